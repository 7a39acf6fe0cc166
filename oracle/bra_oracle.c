/*
 * TEST INFRASTRUCTURE -- CPU oracle for the BRA forward pass (see
 * bra_oracle_impl.h).  Builds the float and the double instance:
 *   oracle_bra_forward_f32(...), oracle_bra_forward_f64(...)
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define REAL float
#define SUFFIX f32
#include "bra_oracle_impl.h"
#undef REAL
#undef SUFFIX

#define REAL double
#define SUFFIX f64
#include "bra_oracle_impl.h"
#undef REAL
#undef SUFFIX
