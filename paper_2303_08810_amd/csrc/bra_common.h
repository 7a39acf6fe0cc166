// Shared host/device declarations of libbra's kernel families (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/bra.h"

namespace bra {

typedef unsigned short bf16_t;  // raw bf16 bits

// Shape plus everything derived from it (Sec. 3.2: n tokens per region, R regions).
struct Dims {
    int B, H, W, C, heads, S, k, dtype;
    float scale;
    int rh, rw, n, R, N, d, kn;
};

__host__ __device__ inline float bf16_to_f32(bf16_t v)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v << 16;
    return c.f;
}

// Round to nearest, ties to even; NaN stays NaN.
__host__ __device__ inline bf16_t f32_to_bf16(float f)
{
    union { uint32_t u; float f; } c;
    c.f = f;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40u);
    uint32_t lsb = (c.u >> 16) & 1u;
    return (bf16_t)((c.u + 0x7fffu + lsb) >> 16);
}

__device__ inline float load_f32(const float *p) { return *p; }
__device__ inline float load_f32(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ inline void store_from_f32(float *p, float v) { *p = v; }
__device__ inline void store_from_f32(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// GELU(t) = t Phi(t) = t / 2 + |t| (1 - erfc(|t| / sqrt 2)) / 2.  erfc by the approximation of
// Abramowitz & Stegun 7.1.28, erfc(x) = (1 + a1 x + .. + a6 x^6)^-16 (absolute error below
// 3e-7, far inside what a bf16 result resolves; one reciprocal is its only slow instruction);
// the coefficients below are a_k / 2^(k/2), so that the polynomial takes |t| itself.
__device__ __forceinline__ float gelu_f32(float t)
{
    const float a = fabsf(t);
    float p = fmaf(5.382975000e-06f, a, 4.889063564e-05f);
    p = fmaf(p, a, 3.800357500e-05f);
    p = fmaf(p, a, 3.277626324e-03f);
    p = fmaf(p, a, 2.114100615e-02f);
    p = fmaf(p, a, 4.986734697e-02f);
    p = fmaf(p, a, 1.0f);
    p *= p;
    p *= p;
    p *= p;
    p *= p;                                                  // overflows to infinity for large |t|: erfc = 0
    const float q = fmaf(__builtin_amdgcn_rcpf(p), -0.5f, 0.5f);
    return fmaf(a, q, 0.5f * t);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Switches for A/B measurements.  The shipped library is built without BRA_EXPERIMENT: the
// switches are then compile-time constants and nothing is read from the environment.
#ifdef BRA_EXPERIMENT
inline long experiment_value(const char *name, long dflt)
{
    const char *v = getenv(name);
    return v ? atol(v) : dflt;
}
inline bool experiment_flag(const char *name) { return getenv(name) != nullptr; }
#else
constexpr long experiment_value(const char *, long dflt) { return dflt; }
constexpr bool experiment_flag(const char *) { return false; }
#endif

// A routing index as the kernels use it: entries of a caller-supplied index outside
// [0, R) (never produced by the library) are clamped instead of addressing outside the map.
__host__ __device__ inline int region_index(int j, int R) { return j < 0 ? 0 : (j >= R ? R - 1 : j); }

// Kernel identifiers for the optional per-launch timing (bra_profile_begin/end).
enum KernelId {
    K_GEN_POOL = 0, K_GEN_REGION_QK, K_GEN_TOPK, K_GEN_GEMM_QKV, K_GEN_ATTENTION, K_GEN_LCE,
    K_GEN_GEMM_WO, K_MFMA_PREP, K_MFMA_QKV, K_MFMA_ATTENTION, K_MFMA_POOL_QK, K_MFMA_ROUTE_ROWS,
    K_MFMA_FUSED_K1, K_MFMA_ATTN_SMALL, K_MFMA_LCE_ADD, K_MFMA_WO,
    K_BLK_POS_LN, K_BLK_ADD_LN, K_BLK_MLP_IN, K_BLK_MLP_OUT, K_BLK_MLP_FUSED, K_GEN_BACKWARD, K_COUNT
};

// Brackets the launches issued during its lifetime with two events on `st` when
// per-launch timing is switched on; does nothing otherwise.
struct ProfScope {
    ProfScope(hipStream_t st, int id);
    ~ProfScope();
    hipStream_t st_;
    int slot_;
};

// Kernel families.  Each returns a BRA_* code; all checks that can fail happen
// before the first launch.
size_t generic_workspace_bytes(const Dims &D);
int generic_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt,
                  void *ws, hipStream_t st);
int generic_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo,
                    const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                    void *ws, hipStream_t st);
bool generic_supported(const Dims &D);

// float32 tensors with 4 x 4 regions, heads of 32 channels and at most 64 routed keys: two launches on
// the float32 matrix-core instruction (bra_f32_small.hip).  qkv [B N, 3C], pq, pk [B R, C] float32.
bool f32_small_ok(const Dims &D);
int f32_small_forward(const Dims &D, const float *X, const float *Wqkv, const float *Wo, const float *Wlce, float *Y,
                      int32_t *Ir_out_opt, const int32_t *Ir_in_opt, float *qkv, float *pq, float *pk, hipStream_t st);
int f32_small_route(const Dims &D, const float *X, const float *Wqkv, int32_t *Ir, float *Ar_opt, float *qkv,
                    float *pq, float *pk, hipStream_t st);

size_t valu_route_scratch_bytes(const Dims &D);
// Rows of A^r = Q^r (K^r)^T and their top-k from float32 Q^r, K^r [B, R, C] (any region count
// that generic_supported accepts).
int valu_affinity_topk(const Dims &D, const float *Qr, const float *Kr, int32_t *Ir, float *Ar_opt,
                       hipStream_t st);
int valu_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt,
               void *scratch, hipStream_t st);

bool mfma_supported(const Dims &D);
size_t mfma_workspace_bytes(const Dims &D);
int mfma_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt, void *ws,
               hipStream_t st);
int mfma_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                 void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st);

// Out[m][o] = act(sum_k In[m][k] W[k][o] + bias[o]) + res[m][o] on the matrix cores; In [M, K],
// W [K, Nout], Out and res [M, Nout] bf16, bias float32; bias and res may be NULL, act is GELU
// or the identity.  K must be a multiple of 64, Nout of 8.
int gemm_bf16(const bf16_t *In, const bf16_t *W, long M, int K, int Nout, bf16_t *Out, const float *bias,
              const bf16_t *res, bool gelu, int kernel_id, hipStream_t st);

// Maps whose sides S does not divide (bra_pad.hip): Dp describes the zero-padded map.
size_t padded_workspace_bytes(const Dims &Dp, size_t bra_bytes);
int padded_forward(const Dims &Dp, int H, int W, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                   void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, int path, hipStream_t st);

// The projection kernels of bra_mfma.hip for other passes (bf16, C = 64, 128 or 256): Q, K, V = X Wqkv
// into three token maps (with WT given, the same launch writes the transposed weights WT [3C][C] and
// WoT [C][C] of Wqkv and Wo); Out = In W for one row-major C x C matrix.
int mfma_project_qkv(const Dims &D, const void *X, const void *Wqkv, bf16_t *Q, bf16_t *K, bf16_t *V,
                     hipStream_t st, const void *Wo = nullptr, bf16_t *WT = nullptr, bf16_t *WoT = nullptr);
int mfma_project(const Dims &D, const void *In, const bf16_t *W, bf16_t *Out, hipStream_t st);

// The same projection for any C that is a multiple of 64 (bra_mfma_wide.hip).
int wide_project_qkv(const Dims &D, const void *X, const void *Wqkv, bf16_t *Q, bf16_t *K, bf16_t *V, hipStream_t st);

// Backward pass with fixed routing on the matrix cores (bra_mfma_bwd.hip).
bool mfma_backward_supported(const Dims &D);
size_t mfma_backward_workspace_bytes(const Dims &D);
int mfma_backward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                  const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                  hipStream_t st);

// Backward pass with fixed routing, scalar float32 kernels (bra_generic.hip).
bool generic_backward_supported(const Dims &D);
size_t generic_backward_workspace_bytes(const Dims &D);
int generic_backward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                     const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                     hipStream_t st);

// Whole block with the scalar float32 kernels (bra_generic.hip): any dtype, C and hidden.
size_t generic_block_workspace_bytes(const Dims &D, int hidden, size_t bra_bytes);
int generic_block_forward(const Dims &D, int hidden, float eps, const void *X, const bra_block_params &p, void *Xout,
                          int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path,
                          hipStream_t st);

// Whole block around BRA (bra_block.hip).  `path` is the kernel family of the BRA stage
// (BRA_PATH_GENERIC or BRA_PATH_MFMA), `bra_bytes` that family's workspace size.
bool block_supported(const Dims &D, int hidden);
size_t block_workspace_bytes(const Dims &D, int hidden, size_t bra_bytes);
int block_forward(const Dims &D, int hidden, float eps, const void *X, const bra_block_params &p, void *Xout,
                  int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path,
                  hipStream_t st);

}  // namespace bra
