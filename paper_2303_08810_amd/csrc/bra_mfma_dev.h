// Device-side building blocks shared by the matrix-core (MFMA) kernels (internal).
//
// All contractions use v_mfma_f32_16x16x32_bf16 (64-lane wavefront; lane l = 16 g + i):
//   A operand: lane holds A[row i][k = 8 g .. 8 g + 7]
//   B operand: lane holds B[k = 8 g .. 8 g + 7][col i]
//   D result : lane holds D[row 4 g .. 4 g + 3][col i]
// so both operands are read as 16-byte runs along the contraction axis, and the
// contraction may use any key order as long as A and B agree on it.
#pragma once

#include "bra_common.h"

namespace bra {
namespace mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kMaxLds = 160 * 1024;   // LDS per workgroup on gfx950
constexpr int kFastRouteMaxS = 8;     // the matrix-core routing kernels hold a row of A^r in one wavefront: S <= 8 (R <= 64)
constexpr int kTopkRoundsMax = 4;     // up to this k the top-k runs k wavefront-maximum rounds, beyond it rank counting
constexpr int kPoolMaxGroup = 8;      // regions pooled by one workgroup, at most

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// v_mfma_f32_32x32x16_bf16: lane l = 32 h + c holds A[row c][k 8 h .. 8 h + 7], B[k 8 h ..][col c]
// and, in result register 4 q + j, D[row 8 q + 4 h + j][col c].  On this chip it runs at twice
// the flop rate of the 16x16x32 form (measured: 2.46 against 1.4 PFLOP/s in register-only loops).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ unsigned pack_bf16(float a, float b)
{
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(unsigned, r);
}

__device__ __forceinline__ bf16x8 pack8(const float *v)
{
    u32x4 u = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
               pack_bf16(v[6], v[7])};
    return __builtin_bit_cast(bf16x8, u);
}

__device__ __forceinline__ u32x2 pack4(f32x4 v)
{
    return u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
}

__device__ __forceinline__ float bf16_lo(unsigned u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// row / width without an integer division; exact for the small non-negative values
// that occur here (row < 2^20).
__device__ __forceinline__ int fast_div(int row, float width_inv)
{
    return (int)(((float)row + 0.5f) * width_inv);
}

// Exact split of 8 float32 values into three bf16 terms each (x = hi + mid + lo: 3 x 8
// mantissa bits), as MFMA operands.
__device__ __forceinline__ void split3(const float (&x)[8], bf16x8 (&t)[3])
{
    u32x4 h, m, l;      // pairs of bf16, rounded by the hardware conversion (nearest even)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        h[p] = pack_bf16(x[2 * p], x[2 * p + 1]);
        const float r0 = x[2 * p] - bf16_lo(h[p]), r1 = x[2 * p + 1] - bf16_hi(h[p]);
        m[p] = pack_bf16(r0, r1);
        l[p] = pack_bf16(r0 - bf16_lo(m[p]), r1 - bf16_hi(m[p]));
    }
    t[0] = __builtin_bit_cast(bf16x8, h);
    t[1] = __builtin_bit_cast(bf16x8, m);
    t[2] = __builtin_bit_cast(bf16x8, l);
}

// v_mfma_f32_4x4x4_16B_bf16: 16 independent 4x4 blocks, 4 contraction elements each.
// Lane l belongs to block l / 4 and holds row l % 4 of A, column l % 4 of B and of D
// (D rows in the 4 result registers).
__device__ __forceinline__ f32x4 mfma4(s16x4 a, s16x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(a, b, c, 0, 0, 0);
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s
// supplies the address of 4 consecutive 16-bit elements; the four lanes 4 j .. 4 j + 3
// together supply a row j of 16 elements.  Lane i receives element i of rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr16(const bf16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)p);
}

// A 16-byte store to global memory.  MODE 0: an ordinary store (the line stays dirty in this
// XCD's L2 until it is evicted or the kernel ends); 1: with the streaming hint; 2: written through
// to memory (system scope), so that the write-back does not wait for the end of the kernel.
template <int MODE>
__device__ __forceinline__ void store16(void *p, u32x4 v)
{
    if constexpr (MODE == 1) __builtin_nontemporal_store(v, (u32x4 *)p);
    else if constexpr (MODE == 2)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else *(u32x4 *)p = v;
}

// max(x, x of the lane that the DPP control CTRL names), for the rows (of 16 lanes) in
// the mask ROWS; the other rows keep x.
template <int CTRL, int ROWS>
__device__ __forceinline__ uint32_t dpp_umax(uint32_t x)
{
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROWS, 0xf, false);
    return o > x ? o : x;
}

// x + x of the lane that the DPP control CTRL names (all rows; every lane has a source, the
// zero fill of bound_ctrl only lets the compiler fold the move into the add).
template <int CTRL>
__device__ __forceinline__ float dpp_fadd(float x)
{
    const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true);
    return x + __builtin_bit_cast(float, o);
}

// Sums over aligned groups of 2 or 4 consecutive lanes (STEPS = 1 or 2) of each of the 16
// accumulators of a projection tile, in a fixed butterfly order; every lane of a group
// ends up with the group's sum.
template <int STEPS>
__device__ __forceinline__ void lane_group_sums(f32x4 (&acc)[4])
{
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            float v = acc[tt][jj];
            if (STEPS >= 1) v = dpp_fadd<0xB1>(v);      // quad_perm [1,0,3,2]
            if (STEPS >= 2) v = dpp_fadd<0x4E>(v);      // quad_perm [2,3,0,1]
            acc[tt][jj] = v;
        }
}

// Maximum of an unsigned value over the 64 lanes of a wavefront (DPP reduction: within
// quads, half rows, rows of 16 lanes, then across the rows), returned to every lane.
__device__ __forceinline__ uint32_t wave_umax(uint32_t v)
{
    v = dpp_umax<0xB1, 0xf>(v);     // quad_perm [1,0,3,2]
    v = dpp_umax<0x4E, 0xf>(v);     // quad_perm [2,3,0,1]
    v = dpp_umax<0x141, 0xf>(v);    // row_half_mirror
    v = dpp_umax<0x140, 0xf>(v);    // row_mirror: every lane of a row holds the row's maximum
    v = dpp_umax<0x142, 0xa>(v);    // row_bcast15: rows 1, 3 take in rows 0, 2
    v = dpp_umax<0x143, 0xc>(v);    // row_bcast31: rows 2, 3 take in rows 0, 1
    return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1);
}

// Indices of the k largest entries of one row of A^r (Eq. 5), the row spread over the
// 64 lanes of a wavefront (lane j holds entry j; entries j >= R do not exist): larger
// value first, equal values by smaller index, NaN as -inf.  The values are mapped to
// unsigned integers of the same order (never zero).  Small k: k rounds of wavefront
// maximum, lowest lane that holds it, remove it.  Large k: each lane forms a 64-bit key
// (mapped value, then 63 - j) that is larger for whatever comes first and counts the
// larger keys with one lane broadcast per other lane; the lane at position p < k writes
// its index to out[p].
__device__ __forceinline__ uint32_t topk_order_key(float v, int j, int R)
{
    if (!(v == v) || j >= R) v = -INFINITY;
    v += 0.0f;                                              // -0 and +0 are equal values
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);     // -inf -> 0x007fffff, the smallest
}

__device__ __forceinline__ void wave_topk(float v, int j, int R, int k, int32_t *out)
{
    const uint32_t u = topk_order_key(v, j, R);
    if (k <= kTopkRoundsMax) {
        bool avail = j < R;
        for (int p = 0; p < k; ++p) {
            const uint32_t m = wave_umax(avail ? u : 0u);
            const uint64_t holders = __ballot(avail && u == m);
            const int best = __builtin_ctzll(holders);      // k <= R: some entry is still available
            if (j == 0) out[p] = best;
            if (j == best) avail = false;
        }
        return;
    }
    const uint64_t key = ((uint64_t)u << 32) | (uint32_t)(kWave - 1 - j);
    int before = 0;
#pragma unroll
    for (int o = 0; o < kWave; ++o) {
        const uint32_t uo = (uint32_t)__builtin_amdgcn_readlane((int)u, o);
        const uint64_t ko = ((uint64_t)uo << 32) | (uint32_t)(kWave - 1 - o);
        before += ko > key ? 1 : 0;
    }
    if (j < R && before < k) out[before] = j;
}

// The same for NR rows held by one wavefront (row rr in v[rr], its index goes to
// out + rr * k; rows rr >= nrows are not written).  For small k the rounds of the rows
// are interleaved: each round is a chain of dependent cross-lane steps, and independent
// chains fill each other's waits.
template <int NR>
__device__ __forceinline__ void wave_topk_rows(const float (&v)[NR], int nrows, int j, int R, int k,
                                               int32_t *out)
{
    if (k > kTopkRoundsMax) {
#pragma unroll
        for (int rr = 0; rr < NR; ++rr)
            if (rr < nrows) wave_topk(v[rr], j, R, k, out + rr * k);
        return;
    }
    uint32_t u[NR];
    bool avail[NR];
#pragma unroll
    for (int rr = 0; rr < NR; ++rr) {
        u[rr] = topk_order_key(v[rr], j, R);
        avail[rr] = j < R;
    }
    for (int p = 0; p < k; ++p) {
        uint32_t m[NR];
#pragma unroll
        for (int rr = 0; rr < NR; ++rr) m[rr] = wave_umax(avail[rr] ? u[rr] : 0u);
#pragma unroll
        for (int rr = 0; rr < NR; ++rr) {
            const uint64_t holders = __ballot(avail[rr] && u[rr] == m[rr]);
            const int best = __builtin_ctzll(holders);      // k <= R: some entry is still available
            if (j == 0 && rr < nrows) out[rr * k + p] = best;
            if (j == best) avail[rr] = false;
        }
    }
}

// Global -> register half of a tile copy: chunk idx (16 bytes) is row idx / (C/8) of
// the tile, token (y0 + row / tw, x0 + row % tw) of the map; chunks past `rows` and
// tokens outside the image read as zero.  NT: threads of the workgroup.
template <int C, int NB, int NT = 256>
__device__ __forceinline__ void tile_load(u32x4 (&r)[NB], const bf16_t *__restrict__ img, int y0,
                                          int x0, int tw, float tw_inv, int rows, int H, int W,
                                          int first)
{
    constexpr int CH = C / 8;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int idx = first + (int)threadIdx.x + NT * u;
        const int row = idx / CH, cc = idx % CH;
        const int ty = fast_div(row, tw_inv);
        const int y = y0 + ty, x = x0 + row - ty * tw;
        // branch-free: a chunk outside the tile or the image reads the first bytes of the
        // image instead and is zeroed afterwards
        const bool ok = row < rows && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
        const unsigned off = ok ? (unsigned)((y * W + x) * C + cc * 8) : 0u;
        const u32x4 v = *(const u32x4 *)(img + off);
        r[u] = ok ? v : u32x4{0u, 0u, 0u, 0u};
    }
}

// Register -> LDS half: rows of CS elements.
template <int C, int CS, int NB, int NT = 256>
__device__ __forceinline__ void tile_store(bf16_t *dst, const u32x4 (&r)[NB], int rows, int first)
{
    constexpr int CH = C / 8;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int idx = first + (int)threadIdx.x + NT * u;
        const int row = idx / CH, cc = idx % CH;
        if (row < rows) *(u32x4 *)(dst + row * CS + cc * 8) = r[u];
    }
}

// LCE weights [C][25] bf16 in memory -> [25][C] float32 in LDS, in two halves so that
// the loads can be issued early and the LDS writes done later.
template <int C>
struct LceWeights {
    static constexpr int NW = (C * 25 / 8 + 255) / 256;   // 16-byte chunks per thread
    u32x4 r[NW];
    __device__ __forceinline__ void load(const bf16_t *__restrict__ Wlce)
    {
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const int t = threadIdx.x + 256 * u;
            r[u] = u32x4{0u, 0u, 0u, 0u};
            if (t < C * 25 / 8) r[u] = *(const u32x4 *)(Wlce + t * 8);
        }
    }
    __device__ __forceinline__ void store(float *Wl) const
    {
#pragma unroll
        for (int u = 0; u < NW; ++u) {
            const int t = threadIdx.x + 256 * u;
            if (t < C * 25 / 8) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int idx = t * 8 + e;             // flat (channel, tap)
                    const unsigned bits = r[u][e / 2];
                    Wl[(idx % 25) * C + idx / 25] = (e & 1) ? bf16_hi(bits) : bf16_lo(bits);
                }
            }
        }
    }
};

// Reductions over the four lanes {i, 16 + i, 32 + i, 48 + i} (one per 16-lane row), result
// in all four: v_permlane16_swap / v_permlane32_swap exchange rows between two copies of
// the value, so that two register-only steps replace two trips through the LDS crossbar.
__device__ __forceinline__ float cross_row_max(float x)
{
    const int xi = __builtin_bit_cast(int, x);
    const auto a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);     // rows (0,1) and (2,3) paired
    const float m = fmaxf(__builtin_bit_cast(float, (int)a[0]), __builtin_bit_cast(float, (int)a[1]));
    const int mi = __builtin_bit_cast(int, m);
    const auto b = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);     // halves paired
    return fmaxf(__builtin_bit_cast(float, (int)b[0]), __builtin_bit_cast(float, (int)b[1]));
}

__device__ __forceinline__ float cross_row_sum(float x)
{
    const int xi = __builtin_bit_cast(int, x);
    const auto a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const float m = __builtin_bit_cast(float, (int)a[0]) + __builtin_bit_cast(float, (int)a[1]);
    const int mi = __builtin_bit_cast(int, m);
    const auto b = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
    return __builtin_bit_cast(float, (int)b[0]) + __builtin_bit_cast(float, (int)b[1]);
}

// The value of the lane that the DPP control CTRL names.
template <int CTRL>
__device__ __forceinline__ float dpp_get(float x)
{
    const int xi = __builtin_bit_cast(int, x);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(xi, xi, CTRL, 0xf, 0xf, false));
}

// Maxima over the 64 lanes of a wavefront of 4 values per lane at once, to every lane.
// Lane pairs, then pairs of pairs, split the 4 values between them (each keeps the values
// it will own and takes in the partner's copies), so the later steps handle one value per
// lane: over the quads of a 16-lane row by rotation, over the rows by the lane swaps;
// the lanes of a quad then hand their results round.  No NaN in s (max as a median).
__device__ __forceinline__ void wave_fmax4(const f32x4 &s, int lane, float (&m)[4])
{
    const auto mx = [](float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); };
    const bool odd = lane & 1, hi = lane & 2;
    float a = mx(odd ? s[2] : s[0], dpp_get<0xB1>(odd ? s[0] : s[2]));      // rows 0 | 2 over lanes l, l ^ 1
    float b = mx(odd ? s[3] : s[1], dpp_get<0xB1>(odd ? s[1] : s[3]));      // rows 1 | 3
    float x = mx(hi ? b : a, dpp_get<0x4E>(hi ? a : b));                    // quad lane q owns row 2 (q & 1) + (q >> 1)
    x = mx(x, dpp_get<0x124>(x));       // row_ror:4
    x = mx(x, dpp_get<0x128>(x));       // row_ror:8
    x = cross_row_max(x);
    m[0] = dpp_get<0x00>(x);            // quad_perm [0,0,0,0]
    m[1] = dpp_get<0xAA>(x);            // [2,2,2,2]
    m[2] = dpp_get<0x55>(x);            // [1,1,1,1]
    m[3] = dpp_get<0xFF>(x);            // [3,3,3,3]
}

// Online-softmax state of one wavefront: 16 queries (one per lane column i), all heads.
template <int HEADS>
struct SoftmaxState {
    float m[HEADS];          // reference score of the exponentials (at most 2^8 below the running maximum)
    f32x4 lacc[HEADS];       // softmax denominator of query i in entry 0 (all four entries when summed by MFMA)
    f32x4 acc[HEADS][2];     // O^T[channel 16 dt + 4 g + j][query i]
    __device__ __forceinline__ float denom(int h) const { return lacc[h][0]; }
    __device__ __forceinline__ void init()
    {
#pragma unroll
        for (int h = 0; h < HEADS; ++h) {
            m[h] = -INFINITY;
            lacc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[h][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[h][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
};

// Online-softmax step of one head for one block of 64 keys, given the scores
// s[t][j] = S^T[key 16 t + 4 g + j][query i] of this wavefront's 16 queries (Eq. 1, one
// softmax over all routed keys), then O^T += V^T P^T with V read by the transposing LDS
// read: the row of key 32 tp + 16 half + 4 g + i / 4 starts vrow(tp, half) elements into
// Vs, the head's channels at column vcol of it.  The head's running state is slot h of st.
// The exponentials are taken against a reference score that follows the running maximum
// lazily: it moves (and the sums are rescaled) only when some query's block maximum exceeds
// it by more than 2^8 in the exponent, so p <= 256 and most blocks skip the rescaling; the
// quotient O / denominator does not depend on the reference.  MFMA_SUM: the denominators
// come from a product of P^T with an all-ones operand (they sum the same bf16-rounded P as O
// does), which pays when many key blocks follow each other; otherwise they are summed in
// float32 on the vector unit (entry 0 of the state's denominator only).
// FIRST: this is the head's first block (state as left by init()), so there is nothing to
// rescale.
template <bool FIRST, int HEADS, typename VRow, bool MFMA_SUM = false>
__device__ __forceinline__ void softmax_pv_rows(const bf16_t *Vs, VRow vrow, const f32x4 (&s)[4],
                                                SoftmaxState<HEADS> &st, int h, int vcol, float c_exp,
                                                int i)
{
    float mx = s[0][0];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) mx = fmaxf(mx, s[t][jj]);
    mx = cross_row_max(mx);
    if (FIRST) {
        st.m[h] = mx;
    } else if (__builtin_amdgcn_ballot_w64(mx > st.m[h] + 8.0f / c_exp) != 0) {
        // some query's scores outgrew the reference by 2^8: move it, rescale what has been summed
        const float m_new = fmaxf(st.m[h], mx);
        const float alpha = __builtin_amdgcn_exp2f((st.m[h] - m_new) * c_exp);
        st.m[h] = m_new;
        if (MFMA_SUM) st.lacc[h] *= alpha;
        else st.lacc[h][0] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) st.acc[h][dt] *= alpha;
    }
    const float mc = st.m[h] * c_exp;
    float p[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) p[t][jj] = __builtin_amdgcn_exp2f(fmaf(s[t][jj], c_exp, -mc));
    const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    if (!MFMA_SUM) {
        float ls = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) ls += p[t][jj];
        st.lacc[h][0] += cross_row_sum(ls);
    }
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        float pv[8] = {p[2 * tp][0], p[2 * tp][1], p[2 * tp][2], p[2 * tp][3],
                       p[2 * tp + 1][0], p[2 * tp + 1][1], p[2 * tp + 1][2], p[2 * tp + 1][3]};
        const bf16x8 pb = pack8(pv);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            const int col = vcol + 16 * dt + 4 * (i % 4);
            const s16x4 v0 = lds_read_tr16(Vs + vrow(tp, 0) + col);
            const s16x4 v1 = lds_read_tr16(Vs + vrow(tp, 1) + col);
            u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
            u32x4 av = {a0[0], a0[1], a1[0], a1[1]};
            st.acc[h][dt] = mfma16(__builtin_bit_cast(bf16x8, av), pb, st.acc[h][dt]);
        }
        if (MFMA_SUM) st.lacc[h] = mfma16(__builtin_bit_cast(bf16x8, ones), pb, st.lacc[h]);   // sums of the rounded P
    }
}

// The same with the 64 keys in consecutive rows of pitch VS.
template <int VS, bool FIRST = false, bool MFMA_SUM = false, int HEADS>
__device__ __forceinline__ void softmax_pv_block(const bf16_t *Vs, const f32x4 (&s)[4],
                                                 SoftmaxState<HEADS> &st, int h, int vcol, float c_exp,
                                                 int g, int i)
{
    auto vrow = [=](int tp, int half) { return (32 * tp + 16 * half + 4 * g + i / 4) * VS; };
    softmax_pv_rows<FIRST, HEADS, decltype(vrow), MFMA_SUM>(Vs, vrow, s, st, h, vcol, c_exp, i);
}

// One block of 64 keys (rows of Ks / Vs, CS elements per row) against the 16 queries of
// this wavefront (qf[h] = B operand of head h): S^T = K Q^T, then the softmax / PV step.
// The wavefront handles the HPG heads from h0 on (slot h of qf / st is head h0 + h).
template <int C, int CS, int HPG = C / 32>
__device__ __forceinline__ void attn_key_block(const bf16_t *Ks, const bf16_t *Vs,
                                               const bf16x8 (&qf)[HPG],
                                               SoftmaxState<HPG> &st, float c_exp, int g, int i, int h0 = 0)
{
#pragma unroll
    for (int h = 0; h < HPG; ++h) {
        const int col = 32 * (h0 + h);
        f32x4 s[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * CS + col + 8 * g);
            s[t] = mfma16(kf, qf[h], f32x4{0.f, 0.f, 0.f, 0.f});   // S^T[key 16t+4g+j][query i]
        }
        // denominators by MFMA while the four accumulator registers per head are affordable
        softmax_pv_block<CS, false, (HPG <= 4)>(Vs, s, st, h, col, c_exp, g, i);
    }
}

// Normalised attention output of this wavefront's 16 queries -> rows 16 wave + i of the
// float32 output tile Os (OS floats per row).
template <int C, int OS, int HPG = C / 32>
__device__ __forceinline__ void attn_write_out(float *Os, const SoftmaxState<HPG> &st, int wave,
                                               int g, int i, int h0 = 0)
{
#pragma unroll
    for (int h = 0; h < HPG; ++h) {
        const float inv = 1.0f / st.denom(h);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            f32x4 o = st.acc[h][dt] * inv;
            *(f32x4 *)(Os + (16 * wave + i) * OS + 32 * (h0 + h) + 16 * dt + 4 * g) = o;
        }
    }
}

// LCE (Eq. 7): 5x5 depth-wise cross-correlation of V over the halo tile Hs (rows of CS
// bf16, (qh + 4) x hw tokens, hw = rw + 4), added to the output tile Os.  One task =
// (row of the query tile, 8-token segment, channel pair); Wl is [25][C] float32.
template <int C, int CS, int OS, int NT = 256>
__device__ __forceinline__ void lce_add_valu(const bf16_t *Hs, const float *Wl, float *Os, int qh,
                                             int rw, int hw)
{
    const int segs = rw / 8, cp_n = C / 2;
    const int tasks = qh * segs * cp_n;
    for (int task = threadIdx.x; task < tasks; task += NT) {
        const int cp = task % cp_n, seg = (task / cp_n) % segs, r = task / (cp_n * segs);
        const int c = 2 * cp;
        float a0[8], a1[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) { a0[x] = 0.f; a1[x] = 0.f; }
#pragma unroll
        for (int ky = 0; ky < 5; ++ky) {
            f32x2 wk[5];
#pragma unroll
            for (int kx = 0; kx < 5; ++kx) wk[kx] = *(const f32x2 *)(Wl + (ky * 5 + kx) * C + c);
            float v0[12], v1[12];
#pragma unroll
            for (int x = 0; x < 12; ++x) {
                const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + seg * 8 + x) * CS + c);
                v0[x] = bf16_lo(u);
                v1[x] = bf16_hi(u);
            }
#pragma unroll
            for (int x = 0; x < 8; ++x)
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) {
                    a0[x] = fmaf(wk[kx][0], v0[x + kx], a0[x]);
                    a1[x] = fmaf(wk[kx][1], v1[x + kx], a1[x]);
                }
        }
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            f32x2 *o = (f32x2 *)(Os + (r * rw + seg * 8 + x) * OS + c);
            f32x2 cur = *o;
            cur[0] += a0[x];
            cur[1] += a1[x];
            *o = cur;
        }
    }
}

// W^o fragments of output-channel group cg for the transposed product Y^T = Wo^T O^T:
// tile tt, A row i  <->  output channel 64 cg + 16 (i / 4) + 4 tt + (i % 4), so that a
// lane ends up with 16 consecutive output channels of one token.
template <int C>
__device__ __forceinline__ bf16x8 wo_fragment(const bf16_t *__restrict__ WoT, int cg, int tt, int ks,
                                              int g, int i)
{
    const int o = cg * 64 + 16 * (i / 4) + 4 * tt + (i % 4);
    return *(const bf16x8 *)(WoT + (size_t)o * C + 32 * ks + 8 * g);
}

// Y = O Wo (Eq. 2) for the 16 tokens of this wavefront: rows 16 wave + i of Os -> yrow
// (this lane's token row of Y).  wof: prefetched fragments (C == 64) or unused.
template <int C, int OS, bool PREFETCHED>
__device__ __forceinline__ void wo_project_store(const float *Os, const bf16x8 (*wof)[C / 32],
                                                 const bf16_t *__restrict__ WoT, bf16_t *yrow,
                                                 int wave, int g, int i)
{
    constexpr int KS = C / 32;
    bf16x8 of[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const float *src = Os + (16 * wave + i) * OS + 32 * ks + 8 * g;
        f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
        float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        of[ks] = pack8(v);
    }
#pragma unroll
    for (int cg = 0; cg < C / 64; ++cg) {
        f32x4 ya[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            ya[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 wf;
                if constexpr (PREFETCHED) wf = wof[tt][ks];
                else wf = wo_fragment<C>(WoT, cg, tt, ks, g, i);
                ya[tt] = mfma16(wf, of[ks], ya[tt]);
            }
        }
        u32x2 p0 = pack4(ya[0]), p1 = pack4(ya[1]), p2 = pack4(ya[2]), p3 = pack4(ya[3]);
        u32x4 *dst = (u32x4 *)(yrow + cg * 64 + 16 * g);
        dst[0] = u32x4{p0[0], p0[1], p1[0], p1[1]};
        dst[1] = u32x4{p2[0], p2[1], p3[0], p3[1]};
    }
}

// Arguments shared by the attention kernels.
struct AttnArgs {
    const bf16_t *X;                // input map [B, H, W, C] (fused kernel)
    const bf16_t *WT;               // [3C][C] transposed projection weights (fused kernel)
    const bf16_t *Q, *K, *V;        // projected maps [B, H, W, C] (staged kernel)
    const int32_t *Ir_src;          // routing index in memory, or NULL: route in the kernel
    int32_t *Ir_out;                // where to report the routing index, or NULL
    const bf16_t *Wlce, *WoT;
    const bf16_t *Wa;               // LCE weights as 4x4x4 A operands (fused kernel)
    const bf16_t *Wf;               // projection weights in fragment order (fused kernel)
    const bf16_t *WoF, *WlT;        // Wo as plain fragments, LCE weights [25][C] (small-region kernels)
    bf16_t *Y;
    const float *Xr, *U;            // region means and routing vectors (fused kernel, Ir_src == NULL)
    float c_exp;                    // softmax scale * log2(e)
    int total;                      // workgroups that have work
    int trace = 0;                  // experiment builds: leave phase timestamps in Y
};

// Workgroup -> work item.  Consecutive block ids are dealt round-robin to the 8 XCDs;
// undo that so that the workgroups of one image share an L2.  gridDim.x % 8 == 0.
__device__ __forceinline__ int swizzled_block()
{
    const int per_xcd = gridDim.x / 8;
    return ((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
}

}  // namespace mfma

// Small-region pipeline tail (bra_mfma_small.hip): either everything up to Y in one kernel,
// or per-(region, head) attention into O and the LCE added in place (then W^o is left).  A.Q/K/V, routing fields, Wlce, WoT, Y set.
bool small_supported(const Dims &D);
size_t small_scratch_bytes(const Dims &D);
bool small_needs_projection(const Dims &D);   // launch_small left O = attention + LCE in its scratch map: Y = O Wo is still to do
int launch_small(const Dims &D, const mfma::AttnArgs &A, bf16_t *O, hipStream_t st);
// Attention of regions of 1, 2, 4 or 8 tokens + LCE into O for any C that is a multiple of 64
// (image-resident attention; A.Q/K/V, Ir_src, Ir_out, Wlce, c_exp set).
bool map_tail_supported(const Dims &D);
int launch_map_tail(const Dims &D, const mfma::AttnArgs &A, bf16_t *O, hipStream_t st);
// O += LCE(V) for any map, C % 64 == 0.  ldo: elements between rows of O (0: C); square_tiles: 4 x 32 token
// tiles instead of full-width rows.
int launch_lce_add_any(const Dims &D, const mfma::AttnArgs &A, bf16_t *O, hipStream_t st, int ldo = 0,
                       bool square_tiles = false);

// Attention + LCE + W^o for regions of 64 n tokens with 32 queries per wavefront
// (bra_mfma_attn.hip); A.Q must hold Q multiplied by scale * log2(e).
bool attn_q32_ok(const Dims &D);
int launch_attn_q32(const Dims &D, const mfma::AttnArgs &A, hipStream_t st);

// Pipeline for other channel counts (bra_mfma_wide.hip): any multiple of 64 with heads of 32
// channels, at most 64 regions of 1, 2, 4 or 8 tokens.
bool wide_shape(const Dims &D);          // not one of the specialised channel counts
bool wide_supported(const Dims &D);
size_t wide_workspace_bytes(const Dims &D);
int wide_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt, void *ws,
               hipStream_t st);
int wide_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce, void *Y,
                 int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st);

}  // namespace bra
