// Matrix-core (MFMA) kernel family for bf16 tensors on gfx950, head width d = 32.
//
// Intermediates Q, K, V (staged kernels) are bf16 tensors in the spatial [B, H, W, C]
// layout; the region structure of Sec. 3.2 lives in address arithmetic only.  The
// routed key/value tokens (Eq. 6) are copied by index from that layout into LDS,
// never into a gathered tensor in memory.
//
// Routing (Eq. 4-5) is computed in float32, in one of two ways.  From X: a pooling
// kernel forms the region means of X, a routing kernel projects them to Q^r and K^r on
// the matrix cores with an exact three-term bf16 split (mean(X^r) W = mean(X^r W), exact
// in real arithmetic), forms A^r and ranks its rows.  Or from the token projection: the
// projection kernel also writes partial sums of its float32 Q / K accumulators, and the
// routing kernel adds them up per region (used when a region has few of them).
//
// For k = 1 neither Q^r nor K^r is formed: the pooling kernel leaves u_r = Wk (Wq^T mean(X^r))
// per region, and row r of A^r is the means of the image times u_r.
//
// Forward pipelines (C = 64, 128, 256; every other shape: bra_mfma_wide.hip):
//   fused  : k_pool -> k_fused                       (k = 1, 64-token regions, C = 64:
//            projections recomputed per workgroup from X, where recomputing K and V
//            costs less than storing them; the workgroup finds its routed region itself)
//   staged : k_pool -> k_route -> k_qkv -> k_attn_big                 (regions of 64 n tokens)
//            k_qkv -> k_route_p -> small-region kernels (bra_mfma_small.hip)
#include "bra_mfma_dev.h"

#include <stdlib.h>

#include <algorithm>
#include <type_traits>

namespace bra {

using namespace mfma;

namespace {

// ---------------------------------------------------------------------------
// WT[o][c] = Wqkv[c][o] (o < 3C) and WoT[o][c] = Wo[c][o]: the weights with the
// contraction axis contiguous, as the MFMA operands want them.  `e` runs over 4 C^2.
// Elements 4 C^2 .. 4 C^2 + 160 C are the LCE weights (Eq. 7) laid out as the A operands
// of the 4x4x4 matrix products of the fused kernel: for the 16-channel slice s, the
// kernel row ky and the half hh of the 8-wide input window, lane 4 lb + xi holds
//   Wa[s][2 ky + hh][lane][k] = w[16 s + lb][ky][4 hh + k - xi]   (zero outside 0..4),
// so that one 8-byte load per lane fetches an operand and a wavefront reads 512
// contiguous bytes.
constexpr int kLceOperandElems = 160;   // per channel: 5 rows x 2 halves x 4 offsets x 4

// For C = 64 the fused kernel reads all projection weights as ready-made fragments of its
// 32x32x16 products: 10 tiles x 4
// contraction steps x 64 lanes x 8 elements, lane 32 h + c, element s = input channel
// 16 kst + 8 h + s of output channel
//   tiles 0..5: 32 (tile % 2) + prow(c) of Wq, Wk, Wv (tile / 2), prow(c) = 16 (c / 16) + 8 ((c / 4) % 2) +
//               4 ((c / 8) % 2) + c % 4 (the row order that leaves a lane with two runs of 8 channels);
//   tiles 6, 7: 32 (tile - 6) + c of Wv (as a B operand);  tiles 8, 9: 32 (tile - 8) + prow(c) of Wo.
constexpr int kFusedFragElems = 10 * 4 * 64 * 8;

// Elements of the small-region kernels' tables (Wo fragments, LCE weights tap-major).
__host__ __device__ constexpr int small_table_elems(int C) { return C * C + 25 * C; }

__device__ inline void prep_weight_element(const bf16_t *__restrict__ Wqkv,
                                           const bf16_t *__restrict__ Wo,
                                           const bf16_t *__restrict__ Wlce, bf16_t *__restrict__ WT,
                                           bf16_t *__restrict__ WoT, bf16_t *__restrict__ Wa,
                                           bf16_t *__restrict__ Wf, int C, int e)
{
    const int base_elems = 4 * C * C + kLceOperandElems * C;
    if (e >= base_elems && e < base_elems + small_table_elems(C)) {
        // tables of the small-region kernels, kept behind Wa: Wo as plain MFMA fragments
        // WoF[ct][ks][lane 16 g + i][s] = Wo[32 ks + 8 g + s][16 ct + i], then the LCE weights
        // tap-major, WlT[t][c] = Wlce[c][t]
        const int f = e - base_elems;
        bf16_t *tab = Wa + kLceOperandElems * C;
        if (f < C * C) {
            const int s = f % 8, lane = (f / 8) % kWave, ks = (f / 512) % (C / 32), ct = f / (512 * (C / 32));
            tab[f] = Wo[(size_t)(32 * ks + 8 * (lane / 16) + s) * C + 16 * ct + lane % 16];
        } else {
            const int t = (f - C * C) / C, c = (f - C * C) % C;
            tab[f] = Wlce[c * 25 + t];
        }
        return;
    }
    if (e >= base_elems) {                              // only when C == 64
        const int f = e - base_elems - small_table_elems(C);
        const int s = f % 8, lane = (f / 8) % kWave, kst = (f / 512) % 4, tile = f / 2048;
        const int h = lane / 32, c = lane % 32;
        const int prow = 16 * (c / 16) + 8 * ((c / 4) % 2) + 4 * ((c / 8) % 2) + c % 4;
        const int in = 16 * kst + 8 * h + s;
        if (tile < 6) Wf[f] = Wqkv[(size_t)in * 3 * C + (tile / 2) * C + 32 * (tile % 2) + prow];
        else if (tile < 8) Wf[f] = Wqkv[(size_t)in * 3 * C + 2 * C + 32 * (tile - 6) + c];
        else Wf[f] = Wo[(size_t)in * C + 32 * (tile - 8) + prow];
        return;
    }
    if (e >= 4 * C * C) {
        const int a = e - 4 * C * C;
        const int k = a % 4, lane = (a / 4) % kWave, r = (a / (4 * kWave)) % 10, s = a / (40 * kWave);
        const int lb = lane / 4, xi = lane % 4, ky = r / 2, hh = r % 2;
        const int kx = 4 * hh + k - xi;
        Wa[a] = (kx >= 0 && kx <= 4) ? Wlce[(16 * s + lb) * 25 + ky * 5 + kx] : (bf16_t)0;
        return;
    }
    const int o = e / C, c = e % C;
    if (o < 3 * C) WT[e] = Wqkv[(size_t)c * 3 * C + o];
    else WoT[(size_t)(o - 3 * C) * C + c] = Wo[(size_t)c * C + (o - 3 * C)];
}

// Number of prep elements of a forward call.
__host__ __device__ constexpr int prep_total(int C)
{
    return 4 * C * C + kLceOperandElems * C + small_table_elems(C) + (C == 64 ? kFusedFragElems : 0);
}

// Everything the weight rearrangement reads and writes, for kernels that carry it along
// in extra workgroups.
struct PrepArgs {
    const bf16_t *Wqkv, *Wo, *Wlce;
    bf16_t *WT, *WoT, *Wa, *Wf;
    int elems;                      // leading prep elements to produce (0: none)
    int trace = 0;                  // experiment builds: leave phase timestamps in Q
    // The projection kernel can carry the routing from pooled X along (it needs WT, so not in a launch
    // whose prep elements are still being produced): workgroups past the prep ones, one per
    // (image, 16 query regions).
    const float *Xr = nullptr;
    int32_t *Ir = nullptr;
    int route_items = 0;
    Dims dims = {};
};

// `total` = prep_total(C) (all weights) or 3 C^2 (projection weights only; Wo and Wlce
// may be NULL).
__global__ void k_prep_weights(const bf16_t *__restrict__ Wqkv, const bf16_t *__restrict__ Wo,
                               const bf16_t *__restrict__ Wlce, bf16_t *__restrict__ WT,
                               bf16_t *__restrict__ WoT, bf16_t *__restrict__ Wa,
                               bf16_t *__restrict__ Wf, int C, int total)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) prep_weight_element(Wqkv, Wo, Wlce, WT, WoT, Wa, Wf, C, e);
}

// ---------------------------------------------------------------------------
// Region pooling (Sec. 3.2, "Region-to-region routing"): Xr[b, r, :] = mean of the
// tokens of region r, in float32 with a fixed summation order.  Workgroup (b, group)
// handles G consecutive regions of image b and reads their tokens exactly once: a pure
// streaming pass over X.  Workgroups beyond `pool_blocks` rearrange the weights instead.
//
// With U (C = 64, k = 1 pipeline) the workgroup also leaves the routing vector of each of
// its regions: row r of A^r (Eq. 4) is Q^r_r (K^r)^T = (xr_r Wq) (Xr Wk)^T = Xr u_r with
// u_r = Wk (Wq^T xr_r), so whoever needs that row later only needs u_r and the means, not
// the region-level projections.  Wq and Wk (bf16, read from Wqkv at kernel start, parked in
// registers while X streams) pass through LDS; the products are those of float32 arithmetic.
template <int C>
__global__ __launch_bounds__(256) void k_pool(const bf16_t *__restrict__ X,
                                              const bf16_t *__restrict__ Wqkv,
                                              const bf16_t *__restrict__ Wo,
                                              const bf16_t *__restrict__ Wlce,
                                              float *__restrict__ Xr, float *__restrict__ U,
                                              bf16_t *__restrict__ WT,
                                              bf16_t *__restrict__ WoT, bf16_t *__restrict__ Wa,
                                              bf16_t *__restrict__ Wf, Dims D, int pool_blocks, int G,
                                              int prep_elems)
{
    __shared__ float part[2048];   // pooling partials
    constexpr bool kWithU = C == 64;
    __shared__ __attribute__((aligned(16))) bf16_t wqk[kWithU ? 2 * 64 * 64 : 8];   // Wq [e][c], Wk [f][c]
    __shared__ __attribute__((aligned(16))) float xs[kWithU ? kPoolMaxGroup * 64 : 4], qs[kWithU ? kPoolMaxGroup * 64 : 4];
    const int tid = threadIdx.x;
#ifdef BRA_EXPERIMENT
    const bool tracing = prep_elems < 0;
    if (tracing) prep_elems = -prep_elems;
#endif
    if ((int)blockIdx.x >= pool_blocks) {
        const int e = ((int)blockIdx.x - pool_blocks) * 256 + tid;
        if (e < prep_elems) prep_weight_element(Wqkv, Wo, Wlce, WT, WoT, Wa, Wf, C, e);
        return;
    }
#ifdef BRA_EXPERIMENT
    unsigned long long trace_t[4] = {0, 0, 0, 0};
#define BRA_TRACE(k) if (tracing) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    BRA_TRACE(0);
    u32x4 wreg[4];
    if (kWithU && U) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * (u % 2);             // 16-byte chunk of Wq (u < 2) or Wk
            wreg[u] = *(const u32x4 *)(Wqkv + (size_t)(idx / 8) * 3 * C + (u / 2) * C + (idx % 8) * 8);
        }
    }
    constexpr int CH = C / 8;
    const int groups = (D.R + G - 1) / G;
    const int b = blockIdx.x / groups, r0 = (blockIdx.x % groups) * G;
    const int ng = min(G, D.R - r0);                           // regions of this workgroup
    const int items = ng * CH;                                 // (region, 8-channel chunk) pairs
    int P = 8;                                                 // power of two >= items, <= 256
    while (P < items) P *= 2;
    const int SUB = 256 / P;                                   // threads that share one pair
    const int item = tid % P, sub = tid / P;
    if (item < items) {
        const int gi = item / CH, cc = item % CH;
        const int r = r0 + gi;
        const int ry0 = (r / D.S) * D.rh, rx0 = (r % D.S) * D.rw;
        const bf16_t *base = X + (((size_t)b * D.H + ry0) * D.W + rx0) * C + cc * 8;
        const float rw_inv = 1.0f / (float)D.rw;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int slot = sub; slot < D.n; slot += SUB) {
            const int ry = fast_div(slot, rw_inv), rx = slot - ry * D.rw;
            const u32x4 v = *(const u32x4 *)(base + ((size_t)ry * D.W + rx) * C);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] += bf16_lo(v[e]);
                acc[2 * e + 1] += bf16_hi(v[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) part[(sub * items + item) * 8 + e] = acc[e];
    }
    BRA_TRACE(1);
    __syncthreads();
    for (int e = tid; e < ng * C; e += 256) {
        const int gi = e / C, c = e % C;
        const int it = gi * CH + c / 8;
        float s = 0.f;
        for (int sb = 0; sb < SUB; ++sb) s += part[(sb * items + it) * 8 + c % 8];
        const float mean = s / (float)D.n;
        if (kWithU && U) xs[e] = mean;      // stored below: a barrier would wait for the store to land
        else Xr[((size_t)b * D.R + r0 + gi) * C + c] = mean;
    }
    if (kWithU && U) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            *(u32x4 *)(wqk + (u / 2) * 64 * 64 + (tid + 256 * (u % 2)) * 8) = wreg[u];
        __syncthreads();
        // Both products on the matrix cores, the float32 factor split exactly into three
        // bf16 terms (as the routing kernel does): wavefront w owns output channels
        // 16 w .. 16 w + 15, the regions are the columns (columns >= ng repeat the last).
        const int wave = tid / kWave, lane = tid % kWave, g = lane / 16, i = lane % 16;
        const int col = min(i, ng - 1);
        const bf16_t *wq_s = wqk, *wk_s = wqk + 64 * 64;
        auto terms = [&](const float *row, bf16x8 (&t)[3]) {   // 8 consecutive floats -> split operands
            const f32x4 lo = *(const f32x4 *)row, hi = *(const f32x4 *)(row + 4);
            const float x[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            split3(x, t);
        };
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};      // q^T[channel 16 w + 4 g + jj][region i] = sum_e Wq[e][c] xr[e]
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // Wq^T as the A operand: rows of the LDS tile are e, the transposing read turns them
            const bf16_t *wp = wq_s + (32 * ks + 8 * g + i / 4) * 64 + 16 * wave + 4 * (i % 4);
            const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
            const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 4 * 64));
            const bf16x8 wf = __builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]});
            bf16x8 t[3];
            terms(xs + col * 64 + 32 * ks + 8 * g, t);
            acc = mfma16(wf, t[2], acc);       // smallest term first
            acc = mfma16(wf, t[1], acc);
            acc = mfma16(wf, t[0], acc);
        }
        if (i < ng) *(f32x4 *)(qs + i * 64 + 16 * wave + 4 * g) = acc;
        __syncthreads();
        acc = f32x4{0.f, 0.f, 0.f, 0.f};       // u^T[f = 16 w + 4 g + jj][region i] = sum_c Wk[f][c] q[c]
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 wf = *(const bf16x8 *)(wk_s + (16 * wave + i) * 64 + 32 * ks + 8 * g);
            bf16x8 t[3];
            terms(qs + col * 64 + 32 * ks + 8 * g, t);
            acc = mfma16(wf, t[2], acc);
            acc = mfma16(wf, t[1], acc);
            acc = mfma16(wf, t[0], acc);
        }
        if (i < ng) *(f32x4 *)(U + ((size_t)b * D.R + r0 + i) * C + 16 * wave + 4 * g) = acc;
        for (int e = tid; e < ng * C; e += 256) Xr[((size_t)b * D.R + r0) * C + e] = xs[e];
    }
#ifdef BRA_EXPERIMENT
    if (tracing && U) {
        BRA_TRACE(2);
        __syncthreads();
        if (tid == 0) {
            unsigned long long *o = (unsigned long long *)(U + ((size_t)b * D.R + r0) * C);
            for (int k = 0; k < 3; ++k) o[k] = trace_t[k];
        }
    }
#endif
#undef BRA_TRACE
}

// Row `reg` of A^r of image b (Eq. 4) from the routing vector u of the region and the means
// Xr_b [R][64] of the image, by a workgroup of 256 threads, and the index of its largest
// entry (Eq. 5 for k = 1: ties to the smaller index, NaN as -inf), returned to every thread.
// Lane group jq = lane / 4 of wavefront w owns region 16 w + jq, its 4 lanes a quarter of
// the channels each.  Two steps, so that a caller can put other memory requests between
// the loads and their use.
struct RouteRowLoads {
    f32x4 xv[4], uv[4];
};

__device__ __forceinline__ void route_row_load(const float *__restrict__ Xr_b, const float *__restrict__ u,
                                               int R, RouteRowLoads &L)
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int jj = 16 * wave + lane / 4, cq = lane % 4;
    const float *xrow = Xr_b + (size_t)min(jj, R - 1) * 64 + 4 * cq;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        L.xv[e] = *(const f32x4 *)(xrow + 16 * e);
        L.uv[e] = *(const f32x4 *)(u + 4 * cq + 16 * e);
    }
}

// slot: 8 words of LDS.  Contains a barrier.
__device__ __forceinline__ int route_row_k1(const RouteRowLoads &L, int R, uint32_t *slot,
                                            float *__restrict__ Ar_row_opt)
{
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int jj = 16 * wave + lane / 4, cq = lane % 4;
    float a = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int t = 0; t < 4; ++t) a = fmaf(L.xv[e][t], L.uv[e][t], a);
    a = dpp_fadd<0xB1>(a);
    a = dpp_fadd<0x4E>(a);
    if (Ar_row_opt && cq == 0 && jj < R) Ar_row_opt[jj] = a;
    const uint32_t key = topk_order_key(a, jj, R);
    const uint32_t kmax = wave_umax(key);
    const int best = __builtin_ctzll(__ballot(key == kmax)) / 4;
    if (lane == 0) {
        slot[2 * wave] = kmax;
        slot[2 * wave + 1] = (uint32_t)(16 * wave + best);
    }
    __syncthreads();
    uint32_t bk = slot[0];
    int bj = (int)slot[1];
#pragma unroll
    for (int ww = 1; ww < 4; ++ww)
        if (slot[2 * ww] > bk) {
            bk = slot[2 * ww];
            bj = (int)slot[2 * ww + 1];
        }
    return bj;
}

// The routing of the k = 1 pipeline on its own (routing-only calls): workgroup (b, reg).
__global__ __launch_bounds__(256) void k_route_u(const float *__restrict__ Xr, const float *__restrict__ U,
                                                 int32_t *__restrict__ Ir, float *__restrict__ Ar, Dims D)
{
    __shared__ uint32_t slot[8];
    const int b = blockIdx.x / D.R, reg = blockIdx.x % D.R;
    const size_t row = (size_t)b * D.R + reg;
    RouteRowLoads L;
    route_row_load(Xr + (size_t)b * D.R * 64, U + row * 64, D.R, L);
    const int j = route_row_k1(L, D.R, slot, Ar ? Ar + row * D.R : nullptr);
    if (threadIdx.x == 0) Ir[row] = j;
}

// Region-level projections, A^r = Q^r (K^r)^T (Eq. 4) and its row-wise top-k index I^r
// (Eq. 5).  Workgroup (b, rt) owns the 16 regions 16 rt .. 16 rt + 15 of image b as
// queries (R <= 64).  Q^r = Xr Wq for those rows and K^r = Xr Wk for all regions of the
// image run on the matrix cores: the float32 means are split exactly into three bf16
// terms (once per workgroup, staged in LDS in chunks of 64 channels), each term
// is multiplied by the bf16 weights with float32 accumulation, so the products are those
// of the float32 computation.  Wavefront w owns output-channel tiles w, w + 4, ..; the
// results go to LDS (K^r transposed), then wavefront w forms rows 4 w .. 4 w + 3 of A^r
// in float32, lane j holding entry j, and ranks them.
constexpr int kRouteRS = 65;   // regions (float4 slots) per 4-channel group of the K^r tile in LDS

// Rows NR w .. NR w + NR - 1 (of the 4 NR query regions of row tile myrt) of A^r = Q^r (K^r)^T in
// float32 from the LDS tiles Kt [C / 4][kRouteRS][4] (K^r: channel group, region, channel in
// the group) and Qs [4 NR][C + 4], lane j
// holding entry j; then their top-k (Eq. 5) and, if asked for, the rows themselves.
template <int C, int NR = 4>
__device__ __forceinline__ void route_rows_from_lds(const float *Kt, const float *Qs, int b, int myrt,
                                                    const Dims &D, int32_t *__restrict__ Ir,
                                                    float *__restrict__ Ar)
{
    constexpr int QS = C + 4;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    float a[NR];
#pragma unroll
    for (int rr = 0; rr < NR; ++rr) a[rr] = 0.f;
    const float *qrow = Qs + NR * wave * QS;
#pragma unroll 4
    for (int c = 0; c < C; c += 4) {
        const f32x4 kv = *(const f32x4 *)(Kt + ((c / 4) * kRouteRS + lane) * 4);
#pragma unroll
        for (int rr = 0; rr < NR; ++rr) {
            const f32x4 q4 = *(const f32x4 *)(qrow + rr * QS + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) a[rr] = fmaf(q4[e], kv[e], a[rr]);
        }
    }
    const int r0 = 4 * NR * myrt + NR * wave;
    if (r0 >= D.R) return;
    const int nrows = min(NR, D.R - r0);
    const size_t row0 = (size_t)b * D.R + r0;
    if (Ar && lane < D.R) {
#pragma unroll
        for (int rr = 0; rr < NR; ++rr)
            if (rr < nrows) Ar[(row0 + rr) * D.R + lane] = a[rr];
    }
    wave_topk_rows<NR>(a, nrows, lane, D.R, D.k, Ir + row0 * D.k);
}

template <int C>
struct RouteSmem {
    static constexpr int CK = 64;                       // channels per staged chunk
    static constexpr int XP = CK + 16;                  // bf16 per row of a staged term
    static constexpr int QS = C + 4;                    // floats per row of the Q^r tile
    static constexpr size_t xs_bytes = (size_t)3 * 64 * XP * 2;
    static constexpr size_t kq_bytes = ((size_t)C * kRouteRS + 16 * QS) * 4;   // takes the place of the terms
    static constexpr size_t bytes = xs_bytes > kq_bytes ? xs_bytes : kq_bytes;
};

// Work item `wid` = (image, 16 query regions), by the first 256 threads of a workgroup (all of them
// reach every barrier of this function); smem: RouteSmem<C>::bytes.
template <int C>
__device__ __forceinline__ void route_body(const float *__restrict__ Xr, const bf16_t *__restrict__ WT,
                                           int32_t *__restrict__ Ir, float *__restrict__ Ar, const Dims &D,
                                           char *smem, int wid)
{
    typedef RouteSmem<C> SM;
    constexpr int CK = SM::CK, XP = SM::XP, QS = SM::QS, KSC = CK / 32, NCW = C / 64;
    bf16_t *xs = (bf16_t *)smem;                  // [3][64][XP]
    float *Kt = (float *)smem;                    // [C / 4][kRouteRS][4]
    float *Qs = Kt + C * kRouteRS;                // [16][QS]
    const int groups = (D.R + 15) / 16;
    const int b = wid / groups, myrt = wid % groups;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int nrt = (D.R + 15) / 16;              // region tiles that exist
    // staging: thread (row, quarter) splits CK / 4 consecutive channels of one region
    const int srow = threadIdx.x / 4, sq = threadIdx.x % 4;
    const float *xsrc = Xr + ((size_t)b * D.R + min(srow, D.R - 1)) * C + sq * (CK / 4);   // rows past R repeat the last region; never used

    f32x4 ak[4][NCW], aq[NCW];
#pragma unroll
    for (int cw = 0; cw < NCW; ++cw) {
        aq[cw] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) ak[rt][cw] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll 1
    for (int c0 = 0; c0 < C; c0 += CK) {
        // requests of this chunk: the means to split and this wavefront's weight fragments
        f32x4 xv[CK / 16];
#pragma unroll
        for (int e = 0; e < CK / 16; ++e) xv[e] = *(const f32x4 *)(xsrc + c0 + 4 * e);
        bf16x8 wqf[KSC][NCW], wkf[KSC][NCW];
#pragma unroll
        for (int ksl = 0; ksl < KSC; ++ksl)
#pragma unroll
            for (int cw = 0; cw < NCW; ++cw) {
                const size_t off = (size_t)(16 * (wave + 4 * cw) + i) * C + c0 + 32 * ksl + 8 * g;
                wqf[ksl][cw] = *(const bf16x8 *)(WT + off);
                wkf[ksl][cw] = *(const bf16x8 *)(WT + (size_t)C * C + off);
            }
        if (c0) __syncthreads();                  // the previous chunk's terms have been read
#pragma unroll
        for (int e0 = 0; e0 < CK / 4; e0 += 8) {
            const f32x4 lo = xv[e0 / 4], hi = xv[e0 / 4 + 1];
            const float x[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            bf16x8 t[3];
            split3(x, t);
#pragma unroll
            for (int q = 0; q < 3; ++q) *(bf16x8 *)(xs + (q * 64 + srow) * XP + sq * (CK / 4) + e0) = t[q];
        }
        __syncthreads();
#pragma unroll
        for (int ksl = 0; ksl < KSC; ++ksl) {
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
                if (rt >= nrt) break;
                bf16x8 t[3];
#pragma unroll
                for (int q = 0; q < 3; ++q)
                    t[q] = *(const bf16x8 *)(xs + (q * 64 + 16 * rt + i) * XP + 32 * ksl + 8 * g);
#pragma unroll
                for (int cw = 0; cw < NCW; ++cw) {
                    ak[rt][cw] = mfma16(wkf[ksl][cw], t[2], ak[rt][cw]);    // smallest term first
                    ak[rt][cw] = mfma16(wkf[ksl][cw], t[1], ak[rt][cw]);
                    ak[rt][cw] = mfma16(wkf[ksl][cw], t[0], ak[rt][cw]);
                }
                if (rt == myrt) {
#pragma unroll
                    for (int cw = 0; cw < NCW; ++cw) {
                        aq[cw] = mfma16(wqf[ksl][cw], t[2], aq[cw]);
                        aq[cw] = mfma16(wqf[ksl][cw], t[1], aq[cw]);
                        aq[cw] = mfma16(wqf[ksl][cw], t[0], aq[cw]);
                    }
                }
            }
        }
    }
    __syncthreads();   // the terms have been read: K^r and Q^r take their place
    // accumulators hold [channel 16 ct + 4 g + jj][region 16 rt + i]
#pragma unroll
    for (int cw = 0; cw < NCW; ++cw) {
        const int ch = 16 * (wave + 4 * cw) + 4 * g;
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) *(f32x4 *)(Kt + ((ch / 4) * kRouteRS + 16 * rt + i) * 4) = ak[rt][cw];
        *(f32x4 *)(Qs + i * QS + ch) = aq[cw];
    }
    __syncthreads();

    route_rows_from_lds<C>(Kt, Qs, b, myrt, D, Ir, Ar);
}

template <int C>
__global__ __launch_bounds__(256) void k_route(const float *__restrict__ Xr,
                                               const bf16_t *__restrict__ WT,
                                               int32_t *__restrict__ Ir, float *__restrict__ Ar,
                                               Dims D)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int wid = swizzled_block();          // the workgroups of an image share an XCD (and its L2)
    if (wid >= D.B * ((D.R + 15) / 16)) return;
    route_body<C>(Xr, WT, Ir, Ar, D, smem, wid);
}

// Routing from the partial sums that the projection kernel leaves behind (P[token / group]
// [2C] = [sum Q | sum K] over `group` = 2^group_log2 consecutive tokens of one region row):
// Q^r and K^r are the region means of Q and K (Sec. 3.2), i.e. the sum of a region's
// rh x (rw / group) partial sums in a fixed order, divided by n.  Workgroup (b, rt) as in
// k_route; no matrix products are left to do here.
// With `whole` the projection kernel ran over region tiles and P[b R + r][2C] already holds the sums
// over each region.
template <int C, int NR>
__global__ __launch_bounds__(256) void k_route_p(const float *__restrict__ P, int32_t *__restrict__ Ir,
                                                 float *__restrict__ Ar, Dims D, int group_log2, int whole)
{
    constexpr int QS = C + 4, C4 = C / 4, QR = 4 * NR;     // query regions of a workgroup
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float *Kt = (float *)smem;                    // [C / 4][kRouteRS][4]
    float *Qs = Kt + C * kRouteRS;                // [QR][QS]
    const int groups = (D.R + QR - 1) / QR;
    const int wid = swizzled_block();          // the workgroups of an image share an XCD (and its L2)
    if (wid >= D.B * groups) return;
    const int b = wid / groups, myrt = wid % groups;
    const int pw = D.W >> group_log2, pc = D.rw >> group_log2;      // partial sums per image row / region row
    const float inv_n = 1.0f / (float)D.n;
#ifdef BRA_EXPERIMENT
    unsigned long long trace_t[4] = {0, 0, 0, 0};
    const bool tracing = whole & 2;
#define BRA_TRACE(k) if (tracing) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    whole &= 1;
    BRA_TRACE(0);
    // Work items (region, 4 channels): all of K^r, then the QR query rows of Q^r.  A thread
    // takes its NI items at once so that their loads are in flight together; the partial sums of
    // an item are added in the order (row of the region, position in the row).
    constexpr int NI = ((64 + QR) * C4 + 255) / 256;       // every item of a workgroup in one round (R <= 64)
    const int nk = D.R * C4, total = nk + QR * C4;
    for (int i0 = threadIdx.x; i0 < total; i0 += 256 * NI) {
        const float *src[NI];
        f32x4 acc[NI];
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int idx = min(i0 + 256 * u, total - 1);
            const bool isq = idx >= nk;
            const int row = (isq ? idx - nk : idx) / C4, c4 = (isq ? idx - nk : idx) % C4;
            const int r = isq ? min(QR * myrt + row, D.R - 1) : row;     // rows past R repeat the last region; never used
            const int ry = r / D.S, rx = r % D.S;
            src[u] = P + (whole ? (size_t)b * D.R + r : ((size_t)b * D.H + ry * D.rh) * pw + rx * pc) * 2 * C +
                     (isq ? 0 : C) + 4 * c4;
            acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const int nyy = whole ? 1 : D.rh, ncc = whole ? 1 : pc;
        for (int yy = 0; yy < nyy; ++yy)
            for (int cc = 0; cc < ncc; ++cc) {
                f32x4 v[NI];
#pragma unroll
                for (int u = 0; u < NI; ++u) v[u] = *(const f32x4 *)(src[u] + ((size_t)yy * pw + cc) * 2 * C);
#pragma unroll
                for (int u = 0; u < NI; ++u) acc[u] += v[u];
            }
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int idx = i0 + 256 * u;
            if (idx >= total) break;
            const f32x4 v = acc[u] * inv_n;
            if (idx < nk) {
                const int r = idx / C4, c4 = idx % C4;
                *(f32x4 *)(Kt + (c4 * kRouteRS + r) * 4) = v;
            } else {
                const int row = (idx - nk) / C4, c4 = (idx - nk) % C4;
                *(f32x4 *)(Qs + row * QS + 4 * c4) = v;
            }
        }
    }
    __syncthreads();
    BRA_TRACE(1);
    route_rows_from_lds<C, NR>(Kt, Qs, b, myrt, D, Ir, Ar);
#ifdef BRA_EXPERIMENT
    if (tracing && Ar) {
        BRA_TRACE(2);
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long *o = (unsigned long long *)(Ar + ((size_t)b * D.R + QR * myrt) * D.R);
            for (int k = 0; k < 3; ++k) o[k] = trace_t[k];
        }
    }
#endif
#undef BRA_TRACE
}

// Routing from whole-region sums (the projection kernel ran over region tiles and left
// P[b R + r][2C] = [sum Q | sum K] over the tokens of region r): A^r = Q^r (K^r)^T (Eq. 4) with
// Q^r, K^r the sums divided by n (Sec. 3.2), and its row-wise top-k (Eq. 5).  Workgroup (b, rt)
// owns the 16 query regions 16 rt .. 16 rt + 15 of image b (R <= 64); wavefront w forms their
// affinities to the keys 16 w .. 16 w + 15 with float32 matrix-core products
// (v_mfma_f32_16x16x4_f32: lane 16 g + i holds A[row i][k g], B[k g][col i] and
// D[rows 4 g + j][col i]), its key operands loaded straight from P, the query rows (the same for the
// four wavefronts) through LDS, every request issued before the first product; the four 16 x 16
// blocks meet in LDS, then wavefront w ranks rows 4 w .. 4 w + 3.
template <int C>
__global__ __launch_bounds__(256) void k_route_w(const float *__restrict__ P, int32_t *__restrict__ Ir,
                                                 float *__restrict__ Ar, Dims D)
{
    __shared__ float At[16][65];
    __shared__ __attribute__((aligned(16))) float Qt[16][C + 4];      // the 16 query rows, shared by the wavefronts
    const int groups = (D.R + 15) / 16;
    const int wid = swizzled_block();          // the workgroups of an image share an XCD (and its L2)
    if (wid >= D.B * groups) return;
    const int b = wid / groups, myrt = wid % groups;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    // rows past R repeat the last region; their results are never used
    const float *ksrc = P + ((size_t)b * D.R + min(16 * wave + i, D.R - 1)) * 2 * C + C + 4 * g;
    constexpr int NQ = 16 * (C / 4) / 256;      // 16-byte chunks of the query rows per thread
    f32x4 qr[NQ], kv[C / 16];      // channels 16 s + 4 g + e: product e of step s contracts over {16 s + 4 g' + e}
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int idx = threadIdx.x + 256 * u, row = idx / (C / 4), c4 = idx % (C / 4);
        qr[u] = *(const f32x4 *)(P + ((size_t)b * D.R + min(16 * myrt + row, D.R - 1)) * 2 * C + 4 * c4);
    }
#pragma unroll
    for (int s = 0; s < C / 16; ++s) kv[s] = *(const f32x4 *)(ksrc + 16 * s);
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int idx = threadIdx.x + 256 * u;
        *(f32x4 *)&Qt[idx / (C / 4)][4 * (idx % (C / 4))] = qr[u];
    }
    __syncthreads();
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < C / 16; ++s) {
        const f32x4 qv = *(const f32x4 *)&Qt[i][16 * s + 4 * g];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qv[e], kv[s][e], acc, 0, 0, 0);
    }
    const float inv_n = 1.0f / (float)D.n, sc = inv_n * inv_n;
#pragma unroll
    for (int j = 0; j < 4; ++j) At[4 * g + j][16 * wave + i] = acc[j] * sc;
    __syncthreads();
    float a[4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) a[rr] = At[4 * wave + rr][lane];
    const int r0 = 16 * myrt + 4 * wave;
    if (r0 >= D.R) return;
    const int nrows = min(4, D.R - r0);
    const size_t row0 = (size_t)b * D.R + r0;
    if (Ar && lane < D.R) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            if (rr < nrows) Ar[(row0 + rr) * D.R + lane] = a[rr];
    }
    wave_topk_rows<4>(a, nrows, lane, D.R, D.k, Ir + row0 * D.k);
}

// LDS of the projection kernel: two X tiles (rows of C + 16 bf16), in whose place every wavefront
// first stages 64 rows of 32 RT + 8 bf16 of weights, then a table of 8 x 64 tokens.
template <int C, int WPB, int RT>
constexpr size_t kQkvTableOff = (size_t)2 * 64 * (C + 16) * 2 > (size_t)WPB * 64 * (32 * RT + 8) * 2
                                    ? (size_t)2 * 64 * (C + 16) * 2
                                    : (size_t)WPB * 64 * (32 * RT + 8) * 2;
template <int C, int WPB, int RT>
constexpr size_t kQkvSmem = kQkvTableOff<C, WPB, RT> + 8 * 64 * 4;

// How the projection kernel's tiles of 64 "slots" map to tokens.  Plain (region_tiles = 0): slot s is
// token s of the [B N] token list.  Region tiles (n divides 64, n <= 16): the slots run over the
// regions in the order (image, region), n slots per region in row-major order inside the region, so
// that a tile holds 64 / n whole regions and the sums over a region's tokens (Sec. 3.2: Q^r and K^r
// are per-region means) are formed inside one tile.
struct TileMap {
    int region_tiles;
    int sum_log2;       // accumulators are summed over aligned groups of 2^sum_log2 consecutive slots
    int map_log2;       // region tiles: log2 n (a region = 2^map_log2 consecutive slots); plain: 0
    int rw_log2;        // region tiles: log2 of the region width
    int R, S, rh, rw, W, N;
    int regions;        // region tiles: B R
};

// ---------------------------------------------------------------------------
// Q, K, V = X [Wq | Wk | Wv]  (Eq. 3; NMAT = 3), or a single projection such as Y = O Wo
// (Eq. 2; NMAT = 1, every output pointer the same).  Each wavefront owns 32 RT output channels of one
// of the NMAT matrices and keeps its weight fragments in registers; a workgroup is
// WPB such wavefronts (the column group of the workgroup selects which; a multiple of 4 per compute unit keeps its four
// SIMDs equally busy) and walks over `tiles_per_wg`
// consecutive tiles of 64 tokens (gx such workgroups; those before them route from pooled X, those
// after them rearrange the weights for the kernels that follow, when the launch carries such work).
// A tile of X is fetched once per workgroup with
// fully coalesced 16-byte loads (one tile ahead, held in registers while the current
// tile is computed), staged in LDS, and read from there as MFMA operands by all the
// wavefronts.  The product is formed transposed (rows = output channels, columns =
// tokens) with the weight rows permuted so that a lane ends up with 16 consecutive
// output channels of one token, i.e. one 32-byte store.
//
// Region pooling of Q and K (Sec. 3.2: Q^r, K^r are the per-region means of Q and K)
// rides along when P is given: the float32 accumulators of aligned groups of 2^sum_log2
// consecutive slots are summed across lanes before the rounding to bf16, and written as
// P[slot >> sum_log2][2C] = [sum Q | sum K].  With region tiles a group is a whole region and the
// routing kernel only divides by n; otherwise a group is min(rw, 4) consecutive tokens of one row of
// one region, and the routing kernel adds the few partial sums of each region.
template <int C, int WPB, int NMAT, int RT>
__global__ __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(C == 256 ? 2 : 3, 4)))
void k_qkv(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W, bf16_t *__restrict__ Q,
           bf16_t *__restrict__ K, bf16_t *__restrict__ V, float *__restrict__ P, TileMap tm, long M,
           int tiles_per_wg, int gx, PrepArgs prep, float qscale)
{
    constexpr int CH = C / 8, XP = C + 16, NTH = 64 * WPB;
    constexpr size_t kTableOff = kQkvTableOff<C, WPB, RT>;  // region tiles: first tokens of the regions of 8 tiles
    constexpr int NL = (64 * CH + NTH - 1) / NTH;       // 16-byte chunks of a tile per thread
    constexpr int CW = 32 * RT;                         // output channels of a wavefront
    constexpr int WP = CW + 8;                          // row pitch of a wavefront's weight staging tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *xs0 = (bf16_t *)smem;
    // The first workgroups route (a long chain of dependent steps: started first, it ends within the
    // projection), the last ones rearrange weights.
    if ((int)blockIdx.x < prep.route_items) {
        // wavefronts past the fourth leave: a barrier waits for the surviving ones only
        if (threadIdx.x < 256)
            route_body<C>(prep.Xr, prep.WT, prep.Ir, nullptr, prep.dims, smem, (int)blockIdx.x);
        return;
    }
    // GY workgroups (column groups of the outputs) share every token range.  The grid is one-dimensional
    // and consecutive workgroups go to the 8 XCDs in turn: the column groups of a range get numbers 8
    // apart, so that they run on one XCD at about the same time and the range's tokens are fetched
    // from memory once instead of GY times.
    constexpr int GY = NMAT * C / (32 * RT) / WPB;
    const int tw = (int)blockIdx.x - prep.route_items;
    if (tw >= gx * GY) {
        const int e = (tw - gx * GY) * NTH + (int)threadIdx.x;
        if (e < prep.elems)
            prep_weight_element(prep.Wqkv, prep.Wo, prep.Wlce, prep.WT, prep.WoT, prep.Wa, prep.Wf, C, e);
        return;
    }
    int bx = tw, by = 0;
    if (GY > 1) {
        const int first = tw / (8 * GY) * 8, within = tw % (8 * GY);
        const int ranges = gx - first < 8 ? gx - first : 8;       // the last group may hold fewer than 8 ranges
        by = within / ranges;
        bx = first + within % ranges;
    }
#ifdef BRA_EXPERIMENT
    unsigned long long trace_t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define BRA_TRACE(k) if (prep.trace) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    BRA_TRACE(0);
#ifdef BRA_EXPERIMENT
    const int smode = (prep.trace >> 3) & 3;
#else
    constexpr int smode = 0;
#endif
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int i = lane % 16;
    const int grp = by * WPB + wave;                    // channel group among NMAT C / CW
    const int sel = grp / (C / CW), base = (grp % (C / CW)) * CW;
    bf16_t *__restrict__ out = sel == 0 ? Q : (sel == 1 ? K : V);
    const int group_log2 = tm.sum_log2, group = 1 << group_log2;
    const long ntiles = (M + 63) / 64;
    const long tile0 = (long)bx * tiles_per_wg;
    const long tile1 = tile0 + tiles_per_wg < ntiles ? tile0 + tiles_per_wg : ntiles;
    // rbase[(tile - tile0) % 8][j] = first token of region j of the tile (plain: token of slot j).  The
    // entry of a tile is written (by the first 64 >> map_log2 threads) at least one barrier before its
    // first use; tiles past the workgroup's last repeat it, regions (tokens) past the last one repeat
    // that one.  Both modes look the token up: a branch between the matrix products and the first read
    // of their results is best avoided.
    int *rbase = (int *)(smem + kTableOff);
    auto table_entry = [&](long it) {
        const int rpt = 64 >> tm.map_log2;
        if ((int)threadIdx.x < rpt) {
            long tile = tile0 + it;
            if (tile > tile1 - 1) tile = tile1 - 1;
            long G = tile * rpt + (int)threadIdx.x;
            int first;
            if (tm.region_tiles) {
                if (G > tm.regions - 1) G = tm.regions - 1;
                const int b = (int)(G / tm.R), r = (int)(G - (long)b * tm.R);
                const int gy = r / tm.S, gx_ = r - gy * tm.S;
                first = b * tm.N + gy * tm.rh * tm.W + gx_ * tm.rw;
            } else {
                first = (int)(G < M ? G : M - 1);
            }
            rbase[(it & 7) * 64 + threadIdx.x] = first;
        }
    };

    // The products are v_mfma_f32_32x32x16_bf16 (twice the matrix-core rate of the 16x16x32 form on
    // this chip): lane l = 32 h + c holds A[row c][k 8 h ..], B[k 8 h ..][col c] and
    // D[rows 8 q + 4 h + j][col c] in result register 4 q + j.
    // This wavefront's weight slice W[:, sel C + base .. + CW - 1] (row-major [C][NMAT C], as the
    // caller holds it) -> A fragments with permuted rows (row 8 q + 4 h' + j of a 32-row tile is
    // output channel 16 (q / 2) + 8 h' + 4 (q % 2) + j, so that a lane's results 0 .. 7 and 8 .. 15 are
    // 8 consecutive channels each and the two half-waves together write 32 contiguous bytes of a
    // token per store): 64 input channels at a time are copied with coalesced loads into a
    // wavefront-private LDS tile and come back through the transposing read (lane s of a 16-lane
    // group supplies the address of 4 columns of row s / 4, lane i receives column i % 4 of the
    // chunk that the lanes s % 4 == i / 4 named, for rows 0 .. 3).  LDS operations of one
    // wavefront complete in order, so no barrier is needed between its own writes and reads.
    constexpr int KST = C / 16;                           // contraction steps
    const int h = lane / 32, c32 = lane % 32;
    bf16x8 af[RT][KST];

    constexpr int ND = C >= 256 ? 1 : (NL <= 3 ? 4 : 2);     // tiles on their way in registers (a tile's X takes about five tiles' arithmetic to arrive)
    if (tile0 >= tile1) return;
    for (int it = 0; it < ND + 2; ++it) table_entry(it);
    __syncthreads();
    // Requests and stores are laid out so that the wait for a tile's X leaves the stores of the tile
    // before it pending: every tile of the main loop stores unconditionally (a ragged last tile is
    // handled after the loop), and every iteration requests a tile (past the end: the last one again).
    u32x4 xr[ND][NL];
    // slot q of a tile: region q >> sum_log2 of the tile, token (row, column) of the region
    auto in_region = [&](int q) {
        const int e = q & ((1 << tm.map_log2) - 1);
        return (e >> tm.rw_log2) * tm.W + (e & ((1 << tm.rw_log2) - 1));
    };
    int f_reg[NL], f_off[NL];                             // region tiles: where this thread's chunks of a tile come from
#pragma unroll
    for (int u = 0; u < NL; ++u) {
        const int q = min((int)threadIdx.x + NTH * u, 64 * CH - 1) / CH;
        f_reg[u] = q >> tm.map_log2;
        f_off[u] = in_region(q);
    }
    auto fetch = [&](long tile, u32x4 (&r)[NL]) {      // rows past M repeat the last token; their results are not stored
        const int it = (int)(tile - tile0);
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int idx = min((int)threadIdx.x + NTH * u, 64 * CH - 1);
            const long t = rbase[(it & 7) * 64 + f_reg[u]] + f_off[u];
            r[u] = *(const u32x4 *)(X + t * C + (idx % CH) * 8);
        }
    };
    auto stage = [&](int b, const u32x4 (&r)[NL]) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int idx = threadIdx.x + NTH * u;
            if (idx < 64 * CH) *(u32x4 *)(xs0 + (b * 64 + idx / CH) * XP + (idx % CH) * 8) = r[u];
        }
    };
    // one tile of 64 tokens from buffer `cur`; FULL: all its tokens exist
    auto project = [&](long tile, int cur, auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
            f32x16 acc[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[rt][e] = 0.f;
            const bf16_t *xrow = xs0 + (cur * 64 + 32 * ct + c32) * XP + 8 * h;
#pragma unroll
            for (int kst = 0; kst < KST; ++kst) {
                const bf16x8 bfr = *(const bf16x8 *)(xrow + 16 * kst);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[rt] = mfma32(af[rt][kst], bfr, acc[rt]);
            }
            // The results are first read on the far side of a branch: the wait that this takes
            // (11 idle issue slots after an 8-pass product) is spelled out here, where no branch
            // lies between.
            __builtin_amdgcn_sched_barrier(0);
            asm volatile("s_nop 11");
            __builtin_amdgcn_sched_barrier(0);
            const long slot = tile * 64 + 32 * ct + c32;
            const long t = rbase[((int)(tile - tile0) & 7) * 64 + ((32 * ct + c32) >> tm.map_log2)] + in_region(32 * ct + c32);
            if ((FULL || slot < M) && !(prep.trace & 2)) {
                // Q may leave multiplied by a factor (the attention kernel that wants its scores in
                // units of log2 passes scale * log2 e): one rounding, of the scaled value
                auto put = [&](float os) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        u32x4 *dst = (u32x4 *)(out + t * C + base + 32 * rt + 8 * h);
                        const u32x4 lo = {pack_bf16(acc[rt][0] * os, acc[rt][1] * os), pack_bf16(acc[rt][2] * os, acc[rt][3] * os),
                                          pack_bf16(acc[rt][4] * os, acc[rt][5] * os), pack_bf16(acc[rt][6] * os, acc[rt][7] * os)};
                        const u32x4 hi = {pack_bf16(acc[rt][8] * os, acc[rt][9] * os), pack_bf16(acc[rt][10] * os, acc[rt][11] * os),
                                          pack_bf16(acc[rt][12] * os, acc[rt][13] * os), pack_bf16(acc[rt][14] * os, acc[rt][15] * os)};
                        if (smode == 1) { store16<1>(dst, lo); store16<1>(dst + 2, hi); }
                        else if (smode == 2) { store16<2>(dst, lo); store16<2>(dst + 2, hi); }
                        else { store16<0>(dst, lo); store16<0>(dst + 2, hi); }
                    }
                };
                if (sel == 0 && qscale != 1.0f) put(qscale);
                else put(1.0f);      // a constant: no multiplication is left
            }
            if (P && sel < 2) {      // M is a multiple of the group: a group is whole or absent
                // one branch around the whole sum, not one per element
                if (group_log2 >= 2) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            acc[rt][e] = dpp_fadd<0x4E>(dpp_fadd<0xB1>(acc[rt][e]));      // quad_perm [1,0,3,2], then [2,3,0,1]
                    if (group_log2 >= 3) {
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                            for (int e = 0; e < 16; ++e) acc[rt][e] = dpp_fadd<0x141>(acc[rt][e]);      // row_half_mirror: the other quad of 8 lanes
                    }
                    if (group_log2 >= 4) {
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                            for (int e = 0; e < 16; ++e) acc[rt][e] = dpp_fadd<0x140>(acc[rt][e]);      // row_mirror: the other half of 16 lanes
                    }
                } else if (group_log2 == 1) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[rt][e] = dpp_fadd<0xB1>(acc[rt][e]);
                }
                if ((FULL || slot < M) && (c32 & (group - 1)) == 0 && !(prep.trace & 4)) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        f32x4 *dst = (f32x4 *)(P + (slot >> group_log2) * 2 * C + sel * C + base + 32 * rt + 8 * h);
#pragma unroll
                        for (int q4 = 0; q4 < 4; ++q4) {
                            const f32x4 pv = {acc[rt][4 * q4], acc[rt][4 * q4 + 1], acc[rt][4 * q4 + 2], acc[rt][4 * q4 + 3]};
                            const u32x4 pu = __builtin_bit_cast(u32x4, pv);
                            f32x4 *d4 = dst + q4 + 2 * (q4 / 2);      // results 8 .. 15: 16 channels on
                            if (smode == 1) store16<1>(d4, pu);
                            else if (smode == 2) store16<2>(d4, pu);
                            else store16<0>(d4, pu);
                        }
                    }
                }
            }
        }
    };
    // Tile tile0 + j travels in register set j % ND.  Every round requests a tile and hands one to
    // LDS, whether or not it exists (past the end: the last tile again, into a buffer nobody reads).
#pragma unroll
    for (int d = 0; d < ND; ++d) fetch(tile0 + d, xr[d]);
    // the weight fragments, while the first tiles are on their way
    {
        bf16_t *wb = (bf16_t *)smem + wave * 64 * WP;      // in the X tiles' place: they are staged afterwards
        const bf16_t *wsrc = W + sel * C + base;
        const int gg = c32 / 16;
#pragma unroll
        for (int kc = 0; kc < C / 64; ++kc) {
            constexpr int WCH = CW / 8;                  // 16-byte chunks of a staged row
            u32x4 wr[WCH];
#pragma unroll
            for (int u = 0; u < WCH; ++u) {
                const int idx = lane + 64 * u;
                wr[u] = *(const u32x4 *)(wsrc + (size_t)(64 * kc + idx / WCH) * (NMAT * C) + (idx % WCH) * 8);
            }
#pragma unroll
            for (int u = 0; u < WCH; ++u) {
                const int idx = lane + 64 * u;
                *(u32x4 *)(wb + (idx / WCH) * WP + (idx % WCH) * 8) = wr[u];
            }
#pragma unroll
            for (int kl = 0; kl < 4; ++kl)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const bf16_t *src = wb + (16 * kl + 8 * h + i / 4) * WP + 32 * rt + 16 * gg + 8 * ((i % 4) % 2) +
                                        4 * ((i % 4) / 2);
                    const s16x4 v0 = lds_read_tr16(src), v1 = lds_read_tr16(src + 4 * WP);
                    const u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
                    const u32x4 av = {a0[0], a0[1], a1[0], a1[1]};
                    af[rt][4 * kc + kl] = __builtin_bit_cast(bf16x8, av);
                }
        }
    }
    __syncthreads();                                       // every wavefront has its fragments: the X tiles may take the weights' place
    BRA_TRACE(1);
    stage(0, xr[0]);
    fetch(tile0 + ND, xr[0]);
    __syncthreads();
    BRA_TRACE(2);
    const long tfull = tile1 * 64 <= M ? tile1 : tile1 - 1;      // tiles below this one are full
    for (long base_tile = tile0; base_tile < tfull; base_tile += ND) {
#pragma unroll
        for (int d = 0; d < ND; ++d) {
            const long tile = base_tile + d;
            const int cur = (int)((tile - tile0) & 1);
            if (tile < tfull) project(tile, cur, std::true_type{});
            stage(cur ^ 1, xr[(d + 1) % ND]);      // the other buffer was last read before the previous barrier
            fetch(tile + 1 + ND, xr[(d + 1) % ND]);
            table_entry(tile - tile0 + ND + 2);
            __syncthreads();
            if (tile == tile0) BRA_TRACE(3);
        }
    }
    const int cur = (int)((tfull - tile0) & 1);
    if (tfull < tile1) project(tfull, cur, std::false_type{});
#ifdef BRA_EXPERIMENT
    if (prep.trace) {
        BRA_TRACE(4);
        __syncthreads();
        if (threadIdx.x == 0 && by == 0) {
            unsigned long long *o = (unsigned long long *)(Q + tile0 * 64 * C);
            for (int k = 0; k < 5; ++k) o[k] = trace_t[k];
            o[5] = (unsigned long long)(tile1 - tile0);
        }
    }
#endif
#undef BRA_TRACE
}

// ---------------------------------------------------------------------------
// LDS map of the staged attention kernel.  Rows of bf16 tiles have CS = C + 16 elements
// (a pitch of 32 bytes x odd: full rate for the 16-byte operand reads and the transposing
// reads), rows of the float32 output tile OS.
template <int C>
struct AttnSmem {
    static constexpr int CS = C + 16;
    static constexpr int OS = C + 4;
    static constexpr size_t k_off = 0;                                // K tile; output tile later
    static constexpr size_t v_off = k_off + (size_t)64 * CS * 2;      // V tile (fused: Q tile first)
    static constexpr size_t w_off = v_off + (size_t)64 * CS * 2;      // LCE weights [25][C] f32
    static constexpr size_t h_off = w_off + (size_t)25 * C * 4;       // V halo tile
    static size_t bytes(int halo_rows) { return h_off + (size_t)halo_rows * CS * 2; }
};

// Routed attention + LCE + W^o for regions of n >= 64 tokens (Eq. 6-7, Eq. 2).
// One workgroup = 64 query tokens (64/rw full rows of one region), all heads; wavefront
// w % 4 owns queries 16 (w % 4) .. + 15.  Keys and values of the k routed regions are copied
// by index, 64 tokens at a time, from the projected maps into LDS; one online softmax runs
// over all k n keys.
// HG = 1: 4 wavefronts, each with all heads.  HG = 2 (C = 64): 8 wavefronts, group w / 4 takes
// half of the heads over the same staged key blocks and, at the end, half of the output
// channels of W^o: twice the wavefronts per compute unit when there are few workgroups.
template <int C, int HG = 1>
__global__ __launch_bounds__(256 * HG) __attribute__((amdgpu_waves_per_eu(2, 2 + HG)))
void k_attn_big(AttnArgs A, Dims D)
{
    typedef AttnSmem<C> SM;
    static_assert(HG == 1 || C == 64, "head groups are laid out for two heads");
    constexpr int CS = SM::CS, OS = SM::OS, HEADS = C / 32, HPG = HEADS / HG, KS = C / 32, CH = C / 8;
    constexpr int NT = 256 * HG;
    constexpr int NBT = 64 * CH / NT;           // 16-byte chunks per thread for a 64-row tile
    constexpr int NBH = 5;                      // halo chunks per thread and batch
    constexpr bool kPrefetchWo = (C == 64);
    constexpr int NWT = 4 / HG;                 // W^o tiles of a wavefront (C == 64)
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)(smem + SM::k_off);
    bf16_t *Vs = (bf16_t *)(smem + SM::v_off);
    float *Wl = (float *)(smem + SM::w_off);
    bf16_t *Hs = (bf16_t *)(smem + SM::h_off);
    float *Os = (float *)(smem + SM::k_off);   // reuses the K/V tiles after the key loop

    const int wid = swizzled_block();
    if (wid >= A.total) return;

    const int wave = (threadIdx.x / kWave) % 4, hg = threadIdx.x / (4 * kWave), lane = threadIdx.x % kWave;
    const int h0 = hg * HPG;
    const int g = lane / 16, i = lane % 16;
    const int chunks = D.n / 64;               // query tiles per region
    const int qh = 64 / D.rw;                  // rows per query tile
    const int b = wid / (D.R * chunks);
    const int reg = (wid / chunks) % D.R;
    const int ch = wid % chunks;
    const float s_inv = 1.0f / (float)D.S;
    const int regy = fast_div(reg, s_inv);
    const int y0 = regy * D.rh + ch * qh, x0 = (reg - regy * D.S) * D.rw;
    const size_t img_off = (size_t)b * D.N * C;
    const int hw = D.rw + 4, hrows = (qh + 4) * hw;
    const float hw_inv = 1.0f / (float)hw, rw_inv = 1.0f / (float)D.rw;

    // Everything that does not depend on the routing is requested first: V halo, LCE
    // weights, this lane's query fragments and (small C) the W^o fragments.
    u32x4 hreg[NBH];
    tile_load<C, NBH, NT>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, 0);
    LceWeights<C> lw;
    lw.load(A.Wlce);
    const int q = 16 * wave + i;
    const int qy = fast_div(q, rw_inv);
    const size_t qtok = (size_t)(y0 + qy) * D.W + x0 + q - qy * D.rw;
    bf16x8 qf[HPG];
#pragma unroll
    for (int h = 0; h < HPG; ++h) qf[h] = *(const bf16x8 *)(A.Q + img_off + qtok * C + 32 * (h0 + h) + 8 * g);
    bf16x8 wof[kPrefetchWo ? NWT : 1][KS];
    if constexpr (kPrefetchWo) {
#pragma unroll
        for (int tt = 0; tt < NWT; ++tt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wof[tt][ks] = wo_fragment<C>(A.WoT, 0, NWT * hg + tt, ks, g, i);
    }

    // Routing row of this region.
    const int32_t *irp = A.Ir_src + ((size_t)b * D.R + reg) * D.k;
    if (A.Ir_out && A.Ir_out != A.Ir_src && ch == 0)
        for (int p = threadIdx.x; p < D.k; p += NT) A.Ir_out[((size_t)b * D.R + reg) * D.k + p] = irp[p];

    tile_store<C, CS, NBH, NT>(Hs, hreg, hrows, 0);
    for (int first = NT * NBH; first < hrows * CH; first += NT * NBH) {
        tile_load<C, NBH, NT>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, first);
        tile_store<C, CS, NBH, NT>(Hs, hreg, hrows, first);
    }
    lw.store(Wl);

    SoftmaxState<HPG> st;
    st.init();
    const int nblocks = D.kn / 64;
    // K / V blocks of 64 routed tokens: the next block is requested as soon as the current
    // one has been handed to LDS, so that its latency hides behind the current block's work.
    u32x4 kreg[NBT], vreg[NBT];
    auto request = [&](int kb) {
        const int j = region_index(irp[kb / chunks], D.R);
        const int jy = fast_div(j, s_inv);
        const int ky0 = jy * D.rh + (kb % chunks) * qh, kx0 = (j - jy * D.S) * D.rw;
        tile_load<C, NBT, NT>(kreg, A.K + img_off, ky0, kx0, D.rw, rw_inv, 64, D.H, D.W, 0);
        tile_load<C, NBT, NT>(vreg, A.V + img_off, ky0, kx0, D.rw, rw_inv, 64, D.H, D.W, 0);
    };
    request(0);
    for (int kb = 0; kb < nblocks; ++kb) {
        __syncthreads();   // the previous block's readers are done with Ks / Vs
        tile_store<C, CS, NBT, NT>(Ks, kreg, 64, 0);
        tile_store<C, CS, NBT, NT>(Vs, vreg, 64, 0);
        if (kb + 1 < nblocks) request(kb + 1);
        __syncthreads();
        attn_key_block<C, CS, HPG>(Ks, Vs, qf, st, A.c_exp, g, i, h0);
    }
    __builtin_amdgcn_s_setprio(2);      // late phases first: the workgroup's LDS is freed sooner
    __syncthreads();   // everyone is done with Ks / Vs: the output tile may overwrite them
    attn_write_out<C, OS, HPG>(Os, st, wave, g, i, h0);
    __syncthreads();
    lce_add_valu<C, CS, OS, NT>(Hs, Wl, Os, qh, D.rw, hw);
    __syncthreads();
    if constexpr (HG == 1) {
        wo_project_store<C, OS, kPrefetchWo>(Os, kPrefetchWo ? wof : nullptr, A.WoT,
                                             A.Y + img_off + qtok * C, wave, g, i);
    } else {
        // group hg forms tiles NWT hg .. of Y^T = Wo^T O^T: 8 of this lane's 16 output channels
        bf16x8 of[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float *src = Os + (16 * wave + i) * OS + 32 * ks + 8 * g;
            const f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
            const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            of[ks] = pack8(v);
        }
        u32x2 yp[NWT];
#pragma unroll
        for (int tt = 0; tt < NWT; ++tt) {
            f32x4 ya = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) ya = mfma16(wof[tt][ks], of[ks], ya);
            yp[tt] = pack4(ya);
        }
        u32x4 *dst = (u32x4 *)(A.Y + img_off + qtok * C + 16 * g);
        dst[hg] = u32x4{yp[0][0], yp[0][1], yp[1][0], yp[1][1]};
    }
}

// ---------------------------------------------------------------------------
// Fused forward for one 64-token query tile whose region attends to a single
// 64-token key block (the k = 1 stage), C = 64: Q, the routed K / V and the V halo
// needed by the LCE are projected from X inside the workgroup (Eq. 3), so Q, K, V never
// travel through memory.  X tiles are staged once through LDS.
//
// Work split over the four wavefronts: see the kernel's own comment.
//   * LCE (Eq. 7) runs on the matrix cores.  The V halo of a wavefront's channels is
//     stored channel-major (a plane of halo tokens per channel) and the 5x5 depth-wise
//     correlation of one channel is a chain of v_mfma_f32_4x4x4_16B_bf16 products:
//     block = channel, D[xi][yj] = out[y0 + yj][x0 + xi], and for every (ky, half hh)
//       A[xi][k] = w[ky][4 hh + k - xi] (zero outside 0..4),
//       B[k][yj] = V[y0 + yj + ky][x0 + 4 hh + k]            (halo coordinates).
//     4x4x4 lane layout: block l / 4; A row, B / D column l % 4.  The result goes to
//     LDS as a float32 tile [channel][query] and is added to the attention output in
//     registers by the wavefront that owns the query.
//
// LDS row pitches are chosen per access pattern (measured on gfx950): rows read with
// the transposing read are fastest at 160 bytes, rows read 8 bytes per lane at 144 bytes,
// the planes (8-byte reads, lane = channel x row offset) at a pitch of 8 x odd words.
// The X tiles (16-byte reads) would also like 160 bytes; at 144 bytes the whole map takes 40 KB and
// three workgroups share a compute unit.  (A fourth needs 36 KB or less and at most 120 registers:
// built with an unpadded, swizzled halo tile, it was measured no faster.)
template <int RW>
struct FusedSmem {
    static constexpr int C = 64;
    static constexpr int XS = C + 8;                                  // X tiles
    static constexpr int KP = C + 8;                                  // K tile
    static constexpr int VP = C + 16;                                 // V tile
    static constexpr int PL = 68;                                     // LCE tile: floats per channel
    static constexpr int QH = 64 / RW;                                // rows of the query tile
    static constexpr int HW = RW + 4, HROWS = (QH + 4) * HW;          // halo tile
    static constexpr int NHT = (HROWS + 15) / 16;                     // 16-token tiles of the halo
    static constexpr int PSW = (NHT % 2) ? NHT * 8 : NHT * 8 + 8;     // plane pitch in 32-bit words
    static constexpr int PS = 2 * PSW;
    static constexpr size_t k_off = 0;                                // routed X tile -> K tile
    static constexpr size_t v_off = k_off + (size_t)64 * XS * 2;      // V tile
    static constexpr size_t l_off = 0;                                // LCE tile, over K and V
    static constexpr size_t h_off = v_off + (size_t)64 * VP * 2;      // X halo -> V halo planes
    static constexpr size_t xh_bytes = (size_t)NHT * 16 * XS * 2;
    static constexpr size_t vt_bytes = (size_t)C * PS * 2;
    static constexpr size_t r_off = h_off + (xh_bytes > vt_bytes ? xh_bytes : vt_bytes);   // routing: 8 words
    static constexpr size_t bytes = r_off + 32;
    static_assert(KP <= XS && (size_t)C * PL * 4 <= h_off, "tiles that share a slot must fit");
};

// The products are v_mfma_f32_32x32x16_bf16 (twice the matrix-core rate of the 16x16x32 form
// on this chip, and half the LDS operand bytes per flop): lane l = 32 h + c holds A[row c][k 8 h ..],
// B[k 8 h ..][col c] and D[rows 8 q + 4 h + j][col c] in result register 4 q + j.
// Wavefront w = (th = w % 2, ch = w / 2).  Projections are formed transposed (rows = output
// channels ch-th half = head ch, columns = tokens th-th half) from ready-made weight fragments (a
// table the weight-prep blocks write: one coalesced 16-byte load per lane and contraction step;
// the same rows taken straight from the transposed weights, 32 scattered rows per load, cost 15 us
// per launch), with the rows permuted so that
// result registers 0 .. 7 and 8 .. 15 of a lane are the channels 8 h .. + 7 and 16 + 8 h .. + 7 of
// its token: exactly the two B operands that the next product wants, so Q feeds S^T = K Q^T and
// O feeds W^o without leaving the registers of a lane.  Attention: wavefront = (head ch, queries
// of half th); a lane of S^T holds 32 of its query's 64 scores (the other half sits in lane
// l ^ 32), and result registers 8 qq .. 8 qq + 7 of key tile t are the B operand of
// O^T += V^T P^T for the keys 32 t + 16 qq + {4 h .. + 3, 8 + 4 h .. + 3}, which is also what the two
// transposing reads of V deliver.  The V halo is projected with the operands swapped (rows =
// halo tokens), 4 consecutive tokens of a channel per register group, into channel-major planes;
// the LCE runs on them as described above.
template <int RW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void k_fused(AttnArgs A, Dims D)
{
    typedef FusedSmem<RW> SM;
    constexpr int C = 64, CH = C / 8, KST = C / 16;
    constexpr int XS = SM::XS, KP = SM::KP, VP = SM::VP, PL = SM::PL;
    constexpr int QH = SM::QH, HW = SM::HW, HROWS = SM::HROWS, NHT = SM::NHT, PS = SM::PS;
    constexpr int NBH = (HROWS * CH + 255) / 256;      // halo chunks per thread
    constexpr int NBT = CH / 4;                 // chunks per thread of a 64-row tile
    constexpr int NYB = QH / 4, NXB = RW / 4;   // 4x4 output blocks of the query tile
    constexpr int NT32 = (HROWS + 31) / 32;     // 32-token tiles of the halo
    constexpr int OP = C + 8;                   // row pitch of the O tile
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)(smem + SM::k_off);   // first the routed X tile
    bf16_t *Vs = (bf16_t *)(smem + SM::v_off);
    bf16_t *Hs = (bf16_t *)(smem + SM::h_off);   // first the X halo tile, then the V planes, then O
    float *Ls = (float *)(smem + SM::l_off);
    static_assert((size_t)64 * OP * 2 <= SM::bytes - SM::h_off, "the O tile takes the planes' place");

    const int wid = swizzled_block();
    if (wid >= A.total) return;
#ifdef BRA_EXPERIMENT
    unsigned long long trace_t[8];
#define BRA_TRACE(k) if (A.trace) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    BRA_TRACE(0);

    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int h = lane / 32, c32 = lane % 32, i = lane % 16, gg = c32 / 16;
    const int th = wave % 2, chh = wave / 2;
    const int b = wid / D.R, reg = wid % D.R;
    const float s_inv = 1.0f / (float)D.S;
    const int regy = fast_div(reg, s_inv);
    const int y0 = regy * D.rh, x0 = (reg - regy * D.S) * RW;
    const size_t img_off = (size_t)b * D.N * C;
    const bf16_t *Ximg = A.X + img_off;
    const float hw_inv = 1.0f / (float)HW, rw_inv = 1.0f / (float)RW;

    // All requests up front: the routed region, X over the halo of the query tile (it contains the
    // query tile) and over the routed region, the weight fragments.  The routed region: given, or
    // found here from this region's row of A^r; the requests for that row go first, so that they are
    // back before the tiles.
    const size_t rrow = (size_t)b * D.R + reg;
    RouteRowLoads rl;
    int j = 0;
    int j_given = 0;            // reported as given, used clamped
    if (A.Ir_src) {
        j_given = A.Ir_src[rrow];
        j = region_index(j_given, D.R);
    }
    else route_row_load(A.Xr + (size_t)b * D.R * C, A.U + rrow * C, D.R, rl);
    u32x4 hreg[NBH];
    tile_load<C, NBH>(hreg, Ximg, y0 - 2, x0 - 2, HW, hw_inv, HROWS, D.H, D.W, 0);
    if (!A.Ir_src) j = route_row_k1(rl, D.R, (uint32_t *)(smem + SM::r_off), nullptr);
    BRA_TRACE(1);
    // weight rows: result row c of a 32-row tile is output channel prow of the tile
    // (ready-made fragments: one coalesced 16-byte load per lane each)
    auto fragment = [&](int tile, int kst) {
#ifdef BRA_EXPERIMENT
        if (A.trace & 4) {      // ablation: no weight traffic (wrong results)
            const u32x4 c = {0x3c003c00u + (unsigned)tile, 0x3c003c00u, 0x3c003c00u + (unsigned)kst, 0x3c003c00u};
            return __builtin_bit_cast(bf16x8, c);
        }
#endif
        return *(const bf16x8 *)(A.Wf + ((size_t)(tile * KST + kst) * kWave + lane) * 8);
    };
    bf16x8 wq[KST], wk[KST], wv[KST], wvb[KST];
#pragma unroll
    for (int kst = 0; kst < KST; ++kst) {
        wq[kst] = fragment(chh, kst);
        wk[kst] = fragment(2 + chh, kst);
        wv[kst] = fragment(4 + chh, kst);
        wvb[kst] = fragment(6 + th, kst);      // as a B operand: column c
    }
    u32x4 kreg[NBT];
    const int jy = fast_div(j, s_inv);
    tile_load<C, NBT>(kreg, Ximg, jy * D.rh, (j - jy * D.S) * RW, RW, rw_inv, 64, D.H, D.W, 0);
    tile_store<C, XS, NBH>(Hs, hreg, HROWS, 0);
    tile_store<C, XS, NBT>(Ks, kreg, 64, 0);
    __syncthreads();
    BRA_TRACE(2);

    // Q of head chh for the queries 32 th .. + 31, kept as the B operands of S^T = K Q^T
    const int q = 32 * th + c32;
    const int qy = fast_div(q, rw_inv);
    bf16x8 qb[2];
    {
        const bf16_t *xq = Hs + ((qy + 2) * HW + q - qy * RW + 2) * XS + 8 * h;   // query token in the halo
        f32x16 a;
#pragma unroll
        for (int e = 0; e < 16; ++e) a[e] = 0.f;
#pragma unroll
        for (int kst = 0; kst < KST; ++kst) a = mfma32(wq[kst], *(const bf16x8 *)(xq + 16 * kst), a);
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = a[e];
        qb[0] = pack8(v);
        qb[1] = pack8(v + 8);
    }
    // K, V of the routed tokens 32 th .. + 31, channels of half chh
    bf16x8 kp[2], vp[2];
    {
        const bf16_t *xk = Ks + (32 * th + c32) * XS + 8 * h;
        f32x16 ka, va;
#pragma unroll
        for (int e = 0; e < 16; ++e) ka[e] = va[e] = 0.f;
#pragma unroll
        for (int kst = 0; kst < KST; ++kst) {
            const bf16x8 bk = *(const bf16x8 *)(xk + 16 * kst);
            ka = mfma32(wk[kst], bk, ka);
            va = mfma32(wv[kst], bk, va);
        }
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = ka[e];
        kp[0] = pack8(v);
        kp[1] = pack8(v + 8);
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = va[e];
        vp[0] = pack8(v);
        vp[1] = pack8(v + 8);
    }
    // V halo: tasks (32-token tile T, channel half th), operands swapped: D[token 8 q + 4 h + j][channel c]
    constexpr int NHU = (2 * NT32 + 3) / 4;
    u32x2 vh[NHU][4];
#pragma unroll
    for (int u = 0; u < NHU; ++u) {
        const int T = chh + 2 * u;      // task wave + 4 u = (T, th)
        if (T < NT32) {
            const bf16_t *xh = Hs + min(32 * T + c32, HROWS - 1) * XS + 8 * h;   // rows past the halo repeat the last one; never used
            f32x16 a;
#pragma unroll
            for (int e = 0; e < 16; ++e) a[e] = 0.f;
#pragma unroll
            for (int kst = 0; kst < KST; ++kst) a = mfma32(*(const bf16x8 *)(xh + 16 * kst), wvb[kst], a);
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) vh[u][qq] = pack4(f32x4{a[4 * qq], a[4 * qq + 1], a[4 * qq + 2], a[4 * qq + 3]});
        }
    }
    __syncthreads();   // every X tile has been read
    BRA_TRACE(3);
    {
        bf16_t *kd = Ks + (32 * th + c32) * KP + 32 * chh + 8 * h, *vd = Vs + (32 * th + c32) * VP + 32 * chh + 8 * h;
        *(bf16x8 *)kd = kp[0];
        *(bf16x8 *)(kd + 16) = kp[1];
        *(bf16x8 *)vd = vp[0];
        *(bf16x8 *)(vd + 16) = vp[1];
        bf16_t *plane = Hs + (32 * th + c32) * PS;      // plane of channel 32 th + c
#pragma unroll
        for (int u = 0; u < NHU; ++u) {
            const int T = chh + 2 * u;
            if (T < NT32) {
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int tok = 32 * T + 8 * qq + 4 * h;
                    if (tok < NHT * 16) *(u32x2 *)(plane + tok) = vh[u][qq];
                }
            }
        }
    }
    __syncthreads();
    __builtin_amdgcn_s_setprio(2);
    BRA_TRACE(4);
    // W^o rows (out channels of half chh) and the LCE operands: requested now, used after the attention
    bf16x8 wo[KST];
#pragma unroll
    for (int kst = 0; kst < KST; ++kst) wo[kst] = fragment(8 + chh, kst);
    const int lb = lane / 4, xi = lane % 4;      // LCE: lane = (channel of the wavefront's 16, output row offset)
    s16x4 aw[5][2];
#pragma unroll
    for (int r = 0; r < 10; ++r)
        aw[r / 2][r % 2] = *(const s16x4 *)(A.Wa + ((size_t)(wave * 10 + r) * kWave + lane) * 4);

    // attention of head chh, queries 32 th .. + 31, over the 64 keys (Eq. 1 with one routed block)
    float p[32];
    {
        f32x16 s0, s1;
#pragma unroll
        for (int e = 0; e < 16; ++e) s0[e] = s1[e] = 0.f;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16_t *kr = Ks + c32 * KP + 32 * chh + 16 * s + 8 * h;
            s0 = mfma32(*(const bf16x8 *)kr, qb[s], s0);
            s1 = mfma32(*(const bf16x8 *)(kr + 32 * KP), qb[s], s1);
        }
        float m = s0[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) m = fmaxf(m, s0[e]);
#pragma unroll
        for (int e = 0; e < 16; ++e) m = fmaxf(m, s1[e]);
        m = fmaxf(m, __shfl_xor(m, 32));
        const float mc = m * A.c_exp;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(s0[e], A.c_exp, -mc));
            p[16 + e] = __builtin_amdgcn_exp2f(fmaf(s1[e], A.c_exp, -mc));
        }
    }
    float lsum = 0.f;
#pragma unroll
    for (int e = 0; e < 32; ++e) lsum += p[e];
    lsum += __shfl_xor(lsum, 32);
    f32x16 oacc;
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[e] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int qq = 0; qq < 2; ++qq) {
            const bf16_t *src = Vs + (32 * t + 16 * qq + 4 * h + i / 4) * VP + 32 * chh + 16 * gg + 8 * ((i % 4) % 2) +
                                4 * ((i % 4) / 2);
            const u32x2 v0 = __builtin_bit_cast(u32x2, lds_read_tr16(src));
            const u32x2 v1 = __builtin_bit_cast(u32x2, lds_read_tr16(src + 8 * VP));
            const bf16x8 vf = __builtin_bit_cast(bf16x8, u32x4{v0[0], v0[1], v1[0], v1[1]});
            oacc = mfma32(vf, pack8(p + 16 * t + 8 * qq), oacc);
        }
    const float inv = 1.0f / lsum;

    // LCE of this wavefront's 16 channels from its halo planes: lane = (channel lb, output row offset xi)
    f32x4 lce[NYB][NXB];
    {
        const bf16_t *plane = Hs + (16 * wave + lb) * PS;
#pragma unroll
        for (int yb = 0; yb < NYB; ++yb) {
#pragma unroll
            for (int xb = 0; xb < NXB; ++xb) lce[yb][xb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                const bf16_t *row = plane + (4 * yb + xi + ky) * HW;   // halo row of output row 4 yb + yj
                s16x4 br[NXB + 1];
#pragma unroll
                for (int xb = 0; xb <= NXB; ++xb) br[xb] = *(const s16x4 *)(row + 4 * xb);
#pragma unroll
                for (int xb = 0; xb < NXB; ++xb) {
                    lce[yb][xb] = mfma4(aw[ky][0], br[xb], lce[yb][xb]);
                    lce[yb][xb] = mfma4(aw[ky][1], br[xb + 1], lce[yb][xb]);
                }
            }
        }
    }
    BRA_TRACE(5);
    __syncthreads();   // K, V and the planes have been read: the LCE tile and the O tile may take their place
#pragma unroll
    for (int yb = 0; yb < NYB; ++yb)
#pragma unroll
        for (int xb = 0; xb < NXB; ++xb)   // queries (row 4 yb + yj, columns 4 xb ..) of channel 16 w + lb
            *(f32x4 *)(Ls + (16 * wave + lb) * PL + (4 * yb + xi) * RW + 4 * xb) = lce[yb][xb];
    __syncthreads();
    BRA_TRACE(6);
    // O = attention + LCE (Eq. 2, 7), rounded once, into the O tile [query][channel]
    {
        float v[16];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            v[e] = fmaf(oacc[e], inv, Ls[(32 * chh + 8 * h + e) * PL + q]);
            v[8 + e] = fmaf(oacc[8 + e], inv, Ls[(32 * chh + 16 + 8 * h + e) * PL + q]);
        }
        bf16_t *od = Hs + q * OP + 32 * chh + 8 * h;
        *(bf16x8 *)od = pack8(v);
        *(bf16x8 *)(od + 16) = pack8(v + 8);
    }
    __syncthreads();
    // Y^T = Wo^T O^T: out channels of half chh, queries of half th
    {
        f32x16 ya;
#pragma unroll
        for (int e = 0; e < 16; ++e) ya[e] = 0.f;
#pragma unroll
        for (int kst = 0; kst < KST; ++kst) ya = mfma32(wo[kst], *(const bf16x8 *)(Hs + q * OP + 16 * kst + 8 * h), ya);
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = ya[e];
        bf16_t *dst = A.Y + img_off + ((size_t)(y0 + qy) * D.W + x0 + q - qy * RW) * C + 32 * chh + 8 * h;
        *(bf16x8 *)dst = pack8(v);
        *(bf16x8 *)(dst + 16) = pack8(v + 8);
    }
    // reported last: a store ahead of the barriers above would have to land before them
    if (A.Ir_out && A.Ir_out != A.Ir_src && threadIdx.x == 0) A.Ir_out[rrow] = A.Ir_src ? j_given : j;
#ifdef BRA_EXPERIMENT
    if (A.trace) {
        BRA_TRACE(7);
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned long long *out = (unsigned long long *)(A.Y + img_off + ((size_t)y0 * D.W + x0) * C);
            for (int k = 0; k < 8; ++k) out[k] = trace_t[k];
        }
    }
#endif
#undef BRA_TRACE
}

// ---------------------------------------------------------------------------
struct MfmaWs {
    bf16_t *q, *k, *v, *o, *wt, *wot, *wa, *wf;
    float *xr, *u, *p;
    void *route;
    int32_t *ir;
    size_t bytes;
};

bool fast_route_ok(const Dims &D) { return D.S <= kFastRouteMaxS; }

int halo_rows(const Dims &D)
{
    const int qh = 64 / D.rw;
    return (qh + 4) * (D.rw + 4);
}

// The fused pipeline pays one extra K/V projection per routed key block.
bool fused_ok(const Dims &D)
{
    static const bool disabled = experiment_flag("BRA_DISABLE_FUSED");
    if (disabled || !fast_route_ok(D)) return false;
    if (D.C != 64) return false;
    return D.n == 64 && D.k == 1 && (D.rw == 8 || D.rw == 16);
}

// Whether the staged pipelines take Q^r, K^r from partial sums written by the projection
// kernel (few partial sums per region: small regions) or from the pooled X (k_pool, k_route).
bool pooled_projection(const Dims &D);

// log2 of the number of consecutive tokens whose Q / K accumulators the projection kernel
// sums: the largest of 1, 2, 4 that divides rw (such tokens lie in one row of one region).
int pool_group_log2(const Dims &D)
{
    int lg = 0;
    while (lg < 2 && D.rw % (2 << lg) == 0) ++lg;
    return lg;
}

// The projection kernel can walk over whole regions (n a power of two, at most 16 tokens, so that a
// region's sum is one reduction inside a row of 16 lanes).
bool region_tiles_ok(const Dims &D)
{
    static const bool off = experiment_flag("BRA_NO_REGION_TILES");
    return !off && D.n <= 16 && (D.n & (D.n - 1)) == 0 && (D.rw & (D.rw - 1)) == 0;
}

TileMap tile_map(const Dims &D, bool pooled)
{
    TileMap tm = {0, 0, 0, 0, D.R, D.S, D.rh, D.rw, D.W, D.N, D.B * D.R};
    if (!pooled) return tm;
    if (region_tiles_ok(D)) {
        tm.region_tiles = 1;
        while ((1 << tm.sum_log2) < D.n) ++tm.sum_log2;
        while ((1 << tm.rw_log2) < D.rw) ++tm.rw_log2;
        tm.map_log2 = tm.sum_log2;
    } else {
        tm.sum_log2 = pool_group_log2(D);
    }
    return tm;
}

bool pooled_projection(const Dims &D)
{
    return fast_route_ok(D) && (region_tiles_ok(D) || D.rh * (D.rw >> pool_group_log2(D)) <= 8);
}

MfmaWs carve(const Dims &D, void *ws)
{
    MfmaWs w;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    const size_t tok = fused_ok(D) ? 0 : (size_t)D.B * D.N;     // the k = 1 kernel projects inside the workgroup
    w.q = (bf16_t *)take(tok * D.C * 2);
    w.k = (bf16_t *)take(tok * D.C * 2);
    w.v = (bf16_t *)take(tok * D.C * 2);
    w.o = (bf16_t *)take(small_supported(D) ? small_scratch_bytes(D) : 0);
    w.wt = (bf16_t *)take((size_t)3 * D.C * D.C * 2);
    w.wot = (bf16_t *)take((size_t)D.C * D.C * 2);
    w.wa = (bf16_t *)take((size_t)(D.C * kLceOperandElems + small_table_elems(D.C)) * 2);
    w.wf = (bf16_t *)take(D.C == 64 ? (size_t)kFusedFragElems * 2 : 0);
    w.xr = (float *)take((size_t)D.B * D.R * D.C * sizeof(float));
    w.u = (float *)take(D.C == 64 && fused_ok(D) ? (size_t)D.B * D.R * D.C * sizeof(float) : 0);
    w.p = (float *)take(pooled_projection(D) ? (size_t)D.B * D.H * (D.W >> pool_group_log2(D)) * 2 * D.C * sizeof(float) : 0);
    w.route = take(fast_route_ok(D) ? 0 : valu_route_scratch_bytes(D));
    w.ir = (int32_t *)take((size_t)D.B * D.R * D.k * sizeof(int32_t));
    w.bytes = off;
    return w;
}

// More than 64 KB of dynamic LDS needs an opt-in, once per kernel.
template <typename K>
bool lds_opt_in(K kernel, bool &done)
{
    if (done) return true;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) !=
        hipSuccess)
        return false;
    done = true;
    return true;
}

// Regions per pooling workgroup: about 8 loads of 16 bytes per thread, at most 256
// (region, 8-channel chunk) pairs, and enough workgroups to fill the chip.
int pool_group(const Dims &D)
{
    static const int forced = (int)experiment_value("BRA_POOL_GROUP", 0);
    if (forced >= 1 && forced <= kPoolMaxGroup && forced * (D.C / 8) <= 256) return forced;
    const int chunks = D.n * (D.C / 8);
    int G = 2048 / chunks;
    const int cap = 256 / (D.C / 8) < kPoolMaxGroup ? 256 / (D.C / 8) : kPoolMaxGroup;
    G = G < 1 ? 1 : (G > cap ? cap : G);
    while (G > 1 && (long)D.B * ((D.R + G - 1) / G) < 512) G /= 2;
    return G;
}

// Pooling (if `pool`) and weight preparation (`prep_elems` leading prep elements) in one launch.
template <int C>
void launch_pool(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, const bf16_t *Wo,
                 const bf16_t *Wlce, const MfmaWs &w, bool pool, int prep_elems, hipStream_t st,
                 bool with_u = false)
{
    const int G = pool_group(D);
    const int pool_blocks = pool ? D.B * ((D.R + G - 1) / G) : 0;
    const int prep_blocks = (prep_elems + 255) / 256;
    if (pool_blocks + prep_blocks == 0) return;
    ProfScope ps(st, K_MFMA_POOL_QK);
    hipLaunchKernelGGL(k_pool<C>, dim3(pool_blocks + prep_blocks), dim3(256), 0, st, X, Wqkv, Wo, Wlce,
                       w.xr, with_u ? w.u : nullptr, w.wt, w.wot, w.wa, w.wf, D, pool_blocks, G,
                       experiment_flag("BRA_POOL_TRACE") ? -prep_elems : prep_elems);
}

template <int C>
int launch_route(const Dims &D, const MfmaWs &w, int32_t *Ir, float *Ar_opt, hipStream_t st)
{
    static bool opted = false;
    if (!lds_opt_in(k_route<C>, opted)) return BRA_ERR_LAUNCH;
    const size_t smem = RouteSmem<C>::bytes;
    ProfScope ps(st, K_MFMA_ROUTE_ROWS);
    hipLaunchKernelGGL(k_route<C>, dim3((D.B * ((D.R + 15) / 16) + 7) / 8 * 8), dim3(256), smem, st, w.xr, w.wt, Ir,
                       Ar_opt, D);
    return BRA_OK;
}

template <int C>
int launch_route_p(const Dims &D, const MfmaWs &w, int32_t *Ir, float *Ar_opt, hipStream_t st)
{
    // 8 query regions per workgroup (2 per wavefront) where two workgroups fit a compute unit
    // (the K^r tile takes C x 260 bytes of LDS): twice the workgroups, half the serial affinity /
    // top-k work in each.  Measured: C = 128 12.6 -> 10.8 us, C = 256 (one per unit) 17.3 -> 22.1 us.
    if (region_tiles_ok(D) && !experiment_flag("BRA_ROUTE_OLD")) {
        ProfScope ps(st, K_MFMA_ROUTE_ROWS);
        hipLaunchKernelGGL((k_route_w<C>), dim3((D.B * ((D.R + 15) / 16) + 7) / 8 * 8), dim3(256), 0, st, w.p, Ir,
                           Ar_opt, D);
        return BRA_OK;
    }
    static const int forced = (int)experiment_value("BRA_ROUTE_ROWS", 0);
    const bool rows8 = forced ? forced == 8 : 2 * RouteSmem<C>::kq_bytes <= (size_t)kMaxLds;
    ProfScope ps(st, K_MFMA_ROUTE_ROWS);
    if (rows8) {
        static bool opted = false;
        if (!lds_opt_in(k_route_p<C, 2>, opted)) return BRA_ERR_LAUNCH;
        hipLaunchKernelGGL((k_route_p<C, 2>), dim3((D.B * ((D.R + 7) / 8) + 7) / 8 * 8), dim3(256),
                           RouteSmem<C>::kq_bytes, st, w.p, Ir, Ar_opt, D, pool_group_log2(D),
                           (int)region_tiles_ok(D) | (experiment_flag("BRA_ROUTE_TRACE") ? 2 : 0));
    } else {
        static bool opted = false;
        if (!lds_opt_in(k_route_p<C, 4>, opted)) return BRA_ERR_LAUNCH;
        hipLaunchKernelGGL((k_route_p<C, 4>), dim3((D.B * ((D.R + 15) / 16) + 7) / 8 * 8), dim3(256),
                           RouteSmem<C>::kq_bytes, st, w.p, Ir, Ar_opt, D, pool_group_log2(D),
                           (int)region_tiles_ok(D) | (experiment_flag("BRA_ROUTE_TRACE") ? 2 : 0));
    }
    return BRA_OK;
}

// Q, K, V of all tokens into the workspace; with `pooled`, also the partial sums of Q and K;
// with prep.elems > 0, extra workgroups rearrange the weights for the kernels that follow.
template <int C>
int launch_qkv(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, const MfmaWs &w, bool pooled,
               const PrepArgs &prep, hipStream_t st, float qscale = 1.0f)
{
    const long M = (long)D.B * D.N;
    constexpr int RT = 1;                                  // 32 output channels per wavefront
    constexpr int WPB = (C == 256) ? 8 : 3 * C / 32;      // wavefronts per workgroup
    const long ntiles = (M + 63) / 64;
    // one workgroup per compute unit (what the registers allow for the wider ones; a second round of
    // workgroups would start when the first is done): every wavefront keeps its weight slice in
    // registers and the workgroup streams its share of the tokens
    const int gy = 3 * C / (32 * RT) / WPB;
    const long slots = experiment_value("BRA_QKV_SLOTS", C == 64 ? 512 : 256);
    // (routing workgroups take slots too: one workgroup too many would start a second round)
    const long tile_slots = slots > 2 * prep.route_items ? slots - prep.route_items : slots;
    long tpw = (ntiles * gy + tile_slots - 1) / tile_slots;
    static const int forced = (int)experiment_value("BRA_QKV_TPW", 0);
    if (forced >= 1 && forced <= 4096) tpw = forced;
    const int gx = (int)((ntiles + tpw - 1) / tpw);
    const int prep_blocks = (prep.elems + 64 * WPB - 1) / (64 * WPB) + prep.route_items;
    const size_t smem = std::max(kQkvSmem<C, WPB, RT>, prep.route_items ? RouteSmem<C>::bytes : (size_t)0);
    static bool opted = false;
    if (!lds_opt_in(k_qkv<C, WPB, 3, RT>, opted)) return BRA_ERR_LAUNCH;
    ProfScope ps(st, K_MFMA_QKV);
    hipLaunchKernelGGL((k_qkv<C, WPB, 3, RT>), dim3(gx * gy + prep_blocks), dim3(64 * WPB), smem, st, X, Wqkv, w.q,
                       w.k, w.v, pooled ? w.p : nullptr, tile_map(D, pooled), M, (int)tpw, gx, prep, qscale);
    return BRA_OK;
}

// Y = O Wo (Eq. 2) as a plain projection of a token map: the projection kernel with Wo as
// its only weight matrix.
template <int C>
int launch_wo(const Dims &D, const bf16_t *O, const bf16_t *Wo, bf16_t *Y, hipStream_t st)
{
    const long M = (long)D.B * D.N;
    constexpr int RT = 1, WPB = C / (32 * RT);
    const long ntiles = (M + 63) / 64;
    const long tpw = (ntiles + 511) / 512;
    const int gx = (int)((ntiles + tpw - 1) / tpw);
    const size_t smem = kQkvSmem<C, WPB, RT>;
    static bool opted = false;
    if (!lds_opt_in(k_qkv<C, WPB, 1, RT>, opted)) return BRA_ERR_LAUNCH;
    ProfScope ps(st, K_MFMA_WO);
    hipLaunchKernelGGL((k_qkv<C, WPB, 1, RT>), dim3(gx), dim3(64 * WPB), smem, st, O, Wo, Y, Y, Y, nullptr,
                       tile_map(D, false), M,
                       (int)tpw, gx, PrepArgs{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0}, 1.0f);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

bool attn_big_ok(const Dims &D);

template <int C>
int forward_c(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, const bf16_t *Wo,
              const bf16_t *Wlce, bf16_t *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
              const MfmaWs &w, hipStream_t st)
{
    // Routing: the k = 1 pipeline pools X and routes before its single kernel; the staged
    // pipelines pool Q and K inside the projection kernel and route after it.
    const int32_t *Ir_src = Ir_in_opt;
    int32_t *Ir_dst = Ir_out_opt ? Ir_out_opt : w.ir;
    const bool fused = C == 64 && fused_ok(D);
    bool prep_pending = false;      // the weights still have to be rearranged, next to the projection
    bool route_with_qkv = false;    // the routing from pooled X rides in the projection kernel's launch
    if (!fast_route_ok(D)) {
        if (!Ir_in_opt) {
            int rc = valu_route(D, X, Wqkv, Ir_dst, nullptr, w.route, st);
            if (rc != BRA_OK) return rc;
            Ir_src = Ir_dst;
        }
        ProfScope ps(st, K_MFMA_PREP);
        const int total = prep_total(C);
        hipLaunchKernelGGL(k_prep_weights, dim3((total + 255) / 256), dim3(256), 0, st, Wqkv, Wo, Wlce,
                           w.wt, w.wot, w.wa, w.wf, C, total);
    } else {
        // pool X and route before the rest, with the weight rearrangement in the same launch;
        // the pooled-projection pipelines need neither and rearrange next to the projection
        static const bool route_launch = experiment_flag("BRA_FUSED_ROUTE_LAUNCH");
        const bool inline_route = fused && !route_launch;     // the k = 1 kernel routes by itself, from the routing vectors
        {
            const bool from_x = (fused || !pooled_projection(D)) && !Ir_in_opt;
            if (fused || from_x)
                launch_pool<C>(D, X, Wqkv, Wo, Wlce, w, /*pool=*/from_x, prep_total(C), st, /*with_u=*/inline_route);
            if (from_x && !inline_route) {
                // next to the projection (which does not depend on it) where there is one
                route_with_qkv = !fused && !experiment_flag("BRA_ROUTE_LAUNCH");
                if (!route_with_qkv) {
                    const int rc = launch_route<C>(D, w, Ir_dst, nullptr, st);
                    if (rc != BRA_OK) return rc;
                }
                Ir_src = Ir_dst;
            }
            prep_pending = !(fused || from_x);
        }
    }
    // the many-block attention kernel takes Q in units of log2 of the softmax weights
    const bool q32 = !fused && attn_big_ok(D) && attn_q32_ok(D) && !experiment_flag("BRA_ATTN_OLD");
    const float c_exp = D.scale * 1.4426950408889634f;
    if (!fused) {
        const bool pooled = pooled_projection(D) && !Ir_in_opt;
        PrepArgs prep = {Wqkv, Wo, Wlce, w.wt, w.wot, w.wa, w.wf, prep_pending ? prep_total(C) : 0};
        prep.trace = (int)experiment_value("BRA_QKV_TRACE", 0);
        if (route_with_qkv) {
            prep.Xr = w.xr;
            prep.Ir = Ir_dst;
            prep.route_items = D.B * ((D.R + 15) / 16);
            prep.dims = D;
        }
        int rc = launch_qkv<C>(D, X, Wqkv, w, pooled, prep, st, q32 ? c_exp : 1.0f);
        if (rc != BRA_OK) return rc;
        if (pooled) {
            rc = launch_route_p<C>(D, w, Ir_dst, nullptr, st);
            if (rc != BRA_OK) return rc;
            Ir_src = Ir_dst;
        }
    }
    AttnArgs A;
    A.X = X; A.WT = w.wt; A.Q = w.q; A.K = w.k; A.V = w.v;
    A.Ir_src = Ir_src; A.Ir_out = Ir_out_opt; A.Wlce = Wlce; A.Wa = w.wa; A.WoF = w.wa + kLceOperandElems * C; A.WlT = A.WoF + C * C; A.Wf = w.wf; A.WoT = w.wot; A.Y = Y;
    A.Xr = w.xr; A.U = w.u;
    A.c_exp = c_exp;
    A.total = D.B * D.R * (D.n / 64);
    A.trace = experiment_flag("BRA_Q32_TRACE");
    const int grid = ((A.total + 7) / 8) * 8;
    const int hrows = halo_rows(D);

    if constexpr (C == 64) {
        if (fused) {
            static bool opted8 = false, opted16 = false;
            ProfScope ps(st, K_MFMA_FUSED_K1);
            if (D.rw == 8) {
                if (!lds_opt_in(k_fused<8>, opted8)) return BRA_ERR_LAUNCH;
                hipLaunchKernelGGL(k_fused<8>, dim3(grid), dim3(256), FusedSmem<8>::bytes, st, A, D);
            } else {
                if (!lds_opt_in(k_fused<16>, opted16)) return BRA_ERR_LAUNCH;
                hipLaunchKernelGGL(k_fused<16>, dim3(grid), dim3(256), FusedSmem<16>::bytes, st, A, D);
            }
            return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
        }
    }
    if (!attn_big_ok(D)) {
        const int rc = launch_small(D, A, w.o, st);
        if (rc != BRA_OK || !small_needs_projection(D)) return rc;
        return launch_wo<C>(D, w.o, Wo, Y, st);
    }
    if (q32) return launch_attn_q32(D, A, st);
    {
        const size_t smem = AttnSmem<C>::bytes(hrows);
        ProfScope ps(st, K_MFMA_ATTENTION);
        if constexpr (C == 64) {
            // few workgroups: twice the wavefronts each
            static const int forced = (int)experiment_value("BRA_ATTN_WAVES", 0);
            if (forced == 8 || (forced != 4 && A.total < 1024)) {
                static bool opted8 = false;
                if (!lds_opt_in(k_attn_big<64, 2>, opted8)) return BRA_ERR_LAUNCH;
                hipLaunchKernelGGL((k_attn_big<64, 2>), dim3(grid), dim3(512), smem, st, A, D);
                return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
            }
        }
        static bool opted = false;
        if (!lds_opt_in(k_attn_big<C, 1>, opted)) return BRA_ERR_LAUNCH;
        hipLaunchKernelGGL((k_attn_big<C, 1>), dim3(grid), dim3(256), smem, st, A, D);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

template <int C>
int route_c(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, int32_t *Ir, float *Ar_opt,
            const MfmaWs &w, hipStream_t st)
{
    // the same kernels as bra_forward runs for this shape, so that both give the same index
    int rc;
    if (C == 64 && fused_ok(D)) {
        launch_pool<C>(D, X, Wqkv, nullptr, nullptr, w, /*pool=*/true, 0, st, /*with_u=*/true);
        ProfScope ps(st, K_MFMA_ROUTE_ROWS);
        hipLaunchKernelGGL(k_route_u, dim3(D.B * D.R), dim3(256), 0, st, w.xr, w.u, Ir, Ar_opt, D);
        rc = BRA_OK;
    } else if (!pooled_projection(D)) {
        launch_pool<C>(D, X, Wqkv, nullptr, nullptr, w, /*pool=*/true, /*prep: Wq^T, Wk^T*/ 2 * C * C, st);
        rc = launch_route<C>(D, w, Ir, Ar_opt, st);
    } else {
        rc = launch_qkv<C>(D, X, Wqkv, w, /*pooled=*/true, PrepArgs{nullptr, nullptr, nullptr, nullptr, nullptr,
                                                                     nullptr, nullptr, 0}, st);
        if (rc == BRA_OK) rc = launch_route_p<C>(D, w, Ir, Ar_opt, st);
    }
    if (rc != BRA_OK) return rc;
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

bool attn_big_ok(const Dims &D)
{
    if (D.n % 64 != 0) return false;
    if (D.rw < 8 || 64 % D.rw != 0) return false;
    const int qh = 64 / D.rw;
    if (D.rh % qh != 0) return false;
    const int halo = ((halo_rows(D) + 15) / 16) * 16;
    size_t smem = 0;
    if (D.C == 64) smem = AttnSmem<64>::bytes(halo);
    else if (D.C == 128) smem = AttnSmem<128>::bytes(halo);
    else smem = AttnSmem<256>::bytes(halo);
    return smem <= (size_t)kMaxLds;
}

}  // namespace

// Shapes of the kernels specialised by channel count.
static bool specialised(const Dims &D)
{
    static const bool general_only = experiment_flag("BRA_GENERAL_PIPELINE");
    if (general_only) return false;
    if (D.dtype != BRA_BF16 || D.d != 32) return false;
    if (D.C != 64 && D.C != 128 && D.C != 256) return false;
    if ((long)D.B * D.R * (D.n / 64 + 1) + 8 > 0x7fffffffL) return false;
    if (!fast_route_ok(D) && !generic_supported(D)) return false;   // fallback routing kernels
    return attn_big_ok(D) || small_supported(D);
}

bool wide_shape(const Dims &D) { return !specialised(D); }

// The matrix-core kernels address a token's channels within its image by 32-bit element
// offsets and divide key / slot numbers with fast_div (exact below 2^20).
static bool addressable(const Dims &D)
{
    return (long)D.N * D.C < (1L << 31) && D.n < (1 << 20) && (long)D.kn < (1L << 20);
}

bool mfma_supported(const Dims &D) { return addressable(D) && (specialised(D) || wide_supported(D)); }

size_t mfma_workspace_bytes(const Dims &D)
{
    return wide_shape(D) ? wide_workspace_bytes(D) : carve(D, nullptr).bytes;
}

int mfma_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt, void *ws,
               hipStream_t st)
{
    if (wide_shape(D)) return wide_route(D, X, Wqkv, Ir, Ar_opt, ws, st);
    MfmaWs w = carve(D, ws);
    if (!fast_route_ok(D)) return valu_route(D, X, Wqkv, Ir, Ar_opt, w.route, st);
    const bf16_t *x = (const bf16_t *)X, *wq = (const bf16_t *)Wqkv;
    switch (D.C) {
    case 64: return route_c<64>(D, x, wq, Ir, Ar_opt, w, st);
    case 128: return route_c<128>(D, x, wq, Ir, Ar_opt, w, st);
    case 256: return route_c<256>(D, x, wq, Ir, Ar_opt, w, st);
    default: return BRA_ERR_UNSUPPORTED;
    }
}

int mfma_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                 void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st)
{
    if (wide_shape(D)) return wide_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, st);
    MfmaWs w = carve(D, ws);
    const bf16_t *x = (const bf16_t *)X, *wq = (const bf16_t *)Wqkv, *wo = (const bf16_t *)Wo,
                 *wl = (const bf16_t *)Wlce;
    bf16_t *y = (bf16_t *)Y;
    switch (D.C) {
    case 64: return forward_c<64>(D, x, wq, wo, wl, y, Ir_out_opt, Ir_in_opt, w, st);
    case 128: return forward_c<128>(D, x, wq, wo, wl, y, Ir_out_opt, Ir_in_opt, w, st);
    case 256: return forward_c<256>(D, x, wq, wo, wl, y, Ir_out_opt, Ir_in_opt, w, st);
    default: return BRA_ERR_UNSUPPORTED;
    }
}

// The projection kernels for the backward pass (bf16, C = 64, 128 or 256): Q, K, V = X Wqkv
// (Eq. 3) into three token maps (with WT given, the launch also writes WT[o][c] = Wqkv[c][o] and
// WoT[o][c] = Wo[c][o]), and Out = In W for one C x C matrix.
int mfma_project_qkv(const Dims &D, const void *X, const void *Wqkv, bf16_t *Q, bf16_t *K, bf16_t *V,
                     hipStream_t st, const void *Wo, bf16_t *WT, bf16_t *WoT)
{
    MfmaWs w = {};
    w.q = Q; w.k = K; w.v = V;
    // extra workgroups leave the transposed weights WT [3C][C], WoT [C][C] when asked for
    const PrepArgs none{(const bf16_t *)Wqkv, (const bf16_t *)Wo, nullptr, WT, WoT, nullptr, nullptr,
                        WT ? 4 * D.C * D.C : 0};
    const bf16_t *x = (const bf16_t *)X, *wq = (const bf16_t *)Wqkv;
    switch (D.C) {
    case 64: return launch_qkv<64>(D, x, wq, w, false, none, st);
    case 128: return launch_qkv<128>(D, x, wq, w, false, none, st);
    case 256: return launch_qkv<256>(D, x, wq, w, false, none, st);
    default: return BRA_ERR_UNSUPPORTED;
    }
}

int mfma_project(const Dims &D, const void *In, const bf16_t *W, bf16_t *Out, hipStream_t st)
{
    const bf16_t *in = (const bf16_t *)In;
    switch (D.C) {
    case 64: return launch_wo<64>(D, in, W, Out, st);
    case 128: return launch_wo<128>(D, in, W, Out, st);
    case 256: return launch_wo<256>(D, in, W, Out, st);
    default: return BRA_ERR_UNSUPPORTED;
    }
}

}  // namespace bra
