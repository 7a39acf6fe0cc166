// Backward pass of the layer on the matrix cores (bf16 tensors, heads of 32 channels, C = 64 or
// 128, at most 64 routed keys per query: k n <= 64), with the routing index held fixed.
//
// Chain rule through Eq. 6-7 and Eq. 1-2, with O = Attention(Q, K^g, V^g) + LCE(V), Y = O Wo:
//     dO = dY Wo^T                     projection kernel with Wo^T as its matrix
//     P  = softmax(scale Q K^T)        recomputed per (region, head) from the re-projected Q, K
//     dP = dO V^T,  dS = scale P o (dP - rowsum(P o dP))
//     dQ = dS K,  dK += dS^T Q,  dV += P^T dO          k_attn_bwd
//     dV += LCE^T(dO)                  the forward's depth-wise kernel with the taps reversed
//     dX = [dQ | dK | dV] Wqkv^T       one product with the transposed weights
//     dWqkv = X^T [dQ | dK | dV],  dWo = O^T dY         k_gemm_tn (contraction over tokens)
//     dWlce[c][ky][kx] = sum_t dO[t][c] V[t + (ky - 2, kx - 2)][c]       k_lce_bwd_w
// All products take bf16 operands and accumulate in float32; dQ, dK, dV and dO are rounded to
// bf16 between the kernels (they are matrix-core operands of the next product).  dK and dV of a
// token collect contributions from every region routed to it: float32 atomic adds into
// accumulators in the workspace, so results are reproducible to rounding, not bit for bit.
#include "bra_mfma_dev.h"

namespace bra {

using namespace mfma;

namespace {

template <typename K>
bool opt_in(K kernel, bool &done)
{
    if (done) return true;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) !=
        hipSuccess)
        return false;
    done = true;
    return true;
}

// Two transposing reads -> one MFMA operand: lane 16 g + i receives column col0 + i of the
// rows row0 + 4 g .. + 3 (contraction slots 0..3) and row0 + 16 + 4 g .. + 3 (slots 4..7) of a
// row-major tile.  The same row-to-slot map on both operands of a product (or the accumulator
// layout of a preceding product as the other operand) keeps the contraction consistent.
__device__ __forceinline__ bf16x8 tr_operand(const bf16_t *T, int pitch, int row0, int col0, int g, int i)
{
    const bf16_t *p = T + (row0 + 4 * g + i / 4) * pitch + col0 + 4 * (i % 4);
    const u32x2 a0 = __builtin_bit_cast(u32x2, lds_read_tr16(p));
    const u32x2 a1 = __builtin_bit_cast(u32x2, lds_read_tr16(p + 16 * pitch));
    const u32x4 av = {a0[0], a0[1], a1[0], a1[1]};
    return __builtin_bit_cast(bf16x8, av);
}

// acc[dt] = T^T[channel col + 16 dt + 4 g + j][..] x vals: T a 64-row tile (keys), vals[t][j] the
// value of key 16 t + 4 g + j for this lane's query (accumulator layout of S^T = K Q^T).
__device__ __forceinline__ void keys_contract(const bf16_t *T, int pitch, const float (&vals)[4][4], int col,
                                              int g, int i, f32x4 (&acc)[2])
{
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        const float pv[8] = {vals[2 * tp][0], vals[2 * tp][1], vals[2 * tp][2], vals[2 * tp][3],
                             vals[2 * tp + 1][0], vals[2 * tp + 1][1], vals[2 * tp + 1][2], vals[2 * tp + 1][3]};
        const bf16x8 pb = pack8(pv);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
            acc[dt] = mfma16(tr_operand(T, pitch, 32 * tp, col + 16 * dt, g, i), pb, acc[dt]);
    }
}

template <int C>
struct BwdSmem {
    static constexpr int CS = C + 16;     // elements per row of the token tiles
    static constexpr int PP = 64 + 8;     // elements per row of the P / dS tiles
    static constexpr int tile = 64 * CS;
    static constexpr int p_off = 4 * tile, ds_off = p_off + 64 * PP, tok_off = ds_off + 64 * PP;
    static constexpr size_t bytes = (size_t)tok_off * 2 + 128 * sizeof(int);
};

// ---------------------------------------------------------------------------
// Attention backward (derivative of Eq. 6 with Eq. 1) of one (image, region, block of up to 64
// queries) over the region's k n <= 64 routed keys.  The workgroup copies the K, V rows of the
// keys (found by index in the projected maps, Eq. 6) and the Q, dO rows of its queries into LDS.
// Per head, wavefront w owns queries 16 w .. 16 w + 15:
//     S^T = K Q^T and dP^T = V dO^T          (A operand: key rows, B operand: the query's row)
//     P = softmax over the keys, D = sum_j P_j dP_j, dS = scale P (dP - D)      (registers)
//     O^T = V^T P^T (attention output, needed for dWo) and dQ^T = K^T dS^T      (stored as bf16)
// then P and dS go to LDS as bf16 [query][key] and wavefront w, now owning keys 16 w .. + 15,
// forms dV = P^T dO and dK = dS^T Q (both operands by transposing reads, contraction over the 64
// queries) and adds them to the float32 accumulators of the keys' tokens.
// dQ has row pitch ldq (it is the first third of the [M][3C] gradient map).
template <int C>
__global__ __launch_bounds__(256) void k_attn_bwd(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                  const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                  const int32_t *__restrict__ Ir, bf16_t *__restrict__ O,
                                                  bf16_t *__restrict__ dQ, int ldq, float *__restrict__ dK,
                                                  float *__restrict__ dV, Dims D, int qchunks)
{
    using L = BwdSmem<C>;
    constexpr int CS = L::CS, PP = L::PP, CH8 = C / 8, NL = 64 * CH8 / 256;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + L::tile, *Qs = Vs + L::tile, *dOs = Qs + L::tile;
    bf16_t *Ps = Ks + L::p_off, *dSs = Ks + L::ds_off;
    int *ktok = (int *)(Ks + L::tok_off), *qtok = ktok + 64;

    const int qc = blockIdx.x % qchunks, r = (blockIdx.x / qchunks) % D.R, b = blockIdx.x / (qchunks * D.R);
    const int nq = min(64, D.n - 64 * qc), kn = D.kn;
    const size_t img = (size_t)b * D.N;

    // token (within the image) of slot s of region j (Sec. 3.2: regions tile the map row-major)
    auto token = [&](int region, int slot) {
        const int ry = region / D.S, rx = region % D.S, sy = slot / D.rw, sx = slot % D.rw;
        return (ry * D.rh + sy) * D.W + rx * D.rw + sx;
    };
    if (threadIdx.x < 64) {
        const int l = threadIdx.x;
        int t = -1;
        if (l < kn) {
            const int j = Ir[((size_t)b * D.R + r) * D.k + l / D.n];
            t = token(min(max(j, 0), D.R - 1), l % D.n);
        }
        ktok[l] = t;
    } else if (threadIdx.x < 128) {
        const int l = threadIdx.x - 64;
        qtok[l] = l < nq ? token(r, 64 * qc + l) : -1;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < NL; ++u) {
        const int idx = threadIdx.x + 256 * u, row = idx / CH8, c8 = idx % CH8;
        const int kt = ktok[row], qt = qtok[row];
        u32x4 kr = {0u, 0u, 0u, 0u}, vr = kr, qr = kr, gr = kr;
        if (kt >= 0) {
            kr = *(const u32x4 *)(K + (img + kt) * C + c8 * 8);
            vr = *(const u32x4 *)(V + (img + kt) * C + c8 * 8);
        }
        if (qt >= 0) {
            qr = *(const u32x4 *)(Q + (img + qt) * C + c8 * 8);
            gr = *(const u32x4 *)(dO + (img + qt) * C + c8 * 8);
        }
        *(u32x4 *)(Ks + row * CS + c8 * 8) = kr;
        *(u32x4 *)(Vs + row * CS + c8 * 8) = vr;
        *(u32x4 *)(Qs + row * CS + c8 * 8) = qr;
        *(u32x4 *)(dOs + row * CS + c8 * 8) = gr;
    }
    __syncthreads();

    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    const int q = 16 * w + i;
    const int my_qtok = qtok[q];
    const float c_exp = D.scale * 1.4426950408889634f;
    int my_ktok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) my_ktok[j] = ktok[16 * w + 4 * g + j];

#pragma unroll 1
    for (int h = 0; h < C / 32; ++h) {
        const int col = 32 * h;
        const bf16x8 qf = *(const bf16x8 *)(Qs + q * CS + col + 8 * g);
        const bf16x8 gf = *(const bf16x8 *)(dOs + q * CS + col + 8 * g);
        f32x4 s[4], dp[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * CS + col + 8 * g);
            const bf16x8 vf = *(const bf16x8 *)(Vs + (16 * t + i) * CS + col + 8 * g);
            s[t] = mfma16(kf, qf, f32x4{0.f, 0.f, 0.f, 0.f});     // S^T[key 16 t + 4 g + j][query i]
            dp[t] = mfma16(vf, gf, f32x4{0.f, 0.f, 0.f, 0.f});    // dP^T, same layout
        }
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (16 * t + 4 * g + j >= kn) s[t][j] = -INFINITY;
                mx = fmaxf(mx, s[t][j]);
            }
        mx = cross_row_max(mx);           // key 0 exists, so the maximum is finite
        const float mc = mx * c_exp;
        float p[4][4], ds[4][4], lsum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[t][j] = __builtin_amdgcn_exp2f(fmaf(s[t][j], c_exp, -mc));
                lsum += p[t][j];
            }
        const float inv = (my_qtok >= 0) ? 1.0f / cross_row_sum(lsum) : 0.f;    // rows of missing queries: P = 0
        float dsum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[t][j] *= inv;
                dsum = fmaf(p[t][j], dp[t][j], dsum);
            }
        dsum = cross_row_sum(dsum);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) ds[t][j] = p[t][j] * (dp[t][j] - dsum) * D.scale;

        f32x4 oacc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
        f32x4 qacc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
        keys_contract(Vs, CS, p, col, g, i, oacc);       // O^T[channel col + 16 dt + 4 g + j][query i]
        keys_contract(Ks, CS, ds, col, g, i, qacc);      // dQ^T, same layout
        if (my_qtok >= 0) {
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                *(u32x2 *)(O + (img + my_qtok) * C + col + 16 * dt + 4 * g) = pack4(oacc[dt]);
                *(u32x2 *)(dQ + (img + my_qtok) * (size_t)ldq + col + 16 * dt + 4 * g) = pack4(qacc[dt]);
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            *(u32x2 *)(Ps + q * PP + 16 * t + 4 * g) = pack4(f32x4{p[t][0], p[t][1], p[t][2], p[t][3]});
            *(u32x2 *)(dSs + q * PP + 16 * t + 4 * g) = pack4(f32x4{ds[t][0], ds[t][1], ds[t][2], ds[t][3]});
        }
        __syncthreads();

        // keys 16 w .. 16 w + 15 against all 64 queries:
        // dV[key 4 g + j][channel col + 16 dt + i] = sum_q P[q][key] dO[q][channel], dK likewise from dS, Q
        f32x4 dv[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
        f32x4 dk[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 pa = tr_operand(Ps, PP, 32 * ks, 16 * w, g, i);
            const bf16x8 da = tr_operand(dSs, PP, 32 * ks, 16 * w, g, i);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                dv[dt] = mfma16(pa, tr_operand(dOs, CS, 32 * ks, col + 16 * dt, g, i), dv[dt]);
                dk[dt] = mfma16(da, tr_operand(Qs, CS, 32 * ks, col + 16 * dt, g, i), dk[dt]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (my_ktok[j] < 0) continue;
            const size_t at = (img + my_ktok[j]) * C + col + i;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                unsafeAtomicAdd(dV + at + 16 * dt, dv[dt][j]);
                unsafeAtomicAdd(dK + at + 16 * dt, dk[dt][j]);
            }
        }
        __syncthreads();      // the next head overwrites Ps, dSs
    }
}

// ---------------------------------------------------------------------------
// Out[a0 + a][b0 + o] += sum_t A[t][a0 + a] Bm[t][b0 + o] over the workgroup's share of the M
// tokens (the token contractions dWqkv = X^T dQKV and dWo = O^T dY): a 64 x 64 block of the
// output per workgroup (blockIdx.y, blockIdx.z), both operands staged as [64 tokens][64 channels]
// LDS tiles and read with transposing reads, float32 atomic adds at the end.  Out is zeroed
// beforehand.  Wavefront w forms rows 16 w .. 16 w + 15 of the block.
__global__ __launch_bounds__(256) void k_gemm_tn(const bf16_t *__restrict__ A, int lda,
                                                 const bf16_t *__restrict__ Bm, int ldb, float *__restrict__ Out,
                                                 int ldo, long M, int tokens_per_wg)
{
    constexpr int TP = 64 + 16;
    __shared__ __attribute__((aligned(16))) bf16_t As[64 * TP];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[64 * TP];
    const int a0 = 64 * blockIdx.y, b0 = 64 * blockIdx.z;
    const long t_begin = (long)blockIdx.x * tokens_per_wg, t_end = min(M, t_begin + tokens_per_wg);
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    f32x4 acc[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 ar[2], br[2];
    auto fetch = [&](long t0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = threadIdx.x + 256 * u, row = idx / 8, c8 = idx % 8;
            ar[u] = u32x4{0u, 0u, 0u, 0u};
            br[u] = ar[u];
            if (t0 + row < t_end) {
                ar[u] = *(const u32x4 *)(A + (size_t)(t0 + row) * lda + a0 + c8 * 8);
                br[u] = *(const u32x4 *)(Bm + (size_t)(t0 + row) * ldb + b0 + c8 * 8);
            }
        }
    };
    if (t_begin < t_end) fetch(t_begin);
    for (long t0 = t_begin; t0 < t_end; t0 += 64) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = threadIdx.x + 256 * u, row = idx / 8, c8 = idx % 8;
            *(u32x4 *)(As + row * TP + c8 * 8) = ar[u];
            *(u32x4 *)(Bs + row * TP + c8 * 8) = br[u];
        }
        __syncthreads();
        if (t0 + 64 < t_end) fetch(t0 + 64);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 af = tr_operand(As, TP, 32 * ks, 16 * w, g, i);
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) acc[ct] = mfma16(af, tr_operand(Bs, TP, 32 * ks, 16 * ct, g, i), acc[ct]);
        }
        __syncthreads();
    }
    if (t_begin >= t_end) return;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            unsafeAtomicAdd(Out + (size_t)(a0 + 16 * w + 4 * g + j) * ldo + b0 + 16 * ct + i, acc[ct][j]);
}

// ---------------------------------------------------------------------------
// dWlce[c][ky][kx] += sum over the tokens (y, x) of the workgroup's tiles of
// dO[y][x][c] V[y + ky - 2][x + kx - 2][c] (derivative of the depth-wise 5x5 correlation of Eq. 7
// with respect to its taps; V is zero outside the image).  A tile is kBwTileH x kBwTileW tokens of
// one image and 64 channels: V with a 2-token halo in LDS, a thread handles a pair of channels
// and 4-token row segments and keeps the 2 x 25 sums in registers; the workgroup reduces them
// through LDS and adds them to dWlce (zeroed beforehand) with float32 atomics.
constexpr int kBwTileH = 4, kBwTileW = 32, kBwPitch = 64 + 8;
constexpr int kBwHaloRows = (kBwTileH + 4) * (kBwTileW + 4);
constexpr size_t kBwSmem = std::max((size_t)kBwHaloRows * kBwPitch * 2, (size_t)4 * 32 * 50 * 4);

__global__ __launch_bounds__(256) void k_lce_bwd_w(const bf16_t *__restrict__ dO, const bf16_t *__restrict__ V,
                                                   float *__restrict__ dW, Dims D, int tiles_total,
                                                   int tiles_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Hs = (bf16_t *)smem;
    const int C = D.C, NCH = C / 64;
    const int ytiles = (D.H + kBwTileH - 1) / kBwTileH, xtiles = (D.W + kBwTileW - 1) / kBwTileW;
    const int cc = blockIdx.x % NCH, c0 = 64 * cc;
    const int first_tile = (blockIdx.x / NCH) * tiles_per_wg;
    const int cpair = threadIdx.x % 32, grp = threadIdx.x / 32;
    constexpr int hw = kBwTileW + 4;
    float g0[25], g1[25];
#pragma unroll
    for (int e = 0; e < 25; ++e) g0[e] = g1[e] = 0.f;

    for (int tile = first_tile; tile < min(tiles_total, first_tile + tiles_per_wg); ++tile) {
        const int xt = tile % xtiles, yt = (tile / xtiles) % ytiles, b = tile / (xtiles * ytiles);
        const int y0 = yt * kBwTileH, x0 = xt * kBwTileW;
        const int th = min(kBwTileH, D.H - y0), tw = min(kBwTileW, D.W - x0);
        const size_t img_off = (size_t)b * D.N * C;
        __syncthreads();          // the previous tile's readers are done
        for (int idx = threadIdx.x; idx < kBwHaloRows * 8; idx += 256) {
            const int row = idx / 8, c8 = idx % 8;
            const int y = y0 - 2 + row / hw, x = x0 - 2 + row % hw;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (y >= 0 && y < D.H && x >= 0 && x < D.W)
                v = *(const u32x4 *)(V + img_off + ((size_t)y * D.W + x) * C + c0 + c8 * 8);
            *(u32x4 *)(Hs + row * kBwPitch + c8 * 8) = v;
        }
        __syncthreads();
        const int segs = (tw + 3) / 4;
        for (int task = grp; task < th * segs; task += 8) {
            const int seg = task % segs, r = task / segs;
            float d0[4], d1[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                unsigned u = 0u;
                if (seg * 4 + x < tw)
                    u = *(const unsigned *)(dO + img_off + ((size_t)(y0 + r) * D.W + x0 + seg * 4 + x) * C + c0 + 2 * cpair);
                d0[x] = bf16_lo(u);
                d1[x] = bf16_hi(u);
            }
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                float v0[8], v1[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + seg * 4 + x) * kBwPitch + 2 * cpair);
                    v0[x] = bf16_lo(u);
                    v1[x] = bf16_hi(u);
                }
#pragma unroll
                for (int kx = 0; kx < 5; ++kx)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        g0[ky * 5 + kx] = fmaf(d0[x], v0[x + kx], g0[ky * 5 + kx]);
                        g1[ky * 5 + kx] = fmaf(d1[x], v1[x + kx], g1[ky * 5 + kx]);
                    }
            }
        }
    }
    // lanes l and l + 32 of a wavefront hold the same channel pair; then the four wavefronts through LDS
    __syncthreads();
    float *Rs = (float *)smem;
    const int wv = threadIdx.x / 64;
#pragma unroll
    for (int e = 0; e < 25; ++e) {
        g0[e] += __shfl_xor(g0[e], 32);
        g1[e] += __shfl_xor(g1[e], 32);
        if (threadIdx.x % 64 < 32) {
            Rs[(wv * 32 + cpair) * 50 + e] = g0[e];
            Rs[(wv * 32 + cpair) * 50 + 25 + e] = g1[e];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * 50; idx += 256) {
        const float v = Rs[idx] + Rs[32 * 50 + idx] + Rs[2 * 32 * 50 + idx] + Rs[3 * 32 * 50 + idx];
        // idx = cpair * 50 + 25 * (channel of the pair) + tap
        unsafeAtomicAdd(dW + (size_t)(c0 + 2 * (idx / 50) + (idx % 50) / 25) * 25 + idx % 25, v);
    }
}

// ---------------------------------------------------------------------------
// Small element-wise kernels.

// WT[o][c] = Wqkv[c][o] ([3C][C]), WoT[o][c] = Wo[c][o], WlF[c][t] = Wlce[c][24 - t] (the taps
// of the transposed correlation), and zeros in the three weight gradients.
__global__ void k_bwd_prep(const bf16_t *__restrict__ Wqkv, const bf16_t *__restrict__ Wo,
                           const bf16_t *__restrict__ Wlce, bf16_t *__restrict__ WT, bf16_t *__restrict__ WoT,
                           bf16_t *__restrict__ WlF, float *__restrict__ dWqkv, float *__restrict__ dWo,
                           float *__restrict__ dWlce, int C)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < 3 * C * C) {
        const int o = e / C, c = e % C;
        WT[e] = Wqkv[(size_t)c * 3 * C + o];
        dWqkv[e] = 0.f;
    } else if (e < 4 * C * C) {
        const int f = e - 3 * C * C, o = f / C, c = f % C;
        WoT[f] = Wo[(size_t)c * C + o];
        dWo[f] = 0.f;
    } else if (e < 4 * C * C + 25 * C) {
        const int f = e - 4 * C * C, c = f / 25, t = f % 25;
        WlF[f] = Wlce[c * 25 + 24 - t];
        dWlce[f] = 0.f;
    }
}

__global__ void k_zero16(u32x4 *__restrict__ p, size_t count)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < count) p[e] = u32x4{0u, 0u, 0u, 0u};
}

// dQKV[t][C + c] = bf16(dK[t][c]), dQKV[t][2C + c] = bf16(dV[t][c] + G[t][c]) with G = LCE^T(dO):
// 8 channels per thread.
__global__ void k_bwd_pack(const float *__restrict__ dK, const float *__restrict__ dV,
                           const bf16_t *__restrict__ G, bf16_t *__restrict__ dQKV, size_t chunks, int C)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= chunks) return;
    const int c8 = C / 8;
    const size_t t = e / c8;
    const int c = (int)(e % c8) * 8;
    const f32x4 k0 = *(const f32x4 *)(dK + t * C + c), k1 = *(const f32x4 *)(dK + t * C + c + 4);
    const f32x4 v0 = *(const f32x4 *)(dV + t * C + c), v1 = *(const f32x4 *)(dV + t * C + c + 4);
    const u32x4 gv = *(const u32x4 *)(G + t * C + c);
    const u32x4 ko = {pack_bf16(k0[0], k0[1]), pack_bf16(k0[2], k0[3]), pack_bf16(k1[0], k1[1]), pack_bf16(k1[2], k1[3])};
    const u32x4 vo = {pack_bf16(v0[0] + bf16_lo(gv[0]), v0[1] + bf16_hi(gv[0])),
                      pack_bf16(v0[2] + bf16_lo(gv[1]), v0[3] + bf16_hi(gv[1])),
                      pack_bf16(v1[0] + bf16_lo(gv[2]), v1[1] + bf16_hi(gv[2])),
                      pack_bf16(v1[2] + bf16_lo(gv[3]), v1[3] + bf16_hi(gv[3]))};
    *(u32x4 *)(dQKV + t * 3 * C + C + c) = ko;
    *(u32x4 *)(dQKV + t * 3 * C + 2 * C + c) = vo;
}

// ---------------------------------------------------------------------------
struct BwdWs {
    bf16_t *q, *k, *v, *dO, *o, *g, *dqkv, *wt, *wot, *wlf;
    float *dk, *dv;
    size_t bytes;
};

BwdWs carve_bwd(const Dims &D, void *ws)
{
    char *base = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    const size_t MC = (size_t)D.B * D.N * D.C, C = D.C;
    BwdWs w;
    w.q = (bf16_t *)take(MC * 2);
    w.k = (bf16_t *)take(MC * 2);
    w.v = (bf16_t *)take(MC * 2);
    w.dO = (bf16_t *)take(MC * 2);
    w.o = (bf16_t *)take(MC * 2);
    w.dqkv = (bf16_t *)take(MC * 6);
    // dk, dv, g are zeroed by one fill: keep them adjacent (MC * 4 and MC * 2 are multiples of 256 or
    // the fill covers the padding too)
    w.dk = (float *)take(MC * 4);
    w.dv = (float *)take(MC * 4);
    w.g = (bf16_t *)take(MC * 2);
    w.wt = (bf16_t *)take(3 * C * C * 2);
    w.wot = (bf16_t *)take(C * C * 2);
    w.wlf = (bf16_t *)take(25 * C * 2);
    w.bytes = off;
    return w;
}

template <int C>
int attn_bwd(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    static bool opted = false;
    if (!opt_in(k_attn_bwd<C>, opted)) return BRA_ERR_LAUNCH;
    const int qchunks = (D.n + 63) / 64;
    const long blocks = (long)D.B * D.R * qchunks;
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL(k_attn_bwd<C>, dim3((unsigned)blocks), dim3(256), BwdSmem<C>::bytes, st, w.q, w.k, w.v, w.dO,
                       Ir, w.o, w.dqkv, 3 * C, w.dk, w.dv, D, qchunks);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

int gemm_tn(const bf16_t *A, int lda, int Ca, const bf16_t *Bm, int ldb, int Cb, float *Out, int ldo, long M,
            hipStream_t st)
{
    const long steps = (M + 63) / 64;
    const long per_wg = (steps + 383) / 384;             // about 384 token shares
    const int gx = (int)((steps + per_wg - 1) / per_wg);
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL(k_gemm_tn, dim3(gx, Ca / 64, Cb / 64), dim3(256), 0, st, A, lda, Bm, ldb, Out, ldo, M,
                       (int)(per_wg * 64));
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

bool launched() { return hipGetLastError() == hipSuccess; }

}  // namespace

bool mfma_backward_supported(const Dims &D)
{
    static const bool off = experiment_flag("BRA_NO_MFMA_BACKWARD");
    if (off || D.dtype != BRA_BF16 || D.d != 32 || (D.C != 64 && D.C != 128) || D.kn > 64) return false;
    const long M = (long)D.B * D.N;
    return M * 3 * D.C < (1L << 40) && (long)D.B * D.R * ((D.n + 63) / 64) <= 0x7fffffffL && M <= 0x7fffffffL;
}

size_t mfma_backward_workspace_bytes(const Dims &D) { return carve_bwd(D, nullptr).bytes; }

int mfma_backward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                  const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                  hipStream_t st)
{
    const BwdWs w = carve_bwd(D, ws);
    const int C = D.C;
    const long M = (long)D.B * D.N;
    const size_t MC = (size_t)M * C;
    {
        ProfScope ps(st, K_GEN_BACKWARD);
        const int total = 4 * C * C + 25 * C;
        hipLaunchKernelGGL(k_bwd_prep, dim3((total + 255) / 256), dim3(256), 0, st, (const bf16_t *)Wqkv,
                           (const bf16_t *)Wo, (const bf16_t *)Wlce, w.wt, w.wot, w.wlf, dWqkv, dWo, dWlce, C);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    {
        ProfScope ps(st, K_GEN_BACKWARD);
        const size_t count = (size_t)((char *)w.g - (char *)w.dk + MC * 2 + 15) / 16;   // dk | dv | g
        hipLaunchKernelGGL(k_zero16, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, (u32x4 *)w.dk, count);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    int rc = mfma_project_qkv(D, X, Wqkv, w.q, w.k, w.v, st);                 // Q, K, V once more (Eq. 3)
    if (rc != BRA_OK) return rc;
    rc = mfma_project(D, dY, w.wot, w.dO, st);                                // dO = dY Wo^T
    if (rc != BRA_OK) return rc;
    rc = (C == 64) ? attn_bwd<64>(D, w, Ir, st) : attn_bwd<128>(D, w, Ir, st);
    if (rc != BRA_OK) return rc;
    AttnArgs A = {};
    A.V = w.v; A.Wlce = (const bf16_t *)Wlce;
    rc = launch_lce_add_any(D, A, w.o, st);                                   // O = attention + LCE(V)  (Eq. 7)
    if (rc != BRA_OK) return rc;
    A.V = w.dO; A.Wlce = w.wlf;
    rc = launch_lce_add_any(D, A, w.g, st);                                   // G = LCE^T(dO)
    if (rc != BRA_OK) return rc;
    {
        ProfScope ps(st, K_GEN_BACKWARD);
        const size_t chunks = MC / 8;
        hipLaunchKernelGGL(k_bwd_pack, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, w.dk, w.dv, w.g,
                           w.dqkv, chunks, C);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    rc = gemm_bf16(w.dqkv, w.wt, M, 3 * C, C, (bf16_t *)dX, nullptr, nullptr, false, K_GEN_BACKWARD, st);
    if (rc != BRA_OK) return rc;
    rc = gemm_tn((const bf16_t *)X, C, C, w.dqkv, 3 * C, 3 * C, dWqkv, 3 * C, M, st);
    if (rc != BRA_OK) return rc;
    rc = gemm_tn(w.o, C, C, (const bf16_t *)dY, C, C, dWo, C, M, st);
    if (rc != BRA_OK) return rc;
    {
        const int ytiles = (D.H + kBwTileH - 1) / kBwTileH, xtiles = (D.W + kBwTileW - 1) / kBwTileW;
        const int tiles = D.B * ytiles * xtiles;
        const int per_wg = (tiles + 511) / 512;
        const int groups = (tiles + per_wg - 1) / per_wg;
        static bool opted = false;
        if (!opt_in(k_lce_bwd_w, opted)) return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_GEN_BACKWARD);
        hipLaunchKernelGGL(k_lce_bwd_w, dim3(groups * (C / 64)), dim3(256), kBwSmem, st, w.dO, w.v, dWlce, D, tiles,
                           per_wg);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    return BRA_OK;
}

}  // namespace bra
