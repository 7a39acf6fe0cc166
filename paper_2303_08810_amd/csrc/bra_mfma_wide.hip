// Matrix-core pipeline for the shapes that the specialised kernels do not take: any C that is
// a multiple of 64, heads of 32 or 64 channels, any region size and count, e.g. the last stage
// of the paper's backbones (7x7 map, S = 7: one token per region, k = S^2, C = 512), the wider
// variants' stages (C = 384, 768), S = 16 on large maps, and the plain-ViT adaptation of the
// appendix (32x32 map, S = 8, k = 12, 12 heads of 64 channels).
//
//   k_pool_wide   Xr[b, r, :] = mean of the region's tokens, float32            (Sec. 3.2)
//   k_gemm<true>  Q^r | K^r = Xr [Wq | Wk] in float32: the means are split exactly into three
//                 bf16 terms, so the products are those of the float32 computation
//   k_route_qk    rows of A^r = Q^r (K^r)^T (Eq. 4) and their top-k (Eq. 5)
//   k_gemm<false> Q | K | V = X Wqkv (Eq. 3), bf16 out
//   image-resident attention (small maps, regions of up to 8 tokens; bra_mfma_small.hip) or
//   k_attn_gen (everything else), then LCE added in place                       (Eq. 6, 7)
//   k_gemm<false> Y = O Wo (Eq. 2)
#include "bra_mfma_dev.h"

#include <stdlib.h>

namespace bra {

using namespace mfma;

namespace {

// SUB (1, 2, 4 or 8) consecutive lanes share one (image, region, 8-channel chunk): lane s adds
// tokens s, s + SUB, .. of the region (row-major), then the partial sums are combined pairwise
// in a fixed order.
__global__ __launch_bounds__(256) void k_pool_wide(const bf16_t *__restrict__ X, float *__restrict__ Xr, Dims D,
                                                   int SUB)
{
    const int CH = D.C / 8;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const long item = idx / SUB;
    const int sub = (int)(idx % SUB);
    const bool valid = item < (long)D.B * D.R * CH;
    const long it = valid ? item : 0;
    const int cc = (int)(it % CH), r = (int)((it / CH) % D.R), b = (int)(it / ((long)CH * D.R));
    const bf16_t *base = X + (((size_t)b * D.H + (r / D.S) * D.rh) * D.W + (r % D.S) * D.rw) * D.C + cc * 8;
    const float rw_inv = 1.0f / (float)D.rw;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int slot = sub; slot < D.n; slot += SUB) {
        const int y = fast_div(slot, rw_inv), x = slot - y * D.rw;
        const u32x4 v = *(const u32x4 *)(base + ((size_t)y * D.W + x) * D.C);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[2 * e] += bf16_lo(v[e]);
            acc[2 * e + 1] += bf16_hi(v[e]);
        }
    }
    for (int off = 1; off < SUB; off *= 2)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
    if (valid && sub == 0) {
        float *dst = Xr + ((size_t)b * D.R + r) * D.C + cc * 8;
        const float inv = 1.0f / (float)D.n;
        *(f32x4 *)dst = f32x4{acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
        *(f32x4 *)(dst + 4) = f32x4{acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv};
    }
}

// ---------------------------------------------------------------------------
// Out[m][o] = sum_k In[m][k] W[k][o] (W row-major with ldw columns, as the caller holds it)
// for a tile of 64 rows m x 32 CW outputs o (128 or 64) per workgroup, the contraction in chunks of 64
// staged in LDS (the next chunk is requested while the current one is multiplied).
// The four wavefronts split the tile 2 x 2 (32 rows x 16 CW outputs each); the product is formed
// transposed (D[output 16 t + 4 g + jj][row i]) so that a lane stores 4 consecutive outputs of one row;
// its W operand (rows = outputs) comes out of the row-major chunk by the transposing LDS read.
// Output column o goes to buffer o / cols (three buffers of `cols` columns each, e.g. Q, K,
// V), column o % cols.
// SPLIT: In is float32 and enters as three exact bf16 terms (smallest first); otherwise In is
// bf16.  F32OUT: Out is float32, else bf16.
constexpr int kGemmPitch = 80;      // bf16 per LDS row of In: 64 + 16 (rows of 160 bytes); W: the tile's width + 16
constexpr int kGemmGroupW = 64;     // W: 128 bytes more after every 8 rows: the neighbouring lane group of a
                                    // transposing read (8 rows further on) then meets the other half of the banks

struct GemmOut {
    void *buf[3];
    int cols;
    float *f32[2];      // optional float32 copies of the results that go to buf[0] and buf[1] (bf16 output only)
    // bf16 output only, all optional: bias[o] is added, then GELU is applied, then res[m][o]
    // (the layout of buf[0]) is added.
    const float *bias;
    const bf16_t *res;
    int gelu;
};

template <bool SPLIT, bool F32OUT = SPLIT, int CW = 4>
__global__ __launch_bounds__(256) void k_gemm(const void *__restrict__ In, const bf16_t *__restrict__ W,
                                              int ldw, int M, int K, int Nout, GemmOut out)
{
    constexpr int P = kGemmPitch, NT = SPLIT ? 3 : 1, COLS = 32 * CW, PW = COLS + 16;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ws = (bf16_t *)smem;                 // [64 k][PW]
    bf16_t *Xs = Ws + 64 * PW + 8 * kGemmGroupW; // [NT][64][P]
    float *bs = (float *)(Xs + NT * 64 * P);     // [128]: the tile's slice of the bias
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave, g = lane / 16, i = lane % 16;
    const int otiles = (Nout + COLS - 1) / COLS;
    const int m0 = (blockIdx.x / otiles) * 64, o0 = (blockIdx.x % otiles) * COLS;

    // this thread's pieces of a chunk: 4 x 16 bytes of W, and 2 x 16 bytes of bf16 In or
    // 2 x 8 floats of float32 In
    u32x4 wreg[CW], xreg[SPLIT ? 4 : 2];
    auto request = [&](int k0) {
#pragma unroll
        for (int u = 0; u < CW; ++u) {
            const int idx = tid + 256 * u;                       // (row k, 8 outputs)
            const int o = min(o0 + (idx % (COLS / 8)) * 8, Nout - 8);    // columns past the end repeat the last; never stored
            wreg[u] = *(const u32x4 *)(W + (size_t)(k0 + idx / (COLS / 8)) * ldw + o);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + 256 * u;
            const int m = min(m0 + idx / 8, M - 1);
            if (SPLIT) {
                const float *src = (const float *)In + (size_t)m * K + k0 + (idx % 8) * 8;
                xreg[2 * u] = *(const u32x4 *)src;
                xreg[2 * u + 1] = *(const u32x4 *)(src + 4);
            } else {
                xreg[u] = *(const u32x4 *)((const bf16_t *)In + (size_t)m * K + k0 + (idx % 8) * 8);
            }
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int u = 0; u < CW; ++u) {
            const int idx = tid + 256 * u;
            const int row = idx / (COLS / 8);
            *(u32x4 *)(Ws + row * PW + (row / 8) * kGemmGroupW + (idx % (COLS / 8)) * 8) = wreg[u];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + 256 * u;
            bf16_t *dst = Xs + (idx / 8) * P + (idx % 8) * 8;
            if (SPLIT) {
                const f32x4 lo = __builtin_bit_cast(f32x4, xreg[2 * u]), hi = __builtin_bit_cast(f32x4, xreg[2 * u + 1]);
                const float x[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                bf16x8 t[3];
                split3(x, t);
#pragma unroll
                for (int q = 0; q < 3; ++q) *(bf16x8 *)(dst + q * 64 * P) = t[q];
            } else {
                *(u32x4 *)dst = xreg[u];
            }
        }
    };

    // wavefront (wr, wc) owns rows 32 wr .. 32 wr + 31 (two 16-row tiles) and outputs 64 wc ..
    // 64 wc + 63 (four tiles) of the workgroup's 64 x 128: a W fragment serves two row tiles
    const int wr = wave / 2, wc = wave % 2;
    f32x4 acc[2][CW];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int t = 0; t < CW; ++t) acc[rt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (!F32OUT && out.bias && tid < COLS) bs[tid] = out.bias[min(o0 + tid, Nout - 1)];   // read after the loop's barriers
    request(0);
    for (int k0 = 0; k0 < K; k0 += 64) {
        if (k0) __syncthreads();          // the previous chunk has been read
        park();
        __syncthreads();
        if (k0 + 64 < K) request(k0 + 64);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 xb[2][NT];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int q = 0; q < NT; ++q)
                    xb[rt][q] = *(const bf16x8 *)(Xs + (q * 64 + 32 * wr + 16 * rt + i) * P + 32 * ks + 8 * g);
#pragma unroll
            for (int t = 0; t < CW; ++t) {
                const bf16_t *wp = Ws + (32 * ks + 8 * g + i / 4) * PW + (4 * ks + g) * kGemmGroupW + 16 * CW * wc + 16 * t +
                                   4 * (i % 4);
                const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
                const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 4 * PW));
                const bf16x8 wf = __builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]});
#pragma unroll
                for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                    for (int q = NT - 1; q >= 0; --q) acc[rt][t] = mfma16(wf, xb[rt][q], acc[rt][t]);
            }
        }
    }
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int m = m0 + 32 * wr + 16 * rt + i;
        if (m >= M) continue;
        // the residual's pieces are requested together, ahead of the arithmetic (one by one
        // behind the loop's exit test their latencies would add up)
        u32x2 rv[CW];
        if (!F32OUT && out.res) {
#pragma unroll
            for (int t = 0; t < CW; ++t) {
                const int o = min(o0 + 16 * CW * wc + 16 * t + 4 * g, Nout - 4);
                rv[t] = *(const u32x2 *)(out.res + (size_t)m * out.cols + o);
            }
        }
#pragma unroll
        for (int t = 0; t < CW; ++t) {
            const int o = o0 + 16 * CW * wc + 16 * t + 4 * g;
            if (o >= Nout) break;
            const int which = o / out.cols, col = o % out.cols;
            if (F32OUT) {
                *(f32x4 *)((float *)out.buf[which] + (size_t)m * out.cols + col) = acc[rt][t];
            } else {
                f32x4 v = acc[rt][t];
                if (out.bias) {
                    const f32x4 bv = *(const f32x4 *)(bs + 16 * CW * wc + 16 * t + 4 * g);
                    v = f32x4{v[0] + bv[0], v[1] + bv[1], v[2] + bv[2], v[3] + bv[3]};
                }
                if (out.gelu) v = f32x4{gelu_f32(v[0]), gelu_f32(v[1]), gelu_f32(v[2]), gelu_f32(v[3])};
                if (out.res)
                    v = f32x4{v[0] + bf16_lo(rv[t][0]), v[1] + bf16_hi(rv[t][0]), v[2] + bf16_lo(rv[t][1]),
                              v[3] + bf16_hi(rv[t][1])};
                *(u32x2 *)((bf16_t *)out.buf[which] + (size_t)m * out.cols + col) = pack4(v);
                if (which < 2 && out.f32[which]) *(f32x4 *)(out.f32[which] + (size_t)m * out.cols + col) = acc[rt][t];
            }
        }
    }
}

constexpr size_t gemm_smem(bool split, int cw = 4)
{
    return (size_t)(64 * (32 * cw + 16) + 8 * kGemmGroupW) * 2 + (size_t)(split ? 3 : 1) * 64 * kGemmPitch * 2 +
           128 * sizeof(float);
}

// ---------------------------------------------------------------------------
// Rows of A^r = Q^r (K^r)^T (Eq. 4) in float32 and their top-k (Eq. 5) for workgroup
// (image, 4 NR query regions), R <= 64: the channels pass through LDS 64 at a time (K^r of all
// regions as [16][kQkRS][4]: channel group, region, channel; Q^r of the workgroup's rows),
// wavefront w accumulates rows NR w .. NR w + NR - 1 with lane j holding entry j.
constexpr int kQkRS = 65;

template <int NR>
__global__ __launch_bounds__(256) void k_route_qk(const float *__restrict__ Qr, const float *__restrict__ Kr,
                                                  int32_t *__restrict__ Ir, float *__restrict__ Ar, Dims D)
{
    __shared__ __attribute__((aligned(16))) float Kt[16 * kQkRS * 4];
    __shared__ __attribute__((aligned(16))) float Qs[16 * 68];
    constexpr int QR = 4 * NR;
    const int groups = (D.R + QR - 1) / QR;
    const int b = blockIdx.x / groups, myrt = blockIdx.x % groups;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const size_t img = (size_t)b * D.R * D.C;
    float a[NR];
#pragma unroll
    for (int rr = 0; rr < NR; ++rr) a[rr] = 0.f;
    f32x4 kv[4], qv;
    auto request = [&](int c0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * u;               // (region, 4-channel group)
            const int r = min(idx / 16, D.R - 1);        // regions past R repeat the last; never used
            kv[u] = *(const f32x4 *)(Kr + img + (size_t)r * D.C + c0 + (idx % 16) * 4);
        }
        const int r = min(QR * myrt + (tid / 16) % QR, D.R - 1);
        qv = *(const f32x4 *)(Qr + img + (size_t)r * D.C + c0 + (tid % 16) * 4);
    };
    request(0);
    for (int c0 = 0; c0 < D.C; c0 += 64) {
        if (c0) __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + 256 * u;
            *(f32x4 *)(Kt + ((idx % 16) * kQkRS + idx / 16) * 4) = kv[u];
        }
        if (tid / 16 < QR) *(f32x4 *)(Qs + (tid / 16) * 68 + (tid % 16) * 4) = qv;
        __syncthreads();
        if (c0 + 64 < D.C) request(c0 + 64);      // the next chunk travels while this one is multiplied
#pragma unroll 4
        for (int c4 = 0; c4 < 16; ++c4) {
            const f32x4 k4 = *(const f32x4 *)(Kt + (c4 * kQkRS + lane) * 4);
#pragma unroll
            for (int rr = 0; rr < NR; ++rr) {
                const f32x4 q4 = *(const f32x4 *)(Qs + (NR * wave + rr) * 68 + 4 * c4);
#pragma unroll
                for (int e = 0; e < 4; ++e) a[rr] = fmaf(q4[e], k4[e], a[rr]);
            }
        }
    }
    const int r0 = QR * myrt + NR * wave;
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

// ---------------------------------------------------------------------------
// Routed attention (Eq. 6, Eq. 1) for any region size and heads of 32 or 64 channels:
// workgroup (image, region, tile of 64 queries of the region, group of 64 channels = 2 or
// 1 heads), wavefront w with queries 16 w .. 16 w + 15 of the tile.  The k n routed keys are
// taken 64 at a time: their K and V rows (the group's 128 bytes each, found by index in the
// projected maps) are copied into LDS with coalesced loads, the next block being requested
// while the current one is worked on; S^T = K Q^T, one softmax over all routed keys (lazy
// reference, see softmax_pv_rows), O^T += V^T P^T by the transposing LDS read.  Queries past
// the end of the region and keys past k n repeat the last one and are masked.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_gen(AttnArgs A, bf16_t *__restrict__ O, Dims D)
{
    constexpr int HPW = 64 / HD;          // heads of this workgroup
    constexpr int KSD = HD / 32;          // contraction steps of a score
    constexpr int NDT = HD / 16;          // 16-channel tiles of a head's output
    constexpr int XP = 64 + 16;
    __shared__ __attribute__((aligned(16))) bf16_t Ks[64 * XP];
    __shared__ __attribute__((aligned(16))) bf16_t Vs[64 * XP];
    const int C = D.C, ncg = C / 64, n = D.n, kn = D.kn;
    const int qtiles = (n + 63) / 64;
    const int cg = blockIdx.x % ncg, qt = (blockIdx.x / ncg) % qtiles;
    const int reg = (blockIdx.x / (ncg * qtiles)) % D.R, b = blockIdx.x / (ncg * qtiles * D.R);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave, g = lane / 16, i = lane % 16;
    const float rw_inv = 1.0f / (float)D.rw, n_inv = 1.0f / (float)n, s_inv = 1.0f / (float)D.S;
    const size_t img_off = (size_t)b * D.N * C + 64 * cg;
    auto region_origin = [&](int r) {
        const int ry = fast_div(r, s_inv);
        return ry * D.rh * D.W + (r - ry * D.S) * D.rw;
    };
    auto in_region = [&](int slot) {
        const int sy = fast_div(slot, rw_inv);
        return sy * D.W + slot - sy * D.rw;
    };
    const int32_t *irp = A.Ir_src + ((size_t)b * D.R + reg) * D.k;
    if (A.Ir_out && A.Ir_out != A.Ir_src && qt == 0 && cg == 0)
        for (int p = tid; p < D.k; p += 256) A.Ir_out[((size_t)b * D.R + reg) * D.k + p] = irp[p];

    const int slot = 64 * qt + 16 * wave + i;
    const size_t qtok = (size_t)region_origin(reg) + in_region(min(slot, n - 1));
    bf16x8 qf[HPW][KSD];
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
        for (int ks = 0; ks < KSD; ++ks)
            qf[hh][ks] = *(const bf16x8 *)(A.Q + img_off + qtok * C + HD * hh + 32 * ks + 8 * g);

    u32x4 kreg[2], vreg[2];
    auto request = [&](int k0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + 256 * u;                       // (key of the block, 16-byte piece)
            const int key = min(k0 + idx / 8, kn - 1);
            const int p = fast_div(key, n_inv);
            const size_t tok = (size_t)region_origin(region_index(irp[p], D.R)) + in_region(key - p * n);
            const size_t off = img_off + tok * C + (idx % 8) * 8;
            kreg[u] = *(const u32x4 *)(A.K + off);
            vreg[u] = *(const u32x4 *)(A.V + off);
        }
    };
    float m[HPW], l[HPW];
    f32x4 acc[HPW][NDT];
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        m[hh] = -INFINITY;
        l[hh] = 0.f;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) acc[hh][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float lim = 8.0f / A.c_exp;
    request(0);
    for (int k0 = 0; k0 < kn; k0 += 64) {
        if (k0) __syncthreads();              // the previous block has been read
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = tid + 256 * u;
            *(u32x4 *)(Ks + (idx / 8) * XP + (idx % 8) * 8) = kreg[u];
            *(u32x4 *)(Vs + (idx / 8) * XP + (idx % 8) * 8) = vreg[u];
        }
        if (k0 + 64 < kn) request(k0 + 64);
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) {
            f32x4 s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KSD; ++ks) {
                    const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * XP + HD * hh + 32 * ks + 8 * g);
                    s[t] = mfma16(kf, qf[hh][ks], s[t]);        // S^T[key 16 t + 4 g + jj][query i]
                }
            }
            if (k0 + 64 > kn) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        if (k0 + 16 * t + 4 * g + jj >= kn) s[t][jj] = -INFINITY;
            }
            float mx = s[0][0];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) mx = fmaxf(mx, s[t][jj]);
            mx = cross_row_max(mx);
            if (__builtin_amdgcn_ballot_w64(mx > m[hh] + lim) != 0) {
                const float m_new = fmaxf(m[hh], mx);
                const float alpha = __builtin_amdgcn_exp2f((m[hh] - m_new) * A.c_exp);
                m[hh] = m_new;
                l[hh] *= alpha;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) acc[hh][dt] *= alpha;
            }
            const float mc = m[hh] * A.c_exp;
            float p[4][4], ls = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    p[t][jj] = __builtin_amdgcn_exp2f(fmaf(s[t][jj], A.c_exp, -mc));
                    ls += p[t][jj];
                }
            l[hh] += cross_row_sum(ls);
#pragma unroll
            for (int tp = 0; tp < 2; ++tp) {
                const float pv[8] = {p[2 * tp][0], p[2 * tp][1], p[2 * tp][2], p[2 * tp][3],
                                     p[2 * tp + 1][0], p[2 * tp + 1][1], p[2 * tp + 1][2], p[2 * tp + 1][3]};
                const bf16x8 pb = pack8(pv);
                const bf16_t *vp = Vs + (32 * tp + 4 * g + i / 4) * XP + HD * hh + 4 * (i % 4);
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const u32x2 v0 = __builtin_bit_cast(u32x2, lds_read_tr16(vp + 16 * dt));
                    const u32x2 v1 = __builtin_bit_cast(u32x2, lds_read_tr16(vp + 16 * XP + 16 * dt));
                    acc[hh][dt] = mfma16(__builtin_bit_cast(bf16x8, u32x4{v0[0], v0[1], v1[0], v1[1]}), pb,
                                         acc[hh][dt]);
                }
            }
        }
    }
    if (slot < n) {
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) {
            const float inv = 1.0f / l[hh];
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                *(u32x2 *)(O + img_off + qtok * C + HD * hh + 16 * dt + 4 * g) = pack4(acc[hh][dt] * inv);
        }
    }
}

struct WideWs {
    bf16_t *q, *k, *v, *o;
    float *xr, *qr, *kr;
    int32_t *ir;
    size_t bytes;
};

bool many_regions(const Dims &D) { return D.S > kFastRouteMaxS; }

WideWs carve(const Dims &D, void *ws)
{
    WideWs w;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    const size_t tok = (size_t)D.B * D.N, reg = (size_t)D.B * D.R;
    w.q = (bf16_t *)take(tok * D.C * 2);
    w.k = (bf16_t *)take(tok * D.C * 2);
    w.v = (bf16_t *)take(tok * D.C * 2);
    w.o = (bf16_t *)take(tok * D.C * 2);
    w.xr = (float *)take(reg * D.C * 4);
    w.qr = (float *)take(reg * D.C * 4);
    w.kr = (float *)take(reg * D.C * 4);
    w.ir = (int32_t *)take(reg * D.k * 4);
    w.bytes = off;
    return w;
}

template <bool SPLIT, bool F32OUT, int CW>
int launch_gemm_tile(const void *In, const bf16_t *W, int ldw, long M, int K, int Nout, GemmOut out, int kernel_id,
                     hipStream_t st)
{
    static bool opted = false;
    if (!opted) {
        if (hipFuncSetAttribute((const void *)k_gemm<SPLIT, F32OUT, CW>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)gemm_smem(SPLIT, CW)) != hipSuccess)
            return BRA_ERR_LAUNCH;
        opted = true;
    }
    const long grid = ((M + 63) / 64) * ((Nout + 32 * CW - 1) / (32 * CW));
    ProfScope ps(st, kernel_id);
    hipLaunchKernelGGL((k_gemm<SPLIT, F32OUT, CW>), dim3((unsigned)grid), dim3(256), gemm_smem(SPLIT, CW), st, In, W,
                       ldw, (int)M, K, Nout, out);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

template <bool SPLIT, bool F32OUT = SPLIT>
int launch_gemm(const void *In, const bf16_t *W, int ldw, long M, int K, int Nout, GemmOut out, int kernel_id,
                hipStream_t st)
{
    // 64 x 64 tiles (twice the workgroups, six wavefronts per SIMD instead of four) where 64 x 128
    // tiles would leave the chip under-filled; measured: the narrow tile wins below a few hundred
    // wide tiles and loses above about a thousand
    static const long narrow_below = experiment_value("BRA_GEMM_NARROW", 400);
    // (and where the output is at most 64 columns wide: half of a wide tile would be idle)
    if (Nout <= 64 || ((M + 63) / 64) * ((Nout + 127) / 128) < narrow_below)
        return launch_gemm_tile<SPLIT, F32OUT, 2>(In, W, ldw, M, K, Nout, out, kernel_id, st);
    return launch_gemm_tile<SPLIT, F32OUT, 4>(In, W, ldw, M, K, Nout, out, kernel_id, st);
}

// A^r rows and top-k from the float32 Q^r, K^r in the workspace.
int affinity_steps(const Dims &D, const WideWs &w, int32_t *Ir, float *Ar_opt, hipStream_t st)
{
    if (many_regions(D)) return valu_affinity_topk(D, w.qr, w.kr, Ir, Ar_opt, st);   // more than one entry per lane
    ProfScope ps(st, K_MFMA_ROUTE_ROWS);
    // 16 query regions per workgroup when that already fills the chip, else 8 or 4
    const long wgs16 = (long)D.B * ((D.R + 15) / 16);
    if (wgs16 >= 1024)
        hipLaunchKernelGGL(k_route_qk<4>, dim3((unsigned)wgs16), dim3(256), 0, st, w.qr, w.kr, Ir, Ar_opt, D);
    else if (2 * wgs16 >= 1024)
        hipLaunchKernelGGL(k_route_qk<2>, dim3(D.B * ((D.R + 7) / 8)), dim3(256), 0, st, w.qr, w.kr, Ir, Ar_opt, D);
    else
        hipLaunchKernelGGL(k_route_qk<1>, dim3(D.B * ((D.R + 3) / 4)), dim3(256), 0, st, w.qr, w.kr, Ir, Ar_opt, D);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

// Pooling, region-level projections, A^r rows and top-k.
int route_steps(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, const WideWs &w, int32_t *Ir, float *Ar_opt,
                hipStream_t st)
{
    if (D.n == 1) {
        // one token per region: the means are the (bf16) tokens themselves, so Q^r | K^r is the
        // plain projection of X with float32 results: no pooling, no split
        const int rc = launch_gemm<false, true>(X, Wqkv, 3 * D.C, (long)D.B * D.R, D.C, 2 * D.C,
                                                GemmOut{{w.qr, w.kr, nullptr}, D.C, {nullptr, nullptr}}, K_MFMA_ROUTE_ROWS, st);
        if (rc != BRA_OK) return rc;
        return affinity_steps(D, w, Ir, Ar_opt, st);
    }
    {
        int sub = 1;                                           // lanes per (region, chunk)
        while (sub < 8 && 2 * sub <= D.n) sub *= 2;
        const long items = (long)D.B * D.R * (D.C / 8) * sub;
        ProfScope ps(st, K_MFMA_POOL_QK);
        hipLaunchKernelGGL(k_pool_wide, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, X, w.xr, D, sub);
    }
    const int rc = launch_gemm<true>(w.xr, Wqkv, 3 * D.C, (long)D.B * D.R, D.C, 2 * D.C, GemmOut{{w.qr, w.kr, nullptr}, D.C, {nullptr, nullptr}},
                                     K_MFMA_ROUTE_ROWS, st);
    if (rc != BRA_OK) return rc;
    return affinity_steps(D, w, Ir, Ar_opt, st);
}

}  // namespace

int gemm_bf16(const bf16_t *In, const bf16_t *W, long M, int K, int Nout, bf16_t *Out, const float *bias,
              const bf16_t *res, bool gelu, int kernel_id, hipStream_t st)
{
    if (M < 1 || M > 0x7fffffffL || K < 64 || K % 64 || Nout < 8 || Nout % 8) return BRA_ERR_UNSUPPORTED;
    GemmOut out{{Out, nullptr, nullptr}, Nout, {nullptr, nullptr}, bias, res, gelu ? 1 : 0};
    return launch_gemm<false>(In, W, Nout, M, K, Nout, out, kernel_id, st);
}

// Q, K, V = X Wqkv into three token maps (Eq. 3) for any C that is a multiple of 64: the projection of
// the wide pipeline, for the backward pass.
int wide_project_qkv(const Dims &D, const void *X, const void *Wqkv, bf16_t *Q, bf16_t *K, bf16_t *V, hipStream_t st)
{
    const long M = (long)D.B * D.N;
    if (D.C % 64 || M > 0x7fffffffL) return BRA_ERR_UNSUPPORTED;
    return launch_gemm<false>(X, (const bf16_t *)Wqkv, 3 * D.C, M, D.C, 3 * D.C,
                              GemmOut{{Q, K, V}, D.C, {nullptr, nullptr}}, K_MFMA_QKV, st);
}

bool wide_supported(const Dims &D)
{
    if (D.dtype != BRA_BF16 || D.C % 64 != 0 || D.C > 4096) return false;
    if (D.d != 32 && D.d != 64) return false;
    if (many_regions(D) && !generic_supported(D)) return false;               // top-k by the generic kernel
    if (((long)D.B * D.N + 63) / 64 * ((3L * D.C + 127) / 128) > 0x7fffffffL) return false;
    if ((long)D.B * D.R * ((D.n + 63) / 64) * (D.C / 64) > 0x7fffffffL) return false;
    return true;
}

size_t wide_workspace_bytes(const Dims &D) { return carve(D, nullptr).bytes; }

int wide_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt, void *ws,
               hipStream_t st)
{
    const WideWs w = carve(D, ws);
    return route_steps(D, (const bf16_t *)X, (const bf16_t *)Wqkv, w, Ir, Ar_opt, st);
}

int wide_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce, void *Y,
                 int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st)
{
    const WideWs w = carve(D, ws);
    const int32_t *Ir_src = Ir_in_opt;
    int32_t *Ir_dst = Ir_out_opt ? Ir_out_opt : w.ir;
    // one token per region: Q^r, K^r are Q, K before their rounding to bf16, which the token
    // projection leaves as float32 copies; the routing then follows the projection
    const bool route_after = !Ir_in_opt && D.n == 1;
    if (!Ir_in_opt && !route_after) {
        const int rc = route_steps(D, (const bf16_t *)X, (const bf16_t *)Wqkv, w, Ir_dst, nullptr, st);
        if (rc != BRA_OK) return rc;
        Ir_src = Ir_dst;
    }
    const long M = (long)D.B * D.N;
    float *fq = route_after ? w.qr : nullptr, *fk = route_after ? w.kr : nullptr;
    int rc = launch_gemm<false>(X, (const bf16_t *)Wqkv, 3 * D.C, M, D.C, 3 * D.C, GemmOut{{w.q, w.k, w.v}, D.C, {fq, fk}}, K_MFMA_QKV, st);
    if (rc != BRA_OK) return rc;
    if (route_after) {
        rc = affinity_steps(D, w, Ir_dst, nullptr, st);
        if (rc != BRA_OK) return rc;
        Ir_src = Ir_dst;
    }
    AttnArgs A = {};
    A.X = (const bf16_t *)X; A.Q = w.q; A.K = w.k; A.V = w.v;
    A.Ir_src = Ir_src; A.Ir_out = Ir_out_opt; A.Wlce = (const bf16_t *)Wlce; A.Y = (bf16_t *)Y;
    A.c_exp = D.scale * 1.4426950408889634f;
    if (map_tail_supported(D)) {
        rc = launch_map_tail(D, A, w.o, st);
    } else {
        {
            const unsigned grid = (unsigned)((long)D.B * D.R * ((D.n + 63) / 64) * (D.C / 64));
            ProfScope ps(st, K_MFMA_ATTENTION);
            if (D.d == 32) hipLaunchKernelGGL(k_attn_gen<32>, dim3(grid), dim3(256), 0, st, A, w.o, D);
            else hipLaunchKernelGGL(k_attn_gen<64>, dim3(grid), dim3(256), 0, st, A, w.o, D);
        }
        rc = launch_lce_add_any(D, A, w.o, st);
    }
    if (rc != BRA_OK) return rc;
    return launch_gemm<false>(w.o, (const bf16_t *)Wo, D.C, M, D.C, D.C, GemmOut{{Y, nullptr, nullptr}, D.C, {nullptr, nullptr}}, K_MFMA_WO, st);
}

}  // namespace bra
