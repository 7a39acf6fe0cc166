// Generic kernel family: scalar (VALU) float32 arithmetic, any valid shape.
//
// Used for float32 tensors and for shapes the matrix-core kernels are not built
// for.  All intermediates (Q, K, V, attention output) are kept in float32 in the
// workspace, whatever the storage type of X and Y.  The steps follow Sec. 3.2:
// projection (Eq. 3), region pooling + affinity (Eq. 4), top-k (Eq. 5), routed
// attention straight from the index (Eq. 6-7, no gathered tensor), LCE, W^o (Eq. 2).
// Region pooling uses mean(X^r) W = mean(X^r W), which is exact in real arithmetic
// (the mean is linear; same argument as Appendix A).
#include "bra_common.h"
#include <type_traits>

#include <math.h>

namespace bra {

namespace {

constexpr int kWave = 64;
constexpr int kTopkSlots = 16;      // affinity values per lane: R <= 64 * 16
constexpr int kAttnChunk = 1024;    // keys per online-softmax chunk
constexpr int kAttnMaxD = 256;      // head width limit of the generic attention kernel

// ---------------------------------------------------------------------------
// out[M, N] = A[M, K] * Bm[K, N]  (row-major with leading dimensions), float32 FMA,
// k ascending.  64 x 64 tile per workgroup, 4 x 4 outputs per thread.
// BT: B is read transposed (B[k][n] = Bm[n * ldb + k]).
template <typename TA, typename TB, typename TO, bool BT = false>
__global__ __launch_bounds__(256) void gen_gemm(const TA *__restrict__ A, int lda,
                                                const TB *__restrict__ Bm, int ldb,
                                                TO *__restrict__ Out, int ldo, int M, int N, int K,
                                                const float *__restrict__ bias = nullptr,
                                                const TO *__restrict__ res = nullptr, int gelu = 0)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const long m0 = (long)blockIdx.x * 64;
    const int n0 = blockIdx.y * 64;
    float acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    // the next 16-deep slice is requested while the current one is multiplied
    float ra[4], rb[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + i * 256;
            const int r = idx / 16, kk = idx % 16;
            const long gm = m0 + r;
            ra[i] = (gm < M && k0 + kk < K) ? load_f32(A + gm * lda + k0 + kk) : 0.f;
            const int kb = idx / 64, nn = idx % 64;
            rb[i] = (k0 + kb < K && n0 + nn < N)
                        ? load_f32(BT ? Bm + (long)(n0 + nn) * ldb + k0 + kb : Bm + (long)(k0 + kb) * ldb + n0 + nn)
                        : 0.f;
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + i * 256;
            As[idx % 16][idx / 16] = ra[i];
            Bs[idx / 64][idx % 64] = rb[i];
        }
        __syncthreads();
        if (k0 + 16 < K) fetch(k0 + 16);
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        long gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
        for (int j = 0; j < 4; ++j) {
            int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            // optional epilogue: + bias[column], GELU, + res[row][column] (the layout of Out)
            float v = acc[i][j];
            if (bias) v += bias[gn];
            if (gelu) v = gelu_f32(v);
            if (res) v += load_f32(res + gm * ldo + gn);
            store_from_f32(Out + gm * ldo + gn, v);
        }
    }
}

// ---------------------------------------------------------------------------
// Xr[b, r, c] = mean over the n tokens of region r of X[b, :, :, c]; tokens are
// summed in row-major order inside the region; one workgroup per (b, r),
// and Qr[b, r, :] = Xr[b, r, :] Wq, Kr[b, r, :] = Xr[b, r, :] Wk from the means in LDS (Sec. 3.2).
template <typename T>
__global__ void gen_pool_qk(const T *__restrict__ X, const T *__restrict__ Wqkv, float *__restrict__ Xr,
                            float *__restrict__ Qr, float *__restrict__ Kr, Dims D)
{
    extern __shared__ float xs[];
    const int b = blockIdx.x / D.R, r = blockIdx.x % D.R;
    const size_t row = blockIdx.x;
    const int y0 = (r / D.S) * D.rh, x0 = (r % D.S) * D.rw;
    const T *img = X + (size_t)b * D.N * D.C;
    for (int c = threadIdx.x; c < D.C; c += blockDim.x) {
        float s = 0.f;
        for (int ry = 0; ry < D.rh; ++ry)
            for (int rx = 0; rx < D.rw; ++rx)
                s += load_f32(img + ((size_t)(y0 + ry) * D.W + x0 + rx) * D.C + c);
        xs[c] = s / (float)D.n;
        Xr[row * D.C + c] = xs[c];
    }
    __syncthreads();
    for (int o = threadIdx.x; o < 2 * D.C; o += blockDim.x) {
        float acc = 0.f;
        for (int c = 0; c < D.C; ++c) acc = fmaf(xs[c], load_f32(Wqkv + (size_t)c * 3 * D.C + o), acc);
        if (o < D.C) Qr[row * D.C + o] = acc;
        else Kr[row * D.C + o - D.C] = acc;
    }
}

// One wavefront per (b, i): row i of A^r = Q^r (K^r)^T (Eq. 4), then k rounds of a
// wave-wide arg-max (Eq. 5).  Order: larger value first, equal values by smaller
// index; NaN counts as -inf so that the k indices are always distinct and valid.
__global__ __launch_bounds__(kWave) void gen_affinity_topk(const float *__restrict__ Qr,
                                                           const float *__restrict__ Kr,
                                                           int32_t *__restrict__ Ir,
                                                           float *__restrict__ Ar_opt, Dims D)
{
    extern __shared__ float qs[];
    const int b = blockIdx.x / D.R, i = blockIdx.x % D.R;
    const int lane = threadIdx.x;
    for (int c = lane; c < D.C; c += kWave) qs[c] = Qr[((size_t)b * D.R + i) * D.C + c];
    __syncthreads();
    float vals[kTopkSlots];
#pragma unroll
    for (int t = 0; t < kTopkSlots; ++t) {
        const int j = lane + t * kWave;
        float a = -INFINITY;
        if (j < D.R) {
            const float *kr = Kr + ((size_t)b * D.R + j) * D.C;
            a = 0.f;
            for (int c = 0; c < D.C; ++c) a = fmaf(qs[c], kr[c], a);
            if (Ar_opt) Ar_opt[((size_t)b * D.R + i) * D.R + j] = a;
            if (!(a == a)) a = -INFINITY;
        }
        vals[t] = a;
    }
    unsigned taken = 0;  // bit t: slot t of this lane already selected
    for (int p = 0; p < D.k; ++p) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < kTopkSlots; ++t) {
            const int j = lane + t * kWave;
            if (j < D.R && !((taken >> t) & 1u)) {
                if (bi == 0x7fffffff || vals[t] > bv) { bv = vals[t]; bi = j; }
            }
        }
        for (int off = 32; off >= 1; off >>= 1) {
            float ov = __shfl_xor(bv, off, kWave);
            int oi = __shfl_xor(bi, off, kWave);
            bool take = (oi != 0x7fffffff) && (bi == 0x7fffffff || ov > bv || (ov == bv && oi < bi));
            if (take) { bv = ov; bi = oi; }
        }
        if (bi % kWave == lane) taken |= 1u << (bi / kWave);
        if (lane == 0) Ir[((size_t)b * D.R + i) * D.k + p] = bi;
    }
}

// Routed attention (Eq. 6, Eq. 1) for heads of at most 64 channels, with the keys staged in
// LDS; QKV is [B, N, 3C] float32 (q | k | v per token).
// Workgroup (b, region, head) takes its queries 16 at a time (4 per wavefront) and, per pass,
// the routed keys 64 at a time: K and V rows of the block are copied into LDS with
// consecutive lanes on consecutive channels, then lane u scores key u against each of the
// wavefront's queries (Eq. 1, scaled), the online softmax state of a query lives in
// registers, and lane c accumulates channel c of P V.
constexpr int kAttnLdsD = 64;

__global__ __launch_bounds__(256) void gen_attention_lds(const float *__restrict__ QKV,
                                                         const int32_t *__restrict__ Ir,
                                                         float *__restrict__ O, Dims D, float scale)
{
    __shared__ float Ks[64][kAttnLdsD + 1];
    __shared__ float Vs[64][kAttnLdsD + 1];
    __shared__ float qs[16][kAttnLdsD];
    __shared__ float sc[16][64];
    const int hd = blockIdx.x % D.heads;
    const int reg = (blockIdx.x / D.heads) % D.R;
    const int b = blockIdx.x / (D.heads * D.R);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int C3 = 3 * D.C, d = D.d;
    const float *img = QKV + (size_t)b * D.N * C3;
    const int32_t *irp = Ir + ((size_t)b * D.R + reg) * D.k;
    const int y0 = (reg / D.S) * D.rh, x0 = (reg % D.S) * D.rw;

    for (int s0 = 0; s0 < D.n; s0 += 16) {
        // the 16 queries of this pass (past the end: the last one again; never stored)
        for (int e = tid; e < 16 * d; e += 256) {
            const int s = min(s0 + e / d, D.n - 1);
            const int qtok = (y0 + s / D.rw) * D.W + x0 + s % D.rw;
            qs[e / d][e % d] = img[(size_t)qtok * C3 + hd * d + e % d];
        }
        float m[4], l[4], acc[4];
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            m[qq] = -INFINITY;
            l[qq] = 0.f;
            acc[qq] = 0.f;
        }
        for (int k0 = 0; k0 < D.kn; k0 += 64) {
            const int cn = min(64, D.kn - k0);
            __syncthreads();               // queries staged; the previous block has been read
            for (int e = tid; e < 64 * d; e += 256) {
                const int u = e / d, c = e % d;
                const int key = min(k0 + u, D.kn - 1);
                const int j = region_index(irp[key / D.n], D.R), slot = key % D.n;
                const int tok = ((j / D.S) * D.rh + slot / D.rw) * D.W + (j % D.S) * D.rw + slot % D.rw;
                const float *row = img + (size_t)tok * C3 + hd * d + c;
                Ks[u][c] = row[D.C];
                Vs[u][c] = row[2 * D.C];
            }
            __syncthreads();
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const float *q = qs[4 * wave + qq];
                float a = 0.f;
                for (int c = 0; c < d; ++c) a = fmaf(q[c], Ks[lane][c], a);
                a = lane < cn ? a * scale : -INFINITY;
                float mx = a;
                for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
                const float m_new = fmaxf(m[qq], mx);
                const float corr = (m[qq] == -INFINITY) ? 0.f : expf(m[qq] - m_new);
                const float pv = lane < cn ? expf(a - m_new) : 0.f;
                float ls = pv;
                for (int off = 32; off >= 1; off >>= 1) ls += __shfl_xor(ls, off, kWave);
                l[qq] = l[qq] * corr + ls;
                m[qq] = m_new;
                sc[4 * wave + qq][lane] = pv;      // read back by this wavefront only
                float o = acc[qq] * corr;
                if (lane < d)
                    for (int u = 0; u < cn; ++u) o = fmaf(sc[4 * wave + qq][u], Vs[u][lane], o);
                acc[qq] = o;
            }
        }
        __syncthreads();                   // the next pass replaces the queries
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            const int s = s0 + 4 * wave + qq;
            if (s < D.n && lane < d) {
                const int qtok = (y0 + s / D.rw) * D.W + x0 + s % D.rw;
                O[((size_t)b * D.N + qtok) * D.C + hd * d + lane] = acc[qq] / l[qq];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Routed attention for wider heads, one workgroup (4 wavefronts) per (b, region i, head).  Each
// wavefront owns one query at a time and runs an online softmax over the k n keys
// of regions Ir[b, i, :] in chunks; keys and values are read in place from the
// projected map by index.  QKV is [B, N, 3C] float32 (q | k | v per token).
__global__ __launch_bounds__(256) void gen_attention(const float *__restrict__ QKV,
                                                     const int32_t *__restrict__ Ir,
                                                     float *__restrict__ O, Dims D, float scale)
{
    __shared__ float qs[4][kAttnMaxD];
    __shared__ float sc[4][kAttnChunk];
    __shared__ int tk[4][kAttnChunk];
    extern __shared__ int regs[];  // k routed regions

    const int hd = blockIdx.x % D.heads;
    const int i = (blockIdx.x / D.heads) % D.R;
    const int b = blockIdx.x / (D.heads * D.R);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int C3 = 3 * D.C;
    const float *img = QKV + (size_t)b * D.N * C3;

    for (int p = threadIdx.x; p < D.k; p += blockDim.x) regs[p] = region_index(Ir[((size_t)b * D.R + i) * D.k + p], D.R);
    __syncthreads();

    const int y0 = (i / D.S) * D.rh, x0 = (i % D.S) * D.rw;
    const int iters = (D.n + 3) / 4;
    for (int it = 0; it < iters; ++it) {
        const int s = it * 4 + wave;
        const bool active = s < D.n;
        int qtok = 0;
        if (active) {
            qtok = (y0 + s / D.rw) * D.W + x0 + s % D.rw;
            for (int c = lane; c < D.d; c += kWave) qs[wave][c] = img[(size_t)qtok * C3 + hd * D.d + c];
        }
        float m = -INFINITY, l = 0.f;
        float acc[kAttnMaxD / kWave];
        for (int t = 0; t < kAttnMaxD / kWave; ++t) acc[t] = 0.f;
        __syncthreads();
        for (int c0 = 0; c0 < D.kn; c0 += kAttnChunk) {
            const int cn = min(kAttnChunk, D.kn - c0);
            float lm = -INFINITY;
            if (active) {
                for (int u = lane; u < cn; u += kWave) {
                    const int g = c0 + u;
                    const int j = regs[g / D.n], slot = g % D.n;
                    const int tok = ((j / D.S) * D.rh + slot / D.rw) * D.W + (j % D.S) * D.rw + slot % D.rw;
                    const float *kr = img + (size_t)tok * C3 + D.C + hd * D.d;
                    float a = 0.f;
                    for (int c = 0; c < D.d; ++c) a = fmaf(qs[wave][c], kr[c], a);
                    a *= scale;
                    sc[wave][u] = a;
                    tk[wave][u] = tok;
                    lm = fmaxf(lm, a);
                }
            }
            for (int off = 32; off >= 1; off >>= 1) lm = fmaxf(lm, __shfl_xor(lm, off, kWave));
            const float m_new = fmaxf(m, lm);
            const float corr = (m == -INFINITY) ? 0.f : expf(m - m_new);
            float ls = 0.f;
            if (active) {
                for (int u = lane; u < cn; u += kWave) {
                    float pv = expf(sc[wave][u] - m_new);
                    sc[wave][u] = pv;
                    ls += pv;
                }
            }
            for (int off = 32; off >= 1; off >>= 1) ls += __shfl_xor(ls, off, kWave);
            l = l * corr + ls;
            m = m_new;
            __syncthreads();
            if (active) {
                for (int t = 0; t < kAttnMaxD / kWave; ++t) {
                    const int c = lane + t * kWave;
                    if (c < D.d) {
                        float a = acc[t] * corr;
                        for (int u = 0; u < cn; ++u)
                            a = fmaf(sc[wave][u], img[(size_t)tk[wave][u] * C3 + 2 * D.C + hd * D.d + c], a);
                        acc[t] = a;
                    }
                }
            }
            __syncthreads();
        }
        if (active) {
            for (int t = 0; t < kAttnMaxD / kWave; ++t) {
                const int c = lane + t * kWave;
                if (c < D.d) O[((size_t)b * D.N + qtok) * D.C + hd * D.d + c] = acc[t] / l;
            }
        }
    }
}

// O[b, y, x, c] += sum_{ky,kx} Wlce[c, ky, kx] * V[b, y+ky-2, x+kx-2, c], V = 0 outside.
template <typename T>
__global__ void gen_lce_add(const float *__restrict__ QKV, const T *__restrict__ Wlce,
                            float *__restrict__ O, Dims D)
{
    const size_t total = (size_t)D.B * D.N * D.C;
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int c = e % D.C;
    const size_t t = e / D.C;
    const int x = t % D.W, y = (t / D.W) % D.H;
    const size_t b = t / D.N;
    const float *img = QKV + b * D.N * 3 * D.C + 2 * D.C + c;
    float acc = 0.f;
    for (int ky = 0; ky < 5; ++ky) {
        const int yy = y + ky - 2;
        if (yy < 0 || yy >= D.H) continue;
        for (int kx = 0; kx < 5; ++kx) {
            const int xx = x + kx - 2;
            if (xx < 0 || xx >= D.W) continue;
            acc = fmaf(load_f32(Wlce + (c * 5 + ky) * 5 + kx), img[((size_t)yy * D.W + xx) * 3 * D.C], acc);
        }
    }
    O[e] += acc;
}

struct GenericWs {
    float *qkv, *o, *xr, *qr, *kr;
    int32_t *ir;
    size_t bytes;
};

GenericWs carve(const Dims &D, void *ws)
{
    GenericWs w;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    const size_t tok = (size_t)D.B * D.N, reg = (size_t)D.B * D.R;
    w.qkv = (float *)take(tok * 3 * D.C * sizeof(float));
    w.o = (float *)take(tok * D.C * sizeof(float));
    w.xr = (float *)take(reg * D.C * sizeof(float));
    w.qr = (float *)take(reg * D.C * sizeof(float));
    w.kr = (float *)take(reg * D.C * sizeof(float));
    w.ir = (int32_t *)take(reg * D.k * sizeof(int32_t));
    w.bytes = off;
    return w;
}

template <typename T>
void launch_route(const Dims &D, const T *X, const T *Wqkv, int32_t *Ir, float *Ar_opt,
                  const GenericWs &w, hipStream_t st)
{
    const int regs = D.B * D.R;
    {
        ProfScope ps(st, K_GEN_POOL);
        hipLaunchKernelGGL(gen_pool_qk<T>, dim3(regs), dim3(256), D.C * sizeof(float), st, X, Wqkv, w.xr, w.qr, w.kr, D);
    }
    {
        ProfScope ps(st, K_GEN_TOPK);
        hipLaunchKernelGGL(gen_affinity_topk, dim3(regs), dim3(kWave), D.C * sizeof(float), st, w.qr,
                           w.kr, Ir, Ar_opt, D);
    }
}

template <typename T>
int forward_t(const Dims &D, const T *X, const T *Wqkv, const T *Wo, const T *Wlce, T *Y,
              int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st)
{
    GenericWs w = carve(D, ws);
    if constexpr (std::is_same<T, float>::value) {
        if (f32_small_ok(D))
            return f32_small_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, w.qkv, w.qr, w.kr, st);
    }
    const long M = (long)D.B * D.N;
    const int32_t *Ir = Ir_in_opt;
    if (!Ir_in_opt) {
        int32_t *dst = Ir_out_opt ? Ir_out_opt : w.ir;
        launch_route<T>(D, X, Wqkv, dst, nullptr, w, st);
        Ir = dst;
    } else if (Ir_out_opt) {
        if (hipMemcpyAsync(Ir_out_opt, Ir_in_opt, sizeof(int32_t) * (size_t)D.B * D.R * D.k,
                           hipMemcpyDeviceToDevice, st) != hipSuccess)
            return BRA_ERR_LAUNCH;
    }
    dim3 g1((unsigned)((M + 63) / 64), (unsigned)((3 * D.C + 63) / 64));
    {
        ProfScope ps(st, K_GEN_GEMM_QKV);
        hipLaunchKernelGGL((gen_gemm<T, T, float>), g1, dim3(256), 0, st, X, D.C, Wqkv, 3 * D.C, w.qkv,
                           3 * D.C, (int)M, 3 * D.C, D.C);
    }
    {
        ProfScope ps(st, K_GEN_ATTENTION);
        if (D.d <= kAttnLdsD)
            hipLaunchKernelGGL(gen_attention_lds, dim3(D.B * D.R * D.heads), dim3(256), 0, st, w.qkv, Ir, w.o, D,
                               D.scale);
        else
            hipLaunchKernelGGL(gen_attention, dim3(D.B * D.R * D.heads), dim3(256), D.k * sizeof(int), st,
                               w.qkv, Ir, w.o, D, D.scale);
    }
    const size_t total = (size_t)M * D.C;
    {
        ProfScope ps(st, K_GEN_LCE);
        hipLaunchKernelGGL(gen_lce_add<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           w.qkv, Wlce, w.o, D);
    }
    dim3 g2((unsigned)((M + 63) / 64), (unsigned)((D.C + 63) / 64));
    {
        ProfScope ps(st, K_GEN_GEMM_WO);
        hipLaunchKernelGGL((gen_gemm<float, T, T>), g2, dim3(256), 0, st, w.o, D.C, Wo, D.C, Y, D.C,
                           (int)M, D.C, D.C);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------
// Whole block (Sec. 3.4) with scalar kernels.  One wavefront per token; lane l owns channels
// l, l + 64, ..  POS: Sum = A + DWConv3x3(A) + bpos (cross-correlation, zero padding 1);
// otherwise Sum = A + Badd.  Norm = LayerNorm(Sum) over the token's C channels from the
// float32 values (biased variance, eps inside the root), which wait in LDS between the passes.
template <typename T, bool POS>
__global__ __launch_bounds__(256) void gen_token_ln(const T *A, const T *__restrict__ Badd, const T *__restrict__ Wpos,
                                                    const float *__restrict__ bpos, const float *__restrict__ gamma,
                                                    const float *__restrict__ beta, T *Sum, T *__restrict__ Norm,
                                                    int H, int W, int C, long tokens, float eps)
{
    extern __shared__ float strips[];                 // [4 wavefronts][C]
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    float *strip = strips + (size_t)wave * C;
    const long tok = (long)blockIdx.x * 4 + wave;
    if (tok >= tokens) return;                        // whole wavefronts leave; no barrier follows
    const int x = (int)(tok % W), y = (int)((tok / W) % H);
    const T *centre = A + (size_t)tok * C;
    float s = 0.f;
    for (int c = lane; c < C; c += kWave) {
        float v = load_f32(centre + c);
        if (POS) {
            float acc = v + bpos[c];
            for (int ky = 0; ky < 3; ++ky) {
                const int yy = y + ky - 1;
                if (yy < 0 || yy >= H) continue;
                for (int kx = 0; kx < 3; ++kx) {
                    const int xx = x + kx - 1;
                    if (xx < 0 || xx >= W) continue;
                    acc = fmaf(load_f32(Wpos + (size_t)c * 9 + 3 * ky + kx),
                               load_f32(centre + ((long)(ky - 1) * W + (kx - 1)) * C + c), acc);
                }
            }
            v = acc;
        } else {
            v += load_f32(Badd + (size_t)tok * C + c);
        }
        strip[c] = v;
        s += v;
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    const float mean = s / (float)C;
    float q = 0.f;
    for (int c = lane; c < C; c += kWave) { const float d = strip[c] - mean; q = fmaf(d, d, q); }
    for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off);
    const float rstd = 1.0f / sqrtf(q / (float)C + eps);
    for (int c = lane; c < C; c += kWave) {
        const float v = strip[c];
        store_from_f32(Sum + (size_t)tok * C + c, v);             // may overwrite A: this lane has read it
        store_from_f32(Norm + (size_t)tok * C + c, fmaf((v - mean) * rstd, gamma[c], beta[c]));
    }
}

struct GenBlockWs {
    void *x1, *xn, *y, *hd, *inner;
    size_t bytes;
};

GenBlockWs carve_gen_block(const Dims &D, int hidden, size_t bra_bytes, void *ws)
{
    char *base = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *ptr = base ? base + off : nullptr;
        off += align256(bytes);
        return ptr;
    };
    const size_t es = D.dtype == BRA_BF16 ? 2 : 4, tokens = (size_t)D.B * D.N;
    GenBlockWs w;
    w.x1 = take(tokens * D.C * es);
    w.xn = take(tokens * D.C * es);
    w.y = take(tokens * D.C * es);
    w.hd = take(tokens * hidden * es);
    w.inner = take(bra_bytes);
    w.bytes = off;
    return w;
}

template <typename T>
int block_t(const Dims &D, int hidden, float eps, const T *X, const bra_block_params &p, T *Xout, int32_t *Ir_out_opt,
            const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path, hipStream_t st)
{
    const GenBlockWs w = carve_gen_block(D, hidden, bra_bytes, ws);
    T *x1 = (T *)w.x1, *xn = (T *)w.xn, *y = (T *)w.y, *hd = (T *)w.hd;
    const long M = (long)D.B * D.N;
    const unsigned tgrid = (unsigned)((M + 3) / 4);
    const size_t strip = (size_t)4 * D.C * sizeof(float);
    {
        ProfScope ps(st, K_BLK_POS_LN);
        hipLaunchKernelGGL((gen_token_ln<T, true>), dim3(tgrid), dim3(256), strip, st, X, (const T *)nullptr,
                           (const T *)p.Wpos, p.bpos, p.ln1_gamma, p.ln1_beta, x1, xn, D.H, D.W, D.C, M, eps);
    }
    if (hipGetLastError() != hipSuccess) return BRA_ERR_LAUNCH;
    int rc = (path == BRA_PATH_MFMA)
                 ? mfma_forward(D, xn, p.Wqkv, p.Wo, p.Wlce, y, Ir_out_opt, Ir_in_opt, w.inner, st)
                 : generic_forward(D, xn, p.Wqkv, p.Wo, p.Wlce, y, Ir_out_opt, Ir_in_opt, w.inner, st);
    if (rc != BRA_OK) return rc;
    {
        ProfScope ps(st, K_BLK_ADD_LN);
        hipLaunchKernelGGL((gen_token_ln<T, false>), dim3(tgrid), dim3(256), strip, st, x1, y, (const T *)nullptr,
                           (const float *)nullptr, p.ln2_gamma, p.ln2_beta, x1, xn, D.H, D.W, D.C, M, eps);
    }
    {
        ProfScope ps(st, K_BLK_MLP_IN);
        dim3 g((unsigned)((M + 63) / 64), (unsigned)((hidden + 63) / 64));
        hipLaunchKernelGGL((gen_gemm<T, T, T>), g, dim3(256), 0, st, xn, D.C, (const T *)p.W1, hidden, hd, hidden,
                           (int)M, hidden, D.C, p.b1, (const T *)nullptr, 1);
    }
    {
        ProfScope ps(st, K_BLK_MLP_OUT);
        dim3 g((unsigned)((M + 63) / 64), (unsigned)((D.C + 63) / 64));
        hipLaunchKernelGGL((gen_gemm<T, T, T>), g, dim3(256), 0, st, hd, hidden, (const T *)p.W2, D.C, Xout, D.C,
                           (int)M, D.C, hidden, p.b2, x1, 0);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

// ---------------------------------------------------------------------------
// Backward pass with fixed routing (the top-k of Eq. 5 has no derivative), scalar kernels.
// With dO = dY Wo^T and, per query token t of region i and head h, P = softmax over the keys G_i:
//   dP_j = dO_h[t] . V_h[j],  dS_j = P_j (dP_j - sum_u P_u dP_u),
//   dQ_h[t] = scale sum_j dS_j K_h[j],  dK_h[j] += scale dS_j Q_h[t],  dV_h[j] += P_j dO_h[t].

__global__ void gen_fill_zero(float *__restrict__ p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.f;
}

// Out[i][j] += sum_m A[m][i] B[m][j] over this workgroup's slice of the rows m (atomic adds into
// float32 Out [KA][N], zeroed beforehand): the weight gradients, a contraction over all tokens.
template <typename TA, typename TB>
__global__ __launch_bounds__(256) void gen_gemm_tn(const TA *__restrict__ A, int lda, const TB *__restrict__ Bm,
                                                   int ldb, float *__restrict__ Out, int ldo, long M, int KA, int N,
                                                   long rows_per_wg)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64];
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int i0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
    const long m_begin = (long)blockIdx.z * rows_per_wg, m_end = min(M, m_begin + rows_per_wg);
    float acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (long m0 = m_begin; m0 < m_end; m0 += 16) {
        for (int u = 0; u < 4; ++u) {
            const int idx = tid + u * 256;
            const int mm = idx / 64, cc = idx % 64;
            const long gm = m0 + mm;
            As[mm][cc] = (gm < m_end && i0 + cc < KA) ? load_f32(A + gm * lda + i0 + cc) : 0.f;
            Bs[mm][cc] = (gm < m_end && n0 + cc < N) ? load_f32(Bm + gm * ldb + n0 + cc) : 0.f;
        }
        __syncthreads();
        for (int mm = 0; mm < 16; ++mm) {
            float a[4], b[4];
            for (int i = 0; i < 4; ++i) a[i] = As[mm][ty * 4 + i];
            for (int j = 0; j < 4; ++j) b[j] = Bs[mm][tx * 4 + j];
            for (int i = 0; i < 4; ++i)
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            const int gi = i0 + ty * 4 + i, gn = n0 + tx * 4 + j;
            if (gi < KA && gn < N) unsafeAtomicAdd(Out + (size_t)gi * ldo + gn, acc[i][j]);
        }
}

// One workgroup per (image, region, head, pass of 16 queries: wavefront w owns 4 of them), the
// routed keys in blocks of 64 staged in LDS.  Sweep 1 over the key blocks: the softmax maximum and
// denominator of each query and, rescaled along with them, sum_j e_j dP_j, which gives
// D_q = sum_j P_j dP_j.  The attention output itself (needed for dWo) falls out of sweep 2.  Sweep 2: per block, a lane per key forms P_j and dS_j
// (kept in LDS for the pass's 16 queries), a lane per channel adds the query's share to dQ
// (registers), then a thread per (key, channel) sums the 16 queries' shares of dK, dV and adds them
// to memory with one atomic add each (other passes and regions route to the same keys).  LDS
// atomics for that sum were measured at about one lane per clock: eight times slower.
constexpr int kBwdMaxD = 64;

__global__ __launch_bounds__(256) void gen_attention_bwd(const float *__restrict__ QKV,
                                                         const int32_t *__restrict__ Ir,
                                                         float *__restrict__ Oatt,
                                                         const float *__restrict__ dO, float *__restrict__ dQKV,
                                                         Dims D, float scale)
{
    extern __shared__ float lds[];
    const int d = D.d, dp = d + 1;
    float *Ks = lds, *Vs = Ks + 64 * dp;
    float *qs = Vs + 64 * dp, *dos = qs + 16 * d, *Psc = dos + 16 * d, *dSsc = Psc + 16 * 64;
    const int passes = (D.n + 15) / 16;
    const int pass = blockIdx.x % passes, rest = blockIdx.x / passes;
    const int hd = rest % D.heads;
    const int reg = (rest / D.heads) % D.R;
    const int b = rest / (D.heads * D.R);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int C3 = 3 * D.C;
    const float *img = QKV + (size_t)b * D.N * C3;
    float *dimg = dQKV + (size_t)b * D.N * C3;
    const int32_t *irp = Ir + ((size_t)b * D.R + reg) * D.k;
    const int y0 = (reg / D.S) * D.rh, x0 = (reg % D.S) * D.rw;
    auto query_token = [&](int s) { return (y0 + s / D.rw) * D.W + x0 + s % D.rw; };
    auto key_token = [&](int key) {
        const int j = region_index(irp[key / D.n], D.R), slot = key % D.n;
        return ((j / D.S) * D.rh + slot / D.rw) * D.W + (j % D.S) * D.rw + slot % D.rw;
    };
    auto stage_keys = [&](int k0, bool with_v) {
        for (int e = tid; e < 64 * d; e += 256) {
            const int u = e / d, c = e % d;
            const float *row = img + (size_t)key_token(min(k0 + u, D.kn - 1)) * C3 + hd * d + c;
            Ks[u * dp + c] = row[D.C];
            if (with_v) Vs[u * dp + c] = row[2 * D.C];
        }
    };

    {
        const int s0 = 16 * pass;
        for (int e = tid; e < 16 * d; e += 256) {
            const int s = min(s0 + e / d, D.n - 1);      // past the end: the last query again; it adds nothing
            const int qtok = query_token(s);
            qs[e] = img[(size_t)qtok * C3 + hd * d + e % d];
            dos[e] = dO[((size_t)b * D.N + qtok) * D.C + hd * d + e % d];
        }
        __syncthreads();
        float m[4], l[4], Dq[4], dq[4], oa[4];
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            m[qq] = -INFINITY;
            l[qq] = 0.f;
            Dq[qq] = 0.f;          // sum_j e_j dP_j until the end of sweep 1, then divided by l
            dq[qq] = 0.f;
            oa[qq] = 0.f;
        }
        for (int k0 = 0; k0 < D.kn; k0 += 64) {        // sweep 1: maximum, denominator and sum_j e_j dP_j
            const int cn = min(64, D.kn - k0);
            __syncthreads();
            stage_keys(k0, true);
            __syncthreads();
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const float *q = qs + (4 * wave + qq) * d, *dov = dos + (4 * wave + qq) * d;
                float a = 0.f, gsum = 0.f;
                for (int c = 0; c < d; ++c) {
                    a = fmaf(q[c], Ks[lane * dp + c], a);
                    gsum = fmaf(dov[c], Vs[lane * dp + c], gsum);
                }
                a = lane < cn ? a * scale : -INFINITY;
                float mx = a;
                for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
                const float m_new = fmaxf(m[qq], mx);
                float e = lane < cn ? expf(a - m_new) : 0.f;
                float eg = e * gsum;
                for (int off = 32; off >= 1; off >>= 1) {
                    e += __shfl_xor(e, off, kWave);
                    eg += __shfl_xor(eg, off, kWave);
                }
                const float corr = (m[qq] == -INFINITY) ? 0.f : expf(m[qq] - m_new);
                l[qq] = l[qq] * corr + e;
                Dq[qq] = Dq[qq] * corr + eg;
                m[qq] = m_new;
            }
        }
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) Dq[qq] /= l[qq];
        for (int k0 = 0; k0 < D.kn; k0 += 64) {        // sweep 2: gradients
            const int cn = min(64, D.kn - k0);
            if (D.kn > 64) {                           // a single block is still in LDS from sweep 1
                __syncthreads();
                stage_keys(k0, true);
                __syncthreads();
            }
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const bool live = s0 + 4 * wave + qq < D.n;      // uniform in the wavefront
                const float *q = qs + (4 * wave + qq) * d, *dov = dos + (4 * wave + qq) * d;
                float *Pw = Psc + (4 * wave + qq) * 64, *dSw = dSsc + (4 * wave + qq) * 64;
                float a = 0.f, gsum = 0.f;
                for (int c = 0; c < d; ++c) {
                    a = fmaf(q[c], Ks[lane * dp + c], a);
                    gsum = fmaf(dov[c], Vs[lane * dp + c], gsum);
                }
                const float pj = (live && lane < cn) ? expf(a * scale - m[qq]) / l[qq] : 0.f;
                Pw[lane] = pj;
                dSw[lane] = pj * (gsum - Dq[qq]) * scale;
                if (live && lane < d) {
                    float acc = dq[qq], o = oa[qq];
                    for (int u = 0; u < cn; ++u) {               // this wavefront's rows only
                        acc = fmaf(dSw[u], Ks[u * dp + lane], acc);
                        o = fmaf(Pw[u], Vs[u * dp + lane], o);
                    }
                    dq[qq] = acc;
                    oa[qq] = o;
                }
            }
            __syncthreads();
            // dK[u][c] += sum_q dS[q][u] Q[q][c], dV[u][c] += sum_q P[q][u] dO[q][c] over the pass's 16
            // queries: a thread per (key, channel), then one atomic add each (other passes and other
            // regions add to the same keys)
            for (int e = tid; e < cn * d; e += 256) {
                const int u = e / d, c = e % d;
                float ak = 0.f, av = 0.f;
#pragma unroll
                for (int qi = 0; qi < 16; ++qi) {
                    ak = fmaf(dSsc[qi * 64 + u], qs[qi * d + c], ak);
                    av = fmaf(Psc[qi * 64 + u], dos[qi * d + c], av);
                }
                const size_t at = (size_t)key_token(k0 + u) * C3 + hd * d + c;
                unsafeAtomicAdd(dimg + at + D.C, ak);
                unsafeAtomicAdd(dimg + at + 2 * D.C, av);
            }
        }
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            const int s = s0 + 4 * wave + qq;
            if (s < D.n && lane < d) {                           // every query has one owner
                dimg[(size_t)query_token(s) * C3 + hd * d + lane] = dq[qq];
                Oatt[((size_t)b * D.N + query_token(s)) * D.C + hd * d + lane] = oa[qq];
            }
        }
    }
}

inline size_t attention_bwd_smem(int d)
{
    return (size_t)(2 * 64 * (d + 1) + 2 * 16 * d + 2 * 16 * 64) * sizeof(float);
}

// dV += LCE^T(dO): dV[y, x, c] += sum w[c, ky, kx] dO[y - ky + 2, x - kx + 2, c]   (after the attention part)
template <typename T>
__global__ void gen_lce_bwd_dv(const float *__restrict__ dO, const T *__restrict__ Wlce, float *__restrict__ dQKV,
                               Dims D)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)D.B * D.N * D.C;
    if (idx >= total) return;
    const int c = (int)(idx % D.C);
    const size_t tok = idx / D.C;
    const int x = (int)(tok % D.W), y = (int)((tok / D.W) % D.H);
    const size_t b = tok / D.N;
    float acc = 0.f;
    for (int ky = 0; ky < 5; ++ky) {
        const int yy = y - ky + 2;
        if (yy < 0 || yy >= D.H) continue;
        for (int kx = 0; kx < 5; ++kx) {
            const int xx = x - kx + 2;
            if (xx < 0 || xx >= D.W) continue;
            acc = fmaf(load_f32(Wlce + (size_t)c * 25 + ky * 5 + kx), dO[((b * D.H + yy) * D.W + xx) * D.C + c], acc);
        }
    }
    dQKV[tok * 3 * D.C + 2 * D.C + c] += acc;
}

// dWlce[c, ky, kx] += sum over this workgroup's tokens of dO[y, x, c] V[y + ky - 2, x + kx - 2, c]:
// blockIdx.y = tap, a thread per channel, atomic adds into the zeroed gradient.
__global__ __launch_bounds__(256) void gen_lce_bwd_dw(const float *__restrict__ dO, const float *__restrict__ QKV,
                                                      float *__restrict__ dW, Dims D, long tokens_per_wg)
{
    const int tap = blockIdx.y, ky = tap / 5, kx = tap % 5;
    const long t_begin = (long)blockIdx.x * tokens_per_wg, t_end = min((long)D.B * D.N, t_begin + tokens_per_wg);
    // 256 / C groups of threads share the workgroup's tokens when C < 256
    const int cw = D.C < 256 ? D.C : 256, groups = 256 / cw, grp = threadIdx.x / cw;
    if (grp >= groups) return;
    for (int c = threadIdx.x % cw; c < D.C; c += cw) {
        float acc = 0.f;
        for (long tok = t_begin + grp; tok < t_end; tok += groups) {
            const int x = (int)(tok % D.W), y = (int)((tok / D.W) % D.H);
            const int yy = y + ky - 2, xx = x + kx - 2;
            if (yy < 0 || yy >= D.H || xx < 0 || xx >= D.W) continue;
            const long vt = tok + (long)(ky - 2) * D.W + (kx - 2);
            acc = fmaf(dO[(size_t)tok * D.C + c], QKV[(size_t)vt * 3 * D.C + 2 * D.C + c], acc);
        }
        unsafeAtomicAdd(dW + (size_t)c * 25 + tap, acc);
    }
}

struct BwdWs {
    float *qkv, *o, *dO, *dqkv;
    size_t bytes;
};

BwdWs carve_bwd(const Dims &D, void *ws)
{
    char *base = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *ptr = base ? base + off : nullptr;
        off += align256(bytes);
        return ptr;
    };
    const size_t tok = (size_t)D.B * D.N;
    BwdWs w;
    w.qkv = (float *)take(tok * 3 * D.C * sizeof(float));
    w.o = (float *)take(tok * D.C * sizeof(float));
    w.dO = (float *)take(tok * D.C * sizeof(float));
    w.dqkv = (float *)take(tok * 3 * D.C * sizeof(float));
    w.bytes = off;
    return w;
}

void fill_zero(float *p, size_t n, hipStream_t st)
{
    hipLaunchKernelGGL(gen_fill_zero, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
}

template <typename T>
int backward_t(const Dims &D, const T *X, const T *Wqkv, const T *Wo, const T *Wlce, const int32_t *Ir, const T *dY,
               T *dX, float *dWqkv, float *dWo, float *dWlce, void *ws, hipStream_t st)
{
    const BwdWs w = carve_bwd(D, ws);
    const long M = (long)D.B * D.N;
    const int C = D.C, C3 = 3 * D.C;
    const size_t total = (size_t)M * C;
    if (attention_bwd_smem(D.d) > 64 * 1024) {
        static bool opted = false;
        if (!opted) {
            if (hipFuncSetAttribute((const void *)gen_attention_bwd, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)attention_bwd_smem(kBwdMaxD)) != hipSuccess)
                return BRA_ERR_LAUNCH;
            opted = true;
        }
    }
    ProfScope ps(st, K_GEN_BACKWARD);
    // forward intermediates again: Q | K | V (the attention output comes out of the backward kernel)
    hipLaunchKernelGGL((gen_gemm<T, T, float>), dim3((unsigned)((M + 63) / 64), (unsigned)((C3 + 63) / 64)), dim3(256), 0,
                       st, X, C, Wqkv, C3, w.qkv, C3, (int)M, C3, C);
    // dO = dY Wo^T
    hipLaunchKernelGGL((gen_gemm<T, T, float, true>), dim3((unsigned)((M + 63) / 64), (unsigned)((C + 63) / 64)), dim3(256),
                       0, st, dY, C, Wo, C, w.dO, C, (int)M, C, C);
    fill_zero(dWo, (size_t)C * C, st);
    fill_zero(dWqkv, (size_t)C * C3, st);
    fill_zero(dWlce, (size_t)C * 25, st);
    fill_zero(w.dqkv, (size_t)M * C3, st);
    // attention: dQ, dK, dV and the attention output; then O = attention + LCE(V) for dWo
    hipLaunchKernelGGL(gen_attention_bwd, dim3((unsigned)((long)D.B * D.R * D.heads * ((D.n + 15) / 16))), dim3(256),
                       attention_bwd_smem(D.d), st, w.qkv, Ir,
                       w.o, w.dO, w.dqkv, D, D.scale);
    hipLaunchKernelGGL(gen_lce_add<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w.qkv, Wlce, w.o, D);
    long splits = (M + 255) / 256;                 // enough workgroups to fill the chip
    splits = splits > 4096 ? 4096 : splits;
    const long rows = ((M + splits - 1) / splits + 15) / 16 * 16;
    hipLaunchKernelGGL((gen_gemm_tn<float, T>), dim3((unsigned)((C + 63) / 64), (unsigned)((C + 63) / 64), (unsigned)splits),
                       dim3(256), 0, st, w.o, C, dY, C, dWo, C, M, C, C, rows);
    // the LCE parts
    hipLaunchKernelGGL(gen_lce_bwd_dv<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, w.dO, Wlce, w.dqkv, D);
    const long tpw = 512;
    hipLaunchKernelGGL(gen_lce_bwd_dw, dim3((unsigned)((M + tpw - 1) / tpw), 25), dim3(256), 0, st, w.dO, w.qkv, dWlce, D,
                       tpw);
    // dX = [dQ | dK | dV] Wqkv^T, dWqkv = X^T [dQ | dK | dV]
    hipLaunchKernelGGL((gen_gemm<float, T, T, true>), dim3((unsigned)((M + 63) / 64), (unsigned)((C + 63) / 64)), dim3(256),
                       0, st, w.dqkv, C3, Wqkv, C3, dX, C, (int)M, C, C3);
    hipLaunchKernelGGL((gen_gemm_tn<T, float>), dim3((unsigned)((C + 63) / 64), (unsigned)((C3 + 63) / 64), (unsigned)splits),
                       dim3(256), 0, st, X, C, w.dqkv, C3, dWqkv, C3, M, C, C3, rows);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

}  // namespace

size_t generic_block_workspace_bytes(const Dims &D, int hidden, size_t bra_bytes)
{
    return carve_gen_block(D, hidden, bra_bytes, nullptr).bytes;
}

int generic_block_forward(const Dims &D, int hidden, float eps, const void *X, const bra_block_params &p, void *Xout,
                          int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path,
                          hipStream_t st)
{
    if (D.dtype == BRA_BF16)
        return block_t<bf16_t>(D, hidden, eps, (const bf16_t *)X, p, (bf16_t *)Xout, Ir_out_opt, Ir_in_opt, ws,
                               bra_bytes, path, st);
    return block_t<float>(D, hidden, eps, (const float *)X, p, (float *)Xout, Ir_out_opt, Ir_in_opt, ws, bra_bytes,
                          path, st);
}

bool generic_backward_supported(const Dims &D)
{
    return generic_supported(D) && D.d <= kBwdMaxD && (long)D.B * D.R * D.heads * ((D.n + 15) / 16) <= 0x7fffffffL;
}

size_t generic_backward_workspace_bytes(const Dims &D) { return carve_bwd(D, nullptr).bytes; }

int generic_backward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                     const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                     hipStream_t st)
{
    if (D.dtype == BRA_BF16)
        return backward_t<bf16_t>(D, (const bf16_t *)X, (const bf16_t *)Wqkv, (const bf16_t *)Wo, (const bf16_t *)Wlce,
                                  Ir, (const bf16_t *)dY, (bf16_t *)dX, dWqkv, dWo, dWlce, ws, st);
    return backward_t<float>(D, (const float *)X, (const float *)Wqkv, (const float *)Wo, (const float *)Wlce, Ir,
                             (const float *)dY, (float *)dX, dWqkv, dWo, dWlce, ws, st);
}

bool generic_supported(const Dims &D)
{
    // grid sizes must fit 31 bits; head width and region count are bounded by the
    // static buffers of the attention and top-k kernels.
    if (D.d > kAttnMaxD) return false;
    if (D.R > kWave * kTopkSlots) return false;
    if ((long)D.B * D.R * D.heads > 0x7fffffffL) return false;
    if (((long)D.B * D.N * D.C + 255) / 256 > 0x7fffffffL) return false;
    if ((size_t)D.k * sizeof(int) > 16 * 1024) return false;
    if ((size_t)D.C * sizeof(float) > 48 * 1024) return false;
    return true;
}

size_t generic_workspace_bytes(const Dims &D) { return carve(D, nullptr).bytes; }

int generic_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt,
                  void *ws, hipStream_t st)
{
    GenericWs w = carve(D, ws);
    if (f32_small_ok(D))      // the kernels that bra_forward runs for this shape, so that both give the same index
        return f32_small_route(D, (const float *)X, (const float *)Wqkv, Ir, Ar_opt, w.qkv, w.qr, w.kr, st);
    if (D.dtype == BRA_F32)
        launch_route<float>(D, (const float *)X, (const float *)Wqkv, Ir, Ar_opt, w, st);
    else
        launch_route<bf16_t>(D, (const bf16_t *)X, (const bf16_t *)Wqkv, Ir, Ar_opt, w, st);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

int generic_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo,
                    const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                    void *ws, hipStream_t st)
{
    if (D.dtype == BRA_F32)
        return forward_t<float>(D, (const float *)X, (const float *)Wqkv, (const float *)Wo,
                                (const float *)Wlce, (float *)Y, Ir_out_opt, Ir_in_opt, ws, st);
    return forward_t<bf16_t>(D, (const bf16_t *)X, (const bf16_t *)Wqkv, (const bf16_t *)Wo,
                             (const bf16_t *)Wlce, (bf16_t *)Y, Ir_out_opt, Ir_in_opt, ws, st);
}

}  // namespace bra

namespace bra {

// Routing with caller-provided scratch (xr, qr, kr: [B, R, C] float32 each), used by
// the matrix-core family for shapes its own routing kernels do not cover.
size_t valu_route_scratch_bytes(const Dims &D)
{
    return 3 * align256((size_t)D.B * D.R * D.C * sizeof(float));
}

int valu_affinity_topk(const Dims &D, const float *Qr, const float *Kr, int32_t *Ir, float *Ar_opt,
                       hipStream_t st)
{
    ProfScope ps(st, K_GEN_TOPK);
    hipLaunchKernelGGL(gen_affinity_topk, dim3(D.B * D.R), dim3(kWave), D.C * sizeof(float), st, Qr, Kr, Ir,
                       Ar_opt, D);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

int valu_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt,
               void *scratch, hipStream_t st)
{
    GenericWs w;
    const size_t each = align256((size_t)D.B * D.R * D.C * sizeof(float));
    w.xr = (float *)scratch;
    w.qr = (float *)((char *)scratch + each);
    w.kr = (float *)((char *)scratch + 2 * each);
    if (D.dtype == BRA_F32)
        launch_route<float>(D, (const float *)X, (const float *)Wqkv, Ir, Ar_opt, w, st);
    else
        launch_route<bf16_t>(D, (const bf16_t *)X, (const bf16_t *)Wqkv, Ir, Ar_opt, w, st);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

}  // namespace bra
