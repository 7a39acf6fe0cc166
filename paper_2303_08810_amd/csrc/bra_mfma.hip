// Matrix-core (MFMA) kernel family for bf16 tensors on gfx950, head width d = 32.
//
// All contractions use v_mfma_f32_16x16x32_bf16 (64-lane wavefront; lane l = 16 g + i):
//   A operand: lane holds A[row i][k = 8 g .. 8 g + 7]
//   B operand: lane holds B[k = 8 g .. 8 g + 7][col i]
//   D result : lane holds D[row 4 g .. 4 g + 3][col i]
// so both operands are read as 16-byte runs along the contraction axis, and the
// contraction may use any key order as long as A and B agree on it.
//
// Intermediates Q, K, V are bf16 tensors in the spatial [B, H, W, C] layout; the
// region structure of Sec. 3.2 lives in address arithmetic only.  The routed
// key/value tokens (Eq. 6) are copied by index from that layout into LDS, never
// into a gathered tensor in memory.
#include "bra_common.h"

namespace bra {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kMaxLds = 160 * 1024;   // LDS per workgroup on gfx950

__device__ inline f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ inline unsigned pack_bf16(float a, float b)
{
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(unsigned, r);
}

__device__ inline bf16x8 pack8(const float *v)
{
    u32x4 u = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
               pack_bf16(v[6], v[7])};
    return __builtin_bit_cast(bf16x8, u);
}

// LDS transpose read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s
// supplies the address of 4 consecutive 16-bit elements; the four lanes 4 j .. 4 j + 3
// together supply a row j of 16 elements.  Lane i receives element i of rows 0..3.
__device__ inline s16x4 lds_read_tr16(const bf16_t *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)p);
}

// ---------------------------------------------------------------------------
// WT[o][c] = Wqkv[c][o] (o < 3C) and WoT[o][c] = Wo[c][o]: the weights with the
// contraction axis contiguous, as the MFMA operands want them.
__global__ void k_prep_weights(const bf16_t *__restrict__ Wqkv, const bf16_t *__restrict__ Wo,
                               bf16_t *__restrict__ WT, bf16_t *__restrict__ WoT, int C)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    const int total = 4 * C * C;
    if (e >= total) return;
    const int o = e / C, c = e % C;
    if (o < 3 * C) WT[e] = Wqkv[(size_t)c * 3 * C + o];
    else WoT[(size_t)(o - 3 * C) * C + c] = Wo[(size_t)c * C + (o - 3 * C)];
}

// ---------------------------------------------------------------------------
// Q, K, V = X [Wq | Wk | Wv]  (Eq. 3).  Each wavefront owns 64 output channels of one
// of the three matrices and keeps its weight fragments in registers; the workgroup
// (3C/64 wavefronts) walks over tiles of 16*NU tokens.  The product is formed
// transposed (rows = output channels, columns = tokens) with the weight rows
// permuted so that a lane ends up with 16 consecutive output channels of one token,
// i.e. one 32-byte store.
template <int C, int NU>
__global__ __launch_bounds__(3 * C) void k_qkv(const bf16_t *__restrict__ X,
                                               const bf16_t *__restrict__ WT,
                                               bf16_t *__restrict__ Q, bf16_t *__restrict__ K,
                                               bf16_t *__restrict__ V, long M)
{
    constexpr int KS = C / 32;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int sel = wave / (C / 64), base = (wave % (C / 64)) * 64;
    bf16_t *__restrict__ out = sel == 0 ? Q : (sel == 1 ? K : V);

    bf16x8 af[4][KS];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
        const int o = sel * C + base + 16 * (i / 4) + 4 * tt + (i % 4);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            af[tt][ks] = *(const bf16x8 *)(WT + (size_t)o * C + 32 * ks + 8 * g);
    }

    const long ntiles = (M + 16 * NU - 1) / (16 * NU);
    for (long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const long tok0 = tile * 16 * NU;
        bf16x8 bfr[NU][KS];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            long t = tok0 + 16 * u + i;
            if (t >= M) t = M - 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                bfr[u][ks] = *(const bf16x8 *)(X + t * C + 32 * ks + 8 * g);
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            f32x4 acc[4];
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                acc[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc[tt] = mfma16(af[tt][ks], bfr[u][ks], acc[tt]);
            }
            const long t = tok0 + 16 * u + i;
            if (t < M) {
                u32x4 lo = {pack_bf16(acc[0][0], acc[0][1]), pack_bf16(acc[0][2], acc[0][3]),
                            pack_bf16(acc[1][0], acc[1][1]), pack_bf16(acc[1][2], acc[1][3])};
                u32x4 hi = {pack_bf16(acc[2][0], acc[2][1]), pack_bf16(acc[2][2], acc[2][3]),
                            pack_bf16(acc[3][0], acc[3][1]), pack_bf16(acc[3][2], acc[3][3])};
                u32x4 *dst = (u32x4 *)(out + t * C + base + 16 * g);
                dst[0] = lo;
                dst[1] = hi;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Routed attention + LCE + W^o for regions of n >= 64 tokens (Eq. 6-7, Eq. 2).
// One workgroup = 64 query tokens (64/rw full rows of one region), all heads,
// 4 wavefronts; wavefront w owns queries 16 w .. 16 w + 15.  Keys and values of the
// k routed regions are copied by index, 64 tokens at a time, from the projected
// maps into LDS; one online softmax runs over all k n keys.
template <int C>
struct AttnBigSmem {
    static constexpr int CS = C + 8;               // bf16 elements per LDS row (16 B pad)
    static constexpr int OS = C + 4;               // floats per row of the output tile
    static constexpr size_t q_off = 0;
    static constexpr size_t k_off = q_off + (size_t)64 * CS * 2;
    static constexpr size_t v_off = k_off + (size_t)64 * CS * 2;
    static constexpr size_t h_off = v_off + (size_t)64 * CS * 2;
    static size_t bytes(int halo_rows) { return h_off + (size_t)halo_rows * CS * 2; }
};

// Copies `rows` token rows of C bf16 from a [.., W, C] map into LDS rows of CS elements.
// Row r is token (y0 + r / tw, x0 + r % tw); rows outside the image are zero-filled.
template <int C, int CS>
__device__ inline void stage_rows(bf16_t *dst, const bf16_t *__restrict__ img, int y0, int x0,
                                  int tw, int rows, int H, int W)
{
    constexpr int CH = C / 8;
    for (int idx = threadIdx.x; idx < rows * CH; idx += blockDim.x) {
        const int r = idx / CH, cc = idx % CH;
        const int y = y0 + r / tw, x = x0 + r % tw;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (y >= 0 && y < H && x >= 0 && x < W) v = *(const u32x4 *)(img + ((size_t)y * W + x) * C + cc * 8);
        *(u32x4 *)(dst + r * CS + cc * 8) = v;
    }
}

template <int C>
__global__ __launch_bounds__(256) void k_attn_big(const bf16_t *__restrict__ Q,
                                                  const bf16_t *__restrict__ K,
                                                  const bf16_t *__restrict__ V,
                                                  const int32_t *__restrict__ Ir,
                                                  const bf16_t *__restrict__ Wlce,
                                                  const bf16_t *__restrict__ WoT,
                                                  bf16_t *__restrict__ Y, Dims D, float c_exp)
{
    typedef AttnBigSmem<C> SM;
    constexpr int CS = SM::CS, OS = SM::OS, HEADS = C / 32, KS = C / 32;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Qs = (bf16_t *)(smem + SM::q_off);
    bf16_t *Ks = (bf16_t *)(smem + SM::k_off);
    bf16_t *Vs = (bf16_t *)(smem + SM::v_off);
    bf16_t *Hs = (bf16_t *)(smem + SM::h_off);
    float *Os = (float *)(smem + SM::k_off);   // reuses the K/V tiles after the key loop

    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;

    const int chunks = D.n / 64;               // query tiles per region
    const int qh = 64 / D.rw;                  // rows per query tile
    const int wid = blockIdx.x;
    const int b = wid / (D.R * chunks);
    const int reg = (wid / chunks) % D.R;
    const int ch = wid % chunks;
    const int y0 = (reg / D.S) * D.rh + ch * qh, x0 = (reg % D.S) * D.rw;
    const size_t img_off = (size_t)b * D.N * C;
    const int32_t *ir = Ir + ((size_t)b * D.R + reg) * D.k;

    stage_rows<C, CS>(Qs, Q + img_off, y0, x0, D.rw, 64, D.H, D.W);
    const int hw = D.rw + 4, hrows = (qh + 4) * hw;
    stage_rows<C, CS>(Hs, V + img_off, y0 - 2, x0 - 2, hw, hrows, D.H, D.W);

    float m_run[HEADS], l_run[HEADS];
    f32x4 acc[HEADS][2];
#pragma unroll
    for (int h = 0; h < HEADS; ++h) {
        m_run[h] = -INFINITY;
        l_run[h] = 0.f;
        acc[h][0] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc[h][1] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int nblocks = D.kn / 64;
    for (int kb = 0; kb < nblocks; ++kb) {
        const int j = ir[kb / chunks];
        const int ky0 = (j / D.S) * D.rh + (kb % chunks) * qh, kx0 = (j % D.S) * D.rw;
        __syncthreads();   // previous block's readers are done (and Qs/Hs writes are ordered)
        stage_rows<C, CS>(Ks, K + img_off, ky0, kx0, D.rw, 64, D.H, D.W);
        stage_rows<C, CS>(Vs, V + img_off, ky0, kx0, D.rw, 64, D.H, D.W);
        __syncthreads();
#pragma unroll
        for (int h = 0; h < HEADS; ++h) {
            const bf16x8 qf = *(const bf16x8 *)(Qs + (16 * wave + i) * CS + 32 * h + 8 * g);
            f32x4 s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * CS + 32 * h + 8 * g);
                s[t] = mfma16(kf, qf, f32x4{0.f, 0.f, 0.f, 0.f});   // S^T[key 16t+4g+j][query i]
            }
            float mx = s[0][0];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) mx = fmaxf(mx, s[t][jj]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
            const float m_new = fmaxf(m_run[h], mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run[h] - m_new) * c_exp);
            const float mc = m_new * c_exp;
            float p[4][4], ls = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    p[t][jj] = __builtin_amdgcn_exp2f(fmaf(s[t][jj], c_exp, -mc));
                    ls += p[t][jj];
                }
            ls += __shfl_xor(ls, 16, kWave);
            ls += __shfl_xor(ls, 32, kWave);
            l_run[h] = l_run[h] * alpha + ls;
            m_run[h] = m_new;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) acc[h][dt] *= alpha;
#pragma unroll
            for (int tp = 0; tp < 2; ++tp) {
                float pv[8] = {p[2 * tp][0], p[2 * tp][1], p[2 * tp][2], p[2 * tp][3],
                               p[2 * tp + 1][0], p[2 * tp + 1][1], p[2 * tp + 1][2], p[2 * tp + 1][3]};
                const bf16x8 pb = pack8(pv);
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const int col = 32 * h + 16 * dt + 4 * (i % 4);
                    const s16x4 v0 = lds_read_tr16(Vs + (32 * tp + 4 * g + i / 4) * CS + col);
                    const s16x4 v1 = lds_read_tr16(Vs + (32 * tp + 16 + 4 * g + i / 4) * CS + col);
                    u32x2 a0 = __builtin_bit_cast(u32x2, v0), a1 = __builtin_bit_cast(u32x2, v1);
                    u32x4 av = {a0[0], a0[1], a1[0], a1[1]};
                    acc[h][dt] = mfma16(__builtin_bit_cast(bf16x8, av), pb, acc[h][dt]);
                }
            }
        }
    }
    __syncthreads();   // everyone is done with Ks / Vs: the output tile may overwrite them
#pragma unroll
    for (int h = 0; h < HEADS; ++h) {
        const float inv = 1.0f / l_run[h];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            f32x4 o = acc[h][dt] * inv;   // O^T[channel 16dt+4g+j][query i]
            *(f32x4 *)(Os + (16 * wave + i) * OS + 32 * h + 16 * dt + 4 * g) = o;
        }
    }
    __syncthreads();

    // LCE: 5x5 depth-wise cross-correlation of V over the halo tile, added to the
    // attention output.  One task = (row of the query tile, 8-token segment, channel pair).
    {
        const int segs = D.rw / 8, cp_n = C / 2;
        const int tasks = qh * segs * cp_n;
        for (int task = threadIdx.x; task < tasks; task += blockDim.x) {
            const int cp = task % cp_n, seg = (task / cp_n) % segs, r = task / (cp_n * segs);
            const int c = 2 * cp;
            float w0[25], w1[25];
#pragma unroll
            for (int t = 0; t < 25; ++t) {
                w0[t] = bf16_to_f32(Wlce[c * 25 + t]);
                w1[t] = bf16_to_f32(Wlce[(c + 1) * 25 + t]);
            }
            float a0[8], a1[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) { a0[x] = 0.f; a1[x] = 0.f; }
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                float v0[12], v1[12];
#pragma unroll
                for (int x = 0; x < 12; ++x) {
                    const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + seg * 8 + x) * CS + c);
                    v0[x] = __builtin_bit_cast(float, u << 16);
                    v1[x] = __builtin_bit_cast(float, u & 0xffff0000u);
                }
#pragma unroll
                for (int x = 0; x < 8; ++x)
#pragma unroll
                    for (int kx = 0; kx < 5; ++kx) {
                        a0[x] = fmaf(w0[ky * 5 + kx], v0[x + kx], a0[x]);
                        a1[x] = fmaf(w1[ky * 5 + kx], v1[x + kx], a1[x]);
                    }
            }
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                f32x2 *o = (f32x2 *)(Os + (r * D.rw + seg * 8 + x) * OS + c);
                f32x2 cur = *o;
                cur[0] += a0[x];
                cur[1] += a1[x];
                *o = cur;
            }
        }
    }
    __syncthreads();

    // Y = O Wo for the 16 tokens of this wavefront, formed transposed as in k_qkv.
    {
        bf16x8 of[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const float *src = Os + (16 * wave + i) * OS + 32 * ks + 8 * g;
            f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
            float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            of[ks] = pack8(v);
        }
        const int q = 16 * wave + i;
        const size_t tok = (size_t)(y0 + q / D.rw) * D.W + x0 + q % D.rw;
        bf16_t *yrow = Y + img_off + tok * C;
#pragma unroll
        for (int cg = 0; cg < C / 64; ++cg) {
            f32x4 ya[4];
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int o = cg * 64 + 16 * (i / 4) + 4 * tt + (i % 4);
                ya[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 wf = *(const bf16x8 *)(WoT + (size_t)o * C + 32 * ks + 8 * g);
                    ya[tt] = mfma16(wf, of[ks], ya[tt]);
                }
            }
            u32x4 lo = {pack_bf16(ya[0][0], ya[0][1]), pack_bf16(ya[0][2], ya[0][3]),
                        pack_bf16(ya[1][0], ya[1][1]), pack_bf16(ya[1][2], ya[1][3])};
            u32x4 hi = {pack_bf16(ya[2][0], ya[2][1]), pack_bf16(ya[2][2], ya[2][3]),
                        pack_bf16(ya[3][0], ya[3][1]), pack_bf16(ya[3][2], ya[3][3])};
            u32x4 *dst = (u32x4 *)(yrow + cg * 64 + 16 * g);
            dst[0] = lo;
            dst[1] = hi;
        }
    }
}

struct MfmaWs {
    bf16_t *q, *k, *v, *wt, *wot;
    void *route;
    int32_t *ir;
    size_t bytes;
};

MfmaWs carve(const Dims &D, void *ws)
{
    MfmaWs w;
    char *p = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *q = p ? p + off : nullptr; off += align256(bytes); return q; };
    const size_t tok = (size_t)D.B * D.N;
    w.q = (bf16_t *)take(tok * D.C * 2);
    w.k = (bf16_t *)take(tok * D.C * 2);
    w.v = (bf16_t *)take(tok * D.C * 2);
    w.wt = (bf16_t *)take((size_t)3 * D.C * D.C * 2);
    w.wot = (bf16_t *)take((size_t)D.C * D.C * 2);
    w.route = take(valu_route_scratch_bytes(D));
    w.ir = (int32_t *)take((size_t)D.B * D.R * D.k * sizeof(int32_t));
    w.bytes = off;
    return w;
}

template <int C>
int forward_c(const Dims &D, const bf16_t *X, const bf16_t *Wqkv, const bf16_t *Wo,
              const bf16_t *Wlce, bf16_t *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
              const MfmaWs &w, hipStream_t st)
{
    const int32_t *Ir = Ir_in_opt;
    if (!Ir_in_opt) {
        int32_t *dst = Ir_out_opt ? Ir_out_opt : w.ir;
        int rc = valu_route(D, X, Wqkv, dst, nullptr, w.route, st);
        if (rc != BRA_OK) return rc;
        Ir = dst;
    } else if (Ir_out_opt) {
        if (hipMemcpyAsync(Ir_out_opt, Ir_in_opt, sizeof(int32_t) * (size_t)D.B * D.R * D.k,
                           hipMemcpyDeviceToDevice, st) != hipSuccess)
            return BRA_ERR_LAUNCH;
    }
    {
        ProfScope ps(st, K_MFMA_PREP);
        hipLaunchKernelGGL(k_prep_weights, dim3((4 * C * C + 255) / 256), dim3(256), 0, st, Wqkv, Wo,
                           w.wt, w.wot, C);
    }
    const long M = (long)D.B * D.N;
    {
        constexpr int NU = (C == 256) ? 1 : 2;
        const long ntiles = (M + 16 * NU - 1) / (16 * NU);
        const int grid = (int)(ntiles < 2048 ? ntiles : 2048);
        ProfScope ps(st, K_MFMA_QKV);
        hipLaunchKernelGGL((k_qkv<C, NU>), dim3(grid), dim3(3 * C), 0, st, X, w.wt, w.q, w.k, w.v, M);
    }
    {
        const int qh = 64 / D.rw;
        const size_t smem = AttnBigSmem<C>::bytes((qh + 4) * (D.rw + 4));
        const int grid = D.B * D.R * (D.n / 64);
        const float c_exp = D.scale * 1.4426950408889634f;
        static bool lds_opt_in = false;   // allow more than 64 KB of dynamic LDS, once
        if (!lds_opt_in) {
            if (hipFuncSetAttribute((const void *)k_attn_big<C>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) != hipSuccess)
                return BRA_ERR_LAUNCH;
            lds_opt_in = true;
        }
        ProfScope ps(st, K_MFMA_ATTENTION);
        hipLaunchKernelGGL(k_attn_big<C>, dim3(grid), dim3(256), smem, st, w.q, w.k, w.v, Ir, Wlce,
                           w.wot, Y, D, c_exp);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

bool attn_big_ok(const Dims &D)
{
    if (D.n % 64 != 0) return false;
    if (D.rw < 8 || 64 % D.rw != 0) return false;
    const int qh = 64 / D.rw;
    if (D.rh % qh != 0) return false;
    size_t smem = 0;
    if (D.C == 64) smem = AttnBigSmem<64>::bytes((qh + 4) * (D.rw + 4));
    else if (D.C == 128) smem = AttnBigSmem<128>::bytes((qh + 4) * (D.rw + 4));
    else smem = AttnBigSmem<256>::bytes((qh + 4) * (D.rw + 4));
    return smem <= (size_t)kMaxLds;
}

}  // namespace

bool mfma_supported(const Dims &D)
{
    if (D.dtype != BRA_BF16 || D.d != 32) return false;
    if (D.C != 64 && D.C != 128 && D.C != 256) return false;
    if ((long)D.B * D.R * (D.n / 64 + 1) > 0x7fffffffL) return false;
    if (!generic_supported(D)) return false;   // routing uses the scalar kernels
    return attn_big_ok(D);
}

size_t mfma_workspace_bytes(const Dims &D) { return carve(D, nullptr).bytes; }

int mfma_route(const Dims &D, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt, void *ws,
               hipStream_t st)
{
    MfmaWs w = carve(D, ws);
    return valu_route(D, X, Wqkv, Ir, Ar_opt, w.route, st);
}

int mfma_forward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                 void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, hipStream_t st)
{
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

}  // namespace bra
