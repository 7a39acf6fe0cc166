// One whole BiFormer block around BRA (Sec. 3.4), bf16 tensors, float32 arithmetic:
//
//   k_token_ln<POS>   X1 = X + DWConv3x3(X) + bpos,  Xn = LayerNorm1(X1)      one pass over X
//   BRA               Y  = BRA(Xn)                   (Eq. 2-7; the kernel family picked for the shape)
//   k_token_ln<ADD>   X2 = X1 + Y,                   Xn = LayerNorm2(X2)
//   gemm_bf16         Hd = GELU(Xn W1 + b1)          bias and activation in the product's epilogue
//   gemm_bf16         Xout = X2 + Hd W2 + b2         bias and residual in the epilogue
//
// The normalisation and residual links follow the pre-norm residual reading stated with the
// entry point's declaration.
#include "bra_mfma_dev.h"

namespace bra {

using namespace mfma;

namespace {

constexpr int kPos = 0, kAdd = 1;

// A token's C channels are shared by G consecutive lanes (G a power of two that divides
// C / 8, at most 64): lane `sub` owns the 8-channel chunks sub, sub + G, ..  A workgroup has
// 256 / G token slots and walks `iters` consecutive groups of that many tokens.
// ONE (C / 8 == G): a lane owns one chunk for every token, so its convolution weights, bias,
// gamma and beta stay in registers and a token's values never leave them.  Otherwise the
// values of a lane's chunks wait in a per-lane strip of LDS between the passes.
// Sum = the pre-norm tensor (X1 or X2), Norm = its LayerNorm; the statistics use the float32
// values, not the rounded ones that are stored.  Sum may be A itself (ADD): a lane reads the
// elements it overwrites before it writes them.
template <int MODE, bool ONE>
__global__ __launch_bounds__(256) void k_token_ln(const bf16_t *A, const bf16_t *__restrict__ Badd,
                                                  const bf16_t *__restrict__ Wpos, const float *__restrict__ bpos,
                                                  const float *__restrict__ gamma, const float *__restrict__ beta,
                                                  bf16_t *Sum, bf16_t *__restrict__ Norm, int H, int W,
                                                  int C, long tokens, int G, int iters, float eps)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, sub = tid % G, slot = tid / G, slots = 256 / G;
    const int CH = C / 8, NC = CH / G;
    float *strip = (float *)smem + (size_t)slot * C;       // this token slot's values (not ONE)
    const float c_inv = 1.0f / (float)C;

    // the 3x3 weights of 8 channels are 72 consecutive bf16: channel-major, (ky, kx) inside
    auto load_w = [&](int c0, float (&w)[8][9]) {
        const u32x4 *src = (const u32x4 *)(Wpos + (size_t)c0 * 9);
        unsigned raw[36];
#pragma unroll
        for (int q = 0; q < 9; ++q) {
            const u32x4 v = src[q];
            raw[4 * q] = v[0]; raw[4 * q + 1] = v[1]; raw[4 * q + 2] = v[2]; raw[4 * q + 3] = v[3];
        }
#pragma unroll
        for (int e = 0; e < 72; ++e) w[e / 9][e % 9] = (e & 1) ? bf16_hi(raw[e / 2]) : bf16_lo(raw[e / 2]);
    };
    auto load8 = [&](const float *p, float (&v)[8]) {
        const f32x4 a = *(const f32x4 *)p, b = *(const f32x4 *)(p + 4);
        v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3]; v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
    };
    auto unpack = [&](u32x4 t, float (&v)[8]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[2 * e] = bf16_lo(t[e]); v[2 * e + 1] = bf16_hi(t[e]); }
    };
    // the pre-norm values of chunk c0 of token (img, y, x)
    auto values = [&](long tok, int y, int x, int c0, const float (&w)[8][9], const float (&bias)[8], float (&v)[8]) {
        const bf16_t *centre = A + (size_t)tok * C + c0;
        float xc[8];
        unpack(*(const u32x4 *)centre, xc);
        if (MODE == kAdd) {
            float yv[8];
            unpack(*(const u32x4 *)(Badd + (size_t)tok * C + c0), yv);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = xc[e] + yv[e];
            return;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = fmaf(w[e][4], xc[e], xc[e] + bias[e]);
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int yy = y + ky - 1;
            if (yy < 0 || yy >= H) continue;
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int xx = x + kx - 1;
                if ((ky == 1 && kx == 1) || xx < 0 || xx >= W) continue;
                float nb[8];
                unpack(*(const u32x4 *)(centre + ((long)(ky - 1) * W + (kx - 1)) * C), nb);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = fmaf(w[e][3 * ky + kx], nb[e], v[e]);
            }
        }
    };
    auto group_sum = [&](float s) {
        for (int off = 1; off < G; off *= 2) s += __shfl_xor(s, off);
        return s;
    };

    float w[8][9], bias[8], gm[8], bt[8];
    if (ONE) {
        if (MODE == kPos) { load_w(8 * sub, w); load8(bpos + 8 * sub, bias); }
        load8(gamma + 8 * sub, gm);
        load8(beta + 8 * sub, bt);
    }
    const long first = (long)blockIdx.x * slots * iters;
    for (int it = 0; it < iters; ++it) {
        const long tok_raw = first + (long)it * slots + slot;
        const bool valid = tok_raw < tokens;
        const long tok = valid ? tok_raw : tokens - 1;          // lanes past the end redo the last token, store nothing
        const int ry = (int)tok / W, x = (int)tok - ry * W;    // tokens < 2^31 (checked on the host)
        const int y = ry % H;

        if (ONE) {
            float v[8];
            values(tok, y, x, 8 * sub, w, bias, v);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[e];
            const float mean = group_sum(s) * c_inv;
            float q = 0.f, d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { d[e] = v[e] - mean; q = fmaf(d[e], d[e], q); }
            const float rstd = 1.0f / sqrtf(group_sum(q) * c_inv + eps);
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(d[e] * rstd, gm[e], bt[e]);
            if (valid) {
                *(bf16x8 *)(Sum + (size_t)tok * C + 8 * sub) = pack8(v);
                *(bf16x8 *)(Norm + (size_t)tok * C + 8 * sub) = pack8(o);
            }
        } else {
            float s = 0.f;
            for (int q = 0; q < NC; ++q) {
                const int c0 = 8 * (sub + G * q);
                if (MODE == kPos) { load_w(c0, w); load8(bpos + c0, bias); }
                float v[8];
                values(tok, y, x, c0, w, bias, v);
#pragma unroll
                for (int e = 0; e < 8; ++e) s += v[e];
                *(f32x4 *)(strip + c0) = f32x4{v[0], v[1], v[2], v[3]};
                *(f32x4 *)(strip + c0 + 4) = f32x4{v[4], v[5], v[6], v[7]};
                if (valid) *(bf16x8 *)(Sum + (size_t)tok * C + c0) = pack8(v);
            }
            const float mean = group_sum(s) * c_inv;
            float qq = 0.f;
            for (int q = 0; q < NC; ++q) {
                float v[8];
                load8(strip + 8 * (sub + G * q), v);
#pragma unroll
                for (int e = 0; e < 8; ++e) { const float d = v[e] - mean; qq = fmaf(d, d, qq); }
            }
            const float rstd = 1.0f / sqrtf(group_sum(qq) * c_inv + eps);
            for (int q = 0; q < NC; ++q) {
                const int c0 = 8 * (sub + G * q);
                float v[8], o[8];
                load8(strip + c0, v);
                load8(gamma + c0, gm);
                load8(beta + c0, bt);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf((v[e] - mean) * rstd, gm[e], bt[e]);
                if (valid) *(bf16x8 *)(Norm + (size_t)tok * C + c0) = pack8(o);
            }
        }
    }
}

// lanes per token: the largest power of two that divides C / 8, at most 64
int lanes_per_token(int C)
{
    int G = 1;
    while (G < 64 && (C / 8) % (2 * G) == 0) G *= 2;
    return G;
}

template <int MODE>
int launch_token_ln(const Dims &D, const bf16_t *A, const bf16_t *Badd, const bra_block_params &p, const float *gamma,
                    const float *beta, bf16_t *Sum, bf16_t *Norm, float eps, hipStream_t st)
{
    const long tokens = (long)D.B * D.N;
    const int G = lanes_per_token(D.C), slots = 256 / G;
    const bool one = D.C / 8 == G;
    // enough workgroups to fill the chip several times over, up to 8 token groups each
    long iters = tokens / ((long)slots * 4096);
    iters = iters < 1 ? 1 : (iters > 8 ? 8 : iters);
    const long grid = (tokens + slots * iters - 1) / (slots * iters);
    ProfScope ps(st, MODE == kPos ? K_BLK_POS_LN : K_BLK_ADD_LN);
    if (one) {
        hipLaunchKernelGGL((k_token_ln<MODE, true>), dim3((unsigned)grid), dim3(256), 0, st, A, Badd,
                           (const bf16_t *)p.Wpos, p.bpos, gamma, beta, Sum, Norm, D.H, D.W, D.C, tokens, G,
                           (int)iters, eps);
    } else {
        const size_t smem = (size_t)slots * D.C * sizeof(float);      // at most 4 x 4096 floats
        hipLaunchKernelGGL((k_token_ln<MODE, false>), dim3((unsigned)grid), dim3(256), smem, st, A, Badd,
                           (const bf16_t *)p.Wpos, p.bpos, gamma, beta, Sum, Norm, D.H, D.W, D.C, tokens, G,
                           (int)iters, eps);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

struct BlockWs {
    bf16_t *x1, *xn, *y, *hd;
    void *inner;
    size_t bytes;
};

BlockWs carve_block(const Dims &D, int hidden, size_t bra_bytes, void *ws)
{
    char *base = (char *)ws;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *ptr = base ? base + off : nullptr;
        off += align256(bytes);
        return ptr;
    };
    const size_t act = (size_t)D.B * D.N * D.C * sizeof(bf16_t);
    BlockWs w;
    w.x1 = (bf16_t *)take(act);
    w.xn = (bf16_t *)take(act);
    w.y = (bf16_t *)take(act);
    w.hd = (bf16_t *)take((size_t)D.B * D.N * hidden * sizeof(bf16_t));
    w.inner = take(bra_bytes);
    w.bytes = off;
    return w;
}

}  // namespace

bool block_supported(const Dims &D, int hidden)
{
    return D.dtype == BRA_BF16 && D.C % 64 == 0 && D.C <= 4096 && hidden % 64 == 0 && hidden <= (1 << 16) &&
           (long)D.B * D.N <= 0x7fffffffL / 64;
}

size_t block_workspace_bytes(const Dims &D, int hidden, size_t bra_bytes)
{
    return carve_block(D, hidden, bra_bytes, nullptr).bytes;
}

int block_forward(const Dims &D, int hidden, float eps, const void *X, const bra_block_params &p, void *Xout,
                  int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path, hipStream_t st)
{
    const BlockWs w = carve_block(D, hidden, bra_bytes, ws);
    const long M = (long)D.B * D.N;
    int rc = launch_token_ln<kPos>(D, (const bf16_t *)X, nullptr, p, p.ln1_gamma, p.ln1_beta, w.x1, w.xn, eps, st);
    if (rc != BRA_OK) return rc;
    rc = (path == BRA_PATH_MFMA)
             ? mfma_forward(D, w.xn, p.Wqkv, p.Wo, p.Wlce, w.y, Ir_out_opt, Ir_in_opt, w.inner, st)
             : generic_forward(D, w.xn, p.Wqkv, p.Wo, p.Wlce, w.y, Ir_out_opt, Ir_in_opt, w.inner, st);
    if (rc != BRA_OK) return rc;
    // X2 takes X1's place: every lane reads the elements it overwrites
    rc = launch_token_ln<kAdd>(D, w.x1, w.y, p, p.ln2_gamma, p.ln2_beta, w.x1, w.xn, eps, st);
    if (rc != BRA_OK) return rc;
    rc = gemm_bf16(w.xn, (const bf16_t *)p.W1, M, D.C, hidden, w.hd, p.b1, nullptr, true, K_BLK_MLP_IN, st);
    if (rc != BRA_OK) return rc;
    return gemm_bf16(w.hd, (const bf16_t *)p.W2, M, hidden, D.C, (bf16_t *)Xout, p.b2, w.x1, false, K_BLK_MLP_OUT, st);
}

}  // namespace bra
