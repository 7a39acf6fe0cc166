// One whole BiFormer block around BRA (Sec. 3.4), bf16 tensors, float32 arithmetic:
//
//   k_token_ln<POS>   X1 = X + DWConv3x3(X) + bpos,  Xn = LayerNorm1(X1)      one pass over X
//   BRA               Y  = BRA(Xn)                   (Eq. 2-7; the kernel family picked for the shape)
//   C <= 256:  k_mlp_fused64 (C = 64, weights resident in LDS) or k_mlp_stream (weights streamed):
//                     Xout = X2 + MLP(LayerNorm2(X2)), X2 = X1 + Y, in one kernel
//   otherwise:
//   k_token_ln<ADD>   X2 = X1 + Y,                   Xn = LayerNorm2(X2)
//   gemm_bf16         Hd = GELU(Xn W1 + b1)          bias and activation in the product's epilogue
//   gemm_bf16         Xout = X2 + Hd W2 + b2         bias and residual in the epilogue
//
// The normalisation and residual links follow the pre-norm residual reading stated with the
// entry point's declaration.  float32 tensors and sizes that are not multiples of 64 go to the
// scalar kernels of the generic family instead.
#include "bra_mfma_dev.h"

#include <stdlib.h>

namespace bra {

using namespace mfma;

namespace {

constexpr int kPos = 0, kAdd = 1;

// A token's C channels are shared by G consecutive lanes (G a power of two that divides
// C / 8, at most 64): lane `sub` owns the 8-channel chunks sub, sub + G, ..  A workgroup has
// 256 / G token slots and walks `iters` consecutive groups of that many tokens.
// ONE (C / 8 <= G): a lane owns one chunk for every token, so its convolution weights (packed),
// bias, gamma and beta stay in registers and a token's values never leave them.  Otherwise the
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
    // they stay packed in 36 registers and are widened where they are used
    auto load_w = [&](int c0, unsigned (&raw)[36]) {
        const u32x4 *src = (const u32x4 *)(Wpos + (size_t)c0 * 9);
#pragma unroll
        for (int q = 0; q < 9; ++q) {
            const u32x4 v = src[q];
            raw[4 * q] = v[0]; raw[4 * q + 1] = v[1]; raw[4 * q + 2] = v[2]; raw[4 * q + 3] = v[3];
        }
    };
    auto weight = [&](const unsigned (&raw)[36], int e, int t) {
        const int idx = 9 * e + t;
        return (idx & 1) ? bf16_hi(raw[idx / 2]) : bf16_lo(raw[idx / 2]);
    };
    auto tap_weights = [&](const unsigned (&raw)[36], int t, float (&wt)[8]) {
#pragma unroll
        for (int e = 0; e < 8; ++e) wt[e] = weight(raw, e, t);
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
    auto values = [&](long tok, bool ok, int y, int x, int c0, const unsigned (&w)[36], const float (&bias)[8], float (&v)[8]) {
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
        // all eight neighbours are requested at once; one outside the map (zero padding) is
        // read from the nearest row / column inside instead and blanked after it arrives
        const bool in_y[3] = {y > 0, true, ok && y < H - 1}, in_x[3] = {x > 0, true, ok && x < W - 1};
        const int off_y[3] = {in_y[0] ? -W * C : 0, 0, in_y[2] ? W * C : 0};
        const int off_x[3] = {in_x[0] ? -C : 0, 0, in_x[2] ? C : 0};
        u32x4 nb[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (t == 4) continue;
            nb[t] = *(const u32x4 *)(centre + (off_y[t / 3] + off_x[t % 3]));
        }
        {
            float wt[8];
            tap_weights(w, 4, wt);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaf(wt[e], xc[e], xc[e] + bias[e]);
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (t == 4) continue;
            const u32x4 z = (in_y[t / 3] && in_x[t % 3]) ? nb[t] : u32x4{0u, 0u, 0u, 0u};
            float f[8], wt[8];
            unpack(z, f);
            tap_weights(w, t, wt);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaf(wt[e], f[e], v[e]);
        }
    };
    auto group_sum = [&](float s) {
        for (int off = 1; off < G; off *= 2) s += __shfl_xor(s, off);
        return s;
    };

    // consecutive workgroups (neighbouring rows of the map) run on one XCD and meet in its L2
    const long first = (long)swizzled_block() * slots * iters;
    if (first >= tokens) return;
    const long row_first = first / W;
    const int x_first = (int)(first - row_first * W), y_first = (int)(row_first % H);
    const float w_inv = 1.0f / (float)W, h_inv = 1.0f / (float)H;
    unsigned w[36];
    float bias[8], gm[8], bt[8];
    // ONE: lanes sub >= C / 8 of a token's group (C / 8 not a power of two) carry no chunk: they
    // stand on the last chunk, add nothing to the sums and store nothing
    const bool lane_on = sub < CH;
    const int c_one = 8 * min(sub, CH - 1);
    if (ONE) {
        if (MODE == kPos) {
            load8(bpos + c_one, bias);
            load_w(c_one, w);
        }
        load8(gamma + c_one, gm);
        load8(beta + c_one, bt);
    }
    for (int it = 0; it < iters; ++it) {
        const long tok_raw = first + (long)it * slots + slot;
        const bool valid = tok_raw < tokens;
        const long tok = valid ? tok_raw : tokens - 1;          // lanes past the end redo the last token, store nothing
        // coordinates from the workgroup's first token (uniform: scalar arithmetic) plus this
        // lane's small distance from it; a lane past the end stands on the map's first token for
        // the neighbour tests (it reads the last token only and stores nothing)
        const int xs = valid ? x_first + it * slots + slot : 0;
        const int qx = fast_div(xs, w_inv), x = xs - qx * W;
        const int ys = valid ? y_first + qx : 0;
        const int y = ys - fast_div(ys, h_inv) * H;

        if (ONE) {
            if (MODE == kPos) {
                // the packed weights are re-declared as changed, so that their widened forms
                // (72 more registers) are formed where they are used instead of kept across tokens
#pragma unroll
                for (int q = 0; q < 36; ++q) asm volatile("" : "+v"(w[q]));
            }
            float v[8];
            values(tok, valid, y, x, c_one, w, bias, v);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[e];
            const float mean = group_sum(lane_on ? s : 0.f) * c_inv;
            float q = 0.f, d[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { d[e] = v[e] - mean; q = fmaf(d[e], d[e], q); }
            const float rstd = __builtin_amdgcn_rsqf(group_sum(lane_on ? q : 0.f) * c_inv + eps);
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = fmaf(d[e] * rstd, gm[e], bt[e]);
            if (valid && lane_on) {
                *(bf16x8 *)(Sum + (size_t)tok * C + c_one) = pack8(v);
                *(bf16x8 *)(Norm + (size_t)tok * C + c_one) = pack8(o);
            }
        } else {
            float s = 0.f;
            for (int q = 0; q < NC; ++q) {
                const int c0 = 8 * (sub + G * q);
                if (MODE == kPos) { load_w(c0, w); load8(bpos + c0, bias); }
                float v[8];
                values(tok, valid, y, x, c0, w, bias, v);
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
            const float rstd = __builtin_amdgcn_rsqf(group_sum(qq) * c_inv + eps);
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

// X2 = X1 + Y, LayerNorm2, both MLP layers and the last residual link in one kernel for C = 64,
// hidden = 64 HT: nothing between X1, Y and Xout passes through memory.
// A wavefront owns 16 tokens at a time, lane (g, i) = token i; everything is formed transposed
// (outputs x tokens) so that the matrix cores' result layout (rows 4 g .. 4 g + 3 of column i)
// is again an operand layout:
//   * the lane reads channels 32 ks + 8 g + (0..7) of X1 and Y (ks = 0, 1), adds and normalises
//     them (sums over the four lane groups of a token) and packs them: the B operands of
//     Hd^T = W1^T Xn^T, whose A operands (contraction slot (g, e) = channel 32 ks + 8 g + e)
//     come out of a row-major copy of W1 in LDS by the transposing read;
//   * two result tiles of Hd^T (hidden units 16 t1 + 4 g + jj), after bias and GELU, are packed
//     as they are: slot (g, e) of contraction step ks2 stands for hidden unit
//     16 (2 ks2 + e / 4) + 4 g + e % 4, and W2's fragments are read from its LDS copy to match;
//   * row 4 g + jj of output tile t stands for channel 32 (t / 2) + 8 g + 4 (t % 2) + jj, so the
//     lane ends up with the channels it started with: X2 is still in its registers for the
//     residual link and it stores 16 contiguous bytes per step.
// The weights are copied to LDS once per workgroup; the wavefronts then walk the 16-token
// tiles in a grid-stride loop, requesting the next tile's rows before they work on the current.
constexpr int kMlpWaves = 8;

// LDS copies of the weights, laid out so that a transposing read (per 16 lanes: 4 rows x 4
// pieces of 8 bytes) of 32 lanes touches every bank once (64 banks of 4 bytes):
//   W1 [64][HID]: row pitch = 160 bytes modulo 256 (rows 0..3 start 40 banks apart, their four
//                 adjacent pieces fill 8 banks each), and 128 bytes more after every 8 rows
//                 (the neighbouring lane group reads 8 rows further on);
//   W2 [HID][64]: row pitch 192 bytes (its pieces are 16 bytes apart and fill half of a 64-byte
//                 span), and 8 bytes more after every 4 rows (the neighbouring lane group, 4 rows
//                 further on, fills the other half).
template <int HT>
struct MlpSmem {
    static constexpr int HID = 64 * HT;
    static constexpr int P1 = HID + ((HT % 2) ? 16 : 80);      // bf16 elements
    static constexpr int G1 = 64;                              // extra elements per 8 rows
    static constexpr int P2 = 96, G2 = 4;                      // W2: pitch, extra elements per 4 rows
    static constexpr size_t w2_off = (size_t)(64 * P1 + 8 * G1) * 2;
    static constexpr size_t b1_off = w2_off + (size_t)(HID * P2 + (HID / 4) * G2) * 2;
    static constexpr size_t bytes = b1_off + (size_t)HID * 4;
    static_assert((P1 / 2) % 64 == 40 && w2_off % 16 == 0 && b1_off % 16 == 0, "layout");
};

template <int HT>
__global__ __launch_bounds__(64 * kMlpWaves) __attribute__((amdgpu_waves_per_eu(4, 4)))
void k_mlp_fused64(const bf16_t *__restrict__ X1, const bf16_t *__restrict__ Y, const bf16_t *__restrict__ W1,
                   const float *__restrict__ b1, const bf16_t *__restrict__ W2, const float *__restrict__ b2,
                   const float *__restrict__ gamma, const float *__restrict__ beta, bf16_t *__restrict__ Xout,
                   long tokens, float eps)
{
    typedef MlpSmem<HT> SM;
    constexpr int C = 64, HID = SM::HID, NK2 = HID / 32, P1 = SM::P1, G1 = SM::G1, P2 = SM::P2, G2 = SM::G2;
    constexpr int NTH = 64 * kMlpWaves;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *W1s = (bf16_t *)smem;                       // row-major copies of the weights; the operand
    bf16_t *W2s = (bf16_t *)(smem + SM::w2_off);        // fragments come out of them by the transposing read
    float *b1s = (float *)(smem + SM::b1_off);
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave, g = lane / 16, i = lane % 16;

    for (int q = tid; q < C * (HID / 8); q += NTH) {
        const int k = q / (HID / 8), cg = q % (HID / 8);
        *(u32x4 *)(W1s + k * P1 + (k / 8) * G1 + 8 * cg) = *(const u32x4 *)(W1 + (size_t)k * HID + 8 * cg);
    }
    for (int q = tid; q < HID * (C / 8); q += NTH) {
        const int hid = q / (C / 8), cg = q % (C / 8);
        const u32x4 v = *(const u32x4 *)(W2 + (size_t)hid * C + 8 * cg);
        u32x2 *dst = (u32x2 *)(W2s + hid * P2 + (hid / 4) * G2 + 8 * cg);      // 8-byte aligned only
        dst[0] = u32x2{v[0], v[1]};
        dst[1] = u32x2{v[2], v[3]};
    }
    for (int q = tid; q < HID; q += NTH) b1s[q] = b1[q];

    // this lane's channels 32 ks + 8 g + e: gamma, beta, b2
    float gm[2][8], bt[2][8], bo[2][8];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int c0 = 32 * ks + 8 * g + 4 * h;
            const f32x4 a = *(const f32x4 *)(gamma + c0), b = *(const f32x4 *)(beta + c0), c = *(const f32x4 *)(b2 + c0);
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) { gm[ks][4 * h + jj] = a[jj]; bt[ks][4 * h + jj] = b[jj]; bo[ks][4 * h + jj] = c[jj]; }
        }
    __syncthreads();

    const long tiles = (tokens + 15) / 16, stride = (long)gridDim.x * kMlpWaves;
    // tile = round * (8 grid) + wave * grid + block: the tiles of the last, partial round go to
    // one wavefront each of as many workgroups as possible, not to all wavefronts of a few
    long wt = (long)wave * gridDim.x + blockIdx.x;
    u32x4 xa[2], ya[2];
    auto request = [&](long tile) {
        const long tok = min(tile * 16 + i, tokens - 1);         // rows past the end repeat the last; never stored
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            xa[ks] = *(const u32x4 *)(X1 + (size_t)tok * C + 32 * ks + 8 * g);
            ya[ks] = *(const u32x4 *)(Y + (size_t)tok * C + 32 * ks + 8 * g);
        }
    };
    if (wt < tiles) request(wt);
    for (; wt < tiles; wt += stride) {
        // The lane's piece of a transposing read (16 lanes hand in 4 rows x 4 pieces of 4
        // elements, lane i receives column i of the 4 rows): row i / 4, piece i % 4.
        //   W1, step ks, tile t1:  rows 32 ks + 8 g + (0..3 | 4..7), columns 16 t1 + (0..15)
        //   W2, step ks2, tile t:  rows 32 ks2 + 4 g + (0..3) and + 16, columns = the channels
        //                          32 (t / 2) + 8 (i / 4) + 4 (t % 2) + i % 4 of result row i
        // The offsets are re-declared as changed for every tile, so that the reads stay where
        // they are used instead of moving out of the loop into 200 registers.
        int off1 = (8 * g + i / 4) * P1 + g * G1 + 4 * (i % 4), off2 = (4 * g + i / 4) * P2 + g * G2 + 8 * (i % 4);
        asm volatile("" : "+v"(off1), "+v"(off2));
        float x2[2][8];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x2[ks][2 * e] = bf16_lo(xa[ks][e]) + bf16_lo(ya[ks][e]);
                x2[ks][2 * e + 1] = bf16_hi(xa[ks][e]) + bf16_hi(ya[ks][e]);
            }
        const long tok = wt * 16 + i;
        if (wt + stride < tiles) request(wt + stride);

        // LayerNorm2 over the token's 64 channels: 16 here, the rest in lanes i + 16, 32, 48
        float s = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += x2[ks][e];
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        const float mean = s * (1.0f / C);
        float qq = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float d = x2[ks][e] - mean; qq = fmaf(d, d, qq); }
        qq += __shfl_xor(qq, 16);
        qq += __shfl_xor(qq, 32);
        const float rstd = __builtin_amdgcn_rsqf(qq * (1.0f / C) + eps);
        bf16x8 bx[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = fmaf((x2[ks][e] - mean) * rstd, gm[ks][e], bt[ks][e]);
            bx[ks] = pack8(v);
        }

        // the accumulators start from the biases (and, for the output, from X2)
        f32x4 acc2[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) acc2[t][jj] = bo[t / 2][4 * (t % 2) + jj] + x2[t / 2][4 * (t % 2) + jj];
#pragma unroll
        for (int ks2 = 0; ks2 < NK2; ++ks2) {
            float hv[8];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int t1 = 2 * ks2 + half;
                f32x4 a = *(const f32x4 *)(b1s + 16 * t1 + 4 * g);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const bf16_t *wp = W1s + off1 + ks * (32 * P1 + 4 * G1) + 16 * t1;
                    const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
                    const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 4 * P1));
                    a = mfma16(__builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]}), bx[ks], a);
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) hv[4 * half + jj] = gelu_f32(a[jj]);
            }
            const bf16x8 hb = pack8(hv);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bf16_t *wp = W2s + off2 + ks2 * (32 * P2 + 8 * G2) + 32 * (t / 2) + 4 * (t % 2);
                const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
                const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 16 * P2 + 4 * G2));
                acc2[t] = mfma16(__builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]}), hb, acc2[t]);
            }
        }
        if (tok < tokens) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = acc2[2 * ks + e / 4][e % 4];
                *(bf16x8 *)(Xout + (size_t)tok * C + 32 * ks + 8 * g) = pack8(v);
            }
        }
    }
}

template <int HT>
int launch_mlp_fused64(const Dims &D, const bf16_t *X1, const bf16_t *Y, const bra_block_params &p, bf16_t *Xout,
                       float eps, hipStream_t st)
{
    constexpr size_t smem = MlpSmem<HT>::bytes;
    static bool opted = false;
    if (!opted) {
        if (hipFuncSetAttribute((const void *)k_mlp_fused64<HT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return BRA_ERR_LAUNCH;
        opted = true;
    }
    const long tokens = (long)D.B * D.N, tiles = (tokens + 15) / 16;
    long grid = 256L * 2;                                        // two workgroups of 8 wavefronts share a compute unit
    if (grid > (tiles + kMlpWaves - 1) / kMlpWaves) grid = (tiles + kMlpWaves - 1) / kMlpWaves;
    ProfScope ps(st, K_BLK_MLP_FUSED);
    hipLaunchKernelGGL((k_mlp_fused64<HT>), dim3((unsigned)grid), dim3(64 * kMlpWaves), smem, st, X1, Y,
                       (const bf16_t *)p.W1, p.b1, (const bf16_t *)p.W2, p.b2, p.ln2_gamma, p.ln2_beta, Xout, tokens, eps);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

// The same single-kernel MLP half for C = 64 CT (CT = 1..4) and any hidden = 64 NB: the weights
// no longer fit in LDS, so the hidden layer is walked in blocks of 64 units.  Per block the
// workgroup (4 wavefronts, 16 tokens each, one tile per wavefront) holds the 64 columns of W1
// and the 64 rows of W2 in LDS (requested into registers one block ahead), forms
// GELU(Xn W1[:, block] + b1[block]) for its tokens and adds its product with W2[block, :] to the
// output accumulators, which start from X2 + b2.  Operand layouts, fragment reads and LDS
// pitches as in k_mlp_fused64 (W1's block has 64 columns: its pitch is that kernel's for
// hidden = 64; W2's rows are C wide: pitch C + 32 elements = 64 bytes modulo 256).
template <int CT>
struct MlpStreamSmem {
    static constexpr int C = 64 * CT;
    static constexpr int P1 = 80, G1 = 64;                    // W1 block [C][64]
    static constexpr int P2 = C + 32, G2 = 4;                 // W2 block [64][C]
    static constexpr size_t w2_off = (size_t)(C * P1 + (C / 8) * G1) * 2;
    static constexpr size_t v_off = w2_off + (size_t)(64 * P2 + 16 * G2) * 2;      // gamma, beta, b2 [C] each, then b1
    static_assert(w2_off % 16 == 0 && v_off % 16 == 0, "layout");
    static size_t bytes(int hidden) { return v_off + (size_t)(3 * C + hidden) * 4; }
};

template <int CT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(CT <= 2 ? 3 : 2, 4))) void k_mlp_stream(const bf16_t *__restrict__ X1, const bf16_t *__restrict__ Y,
                                                    const bf16_t *__restrict__ W1, const float *__restrict__ b1,
                                                    const bf16_t *__restrict__ W2, const float *__restrict__ b2,
                                                    const float *__restrict__ gamma, const float *__restrict__ beta,
                                                    bf16_t *__restrict__ Xout, long tokens, int hidden, float eps)
{
    typedef MlpStreamSmem<CT> SM;
    constexpr int C = SM::C, KS = C / 32, NT = C / 16, P1 = SM::P1, G1 = SM::G1, P2 = SM::P2, G2 = SM::G2;
    constexpr int NP = C / 32;          // 16-byte pieces per thread of one block of W1 (8 C pieces), and of W2
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *W1s = (bf16_t *)smem;
    bf16_t *W2s = (bf16_t *)(smem + SM::w2_off);
    float *gms = (float *)(smem + SM::v_off), *bts = gms + C, *b2s = bts + C, *b1s = b2s + C;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave, g = lane / 16, i = lane % 16;
    const int NB = hidden / 64;

    for (int q = tid; q < C; q += 256) { gms[q] = gamma[q]; bts[q] = beta[q]; b2s[q] = b2[q]; }
    for (int q = tid; q < hidden; q += 256) b1s[q] = b1[q];

    // this thread's pieces of a block: W1 rows k (8 pieces of 8 columns each), W2 rows of C / 8 pieces
    u32x4 r1[NP], r2[NP];
    auto request = [&](int nb) {
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int q = tid + 256 * u;
            r1[u] = *(const u32x4 *)(W1 + (size_t)(q / 8) * hidden + 64 * nb + 8 * (q % 8));
            r2[u] = *(const u32x4 *)(W2 + (size_t)(64 * nb + q / (C / 8)) * C + 8 * (q % (C / 8)));
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int q = tid + 256 * u;
            const int k = q / 8, h = q / (C / 8);
            *(u32x4 *)(W1s + k * P1 + (k / 8) * G1 + 8 * (q % 8)) = r1[u];
            u32x2 *dst = (u32x2 *)(W2s + h * P2 + (h / 4) * G2 + 8 * (q % (C / 8)));      // 8-byte aligned only
            dst[0] = u32x2{r2[u][0], r2[u][1]};
            dst[1] = u32x2{r2[u][2], r2[u][3]};
        }
    };
    request(0);

    const long tile = (long)blockIdx.x * 4 + wave;
    const long tok = tile * 16 + i;
    const long tok_c = min(tok, tokens - 1);                    // rows past the end repeat the last; never stored
    float x2[KS][8];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const u32x4 xa = *(const u32x4 *)(X1 + (size_t)tok_c * C + 32 * ks + 8 * g);
        const u32x4 ya = *(const u32x4 *)(Y + (size_t)tok_c * C + 32 * ks + 8 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x2[ks][2 * e] = bf16_lo(xa[e]) + bf16_lo(ya[e]);
            x2[ks][2 * e + 1] = bf16_hi(xa[e]) + bf16_hi(ya[e]);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) s += x2[ks][e];
    s += __shfl_xor(s, 16);
    s += __shfl_xor(s, 32);
    const float mean = s * (1.0f / C);
    float qq = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float d = x2[ks][e] - mean; qq = fmaf(d, d, qq); }
    qq += __shfl_xor(qq, 16);
    qq += __shfl_xor(qq, 32);
    const float rstd = __builtin_amdgcn_rsqf(qq * (1.0f / C) + eps);
    __syncthreads();                                            // the vectors are in LDS

    bf16x8 bx[KS];
    f32x4 acc2[NT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c0 = 32 * ks + 8 * g;
        float v[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const f32x4 gv = *(const f32x4 *)(gms + c0 + 4 * h), bv = *(const f32x4 *)(bts + c0 + 4 * h);
            const f32x4 ov = *(const f32x4 *)(b2s + c0 + 4 * h);
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                v[4 * h + jj] = fmaf((x2[ks][4 * h + jj] - mean) * rstd, gv[jj], bv[jj]);
                acc2[2 * ks + h][jj] = x2[ks][4 * h + jj] + ov[jj];      // output tile 2 ks + h, row 4 g + jj
            }
        }
        bx[ks] = pack8(v);
    }

    const int off1 = (8 * g + i / 4) * P1 + g * G1 + 4 * (i % 4), off2 = (4 * g + i / 4) * P2 + g * G2 + 8 * (i % 4);
    for (int nb = 0; nb < NB; ++nb) {
        if (nb) __syncthreads();                                // the previous block has been read
        park();
        __syncthreads();
        if (nb + 1 < NB) request(nb + 1);
#pragma unroll 1
        for (int ks2 = 0; ks2 < 2; ++ks2) {
            float hv[8];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int t1 = 2 * ks2 + half;
                f32x4 a = *(const f32x4 *)(b1s + 64 * nb + 16 * t1 + 4 * g);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16_t *wp = W1s + off1 + ks * (32 * P1 + 4 * G1) + 16 * t1;
                    const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
                    const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 4 * P1));
                    a = mfma16(__builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]}), bx[ks], a);
                }
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) hv[4 * half + jj] = gelu_f32(a[jj]);
            }
            const bf16x8 hb = pack8(hv);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const bf16_t *wp = W2s + off2 + ks2 * (32 * P2 + 8 * G2) + 32 * (t / 2) + 4 * (t % 2);
                const u32x2 w0 = __builtin_bit_cast(u32x2, lds_read_tr16(wp));
                const u32x2 w1 = __builtin_bit_cast(u32x2, lds_read_tr16(wp + 16 * P2 + 4 * G2));
                acc2[t] = mfma16(__builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]}), hb, acc2[t]);
            }
        }
    }
    if (tok < tokens) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = acc2[2 * ks + e / 4][e % 4];
            *(bf16x8 *)(Xout + (size_t)tok * C + 32 * ks + 8 * g) = pack8(v);
        }
    }
}

template <int CT>
int launch_mlp_stream(const Dims &D, int hidden, const bf16_t *X1, const bf16_t *Y, const bra_block_params &p,
                      bf16_t *Xout, float eps, hipStream_t st)
{
    const size_t smem = MlpStreamSmem<CT>::bytes(hidden);
    static size_t opted = 0;
    if (smem > opted) {
        if (hipFuncSetAttribute((const void *)k_mlp_stream<CT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)smem) != hipSuccess)
            return BRA_ERR_LAUNCH;
        opted = smem;
    }
    const long tokens = (long)D.B * D.N, grid = (tokens + 63) / 64;
    ProfScope ps(st, K_BLK_MLP_FUSED);
    hipLaunchKernelGGL((k_mlp_stream<CT>), dim3((unsigned)grid), dim3(256), smem, st, X1, Y, (const bf16_t *)p.W1,
                       p.b1, (const bf16_t *)p.W2, p.b2, p.ln2_gamma, p.ln2_beta, Xout, tokens, hidden, eps);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

// C = 64 .. 256 with any hidden that fits the LDS budget takes the block-streaming kernel.
bool mlp_stream_shape(const Dims &D, int hidden)
{
    static const bool off = experiment_flag("BRA_BLOCK_UNFUSED");
    if (off || D.C % 64 || D.C > 256 || hidden % 64) return false;
    const size_t fixed[5] = {0, MlpStreamSmem<1>::v_off, MlpStreamSmem<2>::v_off, MlpStreamSmem<3>::v_off,
                             MlpStreamSmem<4>::v_off};
    return fixed[D.C / 64] + (size_t)(3 * D.C + hidden) * 4 <= 160 * 1024;
}

// The single-kernel MLP half exists for C = 64 and hidden = 64, 128, 192 or 256.
bool mlp_fused_shape(const Dims &D, int hidden)
{
    static const bool off = experiment_flag("BRA_BLOCK_UNFUSED");
    return !off && D.C == 64 && hidden % 64 == 0 && hidden <= 256;
}

// lanes per token: the largest power of two that divides C / 8, at most 64
int lanes_per_token(int C)
{
    int G = 1;
    while (G < 64 && (C / 8) % (2 * G) == 0) G *= 2;
    return G;
}

// One chunk per lane with some lanes idle: the power of two that holds C / 8 chunks, where the
// idle share is at most a third (C = 192, 320, 384 ..); 0 where that does not apply.
int lanes_one_chunk(int C)
{
    const int CH = C / 8;
    if (CH > 64) return 0;
    int G = 1;
    while (G < CH) G *= 2;
    return 3 * (G - CH) <= G ? G : 0;
}

template <int MODE>
int launch_token_ln(const Dims &D, const bf16_t *A, const bf16_t *Badd, const bra_block_params &p, const float *gamma,
                    const float *beta, bf16_t *Sum, bf16_t *Norm, float eps, hipStream_t st)
{
    const long tokens = (long)D.B * D.N;
    const int g_one = lanes_one_chunk(D.C);
    const int G = g_one ? g_one : lanes_per_token(D.C), slots = 256 / G;
    const bool one = D.C / 8 <= G;
    // enough workgroups to fill the chip several times over, up to 8 token groups each
    static const long target = experiment_value("BRA_LN_WGS", 2048);
    long iters = tokens / ((long)slots * target);
    iters = iters < 1 ? 1 : (iters > 8 ? 8 : iters);
    const long grid = ((tokens + slots * iters - 1) / (slots * iters) + 7) / 8 * 8;      // whole rounds over the XCDs
    ProfScope ps(st, MODE == kPos ? K_BLK_POS_LN : K_BLK_ADD_LN);
    auto launch = [&](auto kernel, size_t smem) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), smem, st, A, Badd, (const bf16_t *)p.Wpos, p.bpos,
                           gamma, beta, Sum, Norm, D.H, D.W, D.C, tokens, G, (int)iters, eps);
    };
    if (one) launch(k_token_ln<MODE, true>, 0);
    else launch(k_token_ln<MODE, false>, (size_t)slots * D.C * sizeof(float));      // at most 4 x 4096 floats
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

// The matrix-core kernels of this file take bf16 tensors with C and hidden multiples of 64;
// everything else runs on the scalar kernels.
static bool block_fast(const Dims &D, int hidden)
{
    static const bool off = experiment_flag("BRA_BLOCK_GENERIC");
    return !off && D.dtype == BRA_BF16 && D.C % 64 == 0 && D.C <= 4096 && hidden % 64 == 0 && hidden <= (1 << 16);
}

bool block_supported(const Dims &D, int hidden)
{
    if ((long)D.B * D.N > 0x7fffffffL / 64 || hidden > (1 << 20)) return false;
    return block_fast(D, hidden) || (size_t)D.C * sizeof(float) * 4 <= 64 * 1024;
}

size_t block_workspace_bytes(const Dims &D, int hidden, size_t bra_bytes)
{
    if (!block_fast(D, hidden)) return generic_block_workspace_bytes(D, hidden, bra_bytes);
    return carve_block(D, hidden, bra_bytes, nullptr).bytes;
}

int block_forward(const Dims &D, int hidden, float eps, const void *X, const bra_block_params &p, void *Xout,
                  int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t bra_bytes, int path, hipStream_t st)
{
    if (!block_fast(D, hidden))
        return generic_block_forward(D, hidden, eps, X, p, Xout, Ir_out_opt, Ir_in_opt, ws, bra_bytes, path, st);
    const BlockWs w = carve_block(D, hidden, bra_bytes, ws);
    const long M = (long)D.B * D.N;
    int rc = launch_token_ln<kPos>(D, (const bf16_t *)X, nullptr, p, p.ln1_gamma, p.ln1_beta, w.x1, w.xn, eps, st);
    if (rc != BRA_OK) return rc;
    rc = (path == BRA_PATH_MFMA)
             ? mfma_forward(D, w.xn, p.Wqkv, p.Wo, p.Wlce, w.y, Ir_out_opt, Ir_in_opt, w.inner, st)
             : generic_forward(D, w.xn, p.Wqkv, p.Wo, p.Wlce, w.y, Ir_out_opt, Ir_in_opt, w.inner, st);
    if (rc != BRA_OK) return rc;
    if (mlp_fused_shape(D, hidden)) {
        switch (hidden / 64) {
        case 1: return launch_mlp_fused64<1>(D, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        case 2: return launch_mlp_fused64<2>(D, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        case 3: return launch_mlp_fused64<3>(D, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        default: return launch_mlp_fused64<4>(D, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        }
    }
    if (mlp_stream_shape(D, hidden)) {
        switch (D.C / 64) {
        case 1: return launch_mlp_stream<1>(D, hidden, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        case 2: return launch_mlp_stream<2>(D, hidden, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        case 3: return launch_mlp_stream<3>(D, hidden, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        default: return launch_mlp_stream<4>(D, hidden, w.x1, w.y, p, (bf16_t *)Xout, eps, st);
        }
    }
    // X2 takes X1's place: every lane reads the elements it overwrites
    rc = launch_token_ln<kAdd>(D, w.x1, w.y, p, p.ln2_gamma, p.ln2_beta, w.x1, w.xn, eps, st);
    if (rc != BRA_OK) return rc;
    rc = gemm_bf16(w.xn, (const bf16_t *)p.W1, M, D.C, hidden, w.hd, p.b1, nullptr, true, K_BLK_MLP_IN, st);
    if (rc != BRA_OK) return rc;
    return gemm_bf16(w.hd, (const bf16_t *)p.W2, M, hidden, D.C, (bf16_t *)Xout, p.b2, w.x1, false, K_BLK_MLP_OUT, st);
}

}  // namespace bra
