// float32 tensors, regions of 4 x 4 tokens, heads of 32 channels, at most 64 routed keys: the
// whole layer in two launches, all products on the float32 matrix-core instruction
// v_mfma_f32_16x16x4_f32 (lane 16 g + i holds A[row i][k g], B[k g][col i] and D[rows 4 g + j]
// [col i]; a lane that loads 4 consecutive floats of its row feeds 4 such products, the
// contraction index then runs over {16 s + 4 g' + e} in product e of step s: any order will do
// as long as both operands use the same one).
//
//   k_f32_qkv : workgroup = one region.  Q, K, V = X [Wq | Wk | Wv] (Eq. 3) of its 16 tokens, and
//               the sums of Q and K over them (Sec. 3.2: Q^r, K^r are the per-region means).
//   k_f32_attn: workgroup = one region.  Its row of A^r = Q^r (K^r)^T (Eq. 4) and the top-k of it
//               (Eq. 5), the gathered keys and values (Eq. 6), attention (Eq. 1), LCE (Eq. 7; 5 x 5
//               depth-wise correlation of V, zero padding) and W^o (Eq. 2).
//   k_f32_route: the same routing rows on their own, for routing-only calls.
#include "bra_mfma_dev.h"

namespace bra {

using namespace mfma;

namespace {

constexpr int kN = 16;       // tokens of a region
constexpr int kKeys = 64;    // keys of a region's attention at most

__device__ __forceinline__ f32x4 mfma_f32(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// token (in the image) of slot q of region r
__device__ __forceinline__ int region_token(const Dims &D, int r, int q)
{
    const int gy = r / D.S, gx = r - gy * D.S;
    return (gy * 4 + q / 4) * D.W + gx * 4 + q % 4;
}

template <int C>
__global__ __launch_bounds__(256) void k_f32_qkv(const float *__restrict__ X, const float *__restrict__ Wqkv,
                                                 float *__restrict__ QKV, float *__restrict__ Pq,
                                                 float *__restrict__ Pk, Dims D)
{
    const int b = blockIdx.x / D.R, r = blockIdx.x % D.R;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const size_t img = (size_t)b * D.N;
    const float *xrow = X + (img + region_token(D, r, i)) * C + 4 * g;
    f32x4 xa[C / 16];
#pragma unroll
    for (int s = 0; s < C / 16; ++s) xa[s] = *(const f32x4 *)(xrow + 16 * s);
    size_t orow[4];      // rows 4 g + j of the result
#pragma unroll
    for (int j = 0; j < 4; ++j) orow[j] = (img + region_token(D, r, 4 * g + j)) * 3 * C;
    for (int ct = wave; ct < 3 * C / 16; ct += 4) {      // 16 output channels at a time
        float wb[C / 16][4];
#pragma unroll
        for (int s = 0; s < C / 16; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) wb[s][e] = Wqkv[(size_t)(16 * s + 4 * g + e) * 3 * C + 16 * ct + i];
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < C / 16; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = mfma_f32(xa[s][e], wb[s][e], acc);
#pragma unroll
        for (int j = 0; j < 4; ++j) QKV[orow[j] + 16 * ct + i] = acc[j];
        if (16 * ct < 2 * C) {      // Q and K: sums over the region's tokens, in a fixed order
            float v = (acc[0] + acc[1]) + (acc[2] + acc[3]);
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            if (g == 0) {
                float *dst = 16 * ct < C ? Pq : Pk;
                dst[((size_t)b * D.R + r) * C + (16 * ct) % C + i] = v;
            }
        }
    }
}

// Row r of A^r of image b from the region sums (entry j to aff[j], j < 64; entries past R are not
// meaningful), by 256 threads: 4 lanes per key region, a quarter of the channels each.  Ends with a
// barrier.
template <int C>
__device__ __forceinline__ void route_row(const float *__restrict__ Pq_row, const float *__restrict__ Pk_img,
                                          int R, float sc, float *aff)
{
    const int jj = threadIdx.x / 4, cq = threadIdx.x % 4;
    const float *krow = Pk_img + (size_t)min(jj, R - 1) * C + cq * (C / 4);
    const float *qrow = Pq_row + cq * (C / 4);
    float a = 0.f;
#pragma unroll
    for (int c = 0; c < C / 4; c += 4) {
        const f32x4 q4 = *(const f32x4 *)(qrow + c), k4 = *(const f32x4 *)(krow + c);
#pragma unroll
        for (int e = 0; e < 4; ++e) a = fmaf(q4[e], k4[e], a);
    }
    a = dpp_fadd<0xB1>(a);
    a = dpp_fadd<0x4E>(a);
    if (cq == 0) aff[jj] = a * sc;
    __syncthreads();
}

template <int C>
__global__ __launch_bounds__(256) void k_f32_route(const float *__restrict__ Pq, const float *__restrict__ Pk,
                                                   int32_t *__restrict__ Ir, float *__restrict__ Ar, Dims D)
{
    __shared__ float aff[64];
    const int b = blockIdx.x / D.R, r = blockIdx.x % D.R;
    const size_t row = (size_t)b * D.R + r;
    const float inv_n = 1.0f / (float)kN;
    route_row<C>(Pq + row * C, Pk + (size_t)b * D.R * C, D.R, inv_n * inv_n, aff);
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        const float v = aff[lane];
        if (Ar && lane < D.R) Ar[row * D.R + lane] = v;
        wave_topk(v, lane, D.R, D.k, Ir + row * D.k);
    }
}

template <int C>
struct F32Smem {
    static constexpr int P = C + 4;                       // floats per row of the K, V, halo and O tiles (4 x odd: conflict-free 16-byte reads of 16 rows)
    static constexpr int SP = kKeys + 4;                  // floats per row of a score tile
    static constexpr int HEADS = C / 32;
    static constexpr size_t k_off = 0;
    static constexpr size_t v_off = k_off + (size_t)kKeys * P * 4;
    static constexpr size_t h_off = v_off + (size_t)kKeys * P * 4;        // V over the region and a 2-token halo: 8 x 8 tokens
    static constexpr size_t s_off = h_off + (size_t)64 * P * 4;           // scores / softmax weights [HEADS][16][SP]
    static constexpr size_t o_off = s_off + (size_t)HEADS * 16 * SP * 4;  // Q, later O = attention + LCE: [16][P]
    static constexpr size_t a_off = o_off + (size_t)16 * P * 4;           // affinities [64], routed regions [4]
    static constexpr size_t bytes = a_off + 64 * 4 + 16 * 4;
};

template <int C>
__global__ __launch_bounds__(256) void k_f32_attn(const float *__restrict__ QKV, const float *__restrict__ Pq,
                                                  const float *__restrict__ Pk, const int32_t *__restrict__ Ir_in,
                                                  int32_t *__restrict__ Ir_out, const float *__restrict__ Wlce,
                                                  const float *__restrict__ Wo, float *__restrict__ Y, Dims D)
{
    typedef F32Smem<C> SM;
    constexpr int P = SM::P, SP = SM::SP, HEADS = SM::HEADS;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float *Ks = (float *)(smem + SM::k_off), *Vs = (float *)(smem + SM::v_off), *Hs = (float *)(smem + SM::h_off);
    float *Ss = (float *)(smem + SM::s_off), *Os = (float *)(smem + SM::o_off);
    float *aff = (float *)(smem + SM::a_off);
    int32_t *irs = (int32_t *)(aff + 64);

    const int b = blockIdx.x / D.R, r = blockIdx.x % D.R;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const size_t img = (size_t)b * D.N;
    const size_t row = (size_t)b * D.R + r;
    const int gy = r / D.S, gx = r - gy * D.S;
    const int y0 = 4 * gy, x0 = 4 * gx;
    const int kn = D.k * kN;

    // requests that do not depend on the routing: W^o operands of this wavefront's output tiles,
    // LCE taps of this thread's channel, Q, V over the halo
    constexpr int NOT = C / 64;                            // output-channel tiles of 16 per wavefront
    float wo[NOT][C / 16][4];
#pragma unroll
    for (int u = 0; u < NOT; ++u)
#pragma unroll
        for (int s = 0; s < C / 16; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) wo[u][s][e] = Wo[(size_t)(16 * s + 4 * g + e) * C + 16 * (wave + 4 * u) + i];
    const int lc = threadIdx.x % C, lq0 = threadIdx.x / C;      // LCE: channel, first token; tokens lq0, lq0 + 256 / C, ..
    float tap[25];
#pragma unroll
    for (int t = 0; t < 25; ++t) tap[t] = Wlce[(size_t)lc * 25 + t];
    constexpr int C4 = C / 4;                              // 16-byte chunks of a row
    constexpr int NQ = 16 * C4 / 256, NH = 64 * C4 / 256;
    f32x4 qreg[NQ], hreg[NH];
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int idx = threadIdx.x + 256 * u;
        qreg[u] = *(const f32x4 *)(QKV + (img + region_token(D, r, idx / C4)) * 3 * C + 4 * (idx % C4));
    }
#pragma unroll
    for (int u = 0; u < NH; ++u) {
        const int idx = threadIdx.x + 256 * u;
        const int t = idx / C4, y = y0 - 2 + t / 8, x = x0 - 2 + t % 8;
        const bool ok = (unsigned)y < (unsigned)D.H && (unsigned)x < (unsigned)D.W;
        const f32x4 v = *(const f32x4 *)(QKV + (img + (ok ? y * D.W + x : 0)) * 3 * C + 2 * C + 4 * (idx % C4));
        hreg[u] = ok ? v : f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // routing (Eq. 4, 5): given, or this region's row of A^r and its k largest entries
    if (Ir_in) {
        if (threadIdx.x < D.k) irs[threadIdx.x] = region_index(Ir_in[row * D.k + threadIdx.x], D.R);
    } else {
        const float inv_n = 1.0f / (float)kN;
        route_row<C>(Pq + row * C, Pk + (size_t)b * D.R * C, D.R, inv_n * inv_n, aff);
        if (wave == 0) wave_topk(aff[lane], lane, D.R, D.k, irs);
    }
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int idx = threadIdx.x + 256 * u;
        *(f32x4 *)(Os + (idx / C4) * P + 4 * (idx % C4)) = qreg[u];
    }
#pragma unroll
    for (int u = 0; u < NH; ++u) {
        const int idx = threadIdx.x + 256 * u;
        *(f32x4 *)(Hs + (idx / C4) * P + 4 * (idx % C4)) = hreg[u];
    }
    __syncthreads();
    if (Ir_out && threadIdx.x < D.k) Ir_out[row * D.k + threadIdx.x] = Ir_in ? Ir_in[row * D.k + threadIdx.x] : irs[threadIdx.x];

    // gathered keys and values (Eq. 6): key l is token l % 16 of routed region l / 16
    constexpr int NK = kKeys * C4 / 256;
    {
        f32x4 kr[NK], vr[NK];
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int idx = threadIdx.x + 256 * u;
            const int key = min(idx / C4, kn - 1);      // rows past the end repeat the last key; masked below
            const float *src = QKV + (img + region_token(D, irs[key / kN], key % kN)) * 3 * C + 4 * (idx % C4);
            kr[u] = *(const f32x4 *)(src + C);
            vr[u] = *(const f32x4 *)(src + 2 * C);
        }
#pragma unroll
        for (int u = 0; u < NK; ++u) {
            const int idx = threadIdx.x + 256 * u;
            *(f32x4 *)(Ks + (idx / C4) * P + 4 * (idx % C4)) = kr[u];
            *(f32x4 *)(Vs + (idx / C4) * P + 4 * (idx % C4)) = vr[u];
        }
    }
    __syncthreads();

    // scores S = Q K^T per head, 16 queries x 16 keys per product chain
    for (int task = wave; task < HEADS * 4; task += 4) {
        const int h = task / 4, t = task % 4;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const f32x4 qa = *(const f32x4 *)(Os + i * P + 32 * h + 16 * s + 4 * g);
            const f32x4 kb = *(const f32x4 *)(Ks + (16 * t + i) * P + 32 * h + 16 * s + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = mfma_f32(qa[e], kb[e], acc);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) Ss[(h * 16 + 4 * g + j) * SP + 16 * t + i] = acc[j];
    }
    __syncthreads();
    // softmax over the kn keys of each (head, query) row (Eq. 1): lane = key
    for (int rowi = wave; rowi < HEADS * 16; rowi += 4) {
        float v = lane < kn ? Ss[rowi * SP + lane] * D.scale : -INFINITY;
        float m = v;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
        const float p = lane < kn ? __expf(v - m) : 0.f;
        float sum = p;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
        Ss[rowi * SP + lane] = p / sum;
    }
    __syncthreads();      // also: every wavefront has read Q from the O tile
    // attention output: 16 queries x 16 channels per product chain, into the O tile
    for (int task = wave; task < HEADS * 2; task += 4) {
        const int h = task / 2, ct = task % 2;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kKeys / 16; ++s) {
            const f32x4 pa = *(const f32x4 *)(Ss + (h * 16 + i) * SP + 16 * s + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = mfma_f32(pa[e], Vs[(16 * s + 4 * g + e) * P + 32 * h + 16 * ct + i], acc);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) Os[(4 * g + j) * P + 32 * h + 16 * ct + i] = acc[j];
    }
    __syncthreads();
    // + LCE (Eq. 7): thread = (channel, every (256 / C)-th token)
    for (int q = lq0; q < kN; q += 256 / C) {
        const int qy = q / 4, qx = q % 4;
        float a = 0.f;
#pragma unroll
        for (int ky = 0; ky < 5; ++ky)
#pragma unroll
            for (int kx = 0; kx < 5; ++kx) a = fmaf(tap[ky * 5 + kx], Hs[((qy + ky) * 8 + qx + kx) * P + lc], a);
        Os[q * P + lc] += a;
    }
    __syncthreads();
    // Y = O Wo (Eq. 2)
    f32x4 oa[C / 16];
#pragma unroll
    for (int s = 0; s < C / 16; ++s) oa[s] = *(const f32x4 *)(Os + i * P + 16 * s + 4 * g);
#pragma unroll
    for (int u = 0; u < NOT; ++u) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < C / 16; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = mfma_f32(oa[s][e], wo[u][s][e], acc);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            Y[(img + region_token(D, r, 4 * g + j)) * C + 16 * (wave + 4 * u) + i] = acc[j];
    }
}

template <typename K>
bool opt_in(K kernel, size_t bytes, bool &done)
{
    if (done || bytes <= 64 * 1024) return true;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return false;
    done = true;
    return true;
}

template <int C>
int forward_c(const Dims &D, const float *X, const float *Wqkv, const float *Wo, const float *Wlce, float *Y,
              int32_t *Ir_out_opt, const int32_t *Ir_in_opt, float *qkv, float *pq, float *pk, hipStream_t st)
{
    static bool opted = false;
    if (!opt_in(k_f32_attn<C>, F32Smem<C>::bytes, opted)) return BRA_ERR_LAUNCH;
    {
        ProfScope ps(st, K_GEN_GEMM_QKV);
        hipLaunchKernelGGL(k_f32_qkv<C>, dim3(D.B * D.R), dim3(256), 0, st, X, Wqkv, qkv, pq, pk, D);
    }
    {
        ProfScope ps(st, K_GEN_ATTENTION);
        hipLaunchKernelGGL(k_f32_attn<C>, dim3(D.B * D.R), dim3(256), F32Smem<C>::bytes, st, qkv, pq, pk, Ir_in_opt,
                           Ir_out_opt, Wlce, Wo, Y, D);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

template <int C>
int route_c(const Dims &D, const float *X, const float *Wqkv, int32_t *Ir, float *Ar_opt, float *qkv, float *pq,
            float *pk, hipStream_t st)
{
    {
        ProfScope ps(st, K_GEN_GEMM_QKV);
        hipLaunchKernelGGL(k_f32_qkv<C>, dim3(D.B * D.R), dim3(256), 0, st, X, Wqkv, qkv, pq, pk, D);
    }
    {
        ProfScope ps(st, K_GEN_TOPK);
        hipLaunchKernelGGL(k_f32_route<C>, dim3(D.B * D.R), dim3(256), 0, st, pq, pk, Ir, Ar_opt, D);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

}  // namespace

bool f32_small_ok(const Dims &D)
{
    static const bool off = experiment_flag("BRA_NO_F32_SMALL");
    return !off && D.dtype == BRA_F32 && D.rh == 4 && D.rw == 4 && D.d == 32 && (D.C == 64 || D.C == 128) &&
           D.R <= 64 && D.k * kN <= kKeys && (size_t)D.B * D.N * 3 * D.C < ((size_t)1 << 31);
}

int f32_small_forward(const Dims &D, const float *X, const float *Wqkv, const float *Wo, const float *Wlce, float *Y,
                      int32_t *Ir_out_opt, const int32_t *Ir_in_opt, float *qkv, float *pq, float *pk, hipStream_t st)
{
    if (D.C == 64) return forward_c<64>(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, qkv, pq, pk, st);
    return forward_c<128>(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, qkv, pq, pk, st);
}

int f32_small_route(const Dims &D, const float *X, const float *Wqkv, int32_t *Ir, float *Ar_opt, float *qkv,
                    float *pq, float *pk, hipStream_t st)
{
    if (D.C == 64) return route_c<64>(D, X, Wqkv, Ir, Ar_opt, qkv, pq, pk, st);
    return route_c<128>(D, X, Wqkv, Ir, Ar_opt, qkv, pq, pk, st);
}

}  // namespace bra
