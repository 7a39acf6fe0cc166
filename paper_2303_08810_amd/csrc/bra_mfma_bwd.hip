// Backward pass of the layer on the matrix cores (bf16 tensors, heads of 32 or 64 channels, C a
// multiple of 64 up to 4096, at most 4096 routing entries per image), with the routing index held fixed.
//
// Chain rule through Eq. 6-7 and Eq. 1-2, with O = Attention(Q, K^g, V^g) + LCE(V), Y = O Wo:
//     dO = dY Wo^T                     projection kernel with Wo^T as its matrix
//     P  = softmax(scale Q K^T)        recomputed per (region, head) from the re-projected Q, K
//     dP = dO V^T,  dS = scale P o (dP - D),  D = rowsum(P o dP)
//     dQ = dS K                        k_attn_bwd_q, one workgroup per query region; it also leaves the
//                                      row statistics (log-sum-exp and D) and the attention output
//     dK = dS^T Q,  dV = P^T dO        k_attn_bwd_kv, one workgroup per KEY region: it finds the query
//                                      regions routed to it in Ir, recomputes their P and dS from the
//                                      statistics and sums in registers, so no atomic adds are needed
//     O += LCE(V), dV += LCE^T(dO) (the correlation with the taps reversed) and
//     dWlce[c][ky][kx] = sum_t dO[t][c] V[t + (ky - 2, kx - 2)][c]       k_lce_bwd
//     dX = [dQ | dK | dV] Wqkv^T,  dWqkv = X^T [dQ | dK | dV]      k_bwd_proj, one pass over the gradient map
//     dWo = O^T dY                     k_gemm_tn (contraction over tokens)
// All products take bf16 operands and accumulate in float32; dQ, dK, dV and dO are rounded to
// bf16 between the kernels (they are matrix-core operands of the next product).  The weight
// gradients are summed from per-workgroup partial sums in a fixed order (k_reduce_parts).
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
// value of key 16 t + 4 g + j for this lane's query (accumulator layout of S^T = K Q^T); NDT tiles of
// 16 channels (a head).
template <int NDT>
__device__ __forceinline__ void keys_contract(const bf16_t *T, int pitch, const float (&vals)[4][4], int col,
                                              int g, int i, f32x4 (&acc)[NDT])
{
#pragma unroll
    for (int tp = 0; tp < 2; ++tp) {
        const float pv[8] = {vals[2 * tp][0], vals[2 * tp][1], vals[2 * tp][2], vals[2 * tp][3],
                             vals[2 * tp + 1][0], vals[2 * tp + 1][1], vals[2 * tp + 1][2], vals[2 * tp + 1][3]};
        const bf16x8 pb = pack8(pv);
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
            acc[dt] = mfma16(tr_operand(T, pitch, 32 * tp, col + 16 * dt, g, i), pb, acc[dt]);
    }
}

// The attention kernels are built for heads of DH = 32 or 64 channels and take HPW heads per
// workgroup: up to 128 channels' worth for small regions (a (16-token tile, head) pair per
// wavefront), one head where a region fills several tiles by itself, so that more, lighter workgroups
// share a compute unit.  CW = DH HPW channels of each row are staged; the layer's C and its number
// of heads are run-time values (row pitch of the maps, HPW divides the number of heads).
template <int DH, int HPW, int QR = 64, int KR = 64>
struct BwdSmem {
    static constexpr int CW = DH * HPW;
    // elements per row of the token tiles: the 16-byte row reads and the transposing reads stay
    // conflict-free, and four workgroups of the C = 64 kernels share a compute unit's LDS
    static constexpr int CS = CW + 8;
    // K, V tiles of KR rows, then Q, dO tiles of QR rows: 64 each, or 16 on the side that holds one
    // region's tokens when a region has at most 16 (a third workgroup then fits beside two)
    static constexpr int ktile = KR * CS, qtile = QR * CS;
    static constexpr size_t q_bytes = (size_t)2 * (ktile + qtile) * 2;       // the four tiles
    static constexpr size_t stat_off = q_bytes;                              // float lse[HPW][64], dsum[HPW][64]
    static constexpr size_t list_off = stat_off + 2 * HPW * 64 * sizeof(float);   // int count, pad, list[]
    static size_t kv_bytes(int entries) { return list_off + 16 + (size_t)entries * sizeof(int); }
};

// Token (within the image) of slot s of region j (Sec. 3.2: regions tile the map row-major).
__device__ __forceinline__ int region_token(const Dims &D, int region, int slot)
{
    const int ry = region / D.S, rx = region % D.S, sy = slot / D.rw, sx = slot % D.rw;
    return (ry * D.rh + sy) * D.W + rx * D.rw + sx;
}

// Channels c0 .. c0 + CW - 1 of ROWS rows of two token maps (row pitch C) -> registers -> LDS tiles
// of pitch CW + 8; tok(row) names the token of a tile row within the image (-1: a row of zeros).
template <int CW, int ROWS = 64>
struct RowRegs {
    static constexpr int CHUNKS = ROWS * (CW / 8), NL = (CHUNKS + 255) / 256;
    u32x4 r0[NL], r1[NL];
};

template <int CW, int ROWS, typename Tok>
__device__ __forceinline__ void fetch_rows(RowRegs<CW, ROWS> &R, const bf16_t *__restrict__ M0,
                                           const bf16_t *__restrict__ M1, size_t img, int C, int c0, Tok tok)
{
    constexpr int CH8 = CW / 8;
#pragma unroll
    for (int u = 0; u < RowRegs<CW, ROWS>::NL; ++u) {
        const int idx = threadIdx.x + 256 * u, row = idx / CH8, c8 = idx % CH8;
        const int t = idx < RowRegs<CW, ROWS>::CHUNKS ? tok(row) : -1;
        R.r0[u] = u32x4{0u, 0u, 0u, 0u};
        R.r1[u] = R.r0[u];
        if (t >= 0) {
            R.r0[u] = *(const u32x4 *)(M0 + (img + t) * C + c0 + c8 * 8);
            R.r1[u] = *(const u32x4 *)(M1 + (img + t) * C + c0 + c8 * 8);
        }
    }
}

template <int CW, int ROWS>
__device__ __forceinline__ void store_rows(bf16_t *T0, bf16_t *T1, const RowRegs<CW, ROWS> &R)
{
    constexpr int CS = CW + 8, CH8 = CW / 8;
#pragma unroll
    for (int u = 0; u < RowRegs<CW, ROWS>::NL; ++u) {
        const int idx = threadIdx.x + 256 * u, row = idx / CH8, c8 = idx % CH8;
        if (idx < RowRegs<CW, ROWS>::CHUNKS) {
            *(u32x4 *)(T0 + row * CS + c8 * 8) = R.r0[u];
            *(u32x4 *)(T1 + row * CS + c8 * 8) = R.r1[u];
        }
    }
}

// ---------------------------------------------------------------------------
// Query side of the attention backward (derivative of Eq. 6 with Eq. 1) for one (image, region,
// block of up to 64 queries) over the region's k n <= 64 routed keys.  The workgroup copies the K,
// V rows of the keys (found by index in the projected maps, Eq. 6) and the Q, dO rows of its
// queries into LDS.  A wavefront takes (16-query tile, head) pairs:
//     S^T = K Q^T and dP^T = V dO^T          (A operand: key rows, B operand: the query's row)
//     P = softmax over the keys, D = sum_j P_j dP_j, dS = scale P (dP - D)      (registers)
//     O^T = V^T P^T (attention output, needed for dWo) and dQ^T = K^T dS^T      (stored as bf16)
// and leaves lse = log2 of the softmax denominator (with the scaled maximum folded in, so that
// P = exp2(scale log2(e) s - lse)) and D per (token, head) for the key-side kernel.
// dQ has row pitch ldq (it is the first third of the [M][3C] gradient map).
template <int DH, int HPW, int QR>
__global__ __launch_bounds__(256) void k_attn_bwd_q(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                    const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                    const int32_t *__restrict__ Ir, bf16_t *__restrict__ O,
                                                    bf16_t *__restrict__ dQ, int ldq, float *__restrict__ lse,
                                                    float *__restrict__ dsum, Dims D, int qchunks)
{
    using L = BwdSmem<DH, HPW, QR, 64>;
    constexpr int CS = L::CS, CW = L::CW, NDT = DH / 16, NKS = DH / 32;
    const int C = D.C, HEADS = D.heads, HG = HEADS / HPW;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + L::ktile, *Qs = Vs + L::ktile, *dOs = Qs + L::qtile;

    const int h0 = ((int)blockIdx.x % HG) * HPW, bx = blockIdx.x / HG;       // first head of this workgroup
    const int qc = bx % qchunks, r = (bx / qchunks) % D.R, b = bx / (qchunks * D.R);
    const int nq = min(QR, D.n - 64 * qc), kn = D.kn;      // QR = 16: regions of at most 16 tokens
    const size_t img = (size_t)b * D.N;
    const int32_t *irow = Ir + ((size_t)b * D.R + r) * D.k;
    auto key_token = [&](int l) {          // key l of the gathered set (Eq. 6): slot l % n of routed region l / n
        if (l >= kn) return -1;
        return region_token(D, min(max(irow[l / D.n], 0), D.R - 1), l % D.n);
    };
    auto query_token = [&](int l) { return l < nq ? region_token(D, r, 64 * qc + l) : -1; };
    {
        // the query rows do not wait for the routing index: ask for them first
        RowRegs<CW, QR> qr;
        RowRegs<CW, 64> kr;
        fetch_rows<CW, QR>(qr, Q, dO, img, C, DH * h0, query_token);
        fetch_rows<CW, 64>(kr, K, V, img, C, DH * h0, key_token);
        store_rows<CW, QR>(Qs, dOs, qr);
        store_rows<CW, 64>(Ks, Vs, kr);
    }
    __syncthreads();

    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    const float c_exp = D.scale * 1.4426950408889634f;
    const int qtiles = (nq + 15) / 16;
#pragma unroll 1
    for (int task = w; task < qtiles * HPW; task += 4) {
        const int qt = task % qtiles, hl = task / qtiles, h = h0 + hl, col = DH * hl;   // col: within the tiles
        const int q = 16 * qt + i, my_qtok = query_token(q);
        bf16x8 qf[NKS], gf[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            qf[ks] = *(const bf16x8 *)(Qs + q * CS + col + 32 * ks + 8 * g);
            gf[ks] = *(const bf16x8 *)(dOs + q * CS + col + 32 * ks + 8 * g);
        }
        f32x4 s[4], dp[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            s[t] = dp[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                const bf16x8 vf = *(const bf16x8 *)(Vs + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                s[t] = mfma16(kf, qf[ks], s[t]);      // S^T[key 16 t + 4 g + j][query i]
                dp[t] = mfma16(vf, gf[ks], dp[t]);    // dP^T, same layout
            }
        }
        // a ragged key block: the missing keys get no weight (selects, not a branch between the matrix
        // instructions and the first read of their results)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) s[t][j] = (16 * t + 4 * g + j >= kn) ? -INFINITY : s[t][j];
        float mx = s[0][0];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) mx = fmaxf(mx, s[t][j]);
        mx = cross_row_max(mx);           // key 0 exists, so the maximum is finite
        const float mc = mx * c_exp;
        // the products below take the unnormalised e = exp(s - max): the factors 1 / sum and scale are
        // applied to their 8 results per lane instead of to the 16 weights
        float p[4][4], ds[4][4], lsum = 0.f, dd = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                p[t][j] = __builtin_amdgcn_exp2f(fmaf(s[t][j], c_exp, -mc));
                lsum += p[t][j];
                dd = fmaf(p[t][j], dp[t][j], dd);
            }
        lsum = cross_row_sum(lsum);
        const float inv = 1.0f / lsum;
        dd = cross_row_sum(dd) * inv;     // D = sum_j P_j dP_j
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j) ds[t][j] = p[t][j] * (dp[t][j] - dd);

        f32x4 oacc[NDT], qacc[NDT];
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) oacc[dt] = qacc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        keys_contract(Vs, CS, p, col, g, i, oacc);       // O^T[channel col + 16 dt + 4 g + j][query i]
        keys_contract(Ks, CS, ds, col, g, i, qacc);      // dQ^T, same layout
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            oacc[dt] *= inv;
            qacc[dt] *= inv * D.scale;
        }
        if (my_qtok >= 0) {
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) {
                *(u32x2 *)(O + (img + my_qtok) * C + DH * h + 16 * dt + 4 * g) = pack4(oacc[dt]);
                *(u32x2 *)(dQ + (img + my_qtok) * (size_t)ldq + DH * h + 16 * dt + 4 * g) = pack4(qacc[dt]);
            }
            if (g == 0) {
                lse[(img + my_qtok) * HEADS + h] = mc + __builtin_amdgcn_logf(lsum);     // v_log_f32: log2
                dsum[(img + my_qtok) * HEADS + h] = dd;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The query side for more than 64 routed keys per query: the keys are taken in blocks of 64, twice.
// First sweep, per (16-query tile, head) of a wavefront: the running maximum m, the sum l of
// e = exp(s - m), the unnormalised sums O~ = sum e V and D~ = sum e dP, all rescaled when m grows
// (the online softmax of the forward kernels); at its end O = O~ / l, D = D~ / l and
// lse = log2(l) + scale log2(e) m are final and stored.  Second sweep: P = exp2(scale log2(e) s - lse),
// dS = P (dP - D), dQ^T += K^T dS^T; dQ = scale dQ^T at the end.  The next block's K, V rows travel
// to registers while the current block is worked on.  A wavefront keeps the state of up to HPW pairs.
template <int DH, int HPW>
__global__ __launch_bounds__(256) void k_attn_bwd_q_blocks(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                           const bf16_t *__restrict__ V,
                                                           const bf16_t *__restrict__ dO,
                                                           const int32_t *__restrict__ Ir, bf16_t *__restrict__ O,
                                                           bf16_t *__restrict__ dQ, int ldq, float *__restrict__ lse,
                                                           float *__restrict__ dsum, Dims D, int qchunks)
{
    using L = BwdSmem<DH, HPW>;
    constexpr int CS = L::CS, CW = L::CW, NDT = DH / 16, NKS = DH / 32;
    const int C = D.C, HEADS = D.heads, HG = HEADS / HPW;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + L::ktile, *Qs = Vs + L::ktile, *dOs = Qs + L::qtile;

    const int h0 = ((int)blockIdx.x % HG) * HPW, bx = blockIdx.x / HG;
    const int qc = bx % qchunks, r = (bx / qchunks) % D.R, b = bx / (qchunks * D.R);
    const int nq = min(64, D.n - 64 * qc), kn = D.kn, nblocks = (kn + 63) / 64;
    const size_t img = (size_t)b * D.N;
    // the region's routing row in LDS: key addresses need it block after block
    int *ir_s = (int *)(smem + L::q_bytes);
    for (int e = threadIdx.x; e < D.k; e += 256) ir_s[e] = min(max(Ir[((size_t)b * D.R + r) * D.k + e], 0), D.R - 1);
    auto key_token = [&](int l) {          // key l of the gathered set (Eq. 6): slot l % n of routed region l / n
        return l < kn ? region_token(D, ir_s[l / D.n], l % D.n) : -1;
    };
    auto query_token = [&](int l) { return l < nq ? region_token(D, r, 64 * qc + l) : -1; };
    // DEPTH blocks of K, V rows are in flight in registers.  One is enough: the sweeps are bound by
    // their vector work (about 200 instructions per pair and block), and with three blocks in flight
    // the kernel was slower (99 against 90 us on a 2 x 128 x 128 x 64 map with 1024 keys per query)
    constexpr int DEPTH = 1;
    const int total = 2 * nblocks;        // both sweeps, as one sequence of blocks
    RowRegs<CW, 64> kr[DEPTH];
    {
        RowRegs<CW, 64> qr;
        fetch_rows<CW, 64>(qr, Q, dO, img, C, DH * h0, query_token);
        store_rows<CW, 64>(Qs, dOs, qr);
    }
    __syncthreads();                      // ir_s is in place
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (d < total) fetch_rows<CW, 64>(kr[d], K, V, img, C, DH * h0, [&](int l) { return key_token(64 * (d % nblocks) + l); });
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    const float c_exp = D.scale * 1.4426950408889634f;
    const int qtiles = (nq + 15) / 16, ntasks = qtiles * HPW;

    float m[HPW], l[HPW], dd[HPW];        // per pair: maximum, sum, D~ (first sweep); then lse in m, D in dd
    f32x4 acc[HPW][NDT];                  // O~^T, then dQ^T: [channel 16 dt + 4 g + j of the head][query i]
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
        m[u] = -INFINITY;
        l[u] = dd[u] = 0.f;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) acc[u][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll 1
    for (int t0 = 0; t0 < total; t0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int step = t0 + d;
            if (step >= total) break;
            const int sweep = step >= nblocks ? 1 : 0, kb = step - sweep * nblocks;
            __syncthreads();              // the previous block's readers are done
            store_rows<CW, 64>(Ks, Vs, kr[d]);
            __syncthreads();
            if (step + DEPTH < total) {
                const int nb = (step + DEPTH) % nblocks;
                fetch_rows<CW, 64>(kr[d], K, V, img, C, DH * h0, [&](int l) { return key_token(64 * nb + l); });
            }
#pragma unroll
            for (int u = 0; u < HPW; ++u) {
                const int task = w + 4 * u;
                if (task >= ntasks) continue;
                const int qt = task % qtiles, col = DH * (task / qtiles), q = 16 * qt + i;
                bf16x8 qf[NKS], gf[NKS];
#pragma unroll
                for (int ks = 0; ks < NKS; ++ks) {
                    qf[ks] = *(const bf16x8 *)(Qs + q * CS + col + 32 * ks + 8 * g);
                    gf[ks] = *(const bf16x8 *)(dOs + q * CS + col + 32 * ks + 8 * g);
                }
                f32x4 s[4], dp[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    s[t] = dp[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
                        const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                        const bf16x8 vf = *(const bf16x8 *)(Vs + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                        s[t] = mfma16(kf, qf[ks], s[t]);      // S^T[key 16 t + 4 g + j][query i]
                        dp[t] = mfma16(vf, gf[ks], dp[t]);    // dP^T, same layout
                    }
                }
                // the ragged last block: the missing keys get no weight (selects, not a branch between the
                // matrix instructions and the first read of their results)
                const int left = kn - 64 * kb;
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) s[t][j] = (16 * t + 4 * g + j >= left) ? -INFINITY : s[t][j];
                float e[4][4];
                if (sweep == 0) {
                    float mx = s[0][0];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j) mx = fmaxf(mx, s[t][j]);
                    const float m_new = fmaxf(m[u], cross_row_max(mx));       // finite: key 64 kb exists
                    const float alpha = __builtin_amdgcn_exp2f((m[u] - m_new) * c_exp);   // 0 on the first block
                    m[u] = m_new;
                    const float mc = m_new * c_exp;
                    float ls = 0.f, ds = 0.f;
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            e[t][j] = __builtin_amdgcn_exp2f(fmaf(s[t][j], c_exp, -mc));
                            ls += e[t][j];
                            ds = fmaf(e[t][j], dp[t][j], ds);
                        }
                    l[u] = fmaf(l[u], alpha, cross_row_sum(ls));
                    dd[u] = fmaf(dd[u], alpha, cross_row_sum(ds));
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) acc[u][dt] *= alpha;
                    keys_contract(Vs, CS, e, col, g, i, acc[u]);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            e[t][j] = __builtin_amdgcn_exp2f(fmaf(s[t][j], c_exp, -m[u])) * (dp[t][j] - dd[u]);
                    keys_contract(Ks, CS, e, col, g, i, acc[u]);
                }
            }
            if (kb + 1 < nblocks) continue;
            // end of a sweep: store O and the statistics, or dQ
#pragma unroll
            for (int u = 0; u < HPW; ++u) {
                const int task = w + 4 * u;
                if (task >= ntasks) continue;
                const int qt = task % qtiles, h = h0 + task / qtiles;
                const int tok = query_token(16 * qt + i);
                if (sweep == 0) {
                    const float inv = 1.0f / l[u];
                    const float lse2 = fmaf(m[u], c_exp, __builtin_amdgcn_logf(l[u]));      // v_log_f32: log2
                    const float dfin = dd[u] * inv;
                    if (tok >= 0) {
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt)
                            *(u32x2 *)(O + (img + tok) * C + DH * h + 16 * dt + 4 * g) = pack4(acc[u][dt] * inv);
                        if (g == 0) {
                            lse[(img + tok) * HEADS + h] = lse2;
                            dsum[(img + tok) * HEADS + h] = dfin;
                        }
                    }
                    m[u] = lse2;
                    dd[u] = dfin;
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) acc[u][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
                } else if (tok >= 0) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt)
                        *(u32x2 *)(dQ + (img + tok) * (size_t)ldq + DH * h + 16 * dt + 4 * g) =
                            pack4(acc[u][dt] * D.scale);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Key side of the attention backward for one (image, key region j, block of up to 64 of its
// tokens).  The workgroup collects the routing entries Ir[b][i][.] == j (every query region i
// that attends to region j, once per entry), ordered by entry number when there are at most 256
// (then the summation order, and so the result, is fixed).  The queries of those regions form one
// list of rows, taken 64 at a time: their Q, dO rows and statistics go to LDS, and a wavefront
// holding a (16-key tile, head) pair forms
//     S = Q K^T and dP = dO V^T              (A operand: query rows, B operand: the key's row)
//     P = exp2(scale log2(e) S - lse), dS = scale P (dP - D)               (registers)
//     dV^T += dO^T P and dK^T += Q^T dS      (A operand by transposing reads, B = P, dS as they are)
// in float32 registers across all query blocks; at the end dK, dV of its tokens are stored once as
// bf16 into the second and third thirds of the [M][3C] gradient map (dKV points at the second).
// Regions that no query attends to get zeros.
template <int DH, int HPW, int KR>
__global__ __launch_bounds__(256) void k_attn_bwd_kv(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                     const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                     const int32_t *__restrict__ Ir, const float *__restrict__ lse,
                                                     const float *__restrict__ dsum, bf16_t *__restrict__ dKV,
                                                     int ld, Dims D, int kchunks)
{
    using L = BwdSmem<DH, HPW, 64, KR>;
    constexpr int CS = L::CS, CW = L::CW, NDT = DH / 16, NKS = DH / 32;
    const int C = D.C, HEADS = D.heads, HG = HEADS / HPW;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + L::ktile, *Qs = Vs + L::ktile, *dOs = Qs + L::qtile;
    float *lse_s = (float *)(smem + L::stat_off), *dd_s = lse_s + HPW * 64;
    int *count = (int *)(smem + L::list_off), *list = count + 4;

    const int h0 = ((int)blockIdx.x % HG) * HPW, bx = blockIdx.x / HG;       // first head of this workgroup
    const int kc = bx % kchunks, jr = (bx / kchunks) % D.R, b = bx / (kchunks * D.R);
    const int nk = min(KR, D.n - 64 * kc);                  // KR = 16: regions of at most 16 tokens
    const size_t img = (size_t)b * D.N;
    auto key_token = [&](int l) { return l < nk ? region_token(D, jr, 64 * kc + l) : -1; };
    if (threadIdx.x == 0) *count = 0;
    __syncthreads();
    const int entries = D.R * D.k;
    const int32_t *irb = Ir + (size_t)b * entries;
    {
        RowRegs<CW, KR> kr;               // in flight while the routing index is searched
        fetch_rows<CW, KR>(kr, K, V, img, C, DH * h0, key_token);
        for (int e = threadIdx.x; e < entries; e += 256)
            if (min(max(irb[e], 0), D.R - 1) == jr) list[atomicAdd(count, 1)] = e;
        store_rows<CW, KR>(Ks, Vs, kr);
    }
    __syncthreads();
    const int m = *count;
    if (m > 1 && m <= 256) {              // rank sort: entry numbers are distinct
        const int mine = (int)threadIdx.x < m ? list[threadIdx.x] : 0;
        int rank = 0;
        for (int u = 0; u < m; ++u) rank += list[u] < mine;
        __syncthreads();
        if ((int)threadIdx.x < m) list[rank] = mine;
    }

    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    const float c_exp = D.scale * 1.4426950408889634f;
    const int ktiles = (nk + 15) / 16, ntasks = ktiles * HPW;
    f32x4 acc[HPW][2 * NDT];              // per task of this wavefront: dV^T (NDT channel tiles), then dK^T
#pragma unroll
    for (int u = 0; u < HPW; ++u)
#pragma unroll
        for (int a = 0; a < 2 * NDT; ++a) acc[u][a] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int rows = m * D.n;
    // row r0 + l of the list of queries: slot .. % n of the query region of entry .. / n
    auto query_token = [&](int r0, int l) {
        const int rho = r0 + l;
        return rho < rows ? region_token(D, list[rho / D.n] / D.k, rho % D.n) : -1;
    };
    // the next block's rows and statistics travel to registers while the current block is worked on
    RowRegs<CW, 64> next;
    float next_lse = INFINITY, next_dd = 0.f;
    const int srow = threadIdx.x / HPW, sh = threadIdx.x % HPW;          // statistics: one (row, head) per thread
    auto fetch_block = [&](int r0) {
        fetch_rows<CW, 64>(next, Q, dO, img, C, DH * h0, [&](int l) { return query_token(r0, l); });
        if ((int)threadIdx.x < 64 * HPW) {
            const int t = query_token(r0, srow);
            // a missing row: P = exp2(-inf) = 0 and dS = 0
            next_lse = t >= 0 ? lse[(img + t) * HEADS + h0 + sh] : INFINITY;
            next_dd = t >= 0 ? dsum[(img + t) * HEADS + h0 + sh] : 0.f;
        }
    };
    __syncthreads();                      // the list is in place
    if (rows > 0) fetch_block(0);
    for (int r0 = 0; r0 < rows; r0 += 64) {
        if (r0 > 0) __syncthreads();      // the previous block's readers are done
        store_rows<CW, 64>(Qs, dOs, next);
        if ((int)threadIdx.x < 64 * HPW) {
            lse_s[sh * 64 + srow] = next_lse;
            dd_s[sh * 64 + srow] = next_dd;
        }
        __syncthreads();
        if (r0 + 64 < rows) fetch_block(r0 + 64);
        const int qtiles = (min(64, rows - r0) + 15) / 16;
#pragma unroll
        for (int u = 0; u < HPW; ++u) {
            const int task = w + 4 * u;
            if (task >= ntasks) continue;
            const int kt = task % ktiles, h = task / ktiles, col = DH * h;      // h, col: within the workgroup's heads
            bf16x8 kf[NKS], vf[NKS];
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                kf[ks] = *(const bf16x8 *)(Ks + (16 * kt + i) * CS + col + 32 * ks + 8 * g);
                vf[ks] = *(const bf16x8 *)(Vs + (16 * kt + i) * CS + col + 32 * ks + 8 * g);
            }
            float p[4][4], ds[4][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t < qtiles) {
                    f32x4 s = {0.f, 0.f, 0.f, 0.f}, dp = s;
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) {
                        const bf16x8 qf = *(const bf16x8 *)(Qs + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                        const bf16x8 gf = *(const bf16x8 *)(dOs + (16 * t + i) * CS + col + 32 * ks + 8 * g);
                        s = mfma16(qf, kf[ks], s);        // S[query 16 t + 4 g + j][key i]
                        dp = mfma16(gf, vf[ks], dp);
                    }
                    const f32x4 l4 = *(const f32x4 *)(lse_s + h * 64 + 16 * t + 4 * g);
                    const f32x4 d4 = *(const f32x4 *)(dd_s + h * 64 + 16 * t + 4 * g);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        p[t][j] = __builtin_amdgcn_exp2f(fmaf(s[j], c_exp, -l4[j]));
                        ds[t][j] = p[t][j] * (dp[j] - d4[j]);      // the factor scale: on the sums, at the end
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) p[t][j] = ds[t][j] = 0.f;
                }
            }
#pragma unroll
            for (int tp = 0; tp < 2; ++tp) {
                if (2 * tp >= qtiles) continue;
                const float pv[8] = {p[2 * tp][0], p[2 * tp][1], p[2 * tp][2], p[2 * tp][3],
                                     p[2 * tp + 1][0], p[2 * tp + 1][1], p[2 * tp + 1][2], p[2 * tp + 1][3]};
                const float dv[8] = {ds[2 * tp][0], ds[2 * tp][1], ds[2 * tp][2], ds[2 * tp][3],
                                     ds[2 * tp + 1][0], ds[2 * tp + 1][1], ds[2 * tp + 1][2], ds[2 * tp + 1][3]};
                const bf16x8 pb = pack8(pv), db = pack8(dv);
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    acc[u][dt] = mfma16(tr_operand(dOs, CS, 32 * tp, col + 16 * dt, g, i), pb, acc[u][dt]);
                    acc[u][NDT + dt] = mfma16(tr_operand(Qs, CS, 32 * tp, col + 16 * dt, g, i), db, acc[u][NDT + dt]);
                }
            }
        }
    }
    // acc[u][.][j] = gradient of channel col + 16 dt + 4 g + j of key 16 kt + i
#pragma unroll
    for (int u = 0; u < HPW; ++u) {
        const int task = w + 4 * u;
        if (task >= ntasks) continue;
        const int kt = task % ktiles, h = task / ktiles, col = DH * (h0 + h);
        const int t = key_token(16 * kt + i);
        if (t < 0) continue;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            *(u32x2 *)(dKV + (img + t) * (size_t)ld + col + 16 * dt + 4 * g) = pack4(acc[u][NDT + dt] * D.scale);
            *(u32x2 *)(dKV + (img + t) * (size_t)ld + C + col + 16 * dt + 4 * g) = pack4(acc[u][dt]);
        }
    }
}

// ---------------------------------------------------------------------------
// Part[blockIdx.x][a][o] = sum_t A[t][a] Bm[t][o] over the workgroup's share of the M tokens (the
// token contractions dWqkv = X^T dQKV and dWo = O^T dY): a 64 x 64 block (blockIdx.y, blockIdx.z)
// of the [Ca][ldo] output per workgroup, both operands staged as [64 tokens][64 channels] LDS
// tiles and read with transposing reads.  Wavefront w forms rows 16 w .. 16 w + 15 of the block.
// k_reduce_parts then sums the partial matrices.
__global__ __launch_bounds__(256) void k_gemm_tn(const bf16_t *__restrict__ A, int lda,
                                                 const bf16_t *__restrict__ Bm, int ldb, float *__restrict__ Part,
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
    float *out = Part + (size_t)blockIdx.x * (64 * gridDim.y) * ldo;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j) out[(size_t)(a0 + 16 * w + 4 * g + j) * ldo + b0 + 16 * ct + i] = acc[ct][j];
}

// ---------------------------------------------------------------------------
// The two products that read the gradient map G = [dQ | dK | dV] ([M][3C]), in one pass over it:
//     dX = G Wqkv^T                    (derivative of Eq. 3 with respect to X)
//     dWqkv = X^T G                    (with respect to the weights; contraction over tokens)
// A workgroup of C / 16 wavefronts streams 64-token tiles of G and X through LDS (the next tile
// travels to registers meanwhile).  Wavefront w holds rows 16 w .. 16 w + 15 of Wqkv as A
// operands and forms dX^T[channel][token] = Wqkv G^T tile by tile (B operand: a token's row of G);
// and it keeps rows 16 w .. 16 w + 15 of dWqkv as 3C / 16 accumulators over all its tiles (both
// operands by transposing reads), written at the end as Part[workgroup][C][3C] for k_reduce_parts.
// With WO the same pass also streams O and dY and keeps dWo = O^T dY (rows 16 w .. 16 w + 15, C / 16
// accumulators more: taken where the registers allow it, C = 64).
template <int C, bool WO>
struct ProjSmem {
    static constexpr int GS = 3 * C + 8, XS = C + 8;
    static constexpr size_t bytes = (size_t)64 * (GS + (WO ? 3 : 1) * XS) * 2;
};

template <int C, bool WO>
__global__ __launch_bounds__(4 * C) void k_bwd_proj(const bf16_t *__restrict__ G, const bf16_t *__restrict__ X,
                                                    const bf16_t *__restrict__ Wqkv, bf16_t *__restrict__ dX,
                                                    float *__restrict__ Part, const bf16_t *__restrict__ O,
                                                    const bf16_t *__restrict__ dY, float *__restrict__ PartO, long M,
                                                    int tiles, int tiles_per_wg)
{
    constexpr int NT = 4 * C, GS = ProjSmem<C, WO>::GS, XS = ProjSmem<C, WO>::XS, KS = 3 * C / 32, CT = 3 * C / 16;
    constexpr int GCH = 3 * C / 8, XCH = C / 8, GL = 64 * GCH / NT, XL = 64 * XCH / NT, OT = WO ? C / 16 : 1;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Gs = (bf16_t *)smem, *Xs = Gs + 64 * GS, *Os = Xs + 64 * XS, *Ys = Os + 64 * XS;
    const int w = threadIdx.x / 64, lane = threadIdx.x % 64, g = lane / 16, i = lane % 16;
    bf16x8 wf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) wf[ks] = *(const bf16x8 *)(Wqkv + (size_t)(16 * w + i) * 3 * C + 32 * ks + 8 * g);
    f32x4 acc[CT], acco[OT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ct = 0; ct < OT; ++ct) acco[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 gr[GL], xr[XL], orr[WO ? XL : 1], yr[WO ? XL : 1];
    auto fetch = [&](long tile) {
#pragma unroll
        for (int u = 0; u < GL; ++u) {
            const int idx = threadIdx.x + NT * u;
            const long t = tile * 64 + idx / GCH;
            gr[u] = u32x4{0u, 0u, 0u, 0u};
            if (t < M) gr[u] = *(const u32x4 *)(G + (size_t)t * 3 * C + (idx % GCH) * 8);
        }
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int idx = threadIdx.x + NT * u;
            const long t = tile * 64 + idx / XCH;
            xr[u] = u32x4{0u, 0u, 0u, 0u};
            if (WO) orr[u] = yr[u] = xr[u];
            if (t < M) {
                xr[u] = *(const u32x4 *)(X + (size_t)t * C + (idx % XCH) * 8);
                if (WO) {
                    orr[u] = *(const u32x4 *)(O + (size_t)t * C + (idx % XCH) * 8);
                    yr[u] = *(const u32x4 *)(dY + (size_t)t * C + (idx % XCH) * 8);
                }
            }
        }
    };
    const int first = blockIdx.x * tiles_per_wg, last = min(tiles, first + tiles_per_wg);
    if (first < last) fetch(first);
    for (int tile = first; tile < last; ++tile) {
        if (tile > first) __syncthreads();          // the previous tile's readers are done
#pragma unroll
        for (int u = 0; u < GL; ++u) {
            const int idx = threadIdx.x + NT * u;
            *(u32x4 *)(Gs + (idx / GCH) * GS + (idx % GCH) * 8) = gr[u];
        }
#pragma unroll
        for (int u = 0; u < XL; ++u) {
            const int idx = threadIdx.x + NT * u;
            *(u32x4 *)(Xs + (idx / XCH) * XS + (idx % XCH) * 8) = xr[u];
            if (WO) {
                *(u32x4 *)(Os + (idx / XCH) * XS + (idx % XCH) * 8) = orr[u];
                *(u32x4 *)(Ys + (idx / XCH) * XS + (idx % XCH) * 8) = yr[u];
            }
        }
        __syncthreads();
        if (tile + 1 < last) fetch(tile + 1);
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a = mfma16(wf[ks], *(const bf16x8 *)(Gs + (16 * rt + i) * GS + 32 * ks + 8 * g), a);
            const long t = (long)tile * 64 + 16 * rt + i;       // a[j] = dX[token t][channel 16 w + 4 g + j]
            if (t < M) *(u32x2 *)(dX + (size_t)t * C + 16 * w + 4 * g) = pack4(a);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 xa = tr_operand(Xs, XS, 32 * ks, 16 * w, g, i);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) acc[ct] = mfma16(xa, tr_operand(Gs, GS, 32 * ks, 16 * ct, g, i), acc[ct]);
            if (WO) {
                const bf16x8 oa = tr_operand(Os, XS, 32 * ks, 16 * w, g, i);
#pragma unroll
                for (int ct = 0; ct < OT; ++ct)
                    acco[ct] = mfma16(oa, tr_operand(Ys, XS, 32 * ks, 16 * ct, g, i), acco[ct]);
            }
        }
    }
    float *out = Part + (size_t)blockIdx.x * C * 3 * C;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j) out[(size_t)(16 * w + 4 * g + j) * 3 * C + 16 * ct + i] = acc[ct][j];
    if (WO) {
        float *outo = PartO + (size_t)blockIdx.x * C * C;
#pragma unroll
        for (int ct = 0; ct < OT; ++ct)
#pragma unroll
            for (int j = 0; j < 4; ++j) outo[(size_t)(16 * w + 4 * g + j) * C + 16 * ct + i] = acco[ct][j];
    }
}

// ---------------------------------------------------------------------------
// The three uses of the depth-wise 5x5 correlation (Eq. 7) in the backward pass, in one kernel.
// A tile is kLbTH x kLbTW tokens of one image and 64 channels; a thread handles a pair of channels
// and 4-token row segments.
//   phase 1, V with a 2-token halo in LDS:   O += LCE(V)  (the forward's O, for dWo) and the tap
//            gradients dWlce[c][ky][kx] = sum_t dO[t][c] V[t + (ky - 2, kx - 2)][c], 2 x 25 sums
//            kept in registers across the workgroup's tiles (V is zero outside the image)
//   phase 2, dO with its halo in the same LDS buffer:
//            dV += LCE^T(dO), the correlation with the taps reversed; dV has row pitch ldv
// Two workgroups per compute unit (the 50 tap sums, the unpacked weights and the halo rows in flight
// take that register budget; fetching the next phase's halo into registers ahead of time was
// measured slower, 92 against 68 us on a 64 x 56 x 56 x 64 map).  At the end the workgroup reduces its tap sums through
// LDS and writes Part[tile group][C][25] for k_reduce_parts.
constexpr int kLbTH = 4, kLbTW = 32, kLbHW = kLbTW + 4, kLbRows = (kLbTH + 4) * kLbHW, kLbPitch = 64 + 8;
constexpr int kLbLoads = (kLbRows * 8 + 255) / 256;
constexpr size_t kLbSmem = std::max((size_t)kLbRows * kLbPitch * 2, (size_t)4 * 32 * 50 * 4);

__device__ __forceinline__ void halo_fetch(u32x4 (&h)[kLbLoads], const bf16_t *__restrict__ M, size_t img_off,
                                           int y0, int x0, int c0, const Dims &D)
{
#pragma unroll
    for (int u = 0; u < kLbLoads; ++u) {
        const int idx = threadIdx.x + 256 * u, row = idx / 8, c8 = idx % 8;
        const int y = y0 - 2 + row / kLbHW, x = x0 - 2 + row % kLbHW;
        h[u] = u32x4{0u, 0u, 0u, 0u};
        if (idx < kLbRows * 8 && y >= 0 && y < D.H && x >= 0 && x < D.W)
            h[u] = *(const u32x4 *)(M + img_off + ((size_t)y * D.W + x) * D.C + c0 + c8 * 8);
    }
}

__device__ __forceinline__ void halo_store(bf16_t *Hs, const u32x4 (&h)[kLbLoads])
{
#pragma unroll
    for (int u = 0; u < kLbLoads; ++u) {
        const int idx = threadIdx.x + 256 * u;
        if (idx < kLbRows * 8) *(u32x4 *)(Hs + (idx / 8) * kLbPitch + (idx % 8) * 8) = h[u];
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_lce_bwd(bf16_t *__restrict__ O, bf16_t *__restrict__ dVm, int ldv,
                                                 const bf16_t *__restrict__ V, const bf16_t *__restrict__ dO,
                                                 const bf16_t *__restrict__ Wlce, float *__restrict__ Part, Dims D,
                                                 int tiles_total, int tiles_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Hs = (bf16_t *)smem;
    const int C = D.C, NCH = C / 64;
    const int ytiles = (D.H + kLbTH - 1) / kLbTH, xtiles = (D.W + kLbTW - 1) / kLbTW;
    const int cc = blockIdx.x % NCH, c0 = 64 * cc;
    const int first_tile = (blockIdx.x / NCH) * tiles_per_wg;
    const int last_tile = min(tiles_total, first_tile + tiles_per_wg);
    const int cpair = threadIdx.x % 32, grp = threadIdx.x / 32;
    unsigned wl[25];        // [W(c, 0..24) | W(c + 1, 0..24)] as 25 packed pairs
#pragma unroll
    for (int e = 0; e < 25; ++e) wl[e] = *(const unsigned *)(Wlce + (size_t)(c0 + 2 * cpair) * 25 + 2 * e);
    auto tap = [&](int ch, int t) {   // weight of tap t of channel c + ch
        const int e = 25 * ch + t;
        return (e & 1) ? bf16_hi(wl[e / 2]) : bf16_lo(wl[e / 2]);
    };
    float g0[25], g1[25];
#pragma unroll
    for (int e = 0; e < 25; ++e) g0[e] = g1[e] = 0.f;

    auto origin = [&](int tile, int &b, int &y0, int &x0) {
        b = tile / (xtiles * ytiles);
        y0 = ((tile / xtiles) % ytiles) * kLbTH;
        x0 = (tile % xtiles) * kLbTW;
    };
    for (int tile = first_tile; tile < last_tile; ++tile) {
        int b, y0, x0;
        origin(tile, b, y0, x0);
        const int th = min(kLbTH, D.H - y0), tw = min(kLbTW, D.W - x0);
        const size_t img_off = (size_t)b * D.N * C, img_tok = (size_t)b * D.N;
        __syncthreads();          // the previous tile's readers are done
        {
            u32x4 h[kLbLoads];
            halo_fetch(h, V, img_off, y0, x0, c0, D);
            halo_store(Hs, h);
        }
        __syncthreads();
#pragma unroll 1
        for (int task = grp; task < kLbTH * (kLbTW / 4); task += 8) {
            const int seg = task % (kLbTW / 4), r = task / (kLbTW / 4);
            if (r >= th || seg * 4 >= tw) continue;
            const size_t tok = (size_t)(y0 + r) * D.W + x0 + seg * 4;
            const unsigned *drow = (const unsigned *)(dO + img_off + tok * C + c0 + 2 * cpair);
            unsigned *orow = (unsigned *)(O + img_off + tok * C + c0 + 2 * cpair);
            unsigned o2[4];
            float d0[4], d1[4], a0[4] = {0.f, 0.f, 0.f, 0.f}, a1[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const bool in = seg * 4 + x < tw;
                const unsigned u = in ? drow[(size_t)x * (C / 2)] : 0u;
                o2[x] = in ? orow[(size_t)x * (C / 2)] : 0u;
                d0[x] = bf16_lo(u);
                d1[x] = bf16_hi(u);
            }
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                float v0[8], v1[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const unsigned u = *(const unsigned *)(Hs + ((r + ky) * kLbHW + seg * 4 + x) * kLbPitch + 2 * cpair);
                    v0[x] = bf16_lo(u);
                    v1[x] = bf16_hi(u);
                }
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) {
                    const float w0 = tap(0, ky * 5 + kx), w1 = tap(1, ky * 5 + kx);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        a0[x] = fmaf(w0, v0[x + kx], a0[x]);
                        a1[x] = fmaf(w1, v1[x + kx], a1[x]);
                        g0[ky * 5 + kx] = fmaf(d0[x], v0[x + kx], g0[ky * 5 + kx]);
                        g1[ky * 5 + kx] = fmaf(d1[x], v1[x + kx], g1[ky * 5 + kx]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);      // one halo row at a time: the tap sums fill the registers
            }
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (seg * 4 + x < tw)
                    orow[(size_t)x * (C / 2)] = pack_bf16(bf16_lo(o2[x]) + a0[x], bf16_hi(o2[x]) + a1[x]);
        }
        __syncthreads();
        {
            u32x4 h[kLbLoads];
            halo_fetch(h, dO, img_off, y0, x0, c0, D);
            halo_store(Hs, h);
        }
        __syncthreads();
#pragma unroll 1
        for (int task = grp; task < kLbTH * (kLbTW / 4); task += 8) {
            const int seg = task % (kLbTW / 4), r = task / (kLbTW / 4);
            if (r >= th || seg * 4 >= tw) continue;
            const size_t tok = img_tok + (size_t)(y0 + r) * D.W + x0 + seg * 4;
            unsigned *vrow = (unsigned *)(dVm + tok * ldv + c0 + 2 * cpair);
            unsigned o2[4];
            float a0[4] = {0.f, 0.f, 0.f, 0.f}, a1[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int x = 0; x < 4; ++x) o2[x] = seg * 4 + x < tw ? vrow[(size_t)x * (ldv / 2)] : 0u;
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                float v0[8], v1[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const unsigned u = *(const unsigned *)(Hs + ((r + ky) * kLbHW + seg * 4 + x) * kLbPitch + 2 * cpair);
                    v0[x] = bf16_lo(u);
                    v1[x] = bf16_hi(u);
                }
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) {
                    const float w0 = tap(0, 24 - (ky * 5 + kx)), w1 = tap(1, 24 - (ky * 5 + kx));
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        a0[x] = fmaf(w0, v0[x + kx], a0[x]);
                        a1[x] = fmaf(w1, v1[x + kx], a1[x]);
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (seg * 4 + x < tw)
                    vrow[(size_t)x * (ldv / 2)] = pack_bf16(bf16_lo(o2[x]) + a0[x], bf16_hi(o2[x]) + a1[x]);
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
        Part[((size_t)(blockIdx.x / NCH) * C + c0 + 2 * (idx / 50) + (idx % 50) / 25) * 25 + idx % 25] = v;
    }
}

// ---------------------------------------------------------------------------
// WT[o][c] = Wqkv[c][o] ([3C][C]) and WoT[o][c] = Wo[c][o], for the channel counts whose projection
// launch does not carry the rearrangement along.
__global__ void k_bwd_transpose(const bf16_t *__restrict__ Wqkv, const bf16_t *__restrict__ Wo,
                                bf16_t *__restrict__ WT, bf16_t *__restrict__ WoT, int C)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < 3 * C * C) WT[e] = Wqkv[(size_t)(e % C) * 3 * C + e / C];
    else if (e < 4 * C * C) WoT[e - 3 * C * C] = Wo[(size_t)((e - 3 * C * C) % C) * C + (e - 3 * C * C) / C];
}

// out[e] = sum_p part[p][e], p in a fixed order, for up to three arrays in one launch.  A workgroup
// of 1024 threads takes 1024 / slices elements x `slices` slices of p (a power of two up to 32, about
// the number of partial arrays), the slices summed through LDS.
struct ReduceJob {
    const float *part;
    float *out;
    int nparts, count, slices, blocks;
};

ReduceJob reduce_job(const float *part, float *out, int nparts, int count)
{
    int slices = 1;
    while (slices < 32 && slices < nparts) slices *= 2;
    const int elems = 1024 / slices;
    return ReduceJob{part, out, nparts, count, slices, (count + elems - 1) / elems};
}

__global__ __launch_bounds__(1024) void k_reduce_parts(ReduceJob j0, ReduceJob j1, ReduceJob j2)
{
    __shared__ float red[1024];
    int bi = blockIdx.x;
    ReduceJob job = j0;
    if (bi >= j0.blocks) {
        bi -= j0.blocks;
        job = j1;
        if (bi >= j1.blocks) {
            bi -= j1.blocks;
            job = j2;
        }
    }
    const int elems = 1024 / job.slices;
    const int x = threadIdx.x % elems, y = threadIdx.x / elems, e = bi * elems + x;
    float sum = 0.f;
    if (e < job.count)
#pragma unroll 8
        for (int p = y; p < job.nparts; p += job.slices) sum += job.part[(size_t)p * job.count + e];
    red[y * elems + x] = sum;
    __syncthreads();
    if (y == 0 && e < job.count) {
        float total = 0.f;
        for (int u = 0; u < job.slices; ++u) total += red[u * elems + x];
        job.out[e] = total;
    }
}

// ---------------------------------------------------------------------------
// Token shares of k_gemm_tn: about 384 workgroups over the 64 x 64 output blocks.
struct TnPlan {
    int gx, tokens_per_wg;
};

TnPlan tn_plan(long M, int Ca, int Cb)
{
    const long steps = (M + 63) / 64;
    const long want = std::max(1L, 384L / ((Ca / 64) * (Cb / 64)));
    const long per_wg = (steps + want - 1) / want;
    return TnPlan{(int)((steps + per_wg - 1) / per_wg), (int)(per_wg * 64)};
}

// Tiles of k_bwd_proj per workgroup: all workgroups resident at once.
struct ProjPlan {
    int tiles, per_wg, groups;
};

ProjPlan proj_plan(long M, int C)
{
    ProjPlan p;
    p.tiles = (int)((M + 63) / 64);
    const int slots = C == 64 ? 512 : 256;
    p.per_wg = (p.tiles + slots - 1) / slots;
    p.groups = (p.tiles + p.per_wg - 1) / p.per_wg;
    return p;
}

struct TapPlan {
    int tiles, per_wg, groups;
};

// Tiles of k_lce_bwd per workgroup: all workgroups resident at once (3 per compute unit).
TapPlan tap_plan(const Dims &D)
{
    const int ytiles = (D.H + kLbTH - 1) / kLbTH, xtiles = (D.W + kLbTW - 1) / kLbTW;
    const int slots = (int)experiment_value("BRA_LCE_SLOTS", 512) / (D.C / 64);
    TapPlan t;
    t.tiles = D.B * ytiles * xtiles;
    t.per_wg = (t.tiles + slots - 1) / slots;
    t.groups = (t.tiles + t.per_wg - 1) / t.per_wg;
    return t;
}

// k_bwd_proj keeps 3C / 16 accumulators per wavefront: up to C = 128; wider layers take the plain
// product for dX and k_gemm_tn for dWqkv.
bool fused_projection(int C) { return C <= 128; }

struct BwdWs {
    bf16_t *q, *k, *v, *dO, *o, *dqkv, *wt, *wot;
    float *lse, *dsum, *part_qkv, *part_o, *part_lce;
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
    const long M = (long)D.B * D.N;
    const size_t MC = (size_t)M * D.C, C = D.C;
    BwdWs w;
    w.q = (bf16_t *)take(MC * 2);
    w.k = (bf16_t *)take(MC * 2);
    w.v = (bf16_t *)take(MC * 2);
    w.dO = (bf16_t *)take(MC * 2);
    w.o = (bf16_t *)take(MC * 2);
    w.dqkv = (bf16_t *)take(MC * 6);
    w.lse = (float *)take((size_t)M * D.heads * 4);
    w.dsum = (float *)take((size_t)M * D.heads * 4);
    w.part_qkv = (float *)take((size_t)(fused_projection(D.C) ? proj_plan(M, D.C).groups : tn_plan(M, D.C, 3 * D.C).gx) *
                               3 * C * C * 4);
    w.part_o = (float *)take((size_t)std::max(tn_plan(M, D.C, D.C).gx, proj_plan(M, D.C).groups) * C * C * 4);
    w.part_lce = (float *)take((size_t)tap_plan(D).groups * 25 * C * 4);
    w.wt = (bf16_t *)take(3 * C * C * 2);
    w.wot = (bf16_t *)take(C * C * 2);
    w.bytes = off;
    return w;
}

bool launched() { return hipGetLastError() == hipSuccess; }

template <int DH, int HPW, int QR>
int attn_bwd_q(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    static bool opted = false;
    if (!opt_in(k_attn_bwd_q<DH, HPW, QR>, opted)) return BRA_ERR_LAUNCH;
    using L = BwdSmem<DH, HPW, QR, 64>;
    const int chunks = (D.n + 63) / 64;
    const long blocks = (long)D.B * D.R * chunks * (D.heads / HPW);
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL((k_attn_bwd_q<DH, HPW, QR>), dim3((unsigned)blocks), dim3(256), L::q_bytes, st, w.q, w.k, w.v,
                       w.dO, Ir, w.o, w.dqkv, 3 * D.C, w.lse, w.dsum, D, chunks);
    return launched() ? BRA_OK : BRA_ERR_LAUNCH;
}

template <int DH, int HPW>
int attn_bwd_q_blocks(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    static bool opted = false;
    if (!opt_in(k_attn_bwd_q_blocks<DH, HPW>, opted)) return BRA_ERR_LAUNCH;
    using L = BwdSmem<DH, HPW>;
    const int chunks = (D.n + 63) / 64;
    const long blocks = (long)D.B * D.R * chunks * (D.heads / HPW);
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL((k_attn_bwd_q_blocks<DH, HPW>), dim3((unsigned)blocks), dim3(256),
                       L::q_bytes + (size_t)D.k * sizeof(int), st, w.q, w.k, w.v, w.dO, Ir, w.o, w.dqkv, 3 * D.C, w.lse,
                       w.dsum, D, chunks);
    return launched() ? BRA_OK : BRA_ERR_LAUNCH;
}

template <int DH, int HPW, int KR>
int attn_bwd_kv(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    static bool opted = false;
    if (!opt_in(k_attn_bwd_kv<DH, HPW, KR>, opted)) return BRA_ERR_LAUNCH;
    using L = BwdSmem<DH, HPW, 64, KR>;
    const int chunks = (D.n + 63) / 64;
    const long blocks = (long)D.B * D.R * chunks * (D.heads / HPW);
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL((k_attn_bwd_kv<DH, HPW, KR>), dim3((unsigned)blocks), dim3(256), L::kv_bytes(D.R * D.k), st, w.q,
                       w.k, w.v, w.dO, Ir, w.lse, w.dsum, w.dqkv + D.C, 3 * D.C, D, chunks);
    return launched() ? BRA_OK : BRA_ERR_LAUNCH;
}

// Both attention kernels with HPW heads per workgroup (HPW divides the number of heads, DH HPW <= 128
// channels: the tiles then fill the LDS of half a compute unit at most).  Where a region's tokens
// alone make three or four 16-token tiles, the key side and the multi-block query side take one
// head per workgroup (measured on a 64 x 56 x 56 x 64 map with regions of 64 tokens: query side 40 us
// whole against 45 us split, key side 55 us whole against 52.5 us split).
template <int DH, int HPW>
int attn_bwd_heads(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    static const long split_above = experiment_value("BRA_BWD_HEAD_SPLIT", 32);
    int rc;
    const bool small = D.n <= 16;         // a region's tokens fit one 16-row tile
    if (D.kn <= 64) rc = small ? attn_bwd_q<DH, HPW, 16>(D, w, Ir, st) : attn_bwd_q<DH, HPW, 64>(D, w, Ir, st);
    else if (D.n > split_above) rc = attn_bwd_q_blocks<DH, 1>(D, w, Ir, st);
    else rc = attn_bwd_q_blocks<DH, HPW>(D, w, Ir, st);
    if (rc != BRA_OK) return rc;
    if (D.n > split_above) return attn_bwd_kv<DH, 1, 64>(D, w, Ir, st);
    return small ? attn_bwd_kv<DH, HPW, 16>(D, w, Ir, st) : attn_bwd_kv<DH, HPW, 64>(D, w, Ir, st);
}

// Heads per workgroup: the largest of 4, 2, 1 that divides the number of heads and keeps DH HPW <= 128.
int heads_per_workgroup(const Dims &D)
{
    for (int hpw = 4; hpw > 1; hpw /= 2)
        if (D.heads % hpw == 0 && D.d * hpw <= 128) return hpw;
    return 1;
}

int attn_bwd(const Dims &D, const BwdWs &w, const int32_t *Ir, hipStream_t st)
{
    const int hpw = heads_per_workgroup(D);
    if (D.d == 32) {
        if (hpw == 4) return attn_bwd_heads<32, 4>(D, w, Ir, st);
        if (hpw == 2) return attn_bwd_heads<32, 2>(D, w, Ir, st);
        return attn_bwd_heads<32, 1>(D, w, Ir, st);
    }
    if (hpw == 2) return attn_bwd_heads<64, 2>(D, w, Ir, st);
    return attn_bwd_heads<64, 1>(D, w, Ir, st);
}

int gemm_tn(const bf16_t *A, int lda, int Ca, const bf16_t *Bm, int ldb, int Cb, float *Part, long M, hipStream_t st)
{
    const TnPlan t = tn_plan(M, Ca, Cb);
    ProfScope ps(st, K_GEN_BACKWARD);
    hipLaunchKernelGGL(k_gemm_tn, dim3(t.gx, Ca / 64, Cb / 64), dim3(256), 0, st, A, lda, Bm, ldb, Part, Cb, M,
                       t.tokens_per_wg);
    return launched() ? BRA_OK : BRA_ERR_LAUNCH;
}

// The routing entries of an image must fit the key-side kernel's list in LDS.
constexpr int kBwdMaxEntries = 4096;

}  // namespace

// The projection kernels specialised by channel count (they also carry the weight transposes along).
static bool narrow_projection(int C) { return C == 64 || C == 128 || C == 256; }

bool mfma_backward_supported(const Dims &D)
{
    static const bool off = experiment_flag("BRA_NO_MFMA_BACKWARD");
    if (off || D.dtype != BRA_BF16 || (D.d != 32 && D.d != 64) || D.C % 64 != 0 || D.C > 4096) return false;
    if ((long)D.R * D.k > kBwdMaxEntries) return false;
    const long M = (long)D.B * D.N;
    return M * 3 * D.C < (1L << 40) && (long)D.B * D.R * ((D.n + 63) / 64) * D.heads <= 0x7fffffffL &&
           M <= 0x7fffffffL;
}

size_t mfma_backward_workspace_bytes(const Dims &D) { return carve_bwd(D, nullptr).bytes; }

int mfma_backward(const Dims &D, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                  const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                  hipStream_t st)
{
    const BwdWs w = carve_bwd(D, ws);
    const int C = D.C;
    const long M = (long)D.B * D.N;
    int rc;
    if (narrow_projection(C)) {
        // Q, K, V once more (Eq. 3); the launch also leaves Wqkv^T and Wo^T (a launch of its own for Wo^T
        // alone was measured 4 us slower)
        rc = mfma_project_qkv(D, X, Wqkv, w.q, w.k, w.v, st, Wo, w.wt, w.wot);
        if (rc != BRA_OK) return rc;
        rc = mfma_project(D, dY, w.wot, w.dO, st);                            // dO = dY Wo^T
    } else {
        {
            ProfScope ps(st, K_GEN_BACKWARD);
            hipLaunchKernelGGL(k_bwd_transpose, dim3((4 * C * C + 255) / 256), dim3(256), 0, st, (const bf16_t *)Wqkv,
                               (const bf16_t *)Wo, w.wt, w.wot, C);
            if (!launched()) return BRA_ERR_LAUNCH;
        }
        rc = wide_project_qkv(D, X, Wqkv, w.q, w.k, w.v, st);
        if (rc != BRA_OK) return rc;
        rc = gemm_bf16((const bf16_t *)dY, w.wot, M, C, C, w.dO, nullptr, nullptr, false, K_GEN_BACKWARD, st);
    }
    if (rc != BRA_OK) return rc;
    rc = attn_bwd(D, w, Ir, st);                                              // O, dQ; then dK, dV
    if (rc != BRA_OK) return rc;
    const TapPlan tp = tap_plan(D);
    {
        // O = attention + LCE(V) (Eq. 7), dV += LCE^T(dO), tap-gradient partial sums
        static bool opted = false;
        if (!opt_in(k_lce_bwd, opted)) return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_GEN_BACKWARD);
        hipLaunchKernelGGL(k_lce_bwd, dim3(tp.groups * (C / 64)), dim3(256), kLbSmem, st, w.o, w.dqkv + 2 * C, 3 * C,
                           w.v, w.dO, (const bf16_t *)Wlce, w.part_lce, D, tp.tiles, tp.per_wg);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    const ProjPlan pp = proj_plan(M, C);
    const bool with_o = C == 64;          // dWo = O^T dY rides in the same pass where the registers allow it
    if (fused_projection(C)) {
        // dX = [dQ | dK | dV] Wqkv^T and the partial sums of dWqkv = X^T [dQ | dK | dV] (and of dWo)
        static bool opted[2] = {false, false};
        if (!(C == 64 ? opt_in(k_bwd_proj<64, true>, opted[0]) : opt_in(k_bwd_proj<128, false>, opted[1])))
            return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_GEN_BACKWARD);
        if (C == 64)
            hipLaunchKernelGGL((k_bwd_proj<64, true>), dim3(pp.groups), dim3(256), (ProjSmem<64, true>::bytes), st,
                               w.dqkv, (const bf16_t *)X, (const bf16_t *)Wqkv, (bf16_t *)dX, w.part_qkv, w.o,
                               (const bf16_t *)dY, w.part_o, M, pp.tiles, pp.per_wg);
        else
            hipLaunchKernelGGL((k_bwd_proj<128, false>), dim3(pp.groups), dim3(512), (ProjSmem<128, false>::bytes), st,
                               w.dqkv, (const bf16_t *)X, (const bf16_t *)Wqkv, (bf16_t *)dX, w.part_qkv, nullptr,
                               nullptr, nullptr, M, pp.tiles, pp.per_wg);
        if (!launched()) return BRA_ERR_LAUNCH;
    } else {
        rc = gemm_bf16(w.dqkv, w.wt, M, 3 * C, C, (bf16_t *)dX, nullptr, nullptr, false, K_GEN_BACKWARD, st);
        if (rc != BRA_OK) return rc;
        rc = gemm_tn((const bf16_t *)X, C, C, w.dqkv, 3 * C, 3 * C, w.part_qkv, M, st);
        if (rc != BRA_OK) return rc;
    }
    if (!with_o) {
        rc = gemm_tn(w.o, C, C, (const bf16_t *)dY, C, C, w.part_o, M, st);
        if (rc != BRA_OK) return rc;
    }
    {
        const ReduceJob j0 = reduce_job(w.part_qkv, dWqkv, fused_projection(C) ? pp.groups : tn_plan(M, C, 3 * C).gx,
                                        3 * C * C);
        const ReduceJob j1 = reduce_job(w.part_o, dWo, with_o ? pp.groups : tn_plan(M, C, C).gx, C * C);
        const ReduceJob j2 = reduce_job(w.part_lce, dWlce, tp.groups, 25 * C);
        ProfScope ps(st, K_GEN_BACKWARD);
        hipLaunchKernelGGL(k_reduce_parts, dim3(j0.blocks + j1.blocks + j2.blocks), dim3(1024), 0, st, j0, j1, j2);
        if (!launched()) return BRA_ERR_LAUNCH;
    }
    return BRA_OK;
}

}  // namespace bra
