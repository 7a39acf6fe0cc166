// Routed attention + LCE + W^o for regions of 64 n tokens and many key blocks (Eq. 6-7, Eq. 2),
// the kernel of the dense-prediction shapes (256-token regions, k = 4: 1024 keys per query).
//
// With heads of 32 channels a score costs 128 matrix-core flops but several vector
// instructions, and a workgroup's wavefronts spend most of a key block waiting on each other's
// results (LDS, matrix cores, the block barrier).  The layout answers both:
//   * a wavefront owns 32 queries (two 16-query tiles) of ONE head: every K fragment and every
//     V^T fragment read from LDS feeds two matrix products;
//   * the keys of a block are split between KSPLIT wavefronts with the same queries (each keeps
//     its own online-softmax state; the states are merged once, at the end): twice the
//     wavefronts per SIMD for the same LDS traffic, so that one wavefront's waits are another's work;
//   * Q arrives pre-multiplied by scale * log2(e) (the projection kernel does it on the float32
//     accumulators), and the reference score of the exponentials enters the score product as
//     its accumulator input: the scores leave the matrix cores as the arguments of 2^x;
//   * the reference follows the running maximum lazily (only when a score exceeds it by 2^8),
//     so a key block costs per score: half of a 3-way maximum, the 2^x, half a packed
//     conversion; the softmax denominators come from a product with an all-ones operand;
//   * key-block addresses come from a table built once per workgroup; K / V blocks of 64 routed
//     tokens are copied by index into a two-stage LDS ring, three blocks ahead in registers, with
//     waits that leave the later loads pending; one barrier per block.
#include "bra_mfma_dev.h"

#include <type_traits>

namespace bra {

using namespace mfma;

namespace {

template <int C>
struct Q32Smem {
    static constexpr int CS = C + 16;                                   // bf16 per K / V row (pitch 32 B x odd)
    static constexpr int OS = C + 4;                                    // floats per row of the output tile
    static constexpr size_t stage_bytes = (size_t)2 * 64 * CS * 2;      // K tile, then V tile
    static constexpr size_t x_off = (size_t)64 * OS * 4;                // softmax states to merge, behind the output tile
    static constexpr size_t w_off = 2 * stage_bytes;                    // LCE weights [25][C] float32
    static constexpr size_t h_off = w_off + (size_t)25 * C * 4;         // V halo tile, then the key-block table
    __host__ __device__ static size_t t_off(int halo_rows)      // the float32 LCE tile [64][OS] takes the halo tile's place
    {
        const size_t halo = (size_t)halo_rows * CS * 2, lce = (size_t)64 * OS * 4;
        return h_off + (((halo > lce ? halo : lce) + 15) & ~(size_t)15);
    }
    static size_t bytes(int halo_rows, int nblocks) { return t_off(halo_rows) + (size_t)nblocks * 4; }
};

// Maximum of floats that are known not to be NaN (matrix-core results of finite operands).
__device__ __forceinline__ float max2(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, INFINITY); }
__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

// LCE (Eq. 7) of a 64-token tile: 5x5 depth-wise cross-correlation of V over the halo tile Hs
// (rows of CS bf16, (qh + 4) x hw tokens, hw = rw + 4).  One task = (row of the tile, 4-token
// segment, channel pair): 8 results, kept in registers by lce_tasks and written by lce_store into
// the float32 tile Ls [64][OS] (which may take the halo tile's place once every task is done).
// Wl is [25][C] float32.  NTASK tasks per thread cover the 16 C / 2 tasks of a tile.
template <int C, int CS, int NT, int NTASK>
__device__ __forceinline__ void lce_tasks(const bf16_t *Hs, const float *Wl, int rw, int hw, float (&res)[NTASK][8])
{
    const int segs = rw / 4, cp_n = C / 2;
#pragma unroll
    for (int k = 0; k < NTASK; ++k) {
        const int task = (int)threadIdx.x + NT * k;
        const int cp = task % cp_n, seg = (task / cp_n) % segs, r = task / (cp_n * segs);
        const int c = 2 * cp;
#pragma unroll
        for (int e = 0; e < 8; ++e) res[k][e] = 0.f;
#pragma unroll
        for (int ky = 0; ky < 5; ++ky) {
            f32x2 wk[5];
#pragma unroll
            for (int kx = 0; kx < 5; ++kx) wk[kx] = *(const f32x2 *)(Wl + (ky * 5 + kx) * C + c);
            float v0[8], v1[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + seg * 4 + x) * CS + c);
                v0[x] = bf16_lo(u);
                v1[x] = bf16_hi(u);
            }
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) {
                    res[k][2 * x] = fmaf(wk[kx][0], v0[x + kx], res[k][2 * x]);
                    res[k][2 * x + 1] = fmaf(wk[kx][1], v1[x + kx], res[k][2 * x + 1]);
                }
        }
    }
}

template <int C, int OS, int NT, int NTASK>
__device__ __forceinline__ void lce_store(float *Ls, int rw, const float (&res)[NTASK][8])
{
    const int segs = rw / 4, cp_n = C / 2;
#pragma unroll
    for (int k = 0; k < NTASK; ++k) {
        const int task = (int)threadIdx.x + NT * k;
        const int cp = task % cp_n, seg = (task / cp_n) % segs, r = task / (cp_n * segs);
#pragma unroll
        for (int x = 0; x < 4; ++x)
            *(f32x2 *)(Ls + (r * rw + seg * 4 + x) * OS + 2 * cp) = f32x2{res[k][2 * x], res[k][2 * x + 1]};
    }
}

template <int C, int KSPLIT>
__global__ __launch_bounds__(4 * C * KSPLIT) __attribute__((amdgpu_waves_per_eu(2 * KSPLIT, 2 * KSPLIT)))
void k_attn_q32(AttnArgs A, Dims D)
{
    typedef Q32Smem<C> SM;
    constexpr int CS = SM::CS, OS = SM::OS, HEADS = C / 32, KS = C / 32, CH = C / 8;
    constexpr int NW = 2 * HEADS * KSPLIT, NT = 64 * NW;
    constexpr int NBT = 64 * CH / NT;           // 16-byte chunks per thread of a 64-row tile
    constexpr int NBH = 5;                      // halo chunks per thread and batch
    constexpr int NPF = 3;                      // key blocks held in registers ahead of the ring
    constexpr int TPW = 4 / KSPLIT;             // 16-key tiles of a block per wavefront
    constexpr float kSlack = 8.0f;              // the reference may lag the maximum by 2^8
    static_assert(KSPLIT == 1 || KSPLIT == 2, "one or two wavefronts per query tile pair");
    static_assert(KSPLIT == 1 || SM::x_off + (size_t)(NW / 2) * 64 * 20 * 4 <= 2 * SM::stage_bytes,
                  "the states to merge fit behind the output tile");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float *Wl = (float *)(smem + SM::w_off);
    bf16_t *Hs = (bf16_t *)(smem + SM::h_off);
    float *Os = (float *)smem;                  // O = attention + LCE; reuses the ring after the key loop
    const float *Ls = (const float *)Hs;        // LCE of the tile, in the halo tile's place

    const int wid = swizzled_block();
    if (wid >= A.total) return;
#ifdef BRA_EXPERIMENT
    // phase timestamps (100 MHz counter) of every workgroup, left in the first bytes of its own tile of Y
    unsigned long long trace_t[8];
#define BRA_TRACE(k) if (A.trace) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    BRA_TRACE(0);

    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int ks = wave % KSPLIT, pair = wave / KSPLIT;     // which keys of a block; which (head, query half)
    const int h = pair / 2, qhf = pair % 2;
    const int chunks = D.n / 64;                // query tiles per region
    const int qh = 64 / D.rw;                   // rows per query tile
    const int b = wid / (D.R * chunks);
    const int reg = (wid / chunks) % D.R;
    const int ch = wid % chunks;
    const float s_inv = 1.0f / (float)D.S;
    const int regy = fast_div(reg, s_inv);
    const int y0 = regy * D.rh + ch * qh, x0 = (reg - regy * D.S) * D.rw;
    const size_t img_off = (size_t)b * D.N * C;
    const int hw = D.rw + 4, hrows = (qh + 4) * hw;
    const float hw_inv = 1.0f / (float)hw, rw_inv = 1.0f / (float)D.rw;
    const int nblocks = D.kn / 64;

    const int32_t *irp = A.Ir_src + ((size_t)b * D.R + reg) * D.k;
    if (A.Ir_out && A.Ir_out != A.Ir_src && ch == 0)
        for (int p = threadIdx.x; p < D.k; p += NT) A.Ir_out[((size_t)b * D.R + reg) * D.k + p] = irp[p];

    // Requests that do not depend on the routing go first: V over the tile's halo, the LCE
    // weights, this lane's queries (B operands of S^T = K Q^T: tile qt holds queries
    // 32 qhf + 16 qt + i).
    constexpr int NTASK = (16 * C / 2 + NT - 1) / NT;      // LCE tasks per thread
    float lce[NTASK][8];
    bf16x8 qf[2];
    {
        u32x4 hreg[NBH];
        LceWeights<C> lw;
        lw.load(A.Wlce);
        tile_load<C, NBH, NT>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, 0);
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const int q = 32 * qhf + 16 * qt + i;
            const int qy = fast_div(q, rw_inv);
            const size_t tok = (size_t)(y0 + qy) * D.W + x0 + q - qy * D.rw;
            qf[qt] = *(const bf16x8 *)(A.Q + img_off + tok * C + 32 * h + 8 * g);
        }
        tile_store<C, CS, NBH, NT>(Hs, hreg, hrows, 0);
        for (int first = NT * NBH; first < hrows * CH; first += NT * NBH) {
            tile_load<C, NBH, NT>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, first);
            tile_store<C, CS, NBH, NT>(Hs, hreg, hrows, first);
        }
        lw.store(Wl);
    }

    // Where key block kb starts in the image (element offset of its first token): routed region
    // kb / chunks (Eq. 6: by index), row group kb % chunks of it.  Looked up once per workgroup, so
    // that the key loop issues nothing but the K / V loads themselves.
    int *blk = (int *)(smem + SM::t_off(hrows));
    for (int kb = threadIdx.x; kb < nblocks; kb += NT) {
        const int j = region_index(irp[kb / chunks], D.R);
        const int jy = fast_div(j, s_inv);
        blk[kb] = ((jy * D.rh + (kb % chunks) * qh) * D.W + (j - jy * D.S) * D.rw) * C;
    }
    // this thread's 16-byte chunks of a 64-token block (whole region rows: always inside the image)
    int voff[NBT], soff[NBT];      // where a chunk comes from (relative to the block) and where it goes in a stage
#pragma unroll
    for (int u = 0; u < NBT; ++u) {
        const int idx = (int)threadIdx.x + NT * u, row = idx / CH;
        const int ty = fast_div(row, rw_inv);
        voff[u] = (ty * D.W + row - ty * D.rw) * C + (idx % CH) * 8;
        soff[u] = row * CS + (idx % CH) * 8;
    }
    __syncthreads();
    BRA_TRACE(1);

    // K / V blocks of 64 routed tokens -> registers; block kb lives in set kb % NPF.  Blocks past
    // the end repeat the last one: the number of loads in flight is the same on every path, so
    // the waits before the LDS writes can leave the later blocks' loads pending.
    u32x4 pk[NPF][NBT], pv[NPF][NBT];
    auto request = [&](int kb, u32x4 (&kr)[NBT], u32x4 (&vr)[NBT]) {
        const int base = blk[min(kb, nblocks - 1)];
#pragma unroll
        for (int u = 0; u < NBT; ++u) {
            kr[u] = *(const u32x4 *)(A.K + img_off + (unsigned)(base + voff[u]));
            vr[u] = *(const u32x4 *)(A.V + img_off + (unsigned)(base + voff[u]));
        }
    };
    auto stage_k = [&](int kb) { return (bf16_t *)(smem + (size_t)(kb & 1) * SM::stage_bytes); };
    auto hand_over = [&](int kb, const u32x4 (&kr)[NBT], const u32x4 (&vr)[NBT]) {
        bf16_t *Ks = stage_k(kb);
#pragma unroll
        for (int u = 0; u < NBT; ++u) {
            *(u32x4 *)(Ks + soff[u]) = kr[u];
            *(u32x4 *)(Ks + 64 * CS + soff[u]) = vr[u];
        }
    };
#pragma unroll
    for (int u = 0; u < NPF; ++u) request(u, pk[u], pv[u]);

    // The LCE of the tile while the first key blocks are on their way: results in registers, then,
    // once every task has read the halo tile, into the float32 tile that takes its place.
    lce_tasks<C, CS, NT, NTASK>(Hs, Wl, D.rw, hw, lce);
    __syncthreads();
    BRA_TRACE(2);
    lce_store<C, OS, NT, NTASK>((float *)Hs, D.rw, lce);

    // Online-softmax state of the two query tiles over this wavefront's share of the keys.
    f32x4 acc[2][2], lacc[2], negm[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        acc[qt][0] = acc[qt][1] = lacc[qt] = negm[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const int col = 32 * h;

    // One block of 64 keys in the stage at Ks (V follows K); this wavefront takes its 16-key
    // tiles TPW ks .. TPW ks + TPW - 1.  FIRST: the first block sets the reference score to its own
    // maximum; afterwards the reference only moves when outgrown.
    auto compute = [&](const bf16_t *Ks, auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const bf16_t *Vs = Ks + 64 * CS;
        f32x4 s[2][TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * (TPW * ks + t) + i) * CS + col + 8 * g);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)    // S^T[key 16 t' + 4 g + j][query i] - reference, in units of log2
                s[qt][t] = mfma16(kf, qf[qt], negm[qt]);
        }
        bf16x8 pb[2][TPW / 2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float mx = max3(s[qt][0][0], s[qt][0][1], s[qt][0][2]);
            mx = max2(mx, s[qt][0][3]);
#pragma unroll
            for (int t = 1; t < TPW; ++t) {
                mx = max3(mx, s[qt][t][0], s[qt][t][1]);
                mx = max3(mx, s[qt][t][2], s[qt][t][3]);
            }
            bool move;
            if (FIRST) move = true;
            else move = __builtin_amdgcn_ballot_w64(mx > kSlack) != 0;
            if (move) {
                const float top = cross_row_max(mx);
                const float delta = FIRST ? top : max2(top, 0.f);
                if (!FIRST) {
                    const float alpha = __builtin_amdgcn_exp2f(-delta);
                    acc[qt][0] *= alpha;
                    acc[qt][1] *= alpha;
                    lacc[qt] *= alpha;
                }
#pragma unroll
                for (int t = 0; t < TPW; ++t) s[qt][t] -= delta;
                negm[qt] -= delta;
            }
#pragma unroll
            for (int tp = 0; tp < TPW / 2; ++tp) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(s[qt][2 * tp + e / 4][e % 4]);
                pb[qt][tp] = pack8(p);
            }
        }
#pragma unroll
        for (int tp = 0; tp < TPW / 2; ++tp) {
            const int tpb = (TPW / 2) * ks + tp;          // pair of 16-key tiles within the block
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                // V^T fragment: channels 32 h + 16 dt .., keys in the order of the P^T operand
                const bf16_t *vp = Vs + (32 * tpb + 4 * g + i / 4) * CS + col + 16 * dt + 4 * (i % 4);
                const u32x2 a0 = __builtin_bit_cast(u32x2, lds_read_tr16(vp));
                const u32x2 a1 = __builtin_bit_cast(u32x2, lds_read_tr16(vp + 16 * CS));
                const bf16x8 av = __builtin_bit_cast(bf16x8, u32x4{a0[0], a0[1], a1[0], a1[1]});
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) acc[qt][dt] = mfma16(av, pb[qt][tp], acc[qt][dt]);
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
                lacc[qt] = mfma16(__builtin_bit_cast(bf16x8, ones), pb[qt][tp], lacc[qt]);   // sums of the rounded P
        }
    };

    // Ring schedule (block kb is computed from stage kb % 2):
    //   compute kb | hand block kb + 1 from its registers to stage (kb + 1) % 2 | request block
    //   kb + 1 + NPF into the freed registers | barrier
    // Stage (kb + 1) % 2 was last read in iteration kb - 1, which ended with a barrier.  Only the
    // computation is skipped for blocks past the end (the copies then move the last block once
    // more into a stage that nobody reads): with the same loads and stores on every path, the
    // wait before an LDS write covers exactly the block being handed over.
    hand_over(0, pk[0], pv[0]);
    request(NPF, pk[0], pv[0]);
    __syncthreads();
    BRA_TRACE(3);
    compute(stage_k(0), std::true_type{});
    hand_over(1, pk[1 % NPF], pv[1 % NPF]);
    request(1 + NPF, pk[1 % NPF], pv[1 % NPF]);
    __syncthreads();
    BRA_TRACE(4);
    for (int kb0 = 1; kb0 < nblocks; kb0 += NPF) {
#pragma unroll
        for (int u = 0; u < NPF; ++u) {
            const int kb = kb0 + u;
            constexpr int set_base = 2;         // block kb0 + u + 1 lives in set (u + 2) % NPF (kb0 % NPF == 1)
            if (kb < nblocks) compute(stage_k(kb), std::false_type{});
            hand_over(kb + 1, pk[(u + set_base) % NPF], pv[(u + set_base) % NPF]);
            request(kb + 1 + NPF, pk[(u + set_base) % NPF], pv[(u + set_base) % NPF]);
            __syncthreads();
        }
    }
    BRA_TRACE(5);

    // W^o fragments of this wavefront's share of Y^T = Wo^T O^T (requested now, used after the LCE):
    // tokens 16 (wave % 4) .., output channels 64 cg + 16 (lane group) + (16 / WOS) wo_part .. of each lane
    constexpr int WOS = NW / 4 / (C / 64);      // wavefronts that share a (token tile, 64-channel group)
    constexpr int NWT = 4 / WOS;                // W^o tiles per wavefront
    const int wo_part = (wave / 4) % WOS, cg = (wave / 4) / WOS;
    bf16x8 wof[NWT][KS];
#pragma unroll
    for (int tt = 0; tt < NWT; ++tt)
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) wof[tt][kk] = wo_fragment<C>(A.WoT, cg, NWT * wo_part + tt, kk, g, i);

    // The ring is free (the loop ended with a barrier).  Two wavefronts that split the keys merge
    // their softmax states: the second hands over (reference, denominator, sums), the first
    // combines them against the larger reference.
    if constexpr (KSPLIT == 2) {
        float *Xs = (float *)(smem + SM::x_off) + ((size_t)pair * kWave + lane) * 20;
        if (ks == 1) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                *(f32x4 *)(Xs + 8 * qt) = acc[qt][0];
                *(f32x4 *)(Xs + 8 * qt + 4) = acc[qt][1];
                Xs[16 + qt] = lacc[qt][0];
                Xs[18 + qt] = negm[qt][0];
            }
        }
        __syncthreads();
        if (ks == 0) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const float m0 = -negm[qt][0], m1 = -Xs[18 + qt];
                const float m = max2(m0, m1);
                const float a0 = __builtin_amdgcn_exp2f(m0 - m), a1 = __builtin_amdgcn_exp2f(m1 - m);
                const float inv = 1.0f / (lacc[qt][0] * a0 + Xs[16 + qt] * a1);
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const int at = (32 * qhf + 16 * qt + i) * OS + col + 16 * dt + 4 * g;
                    const f32x4 o = (acc[qt][dt] * a0 + *(const f32x4 *)(Xs + 8 * qt + 4 * dt) * a1) * inv;
                    *(f32x4 *)(Os + at) = o + *(const f32x4 *)(Ls + at);
                }
            }
        }
    } else {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const float inv = 1.0f / lacc[qt][0];
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const int at = (32 * qhf + 16 * qt + i) * OS + col + 16 * dt + 4 * g;
                *(f32x4 *)(Os + at) = acc[qt][dt] * inv + *(const f32x4 *)(Ls + at);
            }
        }
    }
    __syncthreads();
    BRA_TRACE(6);
    // Y = O Wo
    {
        const int q = 16 * (wave % 4) + i;
        const int qy = fast_div(q, rw_inv);
        const size_t tok = (size_t)(y0 + qy) * D.W + x0 + q - qy * D.rw;
        bf16x8 of[KS];
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            const float *src = Os + q * OS + 32 * kk + 8 * g;
            const f32x4 lo = *(const f32x4 *)src, hi = *(const f32x4 *)(src + 4);
            const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            of[kk] = pack8(v);
        }
        u32x2 yp[NWT];
#pragma unroll
        for (int tt = 0; tt < NWT; ++tt) {
            f32x4 ya = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) ya = mfma16(wof[tt][kk], of[kk], ya);
            yp[tt] = pack4(ya);
        }
        bf16_t *dst = A.Y + img_off + tok * C + cg * 64 + 16 * g + 4 * NWT * wo_part;
        if constexpr (NWT == 4) {
            *(u32x4 *)dst = u32x4{yp[0][0], yp[0][1], yp[1][0], yp[1][1]};
            *(u32x4 *)(dst + 8) = u32x4{yp[2][0], yp[2][1], yp[3][0], yp[3][1]};
        } else {
            *(u32x4 *)dst = u32x4{yp[0][0], yp[0][1], yp[1][0], yp[1][1]};
        }
    }
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

template <int C>
size_t q32_smem(const Dims &D)
{
    const int qh = 64 / D.rw;
    return Q32Smem<C>::bytes((qh + 4) * (D.rw + 4), D.kn / 64);
}

template <int C, int KSPLIT>
int launch_q32(const Dims &D, const AttnArgs &A, hipStream_t st)
{
    static bool opted = false;
    if (!opted) {
        if (hipFuncSetAttribute((const void *)k_attn_q32<C, KSPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kMaxLds) != hipSuccess)
            return BRA_ERR_LAUNCH;
        opted = true;
    }
    const int grid = ((A.total + 7) / 8) * 8;
    ProfScope ps(st, K_MFMA_ATTENTION);
    hipLaunchKernelGGL((k_attn_q32<C, KSPLIT>), dim3(grid), dim3(4 * C * KSPLIT), q32_smem<C>(D), st, A, D);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

}  // namespace

// Shapes of this kernel: C = 64 or 128, query tiles of 64 tokens made of whole region rows, key
// blocks of 64 tokens likewise.  Q must have been multiplied by scale * log2(e).
bool attn_q32_ok(const Dims &D)
{
    if (D.C != 64 && D.C != 128) return false;
    if (D.n % 64 != 0 || D.rw < 8 || 64 % D.rw != 0 || D.rh % (64 / D.rw) != 0) return false;
    return (D.C == 64 ? q32_smem<64>(D) : q32_smem<128>(D)) <= (size_t)kMaxLds;
}

int launch_attn_q32(const Dims &D, const AttnArgs &A, hipStream_t st)
{
    if (D.C == 64) return experiment_flag("BRA_Q32_NOSPLIT") ? launch_q32<64, 1>(D, A, st) : launch_q32<64, 2>(D, A, st);
    return launch_q32<128, 1>(D, A, st);
}

}  // namespace bra
