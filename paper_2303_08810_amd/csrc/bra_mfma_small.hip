// Matrix-core kernel for small regions (n = 1, 2, 4, 8 or 16 tokens per region).
//
// With so few queries per region a query tile cannot fill a 64-row workgroup tile from
// one region, and every (region, head) pair has its own routed key set (Eq. 6).  So one
// workgroup handles one (image, region) and the attention runs per head in one
// wavefront: the n queries occupy the first n of the 16 query columns of the 16x16x32
// MFMA tiles, keys are read by index straight from the projected map into the A
// operands, values go through a wavefront-private LDS tile for the transposing read.
// For regions of 16 tokens the same workgroup then adds the LCE of its tokens (Eq. 7; 5x5
// depth-wise correlation of V over the region plus a 2-token halo, staged in LDS) and
// applies W^o (Eq. 2), so the attention output never travels through memory (k_small).
// Smaller regions use separate kernels: on small maps the image-resident attention
// k_attn_map / k_attn_map4 (a head's Q, K, V of a whole image in LDS, the LCE added from the
// same V slice), else k_attn_small (attention output to memory) and k_lce_add (adds the LCE
// in place); then the projection kernel with W^o.
#include "bra_mfma_dev.h"

namespace bra {

using namespace mfma;

namespace {

constexpr int kLTP = 20;    // floats per channel of the LCE tile [C][tokens] (n <= 16)
constexpr int kMaxLceTasks = 2;   // (row, 4-token segment, channel pair) tasks per thread

// ---------------------------------------------------------------------------
// Attention of one (image, region) over its k n routed keys (Eq. 6, Eq. 1), shared by
// both variants.  The keys are taken 64 at a time: the workgroup copies the K and V rows
// of the block (all channels, found by index in the projected maps) into LDS with
// coalesced 16-byte loads, then wavefront w runs heads w, w + 4, .. on it.  Result:
// oacc[hh][dt] = normalised O^T[channel 32 h + 16 dt + 4 g + jj][query i], h = w + 4 hh.
// Ks, Vs: [64][C + 16] bf16 each.  Ends with all wavefronts past their last LDS read only
// after the caller's next barrier.
template <int C>
__device__ __forceinline__ void small_attention(const AttnArgs &A, const Dims &D, int log2n,
                                                size_t img_off, const int32_t *irp, size_t qtok,
                                                bf16_t *Ks, bf16_t *Vs,
                                                f32x4 (&oacc)[(C / 32 + 3) / 4][2])
{
    constexpr int HEADS = C / 32, HPW = (HEADS + 3) / 4, XP = C + 16, CH = C / 8;
    constexpr int NLD = 64 * CH / 256;        // 16-byte chunks of a 64-row tile per thread
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int n = D.n, kn = D.kn;
    const float rw_inv = 1.0f / (float)D.rw, s_inv = 1.0f / (float)D.S;

    bf16x8 qf[HPW];
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        const int h = min(wave + 4 * hh, HEADS - 1);
        qf[hh] = *(const bf16x8 *)(A.Q + img_off + qtok * C + 32 * h + 8 * g);
    }
    SoftmaxState<HPW> st;
    st.init();
    for (int k0 = 0; k0 < kn; k0 += 64) {
        u32x4 kr[NLD], vr[NLD];
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int idx = threadIdx.x + 256 * u;
            int key = k0 + idx / CH;
            if (key >= kn) key = kn - 1;           // rows past the end repeat the last key; masked below
            const int j = region_index(irp[key >> log2n], D.R), slot = key & (n - 1);
            const int sy = fast_div(slot, rw_inv), jy = fast_div(j, s_inv);
            const size_t tok = (size_t)(jy * D.rh + sy) * D.W + (j - jy * D.S) * D.rw + slot - sy * D.rw;
            const size_t off = img_off + tok * C + (idx % CH) * 8;
            kr[u] = *(const u32x4 *)(A.K + off);
            vr[u] = *(const u32x4 *)(A.V + off);
        }
        if (k0) __syncthreads();                   // the previous block has been read
#pragma unroll
        for (int u = 0; u < NLD; ++u) {
            const int idx = threadIdx.x + 256 * u;
            *(u32x4 *)(Ks + (idx / CH) * XP + (idx % CH) * 8) = kr[u];
            *(u32x4 *)(Vs + (idx / CH) * XP + (idx % CH) * 8) = vr[u];
        }
        __syncthreads();
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) {
            const int h = wave + 4 * hh;
            if (h >= HEADS) break;
            f32x4 s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bf16x8 kf = *(const bf16x8 *)(Ks + (16 * t + i) * XP + 32 * h + 8 * g);
                s[t] = mfma16(kf, qf[hh], f32x4{0.f, 0.f, 0.f, 0.f});
            }
            if (k0 + 64 > kn) {   // ragged last block: keys past the end do not count
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        if (k0 + 16 * t + 4 * g + jj >= kn) s[t][jj] = -INFINITY;
            }
            softmax_pv_block<XP>(Vs, s, st, hh, 32 * h, A.c_exp, g, i);
        }
    }
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        const float inv = 1.0f / st.denom(hh);         // heads past the end: 1 / 0 times 0, never used
        oacc[hh][0] = st.acc[hh][0] * inv;
        oacc[hh][1] = st.acc[hh][1] * inv;
    }
}

// LDS map of the one-kernel variant: the K / V key blocks first; once the attention is
// done, the V halo tile and the LCE tile take their place.
template <int C>
struct SmallSmem {
    static constexpr int CS = C + 8, XP = C + 16;
    static constexpr size_t kv_bytes = (size_t)2 * 64 * XP * 2;
    static constexpr size_t lt_bytes = (size_t)C * kLTP * 4;
    __host__ __device__ static size_t o_off(int hrows)   // [16][CS] bf16: O = attention + LCE, behind the halo and LCE tiles
    {
        return (size_t)hrows * CS * 2 + lt_bytes;
    }
    static size_t bytes(int hrows)
    {
        const size_t second = o_off(hrows) + (size_t)16 * CS * 2;
        return kv_bytes > second ? kv_bytes : second;
    }
};

template <int C>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(C <= 128 ? 4 : 2, 4)))
void k_small(AttnArgs A, Dims D, int log2n)
{
    typedef SmallSmem<C> SM;
    constexpr int HEADS = C / 32, HPW = (HEADS + 3) / 4, CS = SM::CS, XP = SM::XP, KS = C / 32, CH = C / 8;
    constexpr int NBH = 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int hw = D.rw + 4, hrows = (D.rh + 4) * hw;
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + 64 * XP;
    bf16_t *Hs = (bf16_t *)smem;                                   // after the attention
    float *Lt = (float *)(smem + (size_t)hrows * CS * 2);
    bf16_t *Ob = (bf16_t *)(smem + SM::o_off(hrows));

    const int wid = swizzled_block();
    if (wid >= A.total) return;
#ifdef BRA_EXPERIMENT
    unsigned long long trace_t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#define BRA_TRACE(k) if (A.trace) trace_t[k] = __builtin_amdgcn_s_memrealtime()
#else
#define BRA_TRACE(k)
#endif
    BRA_TRACE(0);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int b = wid / D.R, reg = wid % D.R;
    const size_t img_off = (size_t)b * D.N * C;
    const int n = D.n;
    const float rw_inv = 1.0f / (float)D.rw, hw_inv = 1.0f / (float)hw;
    const int regy = fast_div(reg, 1.0f / (float)D.S);
    const int y0 = regy * D.rh, x0 = (reg - regy * D.S) * D.rw;

    const int32_t *irp = A.Ir_src + ((size_t)b * D.R + reg) * D.k;
    if (A.Ir_out && A.Ir_out != A.Ir_src)
        for (int p = threadIdx.x; p < D.k; p += 256) A.Ir_out[((size_t)b * D.R + reg) * D.k + p] = irp[p];

    // V over the region and its halo: the first chunks are requested now and parked in
    // registers until the attention has released the LDS
    u32x4 hreg[NBH];
    tile_load<C, NBH>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, 0);

    // query token of this lane's column (columns >= n repeat the last query; never stored)
    const int qs = i < n ? i : n - 1;
    const int qy = fast_div(qs, rw_inv);
    const size_t qtok = (size_t)(y0 + qy) * D.W + x0 + qs - qy * D.rw;

    // LCE task = (row r, 4-token segment, channel pair); a thread keeps its channel pair for
    // all its tasks, so its 2 x 25 weights stay in registers (requested now, used after the attention)
    const int cp_n = C / 2, segs = (D.rw + 3) / 4;
    const int tasks = D.rh * segs * cp_n;
    const int cpair = threadIdx.x % cp_n;
    unsigned wl[25];        // tap t of channels (c, c + 1) as a packed pair, from the tap-major table
#pragma unroll
    for (int t = 0; t < 25; ++t) wl[t] = *(const unsigned *)(A.WlT + (size_t)t * C + 2 * cpair);

    f32x4 oacc[HPW][2];     // normalised attention output of this wavefront's heads
    BRA_TRACE(1);
    small_attention<C>(A, D, log2n, img_off, irp, qtok, Ks, Vs, oacc);
    BRA_TRACE(2);
    __builtin_amdgcn_s_setprio(2);      // late phases first: the workgroup's LDS is freed sooner
    __syncthreads();        // the key blocks have been read: the halo tile takes their place
    BRA_TRACE(3);
    tile_store<C, CS, NBH>(Hs, hreg, hrows, 0);
    for (int first = 256 * NBH; first < hrows * CH; first += 256 * NBH) {
        tile_load<C, NBH>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, first);
        tile_store<C, CS, NBH>(Hs, hreg, hrows, first);
    }

    // LCE (Eq. 7) of the region's tokens
    auto tap = [&](int ch, int t) { return ch ? bf16_hi(wl[t]) : bf16_lo(wl[t]); };
    float lce[kMaxLceTasks][2][4];
    __syncthreads();        // the halo tile is complete
    BRA_TRACE(4);
#pragma unroll
    for (int tk = 0; tk < kMaxLceTasks; ++tk) {
        const int task = threadIdx.x + 256 * tk;
#pragma unroll
        for (int x = 0; x < 4; ++x) lce[tk][0][x] = lce[tk][1][x] = 0.f;
        if (task < tasks) {
            const int seg = (task / cp_n) % segs, r = task / (cp_n * segs);
#pragma unroll
            for (int ky = 0; ky < 5; ++ky) {
                float v0[8], v1[8];
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const int hx = min(seg * 4 + x, hw - 1);    // a ragged segment re-reads the last column; unused
                    const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + hx) * CS + 2 * cpair);
                    v0[x] = bf16_lo(u);
                    v1[x] = bf16_hi(u);
                }
#pragma unroll
                for (int kx = 0; kx < 5; ++kx) {
                    const float w0 = tap(0, ky * 5 + kx), w1 = tap(1, ky * 5 + kx);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        lce[tk][0][x] = fmaf(w0, v0[x + kx], lce[tk][0][x]);
                        lce[tk][1][x] = fmaf(w1, v1[x + kx], lce[tk][1][x]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int tk = 0; tk < kMaxLceTasks; ++tk) {
        const int task = threadIdx.x + 256 * tk;
        if (task < tasks) {
            const int seg = (task / cp_n) % segs, r = task / (cp_n * segs);
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (seg * 4 + x < D.rw) {
                    const int tok = r * D.rw + seg * 4 + x;
                    Lt[(2 * cpair) * kLTP + tok] = lce[tk][0][x];
                    Lt[(2 * cpair + 1) * kLTP + tok] = lce[tk][1][x];
                }
        }
    }
    __syncthreads();
    BRA_TRACE(5);
    // O = attention + LCE, rounded to bf16 once: rows of the B operand of W^o
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        const int h = wave + 4 * hh;
        if (h >= HEADS) break;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
            const int ch = 32 * h + 16 * dt + 4 * g;
            f32x4 o = oacc[hh][dt];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) o[jj] += Lt[(ch + jj) * kLTP + qs];
            *(u32x2 *)(Ob + i * CS + ch) = pack4(o);     // rows >= n repeat the last query
        }
    }
    __syncthreads();
    // Y^T = Wo^T O^T: wavefront w owns output-channel tiles w, w + 4, ..
    bf16x8 of[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) of[ks] = *(const bf16x8 *)(Ob + i * CS + 32 * ks + 8 * g);
    bf16_t *yrow = A.Y + img_off + qtok * C;
#pragma unroll
    for (int ct = wave; ct < C / 16; ct += 4) {
        f32x4 ya = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 wf = *(const bf16x8 *)(A.WoF + ((size_t)(ct * KS + ks) * kWave + lane) * 8);
            ya = mfma16(wf, of[ks], ya);
        }
        if (i < n) *(u32x2 *)(yrow + 16 * ct + 4 * g) = pack4(ya);
    }
#ifdef BRA_EXPERIMENT
    if (A.trace) {
        BRA_TRACE(6);
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
// Two-kernel variant for regions of fewer than 16 tokens, where a workgroup per region
// would re-read all of W^o for a handful of tokens: attention per (image, region) writes
// O_att to memory, then the LCE and W^o run over tiles of full-width image rows.
// One workgroup per (image, region); wavefront w handles heads w, w + 4, ...
// O_att[b, token, head channels] = softmax(scale q K_g^T) V_g over the k n routed keys.
template <int C>
__global__ __launch_bounds__(256) void k_attn_small(AttnArgs A, bf16_t *__restrict__ O, Dims D,
                                                    int log2n)
{
    constexpr int HEADS = C / 32, HPW = (HEADS + 3) / 4, XP = C + 16;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Ks = (bf16_t *)smem, *Vs = Ks + 64 * XP;

    const int wid = swizzled_block();
    if (wid >= A.total) return;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int b = wid / D.R, reg = wid % D.R;
    const size_t img_off = (size_t)b * D.N * C;
    const int n = D.n;
    const float rw_inv = 1.0f / (float)D.rw;

    const int32_t *irp = A.Ir_src + ((size_t)b * D.R + reg) * D.k;
    if (A.Ir_out && A.Ir_out != A.Ir_src)
        for (int p = threadIdx.x; p < D.k; p += 256) A.Ir_out[((size_t)b * D.R + reg) * D.k + p] = irp[p];

    // query token of this lane's column (columns >= n repeat the last query; never stored)
    const int qs = i < n ? i : n - 1;
    const int qy = fast_div(qs, rw_inv);
    const int regy = fast_div(reg, 1.0f / (float)D.S);
    const size_t qtok = (size_t)(regy * D.rh + qy) * D.W + (reg - regy * D.S) * D.rw + qs - qy * D.rw;

    f32x4 oacc[HPW][2];
    small_attention<C>(A, D, log2n, img_off, irp, qtok, Ks, Vs, oacc);
    if (i < n) {
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh) {
            const int h = wave + 4 * hh;
            if (h >= HEADS) break;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
                *(u32x2 *)(O + img_off + qtok * C + 32 * h + 16 * dt + 4 * g) = pack4(oacc[hh][dt]);
        }
    }
}

// ---------------------------------------------------------------------------
// The same attention for maps small enough that one head's K and V of a whole image fit
// in LDS.  Regions of a few tokens route to many regions (k n keys each), so a workgroup
// per region would copy every K / V row of the image about k times from the L2; here
// workgroup (image, head, part) copies the head's 32 channels of all N tokens once and
// its wavefronts walk over the regions of the part, finding the rows of their keys by
// index (Eq. 6 as row addresses of LDS reads).  Ks, Vs: [N][kMapPitch] bf16.
constexpr int kMapPitch = 40;    // 32 channels + 8: rows of 80 bytes (random-row access: the pitch matters little)
constexpr int kMapLcePitch = 32; // floats per token of the LCE tile
constexpr int kMapWaves = 8, kMapThreads = kMapWaves * kWave;   // the walk over the regions is latency-bound: many wavefronts

struct MapWork {
    int b, h, r_begin, r_end;
    size_t img_off;
    bf16_t *Ks, *Vs, *Qs;
    int *rows;       // [R][k]: where the first token of routed region I^r[reg][p] starts in Ks / Vs (elements)
    int *first;      // [R]: first token of a region
    int slot_off;    // this lane's token within a routed region, the same way: key l is token l % n
    char *wave_mem;  // 512 bytes of this wavefront's own
    float *Ls;       // [N][kMapLcePitch]: LCE of the head's channels (variants that add it)
};

// Stages the head's K / V slice and the image's routing index; false: no work.
__device__ __forceinline__ bool map_stage(const AttnArgs &A, const Dims &D, int split, char *smem, MapWork &w)
{
    constexpr int T = kMapThreads;
    const int C = D.C, HEADS = C / 32;
    w.Ks = (bf16_t *)smem;
    w.Vs = w.Ks + (size_t)D.N * kMapPitch;
    w.Qs = w.Vs + (size_t)D.N * kMapPitch;
    w.rows = (int *)(w.Qs + (size_t)D.N * kMapPitch);
    w.first = w.rows + D.R * D.k;
    w.wave_mem = (char *)(w.rows + (D.R * D.k + D.R + 3) / 4 * 4) + (threadIdx.x / kWave) * 512;   // 16-byte aligned
    w.Ls = (float *)((char *)(w.rows + (D.R * D.k + D.R + 3) / 4 * 4) + kMapWaves * 512);
    const int wid = swizzled_block();       // the heads of an image share the memory lines of its K / V rows
    if (wid >= A.total) return false;
    const int part = wid % split;
    w.h = (wid / split) % HEADS;
    w.b = wid / (split * HEADS);
    w.img_off = (size_t)w.b * D.N * C;
    const float rw_inv = 1.0f / (float)D.rw, s_inv = 1.0f / (float)D.S;

    const int chunks = D.N * 4;              // 16-byte chunks of the head's slice
    for (int first = 0; first < chunks; first += T * 4) {
        u32x4 kr[4], vr[4], qr[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = min(first + (int)threadIdx.x + T * u, chunks - 1);
            const size_t off = w.img_off + (size_t)(idx / 4) * C + 32 * w.h + (idx % 4) * 8;
            kr[u] = *(const u32x4 *)(A.K + off);
            vr[u] = *(const u32x4 *)(A.V + off);
            qr[u] = *(const u32x4 *)(A.Q + off);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = first + (int)threadIdx.x + T * u;
            if (idx < chunks) {
                *(u32x4 *)(w.Ks + (idx / 4) * kMapPitch + (idx % 4) * 8) = kr[u];
                *(u32x4 *)(w.Vs + (idx / 4) * kMapPitch + (idx % 4) * 8) = vr[u];
                *(u32x4 *)(w.Qs + (idx / 4) * kMapPitch + (idx % 4) * 8) = qr[u];
            }
        }
    }
    const bool copy_ir = A.Ir_out && A.Ir_out != A.Ir_src && w.h == 0 && part == 0;
    for (int p = threadIdx.x; p < D.R * D.k; p += T) {
        const int j_given = A.Ir_src[(size_t)w.b * D.R * D.k + p];
        const int j = region_index(j_given, D.R);
        const int jy = fast_div(j, s_inv);
        w.rows[p] = (jy * D.rh * D.W + (j - jy * D.S) * D.rw) * kMapPitch;
        if (copy_ir) A.Ir_out[(size_t)w.b * D.R * D.k + p] = j_given;
    }
    for (int r = threadIdx.x; r < D.R; r += T) {
        const int ry = fast_div(r, s_inv);
        w.first[r] = ry * D.rh * D.W + (r - ry * D.S) * D.rw;
    }
    const int slot = (threadIdx.x % kWave) & (D.n - 1), sy = fast_div(slot, rw_inv);
    w.slot_off = (sy * D.W + slot - sy * D.rw) * kMapPitch;
    __syncthreads();
    const int per = (D.R + split - 1) / split;
    w.r_begin = part * per;
    w.r_end = min(D.R, (part + 1) * per);
    return true;
}

// LCE (Eq. 7) of the head's 32 channels over the whole image, from the V slice in LDS into
// w.Ls (float32): thread = (channel pair, group); a group takes (image row, 4-token segment)
// items, the 2 x 25 weights of the pair stay in registers.  Tokens outside the image are zero.
__device__ __forceinline__ void map_lce(const AttnArgs &A, const Dims &D, const MapWork &w)
{
    const int cpair = threadIdx.x % 16, grp = threadIdx.x / 16;
    unsigned wl[25];        // [W(c, 0..24) | W(c + 1, 0..24)] as 25 packed pairs
#pragma unroll
    for (int e = 0; e < 25; ++e) wl[e] = *(const unsigned *)(A.Wlce + (size_t)(32 * w.h + 2 * cpair) * 25 + 2 * e);
    auto tap = [&](int ch, int t) {
        const int e = 25 * ch + t;
        return (e & 1) ? bf16_hi(wl[e / 2]) : bf16_lo(wl[e / 2]);
    };
    const int segs = (D.W + 3) / 4;
    for (int item = grp; item < D.H * segs; item += kMapThreads / 16) {
        const int y = item / segs, x0 = (item % segs) * 4;
        float a0[4] = {0.f, 0.f, 0.f, 0.f}, a1[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ky = 0; ky < 5; ++ky) {
            const int yy = y + ky - 2;
            const bool row_ok = yy >= 0 && yy < D.H;
            float v0[8], v1[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int xx = x0 + x - 2;
                const bool ok = row_ok && xx >= 0 && xx < D.W;
                const unsigned u = *(const unsigned *)(w.Vs + (ok ? yy * D.W + xx : 0) * kMapPitch + 2 * cpair);
                v0[x] = ok ? bf16_lo(u) : 0.f;
                v1[x] = ok ? bf16_hi(u) : 0.f;
            }
#pragma unroll
            for (int kx = 0; kx < 5; ++kx) {
                const float w0 = tap(0, ky * 5 + kx), w1 = tap(1, ky * 5 + kx);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    a0[x] = fmaf(w0, v0[x + kx], a0[x]);
                    a1[x] = fmaf(w1, v1[x + kx], a1[x]);
                }
            }
        }
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (x0 + x < D.W) *(f32x2 *)(w.Ls + (y * D.W + x0 + x) * kMapLcePitch + 2 * cpair) = f32x2{a0[x], a1[x]};
    }
    __syncthreads();
}

// Regions of 8 tokens: the queries take 8 of the 16 query columns of 16x16x32 tiles;
// lane l puts the row of key l into a wavefront-private table, the K operand rows and
// the transposing V reads take their addresses from it.
// LCE: the LCE of the head's channels is computed from the V slice first and added to the
// attention output (no separate LCE pass over memory).
template <bool LCE>
__global__ __launch_bounds__(kMapThreads) void k_attn_map(AttnArgs A, bf16_t *__restrict__ O, Dims D, int log2n,
                                                  int split)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    MapWork w;
    if (!map_stage(A, D, split, smem, w)) return;
    if (LCE) map_lce(A, D, w);
    const bf16_t *Ks = w.Ks, *Vs = w.Vs;
    int *tokw = (int *)w.wave_mem;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int C = D.C, h = w.h, n = D.n, kn = D.kn;
    const float rw_inv = 1.0f / (float)D.rw;

    // query token of this lane's column within its region (columns >= n repeat the last; never stored)
    const int qs = i < n ? i : n - 1;
    const int qy = fast_div(qs, rw_inv);
    const int q_in = qy * D.W + qs - qy * D.rw;
    for (int reg = w.r_begin + wave; reg < w.r_end; reg += kMapWaves) {
        const int tok0 = w.first[reg];
        const bf16x8 qf = *(const bf16x8 *)(w.Qs + (tok0 + q_in) * kMapPitch + 8 * g);
        SoftmaxState<1> st;
        st.init();
        for (int k0 = 0; k0 < kn; k0 += 64) {
            // rows past the end repeat the last region; masked below
            tokw[lane] = w.rows[reg * D.k + (min(k0 + lane, kn - 1) >> log2n)] + w.slot_off;
            f32x4 s[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bf16x8 kf = *(const bf16x8 *)(Ks + tokw[16 * t + i] + 8 * g);
                s[t] = mfma16(kf, qf, f32x4{0.f, 0.f, 0.f, 0.f});
            }
            if (k0 + 64 > kn) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        if (k0 + 16 * t + 4 * g + jj >= kn) s[t][jj] = -INFINITY;
            }
            int vrow[2][2];
#pragma unroll
            for (int tp = 0; tp < 2; ++tp)
#pragma unroll
                for (int half = 0; half < 2; ++half) vrow[tp][half] = tokw[32 * tp + 16 * half + 4 * g + i / 4];
            softmax_pv_rows<false>(
                Vs, [&](int tp, int half) { return vrow[tp][half]; }, s, st, 0, 0, A.c_exp, i);
        }
        const float inv = 1.0f / st.denom(0);
        if (i < n) {
            bf16_t *orow = O + w.img_off + (size_t)(tok0 + q_in) * C + 32 * h + 4 * g;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                f32x4 o = st.acc[0][dt] * inv;
                if (LCE) o += *(const f32x4 *)(w.Ls + (tok0 + q_in) * kMapLcePitch + 16 * dt + 4 * g);
                *(u32x2 *)(orow + 16 * dt) = pack4(o);
            }
        }
    }
}

// Regions of at most 4 tokens: 16 query columns would be three quarters idle and the
// softmax arithmetic with them.  The scores come from v_mfma_f32_4x4x4_16B_bf16 instead
// (16 blocks of 4 queries x 4 keys, 4 channels per product, 8 products for d = 32):
// block l / 4 and column l % 4 make lane l the owner of key l with the scores of the 4
// queries in its 4 result registers, and the K operand is simply the lane's own key row.
// Per query: wavefront maximum, 2^x; the probabilities go through 8 bytes per key of
// wavefront-private LDS and come back, by the transposing read, as the P^T operand of
// O^T = V^T P^T on 16x16x32 tiles (query columns >= 4 see copies).  A product with an
// all-ones operand delivers the softmax denominators (of the same bf16-rounded P) to
// every lane of a query column.
template <bool LCE>
__global__ __launch_bounds__(kMapThreads) void k_attn_map4(AttnArgs A, bf16_t *__restrict__ O, Dims D, int log2n,
                                                   int split)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    MapWork w;
    if (!map_stage(A, D, split, smem, w)) return;
    if (LCE) map_lce(A, D, w);
    const bf16_t *Ks = w.Ks, *Vs = w.Vs;
    bf16_t *Pw = (bf16_t *)w.wave_mem;          // [64 keys][4 queries]
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int C = D.C, h = w.h, n = D.n, kn = D.kn;
    const float rw_inv = 1.0f / (float)D.rw;
    const float c_exp = A.c_exp;

    auto in_region = [&](int q) {   // token offset of query min(q, n - 1) from the region's first token
        const int qs = q < n ? q : n - 1;
        const int qy = fast_div(qs, rw_inv);
        return qy * D.W + qs - qy * D.rw;
    };
    const bf16_t *qbase = w.Qs + in_region(lane % 4) * kMapPitch;               // row of the score operand
    const int qo_in = in_region(i);                                             // column of the output tiles
    bf16_t *obase = O + w.img_off + qo_in * C + 32 * h + 4 * g;
    const u32x4 ones = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bool ragged = (kn % 64) != 0;
    for (int reg = w.r_begin + wave; reg < w.r_end; reg += kMapWaves) {
        const int tok0 = w.first[reg];
        u32x4 q4[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) q4[c] = *(const u32x4 *)(qbase + tok0 * kMapPitch + 8 * c);
        const int *rrow = w.rows + reg * D.k;
        float m[4];
        f32x4 acc[2], lacc;
        // one block of 64 keys; FIRST: the region's first block, nothing to rescale
        auto key_block = [&](int k0, auto first_tag) {
            constexpr bool FIRST = decltype(first_tag)::value;
            int key = k0 + lane;
            if (ragged) key = min(key, kn - 1);         // rows past the end repeat the last region; masked below
            const int row = rrow[key >> log2n] + w.slot_off;
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const u32x4 k4 = *(const u32x4 *)(Ks + row + 8 * c);
                s = mfma4(__builtin_bit_cast(s16x4, u32x2{q4[c][0], q4[c][1]}),
                          __builtin_bit_cast(s16x4, u32x2{k4[0], k4[1]}), s);
                s = mfma4(__builtin_bit_cast(s16x4, u32x2{q4[c][2], q4[c][3]}),
                          __builtin_bit_cast(s16x4, u32x2{k4[2], k4[3]}), s);
            }
            if (ragged && k0 + lane >= kn) s = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            float mb[4];
            wave_fmax4(s, lane, mb);
            if (!FIRST) {
                const int qq = i % 4;
                const float m_old = qq == 0 ? m[0] : qq == 1 ? m[1] : qq == 2 ? m[2] : m[3];
                const float m_blk = qq == 0 ? mb[0] : qq == 1 ? mb[1] : qq == 2 ? mb[2] : mb[3];
                const float al = __builtin_amdgcn_exp2f((m_old - fmaxf(m_old, m_blk)) * c_exp);
                acc[0] *= al;
                acc[1] *= al;
                lacc *= al;
            }
            f32x4 p;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                m[r] = FIRST ? mb[r] : fmaxf(m[r], mb[r]);
                p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c_exp, -m[r] * c_exp));
            }
            asm volatile("" ::: "memory");      // the reads of the previous block precede this write
            *(u32x2 *)(Pw + lane * 4) = pack4(p);
            asm volatile("" ::: "memory");
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int tp = 0; tp < 2; ++tp) {
                const int kk0 = 32 * tp + 4 * g + i / 4, kk1 = kk0 + 16;    // keys of this lane's operand slots
                const u32x2 p0 = __builtin_bit_cast(u32x2, lds_read_tr16(Pw + kk0 * 4));
                const u32x2 p1 = __builtin_bit_cast(u32x2, lds_read_tr16(Pw + kk1 * 4));
                const bf16x8 pb = __builtin_bit_cast(bf16x8, u32x4{p0[0], p0[1], p1[0], p1[1]});
                const int r0 = __builtin_amdgcn_ds_bpermute(4 * kk0, row);
                const int r1 = __builtin_amdgcn_ds_bpermute(4 * kk1, row);
                const bool fresh = FIRST && tp == 0;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const int col = 16 * dt + 4 * (i % 4);
                    const u32x2 v0 = __builtin_bit_cast(u32x2, lds_read_tr16(Vs + r0 + col));
                    const u32x2 v1 = __builtin_bit_cast(u32x2, lds_read_tr16(Vs + r1 + col));
                    acc[dt] = mfma16(__builtin_bit_cast(bf16x8, u32x4{v0[0], v0[1], v1[0], v1[1]}), pb,
                                     fresh ? zero : acc[dt]);
                }
                lacc = mfma16(__builtin_bit_cast(bf16x8, ones), pb, fresh ? zero : lacc);
            }
        };
        key_block(0, std::true_type{});
        for (int k0 = 64; k0 < kn; k0 += 64) key_block(k0, std::false_type{});
        const float inv = __builtin_amdgcn_rcpf(lacc[0]);
        if (i < n) {
            bf16_t *orow = obase + (size_t)tok0 * C;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                f32x4 o = acc[dt] * inv;
                if (LCE) o += *(const f32x4 *)(w.Ls + (tok0 + qo_in) * kMapLcePitch + 16 * dt + 4 * g);
                *(u32x2 *)(orow + 16 * dt) = pack4(o);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// O <- O_att + LCE(V) (Eq. 7) in place, for workgroup (image, tile of TH image rows x TW
// columns (the full width on narrow maps), chunk of 64 channels).  LDS holds the V halo tile
// of the chunk, [(TH + 4) x (TW + 4)] tokens x 64 channels; a thread keeps one channel pair for
// all its (row, 4-token segment) tasks, so its 2 x 25 weights stay in registers.  W^o follows
// as a plain projection.
constexpr int kLceChunk = 64, kLcePitch = kLceChunk + 8;

__global__ __launch_bounds__(256) void k_lce_add(bf16_t *__restrict__ O, const bf16_t *__restrict__ V,
                                                 const bf16_t *__restrict__ Wlce, Dims D, int TH, int TW, int ldo)
{
    constexpr int CH8 = kLceChunk / 8, NBH = 6;
    const int C = D.C, NCH = C / kLceChunk;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Hs = (bf16_t *)smem;
    const int tiles = (D.H + TH - 1) / TH, xtiles = (D.W + TW - 1) / TW;
    const int cc = blockIdx.x % NCH, xt = (blockIdx.x / NCH) % xtiles;
    const int tile = (blockIdx.x / (NCH * xtiles)) % tiles, b = blockIdx.x / (NCH * xtiles * tiles);
    const int y0 = tile * TH, x0 = xt * TW;
    const int th = min(TH, D.H - y0), tw = min(TW, D.W - x0);     // rows and columns of this tile
    const size_t img_off = (size_t)b * D.N * C;
    const int hw = tw + 4, hrows = (th + 4) * hw;
    const float hw_inv = 1.0f / (float)hw;
    const int c0 = cc * kLceChunk;

    const int cpair = threadIdx.x % (kLceChunk / 2);
    unsigned wl[25];        // [W(c, 0..24) | W(c + 1, 0..24)] as 25 packed pairs
#pragma unroll
    for (int e = 0; e < 25; ++e) wl[e] = *(const unsigned *)(Wlce + (size_t)(c0 + 2 * cpair) * 25 + 2 * e);
    auto tap = [&](int ch, int t) {   // weight of tap t of channel c + ch
        const int e = 25 * ch + t;
        return (e & 1) ? bf16_hi(wl[e / 2]) : bf16_lo(wl[e / 2]);
    };
    for (int first = 0; first < hrows * CH8; first += 256 * NBH) {
        u32x4 hreg[NBH];
#pragma unroll
        for (int u = 0; u < NBH; ++u) {
            const int idx = first + (int)threadIdx.x + 256 * u;
            const int row = idx / CH8, c8 = idx % CH8;
            const int ry = fast_div(row, hw_inv);
            const int y = y0 - 2 + ry, x = x0 + row - ry * hw - 2;
            hreg[u] = u32x4{0u, 0u, 0u, 0u};
            if (row < hrows && y >= 0 && y < D.H && x >= 0 && x < D.W)
                hreg[u] = *(const u32x4 *)(V + img_off + ((size_t)y * D.W + x) * C + c0 + c8 * 8);
        }
#pragma unroll
        for (int u = 0; u < NBH; ++u) {
            const int idx = first + (int)threadIdx.x + 256 * u;
            if (idx < hrows * CH8) *(u32x4 *)(Hs + (idx / CH8) * kLcePitch + (idx % CH8) * 8) = hreg[u];
        }
    }
    __syncthreads();

    const int cp_n = kLceChunk / 2, segs = (tw + 3) / 4;
    const int tasks = th * segs * cp_n;
    for (int task = threadIdx.x; task < tasks; task += 256) {
        const int seg = (task / cp_n) % segs, r = task / (cp_n * segs);
        float a0[4] = {0.f, 0.f, 0.f, 0.f}, a1[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ky = 0; ky < 5; ++ky) {
            float v0[8], v1[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const int hx = min(seg * 4 + x, hw - 1);    // a ragged segment re-reads the last column; unused
                const unsigned u = *(const unsigned *)(Hs + ((r + ky) * hw + hx) * kLcePitch + 2 * cpair);
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
                }
            }
        }
        // rows of O are ldo elements apart (C for a map of its own, more for a slice of a wider map)
        unsigned *orow = (unsigned *)(O + ((size_t)b * D.N + (size_t)(y0 + r) * D.W + x0 + seg * 4) * ldo + c0 + 2 * cpair);
        unsigned o2[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) o2[x] = seg * 4 + x < tw ? orow[(size_t)x * (ldo / 2)] : 0u;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (seg * 4 + x < tw) orow[(size_t)x * (ldo / 2)] = pack_bf16(bf16_lo(o2[x]) + a0[x], bf16_hi(o2[x]) + a1[x]);
    }
}

// LCE tile: full-width rows on maps up to 64 columns, else 4 rows x 32 columns.
int tile_cols(const Dims &D) { return D.W <= 64 ? D.W : 32; }
int tile_rows(const Dims &D) { return D.W <= 64 ? 64 / D.W : 4; }

int halo_rows_small(const Dims &D) { return (D.rh + 4) * (D.rw + 4); }

template <int C>
size_t small_smem(const Dims &D) { return SmallSmem<C>::bytes(halo_rows_small(D)); }

}  // namespace

// One kernel per region when a region fills the 16 query columns; else two kernels.
static bool one_kernel(const Dims &D)
{
    if (D.n != 16) return false;
    return D.rh * ((D.rw + 3) / 4) * (D.C / 2) <= 256 * kMaxLceTasks;
}

static size_t lce_add_smem(const Dims &D) { return (size_t)(tile_rows(D) + 4) * (tile_cols(D) + 4) * kLcePitch * 2; }

static size_t map_smem(const Dims &D, bool lce = false)
{
    return (size_t)3 * D.N * kMapPitch * 2 + (size_t)((D.R * D.k + D.R + 3) / 4 * 4) * 4 + kMapWaves * 512 +
           (lce ? (size_t)D.N * kMapLcePitch * 4 : 0);
}

// The LCE rides along in the attention kernel when its float32 tile fits and does not cost
// the second workgroup of a compute unit.
static bool map_adds_lce(const Dims &D)
{
    const size_t with = map_smem(D, true), half = (size_t)kMaxLds / 2;
    return with <= (size_t)kMaxLds && (with <= half || map_smem(D) > half);
}

// Image-resident attention when a head's K and V of one image fit in LDS.
static bool map_attention(const Dims &D) { return map_smem(D) <= (size_t)kMaxLds; }

// Parts per (image, head), so that small batches still fill the chip.
static int map_split(const Dims &D)
{
    static const int forced = (int)experiment_value("BRA_MAP_WGS", 0);
    const int target = forced >= 1 && forced <= 65536 ? forced : 512;
    const int wgs = D.B * (D.C / 32);
    const int split = (target + wgs - 1) / wgs;
    return std::max(1, std::min(split, D.R / kMapWaves));
}

bool small_supported(const Dims &D)
{
    if (D.n > 16 || (D.n & (D.n - 1)) != 0) return false;   // n = 1, 2, 4, 8, 16
    size_t smem;
    if (one_kernel(D)) {
        smem = D.C == 64 ? small_smem<64>(D) : D.C == 128 ? small_smem<128>(D) : small_smem<256>(D);
    } else {
        if (D.W > 64) return false;
        smem = lce_add_smem(D);
        const size_t attn = map_attention(D) ? map_smem(D)
                            : D.C == 64      ? SmallSmem<64>::kv_bytes
                            : D.C == 128     ? SmallSmem<128>::kv_bytes
                                             : SmallSmem<256>::kv_bytes;
        if (attn > smem) smem = attn;
    }
    return smem <= (size_t)kMaxLds;
}

bool small_needs_projection(const Dims &D) { return !one_kernel(D); }

size_t small_scratch_bytes(const Dims &D)
{
    return one_kernel(D) ? 0 : (size_t)D.B * D.N * D.C * 2;     // O_att between the two kernels
}

template <typename K>
static bool opt_in(K kernel, bool &done)
{
    if (done) return true;
    if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds) !=
        hipSuccess)
        return false;
    done = true;
    return true;
}

// Image-resident attention of all regions into O.
static int launch_map(const Dims &D, AttnArgs A, bf16_t *O, int log2n, hipStream_t st)
{
    static bool opted[4] = {false, false, false, false};
    if (!opt_in(k_attn_map<false>, opted[0]) || !opt_in(k_attn_map4<false>, opted[1]) ||
        !opt_in(k_attn_map<true>, opted[2]) || !opt_in(k_attn_map4<true>, opted[3]))
        return BRA_ERR_LAUNCH;
    const int split = map_split(D);
    const bool lce = map_adds_lce(D);
    ProfScope ps(st, K_MFMA_ATTN_SMALL);
    A.total = D.B * (D.C / 32) * split;
    const dim3 grid_map((A.total + 7) / 8 * 8);
    const size_t smem = map_smem(D, lce);
    if (D.n <= 4) {
        if (lce) hipLaunchKernelGGL(k_attn_map4<true>, grid_map, dim3(kMapThreads), smem, st, A, O, D, log2n, split);
        else hipLaunchKernelGGL(k_attn_map4<false>, grid_map, dim3(kMapThreads), smem, st, A, O, D, log2n, split);
    } else {
        if (lce) hipLaunchKernelGGL(k_attn_map<true>, grid_map, dim3(kMapThreads), smem, st, A, O, D, log2n, split);
        else hipLaunchKernelGGL(k_attn_map<false>, grid_map, dim3(kMapThreads), smem, st, A, O, D, log2n, split);
    }
    return BRA_OK;
}

// O += LCE(V) in place.
static int launch_lce_add(const Dims &D, const AttnArgs &A, bf16_t *O, hipStream_t st, int ldo = 0,
                          bool square_tiles = false)
{
    static bool opted = false;
    if (!opt_in(k_lce_add, opted)) return BRA_ERR_LAUNCH;
    // square_tiles: 4 rows x up to 32 columns, fewer halo rows per token than full-width rows
    const int TH = square_tiles ? 4 : tile_rows(D), TW = square_tiles ? std::min(D.W, 32) : tile_cols(D);
    const long blocks = (long)D.B * ((D.H + TH - 1) / TH) * ((D.W + TW - 1) / TW) * (D.C / kLceChunk);
    if (blocks > 0x7fffffffL) return BRA_ERR_UNSUPPORTED;
    const size_t smem = (size_t)(TH + 4) * (TW + 4) * kLcePitch * 2;
    ProfScope ps(st, K_MFMA_LCE_ADD);
    hipLaunchKernelGGL(k_lce_add, dim3((unsigned)blocks), dim3(256), smem, st, O, A.V, A.Wlce, D, TH, TW,
                       ldo ? ldo : D.C);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

template <int C>
static int launch_small_c(const Dims &D, const AttnArgs &A0, bf16_t *O, hipStream_t st)
{
    AttnArgs A = A0;
    A.total = D.B * D.R;
    int log2n = 0;
    while ((1 << log2n) < D.n) ++log2n;
    const int grid = ((A.total + 7) / 8) * 8;
    if (one_kernel(D)) {
        static bool opted = false;
        if (!opt_in(k_small<C>, opted)) return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_MFMA_ATTN_SMALL);
        hipLaunchKernelGGL(k_small<C>, dim3(grid), dim3(256), small_smem<C>(D), st, A, D, log2n);
        return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
    }
    if (map_attention(D)) {
        const int rc = launch_map(D, A, O, log2n, st);
        if (rc != BRA_OK || map_adds_lce(D)) return rc;
    } else {
        static bool opted = false;
        if (!opt_in(k_attn_small<C>, opted)) return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_MFMA_ATTN_SMALL);
        hipLaunchKernelGGL(k_attn_small<C>, dim3(grid), dim3(256), SmallSmem<C>::kv_bytes, st, A, O, D, log2n);
    }
    return launch_lce_add(D, A, O, st);
}

// Any C that is a multiple of 64: regions of fewer than 16 tokens on a map that fits the
// image-resident attention.
bool map_tail_supported(const Dims &D)
{
    if (D.C % 64 != 0 || D.d != 32) return false;
    if (D.n > 8 || (D.n & (D.n - 1)) != 0 || D.W > 64) return false;
    return map_attention(D) && lce_add_smem(D) <= (size_t)kMaxLds;
}

// O += LCE(V) in place for any map (C a multiple of 64).
int launch_lce_add_any(const Dims &D, const AttnArgs &A, bf16_t *O, hipStream_t st, int ldo, bool square_tiles)
{
    return launch_lce_add(D, A, O, st, ldo, square_tiles);
}

int launch_map_tail(const Dims &D, const AttnArgs &A, bf16_t *O, hipStream_t st)
{
    int log2n = 0;
    while ((1 << log2n) < D.n) ++log2n;
    const int rc = launch_map(D, A, O, log2n, st);
    if (rc != BRA_OK || map_adds_lce(D)) return rc;
    return launch_lce_add(D, A, O, st);
}

int launch_small(const Dims &D, const AttnArgs &A, bf16_t *O, hipStream_t st)
{
    switch (D.C) {
    case 64: return launch_small_c<64>(D, A, O, st);
    case 128: return launch_small_c<128>(D, A, O, st);
    case 256: return launch_small_c<256>(D, A, O, st);
    default: return BRA_ERR_UNSUPPORTED;
    }
}

}  // namespace bra
