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
// Smaller regions use separate kernels: k_attn_small (attention output to memory),
// k_lce_add (adds the LCE in place), then the projection kernel with W^o.
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
    const float rw_inv = 1.0f / (float)D.rw;

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
            const int j = irp[key >> log2n], slot = key & (n - 1);
            const int sy = fast_div(slot, rw_inv);
            const size_t tok = (size_t)((j / D.S) * D.rh + sy) * D.W + (j % D.S) * D.rw + slot - sy * D.rw;
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
        const float inv = 1.0f / st.l[hh];         // heads past the end: 1 / 0 times 0, never used
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
    __host__ __device__ static size_t o_off(int hrows)   // [16][CS] bf16: O = attention + LCE
    {
        const size_t second = (size_t)hrows * CS * 2 + lt_bytes;
        return kv_bytes > second ? kv_bytes : second;
    }
    static size_t bytes(int hrows) { return o_off(hrows) + (size_t)16 * CS * 2; }
};

template <int C>
__global__ __launch_bounds__(256) void k_small(AttnArgs A, Dims D, int log2n)
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
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int g = lane / 16, i = lane % 16;
    const int b = wid / D.R, reg = wid % D.R;
    const size_t img_off = (size_t)b * D.N * C;
    const int n = D.n;
    const float rw_inv = 1.0f / (float)D.rw, hw_inv = 1.0f / (float)hw;
    const int y0 = (reg / D.S) * D.rh, x0 = (reg % D.S) * D.rw;

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

    f32x4 oacc[HPW][2];     // normalised attention output of this wavefront's heads
    small_attention<C>(A, D, log2n, img_off, irp, qtok, Ks, Vs, oacc);
    __builtin_amdgcn_s_setprio(2);      // late phases first: the workgroup's LDS is freed sooner
    __syncthreads();        // the key blocks have been read: the halo tile takes their place
    tile_store<C, CS, NBH>(Hs, hreg, hrows, 0);
    for (int first = 256 * NBH; first < hrows * CH; first += 256 * NBH) {
        tile_load<C, NBH>(hreg, A.V + img_off, y0 - 2, x0 - 2, hw, hw_inv, hrows, D.H, D.W, first);
        tile_store<C, CS, NBH>(Hs, hreg, hrows, first);
    }

    // LCE (Eq. 7) of the region's tokens: task = (row r, 4-token segment, channel pair);
    // a thread keeps its channel pair for all its tasks, so its 2 x 25 weights stay in
    // registers.
    const int cp_n = C / 2, segs = (D.rw + 3) / 4;
    const int tasks = D.rh * segs * cp_n;
    const int cpair = threadIdx.x % cp_n;
    unsigned wl[25];        // tap t of channels (c, c + 1) as a packed pair, from the tap-major table
#pragma unroll
    for (int t = 0; t < 25; ++t) wl[t] = *(const unsigned *)(A.WlT + (size_t)t * C + 2 * cpair);
    auto tap = [&](int ch, int t) { return ch ? bf16_hi(wl[t]) : bf16_lo(wl[t]); };
    float lce[kMaxLceTasks][2][4];
    __syncthreads();        // the halo tile is complete
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
    const size_t qtok = (size_t)((reg / D.S) * D.rh + qy) * D.W + (reg % D.S) * D.rw + qs - qy * D.rw;

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
// O <- O_att + LCE(V) (Eq. 7) in place, for workgroup (image, tile of TH full-width image
// rows, chunk of 64 channels).  LDS holds the V halo tile of the chunk, [(TH + 4) x (W + 4)]
// tokens x 64 channels; a thread keeps one channel pair for all its (row, 4-token segment)
// tasks, so its 2 x 25 weights stay in registers.  W^o follows as a plain projection.
constexpr int kLceChunk = 64, kLcePitch = kLceChunk + 8;

template <int C>
__global__ __launch_bounds__(256) void k_lce_add(bf16_t *__restrict__ O, const bf16_t *__restrict__ V,
                                                 const bf16_t *__restrict__ Wlce, Dims D, int TH)
{
    constexpr int NCH = C / kLceChunk, CH8 = kLceChunk / 8, NBH = 6;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *Hs = (bf16_t *)smem;
    const int tiles = (D.H + TH - 1) / TH;
    const int cc = blockIdx.x % NCH, tile = (blockIdx.x / NCH) % tiles, b = blockIdx.x / (NCH * tiles);
    const int y0 = tile * TH;
    const int th = min(TH, D.H - y0);            // rows of this tile
    const size_t img_off = (size_t)b * D.N * C;
    const int hw = D.W + 4, hrows = (th + 4) * hw;
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
            const int y = y0 - 2 + ry, x = row - ry * hw - 2;
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

    const int cp_n = kLceChunk / 2, segs = (D.W + 3) / 4;
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
        unsigned *orow = (unsigned *)(O + img_off + ((size_t)(y0 + r) * D.W + seg * 4) * C + c0 + 2 * cpair);
        unsigned o2[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) o2[x] = seg * 4 + x < D.W ? orow[(size_t)x * C / 2] : 0u;
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (seg * 4 + x < D.W) orow[(size_t)x * C / 2] = pack_bf16(bf16_lo(o2[x]) + a0[x], bf16_hi(o2[x]) + a1[x]);
    }
}

int tile_rows(const Dims &D) { return 64 / D.W; }

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

static size_t lce_add_smem(const Dims &D) { return (size_t)(tile_rows(D) + 4) * (D.W + 4) * kLcePitch * 2; }

bool small_supported(const Dims &D)
{
    if (D.n > 16 || (D.n & (D.n - 1)) != 0) return false;   // n = 1, 2, 4, 8, 16
    size_t smem;
    if (one_kernel(D)) {
        smem = D.C == 64 ? small_smem<64>(D) : D.C == 128 ? small_smem<128>(D) : small_smem<256>(D);
    } else {
        if (D.W > 64) return false;
        smem = lce_add_smem(D);
        const size_t attn = D.C == 64 ? SmallSmem<64>::kv_bytes : D.C == 128 ? SmallSmem<128>::kv_bytes : SmallSmem<256>::kv_bytes;
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
    {
        static bool opted = false;
        if (!opt_in(k_attn_small<C>, opted)) return BRA_ERR_LAUNCH;
        ProfScope ps(st, K_MFMA_ATTN_SMALL);
        hipLaunchKernelGGL(k_attn_small<C>, dim3(grid), dim3(256), SmallSmem<C>::kv_bytes, st, A, O, D, log2n);
    }
    {
        static bool opted = false;
        if (!opt_in(k_lce_add<C>, opted)) return BRA_ERR_LAUNCH;
        const int TH = tile_rows(D);
        const int tiles = (D.H + TH - 1) / TH;
        ProfScope ps(st, K_MFMA_LCE_ADD);
        hipLaunchKernelGGL(k_lce_add<C>, dim3(D.B * tiles * (C / kLceChunk)), dim3(256), lce_add_smem(D), st, O,
                           A.V, A.Wlce, D, TH);
    }
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
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
