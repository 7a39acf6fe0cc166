// C-ABI entry points of libbra: argument checks and dispatch to a kernel family.
#include "bra_common.h"

#include <math.h>

#include <mutex>

// Scratch memory of bra_forward_static: one copy per GPU, held by the code object until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the
// address that kernels, copies and fills take is the one that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[BRA_STATIC_SCRATCH_BYTES];

namespace bra {

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void *ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return BRA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BRA_ERR_LAUNCH;
        if ((uintptr_t)p % 256 != 0) return BRA_ERR_LAUNCH;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return BRA_OK;
}

// Validates `s` and fills D.  Returns a BRA_* code.
static int make_dims(const bra_shape *s, Dims &D)
{
    if (!s) return BRA_ERR_NULL;
    if (s->B < 1 || s->H < 1 || s->W < 1 || s->C < 1 || s->heads < 1 || s->S < 1) return BRA_ERR_SHAPE;
    if (s->H % s->S || s->W % s->S || s->C % s->heads) return BRA_ERR_SHAPE;
    if ((long)s->S * s->S > (1L << 20)) return BRA_ERR_SHAPE;
    if (s->k < 1 || s->k > s->S * s->S) return BRA_ERR_K;
    if (s->dtype != BRA_F32 && s->dtype != BRA_BF16) return BRA_ERR_DTYPE;
    if (s->path != BRA_PATH_AUTO && s->path != BRA_PATH_GENERIC && s->path != BRA_PATH_MFMA)
        return BRA_ERR_DTYPE;
    // element counts must stay addressable with the 31-bit token indices the kernels use
    if ((long)s->H * s->W > (1L << 30) || (long)s->B * s->H * s->W > (1L << 30)) return BRA_ERR_SHAPE;
    D.B = s->B; D.H = s->H; D.W = s->W; D.C = s->C; D.heads = s->heads; D.S = s->S; D.k = s->k;
    D.dtype = s->dtype;
    D.rh = s->H / s->S; D.rw = s->W / s->S; D.n = D.rh * D.rw; D.R = s->S * s->S;
    D.N = s->H * s->W; D.d = s->C / s->heads; D.kn = D.k * D.n;
    D.scale = (s->scale > 0.f) ? s->scale : 1.0f / sqrtf((float)D.d);
    return BRA_OK;
}

// Picks the kernel family: returns BRA_PATH_GENERIC / BRA_PATH_MFMA or an error.
static int pick_path(const bra_shape *s, const Dims &D)
{
    const bool mfma_ok = mfma_supported(D);
    if (s->path == BRA_PATH_MFMA) return mfma_ok ? BRA_PATH_MFMA : BRA_ERR_UNSUPPORTED;
    if (s->path == BRA_PATH_AUTO && mfma_ok) return BRA_PATH_MFMA;
    return generic_supported(D) ? BRA_PATH_GENERIC : BRA_ERR_UNSUPPORTED;
}

// The shape with H and W rounded up to multiples of S (the map after zero padding).
static int make_padded_dims(const bra_shape *s, Dims &Dp)
{
    if (!s) return BRA_ERR_NULL;
    if (s->H < 1 || s->W < 1 || s->S < 1 || s->S > 1024) return BRA_ERR_SHAPE;
    if (s->H > (1 << 24) || s->W > (1 << 24)) return BRA_ERR_SHAPE;
    bra_shape p = *s;
    p.H = (s->H + s->S - 1) / s->S * s->S;
    p.W = (s->W + s->S - 1) / s->S * s->S;
    return make_dims(&p, Dp);
}

static bool ws_ok(const void *ws, size_t have, size_t need)
{
    return ws && ((uintptr_t)ws % 256 == 0) && have >= need;
}

}  // namespace bra

using namespace bra;

extern "C" {

int bra_workspace_bytes(const bra_shape *shape, size_t *out_bytes)
{
    if (!out_bytes) return BRA_ERR_NULL;
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    *out_bytes = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    return BRA_OK;
}

int bra_route(const bra_shape *shape, const void *X, const void *Wqkv, int32_t *Ir, float *Ar_opt,
              void *ws, size_t ws_bytes, void *hip_stream)
{
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (!X || !Wqkv || !Ir) return BRA_ERR_NULL;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    size_t need = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    if (!ws_ok(ws, ws_bytes, need)) return BRA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    if (path == BRA_PATH_MFMA) return mfma_route(D, X, Wqkv, Ir, Ar_opt, ws, st);
    return generic_route(D, X, Wqkv, Ir, Ar_opt, ws, st);
}

int bra_forward(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws,
                size_t ws_bytes, void *hip_stream)
{
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (!X || !Wqkv || !Wo || !Wlce || !Y) return BRA_ERR_NULL;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    size_t need = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    if (!ws_ok(ws, ws_bytes, need)) return BRA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    if (path == BRA_PATH_MFMA)
        return mfma_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, st);
    return generic_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, st);
}

int bra_forward_static(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                       const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                       void *hip_stream)
{
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (!X || !Wqkv || !Wo || !Wlce || !Y) return BRA_ERR_NULL;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    const size_t need = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    if (need > (size_t)BRA_STATIC_SCRATCH_BYTES) return BRA_ERR_TOO_LARGE;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != BRA_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    // no kernel of the forward pass expects zeroed scratch (no counters, no accumulation into it):
    // every buffer carved from it is written before it is read within the call
    if (path == BRA_PATH_MFMA)
        return mfma_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, st);
    return generic_forward(D, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, st);
}

int bra_padded_workspace_bytes(const bra_shape *shape, size_t *out_bytes)
{
    if (!out_bytes) return BRA_ERR_NULL;
    Dims Dp;
    int rc = make_padded_dims(shape, Dp);
    if (rc != BRA_OK) return rc;
    bra_shape ps = *shape;
    ps.H = Dp.H; ps.W = Dp.W;
    int path = pick_path(&ps, Dp);
    if (path < 0) return path;
    const size_t inner = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(Dp) : generic_workspace_bytes(Dp);
    *out_bytes = (Dp.H == shape->H && Dp.W == shape->W) ? inner : padded_workspace_bytes(Dp, inner);
    return BRA_OK;
}

int bra_forward_padded(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                       void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, size_t ws_bytes,
                       void *hip_stream)
{
    Dims Dp;
    int rc = make_padded_dims(shape, Dp);
    if (rc != BRA_OK) return rc;
    if (!X || !Wqkv || !Wo || !Wlce || !Y) return BRA_ERR_NULL;
    bra_shape ps = *shape;
    ps.H = Dp.H; ps.W = Dp.W;
    if (Dp.H == shape->H && Dp.W == shape->W)
        return bra_forward(&ps, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, ws_bytes, hip_stream);
    int path = pick_path(&ps, Dp);
    if (path < 0) return path;
    const size_t inner = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(Dp) : generic_workspace_bytes(Dp);
    if (!ws_ok(ws, ws_bytes, padded_workspace_bytes(Dp, inner))) return BRA_ERR_WORKSPACE;
    return padded_forward(Dp, shape->H, shape->W, X, Wqkv, Wo, Wlce, Y, Ir_out_opt, Ir_in_opt, ws, path,
                          (hipStream_t)hip_stream);
}

// Kernel family of the backward pass: the matrix-core kernels where they apply (bf16, heads of
// 32 or 64 channels, C a multiple of 64, at most 4096 routing entries per image), else the scalar
// float32 kernels.
static int pick_backward_path(const bra_shape *s, const Dims &D)
{
    const bool mfma_ok = mfma_backward_supported(D);
    if (s->path == BRA_PATH_MFMA) return mfma_ok ? BRA_PATH_MFMA : BRA_ERR_UNSUPPORTED;
    if (s->path == BRA_PATH_AUTO && mfma_ok) return BRA_PATH_MFMA;
    return generic_backward_supported(D) ? BRA_PATH_GENERIC : BRA_ERR_UNSUPPORTED;
}

int bra_backward_workspace_bytes(const bra_shape *shape, size_t *out_bytes)
{
    if (!out_bytes) return BRA_ERR_NULL;
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    const int path = pick_backward_path(shape, D);
    if (path < 0) return path;
    *out_bytes = (path == BRA_PATH_MFMA) ? mfma_backward_workspace_bytes(D) : generic_backward_workspace_bytes(D);
    return BRA_OK;
}

int bra_backward(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                 const int32_t *Ir, const void *dY, void *dX, float *dWqkv, float *dWo, float *dWlce, void *ws,
                 size_t ws_bytes, void *hip_stream)
{
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (!X || !Wqkv || !Wo || !Wlce || !Ir || !dY || !dX || !dWqkv || !dWo || !dWlce) return BRA_ERR_NULL;
    const int path = pick_backward_path(shape, D);
    if (path < 0) return path;
    if (path == BRA_PATH_MFMA) {
        if (!ws_ok(ws, ws_bytes, mfma_backward_workspace_bytes(D))) return BRA_ERR_WORKSPACE;
        return mfma_backward(D, X, Wqkv, Wo, Wlce, Ir, dY, dX, dWqkv, dWo, dWlce, ws, (hipStream_t)hip_stream);
    }
    if (!ws_ok(ws, ws_bytes, generic_backward_workspace_bytes(D))) return BRA_ERR_WORKSPACE;
    return generic_backward(D, X, Wqkv, Wo, Wlce, Ir, dY, dX, dWqkv, dWo, dWlce, ws, (hipStream_t)hip_stream);
}

int bra_block_workspace_bytes(const bra_shape *shape, int32_t hidden, size_t *out_bytes)
{
    if (!out_bytes) return BRA_ERR_NULL;
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (hidden < 1) return BRA_ERR_SHAPE;
    if (!block_supported(D, hidden)) return BRA_ERR_UNSUPPORTED;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    const size_t inner = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    *out_bytes = block_workspace_bytes(D, hidden, inner);
    return BRA_OK;
}

int bra_block_forward(const bra_shape *shape, int32_t hidden, float eps, const void *X,
                      const bra_block_params *p, void *Xout, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                      void *ws, size_t ws_bytes, void *hip_stream)
{
    Dims D;
    int rc = make_dims(shape, D);
    if (rc != BRA_OK) return rc;
    if (hidden < 1 || !(eps >= 0.f)) return BRA_ERR_SHAPE;
    if (!X || !p || !Xout) return BRA_ERR_NULL;
    if (!p->Wpos || !p->bpos || !p->ln1_gamma || !p->ln1_beta || !p->Wqkv || !p->Wo || !p->Wlce ||
        !p->ln2_gamma || !p->ln2_beta || !p->W1 || !p->b1 || !p->W2 || !p->b2)
        return BRA_ERR_NULL;
    if (!block_supported(D, hidden)) return BRA_ERR_UNSUPPORTED;
    int path = pick_path(shape, D);
    if (path < 0) return path;
    const size_t inner = (path == BRA_PATH_MFMA) ? mfma_workspace_bytes(D) : generic_workspace_bytes(D);
    if (!ws_ok(ws, ws_bytes, block_workspace_bytes(D, hidden, inner))) return BRA_ERR_WORKSPACE;
    return block_forward(D, hidden, eps, X, *p, Xout, Ir_out_opt, Ir_in_opt, ws, inner, path,
                         (hipStream_t)hip_stream);
}

const char *bra_strerror(int code)
{
    switch (code) {
    case BRA_OK: return "ok";
    case BRA_ERR_NULL: return "a required pointer is NULL";
    case BRA_ERR_SHAPE: return "invalid shape (sizes must be positive, S must divide H and W, heads must divide C)";
    case BRA_ERR_K: return "k must satisfy 1 <= k <= S*S";
    case BRA_ERR_DTYPE: return "unknown dtype or path";
    case BRA_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small";
    case BRA_ERR_UNSUPPORTED: return "shape not supported by the requested kernel family";
    case BRA_ERR_LAUNCH: return "HIP runtime error while enqueueing";
    case BRA_ERR_TOO_LARGE: return "shape needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown error code";
    }
}

int bra_version(void) { return 100; }

}  // extern "C"
