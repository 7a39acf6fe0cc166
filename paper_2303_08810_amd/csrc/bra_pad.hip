// BRA on maps whose sides S does not divide: zero tokens are appended at the bottom and right,
// the layer runs on the padded map, the top-left H x W part of its output is returned
// (the appendix on the choice of S and k: S is a divisor of the training size so that no padding
// is needed; at other sizes the map is padded).
#include "bra_common.h"

namespace bra {

namespace {

typedef unsigned __attribute__((ext_vector_type(4))) u32x4_t;

template <typename U>
__device__ inline U zero_unit() { return U(0); }
template <>
__device__ inline u32x4_t zero_unit<u32x4_t>() { return u32x4_t{0u, 0u, 0u, 0u}; }

// dst [B, Hd, Wd, CU] <- src [B, Hs, Ws, CU] in units U (CU units per token): tokens of dst
// outside src are zero, tokens of src outside dst are dropped.
template <typename U>
__global__ __launch_bounds__(256) void k_resize_map(U *__restrict__ dst, const U *__restrict__ src, int Hd, int Wd,
                                                    int Hs, int Ws, int CU, long units)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= units) return;
    const int cu = (int)(idx % CU);
    const long tok = idx / CU;
    const int x = (int)(tok % Wd);
    const long row = tok / Wd;
    const int y = (int)(row % Hd);
    const long b = row / Hd;
    dst[idx] = (y < Hs && x < Ws) ? src[((b * Hs + y) * Ws + x) * CU + cu] : zero_unit<U>();
}

int resize_map(void *dst, const void *src, int B, int Hd, int Wd, int Hs, int Ws, int C, int esize, hipStream_t st)
{
    const long row_bytes = (long)C * esize;
    const bool wide = row_bytes % 16 == 0 && (uintptr_t)dst % 16 == 0 && (uintptr_t)src % 16 == 0;
    const int unit = wide ? 16 : esize;
    const int CU = (int)(row_bytes / unit);
    const long units = (long)B * Hd * Wd * CU;
    const long grid = (units + 255) / 256;
    if (grid > 0x7fffffffL) return BRA_ERR_SHAPE;
    if (unit == 16)
        hipLaunchKernelGGL(k_resize_map<u32x4_t>, dim3((unsigned)grid), dim3(256), 0, st, (u32x4_t *)dst,
                           (const u32x4_t *)src, Hd, Wd, Hs, Ws, CU, units);
    else if (unit == 4)
        hipLaunchKernelGGL(k_resize_map<uint32_t>, dim3((unsigned)grid), dim3(256), 0, st, (uint32_t *)dst,
                           (const uint32_t *)src, Hd, Wd, Hs, Ws, CU, units);
    else
        hipLaunchKernelGGL(k_resize_map<uint16_t>, dim3((unsigned)grid), dim3(256), 0, st, (uint16_t *)dst,
                           (const uint16_t *)src, Hd, Wd, Hs, Ws, CU, units);
    return hipGetLastError() == hipSuccess ? BRA_OK : BRA_ERR_LAUNCH;
}

size_t map_bytes(const Dims &Dp) { return align256((size_t)Dp.B * Dp.N * Dp.C * (Dp.dtype == BRA_BF16 ? 2 : 4)); }

}  // namespace

size_t padded_workspace_bytes(const Dims &Dp, size_t bra_bytes) { return 2 * map_bytes(Dp) + align256(bra_bytes); }

// Dp: dimensions of the padded map; H, W: the caller's map.
int padded_forward(const Dims &Dp, int H, int W, const void *X, const void *Wqkv, const void *Wo, const void *Wlce,
                   void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt, void *ws, int path, hipStream_t st)
{
    const int esize = Dp.dtype == BRA_BF16 ? 2 : 4;
    char *Xp = (char *)ws, *Yp = Xp + map_bytes(Dp), *inner = Yp + map_bytes(Dp);
    int rc = resize_map(Xp, X, Dp.B, Dp.H, Dp.W, H, W, Dp.C, esize, st);
    if (rc != BRA_OK) return rc;
    rc = (path == BRA_PATH_MFMA) ? mfma_forward(Dp, Xp, Wqkv, Wo, Wlce, Yp, Ir_out_opt, Ir_in_opt, inner, st)
                                 : generic_forward(Dp, Xp, Wqkv, Wo, Wlce, Yp, Ir_out_opt, Ir_in_opt, inner, st);
    if (rc != BRA_OK) return rc;
    return resize_map(Y, Yp, Dp.B, H, W, Dp.H, Dp.W, Dp.C, esize, st);
}

}  // namespace bra
