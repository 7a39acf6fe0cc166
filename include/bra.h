/*
 * libbra -- forward pass of Bi-Level Routing Attention (BRA) on AMD MI355X (gfx950).
 *
 * C ABI.  Every data pointer is CALLER-OWNED DEVICE memory (dense, row-major, no
 * strides); `shape` and `out_bytes` are host pointers.  The compute entry points never
 * allocate, free or synchronise: scratch memory comes from `ws` (size from
 * bra_workspace_bytes, 256-byte aligned) and all work is enqueued on `hip_stream`
 * (a hipStream_t passed as void*; NULL = the default stream).  Outputs are valid
 * once the caller has synchronised that stream.  Calls that share a workspace must
 * be ordered on one stream.  (The measurement aid bra_profile_begin / bra_profile_end is
 * the exception: it creates and destroys HIP events and waits for them.)
 *
 * What is computed (paper: "BiFormer: Vision Transformer with Bi-Level Routing
 * Attention", Sec. 3.2, Eq. 3-7, Algorithm 1; W^o from Eq. 2):
 *   1. the H x W map of each image is cut into S x S non-overlapping regions of
 *      n = (H/S)(W/S) tokens; token (y, x) belongs to region (y / (H/S)) * S + x / (W/S);
 *   2. Q = X W^q, K = X W^k, V = X W^v                                   (Eq. 3);
 *   3. Q^r, K^r = per-region means of Q, K over all C channels;
 *      A^r = Q^r (K^r)^T  in [S^2, S^2]                                  (Eq. 4);
 *   4. I^r = indices of the k largest entries of each row of A^r          (Eq. 5),
 *      descending by value, equal values in ascending index order; the routing is
 *      shared by all heads;
 *   5. each query token of region i attends, per head (head j owns channels
 *      [j d, (j+1) d), d = C / heads), to the k n key/value tokens of regions
 *      I^r[i, 0..k) with ONE softmax over that union                      (Eq. 6-7, Eq. 1);
 *      the gathered K/V tensors of Eq. 6 are never materialised;
 *   6. LCE(V): 5 x 5 depth-wise cross-correlation of V over the whole H x W map,
 *      stride 1, zero padding 2, no bias, is added                        (Eq. 7);
 *   7. Y = (Attention + LCE(V)) W^o                                       (Eq. 2).
 *
 * Layouts:
 *   X, Y   [B, H, W, C]   channels-last (the paper's (H, W, C) with a batch axis)
 *   Wqkv   [C, 3C]        = [W^q | W^k | W^v] column blocks, used as x * W
 *   Wo     [C, C]         used as o * Wo
 *   Wlce   [C, 5, 5]      (channel, ky, kx); out[y,x,c] = sum w[c,ky,kx] V[y+ky-2, x+kx-2, c]
 *   Ir     [B, S*S, k]    int32 region indices
 *   Ar     [B, S*S, S*S]  float32, mean-pooled and unscaled as in Eq. 4
 * dtype is the element type of X, Wqkv, Wo, Wlce and Y; arithmetic accumulates in
 * float32 in every path, and the routing (steps 3-4) is always computed in float32
 * from X so that rounding of stored Q/K never decides an index.
 */
#ifndef BRA_H_
#define BRA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { BRA_F32 = 0, BRA_BF16 = 1 };                 /* bra_shape.dtype */

/* bra_shape.path: which kernel family runs.
 *   AUTO    the fastest family that supports the shape;
 *   GENERIC scalar (VALU) float32 kernels, any valid shape, float32 intermediates;
 *   MFMA    bf16 matrix-core kernels: bf16 tensors, C a multiple of 64, heads of 32 or
 *           64 channels (specialised kernels for C = 64, 128, 256 with heads of 32
 *           and the region sizes of the paper's stages; a general pipeline for the
 *           rest); BRA_ERR_UNSUPPORTED otherwise. */
enum { BRA_PATH_AUTO = 0, BRA_PATH_GENERIC = 1, BRA_PATH_MFMA = 2 };

enum {
    BRA_OK = 0,
    BRA_ERR_NULL = -1,        /* a required pointer is NULL */
    BRA_ERR_SHAPE = -2,       /* B,H,W,C,heads,S < 1; H % S or W % S or C % heads != 0 */
    BRA_ERR_K = -3,           /* k < 1 or k > S*S */
    BRA_ERR_DTYPE = -4,       /* dtype or path is not one of the enums above */
    BRA_ERR_WORKSPACE = -5,   /* ws is NULL, misaligned (256 B) or too small */
    BRA_ERR_UNSUPPORTED = -6, /* valid shape outside what the kernels are built for */
    BRA_ERR_LAUNCH = -7,      /* the HIP runtime reported an error at enqueue time */
    BRA_ERR_TOO_LARGE = -8    /* bra_forward_static: the shape needs more than BRA_STATIC_SCRATCH_BYTES */
};

typedef struct bra_shape {
    int32_t B, H, W, C;   /* batch, map height, map width, channels */
    int32_t heads;        /* attention heads; d = C / heads */
    int32_t S;            /* regions per side; the paper picks S as a divisor of H and W */
    int32_t k;            /* regions each region attends to, 1 <= k <= S*S */
    int32_t dtype;        /* BRA_F32 or BRA_BF16 */
    float scale;          /* softmax logit scale; <= 0 selects 1/sqrt(d) (Eq. 1 on Eq. 2's heads) */
    int32_t path;         /* BRA_PATH_* */
} bra_shape;

/* Host-only.  Bytes of scratch bra_route / bra_forward need for `shape` (the
 * larger of the two).  Errors: NULL, SHAPE, K, DTYPE, UNSUPPORTED. */
int bra_workspace_bytes(const bra_shape *shape, size_t *out_bytes);

/* Region-to-region routing only (Eq. 4-5).  Writes Ir [B,S*S,k]; if Ar_opt is not
 * NULL also the affinity matrix [B,S*S,S*S].  Wqkv's W^v block is not read.
 * All checks run on the host before anything is enqueued. */
int bra_route(const bra_shape *shape, const void *X, const void *Wqkv, int32_t *Ir,
              float *Ar_opt, void *ws, size_t ws_bytes, void *hip_stream);

/* Whole BRA forward (steps 1-7).  Ir_out_opt (or NULL) receives the routing index
 * that was used.  Ir_in_opt (or NULL) forces the routing: steps 3-4 are skipped and
 * these indices are used instead; entries must lie in [0, S*S) and be distinct
 * within a row (not checked on the host: they are device data).  The kernels clamp
 * an out-of-range entry into [0, S*S) where they read it, so a wrong index gives a
 * wrong result, never an access outside the tensors; Ir_out_opt receives the
 * entries as given. */
int bra_forward(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                void *ws, size_t ws_bytes, void *hip_stream);

/* bra_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments and results as bra_forward (bit for bit: the same kernels run), but the scratch
 * memory is a buffer of BRA_STATIC_SCRATCH_BYTES inside the library's code object; every GPU the
 * library runs on holds one such buffer from the time the library is loaded there until the
 * process ends.  The call allocates and frees nothing.  The first call on each device looks up
 * the buffer's address (hipGetSymbolAddress; no allocation, but not to be captured into a
 * graph); later calls only enqueue kernels.  Shapes whose workspace (bra_workspace_bytes)
 * exceeds the buffer are rejected with BRA_ERR_TOO_LARGE before anything is enqueued; the
 * other errors are those of bra_forward.  The buffer keeps the previous call's contents (no
 * kernel of the forward pass needs it zeroed).  All calls on one GPU share it: calls that may
 * overlap on that GPU (different streams, or one stream from several threads) race; order them
 * on one stream. */
#define BRA_STATIC_SCRATCH_BYTES (32u << 20)
int bra_forward_static(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                       const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                       void *hip_stream);

/* BRA on a map whose sides S does not divide (appendix on the choice of S and k: S is picked
 * as a divisor of the training size so that no padding is needed; other sizes are padded).
 * shape->H, shape->W are the caller's map and need not be multiples of S.  Reading of the
 * padding, which the paper does not spell out: zero tokens are appended at the bottom and at
 * the right up to Hp = ceil(H / S) S, Wp = ceil(W / S) S; steps 1-7 run on the padded map
 * (a zero token has zero Q, K, V: it takes part in its region's means, is a key with logit 0 and
 * value 0, and LCE sees it like its own zero padding); Y [B, H, W, C] is the top-left part of
 * the result.  Ir [B, S*S, k] indexes the regions of the padded map.  When S divides H and W this
 * is bra_forward.  Workspace size from bra_padded_workspace_bytes.  Errors as bra_forward. */
int bra_padded_workspace_bytes(const bra_shape *shape, size_t *out_bytes);
int bra_forward_padded(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                       const void *Wlce, void *Y, int32_t *Ir_out_opt, const int32_t *Ir_in_opt,
                       void *ws, size_t ws_bytes, void *hip_stream);

/* One whole BiFormer block around BRA (Sec. 3.4): a 3x3 depth-wise convolution at the start
 * encodes relative position, then the BRA module and a 2-layer MLP (expansion ratio e,
 * hidden = e C channels) follow.  The figure that fixes normalisation and residual links is
 * read as the pre-norm residual form of the works that section cites:
 *     X1   = X  + DWConv3x3(X) + bpos          cross-correlation, stride 1, zero padding 1
 *     X2   = X1 + BRA(LayerNorm1(X1))          steps 1-7 above
 *     Xout = X2 + GELU(LayerNorm2(X2) W1 + b1) W2 + b2
 * LayerNorm: per token over its C channels, biased variance, eps inside the square root,
 * then gamma, beta.  GELU(t) = t Phi(t) (the exact form; evaluated with an erf approximation
 * of absolute error < 3e-7).
 * bra_block_params is a HOST struct of DEVICE pointers, all required:
 *   Wpos [C,3,3] (channel, ky, kx), W1 [C, hidden], W2 [hidden, C], Wqkv, Wo, Wlce as above,
 *   all of shape->dtype; the vectors bpos, ln*_gamma, ln*_beta, b2 [C] and b1 [hidden] float32.
 * bf16 tensors with C and hidden multiples of 64 run on matrix-core kernels; float32 tensors and
 * all other sizes on scalar float32 kernels (C up to 4096).  The
 * BRA stage runs on the family that bra_forward would pick for `shape` (shape->path applies).
 * Intermediate tensors (X1, LayerNorm1's output, BRA's output, X2, the hidden layer) live in
 * `ws` in shape->dtype; arithmetic is float32.  Xout may be the same buffer as X.  Ir_out_opt /
 * Ir_in_opt as in bra_forward.  Errors: as bra_forward; SHAPE for hidden < 1 or eps < 0. */
typedef struct bra_block_params {
    const void *Wpos;
    const float *bpos;
    const float *ln1_gamma, *ln1_beta;
    const void *Wqkv, *Wo, *Wlce;
    const float *ln2_gamma, *ln2_beta;
    const void *W1;
    const float *b1;
    const void *W2;
    const float *b2;
} bra_block_params;

/* Host-only: bytes of scratch bra_block_forward needs. */
int bra_block_workspace_bytes(const bra_shape *shape, int32_t hidden, size_t *out_bytes);

int bra_block_forward(const bra_shape *shape, int32_t hidden, float eps, const void *X,
                      const bra_block_params *params, void *Xout, int32_t *Ir_out_opt,
                      const int32_t *Ir_in_opt, void *ws, size_t ws_bytes, void *hip_stream);

/* Backward pass of the layer with the routing held fixed (the top-k of Eq. 5 has no derivative:
 * training goes through the token-level attention of Eq. 6-7 only).  Given dY = dLoss/dY
 * [B,H,W,C] and the routing index Ir [B,S*S,k] that the forward used, with O = Attention +
 * LCE(V) and, per query token t of region i and head h, P = softmax over the keys of its
 * routed regions:
 *     dO = dY Wo^T,  dWo = O^T dY,  dV += LCE^T(dO),  dWlce[c,ky,kx] = sum dO[y,x,c] V[y+ky-2,x+kx-2,c],
 *     dP_j = dO_h[t] . V_h[j],  dS_j = P_j (dP_j - sum_u P_u dP_u),
 *     dQ_h[t] = scale sum_j dS_j K_h[j],  dK_h[j] += scale dS_j Q_h[t],  dV_h[j] += P_j dO_h[t],
 *     dX = [dQ|dK|dV] Wqkv^T,  dWqkv = X^T [dQ|dK|dV].
 * The forward intermediates are recomputed from X.  dX [B,H,W,C] has shape->dtype; the weight
 * gradients dWqkv [C,3C], dWo [C,C], dWlce [C,5,5] are float32, summed over the batch and
 * OVERWRITTEN.  Two kernel families, chosen by shape->path as in bra_forward:
 *   BRA_PATH_MFMA     bf16 tensors, heads of 32 or 64 channels, C a multiple of 64 and
 *                     S*S*k <= 4096 routing entries per image: matrix-core kernels with bf16
 *                     operands and float32 sums; Q, K, V, dO, P, dS, dQ, dK, dV are rounded to
 *                     bf16 between the products.  No atomic adds: dK, dV are summed per key
 *                     region in registers, the weight gradients from per-workgroup partial sums in
 *                     a fixed order, so a repeat gives the same bits as long as no key region is
 *                     routed to by more than 256 index entries of one image.
 *   BRA_PATH_GENERIC  any dtype, heads up to 64 channels wide: scalar float32 kernels; sums over
 *                     tokens use float32 atomic adds, reproducible to rounding, not bit for bit.
 *   BRA_PATH_AUTO     the first where it applies, else the second.
 * Index values outside [0, S*S) are clamped.  Errors as bra_forward. */
int bra_backward_workspace_bytes(const bra_shape *shape, size_t *out_bytes);
int bra_backward(const bra_shape *shape, const void *X, const void *Wqkv, const void *Wo,
                 const void *Wlce, const int32_t *Ir, const void *dY, void *dX, float *dWqkv,
                 float *dWo, float *dWlce, void *ws, size_t ws_bytes, void *hip_stream);

/* Optional per-launch timing, for benchmarks (Sec. "Limitation": the paper locates
 * BRA's cost in kernel launches and memory transactions, so the benchmark reports
 * time per kernel).  Host-only state, one session at a time, not thread-safe.
 * bra_profile_begin creates 2 * max_records HIP events; from then on every kernel
 * the library enqueues is bracketed by two events on the caller's stream, until
 * max_records launches have been recorded.  bra_profile_end waits for the recorded
 * events, writes up to max_records (kernel id, milliseconds) pairs in launch order
 * to the HOST arrays ids / ms, stores the count in *n_out and destroys the events.
 * bra_kernel_name maps a kernel id to a static string.
 * Errors: SHAPE (begin while active, end while inactive, max_records < 1), NULL,
 * LAUNCH (event API failure). */
int bra_profile_begin(int max_records);
int bra_profile_end(int32_t *ids, float *ms, int max_records, int *n_out);
const char *bra_kernel_name(int id);

/* Measurement aids: plain streaming kernels over `bytes` bytes of device memory
 * (multiple of 16, pointers 16-byte aligned), enqueued on hip_stream.  bra_util_copy
 * copies src to dst; its known traffic (bytes read + bytes written) is what hardware
 * byte counters are scaled against.  bra_util_read only reads src (scratch4: 4 bytes
 * of device memory that are practically never written).  Errors: NULL, SHAPE, LAUNCH. */
int bra_util_copy(void *dst, const void *src, size_t bytes, void *hip_stream);
int bra_util_read(const void *src, size_t bytes, void *scratch4, void *hip_stream);

/* Matrix-core throughput probes: `workgroups` workgroups of 4 wavefronts, each wavefront
 * issuing 8 * iters dense bf16 16x16x32 matrix products (bra_util_mfma; 16384 flops each) or
 * 4 * iters dense bf16 32x32x16 products (bra_util_mfma32; 32768 flops each) on register
 * operands, enqueued on hip_stream; scratch4 as above.  The measured rates stand beside the
 * published peak in the benchmark line.  Errors: NULL, SHAPE, LAUNCH. */
int bra_util_mfma(int workgroups, int iters, void *scratch4, void *hip_stream);
int bra_util_mfma32(int workgroups, int iters, void *scratch4, void *hip_stream);

/* Static, human-readable text for a return code. */
const char *bra_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int bra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BRA_H_ */
