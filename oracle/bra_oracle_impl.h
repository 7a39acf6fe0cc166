/*
 * TEST INFRASTRUCTURE -- CPU oracle for the forward pass of Bi-Level Routing
 * Attention (BRA), "BiFormer: Vision Transformer with Bi-Level Routing Attention".
 *
 * This file is included twice by bra_oracle.c, once with REAL = float and once
 * with REAL = double.  It is a plain, slow, step-by-step transcription of the
 * method's definition (Sec. 3.2, Eq. 3-7, and the data flow of Algorithm 1),
 * with every intermediate tensor the paper names materialised, including the
 * gathered key/value tensors of Eq. 6.  No blocking, fusion or reordering.
 * It shares no code with the HIP library and must never be called by it.
 *
 * Conventions where the paper is silent (all listed in the design notes):
 *   - softmax scale is an argument (default chosen by the caller: 1/sqrt(C/heads),
 *     Eq. 1 applied to the per-head operands of Eq. 2);
 *   - routing (Eq. 4-5) uses all C channels and is shared by the heads;
 *   - top-k rows are ordered by descending affinity, ties to the smaller index;
 *   - LCE (Eq. 7) is a 5x5 depth-wise cross-correlation of V on the H x W map,
 *     stride 1, zero padding 2, no bias;
 *   - Y = (Attention + LCE(V)) W^o  (Eq. 7 followed by the W^o of Eq. 2), no bias.
 */

#define CAT_(a, b) a##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUFFIX)

/* Region partition (Sec. 3.2 "Region partition and input projection"; first step of
 * Algorithm 1): (H, W, C) -> (S^2, HW/S^2, C); token (y, x) goes to region
 * (y / rh) * S + (x / rw), slot (y % rh) * rw + (x % rw). */
static void FN(patchify_)(const REAL *in, REAL *out, int H, int W, int C, int S)
{
    int rh = H / S, rw = W / S, n = rh * rw;
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            int r = (y / rh) * S + (x / rw);
            int s = (y % rh) * rw + (x % rw);
            memcpy(out + ((size_t)r * n + s) * C, in + ((size_t)y * W + x) * C, sizeof(REAL) * C);
        }
}

/* Inverse of patchify (last step of Algorithm 1). */
static void FN(unpatchify_)(const REAL *in, REAL *out, int H, int W, int C, int S)
{
    int rh = H / S, rw = W / S, n = rh * rw;
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            int r = (y / rh) * S + (x / rw);
            int s = (y % rh) * rw + (x % rw);
            memcpy(out + ((size_t)y * W + x) * C, in + ((size_t)r * n + s) * C, sizeof(REAL) * C);
        }
}

/* out[M, N] = a[M, K] * b[K, N], row-major; returns the number of multiply-adds. */
static int64_t FN(matmul_)(const REAL *a, const REAL *b, REAL *out, int M, int K, int N)
{
    for (int i = 0; i < M; ++i)
        for (int j = 0; j < N; ++j) {
            REAL acc = 0;
            for (int c = 0; c < K; ++c)
                acc += a[(size_t)i * K + c] * b[(size_t)c * N + j];
            out[(size_t)i * N + j] = acc;
        }
    return (int64_t)M * K * N;
}

/* Row-wise top-k index (Eq. 5): k largest entries of each row of A[R, R], in
 * descending order; equal values are taken in ascending index order. */
static void FN(topk_index_)(const REAL *A, int32_t *I, int R, int k)
{
    char *taken = (char *)malloc((size_t)R);
    for (int i = 0; i < R; ++i) {
        memset(taken, 0, (size_t)R);
        for (int p = 0; p < k; ++p) {
            int best = -1;
            for (int j = 0; j < R; ++j) {
                if (taken[j]) continue;
                if (best < 0 || A[(size_t)i * R + j] > A[(size_t)i * R + best]) best = j;
            }
            taken[best] = 1;
            I[(size_t)i * k + p] = best;
        }
    }
    free(taken);
}

/* One image.  Pointers marked opt may be NULL. */
static void FN(bra_image_)(int H, int W, int C, int heads, int S, int k, REAL scale,
                           const REAL *X, const REAL *Wqkv, const REAL *Wo, const REAL *Wlce,
                           const int32_t *Ir_in /*opt [R,k]*/, REAL *Y,
                           int32_t *Ir_out /*opt [R,k]*/, REAL *Ar_out /*opt [R,R]*/,
                           REAL *P_out /*opt [heads,R,n,kn]*/, REAL *Oatt_out /*opt [H,W,C]*/,
                           REAL *Lce_out /*opt [H,W,C]*/, int64_t *macs /*[3]*/)
{
    const int rh = H / S, rw = W / S, n = rh * rw, R = S * S, N = H * W, d = C / heads;
    const int kn = k * n;
    const size_t NC = (size_t)N * C;

    REAL *xr = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *qkv = (REAL *)malloc(sizeof(REAL) * NC * 3);
    REAL *q = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *kk = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *v = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *q_r = (REAL *)malloc(sizeof(REAL) * (size_t)R * C);
    REAL *k_r = (REAL *)malloc(sizeof(REAL) * (size_t)R * C);
    REAL *k_rT = (REAL *)malloc(sizeof(REAL) * (size_t)R * C);
    REAL *A_r = (REAL *)malloc(sizeof(REAL) * (size_t)R * R);
    int32_t *I_r = (int32_t *)malloc(sizeof(int32_t) * (size_t)R * k);
    REAL *k_g = (REAL *)malloc(sizeof(REAL) * (size_t)R * kn * C);
    REAL *v_g = (REAL *)malloc(sizeof(REAL) * (size_t)R * kn * C);
    REAL *att = (REAL *)malloc(sizeof(REAL) * (size_t)kn);
    REAL *out_r = (REAL *)malloc(sizeof(REAL) * NC);   /* region layout */
    REAL *v_map = (REAL *)malloc(sizeof(REAL) * NC);   /* V on the H x W map */
    REAL *lce_map = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *lce_r = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *o_map = (REAL *)malloc(sizeof(REAL) * NC);

    /* patchify, then the fused linear projection and its split into q, k, v
     * (Eq. 3; W^q, W^k, W^v are the three column blocks of Wqkv). */
    FN(patchify_)(X, xr, H, W, C, S);
    macs[0] += FN(matmul_)(xr, Wqkv, qkv, N, C, 3 * C);
    for (int t = 0; t < N; ++t)
        for (int c = 0; c < C; ++c) {
            q[(size_t)t * C + c] = qkv[(size_t)t * 3 * C + c];
            kk[(size_t)t * C + c] = qkv[(size_t)t * 3 * C + C + c];
            v[(size_t)t * C + c] = qkv[(size_t)t * 3 * C + 2 * C + c];
        }

    /* region-level queries and keys: per-region average over the n tokens. */
    for (int r = 0; r < R; ++r)
        for (int c = 0; c < C; ++c) {
            REAL sq = 0, sk = 0;
            for (int s = 0; s < n; ++s) {
                sq += q[((size_t)r * n + s) * C + c];
                sk += kk[((size_t)r * n + s) * C + c];
            }
            q_r[(size_t)r * C + c] = sq / (REAL)n;
            k_r[(size_t)r * C + c] = sk / (REAL)n;
        }

    /* region affinity graph A^r = Q^r (K^r)^T (Eq. 4). */
    for (int r = 0; r < R; ++r)
        for (int c = 0; c < C; ++c)
            k_rT[(size_t)c * R + r] = k_r[(size_t)r * C + c];
    macs[1] += FN(matmul_)(q_r, k_rT, A_r, R, C, R);
    if (Ar_out) memcpy(Ar_out, A_r, sizeof(REAL) * (size_t)R * R);

    /* routing index (Eq. 5), or the caller's forced routing. */
    if (Ir_in)
        memcpy(I_r, Ir_in, sizeof(int32_t) * (size_t)R * k);
    else
        FN(topk_index_)(A_r, I_r, R, k);
    if (Ir_out) memcpy(Ir_out, I_r, sizeof(int32_t) * (size_t)R * k);

    /* gather the key/value tokens of the routed regions (Eq. 6):
     * K^g[i] = concat_p K[I^r[i, p]]  ->  (S^2, k n, C). */
    for (int i = 0; i < R; ++i)
        for (int p = 0; p < k; ++p) {
            int j = I_r[(size_t)i * k + p];
            memcpy(k_g + ((size_t)i * kn + (size_t)p * n) * C, kk + (size_t)j * n * C,
                   sizeof(REAL) * (size_t)n * C);
            memcpy(v_g + ((size_t)i * kn + (size_t)p * n) * C, v + (size_t)j * n * C,
                   sizeof(REAL) * (size_t)n * C);
        }

    /* token-to-token attention (Eq. 7 with Eq. 1 per head, heads = channel chunks
     * of width d as in Eq. 2): one softmax over all k n gathered keys. */
    for (int i = 0; i < R; ++i)
        for (int hd = 0; hd < heads; ++hd)
            for (int s = 0; s < n; ++s) {
                const REAL *qv = q + ((size_t)i * n + s) * C + (size_t)hd * d;
                REAL mx = 0;
                for (int u = 0; u < kn; ++u) {
                    const REAL *kv = k_g + ((size_t)i * kn + u) * C + (size_t)hd * d;
                    REAL acc = 0;
                    for (int c = 0; c < d; ++c) acc += qv[c] * kv[c];
                    att[u] = acc * scale;
                    if (u == 0 || att[u] > mx) mx = att[u];
                }
                macs[2] += (int64_t)kn * d;
                REAL den = 0;
                for (int u = 0; u < kn; ++u) {
                    att[u] = (REAL)exp((double)(att[u] - mx));
                    den += att[u];
                }
                for (int u = 0; u < kn; ++u) att[u] /= den;
                if (P_out)
                    memcpy(P_out + (((size_t)hd * R + i) * n + s) * kn, att, sizeof(REAL) * kn);
                REAL *ov = out_r + ((size_t)i * n + s) * C + (size_t)hd * d;
                for (int c = 0; c < d; ++c) {
                    REAL acc = 0;
                    for (int u = 0; u < kn; ++u)
                        acc += att[u] * v_g[((size_t)i * kn + u) * C + (size_t)hd * d + c];
                    ov[c] = acc;
                }
                macs[2] += (int64_t)kn * d;
            }
    if (Oatt_out) FN(unpatchify_)(out_r, Oatt_out, H, W, C, S);

    /* local context enhancement: 5x5 depth-wise convolution of V on the image. */
    FN(unpatchify_)(v, v_map, H, W, C, S);
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
            for (int c = 0; c < C; ++c) {
                REAL acc = 0;
                for (int ky = 0; ky < 5; ++ky)
                    for (int kx = 0; kx < 5; ++kx) {
                        int yy = y + ky - 2, xx = x + kx - 2;
                        if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                        acc += Wlce[((size_t)c * 5 + ky) * 5 + kx] *
                               v_map[((size_t)yy * W + xx) * C + c];
                    }
                lce_map[((size_t)y * W + x) * C + c] = acc;
            }
    if (Lce_out) memcpy(Lce_out, lce_map, sizeof(REAL) * NC);

    /* output = attention + dwconv(value), in region layout, then back to (H, W, C). */
    FN(patchify_)(lce_map, lce_r, H, W, C, S);
    for (size_t e = 0; e < NC; ++e) out_r[e] += lce_r[e];
    FN(unpatchify_)(out_r, o_map, H, W, C, S);

    /* output projection W^o composing the heads (Eq. 2). */
    FN(matmul_)(o_map, Wo, Y, N, C, C);

    free(xr); free(qkv); free(q); free(kk); free(v); free(q_r); free(k_r); free(k_rT);
    free(A_r); free(I_r); free(k_g); free(v_g); free(att); free(out_r); free(v_map);
    free(lce_map); free(lce_r); free(o_map);
}

/* Batched entry: images are independent (routing is per image).  `threads` > 1
 * spreads images over OpenMP threads (used for timing only).  Returns 0, or -1 on
 * an invalid shape.  macs (opt, [3]) receives the multiply-add counts of the
 * projection, region-routing and token-attention parts summed over the batch. */
int FN(oracle_bra_forward_)(int B, int H, int W, int C, int heads, int S, int k, double scale,
                            const REAL *X, const REAL *Wqkv, const REAL *Wo, const REAL *Wlce,
                            const int32_t *Ir_in, REAL *Y, int32_t *Ir_out, REAL *Ar_out,
                            REAL *P_out, REAL *Oatt_out, REAL *Lce_out, int64_t *macs,
                            int threads)
{
    if (B < 1 || H < 1 || W < 1 || C < 1 || heads < 1 || S < 1 || k < 1) return -1;
    if (H % S || W % S || C % heads || k > S * S) return -1;
    const int R = S * S, n = (H / S) * (W / S), N = H * W;
    const size_t NC = (size_t)N * C;
    int64_t m0 = 0, m1 = 0, m2 = 0;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(dynamic, 1) reduction(+ : m0, m1, m2)
    for (int b = 0; b < B; ++b) {
        int64_t m[3] = {0, 0, 0};
        FN(bra_image_)(H, W, C, heads, S, k, (REAL)scale, X + b * NC, Wqkv, Wo, Wlce,
                       Ir_in ? Ir_in + (size_t)b * R * k : NULL, Y + b * NC,
                       Ir_out ? Ir_out + (size_t)b * R * k : NULL,
                       Ar_out ? Ar_out + (size_t)b * R * R : NULL,
                       P_out ? P_out + (size_t)b * heads * R * n * k * n : NULL,
                       Oatt_out ? Oatt_out + b * NC : NULL, Lce_out ? Lce_out + b * NC : NULL, m);
        m0 += m[0]; m1 += m[1]; m2 += m[2];
    }
    if (macs) { macs[0] = m0; macs[1] = m1; macs[2] = m2; }
    return 0;
}

#undef FN
#undef CAT
#undef CAT_
