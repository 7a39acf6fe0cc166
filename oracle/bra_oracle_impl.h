/*
 * TEST INFRASTRUCTURE -- CPU oracle for the forward pass of Bi-Level Routing
 * Attention (BRA), "BiFormer: Vision Transformer with Bi-Level Routing Attention".
 *
 * This file is included twice by bra_oracle.c, once with REAL = float and once
 * with REAL = double.  It writes out the DEFINITION of the layer (Sec. 3.2, Eq. 3-7,
 * with the per-head attention and W^o of Eq. 1-2) token by token on the H x W map:
 * nothing is re-laid-out, blocked, fused or reordered, and no tensor other than the
 * ones the equations name (Q, K, V, Q^r, K^r, A^r, I^r, the output) is formed.  The
 * gathered key/value set of Eq. 6 appears as what it is, a set of tokens: for a query
 * of region i, the tokens of the regions listed in row i of I^r.
 * It shares no code with the HIP library and must never be called by it.
 *
 * Notation: token t = (y, x) of the map; rh = H / S, rw = W / S; region(t) =
 * (y / rh) S + x / rw (Sec. 3.2, "Region partition and input projection");
 * n = rh rw tokens per region; R = S^2 regions; head h owns channels [h d, (h+1) d).
 *
 * Conventions where the paper is silent (all listed in the design notes):
 *   - softmax scale is an argument (default chosen by the caller: 1/sqrt(C/heads),
 *     Eq. 1 applied to the per-head operands of Eq. 2);
 *   - routing (Eq. 4-5) uses all C channels and is shared by the heads;
 *   - row i of I^r lists regions by descending affinity, equal values by ascending index;
 *   - LCE (Eq. 7) is a 5x5 depth-wise cross-correlation of V on the H x W map,
 *     stride 1, zero padding 2, no bias;
 *   - Y = (Attention + LCE(V)) W^o  (Eq. 7 followed by the W^o of Eq. 2), no bias.
 */

#define CAT_(a, b) a##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUFFIX)

/* Eq. 3 for one of the three projections: out[t, o] = sum_c X[t, c] W[c, col0 + o], where W is
 * the [C, ldw] matrix that holds the projection's weights in columns col0 .. col0 + C - 1. */
static void FN(project_)(const REAL *X, const REAL *Wmat, int ldw, int col0, REAL *out, int N, int C)
{
    for (int t = 0; t < N; ++t)
        for (int o = 0; o < C; ++o) {
            REAL acc = 0;
            for (int c = 0; c < C; ++c) acc += X[(size_t)t * C + c] * Wmat[(size_t)c * ldw + col0 + o];
            out[(size_t)t * C + o] = acc;
        }
}

/* Region-level queries / keys (Sec. 3.2, "Region-to-region routing"): mean[r, c] = average of
 * T[t, c] over the tokens t of region r. */
static void FN(region_mean_)(const REAL *T, REAL *mean, int H, int W, int C, int S)
{
    const int rh = H / S, rw = W / S, R = S * S;
    for (int r = 0; r < R; ++r)
        for (int c = 0; c < C; ++c) {
            REAL sum = 0;       /* region r covers rows (r / S) rh .., columns (r % S) rw .. */
            for (int y = (r / S) * rh; y < (r / S + 1) * rh; ++y)
                for (int x = (r % S) * rw; x < (r % S + 1) * rw; ++x) sum += T[((size_t)y * W + x) * C + c];
            mean[(size_t)r * C + c] = sum / (REAL)(rh * rw);
        }
}

/* Eq. 5: row i of I^r holds the indices of the k largest entries of row i of A^r.  Written as a
 * ranking: entry j stands at position (number of entries that come before it), where j' comes
 * before j if it is larger, or equal with a smaller index. */
static void FN(routing_index_)(const REAL *A, int32_t *I, int R, int k)
{
    for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) {
            int before = 0;
            for (int jj = 0; jj < R; ++jj) {
                const REAL a = A[(size_t)i * R + jj], b = A[(size_t)i * R + j];
                if (a > b || (a == b && jj < j)) ++before;
            }
            if (before < k) I[(size_t)i * k + before] = j;
        }
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

    REAL *Q = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *K = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *V = (REAL *)malloc(sizeof(REAL) * NC);
    REAL *Qr = (REAL *)malloc(sizeof(REAL) * (size_t)R * C);
    REAL *Kr = (REAL *)malloc(sizeof(REAL) * (size_t)R * C);
    REAL *Ar = (REAL *)malloc(sizeof(REAL) * (size_t)R * R);
    int32_t *Ir = (int32_t *)malloc(sizeof(int32_t) * (size_t)R * k);
    int *keys = (int *)malloc(sizeof(int) * (size_t)kn);     /* the tokens a query attends to */
    REAL *w = (REAL *)malloc(sizeof(REAL) * (size_t)kn);      /* their softmax weights */
    REAL *O = (REAL *)malloc(sizeof(REAL) * NC);              /* Attention(..) + LCE(V) of Eq. 7 */

    /* Eq. 3: Q = X W^q, K = X W^k, V = X W^v; the three weights are the column blocks of Wqkv. */
    FN(project_)(X, Wqkv, 3 * C, 0, Q, N, C);
    FN(project_)(X, Wqkv, 3 * C, C, K, N, C);
    FN(project_)(X, Wqkv, 3 * C, 2 * C, V, N, C);
    macs[0] += (int64_t)3 * N * C * C;

    /* Q^r, K^r: per-region averages; Eq. 4: A^r = Q^r (K^r)^T. */
    FN(region_mean_)(Q, Qr, H, W, C, S);
    FN(region_mean_)(K, Kr, H, W, C, S);
    for (int i = 0; i < R; ++i)
        for (int j = 0; j < R; ++j) {
            REAL acc = 0;
            for (int c = 0; c < C; ++c) acc += Qr[(size_t)i * C + c] * Kr[(size_t)j * C + c];
            Ar[(size_t)i * R + j] = acc;
        }
    macs[1] += (int64_t)R * R * C;
    if (Ar_out) memcpy(Ar_out, Ar, sizeof(REAL) * (size_t)R * R);

    /* Eq. 5, or the caller's forced routing. */
    if (Ir_in)
        memcpy(Ir, Ir_in, sizeof(int32_t) * (size_t)R * k);
    else
        FN(routing_index_)(Ar, Ir, R, k);
    if (Ir_out) memcpy(Ir_out, Ir, sizeof(int32_t) * (size_t)R * k);

    /* Eq. 6-7 with Eq. 1 per head (Eq. 2): the query token (y, x) of region i attends to every
     * token of the regions I^r[i, 0..k): one softmax over that whole set, then the weighted sum
     * of their values.  The set is listed region by region in the order of row i, tokens of a
     * region in row-major order (the order only fixes where a weight lands in P_out). */
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x) {
            const int t = y * W + x;
            const int i = (y / rh) * S + x / rw;
            int cnt = 0;
            for (int p = 0; p < k; ++p) {
                const int j = Ir[(size_t)i * k + p], jy = j / S, jx = j % S;
                for (int sy = 0; sy < rh; ++sy)
                    for (int sx = 0; sx < rw; ++sx) keys[cnt++] = (jy * rh + sy) * W + jx * rw + sx;
            }
            for (int hd = 0; hd < heads; ++hd) {
                const REAL *q = Q + (size_t)t * C + (size_t)hd * d;
                REAL top = 0;
                for (int u = 0; u < kn; ++u) {
                    const REAL *kv = K + (size_t)keys[u] * C + (size_t)hd * d;
                    REAL dot = 0;
                    for (int c = 0; c < d; ++c) dot += q[c] * kv[c];
                    w[u] = dot * scale;
                    if (u == 0 || w[u] > top) top = w[u];
                }
                REAL den = 0;
                for (int u = 0; u < kn; ++u) {
                    w[u] = (REAL)exp((double)(w[u] - top));
                    den += w[u];
                }
                for (int u = 0; u < kn; ++u) w[u] /= den;
                if (P_out) {
                    const int slot = (y % rh) * rw + x % rw;
                    memcpy(P_out + (((size_t)hd * R + i) * n + slot) * kn, w, sizeof(REAL) * kn);
                }
                for (int c = 0; c < d; ++c) {
                    REAL acc = 0;
                    for (int u = 0; u < kn; ++u) acc += w[u] * V[(size_t)keys[u] * C + (size_t)hd * d + c];
                    O[(size_t)t * C + (size_t)hd * d + c] = acc;
                }
                macs[2] += (int64_t)2 * kn * d;
            }
        }
    if (Oatt_out) memcpy(Oatt_out, O, sizeof(REAL) * NC);

    /* LCE(V) of Eq. 7: 5x5 depth-wise correlation of V over the map, zero outside it. */
    for (int y = 0; y < H; ++y)
        for (int x = 0; x < W; ++x)
            for (int c = 0; c < C; ++c) {
                REAL acc = 0;
                for (int ky = 0; ky < 5; ++ky)
                    for (int kx = 0; kx < 5; ++kx) {
                        const int yy = y + ky - 2, xx = x + kx - 2;
                        if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                        acc += Wlce[((size_t)c * 5 + ky) * 5 + kx] * V[((size_t)yy * W + xx) * C + c];
                    }
                if (Lce_out) Lce_out[((size_t)y * W + x) * C + c] = acc;
                O[((size_t)y * W + x) * C + c] += acc;
            }

    /* Eq. 2: the heads' outputs side by side, times W^o. */
    FN(project_)(O, Wo, C, 0, Y, N, C);

    free(Q); free(K); free(V); free(Qr); free(Kr); free(Ar); free(Ir); free(keys); free(w); free(O);
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
