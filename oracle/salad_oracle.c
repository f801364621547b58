/*
 * CPU oracle for the SALAD attention-layer forward (sparse softmax attention in parallel
 * with ReLU linear attention, combined by static and dynamic scaling).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path, and
 * nothing in the product may call it: only the tests, the smoke check and the benchmark's
 * CPU-baseline leg do.
 *
 * Everything is evaluated in double precision on float32 input arrays (for bf16 workloads
 * the arrays already hold bf16-representable values).  Each function writes the paper's
 * definition out directly: two-pass softmax over exactly the kept keys, sums over all
 * tokens for the linear state, no tiling, no online rescaling, no fusion.  OpenMP only
 * distributes independent output rows over cores; it does not reorder any sum.
 *
 * Passages followed
 *   sparse attention          Sec. 3 "Sparse Attention", Eq. (2); masked positions are excluded
 *   token orders / ST-SWA     App. A.1.1 (default order: time slowest; temporal heads: tokens
 *                             grouped by spatial location so that frames are consecutive)
 *   ReLU linear attention     Sec. 3 "Linear Attention", Eq. (3)
 *   static and dynamic scale  Alg. 1 (Level 1 / Level 2 / residual integration), Sec. 4.2
 *   branch dropping           Sec. 4.3, App. A.3 (the linear branch of a sample is pruned when its
 *                             dynamic scale lies below the threshold)
 *   Top-K block-sparse mask   Sec. 3 "Top-K attention", App. A.1.2 (block means of the keys, query-to-mean
 *                             similarity, the k best blocks per query token, attention on their tokens)
 *
 * Readings where the paper is silent (all listed in the design notes of the repository):
 *   - the sliding window keeps a constant count of `kept` consecutive KV blocks per query
 *     block, centred (extra block on the left for even counts) and shifted inward at the ends;
 *   - sparsity rho maps to kept = clamp(floor((1-rho)*nb + 0.5), 1, nb);
 *   - the linear-attention denominator is (phi(Q_i).Z + eps);
 *   - the static projection is the per-layer scalar lambda times a per-head scalar a_h;
 *   - the gate is Linear: D -> 1 without learned bias (a test-only scalar bias is accepted),
 *     sigmoid per token, then the mean over tokens;
 *   - with a full static projection W_p [D x D] (D = H d; row = input channel h_in d + a, column = output
 *     channel h_out d + c) the residual sum is O_s + lambda s_b (O_l W_p), O_l being the heads' linear
 *     outputs concatenated per token; the per-head form is W_p = blockdiag(a_h I);
 *   - Top-K: key blocks are runs of key_block consecutive tokens of the stored order, the similarity is the
 *     plain dot product q.mean(K_block), every query token selects for itself, ties go to the lower block
 *     index, no block is forced in; the selection is computed in float32 in a fixed order (see there);
 *   - RoPE in the linear branch: rotation of phi(Q), phi(K) in the numerator only, angles supplied as tables,
 *     channel pairs (2p, 2p+1) (see salad_oracle_linear_state_rope);
 *   - "below the threshold" is the strict inequality s_b < tau; a dropped branch contributes
 *     exactly nothing (out = O_s), and tau <= 0 never drops since s_b > 0.
 *
 * Parity pins (tests/test_oracle_*.py): dense attention from a library routine, uniform
 * weights for Q = 0, the quadratic form (phi(Q)phi(K)^T)V, closed forms for the gate and the
 * combination, and structural invariants plus the stated densities for the mask.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SO_OK 0
#define SO_EINVAL 1

/* ---- token order (App. A.1.1) ------------------------------------------------------ */

/* Row index in the stored [N, d] layout (time slowest: n = t*Hh*W + y*W + x) of the token that
 * sits at position p of a head's own order.  kind 0: default order, p = n.  kind 1: tokens
 * grouped by spatial location, frames consecutive: p = (y*W + x)*T + t. */
static int64_t row_of_position(int kind, int64_t p, int T, int64_t HW)
{
    if (kind == 0) return p;
    int64_t loc = p / T;
    int64_t t = p % T;
    return t * HW + loc;
}

int64_t salad_oracle_row_of_position(int kind, int64_t p, int T, int Hh, int W)
{
    return row_of_position(kind, p, T, (int64_t)Hh * W);
}

int salad_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- block mask (Sec. 3 sliding-window attention, App. A.1.1) ----------------------- */

/* Number of KV blocks each query block keeps at sparsity rho ("proportion of computations
 * reduced", Sec. 5.1), counted in block pairs. */
int32_t salad_oracle_kept_from_sparsity(int32_t nb, double sparsity)
{
    double k = floor((1.0 - sparsity) * (double)nb + 0.5);
    if (k < 1.0) k = 1.0;
    if (k > (double)nb) k = (double)nb;
    return (int32_t)k;
}

/* CSR of kept KV blocks.  Row h*nb + i lists, ascending, the kept blocks of query block i of
 * head h; blocks are runs of `block` consecutive positions of that head's token order.
 * row_ptr has H*nb + 1 entries; col_idx needs sum_h nb*kept[h] entries.  Returns nnz, or -1. */
int64_t salad_oracle_block_mask(int T, int Hh, int W, int block, int H,
                                const int32_t *kept, int32_t *row_ptr, int32_t *col_idx)
{
    int64_t N = (int64_t)T * Hh * W;
    if (N <= 0 || block <= 0 || H <= 0) return -1;
    int64_t nb = (N + block - 1) / block;
    int64_t nnz = 0;
    for (int h = 0; h < H; ++h) {
        int64_t k = kept[h];
        if (k < 1 || k > nb) return -1;
        for (int64_t i = 0; i < nb; ++i) {
            int64_t start = i - k / 2;
            if (start < 0) start = 0;
            if (start > nb - k) start = nb - k;
            row_ptr[h * nb + i] = (int32_t)nnz;
            for (int64_t j = start; j < start + k; ++j) col_idx[nnz++] = (int32_t)j;
        }
    }
    row_ptr[(int64_t)H * nb] = (int32_t)nnz;
    return nnz;
}

/* The same sliding window without the inward shift at the sequence ends: query block i of head h keeps
 * the blocks of [i - kept/2, i - kept/2 + kept) that exist, so rows near either end are shorter.  The paper gives
 * no formula for the window (Sec. 3 "Sliding-window attention", App. A.1.1); this is the second plain reading next
 * to the constant-count one above.  col_idx needs at most sum_h nb*kept[h] entries.  Returns nnz, or -1. */
int64_t salad_oracle_block_mask_truncated(int T, int Hh, int W, int block, int H,
                                          const int32_t *kept, int32_t *row_ptr, int32_t *col_idx)
{
    int64_t N = (int64_t)T * Hh * W;
    if (N <= 0 || block <= 0 || H <= 0) return -1;
    int64_t nb = (N + block - 1) / block;
    int64_t nnz = 0;
    for (int h = 0; h < H; ++h) {
        int64_t k = kept[h];
        if (k < 1 || k > nb) return -1;
        for (int64_t i = 0; i < nb; ++i) {
            row_ptr[h * nb + i] = (int32_t)nnz;
            for (int64_t j = i - k / 2; j < i - k / 2 + k; ++j)
                if (j >= 0 && j < nb) col_idx[nnz++] = (int32_t)j;
        }
    }
    row_ptr[(int64_t)H * nb] = (int32_t)nnz;
    return nnz;
}

/* ---- sparse attention, Eq. (2) ------------------------------------------------------ */

/* For the selected query blocks sel[0..nsel) of every (b, h): softmax over exactly the keys of
 * the kept KV blocks (positions >= N do not exist), logits q.k*scale, two passes.
 * q, k, v: float32 [B, H, N, d].  Output compact: out[((b*H + h)*nsel + s)*block + r][d]
 * holds the row for position sel[s]*block + r of head h's order; rows_out (same leading shape)
 * gets that token's stored row index n, or -1 when the position is >= N (output left zero). */
int salad_oracle_sparse_attn(const float *q, const float *k, const float *v,
                             int B, int H, int64_t N, int d,
                             int T, int Hh, int W, int block,
                             const uint8_t *head_kind,
                             const int32_t *row_ptr, const int32_t *col_idx,
                             double scale,
                             const int32_t *sel, int nsel,
                             double *out, int64_t *rows_out)
{
    if ((int64_t)T * Hh * W != N || block <= 0 || d <= 0) return SO_EINVAL;
    const int64_t HW = (int64_t)Hh * W;
    const int64_t nb = (N + block - 1) / block;
    const int64_t total = (int64_t)B * H * nsel * block;
    int bad = 0;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)(nb * block));
        int64_t *krow = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nb * block));
#pragma omp for schedule(dynamic, 16)
        for (int64_t idx = 0; idx < total; ++idx) {
            int r = (int)(idx % block);
            int64_t rest = idx / block;
            int s = (int)(rest % nsel);
            int64_t bh = rest / nsel;
            int h = (int)(bh % H);
            int64_t i = sel[s];
            double *o = out + idx * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            int64_t p = i * block + r;
            if (i < 0 || i >= nb) {
#pragma omp atomic write
                bad = 1;
                rows_out[idx] = -1;
                continue;
            }
            if (p >= N) { rows_out[idx] = -1; continue; }
            int kind = head_kind[h];
            int64_t n = row_of_position(kind, p, T, HW);
            rows_out[idx] = n;
            const float *qi = q + (bh * N + n) * d;
            /* pass 1: logits over the kept set */
            int64_t cnt = 0;
            double m = -INFINITY;
            for (int32_t e = row_ptr[h * nb + i]; e < row_ptr[h * nb + i + 1]; ++e) {
                int64_t j = col_idx[e];
                for (int c = 0; c < block; ++c) {
                    int64_t pk = j * block + c;
                    if (pk >= N) break;
                    int64_t nk = row_of_position(kind, pk, T, HW);
                    const float *kj = k + (bh * N + nk) * d;
                    double acc = 0.0;
                    for (int x = 0; x < d; ++x) acc += (double)qi[x] * (double)kj[x];
                    acc *= scale;
                    logit[cnt] = acc;
                    krow[cnt] = nk;
                    if (acc > m) m = acc;
                    ++cnt;
                }
            }
            if (cnt == 0) continue; /* empty row: defined as zero */
            /* pass 2: weights and weighted sum of V */
            double denom = 0.0;
            for (int64_t t = 0; t < cnt; ++t) { logit[t] = exp(logit[t] - m); denom += logit[t]; }
            for (int64_t t = 0; t < cnt; ++t) {
                const float *vj = v + (bh * N + krow[t]) * d;
                double wgt = logit[t] / denom;
                for (int c = 0; c < d; ++c) o[c] += wgt * (double)vj[c];
            }
        }
        free(logit);
        free(krow);
    }
    return bad ? SO_EINVAL : SO_OK;
}

/* ---- Top-K block-sparse attention, Sec. 3 "Top-K attention", App. A.1.2 ---------------- */

/* Steps 1 and 2 of App. A.1.2: the keys are cut into blocks of key_block consecutive tokens of the head's own
 * token order (App. A.1.1: the stored order for a spatial head, tokens grouped by location for a temporal one;
 * head_kind == NULL: every head spatial), each block is reduced to the mean of its keys, and every query token
 * keeps the topk blocks whose mean has the largest dot product with the query.  mask[(b*H + h)*N + n] (n = the
 * query's stored row) has bit J set when query n keeps block J (nbk = ceil(N / key_block) <= 64 blocks;
 * topk >= nbk keeps all of them).  Block J holds positions J key_block .. (J+1) key_block - 1 of the order.
 *
 * Here floating point decides an integer, so the decision is taken in the arithmetic the device uses for it,
 * written out step by step: float32 throughout; a block's sum is accumulated token by token in ascending order
 * and divided by the token count; a score is accumulated channel by channel in ascending order with a fused
 * multiply-add; a block replaces a kept one only on a strictly larger score, so ties go to the lower index.
 * (tests pin the outcome to the float64 definition wherever the float64 scores leave a clear margin). */
int salad_oracle_topk_select(const float *q, const float *k, int B, int H, int64_t N, int d,
                             int key_block, int topk, const uint8_t *head_kind, int T, int Hh, int W, uint64_t *mask)
{
    if (key_block <= 0 || topk <= 0 || N <= 0 || d <= 0) return SO_EINVAL;
    if (head_kind && (T < 1 || Hh < 1 || W < 1 || (int64_t)T * Hh * W != N)) return SO_EINVAL;
    const int64_t HW = (int64_t)Hh * W;
    const int64_t nbk = (N + key_block - 1) / key_block;
    if (nbk > 64) return SO_EINVAL;
    const int kk = topk < nbk ? topk : (int)nbk;
    const int64_t BH = (int64_t)B * H;
    float *mean = (float *)malloc(sizeof(float) * (size_t)(BH * nbk * d));
    if (!mean) return SO_EINVAL;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < BH * nbk; ++e) {
        const int64_t bh = e / nbk, J = e % nbk;
        const int kind = head_kind ? (int)head_kind[bh % H] : 0;
        const int64_t t0 = J * key_block, t1 = (t0 + key_block < N) ? t0 + key_block : N;
        for (int c = 0; c < d; ++c) {
            volatile float sum = 0.0f;           /* volatile: one rounding per addition, in this order (ascending position) */
            for (int64_t t = t0; t < t1; ++t) sum = sum + k[(bh * N + row_of_position(kind, t, T, HW)) * d + c];
            mean[e * d + c] = sum / (float)(t1 - t0);
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < BH * N; ++e) {
        const int64_t bh = e / N;
        const float *qi = q + e * d;
        float best[64];
        int bidx[64];
        int cnt = 0;
        for (int64_t J = 0; J < nbk; ++J) {
            const float *mj = mean + (bh * nbk + J) * d;
            float sc = 0.0f;
            for (int c = 0; c < d; ++c) sc = fmaf(qi[c], mj[c], sc);
            /* insert into the descending list of the best kk so far; equal scores stay behind earlier blocks */
            int pos = cnt;
            while (pos > 0 && sc > best[pos - 1]) --pos;
            if (pos >= kk) continue;
            const int last = cnt < kk ? cnt : kk - 1;
            for (int i = last; i > pos; --i) { best[i] = best[i - 1]; bidx[i] = bidx[i - 1]; }
            best[pos] = sc;
            bidx[pos] = (int)J;
            if (cnt < kk) ++cnt;
        }
        uint64_t m = 0;
        for (int i = 0; i < cnt; ++i) m |= (uint64_t)1 << bidx[i];
        mask[e] = m;
    }
    free(mean);
    return SO_OK;
}

/* Step 3 of App. A.1.2: every query token attends to the tokens of the key blocks it kept, Eq. (2) with that
 * token-level mask: two-pass softmax in double precision over exactly those keys, logits q.k*scale.
 * rows [B, H, nrows]: stored rows to evaluate (< 0: skipped, output left zero); out [B, H, nrows, d]. */
int salad_oracle_topk_attn(const float *q, const float *k, const float *v, int B, int H, int64_t N, int d,
                           int key_block, const uint64_t *mask, double scale, const uint8_t *head_kind, int T, int Hh, int W,
                           const int64_t *rows, int64_t nrows, double *out)
{
    if (key_block <= 0 || N <= 0 || d <= 0) return SO_EINVAL;
    if (head_kind && (T < 1 || Hh < 1 || W < 1 || (int64_t)T * Hh * W != N)) return SO_EINVAL;
    const int64_t HW = (int64_t)Hh * W;
    const int64_t nbk = (N + key_block - 1) / key_block;
    if (nbk > 64) return SO_EINVAL;
    const int64_t total = (int64_t)B * H * nrows;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)N);
        int64_t *krow = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);
#pragma omp for schedule(dynamic, 16)
        for (int64_t idx = 0; idx < total; ++idx) {
            const int64_t bh = idx / nrows;
            const int64_t n = rows[idx];
            double *o = out + idx * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (n < 0 || n >= N) continue;
            const float *qi = q + (bh * N + n) * d;
            const uint64_t m = mask[bh * N + n];
            const int kind = head_kind ? (int)head_kind[bh % H] : 0;
            int64_t cnt = 0;
            double mx = -INFINITY;
            for (int64_t J = 0; J < nbk; ++J) {
                if (!((m >> J) & 1)) continue;
                const int64_t t1 = ((J + 1) * key_block < N) ? (J + 1) * key_block : N;
                for (int64_t p = J * key_block; p < t1; ++p) {       /* positions of block J in the head's order */
                    const int64_t t = row_of_position(kind, p, T, HW);
                    const float *kj = k + (bh * N + t) * d;
                    double acc = 0.0;
                    for (int x = 0; x < d; ++x) acc += (double)qi[x] * (double)kj[x];
                    acc *= scale;
                    logit[cnt] = acc;
                    krow[cnt] = t;
                    if (acc > mx) mx = acc;
                    ++cnt;
                }
            }
            if (cnt == 0) continue;
            double denom = 0.0;
            for (int64_t t = 0; t < cnt; ++t) { logit[t] = exp(logit[t] - mx); denom += logit[t]; }
            for (int64_t t = 0; t < cnt; ++t) {
                const float *vj = v + (bh * N + krow[t]) * d;
                const double wgt = logit[t] / denom;
                for (int c = 0; c < d; ++c) o[c] += wgt * (double)vj[c];
            }
        }
        free(logit);
        free(krow);
    }
    return SO_OK;
}

/* ---- ReLU linear attention, Eq. (3) ------------------------------------------------- */

static inline double relu(double x) { return x > 0.0 ? x : 0.0; }

/* State of one (b, h): Hs[a][c] = sum_j relu(K[j][a]) * V[j][c], Z[a] = sum_j relu(K[j][a]).
 * k, v: [B, H, N, d]; Hs: [B, H, d, d]; Z: [B, H, d]. */
int salad_oracle_linear_state(const float *k, const float *v, int B, int H, int64_t N, int d,
                              double *Hs, double *Z)
{
    const int64_t BH = (int64_t)B * H;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        for (int a = 0; a < d; ++a) {
            double *hrow = Hs + (bh * d + a) * d;
            for (int c = 0; c < d; ++c) hrow[c] = 0.0;
            double z = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                double ka = relu((double)k[(bh * N + j) * d + a]);
                const float *vj = v + (bh * N + j) * d;
                for (int c = 0; c < d; ++c) hrow[c] += ka * (double)vj[c];
                z += ka;
            }
            Z[bh * d + a] = z;
        }
    }
    return SO_OK;
}

/* O_l[n] = relu(Q[n]) Hs / (relu(Q[n]).Z + eps) for the listed stored rows of every (b, h).
 * rows: [B*H*nrows] stored row indices (entries < 0 are skipped, output zero);
 * out: [B*H*nrows, d]. */
int salad_oracle_linear_apply(const float *q, const double *Hs, const double *Z,
                              int B, int H, int64_t N, int d, double eps,
                              const int64_t *rows, int64_t nrows, double *out)
{
    const int64_t total = (int64_t)B * H * nrows;
#pragma omp parallel for schedule(static)
    for (int64_t idx = 0; idx < total; ++idx) {
        int64_t bh = idx / nrows;
        int64_t n = rows[idx];
        double *o = out + idx * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        if (n < 0 || n >= N) continue;
        const float *qi = q + (bh * N + n) * d;
        double den = 0.0;
        for (int a = 0; a < d; ++a) {
            double qa = relu((double)qi[a]);
            den += qa * Z[bh * d + a];
            const double *hrow = Hs + (bh * d + a) * d;
            for (int c = 0; c < d; ++c) o[c] += qa * hrow[c];
        }
        den += eps;
        for (int c = 0; c < d; ++c) o[c] /= den;
    }
    return SO_OK;
}

/* ---- rotary position embedding inside the linear branch (Sec. 4.1: the linear branch incorporates 3D RoPE) ----
 *
 * The paper gives no formula; the reading taken here: the feature-mapped queries and keys are rotated in the
 * numerator only, the normaliser keeps the unrotated (non-negative) features:
 *   O_l[i] = sum_j (R_i phi(Q_i)) . (R_j phi(K_j)) V_j / (phi(Q_i) . sum_j phi(K_j) + eps),
 * R_n rotating channel pair (2p, 2p+1) of token n by the angle whose cosine and sine are cs[n][p], sn[n][p]
 * (float32 tables [N, d/2] from the caller, who owns the split of the pairs over the t, y, x axes and the
 * frequencies).  Reassociated like Eq. (3): Hr = sum_j (R_j phi(K_j))^T V_j, numerator = (R_i phi(Q_i)) Hr. */
static inline void rope_rotate(const float *x, const float *cs, const float *sn, int d, double *out)
{
    for (int p = 0; p < d / 2; ++p) {
        const double a = relu((double)x[2 * p]), b = relu((double)x[2 * p + 1]);
        out[2 * p] = a * (double)cs[p] - b * (double)sn[p];
        out[2 * p + 1] = a * (double)sn[p] + b * (double)cs[p];
    }
}

/* Hr [B,H,d,d] = sum_j (R_j relu(K_j))^T V_j. */
int salad_oracle_linear_state_rope(const float *k, const float *v, const float *cs, const float *sn,
                                   int B, int H, int64_t N, int d, double *Hr)
{
    if (d % 2) return SO_EINVAL;
    const int64_t BH = (int64_t)B * H;
#pragma omp parallel for schedule(static)
    for (int64_t bh = 0; bh < BH; ++bh) {
        double *kr = (double *)malloc(sizeof(double) * (size_t)d);
        double *h = Hr + bh * d * d;
        for (int64_t e = 0; e < (int64_t)d * d; ++e) h[e] = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            rope_rotate(k + (bh * N + j) * d, cs + j * (d / 2), sn + j * (d / 2), d, kr);
            const float *vj = v + (bh * N + j) * d;
            for (int a = 0; a < d; ++a)
                for (int c = 0; c < d; ++c) h[a * d + c] += kr[a] * (double)vj[c];
        }
        free(kr);
    }
    return SO_OK;
}

/* O_l for the listed stored rows: (R_n relu(Q_n)) Hr / (relu(Q_n).Z + eps); same argument shapes as
 * salad_oracle_linear_apply. */
int salad_oracle_linear_apply_rope(const float *q, const double *Hr, const double *Z, const float *cs, const float *sn,
                                   int B, int H, int64_t N, int d, double eps,
                                   const int64_t *rows, int64_t nrows, double *out)
{
    if (d % 2) return SO_EINVAL;
    const int64_t total = (int64_t)B * H * nrows;
#pragma omp parallel
    {
        double *qr = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int64_t idx = 0; idx < total; ++idx) {
            const int64_t bh = idx / nrows;
            const int64_t n = rows[idx];
            double *o = out + idx * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (n < 0 || n >= N) continue;
            const float *qi = q + (bh * N + n) * d;
            rope_rotate(qi, cs + n * (d / 2), sn + n * (d / 2), d, qr);
            double den = eps;
            for (int a = 0; a < d; ++a) {
                den += relu((double)qi[a]) * Z[bh * d + a];
                const double *hrow = Hr + (bh * d + a) * d;
                for (int c = 0; c < d; ++c) o[c] += qr[a] * hrow[c];
            }
            for (int c = 0; c < d; ++c) o[c] /= den;
        }
        free(qr);
    }
    return SO_OK;
}

/* The same quantity without reassociation: A = relu(Q) relu(K)^T (one row at a time),
 * O_l[i] = (A_i V) / (A_i 1 + eps).  Quadratic in N: tiny inputs only.
 * q, k, v: one head, [N, d]; out: [N, d]. */
int salad_oracle_linear_attn_quadratic(const float *q, const float *k, const float *v,
                                       int64_t N, int d, double eps, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double *o = out + i * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        double rowsum = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            double a = 0.0;
            for (int x = 0; x < d; ++x)
                a += relu((double)q[i * d + x]) * relu((double)k[j * d + x]);
            rowsum += a;
            for (int c = 0; c < d; ++c) o[c] += a * (double)v[j * d + c];
        }
        for (int c = 0; c < d; ++c) o[c] /= (rowsum + eps);
    }
    return SO_OK;
}

/* ---- dynamic scale, Alg. 1 "Level 2" ------------------------------------------------ */

/* s[b] = (1/N) * sum_n sigmoid(x[b][n] . w + bias);  x: [B, N, D], w: [D]. */
int salad_oracle_gate(const float *x, const float *w, double bias, int B, int64_t N, int D,
                      double *s)
{
    double *sig = (double *)malloc(sizeof(double) * (size_t)N);
    if (!sig) return SO_EINVAL;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            const float *xr = x + ((int64_t)b * N + n) * D;
            double z = bias;
            for (int c = 0; c < D; ++c) z += (double)xr[c] * (double)w[c];
            sig[n] = 1.0 / (1.0 + exp(-z));
        }
        double total = 0.0;
        for (int64_t n = 0; n < N; ++n) total += sig[n];
        s[b] = total / (double)N;
    }
    free(sig);
    return SO_OK;
}

/* ---- residual integration, Alg. 1 last block; Eq. (lambda scale), Sec. 4.2 ------------ */

/* Residual integration with the full Level-1 projection (Alg. 1 "Proj", Sec. 4.2 layer-wise static scaling):
 *   out[b, h_out, r, c] = O_s[b, h_out, r, c]
 *                       + lambda s[b] sum_{h_in, a} O_l[b, h_in, n, a] W_p[h_in d + a][h_out d + c],
 * n = rows[b, h_out, r] being the stored row of compact row r (rows differ between heads, so the linear
 * outputs of all heads at row n are evaluated here from Q, Hs, Z: Eq. (3) quotient).
 * o_s, out: [B, H, nrows, d]; rows: [B, H, nrows] (< 0: skipped, out = O_s); W_p: [D, D] double. */
int salad_oracle_combine_proj(const float *q, const double *Hs, const double *Z, int B, int H, int64_t N, int d,
                              double eps, const double *o_s, const int64_t *rows, int64_t nrows,
                              const double *Wp, double lambda, const double *s, double *out)
{
    const int64_t total = (int64_t)B * H * nrows;
    const int64_t D = (int64_t)H * d;
#pragma omp parallel for schedule(static)
    for (int64_t idx = 0; idx < total; ++idx) {
        const int64_t bh = idx / nrows;
        const int b = (int)(bh / H), ho = (int)(bh % H);
        const int64_t n = rows[idx];
        double *o = out + idx * d;
        for (int c = 0; c < d; ++c) o[c] = o_s[idx * d + c];
        if (n < 0 || n >= N) continue;
        for (int hi = 0; hi < H; ++hi) {
            const int64_t bhi = (int64_t)b * H + hi;
            const float *qi = q + (bhi * N + n) * d;
            /* O_l of head hi at row n */
            double den = eps;
            for (int a = 0; a < d; ++a) den += relu((double)qi[a]) * Z[bhi * d + a];
            for (int a2 = 0; a2 < d; ++a2) {
                double num = 0.0;
                for (int a = 0; a < d; ++a) num += relu((double)qi[a]) * Hs[(bhi * d + a) * d + a2];
                const double ol = num / den;
                const double *wrow = Wp + ((int64_t)hi * d + a2) * D + (int64_t)ho * d;
                for (int c = 0; c < d; ++c) o[c] += lambda * s[b] * ol * wrow[c];
            }
        }
    }
    return SO_OK;
}

/* The same residual integration when the linear branch carries the rotary position embedding (Sec. 4.1 together with
 * Alg. 1 "Proj"): O_l of every head at row n is (R_n relu(Q_n)) Hr / (relu(Q_n).Z + eps) with the rotated state Hr
 * (the numerator is rotated, the normaliser is not), then projected across heads as above.  cs, sn: [N, d/2]. */
int salad_oracle_combine_proj_rope(const float *q, const double *Hr, const double *Z, const float *cs, const float *sn,
                                   int B, int H, int64_t N, int d, double eps, const double *o_s, const int64_t *rows,
                                   int64_t nrows, const double *Wp, double lambda, const double *s, double *out)
{
    if (d % 2) return SO_EINVAL;
    const int64_t total = (int64_t)B * H * nrows;
    const int64_t D = (int64_t)H * d;
#pragma omp parallel
    {
        double *qr = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int64_t idx = 0; idx < total; ++idx) {
            const int64_t bh = idx / nrows;
            const int b = (int)(bh / H), ho = (int)(bh % H);
            const int64_t n = rows[idx];
            double *o = out + idx * d;
            for (int c = 0; c < d; ++c) o[c] = o_s[idx * d + c];
            if (n < 0 || n >= N) continue;
            for (int hi = 0; hi < H; ++hi) {
                const int64_t bhi = (int64_t)b * H + hi;
                const float *qi = q + (bhi * N + n) * d;
                rope_rotate(qi, cs + n * (d / 2), sn + n * (d / 2), d, qr);
                double den = eps;
                for (int a = 0; a < d; ++a) den += relu((double)qi[a]) * Z[bhi * d + a];
                for (int a2 = 0; a2 < d; ++a2) {
                    double num = 0.0;
                    for (int a = 0; a < d; ++a) num += qr[a] * Hr[(bhi * d + a) * d + a2];
                    const double ol = num / den;
                    const double *wrow = Wp + ((int64_t)hi * d + a2) * D + (int64_t)ho * d;
                    for (int c = 0; c < d; ++c) o[c] += lambda * s[b] * ol * wrow[c];
                }
            }
        }
        free(qr);
    }
    return SO_OK;
}

/* Post-tuning branch dropping, Sec. 4.3: dropped[b] = 1 when the sample's dynamic scale is below the
 * threshold.  The comparison is made on the float32 value of s, the precision the device holds it in. */
int salad_oracle_branch_drop(const double *s, int B, double tau, int *dropped)
{
    for (int b = 0; b < B; ++b) dropped[b] = ((float)s[b] < (float)tau) ? 1 : 0;
    return SO_OK;
}

/* out = O_s + lambda * a[h] * s[b] * O_l on compact row sets of shape [B, H, nrows, d]. */
int salad_oracle_combine(const double *o_s, const double *o_l, int B, int H, int64_t nrows, int d,
                         double lambda, const float *head_scale, const double *s, double *out)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            double a = head_scale ? (double)head_scale[h] : 1.0;
            double coef = lambda * a * s[b];
            int64_t base = ((int64_t)b * H + h) * nrows * d;
            for (int64_t e = 0; e < nrows * d; ++e) out[base + e] = o_s[base + e] + coef * o_l[base + e];
        }
    return SO_OK;
}
