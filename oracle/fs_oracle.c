/*
 * CPU oracle for the fused LM-head + Gumbel-max sampling path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, direct
 * evaluation of what the method computes, used only by the tests, by the smoke
 * check and by the CPU-baseline leg of the benchmark.  It shares no code,
 * header, table or helper with the HIP library and neither includes the other.
 *
 * What it computes (one row b at a time, rows are independent):
 *   1. logits            y_i = sum_d H[b,d] * W[i,d]            (Alg. 1, tiled matmul line;
 *                        bf16 inputs widened exactly, accumulated in fp64, d ascending)
 *   2. transform         z_i = y_i / tau_b                       (Alg. 1, "transform": temperature)
 *   3. noise             r_i = word (i & 3) of Philox4x32-10(counter = (i >> 2, row, 0, 0),
 *                        key = (lo32(seed_b), hi32(seed_b)))     (Section "RNG determinism":
 *                        a counter-based generator indexed by the logical position (b, i))
 *                        x_i = min(fma((float)r_i, 2^-32, 2^-33), 1 - 2^-24)   in fp32
 *                        u_i = 1 - x_i  in the open interval (0,1)
 *                        g_i = -log(-log u_i) = -log(-log1p(-x_i))             in fp64
 *                        (Alg. 1 "Draw u in (0,1)"; appendix "Numerically Stable and Fast
 *                        Gumbel Generation"; the paper's (r+1)/(2^32+1) is NOT used because in
 *                        fp32 it rounds to 1.0 for the top 129 values of r)
 *   4. perturbed score   s_i = z_i + g_i                          (Alg. 1)
 *   5. streaming argmax  keep (m, i*) with a strict s_i > m update, i ascending, so the lowest
 *                        index wins exact ties (appendix Alg. "Gumbel-Max sampling (standalone
 *                        logits)"; Theorem "Gumbel-Max")
 *   6. out_idx[b] = i* (0-based), out_val[b] = (float) m.
 *
 * A tiled variant (per-tile (m, idx) candidates, then an argmax over tiles) exists only to
 * demonstrate the Lemma "Max over vocabulary tiles" on the oracle itself and to check the
 * GPU's candidate buffer.
 *
 * The full transform (additive bias, temperature, -inf mask) and the log-normaliser
 * log sum_i exp(z_i) are the second group of functions (fso_transform_row and below); the
 * grouped variants (parallel and online Group-Gumbel-Max) are the third (fso_group_word and below);
 * FP8 (E4M3) weights with per-row scales are the fourth (fso_e4m3_to_double and below), MXFP4
 * weights the fifth (fso_e2m1_to_double and below); truncated supports (top-k, nucleus on the k
 * candidates, Gumbel-top-k) the sixth (fso_topk_row and below).
 *
 * NaN scores never win (the strict > comparison is false for NaN); a row with no
 * score > -inf returns idx = -1, val = -inf.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ Philox4x32-10 */
/* Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3" (SC'11). */

void fso_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32-bit random word for logical position (row, vocab_id) under a 64-bit seed. */
uint32_t fso_random_word(uint64_t seed, int64_t row, int64_t vocab_id)
{
    uint32_t ctr[4] = { (uint32_t)((uint64_t)vocab_id >> 2), (uint32_t)(uint64_t)row, 0u, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    fso_philox4x32_10(ctr, key, out);
    return out[(uint64_t)vocab_id & 3u];
}

/* ------------------------------------------------------------------ uniform -> Gumbel */

/* x = 1 - u as an fp32 value in (0, 1): the shared starting point of both implementations. */
float fso_uniform_x(uint32_t r)
{
    float x = fmaf((float)r, 0x1p-32f, 0x1p-33f);
    float cap = 1.0f - 0x1p-24f;
    return x < cap ? x : cap;
}

/* g = -log(-log u), u = 1 - x, evaluated in fp64. */
double fso_gumbel_from_word(uint32_t r)
{
    double x = (double)fso_uniform_x(r);
    return -log(-log1p(-x));
}

double fso_gumbel(uint64_t seed, int64_t row, int64_t vocab_id)
{
    return fso_gumbel_from_word(fso_random_word(seed, row, vocab_id));
}

/* ------------------------------------------------------------------ logits */

static inline double bf16_to_double(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* One logit: y = sum_d H[b,d] * W[i,d], fp64, d ascending. */
double fso_logit(const uint16_t* H, const uint16_t* W, int64_t D, int64_t b, int64_t i)
{
    const uint16_t* h = H + b * D;
    const uint16_t* w = W + i * D;
    double acc = 0.0;
    for (int64_t d = 0; d < D; ++d)
        acc += bf16_to_double(h[d]) * bf16_to_double(w[d]);
    return acc;
}

/* All logits Y[B,V] (row-major, fp64).  Returns the number of threads used. */
int fso_logits(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V, double* Y)
{
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < V; ++i)
        for (int64_t b = 0; b < B; ++b)
            Y[b * V + i] = fso_logit(H, W, D, b, i);
    return nthreads;
}

/* ------------------------------------------------------------------ streaming Gumbel-max */

/*
 * One row of raw logits y[0..V) -> sample.  vocab ids are vocab_offset + i (global ids, so a
 * vocabulary shard reproduces the unsharded noise).  Also returns the runner-up
 * (second-largest perturbed score and its index; -inf / -1 if V < 2) for the near-tie rule.
 */
void fso_gumbel_max_row(const double* y, int64_t V, double tau, uint64_t seed, int64_t row,
                        int64_t vocab_offset, int64_t* best_idx, double* best_val,
                        int64_t* second_idx, double* second_val)
{
    double m = -INFINITY, m2 = -INFINITY;
    int64_t im = -1, im2 = -1;
    for (int64_t i = 0; i < V; ++i) {
        int64_t vid = vocab_offset + i;
        double z = y[i] / tau;
        double g = fso_gumbel(seed, row, vid);
        double s = z + g;
        if (s > m) {
            m2 = m; im2 = im;
            m = s; im = vid;
        } else if (s > m2) {
            m2 = s; im2 = vid;
        }
    }
    *best_idx = im; *best_val = m;
    if (second_idx) *second_idx = im2;
    if (second_val) *second_val = m2;
}

/* Perturbed score of a single (row, vocab id): s = y/tau + g. */
double fso_score_at(const uint16_t* H, const uint16_t* W, int64_t D, int64_t b_local,
                    int64_t i_local, double tau, uint64_t seed, int64_t row, int64_t vocab_id)
{
    return fso_logit(H, W, D, b_local, i_local) / tau + fso_gumbel(seed, row, vocab_id);
}

static inline uint64_t row_seed(uint64_t seed, const uint64_t* row_seeds, int64_t b)
{
    return row_seeds ? row_seeds[b] : seed;
}
static inline int64_t row_id(const int64_t* row_ids, int64_t row_offset, int64_t b)
{
    return row_ids ? row_ids[b] : row_offset + b;
}

/*
 * Full path: i*_b ~ Cat(softmax(H W^T / tau)) by Gumbel-max with the noise above.
 *   H [B,D], W [V,D] bf16 bits; tau [B]; row_seeds [B] or NULL (then `seed` for all rows);
 *   row_ids [B] or NULL (then row_offset + b) is the row word of the counter.
 * Outputs (each may be NULL except out_idx): out_idx/out_val [B]; top1/top2 perturbed values in
 * fp64 and the runner-up index, for the acceptance rule.  Returns threads used, or -1 on OOM.
 */
int fso_sample(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V,
               const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
               const int64_t* row_ids, int64_t vocab_offset, int32_t* out_idx, float* out_val,
               double* top1_val, int64_t* top2_idx, double* top2_val)
{
    if (B <= 0 || V <= 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits(H, W, B, D, V, Y);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        int64_t i1, i2;
        double m1, m2;
        fso_gumbel_max_row(Y + b * V, V, (double)tau[b], row_seed(seed, row_seeds, b),
                           row_id(row_ids, row_offset, b), vocab_offset, &i1, &m1, &i2, &m2);
        out_idx[b] = (int32_t)i1;
        if (out_val) out_val[b] = (float)m1;
        if (top1_val) top1_val[b] = m1;
        if (top2_idx) top2_idx[b] = i2;
        if (top2_val) top2_val[b] = m2;
    }
    free(Y);
    return nthreads;
}

/*
 * Two-stage form of Alg. 1 with an arbitrary vocabulary tile size: stage 1 keeps one
 * (m, global idx) candidate per (row, tile); stage 2 takes the argmax over tiles, lowest tile
 * first on exact ties.  cand_val/cand_idx are [B, T], T = ceil(V / tile).
 */
int fso_sample_tiled(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V,
                     const float* tau, uint64_t seed, const uint64_t* row_seeds,
                     int64_t row_offset, int64_t vocab_offset, int64_t tile, double* cand_val,
                     int64_t* cand_idx, int32_t* out_idx, float* out_val)
{
    if (B <= 0 || V <= 0 || tile <= 0) return 0;
    int64_t T = (V + tile - 1) / tile;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits(H, W, B, D, V, Y);
    for (int64_t b = 0; b < B; ++b) {
        /* Stage 1 */
        for (int64_t t = 0; t < T; ++t) {
            int64_t lo = t * tile, hi = lo + tile < V ? lo + tile : V;
            int64_t i1;
            double m1;
            fso_gumbel_max_row(Y + b * V + lo, hi - lo, (double)tau[b],
                               row_seed(seed, row_seeds, b), row_offset + b, vocab_offset + lo,
                               &i1, &m1, NULL, NULL);
            cand_val[b * T + t] = m1;
            cand_idx[b * T + t] = i1;
        }
        /* Stage 2 */
        double m = -INFINITY;
        int64_t im = -1;
        for (int64_t t = 0; t < T; ++t)
            if (cand_val[b * T + t] > m) { m = cand_val[b * T + t]; im = cand_idx[b * T + t]; }
        out_idx[b] = (int32_t)im;
        if (out_val) out_val[b] = (float)m;
    }
    free(Y);
    return nthreads;
}

/* ------------------------------------------------------------------ full transform + log-normaliser */
/*
 * Transformed logits of one row (Section "Background", Notation: the logits after the deterministic
 * steps, of which it names a bias added, a temperature and a mask; Alg. 1, "transform"; Section
 * "Top-k, Nucleus Sampling, and Masking": forbidden ids are set to -inf before perturbation):
 *      z_i = (y_i + bias_i) / tau            if id i is allowed
 *      z_i = -inf                             if id i is masked out
 * bias is fp32 [V] or NULL (indexed by the local id i); allowed is a bit array of V bits packed in
 * 32-bit words (bit i%32 of word i/32 set = allowed) or NULL (everything allowed).
 * The order bias -> temperature -> mask is this build's reading; the paper does not fix it.
 */
void fso_transform_row(const double* y, int64_t V, double tau, const float* bias,
                       const uint32_t* allowed, double* z)
{
    for (int64_t i = 0; i < V; ++i) {
        double v = y[i];
        if (bias) v += (double)bias[i];
        v /= tau;
        if (allowed && !((allowed[i >> 5] >> (i & 31)) & 1u)) v = -INFINITY;
        z[i] = v;
    }
}

/* Streaming Gumbel-max over already transformed logits z (same noise, same tie rule as
 * fso_gumbel_max_row; -inf entries can never win because the update is a strict >). */
void fso_gumbel_max_transformed(const double* z, int64_t V, uint64_t seed, int64_t row,
                                int64_t vocab_offset, int64_t* best_idx, double* best_val,
                                int64_t* second_idx, double* second_val)
{
    double m = -INFINITY, m2 = -INFINITY;
    int64_t im = -1, im2 = -1;
    for (int64_t i = 0; i < V; ++i) {
        int64_t vid = vocab_offset + i;
        double s = z[i] + fso_gumbel(seed, row, vid);
        if (s > m) { m2 = m; im2 = im; m = s; im = vid; }
        else if (s > m2) { m2 = s; im2 = vid; }
    }
    *best_idx = im; *best_val = m;
    if (second_idx) *second_idx = im2;
    if (second_val) *second_val = m2;
}

/* log Z = log sum_i exp(z_i) (appendix "Returning Log-Normalizers or Max Values"), max-shifted,
 * fp64; -inf when no entry is finite. */
double fso_log_sum_exp(const double* z, int64_t V)
{
    double zmax = -INFINITY;
    for (int64_t i = 0; i < V; ++i) if (z[i] > zmax) zmax = z[i];
    if (!(zmax > -INFINITY)) return -INFINITY;
    if (zmax == INFINITY) return INFINITY;
    double sum = 0.0;
    for (int64_t i = 0; i < V; ++i) sum += exp(z[i] - zmax);
    return zmax + log(sum);
}

/*
 * Full path with the whole transform and the log-normaliser:
 *   i*_b ~ Cat(softmax(z_b)), z_b = transform(H_b W^T), out_lse[b] = log sum_i exp(z_{b,i}).
 * allowed: NULL, or bit rows of `mask_stride_words` 32-bit words per batch row
 * (mask_stride_words == 0: one row of bits shared by every batch row).
 */
int fso_sample_full(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V,
                    const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                    const int64_t* row_ids, int64_t vocab_offset, const float* bias,
                    const uint32_t* allowed, int64_t mask_stride_words, int32_t* out_idx,
                    float* out_val, double* out_lse, double* top1_val, int64_t* top2_idx,
                    double* top2_val)
{
    if (B <= 0 || V <= 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits(H, W, B, D, V, Y);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double* z = Y + b * V;   /* transformed in place */
        const uint32_t* arow = allowed ? allowed + (size_t)b * (size_t)mask_stride_words : NULL;
        fso_transform_row(z, V, (double)tau[b], bias, arow, z);
        int64_t i1, i2;
        double m1, m2;
        fso_gumbel_max_transformed(z, V, row_seed(seed, row_seeds, b), row_id(row_ids, row_offset, b),
                                   vocab_offset, &i1, &m1, &i2, &m2);
        out_idx[b] = (int32_t)i1;
        if (out_val) out_val[b] = (float)m1;
        if (out_lse) out_lse[b] = fso_log_sum_exp(z, V);
        if (top1_val) top1_val[b] = m1;
        if (top2_idx) top2_idx[b] = i2;
        if (top2_val) top2_val[b] = m2;
    }
    free(Y);
    return nthreads;
}

/* Transformed score of a single (row, id): z + g, or -inf if the id is masked. */
double fso_score_at_full(const uint16_t* H, const uint16_t* W, int64_t D, int64_t b_local,
                         int64_t i_local, double tau, uint64_t seed, int64_t row, int64_t vocab_id,
                         const float* bias, const uint32_t* allowed_row)
{
    double y = fso_logit(H, W, D, b_local, i_local), z;
    fso_transform_row(&y, 1, tau, bias ? bias + i_local : NULL, NULL, &z);
    if (allowed_row && !((allowed_row[i_local >> 5] >> (i_local & 31)) & 1u)) return -INFINITY;
    return z + fso_gumbel(seed, row, vocab_id);
}

/* ------------------------------------------------------------------ grouped variants */

/*
 * Group-Gumbel-Max (Section "Group-Gumbel-Max: Hierarchical Exact Sampling"; appendix algorithms
 * "FlashSampling (parallel)" and "FlashSampling (sequential/online)").  The vocabulary is cut into
 * groups of `g` consecutive ids (the last one may be shorter).  For every group k of a row:
 *      z_k  = Gumbel-max sample inside the group, with the same per-(row, id) noise as the main
 *             path (so z_k is also the best of the main path's candidates inside the group)
 *      L_k  = log sum_{i in group} exp(z_i)                       (group log-mass)
 * A zero-mass group (L_k = -inf) is skipped.  The two variants differ in how the group is chosen;
 * both are exact in distribution (Lemma "Exact group factorization", Lemma "binary merge"), not
 * pathwise equal to the main path.
 *
 * Noise of the group choice (this build's reading; the paper only asks for fresh uniforms):
 * word (k & 3) of Philox4x32-10(counter = (k >> 2, row, stream, 0), same key), k the global group
 * id, stream = 1 for the parallel variant's outer Gumbels and 2 for the online variant's
 * accept/reject uniforms (stream 0 is the per-id noise), mapped to x in (0,1) as in fso_uniform_x.
 */
uint32_t fso_group_word(uint64_t seed, int64_t row, int64_t group_id, uint32_t stream)
{
    uint32_t ctr[4] = { (uint32_t)((uint64_t)group_id >> 2), (uint32_t)(uint64_t)row, stream, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    fso_philox4x32_10(ctr, key, out);
    return out[(uint64_t)group_id & 3u];
}

/* Per-group local sample (global id, -1 for a zero-mass group), its top-two perturbed scores and
 * the group log-mass, for one row of transformed logits z[0..V).  m = ceil(V / g) groups. */
void fso_group_stats(const double* z, int64_t V, int64_t g, uint64_t seed, int64_t row,
                     int64_t vocab_offset, int64_t* zk, double* s1, double* s2, double* L)
{
    int64_t m = (V + g - 1) / g;
    for (int64_t k = 0; k < m; ++k) {
        int64_t lo = k * g, n = (V - lo < g) ? V - lo : g;
        int64_t i1, i2;
        double m1, m2;
        fso_gumbel_max_transformed(z + lo, n, seed, row, vocab_offset + lo, &i1, &m1, &i2, &m2);
        zk[k] = i1;
        if (s1) s1[k] = m1;
        if (s2) s2[k] = m2;
        L[k] = fso_log_sum_exp(z + lo, n);
    }
}

/* Parallel variant: k* = argmax_k (L_k - log(-log ubar_k)), lowest k on exact ties; score[k] is
 * the perturbed log-mass (-inf for a zero-mass group).  Returns k* or -1 when every group has
 * zero mass. */
int64_t fso_group_choose_parallel(const double* L, int64_t m, uint64_t seed, int64_t row,
                                  int64_t group_offset, double* score)
{
    double best = -INFINITY;
    int64_t kstar = -1;
    for (int64_t k = 0; k < m; ++k) {
        double s = -INFINITY;
        if (L[k] > -INFINITY)
            s = L[k] + fso_gumbel_from_word(fso_group_word(seed, row, group_offset + k, 1u));
        if (score) score[k] = s;
        if (s > best) { best = s; kstar = k; }
    }
    return kstar;
}

/* log(e^a + e^b) for a, b in [-inf, +inf). */
static double lse2(double a, double b)
{
    double hi = a > b ? a : b, lo = a > b ? b : a;
    if (!(hi > -INFINITY)) return -INFINITY;
    return hi + log1p(exp(lo - hi));
}

/* Online variant: running (ell, k*) over the groups in ascending order; group k replaces the
 * running sample when u_k < p_k = exp(L_k - lse(ell, L_k)).  The first nonzero-mass group has
 * p = 1 and u < 1 always, which is the algorithm's initialisation.  u[k], p[k] are reported for
 * every nonzero-mass group (NaN otherwise).  Returns k* or -1; *lse_out = final ell. */
int64_t fso_group_choose_online(const double* L, int64_t m, uint64_t seed, int64_t row,
                                int64_t group_offset, double* u, double* p, double* lse_out)
{
    double ell = -INFINITY;
    int64_t kstar = -1;
    for (int64_t k = 0; k < m; ++k) {
        if (u) u[k] = NAN;
        if (p) p[k] = NAN;
        if (!(L[k] > -INFINITY)) continue;
        double ell_new = lse2(ell, L[k]);
        double p_replace = exp(L[k] - ell_new);
        double uk = (double)fso_uniform_x(fso_group_word(seed, row, group_offset + k, 2u));
        if (u) u[k] = uk;
        if (p) p[k] = p_replace;
        if (uk < p_replace) kstar = k;
        ell = ell_new;
    }
    if (lse_out) *lse_out = ell;
    return kstar;
}

/* One row, from transformed logits: mode 0 = parallel, 1 = online.  Returns the sampled global id
 * (-1 when the row has no mass); *lse_out = log sum_i exp(z_i) = lse over the group log-masses. */
int64_t fso_grouped_row(const double* z, int64_t V, int64_t g, int mode, uint64_t seed, int64_t row,
                        int64_t vocab_offset, double* lse_out, int64_t* zk, double* s1, double* s2,
                        double* L, double* outer, double* p)
{
    int64_t m = (V + g - 1) / g, kstar;
    int own = 0;
    if (!zk) { zk = (int64_t*)malloc(sizeof(int64_t) * (size_t)m); own |= 1; }
    if (!L) { L = (double*)malloc(sizeof(double) * (size_t)m); own |= 2; }
    fso_group_stats(z, V, g, seed, row, vocab_offset, zk, s1, s2, L);
    int64_t group_offset = vocab_offset / g;
    double lse = -INFINITY;
    if (mode == 0) {
        kstar = fso_group_choose_parallel(L, m, seed, row, group_offset, outer);
        lse = fso_log_sum_exp(L, m);
    } else {
        kstar = fso_group_choose_online(L, m, seed, row, group_offset, outer, p, &lse);
    }
    int64_t id = kstar < 0 ? -1 : zk[kstar];
    if (lse_out) *lse_out = lse;
    if (own & 1) free(zk);
    if (own & 2) free(L);
    return id;
}

/*
 * Whole batch: logits, full transform, then the grouped choice.  Diagnostics (each NULL or
 * [B, m], m = ceil(V / g)): zk local samples, s1/s2 their top-two perturbed scores, L log-masses,
 * outer = perturbed log-mass (parallel) or the uniform u_k (online), p = replace probability
 * (online only).  vocab_offset must be a multiple of g (global group ids index the noise).
 */
int fso_sample_grouped(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V,
                       const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                       const int64_t* row_ids, int64_t vocab_offset, const float* bias,
                       const uint32_t* allowed, int64_t mask_stride_words, int64_t g, int mode,
                       int32_t* out_idx, double* out_lse, int64_t* zk, double* s1, double* s2,
                       double* L, double* outer, double* p)
{
    if (B <= 0 || V <= 0 || g <= 0 || vocab_offset % g != 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits(H, W, B, D, V, Y);
    int64_t m = (V + g - 1) / g;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        double* z = Y + b * V;
        const uint32_t* arow = allowed ? allowed + (size_t)b * (size_t)mask_stride_words : NULL;
        fso_transform_row(z, V, (double)tau[b], bias, arow, z);
        double lse;
        int64_t id = fso_grouped_row(z, V, g, mode, row_seed(seed, row_seeds, b),
                                     row_id(row_ids, row_offset, b), vocab_offset, &lse,
                                     zk ? zk + b * m : NULL, s1 ? s1 + b * m : NULL,
                                     s2 ? s2 + b * m : NULL, L ? L + b * m : NULL,
                                     outer ? outer + b * m : NULL, p ? p + b * m : NULL);
        out_idx[b] = (int32_t)id;
        if (out_lse) out_lse[b] = lse;
    }
    free(Y);
    return nthreads;
}

/* counts[i] += draws of the grouped sampler that picked i, draw d using (seed, row = row0 + d),
 * on a fixed row of transformed logits z. */
void fso_grouped_draw_counts(const double* z, int64_t V, int64_t g, int mode, uint64_t seed,
                             int64_t row0, int64_t ndraws, int64_t* counts)
{
#pragma omp parallel
    {
        int64_t* local = (int64_t*)calloc((size_t)V, sizeof(int64_t));
#pragma omp for schedule(static)
        for (int64_t d = 0; d < ndraws; ++d) {
            int64_t id = fso_grouped_row(z, V, g, mode, seed, row0 + d, 0, NULL, NULL, NULL, NULL,
                                         NULL, NULL, NULL);
            if (id >= 0) local[id] += 1;
        }
#pragma omp critical
        for (int64_t i = 0; i < V; ++i) counts[i] += local[i];
        free(local);
    }
}

/* ------------------------------------------------------------------ FP8 weights */

/*
 * Lower-precision weights (Section "Limitations and Future Work": FP8 weights as the next byte
 * saving in the bandwidth-bound regime).  This build's reading: W is stored as OCP FP8 E4M3
 * ("e4m3fn": 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities, S.1111.111 = NaN,
 * subnormals m/8 * 2^-6) with one fp32 scale per vocabulary row; the hidden states stay bf16:
 *      y_i = scale_i * sum_d H[b,d] * e4m3(W8[i,d])
 * Every e4m3 value is exactly representable in bf16, so the products are the same exact products
 * as on the bf16 path; everything after y is unchanged.
 */
double fso_e4m3_to_double(uint8_t code)
{
    int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

double fso_logit_w8(const uint16_t* H, const uint8_t* W8, const float* scale, int64_t D, int64_t b, int64_t i)
{
    const uint16_t* h = H + b * D;
    const uint8_t* w = W8 + i * D;
    double acc = 0.0;
    for (int64_t d = 0; d < D; ++d) acc += bf16_to_double(h[d]) * fso_e4m3_to_double(w[d]);
    return scale ? (double)scale[i] * acc : acc;
}

int fso_logits_w8(const uint16_t* H, const uint8_t* W8, const float* scale, int64_t B, int64_t D, int64_t V,
                  double* Y)
{
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < V; ++i)
        for (int64_t b = 0; b < B; ++b) Y[b * V + i] = fso_logit_w8(H, W8, scale, D, b, i);
    return nthreads;
}

/* The default path on FP8 weights: i*_b ~ Cat(softmax(y_b / tau_b)), y as above. */
int fso_sample_w8(const uint16_t* H, const uint8_t* W8, const float* scale, int64_t B, int64_t D, int64_t V,
                  const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                  const int64_t* row_ids, int64_t vocab_offset, int32_t* out_idx, float* out_val,
                  double* top1_val, int64_t* top2_idx, double* top2_val)
{
    if (B <= 0 || V <= 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits_w8(H, W8, scale, B, D, V, Y);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        int64_t i1, i2;
        double m1, m2;
        fso_gumbel_max_row(Y + b * V, V, (double)tau[b], row_seed(seed, row_seeds, b),
                           row_id(row_ids, row_offset, b), vocab_offset, &i1, &m1, &i2, &m2);
        out_idx[b] = (int32_t)i1;
        if (out_val) out_val[b] = (float)m1;
        if (top1_val) top1_val[b] = m1;
        if (top2_idx) top2_idx[b] = i2;
        if (top2_val) top2_val[b] = m2;
    }
    free(Y);
    return nthreads;
}

double fso_score_at_w8(const uint16_t* H, const uint8_t* W8, const float* scale, int64_t D, int64_t b_local,
                       int64_t i_local, double tau, uint64_t seed, int64_t row, int64_t vocab_id)
{
    return fso_logit_w8(H, W8, scale, D, b_local, i_local) / tau + fso_gumbel(seed, row, vocab_id);
}

/* ------------------------------------------------------------------ MXFP4 weights */

/*
 * Four-bit weights in the OCP microscaling format MXFP4 (the second lower-precision format the
 * paper names as future work): elements are FP4 E2M1 codes (1 sign, 2 exponent bits with bias 1,
 * 1 mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), two per byte (element 2j in the low
 * nibble of byte j), and every block of 32 consecutive elements of a row shares one E8M0 scale
 * byte e, worth 2^(e - 127) (e = 255 is NaN).  Hidden states stay bf16:
 *      y_i = sum_d H[b,d] * e2m1(W4[i,d]) * 2^(S[i, d / 32] - 127)
 * A scaled element is a bf16 value (a power-of-two multiple of a one-mantissa-bit number), so the
 * products are again the exact products of the bf16 path.
 */
double fso_e2m1_to_double(uint8_t nibble)
{
    static const double mag[8] = { 0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0 };
    double v = mag[nibble & 7];
    return (nibble & 8) ? -v : v;
}

double fso_e8m0_to_double(uint8_t e)
{
    if (e == 255) return NAN;
    return ldexp(1.0, (int)e - 127);
}

double fso_logit_w4(const uint16_t* H, const uint8_t* W4, const uint8_t* S, int64_t D, int64_t b, int64_t i)
{
    const uint16_t* h = H + b * D;
    const uint8_t* w = W4 + i * (D / 2);
    const uint8_t* sc = S + i * (D / 32);
    double acc = 0.0;
    for (int64_t d = 0; d < D; ++d) {
        uint8_t byte = w[d >> 1];
        uint8_t nib = (d & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15);
        acc += bf16_to_double(h[d]) * (fso_e2m1_to_double(nib) * fso_e8m0_to_double(sc[d >> 5]));
    }
    return acc;
}

int fso_logits_w4(const uint16_t* H, const uint8_t* W4, const uint8_t* S, int64_t B, int64_t D, int64_t V,
                  double* Y)
{
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < V; ++i)
        for (int64_t b = 0; b < B; ++b) Y[b * V + i] = fso_logit_w4(H, W4, S, D, b, i);
    return nthreads;
}

int fso_sample_w4(const uint16_t* H, const uint8_t* W4, const uint8_t* S, int64_t B, int64_t D, int64_t V,
                  const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                  const int64_t* row_ids, int64_t vocab_offset, int32_t* out_idx, float* out_val,
                  double* top1_val, int64_t* top2_idx, double* top2_val)
{
    if (B <= 0 || V <= 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits_w4(H, W4, S, B, D, V, Y);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        int64_t i1, i2;
        double m1, m2;
        fso_gumbel_max_row(Y + b * V, V, (double)tau[b], row_seed(seed, row_seeds, b),
                           row_id(row_ids, row_offset, b), vocab_offset, &i1, &m1, &i2, &m2);
        out_idx[b] = (int32_t)i1;
        if (out_val) out_val[b] = (float)m1;
        if (top1_val) top1_val[b] = m1;
        if (top2_idx) top2_idx[b] = i2;
        if (top2_val) top2_val[b] = m2;
    }
    free(Y);
    return nthreads;
}

double fso_score_at_w4(const uint16_t* H, const uint8_t* W4, const uint8_t* S, int64_t D, int64_t b_local,
                       int64_t i_local, double tau, uint64_t seed, int64_t row, int64_t vocab_id)
{
    return fso_logit_w4(H, W4, S, D, b_local, i_local) / tau + fso_gumbel(seed, row, vocab_id);
}

/* ------------------------------------------------------------------ helpers for the pins */

/* ------------------------------------------------------------------ truncated supports */

/*
 * Section "Top-k, Nucleus Sampling, and Masking".  Two uses of "the k largest of a row":
 *   truncation     the support is cut to the k ids with the largest transformed logits z_i, and
 *                  the draw is a Gumbel-max over that support (which is the masked draw of the same
 *                  section with every other id set to -inf, hence exact on the restricted support);
 *                  optionally the nucleus rule is applied on those k candidates first;
 *   Gumbel-top-k   the k ids with the largest PERTURBED scores s_i = z_i + g_i, in descending
 *                  order: a draw of k ids without replacement (the trick the section cites); its
 *                  first element is the plain Gumbel-max sample.
 * Order used everywhere: larger key first; equal keys: lower id first.  NaN keys count as -inf
 * (they never win).  The paper fixes none of these details.
 */
typedef struct { double key; int64_t id; } fso_pair;

static int fso_pair_cmp(const void* a, const void* b)
{
    const fso_pair* x = (const fso_pair*)a;
    const fso_pair* y = (const fso_pair*)b;
    if (x->key > y->key) return -1;
    if (x->key < y->key) return 1;
    return x->id < y->id ? -1 : (x->id > y->id ? 1 : 0);
}

/* The k largest keys of key[0..V) by a full sort: out_key/out_id [k] in descending order (lower id
 * first on ties), ids reported as vocab_offset + i; slots past V are (-inf, -1).  If kth1 is not
 * NULL it receives the (k+1)-th largest key (-inf if there is none): the runner-up of the cut. */
int fso_topk_row(const double* key, int64_t V, int64_t k, int64_t vocab_offset, double* out_key,
                 int64_t* out_id, double* kth1)
{
    fso_pair* p = (fso_pair*)malloc(sizeof(fso_pair) * (size_t)V);
    if (!p) return -1;
    for (int64_t i = 0; i < V; ++i) {
        p[i].key = isnan(key[i]) ? -INFINITY : key[i];
        p[i].id = vocab_offset + i;
    }
    qsort(p, (size_t)V, sizeof(fso_pair), fso_pair_cmp);
    for (int64_t j = 0; j < k; ++j) {
        out_key[j] = j < V ? p[j].key : -INFINITY;
        out_id[j] = j < V ? p[j].id : -1;
    }
    if (kth1) *kth1 = k < V ? p[k].key : -INFINITY;
    free(p);
    return 0;
}

/*
 * Nucleus rule on k candidates given in descending order of z: q_j = exp(z_j) / sum_{l<k} exp(z_l)
 * (the softmax over the candidates only, as the section applies top-p after top-k); keep the
 * shortest prefix whose mass reaches top_p, at least one candidate.  Candidates with z = -inf
 * (padding) carry no mass.  Returns the number kept; *mass_before (if not NULL) receives the
 * cumulative mass of the kept prefix WITHOUT its last element (how close the cut was to moving).
 * top_p >= 1 keeps every candidate that has mass.
 */
int64_t fso_top_p_cut(const double* z_sorted, int64_t k, double top_p, double* mass_before)
{
    if (mass_before) *mass_before = 0.0;
    if (k <= 0 || !(z_sorted[0] > -INFINITY)) return 0;
    double zmax = z_sorted[0], sum = 0.0;
    int64_t live = 0;
    for (int64_t j = 0; j < k; ++j)
        if (z_sorted[j] > -INFINITY) { sum += exp(z_sorted[j] - zmax); ++live; }
    if (top_p >= 1.0) {
        if (mass_before) *mass_before = live > 0 ? (sum - exp(z_sorted[live - 1] - zmax)) / sum : 0.0;
        return live;
    }
    double cum = 0.0;
    for (int64_t j = 0; j < live; ++j) {
        if (mass_before) *mass_before = cum / sum;
        cum += exp(z_sorted[j] - zmax);
        if (cum / sum >= top_p) return j + 1;
    }
    return live;
}

/*
 * One row.  mode 0 (truncation): z_i = y_i / tau; S = top-k of z; nucleus cut on S; the sample is
 * argmax_{i in kept} (z_i + g_i) with the per-(row, id) noise of the main path, lowest id on ties.
 * mode 1 (Gumbel-top-k): S = top-k of s_i = z_i + g_i; the sample is its first element.
 * Outputs: top_key/top_id [k] (z or s, sorted), *n_kept, *best_id / *best_val (perturbed score),
 * *kth1 = the (k+1)-th key, *mass_before as in fso_top_p_cut, *second_val = runner-up perturbed
 * score among the kept candidates (mode 0) or the second key (mode 1).
 */
int fso_sample_topk_row(const double* y, int64_t V, double tau, uint64_t seed, int64_t row,
                        int64_t vocab_offset, int64_t k, double top_p, int mode, double* top_key,
                        int64_t* top_id, int64_t* n_kept, int64_t* best_id, double* best_val,
                        double* kth1, double* mass_before, double* second_val)
{
    double* key = (double*)malloc(sizeof(double) * (size_t)V);
    if (!key) return -1;
    for (int64_t i = 0; i < V; ++i) {
        key[i] = y[i] / tau;
        if (mode == 1) key[i] += fso_gumbel(seed, row, vocab_offset + i);
    }
    int rc = fso_topk_row(key, V, k, vocab_offset, top_key, top_id, kth1);
    free(key);
    if (rc != 0) return rc;
    if (mode == 1) {
        int64_t live = 0;
        for (int64_t j = 0; j < k; ++j) if (top_id[j] >= 0 && top_key[j] > -INFINITY) ++live;
        *n_kept = live;
        *best_id = live > 0 ? top_id[0] : -1;
        *best_val = live > 0 ? top_key[0] : -INFINITY;
        if (second_val) *second_val = live > 1 ? top_key[1] : -INFINITY;
        if (mass_before) *mass_before = 0.0;
        return 0;
    }
    *n_kept = fso_top_p_cut(top_key, k, top_p, mass_before);
    double m = -INFINITY, m2 = -INFINITY;
    int64_t im = -1;
    /* Gumbel-max over the kept candidates in ascending id order with a strict >: lowest id on ties */
    fso_pair* q = (fso_pair*)malloc(sizeof(fso_pair) * (size_t)(*n_kept > 0 ? *n_kept : 1));
    if (!q) return -1;
    for (int64_t j = 0; j < *n_kept; ++j) { q[j].key = -(double)top_id[j]; q[j].id = j; }   /* by id, ascending */
    qsort(q, (size_t)*n_kept, sizeof(fso_pair), fso_pair_cmp);
    for (int64_t t = 0; t < *n_kept; ++t) {
        const int64_t j = q[t].id;
        const double s = top_key[j] + fso_gumbel(seed, row, top_id[j]);
        if (s > m) { m2 = m; m = s; im = top_id[j]; }
        else if (s > m2) m2 = s;
    }
    free(q);
    *best_id = im;
    *best_val = m;
    if (second_val) *second_val = m2;
    return 0;
}

/* Batch form.  Arrays: top_key/top_id [B, k]; n_kept, kth1, mass_before, top1, top2 [B]. */
int fso_sample_topk(const uint16_t* H, const uint16_t* W, int64_t B, int64_t D, int64_t V,
                    const float* tau, uint64_t seed, const uint64_t* row_seeds, int64_t row_offset,
                    int64_t vocab_offset, int64_t k, double top_p, int mode, int32_t* out_idx,
                    float* out_val, double* top_key, int64_t* top_id, int64_t* n_kept, double* kth1,
                    double* mass_before, double* top1_val, double* top2_val)
{
    if (B <= 0 || V <= 0 || k <= 0) return 0;
    double* Y = (double*)malloc(sizeof(double) * (size_t)B * (size_t)V);
    if (!Y) return -1;
    int nthreads = fso_logits(H, W, B, D, V, Y);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < B; ++b) {
        int64_t bid;
        double bval, second;
        int rc = fso_sample_topk_row(Y + b * V, V, (double)tau[b], row_seed(seed, row_seeds, b), row_offset + b,
                                     vocab_offset, k, top_p, mode, top_key + b * k, top_id + b * k, n_kept + b,
                                     &bid, &bval, kth1 + b, mass_before + b, &second);
        if (rc != 0) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        out_idx[b] = (int32_t)bid;
        if (out_val) out_val[b] = (float)bval;
        if (top1_val) top1_val[b] = bval;
        if (top2_val) top2_val[b] = second;
    }
    free(Y);
    return failed ? -1 : nthreads;
}

/* counts[i] += number of draws that picked i, over draws k = 0..ndraws-1.
 * by_row != 0: draw k uses (seed, row = row0 + k); else (seed + k, row = row0). */
void fso_draw_counts(const double* y, int64_t V, double tau, uint64_t seed, int64_t row0,
                     int64_t ndraws, int by_row, int64_t* counts, double* vals)
{
#pragma omp parallel
    {
        int64_t* local = (int64_t*)calloc((size_t)V, sizeof(int64_t));
#pragma omp for schedule(static)
        for (int64_t k = 0; k < ndraws; ++k) {
            int64_t i1;
            double m1;
            uint64_t s = by_row ? seed : seed + (uint64_t)k;
            int64_t row = by_row ? row0 + k : row0;
            fso_gumbel_max_row(y, V, tau, s, row, 0, &i1, &m1, NULL, NULL);
            if (i1 >= 0) local[i1] += 1;
            if (vals) vals[k] = m1;
        }
#pragma omp critical
        for (int64_t i = 0; i < V; ++i) counts[i] += local[i];
        free(local);
    }
}

/* Brute-force softmax probabilities of z = y / tau in fp64 (max-shifted). */
void fso_softmax(const double* y, int64_t V, double tau, double* p, double* lse)
{
    double zmax = -INFINITY;
    for (int64_t i = 0; i < V; ++i) { double z = y[i] / tau; if (z > zmax) zmax = z; }
    double sum = 0.0;
    for (int64_t i = 0; i < V; ++i) { p[i] = exp(y[i] / tau - zmax); sum += p[i]; }
    for (int64_t i = 0; i < V; ++i) p[i] /= sum;
    if (lse) *lse = zmax + log(sum);
}

/* Gumbel variates for words r[0..n): bulk form of fso_gumbel_from_word. */
void fso_gumbel_from_words(const uint32_t* r, int64_t n, double* g, float* x)
{
    for (int64_t k = 0; k < n; ++k) {
        g[k] = fso_gumbel_from_word(r[k]);
        if (x) x[k] = fso_uniform_x(r[k]);
    }
}

/* Random words for vocab ids [v0, v0+n) of one row: bulk form of fso_random_word. */
void fso_random_words(uint64_t seed, int64_t row, int64_t v0, int64_t n, uint32_t* out)
{
    for (int64_t k = 0; k < n; ++k) out[k] = fso_random_word(seed, row, v0 + k);
}

int fso_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
