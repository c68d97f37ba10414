/*
 * hola_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, float64 CPU statement of what one batched verify step of
 * HOLA's Hierarchical Speculative Decoding (HSD) computes.  It exists so that
 * the HIP path can be checked element by element; it shares no code, header,
 * table or helper with the HIP path, and only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.
 *
 * What the paper fixes (Section 3.1, "HSD Module"; Algorithm 1, Step 1;
 * Equation (1); Section 4.3 for the magnitude of tau):
 *   - the per-position entropy of the DRAFT distribution, H = -sum_i q_i log q_i;
 *   - the gate g(t) = 1[H < tau] with a strict inequality;
 *   - gate = 1 keeps the drafted token without consulting the verifier,
 *     gate = 0 falls back to the verifier.
 * What the paper leaves open and this file fills in with the standard
 * draft-and-verify rule of the literature the paper's related-work section
 * points at (all of it restated here, every reading listed in the design
 * notes of the repository):
 *   - temperature-scaled softmax of both models' logits;
 *   - verifier branch = acceptance test  u * q(x) < p(x),  u uniform on [0,1);
 *   - the sequence stops at its first rejected position;
 *   - at a rejection the next token is drawn from  max(0, p - q) / Z  by
 *     inverse CDF; when every draft is accepted a bonus token is drawn from p;
 *   - uniforms come from Philox4x32-10 keyed on (seed, sequence, position, level);
 *   - "hierarchical": the output of one verify level is the draft of the next.
 *
 * Arithmetic: IEEE double, libm exp/log, sums taken in ascending index order,
 * no blocking, no fusion.  bf16 inputs are widened exactly (bits << 16).
 *
 * Parity pins (tests/test_oracle_*.py, all CPU): Philox known-answer vectors of
 * the published generator; scipy logsumexp / entropy; closed forms for uniform,
 * one-hot, two-point and geometric logits; q = p accepts everything; p(x) = 0
 * always rejects; full-lattice enumeration of the uniform; numpy cumsum +
 * searchsorted for the inverse CDF; Z = 1 - sum min(p,q); brute-force output
 * marginal = p on tiny vocabularies; monotonicity of accept length in tau;
 * tile merge = statistics of the whole row (itself pinned to scipy); top-k /
 * top-p keep sets = numpy stable sort + cumsum, filtered statistics = scipy on
 * the kept subset, filters off = the unfiltered step, output marginal = the
 * filtered target; token trees: a chain = the one-token step, several
 * candidates = a direct numpy restatement, closed-form accept rates, output
 * marginal = p by brute force over the candidates.
 * No function in this file is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11).  Ten rounds; the key is bumped between rounds.   */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += W0; k1 += W1; }
        uint64_t prod0 = (uint64_t)M0 * c0;
        uint64_t prod1 = (uint64_t)M1 * c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 24-bit uniform on the lattice {0, 1, ..., 2^24 - 1} * 2^-24, a subset of [0,1). */
double oracle_u24(uint32_t r) { return (double)(r >> 8) * (1.0 / 16777216.0); }

/* The random block of one (sequence, position, level): counter words are
 * (position, low and high half of the global sequence index, level), the key
 * is the 64-bit seed split in halves. */
static void hsd_random_block(uint64_t seed, int64_t seq, uint32_t pos, uint32_t level, uint32_t out[4])
{
    uint32_t ctr[4] = { pos, (uint32_t)((uint64_t)seq & 0xffffffffu), (uint32_t)((uint64_t)seq >> 32), level };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    oracle_philox4x32_10(ctr, key, out);
}

/* ------------------------------------------------------------------------- */
/* Logit access.  dtype 0: IEEE float; dtype 1: bfloat16 as raw 16-bit words. */
/* ------------------------------------------------------------------------- */
static double logit_at(const void* base, int32_t dtype, int64_t idx)
{
    if (dtype == 0) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Scaled logit z_i = x_i / T.  For a greedy row (T == 0) the entropy gate is
 * evaluated on the unscaled logits, i.e. as if T = 1. */
static double scaled(double x, double T) { return T > 0.0 ? x / T : x; }

/* ------------------------------------------------------------------------- */
/* Row statistics: log-sum-exp, Shannon entropy (nats), argmax.               */
/* Entropy as Section 3.1 defines it, H = -sum_i p_i log p_i, with             */
/* p_i = exp(z_i - lse) and log p_i = z_i - lse, so                            */
/*   H = lse - sum_i z_i exp(z_i - lse);   a term whose probability is 0       */
/* (including z_i = -inf) contributes 0.                                       */
/* A row with no finite logit has no distribution: lse = -inf, H = NaN; a row   */
/* holding +inf or NaN has no softmax either: lse = NaN, H = NaN.              */
/* Shannon entropy is >= 0; on a nearly one-hot row the subtraction above can  */
/* leave a rounding residue below zero, which is returned as 0 (so a threshold */
/* of 0 with the strict gate never fires).                                     */
/* ------------------------------------------------------------------------- */
void oracle_row_stats(const void* logits, int32_t dtype, int64_t offset, int32_t V, double T,
                      double* lse_out, double* H_out, int32_t* argmax_out)
{
    double m = -INFINITY;
    int32_t am = -1;
    for (int32_t i = 0; i < V; ++i) {
        double z = scaled(logit_at(logits, dtype, offset + i), T);
        if (z > m) { m = z; am = i; }          /* strict: lowest index wins ties */
    }
    if (argmax_out) *argmax_out = am;
    if (!(m > -INFINITY) || !(m < INFINITY)) {  /* all -inf, or +inf present */
        if (lse_out) *lse_out = (m == INFINITY) ? NAN : -INFINITY;
        if (H_out) *H_out = NAN;
        return;
    }
    double S = 0.0;
    for (int32_t i = 0; i < V; ++i) {
        double z = scaled(logit_at(logits, dtype, offset + i), T);
        S += exp(z - m);
    }
    double lse = m + log(S);
    double acc = 0.0;
    for (int32_t i = 0; i < V; ++i) {
        double z = scaled(logit_at(logits, dtype, offset + i), T);
        double p = exp(z - lse);
        if (p > 0.0) acc += z * p;
    }
    double H = lse - acc;
    if (H < 0.0) H = 0.0;                       /* rounding residue; NaN passes through */
    if (lse_out) *lse_out = lse;
    if (H_out) *H_out = H;
}

/* ------------------------------------------------------------------------- */
/* Statistics of a row from the statistics of its column tiles (the row is     */
/* the concatenation of the tiles; tile t has log-sum-exp lse_t and entropy    */
/* H_t of its own normalised distribution).  With w_t = exp(lse_t - lse) the   */
/* probability of element i of tile t is w_t p_{i|t}, so Section 3.1's         */
/*   H = -sum_i p_i log p_i = sum_t w_t (H_t - log w_t),                       */
/*   lse = log sum_t exp(lse_t).                                               */
/* A tile with lse_t = -inf (no finite logit) has w_t = 0 and contributes      */
/* nothing, whatever its H_t; a row of such tiles gives lse = -inf, H = NaN.   */
/* A NaN or +inf lse_t makes the row (NaN, NaN), as in oracle_row_stats.       */
/* ------------------------------------------------------------------------- */
void oracle_merge_tile_stats(const double* tile_stats /* [ntiles][2] = (lse_t, H_t) */, int32_t ntiles,
                             double* lse_out, double* H_out)
{
    double m = -INFINITY;
    int bad = 0;
    for (int32_t t = 0; t < ntiles; ++t) {
        double l = tile_stats[2 * t];
        if (l != l) bad = 1;
        if (l > m) m = l;
    }
    if (bad) { *lse_out = NAN; *H_out = NAN; return; }
    if (!(m > -INFINITY) || !(m < INFINITY)) { *lse_out = (m == INFINITY) ? NAN : -INFINITY; *H_out = NAN; return; }
    double S = 0.0;
    for (int32_t t = 0; t < ntiles; ++t) S += exp(tile_stats[2 * t] - m);
    double lse = m + log(S);
    double H = 0.0;
    for (int32_t t = 0; t < ntiles; ++t) {
        double logw = tile_stats[2 * t] - lse;
        double w = exp(logw);
        if (w > 0.0) H += w * (tile_stats[2 * t + 1] - logw);
    }
    *lse_out = lse;
    *H_out = H;
}

/* Probability of token x in the row whose log-sum-exp is lse. */
static double prob_at(const void* logits, int32_t dtype, int64_t offset, int32_t x, double T, double lse)
{
    double z = scaled(logit_at(logits, dtype, offset + x), T);
    return exp(z - lse);
}

/* ------------------------------------------------------------------------- */
/* The acceptance test of the verifier branch:  accept  iff  u * q_x < p_x.   */
/* With u in [0,1): p_x = 0 rejects for every u (also u = 0); q_x = 0 < p_x   */
/* accepts; p_x >= q_x > 0 accepts for every u.  Accept probability is         */
/* min(1, p_x / q_x).                                                          */
/* ------------------------------------------------------------------------- */
int32_t oracle_ratio_accept(double u, double p_x, double q_x) { return (u * q_x < p_x) ? 1 : 0; }

/* ------------------------------------------------------------------------- */
/* Inverse-CDF draw from unnormalised weights w[0..V): the smallest i whose    */
/* inclusive running sum C_i (ascending order) exceeds t = u * Z, Z = C_{V-1}. */
/* If rounding leaves no such i, the largest i with w_i > 0; if no weight is   */
/* positive, -1.  margin_out = distance from t to the nearer end of the chosen */
/* interval, in units of Z.                                                    */
/* ------------------------------------------------------------------------- */
int32_t oracle_inverse_cdf(const double* w, int32_t V, double u, double* Z_out, double* margin_out)
{
    double Z = 0.0;
    for (int32_t i = 0; i < V; ++i) Z += w[i];
    if (Z_out) *Z_out = Z;
    if (margin_out) *margin_out = NAN;
    if (!(Z > 0.0)) return -1;
    double t = u * Z;
    double C = 0.0;
    int32_t last_pos = -1;
    for (int32_t i = 0; i < V; ++i) {
        double prev = C;
        C += w[i];
        if (w[i] > 0.0) last_pos = i;
        if (C > t) {
            if (margin_out) {
                double lo = t - prev, hi = C - t;
                *margin_out = (lo < hi ? lo : hi) / Z;
            }
            return i;
        }
    }
    if (margin_out) *margin_out = 0.0;
    return last_pos;
}

/* Test aids: exact accept / selection frequencies over the whole 24-bit lattice
 * of the uniform (stride > 1 walks a coarser sub-lattice), obtained by calling
 * the two functions above once per lattice point. */
int64_t oracle_ratio_accept_lattice_count(double p_x, double q_x, int32_t stride)
{
    int64_t n = 0;
    for (uint32_t k = 0; k < (1u << 24); k += (uint32_t)stride)
        n += oracle_ratio_accept((double)k * (1.0 / 16777216.0), p_x, q_x);
    return n;
}

void oracle_inverse_cdf_lattice_hist(const double* w, int32_t V, int32_t stride, int64_t* hist)
{
    for (int32_t i = 0; i < V; ++i) hist[i] = 0;
    for (uint32_t k = 0; k < (1u << 24); k += (uint32_t)stride) {
        int32_t t = oracle_inverse_cdf(w, V, (double)k * (1.0 / 16777216.0), NULL, NULL);
        if (t >= 0) hist[t] += 1;
    }
}

/* Residual weights at one position: w_i = max(0, p_i - q_i); bonus: w_i = p_i. */
void oracle_residual_weights(const void* target, const void* draft, int32_t dtype,
                             int64_t t_off, int64_t d_off, int32_t V, double T,
                             double lseP, double lseD, int32_t bonus, double* w)
{
    for (int32_t i = 0; i < V; ++i) {
        double p = prob_at(target, dtype, t_off, i, T, lseP);
        if (bonus) { w[i] = p; continue; }
        double q = prob_at(draft, dtype, d_off, i, T, lseD);
        double d = p - q;
        w[i] = d > 0.0 ? d : 0.0;
    }
}

/* ------------------------------------------------------------------------- */
/* One verify level.                                                           */
/* ------------------------------------------------------------------------- */
typedef struct {
    const void* target_logits;      /* [B, gamma+1, V], row stride target_ld elements (0 => V) */
    const void* draft_logits;       /* [B, gamma,   V], row stride draft_ld  elements (0 => V) */
    int32_t dtype;                  /* 0 = float, 1 = bfloat16 bits */
    int64_t target_ld, draft_ld;
    const int32_t* draft_tokens;    /* [B, gamma] */
    const int32_t* draft_len;       /* [B] in [0, gamma], or NULL => gamma */
    const float* row_temperature;   /* [B] or NULL => temperature; 0 => greedy row */
    const int32_t* force_accept_len;/* [B] or NULL; entry >= 0 overrides the scan result (test aid) */
    uint64_t seed;
    uint32_t level;
    int64_t seq_base;
    int32_t B, gamma, V;
    float temperature, entropy_threshold;
    /* outputs; any may be NULL */
    int32_t* out_accept_len;        /* [B] */
    int32_t* out_next_token;        /* [B] */
    float* out_entropy;             /* [B, gamma], -1 beyond draft_len */
    double* out_entropy64;          /* [B, gamma], NaN beyond draft_len */
    double* out_lse_draft;          /* [B, gamma] */
    double* out_lse_target;         /* [B, gamma+1] */
    double* out_H_target;           /* [B, gamma+1] entropy of the target rows (next level's gate) */
    uint8_t* out_gate;              /* [B, gamma] */
    uint8_t* out_ratio_ok;          /* [B, gamma] */
    double* out_gate_margin;        /* [B, gamma] |H - tau| */
    double* out_ratio_margin;       /* [B, gamma] |u - p_x/q_x|, NaN when q_x == 0 or greedy */
    double* out_sample_margin;      /* [B] */
    double* out_Z;                  /* [B] total residual (or bonus) weight; NaN for greedy */
    int32_t num_threads;            /* <= 0: library default */
} oracle_verify_args;

static void verify_one_sequence(const oracle_verify_args* a, int32_t b, double* w)
{
    const int32_t g = a->gamma, V = a->V;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    const int32_t len = a->draft_len ? a->draft_len[b] : g;
    const double T = (double)(a->row_temperature ? a->row_temperature[b] : a->temperature);
    const int greedy = !(T > 0.0);
    const double tau = (double)a->entropy_threshold;
    const int64_t seq = a->seq_base + b;

    double lseD[64], HD[64], lseP[65], HP[65];
    int32_t amP[65];

    for (int32_t j = 0; j < g; ++j) {
        if (a->out_entropy) a->out_entropy[(int64_t)b * g + j] = -1.0f;
        if (a->out_entropy64) a->out_entropy64[(int64_t)b * g + j] = NAN;
        if (a->out_gate) a->out_gate[(int64_t)b * g + j] = 0;
        if (a->out_ratio_ok) a->out_ratio_ok[(int64_t)b * g + j] = 0;
        if (a->out_gate_margin) a->out_gate_margin[(int64_t)b * g + j] = NAN;
        if (a->out_ratio_margin) a->out_ratio_margin[(int64_t)b * g + j] = NAN;
        if (a->out_lse_draft) a->out_lse_draft[(int64_t)b * g + j] = NAN;
    }
    for (int32_t j = 0; j <= g; ++j) {
        if (a->out_lse_target) a->out_lse_target[(int64_t)b * (g + 1) + j] = NAN;
        if (a->out_H_target) a->out_H_target[(int64_t)b * (g + 1) + j] = NAN;
    }

    /* draft rows: lse and entropy of q */
    for (int32_t j = 0; j < len; ++j) {
        oracle_row_stats(a->draft_logits, a->dtype, ((int64_t)b * g + j) * dld, V, T, &lseD[j], &HD[j], NULL);
        if (a->out_entropy) a->out_entropy[(int64_t)b * g + j] = (float)HD[j];
        if (a->out_entropy64) a->out_entropy64[(int64_t)b * g + j] = HD[j];
        if (a->out_lse_draft) a->out_lse_draft[(int64_t)b * g + j] = lseD[j];
    }
    /* target rows: lse (argmax for greedy rows); entropy kept for a following level */
    for (int32_t j = 0; j <= len; ++j) {
        oracle_row_stats(a->target_logits, a->dtype, ((int64_t)b * (g + 1) + j) * tld, V, T, &lseP[j], &HP[j], &amP[j]);
        if (a->out_lse_target) a->out_lse_target[(int64_t)b * (g + 1) + j] = lseP[j];
        if (a->out_H_target) a->out_H_target[(int64_t)b * (g + 1) + j] = HP[j];
    }

    /* gate, ratio test, first rejection */
    int32_t acc_len = len;
    for (int32_t j = 0; j < len; ++j) {
        int gate = (HD[j] < tau) ? 1 : 0;                 /* Algorithm 1, Step 1: H < tau, strict */
        int32_t x = a->draft_tokens[(int64_t)b * g + j];
        uint32_t r[4];
        hsd_random_block(a->seed, seq, (uint32_t)j, a->level, r);
        double u = oracle_u24(r[0]);
        int ok;
        double rmargin = NAN;
        if (greedy) {
            ok = (x == amP[j]);
        } else {
            double p_x = 0.0, q_x = 1.0;
            if (x >= 0 && x < V) {
                p_x = prob_at(a->target_logits, a->dtype, ((int64_t)b * (g + 1) + j) * tld, x, T, lseP[j]);
                q_x = prob_at(a->draft_logits, a->dtype, ((int64_t)b * g + j) * dld, x, T, lseD[j]);
            }
            ok = oracle_ratio_accept(u, p_x, q_x);
            if (q_x > 0.0) rmargin = fabs(u - p_x / q_x);
        }
        if (a->out_gate) a->out_gate[(int64_t)b * g + j] = (uint8_t)gate;
        if (a->out_ratio_ok) a->out_ratio_ok[(int64_t)b * g + j] = (uint8_t)ok;
        if (a->out_gate_margin) a->out_gate_margin[(int64_t)b * g + j] = fabs(HD[j] - tau);
        if (a->out_ratio_margin) a->out_ratio_margin[(int64_t)b * g + j] = rmargin;
        if (!(gate || ok) && acc_len == len) acc_len = j; /* Equation (1): gate keeps the draft, else verifier */
    }
    if (a->force_accept_len && a->force_accept_len[b] >= 0) acc_len = a->force_accept_len[b];
    if (a->out_accept_len) a->out_accept_len[b] = acc_len;

    /* next token at the stop row */
    const int32_t rrow = acc_len;
    int32_t tok;
    double smargin = NAN, Z = NAN;
    if (greedy) {
        tok = amP[rrow];
    } else {
        uint32_t r[4];
        hsd_random_block(a->seed, seq, (uint32_t)rrow, a->level, r);
        double u2 = oracle_u24(r[1]);
        int32_t bonus = (acc_len >= len);
        int64_t t_off = ((int64_t)b * (g + 1) + rrow) * tld;
        int64_t d_off = ((int64_t)b * g + (bonus ? 0 : rrow)) * dld;
        oracle_residual_weights(a->target_logits, a->draft_logits, a->dtype, t_off, d_off, V, T,
                                lseP[rrow], bonus ? 0.0 : lseD[rrow], bonus, w);
        tok = oracle_inverse_cdf(w, V, u2, &Z, &smargin);
        if (!bonus && !(Z > 0.0)) {                        /* p == q everywhere: fall back to p */
            oracle_residual_weights(a->target_logits, a->draft_logits, a->dtype, t_off, d_off, V, T,
                                    lseP[rrow], 0.0, 1, w);
            tok = oracle_inverse_cdf(w, V, u2, &Z, &smargin);
        }
    }
    if (a->out_next_token) a->out_next_token[b] = tok;
    if (a->out_sample_margin) a->out_sample_margin[b] = smargin;
    if (a->out_Z) a->out_Z[b] = Z;
}

/* Returns 0, or -1 on an argument the oracle does not take. */
int32_t oracle_verify(const oracle_verify_args* a)
{
    if (!a || a->B < 0 || a->gamma < 1 || a->gamma > 63 || a->V < 1) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = a->num_threads > 0 ? a->num_threads : omp_get_max_threads();
#endif
    (void)nthreads;
#pragma omp parallel num_threads(nthreads)
    {
        double* w = (double*)malloc((size_t)a->V * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < a->B; ++b) verify_one_sequence(a, b, w);
        free(w);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Filtered distributions: top-k, then top-p (nucleus) on what top-k left.     */
/* The paper does not filter; these are the usual sampling-time truncations,   */
/* applied to both models before the acceptance test so that the drafted       */
/* token, the test and the residual all speak of the distributions that are    */
/* actually sampled.  Definition used here: order the tokens by scaled logit,  */
/* largest first, equal logits by ascending index (a stable order); top-k      */
/* keeps the first k (k <= 0 or k >= V: all); top-p then keeps the shortest    */
/* prefix of those whose probability, as a fraction of the top-k mass,         */
/* reaches top_p (top_p >= 1: all of them; at least one token is kept).        */
/* Tokens with logit -inf are never kept.  The kept tokens are renormalised:   */
/* lse_out / H_out are the log-sum-exp and entropy (nats) over the kept set.   */
/* margin_out: distance of the nucleus target from the nearer of the two       */
/* cumulative sums that decide the cut, as a fraction of the top-k mass (NaN   */
/* when top-p is off).  Returns the number of kept tokens.                     */
/* force_m >= 0 (test aid) overrides the length of the kept prefix, so that a  */
/* cut that differs within rounding can be followed through the later steps.   */
/* ------------------------------------------------------------------------- */
typedef struct { double z; int32_t i; } oracle_zi;

static int zi_desc(const void* pa, const void* pb)
{
    const oracle_zi* a = (const oracle_zi*)pa;
    const oracle_zi* b = (const oracle_zi*)pb;
    if (a->z > b->z) return -1;
    if (a->z < b->z) return 1;
    return (a->i > b->i) - (a->i < b->i);
}

int32_t oracle_filter_row(const void* logits, int32_t dtype, int64_t offset, int32_t V, double T,
                          int32_t top_k, double top_p, int32_t force_m, uint8_t* keep, double* lse_out,
                          double* H_out, double* margin_out)
{
    double lse, H;
    oracle_row_stats(logits, dtype, offset, V, T, &lse, &H, NULL);
    for (int32_t i = 0; i < V; ++i) keep[i] = 0;
    if (margin_out) *margin_out = NAN;
    if (!(lse > -INFINITY) || !(lse < INFINITY)) { *lse_out = lse; *H_out = NAN; return 0; }

    oracle_zi* o = (oracle_zi*)malloc((size_t)V * sizeof(oracle_zi));
    int32_t n_finite = 0;
    for (int32_t i = 0; i < V; ++i) {
        o[i].z = scaled(logit_at(logits, dtype, offset + i), T);
        o[i].i = i;
        if (o[i].z > -INFINITY) ++n_finite;
    }
    qsort(o, (size_t)V, sizeof(oracle_zi), zi_desc);

    int32_t m = (top_k > 0 && top_k < V) ? top_k : V;
    if (m > n_finite) m = n_finite;
    if (top_p < 1.0) {
        double Zk = 0.0;
        for (int32_t r = 0; r < m; ++r) Zk += exp(o[r].z - lse);
        const double target = top_p * Zk;
        double c = 0.0;
        for (int32_t r = 0; r < m; ++r) {
            const double c_prev = c;
            c += exp(o[r].z - lse);
            if (c >= target) {
                if (margin_out) { double hi = c - target, lo = target - c_prev; *margin_out = (hi < lo ? hi : lo) / Zk; }
                m = r + 1;
                break;
            }
        }
    }
    if (force_m >= 0) m = force_m < n_finite ? force_m : n_finite;
    for (int32_t r = 0; r < m; ++r) keep[o[r].i] = 1;
    free(o);

    /* statistics of the kept tokens, in index order */
    double mx = -INFINITY;
    for (int32_t i = 0; i < V; ++i)
        if (keep[i]) { double z = scaled(logit_at(logits, dtype, offset + i), T); if (z > mx) mx = z; }
    double S = 0.0;
    for (int32_t i = 0; i < V; ++i)
        if (keep[i]) S += exp(scaled(logit_at(logits, dtype, offset + i), T) - mx);
    const double lseK = mx + log(S);
    double acc = 0.0;
    for (int32_t i = 0; i < V; ++i)
        if (keep[i]) { double z = scaled(logit_at(logits, dtype, offset + i), T); acc += z * exp(z - lseK); }
    *lse_out = lseK;
    *H_out = lseK - acc;
    return m;
}

/* Probability of token x under the filtered, renormalised distribution. */
static double filtered_prob_at(const void* logits, int32_t dtype, int64_t offset, int32_t x, double T,
                               const uint8_t* keep, double lseK)
{
    return keep[x] ? prob_at(logits, dtype, offset, x, T, lseK) : 0.0;
}

/* One verify level on filtered distributions: the steps of oracle_verify with
 * q and p replaced by their filtered, renormalised versions everywhere (gate
 * entropy, acceptance test, residual, bonus).  Stochastic rows only (every
 * temperature > 0).  Extra outputs, any may be NULL: out_filter_margin
 * [B, 2 gamma + 1] (draft rows 0..gamma-1, then target rows 0..gamma; NaN for
 * rows not needed or with top-p off), out_keep_count likewise (-1 unused).
 * force_accept_len and the out_lse / out_H_target arrays refer to the filtered
 * statistics.  Returns 0, or -1 on an argument the oracle does not take. */
static void verify_filtered_one_sequence(const oracle_verify_args* a, int32_t top_k, double top_p, int32_t b,
                                         double* w, uint8_t* keepD, uint8_t* keepP,
                                         double* out_filter_margin, int32_t* out_keep_count,
                                         const int32_t* force_keep_count)
{
    const int32_t g = a->gamma, V = a->V;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    const int32_t len = a->draft_len ? a->draft_len[b] : g;
    const double T = (double)(a->row_temperature ? a->row_temperature[b] : a->temperature);
    const double tau = (double)a->entropy_threshold;
    const int64_t seq = a->seq_base + b;
    const int32_t R = 2 * g + 1;

    double lseD[64], HD[64], lseP[65], HP[65];
    for (int32_t j = 0; j < g; ++j) {
        if (a->out_entropy) a->out_entropy[(int64_t)b * g + j] = -1.0f;
        if (a->out_entropy64) a->out_entropy64[(int64_t)b * g + j] = NAN;
        if (a->out_gate) a->out_gate[(int64_t)b * g + j] = 0;
        if (a->out_ratio_ok) a->out_ratio_ok[(int64_t)b * g + j] = 0;
        if (a->out_gate_margin) a->out_gate_margin[(int64_t)b * g + j] = NAN;
        if (a->out_ratio_margin) a->out_ratio_margin[(int64_t)b * g + j] = NAN;
        if (a->out_lse_draft) a->out_lse_draft[(int64_t)b * g + j] = NAN;
    }
    for (int32_t j = 0; j <= g; ++j) {
        if (a->out_lse_target) a->out_lse_target[(int64_t)b * (g + 1) + j] = NAN;
        if (a->out_H_target) a->out_H_target[(int64_t)b * (g + 1) + j] = NAN;
    }
    for (int32_t k = 0; k < R; ++k) {
        if (out_filter_margin) out_filter_margin[(int64_t)b * R + k] = NAN;
        if (out_keep_count) out_keep_count[(int64_t)b * R + k] = -1;
    }

    for (int32_t j = 0; j < len; ++j) {
        double mg;
        int32_t n = oracle_filter_row(a->draft_logits, a->dtype, ((int64_t)b * g + j) * dld, V, T, top_k, top_p,
                                      force_keep_count ? force_keep_count[(int64_t)b * R + j] : -1,
                                      keepD + (size_t)j * V, &lseD[j], &HD[j], &mg);
        if (out_filter_margin) out_filter_margin[(int64_t)b * R + j] = mg;
        if (out_keep_count) out_keep_count[(int64_t)b * R + j] = n;
        if (a->out_entropy) a->out_entropy[(int64_t)b * g + j] = (float)HD[j];
        if (a->out_entropy64) a->out_entropy64[(int64_t)b * g + j] = HD[j];
        if (a->out_lse_draft) a->out_lse_draft[(int64_t)b * g + j] = lseD[j];
    }
    for (int32_t j = 0; j <= len; ++j) {
        double mg;
        int32_t n = oracle_filter_row(a->target_logits, a->dtype, ((int64_t)b * (g + 1) + j) * tld, V, T, top_k, top_p,
                                      force_keep_count ? force_keep_count[(int64_t)b * R + g + j] : -1,
                                      keepP + (size_t)j * V, &lseP[j], &HP[j], &mg);
        if (out_filter_margin) out_filter_margin[(int64_t)b * R + g + j] = mg;
        if (out_keep_count) out_keep_count[(int64_t)b * R + g + j] = n;
        if (a->out_lse_target) a->out_lse_target[(int64_t)b * (g + 1) + j] = lseP[j];
        if (a->out_H_target) a->out_H_target[(int64_t)b * (g + 1) + j] = HP[j];
    }

    int32_t acc_len = len;
    for (int32_t j = 0; j < len; ++j) {
        int gate = (HD[j] < tau) ? 1 : 0;
        int32_t x = a->draft_tokens[(int64_t)b * g + j];
        uint32_t r[4];
        hsd_random_block(a->seed, seq, (uint32_t)j, a->level, r);
        double u = oracle_u24(r[0]);
        double p_x = 0.0, q_x = 1.0, rmargin = NAN;
        if (x >= 0 && x < V) {
            p_x = filtered_prob_at(a->target_logits, a->dtype, ((int64_t)b * (g + 1) + j) * tld, x, T, keepP + (size_t)j * V, lseP[j]);
            q_x = filtered_prob_at(a->draft_logits, a->dtype, ((int64_t)b * g + j) * dld, x, T, keepD + (size_t)j * V, lseD[j]);
        }
        int ok = oracle_ratio_accept(u, p_x, q_x);
        if (q_x > 0.0) rmargin = fabs(u - p_x / q_x);
        if (a->out_gate) a->out_gate[(int64_t)b * g + j] = (uint8_t)gate;
        if (a->out_ratio_ok) a->out_ratio_ok[(int64_t)b * g + j] = (uint8_t)ok;
        if (a->out_gate_margin) a->out_gate_margin[(int64_t)b * g + j] = fabs(HD[j] - tau);
        if (a->out_ratio_margin) a->out_ratio_margin[(int64_t)b * g + j] = rmargin;
        if (!(gate || ok) && acc_len == len) acc_len = j;
    }
    if (a->force_accept_len && a->force_accept_len[b] >= 0) acc_len = a->force_accept_len[b];
    if (a->out_accept_len) a->out_accept_len[b] = acc_len;

    const int32_t rrow = acc_len;
    uint32_t r[4];
    hsd_random_block(a->seed, seq, (uint32_t)rrow, a->level, r);
    const double u2 = oracle_u24(r[1]);
    const int32_t bonus = (acc_len >= len);
    const int64_t t_off = ((int64_t)b * (g + 1) + rrow) * tld;
    const int64_t d_off = ((int64_t)b * g + (bonus ? 0 : rrow)) * dld;
    const uint8_t* kP = keepP + (size_t)rrow * V;
    const uint8_t* kD = keepD + (size_t)(bonus ? 0 : rrow) * V;
    for (int pass = 0; pass < 2; ++pass) {
        const int as_bonus = bonus || pass == 1;             /* second pass: residual without mass, sample p itself */
        for (int32_t i = 0; i < V; ++i) {
            double p = filtered_prob_at(a->target_logits, a->dtype, t_off, i, T, kP, lseP[rrow]);
            if (as_bonus) { w[i] = p; continue; }
            double q = filtered_prob_at(a->draft_logits, a->dtype, d_off, i, T, kD, lseD[rrow]);
            double d = p - q;
            w[i] = d > 0.0 ? d : 0.0;
        }
        double Z, smargin;
        int32_t tok = oracle_inverse_cdf(w, V, u2, &Z, &smargin);
        if (as_bonus || Z > 0.0) {
            if (a->out_next_token) a->out_next_token[b] = tok;
            if (a->out_sample_margin) a->out_sample_margin[b] = smargin;
            if (a->out_Z) a->out_Z[b] = Z;
            break;
        }
    }
}

int32_t oracle_verify_filtered(const oracle_verify_args* a, int32_t top_k, double top_p,
                               double* out_filter_margin, int32_t* out_keep_count,
                               const int32_t* force_keep_count /* [B, 2 gamma + 1] or NULL; entries < 0: not forced */)
{
    if (!a || a->B < 0 || a->gamma < 1 || a->gamma > 63 || a->V < 1) return -1;
    if (!(top_p > 0.0)) return -1;
    if (!a->row_temperature && !(a->temperature > 0.f)) return -1;
    if (a->row_temperature)
        for (int32_t b = 0; b < a->B; ++b) if (!(a->row_temperature[b] > 0.f)) return -1;
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = a->num_threads > 0 ? a->num_threads : omp_get_max_threads();
#endif
    (void)nthreads;
#pragma omp parallel num_threads(nthreads)
    {
        double* w = (double*)malloc((size_t)a->V * sizeof(double));
        uint8_t* keepD = (uint8_t*)malloc((size_t)a->gamma * a->V);
        uint8_t* keepP = (uint8_t*)malloc((size_t)(a->gamma + 1) * a->V);
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < a->B; ++b)
            verify_filtered_one_sequence(a, top_k, top_p, b, w, keepD, keepP, out_filter_margin, out_keep_count,
                                         force_keep_count);
        free(w); free(keepD); free(keepP);
    }
    return 0;
}

/* The interval [C_{tok-1}, C_tok] / Z of token `tok` in the distribution the
 * stop row of sequence b is sampled from (residual when acc_len < len, bonus
 * otherwise), for judging a sample that differs from the oracle's. */
int32_t oracle_sample_interval(const oracle_verify_args* a, int32_t b, int32_t acc_len, int32_t tok,
                               double* lo_out, double* hi_out)
{
    const int32_t g = a->gamma, V = a->V;
    if (tok < 0 || tok >= V || acc_len < 0 || acc_len > g) return -1;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    const int32_t len = a->draft_len ? a->draft_len[b] : g;
    const double T = (double)(a->row_temperature ? a->row_temperature[b] : a->temperature);
    if (!(T > 0.0)) return -1;
    int32_t bonus = (acc_len >= len);
    int64_t t_off = ((int64_t)b * (g + 1) + acc_len) * tld;
    int64_t d_off = ((int64_t)b * g + (bonus ? 0 : acc_len)) * dld;
    double lseP, lseD = 0.0;
    oracle_row_stats(a->target_logits, a->dtype, t_off, V, T, &lseP, NULL, NULL);
    if (!bonus) oracle_row_stats(a->draft_logits, a->dtype, d_off, V, T, &lseD, NULL, NULL);
    double* w = (double*)malloc((size_t)V * sizeof(double));
    oracle_residual_weights(a->target_logits, a->draft_logits, a->dtype, t_off, d_off, V, T, lseP, lseD, bonus, w);
    double Z = 0.0;
    for (int32_t i = 0; i < V; ++i) Z += w[i];
    if (!bonus && !(Z > 0.0)) {
        oracle_residual_weights(a->target_logits, a->draft_logits, a->dtype, t_off, d_off, V, T, lseP, 0.0, 1, w);
        Z = 0.0;
        for (int32_t i = 0; i < V; ++i) Z += w[i];
    }
    double C = 0.0, prev = 0.0;
    for (int32_t i = 0; i <= tok; ++i) { prev = C; C += w[i]; }
    free(w);
    if (!(Z > 0.0)) return -1;
    *lo_out = prev / Z;
    *hi_out = C / Z;
    return 0;
}

/* The same interval on filtered distributions (test aid): the keep sets of the
 * stop row pair are those of oracle_filter_row with the given top_k / top_p,
 * their lengths overridden by force_keep_count where that is given and >= 0. */
int32_t oracle_sample_interval_filtered(const oracle_verify_args* a, int32_t top_k, double top_p,
                                        const int32_t* force_keep_count /* [B, 2 gamma + 1] or NULL */,
                                        int32_t b, int32_t acc_len, int32_t tok, double* lo_out, double* hi_out)
{
    const int32_t g = a->gamma, V = a->V, R = 2 * g + 1;
    if (tok < 0 || tok >= V || acc_len < 0 || acc_len > g) return -1;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    const int32_t len = a->draft_len ? a->draft_len[b] : g;
    const double T = (double)(a->row_temperature ? a->row_temperature[b] : a->temperature);
    if (!(T > 0.0)) return -1;
    const int32_t bonus = (acc_len >= len);
    const int64_t t_off = ((int64_t)b * (g + 1) + acc_len) * tld;
    const int64_t d_off = ((int64_t)b * g + (bonus ? 0 : acc_len)) * dld;
    uint8_t* kP = (uint8_t*)malloc((size_t)V);
    uint8_t* kD = (uint8_t*)malloc((size_t)V);
    double* w = (double*)malloc((size_t)V * sizeof(double));
    double lseP, lseD = 0.0, H, mg;
    oracle_filter_row(a->target_logits, a->dtype, t_off, V, T, top_k, top_p,
                      force_keep_count ? force_keep_count[(int64_t)b * R + g + acc_len] : -1, kP, &lseP, &H, &mg);
    if (!bonus)
        oracle_filter_row(a->draft_logits, a->dtype, d_off, V, T, top_k, top_p,
                          force_keep_count ? force_keep_count[(int64_t)b * R + acc_len] : -1, kD, &lseD, &H, &mg);
    double Z = 0.0;
    for (int pass = 0; pass < 2; ++pass) {
        const int as_bonus = bonus || pass == 1;
        Z = 0.0;
        for (int32_t i = 0; i < V; ++i) {
            double p = filtered_prob_at(a->target_logits, a->dtype, t_off, i, T, kP, lseP);
            if (as_bonus) { w[i] = p; Z += p; continue; }
            double q = filtered_prob_at(a->draft_logits, a->dtype, d_off, i, T, kD, lseD);
            double d = p - q;
            w[i] = d > 0.0 ? d : 0.0;
            Z += w[i];
        }
        if (as_bonus || Z > 0.0) break;
    }
    double C = 0.0, prev = 0.0;
    for (int32_t i = 0; i <= tok; ++i) { prev = C; C += w[i]; }
    free(w); free(kP); free(kD);
    if (!(Z > 0.0)) return -1;
    *lo_out = prev / Z;
    *hi_out = C / Z;
    return 0;
}

/* The interval [C_{tok-1}, C_tok] / Z of token `tok` under softmax(row / T) itself
 * (test aid for draws taken straight from a target row). */
int32_t oracle_row_interval(const void* logits, int32_t dtype, int64_t offset, int32_t V, double T, int32_t tok,
                            double* lo_out, double* hi_out)
{
    if (tok < 0 || tok >= V || !(T > 0.0)) return -1;
    double lse;
    oracle_row_stats(logits, dtype, offset, V, T, &lse, NULL, NULL);
    double Z = 0.0, C = 0.0, prev = 0.0;
    for (int32_t i = 0; i < V; ++i) {
        const double p = prob_at(logits, dtype, offset, i, T, lse);
        Z += p;
        if (i <= tok) { prev = C; C += p; }
    }
    if (!(Z > 0.0)) return -1;
    *lo_out = prev / Z;
    *hi_out = C / Z;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Hierarchical verify over n_models logit sets, smallest drafter first.       */
/* Level k (k = 1 .. n_models-1) verifies with models[k] the drafts that       */
/* level k-1 produced: its accepted tokens followed by its next token (or,     */
/* with survivors_only, its accepted tokens alone: the other reading of "the   */
/* target verifies the survivors", which is not lossless).                     */
/* models[k] has gamma+k rows per sequence; tau[k-1] gates level k on the      */
/* entropy of models[k-1] (of its filtered distribution when filters are on).  */
/* ------------------------------------------------------------------------- */
int32_t oracle_hsd_verify(const void* const* model_logits, const int64_t* model_ld, int32_t n_models,
                          int32_t dtype, const int32_t* draft_tokens, uint64_t seed, int64_t seq_base,
                          int32_t B, int32_t gamma, int32_t V,
                          const float* row_temperature, float temperature, const float* tau,
                          int32_t* out_tokens,      /* [B, gamma + n_models - 1], -1 beyond the drafts */
                          int32_t* out_accept_len,  /* [B] final level */
                          int32_t* out_next_token,  /* [B] final level */
                          float* out_entropy,       /* [n_models-1, B, gamma + n_models - 2], -1 where unused */
                          int32_t* out_level_accept,/* [n_models-1, B] or NULL */
                          int32_t* out_level_next,  /* [n_models-1, B] or NULL */
                          int32_t survivors_only,   /* alternative reading: pass on the kept tokens only */
                          int32_t top_k, double top_p, /* filters on both models of every level; 0 and 1: none */
                          int32_t num_threads)
{
    if (n_models < 2 || B < 0 || gamma < 1 || gamma + n_models - 2 > 63) return -1;
    const int32_t L = n_models - 1;
    const int32_t gmax = gamma + L - 1;           /* drafts at the last level */
    const int32_t wout = gamma + L;               /* width of out_tokens */
    int32_t* toks = (int32_t*)malloc((size_t)B * (gmax + 1) * sizeof(int32_t));
    int32_t* lens = (int32_t*)malloc((size_t)B * sizeof(int32_t));
    int32_t* acc = (int32_t*)malloc((size_t)B * sizeof(int32_t));
    int32_t* nxt = (int32_t*)malloc((size_t)B * sizeof(int32_t));
    float* ent = (float*)malloc((size_t)B * gmax * sizeof(float));
    int32_t* cur = (int32_t*)malloc((size_t)B * gmax * sizeof(int32_t));
    for (int32_t b = 0; b < B; ++b) {
        lens[b] = gamma;
        for (int32_t j = 0; j < gamma; ++j) toks[(int64_t)b * (gmax + 1) + j] = draft_tokens[(int64_t)b * gamma + j];
    }
    if (out_entropy)
        for (int64_t i = 0; i < (int64_t)L * B * gmax; ++i) out_entropy[i] = -1.0f;
    int32_t rc = 0;
    for (int32_t k = 1; k <= L && rc == 0; ++k) {
        const int32_t gk = gamma + k - 1;         /* drafts offered at this level */
        for (int32_t b = 0; b < B; ++b)
            for (int32_t j = 0; j < gk; ++j)
                cur[(int64_t)b * gk + j] = (j < lens[b]) ? toks[(int64_t)b * (gmax + 1) + j] : -1;
        oracle_verify_args a;
        memset(&a, 0, sizeof a);
        a.target_logits = model_logits[k];
        a.draft_logits = model_logits[k - 1];
        a.dtype = dtype;
        a.target_ld = model_ld ? model_ld[k] : 0;
        a.draft_ld = model_ld ? model_ld[k - 1] : 0;
        a.draft_tokens = cur;
        a.draft_len = lens;
        a.row_temperature = row_temperature;
        a.seed = seed;
        a.level = (uint32_t)(k - 1);
        a.seq_base = seq_base;
        a.B = B; a.gamma = gk; a.V = V;
        a.temperature = temperature;
        a.entropy_threshold = tau[k - 1];
        a.out_accept_len = acc;
        a.out_next_token = nxt;
        a.out_entropy = ent;
        a.num_threads = num_threads;
        /* A level on filtered distributions is the filtered step with that level's pair of models: both sides
           of its ratio test and its residual are the renormalised kept sets, so each level stays exact with
           respect to its own filtered verifier. */
        const int filtered = (top_k > 0 && top_k < V) || top_p < 1.0;
        rc = filtered ? oracle_verify_filtered(&a, top_k, top_p, NULL, NULL, NULL) : oracle_verify(&a);
        for (int32_t b = 0; b < B && rc == 0; ++b) {
            if (out_entropy)
                for (int32_t j = 0; j < gk; ++j)
                    out_entropy[((int64_t)(k - 1) * B + b) * gmax + j] = ent[(int64_t)b * gk + j];
            if (out_level_accept) out_level_accept[(int64_t)(k - 1) * B + b] = acc[b];
            if (out_level_next) out_level_next[(int64_t)(k - 1) * B + b] = nxt[b];
            if (k < L) {
                if (survivors_only) {             /* alternative reading: the kept tokens only */
                    lens[b] = acc[b];
                } else {                          /* next level's drafts: accepted prefix + next token */
                    toks[(int64_t)b * (gmax + 1) + acc[b]] = nxt[b];
                    lens[b] = acc[b] + 1;
                }
            }
        }
    }
    if (rc == 0) {
        for (int32_t b = 0; b < B; ++b) {
            if (out_accept_len) out_accept_len[b] = acc[b];
            if (out_next_token) out_next_token[b] = nxt[b];
            if (out_tokens)
                for (int32_t j = 0; j < wout; ++j)
                    out_tokens[(int64_t)b * wout + j] = (j < lens[b]) ? toks[(int64_t)b * (gmax + 1) + j] : -1;
        }
    }
    free(toks); free(lens); free(acc); free(nxt); free(ent); free(cur);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Equation (1) taken literally (no stop at a replaced token): for every       */
/* drafted position t, y_t = draft token if g(t) = 1[H(draft_t) < tau] = 1,     */
/* otherwise y_t = f_ver(x, draft_<t): a token of the verifier's distribution  */
/* at position t given the drafted prefix, i.e. a draw from                    */
/* p_t = softmax(target[b, t] / T) (argmax on greedy rows) with the sampling   */
/* uniform of position t.  Target row gamma is not used.  Section 3.1 counts   */
/* the verifier invocations k; out_calls returns them per sequence.            */
/* Uses the fields of oracle_verify_args; out_accept_len / out_next_token /    */
/* ratio outputs are ignored.                                                  */
/* ------------------------------------------------------------------------- */
int32_t oracle_verify_literal(const oracle_verify_args* a, int32_t* out_tokens /* [B, gamma], -1 beyond len */,
                              int32_t* out_calls /* [B] */, double* out_pos_sample_margin /* [B, gamma] or NULL */,
                              const int8_t* force_gate /* [B, gamma] or NULL; 0 / 1 overrides that gate (test aid) */)
{
    if (!a || a->B < 0 || a->gamma < 1 || a->gamma > 63 || a->V < 1) return -1;
    const int32_t g = a->gamma, V = a->V;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    const double tau = (double)a->entropy_threshold;
    double* w = (double*)malloc((size_t)V * sizeof(double));
    for (int32_t b = 0; b < a->B; ++b) {
        const int32_t len = a->draft_len ? a->draft_len[b] : g;
        const double T = (double)(a->row_temperature ? a->row_temperature[b] : a->temperature);
        const int greedy = !(T > 0.0);
        int32_t calls = 0;
        for (int32_t t = 0; t < g; ++t) {
            const int64_t o = (int64_t)b * g + t;
            out_tokens[o] = -1;
            if (a->out_entropy) a->out_entropy[o] = -1.0f;
            if (a->out_entropy64) a->out_entropy64[o] = NAN;
            if (a->out_gate) a->out_gate[o] = 0;
            if (a->out_gate_margin) a->out_gate_margin[o] = NAN;
            if (out_pos_sample_margin) out_pos_sample_margin[o] = NAN;
            if (t >= len) continue;
            double lseD, HD;
            oracle_row_stats(a->draft_logits, a->dtype, o * dld, V, T, &lseD, &HD, NULL);
            int gate = (HD < tau) ? 1 : 0;
            if (force_gate && force_gate[o] >= 0) gate = force_gate[o] ? 1 : 0;
            if (a->out_entropy) a->out_entropy[o] = (float)HD;
            if (a->out_entropy64) a->out_entropy64[o] = HD;
            if (a->out_gate) a->out_gate[o] = (uint8_t)gate;
            if (a->out_gate_margin) a->out_gate_margin[o] = fabs(HD - tau);
            if (gate) { out_tokens[o] = a->draft_tokens[o]; continue; }
            ++calls;
            const int64_t t_off = ((int64_t)b * (g + 1) + t) * tld;
            double lseP, HP, Z, m = NAN;
            int32_t am;
            oracle_row_stats(a->target_logits, a->dtype, t_off, V, T, &lseP, &HP, &am);
            if (greedy) { out_tokens[o] = am; continue; }
            uint32_t r[4];
            hsd_random_block(a->seed, a->seq_base + b, (uint32_t)t, a->level, r);
            oracle_residual_weights(a->target_logits, a->draft_logits, a->dtype, t_off, 0, V, T, lseP, 0.0, 1, w);
            out_tokens[o] = oracle_inverse_cdf(w, V, oracle_u24(r[1]), &Z, &m);
            if (out_pos_sample_margin) out_pos_sample_margin[o] = m;
        }
        if (out_calls) out_calls[b] = calls;
    }
    free(w);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Token trees (several drafted tokens per position).  The paper drafts one    */
/* token per position; this is the multi-candidate generalisation of the same  */
/* step, with the published recursive rejection rule for several candidates    */
/* drawn independently from the same draft distribution (Miao et al.,          */
/* "SpecInfer", multi-step speculative sampling):                              */
/*   context c = the prefix plus the tokens on the path to node c-1 (c = 0:    */
/*   the prefix alone); q_c, p_c = the two models' distributions after it.     */
/*   The children of a context are tried in node order against a running       */
/*   distribution r, r = p_c at first: child x is kept iff u q_c(x) < r(x);    */
/*   after a rejection r <- max(0, r - q_c) / its sum.  A kept child becomes   */
/*   the context; when every child is rejected the next token is drawn from    */
/*   r and the walk stops; a context without children draws from p_c.          */
/* The gate of Algorithm 1, Step 1 acts on the context's draft entropy: with   */
/* H(q_c) < tau the first child is kept without a test (Equation (1), draft    */
/* branch).  A chain (node n's parent is n-1) is exactly the one-token step    */
/* above, uniforms included: node n's test uses word 0 of block (n, level),    */
/* the draw at context c uses word 1 of block (c, level).                      */
/* A residual without mass after a rejection (impossible in exact arithmetic)  */
/* ends the walk with a draw from p_c, like the one-token step.                */
/* Margins: gate |H - tau| per context; test |u - r(x)/q(x)| scaled by         */
/* Z / max(1, C), Z the product of the residual sums so far and C the sum of   */
/* those products before it (the size of the test in the unnormalised terms    */
/* max(0, p - C q) that an implementation may use); both 1, 0 for a first      */
/* child.                                                                      */
/* ------------------------------------------------------------------------- */
typedef struct {
    const void* target_logits;      /* [B, N+1, V] row c: context c */
    const void* draft_logits;       /* [B, N, V]   row c: context c (rows of contexts without children are not read) */
    int32_t dtype;
    int64_t target_ld, draft_ld;
    const int32_t* node_token;      /* [B, N] */
    const int32_t* node_parent;     /* [B, N] -1: child of the prefix; else an earlier node */
    const int32_t* n_nodes;         /* [B] in [0, N] or NULL => N */
    uint64_t seed;
    uint32_t level;
    int64_t seq_base;
    int32_t B, N, V;
    float temperature, entropy_threshold;
    /* outputs; any may be NULL */
    int32_t* out_accept_len;        /* [B] kept nodes */
    int32_t* out_path;              /* [B, N] kept nodes from the prefix on, -1 beyond */
    int32_t* out_next_token;        /* [B] */
    float* out_entropy;             /* [B, N] H(q_c) of contexts with children, -1 elsewhere */
    double* out_entropy64;          /* [B, N] NaN elsewhere */
    double* out_gate_margin;        /* [B, N] per context, NaN where unused or not visited */
    double* out_ratio_margin;       /* [B, N] per node, NaN where not tested */
    double* out_sample_margin;      /* [B] */
    int32_t num_threads;
    /* test aids; any may be NULL */
    const int32_t* force_node;      /* [B] node whose decision (gate or test) is overridden, -1: none */
    const int32_t* force_outcome;   /* [B] 1: that node is kept, 0: it is rejected */
    const int32_t* probe_token;     /* [B] token whose interval in the walk's final draw is wanted, -1: none */
    double* out_probe_lo;           /* [B] its interval [C_{tok-1}, C_tok] / Z, NaN when not asked or without mass */
    double* out_probe_hi;
} oracle_tree_args;

static void tree_one_sequence(const oracle_tree_args* a, int32_t b, double* pr, double* q, double* w)
{
    const int32_t N = a->N, V = a->V;
    const int64_t tld = a->target_ld ? a->target_ld : V;
    const int64_t dld = a->draft_ld ? a->draft_ld : V;
    int32_t len = a->n_nodes ? a->n_nodes[b] : N;
    if (len < 0) len = 0;
    if (len > N) len = N;
    const double T = (double)a->temperature;
    const double tau = (double)a->entropy_threshold;
    const int64_t seq = a->seq_base + b;
    const int32_t* tok = a->node_token + (int64_t)b * N;
    const int32_t* par = a->node_parent + (int64_t)b * N;

    for (int32_t c = 0; c < N; ++c) {
        const int64_t o = (int64_t)b * N + c;
        if (a->out_path) a->out_path[o] = -1;
        if (a->out_entropy) a->out_entropy[o] = -1.0f;
        if (a->out_entropy64) a->out_entropy64[o] = NAN;
        if (a->out_gate_margin) a->out_gate_margin[o] = NAN;
        if (a->out_ratio_margin) a->out_ratio_margin[o] = NAN;
    }
    /* the draft entropy of every context that has a child */
    for (int32_t c = 0; c < len; ++c) {
        int has = 0;
        for (int32_t n = c; n < len; ++n) if (par[n] == c - 1) has = 1;
        if (!has) continue;
        double lse, H;
        oracle_row_stats(a->draft_logits, a->dtype, ((int64_t)b * N + c) * dld, V, T, &lse, &H, NULL);
        if (a->out_entropy) a->out_entropy[(int64_t)b * N + c] = (float)H;
        if (a->out_entropy64) a->out_entropy64[(int64_t)b * N + c] = H;
    }

    int32_t ctx = 0, depth = 0, next = -1;
    double smargin = NAN;
    const double* final_w = pr;                            /* the weights the final draw was taken from (probe aid) */
    for (;;) {
        const int64_t t_off = ((int64_t)b * (N + 1) + ctx) * tld;
        double lseP, HP;
        oracle_row_stats(a->target_logits, a->dtype, t_off, V, T, &lseP, &HP, NULL);
        for (int32_t i = 0; i < V; ++i) pr[i] = prob_at(a->target_logits, a->dtype, t_off, i, T, lseP);
        int32_t nkids = 0;
        for (int32_t n = ctx; n < len; ++n) if (par[n] == ctx - 1) ++nkids;
        uint32_t rb[4];
        hsd_random_block(a->seed, seq, (uint32_t)ctx, a->level, rb);
        const double u2 = oracle_u24(rb[1]);
        double Zs;
        if (nkids == 0) {                                  /* nothing drafted here: the token is the verifier's */
            next = oracle_inverse_cdf(pr, V, u2, &Zs, &smargin);
            final_w = pr;
            break;
        }
        const int64_t d_off = ((int64_t)b * N + ctx) * dld;
        double lseD, HD;
        oracle_row_stats(a->draft_logits, a->dtype, d_off, V, T, &lseD, &HD, NULL);
        for (int32_t i = 0; i < V; ++i) q[i] = prob_at(a->draft_logits, a->dtype, d_off, i, T, lseD);
        const int gate = (HD < tau) ? 1 : 0;
        if (a->out_gate_margin) a->out_gate_margin[(int64_t)b * N + ctx] = fabs(HD - tau);
        int32_t kept = -1, first = 1, dead = 0, rejected = 0;
        double Zprod = 1.0, Csum = 0.0;
        for (int32_t n = ctx; n < len && kept < 0 && !dead; ++n) {
            if (par[n] != ctx - 1) continue;
            const int32_t x = tok[n];
            int ok;
            if (first && gate) {
                ok = 1;
            } else {
                uint32_t r[4];
                hsd_random_block(a->seed, seq, (uint32_t)n, a->level, r);
                const double u = oracle_u24(r[0]);
                double r_x = 0.0, q_x = 1.0;
                if (x >= 0 && x < V) { r_x = pr[x]; q_x = q[x]; }
                ok = oracle_ratio_accept(u, r_x, q_x);
                if (a->out_ratio_margin && q_x > 0.0)
                    a->out_ratio_margin[(int64_t)b * N + n] = fabs(u - r_x / q_x) * Zprod / (Csum > 1.0 ? Csum : 1.0);
            }
            if (a->force_node && a->force_node[b] == n) ok = a->force_outcome[b] ? 1 : 0;
            first = 0;
            if (ok) { kept = n; break; }
            double z = 0.0;                                /* r <- max(0, r - q) / its sum */
            for (int32_t i = 0; i < V; ++i) { const double d = pr[i] - q[i]; w[i] = d > 0.0 ? d : 0.0; z += w[i]; }
            if (!(z > 0.0)) { dead = 1; break; }
            rejected = 1;
            for (int32_t i = 0; i < V; ++i) pr[i] = w[i] / z;
            Csum += Zprod;
            Zprod *= z;
        }
        if (kept >= 0) {
            if (a->out_path) a->out_path[(int64_t)b * N + depth] = kept;
            ++depth;
            ctx = kept + 1;
            continue;
        }
        if (dead) {                                        /* no residual mass: the verifier's own distribution */
            for (int32_t i = 0; i < V; ++i) pr[i] = prob_at(a->target_logits, a->dtype, t_off, i, T, lseP);
            rejected = 0;
        }
        /* the draw needs no normalised weights: the last residual as it was before its division */
        next = oracle_inverse_cdf(rejected ? w : pr, V, u2, &Zs, &smargin);
        final_w = rejected ? w : pr;
        break;
    }
    if (a->out_probe_lo) a->out_probe_lo[b] = NAN;
    if (a->out_probe_hi) a->out_probe_hi[b] = NAN;
    if (a->probe_token && a->out_probe_lo && a->out_probe_hi && a->probe_token[b] >= 0 && a->probe_token[b] < V) {
        const int32_t t = a->probe_token[b];
        double Z = 0.0, C = 0.0, prev = 0.0;
        for (int32_t i = 0; i < V; ++i) Z += final_w[i];
        for (int32_t i = 0; i <= t; ++i) { prev = C; C += final_w[i]; }
        if (Z > 0.0) { a->out_probe_lo[b] = prev / Z; a->out_probe_hi[b] = C / Z; }
    }
    if (a->out_accept_len) a->out_accept_len[b] = depth;
    if (a->out_next_token) a->out_next_token[b] = next;
    if (a->out_sample_margin) a->out_sample_margin[b] = smargin;
}

/* Returns 0, or -1 on arguments it does not take (a parent that is not an earlier node included). */
int32_t oracle_verify_tree(const oracle_tree_args* a)
{
    if (!a || a->B < 0 || a->N < 1 || a->N > 63 || a->V < 1 || !(a->temperature > 0.f)) return -1;
    if (!a->node_token || !a->node_parent) return -1;
    for (int32_t b = 0; b < a->B; ++b) {
        int32_t len = a->n_nodes ? a->n_nodes[b] : a->N;
        if (len > a->N) len = a->N;
        for (int32_t n = 0; n < len; ++n) {
            const int32_t p = a->node_parent[(int64_t)b * a->N + n];
            if (p < -1 || p >= n) return -1;
        }
    }
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = a->num_threads > 0 ? a->num_threads : omp_get_max_threads();
#endif
    (void)nthreads;
#pragma omp parallel num_threads(nthreads)
    {
        double* buf = (double*)malloc((size_t)a->V * 3 * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < a->B; ++b) tree_one_sequence(a, b, buf, buf + a->V, buf + 2 * (size_t)a->V);
        free(buf);
    }
    return 0;
}

int32_t oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
