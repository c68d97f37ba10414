/*
 * Sanitizer driver for the CPU oracle (test infrastructure).  Linked with hola_oracle.c under
 * -fsanitize=address,undefined by tests/test_sanitizers.py; it calls every entry point of the oracle on small seeded
 * inputs, among them the ragged and degenerate ones (V = 1, empty drafts, tokens outside the vocabulary, masked
 * logits, forced decisions, probes), so that an out-of-bounds access, a use of uninitialised stack arrays beyond
 * their filled part, a signed overflow or a misaligned access in the oracle ends the run with a report.
 * It checks no values: the pins do that.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const void* target_logits; const void* draft_logits; int32_t dtype; int64_t target_ld, draft_ld;
    const int32_t* draft_tokens; const int32_t* draft_len; const float* row_temperature; const int32_t* force_accept_len;
    uint64_t seed; uint32_t level; int64_t seq_base; int32_t B, gamma, V; float temperature, entropy_threshold;
    int32_t* out_accept_len; int32_t* out_next_token; float* out_entropy; double* out_entropy64; double* out_lse_draft;
    double* out_lse_target; double* out_H_target; uint8_t* out_gate; uint8_t* out_ratio_ok; double* out_gate_margin;
    double* out_ratio_margin; double* out_sample_margin; double* out_Z; int32_t num_threads;
} verify_args;

typedef struct {
    const void* target_logits; const void* draft_logits; int32_t dtype; int64_t target_ld, draft_ld;
    const int32_t* node_token; const int32_t* node_parent; const int32_t* n_nodes;
    uint64_t seed; uint32_t level; int64_t seq_base; int32_t B, N, V; float temperature, entropy_threshold;
    int32_t* out_accept_len; int32_t* out_path; int32_t* out_next_token; float* out_entropy; double* out_entropy64;
    double* out_gate_margin; double* out_ratio_margin; double* out_sample_margin; int32_t num_threads;
    const int32_t* force_node; const int32_t* force_outcome; const int32_t* probe_token; double* out_probe_lo; double* out_probe_hi;
} tree_args;

int32_t oracle_verify(const verify_args*);
int32_t oracle_verify_filtered(const verify_args*, int32_t, double, double*, int32_t*, const int32_t*);
int32_t oracle_sample_interval(const verify_args*, int32_t, int32_t, int32_t, double*, double*);
int32_t oracle_sample_interval_filtered(const verify_args*, int32_t, double, const int32_t*, int32_t, int32_t, int32_t, double*, double*);
int32_t oracle_row_interval(const void*, int32_t, int64_t, int32_t, double, int32_t, double*, double*);
int32_t oracle_verify_literal(const verify_args*, int32_t*, int32_t*, double*, const int8_t*);
int32_t oracle_verify_tree(const tree_args*);
int32_t oracle_hsd_verify(const void* const*, const int64_t*, int32_t, int32_t, const int32_t*, uint64_t, int64_t, int32_t,
                          int32_t, int32_t, const float*, float, const float*, int32_t*, int32_t*, int32_t*, float*, int32_t*,
                          int32_t*, int32_t, int32_t, double, int32_t);
void oracle_merge_tile_stats(const double*, int32_t, double*, double*);
void oracle_row_stats(const void*, int32_t, int64_t, int32_t, double, double*, double*, int32_t*);

static uint64_t g_state = 88172645463325252ull;
static double rnd(void)                                  /* xorshift64*, uniform in [0, 1) */
{
    g_state ^= g_state >> 12; g_state ^= g_state << 25; g_state ^= g_state >> 27;
    return (double)((g_state * 2685821657736338717ull) >> 11) * (1.0 / 9007199254740992.0);
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(1.0 - rnd())) * cos(6.283185307179586 * rnd())); }

static void* fill_logits(int64_t n, int32_t dtype, double mask_prob)
{
    if (dtype == 0) {
        float* p = (float*)malloc((size_t)n * sizeof(float));
        for (int64_t i = 0; i < n; ++i) p[i] = rnd() < mask_prob ? -INFINITY : 2.0f * gauss();
        return p;
    }
    uint16_t* p = (uint16_t*)malloc((size_t)n * sizeof(uint16_t));
    for (int64_t i = 0; i < n; ++i) {
        float f = rnd() < mask_prob ? -INFINITY : 2.0f * gauss();
        uint32_t bits; memcpy(&bits, &f, 4);
        p[i] = (uint16_t)(bits >> 16);
    }
    return p;
}

static int one_level(int32_t B, int32_t g, int32_t V, int32_t dtype, double mask_prob, int ragged)
{
    void* P = fill_logits((int64_t)B * (g + 1) * V, dtype, mask_prob);
    void* D = fill_logits((int64_t)B * g * V, dtype, mask_prob);
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * B * g);
    int32_t* len = (int32_t*)malloc(sizeof(int32_t) * B);
    float* rowT = (float*)malloc(sizeof(float) * B);
    for (int i = 0; i < B * g; ++i) tok[i] = (int32_t)(rnd() * (V + 2)) - 1;     /* -1 and V occur */
    for (int b = 0; b < B; ++b) { len[b] = ragged ? (int32_t)(rnd() * (g + 1)) : g; rowT[b] = (b % 3 == 0) ? 0.f : 0.8f; }
    int32_t* acc = (int32_t*)malloc(sizeof(int32_t) * B); int32_t* nxt = (int32_t*)malloc(sizeof(int32_t) * B);
    float* ent = (float*)malloc(sizeof(float) * B * g); double* ent64 = (double*)malloc(sizeof(double) * B * g);
    double* lsd = (double*)malloc(sizeof(double) * B * g); double* lst = (double*)malloc(sizeof(double) * B * (g + 1));
    double* Ht = (double*)malloc(sizeof(double) * B * (g + 1));
    uint8_t* gate = (uint8_t*)malloc(B * g); uint8_t* rok = (uint8_t*)malloc(B * g);
    double* gm = (double*)malloc(sizeof(double) * B * g); double* rm = (double*)malloc(sizeof(double) * B * g);
    double* sm = (double*)malloc(sizeof(double) * B); double* Z = (double*)malloc(sizeof(double) * B);
    verify_args a; memset(&a, 0, sizeof a);
    a.target_logits = P; a.draft_logits = D; a.dtype = dtype; a.draft_tokens = tok; a.draft_len = ragged ? len : NULL;
    a.seed = 12345; a.level = 2; a.seq_base = ((int64_t)1 << 33) + 5; a.B = B; a.gamma = g; a.V = V;
    a.temperature = 0.9f; a.entropy_threshold = (float)(0.4 * log((double)(V > 1 ? V : 2)));
    a.out_accept_len = acc; a.out_next_token = nxt; a.out_entropy = ent; a.out_entropy64 = ent64; a.out_lse_draft = lsd;
    a.out_lse_target = lst; a.out_H_target = Ht; a.out_gate = gate; a.out_ratio_ok = rok; a.out_gate_margin = gm;
    a.out_ratio_margin = rm; a.out_sample_margin = sm; a.out_Z = Z; a.num_threads = 2;
    int rc = oracle_verify(&a);
    a.row_temperature = rowT;                               /* greedy rows mixed in */
    rc |= oracle_verify(&a);
    a.row_temperature = NULL;
    int32_t* force = (int32_t*)malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b) force[b] = (b & 1) ? -1 : (ragged ? len[b] : g);
    a.force_accept_len = force;
    rc |= oracle_verify(&a);
    a.force_accept_len = NULL;
    double lo, hi;
    for (int b = 0; b < B; ++b) {
        (void)oracle_sample_interval(&a, b, acc[b], nxt[b] < 0 ? 0 : nxt[b], &lo, &hi);
        (void)oracle_sample_interval(&a, b, 0, V - 1, &lo, &hi);
        (void)oracle_sample_interval(&a, b, 0, V, &lo, &hi);            /* refused */
    }
    /* filtered step, keep counts forced on some rows, intervals */
    const int R = 2 * g + 1;
    double* fm = (double*)malloc(sizeof(double) * B * R); int32_t* kc = (int32_t*)malloc(sizeof(int32_t) * B * R);
    int32_t* fk = (int32_t*)malloc(sizeof(int32_t) * B * R);
    const int32_t ks[3] = {0, 3, V + 5}; const double ps[3] = {0.9, 1.0, 0.05};
    for (int i = 0; i < 3; ++i) {
        rc |= oracle_verify_filtered(&a, ks[i], ps[i], fm, kc, NULL);
        for (int j = 0; j < B * R; ++j) fk[j] = (j % 4 == 0) ? 1 : ((j % 4 == 1) ? V + 3 : -1);
        rc |= oracle_verify_filtered(&a, ks[i], ps[i], fm, kc, fk);
        for (int b = 0; b < B; ++b)
            (void)oracle_sample_interval_filtered(&a, ks[i], ps[i], fk, b, acc[b], nxt[b] < 0 ? 0 : nxt[b], &lo, &hi);
    }
    /* Equation (1) literal mode with forced gates */
    int32_t* lt = (int32_t*)malloc(sizeof(int32_t) * B * g); int32_t* calls = (int32_t*)malloc(sizeof(int32_t) * B);
    int8_t* fg = (int8_t*)malloc(B * g);
    for (int i = 0; i < B * g; ++i) fg[i] = (int8_t)(i % 3 - 1);
    rc |= oracle_verify_literal(&a, lt, calls, gm, NULL);
    rc |= oracle_verify_literal(&a, lt, calls, gm, fg);
    a.row_temperature = rowT;
    rc |= oracle_verify_literal(&a, lt, calls, NULL, NULL);
    (void)oracle_row_interval(P, dtype, 0, V, 0.7, V - 1, &lo, &hi);
    (void)oracle_row_interval(P, dtype, 0, V, 0.7, -1, &lo, &hi);
    free(P); free(D); free(tok); free(len); free(rowT); free(acc); free(nxt); free(ent); free(ent64); free(lsd); free(lst);
    free(Ht); free(gate); free(rok); free(gm); free(rm); free(sm); free(Z); free(force); free(fm); free(kc); free(fk);
    free(lt); free(calls); free(fg);
    return rc;
}

static int hierarchy(int32_t n_models, int32_t B, int32_t g, int32_t V, int32_t dtype)
{
    const void* models[8];
    for (int k = 0; k < n_models; ++k) models[k] = fill_logits((int64_t)B * (g + k) * V, dtype, 0.05);
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * B * g);
    for (int i = 0; i < B * g; ++i) tok[i] = (int32_t)(rnd() * V);
    float tau[8];
    for (int k = 0; k < n_models - 1; ++k) tau[k] = (float)(0.2 * (k + 1) * log((double)V));
    const int L = n_models - 1, gmax = g + L - 1;
    int32_t* ot = (int32_t*)malloc(sizeof(int32_t) * B * (g + L)); int32_t* acc = (int32_t*)malloc(sizeof(int32_t) * B);
    int32_t* nxt = (int32_t*)malloc(sizeof(int32_t) * B); float* ent = (float*)malloc(sizeof(float) * L * B * gmax);
    int32_t* la = (int32_t*)malloc(sizeof(int32_t) * L * B); int32_t* ln = (int32_t*)malloc(sizeof(int32_t) * L * B);
    int rc = 0;
    for (int so = 0; so < 2; ++so) {
        rc |= oracle_hsd_verify(models, NULL, n_models, dtype, tok, 7, 3, B, g, V, NULL, 1.0f, tau, ot, acc, nxt, ent, la, ln, so, 0, 1.0, 2);
        rc |= oracle_hsd_verify(models, NULL, n_models, dtype, tok, 7, 3, B, g, V, NULL, 1.0f, tau, ot, acc, nxt, ent, NULL, NULL, so, 5, 0.9, 1);
    }
    for (int k = 0; k < n_models; ++k) free((void*)models[k]);
    free(tok); free(ot); free(acc); free(nxt); free(ent); free(la); free(ln);
    return rc;
}

static int tree(int32_t B, int32_t N, int32_t V, int32_t dtype)
{
    void* P = fill_logits((int64_t)B * (N + 1) * V, dtype, 0.02);
    void* D = fill_logits((int64_t)B * N * V, dtype, 0.02);
    int32_t* tok = (int32_t*)malloc(sizeof(int32_t) * B * N); int32_t* par = (int32_t*)malloc(sizeof(int32_t) * B * N);
    int32_t* nn = (int32_t*)malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b) {
        nn[b] = (int32_t)(rnd() * (N + 1));
        for (int n = 0; n < N; ++n) { tok[b * N + n] = (int32_t)(rnd() * (V + 2)) - 1; par[b * N + n] = (int32_t)(rnd() * (n + 1)) - 1; }
    }
    int32_t* acc = (int32_t*)malloc(sizeof(int32_t) * B); int32_t* path = (int32_t*)malloc(sizeof(int32_t) * B * N);
    int32_t* nxt = (int32_t*)malloc(sizeof(int32_t) * B); float* ent = (float*)malloc(sizeof(float) * B * N);
    double* e64 = (double*)malloc(sizeof(double) * B * N); double* gm = (double*)malloc(sizeof(double) * B * N);
    double* rm = (double*)malloc(sizeof(double) * B * N); double* sm = (double*)malloc(sizeof(double) * B);
    int32_t* fn = (int32_t*)malloc(sizeof(int32_t) * B); int32_t* fo = (int32_t*)malloc(sizeof(int32_t) * B);
    int32_t* pt = (int32_t*)malloc(sizeof(int32_t) * B); double* plo = (double*)malloc(sizeof(double) * B);
    double* phi = (double*)malloc(sizeof(double) * B);
    tree_args a; memset(&a, 0, sizeof a);
    a.target_logits = P; a.draft_logits = D; a.dtype = dtype; a.node_token = tok; a.node_parent = par; a.n_nodes = nn;
    a.seed = 99; a.level = 1; a.seq_base = 17; a.B = B; a.N = N; a.V = V; a.temperature = 0.8f;
    a.entropy_threshold = (float)(0.3 * log((double)(V > 1 ? V : 2)));
    a.out_accept_len = acc; a.out_path = path; a.out_next_token = nxt; a.out_entropy = ent; a.out_entropy64 = e64;
    a.out_gate_margin = gm; a.out_ratio_margin = rm; a.out_sample_margin = sm; a.num_threads = 2;
    int rc = oracle_verify_tree(&a);
    for (int b = 0; b < B; ++b) { fn[b] = (b & 1) ? -1 : (int32_t)(rnd() * N); fo[b] = b & 2 ? 1 : 0; pt[b] = (b % 3) ? (int32_t)(rnd() * V) : -1; }
    a.force_node = fn; a.force_outcome = fo; a.probe_token = pt; a.out_probe_lo = plo; a.out_probe_hi = phi;
    rc |= oracle_verify_tree(&a);
    a.n_nodes = NULL;
    rc |= oracle_verify_tree(&a);
    free(P); free(D); free(tok); free(par); free(nn); free(acc); free(path); free(nxt); free(ent); free(e64); free(gm);
    free(rm); free(sm); free(fn); free(fo); free(pt); free(plo); free(phi);
    return rc;
}

int main(void)
{
    int rc = 0;
    const int32_t shapes[][3] = {{1, 1, 1}, {3, 1, 7}, {2, 2, 8}, {5, 3, 101}, {4, 63, 19}, {2, 5, 1000}};
    for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
        for (int32_t dtype = 0; dtype < 2; ++dtype)
            for (int ragged = 0; ragged < 2; ++ragged)
                rc |= one_level(shapes[i][0], shapes[i][1], shapes[i][2], dtype, i % 2 ? 0.3 : 0.0, ragged);
    rc |= hierarchy(2, 4, 3, 33, 0);
    rc |= hierarchy(4, 5, 2, 40, 1);
    rc |= hierarchy(3, 2, 61, 9, 0);                        /* widest level at the limit of 63 drafted positions */
    rc |= tree(6, 1, 5, 0);
    rc |= tree(9, 12, 64, 1);
    rc |= tree(3, 63, 11, 0);
    double ts[8] = {-INFINITY, NAN, 0.3, 1.1, -INFINITY, 5.0, 2.0, 0.5}, lse, H;
    oracle_merge_tile_stats(ts, 4, &lse, &H);
    float row[4] = {INFINITY, 0.f, -1.f, NAN};
    oracle_row_stats(row, 0, 0, 4, 1.0, &lse, &H, NULL);
    printf("oracle sanitizer driver: rc=%d\n", rc);
    return rc ? 1 : 0;
}
