/*
 * hola.h -- C ABI of libhola.so: the batched verify step of HOLA's Hierarchical
 * Speculative Decoding (HSD) on one AMD MI355X (gfx950).
 *
 * What one call computes, for B sequences each carrying gamma drafted tokens over a
 * vocabulary of V entries (paper Section 3.1 "HSD Module", Algorithm 1 Step 1, Equation (1)):
 *
 *   1. p = softmax(target_logits / T) and q = softmax(draft_logits / T) per position
 *      (temperature scaling is not in the paper; T = 1 reproduces it);
 *   2. the entropy of the DRAFT distribution, H = -sum_i q_i ln q_i, per position
 *      (Section 3.1; natural log, so the threshold is in nats);
 *   3. the entropy gate g = 1[H < tau], strict (Algorithm 1 Step 1; Section 4.3 for tau);
 *   4. Equation (1): gate = 1 keeps the drafted token without consulting the verifier;
 *      gate = 0 falls back to the verifier, here the draft-and-verify acceptance test
 *      u * q(x) < p(x) with u uniform on [0,1);
 *   5. the first position that is neither gated nor accepted ends the sequence
 *      (accept_len = number of drafts kept);
 *   6. the next token: at a rejection, drawn by inverse CDF from max(0, p - q) / Z at that
 *      position; when all drafts were kept, a bonus token drawn from p at position len;
 *   7. "Hierarchical": the kept tokens plus the next token of one level are the drafts of
 *      the next level, verified by the next larger model (hola_hsd_verify).
 * Beyond the paper's step, declared further down with their own definitions: top-k / top-p filtered
 * distributions (hola_verify_args.top_k / top_p), Equation (1) taken literally (hola_verify_literal_ex),
 * several drafted candidates per position (hola_verify_tree), statistics by column tiles (hola_tile_stats,
 * hola_merge_tile_stats).
 *
 * Uniforms: Philox4x32-10 with key = (seed low, seed high) and counter =
 * (position, sequence low, sequence high, level), sequence = seq_base + b; output word 0
 * drives the acceptance test of that position, word 1 the sample taken at that position;
 * each is reduced to 24 bits, u = (word >> 8) * 2^-24.
 *
 * Layout.  All tensors are row-major and contiguous unless a leading dimension is given:
 *   target_logits [B, gamma+1, V]   (row gamma is the bonus position)
 *   draft_logits  [B, gamma,   V]
 *   draft_tokens  [B, gamma]        int32
 *   out_accept_len[B], out_next_token[B]  int32;  out_entropy [B, gamma] float (nats)
 * bf16 logits are passed as raw 16-bit patterns.  gamma <= HOLA_MAX_GAMMA = 63.
 *
 * Ownership and memory spaces.  Every pointer named "device" is caller-owned DEVICE memory
 * (for PyTorch: tensor.data_ptr()); host pointers are marked "host".  The library never
 * frees caller memory.  hola_verify_f32 / hola_verify_bf16 use one library-owned workspace
 * per device, allocated on first use and grown when a larger shape arrives (hipMalloc, which
 * synchronises the device; not on the steady-state path), released by hola_shutdown().  Because
 * that workspace is shared, the two short forms are for ONE stream and ONE calling thread per
 * device at a time: calls that overlap on a device race on it.  hola_verify_ex, hola_hsd_verify
 * and the other forms that take a workspace use the caller's only, never allocate, and are
 * reentrant across threads and streams when each call in flight has a workspace of its own.
 * Launch-shape defaults (hola_set_tuning) and the timing aid (hola_profile_*) belong to the
 * calling thread.
 *
 * Asynchrony.  All work is enqueued on `stream`; nothing synchronises with the host.
 * Outputs are valid once the stream has been synchronised; inputs and the workspace must
 * stay alive and unmodified until then.  Calls sharing a workspace must be on one stream
 * (or otherwise ordered).
 *
 * Errors.  Return codes only.  Argument errors (a required pointer NULL, B < 0, gamma < 1 or
 * > HOLA_MAX_GAMMA, V < 1, a negative or NaN temperature, NaN tau, a leading dimension < V, a logits
 * pointer not aligned to its element size, a workspace that is too small or not 256-byte
 * aligned) are detected on the host before any launch and leave the outputs untouched.
 * HIP launch or allocation failures return HOLA_ERR_HIP; hola_last_hip_error() names the last
 * one seen by the calling thread.  B == 0 is a successful no-op.
 * Data problems cannot be reported synchronously: a drafted token outside [0, V) has
 * p(x) = 0 (never ratio-accepted, still gate-acceptable); a target row with no finite
 * probability mass yields next_token = -1; -inf logits are allowed (masked vocabulary);
 * +inf or NaN logits give NaN statistics for that row (never a fault).
 */
#ifndef HOLA_H
#define HOLA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t* hola_stream_t;   /* == hipStream_t; NULL is the default stream */

typedef enum {
    HOLA_OK = 0,
    HOLA_ERR_INVALID_ARG = 1,
    HOLA_ERR_UNSUPPORTED = 2,
    HOLA_ERR_WORKSPACE = 3,
    HOLA_ERR_HIP = 4
} hola_status;

enum { HOLA_DTYPE_F32 = 0, HOLA_DTYPE_BF16 = 1 };
enum { HOLA_MAX_GAMMA = 63 };   /* drafted positions (or tree nodes) per sequence: one lane of a wavefront each */

/* One verify level on float logits.  Steps 1-6 above with a single temperature (> 0) and
 * threshold; seq_base = 0, level = 0.  All pointers device; stream may be NULL. */
hola_status hola_verify_f32(const float* target_logits, const float* draft_logits,
                            const int32_t* draft_tokens, uint64_t seed,
                            int32_t B, int32_t gamma, int32_t V,
                            float temperature, float entropy_threshold,
                            int32_t* out_accept_len, int32_t* out_next_token, float* out_entropy,
                            hola_stream_t stream);

/* Same on bfloat16 logits given as raw 16-bit patterns. */
hola_status hola_verify_bf16(const uint16_t* target_logits, const uint16_t* draft_logits,
                             const int32_t* draft_tokens, uint64_t seed,
                             int32_t B, int32_t gamma, int32_t V,
                             float temperature, float entropy_threshold,
                             int32_t* out_accept_len, int32_t* out_next_token, float* out_entropy,
                             hola_stream_t stream);

/* Launch-shape knobs.  Zero in a field keeps the built-in choice for MI355X.  Every setting computes the same
 * decisions; only partial sums are grouped differently (entropies may differ in the last bits). */
typedef struct {
    int32_t stats_split;            /* workgroups per logits row in the split-row statistics kernel (1..16) */
    int32_t stats_unroll;           /* 16-byte loads in flight per lane while streaming a row: 2, 4, 8 or 16 */
    int32_t path;                   /* 1: split-row statistics + per-sequence tail kernel (2 launches);
                                       2: fused per-sequence kernel (1 launch; gamma <= 32, else as 1);
                                       3: split-row statistics, accept, tile sums, select (4 launches);
                                       0: the library's choice for the shape (path 1 whenever the
                                          per-sequence kernels support it, else path 3) */
    int32_t fused_waves;            /* wavefronts per workgroup of the per-sequence kernels: 4 (tail kernel
                                       only; the fused kernel then uses 8), 8 or 16; 0: 16 for the fused
                                       kernel, and for the tail kernel 16 / 8 / 4 as the batch grows past
                                       one / three sequences per compute unit */
    int32_t filter_path;            /* top-k / top-p keep sets.  0: a split-row scan lists the candidates of every
                                       row, one wavefront per row decides, and only rows that step cannot settle
                                       go to the one-workgroup-per-row kernel; 1: that kernel for every row */
    int32_t tail_split;             /* workgroups that share one sequence's tail (the sweep of its stop rows): 1, 2, 4
                                       or 8; 0: the library's choice (more than one only for small batches of wide
                                       rows, where compute units would otherwise idle while one of them sweeps).  A
                                       wish: where B * tail_split exceeds the compute units, or the call is filtered,
                                       one workgroup is used.  The result does not depend on it. */
} hola_tuning;
/* Sets the defaults of the CALLING THREAD (thread-local; NULL restores the built-in choices).  A call whose args
 * structure carries its own `tuning` ignores them, so no state outside a call's arguments need decide its path. */
hola_status hola_set_tuning(const hola_tuning* t /* host; NULL restores defaults */);

/* Extended form of one verify level. */
typedef struct {
    const void* target_logits;      /* device [B, gamma+1, V] */
    const void* draft_logits;       /* device [B, gamma,   V] */
    int32_t dtype;                  /* HOLA_DTYPE_F32 | HOLA_DTYPE_BF16 */
    int64_t target_ld, draft_ld;    /* row stride in elements, >= V; 0 => V */
    const int32_t* draft_tokens;    /* device [B, gamma] */
    const int32_t* draft_len;       /* device [B], each in [0, gamma]; NULL => gamma everywhere */
    const float* row_temperature;   /* device [B]; NULL => `temperature` everywhere.  An entry of
                                       0 marks a greedy row: accept iff token == argmax(target) (lowest
                                       index on ties), next token = argmax at the stop row, gate entropy
                                       taken at T = 1 */
    const double* draft_stats_in;   /* device [B, gamma, 2] = (lse, H) of the draft rows in nats, as a
                                       previous level's target_stats_out produced them; NULL => computed
                                       here.  When given, the draft rows are read only for the gathers and
                                       at the stop row */
    double* target_stats_out;       /* device [B, gamma+1, 2] = (lse, H) of the target rows j <= len;
                                       NULL => not wanted */
    const double* target_stats_in;  /* device [B, gamma+1, 2] = (lse, H) of the target rows in nats (H is not
                                       used), e.g. merged from the tile statistics of the LM head that
                                       produced the logits (hola_merge_tile_stats); NULL => computed here.
                                       With draft_stats_in also given no logits row is streamed: the call
                                       reads only the gathered logits of the drafted tokens and the stop
                                       rows.  Needs temperature > 0 and row_temperature == NULL (the
                                       statistics carry no argmax for greedy rows), else
                                       HOLA_ERR_UNSUPPORTED; also unsupported above 2048 sampler tiles per row */
    int32_t top_k;                  /* > 0: both models' distributions are truncated to their top_k largest
                                       logits (equal logits: lower index first) and renormalised before the
                                       gate entropy, the acceptance test and the residual; 0 or >= V: off */
    float top_p;                    /* in (0, 1): after top_k, keep the shortest prefix of the tokens in
                                       descending order whose probability reaches top_p of the top_k mass
                                       (at least one token), renormalised; 0 or >= 1: off.  With either filter
                                       on: temperature > 0, row_temperature / draft_stats_in / target_stats_in
                                       / target_stats_out NULL, V < 2^22 and at most 2048 sampler tiles per
                                       row, else HOLA_ERR_UNSUPPORTED; out_entropy is the entropy of the
                                       filtered draft distribution */
    int32_t* out_keep_count;        /* device [B, 2*gamma+1] or NULL; written only with a filter on: the
                                       number of tokens kept in draft rows 0..gamma-1, then in target rows
                                       0..gamma, of each sequence; -1 for rows the call does not use */
    uint64_t seed;
    uint32_t level;                 /* Philox counter word 3 */
    int64_t seq_base;               /* global index of sequence 0 of this call (Philox counter words 1,2) */
    int32_t B, gamma, V;
    float temperature;              /* >= 0; used where row_temperature is NULL */
    float entropy_threshold;        /* tau, nats.  tau <= 0 never gates; +inf gates everything */
    int32_t* out_accept_len;        /* device [B] */
    int32_t* out_next_token;        /* device [B] */
    float* out_entropy;             /* device [B, entropy_ld]: draft entropy for j < len, -1 beyond; NULL ok */
    int64_t entropy_ld;             /* row stride of out_entropy in elements, >= gamma; 0 => gamma */
    void* workspace;                /* device, 256-byte aligned, >= hola_workspace_bytes_ex(this) */
    size_t workspace_bytes;
    hola_stream_t stream;
    const hola_tuning* tuning;      /* host; launch shape of this call, NULL => the calling thread's defaults */
} hola_verify_args;

/* Bytes of workspace that any hola_verify_ex call of this shape can need (either dtype, filters on or off);
 * 0 on invalid shape. */
size_t hola_workspace_bytes(int32_t B, int32_t gamma, int32_t V);

/* Bytes of workspace this very call needs, <= hola_workspace_bytes(B, gamma, V): the candidate lists of the top-k /
 * top-p filters (most of the larger figure: 16 KB per logits row) are counted only when a filter is on.  Reads B,
 * gamma, V, top_k and top_p; 0 on NULL or an invalid shape. */
size_t hola_workspace_bytes_ex(const hola_verify_args* args /* host */);

hola_status hola_verify_ex(const hola_verify_args* args /* host */);

/* hola_verify_ex for callers that cannot allocate device memory and have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  args->workspace and workspace_bytes
 * are ignored; the workspace is an array of HOLA_STATIC_SCRATCH_BYTES in the library's device image (each GPU the
 * library runs on holds its copy until the process ends).  The call allocates and frees nothing (keep the timing
 * aid off: it creates events) and enqueues the same kernels as hola_verify_ex, so the outputs are bit-identical.
 * HOLA_ERR_WORKSPACE when hola_workspace_bytes_ex(args) exceeds HOLA_STATIC_SCRATCH_BYTES (the headline shape
 * B=256, gamma=8 needs 9 MB and fits; filtered calls need 16 KB more per logits row and fit up to ~900 rows);
 * other errors as hola_verify_ex.  Nothing in the array has to start at zero and no call relies on what an
 * earlier one left there, but every call on a GPU uses that GPU's one array: calls that overlap on a GPU (two
 * streams, two threads) race on it. */
enum { HOLA_STATIC_SCRATCH_BYTES = 16 << 20 };
hola_status hola_verify_ex_static(const hola_verify_args* args /* host */);

/* Equation (1) of the paper taken literally, as an alternative to steps 4-6: no ratio test and no stop.
 * For every drafted position t < len, y_t = the drafted token if H(draft_t) < tau, otherwise
 * f_ver(x, draft_<t): a draw from softmax(target_logits[b, t] / T) with the sampling uniform of position t
 * (the argmax on greedy rows).  Target row gamma is not read.  args is used as in hola_verify_ex except that
 * out_accept_len / out_next_token are ignored (may be NULL) and draft_stats_in / target_stats_out must be
 * NULL.  out_tokens: device [B, gamma], -1 beyond draft_len.  out_verifier_calls: device [B] or NULL, the
 * number of positions that fell back to the verifier (the k of Section 3.1).  HOLA_ERR_UNSUPPORTED above
 * 2048 sampler tiles per row (V > 4.2 M bf16 / 2.1 M float). */
hola_status hola_verify_literal_ex(const hola_verify_args* args /* host */, int32_t* out_tokens, int32_t* out_verifier_calls);

/* Hierarchical driver (step 7).  models[0] is the smallest drafter, models[n_models-1] the
 * target; n_models - 1 verify levels.  models[k].logits is device [B, gamma+k, V].
 * Level k (1-based) verifies with models[k] the drafts level k-1 produced (its kept tokens
 * followed by its next token; level 1 takes draft_tokens), gated by tau[k-1] on the entropy of
 * models[k-1], with Philox level word k-1.  The statistics of each middle model are computed
 * once, when it is the target, and reused when it is the draft. */
typedef struct {
    const void* logits;             /* device */
    int64_t ld;                     /* row stride in elements; 0 => V */
} hola_model_logits;

hola_status hola_hsd_verify(const hola_model_logits* models /* host array */, int32_t n_models, int32_t dtype,
                            const int32_t* draft_tokens /* device [B, gamma], drawn from models[0] */,
                            uint64_t seed, int64_t seq_base, int32_t B, int32_t gamma, int32_t V,
                            const float* row_temperature /* device [B] or NULL */, float temperature,
                            const float* tau /* host array [n_models-1] */,
                            int32_t* out_tokens     /* device [B, gamma+n_models-1]: the last level's drafts, -1 beyond */,
                            int32_t* out_accept_len /* device [B], last level */,
                            int32_t* out_next_token /* device [B], last level */,
                            float* out_entropy      /* device [n_models-1, B, gamma+n_models-2], -1 where unused; NULL ok */,
                            void* workspace, size_t workspace_bytes, hola_stream_t stream);

size_t hola_hsd_workspace_bytes(int32_t n_models, int32_t B, int32_t gamma, int32_t V);

/* The same driver with its options in a struct.  survivors_only = 1 selects the other reading of "the
 * target verifies the survivors": level k passes on only the tokens it kept (length accept_len, possibly
 * 0), not its next token; that chain conditions on acceptance and is not lossless, it is offered because
 * the paper does not say which one HSD means.  Every other field is as in hola_hsd_verify. */
typedef struct {
    const hola_model_logits* models;  /* host array [n_models] */
    int32_t n_models, dtype;
    const int32_t* draft_tokens;      /* device [B, gamma] */
    uint64_t seed; int64_t seq_base;
    int32_t B, gamma, V;
    const float* row_temperature;     /* device [B] or NULL */
    float temperature;
    const float* tau;                 /* host array [n_models-1] */
    int32_t survivors_only;
    int32_t* out_tokens;              /* device [B, gamma+n_models-1] or NULL */
    int32_t* out_accept_len; int32_t* out_next_token;   /* device [B] */
    float* out_entropy;               /* device [n_models-1, B, gamma+n_models-2] or NULL */
    void* workspace; size_t workspace_bytes; hola_stream_t stream;
    int32_t top_k; float top_p;       /* as in hola_verify_args, applied to both models of every level (0 / 0: off).
                                         A middle model's keep sets and filtered statistics are found once, at the
                                         level where it is the target, and handed to the level where it is the draft,
                                         as the unfiltered statistics are.  Needs row_temperature == NULL. */
    const hola_tuning* tuning;        /* host; launch shape of every level, NULL => the calling thread's defaults */
} hola_hsd_args;
hola_status hola_hsd_verify_ex(const hola_hsd_args* args /* host */);

/* Token trees: several drafted tokens per position (the paper drafts one; Section 3.1's gate and
 * Equation (1)'s two branches carry over as stated below).  A sequence has N nodes; node n holds a token and
 * a parent, -1 (the prefix) or an earlier node.  Context c is the prefix (c = 0) or the prefix followed by the
 * path to node c - 1; target row c and draft row c are the two models' logits after context c, laid out as
 * for hola_verify_ex with gamma = N (draft rows of contexts without children are never read).  From the
 * prefix on, the children of the current context are tried in node order: with H(q_c) < tau (strict) the
 * first child is kept without a test; otherwise child x is kept iff u q_c(x) < r(x), r = p_c at first and
 * after every rejection r <- max(0, r - q_c) renormalised (the rule for candidates drawn independently from
 * q_c, under which the kept token follows p_c whatever their number).  A kept child becomes the context; when
 * every child is rejected the next token is drawn from r, and at a context without children from p_c.
 * A chain (parent[n] = n - 1) gives exactly hola_verify_ex's results, uniforms included: node n's test takes
 * word 0 of Philox block (n, seq, level), the draw at context c word 1 of block (c, seq, level).
 * A node whose parent is neither -1 nor an earlier node is ignored, like the nodes beyond n_nodes[b].
 * Stochastic rows with one temperature > 0 only (HOLA_ERR_UNSUPPORTED otherwise); N <= HOLA_MAX_GAMMA.
 * All pointers but the struct itself are device memory; outputs are written on `stream`; the caller owns
 * every buffer; workspace: 256-byte aligned, >= hola_tree_workspace_bytes(B, N, V). */
typedef struct {
    const void* target_logits;        /* [B, N+1, V] */
    const void* draft_logits;         /* [B, N, V] */
    int32_t dtype;                    /* HOLA_DTYPE_* */
    int64_t target_ld, draft_ld;      /* row strides in elements, 0 = V */
    const int32_t* node_token;        /* [B, N] */
    const int32_t* node_parent;       /* [B, N] */
    const int32_t* n_nodes;           /* [B] in [0, N], or NULL = N */
    uint64_t seed; uint32_t level; int64_t seq_base;
    int32_t B, N, V;
    float temperature, entropy_threshold;
    int32_t* out_accept_len;          /* [B] number of kept nodes */
    int32_t* out_path;                /* [B, N] kept nodes from the prefix on, -1 beyond; or NULL */
    int32_t* out_next_token;          /* [B]; -1 if the stop row has no finite logit */
    float* out_entropy;               /* [B, N] H(q_c) in nats for contexts with children, -1 elsewhere; or NULL */
    void* workspace; size_t workspace_bytes; hola_stream_t stream;
    const hola_tuning* tuning;        /* host; NULL => the calling thread's defaults (stats_split, stats_unroll, fused_waves) */
} hola_tree_args;
hola_status hola_verify_tree(const hola_tree_args* args /* host */);
size_t hola_tree_workspace_bytes(int32_t B, int32_t N, int32_t V);   /* 0 on invalid shape */

/* Row statistics alone (steps 1-2): (lse, H) in nats of softmax(logits[r, :] / T) for R rows,
 * written to stats_out as device [R, 2] doubles.  Greedy convention does not apply (T > 0).
 * workspace as for hola_verify_ex with B = R, gamma = 1. */
hola_status hola_row_stats(const void* logits /* device [R, V] */, int32_t dtype, int64_t ld,
                           int32_t R, int32_t V, float temperature,
                           double* stats_out /* device [R, 2] */,
                           void* workspace, size_t workspace_bytes, hola_stream_t stream);

/* Vocabulary-tiled statistics: what the epilogue of a vocabulary-tiled LM-head GEMM, or each rank of a
 * vocabulary-sharded head, can compute from the tile of logits it holds, and their merge.  For row r and
 * column tile t = [t * tile_cols, min(V, (t+1) * tile_cols)), tile_stats_out[r, t] = (lse_t, H_t): the
 * log-sum-exp and the entropy (Section 3.1, nats) of softmax(logits[r, tile] / T) taken over the tile alone;
 * a tile with no finite logit gives (-inf, NaN).  ntiles = ceil(V / tile_cols).  Tiles need no alignment.
 * workspace: device, 256-byte aligned, >= hola_tile_stats_workspace_bytes(R, V, tile_cols). */
hola_status hola_tile_stats(const void* logits /* device [R, V] */, int32_t dtype, int64_t ld,
                            int32_t R, int32_t V, int32_t tile_cols, float temperature /* > 0 */,
                            double* tile_stats_out /* device [R, ntiles, 2] */,
                            void* workspace, size_t workspace_bytes, hola_stream_t stream);
size_t hola_tile_stats_workspace_bytes(int32_t R, int32_t V, int32_t tile_cols);   /* 0 on invalid shape */

/* Row statistics from tile statistics: the row's distribution is the mixture of its tiles' with weights
 * w_t = exp(lse_t - lse), so lse = ln sum_t exp(lse_t) and, by Section 3.1's definition of the entropy,
 * H = sum_t w_t (H_t - ln w_t).  Tiles with lse_t = -inf carry no mass (their H_t is ignored); a row of
 * such tiles gives (-inf, NaN); a NaN lse_t gives (NaN, NaN).  The tiles may come from hola_tile_stats, from
 * another device, or from a GEMM epilogue.  No workspace; both arrays are device memory. */
hola_status hola_merge_tile_stats(const double* tile_stats /* device [R, ntiles, 2] */, int32_t R, int32_t ntiles,
                                  double* stats_out /* device [R, 2] = (lse, H) */, hola_stream_t stream);

/* Per-kernel timing aid for benchmarks (state of the calling thread).  While enabled, each call this thread makes
 * records HIP events around each of its kernels on the call's stream.  hola_profile_collect() waits for the recorded
 * events, ADDS elapsed milliseconds and launch counts per stage to the host arrays, and
 * forgets the events.  Stages: 0 split-row statistics, 1 accept/first-reject, 2 residual tile sums,
 * 3 inverse-CDF select, 4 level glue / tile merge, 5 fused per-sequence kernel, 6 per-sequence tail kernel,
 * 7 top-k / top-p keep sets by the per-row kernel (every row, or those the next two left), 8 candidate scan,
 * 9 per-row decide step. */
enum { HOLA_N_STAGES = 11 };      /* stage 10: the read probe below */
hola_status hola_profile_enable(int32_t on);
hola_status hola_profile_collect(double* ms_out /* host [HOLA_N_STAGES] */, int64_t* launches_out /* host [HOLA_N_STAGES] */);
/* The same per launch instead of per stage: for the i-th kernel recorded since the last collect, its stage and its
 * elapsed milliseconds (i < capacity; later ones are dropped); *n_out = kernels recorded.  Forgets the events. */
hola_status hola_profile_collect_launches(int32_t* stage_out /* host [capacity] */, float* ms_out /* host [capacity] */,
                                          int64_t capacity, int64_t* n_out /* host */);

/* A plain copy kernel (16-byte vector loads and stores, nothing else): bytes of device memory from src
 * to dst, bytes a multiple of 16, both 16-byte aligned.  It is not part of the verify step; it exists so
 * that hardware byte counters read for the verify kernels (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) can
 * be scaled against a transfer of known size measured the same way. */
hola_status hola_copy_bytes(void* dst /* device */, const void* src /* device */, size_t bytes, hola_stream_t stream);

/* A read-only streaming kernel (not part of the verify step): reads `bytes` of device memory once, in 16-byte
 * loads, with the launch shape of the statistics pass (workgroups of 256 threads, each over block_bytes contiguous
 * bytes, eight loads in flight per lane), and keeps nothing.  nontemporal != 0: the loads carry the non-temporal
 * hint the statistics pass uses; arithmetic != 0: every 16 bytes also go through the arithmetic that pass performs
 * on eight bf16 logits (24 FMAs, 8 exp2, 7 adds, a running maximum, 2 double adds).  Its rate is the practical
 * ceiling the benchmark quotes beside the published HBM peak.  bytes a multiple of 16, src 16-byte aligned. */
hola_status hola_read_probe(const void* src /* device */, size_t bytes, size_t block_bytes, int32_t nontemporal,
                            int32_t arithmetic, hola_stream_t stream);

/* Frees the library-owned workspaces of every device and the calling thread's profiling events. */
void hola_shutdown(void);

const char* hola_status_string(hola_status s);
const char* hola_last_hip_error(void);
const char* hola_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HOLA_H */
