// Internal declarations shared by the translation units of libhola.so (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include "../../include/hola.h"

namespace hola {

constexpr int kWaves = 4;              // wavefronts per workgroup in the streaming kernels
constexpr int kBlock = 64 * kWaves;    // 256 threads
constexpr int kMaxSplit = 16;          // workgroups per row, upper bound (sizes the partials)
constexpr int kTileChunks = 4;         // 16-byte chunks per lane in one sampler tile
constexpr int kKeptListMax = 1024;     // longest top-k / top-p keep set handed from the filter to the sampler as a list

// One wavefront's share of a row: the sums are S = sum 2^(x*c + bref), T = sum (x*c + bref) 2^(x*c + bref)
// with c = log2(e)/T and bref an integer-valued reference chosen so the largest term is O(1).
struct Partial {
    double bref, S, T;
    float vmax;                        // largest logit seen (argmax rows only)
    int32_t imax;                      // its lowest index
};

// Per-sequence hand-over from the accept kernel to the sampler.
struct SeqInfo {
    double lseP, lseD;                 // natural-log lse of the stop row in target and draft
    float u;                           // sampling uniform
    int32_t row;                       // stop row (= accept length)
    int32_t mode;                      // 0 residual, 1 bonus, 2 nothing to sample (greedy / done)
    int32_t greedy_tok;                // next token of a greedy row (mode 2)
};

// Keep set and statistics of one top-k / top-p filtered row: token i with logit x is kept iff x > theta, or
// x == theta and i <= idx_cut.  lse and H (nats) are those of the kept, renormalised tokens.
struct RowFilter {
    double lse, H;
    float theta;
    int32_t idx_cut;
    int32_t n_keep;                    // kept tokens (-1: every finite logit)
    int32_t pad;
};

// Constants of the exponent argument y = x * cstar + b.  make_scale (device) and host_scale compute the same bits:
// a call with one temperature has them made once on the host instead of by every wavefront.
struct ExpScale {
    double cstar;          // log2(e) / temperature
    float c_hi, c_lo;      // cstar = c_hi + c_lo (fp32 pair)
    float c1, c2;          // cstar = c1 + c2 with c1 of 16 significant bits (bf16 path)
    float inv_c;           // 1 / c_hi
};
inline ExpScale host_scale(double temperature)
{
    ExpScale s;
    s.cstar = 1.4426950408889634074 / temperature;
    s.c_hi = (float)s.cstar;
    s.c_lo = (float)(s.cstar - (double)s.c_hi);
    uint32_t bits;
    memcpy(&bits, &s.c_hi, 4);
    bits = (bits + 0x80u) & 0xffffff00u;
    memcpy(&s.c1, &bits, 4);
    s.c2 = (float)(s.cstar - (double)s.c1);
    s.inv_c = 1.0f / s.c_hi;
    return s;
}

struct Shape {
    int32_t B, gamma, V, dtype;
    int64_t target_ld, draft_ld;
    int32_t nsplit;                    // workgroups per row (row statistics)
    int32_t nparts;                    // partials per row = nsplit * kWaves
    int32_t ntiles;                    // sampler tiles per row
};

// Workspace carve-up (all offsets 256-byte aligned).
struct Workspace {
    Partial* partials;                 // [(B*gamma) + B*(gamma+1)] * nparts
    double* statsD;                    // [B, gamma, 2]   (lse, H) nats
    double* statsP;                    // [B, gamma+1, 2]
    int32_t* argmaxP;                  // [B, gamma+1]
    SeqInfo* seq;                      // [B]
    double* tiles;                     // [B, ntiles]
    RowFilter* filters;                // [(B*gamma) + B*(gamma+1)], filtered calls only
    unsigned long long* tickets;       // [B] completion tickets of a tail shared by several workgroups per sequence
    void* filter_scan;                 // candidate lists, counters, flags and segment records of the filter scan
    size_t bytes;
};

struct Tuning {
    int split = 0, unroll = 0;
    int path = 0;                      // 0 auto, 1 split rows + tail kernel, 2 fused kernel, 3 split rows + 3 kernels
    int fused_waves = 0;               // 0 (= 16), 8 or 16 wavefronts per workgroup in the fused kernel
    int tail_split = 0;                // workgroups per sequence in the tail kernel: 0 auto, 1, 2, 4 or 8
    int filter_path = 0;               // 1: the per-row filter kernel for every row
};

struct RowStatsParams {
    const void* target; const void* draft;
    int64_t target_ld, draft_ld;
    const int32_t* draft_len;          // device or null
    const float* row_temperature;      // device or null
    float temperature;
    int32_t B, gamma, V;
    int32_t nsplit;
    int32_t skip_draft;                // draft statistics come from a previous level
    int32_t skip_target;               // target statistics are given by the caller
    int32_t lse_only_targets;          // nobody asks for the entropy of the target rows: their pass leaves T out
    int32_t tile_cols, ntiles;         // ntiles > 0: "sequence" b is column tile b % ntiles of plain row b / ntiles
    int32_t literal;                   // Equation (1) literal mode: target row j is needed only for j < len
    const int32_t* tree_parent;        // device [B, gamma] or null: token trees, node parents; draft rows of
                                       // contexts without children are skipped
    Partial* partials;
    ExpScale sc;                       // set by the launcher when the call has one temperature > 0 (sc_given)
    int32_t sc_given;
};

struct AcceptParams {
    const void* target; const void* draft; int32_t dtype;
    int64_t target_ld, draft_ld;
    const int32_t* tokens; const int32_t* draft_len; const float* row_temperature;
    const double* draft_stats_in; double* target_stats_out;
    uint64_t seed; uint32_t level; int64_t seq_base;
    int32_t B, gamma, V, nparts;
    int64_t tokens_ld;                 // row stride of tokens (>= gamma)
    int32_t pad_entropy;               // also write -1 into out_entropy columns gamma .. entropy_ld-1
    float temperature, tau;
    const Partial* partials;
    double* statsD; double* statsP; int32_t* argmaxP; SeqInfo* seq;
    int32_t* out_accept_len; int32_t* out_next_token; float* out_entropy; int64_t entropy_ld;
};

struct SamplerParams {
    const void* target; const void* draft; int32_t dtype;
    int64_t target_ld, draft_ld;
    const float* row_temperature; float temperature;
    int32_t B, gamma, V, ntiles;
    const SeqInfo* seq; double* tiles;
    int32_t* out_next_token;
};

struct FusedParams {
    const void* target; const void* draft; int32_t dtype;
    int64_t target_ld, draft_ld;
    const int32_t* tokens; const int32_t* draft_len; const float* row_temperature;
    const double* draft_stats_in; double* target_stats_out; const double* target_stats_in;
    uint64_t seed; uint32_t level; int64_t seq_base;
    int32_t B, gamma, V, ntiles;
    int64_t tokens_ld;                 // row stride of tokens (>= gamma)
    int32_t pad_entropy;               // also write -1 into out_entropy columns gamma .. entropy_ld-1
    float temperature, tau;
    int32_t* out_accept_len; int32_t* out_next_token; float* out_entropy; int64_t entropy_ld;
    // drafts of the next verify level, written by the per-sequence kernels when given: the kept tokens
    // followed by the next token, -1 up to glue_ld; glue_len[b] = accept length + 1
    int32_t* glue_tok; int32_t* glue_len; int64_t glue_ld;
    int32_t glue_keep_next;            // 1: append the next token; 0: the kept tokens only
    const RowFilter* filters;          // top-k / top-p keep sets (slots as the partials), or null
    const RowFilter* draft_filters;    // where the draft rows' keep sets are read from: `filters`, or an array [B, gamma]
                                       // handed over by the previous level of a hierarchy
    // short keep sets written out as lists of (order key << 32 | index), at most kKeptListMax entries, kept_stride
    // apart, for row r = b (2 gamma + 1) + k, and their lengths (-1: no list); null when the filter's scan did not run
    const unsigned long long* kept; const int32_t* kept_n; int64_t kept_stride;
    // a tail shared by `coop` workgroups per sequence (1: one workgroup, as ever): where they leave their tile weights
    // for each other ([B, ntiles]), the sequences' completion tickets ([B], any contents) and this call's tag for them
    int32_t coop;
    double* coop_tiles; unsigned long long* coop_tickets; unsigned long long coop_tag;
    // the scale constants of a call with one temperature > 0, made once on the host (sc_given), as in RowStatsParams
    ExpScale sc; int32_t sc_given;
};

// Token trees: N nodes per sequence, rows by context as the one-token step lays them out with gamma = N.
struct TreeParams {
    const void* target; const void* draft; int32_t dtype;
    int64_t target_ld, draft_ld;
    const int32_t* tokens; const int32_t* parent; const int32_t* n_nodes;
    uint64_t seed; uint32_t level; int64_t seq_base;
    int32_t B, N, V, ntiles;
    float temperature, tau;
    int32_t* out_accept_len; int32_t* out_path; int32_t* out_next_token; float* out_entropy;
    ExpScale sc;                       // host_scale(temperature)
};
bool tree_supported(int32_t N, int32_t V, int dtype);
hipError_t launch_tree_tail(const TreeParams& p, const Partial* partials, int nparts, int waves, hipStream_t s);

hipError_t launch_fused(const FusedParams& p, const Tuning& t, hipStream_t s);
hipError_t launch_tail(const FusedParams& p, const Partial* partials, int nparts, const Tuning& t, hipStream_t s);
bool fused_supported(int32_t gamma, int32_t V, int dtype);   // the one-launch fused kernel
bool tail_supported(int32_t gamma, int32_t V, int dtype);    // the per-sequence tail kernel after the split-row pass
bool literal_supported(int32_t gamma, int32_t V, int dtype);
hipError_t launch_literal(const FusedParams& p, const Partial* partials, int nparts, int32_t* out_tokens,
                          int32_t* out_calls, hipStream_t s);
hipError_t launch_row_stats(const RowStatsParams& p, int dtype, const Tuning& t, hipStream_t s);
// Keep sets of top-k / top-p filtered rows by the one-workgroup-per-row kernel: every row, or with `flags`
// ([B (2 gamma + 1)]) only the rows flagged 1.  skip_draft (here and in the two launchers below): the draft rows'
// keep sets come from elsewhere (the level of a hierarchy at which that model was the target); only target rows are done.
hipError_t launch_filter(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                         const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                         int32_t top_k, float top_p, RowFilter* filters, int32_t* out_keep_count, const int32_t* flags,
                         int32_t skip_draft, hipStream_t s);
// The usual course of the filter: a split-row scan that lists candidates, then a per-row decide step; rows it
// cannot settle come back flagged in *flags_out ([B (2 gamma + 1)], 1 = still to do).
size_t filter_scan_bytes(int64_t rows);
bool filter_scan_applies(int dtype, int32_t V, int32_t top_k);
hipError_t launch_filter_scan(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                              const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                              int32_t top_k, float top_p, void* scratch, int32_t skip_draft, hipStream_t s);
hipError_t launch_filter_decide(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                                const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                                int32_t top_k, float top_p, RowFilter* filters, int32_t* out_keep_count, void* scratch,
                                int32_t** flags_out, const unsigned long long** kept_out, int64_t* kept_stride_out,
                                const int32_t** kept_n_out, int32_t skip_draft, hipStream_t s);
hipError_t launch_accept(const AcceptParams& p, hipStream_t s);
hipError_t launch_merge_tile_stats(const double* ts, int32_t R, int32_t nt, double* out, hipStream_t s);
hipError_t launch_finalize_rows(const Partial* partials, int nparts, int32_t R, double* out, hipStream_t s);
hipError_t launch_tile_sums(const SamplerParams& p, hipStream_t s);
hipError_t launch_select(const SamplerParams& p, hipStream_t s);

// Read-only streaming probe (measurement aid): workgroups of kBlock threads, each over block_bytes of src.
hipError_t launch_read_probe(const void* src, size_t bytes, int64_t block_bytes, int nontemporal, int arith, hipStream_t s);

int choose_split(int64_t rows, int V, int dtype, const Tuning& t);
int sampler_tiles(int V, int dtype);

}  // namespace hola
