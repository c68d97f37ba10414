// Host side of libhola.so: the C ABI, argument checks, workspace carving, the per-level launch
// sequence and the hierarchical level driver.  No host synchronisation and no allocation on the
// steady-state path; everything is enqueued on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "device_common.h"
#include "hola_internal.h"

namespace hola {

// ---------------------------------------------------------------------------------------------
// small device kernels of the driver
// ---------------------------------------------------------------------------------------------
// Drafts of the next level: the kept tokens of this level followed by its next token (only used on the
// four-kernel path; the per-sequence kernels write them themselves).
__global__ void level_glue_kernel(const int32_t* __restrict__ cur_tok, int64_t cur_ld, int32_t gk,
                                  const int32_t* __restrict__ acc, const int32_t* __restrict__ nxt, int32_t B,
                                  int32_t* __restrict__ new_tok, int64_t new_ld, int32_t* __restrict__ new_len,
                                  int32_t keep_next)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int a = acc[b];
    a = a < 0 ? 0 : (a > gk ? gk : a);
    for (int64_t j = 0; j < new_ld; ++j)
        new_tok[(int64_t)b * new_ld + j] = j < a ? cur_tok[(int64_t)b * cur_ld + j] : ((j == a && keep_next) ? nxt[b] : -1);
    new_len[b] = a + (keep_next ? 1 : 0);
}

// Plain copy: one 16-byte load and one 16-byte store per lane per step, grid-stride.
__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__global__ void export_tokens_kernel(const int32_t* __restrict__ tok, int64_t tok_ld, int32_t gk,
                                     const int32_t* __restrict__ len, int32_t B, int32_t width, int32_t* __restrict__ out)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int l = len ? len[b] : gk;
    for (int j = 0; j < width; ++j) out[(int64_t)b * width + j] = (j < l && j < gk) ? tok[(int64_t)b * tok_ld + j] : -1;
}

// ---------------------------------------------------------------------------------------------
// state: launch-shape defaults and the profiling aid belong to the calling thread (a call never sees another
// thread's settings); the only process-wide state is the short forms' workspace per device and the address of
// the static scratch array per device, both behind g_mu.
// ---------------------------------------------------------------------------------------------
static thread_local char g_last_hip[256] = "";
static thread_local Tuning g_tuning;
static std::mutex g_mu;

// Tag of a call's completion tickets (a tail shared by several workgroups per sequence): 48 bits, never 0, different
// from call to call and (by the start value) from process to process, so that nothing a workspace may hold from
// before reads as a ticket of this call.
static unsigned long long next_ticket_tag()
{
    static std::atomic<unsigned long long> counter{0};
    static const unsigned long long salt = [] {
        unsigned long long x = (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
        x ^= (unsigned long long)(uintptr_t)&counter * 0x9E3779B97F4A7C15ull;
        x ^= x >> 29; x *= 0xBF58476D1CE4E5B9ull; x ^= x >> 32;
        return x;
    }();
    const unsigned long long t = (salt + counter.fetch_add(1, std::memory_order_relaxed) * 0x9E3779B97F4A7C15ull) & 0xffffffffffffull;
    return t ? t : 1ull;
}

struct DeviceWs { void* ptr = nullptr; size_t bytes = 0; };
static DeviceWs g_ws[64];

struct ProfEvent { int stage; hipEvent_t a, b; };
static thread_local bool g_prof_on = false;
static thread_local std::vector<ProfEvent> g_prof_live;
static thread_local std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_free;

static hola_status hip_fail(hipError_t e, const char* what)
{
    snprintf(g_last_hip, sizeof g_last_hip, "%s: %s", what, hipGetErrorString(e));
    return HOLA_ERR_HIP;
}

struct StageTimer {
    int stage; hipStream_t s; bool on; hipEvent_t a = nullptr, b = nullptr;
    StageTimer(int stage_, hipStream_t s_) : stage(stage_), s(s_), on(g_prof_on)
    {
        if (!on) return;
        if (!g_prof_free.empty()) { a = g_prof_free.back().first; b = g_prof_free.back().second; g_prof_free.pop_back(); }
        else if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
        if (hipEventRecord(a, s) != hipSuccess) { g_prof_free.emplace_back(a, b); on = false; }
    }
    ~StageTimer()
    {
        if (!on) return;
        const bool timed = hipEventRecord(b, s) == hipSuccess;
        if (timed) g_prof_live.push_back(ProfEvent{stage, a, b});
        else g_prof_free.emplace_back(a, b);
    }
};

// The library's own choices.  Path: the split-row pass, which spreads rows over the whole chip, followed by
// the per-sequence tail kernel; the fused per-sequence kernel stays selectable but was slower at every batch
// size measured (B = 1 .. 8192) once the split-row kernel streamed at ~6.6 TB/s.  Tail workgroup: 16
// wavefronts while every sequence has a compute unit of its own, smaller workgroups (several sequences per
// compute unit, their latency-bound phases overlapping) beyond that (measured: B=512 8 wavefronts 4-12 %
// faster than 16, B>=2048 4 wavefronts 4-15 % faster than 8 unless the rows are very long).
static int device_cu_count()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

static int auto_tail_waves(int32_t B, int64_t row_bytes)
{
    const int cus = device_cu_count();
    if (B <= cus) return 16;
    return (B > 3 * cus && row_bytes < (512 << 10)) ? 4 : 8;   // 1 MB rows: 8 beats 4 by 2 % (sweep is bandwidth-bound)
}

// Workgroups that share one sequence's tail.  One compute unit sweeps a sequence's stop rows at what its vector
// units allow (~20 us for two 256 KB rows); with few sequences most of the chip idles meanwhile, so their sweeps are
// split over two, four or eight compute units, at the price of ~5 us for handing the tile weights over through memory.
static int auto_tail_split(int32_t B, int64_t row_bytes)
{
    const int cus = device_cu_count();
    if (row_bytes < (128 << 10)) return 1;
    if ((int64_t)B * 8 <= cus) return 8;
    if ((int64_t)B * 4 <= cus) return 4;
    if ((int64_t)B * 2 <= cus) return 2;
    return 1;
}

static inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static bool tuning_from(const hola_tuning* t, Tuning* out)
{
    Tuning n;
    if (t) {
        if (t->stats_split < 0 || t->stats_split > kMaxSplit) return false;
        if (t->stats_unroll != 0 && t->stats_unroll != 2 && t->stats_unroll != 4 && t->stats_unroll != 8 && t->stats_unroll != 16)
            return false;
        if (t->path < 0 || t->path > 3) return false;
        if (t->fused_waves != 0 && t->fused_waves != 4 && t->fused_waves != 8 && t->fused_waves != 16) return false;
        if (t->filter_path < 0 || t->filter_path > 1) return false;
        if (t->tail_split != 0 && t->tail_split != 1 && t->tail_split != 2 && t->tail_split != 4 && t->tail_split != 8) return false;
        n.split = t->stats_split; n.unroll = t->stats_unroll; n.path = t->path; n.fused_waves = t->fused_waves;
        n.filter_path = t->filter_path; n.tail_split = t->tail_split;
    }
    *out = n;
    return true;
}

// Launch shape of one call: its own hola_tuning when given, else the calling thread's defaults.
static bool call_tuning(const hola_tuning* t, Tuning* out)
{
    if (!t) { *out = g_tuning; return true; }
    return tuning_from(t, out);
}

// base == nullptr: only the size is wanted (no pointer is formed).
static Workspace carve(void* base, int32_t B, int32_t gamma, int32_t V, bool with_filters = true)
{
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) -> char* {
        char* at = base ? (char*)base + off : nullptr;
        off = align_up(off + bytes);
        return at;
    };
    const size_t rows = (size_t)B * (2 * (size_t)gamma + 1);
    const int ntiles = sampler_tiles(V, HOLA_DTYPE_F32);       // the larger of the two dtypes
    w.partials = (Partial*)take(rows * kMaxSplit * kWaves * sizeof(Partial));
    w.statsD = (double*)take((size_t)B * gamma * 2 * sizeof(double));
    w.statsP = (double*)take((size_t)B * (gamma + 1) * 2 * sizeof(double));
    w.argmaxP = (int32_t*)take((size_t)B * (gamma + 1) * sizeof(int32_t));
    w.seq = (SeqInfo*)take((size_t)B * sizeof(SeqInfo));
    w.tiles = (double*)take((size_t)B * ntiles * sizeof(double));
    w.tickets = (unsigned long long*)take((size_t)B * sizeof(unsigned long long));
    w.filters = nullptr;
    w.filter_scan = nullptr;
    if (with_filters) {                                        // keep sets and candidate lists: filtered calls only
        w.filters = (RowFilter*)take(rows * sizeof(RowFilter));
        const size_t scan_bytes = filter_scan_bytes((int64_t)rows);
        char* at = take(scan_bytes);
        w.filter_scan = scan_bytes ? at : nullptr;
    }
    w.bytes = off;
    return w;
}

static bool shape_ok(int32_t B, int32_t gamma, int32_t V)
{
    return B >= 0 && gamma >= 1 && gamma <= HOLA_MAX_GAMMA && V >= 1;
}

static bool filters_on(const hola_verify_args& a)
{
    return (a.top_k != 0 && a.top_k < a.V) || (a.top_p != 0.f && !(a.top_p >= 1.f));
}

static hola_status check_args(const hola_verify_args& a, bool literal = false)
{
    if (!shape_ok(a.B, a.gamma, a.V)) return HOLA_ERR_INVALID_ARG;
    if (a.dtype != HOLA_DTYPE_F32 && a.dtype != HOLA_DTYPE_BF16) return HOLA_ERR_UNSUPPORTED;
    if (a.B == 0) return HOLA_OK;
    if (!a.target_logits || !a.draft_logits || !a.draft_tokens) return HOLA_ERR_INVALID_ARG;
    if (!literal && (!a.out_accept_len || !a.out_next_token)) return HOLA_ERR_INVALID_ARG;
    const size_t es = a.dtype == HOLA_DTYPE_BF16 ? 2 : 4;
    if (((uintptr_t)a.target_logits % es) || ((uintptr_t)a.draft_logits % es)) return HOLA_ERR_INVALID_ARG;
    if ((a.target_ld && a.target_ld < a.V) || (a.draft_ld && a.draft_ld < a.V)) return HOLA_ERR_INVALID_ARG;
    if (a.entropy_ld && a.entropy_ld < a.gamma) return HOLA_ERR_INVALID_ARG;
    if (!(a.temperature >= 0.f) || std::isinf(a.temperature)) return HOLA_ERR_INVALID_ARG;   // rejects NaN too
    if (std::isnan(a.entropy_threshold)) return HOLA_ERR_INVALID_ARG;
    // Filtered distributions: stochastic rows with one temperature; their statistics are not interchangeable
    // with unfiltered ones, so none are taken or handed on.
    if (filters_on(a)) {
        if (a.top_k < 0 || !(a.top_p >= 0.f)) return HOLA_ERR_INVALID_ARG;
        if (literal || a.row_temperature || !(a.temperature > 0.f) || a.draft_stats_in || a.target_stats_in ||
            a.target_stats_out || a.V >= (1 << 22) || !tail_supported(a.gamma, a.V, a.dtype))
            return HOLA_ERR_UNSUPPORTED;
    }
    // Supplied target statistics carry no argmax, which greedy rows need.
    if (a.target_stats_in && (a.row_temperature || !(a.temperature > 0.f))) return HOLA_ERR_UNSUPPORTED;
    if (a.tuning) { Tuning t; if (!tuning_from(a.tuning, &t)) return HOLA_ERR_INVALID_ARG; }
    if (!a.workspace || ((uintptr_t)a.workspace & 255)) return HOLA_ERR_WORKSPACE;
    if (a.workspace_bytes < carve(nullptr, a.B, a.gamma, a.V, filters_on(a)).bytes + 256) return HOLA_ERR_WORKSPACE;
    return HOLA_OK;
}

// What the hierarchical driver adds to one level: a row stride for the drafted tokens, -1 padding of the
// entropy row up to entropy_ld, and the next level's drafts written by the level itself.
struct LevelExtras {
    int64_t tokens_ld = 0;             // 0 => gamma
    int32_t pad_entropy = 0;
    int32_t* glue_tok = nullptr; int32_t* glue_len = nullptr; int64_t glue_ld = 0;
    int32_t glue_keep_next = 1;
    // filtered levels: the keep sets and statistics of the draft rows as the previous level found them when that
    // model was its target ([B, gamma], so those rows are not scanned again), and where this level leaves its
    // target rows' ([B, gamma + 1]) for the next one
    const RowFilter* draft_filters_in = nullptr;
    RowFilter* target_filters_out = nullptr;
};

static hola_status run_level(const hola_verify_args& a, const LevelExtras& x = LevelExtras())
{
    hola_status st = check_args(a);
    if (st != HOLA_OK || a.B == 0) return st;
    hipStream_t s = (hipStream_t)a.stream;
    const Workspace w = carve(a.workspace, a.B, a.gamma, a.V, filters_on(a));
    const int64_t tld = a.target_ld ? a.target_ld : a.V, dld = a.draft_ld ? a.draft_ld : a.V;
    const int skip_draft = a.draft_stats_in ? 1 : 0, skip_target = a.target_stats_in ? 1 : 0;
    const int64_t rows = (int64_t)a.B * ((skip_draft ? 0 : a.gamma) + (skip_target ? 0 : a.gamma + 1));
    Tuning tune;
    call_tuning(a.tuning, &tune);                             // validated by check_args
    const int nsplit = choose_split(rows > 0 ? rows : 1, a.V, a.dtype, tune);

    // Per-sequence parameters shared by the fused kernel and the tail kernel.
    const bool per_seq_ok = tail_supported(a.gamma, a.V, a.dtype);
    if (skip_target && !per_seq_ok) return HOLA_ERR_UNSUPPORTED;    // only the tail kernel takes them
    if (skip_target) tune.path = 1;
    FusedParams fp{};
    fp.target = a.target_logits; fp.draft = a.draft_logits; fp.dtype = a.dtype; fp.target_ld = tld; fp.draft_ld = dld;
    fp.tokens = a.draft_tokens; fp.draft_len = a.draft_len; fp.row_temperature = a.row_temperature;
    fp.draft_stats_in = a.draft_stats_in; fp.target_stats_out = a.target_stats_out; fp.target_stats_in = a.target_stats_in;
    fp.seed = a.seed; fp.level = a.level; fp.seq_base = a.seq_base;
    fp.B = a.B; fp.gamma = a.gamma; fp.V = a.V; fp.ntiles = sampler_tiles(a.V, a.dtype);
    fp.tokens_ld = x.tokens_ld ? x.tokens_ld : a.gamma; fp.pad_entropy = x.pad_entropy;
    fp.glue_tok = x.glue_tok; fp.glue_len = x.glue_len; fp.glue_ld = x.glue_ld; fp.glue_keep_next = x.glue_keep_next;
    fp.temperature = a.temperature; fp.tau = a.entropy_threshold;
    fp.sc_given = (a.row_temperature == nullptr && a.temperature > 0.f) ? 1 : 0;
    if (fp.sc_given) fp.sc = host_scale((double)a.temperature);
    fp.out_accept_len = a.out_accept_len; fp.out_next_token = a.out_next_token;
    fp.out_entropy = a.out_entropy; fp.entropy_ld = a.entropy_ld;

    const bool filtered = filters_on(a);
    if (filtered) tune.path = 1;                                  // statistics, keep sets, then the tail kernel
    // Path 2: one fused launch per level (one workgroup per sequence streams its own rows).
    const bool want_fused = tune.path == 2;
    if (want_fused && fused_supported(a.gamma, a.V, a.dtype)) {
        hipError_t fe;
        { StageTimer t(5, s); fe = launch_fused(fp, tune, s); }
        if (fe != hipSuccess) return hip_fail(fe, "fused verify launch");
        return HOLA_OK;
    }

    RowStatsParams rs{};
    rs.target = a.target_logits; rs.draft = a.draft_logits; rs.target_ld = tld; rs.draft_ld = dld;
    rs.draft_len = a.draft_len; rs.row_temperature = a.row_temperature; rs.temperature = a.temperature;
    rs.B = a.B; rs.gamma = a.gamma; rs.V = a.V; rs.nsplit = nsplit; rs.skip_draft = skip_draft; rs.skip_target = skip_target;
    rs.lse_only_targets = a.target_stats_out ? 0 : 1;           // the accept stage and the sampler use only their lse
    rs.partials = w.partials;
    hipError_t e = hipSuccess;
    // nothing to stream when both statistics are supplied; the filter kernel takes its own from the logits
    if (rows > 0 && !filtered) { StageTimer t(0, s); e = launch_row_stats(rs, a.dtype, tune, s); }
    if (e != hipSuccess) return hip_fail(e, "row statistics launch");

    if (filtered) {
        const float top_p = (a.top_p > 0.f && a.top_p < 1.f) ? a.top_p : 1.f;
        const int32_t skip_d = x.draft_filters_in ? 1 : 0;     // the draft rows' keep sets are handed over
        int32_t* flags = nullptr;
        if (tune.filter_path != 1 && w.filter_scan && filter_scan_applies(a.dtype, a.V, a.top_k)) {
            { StageTimer t(8, s);
              e = launch_filter_scan(a.target_logits, a.draft_logits, a.dtype, tld, dld, a.draft_len, a.temperature, a.B, a.gamma,
                                     a.V, a.top_k, top_p, w.filter_scan, skip_d, s); }
            if (e != hipSuccess) return hip_fail(e, "filter scan launch");
            { StageTimer t(9, s);
              e = launch_filter_decide(a.target_logits, a.draft_logits, a.dtype, tld, dld, a.draft_len, a.temperature, a.B, a.gamma,
                                       a.V, a.top_k, top_p, w.filters, a.out_keep_count, w.filter_scan, &flags, &fp.kept,
                                       &fp.kept_stride, &fp.kept_n, skip_d, s); }
            if (e != hipSuccess) return hip_fail(e, "filter decide launch");
        }
        { StageTimer t(7, s);
          e = launch_filter(a.target_logits, a.draft_logits, a.dtype, tld, dld, a.draft_len, a.temperature, a.B, a.gamma, a.V,
                            a.top_k, top_p, w.filters, a.out_keep_count, flags, skip_d, s); }
        if (e != hipSuccess) return hip_fail(e, "filter launch");
        fp.filters = w.filters;
        fp.draft_filters = x.draft_filters_in ? x.draft_filters_in : w.filters;
    }

    // Paths 0/1: the split-row pass spreads the rows over the chip, then one per-sequence tail kernel does
    // accept + sampling.  Path 3 keeps accept, tile sums and select as three kernels of their own.
    if (tune.path != 3 && per_seq_ok) {
        const int64_t row_bytes = (int64_t)a.V * (a.dtype == HOLA_DTYPE_BF16 ? 2 : 4);
        if (tune.fused_waves == 0) tune.fused_waves = auto_tail_waves(a.B, row_bytes);
        // several workgroups per sequence: only the 16-wavefront tail of unfiltered calls, each on a compute unit of its own
        int coop = tune.tail_split ? tune.tail_split : auto_tail_split(a.B, row_bytes);
        if (filtered || tune.fused_waves != 16 || (int64_t)a.B * coop > device_cu_count() || fp.ntiles < 2 * coop) coop = 1;
        fp.coop = coop;
        if (coop > 1) { fp.coop_tiles = w.tiles; fp.coop_tickets = w.tickets; fp.coop_tag = next_ticket_tag(); }
        { StageTimer t(6, s); e = launch_tail(fp, w.partials, nsplit * kWaves, tune, s); }
        if (e != hipSuccess) return hip_fail(e, "tail launch");
        if (filtered && x.target_filters_out) {                // this level's target rows are the next level's draft rows
            StageTimer t(4, s);
            const size_t n16 = (size_t)a.B * (a.gamma + 1) * sizeof(RowFilter) / 16;
            hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s, (uint4*)x.target_filters_out,
                               (const uint4*)(w.filters + (size_t)a.B * a.gamma), n16);
            e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e, "filter hand-over launch");
        }
        return HOLA_OK;
    }

    AcceptParams ap{};
    ap.target = a.target_logits; ap.draft = a.draft_logits; ap.dtype = a.dtype; ap.target_ld = tld; ap.draft_ld = dld;
    ap.tokens = a.draft_tokens; ap.draft_len = a.draft_len; ap.row_temperature = a.row_temperature;
    ap.draft_stats_in = a.draft_stats_in; ap.target_stats_out = a.target_stats_out;
    ap.seed = a.seed; ap.level = a.level; ap.seq_base = a.seq_base;
    ap.B = a.B; ap.gamma = a.gamma; ap.V = a.V; ap.nparts = nsplit * kWaves;
    ap.tokens_ld = fp.tokens_ld; ap.pad_entropy = x.pad_entropy;
    ap.temperature = a.temperature; ap.tau = a.entropy_threshold;
    ap.partials = w.partials; ap.statsD = w.statsD; ap.statsP = w.statsP; ap.argmaxP = w.argmaxP; ap.seq = w.seq;
    ap.out_accept_len = a.out_accept_len; ap.out_next_token = a.out_next_token;
    ap.out_entropy = a.out_entropy; ap.entropy_ld = a.entropy_ld;
    { StageTimer t(1, s); e = launch_accept(ap, s); }
    if (e != hipSuccess) return hip_fail(e, "accept launch");

    SamplerParams sp{};
    sp.target = a.target_logits; sp.draft = a.draft_logits; sp.dtype = a.dtype; sp.target_ld = tld; sp.draft_ld = dld;
    sp.row_temperature = a.row_temperature; sp.temperature = a.temperature;
    sp.B = a.B; sp.gamma = a.gamma; sp.V = a.V; sp.ntiles = sampler_tiles(a.V, a.dtype);
    sp.seq = w.seq; sp.tiles = w.tiles; sp.out_next_token = a.out_next_token;
    { StageTimer t(2, s); e = launch_tile_sums(sp, s); }
    if (e != hipSuccess) return hip_fail(e, "tile sums launch");
    { StageTimer t(3, s); e = launch_select(sp, s); }
    if (e != hipSuccess) return hip_fail(e, "select launch");
    if (x.glue_tok) {                                  // this path has no per-sequence kernel to do it
        StageTimer t(4, s);
        const int tpb = 128;
        hipLaunchKernelGGL(level_glue_kernel, dim3((a.B + tpb - 1) / tpb), dim3(tpb), 0, s, a.draft_tokens, fp.tokens_ld,
                           a.gamma, a.out_accept_len, a.out_next_token, a.B, x.glue_tok, x.glue_ld, x.glue_len, x.glue_keep_next);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "glue launch");
    }
    return HOLA_OK;
}

// Equation (1) literal mode: split-row statistics of the draft rows and of target rows j < len, then one
// per-sequence kernel that gates every position and draws the non-gated ones from their target rows.
static hola_status run_literal(const hola_verify_args& a, int32_t* out_tokens, int32_t* out_calls)
{
    hola_status st = check_args(a, true);
    if (st != HOLA_OK) return st;
    if (a.B == 0) return HOLA_OK;
    if (!out_tokens) return HOLA_ERR_INVALID_ARG;
    if (a.draft_stats_in || a.target_stats_out || a.target_stats_in) return HOLA_ERR_UNSUPPORTED;
    if (!literal_supported(a.gamma, a.V, a.dtype)) return HOLA_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)a.stream;
    const Workspace w = carve(a.workspace, a.B, a.gamma, a.V, false);
    const int64_t tld = a.target_ld ? a.target_ld : a.V, dld = a.draft_ld ? a.draft_ld : a.V;
    Tuning tune;
    call_tuning(a.tuning, &tune);
    const int nsplit = choose_split((int64_t)a.B * (2 * a.gamma + 1), a.V, a.dtype, tune);
    RowStatsParams rs{};
    rs.target = a.target_logits; rs.draft = a.draft_logits; rs.target_ld = tld; rs.draft_ld = dld;
    rs.draft_len = a.draft_len; rs.row_temperature = a.row_temperature; rs.temperature = a.temperature;
    rs.B = a.B; rs.gamma = a.gamma; rs.V = a.V; rs.nsplit = nsplit; rs.skip_draft = 0; rs.literal = 1;
    rs.partials = w.partials;
    hipError_t e;
    { StageTimer t(0, s); e = launch_row_stats(rs, a.dtype, tune, s); }
    if (e != hipSuccess) return hip_fail(e, "row statistics launch");
    FusedParams fp{};
    fp.target = a.target_logits; fp.draft = a.draft_logits; fp.dtype = a.dtype; fp.target_ld = tld; fp.draft_ld = dld;
    fp.tokens = a.draft_tokens; fp.draft_len = a.draft_len; fp.row_temperature = a.row_temperature;
    fp.seed = a.seed; fp.level = a.level; fp.seq_base = a.seq_base;
    fp.B = a.B; fp.gamma = a.gamma; fp.V = a.V; fp.ntiles = sampler_tiles(a.V, a.dtype);
    fp.tokens_ld = a.gamma; fp.temperature = a.temperature; fp.tau = a.entropy_threshold;
    fp.sc_given = (a.row_temperature == nullptr && a.temperature > 0.f) ? 1 : 0;
    if (fp.sc_given) fp.sc = host_scale((double)a.temperature);
    fp.out_entropy = a.out_entropy; fp.entropy_ld = a.entropy_ld;
    { StageTimer t(6, s); e = launch_literal(fp, w.partials, nsplit * kWaves, out_tokens, out_calls, s); }
    if (e != hipSuccess) return hip_fail(e, "literal launch");
    return HOLA_OK;
}

// Library-owned workspace of the current device for the short forms.
static hola_status own_workspace(size_t need, void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return HOLA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_mu);
    DeviceWs& d = g_ws[dev];
    if (d.bytes < need) {
        if (d.ptr) { e = hipFree(d.ptr); d.ptr = nullptr; d.bytes = 0; if (e != hipSuccess) return hip_fail(e, "hipFree"); }
        size_t want = need + need / 4;
        e = hipMalloc(&d.ptr, want);
        if (e != hipSuccess) { d.ptr = nullptr; return hip_fail(e, "hipMalloc(workspace)"); }
        d.bytes = want;
    }
    *out = d.ptr;
    return HOLA_OK;
}

static hola_status verify_short(const void* target, const void* draft, int dtype, const int32_t* tokens, uint64_t seed,
                                int32_t B, int32_t gamma, int32_t V, float temperature, float tau,
                                int32_t* out_accept_len, int32_t* out_next_token, float* out_entropy, hola_stream_t stream)
{
    if (!shape_ok(B, gamma, V)) return HOLA_ERR_INVALID_ARG;
    if (!(temperature > 0.f)) return HOLA_ERR_INVALID_ARG;     // the short forms have no greedy rows
    if (B == 0) return HOLA_OK;
    hola_verify_args a;
    memset(&a, 0, sizeof a);
    a.target_logits = target; a.draft_logits = draft; a.dtype = dtype;
    a.draft_tokens = tokens; a.seed = seed; a.B = B; a.gamma = gamma; a.V = V;
    a.temperature = temperature; a.entropy_threshold = tau;
    a.out_accept_len = out_accept_len; a.out_next_token = out_next_token; a.out_entropy = out_entropy;
    a.stream = stream;
    // argument errors first, so that a bad call never allocates
    a.workspace = (void*)(uintptr_t)256; a.workspace_bytes = (size_t)-1;
    hola_status st = check_args(a);
    if (st != HOLA_OK) return st;
    a.workspace_bytes = hola_workspace_bytes(B, gamma, V);
    st = own_workspace(a.workspace_bytes, &a.workspace);
    if (st != HOLA_OK) return st;
    return run_level(a);
}

// ---------------------------------------------------------------------------------------------
// The entry point that allocates nothing: its workspace is this array in the library's own device image.  In host
// code the array's name is only a handle; the device address comes from hipGetSymbolAddress, once per device
// (every GPU holds its own copy at its own address), and is what the kernels are given.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[HOLA_STATIC_SCRATCH_BYTES];
static void* g_scratch_addr[64];                             // per device, behind g_mu

static hola_status static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= 64) return HOLA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_addr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return HOLA_OK;
}

}  // namespace hola

using namespace hola;

extern "C" {

size_t hola_workspace_bytes(int32_t B, int32_t gamma, int32_t V)
{
    if (!shape_ok(B, gamma, V)) return 0;
    return carve(nullptr, B, gamma, V).bytes + 256;
}

size_t hola_workspace_bytes_ex(const hola_verify_args* args)
{
    if (!args || !shape_ok(args->B, args->gamma, args->V)) return 0;
    return carve(nullptr, args->B, args->gamma, args->V, filters_on(*args)).bytes + 256;
}

hola_status hola_verify_ex(const hola_verify_args* args)
{
    if (!args) return HOLA_ERR_INVALID_ARG;
    return run_level(*args);
}

hola_status hola_verify_ex_static(const hola_verify_args* args)
{
    if (!args) return HOLA_ERR_INVALID_ARG;
    hola_verify_args a = *args;
    a.workspace = (void*)(uintptr_t)256; a.workspace_bytes = (size_t)-1;   // argument errors first; the fields are ignored
    hola_status st = check_args(a);
    if (st != HOLA_OK || a.B == 0) return st;
    if (hola_workspace_bytes_ex(&a) > (size_t)HOLA_STATIC_SCRATCH_BYTES) return HOLA_ERR_WORKSPACE;
    st = static_scratch(&a.workspace);
    if (st != HOLA_OK) return st;
    a.workspace_bytes = (size_t)HOLA_STATIC_SCRATCH_BYTES;
    return run_level(a);                                       // kernels only: every partial a call reads it has written
}

hola_status hola_verify_literal_ex(const hola_verify_args* args, int32_t* out_tokens, int32_t* out_verifier_calls)
{
    if (!args) return HOLA_ERR_INVALID_ARG;
    return run_literal(*args, out_tokens, out_verifier_calls);
}

hola_status hola_verify_f32(const float* target_logits, const float* draft_logits, const int32_t* draft_tokens,
                            uint64_t seed, int32_t B, int32_t gamma, int32_t V, float temperature,
                            float entropy_threshold, int32_t* out_accept_len, int32_t* out_next_token,
                            float* out_entropy, hola_stream_t stream)
{
    return verify_short(target_logits, draft_logits, HOLA_DTYPE_F32, draft_tokens, seed, B, gamma, V, temperature,
                        entropy_threshold, out_accept_len, out_next_token, out_entropy, stream);
}

hola_status hola_verify_bf16(const uint16_t* target_logits, const uint16_t* draft_logits, const int32_t* draft_tokens,
                             uint64_t seed, int32_t B, int32_t gamma, int32_t V, float temperature,
                             float entropy_threshold, int32_t* out_accept_len, int32_t* out_next_token,
                             float* out_entropy, hola_stream_t stream)
{
    return verify_short(target_logits, draft_logits, HOLA_DTYPE_BF16, draft_tokens, seed, B, gamma, V, temperature,
                        entropy_threshold, out_accept_len, out_next_token, out_entropy, stream);
}

// Workspace of the hierarchical driver: one level workspace at the widest level, two token / length /
// statistics buffers that alternate between levels.
namespace {
struct HsdWs {
    void* level; size_t level_bytes;
    int32_t* tok[2]; int32_t* len[2]; double* stats[2];
    RowFilter* filt[2];                 // filtered chains: a middle model's keep sets, from the level where it is the target
    size_t bytes;
};
HsdWs carve_hsd(void* base, int32_t n_models, int32_t B, int32_t gamma, int32_t V)
{
    HsdWs h;
    const int32_t gmax = gamma + n_models - 2;
    size_t off = 0;
    auto take = [&](size_t bytes) -> char* {                   // base == nullptr: only the size is wanted
        char* at = base ? (char*)base + off : nullptr;
        off = align_up(off + bytes);
        return at;
    };
    h.level_bytes = hola_workspace_bytes(B, gmax, V);
    h.level = take(h.level_bytes);
    for (int i = 0; i < 2; ++i) h.tok[i] = (int32_t*)take((size_t)B * (gmax + 1) * sizeof(int32_t));
    for (int i = 0; i < 2; ++i) h.len[i] = (int32_t*)take((size_t)B * sizeof(int32_t));
    for (int i = 0; i < 2; ++i) h.stats[i] = (double*)take((size_t)B * (gmax + 1) * 2 * sizeof(double));
    for (int i = 0; i < 2; ++i) h.filt[i] = (RowFilter*)take((size_t)B * (gmax + 1) * sizeof(RowFilter));
    h.bytes = off;
    return h;
}
}  // namespace

size_t hola_hsd_workspace_bytes(int32_t n_models, int32_t B, int32_t gamma, int32_t V)
{
    if (n_models < 2 || !shape_ok(B, gamma, V) || gamma + n_models - 2 > HOLA_MAX_GAMMA) return 0;
    return carve_hsd(nullptr, n_models, B, gamma, V).bytes + 256;
}

hola_status hola_hsd_verify(const hola_model_logits* models, int32_t n_models, int32_t dtype,
                            const int32_t* draft_tokens, uint64_t seed, int64_t seq_base, int32_t B, int32_t gamma,
                            int32_t V, const float* row_temperature, float temperature, const float* tau,
                            int32_t* out_tokens, int32_t* out_accept_len, int32_t* out_next_token, float* out_entropy,
                            void* workspace, size_t workspace_bytes, hola_stream_t stream)
{
    hola_hsd_args a;
    memset(&a, 0, sizeof a);
    a.models = models; a.n_models = n_models; a.dtype = dtype; a.draft_tokens = draft_tokens;
    a.seed = seed; a.seq_base = seq_base; a.B = B; a.gamma = gamma; a.V = V;
    a.row_temperature = row_temperature; a.temperature = temperature; a.tau = tau; a.survivors_only = 0;
    a.out_tokens = out_tokens; a.out_accept_len = out_accept_len; a.out_next_token = out_next_token;
    a.out_entropy = out_entropy; a.workspace = workspace; a.workspace_bytes = workspace_bytes; a.stream = stream;
    return hola_hsd_verify_ex(&a);
}

hola_status hola_hsd_verify_ex(const hola_hsd_args* args)
{
    if (!args) return HOLA_ERR_INVALID_ARG;
    const hola_model_logits* models = args->models;
    const int32_t n_models = args->n_models, dtype = args->dtype, B = args->B, gamma = args->gamma, V = args->V;
    const int32_t* draft_tokens = args->draft_tokens;
    const uint64_t seed = args->seed;
    const int64_t seq_base = args->seq_base;
    const float* row_temperature = args->row_temperature;
    const float temperature = args->temperature;
    const float* tau = args->tau;
    int32_t* out_tokens = args->out_tokens;
    int32_t* out_accept_len = args->out_accept_len;
    int32_t* out_next_token = args->out_next_token;
    float* out_entropy = args->out_entropy;
    void* workspace = args->workspace;
    const size_t workspace_bytes = args->workspace_bytes;
    hola_stream_t stream = args->stream;
    if (!models || !tau || n_models < 2 || !shape_ok(B, gamma, V) || gamma + n_models - 2 > HOLA_MAX_GAMMA)
        return HOLA_ERR_INVALID_ARG;
    if (dtype != HOLA_DTYPE_F32 && dtype != HOLA_DTYPE_BF16) return HOLA_ERR_UNSUPPORTED;
    if (B == 0) return HOLA_OK;
    if (!draft_tokens || !out_accept_len || !out_next_token) return HOLA_ERR_INVALID_ARG;
    for (int k = 0; k < n_models; ++k) {
        if (!models[k].logits) return HOLA_ERR_INVALID_ARG;
        if (models[k].ld && models[k].ld < V) return HOLA_ERR_INVALID_ARG;
        if (k < n_models - 1 && std::isnan(tau[k])) return HOLA_ERR_INVALID_ARG;
    }
    if (!(temperature >= 0.f) || std::isinf(temperature)) return HOLA_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return HOLA_ERR_WORKSPACE;
    if (workspace_bytes < hola_hsd_workspace_bytes(n_models, B, gamma, V)) return HOLA_ERR_WORKSPACE;

    hipStream_t s = (hipStream_t)stream;
    const int L = n_models - 1;
    const int32_t gmax = gamma + L - 1;
    const int64_t out_ld = gamma + L;                  // width of out_tokens
    const HsdWs h = carve_hsd(workspace, n_models, B, gamma, V);
    const int32_t* cur_tok = draft_tokens;
    int64_t cur_ld = gamma;
    const int32_t* cur_len = nullptr;
    const double* cur_stats = nullptr;
    const RowFilter* cur_filt = nullptr;
    for (int k = 1; k <= L; ++k) {
        const int32_t gk = gamma + k - 1;
        hola_verify_args a;
        memset(&a, 0, sizeof a);
        a.target_logits = models[k].logits; a.draft_logits = models[k - 1].logits; a.dtype = dtype;
        a.target_ld = models[k].ld; a.draft_ld = models[k - 1].ld;
        a.draft_tokens = cur_tok; a.draft_len = cur_len; a.row_temperature = row_temperature;
        a.top_k = args->top_k; a.top_p = args->top_p;
        const bool filtered = (args->top_k != 0 && args->top_k < V) || (args->top_p != 0.f && !(args->top_p >= 1.f));
        a.draft_stats_in = filtered ? nullptr : cur_stats;
        a.target_stats_out = (k < L && !filtered) ? h.stats[k & 1] : nullptr;
        a.seed = seed; a.level = (uint32_t)(k - 1); a.seq_base = seq_base;
        a.B = B; a.gamma = gk; a.V = V; a.temperature = temperature; a.entropy_threshold = tau[k - 1];
        a.out_accept_len = out_accept_len; a.out_next_token = out_next_token;
        a.out_entropy = out_entropy ? out_entropy + (int64_t)(k - 1) * B * gmax : nullptr;
        a.entropy_ld = gmax;
        a.workspace = h.level; a.workspace_bytes = h.level_bytes; a.stream = stream;
        a.tuning = args->tuning;
        LevelExtras x;
        x.tokens_ld = cur_ld;
        x.pad_entropy = 1;
        x.glue_keep_next = args->survivors_only ? 0 : 1;
        if (filtered) {
            x.draft_filters_in = cur_filt;                     // null at the first level: it scans its draft rows itself
            x.target_filters_out = k < L ? h.filt[k & 1] : nullptr;
        }
        if (k < L) {
            // The next level's drafts are written by this level.  The last middle level writes them
            // straight into out_tokens (when given), which the last level then reads in place.
            x.glue_len = h.len[k & 1];
            if (k == L - 1 && out_tokens) { x.glue_tok = out_tokens; x.glue_ld = out_ld; }
            else { x.glue_tok = h.tok[k & 1]; x.glue_ld = gk + 1; }
        }
        hola_status st = run_level(a, x);
        if (st != HOLA_OK) return st;
        if (k < L) {
            cur_tok = x.glue_tok; cur_ld = x.glue_ld;
            cur_len = x.glue_len;
            cur_stats = h.stats[k & 1];
            cur_filt = filtered ? h.filt[k & 1] : nullptr;
        }
    }
    if (out_tokens && cur_tok != out_tokens) {          // a single level: its drafts are the caller's tokens
        StageTimer t(4, s);
        const int tpb = 128, nb = (B + tpb - 1) / tpb;
        hipLaunchKernelGGL(export_tokens_kernel, dim3(nb), dim3(tpb), 0, s, cur_tok, cur_ld, gmax, cur_len, B,
                           (int32_t)out_ld, out_tokens);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "export launch");
    }
    return HOLA_OK;
}

size_t hola_tree_workspace_bytes(int32_t B, int32_t N, int32_t V)
{
    if (!shape_ok(B, N, V)) return 0;
    // the wavefront partials of the N draft and N + 1 target rows of every sequence; nothing else
    return align_up((size_t)B * (2 * (size_t)N + 1) * kMaxSplit * kWaves * sizeof(Partial)) + 256;
}

hola_status hola_verify_tree(const hola_tree_args* args)
{
    if (!args) return HOLA_ERR_INVALID_ARG;
    const hola_tree_args& a = *args;
    if (!shape_ok(a.B, a.N, a.V)) return HOLA_ERR_INVALID_ARG;
    if (a.dtype != HOLA_DTYPE_F32 && a.dtype != HOLA_DTYPE_BF16) return HOLA_ERR_UNSUPPORTED;
    if (a.B == 0) return HOLA_OK;
    if (!a.target_logits || !a.draft_logits || !a.node_token || !a.node_parent || !a.out_accept_len || !a.out_next_token)
        return HOLA_ERR_INVALID_ARG;
    const size_t es = a.dtype == HOLA_DTYPE_BF16 ? 2 : 4;
    if (((uintptr_t)a.target_logits % es) || ((uintptr_t)a.draft_logits % es)) return HOLA_ERR_INVALID_ARG;
    if ((a.target_ld && a.target_ld < a.V) || (a.draft_ld && a.draft_ld < a.V)) return HOLA_ERR_INVALID_ARG;
    if (std::isnan(a.temperature) || std::isinf(a.temperature) || a.temperature < 0.f) return HOLA_ERR_INVALID_ARG;
    if (std::isnan(a.entropy_threshold)) return HOLA_ERR_INVALID_ARG;
    if (!(a.temperature > 0.f) || !tree_supported(a.N, a.V, a.dtype)) return HOLA_ERR_UNSUPPORTED;
    if (!a.workspace || ((uintptr_t)a.workspace & 255)) return HOLA_ERR_WORKSPACE;
    if (a.workspace_bytes < hola_tree_workspace_bytes(a.B, a.N, a.V)) return HOLA_ERR_WORKSPACE;

    hipStream_t s = (hipStream_t)a.stream;
    Partial* partials = (Partial*)a.workspace;
    const int64_t tld = a.target_ld ? a.target_ld : a.V, dld = a.draft_ld ? a.draft_ld : a.V;
    Tuning tune;
    if (!call_tuning(a.tuning, &tune)) return HOLA_ERR_INVALID_ARG;
    const int64_t rows = (int64_t)a.B * (2 * (int64_t)a.N + 1);
    const int nsplit = choose_split(rows, a.V, a.dtype, tune);

    hipError_t e;
    RowStatsParams rs{};
    rs.target = a.target_logits; rs.draft = a.draft_logits; rs.target_ld = tld; rs.draft_ld = dld;
    rs.draft_len = a.n_nodes; rs.temperature = a.temperature;
    rs.B = a.B; rs.gamma = a.N; rs.V = a.V; rs.nsplit = nsplit;
    rs.lse_only_targets = 1;                                    // only the drafts' entropy gates
    rs.tree_parent = a.node_parent;                             // draft rows of childless contexts are not read
    rs.partials = partials;
    { StageTimer t(0, s); e = launch_row_stats(rs, a.dtype, tune, s); }
    if (e != hipSuccess) return hip_fail(e, "row statistics launch");

    TreeParams tp{};
    tp.target = a.target_logits; tp.draft = a.draft_logits; tp.dtype = a.dtype; tp.target_ld = tld; tp.draft_ld = dld;
    tp.tokens = a.node_token; tp.parent = a.node_parent; tp.n_nodes = a.n_nodes;
    tp.seed = a.seed; tp.level = a.level; tp.seq_base = a.seq_base;
    tp.B = a.B; tp.N = a.N; tp.V = a.V; tp.ntiles = sampler_tiles(a.V, a.dtype);
    tp.temperature = a.temperature; tp.tau = a.entropy_threshold;
    tp.sc = host_scale((double)a.temperature);
    tp.out_accept_len = a.out_accept_len; tp.out_path = a.out_path; tp.out_next_token = a.out_next_token;
    tp.out_entropy = a.out_entropy;
    const int waves = tune.fused_waves ? tune.fused_waves : (a.B <= device_cu_count() ? 16 : 8);
    { StageTimer t(6, s); e = launch_tree_tail(tp, partials, nsplit * kWaves, waves, s); }
    if (e != hipSuccess) return hip_fail(e, "tree tail launch");
    return HOLA_OK;
}

hola_status hola_row_stats(const void* logits, int32_t dtype, int64_t ld, int32_t R, int32_t V, float temperature,
                           double* stats_out, void* workspace, size_t workspace_bytes, hola_stream_t stream)
{
    if (R < 0 || V < 1) return HOLA_ERR_INVALID_ARG;
    if (dtype != HOLA_DTYPE_F32 && dtype != HOLA_DTYPE_BF16) return HOLA_ERR_UNSUPPORTED;
    if (R == 0) return HOLA_OK;
    if (!logits || !stats_out || !(temperature > 0.f) || std::isinf(temperature)) return HOLA_ERR_INVALID_ARG;
    if (ld && ld < V) return HOLA_ERR_INVALID_ARG;
    if ((uintptr_t)logits % (dtype == HOLA_DTYPE_BF16 ? 2 : 4)) return HOLA_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return HOLA_ERR_WORKSPACE;
    if (workspace_bytes < carve(nullptr, R, 1, V, false).bytes + 256) return HOLA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const Workspace w = carve(workspace, R, 1, V, false);
    const Tuning tune = g_tuning;
    const int nsplit = choose_split(R, V, dtype, tune);
    // R plain rows are laid out as R "sequences" with no draft and one target row each.
    RowStatsParams rs{};
    rs.target = logits; rs.draft = logits; rs.target_ld = ld ? ld : V; rs.draft_ld = rs.target_ld;
    rs.temperature = temperature; rs.B = R; rs.gamma = 0; rs.V = V; rs.nsplit = nsplit; rs.skip_draft = 1;
    rs.partials = w.partials;
    hipError_t e;
    { StageTimer t(0, s); e = launch_row_stats(rs, dtype, tune, s); }
    if (e != hipSuccess) return hip_fail(e, "row statistics launch");
    {
        StageTimer t(1, s);
        e = launch_finalize_rows(w.partials, nsplit * kWaves, R, stats_out, s);
    }
    if (e != hipSuccess) return hip_fail(e, "finalize launch");
    return HOLA_OK;
}

// Vocabulary-tiled statistics.  A tile is a row of its own to the split-row kernel (R * ntiles virtual rows).
static int tiles_of(int32_t V, int32_t tile_cols) { return (int)(((int64_t)V + tile_cols - 1) / tile_cols); }

size_t hola_tile_stats_workspace_bytes(int32_t R, int32_t V, int32_t tile_cols)
{
    if (R < 0 || V < 1 || tile_cols < 1) return 0;
    const int64_t vr = (int64_t)R * tiles_of(V, tile_cols);
    if (vr > 0x7fffffffLL) return 0;
    return carve(nullptr, (int32_t)vr, 1, tile_cols < V ? tile_cols : V, false).bytes + 256;
}

hola_status hola_tile_stats(const void* logits, int32_t dtype, int64_t ld, int32_t R, int32_t V, int32_t tile_cols,
                            float temperature, double* tile_stats_out, void* workspace, size_t workspace_bytes,
                            hola_stream_t stream)
{
    if (R < 0 || V < 1 || tile_cols < 1) return HOLA_ERR_INVALID_ARG;
    if (dtype != HOLA_DTYPE_F32 && dtype != HOLA_DTYPE_BF16) return HOLA_ERR_UNSUPPORTED;
    if (R == 0) return HOLA_OK;
    if (!logits || !tile_stats_out || !(temperature > 0.f) || std::isinf(temperature)) return HOLA_ERR_INVALID_ARG;
    if (ld && ld < V) return HOLA_ERR_INVALID_ARG;
    if ((uintptr_t)logits % (dtype == HOLA_DTYPE_BF16 ? 2 : 4)) return HOLA_ERR_INVALID_ARG;
    const int nt = tiles_of(V, tile_cols);
    const int64_t vr = (int64_t)R * nt;
    if (vr > 0x7fffffffLL) return HOLA_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255)) return HOLA_ERR_WORKSPACE;
    if (workspace_bytes < hola_tile_stats_workspace_bytes(R, V, tile_cols)) return HOLA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int32_t tc = tile_cols < V ? tile_cols : V;
    const Workspace w = carve(workspace, (int32_t)vr, 1, tc, false);
    const Tuning tune = g_tuning;
    const int nsplit = choose_split(vr, tc, dtype, tune);
    RowStatsParams rs{};
    rs.target = logits; rs.draft = logits; rs.target_ld = ld ? ld : V; rs.draft_ld = rs.target_ld;
    rs.temperature = temperature; rs.B = (int32_t)vr; rs.gamma = 0; rs.V = V; rs.nsplit = nsplit; rs.skip_draft = 1;
    rs.tile_cols = tc; rs.ntiles = nt;
    rs.partials = w.partials;
    hipError_t e;
    { StageTimer t(0, s); e = launch_row_stats(rs, dtype, tune, s); }
    if (e != hipSuccess) return hip_fail(e, "tile statistics launch");
    { StageTimer t(1, s); e = launch_finalize_rows(w.partials, nsplit * kWaves, (int32_t)vr, tile_stats_out, s); }
    if (e != hipSuccess) return hip_fail(e, "finalize launch");
    return HOLA_OK;
}

hola_status hola_merge_tile_stats(const double* tile_stats, int32_t R, int32_t ntiles, double* stats_out, hola_stream_t stream)
{
    if (R < 0 || ntiles < 1) return HOLA_ERR_INVALID_ARG;
    if (R == 0) return HOLA_OK;
    if (!tile_stats || !stats_out) return HOLA_ERR_INVALID_ARG;
    hipError_t e;
    { StageTimer t(4, (hipStream_t)stream); e = launch_merge_tile_stats(tile_stats, R, ntiles, stats_out, (hipStream_t)stream); }
    return e == hipSuccess ? HOLA_OK : hip_fail(e, "tile merge launch");
}

hola_status hola_copy_bytes(void* dst, const void* src, size_t bytes, hola_stream_t stream)
{
    if (bytes == 0) return HOLA_OK;
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return HOLA_ERR_INVALID_ARG;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst, (const uint4*)src, n);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HOLA_OK : hip_fail(e, "copy launch");
}

hola_status hola_read_probe(const void* src, size_t bytes, size_t block_bytes, int32_t nontemporal, int32_t arithmetic,
                            hola_stream_t stream)
{
    if (bytes == 0) return HOLA_OK;
    if (!src || (bytes & 15) || ((uintptr_t)src & 15) || block_bytes < 16 || block_bytes > ((size_t)1 << 40)) return HOLA_ERR_INVALID_ARG;
    hipError_t e;
    { StageTimer t(10, (hipStream_t)stream); e = launch_read_probe(src, bytes, (int64_t)block_bytes, nontemporal, arithmetic, (hipStream_t)stream); }
    return e == hipSuccess ? HOLA_OK : hip_fail(e, "read probe launch");
}

hola_status hola_set_tuning(const hola_tuning* t)
{
    Tuning n;
    if (!tuning_from(t, &n)) return HOLA_ERR_INVALID_ARG;
    g_tuning = n;                                              // the calling thread's defaults
    return HOLA_OK;
}

hola_status hola_profile_enable(int32_t on)
{
    g_prof_on = on != 0;                                       // the calling thread's calls only
    return HOLA_OK;
}

hola_status hola_profile_collect(double* ms_out, int64_t* launches_out)
{
    if (!ms_out || !launches_out) return HOLA_ERR_INVALID_ARG;
    std::vector<ProfEvent> live;
    live.swap(g_prof_live);
    hola_status st = HOLA_OK;
    for (const ProfEvent& ev : live) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ev.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
        if (e != hipSuccess) st = hip_fail(e, "profile event");
        else if (ev.stage >= 0 && ev.stage < HOLA_N_STAGES) { ms_out[ev.stage] += ms; launches_out[ev.stage] += 1; }
    }
    for (const ProfEvent& ev : live) g_prof_free.emplace_back(ev.a, ev.b);
    return st;
}

hola_status hola_profile_collect_launches(int32_t* stage_out, float* ms_out, int64_t capacity, int64_t* n_out)
{
    if (!stage_out || !ms_out || !n_out || capacity < 0) return HOLA_ERR_INVALID_ARG;
    std::vector<ProfEvent> live;
    live.swap(g_prof_live);
    hola_status st = HOLA_OK;
    int64_t n = 0;
    for (const ProfEvent& ev : live) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ev.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
        if (e != hipSuccess) { st = hip_fail(e, "profile event"); continue; }
        if (n < capacity) { stage_out[n] = ev.stage; ms_out[n] = ms; }
        ++n;
    }
    *n_out = n;
    for (const ProfEvent& ev : live) g_prof_free.emplace_back(ev.a, ev.b);
    return st;
}

void hola_shutdown(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int cur = 0;
    bool have_dev = hipGetDevice(&cur) == hipSuccess;
    for (int d = 0; d < 64; ++d) {
        if (!g_ws[d].ptr) continue;
        if (have_dev) (void)hipSetDevice(d);
        (void)hipFree(g_ws[d].ptr);
        g_ws[d].ptr = nullptr; g_ws[d].bytes = 0;
    }
    if (have_dev) (void)hipSetDevice(cur);
    for (auto& ev : g_prof_live) { (void)hipEventDestroy(ev.a); (void)hipEventDestroy(ev.b); }
    for (auto& ev : g_prof_free) { (void)hipEventDestroy(ev.first); (void)hipEventDestroy(ev.second); }
    g_prof_live.clear();
    g_prof_free.clear();
}

const char* hola_status_string(hola_status s)
{
    switch (s) {
        case HOLA_OK: return "ok";
        case HOLA_ERR_INVALID_ARG: return "invalid argument";
        case HOLA_ERR_UNSUPPORTED: return "unsupported";
        case HOLA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case HOLA_ERR_HIP: return "HIP error";
    }
    return "unknown status";
}

const char* hola_last_hip_error(void) { return g_last_hip; }
const char* hola_version(void) { return "hola-verify 0.2 (gfx950)"; }

}  // extern "C"
