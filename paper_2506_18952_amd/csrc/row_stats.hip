// Split-row statistics kernel: one streaming pass over every logit of the draft and target rows,
// one workgroup of 4 wavefronts per (row, segment).  Used when there are too few sequences to give
// every compute unit a sequence of its own (see fused.hip for that case) and by hola_row_stats.
//
// A lane reads 16-byte chunks with workgroup stride, UNROLL of them in flight; each wavefront writes
// one Partial (stats_device.h), merged later in double by the accept kernel.  HBM-bound: no LDS, no
// barrier, no matrix cores (there is no contraction here).
#include "stats_device.h"

namespace hola {

template <bool BF16, bool ARGMAX, int U, bool WITH_T = true>
__device__ __forceinline__ void row_segment(const void* row, int32_t V, int seg, int nsplit, bool slabs, const ExpScale& sc,
                                            Partial* __restrict__ out /* [kWaves] of this (row, segment) */)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const RowGeom g = make_geom<BF16>(row, V);
    // The segment's chunks go to the four wavefronts interleaved in blocks of 64 (the fastest order: 3.5 % faster
    // than four contiguous slabs), except on the row a bonus token would be drawn from, where each wavefront
    // takes a contiguous slab so that the sampler can pick a slab from the partial sums.
    int64_t seg_lo, seg_hi, lo, hi;
    wave_slab(g, seg, nsplit, wave, seg_lo, seg_hi, lo, hi);
    const bool do_edges = (seg == 0 && wave == 0);
    const Partial res = wave_row_share<BF16, ARGMAX, U, WITH_T>(g, slabs ? lo + lane : seg_lo + tid, slabs ? hi : seg_hi,
                                                                slabs ? 64 : kBlock, do_edges, sc, lane);
    if (lane == 0) out[wave] = res;
}

// GREEDY: the call has per-row temperatures (or temperature 0), so target rows of greedy sequences also look for
// their argmax.  Calls with one temperature > 0 take the instantiation without that path: 68 instead of 79 vector registers, seven instead
// of six wavefronts per SIMD.
template <bool BF16, int U, bool GREEDY>
__global__ __launch_bounds__(kBlock) void row_stats_kernel(RowStatsParams p)
{
    const int nsplit = p.nsplit;
    const int64_t blk = blockIdx.x;
    const int seg = (int)(blk % nsplit);
    const int64_t r = blk / nsplit;
    const int g = p.gamma;
    const int n_d = p.skip_draft ? 0 : g, n_t = p.skip_target ? 0 : g + 1;
    const int rows_per_seq = n_d + n_t;
    const int b = (int)(r / rows_per_seq);
    const int k = (int)(r % rows_per_seq);
    const bool is_draft = k < n_d;
    const int j = is_draft ? k : k - n_d;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    if (is_draft ? (j >= len) : (p.literal ? (j >= len) : (j > len))) return;   // row not needed (uniform exit)
    if (is_draft && p.tree_parent) {                             // token trees: context j needs a child among the nodes
        const int n = threadIdx.x & 63;                          // (node n hangs under context parent[n] + 1, n >= j)
        const bool child = n >= j && n < len && p.tree_parent[(int64_t)b * g + n] == j - 1;
        if (!__ballot(child)) return;                            // the same answer in every wavefront
    }

    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const bool greedy = !(Tb > 0.f);
    const ExpScale sc = p.sc_given ? p.sc : make_scale(greedy ? kLog2e : kLog2e / (double)Tb);
    constexpr int ES = BF16 ? 2 : 4;
    const char* row;
    int64_t slot;
    int32_t Vrow = p.V;
    if (p.ntiles > 0) {                                          // column tile of a plain row
        const int64_t pr = b / p.ntiles, t = b % p.ntiles;
        row = (const char*)p.target + (pr * p.target_ld + t * p.tile_cols) * ES;
        const int64_t left = (int64_t)p.V - t * p.tile_cols;
        Vrow = (int32_t)(left < p.tile_cols ? left : p.tile_cols);
        slot = b;
    } else if (is_draft) {
        row = (const char*)p.draft + ((int64_t)b * g + j) * p.draft_ld * ES;
        slot = (int64_t)b * g + j;
    } else {
        row = (const char*)p.target + ((int64_t)b * (g + 1) + j) * p.target_ld * ES;
        slot = (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
    }
    Partial* out = p.partials + (slot * nsplit + seg) * kWaves;
    // rows a token may be drawn from with p itself as the weights: the row of the bonus token, or, in the literal mode,
    // every target row (a verifier draw at each position that is not gated)
    const bool slabs = !is_draft && p.ntiles == 0 && (p.literal ? true : j == len);
    if (GREEDY && greedy && !is_draft) row_segment<BF16, true, U>(row, Vrow, seg, nsplit, slabs, sc, out);
    else if (!is_draft && p.lse_only_targets) row_segment<BF16, false, U, false>(row, Vrow, seg, nsplit, slabs, sc, out);
    else row_segment<BF16, false, U>(row, Vrow, seg, nsplit, slabs, sc, out);
}

int choose_split(int64_t rows, int V, int dtype, const Tuning& t)
{
    const int epl = (dtype == HOLA_DTYPE_BF16) ? 8 : 4;
    const int64_t chunks = ((int64_t)V + epl - 1) / epl;
    int max_useful = (int)((chunks + kBlock - 1) / kBlock);  // at least one chunk per lane per segment
    if (max_useful < 1) max_useful = 1;
    int s = t.split;
    if (s <= 0) {
        // Workgroups cost dispatch time (about 1.3 us per thousand on MI355X), so a row is split only as far as it
        // pays.  Fewer rows than compute units: split down to two chunks per lane, so that every unit gets work.
        // Up to ~2048 workgroups (8 per compute unit): split while a lane keeps two groups of 8 loads.  Beyond
        // that, towards 8192 workgroups, only while a lane keeps at least 24 chunks (three groups of 8 loads):
        // shorter segments cost more in ramp-up than the shorter last round of the grid gains.
        s = 1;
        while (rows * s < 256 && s < kMaxSplit && chunks / (s * 2) >= (int64_t)kBlock * 2) s *= 2;
        while (rows * s < 2048 && s < kMaxSplit && chunks / (s * 2) >= (int64_t)kBlock * 8) s *= 2;
        while (rows * s < 8192 && s < kMaxSplit && chunks / (s * 2) >= (int64_t)kBlock * 24) s *= 2;
    }
    if (s > kMaxSplit) s = kMaxSplit;
    if (s > max_useful) s = max_useful;
    return s < 1 ? 1 : s;
}

template <bool BF16>
static hipError_t launch_typed(const RowStatsParams& p_in, const Tuning& t, hipStream_t s)
{
    RowStatsParams p = p_in;
    p.sc_given = (p.row_temperature == nullptr && p.temperature > 0.f) ? 1 : 0;
    if (p.sc_given) p.sc = host_scale((double)p.temperature);
    const int g = p.gamma;
    const int64_t rows = (int64_t)p.B * ((p.skip_draft ? 0 : g) + (p.skip_target ? 0 : g + 1));
    const int64_t nblk = rows * p.nsplit;
    if (nblk <= 0) return hipSuccess;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)nblk), block(kBlock);
    const int U = t.unroll ? t.unroll : 8;
    const bool greedy_rows = p.row_temperature != nullptr || !(p.temperature > 0.f);   // some row may want its argmax
#define HOLA_ROW_STATS(UU) do { \
        if (greedy_rows) hipLaunchKernelGGL((row_stats_kernel<BF16, UU, true>), grid, block, 0, s, p); \
        else hipLaunchKernelGGL((row_stats_kernel<BF16, UU, false>), grid, block, 0, s, p); } while (0)
    if (U == 16) HOLA_ROW_STATS(16);
    else if (U == 2) HOLA_ROW_STATS(2);
    else if (U == 4) HOLA_ROW_STATS(4);
    else HOLA_ROW_STATS(8);
#undef HOLA_ROW_STATS
    return hipGetLastError();
}

hipError_t launch_row_stats(const RowStatsParams& p, int dtype, const Tuning& t, hipStream_t s)
{
    return dtype == HOLA_DTYPE_BF16 ? launch_typed<true>(p, t, s) : launch_typed<false>(p, t, s);
}

}  // namespace hola
