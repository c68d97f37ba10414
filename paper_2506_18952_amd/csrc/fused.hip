// Per-sequence kernels: one workgroup of 4, 8 or 16 wavefronts owns one sequence.
//
// fused_kernel runs the whole verify step for its sequence without leaving the compute unit: row
// statistics of its gamma draft and gamma+1 target rows (streamed once from HBM, wavefront partials
// parked in LDS), the accept / first-reject stage (wavefront 0), the residual or bonus tile weights of
// the stop row (all wavefronts, tile weights in LDS) and the inverse-CDF selection (wavefront 0).
//
// tail_kernel is the same minus the streaming pass: it takes the row partials the split-row kernel
// left in HBM (a segment of lanes merges one row, a lane per partial) and does accept + sampling, so the
// split path is two launches instead of four.  Its phases are arranged so that memory round trips overlap:
// see tail_kernel and sequence_tail.
//
// HBM-bound: every logit is read once, the stop row pair once more.  No spin waits anywhere; the one atomic is the
// completion ticket of a tail that several workgroups share (small batches of wide rows, see sequence_tail), which
// nobody waits for: whoever takes the last ticket carries on, the others leave.
#include "accept_device.h"
#include "filter_device.h"
#include "sampler_device.h"

namespace hola {

constexpr int kFusedMaxTiles = 2048;
constexpr int kFusedMaxGamma = 32;           // the fused kernel parks the partials of its 2 gamma + 1 rows in shared memory

constexpr int kSlabKeepChunks = 8 * 64 * kTileChunks;   // a slab of up to eight tiles is kept in shared memory (32 KB)

struct SeqShared {
    RowStat stat[2 * HOLA_MAX_GAMMA + 1];      // per row: draft rows 0..g-1, target rows g..2g
    double tiles[kFusedMaxTiles];
    SeqInfo si;
    int32_t tok;
    // bonus draw from one slab of the row (split-row partials at hand): its chunks, and where in its mass to land
    int64_t slab_lo, slab_hi;
    double slab_u;
    int32_t slab_ok;
};

// Next token of a filtered stop row whose keep set (at most kKeptListMax tokens) is at hand as a list of
// (order key << 32 | index): the weights of these tokens alone, by the sampler's own element formula (every other
// token has weight 0).  The draw is the inverse CDF in index order, found without putting the list in order: the
// weights become integers in fixed point (2^60 for the total, so sums are exact and the same in any order) and the
// index of the token is built bit by bit, each bit from one sum over the wavefront of the weights that lie below
// the half of the index range in question.  One wavefront, up to 16 entries per lane.
// Returns the token, -1 if the weights carry no mass, or -2 if the caller should draw from the target's
// distribution itself (residual without mass).
template <bool BF16, int KL>
__device__ __forceinline__ int32_t sample_kept_list_n(const RowPair& rp, const unsigned long long* kept, int nk, double u, int lane)
{
    const int nslots = (nk + 63) / 64;
    uint32_t idx[KL];
    float wk[KL];
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < KL; ++j) {
        idx[j] = 0xffffffffu;
        wk[j] = 0.f;
        const int i = j * 64 + lane;
        if (j < nslots && i < nk) {
            const unsigned long long ent = kept[i];
            idx[j] = (uint32_t)(ent & 0xffffffffu);
            const float xp = key_to_logit<BF16>((uint32_t)(ent >> 32));
            const float ep = fast_exp2(exp_arg<BF16>(xp, rp.refP, rp.sc));
            if (rp.bonus) {
                wk[j] = fmaxf(ep, 0.f);
            } else {
                const float xd = load_logit<BF16>(rp.D, (int32_t)idx[j]);
                float eq = fast_exp2(exp_arg<BF16>(xd, rp.refQ, rp.sc));
                if (!(xd > rp.thQ || (xd == rp.thQ && (int32_t)idx[j] <= rp.cutQ))) eq = 0.f;   // outside the draft's keep set
                wk[j] = fmaxf(0.f, __builtin_fmaf(-rp.k_lo, eq, __builtin_fmaf(-rp.k_hi, eq, ep)));
            }
            mine += (double)wk[j];
        }
    }
    const double Zs = wave_sum(mine);                            // in the weights' own unit (the common factor left out)
    const double Z = Zs * rp.scale;
    if (!(Z > 0.0) || !(Z - Z == 0.0)) return rp.bonus ? -1 : -2;
    const double unit = 1152921504606846976.0 / Zs;              // 2^60 for the whole list
    unsigned long long fx[KL], fsum = 0ull;
#pragma unroll
    for (int j = 0; j < KL; ++j) {
        fx[j] = (j < nslots) ? (unsigned long long)((double)wk[j] * unit) : 0ull;
        fsum += fx[j];
    }
    const unsigned long long total = wave_sum_u64(fsum);
    if (total == 0ull) return -1;
    unsigned long long target = (unsigned long long)(u * (double)total);
    if (target >= total) target = total - 1;                     // u < 1: the draw lies inside the mass
    // smallest index x with (sum of the weights at indices <= x) > target
    int vbits = 0;
    while (vbits < 31 && ((int64_t)1 << vbits) < (int64_t)rp.V) ++vbits;
    uint32_t prefix = 0;
    unsigned long long below = 0ull;                             // mass at indices < prefix
    for (int bit = vbits - 1; bit >= 0; --bit) {
        const uint32_t want = prefix >> bit;                     // the half with this bit clear
        unsigned long long s0 = 0ull;
#pragma unroll
        for (int j = 0; j < KL; ++j)
            if (j < nslots && (idx[j] >> bit) == want) s0 += fx[j];
        s0 = wave_sum_u64(s0);
        if (below + s0 <= target) { below += s0; prefix |= 1u << bit; }
    }
    return (int32_t)prefix;
}

// Lists of up to 64, 256 and kKeptListMax tokens, each with as many entries per lane as it needs.
template <bool BF16>
__device__ __forceinline__ int32_t sample_kept_list(const RowPair& rp, const unsigned long long* kept, int nk, double u, int lane)
{
    if (nk <= 64) return sample_kept_list_n<BF16, 1>(rp, kept, nk, u, lane);
    if (nk <= 256) return sample_kept_list_n<BF16, 4>(rp, kept, nk, u, lane);
    return sample_kept_list_n<BF16, kKeptListMax / 64>(rp, kept, nk, u, lane);
}

__device__ __forceinline__ AcceptCtx accept_ctx(const FusedParams& p)
{
    AcceptCtx c;
    c.target = p.target; c.draft = p.draft; c.target_ld = p.target_ld; c.draft_ld = p.draft_ld;
    c.tokens = p.tokens; c.tokens_ld = p.tokens_ld; c.pad_entropy = p.pad_entropy; c.seed = p.seed; c.level = p.level; c.seq_base = p.seq_base;
    c.gamma = p.gamma; c.V = p.V; c.tau = p.tau; c.target_stats_out = p.target_stats_out;
    c.out_accept_len = p.out_accept_len; c.out_next_token = p.out_next_token;
    c.out_entropy = p.out_entropy; c.entropy_ld = p.entropy_ld;
    c.filters = p.filters; c.draft_filters = p.draft_filters ? p.draft_filters : p.filters; c.B = p.B;
    return c;
}

// Drafts of the next verify level: the kept tokens of this level followed by its next token.
__device__ __forceinline__ void write_glue(const FusedParams& p, int b, int a, int32_t next)
{
    if (!p.glue_tok) return;
    for (int64_t j = threadIdx.x; j < p.glue_ld; j += blockDim.x)
        p.glue_tok[(int64_t)b * p.glue_ld + j] =
            j < a ? p.tokens[(int64_t)b * p.tokens_ld + j] : ((j == a && p.glue_keep_next) ? next : -1);
    if (threadIdx.x == 0) p.glue_len[b] = a + (p.glue_keep_next ? 1 : 0);
}

// Bonus draw from one slab of the row, decided before the accept stage has run: pick_row_slab (sampler_device.h) for
// target row len with the sampling uniform of position len.  Neither depends on the accept stage, so one wavefront
// does this while the others merge statistics and gather the drafted tokens' logits, and the slab can be swept while
// the accept stage decides.  If the sequence turns out rejected, the work is dropped.  Called by one whole
// wavefront; fills sh.slab_*.
template <bool BF16>
__device__ __forceinline__ bool pick_bonus_slab(const FusedParams& p, int b, int len, const Partial* parts, int nparts, int lane,
                                                int64_t& lo, int64_t& hi, double& frac)
{
    const uint64_t seq = (uint64_t)(p.seq_base + b);
    const Philox4 r = philox4x32_10((uint32_t)len, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                    (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
    return pick_row_slab<BF16>(p.target, p.target_ld, p.gamma, p.V, p.B, b, len, parts, nparts, (double)u24(r.y), lane,
                               lo, hi, frac);
}

// Accept stage (wavefront 0) and sampling (all wavefronts) of sequence b, given sh.stat[] and, in wavefront 0, the
// gathered token logits tg.  Called by every thread of the workgroup, after a barrier that made sh.stat (and, with
// pre_slab, sh.slab_*) visible.  pre_slab: pick_bonus_slab has run; while wavefront 0 decides, the others sweep the
// slab it chose, so that a sequence whose drafts are all kept finds its tile weights ready.
// slab_raw: kSlabKeepChunks chunks of shared memory in which the sweep of a slab that fits leaves the chunks it
// loaded, so that the selection does not read its tile from global memory again; or null.
// chunk_sums: kSumsKeepTiles x 64 entries of shared memory in which a sweep of at most that many tiles leaves every
// lane's chunk sums, so that the selection rebuilds one chunk of the crossing tile instead of four; or null.
// part, G: this workgroup is one of G that share sequence b's tail (G = 1: the usual case).  Every one of them
// decides (the decision costs little and all need it); only part 0 writes the decision's outputs.  Where the
// stop row must be swept whole, each part sweeps a contiguous G-th of its tiles, leaves the tile weights in
// p.coop_tiles and takes a ticket; the last to arrive reads the others' weights and draws the token.  The weights
// and the draw are those of a workgroup on its own: every tile is summed by one wavefront either way.
template <bool BF16, int NW, bool FILT = false, bool COOP = false>
__device__ __forceinline__ void sequence_tail(const FusedParams& p, SeqShared& sh, int b, int len, float Tb,
                                              const TokenGather& tg, bool pre_slab = false, uint4* slab_raw = nullptr,
                                              float4* chunk_sums = nullptr, int part = 0, int G = 1,
                                              const TilePre pre = TilePre{})
{
    static_assert(!COOP || (NW == 16 && !FILT), "a shared tail is the 16-wavefront unfiltered variant's alone");
    if (!COOP) { part = 0; G = 1; }
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const int g = p.gamma;
    constexpr int N = BF16 ? 8 : 4;
    const ExpScale* const scp = p.sc_given ? &p.sc : nullptr;       // one temperature: the host made the constants
    const bool slab_ready = pre_slab && sh.slab_ok;                 // uniform over the workgroup
    const int64_t slab_lo = slab_ready ? sh.slab_lo : 0, slab_hi = slab_ready ? sh.slab_hi : 0;
    const int slab_tiles = (int)((slab_hi - slab_lo + 64 * kTileChunks - 1) / (64 * kTileChunks));
    uint4* keep = (slab_ready && slab_hi - slab_lo <= kSlabKeepChunks) ? slab_raw : nullptr;
    if (wave == 0) {
        const int j = lane;
        RowStat sd = {NAN, NAN, -1}, sp = {NAN, NAN, -1};
        if (j < len) {
            if (p.draft_stats_in) {
                sd.lse = p.draft_stats_in[((int64_t)b * g + j) * 2 + 0];
                sd.H = p.draft_stats_in[((int64_t)b * g + j) * 2 + 1];
            } else {
                sd = sh.stat[j];
            }
        }
        if (j <= len) {
            if (p.target_stats_in) {
                sp.lse = p.target_stats_in[((int64_t)b * (g + 1) + j) * 2 + 0];
                sp.H = p.target_stats_in[((int64_t)b * (g + 1) + j) * 2 + 1];
            } else {
                sp = sh.stat[g + j];
            }
        }
        if constexpr (COOP) {
            AcceptCtx c = accept_ctx(p);
            c.write_outputs = part == 0;
            accept_decide<BF16>(c, b, j, len, Tb, sd, sp, tg, &sh.si);
        } else {
            const AcceptCtx c = accept_ctx(p);
            accept_decide<BF16>(c, b, j, len, Tb, sd, sp, tg, &sh.si);
        }
    }
    else if (slab_ready && (!COOP || part == 0)) {
        // the slab's tile weights as bonus weights of target row len, by the wavefronts that do not decide
        SeqInfo sb;
        sb.lseP = sh.stat[g + len].lse; sb.lseD = 0.0; sb.u = 0.f; sb.row = len; sb.mode = 1; sb.greedy_tok = -1;
        RowPair rq;
        make_row_pair<BF16>(rq, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, sb, 0, nullptr, p.B, nullptr, scp);
        if (rq.ok) {
            narrow_to_slab<BF16>(rq, slab_lo, slab_hi);
            // a slab is a few tiles: one per wavefront, the last wavefront first (those are the ones with nothing to
            // merge, which had their tile's chunks in flight since before the statistics were there: pre)
            float4* const ssums = slab_tiles <= kSumsKeepTiles ? chunk_sums : nullptr;
            int t = (NW - 1) - wave;
            if (pre.ok) {
                const double w0 = tile_weight_preloaded<BF16>(rq, t, lane, pre, keep, ssums);
                if (lane == 0) sh.tiles[t] = w0;
                t += NW - 1;
            }
            for (; t < slab_tiles; t += NW - 1) {
                const double w0 = tile_weight<BF16>(rq, t, lane, keep, ssums);
                if (lane == 0) sh.tiles[t] = w0;
            }
        }
    }
    __syncthreads();
    const SeqInfo si = sh.si;
    if (si.mode == 2) {                                          // greedy: next token already written
        if (!COOP || part == 0) write_glue(p, b, si.row, si.greedy_tok);
        return;
    }

    RowPair rp;
    make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 0, FILT ? p.filters : nullptr, p.B, FILT ? p.draft_filters : nullptr, scp);
    int ntiles = p.ntiles;
    int32_t tok_off = 0;
    double u_eff = (double)si.u;
    bool slab_mode = false;
    if (slab_ready && si.mode == 1 && rp.ok && si.row == len) {  // every draft kept: the slab's tiles are there
        slab_mode = true;
        narrow_to_slab<BF16>(rp, slab_lo, slab_hi);
        tok_off = (int32_t)(slab_lo * N);
        ntiles = slab_tiles;
        u_eff = sh.slab_u;
    }

    // the sweep of the whole stop row is shared; a draw from a slab, or a row without mass, is part 0's alone
    bool coop_now = COOP && G > 1 && !slab_mode && rp.ok;
    if (COOP && G > 1 && !coop_now && part != 0) return;
    int own_lo = 0, own_hi = 0x7fffffff;                         // the tiles whose chunk sums this workgroup holds
    (void)own_lo; (void)own_hi;

    // ---- filtered call whose stop row's keep set is at hand as a short list: no sweep of the row at all
    int list_n = 0;
    const unsigned long long* list = nullptr;
    if (FILT && p.kept != nullptr && rp.ok) {
        const int64_t rid = (int64_t)b * (2 * g + 1) + g + si.row;
        list_n = p.kept_n[rid];
        list = p.kept + rid * p.kept_stride;
        if (list_n < 1 || list_n > kKeptListMax) list_n = 0;
    }

    int32_t tok = -1;
    for (int attempt = 0; attempt < 3; ++attempt) {
        float4* const sums = (ntiles <= kSumsKeepTiles) ? chunk_sums : nullptr;   // uniform over the workgroup
        if (FILT && list_n > 0) {
            if (wave == 0) {
                const int32_t tk = sample_kept_list<BF16>(rp, list, list_n, u_eff, lane);
                if (lane == 0) sh.tok = tk;
            }
            __syncthreads();
            tok = sh.tok;
            if (tok != -2) break;
            __syncthreads();
            make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 1, FILT ? p.filters : nullptr, p.B, FILT ? p.draft_filters : nullptr, scp);
            continue;
        }
        if (!(slab_mode && attempt == 0)) {
            if constexpr (COOP) {
                int t_lo = 0, t_hi = ntiles;
                if (coop_now) {
                    const int per = (ntiles + G - 1) / G;
                    t_lo = part * per;
                    t_hi = t_lo + per < ntiles ? t_lo + per : ntiles;
                }
                own_lo = t_lo; own_hi = t_hi;
                double* const shared_tiles = p.coop_tiles + (int64_t)b * p.ntiles;
                for (int t = t_lo + wave; t < t_hi; t += 2 * NW) {
                    double w0 = 0.0, w1 = 0.0;
                    const int t1 = t + NW < t_hi ? t + NW : p.ntiles;    // p.ntiles: past the row, no loads and no weight
                    if (rp.ok) tile_weight2<BF16, FILT>(rp, t, t1, lane, w0, w1, sums, t_hi);
                    if (lane == 0) {
                        sh.tiles[t] = w0;
                        if (t + NW < t_hi) sh.tiles[t + NW] = w1;
                        if (coop_now) {                          // and for the other parts, straight to memory
                            store_through(shared_tiles + t, w0);
                            if (t + NW < t_hi) store_through(shared_tiles + t + NW, w1);
                        }
                    }
                }
                if (coop_now) stores_through_done();             // this wavefront's stores have reached memory
                __syncthreads();
                if (coop_now) {
                    if (tid == 0) sh.tok = take_ticket(p.coop_tickets + b, p.coop_tag, (uint32_t)G) ? 1 : 0;
                    __syncthreads();
                    const bool last = sh.tok != 0;
                    __syncthreads();                             // sh.tok is written again below
                    if (!last) return;
                    for (int t = tid; t < ntiles; t += NW * 64)
                        if (t < t_lo || t >= t_hi) sh.tiles[t] = load_through(shared_tiles + t);
                    __syncthreads();
                    coop_now = false;                            // a later sweep, if any, is this workgroup's alone
                }
            } else {
                // tile weights of the stop row: two tiles per round trip and wavefront
                for (int t = wave; t < ntiles; t += 2 * NW) {
                    double w0 = 0.0, w1 = 0.0;
                    if (rp.ok) tile_weight2<BF16, FILT>(rp, t, t + NW, lane, w0, w1, sums, ntiles);
                    if (lane == 0) {
                        sh.tiles[t] = w0;
                        if (t + NW < ntiles) sh.tiles[t + NW] = w1;
                    }
                }
                __syncthreads();
            }
        }
        if (wave == 0) {
            int32_t tk = -1;
            if constexpr (COOP) {
                if (rp.ok) tk = select_token<BF16, true, FILT>(rp, sh.tiles, ntiles, u_eff, lane,
                                                               (slab_mode && attempt == 0) ? keep : nullptr, sums, own_lo, own_hi);
            } else {
                if (rp.ok) tk = select_token<BF16, true, FILT>(rp, sh.tiles, ntiles, u_eff, lane,
                                                               (slab_mode && attempt == 0) ? keep : nullptr, sums);
            }
            if (lane == 0) sh.tok = tk;
        }
        __syncthreads();
        tok = sh.tok;
        if (slab_mode) {
            if (tok >= 0) { tok += tok_off; break; }
            // no mass in the slab by the sampler's arithmetic (an underflow the partials did not have): the whole row
            slab_mode = false;
            make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 0, FILT ? p.filters : nullptr, p.B, FILT ? p.draft_filters : nullptr, scp);
            ntiles = p.ntiles;
            u_eff = (double)si.u;
            continue;
        }
        if (tok != -2) break;                                    // -2: no residual mass, sample p itself
        make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 1, FILT ? p.filters : nullptr, p.B, FILT ? p.draft_filters : nullptr, scp);
    }
    if (tid == 0) p.out_next_token[b] = tok < 0 ? -1 : tok;
    write_glue(p, b, si.row, tok < 0 ? -1 : tok);
}

template <bool BF16, int NW, int U>
__global__ __launch_bounds__(NW * 64) void fused_kernel(FusedParams p)
{
    __shared__ Partial s_part[2 * kFusedMaxGamma + 1][NW];
    __shared__ SeqShared sh;
    __shared__ int32_t s_prog[NW];

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const int g = p.gamma;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const bool greedy = !(Tb > 0.f);
    const ExpScale sc = make_scale(greedy ? kLog2e : kLog2e / (double)Tb);
    constexpr int ES = BF16 ? 2 : 4;

    // ---- statistics of the rows this sequence needs: every row is split statically over the
    // wavefronts (so the result does not depend on timing).  The hardware issues oldest-first, which
    // lets the first wavefronts run rows ahead of the last ones; a wavefront that is ahead of the slowest
    // one therefore lowers its issue priority, so that the workgroup advances evenly.
    if (tid < NW) s_prog[tid] = 0;
    __syncthreads();
    const int n_draft = p.draft_stats_in ? 0 : len;             // draft statistics may come from a previous level
    const int n_rows = n_draft + len + 1;
    int done = 0;
    for (int ri = 0; ri < n_rows; ++ri) {
        const bool is_draft = ri < n_draft;
        const int j = is_draft ? ri : ri - n_draft;
        const int r = is_draft ? j : g + j;
        const char* row = is_draft ? (const char*)p.draft + ((int64_t)b * g + j) * p.draft_ld * ES
                                   : (const char*)p.target + ((int64_t)b * (g + 1) + j) * p.target_ld * ES;
        const RowGeom geom = make_geom<BF16>(row, p.V);
        Partial res;
        if (greedy && !is_draft)
            res = wave_row_share<BF16, true, U>(geom, geom.c_first + tid, geom.c_end, NW * 64, wave == 0, sc, lane);
        else
            res = wave_row_share<BF16, false, U>(geom, geom.c_first + tid, geom.c_end, NW * 64, wave == 0, sc, lane);
        ++done;
        if (lane == 0) { s_part[r][wave] = res; *(volatile int32_t*)&s_prog[wave] = done; }
        int slowest = (lane < NW) ? *(volatile int32_t*)&s_prog[lane] : 0x7fffffff;
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) { const int o = __shfl_xor(slowest, m, 64); slowest = o < slowest ? o : slowest; }
        slowest = __shfl(slowest, 0, 64);
        if (done > slowest) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(3);
    }
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();
    for (int ri = wave; ri < n_rows; ri += NW) {                 // one wavefront per row, one lane per partial
        const bool is_draft = ri < n_draft;
        const int r = is_draft ? ri : g + (ri - n_draft);
        const RowStat rs = merge_partials_wave(&s_part[r][0], NW, lane);
        if (lane == 0) sh.stat[r] = rs;
    }
    TokenGather tg{};
    tg.x = -1;
    if (wave == 0) tg = accept_gather<BF16>(accept_ctx(p), b, lane, len, Tb);
    __syncthreads();
    sequence_tail<BF16, NW>(p, sh, b, len, Tb, tg);
}

// Accept + sampling of one sequence from the row partials of the split-row kernel.  What does not depend on the
// statistics is started first and by wavefronts of its own, so that the memory round trips of a sequence overlap
// instead of following one another: wavefront 0 fetches the drafted tokens and their logits and computes the
// positions' Philox blocks, the first few of the others merge the rows' partials, and every wavefront with nothing to
// merge picks the slab a bonus token would come from and puts its tile of that slab in flight.
template <bool BF16, int NW, bool FILT = false, bool COOP = false>
__global__ __launch_bounds__(NW * 64) void tail_kernel(FusedParams p, const Partial* __restrict__ partials, int nparts)
{
    __shared__ SeqShared sh;
    // the chunks of the slab a bonus token comes from, kept for the selection; only where a workgroup has a compute
    // unit to itself (smaller workgroups share one, and there the shared memory is better left to more of them)
    __shared__ uint4 s_raw[(NW == 16 && !FILT) ? kSlabKeepChunks : 1];
    uint4* const slab_raw = (NW == 16 && !FILT) ? s_raw : nullptr;
    __shared__ float4 s_sums[(NW == 16 && !FILT) ? kSumsKeepTiles * 64 : 1];   // likewise
    float4* const chunk_sums = (NW == 16 && !FILT) ? s_sums : nullptr;
    const int G = (COOP && p.coop > 1) ? p.coop : 1;             // workgroups per sequence (see sequence_tail)
    const int b = (int)blockIdx.x / G, part = (int)blockIdx.x % G;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const int g = p.gamma;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const int first_row = p.draft_stats_in ? g : 0;
    const int end_row = (p.target_stats_in || FILT) ? g : 2 * g + 1;   // supplied or filtered statistics are not merged here
    const bool pre_slab = !FILT && !p.target_stats_in && nparts >= 4 && Tb > 0.f;
    TokenGather tg{};
    tg.x = -1;
    // `width` lanes per row (one lane per partial), 64 / width rows per wavefront; with pre_slab the last wavefront
    // never merges
    const int mergers = pre_slab ? NW - 2 : NW - 1, mw = wave - 1;
    int width = 4;
    while (width < nparts) width <<= 1;
    const int per_wave = 64 / width, seg = lane / width, sl = lane % width;
    const int base_row = FILT ? g : first_row;
    const bool merges = wave >= 1 && wave <= mergers && base_row + mw * per_wave < end_row;
    TilePre pre{};                                               // ok = false
    if (wave == 0) {
        tg = accept_gather<BF16>(accept_ctx(p), b, lane, len, Tb);
    } else if (merges) {
        for (int r0 = base_row + mw * per_wave; r0 < end_row; r0 += mergers * per_wave) {
            const int r = r0 + seg;
            const bool is_draft = r < g;
            const int j = is_draft ? r : r - g;
            const bool need = r < end_row && (is_draft ? (j < len) : (j <= len));
            const int64_t slot = is_draft ? (int64_t)b * g + j : (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
            const RowStat s = merge_partials_seg(need ? partials + slot * nparts : nullptr, nparts, sl, width);
            if (need && sl == 0) sh.stat[r] = s;
        }
    } else if (pre_slab) {
        // Nothing to merge: pick the slab a bonus token would come from (every such wavefront by itself: the same
        // loads and arithmetic, the same answer, and no trip through shared memory) and put this wavefront's tile of it
        // in flight, so that its chunks are there when the statistics are.
        int64_t lo = 0, hi = 0;
        double frac = 0.0;
        const bool ok = pick_bonus_slab<BF16>(p, b, len, partials, nparts, lane, lo, hi, frac);
        if (wave == NW - 1 && lane == 0) { sh.slab_lo = lo; sh.slab_hi = hi; sh.slab_u = frac; sh.slab_ok = ok ? 1 : 0; }
        const int64_t t = (NW - 1) - wave;
        if (ok && (!COOP || part == 0) && t * (64 * kTileChunks) < hi - lo) {
            constexpr int ES = BF16 ? 2 : 4;
            const char* row = (const char*)p.target + ((int64_t)b * (g + 1) + len) * p.target_ld * ES;
            pre = tile_preload((const uint4*)row, lo, hi - lo, t, lane);   // rows with slabs start on the chunk grid
        }
    }
    __syncthreads();
    sequence_tail<BF16, NW, FILT, COOP>(p, sh, b, len, Tb, tg, pre_slab, slab_raw, chunk_sums, part, G, pre);
}

bool fused_supported(int32_t gamma, int32_t V, int dtype)
{
    return gamma <= kFusedMaxGamma && sampler_tiles(V, dtype) <= kFusedMaxTiles;
}

bool tail_supported(int32_t gamma, int32_t V, int dtype)
{
    return gamma <= HOLA_MAX_GAMMA && sampler_tiles(V, dtype) <= kFusedMaxTiles;
}

template <bool BF16>
static hipError_t launch_fused_typed(const FusedParams& p, const Tuning& t, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    dim3 grid((unsigned)p.B);
    const int nw = t.fused_waves ? t.fused_waves : 16;
    const int U = t.unroll ? t.unroll : 8;
#define HOLA_FUSED(NW, UU) hipLaunchKernelGGL((fused_kernel<BF16, NW, UU>), grid, dim3(NW * 64), 0, s, p)
    if (nw <= 8) { if (U == 2) HOLA_FUSED(8, 2); else if (U == 4) HOLA_FUSED(8, 4); else if (U == 16) HOLA_FUSED(8, 16); else HOLA_FUSED(8, 8); }
    else { if (U == 2) HOLA_FUSED(16, 2); else if (U == 4) HOLA_FUSED(16, 4); else if (U == 16) HOLA_FUSED(16, 16); else HOLA_FUSED(16, 8); }
#undef HOLA_FUSED
    return hipGetLastError();
}

hipError_t launch_fused(const FusedParams& p, const Tuning& t, hipStream_t s)
{
    return p.dtype == HOLA_DTYPE_BF16 ? launch_fused_typed<true>(p, t, s) : launch_fused_typed<false>(p, t, s);
}

hipError_t launch_tail(const FusedParams& p, const Partial* partials, int nparts, const Tuning& t, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    if (nparts > 64) return hipErrorInvalidValue;
    const int nw = t.fused_waves ? t.fused_waves : 16;
    const bool coop = p.coop > 1 && nw == 16 && !p.filters;      // the caller checked the rest (hola_api.hip)
    dim3 grid((unsigned)p.B * (coop ? (unsigned)p.coop : 1u));
    if (p.filters) {                                             // filtered distributions: 8 wavefronts, more registers
        if (p.dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((tail_kernel<true, 8, true>), grid, dim3(512), 0, s, p, partials, nparts);
        else hipLaunchKernelGGL((tail_kernel<false, 8, true>), grid, dim3(512), 0, s, p, partials, nparts);
        return hipGetLastError();
    }
    if (p.dtype == HOLA_DTYPE_BF16) {
        if (nw == 4) hipLaunchKernelGGL((tail_kernel<true, 4>), grid, dim3(256), 0, s, p, partials, nparts);
        else if (nw == 8) hipLaunchKernelGGL((tail_kernel<true, 8>), grid, dim3(512), 0, s, p, partials, nparts);
        else if (coop) hipLaunchKernelGGL((tail_kernel<true, 16, false, true>), grid, dim3(1024), 0, s, p, partials, nparts);
        else hipLaunchKernelGGL((tail_kernel<true, 16>), grid, dim3(1024), 0, s, p, partials, nparts);
    } else {
        if (nw == 4) hipLaunchKernelGGL((tail_kernel<false, 4>), grid, dim3(256), 0, s, p, partials, nparts);
        else if (nw == 8) hipLaunchKernelGGL((tail_kernel<false, 8>), grid, dim3(512), 0, s, p, partials, nparts);
        else if (coop) hipLaunchKernelGGL((tail_kernel<false, 16, false, true>), grid, dim3(1024), 0, s, p, partials, nparts);
        else hipLaunchKernelGGL((tail_kernel<false, 16>), grid, dim3(1024), 0, s, p, partials, nparts);
    }
    return hipGetLastError();
}

}  // namespace hola
