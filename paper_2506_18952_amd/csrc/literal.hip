// Equation (1) taken literally, one workgroup per sequence: every drafted position t yields
// y_t = draft token if g(t) = 1[H(draft_t) < tau] = 1 (Section 3.1, Algorithm 1 Step 1), otherwise
// y_t = f_ver(x, draft_<t), a draw from the verifier's distribution at position t (argmax on greedy
// rows).  There is no ratio test and no stop at a replaced token; the number of verifier draws per
// sequence is the k of Section 3.1.  Row statistics come from the split-row kernel's partials; each
// non-gated position costs one more sweep of a slab of its target row by one wavefront (or, where the row has no
// slabs, of the whole row by the workgroup).
#include "accept_device.h"
#include "sampler_device.h"

namespace hola {

constexpr int kLiteralMaxTiles = 2048;

constexpr int kWaveSlabTiles = 16;     // largest slab a single wavefront sweeps for a draw of its own

struct LiteralShared {
    RowStat stat[2 * HOLA_MAX_GAMMA + 1];
    double tiles[kLiteralMaxTiles];
    double wave_tiles[16][kWaveSlabTiles];   // per wavefront: the tile weights of the slab it sweeps
    unsigned long long mask;
    unsigned long long mask_left;      // draws left to the whole-workgroup loop
    int32_t tok;
};

template <bool BF16, int NW>
__global__ __launch_bounds__(NW * 64) void literal_kernel(FusedParams p, const Partial* __restrict__ partials, int nparts,
                                                          int32_t* __restrict__ out_tokens, int32_t* __restrict__ out_calls)
{
    __shared__ LiteralShared sh;
    __shared__ float4 s_sums[NW == 16 ? kSumsKeepTiles * 64 : 1];   // the lanes' chunk sums of a sweep, for its selection
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const int g = p.gamma;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const bool greedy = !(Tb > 0.f);
    for (int r = wave; r < 2 * g; r += NW) {                     // draft rows 0..g-1, target rows 0..g-1
        const bool is_draft = r < g;
        const int j = is_draft ? r : r - g;
        if (j >= len) continue;
        const int64_t slot = is_draft ? (int64_t)b * g + j : (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
        const RowStat s = merge_partials_wave(partials + slot * nparts, nparts, lane);
        if (lane == 0) sh.stat[is_draft ? j : g + j] = s;
    }
    __syncthreads();
    if (wave == 0) {
        const int j = lane;
        bool need = false;
        if (j < g) {
            float ent = -1.0f;
            int32_t y = -1;
            if (j < len) {
                const RowStat sd = sh.stat[j];
                ent = (float)sd.H;
                if (sd.H < (double)p.tau) {                      // strict; NaN never gates
                    y = p.tokens[(int64_t)b * p.tokens_ld + j];
                } else {
                    need = true;
                    if (greedy) y = sh.stat[g + j].argmax;
                }
            }
            if (p.out_entropy) p.out_entropy[(int64_t)b * (p.entropy_ld ? p.entropy_ld : g) + j] = ent;
            out_tokens[(int64_t)b * g + j] = y;
        }
        const unsigned long long m = __ballot(need);
        if (lane == 0) {
            sh.mask_left = 0ull;
            sh.mask = greedy ? 0ull : m;
            if (out_calls) out_calls[b] = __popcll(m);
        }
    }
    __syncthreads();
    unsigned long long mask = sh.mask;
    const uint64_t seq = (uint64_t)(p.seq_base + b);

    // ---- the verifier draws of a sequence do not depend on one another, so each wavefront takes one and does it by
    // itself: the statistics pass took this mode's target rows over contiguous slabs, so the slab that holds the draw
    // follows from the row's partials and the position's sampling uniform (pick_row_slab), and a wavefront sweeps and
    // searches that slab (an eighth of the row on the headline shape) alone.  Draws that cannot go this way (ragged
    // rows, a slab of more than kWaveSlabTiles tiles, no mass found by the sampler's arithmetic) are left to the
    // loop below, which gives the whole workgroup to one draw after the other.
    if (nparts >= 4 && mask) {
        unsigned long long todo = mask, left = 0ull;
        int nth = 0;
        while (todo) {                                           // workgroup-uniform
            const int t = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            if ((nth++ % NW) != wave) continue;
            const Philox4 r = philox4x32_10((uint32_t)t, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                            (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
            int64_t lo = 0, hi = 0;
            double frac = 0.0;
            bool ok = pick_row_slab<BF16>(p.target, p.target_ld, g, p.V, p.B, b, t, partials, nparts, (double)u24(r.y), lane, lo, hi, frac);
            const int slab_tiles = (int)((hi - lo + 64 * kTileChunks - 1) / (64 * kTileChunks));
            if (ok && slab_tiles > kWaveSlabTiles) ok = false;
            int32_t tk = -1;
            if (ok) {
                SeqInfo si;
                si.row = t; si.mode = 1; si.greedy_tok = -1; si.u = 0.f;
                si.lseP = sh.stat[g + t].lse; si.lseD = 0.0;
                RowPair rp;
                make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 1);
                if (rp.ok) {
                    narrow_to_slab<BF16>(rp, lo, hi);
                    double* const my_tiles = sh.wave_tiles[wave];
                    for (int tl = 0; tl < slab_tiles; tl += 2) {
                        double w0 = 0.0, w1 = 0.0;
                        tile_weight2<BF16>(rp, tl, tl + 1, lane, w0, w1);
                        if (lane == 0) {
                            my_tiles[tl] = w0;
                            if (tl + 1 < slab_tiles) my_tiles[tl + 1] = w1;
                        }
                    }
                    wave_handoff();             // the wavefront reads what its own lane 0 stored
                    tk = select_token<BF16, true>(rp, my_tiles, slab_tiles, frac, lane);
                    if (tk >= 0) tk += (int32_t)(lo * (BF16 ? 8 : 4));
                }
            }
            if (tk >= 0) { if (lane == 0) out_tokens[(int64_t)b * g + t] = tk; }
            else left |= 1ull << t;
        }
        __syncthreads();
        if (lane == 0 && left) atomicOr(&sh.mask_left, left);
        __syncthreads();
        mask = sh.mask_left;
    }
    while (mask) {                                               // workgroup-uniform
        const int t = __ffsll((long long)mask) - 1;
        mask &= mask - 1;
        SeqInfo si;
        si.row = t; si.mode = 1; si.greedy_tok = -1;
        si.lseP = sh.stat[g + t].lse; si.lseD = 0.0;
        const Philox4 r = philox4x32_10((uint32_t)t, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                        (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
        si.u = u24(r.y);
        RowPair rp;
        make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 1);
        float4* const sums = (NW == 16 && p.ntiles <= kSumsKeepTiles) ? s_sums : nullptr;   // uniform
        for (int tl = wave; tl < p.ntiles; tl += 2 * NW) {
            double w0 = 0.0, w1 = 0.0;
            if (rp.ok) tile_weight2<BF16>(rp, tl, tl + NW, lane, w0, w1, sums, p.ntiles);
            if (lane == 0) {
                sh.tiles[tl] = w0;
                if (tl + NW < p.ntiles) sh.tiles[tl + NW] = w1;
            }
        }
        __syncthreads();
        if (wave == 0) {
            const int32_t tk = rp.ok ? select_token<BF16, true>(rp, sh.tiles, p.ntiles, si.u, lane, nullptr, sums) : -1;
            if (lane == 0) out_tokens[(int64_t)b * g + t] = tk < 0 ? -1 : tk;
        }
        __syncthreads();
    }
}

bool literal_supported(int32_t gamma, int32_t V, int dtype)
{
    return gamma <= HOLA_MAX_GAMMA && sampler_tiles(V, dtype) <= kLiteralMaxTiles;
}

hipError_t launch_literal(const FusedParams& p, const Partial* partials, int nparts, int32_t* out_tokens,
                          int32_t* out_calls, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    if (nparts > 64) return hipErrorInvalidValue;
    dim3 grid((unsigned)p.B), block(1024);
    if (p.dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((literal_kernel<true, 16>), grid, block, 0, s, p, partials, nparts, out_tokens, out_calls);
    else hipLaunchKernelGGL((literal_kernel<false, 16>), grid, block, 0, s, p, partials, nparts, out_tokens, out_calls);
    return hipGetLastError();
}

}  // namespace hola
