// Fused per-sequence kernel: one workgroup of 8 or 16 wavefronts owns one sequence and runs the whole
// verify step for it without leaving the compute unit: row statistics of its gamma draft and
// gamma+1 target rows (streamed once from HBM, wavefront partials parked in LDS), the accept /
// first-reject stage (wavefront 0), the residual or bonus tile weights of the stop row (all
// wavefronts, tile weights in LDS) and the inverse-CDF selection (wavefront 0).
//
// Used when there are enough sequences to occupy the chip (one launch, no partials in HBM, no
// kernel boundaries); otherwise the split-row kernels spread the rows of few sequences over the chip.
// HBM-bound: every logit is read once, the stop row pair once more.
#include "accept_device.h"
#include "sampler_device.h"

namespace hola {

constexpr int kFusedMaxTiles = 2048;

template <bool BF16, int NW, int U>
__global__ __launch_bounds__(NW * 64) void fused_kernel(FusedParams p)
{
    __shared__ Partial s_part[2 * HOLA_MAX_GAMMA + 1][NW];
    __shared__ double s_tiles[kFusedMaxTiles];
    __shared__ SeqInfo s_si;
    __shared__ int32_t s_tok;

    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = p.gamma;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const bool greedy = !(Tb > 0.f);
    const ExpScale sc = make_scale(greedy ? kLog2e : kLog2e / (double)Tb);
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int64_t kStride = NW * 64;

    // ---- phase 1: statistics of the rows this sequence needs
    const int first_row = p.draft_stats_in ? g : 0;             // draft statistics may come from a previous level
    for (int r = first_row; r < 2 * g + 1; ++r) {
        const bool is_draft = r < g;
        const int j = is_draft ? r : r - g;
        if (is_draft ? (j >= len) : (j > len)) continue;         // workgroup-uniform
        const char* row = is_draft ? (const char*)p.draft + ((int64_t)b * g + j) * p.draft_ld * ES
                                   : (const char*)p.target + ((int64_t)b * (g + 1) + j) * p.target_ld * ES;
        const RowGeom geom = make_geom<BF16>(row, p.V);
        Partial res;
        if (greedy && !is_draft)
            res = wave_row_share<BF16, true, U>(geom, geom.c_first + tid, geom.c_end, kStride, wave == 0, sc, lane);
        else
            res = wave_row_share<BF16, false, U>(geom, geom.c_first + tid, geom.c_end, kStride, wave == 0, sc, lane);
        if (lane == 0) s_part[r][wave] = res;
    }
    __syncthreads();

    // ---- phase 2: accept / first reject (wavefront 0, lane j = position j)
    if (wave == 0) {
        const int j = lane;
        RowStat sd = {NAN, NAN, -1}, sp = {NAN, NAN, -1};
        if (j < len) {
            if (p.draft_stats_in) {
                sd.lse = p.draft_stats_in[((int64_t)b * g + j) * 2 + 0];
                sd.H = p.draft_stats_in[((int64_t)b * g + j) * 2 + 1];
            } else {
                sd = merge_partials(&s_part[j][0], NW);
            }
        }
        if (j <= len) sp = merge_partials(&s_part[g + j][0], NW);
        AcceptCtx c;
        c.target = p.target; c.draft = p.draft; c.target_ld = p.target_ld; c.draft_ld = p.draft_ld;
        c.tokens = p.tokens; c.seed = p.seed; c.level = p.level; c.seq_base = p.seq_base;
        c.gamma = g; c.V = p.V; c.tau = p.tau; c.target_stats_out = p.target_stats_out;
        c.out_accept_len = p.out_accept_len; c.out_next_token = p.out_next_token;
        c.out_entropy = p.out_entropy; c.entropy_ld = p.entropy_ld;
        accept_wave<BF16>(c, b, j, len, Tb, sd, sp, &s_si);
    }
    __syncthreads();
    const SeqInfo si = s_si;
    if (si.mode == 2) return;                                    // greedy: next token already written

    // ---- phase 3: tile weights of the stop row (all wavefronts), then selection (wavefront 0)
    RowPair rp;
    make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 0);
    int32_t tok = -1;
    for (int attempt = 0; attempt < 2; ++attempt) {
        for (int t = wave; t < p.ntiles; t += NW) {
            const double wsum = rp.ok ? tile_weight<BF16>(rp, t, lane) : 0.0;
            if (lane == 0) s_tiles[t] = wsum;
        }
        __syncthreads();
        if (wave == 0) {
            const int32_t tk = rp.ok ? select_token<BF16, true>(rp, s_tiles, p.ntiles, si.u, lane) : -1;
            if (lane == 0) s_tok = tk;
        }
        __syncthreads();
        tok = s_tok;
        if (tok != -2) break;                                    // -2: no residual mass, sample p itself
        make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, g, p.V, Tb, b, si, 1);
    }
    if (tid == 0) p.out_next_token[b] = tok < 0 ? -1 : tok;
}

bool fused_supported(int32_t gamma, int32_t V, int dtype)
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
    if (nw == 8) { if (U == 2) HOLA_FUSED(8, 2); else if (U == 4) HOLA_FUSED(8, 4); else if (U == 16) HOLA_FUSED(8, 16); else HOLA_FUSED(8, 8); }
    else { if (U == 2) HOLA_FUSED(16, 2); else if (U == 4) HOLA_FUSED(16, 4); else if (U == 16) HOLA_FUSED(16, 16); else HOLA_FUSED(16, 8); }
#undef HOLA_FUSED
    return hipGetLastError();
}

hipError_t launch_fused(const FusedParams& p, const Tuning& t, hipStream_t s)
{
    return p.dtype == HOLA_DTYPE_BF16 ? launch_fused_typed<true>(p, t, s) : launch_fused_typed<false>(p, t, s);
}

}  // namespace hola
