// Equation (1) taken literally, one workgroup per sequence: every drafted position t yields
// y_t = draft token if g(t) = 1[H(draft_t) < tau] = 1 (Section 3.1, Algorithm 1 Step 1), otherwise
// y_t = f_ver(x, draft_<t), a draw from the verifier's distribution at position t (argmax on greedy
// rows).  There is no ratio test and no stop at a replaced token; the number of verifier draws per
// sequence is the k of Section 3.1.  Row statistics come from the split-row kernel's partials; each
// non-gated position costs one more sweep of its target row (tile weights in LDS) and one tile re-read.
#include "accept_device.h"
#include "sampler_device.h"

namespace hola {

constexpr int kLiteralMaxTiles = 2048;

struct LiteralShared {
    RowStat stat[2 * HOLA_MAX_GAMMA + 1];
    double tiles[kLiteralMaxTiles];
    unsigned long long mask;
    int32_t tok;
};

template <bool BF16, int NW>
__global__ __launch_bounds__(NW * 64) void literal_kernel(FusedParams p, const Partial* __restrict__ partials, int nparts,
                                                          int32_t* __restrict__ out_tokens, int32_t* __restrict__ out_calls)
{
    __shared__ LiteralShared sh;
    __shared__ float4 s_sums[NW == 16 ? kSumsKeepTiles * 64 : 1];   // the lanes' chunk sums of a sweep, for its selection
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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
            sh.mask = greedy ? 0ull : m;
            if (out_calls) out_calls[b] = __popcll(m);
        }
    }
    __syncthreads();
    unsigned long long mask = sh.mask;
    const uint64_t seq = (uint64_t)(p.seq_base + b);
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
