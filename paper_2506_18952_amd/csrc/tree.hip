// Verify step over token trees: several drafted tokens per position, each with the rows of its own context.
//
// Rows are laid out as in the one-token step with gamma = N nodes: draft row c and target row c belong to context c
// (0: the prefix, n + 1: the prefix followed by the path to node n), so the split-row statistics kernel serves
// unchanged; only the draft rows of contexts without children leave it at once (it looks the children up itself).
//
// tree_tail_kernel, one workgroup per sequence: merges the row partials, gathers the two logits of every node's
// token in one go, then walks from the prefix.  The children of a context are tried in node order by the recursive
// rejection rule for candidates drawn independently from the same draft distribution: after i rejections the
// running distribution is max(0, p - C q) / Z with Z its sum and C the sum of the earlier Z's (C = 0, Z = 1 at
// first, which is the acceptance test u q(x) < p(x) of Equation (1)'s verifier branch); the strict gate H(q) < tau
// (Algorithm 1, Step 1) keeps the first child without a test.  Every rejection but the last costs one sweep of
// the context's row pair for the next Z; after the last the next token is drawn from max(0, p - C q) by the
// sampler of the one-token step, whose weights take C through the factor it already applies to q.
// The walk is wavefront 0's; the sweeps are the whole workgroup's, handed over through shared memory.
// HBM-bound like the tail of the one-token step: no atomics, no spin waits, every loop bounded by the node count.
#include "accept_device.h"
#include "sampler_device.h"

namespace hola {

constexpr int kTreeMaxTiles = 2048;

struct TreeShared {
    RowStat stat[2 * HOLA_MAX_GAMMA + 1];      // draft contexts 0..N-1, target contexts N..2N
    double tiles[kTreeMaxTiles];
    double px[64], qx[64], u[64];              // per node: the two probabilities of its token, its test uniform
    int32_t path[64];                          // kept nodes, from the prefix on
    int32_t ctx_of[64];                        // per node: the context it hangs under, -1: no node
    int32_t used[64];                          // per context: it has a child
    // the walk's state between rounds
    int32_t w_ctx, w_depth, w_first, w_dead;
    double w_C, w_Z;
    unsigned long long w_kids, w_all;
    // the row operation wavefront 0 asks of the workgroup
    int32_t op_ctx, op_bonus, op_sample, done;
    double op_C;
    int32_t tok;
};

// Sum of the tile weights, in the order the selecting wavefront adds them.
__device__ __forceinline__ double tiles_total(const double* tiles, int ntiles, int lane)
{
    const int per = (ntiles + 63) / 64;
    double mine = 0.0;
    for (int i = 0; i < per; ++i) {
        const int t = lane * per + i;
        if (t < ntiles) mine += read_tile<true>(tiles + t);
    }
    const double incl = wave_inclusive_scan(mine, lane);
    return __shfl(incl, 63, 64);
}

template <bool BF16, int NW>
__global__ __launch_bounds__(NW * 64) void tree_tail_kernel(TreeParams p, const Partial* __restrict__ partials, int nparts)
{
    __shared__ TreeShared sh;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    const int N = p.N;
    int len = p.n_nodes ? p.n_nodes[b] : N;
    len = len < 0 ? 0 : (len > N ? N : len);
    const float Tb = p.temperature;

    // ---- every node's context; contexts with children (a node whose parent is not -1 or an earlier node hangs
    // under none)
    if (tid < 64) sh.used[tid] = 0;
    __syncthreads();
    if (wave == 0) {
        int c = -1;
        if (lane < len) {
            const int32_t pr = p.parent[(int64_t)b * N + lane];
            if (pr >= -1 && pr < lane) c = pr + 1;
        }
        sh.ctx_of[lane] = c;
        if (c >= 0) sh.used[c] = 1;                              // the same value from every child
    }
    __syncthreads();

    // ---- row statistics from the split-row partials: `width` lanes per row, 64 / width rows per wavefront
    int width = 4;
    while (width < nparts) width <<= 1;
    const int per_wave = 64 / width, seg = lane / width, sl = lane % width;
    for (int r0 = wave * per_wave; r0 < 2 * N + 1; r0 += NW * per_wave) {
        const int r = r0 + seg;
        const bool is_draft = r < N;
        const int c = is_draft ? r : r - N;
        const bool need = r < 2 * N + 1 && (is_draft ? (c < len && sh.used[c]) : (c <= len));
        const int64_t slot = is_draft ? (int64_t)b * N + c : (int64_t)p.B * N + (int64_t)b * (N + 1) + c;
        const RowStat s = merge_partials_seg(need ? partials + slot * nparts : nullptr, nparts, sl, width);
        if (need && sl == 0) sh.stat[r] = s;
    }
    __syncthreads();

    // ---- per node (lane n of wavefront 0): context, probabilities of its token, test uniform
    int my_ctx = -1;
    if (wave == 0) {
        const uint64_t seq = (uint64_t)(p.seq_base + b);
        const int n = lane;
        double p_x = 0.0, q_x = 1.0, un = 0.0;
        my_ctx = sh.ctx_of[n];
        if (my_ctx >= 0) {
            const int32_t x = p.tokens[(int64_t)b * N + n];
            if (x >= 0 && x < p.V) {
                const double invT = 1.0 / (double)Tb;
                const float xp = load_logit<BF16>(p.target, ((int64_t)b * (N + 1) + my_ctx) * p.target_ld + x);
                const float xq = load_logit<BF16>(p.draft, ((int64_t)b * N + my_ctx) * p.draft_ld + x);
                p_x = exp((double)xp * invT - sh.stat[N + my_ctx].lse);
                q_x = exp((double)xq * invT - sh.stat[my_ctx].lse);
            }
            const Philox4 r = philox4x32_10((uint32_t)n, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                            (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
            un = (double)u24(r.x);
        }
        sh.px[n] = p_x; sh.qx[n] = q_x; sh.u[n] = un;
        if (p.out_entropy && n < N) p.out_entropy[(int64_t)b * N + n] = (n < len && sh.used[n]) ? (float)sh.stat[n].H : -1.0f;
        if (lane == 0) sh.done = 0;
    }
    wave_handoff();

    // ---- the walk (wavefront 0, every lane the same values) and the row sweeps it asks for (all wavefronts).
    // Between rounds the walk's state rests in shared memory, so that no register holds it during a sweep.
    if (wave == 0) {
        const unsigned long long k0 = __ballot(my_ctx == 0);    // the children of the prefix
        if (lane == 0) {
            sh.w_ctx = 0; sh.w_depth = 0; sh.w_first = 1; sh.w_dead = 0; sh.w_C = 0.0; sh.w_Z = 1.0;
            sh.w_kids = k0; sh.w_all = k0;
        }
    }
    for (int it = 0; it < 2 * 64 + 4; ++it) {                   // every round ends the walk or uses up a child
        if (wave == 0) {
            wave_handoff();
            const int mine = sh.ctx_of[lane];
            int ctx = sh.w_ctx, depth = sh.w_depth;
            bool first = sh.w_first != 0;
            const bool dead = sh.w_dead != 0;
            double C = sh.w_C;
            const double Z = sh.w_Z, tau = (double)p.tau;
            unsigned long long kids = sh.w_kids, all_kids = sh.w_all;
            int sample = 1, bonus = 1;
            for (;;) {
                if (dead || all_kids == 0) { bonus = 1; break; } // nothing drafted here (or a residual without mass)
                if (kids == 0) { bonus = 0; break; }             // every child rejected
                const int n = __ffsll((long long)kids) - 1;
                kids &= kids - 1;
                const double q_x = sh.qx[n], p_x = sh.px[n], un = sh.u[n];
                bool ok;
                if (first) ok = (sh.stat[ctx].H < tau) || (un * q_x < p_x);
                else ok = (un * q_x * Z < fmax(0.0, p_x - C * q_x));
                if (ok) {
                    if (lane == 0) sh.path[depth] = n;
                    ++depth;
                    ctx = n + 1;
                    all_kids = __ballot(mine == ctx);
                    kids = all_kids;
                    C = 0.0; first = true;
                    continue;                                    // Z is not read before the next rejection's sweep
                }
                C += first ? 1.0 : Z;
                first = false;
                if (kids == 0) { bonus = 0; break; }
                sample = 0; bonus = 0;                           // more children to try: the next Z
                break;
            }
            wave_handoff();
            if (lane == 0) {
                sh.op_ctx = ctx; sh.op_bonus = bonus; sh.op_sample = sample; sh.op_C = C;
                sh.w_ctx = ctx; sh.w_depth = depth; sh.w_first = first ? 1 : 0; sh.w_C = C;
                sh.w_kids = kids; sh.w_all = all_kids;
            }
        }
        __syncthreads();
        const int o_ctx = sh.op_ctx, o_bonus = sh.op_bonus, o_sample = sh.op_sample;
        const double o_C = sh.op_C;
        SeqInfo si;
        si.row = o_ctx;
        si.lseP = sh.stat[N + o_ctx].lse;
        si.lseD = o_bonus ? 0.0 : sh.stat[o_ctx].lse;
        si.mode = o_bonus ? 1 : 0;
        si.u = 0.f; si.greedy_tok = -1;
        RowPair rp;
        make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, N, p.V, Tb, b, si, o_bonus, nullptr, 0, nullptr, &p.sc);
        if (!rp.bonus && o_C != 1.0) {                           // weights max(0, p - C q): C joins the factor on q
            const double kappa = ((double)rp.k_hi + (double)rp.k_lo) * o_C;
            rp.k_hi = (float)kappa;
            rp.k_lo = (float)(kappa - (double)rp.k_hi);
        }
        for (int t = wave; t < p.ntiles; t += 2 * NW) {
            double w0 = 0.0, w1 = 0.0;
            if (rp.ok) tile_weight2<BF16>(rp, t, t + NW, lane, w0, w1);
            if (lane == 0) {
                sh.tiles[t] = w0;
                if (t + NW < p.ntiles) sh.tiles[t + NW] = w1;
            }
        }
        __syncthreads();
        if (wave == 0) {
            if (!o_sample) {
                const double Z = rp.ok ? tiles_total(sh.tiles, p.ntiles, lane) : 0.0;
                if (lane == 0) {
                    sh.w_Z = Z;
                    if (!(Z > 0.0) || !(Z - Z == 0.0) || rp.bonus) sh.w_dead = 1;   // no residual mass: draw from p itself
                }
            } else {
                const uint64_t seq = (uint64_t)(p.seq_base + b);
                const Philox4 r = philox4x32_10((uint32_t)o_ctx, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                                (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
                const int32_t tk = rp.ok ? select_token<BF16, true>(rp, sh.tiles, p.ntiles, (double)u24(r.y), lane) : -1;
                if (lane == 0) {
                    if (tk == -2 && !sh.w_dead) {
                        sh.w_dead = 1;                            // residual without mass: once more, as a draw from p
                    } else {
                        sh.tok = tk < 0 ? -1 : tk;
                        sh.done = 1;
                    }
                }
            }
        }
        __syncthreads();
        if (sh.done) break;
    }
    if (wave == 0) {
        const int depth = sh.w_depth;
        if (lane == 0) {
            p.out_next_token[b] = sh.done ? sh.tok : -1;
            p.out_accept_len[b] = depth;
        }
        if (p.out_path && lane < N) p.out_path[(int64_t)b * N + lane] = lane < depth ? sh.path[lane] : -1;
    }
}

bool tree_supported(int32_t N, int32_t V, int dtype)
{
    return N >= 1 && N <= HOLA_MAX_GAMMA && sampler_tiles(V, dtype) <= kTreeMaxTiles;
}

hipError_t launch_tree_tail(const TreeParams& p, const Partial* partials, int nparts, int waves, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    if (nparts > 64 || p.ntiles > kTreeMaxTiles) return hipErrorInvalidValue;
    dim3 grid((unsigned)p.B);
    if (p.dtype == HOLA_DTYPE_BF16) {
        if (waves <= 8) hipLaunchKernelGGL((tree_tail_kernel<true, 8>), grid, dim3(512), 0, s, p, partials, nparts);
        else hipLaunchKernelGGL((tree_tail_kernel<true, 16>), grid, dim3(1024), 0, s, p, partials, nparts);
    } else {
        if (waves <= 8) hipLaunchKernelGGL((tree_tail_kernel<false, 8>), grid, dim3(512), 0, s, p, partials, nparts);
        else hipLaunchKernelGGL((tree_tail_kernel<false, 16>), grid, dim3(1024), 0, s, p, partials, nparts);
    }
    return hipGetLastError();
}

}  // namespace hola
