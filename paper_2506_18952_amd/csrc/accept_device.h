// Device code of the accept / first-reject stage (shared by the split accept kernel and the fused
// per-sequence kernel).  One wavefront per sequence, lane j owns position j.
//
// Given the statistics of draft row j and target row j, a lane applies the strict gate H < tau
// (Algorithm 1, Step 1; Section 3.1), and where the gate is open falls back to the verifier
// (Equation (1)) through the acceptance test u * q(x) < p(x) with a Philox uniform keyed on
// (seed, sequence, position, level).  A ballot over the lanes gives the first rejected position.
// All of it is O(gamma) scalar work in double.
#pragma once
#include "stats_device.h"

namespace hola {

struct AcceptCtx {
    const void* target; const void* draft;
    int64_t target_ld, draft_ld;
    const int32_t* tokens; int64_t tokens_ld;
    int32_t pad_entropy;
    uint64_t seed; uint32_t level; int64_t seq_base;
    int32_t gamma, V;
    float tau;
    double* target_stats_out;          // [B, gamma+1, 2] or null
    int32_t* out_accept_len; int32_t* out_next_token;
    float* out_entropy; int64_t entropy_ld;
    const RowFilter* filters = nullptr; // top-k / top-p keep sets and statistics, slots as the partials; or null
    const RowFilter* draft_filters = nullptr;   // the draft rows' ([B, gamma]): `filters` itself unless handed over
    int32_t B = 0;
    int32_t write_outputs = 1;         // 0: decide only (a workgroup that shares a sequence's tail with the one that writes)
};

// Membership of token i with logit x in a filtered row's keep set.
__device__ __forceinline__ bool filter_keeps(float x, int32_t i, float theta, int32_t idx_cut)
{
    return x > theta || (x == theta && i <= idx_cut);
}

// What lane j can have ready for its position before the row statistics are: the drafted token and, on stochastic
// rows, its logit in both models (also divided by the temperature) and the position's Philox block.  Kept apart from
// the decision so that a caller has the loads in flight, and this arithmetic done, while the statistics are still
// being merged.
struct TokenGather {
    int32_t x;                         // drafted token (-1 beyond len)
    float xp, xq;                      // its target and draft logits (0 where not loaded)
    double ap, aq;                     // xp / T and xq / T as the decision uses them
    float u_test, u_draw;              // words 0 and 1 of position j's Philox block as uniforms (0 where there is none)
};

template <bool BF16>
__device__ __forceinline__ TokenGather accept_gather(const AcceptCtx& c, int b, int j, int len, float Tb)
{
    TokenGather t;
    t.x = -1; t.xp = 0.f; t.xq = 0.f; t.ap = 0.0; t.aq = 0.0; t.u_test = 0.f; t.u_draw = 0.f;
    const int g = c.gamma;
    const bool greedy = !(Tb > 0.f);
    if (j < len) {
        t.x = c.tokens[(int64_t)b * c.tokens_ld + j];
        if (!greedy && t.x >= 0 && t.x < c.V) {
            t.xp = load_logit<BF16>(c.target, ((int64_t)b * (g + 1) + j) * c.target_ld + t.x);
            t.xq = load_logit<BF16>(c.draft, ((int64_t)b * g + j) * c.draft_ld + t.x);
        }
    }
    // Position j's Philox block: word 0 decides the acceptance test of drafted position j, word 1 draws the next token
    // if the sequence stops at row j, so the lane that turns out to hold the stop row has its uniform at hand.
    if (!greedy && j <= len) {
        const uint64_t seq = (uint64_t)(c.seq_base + b);
        const Philox4 r = philox4x32_10((uint32_t)j, (uint32_t)seq, (uint32_t)(seq >> 32), c.level, (uint32_t)c.seed, (uint32_t)(c.seed >> 32));
        t.u_test = u24(r.x);
        t.u_draw = u24(r.y);
    }
    const double invT = greedy ? 1.0 : 1.0 / (double)Tb;
    t.ap = (double)t.xp * invT;
    t.aq = (double)t.xq * invT;
    return t;
}

// Called by all 64 lanes of one wavefront.  sd / sp: statistics of draft row j (valid for j < len) and
// target row j (valid for j <= len); tg: what accept_gather returned for this lane.  Writes accept_len, the
// entropies, the optional target statistics and, for greedy rows, the next token; the lane at the stop row fills
// *si_out.
template <bool BF16>
__device__ __forceinline__ void accept_decide(const AcceptCtx& c, int b, int j, int len, float Tb,
                                              const RowStat& sd_in, const RowStat& sp_in, const TokenGather& tg,
                                              SeqInfo* si_out)
{
    const int g = c.gamma;
    RowStat sd = sd_in, sp = sp_in;
    float thD = -INFINITY, thP = -INFINITY;
    int32_t cutD = 0x7fffffff, cutP = 0x7fffffff;
    if (c.filters) {                                    // filtered distributions: their own statistics and keep sets
        if (j < len) {
            const RowFilter f = c.draft_filters[(int64_t)b * g + j];
            sd.lse = f.lse; sd.H = f.H; thD = f.theta; cutD = f.idx_cut;
        }
        if (j <= len) {
            const RowFilter f = c.filters[(int64_t)c.B * g + (int64_t)b * (g + 1) + j];
            sp.lse = f.lse; sp.H = f.H; thP = f.theta; cutP = f.idx_cut;
        }
    }
    const bool greedy = !(Tb > 0.f);
    const double tau = (double)c.tau;
    if (c.write_outputs && c.target_stats_out && j <= len) {
        c.target_stats_out[((int64_t)b * (g + 1) + j) * 2 + 0] = sp.lse;
        c.target_stats_out[((int64_t)b * (g + 1) + j) * 2 + 1] = sp.H;
    }
    if (c.write_outputs && c.out_entropy) {
        const int64_t eld = c.entropy_ld ? c.entropy_ld : g;
        const int64_t width = c.pad_entropy ? eld : g;
        for (int64_t jj = j; jj < width; jj += 64)
            c.out_entropy[(int64_t)b * eld + jj] = (jj < len) ? (float)sd.H : -1.0f;
    }
    bool reject = false;
    if (j < len) {
        const bool gate = sd.H < tau;                   // strict; NaN never gates
        const int32_t x = tg.x;
        bool ok;
        if (greedy) {
            ok = (x == sp.argmax);
        } else {
            double p_x = 0.0, q_x = 1.0;
            if (x >= 0 && x < c.V) {
                p_x = exp(tg.ap - sp.lse);
                q_x = exp(tg.aq - sd.lse);
                if (c.filters) {
                    if (!filter_keeps(tg.xp, x, thP, cutP)) p_x = 0.0;
                    if (!filter_keeps(tg.xq, x, thD, cutD)) q_x = 0.0;
                }
            }
            const double u = (double)tg.u_test;
            ok = (u * q_x < p_x);
        }
        reject = !(gate || ok);
    }
    const unsigned long long rej = __ballot(reject);
    const int a = rej ? (__ffsll((long long)rej) - 1) : len;
    if (j == a) {                                       // exactly one lane: a <= len <= gamma < 64
        if (c.write_outputs) c.out_accept_len[b] = a;
        SeqInfo si;
        si.row = a;
        si.lseP = sp.lse;
        si.lseD = (a < len) ? sd.lse : 0.0;
        si.greedy_tok = -1;
        if (greedy) {
            si.mode = 2;
            si.u = 0.f;
            si.greedy_tok = sp.argmax;
            if (c.write_outputs) c.out_next_token[b] = sp.argmax;
        } else {
            si.u = tg.u_draw;                            // j == a: this lane's own block
            si.mode = (a < len) ? 0 : 1;
        }
        *si_out = si;
    }
}

// Gather and decision in one step.
template <bool BF16>
__device__ __forceinline__ void accept_wave(const AcceptCtx& c, int b, int j, int len, float Tb,
                                            const RowStat& sd, const RowStat& sp, SeqInfo* si_out)
{
    const TokenGather tg = accept_gather<BF16>(c, b, j, len, Tb);
    accept_decide<BF16>(c, b, j, len, Tb, sd, sp, tg, si_out);
}

}  // namespace hola
