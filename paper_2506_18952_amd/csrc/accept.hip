// Accept / first-reject kernel: one wavefront per sequence, lane j owns position j.
//
// Lane j merges the row partials of draft row j and target row j in double, forms
// lse = ln S - bref ln 2 and the draft entropy H = ln S - ln2 T / S (Section 3.1), applies the
// strict gate H < tau (Algorithm 1, Step 1), and where the gate is open falls back to the verifier
// (Equation (1)) through the acceptance test u * q(x) < p(x) with a Philox uniform keyed on
// (seed, sequence, position, level).  A ballot over the lanes gives the first rejected position.
// All of it is O(B * gamma) scalar work in double; the kernel is latency-, not bandwidth-bound.
#include "stats_device.h"

namespace hola {

template <bool BF16>
__global__ __launch_bounds__(64) void accept_kernel(AcceptParams p)
{
    const int b = blockIdx.x;
    const int j = threadIdx.x;                          // position (lane)
    const int g = p.gamma;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    const bool greedy = !(Tb > 0.f);
    const double invT = greedy ? 1.0 : 1.0 / (double)Tb;
    const double tau = (double)p.tau;

    RowStat sd = {NAN, NAN, -1}, sp = {NAN, NAN, -1};
    if (j < len) {
        if (p.draft_stats_in) {
            sd.lse = p.draft_stats_in[((int64_t)b * g + j) * 2 + 0];
            sd.H = p.draft_stats_in[((int64_t)b * g + j) * 2 + 1];
        } else {
            sd = merge_partials(p.partials + ((int64_t)b * g + j) * p.nparts, p.nparts);
        }
        p.statsD[((int64_t)b * g + j) * 2 + 0] = sd.lse;
        p.statsD[((int64_t)b * g + j) * 2 + 1] = sd.H;
    }
    if (j <= len) {
        const int64_t slot = (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
        sp = merge_partials(p.partials + slot * p.nparts, p.nparts);
        p.statsP[((int64_t)b * (g + 1) + j) * 2 + 0] = sp.lse;
        p.statsP[((int64_t)b * (g + 1) + j) * 2 + 1] = sp.H;
        p.argmaxP[(int64_t)b * (g + 1) + j] = sp.argmax;
        if (p.target_stats_out) {
            p.target_stats_out[((int64_t)b * (g + 1) + j) * 2 + 0] = sp.lse;
            p.target_stats_out[((int64_t)b * (g + 1) + j) * 2 + 1] = sp.H;
        }
    }
    if (p.out_entropy && j < g) {
        const int64_t eld = p.entropy_ld ? p.entropy_ld : g;
        p.out_entropy[(int64_t)b * eld + j] = (j < len) ? (float)sd.H : -1.0f;
    }

    const uint64_t seq = (uint64_t)(p.seq_base + b);
    bool reject = false;
    if (j < len) {
        const bool gate = sd.H < tau;                   // strict; NaN never gates
        const int32_t x = p.tokens[(int64_t)b * g + j];
        bool ok;
        if (greedy) {
            ok = (x == sp.argmax);
        } else {
            double p_x = 0.0, q_x = 1.0;
            if (x >= 0 && x < p.V) {
                double zp = (double)load_logit<BF16>(p.target, ((int64_t)b * (g + 1) + j) * p.target_ld + x) * invT;
                double zq = (double)load_logit<BF16>(p.draft, ((int64_t)b * g + j) * p.draft_ld + x) * invT;
                p_x = exp(zp - sp.lse);
                q_x = exp(zq - sd.lse);
            }
            Philox4 r = philox4x32_10((uint32_t)j, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                      (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
            double u = (double)u24(r.x);
            ok = (u * q_x < p_x);
        }
        reject = !(gate || ok);
    }
    const unsigned long long rej = __ballot(reject);
    const int a = rej ? (__ffsll((long long)rej) - 1) : len;

    if (j == a) {                                       // exactly one lane: a <= len <= gamma < 64
        p.out_accept_len[b] = a;
        SeqInfo si;
        si.row = a;
        si.lseP = sp.lse;
        si.lseD = (a < len) ? sd.lse : 0.0;
        si.pad = 0;
        if (greedy) {
            si.mode = 2;
            si.u = 0.f;
            p.out_next_token[b] = sp.argmax;
        } else {
            Philox4 r = philox4x32_10((uint32_t)a, (uint32_t)seq, (uint32_t)(seq >> 32), p.level,
                                      (uint32_t)p.seed, (uint32_t)(p.seed >> 32));
            si.u = u24(r.y);
            si.mode = (a < len) ? 0 : 1;
        }
        p.seq[b] = si;
    }
}

// (lse, H) of plain rows from their partials, one thread per row.
__global__ void finalize_rows_kernel(const Partial* __restrict__ partials, int nparts, int32_t R, double* __restrict__ out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    RowStat s = merge_partials(partials + (int64_t)r * nparts, nparts);
    out[2 * (int64_t)r + 0] = s.lse;
    out[2 * (int64_t)r + 1] = s.H;
}

hipError_t launch_finalize_rows(const Partial* partials, int nparts, int32_t R, double* out, hipStream_t s)
{
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_rows_kernel, dim3((unsigned)((R + 127) / 128)), dim3(128), 0, s, partials, nparts, R, out);
    return hipGetLastError();
}

hipError_t launch_accept(const AcceptParams& p, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    dim3 grid((unsigned)p.B), block(64);
    if (p.dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((accept_kernel<true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((accept_kernel<false>), grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace hola
