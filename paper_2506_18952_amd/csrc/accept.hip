// Split accept kernel: one wavefront per sequence; lane j merges the row partials of draft row j and
// target row j in double (lse = ln S - beta ln 2, H = ln S - ln2 T / S) and runs the accept stage
// (accept_device.h).  Latency-, not bandwidth-bound: O(B * gamma) scalar work.
#include "accept_device.h"

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

    RowStat sd = {NAN, NAN, -1}, sp = {NAN, NAN, -1};
    if (j < len) {
        if (p.draft_stats_in) {
            sd.lse = p.draft_stats_in[((int64_t)b * g + j) * 2 + 0];
            sd.H = p.draft_stats_in[((int64_t)b * g + j) * 2 + 1];
        } else {
            sd = merge_partials(p.partials + ((int64_t)b * g + j) * p.nparts, p.nparts);
        }
    }
    if (j <= len) {
        const int64_t slot = (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
        sp = merge_partials(p.partials + slot * p.nparts, p.nparts);
    }
    AcceptCtx c;
    c.target = p.target; c.draft = p.draft; c.target_ld = p.target_ld; c.draft_ld = p.draft_ld;
    c.tokens = p.tokens; c.tokens_ld = p.tokens_ld; c.pad_entropy = p.pad_entropy; c.seed = p.seed; c.level = p.level; c.seq_base = p.seq_base;
    c.gamma = g; c.V = p.V; c.tau = p.tau; c.target_stats_out = p.target_stats_out;
    c.out_accept_len = p.out_accept_len; c.out_next_token = p.out_next_token;
    c.out_entropy = p.out_entropy; c.entropy_ld = p.entropy_ld;
    accept_wave<BF16>(c, b, j, len, Tb, sd, sp, p.seq + b);
}

// (lse, H) of plain rows from their partials, one thread per row.
__global__ void finalize_rows_kernel(const Partial* __restrict__ partials, int nparts, int32_t R, double* __restrict__ out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const RowStat s = merge_partials(partials + (int64_t)r * nparts, nparts);
    out[2 * (int64_t)r + 0] = s.lse;
    out[2 * (int64_t)r + 1] = s.H;
}

hipError_t launch_finalize_rows(const Partial* partials, int nparts, int32_t R, double* out, hipStream_t s)
{
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(finalize_rows_kernel, dim3((unsigned)((R + 127) / 128)), dim3(128), 0, s, partials, nparts, R, out);
    return hipGetLastError();
}

// Row statistics from the statistics of the row's column tiles, one thread per row, double.  The row's
// distribution is the mixture of the tiles' with weights w_t = exp(lse_t - lse), so Section 3.1's entropy is
// H = sum_t w_t (H_t - ln w_t); tiles without a finite logit (lse_t = -inf) carry no mass.
__global__ void merge_tile_stats_kernel(const double* __restrict__ ts, int32_t R, int32_t nt, double* __restrict__ out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const double* t = ts + (int64_t)r * nt * 2;
    double m = -INFINITY;
    bool bad = false;
    for (int i = 0; i < nt; ++i) {
        const double l = t[2 * i];
        if (!(l == l)) bad = true;
        m = fmax(m, l);
    }
    double lse, H = NAN;
    if (bad) {
        lse = NAN;
    } else if (!(m > -INFINITY) || !(m < INFINITY)) {
        lse = m;
    } else {
        double S = 0.0;
        for (int i = 0; i < nt; ++i) S += exp(t[2 * i] - m);
        lse = m + log(S);
        H = 0.0;
        for (int i = 0; i < nt; ++i) {
            const double lw = t[2 * i] - lse;
            const double wt = exp(lw);
            if (wt > 0.0) H += wt * (t[2 * i + 1] - lw);
        }
    }
    out[2 * (int64_t)r + 0] = lse;
    out[2 * (int64_t)r + 1] = H;
}

hipError_t launch_merge_tile_stats(const double* ts, int32_t R, int32_t nt, double* out, hipStream_t s)
{
    if (R <= 0) return hipSuccess;
    hipLaunchKernelGGL(merge_tile_stats_kernel, dim3((unsigned)((R + 127) / 128)), dim3(128), 0, s, ts, R, nt, out);
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
