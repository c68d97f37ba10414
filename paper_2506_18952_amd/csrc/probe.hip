// Measurement aids, not part of the verify step: a read-only streaming kernel that shows what this machine gives
// a reader shaped like the statistics pass (one workgroup of 256 threads per segment of a row, 8 loads of 16
// bytes in flight per lane), with plain or non-temporal loads and, optionally, the arithmetic the bf16 statistics
// pass performs per 16 bytes.  The benchmark reports its rate beside the published HBM peak as the practical ceiling.
#include "device_common.h"
#include "hola_internal.h"

namespace hola {

static __device__ volatile float g_probe_sink;                      // written only on a value the sums never take

// ARITH: per 16-byte chunk 8 unpacks, 16 + 8 FMAs, 8 exp2, 7 adds, most of a max, 2 converts and 2 double adds:
// what accum_chunk does for eight bf16 logits, on the loaded bits taken as they come.
template <bool NT, bool ARITH>
__global__ __launch_bounds__(kBlock) void read_probe_kernel(const uint4* __restrict__ src, int64_t chunks_per_block, int64_t total,
                                                            float c1, float c2, float ref)
{
    constexpr int U = 8;
    const int64_t lo = (int64_t)blockIdx.x * chunks_per_block;
    int64_t hi = lo + chunks_per_block;
    if (hi > total) hi = total;
    uint32_t x = 0;
    double Sd = 0.0, Td = 0.0;
    float mxall = -INFINITY;
    int64_t c = lo + threadIdx.x;
    while (c + (int64_t)(U - 1) * kBlock < hi) {
        uint4 b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) b[u] = NT ? load_stream(src + c + u * kBlock) : src[c + u * kBlock];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ARITH) {
                float e[8], t0 = 0.f, t1 = 0.f, mx = -INFINITY;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const float v = chunk_elem<true>(b[u], k);
                    mx = fmaxf(mx, v);
                    const float y = __builtin_fmaf(v, c2, __builtin_fmaf(v, c1, ref));
                    e[k] = fast_exp2(y);
                    if (k & 1) t1 = __builtin_fmaf(y, e[k], t1); else t0 = __builtin_fmaf(y, e[k], t0);
                }
                mxall = fmaxf(mxall, mx);
                Sd += (double)(((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7])));
                Td += (double)(t0 + t1);
            } else {
                x ^= b[u].x ^ b[u].y ^ b[u].z ^ b[u].w;
            }
        }
        c += (int64_t)U * kBlock;
    }
    for (; c < hi; c += kBlock) { const uint4 v = src[c]; x ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (ARITH ? (Sd + Td + (double)mxall == 12345.678) : (x == 0x9e3779b9u && threadIdx.x == 77)) g_probe_sink = (float)Sd + (float)x;
}

hipError_t launch_read_probe(const void* src, size_t bytes, int64_t block_bytes, int nontemporal, int arith, hipStream_t s)
{
    const int64_t total = (int64_t)(bytes / 16);
    int64_t cpb = block_bytes / 16;
    if (cpb < kBlock) cpb = kBlock;
    const int64_t nblk = (total + cpb - 1) / cpb;
    if (nblk <= 0) return hipSuccess;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nblk), block(kBlock);
    const uint4* p = (const uint4*)src;
    // scale constants of T = 0.8 as the statistics pass splits them; the reference keeps the exponent arguments small
    const float c1 = 1.8033447265625f, c2 = 2.4061e-5f, ref = -8.f;
    if (nontemporal) {
        if (arith) hipLaunchKernelGGL((read_probe_kernel<true, true>), grid, block, 0, s, p, cpb, total, c1, c2, ref);
        else hipLaunchKernelGGL((read_probe_kernel<true, false>), grid, block, 0, s, p, cpb, total, c1, c2, ref);
    } else {
        if (arith) hipLaunchKernelGGL((read_probe_kernel<false, true>), grid, block, 0, s, p, cpb, total, c1, c2, ref);
        else hipLaunchKernelGGL((read_probe_kernel<false, false>), grid, block, 0, s, p, cpb, total, c1, c2, ref);
    }
    return hipGetLastError();
}

}  // namespace hola
