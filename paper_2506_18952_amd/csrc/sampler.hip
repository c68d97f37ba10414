// Split sampler kernels: tile_sums_kernel sweeps the stop row pair of every sequence once (one
// wavefront per tile) and writes the tile weights; select_kernel (one wavefront per sequence) scans
// them and picks the token (sampler_device.h).  Used with the split-row statistics path.
#include "sampler_device.h"

namespace hola {

template <bool BF16>
__device__ __forceinline__ void row_pair_of(RowPair& rp, const SamplerParams& p, int b, const SeqInfo& si, int force_bonus)
{
    const float Tb = p.row_temperature ? p.row_temperature[b] : p.temperature;
    make_row_pair<BF16>(rp, p.target, p.draft, p.target_ld, p.draft_ld, p.gamma, p.V, Tb, b, si, force_bonus);
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void tile_sums_kernel(SamplerParams p)
{
    const int blocks_per_seq = (p.ntiles + kWaves - 1) / kWaves;
    const int b = blockIdx.x / blocks_per_seq;
    const int tb = blockIdx.x % blocks_per_seq;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile = tb * kWaves + wave;
    if (tile >= p.ntiles) return;
    const SeqInfo si = p.seq[b];
    if (si.mode == 2) return;                                        // greedy: token already written
    RowPair rp;
    row_pair_of<BF16>(rp, p, b, si, 0);
    double wsum = 0.0;
    if (rp.ok) wsum = tile_weight<BF16>(rp, tile, lane);
    if (lane == 0) p.tiles[(int64_t)b * p.ntiles + tile] = wsum;
}

template <bool BF16>
__global__ __launch_bounds__(64) void select_kernel(SamplerParams p)
{
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    const SeqInfo si = p.seq[b];
    if (si.mode == 2) return;
    double* tiles = p.tiles + (int64_t)b * p.ntiles;
    RowPair rp;
    row_pair_of<BF16>(rp, p, b, si, 0);
    int32_t token = -1;
    if (rp.ok) {
        token = select_token<BF16, false>(rp, tiles, p.ntiles, si.u, lane);
        if (token == -2) {
            // No residual mass: fall back to p itself, once.
            row_pair_of<BF16>(rp, p, b, si, 1);
            for (int t = 0; t < p.ntiles; ++t) {
                const double wsum = tile_weight<BF16>(rp, t, lane);
                if (lane == 0) tiles[t] = wsum;
            }
            __threadfence();
            token = select_token<BF16, false>(rp, tiles, p.ntiles, si.u, lane);
            if (token < 0) token = -1;
        }
    }
    if (lane == 0) p.out_next_token[b] = token;
}

int sampler_tiles(int V, int dtype)
{
    const int epl = (dtype == HOLA_DTYPE_BF16) ? 8 : 4;
    const int64_t chunks = ((int64_t)V + epl - 1) / epl + 1;         // +1: a misaligned row spills into one more chunk
    return (int)((chunks + 64 * kTileChunks - 1) / (64 * kTileChunks));
}

hipError_t launch_tile_sums(const SamplerParams& p, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    const int64_t blocks_per_seq = (p.ntiles + kWaves - 1) / kWaves;
    const int64_t nblk = blocks_per_seq * p.B;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)nblk), block(kBlock);
    if (p.dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((tile_sums_kernel<true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((tile_sums_kernel<false>), grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_select(const SamplerParams& p, hipStream_t s)
{
    if (p.B <= 0) return hipSuccess;
    dim3 grid((unsigned)p.B), block(64);
    if (p.dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((select_kernel<true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((select_kernel<false>), grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace hola
