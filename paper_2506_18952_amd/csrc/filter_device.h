// Pieces shared by the kernels that find the keep sets of top-k / top-p filtered rows: order-preserving keys of
// logits, the description of a row as 16-byte chunks, and the fixed-point mass of a listed token.
#pragma once
#include "sampler_device.h"

namespace hola {

// Masses of listed tokens are taken relative to the reference of the row's largest logit (each <= ~1) and
// summed as integers in units of 2^-38, so a sum does not depend on the order of its terms; packed histogram
// entries keep a count above the 51 mass bits.
constexpr int kListMassBits = 51;
constexpr uint64_t kListMassMask = (1ull << kListMassBits) - 1;
constexpr double kListMassUnit = 274877906944.0;               // 2^38

// Order-preserving key of a logit (larger logit, larger key); -0 and +0 share a key.
template <bool BF16>
__device__ __forceinline__ uint32_t order_key(float x)
{
    if (x == 0.f) x = 0.f;
    const uint32_t b = __float_as_uint(x);
    const uint32_t k = b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
    return BF16 ? (k >> 16) : k;
}
template <bool BF16>
__device__ __forceinline__ float key_to_logit(uint32_t key)
{
    const uint32_t k = BF16 ? (key << 16) : key;
    uint32_t b = (k >> 31) ? (k ^ 0x80000000u) : ~k;
    if (BF16) b &= 0xffff0000u;                                 // the low half of a widened bf16 is zero
    return __uint_as_float(b);
}

struct FilterRow {
    const uint4* rowv; int32_t head, V; int64_t nchunks;
    ExpScale sc; float ref; double scale;                       // p_i = 2^(exp_arg(x_i)) * scale
};

template <bool BF16>
__device__ __forceinline__ uint64_t list_mass_fixed(const FilterRow& fr, float x)
{
    const double p = (double)fast_exp2(exp_arg<BF16>(x, fr.ref, fr.sc)) * fr.scale;
    return (uint64_t)(p * kListMassUnit + 0.5);
}

// Row r of a filtered call, r in [0, B (2 gamma + 1)): per sequence the gamma draft rows, then the gamma + 1
// target rows.  Returns false for a row the call does not use (beyond the sequence's draft length, or a draft row
// when the draft rows' keep sets were handed over by the previous level: skip_draft).
struct FilterRowId { int b, j; bool is_draft; int64_t slot; };
__device__ __forceinline__ bool filter_row_id(int r, int32_t B, int32_t gamma, const int32_t* draft_len, FilterRowId& id,
                                              int32_t skip_draft = 0)
{
    const int rows_per_seq = 2 * gamma + 1;
    id.b = r / rows_per_seq;
    const int k = r % rows_per_seq;
    id.is_draft = k < gamma;
    id.j = id.is_draft ? k : k - gamma;
    int len = draft_len ? draft_len[id.b] : gamma;
    len = len < 0 ? 0 : (len > gamma ? gamma : len);
    id.slot = id.is_draft ? (int64_t)id.b * gamma + id.j : (int64_t)B * gamma + (int64_t)id.b * (gamma + 1) + id.j;
    return id.is_draft ? (!skip_draft && id.j < len) : (id.j <= len);
}

template <bool BF16>
__device__ __forceinline__ FilterRow make_filter_row(const void* target, const void* draft, int64_t target_ld, int64_t draft_ld,
                                                     int32_t gamma, int32_t V, float temperature, const FilterRowId& id)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    const char* row = id.is_draft ? (const char*)draft + ((int64_t)id.b * gamma + id.j) * draft_ld * ES
                                  : (const char*)target + ((int64_t)id.b * (gamma + 1) + id.j) * target_ld * ES;
    FilterRow fr;
    const uintptr_t addr = (uintptr_t)row;
    fr.head = (int32_t)((addr & 15) / ES);
    fr.rowv = (const uint4*)(addr & ~(uintptr_t)15);
    fr.V = V;
    fr.nchunks = ((int64_t)V + fr.head + N - 1) / N;
    fr.sc = make_scale(kLog2e / (double)temperature);
    fr.ref = 0.f;
    fr.scale = 1.0;
    return fr;
}

// Sum over the wavefront of a 64-bit integer, the same value in every lane.  Four data-parallel-primitive steps
// (lane ^ 1, lane ^ 2, reversal within 8, reversal within 16) leave each lane with the sum of its row of 16
// lanes; the four row sums are read into scalars and added there.  An order of magnitude less latency than six
// cross-lane permutes through the LDS crossbar, which matters where a radix descent needs one sum per key bit.
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v)
{
#define HOLA_DPP_STEP(ctrl)                                                                                       \
    {                                                                                                             \
        const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, ctrl, 0xf, 0xf, true);     \
        const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), ctrl, 0xf, 0xf, true); \
        v += ((unsigned long long)hi << 32) | lo;                                                                 \
    }
    HOLA_DPP_STEP(0xb1)                                         // quad_perm [1,0,3,2]
    HOLA_DPP_STEP(0x4e)                                         // quad_perm [2,3,0,1]
    HOLA_DPP_STEP(0x141)                                        // row_half_mirror
    HOLA_DPP_STEP(0x140)                                        // row_mirror
#undef HOLA_DPP_STEP
    unsigned long long total = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 16 * row);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 16 * row);
        total += ((unsigned long long)hi << 32) | lo;
    }
    return total;
}

}  // namespace hola
