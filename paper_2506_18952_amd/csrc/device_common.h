// Device-side helpers for the gfx950 kernels of libhola.so: logit unpacking, the scaled
// exponent, 64-lane reductions and scans, Philox4x32-10.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hola {

constexpr double kLog2e = 1.4426950408889634074;
constexpr double kLn2 = 0.69314718055994530942;

__device__ __forceinline__ float bits_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 2^y on the transcendental unit (v_exp_f32); y below -126 gives 0.
__device__ __forceinline__ float fast_exp2(float y) { return __builtin_amdgcn_exp2f(y); }

// Scaled exponent y = x*c + b with c = c_hi + c_lo carried in two floats: the product with
// c_hi is added to the reference first, so the small correction lands on a small number.
template <bool SINGLE_C>
__device__ __forceinline__ float scaled_exponent(float x, float c_hi, float c_lo, float b)
{
    float y = __builtin_fmaf(x, c_hi, b);
    if (!SINGLE_C) y = __builtin_fmaf(x, c_lo, y);
    return y;
}

// Streaming 16-byte load: the logits are read once, so the load carries the non-temporal hint and does not
// allocate in the caches (on MI355X a pure reader goes from ~6.1 TB/s with plain loads to ~7.0 TB/s).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4_t* global_chunk_ptr;   // global (not flat) addressing
typedef const __attribute__((address_space(1))) char* global_byte_ptr;
__device__ __forceinline__ uint4 load_stream(global_chunk_ptr p)
{
    const u32x4_t v = __builtin_nontemporal_load(p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 load_stream(const uint4* p) { return load_stream((global_chunk_ptr)p); }

// Element k (0..EPL-1) of a 16-byte chunk as float.
template <bool BF16>
__device__ __forceinline__ float chunk_elem(const uint4& v, int k)
{
    if (BF16) {
        uint32_t w = (k < 2) ? v.x : (k < 4) ? v.y : (k < 6) ? v.z : v.w;
        return (k & 1) ? bf16_hi(w) : bf16_lo(w);
    } else {
        uint32_t w = (k == 0) ? v.x : (k == 1) ? v.y : (k == 2) ? v.z : v.w;
        return bits_f32(w);
    }
}

template <bool BF16>
__device__ __forceinline__ float load_logit(const void* base, int64_t idx)
{
    if (BF16) return __uint_as_float((uint32_t)((const uint16_t*)base)[idx] << 16);
    return ((const float*)base)[idx];
}

// A value that is the same in every lane, moved to scalar registers so that the compiler knows it.
__device__ __forceinline__ int64_t wave_uniform(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Lanes of ONE wavefront hand values to one another through memory (one lane stores, the others load): the hardware
// keeps a wavefront's accesses to one kind of memory in order, but to the compiler a lane's load is unrelated to
// another lane's store and may be moved ahead of it.  The fence (wavefront scope: no instruction of its own) pins
// the order in the program; the barrier keeps the lanes' code together.
__device__ __forceinline__ void wave_handoff()
{
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// ---- 64-lane wavefront collectives (not on the streaming path) ------------------------------
// Sums, scans, maxima and minima over the wavefront move data with data-parallel-primitive controls of the vector
// unit (shifts inside the rows of 16 lanes, then the last lane of a row broadcast into the rows after it) instead of
// permutes through the shared-memory crossbar: six dependent steps of a few cycles each instead of six of ~100.
// A lane without a source (shifted in from outside its row, or in a row the step does not write) takes the
// operation's identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_take(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_take_f64(double identity, double v)
{
    const int lo = dpp_take<CTRL, ROW_MASK>(__double2loint(identity), __double2loint(v));
    const int hi = dpp_take<CTRL, ROW_MASK>(__double2hiint(identity), __double2hiint(v));
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double lane63(double v)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// Inclusive prefix sum over the lanes of a wavefront (lane i: v_0 + ... + v_i).
__device__ __forceinline__ double wave_inclusive_scan(double v, int /*lane*/)
{
    v += dpp_take_f64<kDppRowShr1, 0xf>(0.0, v);
    v += dpp_take_f64<kDppRowShr2, 0xf>(0.0, v);
    v += dpp_take_f64<kDppRowShr4, 0xf>(0.0, v);
    v += dpp_take_f64<kDppRowShr8, 0xf>(0.0, v);
    v += dpp_take_f64<kDppRowBcast15, 0xa>(0.0, v);               // rows 1 and 3 take the total of the row before
    v += dpp_take_f64<kDppRowBcast31, 0xc>(0.0, v);               // rows 2 and 3 take the total of the first two
    return v;
}
__device__ __forceinline__ double wave_sum(double v) { return lane63(wave_inclusive_scan(v, 0)); }

__device__ __forceinline__ float wave_max(float v)
{
    const int ninf = (int)0xff800000u;
#define HOLA_MAX_STEP(CTRL, MASK) v = fmaxf(v, __int_as_float(dpp_take<CTRL, MASK>(ninf, __float_as_int(v))))
    HOLA_MAX_STEP(kDppRowShr1, 0xf); HOLA_MAX_STEP(kDppRowShr2, 0xf); HOLA_MAX_STEP(kDppRowShr4, 0xf);
    HOLA_MAX_STEP(kDppRowShr8, 0xf); HOLA_MAX_STEP(kDppRowBcast15, 0xa); HOLA_MAX_STEP(kDppRowBcast31, 0xc);
#undef HOLA_MAX_STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_min(float v)
{
    const int pinf = 0x7f800000;
#define HOLA_MIN_STEP(CTRL, MASK) v = fminf(v, __int_as_float(dpp_take<CTRL, MASK>(pinf, __float_as_int(v))))
    HOLA_MIN_STEP(kDppRowShr1, 0xf); HOLA_MIN_STEP(kDppRowShr2, 0xf); HOLA_MIN_STEP(kDppRowShr4, 0xf);
    HOLA_MIN_STEP(kDppRowShr8, 0xf); HOLA_MIN_STEP(kDppRowBcast15, 0xa); HOLA_MIN_STEP(kDppRowBcast31, 0xc);
#undef HOLA_MIN_STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Smallest of a double over the wavefront (every lane gets it).
__device__ __forceinline__ double wave_min(double v)
{
#define HOLA_MIN_STEP(CTRL, MASK) v = fmin(v, dpp_take_f64<CTRL, MASK>((double)INFINITY, v))
    HOLA_MIN_STEP(kDppRowShr1, 0xf); HOLA_MIN_STEP(kDppRowShr2, 0xf); HOLA_MIN_STEP(kDppRowShr4, 0xf);
    HOLA_MIN_STEP(kDppRowShr8, 0xf); HOLA_MIN_STEP(kDppRowBcast15, 0xa); HOLA_MIN_STEP(kDppRowBcast31, 0xc);
#undef HOLA_MIN_STEP
    return lane63(v);
}

// ---- values that cross from one workgroup to another INSIDE a launch ------------------------------------------
// The compute units' vector caches and the chip's eight second-level caches are not coherent with one another
// within a launch.  Such a value is therefore written and read with device-scope relaxed atomic accesses: the
// store goes through to memory, the load comes from it, and no cache has to be written back or emptied as a whole
// (which is what a device-scope fence does: measured at 10 x the cost of a whole launch when every workgroup
// does it).  Ordering is the caller's business: wait for the stores (stores_through_done) before telling anybody,
// and load only after having been told.
__device__ __forceinline__ void store_through(double* dst, double v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), (unsigned long long)__double_as_longlong(v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double load_through(const double* src)
{
    return __longlong_as_double((long long)__hip_atomic_load(reinterpret_cast<const unsigned long long*>(src),
                                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
// Every store this wavefront has issued has been acknowledged by the memory system.
__device__ __forceinline__ void stores_through_done()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// A sequence's completion ticket: one 64-bit word in the workspace, (tag << 16 | count).  The workspace arrives with
// any contents, so a word counts only if it carries this call's tag (48 bits, drawn per call); anything else reads
// as count 0.  Whoever takes the last of `expected` tickets is told so (returns true) and leaves the word at 0, so
// that a replay of a captured launch (same tag) starts afresh.  Nobody waits for anybody; one load and one
// single-shot atomic per caller (only the first ticket of a call swaps).  Called by one thread per workgroup.
__device__ __forceinline__ bool take_ticket(unsigned long long* word, unsigned long long tag, uint32_t expected)
{
    const unsigned long long mine = tag << 16;
    unsigned long long cur = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long prev;                                     // the word before this ticket
    if ((cur >> 16) == tag) prev = __hip_atomic_fetch_add(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else if (__hip_atomic_compare_exchange_strong(word, &cur, mine | 1ull, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        prev = mine;
    else prev = __hip_atomic_fetch_add(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = (uint32_t)(prev & 0xffffu) + 1u >= expected;
    if (last) __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return last;
}

// ---- Philox4x32-10 (Salmon et al., SC'11) ---------------------------------------------------
struct Philox4 { uint32_t x, y, z, w; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return Philox4{c0, c1, c2, c3};
}

// Uniform on the 24-bit lattice in [0,1): exact in float and double.
__device__ __forceinline__ float u24(uint32_t r) { return (float)(r >> 8) * 5.9604644775390625e-8f; }

}  // namespace hola
