// Device code of the row statistics (shared by the split-row kernel and the fused per-sequence kernel).
//
// For one logits row the entropy of Section 3.1 (H = -sum p_i log p_i) and the softmax normaliser
// follow from two sums over y_i = x_i * c + beta, c = log2(e)/temperature:
//     S = sum_i 2^(y_i),   T = sum_i y_i 2^(y_i);   lse = ln S - beta ln 2,   H = ln S - ln2 * T / S.
// Each lane streams 16-byte chunks and keeps (S, T) in DOUBLE, fed by fp32 chunk sums of 4-8 terms, so a
// dominant term never sits in an fp32 accumulator while hundreds of small ones are added to it.
//
// The exponent argument is formed so that its rounding is unbiased and consistent over the row:
//   bf16 logits: c = c1 + c2 with c1 cut to 16 significant bits, so x * c1 is exact in fp32;
//                y = fma(x, c2, fma(x, c1, b)) with an integer-valued reference b (beta = b).
//   fp32 logits: d = x - m against a reference logit m, y = fma(d, c_hi, d * c_lo) (beta = -m c).
// The reference comes from the wavefront's first chunk and moves only when a logit exceeds it by more
// than a binade (rare); the lane's double sums are then re-referenced exactly in double.
#pragma once
#include "device_common.h"
#include "hola_internal.h"

namespace hola {

__device__ __forceinline__ ExpScale make_scale(double cstar)
{
    ExpScale s;
    s.cstar = cstar;
    s.c_hi = (float)cstar;
    s.c_lo = (float)(cstar - (double)s.c_hi);
    s.c1 = __uint_as_float((__float_as_uint(s.c_hi) + 0x80u) & 0xffffff00u);
    s.c2 = (float)(cstar - (double)s.c1);
    s.inv_c = 1.0f / s.c_hi;
    return s;
}

// Exponent argument y for logit x against reference ref.
template <bool BF16>
__device__ __forceinline__ float exp_arg(float x, float ref, const ExpScale& sc)
{
    if (BF16) return __builtin_fmaf(x, sc.c2, __builtin_fmaf(x, sc.c1, ref));
    const float d = x - ref;
    return __builtin_fmaf(d, sc.c_hi, d * sc.c_lo);
}

// Offset beta such that y = x * cstar + beta.
template <bool BF16>
__device__ __forceinline__ double ref_offset(float ref, const ExpScale& sc)
{
    return BF16 ? (double)ref : -(double)ref * sc.cstar;
}

// Reference that puts logit mx at y ~ 0, and the logit above which y would exceed ~1.
template <bool BF16>
__device__ __forceinline__ float ref_for(float mx, const ExpScale& sc) { return BF16 ? -rintf(mx * sc.c_hi) : mx; }
template <bool BF16>
__device__ __forceinline__ float thr_for(float ref, const ExpScale& sc)
{
    return BF16 ? (1.f - ref) * sc.inv_c : ref + sc.inv_c;
}

struct LaneState {
    double Sd, Td;         // sums at offset ref_offset(ref)
    float ref, thr_ref;    // current reference; logit above which it must move
    float thr;             // trigger of the rare path (thr_ref, or the running maximum on argmax rows)
    float vmax; int32_t imax;
};

__device__ __forceinline__ void lane_init(LaneState& st)
{
    st.Sd = 0.0; st.Td = 0.0; st.ref = 0.f; st.thr_ref = -INFINITY; st.thr = -INFINITY;
    st.vmax = -INFINITY; st.imax = -1;
}

// 2^d in double for the rare path.  Kept out of line: inlined into the streaming loop, the constants of its
// polynomial would occupy vector registers for the whole loop.
__device__ __noinline__ double exp2_out_of_line(double d) { return exp2(d); }

// Move the lane to a reference built from logit mx; the sums are rescaled exactly in double.
template <bool BF16>
__device__ __forceinline__ void re_reference(LaneState& st, float mx, const ExpScale& sc)
{
    const float nref = ref_for<BF16>(mx, sc);
    if (st.Sd != 0.0 || st.Td != 0.0) {
        const double delta = ref_offset<BF16>(nref, sc) - ref_offset<BF16>(st.ref, sc);   // < 0
        // bf16 references are integers, so the factor is an exact power of two
        const double f = BF16 ? ldexp(1.0, (int)fmax(delta, -4096.0)) : exp2_out_of_line(delta);
        st.Td = (st.Td + delta * st.Sd) * f;
        st.Sd *= f;
    }
    st.ref = nref;
    st.thr_ref = thr_for<BF16>(nref, sc);
}

// Rare path: a logit above the lane's trigger arrived.
template <bool BF16, bool ARGMAX>
__device__ __forceinline__ void on_exceed(LaneState& st, float mx, int32_t idx, const ExpScale& sc)
{
    if (ARGMAX && mx > st.vmax) { st.vmax = mx; st.imax = idx; }
    if (mx > st.thr_ref) re_reference<BF16>(st, mx, sc);
    st.thr = ARGMAX ? st.vmax : st.thr_ref;
}

// One element with every guard (edge elements and the fallback pass): -inf logits carry no mass.
template <bool BF16, bool ARGMAX>
__device__ __forceinline__ void accum_elem(LaneState& st, float x, int32_t idx, const ExpScale& sc)
{
    if (x == -INFINITY) return;
    if (x > st.thr) on_exceed<BF16, ARGMAX>(st, x, idx, sc);
    const float y = exp_arg<BF16>(x, st.ref, sc);
    const float e = fast_exp2(y);
    st.Sd += (double)e;
    st.Td += (double)(y * e);
}

// The sums of one chunk's terms with -inf logits left out, in the order of the fast path.  A -inf logit (a masked
// or padded vocabulary entry) carries no mass, but the unguarded arithmetic turns it into NaN: y 2^y = -inf x 0, and
// y itself when the low part of the scale constant is negative (-inf x c2 = +inf, added to -inf).
template <bool BF16, bool WITH_T>
__device__ __forceinline__ void chunk_sums_guarded(const uint4& v, float ref, const ExpScale& sc, float& s_out, float& t_out)
{
    constexpr int N = BF16 ? 8 : 4;
    float s = 0.f, t[2] = {0.f, 0.f};
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float x = chunk_elem<BF16>(v, k);
        if (x == -INFINITY) continue;
        const float y = exp_arg<BF16>(x, ref, sc);
        const float e = fast_exp2(y);
        s += e;
        if (WITH_T) t[k & 1] = __builtin_fmaf(y, e, t[k & 1]);
    }
    s_out = s;
    t_out = t[0] + t[1];
}

// Fast path: one 16-byte chunk, no per-element guards.  WITH_T = false leaves out T = sum y 2^y (rows of which
// only the normaliser is wanted).  GUARDED: -inf logits are left out of the sums (the second try of a wavefront
// whose unguarded sums came out NaN).
template <bool BF16, bool ARGMAX, bool WITH_T = true, bool GUARDED = false>
__device__ __forceinline__ void accum_chunk(LaneState& st, const uint4& v, int32_t elem0, const ExpScale& sc)
{
    constexpr int N = BF16 ? 8 : 4;
    float x[N];
#pragma unroll
    for (int k = 0; k < N; ++k) x[k] = chunk_elem<BF16>(v, k);
    float mx = x[0];
#pragma unroll
    for (int k = 1; k < N; ++k) mx = fmaxf(mx, x[k]);
    if (mx > st.thr) {
        int32_t idx = elem0;
        if (ARGMAX) {
#pragma unroll
            for (int k = N - 1; k >= 0; --k) if (x[k] == mx) idx = elem0 + k;   // lowest index wins
        }
        on_exceed<BF16, ARGMAX>(st, mx, idx, sc);
    }
    if (GUARDED) {
        float s, tt;
        chunk_sums_guarded<BF16, WITH_T>(v, st.ref, sc, s, tt);
        st.Sd += (double)s;
        if (WITH_T) st.Td += (double)tt;
        return;
    }
    float e[N], t[2] = {0.f, 0.f};
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float y = exp_arg<BF16>(x[k], st.ref, sc);
        e[k] = fast_exp2(y);
        if (WITH_T) t[k & 1] = __builtin_fmaf(y, e[k], t[k & 1]);
    }
    float s;
    if (N == 8) s = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
    else s = (e[0] + e[1]) + (e[2] + e[3]);
    float tt = WITH_T ? t[0] + t[1] : 0.f;
    if (!ARGMAX) {                                              // the few chunks of a wavefront's last, partial group
        const float chk = WITH_T ? tt : s;
        if (!(chk == chk)) chunk_sums_guarded<BF16, WITH_T>(v, st.ref, sc, s, tt);   // a -inf logit in the chunk (a NaN stays one)
    }
    st.Sd += (double)s;
    if (WITH_T) st.Td += (double)tt;
}

// The sums of one chunk's terms against the lane's reference, added to its state; no trigger.
template <bool BF16, bool WITH_T, bool GUARDED = false>
__device__ __forceinline__ void accum_chunk_terms(LaneState& st, const uint4& v, const ExpScale& sc)
{
    constexpr int N = BF16 ? 8 : 4;
    if (GUARDED) {
        float s, tt;
        chunk_sums_guarded<BF16, WITH_T>(v, st.ref, sc, s, tt);
        st.Sd += (double)s;
        if (WITH_T) st.Td += (double)tt;
        return;
    }
    float e[N], t[2] = {0.f, 0.f};
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float y = exp_arg<BF16>(chunk_elem<BF16>(v, k), st.ref, sc);
        e[k] = fast_exp2(y);
        if (WITH_T) t[k & 1] = __builtin_fmaf(y, e[k], t[k & 1]);
    }
    float s;
    if (N == 8) s = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
    else s = (e[0] + e[1]) + (e[2] + e[3]);
    st.Sd += (double)s;
    if (WITH_T) st.Td += (double)(t[0] + t[1]);
}

// Largest logit of a chunk (NaN elements are passed over, as everywhere the reference is chosen).
template <bool BF16>
__device__ __forceinline__ float chunk_max(const uint4& v)
{
    constexpr int N = BF16 ? 8 : 4;
    float mx = chunk_elem<BF16>(v, 0);
#pragma unroll
    for (int k = 1; k < N; ++k) mx = fmaxf(mx, chunk_elem<BF16>(v, k));
    return mx;
}

template <bool BF16, bool ARGMAX>
__device__ __forceinline__ void accum_chunk_robust(LaneState& st, const uint4& v, int32_t elem0, const ExpScale& sc)
{
    constexpr int N = BF16 ? 8 : 4;
#pragma unroll
    for (int k = 0; k < N; ++k) accum_elem<BF16, ARGMAX>(st, chunk_elem<BF16>(v, k), elem0 + k, sc);
}

// 2^d for d <= 0 in the merges of partial sums.  The offsets of bf16 rows are integers, so their differences are
// too, and the factor is a power of two that needs no polynomial (the same value: 2^d is exact there).
__device__ __forceinline__ double exp2_offset_diff(double d)
{
    if (d == rint(d)) return ldexp(1.0, (int)fmax(d, -4096.0));
    return exp2(d);
}

// Merge the 64 lane states in double; every lane returns the wavefront's Partial.
template <bool BF16, bool ARGMAX>
__device__ __forceinline__ Partial wave_merge(const LaneState& st, const ExpScale& sc)
{
    const bool has = !(st.Sd == 0.0 && st.Td == 0.0);   // also true for NaN
    const double beta = ref_offset<BF16>(st.ref, sc);
    const double bmin = wave_min(has ? beta : (double)INFINITY);
    double S = 0.0, T = 0.0;
    if (has) {
        const double diff = bmin - beta;                // <= 0
        S = st.Sd; T = st.Td;
        if (diff != 0.0) {
            const double f = exp2_offset_diff(diff);
            T = (T + diff * S) * f;
            S *= f;
        }
        if (!(beta == beta)) { S = NAN; T = NAN; }
    }
    Partial out;
    out.S = wave_sum(S);
    out.T = wave_sum(T);
    out.bref = (bmin == INFINITY) ? 0.0 : bmin;
    out.vmax = -INFINITY;
    out.imax = -1;
    if (ARGMAX) {
        float v = st.vmax;
        int32_t i = st.imax;
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            const float ov = __shfl_xor(v, m, 64);
            const int32_t oi = __shfl_xor(i, m, 64);
            const bool take = (oi >= 0) && (i < 0 || ov > v || (ov == v && oi < i));
            if (take) { v = ov; i = oi; }
        }
        out.vmax = v;
        out.imax = i;
    }
    return out;
}

// Geometry of a row on the 16-byte chunk grid anchored at the row pointer aligned down to 16 bytes.
struct RowGeom {
    const uint4* rowv;       // aligned chunk grid
    const void* row;         // the row itself (element addressing of the edges)
    int32_t head;            // elements of chunk 0 that precede the row
    int32_t V;
    int64_t c_first, c_end;  // full chunks [c_first, c_end)
    int32_t edge_lo_end;     // row elements [0, edge_lo_end) precede the first full chunk
    int32_t edge_hi_begin;   // row elements [edge_hi_begin, V) follow the last full chunk
};

template <bool BF16>
__device__ __forceinline__ RowGeom make_geom(const void* row, int32_t V)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    RowGeom g;
    const uintptr_t addr = (uintptr_t)row;
    g.row = row;
    g.V = V;
    g.head = (int32_t)((addr & 15) / ES);
    g.rowv = (const uint4*)(addr & ~(uintptr_t)15);
    g.c_first = g.head ? 1 : 0;
    g.c_end = ((int64_t)V + g.head) / N;
    if (g.c_end < g.c_first) g.c_end = g.c_first;
    int32_t lo = g.head ? (N - g.head) : 0;
    if (lo > V) lo = V;
    g.edge_lo_end = lo;
    int32_t hi = (int32_t)(g.c_end * N) - g.head;
    if (hi < lo) hi = lo;
    g.edge_hi_begin = hi;
    return g;
}

// The split-row kernel's division of a row: its full chunks go to nsplit segments [seg_lo, seg_hi) of equal length
// (a multiple of the workgroup's 256 lanes).  Within a segment the four wavefronts either interleave in blocks of
// 64 chunks, or, on the row a bonus token would be drawn from, take four contiguous slabs [lo, hi) (a multiple of
// 64 chunks each): partial (segment, wavefront) of that row is then the sum over one contiguous range of tokens, in
// index order, and the sampler can pick a slab from these sums and read only that slab again.
__device__ __forceinline__ void wave_slab(const RowGeom& g, int seg, int nsplit, int wave, int64_t& seg_lo, int64_t& seg_hi,
                                          int64_t& lo, int64_t& hi)
{
    const int64_t nfull = g.c_end - g.c_first;
    int64_t per = (nfull + nsplit - 1) / nsplit;            // full chunks per segment,
    per = (per + 255) / 256 * 256;                          // a multiple of the workgroup's lanes
    seg_lo = g.c_first + (int64_t)seg * per;
    seg_hi = seg_lo + per;
    if (seg_lo > g.c_end) seg_lo = g.c_end;
    if (seg_hi > g.c_end) seg_hi = g.c_end;
    int64_t wl = (seg_hi - seg_lo + 3) / 4;
    wl = (wl + 63) / 64 * 64;
    lo = seg_lo + (int64_t)wave * wl;
    if (lo > seg_hi) lo = seg_hi;
    hi = lo + wl < seg_hi ? lo + wl : seg_hi;
}

// One wavefront's pass over the chunks c0, c0 + stride, ... < c_hi of a row (c0 already holds the lane's
// offset), plus, if do_edges, the edge elements (fewer than two chunks' worth, one per lane).
template <bool BF16, bool ARGMAX, int U, bool ROBUST, bool WITH_T = true, bool GUARDED = false>
__device__ __forceinline__ void wave_pass(LaneState& st, const RowGeom& g, int64_t c0, int64_t c_hi_in, int64_t stride_in,
                                          bool do_edges, const ExpScale& sc, int lane)
{
    const int64_t c_hi = wave_uniform(c_hi_in), stride = wave_uniform(stride_in);
    constexpr int N = BF16 ? 8 : 4;
    lane_init(st);
    // The wavefront's lanes start from a common reference taken from the first chunks it loads (with
    // the whole first group already in flight), so that lanes rarely re-reference.
    bool need_ref = !ARGMAX && !ROBUST;
    // Loop control and addresses are wavefront-uniform (scalar registers): a load is scalar base + lane offset.
    const int64_t w0 = wave_uniform(c0 - lane);                  // chunk of the wavefront's first lane
    int64_t w = w0;
    global_byte_ptr wb = (global_byte_ptr)wave_uniform((int64_t)(uintptr_t)(g.rowv + w0));
    const uint32_t voff = (uint32_t)lane * 16u;
    const int64_t sb = stride * 16;
    // The fast pass looks after -inf logits (masked or padded vocabulary entries, whose unguarded terms are NaN)
    // one group late: once the NEXT group's loads are in flight, a lane whose sums the previous group spoiled takes
    // them back to what they were before it and redoes that group's chunks with the guarded sums (loaded again:
    // keeping them would cost the loop 28 registers).  Looked at right after the group, the same test held up the
    // next loads behind the group's last addition (+2 us on the headline); here it costs nothing measurable.
    constexpr bool REPAIR = !ROBUST && !ARGMAX && !GUARDED;
    double Sd_before = 0.0, Td_before = 0.0;                    // the lane's sums before the terms of the previous group
    bool have_prev = false;                                     // wavefront-uniform
    auto repair_previous = [&]() {
        const double chk = WITH_T ? st.Td : st.Sd;              // one sum tells: a -inf logit always spoils T, and S when it spoils y
        if (!(chk == chk)) {
            st.Sd = Sd_before; st.Td = Td_before;
            const global_byte_ptr pb = wb - (int64_t)U * sb;
            constexpr int R = U >= 2 ? 2 : U;                   // chunks loaded together: a rolled loop over U / R rounds, because
#pragma unroll 1                                                // few registers matter more here than speed
            for (int u0 = 0; u0 < U; u0 += R) {
                uint4 again[R];
#pragma unroll
                for (int r = 0; r < R; ++r) again[r] = load_stream((global_chunk_ptr)(pb + (u0 + r) * sb + voff));
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float s1, t1;
                    chunk_sums_guarded<BF16, WITH_T>(again[r], st.ref, sc, s1, t1);
                    st.Sd += (double)s1;
                    if (WITH_T) st.Td += (double)t1;
                }
            }
        }
    };
    // groups in which every lane of the wavefront has U chunks: no guards
    while (w + 63 + (int64_t)(U - 1) * stride < c_hi) {
        uint4 buf[U];
#pragma unroll
        for (int u = 0; u < U; ++u) buf[u] = load_stream((global_chunk_ptr)(wb + u * sb + voff));
        __builtin_amdgcn_sched_barrier(0);                      // every load of the group is issued before any is used
        if (REPAIR && have_prev) repair_previous();
        const int64_t c = w + lane;
        if (need_ref) {
            float mx = -INFINITY;
#pragma unroll
            for (int k = 0; k < N; ++k) mx = fmaxf(mx, chunk_elem<BF16>(buf[0], k));
            mx = wave_max(mx);
            if (mx > -INFINITY && mx < INFINITY) {
                st.ref = ref_for<BF16>(mx, sc);
                st.thr_ref = thr_for<BF16>(st.ref, sc);
                st.thr = st.thr_ref;
            }
            need_ref = false;
        }
        if (!ROBUST && !ARGMAX) {
            // The lane's reference is looked at once per group of loads: the largest logit of the whole group
            // decides whether it has to move (one test, rarely taken once the reference sits near the row's
            // top), and then the terms of all the group's chunks are formed against one reference in a single
            // piece of straight-line code.
            float mx = chunk_max<BF16>(buf[0]);
#pragma unroll
            for (int u = 1; u < U; ++u) mx = fmaxf(mx, chunk_max<BF16>(buf[u]));
            if (mx > st.thr) on_exceed<BF16, ARGMAX>(st, mx, 0, sc);
            if (REPAIR) { Sd_before = st.Sd; Td_before = st.Td; have_prev = true; }
#pragma unroll
            for (int u = 0; u < U; ++u) accum_chunk_terms<BF16, WITH_T, GUARDED>(st, buf[u], sc);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t e0 = (int32_t)((c + u * stride) * N) - g.head;
                if (ROBUST) accum_chunk_robust<BF16, ARGMAX>(st, buf[u], e0, sc);
                else accum_chunk<BF16, ARGMAX, WITH_T, GUARDED>(st, buf[u], e0, sc);
            }
        }
        w += (int64_t)U * stride;
        wb += (int64_t)U * sb;
    }
    if (REPAIR && have_prev) repair_previous();                 // the last full group
    // the last, partial group: all its loads are issued together, each one guarded
    if (w < c_hi) {
        const int64_t c = w + lane;
        uint4 buf[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            buf[u] = make_uint4(0, 0, 0, 0);
            if (c + u * stride < c_hi) buf[u] = load_stream((global_chunk_ptr)(wb + u * sb + voff));
        }
        if (need_ref) {
            float mx = -INFINITY;
            if (c < c_hi) {
#pragma unroll
                for (int k = 0; k < N; ++k) mx = fmaxf(mx, chunk_elem<BF16>(buf[0], k));
            }
            mx = wave_max(mx);
            if (mx > -INFINITY && mx < INFINITY) {
                st.ref = ref_for<BF16>(mx, sc);
                st.thr_ref = thr_for<BF16>(st.ref, sc);
                st.thr = st.thr_ref;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (c + u * stride < c_hi) {
                const int32_t e0 = (int32_t)((c + u * stride) * N) - g.head;
                if (ROBUST) accum_chunk_robust<BF16, ARGMAX>(st, buf[u], e0, sc);
                else accum_chunk<BF16, ARGMAX, WITH_T, GUARDED>(st, buf[u], e0, sc);
            }
        }
    }
    if (do_edges) {
        const int32_t n_lo = g.edge_lo_end, n_hi = g.V - g.edge_hi_begin;
        int32_t e = -1;
        if (lane < n_lo) e = lane;
        else if (lane - n_lo < n_hi) e = g.edge_hi_begin + (lane - n_lo);
        if (e >= 0) accum_elem<BF16, ARGMAX>(st, load_logit<BF16>(g.row, e), e, sc);
    }
}

// A wavefront's share of a row.  The fast pass has no guards; if its sums are not finite the wavefront goes over
// its share again: first with -inf logits left out of the sums (masked or padded vocabulary entries, whose
// unguarded terms are NaN: the usual cause, and this second try costs about as much as the first), and only if that
// fails too (a NaN or +inf logit, an overflow) element by element with every guard.
template <bool BF16, bool ARGMAX, int U, bool WITH_T = true>
__device__ __forceinline__ Partial wave_row_share(const RowGeom& g, int64_t c0, int64_t c_hi, int64_t stride,
                                                  bool do_edges, const ExpScale& sc, int lane)
{
    LaneState st;
    wave_pass<BF16, ARGMAX, U, false, WITH_T>(st, g, c0, c_hi, stride, do_edges, sc, lane);
    Partial res = wave_merge<BF16, ARGMAX>(st, sc);
    bool finite = (res.S - res.S == 0.0) && (res.T - res.T == 0.0);
    if (!finite) {                                      // wavefront-uniform
        wave_pass<BF16, ARGMAX, U, false, WITH_T, true>(st, g, c0, c_hi, stride, do_edges, sc, lane);
        res = wave_merge<BF16, ARGMAX>(st, sc);
        finite = (res.S - res.S == 0.0) && (res.T - res.T == 0.0);
    }
    if (!finite) {
        wave_pass<BF16, ARGMAX, 2, true>(st, g, c0, c_hi, stride, do_edges, sc, lane);
        res = wave_merge<BF16, ARGMAX>(st, sc);
    }
    return res;
}

// ---- merging partials of one row (accept stage) ------------------------------------------------
struct RowStat { double lse, H; int32_t argmax; };

__device__ __forceinline__ RowStat merge_partials(const Partial* __restrict__ ps, int n)
{
    double bmin = INFINITY;
    bool bad = false;
    for (int i = 0; i < n; ++i) {
        const double S = ps[i].S;
        if (!(S == S)) bad = true;
        if (S > 0.0 && ps[i].bref < bmin) bmin = ps[i].bref;
    }
    double S = 0.0, T = 0.0;
    float vmax = -INFINITY;
    int32_t imax = -1;
    for (int i = 0; i < n; ++i) {
        const Partial q = ps[i];
        if (q.S > 0.0) {
            const double d = bmin - q.bref;             // <= 0
            if (d == 0.0) { S += q.S; T += q.T; }
            else { const double f = exp2_offset_diff(d); S += q.S * f; T += (q.T + d * q.S) * f; }
        }
        if (q.imax >= 0 && (imax < 0 || q.vmax > vmax || (q.vmax == vmax && q.imax < imax))) {
            vmax = q.vmax;
            imax = q.imax;
        }
    }
    RowStat r;
    r.argmax = imax;
    if (bad || !(T == T)) { r.lse = NAN; r.H = NAN; return r; }
    if (!(S > 0.0)) { r.lse = -INFINITY; r.H = NAN; return r; }   // no finite logit in the row
    const double lnS = log(S);
    r.lse = lnS - bmin * kLn2;
    r.H = lnS - kLn2 * (T / S);
    if (r.H < 0.0) r.H = 0.0;                           // rounding on a one-hot row; keeps "tau <= 0 never gates" exact
    return r;
}

}  // namespace hola

namespace hola {

// The same merge done by a whole wavefront: lane i holds partial i (n <= 64), one load per lane.
__device__ __forceinline__ RowStat merge_partials_wave(const Partial* __restrict__ ps, int n, int lane)
{
    Partial q;
    q.bref = 0.0; q.S = 0.0; q.T = 0.0; q.vmax = -INFINITY; q.imax = -1;
    if (lane < n) q = ps[lane];
    const bool bad = __any(!(q.S == q.S));
    const double bmin = wave_min((q.S > 0.0) ? q.bref : (double)INFINITY);
    double S = 0.0, T = 0.0;
    if (q.S > 0.0) {
        const double d = bmin - q.bref;
        if (d == 0.0) { S = q.S; T = q.T; }
        else { const double f = exp2_offset_diff(d); S = q.S * f; T = (q.T + d * q.S) * f; }
    }
    S = wave_sum(S);
    T = wave_sum(T);
    float v = q.vmax;
    int32_t i = q.imax;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const float ov = __shfl_xor(v, m, 64);
        const int32_t oi = __shfl_xor(i, m, 64);
        const bool take = (oi >= 0) && (i < 0 || ov > v || (ov == v && oi < i));
        if (take) { v = ov; i = oi; }
    }
    RowStat r;
    r.argmax = i;
    if (bad || !(T == T)) { r.lse = NAN; r.H = NAN; return r; }
    if (!(S > 0.0)) { r.lse = -INFINITY; r.H = NAN; return r; }
    const double lnS = log(S);
    r.lse = lnS - bmin * kLn2;
    r.H = lnS - kLn2 * (T / S);
    if (r.H < 0.0) r.H = 0.0;                           // rounding on a one-hot row; keeps "tau <= 0 never gates" exact
    return r;
}

// The same merge on a segment of the wavefront: `width` (a power of two >= n) consecutive lanes hold the
// partials of one row, so a wavefront merges 64 / width rows at once.  ps is the row's first partial (null:
// the segment has no row), sl the lane's index inside its segment.  Butterflies with masks below `width` stay
// inside a segment (the whole-wavefront merge adds in another order: the two agree to rounding, not to the bit).
__device__ __forceinline__ RowStat merge_partials_seg(const Partial* __restrict__ ps, int n, int sl, int width)
{
    Partial q;
    q.bref = 0.0; q.S = 0.0; q.T = 0.0; q.vmax = -INFINITY; q.imax = -1;
    if (ps && sl < n) q = ps[sl];
    int badi = !(q.S == q.S) ? 1 : 0;
    double bmin = (q.S > 0.0) ? q.bref : INFINITY;
    for (int m = width >> 1; m >= 1; m >>= 1) {
        bmin = fmin(bmin, __shfl_xor(bmin, m, 64));
        badi |= __shfl_xor(badi, m, 64);
    }
    double S = 0.0, T = 0.0;
    if (q.S > 0.0) {
        const double d = bmin - q.bref;
        if (d == 0.0) { S = q.S; T = q.T; }
        else { const double f = exp2_offset_diff(d); S = q.S * f; T = (q.T + d * q.S) * f; }
    }
    float v = q.vmax;
    int32_t i = q.imax;
    for (int m = width >> 1; m >= 1; m >>= 1) {
        S += __shfl_xor(S, m, 64);
        T += __shfl_xor(T, m, 64);
        const float ov = __shfl_xor(v, m, 64);
        const int32_t oi = __shfl_xor(i, m, 64);
        const bool take = (oi >= 0) && (i < 0 || ov > v || (ov == v && oi < i));
        if (take) { v = ov; i = oi; }
    }
    RowStat r;
    r.argmax = i;
    if (badi || !(T == T)) { r.lse = NAN; r.H = NAN; return r; }
    if (!(S > 0.0)) { r.lse = -INFINITY; r.H = NAN; return r; }
    const double lnS = log(S);
    r.lse = lnS - bmin * kLn2;
    r.H = lnS - kLn2 * (T / S);
    if (r.H < 0.0) r.H = 0.0;
    return r;
}

}  // namespace hola
