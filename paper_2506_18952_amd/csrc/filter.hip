// Keep sets of top-k / top-p filtered rows and the statistics of the kept, renormalised tokens.
//
// Definition (the usual sampling-time truncation; the paper does not filter): order the tokens of a row by
// logit, largest first, equal logits by ascending index; top-k keeps the first k; top-p then keeps the shortest
// prefix of those whose probability, as a fraction of the top-k mass, reaches top_p.  Logits of -inf are never
// kept.  The kept set is described by (theta, idx_cut): x > theta, or x == theta and index <= idx_cut.
//
// This kernel settles any row by itself, one workgroup of 512 threads per row, from nothing but the logits.  It is
// the course of last resort: a filtered call first lets the split-row scan and the per-row decide step of
// filter_scan.hip try, which settle the usual rows several times faster, and runs this kernel only on the rows those
// flagged (or on every row when the scan does not apply: a large top_k, a very large batch, or on request).
// Selection is a radix select over order-preserving integer keys of the logits (16 key bits for bf16, 32 for
// float), 11 bits per level, most significant first.  A level builds a histogram in LDS whose 64-bit entries
// pack an element count and a probability mass in fixed point, so one integer LDS atomic per element serves both
// the by-count (top-k) and the by-mass (top-p) search and the result does not depend on the order in which the
// atomics land.
//
// Usual course, one pass over the row: an exact select on a sample (32 evenly spaced 1 KB blocks) gives a value
// `edge` at or below the cut (top-k: the sample's k-th largest bounds the row's from below; top-p alone: a
// guess); one streaming pass lists every token at or above the edge in LDS (key, index) and, for top-p, sums
// the mass of the others relative to the edge; the guess is then verified (at least k listed; nucleus target
// inside the list's mass) and the cut, the top-k mass, the nucleus, the statistics of the kept tokens (integer
// fixed-point sums, order-independent) and the index of the last kept tie all come from radix selects over the
// list, with masses relative to the row's largest logit.  If the guess fails or the list would exceed 4096
// tokens: two passes (first-level histogram of the whole row, then the list), and for very large keep sets a
// radix select with one pass over the row per level plus a pass for the statistics; those need absolute
// probabilities, whose normaliser the first pass has already summed.
#include "filter_device.h"

namespace hola {

constexpr int kFilterThreads = 512;
constexpr int kFilterWaves = kFilterThreads / 64;
constexpr int kLevelBits = 11;
constexpr int kFilterBins = 1 << kLevelBits;
// Histogram entries.  Whole rows: count in the top 22 bits, mass of absolute probabilities (sum <= 1) in 42 bits,
// unit 2^-40.  Candidate list (at most 4096 tokens): count in 13 bits, mass relative to the reference of the
// row's largest logit (each <= ~1) in 51 bits, unit 2^-38.
constexpr int kMassBits = 42;
constexpr double kMassUnit = 1099511627776.0;                  // 2^40
constexpr uint64_t kMassMask = (1ull << kMassBits) - 1;
constexpr int kFilterCand = 4096;                               // candidate list in LDS (fast path)
constexpr int kMaximaRank = 448;                                // largest rank looked up among the 512 threads' sample maxima

struct FilterShared {
    unsigned long long hist[kFilterBins];
    unsigned long long cand[kFilterCand];                       // (key << 32) | index of the tokens near the top
    unsigned int ncand;
    unsigned int kmax;                                          // largest key met at or above the edge
    unsigned int bad;                                           // a NaN or +inf logit was met
    double red[2 * kFilterWaves];
    unsigned long long wsum[kFilterWaves];
    unsigned int wave_cnt[kFilterWaves];
    unsigned int bin; unsigned long long above;                 // result of a level scan
    int idx_cut; unsigned int sb; unsigned int rank_in_sb;
};

// Calls f(x, index) for every element of chunks [c_lo, c_hi) with a logit above -inf, eight chunks per lane in
// flight.
template <bool BF16, typename F>
__device__ __forceinline__ void for_each_logit(const FilterRow& fr, int64_t c_lo, int64_t c_hi, F f)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int U = 8;
    for (int64_t c0 = c_lo + threadIdx.x; c0 < c_hi; c0 += (int64_t)U * kFilterThreads) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = c0 + (int64_t)u * kFilterThreads;
            v[u] = make_uint4(0, 0, 0, 0);
            if (c < c_hi) v[u] = fr.rowv[c];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = c0 + (int64_t)u * kFilterThreads;
            if (c >= c_hi) continue;
            const int32_t e0 = (int32_t)(c * N) - fr.head;
            const bool edge = (c == 0) || (c == fr.nchunks - 1);
#pragma unroll
            for (int k = 0; k < N; ++k) {
                const int32_t e = e0 + k;
                if (edge && (e < 0 || e >= fr.V)) continue;
                const float x = chunk_elem<BF16>(v[u], k);
                if (x > -INFINITY) f(x, e);
            }
        }
    }
}

// The same over a sample of the row: ns chunks (at most four per thread) taken as blocks of 64 chunks (1 KB)
// that start bstride chunks apart.
template <bool BF16, typename F>
__device__ __forceinline__ void for_each_sample_logit(const FilterRow& fr, int32_t ns, int32_t bstride, F f)
{
    constexpr int N = BF16 ? 8 : 4;
    uint4 v[4];
    int32_t cc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int32_t c = (int32_t)threadIdx.x + u * kFilterThreads;
        cc[u] = (c >> 6) * bstride + (c & 63);
        v[u] = make_uint4(0, 0, 0, 0);
        if (c < ns) v[u] = fr.rowv[cc[u]];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if ((int32_t)threadIdx.x + u * kFilterThreads >= ns) continue;
        const int32_t e0 = cc[u] * N - fr.head;
        const bool edge = (cc[u] == 0) || (cc[u] == (int32_t)fr.nchunks - 1);
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const int32_t e = e0 + k;
            if (edge && (e < 0 || e >= fr.V)) continue;
            const float x = chunk_elem<BF16>(v[u], k);
            if (x > -INFINITY) f(x, e);
        }
    }
}

// One streaming pass that splits the row at a logit value: above(x, index) for x >= edge (edge is finite, so
// -inf never qualifies) and, when BELOW is set, below(s) with s the sum of 2^(exp_arg(x, ref_below)) over some of
// the other logits above -inf.  Non-temporal loads, eight chunks per lane in flight; a chunk without a
// logit at or above the edge costs one compare per element (which also catches NaN) and one call of below.
// Returns true if the thread met a NaN or +inf logit.
template <bool BF16, bool BELOW, typename FA, typename FB>
__device__ __forceinline__ bool split_pass(const FilterRow& fr, float edge, float ref_below, FA above, FB below)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int U = 8;
    bool bad = false;
    for (int64_t c0 = threadIdx.x; c0 < fr.nchunks; c0 += (int64_t)U * kFilterThreads) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = c0 + (int64_t)u * kFilterThreads;
            v[u] = make_uint4(0, 0, 0, 0);
            if (c < fr.nchunks) v[u] = load_stream(fr.rowv + c);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t c = c0 + (int64_t)u * kFilterThreads;
            if (c >= fr.nchunks) continue;
            const bool edge_chunk = (c == 0) || (c == fr.nchunks - 1);
            float x[N];
            bool any = edge_chunk;                              // a logit at or above the edge, a NaN, or a ragged chunk
#pragma unroll
            for (int k = 0; k < N; ++k) { x[k] = chunk_elem<BF16>(v[u], k); any = any || !(x[k] < edge); }
            if (any) {
                const int32_t e0 = (int32_t)(c * N) - fr.head;
#pragma unroll
                for (int k = 0; k < N; ++k) {
                    const int32_t e = e0 + k;
                    if (edge_chunk && (e < 0 || e >= fr.V)) continue;
                    if (!(x[k] < INFINITY)) bad = true;
                    else if (x[k] >= edge) above(x[k], e);
                    else if (BELOW && x[k] > -INFINITY) below(fast_exp2(exp_arg<BF16>(x[k], ref_below, fr.sc)));
                }
            } else if (BELOW) {
                float s = 0.f;
#pragma unroll
                for (int k = 0; k < N; ++k) s += fast_exp2(exp_arg<BF16>(x[k], ref_below, fr.sc));
                if (!(s >= 0.f)) {                              // a -inf logit can turn its exponent into NaN: leave those out
                    s = 0.f;
#pragma unroll
                    for (int k = 0; k < N; ++k)
                        if (x[k] > -INFINITY) s += fast_exp2(exp_arg<BF16>(x[k], ref_below, fr.sc));
                }
                below(s);
            }
        }
    }
    return bad;
}

// A sum of powers of two whose exponents may lie anywhere: value = s * 2^m with m the largest exponent met.
struct RefSum { double m, s; };
__device__ __forceinline__ void refsum_add(RefSum& r, double y)
{
    if (y > r.m) { r.s = r.s * exp2(r.m - y) + 1.0; r.m = y; }
    else r.s += exp2(y - r.m);
}
__device__ __forceinline__ RefSum refsum_merge(const RefSum& a, const RefSum& b)
{
    RefSum r;
    r.m = fmax(a.m, b.m);
    r.s = (r.m == -INFINITY) ? 0.0 : a.s * exp2(a.m - r.m) + b.s * exp2(b.m - r.m);
    return r;
}

// Fixed-point mass of one logit: 2^(exp_arg(x)) * scale in the unit of the whole-row histograms (scale makes it
// the absolute probability) or of the list histograms.
template <bool BF16>
__device__ __forceinline__ uint64_t mass_fixed(const FilterRow& fr, float x)
{
    const double p = (double)fast_exp2(exp_arg<BF16>(x, fr.ref, fr.sc)) * fr.scale;
    return (uint64_t)(p * kMassUnit + 0.5);
}
// Wavefront 0: walk the bins from the top and find the first one at which the running (count or mass), added
// to what lies above the current prefix, reaches `need`.  Leaves the bin and the packed sum of the bins above
// it in shared memory.
template <int MB>
__device__ __forceinline__ void scan_level(FilterShared& sh, int nbins, bool by_mass, uint64_t need)
{
    constexpr uint64_t kMask = (1ull << MB) - 1;
    const int lane = threadIdx.x & 63;
    const int per = nbins >= 64 ? nbins / 64 : 1;
    const int top = nbins - lane * per;                         // this lane covers bins [top - per, top)
    uint64_t mine = 0;
    if (top > 0)
        for (int i = 1; i <= per; ++i) mine += sh.hist[top - i];
    uint64_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = __shfl_up((unsigned long long)incl, d, 64);
        if (lane >= d) incl += o;
    }
    const uint64_t val = by_mass ? (incl & kMask) : (incl >> MB);
    const unsigned long long hit = __ballot(val >= need);
    // If rounding keeps the mass from reaching `need`, settle for the lowest occupied bin.
    const unsigned long long occ = __ballot(mine != 0);
    const int src = hit ? (__ffsll((long long)hit) - 1) : (occ ? 63 - __clzll((long long)occ) : 0);
    if (lane == src) {
        uint64_t run = incl - mine;
        int found = -1, last_occ = -1;
        uint64_t run_last = run;
        for (int i = 1; i <= per && found < 0; ++i) {
            const uint64_t h = sh.hist[top - i];
            const uint64_t nx = run + h;
            if (h != 0) { last_occ = top - i; run_last = run; }
            const uint64_t v = by_mass ? (nx & kMask) : (nx >> MB);
            if (v >= need && h != 0) found = top - i; else run = nx;
        }
        if (found < 0) { found = last_occ < 0 ? 0 : last_occ; run = run_last; }
        sh.bin = (unsigned int)found;
        sh.above = run;
    }
}

struct Cut {
    uint32_t key;          // key of theta
    uint32_t n_ties;       // elements equal to theta
    uint64_t f_theta;      // fixed-point mass of one of them
    uint64_t cnt_above, mass_above;   // strictly above theta
};

// Radix select: by count (the need-th largest element) or by mass (the element at which the cumulative mass,
// largest first, reaches need; with frac > 0 the need is frac times the mass of the whole row, which the first
// level's histogram gives, and is returned in *need_out).  MASS = false leaves the masses out of the
// histograms (count search only).  Every thread returns the same Cut.
template <bool BF16, bool MASS>
__device__ __forceinline__ Cut radix_select(FilterShared& sh, const FilterRow& fr, bool by_mass, uint64_t need,
                                            double frac = 0.0, uint64_t* need_out = nullptr, int32_t sample_n = 0,
                                            int32_t sample_bstride = 64)
{
    constexpr int KB = BF16 ? 16 : 32;
    uint32_t prefix = 0;
    int done = 0;
    uint64_t cnt_above = 0, mass_above = 0;
    Cut cut{};
    while (done < KB) {
        const int nb = (KB - done) < kLevelBits ? (KB - done) : kLevelBits;
        const int shift = KB - done - nb;
        const int nbins = 1 << nb;
        for (int i = threadIdx.x; i < nbins; i += kFilterThreads) sh.hist[i] = 0;
        __syncthreads();
        const int pshift = KB - done;
        auto tally = [&](float x, int32_t) {
            const uint32_t key = order_key<BF16>(x);
            if (done == 0 || (key >> pshift) == prefix) {
                const uint32_t bin = (key >> shift) & (uint32_t)(nbins - 1);
                atomicAdd(&sh.hist[bin], (1ull << kMassBits) + (MASS ? mass_fixed<BF16>(fr, x) : 0ull));
            }
        };
        if (sample_n > 0) for_each_sample_logit<BF16>(fr, sample_n, sample_bstride, tally);   // a sample of the row only
        else for_each_logit<BF16>(fr, 0, fr.nchunks, tally);
        __syncthreads();
        if (MASS && done == 0 && frac > 0.0) {                  // need = frac * mass of the row
            uint64_t s = 0;
            for (int i = threadIdx.x; i < nbins; i += kFilterThreads) s += sh.hist[i];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor((unsigned long long)s, m, 64);
            if ((threadIdx.x & 63) == 0) sh.wsum[threadIdx.x >> 6] = s;
            __syncthreads();
            uint64_t tot = 0;
            for (int i = 0; i < kFilterWaves; ++i) tot += sh.wsum[i];
            need = (uint64_t)(frac * (double)(tot & kMassMask) + 0.5);
            if (need < 1) need = 1;
            if (need_out) *need_out = need;
        }
        const uint64_t rest = by_mass ? (need > mass_above ? need - mass_above : 1) : need - cnt_above;
        if (threadIdx.x < 64) scan_level<kMassBits>(sh, nbins, by_mass, rest);
        __syncthreads();
        const uint32_t bin = sh.bin;
        const uint64_t above = sh.above;
        cnt_above += above >> kMassBits;
        mass_above += above & kMassMask;
        prefix = (prefix << nb) | bin;
        done += nb;
        if (done >= KB) {
            const uint64_t h = sh.hist[bin];
            cut.n_ties = (uint32_t)(h >> kMassBits);
            cut.f_theta = cut.n_ties ? (h & kMassMask) / cut.n_ties : 0;
        }
        __syncthreads();
    }
    cut.key = prefix;
    cut.cnt_above = cnt_above;
    cut.mass_above = mass_above;
    return cut;
}

// The same search over the candidate list in LDS: entries that satisfy pred, ordered by keyfn (KB bits); masses
// in the list unit.
template <bool BF16, bool MASS, typename Pred, typename KeyFn>
__device__ __forceinline__ Cut list_select(FilterShared& sh, const FilterRow& fr, int n, int KB, Pred pred, KeyFn keyfn,
                                           bool by_mass, uint64_t need)
{
    uint32_t prefix = 0;
    int done = 0;
    uint64_t cnt_above = 0, mass_above = 0;
    Cut cut{};
    while (done < KB) {
        const int nb = (KB - done) < kLevelBits ? (KB - done) : kLevelBits;
        const int shift = KB - done - nb;
        const int nbins = 1 << nb;
        for (int i = threadIdx.x; i < nbins; i += kFilterThreads) sh.hist[i] = 0;
        __syncthreads();
        const int pshift = KB - done;
        for (int i = threadIdx.x; i < n; i += kFilterThreads) {
            const unsigned long long ent = sh.cand[i];
            if (!pred(ent)) continue;
            const uint32_t key = keyfn(ent);
            if (done == 0 || (key >> pshift) == prefix) {
                const uint32_t bin = (key >> shift) & (uint32_t)(nbins - 1);
                atomicAdd(&sh.hist[bin], (1ull << kListMassBits) + (MASS ? list_mass_fixed<BF16>(fr, key_to_logit<BF16>(key)) : 0ull));
            }
        }
        __syncthreads();
        const uint64_t rest = by_mass ? (need > mass_above ? need - mass_above : 1) : need - cnt_above;
        if (threadIdx.x < 64) scan_level<kListMassBits>(sh, nbins, by_mass, rest);
        __syncthreads();
        const uint32_t bin = sh.bin;
        const uint64_t above = sh.above;
        cnt_above += above >> kListMassBits;
        mass_above += above & kListMassMask;
        prefix = (prefix << nb) | bin;
        done += nb;
        if (done >= KB) {
            const uint64_t h = sh.hist[bin];
            cut.n_ties = (uint32_t)(h >> kListMassBits);
            cut.f_theta = cut.n_ties ? (h & kListMassMask) / cut.n_ties : 0;
        }
        __syncthreads();
    }
    cut.key = prefix;
    cut.cnt_above = cnt_above;
    cut.mass_above = mass_above;
    return cut;
}

struct FilterParams {
    const void* target; const void* draft;
    int64_t target_ld, draft_ld;
    const int32_t* draft_len;
    float temperature;
    int32_t B, gamma, V;
    int32_t top_k; float top_p;
    RowFilter* filters;
    int32_t* out_keep_count;           // [B, 2 gamma + 1] or null
    const int32_t* flags;              // [B (2 gamma + 1)] or null: only rows flagged 1 are done here
    int32_t skip_draft;                // the draft rows' keep sets are given: only target rows are done here
};

template <bool BF16>
__global__ __launch_bounds__(kFilterThreads) __attribute__((amdgpu_waves_per_eu(6, 6))) void filter_kernel(FilterParams p)
{
    __shared__ FilterShared sh;
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int KB = BF16 ? 16 : 32;
    constexpr int sh0 = KB - kLevelBits;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    if (p.flags && !p.flags[blockIdx.x]) return;                // settled by the scan (uniform exit)
    const int g = p.gamma;
    const int rows_per_seq = 2 * g + 1;
    const int b = blockIdx.x / rows_per_seq, k = blockIdx.x % rows_per_seq;
    const bool is_draft = k < g;
    const int j = is_draft ? k : k - g;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    if (is_draft ? (p.skip_draft || j >= len) : (j > len)) {    // row not needed (uniform exit)
        if (p.out_keep_count && threadIdx.x == 0) p.out_keep_count[blockIdx.x] = -1;
        return;
    }
    const int64_t slot = is_draft ? (int64_t)b * g + j : (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
    const char* row = is_draft ? (const char*)p.draft + ((int64_t)b * g + j) * p.draft_ld * ES
                               : (const char*)p.target + ((int64_t)b * (g + 1) + j) * p.target_ld * ES;

    FilterRow fr;
    const uintptr_t addr = (uintptr_t)row;
    fr.head = (int32_t)((addr & 15) / ES);
    fr.rowv = (const uint4*)(addr & ~(uintptr_t)15);
    fr.V = p.V;
    fr.nchunks = ((int64_t)p.V + fr.head + N - 1) / N;
    fr.sc = make_scale(kLog2e / (double)p.temperature);
    fr.ref = 0.f;
    fr.scale = 1.0;

    const uint64_t kbig = ~0ull;
    const bool want_k = p.top_k > 0 && p.top_k < p.V;
    const bool want_p = p.top_p > 0.f && p.top_p < 1.f;
    bool have_cut = false;
    Cut cut{};
    uint64_t r_keep = 0;                                        // ties at theta that are kept
    float theta = -INFINITY;
    int idx_cut = 0x7fffffff;                                   // every tie is kept
    double S = 0.0, T = 0.0;

    // ---- decisions from a list in LDS that holds every token at or above some value (the cut among them);
    // masses and sums use fr.ref / fr.scale; target_list is the nucleus target in the list unit (top-p alone)
    auto decide_from_list = [&](int n, uint64_t target_list) {
        auto logit_key = [](unsigned long long ent) { return (uint32_t)(ent >> 32); };
        auto every = [](unsigned long long) { return true; };
        uint64_t zk = kbig;
        if (want_k) {
            cut = want_p ? list_select<BF16, true>(sh, fr, n, KB, every, logit_key, false, (uint64_t)p.top_k)
                         : list_select<BF16, false>(sh, fr, n, KB, every, logit_key, false, (uint64_t)p.top_k);
            const uint64_t total = cut.cnt_above + cut.n_ties;
            r_keep = total >= (uint64_t)p.top_k ? (uint64_t)p.top_k - cut.cnt_above : cut.n_ties;
            zk = cut.mass_above + r_keep * cut.f_theta;
            have_cut = true;
        }
        if (want_p) {
            uint64_t target = target_list;
            if (zk != kbig) {
                target = (uint64_t)((double)p.top_p * (double)zk + 0.5);
                if (target < 1) target = 1;
            }
            const Cut cp = list_select<BF16, true>(sh, fr, n, KB, every, logit_key, true, target);
            uint64_t r = 1;
            if (cp.f_theta > 0 && target > cp.mass_above) r = (target - cp.mass_above + cp.f_theta - 1) / cp.f_theta;
            if (r < 1) r = 1;
            if (r > cp.n_ties) r = cp.n_ties;
            if (have_cut && cp.key == cut.key && r > r_keep) r = r_keep;   // never beyond the top-k cut
            cut = cp;
            r_keep = r;
            have_cut = true;
        }
        theta = key_to_logit<BF16>(cut.key);
        // sums over the kept tokens above theta, in fixed point so that the order of the list does not matter
        uint32_t kmax = 0;
        for (int i = tid; i < n; i += kFilterThreads) { const uint32_t kk = (uint32_t)(sh.cand[i] >> 32); kmax = kk > kmax ? kk : kmax; }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { const uint32_t o = __shfl_xor(kmax, m, 64); kmax = o > kmax ? o : kmax; }
        if (lane == 0) sh.wave_cnt[wave] = kmax;
        __syncthreads();
        for (int i = 0; i < kFilterWaves; ++i) kmax = sh.wave_cnt[i] > kmax ? sh.wave_cnt[i] : kmax;
        const float y_top = exp_arg<BF16>(key_to_logit<BF16>(kmax), fr.ref, fr.sc);
        int sft = (int)floorf(-y_top);
        sft = sft < -60 ? -60 : (sft > 900 ? 900 : sft);
        const double up = ldexp(1.0, sft);
        unsigned long long Sfix = 0;
        long long Tfix = 0;
        for (int i = tid; i < n; i += kFilterThreads) {
            const uint32_t kk = (uint32_t)(sh.cand[i] >> 32);
            if (kk > cut.key) {
                const float y = exp_arg<BF16>(key_to_logit<BF16>(kk), fr.ref, fr.sc);
                const double ex = (double)fast_exp2(y) * up;
                Sfix += (unsigned long long)(ex * 562949953421312.0 + 0.5);            // 2^49
                Tfix += (long long)rint((double)y * ex * 2199023255552.0);            // 2^41
            }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            Sfix += __shfl_xor(Sfix, m, 64);
            Tfix += (long long)__shfl_xor((unsigned long long)Tfix, m, 64);
        }
        __syncthreads();
        if (lane == 0) { sh.wsum[wave] = Sfix; sh.red[wave] = __longlong_as_double(Tfix); }
        __syncthreads();
        unsigned long long Sall = 0;
        long long Tall = 0;
        for (int i = 0; i < kFilterWaves; ++i) { Sall += sh.wsum[i]; Tall += __double_as_longlong(sh.red[i]); }
        S = ldexp((double)Sall, -49 - sft);
        T = ldexp((double)Tall, -41 - sft);
        if (r_keep > 0) {
            const float y = exp_arg<BF16>(theta, fr.ref, fr.sc);
            const double ex = (double)fast_exp2(y);
            S += (double)r_keep * ex;
            T += (double)r_keep * ((double)y * ex);
        }
        if (r_keep < cut.n_ties) {
            // the r-th smallest index among the ties: largest-first select on the complemented index
            const uint32_t tkey = cut.key;
            auto is_tie = [tkey](unsigned long long ent) { return (uint32_t)(ent >> 32) == tkey; };
            auto inv_index = [](unsigned long long ent) { return 0x3fffffu - (uint32_t)(ent & 0xffffffffu); };
            __syncthreads();
            const Cut ci = list_select<BF16, false>(sh, fr, n, 22, is_tie, inv_index, false, r_keep);
            idx_cut = (int)(0x3fffffu - ci.key);
        }
    };

    // ---- sample: a value at or below the cut.  A row that fits the list needs none: everything is listed.
    const int64_t row_elems = fr.nchunks * N;
    const bool tiny = row_elems <= (int64_t)(kFilterCand * 3 / 4);
    const int64_t sample_chunks = fr.nchunks < 4 * kFilterThreads ? fr.nchunks : 4 * kFilterThreads;
    int64_t sample_step = 64;                                   // 32 evenly spaced blocks of 64 chunks
    if (fr.nchunks > sample_chunks) sample_step = (fr.nchunks - 64) / (sample_chunks / 64 - 1) / 8 * 8;
    bool sample_ok = false;                                     // x_low is at or below the cut (top-k) / a guess (top-p)
    bool try_list = tiny;                                       // the list is expected to hold the cut
    float x_low = 0.f;
    if (!tiny) {
        const float per_thread = (float)(sample_chunks * N) / (float)kFilterThreads;   // sample logits per thread
        uint64_t need_g = (uint64_t)p.top_k;
        if (!want_k) {
            // top-p alone: the rank among the threads' maxima at which a list of ~3/8 of its capacity is expected
            const float q = fminf(1.f, (float)(kFilterCand * 3 / 8) / (float)row_elems);
            need_g = (uint64_t)((float)kFilterThreads * (1.f - powf(1.f - q, per_thread)) + 0.5f);
            need_g = need_g < 1 ? 1 : (need_g > (uint64_t)kMaximaRank ? (uint64_t)kMaximaRank : need_g);
        }
        if (need_g <= (uint64_t)kMaximaRank) {
            // each thread's largest sample logit: the need_g-th largest of these distinct tokens bounds the row's
            // need_g-th largest from below, and 512 values select much faster than the whole sample
            uint32_t km = 0;                                    // no finite logit: key 0 (never a finite logit's key)
            for_each_sample_logit<BF16>(fr, (int32_t)sample_chunks, (int32_t)sample_step, [&](float x, int32_t) {
                const uint32_t key = order_key<BF16>(x);
                km = key > km ? key : km;
            });
            sh.cand[tid] = ((unsigned long long)km << 32) | (uint32_t)tid;
            __syncthreads();
            auto logit_key = [](unsigned long long ent) { return (uint32_t)(ent >> 32); };
            auto seen = [](unsigned long long ent) { return (ent >> 32) != 0; };
            const Cut cs = list_select<BF16, false>(sh, fr, kFilterThreads, KB, seen, logit_key, false, need_g);
            const uint64_t got = cs.cnt_above + cs.n_ties;      // maxima at or above that value
            sample_ok = got >= need_g;
            if (sample_ok) {
                x_low = key_to_logit<BF16>(cs.key);
                // fraction of the row expected at or above x_low, from the fraction of threads that met such a logit
                const float frac = (float)got / (float)kFilterThreads;
                const float q = frac < 1.f ? 1.f - powf(1.f - frac, 1.f / per_thread) : 1.f;
                try_list = q * (float)row_elems <= (float)(kFilterCand * 3 / 4);
            }
        } else {
            // a large k: exact select on the whole sample
            const Cut cs = radix_select<BF16, false>(sh, fr, false, need_g, 0.0, nullptr, (int32_t)sample_chunks, (int32_t)sample_step);
            const uint64_t samp = cs.cnt_above + cs.n_ties;     // sample logits at or above that value
            sample_ok = samp >= need_g;                         // else the sample has fewer finite logits than asked
            if (sample_ok) {
                x_low = key_to_logit<BF16>(cs.key);
                try_list = samp * (uint64_t)fr.nchunks <= (uint64_t)(kFilterCand * 3 / 4) * (uint64_t)sample_chunks;
            }
        }
    }
    // edge: logits below it are not among the k largest of the row (top-k); without a usable sample every finite
    // logit is "at or above the edge".  x_low is also the reference of the masses below the edge.
    const float edge_v = sample_ok ? x_low : -3.4028234e38f;
    const bool first_pass = (want_p && !want_k) || try_list;    // with top-k no mass outside the list is needed: skip a hopeless list

    // ---- first pass: list at or above the edge, largest key, and (top-p) the mass of everything else
    const float ref_e = ref_for<BF16>(x_low, fr.sc);
    const double beta_e = ref_offset<BF16>(ref_e, fr.sc);
    if (tid == 0) { sh.ncand = 0; sh.kmax = 0; sh.bad = 0; }
    __syncthreads();
    double others = 0.0;                                        // mass, relative to the edge reference, outside the list
    unsigned int n_all = 0;
    bool solved = false, need_norm = false;
    if (first_pass) {
        uint32_t kmax_t = 0;                                    // largest key this thread met at or above the edge
        auto to_list = [&](float x, int32_t e) {
            const uint32_t key = order_key<BF16>(x);
            kmax_t = key > kmax_t ? key : kmax_t;
            const unsigned int slt = atomicAdd(&sh.ncand, 1u);
            if (slt < (unsigned int)kFilterCand) sh.cand[slt] = ((unsigned long long)key << 32) | (uint32_t)e;
        };
        bool bad;
        if (want_p && !want_k) bad = split_pass<BF16, true>(fr, edge_v, ref_e, to_list, [&](float s) { others += (double)s; });
        else bad = split_pass<BF16, false>(fr, edge_v, ref_e, to_list, [](float) {});   // with top-k the masses come from the list
        if (bad) sh.bad = 1;
        others = wave_sum(others);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { const uint32_t o = __shfl_xor(kmax_t, m, 64); kmax_t = o > kmax_t ? o : kmax_t; }
        if (lane == 0) { sh.red[wave] = others; sh.wave_cnt[wave] = kmax_t; }
        __syncthreads();
        others = 0.0;
        for (int i = 0; i < kFilterWaves; ++i) { others += sh.red[i]; kmax_t = sh.wave_cnt[i] > kmax_t ? sh.wave_cnt[i] : kmax_t; }
        if (tid == 0) sh.kmax = kmax_t;
        n_all = sh.ncand;
    }
    const bool bad_row = first_pass && sh.bad != 0;
    RowFilter out;
    out.lse = NAN; out.H = NAN; out.theta = INFINITY; out.idx_cut = -1; out.n_keep = 0; out.pad = 0;
    if (bad_row || (first_pass && n_all == 0)) {                // NaN / +inf logits, or no finite logit: nothing is kept
        if (!bad_row) out.lse = -INFINITY;
        if (tid == 0) { p.filters[slot] = out; if (p.out_keep_count) p.out_keep_count[blockIdx.x] = 0; }
        return;
    }
    __syncthreads();

    if (first_pass) {
        const bool complete = n_all <= (unsigned int)kFilterCand;   // every logit at or above the edge is listed
        const int n = (int)(complete ? n_all : (unsigned int)kFilterCand);
        // from here on masses are taken against the reference of the row's largest logit
        fr.ref = ref_for<BF16>(key_to_logit<BF16>(sh.kmax), fr.sc);
        fr.scale = 1.0;
        const double beta_m = ref_offset<BF16>(fr.ref, fr.sc);
        bool ok = complete && try_list;
        uint64_t target_list = 0;
        // fewer than k listed: the guess was wrong, unless the list holds every finite logit of the row
        if (want_k) ok = ok && (n_all >= (unsigned int)p.top_k || !sample_ok);
        // mass of the list (top-p): in the list unit for the nucleus target, and in double for the normaliser
        double list_m = 0.0;
        unsigned long long lm = 0;
        if (want_p && complete) {
            for (int i = tid; i < n; i += kFilterThreads) {
                const float x = key_to_logit<BF16>((uint32_t)(sh.cand[i] >> 32));
                lm += list_mass_fixed<BF16>(fr, x);
                list_m += exp2((double)x * fr.sc.cstar + beta_m);   // at most ~1 each
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) lm += __shfl_xor(lm, m, 64);
            list_m = wave_sum(list_m);
            if (lane == 0) { sh.wsum[wave] = lm; sh.red[wave] = list_m; }
            __syncthreads();
            lm = 0; list_m = 0.0;
            for (int i = 0; i < kFilterWaves; ++i) { lm += sh.wsum[i]; list_m += sh.red[i]; }
            __syncthreads();
            if (!want_k) {
                const double others_list = others * exp2(beta_m - beta_e) * kListMassUnit;   // the rest of the row, list unit
                target_list = (uint64_t)((double)p.top_p * ((double)lm + others_list) + 0.5);
                if (target_list < 1) target_list = 1;
                ok = ok && lm >= target_list;
            }
        }
        if (ok) {
            decide_from_list(n, target_list);
            solved = true;
        } else if (want_p && !want_k && complete) {
            // absolute probabilities for the whole-row histograms: the normaliser is what this pass summed
            const double L = log2(list_m + others * exp2(beta_m - beta_e)) - beta_m;   // log2-sum-exp of the row
            fr.ref = ref_for_norm<BF16>(L, fr.sc);
            fr.scale = exp2(-L - ref_offset<BF16>(fr.ref, fr.sc));
        } else if (want_p) {
            need_norm = true;                                   // a list that overflowed did not see every mass
        }
    } else {
        // a list that would not fit: the reference is set once the next pass has met the largest logit
        fr.ref = ref_for<BF16>(x_low, fr.sc);
        fr.scale = 1.0;
        need_norm = want_p;
    }
    if (need_norm) {
        // the whole-row histograms need absolute probabilities, so one pass sums the row's normaliser: logits
        // below the edge against the edge reference, the others (which may lie far above it) against their own
        // running maximum
        double lo_sum = 0.0;
        RefSum hi_sum{-INFINITY, 0.0};
        auto hi = [&](float x, int32_t) { refsum_add(hi_sum, (double)x * fr.sc.cstar); };
        auto lo = [&](float s) { lo_sum += (double)s; };
        const bool bad = split_pass<BF16, true>(fr, edge_v, ref_e, hi, lo);
        if (bad) sh.bad = 1;
        lo_sum = wave_sum(lo_sum);
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) {
            RefSum o;
            o.m = __shfl_xor(hi_sum.m, m, 64);
            o.s = __shfl_xor(hi_sum.s, m, 64);
            hi_sum = refsum_merge(hi_sum, o);
        }
        __syncthreads();
        if (lane == 0) { sh.red[wave] = lo_sum; sh.red[kFilterWaves + wave] = hi_sum.m; sh.wsum[wave] = (unsigned long long)__double_as_longlong(hi_sum.s); }
        __syncthreads();
        lo_sum = 0.0;
        hi_sum.m = -INFINITY; hi_sum.s = 0.0;
        for (int i = 0; i < kFilterWaves; ++i) {
            lo_sum += sh.red[i];
            RefSum o;
            o.m = sh.red[kFilterWaves + i];
            o.s = __longlong_as_double((long long)sh.wsum[i]);
            hi_sum = refsum_merge(hi_sum, o);
        }
        if (sh.bad || !(lo_sum > 0.0 || hi_sum.s > 0.0)) {
            if (!sh.bad) out.lse = -INFINITY;
            if (tid == 0) { p.filters[slot] = out; if (p.out_keep_count) p.out_keep_count[blockIdx.x] = 0; }
            return;
        }
        // log2-sum-exp of the row from the two parts
        const double la = hi_sum.s > 0.0 ? hi_sum.m + log2(hi_sum.s) : -INFINITY;
        const double lb = lo_sum > 0.0 ? log2(lo_sum) - beta_e : -INFINITY;
        const double lmax = fmax(la, lb), lmin = fmin(la, lb);
        const double L = lmax + log2(1.0 + exp2(lmin - lmax));
        fr.ref = ref_for_norm<BF16>(L, fr.sc);
        fr.scale = exp2(-L - ref_offset<BF16>(fr.ref, fr.sc));
        __syncthreads();
    }

    if (!solved) {
        // ---- pass A: first-level histogram of the whole row (top-k: of the logits at or above the edge only);
        // the bin that holds the cut, and how many tokens lie at or above it
        for (int i = tid; i < kFilterBins; i += kFilterThreads) sh.hist[i] = 0;
        __syncthreads();
        if (want_p && !want_k)
            for_each_logit<BF16>(fr, 0, fr.nchunks, [&](float x, int32_t) {
                atomicAdd(&sh.hist[order_key<BF16>(x) >> sh0], (1ull << kMassBits) + mass_fixed<BF16>(fr, x));
            });
        else if (want_p)                                        // logits below the sample's k-th largest cannot matter
            split_pass<BF16, false>(fr, edge_v, ref_e, [&](float x, int32_t) {
                atomicAdd(&sh.hist[order_key<BF16>(x) >> sh0], (1ull << kMassBits) + mass_fixed<BF16>(fr, x)); }, [](float) {});
        else {
            uint32_t kmax_t = 0;
            const bool bad = split_pass<BF16, false>(fr, edge_v, ref_e, [&](float x, int32_t) {
                const uint32_t key = order_key<BF16>(x);
                kmax_t = key > kmax_t ? key : kmax_t;
                atomicAdd(&sh.hist[key >> sh0], 1ull << kMassBits); }, [](float) {});
            if (bad) sh.bad = 1;
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) { const uint32_t o = __shfl_xor(kmax_t, m, 64); kmax_t = o > kmax_t ? o : kmax_t; }
            if (lane == 0) atomicMax(&sh.kmax, kmax_t);         // one atomic per wavefront
        }
        __syncthreads();
        if (!first_pass && !want_p) {
            if (sh.bad) {                                       // NaN / +inf logits: nothing is kept
                if (tid == 0) { p.filters[slot] = out; if (p.out_keep_count) p.out_keep_count[blockIdx.x] = 0; }
                return;
            }
            fr.ref = ref_for<BF16>(key_to_logit<BF16>(sh.kmax), fr.sc);   // the sums are taken against the largest logit
        }
        uint64_t row_total = 0;                                 // packed count and mass of what was tallied
        {
            uint64_t sacc = 0;
            for (int i = tid; i < kFilterBins; i += kFilterThreads) sacc += sh.hist[i];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) sacc += __shfl_xor((unsigned long long)sacc, m, 64);
            if (lane == 0) sh.wsum[wave] = sacc;
            __syncthreads();
            for (int i = 0; i < kFilterWaves; ++i) row_total += sh.wsum[i];
        }
        uint64_t target_p = 0;
        if (want_p && !want_k) {
            target_p = (uint64_t)((double)p.top_p * (double)(row_total & kMassMask) + 0.5);
            if (target_p < 1) target_p = 1;
        }
        if (wave == 0) scan_level<kMassBits>(sh, kFilterBins, !want_k, want_k ? (uint64_t)p.top_k : target_p);
        __syncthreads();
        const uint32_t bin0 = sh.bin;
        const uint64_t n_cand = (sh.above >> kMassBits) + (sh.hist[bin0] >> kMassBits);
        const bool fast = n_cand <= (uint64_t)kFilterCand;
        __syncthreads();

        if (fast) {
            // ---- pass B: the tokens at or above that bin go to the list; everything else is decided there
            if (tid == 0) sh.ncand = 0;
            __syncthreads();
            for_each_logit<BF16>(fr, 0, fr.nchunks, [&](float x, int32_t e) {
                const uint32_t key = order_key<BF16>(x);
                if ((key >> sh0) >= bin0) {
                    const unsigned int slt = atomicAdd(&sh.ncand, 1u);
                    if (slt < (unsigned int)kFilterCand) sh.cand[slt] = ((unsigned long long)key << 32) | (uint32_t)e;
                }
            });
            __syncthreads();
            // the whole-row target (unit 2^-40 of absolute probabilities) in the list unit (2^-38, same scale)
            decide_from_list((int)(sh.ncand < (unsigned int)kFilterCand ? sh.ncand : (unsigned int)kFilterCand), (target_p + 2) / 4);
        } else {
            // ---- top-k: the k-th largest logit
            uint64_t zk = kbig;                                         // fixed-point mass of the top-k set (kbig: whole row)
            if (p.top_k > 0 && p.top_k < p.V) {
                cut = want_p ? radix_select<BF16, true>(sh, fr, false, (uint64_t)p.top_k)
                             : radix_select<BF16, false>(sh, fr, false, (uint64_t)p.top_k);
                // fewer than k finite logits: everything finite is kept (the scan then settled on the lowest key)
                const uint64_t total = cut.cnt_above + cut.n_ties;
                if (total >= (uint64_t)p.top_k) {
                    r_keep = (uint64_t)p.top_k - cut.cnt_above;
                } else {
                    r_keep = cut.n_ties;
                }
                zk = cut.mass_above + r_keep * cut.f_theta;
                have_cut = true;
            }
            // ---- top-p: the shortest prefix whose mass reaches top_p of the top-k mass
            if (want_p) {
                uint64_t target = 0;
                Cut cp;
                if (zk == kbig) {
                    cp = radix_select<BF16, true>(sh, fr, true, 0, (double)p.top_p, &target);   // of the whole row's mass
                } else {
                    target = (uint64_t)((double)p.top_p * (double)zk + 0.5);
                    if (target < 1) target = 1;
                    cp = radix_select<BF16, true>(sh, fr, true, target);
                }
                uint64_t r = 1;
                if (cp.f_theta > 0 && target > cp.mass_above) r = (target - cp.mass_above + cp.f_theta - 1) / cp.f_theta;
                if (r < 1) r = 1;
                if (r > cp.n_ties) r = cp.n_ties;
                if (have_cut && cp.key == cut.key && r > r_keep) r = r_keep;   // never beyond the top-k cut
                cut = cp;
                r_keep = r;
                have_cut = true;
            }

            // ---- statistics of the kept tokens; position of the last kept tie
            theta = have_cut ? key_to_logit<BF16>(cut.key) : -INFINITY;
            const bool partial_ties = have_cut && r_keep < cut.n_ties;
            const int64_t cps = ((fr.nchunks + kFilterBins - 1) / kFilterBins + kFilterThreads - 1) / kFilterThreads * kFilterThreads;
            unsigned int* sbties = (unsigned int*)sh.hist;
            if (partial_ties) {
                for (int i = tid; i < kFilterBins; i += kFilterThreads) sbties[i] = 0;
                __syncthreads();
            }
            double Sd = 0.0, Td = 0.0;
            {
                constexpr int U = 4;
                for (int64_t c0 = tid; c0 < fr.nchunks; c0 += (int64_t)U * kFilterThreads) {
                    uint4 v[U];
        #pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t c = c0 + (int64_t)u * kFilterThreads;
                        v[u] = make_uint4(0, 0, 0, 0);
                        if (c < fr.nchunks) v[u] = fr.rowv[c];
                    }
        #pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t c = c0 + (int64_t)u * kFilterThreads;
                        if (c >= fr.nchunks) continue;
                        const int32_t e0 = (int32_t)(c * N) - fr.head;
                        const bool edge = (c == 0) || (c == fr.nchunks - 1);
                        float s = 0.f, t = 0.f;
                        unsigned int ties = 0;
        #pragma unroll
                        for (int kk = 0; kk < N; ++kk) {
                            const int32_t e = e0 + kk;
                            const bool valid = !edge || (e >= 0 && e < fr.V);
                            const float x = chunk_elem<BF16>(v[u], kk);
                            if (valid && x > theta) {
                                const float y = exp_arg<BF16>(x, fr.ref, fr.sc);
                                const float ex = fast_exp2(y);
                                s += ex;
                                t = __builtin_fmaf(y, ex, t);
                            }
                            if (valid && x == theta) ++ties;
                        }
                        Sd += (double)s;
                        Td += (double)t;
                        if (partial_ties && ties) atomicAdd(&sbties[c / cps], ties);
                    }
                }
            }
            Sd = wave_sum(Sd);
            Td = wave_sum(Td);
            if (lane == 0) { sh.red[2 * wave] = Sd; sh.red[2 * wave + 1] = Td; }
            __syncthreads();
            for (int i = 0; i < kFilterWaves; ++i) { S += sh.red[2 * i]; T += sh.red[2 * i + 1]; }
            if (have_cut && r_keep > 0) {                               // the kept ties, all with the same term
                const float y = exp_arg<BF16>(theta, fr.ref, fr.sc);
                const double ex = (double)fast_exp2(y);
                S += (double)r_keep * ex;
                T += (double)r_keep * ((double)y * ex);
            }

            if (partial_ties) {
                // super-block that holds the r-th tie (ascending index), then the element inside it
                if (wave == 0) {
                    const int nsb = (int)((fr.nchunks + cps - 1) / cps);
                    const int per = (nsb + 63) / 64;
                    unsigned int mine = 0;
                    for (int i = 0; i < per; ++i) { const int q = lane * per + i; if (q < nsb) mine += sbties[q]; }
                    unsigned int incl = mine;
        #pragma unroll
                    for (int d = 1; d < 64; d <<= 1) { const unsigned int o = __shfl_up(incl, d, 64); if (lane >= d) incl += o; }
                    const unsigned long long hit = __ballot((uint64_t)incl >= r_keep);
                    const int src = hit ? (__ffsll((long long)hit) - 1) : 63;
                    if (lane == src) {
                        unsigned int run = incl - mine;
                        int found = nsb - 1;
                        for (int i = 0; i < per; ++i) {
                            const int q = lane * per + i;
                            if (q >= nsb) break;
                            if ((uint64_t)run + sbties[q] >= r_keep) { found = q; break; }
                            run += sbties[q];
                        }
                        sh.sb = (unsigned int)found;
                        sh.rank_in_sb = (unsigned int)(r_keep - run);
                    }
                }
                if (tid == 0) sh.idx_cut = fr.V - 1;
                __syncthreads();
                const int64_t c_lo = (int64_t)sh.sb * cps;
                const int64_t c_hi = c_lo + cps < fr.nchunks ? c_lo + cps : fr.nchunks;
                unsigned int want = sh.rank_in_sb;                      // 1-based rank inside the super-block
                bool finished = false;
                for (int64_t base = c_lo; base < c_hi; base += kFilterThreads) {   // uniform trip count
                    const int64_t c = base + tid;
                    unsigned int ties = 0;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    int32_t e0 = 0;
                    if (c < c_hi) {
                        v = fr.rowv[c];
                        e0 = (int32_t)(c * N) - fr.head;
        #pragma unroll
                        for (int kk = 0; kk < N; ++kk) {
                            const int32_t e = e0 + kk;
                            if (e >= 0 && e < fr.V && chunk_elem<BF16>(v, kk) == theta) ++ties;
                        }
                    }
                    unsigned int incl = ties;
        #pragma unroll
                    for (int d = 1; d < 64; d <<= 1) { const unsigned int o = __shfl_up(incl, d, 64); if (lane >= d) incl += o; }
                    if (lane == 63) sh.wave_cnt[wave] = incl;
                    __syncthreads();
                    unsigned int before = 0, total = 0;
                    for (int i = 0; i < kFilterWaves; ++i) { const unsigned int wc = sh.wave_cnt[i]; if (i < wave) before += wc; total += wc; }
                    const unsigned int excl = before + incl - ties;
                    if (!finished && want > excl && want <= excl + ties) {
                        unsigned int seen = excl;
        #pragma unroll
                        for (int kk = 0; kk < N; ++kk) {
                            const int32_t e = e0 + kk;
                            if (e >= 0 && e < fr.V && chunk_elem<BF16>(v, kk) == theta) {
                                ++seen;
                                if (seen == want) sh.idx_cut = e;
                            }
                        }
                    }
                    if (want <= total) finished = true; else want -= total;
                    __syncthreads();
                    if (finished) break;                                // uniform: every thread saw the same totals
                }
                idx_cut = sh.idx_cut;
            }
        }
    }

    out.theta = theta;
    out.idx_cut = idx_cut;
    out.n_keep = have_cut ? (int32_t)(cut.cnt_above + r_keep) : -1;   // -1: every finite logit
    if (S > 0.0) {
        const double lnS = log(S);
        out.lse = lnS - ref_offset<BF16>(fr.ref, fr.sc) * kLn2;   // the sums were taken against fr.ref
        out.H = lnS - kLn2 * (T / S);
        if (out.H < 0.0) out.H = 0.0;                           // a single kept token: exactly zero
    } else {
        out.lse = -INFINITY;
        out.H = NAN;
    }
    if (tid == 0) { p.filters[slot] = out; if (p.out_keep_count) p.out_keep_count[blockIdx.x] = out.n_keep; }
}

hipError_t launch_filter(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                         const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                         int32_t top_k, float top_p, RowFilter* filters, int32_t* out_keep_count, const int32_t* flags,
                         int32_t skip_draft, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    FilterParams p{};
    p.target = target; p.draft = draft; p.target_ld = target_ld; p.draft_ld = draft_ld; p.draft_len = draft_len;
    p.temperature = temperature; p.B = B; p.gamma = gamma; p.V = V; p.top_k = top_k; p.top_p = top_p;
    p.filters = filters; p.out_keep_count = out_keep_count; p.flags = flags; p.skip_draft = skip_draft;
    const int64_t nblk = (int64_t)B * (2 * gamma + 1);
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((filter_kernel<true>), dim3((unsigned)nblk), dim3(kFilterThreads), 0, s, p);
    else hipLaunchKernelGGL((filter_kernel<false>), dim3((unsigned)nblk), dim3(kFilterThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace hola
