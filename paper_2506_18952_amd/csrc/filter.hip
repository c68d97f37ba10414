// Keep sets of top-k / top-p filtered rows and the statistics of the kept, renormalised tokens.
//
// Definition (the usual sampling-time truncation; the paper does not filter): order the tokens of a row by
// logit, largest first, equal logits by ascending index; top-k keeps the first k; top-p then keeps the shortest
// prefix of those whose probability, as a fraction of the top-k mass, reaches top_p.  Logits of -inf are never
// kept.  The kept set is described by (theta, idx_cut): x > theta, or x == theta and index <= idx_cut.
//
// One workgroup of 512 threads per row.  Selection is a radix select over order-preserving integer keys of the
// logits (16 key bits for bf16, 32 for float), 11 bits per level, most significant first.  A level builds a
// histogram in LDS over the elements that match the key prefix found so far; an entry packs the element count
// (22 bits) and the probability mass in fixed point (42 bits, unit 2^-40), so one 64-bit LDS atomic per element
// serves both the by-count (top-k) and the by-mass (top-p) search, and integer addition keeps the result
// independent of the order in which the atomics land.  Probabilities use the row's unfiltered normaliser, merged
// from the partials of the split-row statistics kernel.  The first pass over a row comes from HBM, the others
// find it in L2.  A last pass sums S = sum 2^y and T = sum y 2^y over x > theta (ties at theta are added in
// closed form) and, when the cut falls inside a run of equal logits, locates the index of the last kept one.
#include "sampler_device.h"

namespace hola {

constexpr int kFilterThreads = 512;
constexpr int kFilterWaves = kFilterThreads / 64;
constexpr int kLevelBits = 11;
constexpr int kFilterBins = 1 << kLevelBits;
constexpr int kMassBits = 42;
constexpr uint64_t kMassMask = (1ull << kMassBits) - 1;
constexpr double kMassUnit = 1099511627776.0;                  // 2^40

struct FilterShared {
    unsigned long long hist[kFilterBins];
    double red[2 * kFilterWaves];
    unsigned long long wsum[kFilterWaves];
    unsigned int wave_cnt[kFilterWaves];
    double lse;
    unsigned int bin; unsigned long long above;                 // result of a level scan
    int idx_cut; unsigned int sb; unsigned int rank_in_sb;
};

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

// Calls f(x, index) for every element of the row with a logit above -inf, four chunks per lane in flight.
template <bool BF16, typename F>
__device__ __forceinline__ void for_each_logit(const FilterRow& fr, int64_t c_lo, int64_t c_hi, F f)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int U = 4;
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

template <bool BF16>
__device__ __forceinline__ uint64_t mass_fixed(const FilterRow& fr, float x)
{
    const double p = (double)fast_exp2(exp_arg<BF16>(x, fr.ref, fr.sc)) * fr.scale;
    return (uint64_t)(p * kMassUnit + 0.5);
}

// Wavefront 0: walk the bins from the top and find the first one at which the running (count or mass), added
// to what lies above the current prefix, reaches `need`.  Leaves the bin and the packed sum of the bins above
// it in shared memory.
__device__ __forceinline__ void scan_level(FilterShared& sh, int nbins, bool by_mass, uint64_t need)
{
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
    const uint64_t val = by_mass ? (incl & kMassMask) : (incl >> kMassBits);
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
            const uint64_t v = by_mass ? (nx & kMassMask) : (nx >> kMassBits);
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
// largest first, reaches need).  Every thread returns the same Cut.
template <bool BF16>
__device__ __forceinline__ Cut radix_select(FilterShared& sh, const FilterRow& fr, bool by_mass, uint64_t need)
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
        for_each_logit<BF16>(fr, 0, fr.nchunks, [&](float x, int32_t) {
            const uint32_t key = order_key<BF16>(x);
            if (done == 0 || (key >> pshift) == prefix) {
                const uint32_t bin = (key >> shift) & (uint32_t)(nbins - 1);
                atomicAdd(&sh.hist[bin], (1ull << kMassBits) + mass_fixed<BF16>(fr, x));
            }
        });
        __syncthreads();
        const uint64_t rest = by_mass ? (need > mass_above ? need - mass_above : 1) : need - cnt_above;
        if (threadIdx.x < 64) scan_level(sh, nbins, by_mass, rest);
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

struct FilterParams {
    const void* target; const void* draft;
    int64_t target_ld, draft_ld;
    const int32_t* draft_len;
    float temperature;
    int32_t B, gamma, V;
    int32_t top_k; float top_p;
    const Partial* partials; int32_t nparts;
    RowFilter* filters;
    int32_t* out_keep_count;           // [B, 2 gamma + 1] or null
};

template <bool BF16>
__global__ __launch_bounds__(kFilterThreads) void filter_kernel(FilterParams p)
{
    __shared__ FilterShared sh;
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = p.gamma;
    const int rows_per_seq = 2 * g + 1;
    const int b = blockIdx.x / rows_per_seq, k = blockIdx.x % rows_per_seq;
    const bool is_draft = k < g;
    const int j = is_draft ? k : k - g;
    int len = p.draft_len ? p.draft_len[b] : g;
    len = len < 0 ? 0 : (len > g ? g : len);
    if (is_draft ? (j >= len) : (j > len)) {                    // row not needed (uniform exit)
        if (p.out_keep_count && threadIdx.x == 0) p.out_keep_count[blockIdx.x] = -1;
        return;
    }
    const int64_t slot = is_draft ? (int64_t)b * g + j : (int64_t)p.B * g + (int64_t)b * (g + 1) + j;
    const char* row = is_draft ? (const char*)p.draft + ((int64_t)b * g + j) * p.draft_ld * ES
                               : (const char*)p.target + ((int64_t)b * (g + 1) + j) * p.target_ld * ES;

    if (wave == 0) {
        const RowStat rs = merge_partials_wave(p.partials + slot * p.nparts, p.nparts, lane);
        if (lane == 0) sh.lse = rs.lse;
    }
    __syncthreads();
    const double lse = sh.lse;
    RowFilter out;
    out.lse = lse; out.H = NAN; out.theta = INFINITY; out.idx_cut = -1; out.n_keep = 0; out.pad = 0;
    if (!(lse - lse == 0.0)) {                                  // no finite normaliser: nothing is kept
        if (tid == 0) { p.filters[slot] = out; if (p.out_keep_count) p.out_keep_count[blockIdx.x] = 0; }
        return;
    }

    FilterRow fr;
    const uintptr_t addr = (uintptr_t)row;
    fr.head = (int32_t)((addr & 15) / ES);
    fr.rowv = (const uint4*)(addr & ~(uintptr_t)15);
    fr.V = p.V;
    fr.nchunks = ((int64_t)p.V + fr.head + N - 1) / N;
    fr.sc = make_scale(kLog2e / (double)p.temperature);
    const double L = lse / kLn2;
    fr.ref = ref_for_norm<BF16>(L, fr.sc);
    const double beta = ref_offset<BF16>(fr.ref, fr.sc);
    fr.scale = exp2(-L - beta);

    // ---- top-k: the k-th largest logit
    const uint64_t kbig = ~0ull;
    bool have_cut = false;
    Cut cut{};
    uint64_t r_keep = 0;                                        // ties at theta that are kept
    uint64_t zk = kbig;                                         // fixed-point mass of the top-k set (kbig: whole row)
    uint64_t n_finite = kbig;
    if (p.top_k > 0 && p.top_k < p.V) {
        cut = radix_select<BF16>(sh, fr, false, (uint64_t)p.top_k);
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
    if (p.top_p > 0.f && p.top_p < 1.f) {
        if (zk == kbig) {
            // mass of the whole row in the same fixed point: one more counting pass, level 0 only
            for (int i = tid; i < kFilterBins; i += kFilterThreads) sh.hist[i] = 0;
            __syncthreads();
            for_each_logit<BF16>(fr, 0, fr.nchunks, [&](float x, int32_t) {
                atomicAdd(&sh.hist[order_key<BF16>(x) >> ((BF16 ? 16 : 32) - kLevelBits)], (1ull << kMassBits) + mass_fixed<BF16>(fr, x));
            });
            __syncthreads();
            uint64_t s = 0;
            for (int i = tid; i < kFilterBins; i += kFilterThreads) s += sh.hist[i];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor((unsigned long long)s, m, 64);
            if (lane == 0) sh.wsum[wave] = s;
            __syncthreads();
            uint64_t tot = 0;
            for (int i = 0; i < kFilterWaves; ++i) tot += sh.wsum[i];
            __syncthreads();
            zk = tot & kMassMask;
            n_finite = tot >> kMassBits;
        }
        uint64_t target = (uint64_t)((double)p.top_p * (double)zk + 0.5);
        if (target < 1) target = 1;
        const Cut cp = radix_select<BF16>(sh, fr, true, target);
        uint64_t r = 1;
        if (cp.f_theta > 0 && target > cp.mass_above) r = (target - cp.mass_above + cp.f_theta - 1) / cp.f_theta;
        if (r < 1) r = 1;
        if (r > cp.n_ties) r = cp.n_ties;
        if (have_cut && cp.key == cut.key && r > r_keep) r = r_keep;   // never beyond the top-k cut
        cut = cp;
        r_keep = r;
        have_cut = true;
    }
    (void)n_finite;

    // ---- statistics of the kept tokens; position of the last kept tie
    const float theta = have_cut ? key_to_logit<BF16>(cut.key) : -INFINITY;
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
    double S = 0.0, T = 0.0;
    for (int i = 0; i < kFilterWaves; ++i) { S += sh.red[2 * i]; T += sh.red[2 * i + 1]; }
    if (have_cut && r_keep > 0) {                               // the kept ties, all with the same term
        const float y = exp_arg<BF16>(theta, fr.ref, fr.sc);
        const double ex = (double)fast_exp2(y);
        S += (double)r_keep * ex;
        T += (double)r_keep * ((double)y * ex);
    }

    int idx_cut = 0x7fffffff;                                   // every tie is kept
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

    out.theta = theta;
    out.idx_cut = idx_cut;
    out.n_keep = have_cut ? (int32_t)(cut.cnt_above + r_keep) : -1;   // -1: every finite logit
    if (S > 0.0) {
        const double lnS = log(S);
        out.lse = lnS - beta * kLn2;
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
                         int32_t top_k, float top_p, const Partial* partials, int nparts, RowFilter* filters,
                         int32_t* out_keep_count, hipStream_t s)
{
    if (B <= 0) return hipSuccess;
    if (nparts > 64) return hipErrorInvalidValue;
    FilterParams p{};
    p.target = target; p.draft = draft; p.target_ld = target_ld; p.draft_ld = draft_ld; p.draft_len = draft_len;
    p.temperature = temperature; p.B = B; p.gamma = gamma; p.V = V; p.top_k = top_k; p.top_p = top_p;
    p.partials = partials; p.nparts = nparts; p.filters = filters; p.out_keep_count = out_keep_count;
    const int64_t nblk = (int64_t)B * (2 * gamma + 1);
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == HOLA_DTYPE_BF16) hipLaunchKernelGGL((filter_kernel<true>), dim3((unsigned)nblk), dim3(kFilterThreads), 0, s, p);
    else hipLaunchKernelGGL((filter_kernel<false>), dim3((unsigned)nblk), dim3(kFilterThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace hola
