// Keep sets of top-k / top-p filtered rows, the usual course: one streaming launch that spreads every row over
// several workgroups and lists the few tokens that can lie in the keep set, and one launch in which a single
// wavefront per row decides the cut from that list.  Rows it cannot settle (a list that overflowed, a nucleus
// that reaches beyond the list, NaN or +inf logits) are flagged and left to the one-workgroup-per-row kernel.
//
// Scan: a workgroup of 256 threads owns one segment of up to 256 x 64 logits of a row (the row's chunks are
// shared evenly by its segments) and holds it in registers.  Each thread takes the largest logit of each of its
// chunks and of all of them (bf16: from the raw 16-bit patterns, two per packed operation).  Each wavefront then finds,
// by a bit-by-bit radix descent on ballots, the r-th largest of its lanes' maxima, r being the wavefront's share
// of a rank; the lowest of the wavefronts' values, the edge, has at least `rank` distinct tokens of the segment
// at or above it.  With rank = top_k no token below the edge is among the row's k largest.  (Top-p alone has no
// such bound: the rank is chosen so that the lists of a row hold a few hundred tokens, and the decide step checks
// that the nucleus ends at or above every segment's edge.)  Chunks whose maximum reaches the edge are few, but
// nearly every wavefront has some: it packs them into shared memory and examines their elements with all lanes
// busy.  Tokens at or above the edge go to the segment's own part of the row's list in global memory as
// (key << 32 | index); the segment reports their number, its edge, whether it met NaN / +inf, and for top-p alone
// the mass of its other tokens relative to the edge.  No global atomics, nothing to clear beforehand.
//
// For a larger top_k (69 .. 137 on eight segments) the 64 maxima of a wavefront run out: the rank is then looked up
// among two maxima per lane (those of the two halves of its chunks, disjoint sets of tokens as well).
//
// Decide: the wavefront holds the row's list in registers (16 entries per lane, 32 for the larger top_k), drops what
// lies below the highest segment edge, finds the k-th largest key by a radix descent over ballots (skipping the key
// bits on which all entries agree), keeps the tokens at or above it, and finds the end of the nucleus either by
// walking the cumulative mass of those tokens in the order of the definition (when they fit one lane each) or by a
// radix descent with wavefront sums.  Sums over the kept tokens are integers in fixed point, so neither the order
// of the list nor the number of segments changes a bit of the result.  A keep set of at most 256 tokens is also
// written out as a list: the sampler then draws from those tokens alone.  The kernel is compiled per combination
// of filters, so each carries only its own code and registers.
#include "filter_device.h"

namespace hola {

constexpr int kScanThreads = 256;
constexpr int kScanWaves = kScanThreads / 64;
// Chunks per thread: 64 logits in registers for either type (8 chunks of 8 bf16, 16 chunks of 4 floats), so a
// segment is 16 384 logits and rows of one vocabulary have the same number of segments in both types.
template <bool BF16> struct ScanU { static constexpr int value = BF16 ? 8 : 16; };
constexpr int scan_seg_chunks(int dtype) { return kScanThreads * (dtype == HOLA_DTYPE_BF16 ? 8 : 16); }
constexpr int kScanSlots = 16;                                  // list entries per lane in the decide step
constexpr int kScanSlotsWide = 32;                              // the same for a large top_k, whose lists are longer
constexpr int kScanCap = 64 * kScanSlots;                       // list entries per row that the decide step holds
constexpr int kScanStore = 2 * kScanCap;                        // list entries per row in memory, shared evenly by its segments
constexpr int kScanMaxSeg = 16;                                 // segments per row (64 list entries each at least)
constexpr int kScanTiny = kScanCap * 3 / 4;                     // rows up to this many elements are listed whole
constexpr int kScanTopPList = kScanCap * 5 / 8;                 // list size aimed at for top-p alone (measured: 512 .. 640 alike, 768 spills)

struct SegInfo {
    double others;                     // mass of the segment's tokens below its edge, relative to ref_for(edge)
    float edge;                        // the edge (a logit value)
    uint32_t status;                   // bit 0: NaN / +inf met; bit 1: every finite logit of the segment was listed;
                                       // bits 2..: tokens at or above the edge (listed up to the segment's capacity)
};

struct ScanParams {
    const void* target; const void* draft;
    int64_t target_ld, draft_ld;
    const int32_t* draft_len;
    float temperature;
    int32_t B, gamma, V;
    int32_t top_k; float top_p;
    int32_t nseg, cap_seg;             // segments per row; list entries per segment = kScanStore / nseg
    int32_t seg_len;                   // chunks per segment (the last segments of a row may be short or empty)
    int32_t two_maxima;                // the edge is looked up among two maxima per lane (large top_k)
    unsigned long long* cand;          // [rows, nseg, cap_seg]
    SegInfo* segs;                     // [rows, nseg]
    int32_t* flags;                    // [rows]: 1 = left to the per-row kernel
    int32_t* kept_n;                   // [rows]: its length, -1 when not written
    RowFilter* filters;
    int32_t* out_keep_count;
    int32_t skip_draft;                // the draft rows' keep sets are given: only target rows are scanned and decided
    ExpScale sc;                       // of the call's temperature
};

// The need-th largest of the keys (kbits wide) that satisfy pred, need >= 1 and at most their number, over a
// wavefront that holds E entries per lane of which the first nslots may be occupied.  Bits set in `same` are
// known to be equal in all those keys (their value is in `bits`) and cost nothing.  Wavefront-uniform result.
template <int E, typename T, typename Pred, typename KeyFn>
__device__ __forceinline__ uint32_t wave_select_by_count(const T (&ent)[E], int nslots, int kbits, Pred pred, KeyFn keyfn,
                                                         uint32_t need, uint32_t same = 0, uint32_t bits = 0)
{
    uint32_t prefix = 0;
    for (int bit = kbits - 1; bit >= 0; --bit) {
        if ((same >> bit) & 1u) { prefix |= bits & (1u << bit); continue; }
        const uint32_t want = (prefix >> bit) | 1u;
        uint32_t cnt = 0;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (j < nslots) cnt += (uint32_t)__popcll(__ballot(pred(ent[j]) && (keyfn(ent[j]) >> bit) == want));
        if (cnt >= need) prefix |= 1u << bit;
        else need -= cnt;
    }
    return prefix;
}

// Signed 16-bit order keys of two packed bf16 logits (larger logit, larger key; -0 one below +0).
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
constexpr int kBf16NegInfKey = -32641;                          // key of -inf (0xff80 ^ 0x7fff as a signed 16-bit number)
__device__ __forceinline__ short2_t bf16_keys(uint32_t w)
{
    const short2_t sx = __builtin_bit_cast(short2_t, w);
    const short2_t sign = sx >> 15;                             // 0 or -1 per half
    return __builtin_bit_cast(short2_t, w ^ (__builtin_bit_cast(uint32_t, sign) & 0x7fff7fffu));
}

constexpr int kKeptList = kKeptListMax;                         // longest keep set handed to the sampler as a list
constexpr int kScanHot = 64;                                    // hot chunks a wavefront packs into shared memory

struct ScanShared {
    uint4 hot_chunk[kScanWaves][kScanHot];                      // chunks that hold a logit at or above the edge
    int32_t hot_e0[kScanWaves][kScanHot];                       // index of their first element
    uint32_t edge[kScanWaves];
    uint32_t count;
    uint32_t status;                                            // bit 0: NaN / +inf met
    double red[kScanWaves];
};

// One segment of one row: what a workgroup needs to load it and to interpret the loaded chunks.
struct ScanItem {
    const uint4* rowv;                                          // chunk c_lo of the row's 16-byte grid
    int32_t nchunks, c_lo;                                      // V < 2^22, so chunk and element numbers fit 32 bits
    int32_t head, n_c;                                          // n_c <= 0: nothing to do (row unused or segment empty)
    int32_t r, seg;
    bool used;                                                  // the row is needed (an empty segment still reports)
};

// Segment `seg` of row k (0 .. 2 gamma: the draft rows, then the target rows) of sequence b.  The grid gives the
// three numbers, and every row uses the same segment length, so nothing here divides by a run-time value.
template <bool BF16>
__device__ __forceinline__ ScanItem scan_item(const ScanParams& p, int seg, int k, int b)
{
    ScanItem it;
    it.rowv = nullptr; it.nchunks = 0; it.c_lo = 0; it.head = 0; it.n_c = 0; it.used = false;
    it.r = b * (2 * p.gamma + 1) + k;
    it.seg = seg;
    const bool is_draft = k < p.gamma;
    const int j = is_draft ? k : k - p.gamma;
    int len = p.draft_len ? p.draft_len[b] : p.gamma;
    len = len < 0 ? 0 : (len > p.gamma ? p.gamma : len);
    if (is_draft ? (p.skip_draft || j >= len) : (j > len)) return it;   // row not needed
    it.used = true;
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    const char* row = is_draft ? (const char*)p.draft + ((int64_t)b * p.gamma + j) * p.draft_ld * ES
                               : (const char*)p.target + ((int64_t)b * (p.gamma + 1) + j) * p.target_ld * ES;
    const uintptr_t addr = (uintptr_t)row;
    it.head = (int32_t)((addr & 15) / ES);
    it.nchunks = (p.V + it.head + N - 1) / N;
    it.c_lo = seg * p.seg_len;
    it.rowv = (const uint4*)(addr & ~(uintptr_t)15) + it.c_lo;
    const int32_t c_hi = it.c_lo + p.seg_len < it.nchunks ? it.c_lo + p.seg_len : it.nchunks;
    it.n_c = c_hi > it.c_lo ? c_hi - it.c_lo : 0;               // <= 256 x ScanU (the launcher's choice of seg_len)
    return it;
}

// The segment's chunks, ScanU per thread; chunks past its end read as -inf.
template <bool BF16>
__device__ __forceinline__ void scan_load(const ScanItem& it, uint4 (&v)[ScanU<BF16>::value])
{
    const uint32_t ninf = BF16 ? 0xff80ff80u : 0xff800000u;
#pragma unroll
    for (int u = 0; u < ScanU<BF16>::value; ++u) {
        const int i = (int)threadIdx.x + u * kScanThreads;
        v[u] = make_uint4(ninf, ninf, ninf, ninf);
        if (i < it.n_c) v[u] = load_stream(it.rowv + i);
    }
}

// Edge, list and report of one loaded segment.  Two barriers; the shared words are free for the next segment once
// thread 0 has written the report.
template <bool BF16, bool MASS>
__device__ __forceinline__ void scan_segment(const ScanParams& p, const ScanItem& it, uint4 (&v)[ScanU<BF16>::value], const ExpScale& sc,
                                             ScanShared& sh)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int KB = BF16 ? 16 : 32;
    constexpr int U = ScanU<BF16>::value;
    constexpr int NT = kScanThreads;
    constexpr int NW = kScanWaves;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: a scalar
    if (!it.used) return;                                       // uniform
    SegInfo* seg_out = p.segs + (int64_t)it.r * p.nseg + it.seg;
    if (it.n_c <= 0) {                                          // fewer chunks than segments
        if (tid == 0) { SegInfo si; si.others = 0.0; si.edge = 0.f; si.status = 2u; *seg_out = si; }
        return;
    }
    // elements outside the row read as -inf
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = tid + u * NT;
        const int32_t c = it.c_lo + i;
        if (i < it.n_c && (c == 0 || c == it.nchunks - 1)) {
            const int32_t e0 = c * N - it.head;
            uint32_t* w = (uint32_t*)&v[u];
#pragma unroll
            for (int k = 0; k < N; ++k) {
                if (e0 + k >= 0 && e0 + k < p.V) continue;
                if (BF16) w[k >> 1] = (w[k >> 1] & ((k & 1) ? 0x0000ffffu : 0xffff0000u)) | ((k & 1) ? 0xff800000u : 0x0000ff80u);
                else w[k] = 0xff800000u;
            }
        }
    }

    // ---- largest logit of every chunk and of the thread, NaN / +inf detection.  bf16: from the raw 16-bit
    // patterns, two per packed operation, the result as a signed order key; float: a maximum that skips NaN,
    // which the largest magnitude pattern then reveals.
    int cm_key[U];                                              // bf16: chunk maximum as a signed key
    float cm_val[U];                                            // float: chunk maximum
    bool bad = false;
    uint32_t lane_key = 0;                                      // unsigned order key of the thread's maximum; 0: no finite logit
    if constexpr (BF16) {
        // A positive bf16 is its own key, and as signed 16-bit integers the positives lie above the negatives, so the
        // largest raw pattern of a chunk is its largest key unless every logit in it is negative; then the largest
        // logit is the one of smallest magnitude, the smallest raw pattern, whose key is that pattern with its low
        // 15 bits flipped.  The largest raw pattern taken unsigned exposes a NaN with the sign set (above -inf = 0xff80).
        ushort2_t umax = {0, 0};
        int tmax = -32768;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const short2_t r0 = __builtin_bit_cast(short2_t, v[u].x), r1 = __builtin_bit_cast(short2_t, v[u].y);
            const short2_t r2 = __builtin_bit_cast(short2_t, v[u].z), r3 = __builtin_bit_cast(short2_t, v[u].w);
            const short2_t mx = __builtin_elementwise_max(__builtin_elementwise_max(r0, r1), __builtin_elementwise_max(r2, r3));
            const short2_t mn = __builtin_elementwise_min(__builtin_elementwise_min(r0, r1), __builtin_elementwise_min(r2, r3));
            umax = __builtin_elementwise_max(__builtin_elementwise_max(umax, __builtin_bit_cast(ushort2_t, r0)),
                                             __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, r1),
                                                                       __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, r2),
                                                                                                 __builtin_bit_cast(ushort2_t, r3))));
            const int hi = (int)mx.x > (int)mx.y ? (int)mx.x : (int)mx.y;
            const int lo = (int)mn.x < (int)mn.y ? (int)mn.x : (int)mn.y;
            const int cm = hi >= 0 ? hi : (int)(short)(lo ^ 0x7fff);
            cm_key[u] = cm;
            tmax = cm > tmax ? cm : tmax;
        }
        const uint32_t top_raw = (uint32_t)umax.x > (uint32_t)umax.y ? (uint32_t)umax.x : (uint32_t)umax.y;
        bad = tmax >= 0x7f80 || top_raw > 0xff80u;               // +inf or NaN; NaN with the sign set
        lane_key = tmax > kBf16NegInfKey ? ((uint32_t)tmax ^ 0x8000u) & 0xffffu : 0u;
    } else {
        float tmax = -INFINITY;
        uint32_t amax = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t* w = (const uint32_t*)&v[u];
            cm_val[u] = fmaxf(fmaxf(__uint_as_float(w[0]), __uint_as_float(w[1])), fmaxf(__uint_as_float(w[2]), __uint_as_float(w[3])));
            tmax = fmaxf(tmax, cm_val[u]);
#pragma unroll
            for (int k = 0; k < 4; ++k) { const uint32_t m = w[k] & 0x7fffffffu; amax = m > amax ? m : amax; }
        }
        bad = amax > 0x7f800000u || tmax == INFINITY;
        lane_key = tmax > -INFINITY ? order_key<false>(tmax) : 0u;
    }

    // ---- edge.  Each wavefront takes its share of the rank among its lanes' maxima; the lowest of the
    // wavefronts' values has at least `rank` distinct tokens of the segment at or above it.
    const int32_t row_elems = it.nchunks * N;
    const bool tiny = row_elems <= kScanTiny;
    if (!tiny) {
        // the values the rank is looked up among: each lane's maximum, or (a large top_k, where 64 maxima per
        // wavefront run out) the maxima of the two halves of its chunks, which are disjoint sets of tokens too
        uint32_t keys[2] = {lane_key, 0u};
        if (p.two_maxima) {
            if constexpr (BF16) {
                int h0 = -32768, h1 = -32768;
#pragma unroll
                for (int u = 0; u < U / 2; ++u) { h0 = cm_key[u] > h0 ? cm_key[u] : h0; h1 = cm_key[U / 2 + u] > h1 ? cm_key[U / 2 + u] : h1; }
                keys[0] = h0 > kBf16NegInfKey ? ((uint32_t)h0 ^ 0x8000u) & 0xffffu : 0u;
                keys[1] = h1 > kBf16NegInfKey ? ((uint32_t)h1 ^ 0x8000u) & 0xffffu : 0u;
            } else {
                float h0 = -INFINITY, h1 = -INFINITY;
#pragma unroll
                for (int u = 0; u < U / 2; ++u) { h0 = fmaxf(h0, cm_val[u]); h1 = fmaxf(h1, cm_val[U / 2 + u]); }
                keys[0] = h0 > -INFINITY ? order_key<false>(h0) : 0u;
                keys[1] = h1 > -INFINITY ? order_key<false>(h1) : 0u;
            }
        }
        const int nkeys = p.two_maxima ? 2 : 1;
        const int threads = it.n_c < NT ? it.n_c : NT;          // threads that hold a chunk
        int my_lanes = threads - 64 * wave;
        my_lanes = my_lanes < 0 ? 0 : (my_lanes > 64 ? 64 : my_lanes);
        uint32_t rank = (uint32_t)p.top_k;
        if (MASS) {
            // top-p alone: the rank at which about kScanTopPList tokens of the row are expected at or above the edge
            const float per_thread = (float)(it.n_c * N) / (float)threads;
            const float q = fminf(1.f, (float)kScanTopPList / (float)row_elems);
            // (1 - q)^per_thread on the transcendental unit: the rank only sizes the lists, it decides nothing
            const float rk = (float)threads * (1.f - __builtin_amdgcn_exp2f(per_thread * __builtin_amdgcn_logf(1.f - q)));
            const uint32_t top = (uint32_t)((float)threads * 0.75f);
            rank = (uint32_t)(rk + 0.5f);
            rank = rank > top ? top : rank;
            rank = rank < 1 ? 1 : rank;
        }
        uint32_t wkey = 0xffffffffu;                            // a wavefront without lanes does not bound the edge
        if (my_lanes > 0) {
            const uint32_t need = (rank * (uint32_t)my_lanes + (uint32_t)threads - 1) / (uint32_t)threads;   // shares add up to >= rank
            const uint32_t have = (uint32_t)__popcll(__ballot(keys[0] != 0)) + (uint32_t)__popcll(__ballot(keys[1] != 0));
            wkey = 0;                                           // too few maxima: the whole segment is listed
            if (have >= need)
                wkey = wave_select_by_count<2>(keys, nkeys, KB, [](uint32_t e) { return e != 0; }, [](uint32_t e) { return e; }, need);
        }
        if (lane == 0) sh.edge[wave] = wkey;
    }
    __syncthreads();
    uint32_t edge_key = 0;
    if (!tiny) {
        edge_key = 0xffffffffu;
#pragma unroll
        for (int i = 0; i < NW; ++i) edge_key = sh.edge[i] < edge_key ? sh.edge[i] : edge_key;
        if (edge_key == 0xffffffffu) edge_key = 0;
    }
    const bool lowest = edge_key == 0;                          // every finite logit of the segment is listed
    float edge = lowest ? -3.4028234e38f : key_to_logit<BF16>(edge_key);
    if (!(edge >= -3.4028234e38f)) edge = -3.4028234e38f;
    const float x_low = lowest ? 0.f : edge;
    const float ref_e = MASS ? ref_for<BF16>(x_low, sc) : 0.f;
    // bf16: the signed key a chunk maximum must reach for the chunk to hold a logit >= edge (-0 and +0 compare
    // equal as logits but not as keys: an edge of zero takes the lower key)
    int edge_s = kBf16NegInfKey + 1;
    if (BF16 && !lowest) {
        edge_s = (int)(short)(uint16_t)(edge_key ^ 0x8000u);
        if (edge_s == 0) edge_s = -1;
    }

    // ---- tokens at or above the edge, and the mass of the others (top-p alone).  Few chunks hold such a token
    // (a few per cent), but nearly every wavefront has a lane with one: walking them lane by lane would run the
    // per-element code for every chunk slot with most lanes idle.  Instead each wavefront packs its hot chunks
    // into shared memory and then looks at their elements with all lanes busy.
    double others = 0.0;
    uint32_t hot = 0;                                           // bit u: chunk u holds a logit at or above the edge
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool any = BF16 ? cm_key[u] >= edge_s : cm_val[u] >= edge;
        if (any) hot |= 1u << u;
        if (MASS && !any) {
            float s = 0.f;
#pragma unroll
            for (int k = 0; k < N; ++k) s += fast_exp2(exp_arg<BF16>(chunk_elem<BF16>(v[u], k), ref_e, sc));
            if (!(s >= 0.f)) {                                  // a -inf logit can turn its exponent into NaN: leave those out
                s = 0.f;
#pragma unroll
                for (int k = 0; k < N; ++k) {
                    const float x = chunk_elem<BF16>(v[u], k);
                    if (x > -INFINITY && x < INFINITY) s += fast_exp2(exp_arg<BF16>(x, ref_e, sc));
                }
            }
            others += (double)s;
        }
    }
    int nh = 0;                                                 // hot chunks of the wavefront (uniform)
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool mine = (hot >> u) & 1u;
        const unsigned long long bl = __ballot(mine);
        if (bl) {
            const int at = nh + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bl >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bl, 0u));
            if (mine && at < kScanHot) {
                sh.hot_chunk[wave][at] = v[u];
                sh.hot_e0[wave][at] = (it.c_lo + tid + u * NT) * N - it.head;
            }
            nh += (int)__popcll(bl);
        }
    }
    unsigned long long* list = p.cand + ((int64_t)it.r * p.nseg + it.seg) * p.cap_seg;
    if (nh <= kScanHot) {
        wave_handoff();                        // the wavefront reads what its own lanes stored
        constexpr int IT = kScanHot * N / 64;
        const int nel = nh * N;
        float xs[IT];
        unsigned long long bal[IT];
        int total = 0;
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            bal[i] = 0ull;
            xs[i] = -INFINITY;
            if (i * 64 < nel) {
                const int t = i * 64 + lane;
                if (t < nel) {
                    if (BF16) xs[i] = __uint_as_float((uint32_t)((const uint16_t*)sh.hot_chunk[wave])[t] << 16);
                    else xs[i] = ((const float*)sh.hot_chunk[wave])[t];
                }
                const bool c = xs[i] >= edge && xs[i] < INFINITY;
                if (MASS && !c && xs[i] > -INFINITY && xs[i] < INFINITY) others += (double)fast_exp2(exp_arg<BF16>(xs[i], ref_e, sc));
                bal[i] = __ballot(c);
                total += (int)__popcll(bal[i]);
            }
        }
        int at = 0;
        if (lane == 0 && total > 0) at = (int)atomicAdd(&sh.count, (uint32_t)total);
        at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            if (bal[i]) {
                const int t = i * 64 + lane;
                const int pos = at + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal[i] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal[i], 0u));
                if (((bal[i] >> lane) & 1ull) && pos < p.cap_seg)
                    list[pos] = ((unsigned long long)order_key<BF16>(xs[i]) << 32) | (uint32_t)(sh.hot_e0[wave][t / N] + t % N);
                at += (int)__popcll(bal[i]);
            }
        }
    } else {
        // many hot chunks (a segment listed whole, long runs of equal logits): lane by lane
        int cnt = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!((hot >> u) & 1u)) continue;
#pragma unroll
            for (int k = 0; k < N; ++k) {
                const float x = chunk_elem<BF16>(v[u], k);
                if (x >= edge && x < INFINITY) ++cnt;
                else if (MASS && x > -INFINITY && x < INFINITY) others += (double)fast_exp2(exp_arg<BF16>(x, ref_e, sc));
            }
        }
        int incl = cnt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int o = __shfl_up(incl, d, 64); if (lane >= d) incl += o; }
        const int wave_total = __shfl(incl, 63, 64);
        int base = 0;
        if (lane == 0 && wave_total > 0) base = (int)atomicAdd(&sh.count, (uint32_t)wave_total);
        base = __shfl(base, 0, 64);
        if (cnt > 0) {
            int pos = base + incl - cnt;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!((hot >> u) & 1u)) continue;
                const int32_t e0 = (it.c_lo + tid + u * NT) * N - it.head;
#pragma unroll
                for (int k = 0; k < N; ++k) {
                    const float x = chunk_elem<BF16>(v[u], k);
                    if (x >= edge && x < INFINITY) {
                        if (pos < p.cap_seg) list[pos] = ((unsigned long long)order_key<BF16>(x) << 32) | (uint32_t)(e0 + k);
                        ++pos;
                    }
                }
            }
        }
    }
    if (bad) atomicOr(&sh.status, 1u);
    if (MASS) {
        others = wave_sum(others);
        if (lane == 0) sh.red[wave] = others;
    }
    __syncthreads();
    if (tid == 0) {
        SegInfo si;
        si.others = 0.0;
        if (MASS)
            for (int i = 0; i < NW; ++i) si.others += sh.red[i];
        si.edge = x_low;
        si.status = (sh.status & 1u) | (lowest ? 2u : 0u) | (sh.count << 2);
        *seg_out = si;
        sh.status = 0;                                          // for the workgroup's next segment: the other threads
        sh.count = 0;                                           // touch these words only after its first barrier
    }
}

// One workgroup per segment.  (Persistent workgroups that loaded their next segment while working on the current
// one were slower: twice the registers, and the waits on the stores of the list also waited on the prefetch.)
template <bool BF16, bool MASS>
__global__ __launch_bounds__(kScanThreads) void filter_scan_kernel(ScanParams p)
{
    __shared__ ScanShared sh;
    if (threadIdx.x == 0) { sh.status = 0; sh.count = 0; }
    const ExpScale sc = p.sc;
    uint4 v[ScanU<BF16>::value];
    const ScanItem it = scan_item<BF16>(p, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z);   // grid: nseg x (2 gamma + 1) x B
    scan_load<BF16>(it, v);
    __syncthreads();
    scan_segment<BF16, MASS>(p, it, v, sc, sh);
}

// WANT_K / WANT_P: which of the two filters is on (at least one is), so that each combination carries only its own
// code and registers.
template <bool BF16, bool WANT_K, bool WANT_P, int E>
__global__ __launch_bounds__(64, E > kScanSlots ? 2 : ((WANT_K && WANT_P) ? 4 : 5)) void filter_decide_kernel(ScanParams p)
{
    constexpr int KB = BF16 ? 16 : 32;
    const int lane = threadIdx.x;
    const int r = blockIdx.x;
    FilterRowId id;
    if (!filter_row_id(r, p.B, p.gamma, p.draft_len, id, p.skip_draft)) {   // row not needed
        if (lane == 0) { p.flags[r] = 0; p.kept_n[r] = -1; if (p.out_keep_count) p.out_keep_count[r] = -1; }
        return;
    }
    FilterRow fr = make_filter_row<BF16>(p.target, p.draft, p.target_ld, p.draft_ld, p.gamma, p.V, p.temperature, id);
    constexpr bool want_k = WANT_K, want_p = WANT_P;
    if (lane == 0) p.kept_n[r] = -1;                            // until the keep set itself has been written

    // lane s holds the record of segment s (at most kScanMaxSeg of them)
    SegInfo si;
    si.others = 0.0; si.edge = 0.f; si.status = 2u;
    if (lane < p.nseg) si = p.segs[(int64_t)r * p.nseg + lane];
    const int my_count = (int)(si.status >> 2);
    const bool bad = __ballot((si.status & 1u) != 0) != 0;
    const bool partial = __ballot(!(si.status & 2u)) != 0;      // some segment listed only its top
    const bool spilled = __ballot(my_count > p.cap_seg) != 0;
    uint32_t edge_max = (si.status & 2u) ? 0u : order_key<BF16>(si.edge);   // the highest edge among those segments
    int n = my_count;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const uint32_t o = __shfl_xor(edge_max, m, 64); edge_max = o > edge_max ? o : edge_max;
        n += __shfl_xor(n, m, 64);
    }
    if (bad || spilled || n > 64 * E) {                         // left to the per-row kernel
        if (lane == 0) p.flags[r] = 1;
        return;
    }
    RowFilter out;
    out.lse = -INFINITY; out.H = NAN; out.theta = INFINITY; out.idx_cut = -1; out.n_keep = 0; out.pad = 0;
    if (n == 0) {                                               // no finite logit: nothing is kept
        if (lane == 0) { p.filters[id.slot] = out; p.flags[r] = 0; if (p.out_keep_count) p.out_keep_count[r] = 0; }
        return;
    }
    if (want_k && n < p.top_k && partial) {                     // cannot happen (a segment with an edge lists >= k); be safe
        if (lane == 0) p.flags[r] = 1;
        return;
    }

    // the lists of the segments one after the other: entry f belongs to the segment whose running count passes f
    int run = my_count;                                         // inclusive running count over the segments (lanes)
#pragma unroll
    for (int d = 1; d < kScanMaxSeg; d <<= 1) { const int o = __shfl_up(run, d, 64); if (lane >= d) run += o; }
    int nslots = (n + 63) / 64;
    unsigned long long ent[E];
    const unsigned long long* list = p.cand + (int64_t)r * p.nseg * p.cap_seg;
#pragma unroll
    for (int j = 0; j < E; ++j) {
        ent[j] = 0ull;
        if (j < nslots) {
            const int f = j * 64 + lane;
            int sg = 0;                                         // segments that end at or before f
#pragma unroll
            for (int step = kScanMaxSeg / 2; step >= 1; step >>= 1) {
                const int probe = sg + step - 1;
                const int end_q = __shfl(run, probe & 63, 64);
                if (probe < p.nseg - 1 && f >= end_q) sg += step;
            }
            const int before = __shfl(run, (sg + 63) & 63, 64);   // every lane takes part in the exchange
            const int start = sg > 0 ? before : 0;
            if (f < n) ent[j] = list[(int64_t)sg * p.cap_seg + (f - start)];
        }
    }
    auto valid = [](unsigned long long e) { return e != 0; };   // the key of a finite logit is never 0
    auto logit_key = [](unsigned long long e) { return (uint32_t)(e >> 32); };

    // masses are taken against the reference of the row's largest logit
    uint32_t kmax = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) { const uint32_t kk = logit_key(ent[j]); kmax = kk > kmax ? kk : kmax; }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) { const uint32_t o = __shfl_xor(kmax, m, 64); kmax = o > kmax ? o : kmax; }
    fr.ref = ref_for<BF16>(key_to_logit<BF16>(kmax), fr.sc);
    fr.scale = 1.0;
    const double beta_m = ref_offset<BF16>(fr.ref, fr.sc);
    // Shorter lists make every later step cheaper: entries that cannot matter are dropped and the rest packed into
    // the first slots (through shared memory; the order of a list never matters).
    __shared__ unsigned long long s_pack[64 * E];
    auto pack = [&](auto keep_key) {
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            if (j < nslots) {
                const bool keep = valid(ent[j]) && keep_key(logit_key(ent[j]));
                const unsigned long long bl = __ballot(keep);
                if (bl) {
                    const int at = cnt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bl >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bl, 0u));
                    if (keep) s_pack[at] = ent[j];
                    cnt += (int)__popcll(bl);
                }
            }
        }
        wave_handoff();
        n = cnt;
        nslots = (cnt + 63) / 64;
#pragma unroll
        for (int j = 0; j < E; ++j) ent[j] = (j < nslots && j * 64 + lane < cnt) ? s_pack[j * 64 + lane] : 0ull;
        wave_handoff();
    };
    // key bits on which every listed token agrees (the list spans a narrow range of logits): the descents skip them
    uint32_t same = 0, same_bits = 0;
    auto agree = [&]() {
        uint32_t k_or = 0, k_and = 0xffffffffu;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (j < nslots && valid(ent[j])) { k_or |= logit_key(ent[j]); k_and &= logit_key(ent[j]); }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { k_or |= __shfl_xor(k_or, m, 64); k_and &= __shfl_xor(k_and, m, 64); }
        same = ~(k_or ^ k_and);
        same_bits = k_and;
    };
    auto count_where = [&](auto pred) {
        uint32_t c = 0;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (j < nslots) c += (uint32_t)__popcll(__ballot(valid(ent[j]) && pred(logit_key(ent[j]))));
        return c;
    };

    bool have_cut = false;
    uint32_t cut_key = 0, n_ties = 0, cnt_above = 0;
    unsigned long long r_keep = 0, zk = ~0ull;
    if (want_k) {
        // the segment with the highest edge alone holds k tokens at or above it: nothing below that edge is kept
        if (partial) pack([&](uint32_t kk) { return kk >= edge_max; });
        agree();
        const uint32_t need = (uint32_t)p.top_k < (uint32_t)n ? (uint32_t)p.top_k : (uint32_t)n;
        cut_key = wave_select_by_count<E>(ent, nslots, KB, valid, logit_key, need, same, same_bits);
        pack([&](uint32_t kk) { return kk >= cut_key; });        // the kept tokens and the ties at the cut
        cnt_above = count_where([&](uint32_t kk) { return kk > cut_key; });
        n_ties = count_where([&](uint32_t kk) { return kk == cut_key; });
        const unsigned long long total = (unsigned long long)cnt_above + n_ties;
        r_keep = total >= (unsigned long long)p.top_k ? (unsigned long long)p.top_k - cnt_above : n_ties;
        have_cut = true;
    }
    // ---- top-k with top-p, the kept tokens and the ties at the cut on one lane each (the usual case): put them in
    // the order of the definition (logit descending, equal logits by ascending index) and walk the cumulative mass.
    // The first k of them are the top-k set; the nucleus is the shortest prefix that reaches top_p of their mass.
    bool nucleus_done = false;
    int idx_cut = 0x7fffffff;                                   // every tie is kept
    if (want_k && want_p && n <= 64) {
        __shared__ unsigned long long s_ord_e[64], s_ord_m[64];
        const unsigned long long e = ent[0];
        const uint32_t key = logit_key(e), idx = (uint32_t)(e & 0xffffffffu);
        s_pack[lane] = e;
        wave_handoff();
        int rank = 0;
        for (int q = 0; q < n; ++q) {
            const unsigned long long o = s_pack[q];
            const uint32_t ok = logit_key(o), oi = (uint32_t)(o & 0xffffffffu);
            rank += (ok > key || (ok == key && oi < idx)) ? 1 : 0;
        }
        if (valid(e)) {
            s_ord_e[rank] = e;
            s_ord_m[rank] = list_mass_fixed<BF16>(fr, key_to_logit<BF16>(key));
        }
        wave_handoff();
        const unsigned long long er = lane < n ? s_ord_e[lane] : 0ull;
        unsigned long long incl = lane < n ? s_ord_m[lane] : 0ull;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const unsigned long long o = __shfl_up(incl, d, 64); if (lane >= d) incl += o; }
        const int kk = p.top_k < n ? p.top_k : n;               // the top-k set: the first kk in this order
        zk = __shfl(incl, kk - 1, 64);
        unsigned long long target = (unsigned long long)((double)p.top_p * (double)zk + 0.5);
        if (target < 1) target = 1;
        const unsigned long long hit = __ballot(lane < kk && incl >= target);
        const int last = hit ? __ffsll((long long)hit) - 1 : kk - 1;   // the last kept token
        const unsigned long long ec = __shfl(er, last, 64);
        cut_key = logit_key(ec);
        idx_cut = (int)(uint32_t)(ec & 0xffffffffu);            // kept ties have indices up to this one
        cnt_above = (uint32_t)__popcll(__ballot(lane <= last && logit_key(er) > cut_key));
        r_keep = (unsigned long long)(last + 1) - cnt_above;
        n_ties = (uint32_t)r_keep;                              // nothing left for the tie search below
        have_cut = true;
        nucleus_done = true;
    }
    if (!nucleus_done) agree();

    unsigned long long mass[E];
    unsigned long long lm = 0;                                  // mass of the whole list
#pragma unroll
    for (int j = 0; j < E; ++j) {
        mass[j] = 0ull;
        if (want_p && !nucleus_done && j < nslots && valid(ent[j])) mass[j] = list_mass_fixed<BF16>(fr, key_to_logit<BF16>(logit_key(ent[j])));
        lm += mass[j];
    }
    if (want_p && !nucleus_done) lm = wave_sum_u64(lm);
    auto mass_where = [&](auto pred) {
        unsigned long long s = 0;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (j < nslots && valid(ent[j]) && pred(logit_key(ent[j]))) s += mass[j];
        return wave_sum_u64(s);
    };
    if (want_k && want_p && !nucleus_done) {
        const unsigned long long f_theta = list_mass_fixed<BF16>(fr, key_to_logit<BF16>(cut_key));
        zk = mass_where([&](uint32_t kk) { return kk > cut_key; }) + r_keep * f_theta;
    }
    if (want_p && !nucleus_done) {
        unsigned long long target;
        if (zk != ~0ull) {
            target = (unsigned long long)((double)p.top_p * (double)zk + 0.5);
        } else {
            // top-p alone: of the mass of the whole row = the list plus what the segments left below their edges
            double others_list = 0.0;
            if (si.others > 0.0) {
                const double beta_e = ref_offset<BF16>(ref_for<BF16>(si.edge, fr.sc), fr.sc);
                others_list = si.others * exp2(beta_m - beta_e);
            }
            others_list = wave_sum(others_list) * kListMassUnit;
            target = (unsigned long long)((double)p.top_p * ((double)lm + others_list) + 0.5);
            if (partial && lm < target) {                       // the nucleus reaches beyond the list
                if (lane == 0) p.flags[r] = 1;
                return;
            }
        }
        if (target < 1) target = 1;
        if (target > lm) target = lm;                           // rounding only: the list holds the target mass
        // the key at which the cumulative mass, largest first, reaches the target
        uint32_t prefix = 0;
        unsigned long long above = 0;
        for (int bit = KB - 1; bit >= 0; --bit) {
            if ((same >> bit) & 1u) { prefix |= same_bits & (1u << bit); continue; }
            const uint32_t want = (prefix >> bit) | 1u;
            unsigned long long s = 0;
#pragma unroll
            for (int j = 0; j < E; ++j)
                if (j < nslots && valid(ent[j]) && (logit_key(ent[j]) >> bit) == want) s += mass[j];
            s = wave_sum_u64(s);
            if (above + s >= target) prefix |= 1u << bit;
            else above += s;
        }
        const uint32_t ties_p = count_where([&](uint32_t kk) { return kk == prefix; });
        const unsigned long long f_theta = list_mass_fixed<BF16>(fr, key_to_logit<BF16>(prefix));
        unsigned long long rr = 1;
        if (f_theta > 0 && target > above) rr = (target - above + f_theta - 1) / f_theta;
        if (rr < 1) rr = 1;
        if (rr > ties_p) rr = ties_p;
        if (have_cut && prefix == cut_key && rr > r_keep) rr = r_keep;   // never beyond the top-k cut
        if (ties_p == 0) {                                      // every mass below the unit: keep the largest logit
            prefix = kmax;
            rr = 1;
        }
        // top-p alone: a segment lists only what lies at or above its own edge, so the tokens at or above theta
        // are all listed only if theta is not below the highest edge
        if (!want_k && partial && prefix < edge_max) {
            if (lane == 0) p.flags[r] = 1;
            return;
        }
        cut_key = prefix;
        n_ties = count_where([&](uint32_t kk) { return kk == cut_key; });
        cnt_above = count_where([&](uint32_t kk) { return kk > cut_key; });
        r_keep = rr > n_ties ? n_ties : rr;
        have_cut = true;
    }
    const float theta = key_to_logit<BF16>(cut_key);

    // ---- sums over the kept tokens above theta, the kept ties added once.  Each term is a float (the library's
    // terms 2^y are) and is added as an integer in fixed point, so the order of the list does not matter: a float
    // below 2^31 splits exactly into its integer part and a remainder that the second conversion takes.
    const float y_top = exp_arg<BF16>(key_to_logit<BF16>(kmax), fr.ref, fr.sc);   // near 0: the reference is the largest logit's
    int sft = (int)floorf(-y_top);
    sft = sft < -8 ? -8 : (sft > 8 ? 8 : sft);
    unsigned long long Sfix = 0;                                // unit 2^-52 (each term < 2)
    long long Tfix = 0;                                         // unit 2^-42 (|y 2^y| < 2^9 for a term that does not underflow)
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const uint32_t kk = logit_key(ent[j]);
        if (j < nslots && valid(ent[j]) && kk > cut_key) {
            const float y = exp_arg<BF16>(key_to_logit<BF16>(kk), fr.ref, fr.sc);
            const float ex = ldexpf(fast_exp2(y), sft);
            const float a = ex * 1048576.f;                     // 2^20
            const uint32_t a_hi = (uint32_t)a;
            const uint32_t a_lo = (uint32_t)((a - (float)a_hi) * 4294967296.f);
            Sfix += ((unsigned long long)a_hi << 32) | a_lo;
            const float pt = y * ex;
            const float bq = fabsf(pt) * 1024.f;                // 2^10
            const uint32_t b_hi = (uint32_t)bq;
            const uint32_t b_lo = (uint32_t)((bq - (float)b_hi) * 4294967296.f);
            const long long mag = (long long)(((unsigned long long)b_hi << 32) | b_lo);
            Tfix += pt < 0.f ? -mag : mag;
        }
    }
    Sfix = wave_sum_u64(Sfix);
    Tfix = (long long)wave_sum_u64((unsigned long long)Tfix);
    double S = ldexp((double)Sfix, -52 - sft);
    double T = ldexp((double)Tfix, -42 - sft);
    if (r_keep > 0) {
        const float y = exp_arg<BF16>(theta, fr.ref, fr.sc);
        const double ex = (double)fast_exp2(y);
        S += (double)r_keep * ex;
        T += (double)r_keep * ((double)y * ex);
    }

    // ---- the last kept tie: the r-th smallest index among the ties
    if (r_keep < n_ties && n_ties <= 64) {
        // few ties (the usual case): their indices go to shared memory, lane l counts those below the l-th
        __shared__ uint32_t s_tie[64];
        int nt = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            if (j < nslots) {
                const bool tie = valid(ent[j]) && logit_key(ent[j]) == cut_key;
                const unsigned long long bl = __ballot(tie);
                if (bl) {
                    const int at = nt + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bl >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bl, 0u));
                    if (tie) s_tie[at] = (uint32_t)(ent[j] & 0xffffffffu);
                    nt += (int)__popcll(bl);
                }
            }
        }
        wave_handoff();
        const uint32_t mine = lane < (int)n_ties ? s_tie[lane] : 0xffffffffu;
        uint32_t below = 0;
        for (int q = 0; q < (int)n_ties; ++q) below += s_tie[q] < mine ? 1u : 0u;
        const unsigned long long hit = __ballot(lane < (int)n_ties && (unsigned long long)below + 1 == r_keep);
        const int src = hit ? __ffsll((long long)hit) - 1 : 0;
        idx_cut = (int)__shfl(mine, src, 64);
    } else if (r_keep < n_ties) {
        // long runs of equal logits: the r-th largest complemented index by radix descent
        const uint32_t tkey = cut_key;
        auto is_tie = [tkey](unsigned long long e) { return e != 0 && (uint32_t)(e >> 32) == tkey; };
        auto inv_index = [](unsigned long long e) { return 0x3fffffu - (uint32_t)(e & 0xffffffffu); };
        const uint32_t ci = wave_select_by_count<E>(ent, nslots, 22, is_tie, inv_index, (uint32_t)r_keep);
        idx_cut = (int)(0x3fffffu - ci);
    }

    // ---- a short keep set of a target row is written out itself: the sampler then needs no sweep of the row
    const long long n_keep = have_cut ? (long long)cnt_above + (long long)r_keep : -1;
    if (!id.is_draft && n_keep >= 1 && n_keep <= kKeptList) {
        // (into the row's own candidate area: every entry of it has been in registers since the start)
        unsigned long long* kl = p.cand + (int64_t)r * p.nseg * p.cap_seg;
        int nk = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            if (j < nslots) {
                const uint32_t kk = logit_key(ent[j]);
                const bool keep = valid(ent[j]) && (kk > cut_key || (kk == cut_key && (int)(uint32_t)(ent[j] & 0xffffffffu) <= idx_cut));
                const unsigned long long bl = __ballot(keep);
                if (bl) {
                    const int at = nk + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bl >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bl, 0u));
                    if (keep && at < kKeptList) kl[at] = ent[j];
                    nk += (int)__popcll(bl);
                }
            }
        }
        if (lane == 0) p.kept_n[r] = nk == (int)n_keep ? nk : -1;
    }

    out.theta = theta;
    out.idx_cut = idx_cut;
    out.n_keep = have_cut ? (int32_t)(cnt_above + r_keep) : -1;
    if (S > 0.0) {
        const double lnS = log(S);
        out.lse = lnS - beta_m * kLn2;
        out.H = lnS - kLn2 * (T / S);
        if (out.H < 0.0) out.H = 0.0;                           // a single kept token: exactly zero
    }
    if (lane == 0) { p.filters[id.slot] = out; p.flags[r] = 0; if (p.out_keep_count) p.out_keep_count[r] = out.n_keep; }
}

// Segments per row: as few as hold a row of V elements of either type at any alignment.
static int scan_segments(int dtype, int32_t V)
{
    const int N = dtype == HOLA_DTYPE_BF16 ? 8 : 4;
    const int64_t nchunks_max = ((int64_t)V + N - 1) / N + 1;
    return (int)((nchunks_max + scan_seg_chunks(dtype) - 1) / scan_seg_chunks(dtype));
}

// Scratch of the scan + decide pair: 16 KB of candidate list per row, which is why very large batches (beyond
// 256 MB of lists) go without it and use the per-row kernel alone.
size_t filter_scan_bytes(int64_t rows)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    if (rows <= 0 || (size_t)rows * kScanStore * sizeof(unsigned long long) > ((size_t)256 << 20)) return 0;
    return up((size_t)rows * kScanStore * sizeof(unsigned long long)) + 2 * up((size_t)rows * sizeof(int32_t)) +
           up((size_t)rows * kScanMaxSeg * sizeof(SegInfo));
}

// Entries per lane the decide step needs for this call (0: the scan + decide pair is not worth running).  A segment
// lists about 1.45 top_k tokens for top_k up to ~64 (the lowest of four wavefronts' values lets that many through)
// and more beyond, as the lanes' maxima run out (1.7 top_k at 136), give or take 20 %; a segment that lists more than
// its share of the stored list (kScanStore / nseg) sends its row to the per-row kernel, which costs more than the
// scan saves once it happens in a call.  Measured on 8 segments: no such row up to top_k = 85, some at 100, most
// at 136.
static int scan_decide_slots(int dtype, int32_t V, int32_t top_k)
{
    const int nseg = scan_segments(dtype, V);
    if (nseg > kScanMaxSeg) return 0;
    const bool want_k = top_k > 0 && top_k < V;
    if (!want_k || (int64_t)V <= kScanTiny) return kScanSlots;
    const int64_t listed = (int64_t)top_k * nseg;
    // a wavefront looks its share of top_k (a quarter) up among its 64 maxima, or 128 with two per lane
    if (top_k <= kScanThreads * 3 / 4 && listed * 3 / 2 * 5 / 4 <= 64 * kScanSlots) return kScanSlots;   // top_k <= 68 on 8 segments
    if (top_k <= kScanThreads * 3 / 2 && listed <= 1100) return kScanSlotsWide;   // top_k <= 137 on 8 segments (two maxima per lane)
    return 0;
}

bool filter_scan_applies(int dtype, int32_t V, int32_t top_k) { return scan_decide_slots(dtype, V, top_k) > 0; }

static ScanParams scan_params(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                              const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                              int32_t top_k, float top_p, RowFilter* filters, int32_t* out_keep_count, void* scratch,
                              int32_t skip_draft)
{
    const int64_t rows = (int64_t)B * (2 * gamma + 1);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    char* base = (char*)scratch;
    ScanParams p{};
    p.target = target; p.draft = draft; p.target_ld = target_ld; p.draft_ld = draft_ld; p.draft_len = draft_len;
    p.temperature = temperature; p.B = B; p.gamma = gamma; p.V = V; p.top_k = top_k; p.top_p = top_p;
    p.filters = filters; p.out_keep_count = out_keep_count; p.skip_draft = skip_draft;
    p.sc = host_scale((double)temperature);
    p.nseg = scan_segments(dtype, V);
    p.cap_seg = kScanStore / p.nseg;
    const int N = dtype == HOLA_DTYPE_BF16 ? 8 : 4;
    const int64_t nchunks_max = ((int64_t)V + N - 1) / N + 1;   // any alignment of the row
    p.seg_len = (int32_t)((nchunks_max + p.nseg - 1) / p.nseg);
    p.two_maxima = scan_decide_slots(dtype, V, top_k) > kScanSlots ? 1 : 0;
    size_t off = 0;
    p.cand = (unsigned long long*)(base + off); off += up((size_t)rows * kScanStore * sizeof(unsigned long long));
    p.flags = (int32_t*)(base + off);           off += up((size_t)rows * sizeof(int32_t));
    p.kept_n = (int32_t*)(base + off);          off += up((size_t)rows * sizeof(int32_t));
    p.segs = (SegInfo*)(base + off);
    return p;
}

hipError_t launch_filter_scan(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                              const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                              int32_t top_k, float top_p, void* scratch, int32_t skip_draft, hipStream_t s)
{
    const ScanParams p = scan_params(target, draft, dtype, target_ld, draft_ld, draft_len, temperature, B, gamma, V, top_k, top_p,
                                     nullptr, nullptr, scratch, skip_draft);
    if (p.nseg > kScanMaxSeg || p.seg_len > scan_seg_chunks(dtype) || B > 65535) return hipErrorInvalidValue;
    const bool mass = !(top_k > 0 && top_k < V);                // top-p alone: the segments also sum the mass below their edges
    const dim3 grid((unsigned)p.nseg, (unsigned)(2 * gamma + 1), (unsigned)B);
    if (dtype == HOLA_DTYPE_BF16) {
        if (mass) hipLaunchKernelGGL((filter_scan_kernel<true, true>), grid, dim3(kScanThreads), 0, s, p);
        else hipLaunchKernelGGL((filter_scan_kernel<true, false>), grid, dim3(kScanThreads), 0, s, p);
    } else {
        if (mass) hipLaunchKernelGGL((filter_scan_kernel<false, true>), grid, dim3(kScanThreads), 0, s, p);
        else hipLaunchKernelGGL((filter_scan_kernel<false, false>), grid, dim3(kScanThreads), 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_filter_decide(const void* target, const void* draft, int dtype, int64_t target_ld, int64_t draft_ld,
                                const int32_t* draft_len, float temperature, int32_t B, int32_t gamma, int32_t V,
                                int32_t top_k, float top_p, RowFilter* filters, int32_t* out_keep_count, void* scratch,
                                int32_t** flags_out, const unsigned long long** kept_out, int64_t* kept_stride_out,
                                const int32_t** kept_n_out, int32_t skip_draft, hipStream_t s)
{
    const ScanParams p = scan_params(target, draft, dtype, target_ld, draft_ld, draft_len, temperature, B, gamma, V, top_k, top_p,
                                     filters, out_keep_count, scratch, skip_draft);
    *flags_out = p.flags;
    *kept_out = p.cand;                                         // a short keep set replaces the row's candidates
    *kept_stride_out = (int64_t)p.nseg * p.cap_seg;
    *kept_n_out = p.kept_n;
    const int64_t rows = (int64_t)B * (2 * gamma + 1);
    const bool want_k = top_k > 0 && top_k < V, want_p = top_p > 0.f && top_p < 1.f;
    const dim3 grid((unsigned)rows), block(64);
    const bool wide = scan_decide_slots(dtype, V, top_k) > kScanSlots;   // only with top-k
#define HOLA_DECIDE(BF, K, P, EE) hipLaunchKernelGGL((filter_decide_kernel<BF, K, P, EE>), grid, block, 0, s, p)
    if (dtype == HOLA_DTYPE_BF16) {
        if (want_k && want_p) { if (wide) HOLA_DECIDE(true, true, true, kScanSlotsWide); else HOLA_DECIDE(true, true, true, kScanSlots); }
        else if (want_k) { if (wide) HOLA_DECIDE(true, true, false, kScanSlotsWide); else HOLA_DECIDE(true, true, false, kScanSlots); }
        else HOLA_DECIDE(true, false, true, kScanSlots);
    } else {
        if (want_k && want_p) { if (wide) HOLA_DECIDE(false, true, true, kScanSlotsWide); else HOLA_DECIDE(false, true, true, kScanSlots); }
        else if (want_k) { if (wide) HOLA_DECIDE(false, true, false, kScanSlotsWide); else HOLA_DECIDE(false, true, false, kScanSlots); }
        else HOLA_DECIDE(false, false, true, kScanSlots);
    }
#undef HOLA_DECIDE
    return hipGetLastError();
}

}  // namespace hola
