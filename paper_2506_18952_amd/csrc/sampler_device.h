// Device code of the next-token sampler (shared by the split kernels and the fused per-sequence kernel):
// inverse CDF over the residual max(0, p - q) at the first rejected position, or over p at the bonus
// position when every draft was kept.
//
// A row is cut into tiles of 64 lanes x 4 chunks of 16 bytes.  Tile weights are summed in double; the
// selecting wavefront scans them, finds the tile where the running sum first exceeds u * Z, re-reads
// only that tile and scans inside it: lanes, then the 4 or 8 elements of one chunk.  Element weights
// come from one device function, so the sweep and the re-read agree bit for bit.
//
// Numerics: p_i = 2^(x_i c - L), L = lse / ln 2 from the accept stage.  The exponent argument is
// formed against a float reference as in the row statistics (exact bf16 product / fp32 difference);
// what the reference misses is put back exactly: w_i = 2^rP * max(0, eP_i - kappa eQ_i) with
// kappa = 2^(rQ - rP) carried as a float pair and the common factor applied to chunk sums in double.
// Chunk sums are fp32 over 4-8 elements, everything above a chunk is double.
#pragma once
#include "stats_device.h"

namespace hola {

struct RowPair {
    const uint4* Pv; const uint4* Dv;   // 16-byte aligned chunk grids (Dv null => element loads of D)
    const void* D;                      // draft row (element addressing)
    int32_t head;                       // elements of chunk 0 that precede the target row
    int32_t V;
    int64_t nchunks;                    // chunks that hold at least one element of the row
    ExpScale sc;
    float refP, refQ, k_hi, k_lo;
    double scale;                       // 2^rP
    int32_t bonus;                      // weights are p itself
    int32_t ok;                         // the target row has a finite normaliser
    float thP, thQ; int32_t cutP, cutQ; // keep sets of filtered rows (x > th, or x == th and index <= cut)
};

// Reference for rows whose log2-normaliser is L: bf16 an integer near -L, fp32 a logit near L / c.
template <bool BF16>
__device__ __forceinline__ float ref_for_norm(double L, const ExpScale& sc)
{
    return BF16 ? (float)rint(-L) : (float)(L / sc.cstar);
}

template <bool BF16>
__device__ __forceinline__ void make_row_pair(RowPair& rp, const void* target, const void* draft, int64_t target_ld,
                                              int64_t draft_ld, int32_t gamma, int32_t V, float Tb, int b,
                                              const SeqInfo& si, int force_bonus, const RowFilter* filters = nullptr,
                                              int32_t B = 0, const RowFilter* draft_filters = nullptr,
                                              const ExpScale* sc = nullptr /* the constants for Tb, if the caller has them */)
{
    constexpr int N = BF16 ? 8 : 4;
    constexpr int ES = BF16 ? 2 : 4;
    const int g = gamma;
    rp.sc = sc ? *sc : make_scale(kLog2e / (double)Tb);
    rp.V = V;
    const char* rowP = (const char*)target + ((int64_t)b * (g + 1) + si.row) * target_ld * ES;
    const uintptr_t aP = (uintptr_t)rowP;
    rp.head = (int32_t)((aP & 15) / ES);
    rp.Pv = (const uint4*)(aP & ~(uintptr_t)15);
    rp.nchunks = ((int64_t)V + rp.head + N - 1) / N;
    rp.ok = (si.lseP - si.lseP == 0.0) ? 1 : 0;                      // finite
    rp.bonus = (force_bonus || si.mode == 1 || !(si.lseD - si.lseD == 0.0)) ? 1 : 0;
    const double LP = si.lseP / kLn2;
    rp.refP = ref_for_norm<BF16>(LP, rp.sc);
    const double rP = -LP - ref_offset<BF16>(rp.refP, rp.sc);          // p_i = 2^(y_i + rP)
    rp.scale = exp2(rP);
    rp.Dv = nullptr; rp.D = nullptr; rp.refQ = 0.f; rp.k_hi = 0.f; rp.k_lo = 0.f;
    rp.thP = rp.thQ = -INFINITY; rp.cutP = rp.cutQ = 0x7fffffff;
    if (filters) {
        const RowFilter f = filters[(int64_t)B * g + (int64_t)b * (g + 1) + si.row];
        rp.thP = f.theta; rp.cutP = f.idx_cut;
        if (!rp.bonus) {
            const RowFilter fq = (draft_filters ? draft_filters : filters)[(int64_t)b * g + (si.row < g ? si.row : g - 1)];
            rp.thQ = fq.theta; rp.cutQ = fq.idx_cut;
        }
    }
    if (!rp.bonus) {
        const int jd = si.row < g ? si.row : g - 1;
        const char* rowD = (const char*)draft + ((int64_t)b * g + jd) * draft_ld * ES;
        const uintptr_t aD = (uintptr_t)rowD;
        rp.D = rowD;
        if ((int32_t)((aD & 15) / ES) == rp.head) rp.Dv = (const uint4*)(aD & ~(uintptr_t)15);
        const double LD = si.lseD / kLn2;
        rp.refQ = ref_for_norm<BF16>(LD, rp.sc);
        const double rQ = -LD - ref_offset<BF16>(rp.refQ, rp.sc);
        const double kappa = exp2(rQ - rP);
        rp.k_hi = (float)kappa;
        rp.k_lo = (float)(kappa - (double)rp.k_hi);
    }
}

// The 16-byte chunks c of the target row and (when it shares the alignment) of the draft row.  In the first
// and last chunk the elements that lie outside the row are replaced by -inf logits (weight 0), so the weight
// loop needs no guard.
//
// MODE (here and in chunk_weights_loaded): what kind of weights the row pair asks for is the same for every chunk of
// a sweep, so the sweep decides it once and runs straight-line code.  kModeAny: look at rp for every chunk (same
// arithmetic, for the few chunks of a selection); kModeBonus: p itself; kModeResidualVec: max(0, p - kappa q) with
// the draft row on the target row's chunk grid; kModeResidualElem: the same with element loads of the draft row.
constexpr int kModeAny = 0, kModeBonus = 1, kModeResidualVec = 2, kModeResidualElem = 3;

template <bool BF16, int MODE = kModeAny>
__device__ __forceinline__ void load_chunk_pair(const RowPair& rp, int64_t c, uint4& vp, uint4& vd)
{
    constexpr int N = BF16 ? 8 : 4;
    vp = make_uint4(0, 0, 0, 0);
    vd = make_uint4(0, 0, 0, 0);
    if (c < rp.nchunks) {
        vp = load_stream(rp.Pv + c);
        const bool dvec = MODE == kModeAny ? (!rp.bonus && rp.Dv != nullptr) : MODE == kModeResidualVec;
        if (dvec) vd = load_stream(rp.Dv + c);
        if (c == 0 || c == rp.nchunks - 1) {
            const int32_t e0 = (int32_t)(c * N) - rp.head;
            uint32_t* wp = (uint32_t*)&vp;
            uint32_t* wd = (uint32_t*)&vd;
#pragma unroll
            for (int k = 0; k < N; ++k) {
                if (e0 + k >= 0 && e0 + k < rp.V) continue;
                if (BF16) {
                    const uint32_t m = (k & 1) ? 0x0000ffffu : 0xffff0000u, v = (k & 1) ? 0xff800000u : 0x0000ff80u;
                    wp[k >> 1] = (wp[k >> 1] & m) | v;
                    wd[k >> 1] = (wd[k >> 1] & m) | v;
                } else {
                    wp[k] = 0xff800000u;
                    wd[k] = 0xff800000u;
                }
            }
        }
    }
}

// Weights of the N elements of chunk c (0 for elements outside the row) and their fp32 sum in index
// order, from chunks already loaded.
template <bool BF16, bool FILT = false, int MODE = kModeAny>
__device__ __forceinline__ float chunk_weights_loaded(const RowPair& rp, int64_t c, const uint4& vp, const uint4& vd, float* w)
{
    constexpr int N = BF16 ? 8 : 4;
    if (c >= rp.nchunks) {
#pragma unroll
        for (int k = 0; k < N; ++k) w[k] = 0.f;
        return 0.f;
    }
    const int32_t e0 = (int32_t)(c * N) - rp.head;
    const bool bonus = MODE == kModeAny ? rp.bonus != 0 : MODE == kModeBonus;
    const bool dvec = MODE == kModeAny ? (!rp.bonus && rp.Dv != nullptr) : MODE == kModeResidualVec;
    // Out-of-row elements of an edge chunk arrive as -inf logits (load_chunk_pair), so the loop carries no
    // per-element guard; a NaN weight is dropped by the max with 0.
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const int32_t e = e0 + k;
        const float xp = chunk_elem<BF16>(vp, k);
        float ep = fast_exp2(exp_arg<BF16>(xp, rp.refP, rp.sc));
        if (FILT && !(xp > rp.thP || (xp == rp.thP && e <= rp.cutP))) ep = 0.f;
        float wk;
        if (bonus) {
            wk = fmaxf(ep, 0.f);
        } else {
            float xd;
            if (dvec) xd = chunk_elem<BF16>(vd, k);
            else xd = (e >= 0 && e < rp.V) ? load_logit<BF16>(rp.D, e) : 0.f;
            float eq = fast_exp2(exp_arg<BF16>(xd, rp.refQ, rp.sc));
            if (FILT && !(xd > rp.thQ || (xd == rp.thQ && e <= rp.cutQ))) eq = 0.f;
            wk = fmaxf(0.f, __builtin_fmaf(-rp.k_lo, eq, __builtin_fmaf(-rp.k_hi, eq, ep)));
        }
        w[k] = wk;
        sum += wk;
    }
    return sum;
}

template <bool BF16, bool FILT = false>
__device__ __forceinline__ float chunk_weights(const RowPair& rp, int64_t c, float* w)
{
    uint4 vp, vd;
    load_chunk_pair<BF16>(rp, c, vp, vd);
    return chunk_weights_loaded<BF16, FILT>(rp, c, vp, vd, w);
}

// A draw from p itself (bonus weights) out of ONE slab of target row j.  On a row whose split-row partials were taken
// over contiguous slabs (the statistics pass does that for the rows such a draw can come from), every partial is the
// mass of one contiguous range of tokens, in index order, so the slab that holds the draw follows from the partials
// and the sampling uniform u alone: an inverse CDF over at most 64 slab masses.  Returns false when the row has
// ragged ends or the partials carry no usable mass (the caller then sweeps the whole row); otherwise the slab's
// chunks [lo, hi) and where in its mass to land (frac, to be used as the uniform of a draw from the slab alone).
// Called by one whole wavefront; the results are wavefront-uniform.
template <bool BF16>
__device__ __forceinline__ bool pick_row_slab(const void* target, int64_t target_ld, int32_t gamma, int32_t V, int32_t B, int b, int j,
                                              const Partial* parts, int nparts, double u, int lane,
                                              int64_t& lo, int64_t& hi, double& frac)
{
    constexpr int ES = BF16 ? 2 : 4;
    const int g = gamma;
    lo = 0; hi = 0; frac = 0.0;
    const RowGeom geo = make_geom<BF16>((const char*)target + ((int64_t)b * (g + 1) + j) * target_ld * ES, V);
    if (!(geo.edge_lo_end == 0 && geo.edge_hi_begin == V)) return false;   // ragged ends: the slabs are not all of the row
    const Partial* ps = parts + ((int64_t)B * g + (int64_t)b * (g + 1) + j) * nparts;
    double S = 0.0, br = 0.0;
    if (lane < nparts) { S = ps[lane].S; br = ps[lane].bref; }
    const bool has = S > 0.0 && S < INFINITY;
    const double bmin = wave_min(has ? br : (double)INFINITY);
    const double W = has ? S * exp2_offset_diff(bmin - br) : 0.0;              // the slab's mass against a common reference
    const double incl = wave_inclusive_scan(W, lane);
    const double Z = __shfl(incl, 63, 64);
    const double target_mass = u * Z;
    const unsigned long long hit = __ballot(incl > target_mass);
    const int src = hit ? __ffsll((long long)hit) - 1 : 0;
    const double w_src = __shfl(W, src, 64), excl = __shfl(incl - W, src, 64);
    bool ok = Z > 0.0 && Z < INFINITY && hit && w_src > 0.0;
    double f = ok ? (target_mass - excl) / w_src : 0.0;
    f = f < 0.0 ? 0.0 : (f > 0.999999999 ? 0.999999999 : f);
    int64_t seg_lo, seg_hi;
    wave_slab(geo, src / kWaves, nparts / kWaves, src % kWaves, seg_lo, seg_hi, lo, hi);
    if (hi <= lo) ok = false;
    frac = f;
    return ok;
}

// A row pair narrowed to the chunks [lo, hi) of the target row, as a row of its own (bonus weights only).
template <bool BF16>
__device__ __forceinline__ void narrow_to_slab(RowPair& rp, int64_t lo, int64_t hi)
{
    constexpr int N = BF16 ? 8 : 4;
    rp.Pv += lo;                                                   // head is 0 on rows that have slabs
    rp.nchunks = hi - lo;
    rp.V = (int32_t)((hi - lo) * N);
}

// A sweep of up to this many tiles can leave every lane's chunk sums in shared memory (1 KB per tile) for
// select_token, in the kernels whose workgroup has a compute unit to itself.
constexpr int kSumsKeepTiles = 80;

// Weight of one tile: lanes take chunks tile*256 + g*64 + lane, g = 0..3.  Every lane returns the sum.
// keep: shared-memory copy of the target row's chunks for select_token (indexed by chunk), or null.
// sums: shared memory for the lanes' four chunk sums of every tile ([tile][lane]), which select_token then need
// not rebuild from the row; or null.
template <bool BF16>
__device__ __forceinline__ double tile_weight_of(const RowPair& rp, int64_t tile, int lane, const uint4* vp, const uint4* vd,
                                                 uint4* keep, float4* sums)
{
    constexpr int N = BF16 ? 8 : 4;
    if (keep != nullptr) {
#pragma unroll
        for (int g = 0; g < kTileChunks; ++g) {
            const int64_t c = tile * (64 * kTileChunks) + g * 64 + lane;
            if (c < rp.nchunks) keep[c] = vp[g];
        }
    }
    double acc = 0.0;
    float cs[kTileChunks];
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) {
        float w[N];
        cs[g] = chunk_weights_loaded<BF16>(rp, tile * (64 * kTileChunks) + g * 64 + lane, vp[g], vd[g], w);
        acc += (double)cs[g];
    }
    if (sums != nullptr) sums[tile * 64 + lane] = make_float4(cs[0], cs[1], cs[2], cs[3]);
    return wave_sum(acc) * rp.scale;
}

template <bool BF16>
__device__ __forceinline__ double tile_weight(const RowPair& rp, int64_t tile, int lane, uint4* keep = nullptr,
                                              float4* sums = nullptr)
{
    uint4 vp[kTileChunks], vd[kTileChunks];
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) load_chunk_pair<BF16>(rp, tile * (64 * kTileChunks) + g * 64 + lane, vp[g], vd[g]);
    return tile_weight_of<BF16>(rp, tile, lane, vp, vd, keep, sums);
}

// One tile's chunks of a lane, fetched ahead of the weights (ok: wavefront-uniform, the chunks are there).  Four named
// members rather than an array, so that the chunks stay in registers on their way through the callers.
struct TilePre {
    uint4 v0, v1, v2, v3;
    bool ok;
};
static_assert(kTileChunks == 4, "TilePre holds one tile's four chunks per lane");

// The lane's chunks of tile `tile` of a slab [lo, lo + n) of a target row whose chunk grid starts at rowv (a row with
// slabs: no ragged ends, so no chunk needs patching), loaded before the row pair exists; zeros past the slab.
__device__ __forceinline__ TilePre tile_preload(const uint4* rowv, int64_t lo, int64_t n, int64_t tile, int lane)
{
    const int64_t c = tile * (64 * kTileChunks) + lane;
    TilePre t;
    t.v0 = t.v1 = t.v2 = t.v3 = make_uint4(0, 0, 0, 0);
    if (c < n) t.v0 = load_stream(rowv + lo + c);
    if (c + 64 < n) t.v1 = load_stream(rowv + lo + c + 64);
    if (c + 128 < n) t.v2 = load_stream(rowv + lo + c + 128);
    if (c + 192 < n) t.v3 = load_stream(rowv + lo + c + 192);
    t.ok = true;
    return t;
}

// Bonus weight of a tile of a row pair narrowed to that slab, from chunks tile_preload fetched.
template <bool BF16>
__device__ __forceinline__ double tile_weight_preloaded(const RowPair& rp, int64_t tile, int lane, const TilePre& pre,
                                                        uint4* keep = nullptr, float4* sums = nullptr)
{
    const uint4 vp[kTileChunks] = {pre.v0, pre.v1, pre.v2, pre.v3};
    uint4 vd[kTileChunks];
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) vd[g] = make_uint4(0, 0, 0, 0);
    return tile_weight_of<BF16>(rp, tile, lane, vp, vd, keep, sums);
}

// Two tiles with all their loads in flight together (twice the bytes per round trip).
template <bool BF16, bool FILT, int MODE>
__device__ __forceinline__ void tile_weight2_mode(const RowPair& rp, int64_t t0, int64_t t1, int lane, double& w0, double& w1,
                                                  float4* sums, int ntiles)
{
    constexpr int N = BF16 ? 8 : 4;
    uint4 vp[2][kTileChunks], vd[2][kTileChunks];
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) {
        load_chunk_pair<BF16, MODE>(rp, t0 * (64 * kTileChunks) + g * 64 + lane, vp[0][g], vd[0][g]);
        load_chunk_pair<BF16, MODE>(rp, t1 * (64 * kTileChunks) + g * 64 + lane, vp[1][g], vd[1][g]);
    }

    double a0 = 0.0, a1 = 0.0;
    float c0[kTileChunks], c1[kTileChunks];
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) {
        float w[N];
        c0[g] = chunk_weights_loaded<BF16, FILT, MODE>(rp, t0 * (64 * kTileChunks) + g * 64 + lane, vp[0][g], vd[0][g], w);
        c1[g] = chunk_weights_loaded<BF16, FILT, MODE>(rp, t1 * (64 * kTileChunks) + g * 64 + lane, vp[1][g], vd[1][g], w);
        a0 += (double)c0[g];
        a1 += (double)c1[g];
    }
    if (sums != nullptr) {
        sums[t0 * 64 + lane] = make_float4(c0[0], c0[1], c0[2], c0[3]);
        if (t1 < ntiles) sums[t1 * 64 + lane] = make_float4(c1[0], c1[1], c1[2], c1[3]);
    }
    w0 = wave_sum(a0) * rp.scale;
    w1 = wave_sum(a1) * rp.scale;
}

// The kind of weights is looked up once per pair of tiles (see kModeAny above): the element loops then carry no
// branch on it.
template <bool BF16, bool FILT = false>
__device__ __forceinline__ void tile_weight2(const RowPair& rp, int64_t t0, int64_t t1, int lane, double& w0, double& w1,
                                             float4* sums = nullptr, int ntiles = 0)
{
    if (rp.bonus) tile_weight2_mode<BF16, FILT, kModeBonus>(rp, t0, t1, lane, w0, w1, sums, ntiles);
    else if (rp.Dv != nullptr) tile_weight2_mode<BF16, FILT, kModeResidualVec>(rp, t0, t1, lane, w0, w1, sums, ntiles);
    else tile_weight2_mode<BF16, FILT, kModeResidualElem>(rp, t0, t1, lane, w0, w1, sums, ntiles);
}

// Tile weights may be rewritten by one lane and read by the others of the same wavefront (fallback
// below); global memory is read with device-scope loads so no stale first-level-cache line is seen.
template <bool LDS>
__device__ __forceinline__ double read_tile(const double* t)
{
    if (LDS) return *(const volatile double*)t;
    unsigned long long bits = __hip_atomic_load((const unsigned long long*)t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return __longlong_as_double((long long)bits);
}

// One wavefront selects the token from the tile weights: returns the token (all lanes), -1 if the
// weights carry no mass, or -2 if the caller should recompute the tiles as bonus weights (residual with
// Z == 0: p == q everywhere, or a broken draft row) and call again.
// raw: the target row's chunks as the sweep loaded them, kept in shared memory (bonus weights, whole chunks: the
// crossing tile is then not read from global memory again), or null.
// sums: every lane's four chunk sums of the tiles [sums_lo, sums_hi) as the sweep left them in shared memory
// ([tile][lane]), or null; with them only the one chunk that holds the crossing is rebuilt element by element.
template <bool BF16, bool LDS, bool FILT = false>
__device__ __forceinline__ int32_t select_token(const RowPair& rp, const double* tiles, int ntiles, double u, int lane,
                                                const uint4* raw = nullptr, const float4* sums = nullptr,
                                                int sums_lo = 0, int sums_hi = 0x7fffffff)
{
    constexpr int N = BF16 ? 8 : 4;
    const int per = (ntiles + 63) / 64;
    // ---- tile level: each lane sums a contiguous run of tiles, then a scan over lanes
    double mine = 0.0;
    for (int i = 0; i < per; ++i) {
        const int t = lane * per + i;
        if (t < ntiles) mine += read_tile<LDS>(tiles + t);
    }
    const double incl = wave_inclusive_scan(mine, lane);
    const double Z = __shfl(incl, 63, 64);
    if (!(Z > 0.0) || !(Z - Z == 0.0)) return rp.bonus ? -1 : -2;
    const double target = u * Z;
    const unsigned long long hit = __ballot(incl > target);
    // The lane whose run of tiles holds the crossing walks it; if rounding hides the crossing it settles
    // for its last tile with weight.  With no such lane at all (rounding at the top end) the last lane that
    // holds weight does the same.
    const unsigned long long haveW = __ballot(mine > 0.0);
    if (!haveW) return -1;
    const int src = hit ? (__ffsll((long long)hit) - 1) : (63 - __clzll((long long)haveW));
    int tl = -1, tl_last = -1;
    double run = incl - mine, run_last = 0.0;                        // exclusive prefix of this lane
    for (int i = 0; i < per; ++i) {
        const int t = lane * per + i;
        if (t < ntiles && tl < 0) {
            const double wt = read_tile<LDS>(tiles + t);
            const double nx = run + wt;
            if (wt > 0.0) { tl_last = t; run_last = run; }
            if (nx > target) tl = t; else run = nx;
        }
    }
    const bool force_last = __shfl((int)(tl < 0), src, 64) != 0;
    if (tl < 0) { tl = tl_last; run = run_last; }
    const int tile = __shfl(tl, src, 64);
    const double before = __shfl(run, src, 64);
    if (tile < 0) return -1;
    // ---- inside the tile
    // the weights of the lane's chunk g of the tile, element by element (and their sum)
    auto chunk_w = [&](int g, float* wout) -> float {
        const int64_t c = (int64_t)tile * (64 * kTileChunks) + g * 64 + lane;
        if (raw != nullptr) {
            const uint4 none = make_uint4(0, 0, 0, 0);
            return chunk_weights_loaded<BF16, FILT>(rp, c, c < rp.nchunks ? raw[c] : none, none, wout);
        }
        return chunk_weights<BF16, FILT>(rp, c, wout);
    };
    const bool have_sums = sums != nullptr && tile >= sums_lo && tile < sums_hi;   // the sweep left every lane's chunk sums
    float w[kTileChunks][N];
    float cs[kTileChunks];
    if (have_sums) {
        const float4 k = sums[tile * 64 + lane];
        cs[0] = k.x; cs[1] = k.y; cs[2] = k.z; cs[3] = k.w;
    } else {
#pragma unroll
        for (int g = 0; g < kTileChunks; ++g) cs[g] = chunk_w(g, w[g]);
    }
    double base = before;
    int found_g = -1, found_lane = -1;
    double found_excl = 0.0;
#pragma unroll
    for (int g = 0; g < kTileChunks; ++g) {
        const double v = (double)cs[g] * rp.scale;
        const double inc = wave_inclusive_scan(v, lane);
        const unsigned long long h = force_last ? 0ull : __ballot(base + inc > target);
        if (h && found_g < 0) {
            found_g = g;
            found_lane = __ffsll((long long)h) - 1;
            found_excl = base + __shfl(inc - v, found_lane, 64);
        }
        base += __shfl(inc, 63, 64);
    }
    int32_t tok = -1;
    if (found_g >= 0) {
        // the elements of the one chunk that holds the crossing: rebuilt now (one chunk per lane instead of the
        // tile's four) when the sums came from the sweep
        float ws[N];
        if (have_sums) {
            chunk_w(found_g, ws);
        } else {
#pragma unroll
            for (int g = 0; g < kTileChunks; ++g) {
                if (g != found_g) continue;
#pragma unroll
                for (int k = 0; k < N; ++k) ws[k] = w[g][k];
            }
        }
        if (lane == found_lane) {
            double r = found_excl;
            int32_t lastpos = -1;
            const int64_t c = (int64_t)tile * (64 * kTileChunks) + found_g * 64 + lane;
#pragma unroll
            for (int k = 0; k < N; ++k) {
                if (ws[k] > 0.f) lastpos = (int32_t)(c * N) + k - rp.head;
                r += (double)ws[k] * rp.scale;
                if (tok < 0 && r > target) tok = (int32_t)(c * N) + k - rp.head;
            }
            if (tok < 0) tok = lastpos;
        }
        tok = __shfl(tok, found_lane, 64);
    } else {
        // the last element of the tile with positive weight
        if (have_sums) {
#pragma unroll
            for (int g = 0; g < kTileChunks; ++g) chunk_w(g, w[g]);
        }
        int32_t lastpos = -1;
#pragma unroll
        for (int g = 0; g < kTileChunks; ++g) {
            const int64_t c = (int64_t)tile * (64 * kTileChunks) + g * 64 + lane;
#pragma unroll
            for (int k = 0; k < N; ++k)
                if (w[g][k] > 0.f) { const int32_t e = (int32_t)(c * N) + k - rp.head; lastpos = e > lastpos ? e : lastpos; }
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) { const int32_t o = __shfl_xor(lastpos, m, 64); lastpos = o > lastpos ? o : lastpos; }
        tok = lastpos;
    }
    return tok;
}

}  // namespace hola
