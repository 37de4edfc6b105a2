// Gate scoring and causal top-k on bf16 MFMA (paper Section 2; Appendix C.1, fused
// top-k selection: scores are produced tile by tile and never written to memory).
//
// Scores must be fp32-accurate (the routing is compared with a 1e-4 score gap), so the
// fp32 centroids are split into three bf16 terms hi + mid + lo (24 mantissa bits); the
// queries are bf16 already, every product is exact in fp32 and only the fp32 accumulation
// rounds.  A workgroup of two waves owns 64 consecutive queries; the waves take alternate
// centroid tiles of the queries' past blocks: 16 blocks x 64 queries per step, 3 terms x d/32
// MFMAs per 16 queries.
//
// Selection replaces the paper's per-row insertion sort (k = 64 of ~1000 candidates makes
// insertion far too long) by a search that recomputes the cheap scores instead of storing them.
//
// First look (approximate): scores from the hi term alone -- a third of the operand loads and
// MFMAs, within about 2^-8 of the score's scale.  One sweep finds about the largest score of
// every query, a second one histograms the order-preserving integer keys of the scores below it
// into 64 bins (LDS integer atomics) and walks the bins to the one that holds the k-th largest
// approximate score.  That bin, widened by the error of the first look, is a band [lo, hi) of
// scores in which the k-th largest EXACT score is expected.
// Decision (exact): one sweep with all three terms marks every block with score >= hi ("sure") in
// a per-query bit row and collects the few blocks inside the band with their exact keys; with S
// sure blocks and C collected ones, S <= k <= S + C proves that the kept set is the sure blocks
// plus the best k - S of the collected ones (ties: lower block) -- whatever the first look got
// wrong can only break that inequality, never the result.
// Queries that fail the test (a band with more blocks than the collection holds: many equal
// scores; non-finite scores) fall back to the exact radix search: each sweep histograms the exact
// keys of the still-undecided interval of every query, the bin that holds the k-th largest key
// becomes the next interval, until that bin holds exactly as many keys as are still needed, few
// enough to collect, or is one key wide (ties; the lower block index wins).
// The bit rows are written out in ascending block order.
#include <type_traits>

#include "mfma.h"

namespace moba {

constexpr int kHistWords = 32;            // exact search: 64 bins of 16 bits per query
constexpr int kHistStride = 65;           // first look: 64 bins of 32 bits; odd row stride: queries land on different LDS banks
constexpr int kCand = 32;                 // blocks inside a band that the ranking takes
constexpr int kRecWave = 512;             // records (blocks inside bands) a wave can write during one marking sweep
constexpr int kCandExact = kRecWave / 64; // exact search: a final bin this small is collected (64 queries always fit one wave's records)
constexpr int kBandBins = 24;             // first look: a bin with more approximate scores than this is cut again
constexpr int kLookSweeps = 3;            // histogram sweeps of the first look at most
constexpr int kTopkMfmaMaxBlocks = 16384; // the bit rows of a strip (8 bytes per block) still fit the LDS; 16-bit bins and block ids hold it

// c3 <- the three bf16 terms of the fp32 centroids, in MFMA operand order: the 16 bytes lane
// (m, g) feeds to the MFMA for blocks 16 jt + m, channels 32 ks + 8 g .. + 8, term t, sit at
// (((slice * ntile + jt) * 3 + t) * (D / 32) + ks) * 1024 + 16 * lane, so that one load
// instruction of a wave covers 1 KB of consecutive bytes.  Blocks beyond n read as zero.
template <int D>
__global__ void split3_kernel(const float* __restrict__ c, bf16_t* __restrict__ out, int n, int ntile,
                              int64_t chunks)
{
    constexpr int KS = D / 32;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= chunks) return;
    const int lane = (int)(i % 64), ks = (int)((i / 64) % KS), term = (int)((i / (64 * KS)) % 3);
    const int64_t tile = i / (64 * KS * 3);
    const int jt = (int)(tile % ntile);
    const int64_t s = tile / ntile;
    const int row = 16 * jt + (lane & 15), g = lane >> 4;
    bf16_t o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float x = row < n ? c[(s * n + row) * D + 32 * ks + 8 * g + e] : 0.f;
        const bf16_t hi = f32_to_bf16(x);
        const float r1 = x - bf16_to_f32(hi);
        const bf16_t mid = f32_to_bf16(r1);
        const float r2 = r1 - bf16_to_f32(mid);
        o[e] = term == 0 ? hi : term == 1 ? mid : f32_to_bf16(r2);
    }
    *reinterpret_cast<uint4*>(out + i * 8) = *reinterpret_cast<const uint4*>(o);
}

// the score whose order_key is `key`; `none` when the key does not belong to a number
__device__ __forceinline__ float key_score(uint32_t key, float none)
{
    const uint32_t bits = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    return (bits & 0x7fffffffu) > 0x7f800000u ? none : __uint_as_float(bits);
}

// One wave's share (tiles tile_lo, tile_lo + step, ...) of a sweep over the centroid tiles of a
// 64-query strip.  f(qt, sc, j0): sc[i] is the score of
// query 16*qt + m16 against block j0 + i (j0 = 16*tile + 4*g).
// TOP = 2: the fp32-accurate score from all three terms; TOP = 0: the hi term alone, a third of the
// loads and MFMAs, within about 2^-8 of the score's scale.
// The operands of a tile are loaded a whole tile ahead into a second set of registers (the loop
// is unrolled by two so that the sets swap without copies): a load that is waited for in the
// iteration that issues it leaves the wave idle for an L2 round trip per tile.
template <int D, int TOP, typename F>
__device__ __forceinline__ void sweep_tiles(const char* __restrict__ c3s, int tile_lo, int tile_hi,
                                            int step, const Frag (&qb)[4][D / 32], int lane, int g, F f)
{
    constexpr int KS = D / 32;
    if (tile_lo >= tile_hi) return;
    Frag a[2][TOP + 1][KS];
    auto load = [&](int buf, int jt) {
        const char* tb = c3s + (int64_t)jt * (3 * KS * 1024) + lane * 16;
#pragma unroll
        for (int term = 0; term <= TOP; ++term)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                a[buf][term][ks].q = *reinterpret_cast<const uint4*>(tb + (term * KS + ks) * 1024);
    };
    auto compute = [&](int buf, int jt) {
        // the four 16-query tiles are independent accumulation chains: issue them interleaved so
        // that no MFMA waits for the one before it
        f32x4_t sc[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) sc[qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int term = TOP; term >= 0; --term)       // smallest terms first
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int qt = 0; qt < 4; ++qt) sc[qt] = mfma16(a[buf][term][ks], qb[qt][ks], sc[qt]);
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) f(qt, sc[qt], 16 * jt + 4 * g);
    };
    int jt = tile_lo;
    load(0, jt);
    // (past the last tile the loads repeat that tile: unconditional, always valid)
    // The compiler would move each load down to the block of its first use (past the loop's exit
    // test), next to the MFMAs that wait for it: the scheduling barrier keeps it above the tile's
    // work, and an empty asm statement that names the loaded registers, after that work, keeps it
    // in this block.
    auto pin = [&](int buf) {
#pragma unroll
        for (int term = 0; term <= TOP; ++term)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(a[buf][term][ks].n));
    };
    while (true) {
        const int n1 = jt + step;
        load(1, n1 < tile_hi ? n1 : jt);
        __builtin_amdgcn_sched_barrier(0);
        compute(0, jt);
        __builtin_amdgcn_sched_barrier(0);
        pin(1);
        if (n1 >= tile_hi) break;
        const int n2 = n1 + step;
        load(0, n2 < tile_hi ? n2 : n1);
        __builtin_amdgcn_sched_barrier(0);
        compute(1, n1);
        __builtin_amdgcn_sched_barrier(0);
        pin(0);
        if (n2 >= tile_hi) break;
        jt = n2;
    }
}

constexpr int kTopkWaves = 2;             // waves per 64-query strip (= per workgroup)
// The kept blocks of a query are collected in LDS either as a bit row over the n blocks (KL = 0)
// or as a list of at most KL block ids: 16 for a small top-k (2 KB per strip instead of 8 n
// bytes: with thousands of blocks the bit rows would cap the workgroups per CU), 64 for a top-k
// up to 64 of more than kBitRowBlocks blocks (8 KB per strip where the bit rows would take 32 KB
// and more; each kept block costs a returning LDS atomic there, which only pays when few of the
// blocks that go by are kept).
constexpr int kKeptList = 16;
constexpr int kKeptListLong = 64;
constexpr int kBitRowBlocks = 4096;

// states of a query
enum : uint32_t {
    kUndecided = 0,   // the search goes on in [lo, hi), 64 bins of 2^sh keys
    kKeepFrom = 1,    // keep every block with key >= lo
    kKeepTies = 2,    // keep key > lo and the lowest blocks among key == lo
    kBand = 3,        // keep score >= thi and the best of the blocks with tlo <= score < thi
    kDone = 4
};

template <int D, int KL>
__global__ __launch_bounds__(kTopkWaves * kWave) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2)))
void topk_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ c3, int ntile_all,
    int32_t* __restrict__ idx, int N, int B, int n, int k, int strips_per_slice, int Wn, int G,
    int exact_only, const int32_t* __restrict__ blk_first)
{
    extern __shared__ uint32_t smem[];
    constexpr int KS = D / 32;
    constexpr bool LISTS = KL > 0;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int m16 = lane & 15, g = lane >> 4;
    const int strip = blockIdx.x;
    uint32_t* hist = smem;
    uint32_t* st_lo = hist + 64 * kHistStride + 64;   // (the first look's rows start one word in, see there)
    uint32_t* st_sh = st_lo + 64;
    uint32_t* st_need = st_sh + 64;                // blocks still to find inside the current interval
    uint32_t* st_state = st_need + 64;
    uint32_t* st_past = st_state + 64;             // candidates of the query: blocks first .. past - 1
    uint32_t* st_first = st_past + 64;
    uint32_t* st_hi = st_first + 64;                // the current interval is [lo, hi): at most 64 bins of 2^sh keys
    float* st_tlo = reinterpret_cast<float*>(st_hi + 64);   // marking thresholds, see kBand
    float* st_thi = st_tlo + 64;
    uint32_t* st_cnt = reinterpret_cast<uint32_t*>(st_thi + 64);   // marking: blocks met inside the band
    float* st_top = reinterpret_cast<float*>(st_cnt + 64);         // first look: about the largest |score|,
    float* st_min = st_top + 64;                                   //   about the smallest score,
    float* st_a = st_min + 64;                                     //   the window [a, a + 64 w) of the histogram,
    float* st_w = st_a + 64;
    uint32_t* st_open = reinterpret_cast<uint32_t*>(st_w + 64);    //   whether its last bin also takes everything above
    uint32_t* st_off = st_open + 64;               // marking: where the query's records start, and
    uint32_t* st_fill = st_off + 64;               //   the next free place among them
    uint32_t* wrec = st_fill + 64;                 // [kTopkWaves, padded to 64] records each wave wrote
    uint32_t* selm = wrec + 64;                    // [64][Wn] kept-block bits, or:
    uint16_t* lst = reinterpret_cast<uint16_t*>(selm);      // [64][KL] kept blocks, any order
    uint32_t* lcnt = selm + 64 * KL / 2;                    // [64] their number
    const int sel_words = LISTS ? 64 * KL / 2 + 64 : 64 * Wn;
    // one more kept block of query q (concurrent callers) / (only caller for q)
    auto keep_atomic = [&](int q, int blk) {
        if constexpr (LISTS) {
            const uint32_t slot = atomicAdd(&lcnt[q], 1u);
            if (slot < (uint32_t)KL) lst[q * KL + slot] = (uint16_t)blk;
        } else {
            atomicOr(&selm[q * Wn + (blk >> 5)], 1u << (blk & 31));
        }
    };
    auto keep_plain = [&](int q, int blk) {
        if constexpr (LISTS) {
            const uint32_t slot = lcnt[q]++;
            if (slot < (uint32_t)KL) lst[q * KL + slot] = (uint16_t)blk;
        } else {
            selm[q * Wn + (blk >> 5)] |= 1u << (blk & 31);
        }
    };
    // forget the kept blocks of query q
    auto kept_clear = [&](int q) {
        if constexpr (LISTS) lcnt[q] = 0u;
        else for (int w = 0; w < Wn; ++w) selm[q * Wn + w] = 0u;
    };

    const int s = strip / strips_per_slice;
    // (the late strips of a slice, which have the most candidates, start first: the kernel then
    // ends on short strips)
    const int t0 = (strips_per_slice - 1 - strip % strips_per_slice) * 64;
    const int rows_here = min(64, N - t0);
    const char* c3s = reinterpret_cast<const char*>(c3) + (int64_t)(s / G) * ntile_all * (3 * KS * 1024);   // G query heads share the centroids
    int32_t* out = idx + ((int64_t)s * N + t0) * k;

    if (wave == 0) {   // lane = query: initial state
        // (packed variable-length batches: the blocks of a query's own sequence start at blk_first)
        const int own = lane < rows_here ? (t0 + lane) / B : 0;
        const int first = blk_first && lane < rows_here ? blk_first[own] : 0;
        const int past = own - first;                          // number of candidates
        st_past[lane] = own;
        st_first[lane] = first;
        st_lo[lane] = 0u;
        st_sh[lane] = 26u;
        st_hi[lane] = 0xffffffffu;
        st_need[lane] = (uint32_t)min(k, past);
        st_state[lane] = past <= k ? kKeepFrom : kUndecided;      // few candidates: keep them all (every key >= 0)
        st_tlo[lane] = -INFINITY;
        st_thi[lane] = -INFINITY;
        st_cnt[lane] = (uint32_t)min(k, past);   // (first look: blocks still to find inside the window)
        st_top[lane] = 0.f;
        st_min[lane] = 0.f;
        st_a[lane] = 0.f;
        st_w[lane] = 0.f;
        st_open[lane] = 0u;
    }
    for (int i = tid; i < sel_words; i += kTopkWaves * kWave) selm[i] = 0u;
    const int pmax = (t0 + rows_here - 1) / B;
    const int ntile = (pmax + 15) / 16;
    // first candidate block of the strip's first and last query (the queries of a strip are
    // consecutive, so these are the smallest and the largest)
    const int fmin = blk_first ? blk_first[t0 / B] : 0;
    const int fmax = blk_first ? blk_first[pmax] : 0;
    const int tbeg = fmin / 16;

    Frag qb[4][KS];
#pragma unroll
    for (int qt = 0; qt < 4; ++qt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int64_t r = min(t0 + 16 * qt + m16, N - 1);
            qb[qt][ks].q = *reinterpret_cast<const uint4*>(Q + ((int64_t)s * N + r) * D + 8 * g + 32 * ks);
        }
    __syncthreads();

    // Interior tiles hold only blocks that are candidates of every query of the strip; the tiles
    // before and after them need the per-query test.  The waves of the strip take alternate tiles
    // (every sm-th tile in a sampled sweep): tile t belongs to wave ((t - tbeg) / sm) mod waves.
    const int ihi = min(ntile, (t0 / B) / 16);
    const int ilo = min(ihi, max(tbeg, (fmax + 15) / 16));
    auto sweep_any = [&](auto top, int tlo, int thi, int sm, auto f) {
        constexpr int TOP = decltype(top)::value;
        const int step = kTopkWaves * sm, base = tbeg + sm * wave;
        auto segment = [&](int a, int b, auto checked) {
            a = max(a, max(tlo, tbeg));
            b = min(b, thi);
            const int first = a <= base ? base : base + (a - base + step - 1) / step * step;
            sweep_tiles<D, TOP>(c3s, first, b, step, qb, lane, g,
                                [&](int qt, const f32x4_t& sc, int j0) { f(qt, sc, j0, checked); });
        };
        segment(tbeg, ilo, std::true_type());
        segment(ilo, ihi, std::false_type());
        segment(ihi, ntile, std::true_type());
    };
    auto sweep = [&](int tlo, int thi, auto f) { sweep_any(std::integral_constant<int, 2>(), tlo, thi, 1, f); };
    // every sm-th tile only, scores from the hi term alone
    auto sweep_sample = [&](int sm, auto f) { sweep_any(std::integral_constant<int, 0>(), 0, ntile, sm, f); };

    // ---- first look, on hi-term scores (a third of the operand loads and MFMAs; the selection
    // below does not depend on these being right).
    // Where to look: the largest and the smallest score of every undecided query, over all its
    // blocks when there are few tiles, over every sm-th tile otherwise.  The first window is
    // [max / 4, max] (from the smallest score when no score is positive, or when the query keeps
    // more than a fifth of its candidates), 64 bins, open at the top (its last bin also takes
    // whatever lies above).
    const int sm = min(max((ntile - tbeg) / 8, 1), LISTS ? 8 : 4);
    if (!exact_only && __syncthreads_or(st_state[lane] == kUndecided)) {
        for (int i = tid; i < 64; i += kTopkWaves * kWave) { hist[i * kHistStride] = 0u; hist[i * kHistStride + 1] = 0xffffffffu; }
        uint32_t first4[4], span4[4];
        float mx4[4], mn4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            first4[qt] = st_first[16 * qt + m16];
            span4[qt] = st_past[16 * qt + m16] - first4[qt];
            mx4[qt] = -INFINITY;
            mn4[qt] = INFINITY;
        }
        __syncthreads();
        sweep_sample(sm, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
            if (decltype(tail)::value) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if ((uint32_t)(j0 + i) - first4[qt] < span4[qt]) { mx4[qt] = fmaxf(mx4[qt], sc[i]); mn4[qt] = fminf(mn4[qt], sc[i]); }
            } else {                               // (NaN scores are ignored here as in the counts)
                mx4[qt] = fmaxf(fmaxf(mx4[qt], sc[0]), fmaxf(sc[1], fmaxf(sc[2], sc[3])));
                mn4[qt] = fminf(fminf(mn4[qt], sc[0]), fminf(sc[1], fminf(sc[2], sc[3])));
            }
        });
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            atomicMax(&hist[(16 * qt + m16) * kHistStride], order_key(mx4[qt]));
            atomicMin(&hist[(16 * qt + m16) * kHistStride + 1], order_key(mn4[qt]));
        }
        __syncthreads();
        if (wave == 0 && st_state[lane] == kUndecided) {
            const float M = key_score(hist[lane * kHistStride], NAN);
            const float m = key_score(hist[lane * kHistStride + 1], NAN);
            float w = 0.f, a = 0.f;
            if (M >= m && fabsf(M) < INFINITY && fabsf(m) < INFINITY) {
                // (a query that keeps more than a fifth of its candidates looks at all of them)
                const bool many = 5u * st_cnt[lane] > st_past[lane] - st_first[lane];
                a = M > 0.f && !many ? fmaxf(0.25f * M, m) : m;
                const float top = M + (sm > 1 ? 0.5f : 0.0625f) * fabsf(M) + 1e-30f;
                w = (top - a) * (1.f / 64.f);
            }
            st_a[lane] = a;
            st_w[lane] = w > 0.f ? w : 0.f;            // 0: no first look for this query
            st_open[lane] = 1u;
            st_min[lane] = m;
            st_top[lane] = fabsf(M);
        }
        __syncthreads();
    }

    // Histogram sweeps until the bin of the k-th largest approximate score holds few enough
    // scores; that bin, widened by the error of the hi term (about 2^-8 of the scale of the
    // scores, taken from the largest one), becomes the query's band.
    for (int it = 0; it < kLookSweeps && !exact_only; ++it) {
        if (!__syncthreads_or(st_state[lane] == kUndecided && st_w[lane] > 0.f)) break;
        for (int i = tid; i < 64 * kHistStride; i += kTopkWaves * kWave) hist[i] = 0u;
        // bin = floor(x), x = (score - a) / w, taken from the mantissa of (x - 0.5) + 1.5 * 2^23
        // (off by one bin where x is a whole number, which the first look can afford), clamped
        // to -1 .. 64: a query's row of bins starts one word into its 65, so that scores below the
        // window (and queries without a window: x = -2) count into a word in front of it and
        // scores above a closed window into the word behind it, neither of which is ever read --
        // no branch and no compare per score.
        constexpr float kMagic = 12582912.f;                   // 1.5 * 2^23
        constexpr int kMagicBits = 0x4B400000;
        uint32_t first4[4], span4[4];
        float inv4[4], off4[4], cap4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            const float w = st_state[q] == kUndecided ? st_w[q] : 0.f;
            first4[qt] = st_first[q];
            span4[qt] = st_past[q] - first4[qt];
            inv4[qt] = w > 0.f ? 1.f / w : 0.f;
            off4[qt] = (w > 0.f ? -st_a[q] / w : -1.f) - 0.5f;
            cap4[qt] = kMagic + (st_open[q] ? 63.f : 64.f);    // open at the top: the last bin takes the rest
        }
        __syncthreads();
        sweep_sample(1, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
            uint32_t* row = hist + 1 + (16 * qt + m16) * kHistStride;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // (fminf takes a NaN to the cap, like the scores above the window)
                const float x = fmaxf(fminf(fmaf(sc[i], inv4[qt], off4[qt]) + kMagic, cap4[qt]), kMagic - 1.f);
                int bi = __float_as_int(x) - kMagicBits;
                if (decltype(tail)::value) bi = (uint32_t)(j0 + i) - first4[qt] < span4[qt] ? bi : -1;
                atomicAdd(&row[bi], 1u);
            }
        });
        __syncthreads();
        if (wave == 0 && st_state[lane] == kUndecided && st_w[lane] > 0.f) {     // lane = query: walk the bins from the top
            const uint32_t need = st_cnt[lane];
            const float a = st_a[lane], w = st_w[lane];
            const bool open = st_open[lane] != 0u;
            const uint32_t* row = hist + 1 + lane * kHistStride;
            uint32_t cum = 0, c = 0;
            int b = -1;
            for (int b0 = 60; b0 >= 0 && b < 0; b0 -= 4) {
                const uint32_t c4[4] = {row[b0], row[b0 + 1], row[b0 + 2], row[b0 + 3]};
#pragma unroll
                for (int u = 3; u >= 0; --u) {
                    if (b < 0) {
                        if (cum + c4[u] >= need) { b = b0 + u; c = c4[u]; }
                        else cum += c4[u];
                    }
                }
            }
            if (b < 0) {
                // fewer scores in the window than needed: go on below it, down to the smallest score
                const float m = st_min[lane];
                if (a > m) {
                    st_cnt[lane] = need - cum;
                    st_a[lane] = m;
                    st_w[lane] = (a - m) * (1.f / 64.f) + 1e-30f;
                    st_open[lane] = 0u;
                } else {
                    st_w[lane] = 0.f;                          // (sampled minimum too high, non-finite scores)
                }
            } else {
                const float lo = a + (float)b * w;
                const bool open63 = open && b == 63;
                if (c > (uint32_t)kBandBins) {
                    const float w2 = open63 ? 4.f * w : w * (1.f / 64.f);      // more room above / cut the bin into 64 again
                    st_cnt[lane] = need - cum;
                    st_a[lane] = lo;
                    st_w[lane] = lo + w2 > lo ? w2 : 0.f;     // (bins below the resolution of the scores: equal scores)
                    st_open[lane] = open63 ? 1u : 0u;
                } else {
                    const float eps = 0.00390625f * fmaxf(st_top[lane], fabsf(lo)) + 1e-37f;
                    st_tlo[lane] = lo - eps;
                    st_thi[lane] = open63 ? INFINITY : lo + w + eps;
                    st_state[lane] = kBand;
                }
            }
        }
        __syncthreads();
    }

    // ---- marking sweep over the exact scores, for every query that is not kUndecided or kDone:
    // blocks with score >= thi go to the kept blocks; blocks with tlo <= score < thi are written
    // as records (key, query << 16 | block) to the wave's own half of a buffer that lies over the
    // histograms.  A wave counts its records in a scalar register (ballot + popcount), so the
    // sweep never waits for an LDS atomic to come back.
    uint2* rec = reinterpret_cast<uint2*>(hist);                  // [kTopkWaves][kRecWave], then:
    uint2* sorted = rec + kTopkWaves * kRecWave;                  // [kTopkWaves * kRecWave] records by query
    static_assert(2 * kTopkWaves * kRecWave * sizeof(uint2) <= 64 * kHistStride * sizeof(uint32_t), "records lie over the histograms");
    auto mark = [&]() {
        for (int i = tid; i < 64; i += kTopkWaves * kWave) st_cnt[i] = 0u;
        // The sign of score - threshold is shifted into a mask, one bit per score (two instructions
        // per score and threshold, none of them waiting for a compare); a threshold of +0 is taken
        // as -0 so that a score of -0 does not come out below it.
        int past4[4], first4[4];
        uint32_t on4[4];
        float tlo4[4], thi4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            past4[qt] = (int)st_past[q];
            first4[qt] = (int)st_first[q];
            const uint32_t st = st_state[q];
            on4[qt] = st != kUndecided && st != kDone ? 0xfu : 0u;
            const float lo = st_tlo[q], hi = st_thi[q];
            tlo4[qt] = lo == 0.f ? -0.f : lo;
            thi4[qt] = hi == 0.f ? -0.f : hi;
        }
        __syncthreads();
        uint2* mine = rec + wave * kRecWave;
        uint32_t nrec = 0;                                        // the same in all lanes
        sweep(0, ntile, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
            uint32_t below_hi = 0, below_lo = 0;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                below_hi = __builtin_amdgcn_alignbit(below_hi, __float_as_uint(sc[i] - thi4[qt]), 31);
                below_lo = __builtin_amdgcn_alignbit(below_lo, __float_as_uint(sc[i] - tlo4[qt]), 31);
            }
            uint32_t ok = on4[qt];
            if (decltype(tail)::value)                            // blocks first .. past - 1 only
                ok &= ((1u << min(max(past4[qt] - j0, 0), 4)) - 1u) & ~((1u << min(max(first4[qt] - j0, 0), 4)) - 1u);
            const uint32_t bits = ~below_hi & ok;                 // score >= thi
            const uint32_t cand = below_hi & ~below_lo & ok;      // tlo <= score < thi
            if (__ballot(cand != 0u)) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool ci = (cand >> i) & 1u;
                    const uint64_t m = __ballot(ci);
                    if (m) {
                        const uint32_t slot = nrec + (uint32_t)lanes_below(m);
                        if (ci && slot < (uint32_t)kRecWave)
                            mine[slot] = make_uint2(order_key(sc[i]), ((uint32_t)(16 * qt + m16) << 16) | (uint32_t)(j0 + i));
                        nrec += (uint32_t)__popcll(m);
                    }
                }
            }
            if constexpr (LISTS) {
                uint32_t b = bits;
                while (b) {
                    keep_atomic(16 * qt + m16, j0 + __ffs(b) - 1);
                    b &= b - 1;
                }
            } else {
                if (bits) atomicOr(&selm[(16 * qt + m16) * Wn + (j0 >> 5)], bits << (j0 & 31));
            }
        });
        if (lane == 0) wrec[wave] = nrec;
        __syncthreads();
    };
    // After a marking sweep: the records are counted per query and put in query order (counting
    // sort); then, two threads per query, a band's records are ranked by (key descending, block
    // ascending); with S kept blocks so far the best need - S of them are kept as well.
    // A band that does not hold the k-th score (S > need or S + records < need), more records than
    // kCand, or a wave that ran out of room for records: `retry` sends the query to the exact
    // search, else it keeps what there is.
    auto resolve = [&](bool retry) {
        bool room = true;
#pragma unroll
        for (int wv = 0; wv < kTopkWaves; ++wv) room = room && wrec[wv] <= (uint32_t)kRecWave;
        const int q = tid >> 1, half = tid & 1;
        const bool band = st_state[q] == kBand;
        // 1. records per query (st_cnt is zero on entry)
        for (int wv = 0; wv < kTopkWaves; ++wv) {
            const int nr = (int)min(wrec[wv], (uint32_t)kRecWave);
            for (int r = tid; r < nr; r += kTopkWaves * kWave) atomicAdd(&st_cnt[rec[wv * kRecWave + r].y >> 16], 1u);
        }
        int kept = 0;
        if (band) {
            if constexpr (LISTS) {
                kept = (int)lcnt[q];
            } else {                               // the two threads of the query count alternate words
                for (int w = half; w < Wn; w += 8) {          // four reads in flight
                    uint32_t v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) v[u] = w + 2 * u < Wn ? selm[q * Wn + w + 2 * u] : 0u;
#pragma unroll
                    for (int u = 0; u < 4; ++u) kept += __popc(v[u]);
                }
                kept += __shfl_xor(kept, 1, 64);
            }
        }
        __syncthreads();
        // 2. where each query's records start (wave 0, lane = query)
        if (wave == 0) {
            const uint32_t c = st_cnt[lane];
            uint32_t incl = c;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t up = __shfl_up(incl, o, 64);
                if (lane >= o) incl += up;
            }
            st_off[lane] = incl - c;
            st_fill[lane] = incl - c;
        }
        __syncthreads();
        // 3. records in query order
        for (int wv = 0; wv < kTopkWaves; ++wv) {
            const int nr = (int)min(wrec[wv], (uint32_t)kRecWave);
            for (int r = tid; r < nr; r += kTopkWaves * kWave) {
                const uint2 v = rec[wv * kRecWave + r];
                sorted[atomicAdd(&st_fill[v.y >> 16], 1u)] = v;
            }
        }
        __syncthreads();
        // 4. the best of each band: how many of its records a query still wants (st_fill, free
        // again), then a thread per record ranks it among the records of its query
        bool fits = true;
        if (band) {
            const int met = (int)st_cnt[q];
            const int want = (int)min((uint32_t)k, st_past[q] - st_first[q]) - kept;
            fits = room && met <= kCand && want >= 0 && want <= min(met, kCand);
            if (half == 0) st_fill[q] = fits || !retry ? (uint32_t)max(want, 0) : 0u;
        } else if (half == 0) {
            st_fill[q] = 0u;
        }
        __syncthreads();
        {
            // (key, then lower block first) as one 64-bit number: larger = better
            auto order = [](const uint2& r) { return ((uint64_t)r.x << 32) | (uint64_t)(~r.y); };
            const int nrec_all = (int)(st_off[63] + st_cnt[63]);
            for (int r = tid; r < nrec_all; r += kTopkWaves * kWave) {
                const uint2 me = sorted[r];
                const int rq = (int)(me.y >> 16);
                const int want = (int)st_fill[rq];
                const int c = min((int)st_cnt[rq], kCand);
                const int base = (int)st_off[rq];
                if (want == 0 || r - base >= c) continue;            // (records beyond kCand are not ranked)
                const uint2* seg = sorted + base;
                const uint64_t mine64 = order(me);
                int rank = 0;
                // (eight records are read at a time, so that the loop waits for LDS once per eight)
                for (int o = 0; o < c; o += 8) {
                    uint2 v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = seg[min(o + u, c - 1)];          // unconditional loads
#pragma unroll
                    for (int u = 0; u < 8; ++u) rank += (int)(o + u < c) & (int)(order(v[u]) > mine64);
                }
                if (rank < want) keep_atomic(rq, (int)(me.y & 0xffffu));
            }
        }
        __syncthreads();
        if (half == 0 && st_state[q] != kUndecided && st_state[q] != kKeepTies) {
            if (band && !fits && retry) {
                kept_clear(q);
                st_lo[q] = 0u;
                st_sh[q] = 26u;
                st_hi[q] = 0xffffffffu;
                st_need[q] = min((uint32_t)k, st_past[q] - st_first[q]);
                st_state[q] = kUndecided;
            } else {
                st_state[q] = kDone;
            }
        }
        __syncthreads();
    };
    if (!exact_only) {
        mark();
        resolve(true);
    }

    // ---- exact radix search for the k-th largest key of every query still undecided.
    // Membership of a score in the query's current key interval is tested on the float itself
    // (two compares); only members pay for the key, the bin and the atomic.
    const bool leftovers = __syncthreads_or(st_state[lane] != kDone);
    while (__syncthreads_or(st_state[lane] == kUndecided)) {
        for (int i = tid; i < 64 * kHistStride; i += kTopkWaves * kWave) hist[i] = 0u;
        uint32_t lo4[4], sh4[4], first4[4], span4[4];
        float flo4[4], fhi4[4];
        bool act4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            lo4[qt] = st_lo[q]; sh4[qt] = st_sh[q];
            first4[qt] = st_first[q];
            span4[qt] = st_past[q] - first4[qt];
            act4[qt] = st_state[q] == kUndecided;
            flo4[qt] = key_score(lo4[qt], -INFINITY);
            const uint32_t hi = st_hi[q];
            fhi4[qt] = hi > 0xff800000u ? NAN : key_score(hi, NAN);   // NaN: no upper end
        }
        __syncthreads();
        sweep(0, ntile, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
            if (!act4[qt]) return;
            uint32_t* row = hist + (16 * qt + m16) * kHistStride;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bool in = sc[i] >= flo4[qt] && !(sc[i] >= fhi4[qt]);
                if (decltype(tail)::value) in = in && (uint32_t)(j0 + i) - first4[qt] < span4[qt];
                if (in) {
                    // (an interval open at the top: its last bin takes everything above as well)
                    const uint32_t bin = min((order_key(sc[i]) - lo4[qt]) >> sh4[qt], 63u);
                    atomicAdd(&row[bin >> 1], 1u << (16 * (bin & 1u)));
                }
            }
        });
        __syncthreads();
        if (wave == 0 && st_state[lane] == kUndecided) {     // lane = query: walk the bins from the top
            const uint32_t need = st_need[lane], lo = st_lo[lane], sh = st_sh[lane], hi = st_hi[lane];
            uint32_t cum = 0, c = 0;
            int b = 63;
            for (; b >= 0; --b) {
                c = (hist[lane * kHistStride + (b >> 1)] >> (16 * (b & 1))) & 0xffffu;
                if (cum + c >= need) break;
                cum += c;
            }
            if (b < 0 && lo > 0u) {
                // fewer keys in the interval than needed (only a guessed interval can
                // miss): go on below it, [0, lo) in at most 64 bins
                const int width = 32 - __clz((int)(lo - 1u));                 // lo > 0 here
                const uint32_t sh2 = (uint32_t)max(width - 6, 0);
                st_lo[lane] = 0u;
                st_need[lane] = need - cum;
                st_sh[lane] = sh2;
                st_hi[lane] = lo;
            } else {
                b = max(b, 0);                 // (only NaN scores can leave [0, ..) short: keep all)
                const uint32_t need2 = need - cum;
                const uint32_t lo2 = lo + ((uint32_t)b << sh);
                // the last bin of an interval that is open at the top and narrower than the keys
                // above it: [lo2, 2^32), not [lo2, lo2 + 2^sh)
                const bool open63 = b == 63 && hi == 0xffffffffu && (uint64_t)lo + (64ull << sh) < (1ull << 32);
                const uint32_t hi2 = open63 ? 0xffffffffu
                                            : (uint32_t)min((uint64_t)lo2 + (1ull << sh), (uint64_t)hi);   // the chosen bin
                st_lo[lane] = lo2;
                st_hi[lane] = hi2;
                st_need[lane] = need2;
                const float flo = key_score(lo2, -INFINITY);
                uint32_t state = kUndecided;
                if (c == need2) state = kKeepFrom;
                else if (open63) {
                    if (c <= (uint32_t)kCandExact) state = kBand;
                    else st_sh[lane] = (uint32_t)max(32 - __clz((int)(0xffffffffu - lo2)) - 6, 0);   // 64 bins over [lo2, 2^32)
                }
                else if (sh == 0u) state = kKeepTies;
                else if (c <= (uint32_t)kCandExact) state = kBand;
                else st_sh[lane] = sh >= 6u ? sh - 6u : 0u;                     // cut the bin into 64 again
                if (state == kKeepFrom) { st_tlo[lane] = flo; st_thi[lane] = flo; }
                if (state == kKeepTies) {                                       // score > the threshold now, ties below
                    const float above = lo2 == 0xffffffffu ? INFINITY : key_score(lo2 + 1u, INFINITY);
                    st_tlo[lane] = above;
                    st_thi[lane] = above;
                }
                if (state == kBand) {
                    st_tlo[lane] = flo;
                    st_thi[lane] = hi2 > 0xff800000u ? INFINITY : key_score(hi2, INFINITY);   // nothing above
                }
                st_state[lane] = state;
            }
        }
        __syncthreads();
    }

    if (leftovers) {
        bool strict4[4];
        uint32_t first4[4], span4[4];
        float thr4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            strict4[qt] = st_state[q] == kKeepTies;
            first4[qt] = st_first[q];
            span4[qt] = st_past[q] - first4[qt];
            thr4[qt] = key_score(st_lo[q], -INFINITY);
        }
        mark();
        resolve(false);
        // ties at the threshold: the lowest block indices among the equal scores, 1024 blocks at a time
        if (__syncthreads_or(st_state[lane] == kKeepTies)) {
            for (int r0 = 0; r0 < 16 * ntile; r0 += 1024) {
                for (int i = tid; i < 64 * kHistStride; i += kTopkWaves * kWave) hist[i] = 0u;
                __syncthreads();
                sweep(r0 / 16, min(ntile, (r0 + 1024) / 16), [&](int qt, const f32x4_t& sc, int j0, auto tail) {
                    if (!strict4[qt]) return;
                    uint32_t bits = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((uint32_t)(j0 + i) - first4[qt] < span4[qt] && sc[i] == thr4[qt]) bits |= 1u << i;
                    if (bits) atomicOr(&hist[(16 * qt + m16) * kHistStride + ((j0 - r0) >> 5)], bits << (j0 & 31));
                });
                __syncthreads();
                if (wave == 0 && st_state[lane] == kKeepTies) {
                    uint32_t need = st_need[lane];
                    for (int w = 0; w < kHistWords && need > 0; ++w) {
                        uint32_t word = hist[lane * kHistStride + w];
                        while (word && need > 0) {
                            const int b = __ffs(word) - 1;
                            keep_plain(lane, r0 + 32 * w + b);
                            word &= word - 1;
                            --need;
                        }
                    }
                    st_need[lane] = need;
                }
                __syncthreads();
            }
        }
    }

    // ---- write the rows: kept blocks ascending, then -1.  Rows of at most 64 entries are put
    // together in LDS (over the histograms) and leave as one run of consecutive 16-byte stores.
    __syncthreads();
    if (k <= 64) {
        // (rows of k + 1 words: the queries of a wave, which fill their rows side by side, then
        // land on different banks)
        int32_t* stage = reinterpret_cast<int32_t*>(hist);           // [64][k + 1]
        const int ks1 = k + 1;
        for (int i = tid; i < 64 * ks1; i += kTopkWaves * kWave) stage[i] = -1;
        __syncthreads();
        if constexpr (LISTS) {
            // two threads per query: a kept block goes to the place given by the number of
            // smaller ones (block ids are distinct)
            const int q = tid >> 1;
            const uint16_t* mine = lst + q * KL;
            const int c = min((int)lcnt[q], min(k, KL));
            for (int a = tid & 1; a < c; a += 2) {
                const uint16_t v = mine[a];
                int rank = 0;
                for (int b = 0; b < c; ++b) rank += (int)(mine[b] < v);
                stage[q * ks1 + rank] = v;
            }
        } else {
            // wave 0 takes the first half of a query's bit row, wave 1 the second, starting
            // after the bits of the first
            const int half_w = (Wn + 1) / 2;
            const int w0 = wave == 0 ? 0 : half_w, w1 = wave == 0 ? half_w : Wn;
            int pos = 0;
            if (wave != 0)
                for (int w = 0; w < half_w; ++w) pos += __popc(selm[lane * Wn + w]);
            for (int w = w0; w < w1; ++w) {
                uint32_t word = selm[lane * Wn + w];
                while (word) {
                    const int b = __ffs(word) - 1;
                    if (pos < k) stage[lane * ks1 + pos] = 32 * w + b;
                    ++pos;
                    word &= word - 1;
                }
            }
        }
        __syncthreads();
        const int total = rows_here * k;                              // the strip's rows are one run in memory
        constexpr int NTH = kTopkWaves * kWave;
        const int dq = NTH / k, dp = NTH % k;
        int sq = tid / k, sp = tid % k;
        for (int i = tid; i < total; i += NTH) {                      // a wave stores 256 consecutive bytes
            out[i] = stage[sq * ks1 + sp];
            sq += dq;
            sp += dp;
            if (sp >= k) { sp -= k; ++sq; }
        }
    } else if (wave == 0 && lane < rows_here) {                       // lane = query
        int32_t* row = out + (int64_t)lane * k;
        int pos = 0;
        for (int w = 0; w < Wn; ++w) {
            uint32_t word = selm[lane * Wn + w];
            while (word) {
                const int b = __ffs(word) - 1;
                if (pos < k) row[pos] = 32 * w + b;
                ++pos;
                word &= word - 1;
            }
        }
        for (; pos < k; ++pos) row[pos] = -1;
    }
}

size_t topk_mfma_ws_bytes(const Dims& s)
{
    return 3 * sizeof(bf16_t) * (size_t)s.bhk * ((s.n + 15) / 16 * 16) * s.D;
}

bool topk_mfma_supported(const Dims& s)
{
    return s.dtype == MOBA_BF16 && !(s.flags & MOBA_FLAG_REFERENCE_KERNELS) &&
           s.n <= kTopkMfmaMaxBlocks && s.k > 0;
}

template <int D, int KL>
static hipError_t topk_launch2(const Dims& s, const void* Q, const bf16_t* c3, int32_t* idx,
                               hipStream_t st)
{
    const int sps = (s.N + 63) / 64;
    const int64_t strips = (int64_t)sps * s.bh;
    const int Wn = ((s.n + 31) / 32) | 1;      // words per bit row, odd for the same reason
    const size_t lds = sizeof(uint32_t) * (size_t)(64 * kHistStride + 64 + 18 * 64 +
                                                   (KL > 0 ? 64 * KL / 2 + 64 : 64 * Wn));
    hipError_t e = ensure_dynamic_lds((const void*)topk_mfma_kernel<D, KL>, (size_t)lds);
    if (e != hipSuccess) return e;
    ProfileScope timing(MOBA_PROFILE_TOPK, st);
    hipLaunchKernelGGL((topk_mfma_kernel<D, KL>), dim3((unsigned)strips), dim3(kTopkWaves * kWave), lds, st,
                       (const bf16_t*)Q, c3, (s.n + 15) / 16, idx, s.N, s.B, s.n, s.k, sps, Wn, s.G,
                       (s.flags & MOBA_FLAG_GATE_EXACT_SEARCH) ? 1 : 0, s.blk_first);
    return hipGetLastError();
}

template <int D>
static hipError_t topk_launch(const Dims& s, const void* Q, const bf16_t* c3, int32_t* idx,
                              hipStream_t st)
{
    if (s.k <= kKeptList) return topk_launch2<D, kKeptList>(s, Q, c3, idx, st);
    if (s.k <= kKeptListLong && s.n > kBitRowBlocks) return topk_launch2<D, kKeptListLong>(s, Q, c3, idx, st);
    return topk_launch2<D, 0>(s, Q, c3, idx, st);
}

hipError_t launch_topk_mfma(const Dims& s, const void* Q, const float* cent, int32_t* idx, void* ws,
                            hipStream_t st)
{
    const int ntile = (s.n + 15) / 16;
    const int64_t chunks = (int64_t)s.bhk * ntile * 3 * (s.D / 32) * 64;     // centroids: per key/value head
    if (chunks == 0) return hipSuccess;
    bf16_t* c3 = (bf16_t*)ws;
    const unsigned grid = (unsigned)((chunks + 255) / 256);
    if (s.D == 64)
        hipLaunchKernelGGL(split3_kernel<64>, dim3(grid), dim3(256), 0, st, cent, c3, s.n, ntile, chunks);
    else
        hipLaunchKernelGGL(split3_kernel<128>, dim3(grid), dim3(256), 0, st, cent, c3, s.n, ntile, chunks);
    return s.D == 64 ? topk_launch<64>(s, Q, c3, idx, st) : topk_launch<128>(s, Q, c3, idx, st);
}

}  // namespace moba
