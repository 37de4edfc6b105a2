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
// insertion far too long) by an exact radix search that recomputes the cheap scores instead
// of storing them: each sweep histograms the order-preserving integer keys of the
// still-undecided interval of every query into 64 bins (LDS integer atomics), the bin that
// holds the k-th largest key becomes the next interval, and a query is decided as soon as
// that bin holds exactly as many keys as are still needed (typically after two sweeps) or
// its width reaches one key (ties; the lower block index wins).  A last sweep marks the kept
// blocks in a per-query bit row, which is written out in ascending block order.
#include <type_traits>

#include "mfma.h"

namespace moba {

constexpr int kHistWords = 32;            // 64 bins of 16 bits per query
constexpr int kHistStride = 33;           // odd row stride: queries land on different LDS banks
constexpr int kCand = 16;                 // a final bin this small is resolved from a candidate list
constexpr int kTopkMfmaMaxBlocks = 4096;  // a 16-bit histogram bin holds any count of blocks up to this

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
// loads and MFMAs, within about 1 % of the score (enough to say where to look first).
template <int D, int TOP, typename F>
__device__ __forceinline__ void sweep_tiles(const char* __restrict__ c3s, int tile_lo, int tile_hi,
                                            int step, const Frag (&qb)[4][D / 32], int lane, int g, F f)
{
    constexpr int KS = D / 32;
    // One tile of operands in registers: the MFMAs of a term are issued, then the same term of
    // the wave's next tile is loaded over it, so every load has a whole tile of work to arrive.
    // (Past the last tile the loads repeat that tile: unconditional, always valid.)
    Frag a[3][KS];
    auto load = [&](int jt, int term) {
        const char* tb = c3s + (int64_t)jt * (3 * KS * 1024) + lane * 16 + term * (KS * 1024);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[term][ks].q = *reinterpret_cast<const uint4*>(tb + ks * 1024);
    };
    int jt = tile_lo;
    if (jt >= tile_hi) return;
#pragma unroll
    for (int term = TOP; term >= 0; --term) load(jt, term);
    while (jt < tile_hi) {
        const int nx = jt + step, ld = nx < tile_hi ? nx : jt;
        // the four 16-query tiles are independent accumulation chains: issue them interleaved so
        // that no MFMA waits for the one before it
        f32x4_t sc[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) sc[qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int term = TOP; term >= 0; --term) {       // smallest terms first
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int qt = 0; qt < 4; ++qt) sc[qt] = mfma16(a[term][ks], qb[qt][ks], sc[qt]);
            load(ld, term);
        }
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) f(qt, sc[qt], 16 * jt + 4 * g);
        jt = nx;
    }
}

constexpr int kTopkWaves = 2;             // waves per 64-query strip (= per workgroup)
// The kept blocks of a query are collected in LDS either as a bit row over the n blocks or, for
// small top-k, as a list of at most kKeptList block ids (2 KB per strip instead of 8 n bytes:
// with thousands of blocks the bit rows would cap the workgroups per CU).
constexpr int kKeptList = 16;

template <int D, bool LISTS>
__global__ __launch_bounds__(kTopkWaves * kWave) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 3)))
void topk_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ c3, int ntile_all,
    int32_t* __restrict__ idx, int N, int B, int n, int k, int strips_per_slice, int Wn, int G)
{
    extern __shared__ uint32_t smem[];
    constexpr int KS = D / 32;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int m16 = lane & 15, g = lane >> 4;
    const int strip = blockIdx.x;
    uint32_t* hist = smem;
    uint32_t* st_lo = hist + 64 * kHistStride;
    uint32_t* st_sh = st_lo + 64;
    uint32_t* st_need = st_sh + 64;
    // 0 undecided, 1 keep key >= lo, 2 keep key > lo + ties at lo, 3 keep key >= lo + 2^sh and
    // the best `need` of the (at most kCand) keys inside [lo, lo + 2^sh)
    uint32_t* st_state = st_need + 64;
    uint32_t* st_past = st_state + 64;
    uint32_t* st_hi = st_past + 64;                // the current interval is [lo, hi): at most 64 bins of 2^sh keys
    uint32_t* selm = st_hi + 64;                   // [64][Wn] kept-block bits, or:
    uint16_t* lst = reinterpret_cast<uint16_t*>(selm);      // [64][kKeptList] kept blocks, any order
    uint32_t* lcnt = selm + 64 * kKeptList / 2;             // [64] their number
    const int sel_words = LISTS ? 64 * kKeptList / 2 + 64 : 64 * Wn;
    // one more kept block of query q (concurrent callers) / (only caller for q)
    auto keep_atomic = [&](int q, int blk) {
        if constexpr (LISTS) {
            const uint32_t slot = atomicAdd(&lcnt[q], 1u);
            if (slot < (uint32_t)kKeptList) lst[q * kKeptList + slot] = (uint16_t)blk;
        } else {
            atomicOr(&selm[q * Wn + (blk >> 5)], 1u << (blk & 31));
        }
    };
    auto keep_plain = [&](int q, int blk) {
        if constexpr (LISTS) {
            const uint32_t slot = lcnt[q]++;
            if (slot < (uint32_t)kKeptList) lst[q * kKeptList + slot] = (uint16_t)blk;
        } else {
            selm[q * Wn + (blk >> 5)] |= 1u << (blk & 31);
        }
    };

    const int s = strip / strips_per_slice;
    const int t0 = (strip % strips_per_slice) * 64;
    const int rows_here = min(64, N - t0);
    const char* c3s = reinterpret_cast<const char*>(c3) + (int64_t)(s / G) * ntile_all * (3 * KS * 1024);   // G query heads share the centroids
    int32_t* out = idx + ((int64_t)s * N + t0) * k;

    if (wave == 0) {   // lane = query: initial state
        const int past = lane < rows_here ? (t0 + lane) / B : 0;
        st_past[lane] = past;
        st_lo[lane] = 0u;
        st_sh[lane] = 26u;
        st_hi[lane] = 0xffffffffu;
        st_need[lane] = (uint32_t)min(k, past);
        st_state[lane] = past <= k ? 1u : 0u;      // few candidates: keep them all (every key >= 0)
    }
    for (int i = tid; i < sel_words; i += kTopkWaves * kWave) selm[i] = 0u;
    const int pmax = (t0 + rows_here - 1) / B;
    const int ntile = (pmax + 15) / 16;

    Frag qb[4][KS];
#pragma unroll
    for (int qt = 0; qt < 4; ++qt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int64_t r = min(t0 + 16 * qt + m16, N - 1);
            qb[qt][ks].q = *reinterpret_cast<const uint4*>(Q + ((int64_t)s * N + r) * D + 8 * g + 32 * ks);
        }
    __syncthreads();

    // Interior tiles hold only blocks that are past blocks of every query of the strip; the
    // tail tiles need the per-query causal test.  The waves of the strip take alternate tiles.
    const int ntile_int = min(ntile, (t0 / B) / 16);
    auto sweep = [&](int tlo, int thi, auto f) {
        const int mid = min(max(ntile_int, tlo), thi);
        sweep_tiles<D, 2>(c3s, tlo + wave, mid, kTopkWaves, qb, lane, g,
                          [&](int qt, const f32x4_t& sc, int j0) { f(qt, sc, j0, std::false_type()); });
        // first tail tile of this wave: same parity as its interior tiles
        const int tail0 = mid + ((wave - (mid - tlo)) & (kTopkWaves - 1));
        sweep_tiles<D, 2>(c3s, tail0, thi, kTopkWaves, qb, lane, g,
                          [&](int qt, const f32x4_t& sc, int j0) { f(qt, sc, j0, std::true_type()); });
    };
    // every sm-th tile only (tiles 0, sm, 2 sm, ..., alternating between the waves), scores from
    // the hi term alone
    auto sweep_sample = [&](int sm, auto f) {
        const int step = kTopkWaves * sm;
        const int mid = min(ntile_int, ntile);
        sweep_tiles<D, 0>(c3s, sm * wave, mid, step, qb, lane, g,
                          [&](int qt, const f32x4_t& sc, int j0) { f(qt, sc, j0, std::false_type()); });
        int tail0 = sm * wave;
        if (tail0 < mid) tail0 += (mid - tail0 + step - 1) / step * step;
        sweep_tiles<D, 0>(c3s, tail0, ntile, step, qb, lane, g,
                          [&](int qt, const f32x4_t& sc, int j0) { f(qt, sc, j0, std::true_type()); });
    };

    // ---- where to look first: about the largest key of every undecided query -- from hi-term
    // scores, over all its blocks when there are few tiles, over every sm-th tile otherwise (the
    // search below does not depend on the guess being right).  The first interval of the search
    // is 2^24 keys (two binades of the score), 64 bins of 2^18 keys, reaching two bins (6 %) above
    // the largest approximate key, half a binade above a sampled one, and open at the top (its
    // last bin also takes whatever lies above).
    // (sampling pays with a small top-k; with top-k 64 of 1024 blocks it measured 10 % slower)
    const int sm = LISTS ? min(max(ntile / 8, 1), 8) : 1;
    if (__syncthreads_or(st_state[lane] == 0u)) {
        for (int i = tid; i < 64; i += kTopkWaves * kWave) hist[i * kHistStride] = 0u;
        uint32_t past4[4];
        float mx4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) { past4[qt] = st_past[16 * qt + m16]; mx4[qt] = -INFINITY; }
        __syncthreads();
        sweep_sample(sm, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bool ok = true;
                if (decltype(tail)::value) ok = (uint32_t)(j0 + i) < past4[qt];
                if (ok) mx4[qt] = fmaxf(mx4[qt], sc[i]);      // NaN scores are ignored here as in the counts
            }
        });
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) atomicMax(&hist[(16 * qt + m16) * kHistStride], order_key(mx4[qt]));
        __syncthreads();
        if (wave == 0 && st_state[lane] == 0u) {
            const uint32_t kmax = hist[lane * kHistStride];
            const uint64_t above = sm > 1 ? (1ull << 22) : (1ull << 19);
            const uint32_t top = (uint32_t)min((uint64_t)kmax + 1u + above, 0xffffffffull);
            st_lo[lane] = top > (1u << 24) ? top - (1u << 24) : 0u;
            st_hi[lane] = 0xffffffffu;
            st_sh[lane] = 18u;
        }
    }

    // ---- radix search for the k-th largest key of every undecided query.  Membership of a
    // score in the query's current key interval is tested on the float itself (two compares);
    // only members pay for the key, the bin and the atomic.
    while (__syncthreads_or(st_state[lane] == 0u)) {
        for (int i = tid; i < 64 * kHistStride; i += kTopkWaves * kWave) hist[i] = 0u;
        uint32_t lo4[4], sh4[4], past4[4];
        float flo4[4], fhi4[4];
        bool act4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            lo4[qt] = st_lo[q]; sh4[qt] = st_sh[q]; past4[qt] = st_past[q];
            act4[qt] = st_state[q] == 0u;
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
                if (decltype(tail)::value) in = in && (uint32_t)(j0 + i) < past4[qt];
                if (in) {
                    // (an interval open at the top: its last bin takes everything above as well)
                    const uint32_t bin = min((order_key(sc[i]) - lo4[qt]) >> sh4[qt], 63u);
                    atomicAdd(&row[bin >> 1], 1u << (16 * (bin & 1u)));
                }
            }
        });
        __syncthreads();
        if (wave == 0 && st_state[lane] == 0u) {     // lane = query: walk the bins from the top
            const uint32_t need = st_need[lane], lo = st_lo[lane], sh = st_sh[lane], hi = st_hi[lane];
            uint32_t cum = 0, c = 0;
            int b = 63;
            for (; b >= 0; --b) {
                c = (hist[lane * kHistStride + (b >> 1)] >> (16 * (b & 1))) & 0xffffu;
                if (cum + c >= need) break;
                cum += c;
            }
            if (b < 0 && lo > 0u) {
                // fewer keys in the interval than needed (only the first, guessed interval can
                // miss): keep them all and go on below it, [0, lo) in at most 64 bins
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
                st_lo[lane] = lo2;
                st_hi[lane] = open63 ? 0xffffffffu
                                     : (uint32_t)min((uint64_t)lo2 + (1ull << sh), (uint64_t)hi);   // the chosen bin
                st_need[lane] = need2;
                if (c == need2) st_state[lane] = 1u;
                else if (open63) {
                    if (c <= (uint32_t)kCand) st_state[lane] = 3u;
                    else st_sh[lane] = (uint32_t)max(32 - __clz((int)(0xffffffffu - lo2)) - 6, 0);   // 64 bins over [lo2, 2^32)
                }
                else if (sh == 0u) st_state[lane] = 2u;
                else if (c <= (uint32_t)kCand) st_state[lane] = 3u;
                else st_sh[lane] = sh >= 6u ? sh - 6u : 0u;                     // cut the bin into 64 again
            }
        }
        __syncthreads();
    }

    // ---- mark the kept blocks: score >= threshold (state 1), > threshold plus ties (state 2), or
    // above the last bin plus the best of the few scores inside it (state 3; those are collected
    // as (key, block) pairs in the query's histogram row, whose word 32 counts them)
    {
        uint32_t past4[4], st4[4];
        float thr4[4], top4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int q = 16 * qt + m16;
            past4[qt] = st_past[q];
            st4[qt] = st_state[q];
            thr4[qt] = key_score(st_lo[q], -INFINITY);
            const uint32_t top = st_hi[q];
            top4[qt] = top > 0xff800000u ? NAN : key_score(top, NAN);               // NaN: nothing above
        }
        bool strict4[4];
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) strict4[qt] = st4[qt] == 2u;
        sweep(0, ntile, [&](int qt, const f32x4_t& sc, int j0, auto tail) {
            uint32_t bits = 0;
            uint32_t* row = hist + (16 * qt + m16) * kHistStride;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                bool ok = true;
                if (decltype(tail)::value) ok = (uint32_t)(j0 + i) < past4[qt];
                bool keep;
                if (st4[qt] == 3u) {
                    keep = sc[i] >= top4[qt];
                    if (ok && !keep && sc[i] >= thr4[qt]) {
                        const uint32_t slot = atomicAdd(&row[32], 1u);
                        if (slot < (uint32_t)kCand) { row[2 * slot] = order_key(sc[i]); row[2 * slot + 1] = (uint32_t)(j0 + i); }
                    }
                } else {
                    keep = strict4[qt] ? sc[i] > thr4[qt] : sc[i] >= thr4[qt];
                }
                if (keep && ok) bits |= 1u << i;
            }
            if constexpr (LISTS) {
                while (bits) {
                    keep_atomic(16 * qt + m16, j0 + __ffs(bits) - 1);
                    bits &= bits - 1;
                }
            } else {
                if (bits) atomicOr(&selm[(16 * qt + m16) * Wn + (j0 >> 5)], bits << (j0 & 31));
            }
        });
        __syncthreads();
        if (wave == 0 && st_state[lane] == 3u) {     // lane = query: the best `need` candidates
            uint32_t* row = hist + lane * kHistStride;
            const int c = (int)min(row[32], (uint32_t)kCand);
            uint32_t used = 0;
            for (uint32_t need = st_need[lane]; need > 0; --need) {
                int best = -1;
                uint32_t bkey = 0, bj = 0;
                for (int i = 0; i < c; ++i) {
                    if ((used >> i) & 1u) continue;
                    const uint32_t ky = row[2 * i], jj = row[2 * i + 1];
                    if (best < 0 || ky > bkey || (ky == bkey && jj < bj)) { best = i; bkey = ky; bj = jj; }
                }
                if (best < 0) break;
                used |= 1u << best;
                keep_plain(lane, (int)bj);
            }
        }
        // ties at the threshold: the lowest block indices among the equal scores, 1024 blocks at a time
        if (__syncthreads_or(st_state[lane] == 2u)) {
            for (int r0 = 0; r0 < 16 * ntile; r0 += 1024) {
                for (int i = tid; i < 64 * kHistStride; i += kTopkWaves * kWave) hist[i] = 0u;
                __syncthreads();
                sweep(r0 / 16, min(ntile, (r0 + 1024) / 16), [&](int qt, const f32x4_t& sc, int j0, auto tail) {
                    if (!strict4[qt]) return;
                    uint32_t bits = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if ((uint32_t)(j0 + i) < past4[qt] && sc[i] == thr4[qt]) bits |= 1u << i;
                    if (bits) atomicOr(&hist[(16 * qt + m16) * kHistStride + ((j0 - r0) >> 5)], bits << (j0 & 31));
                });
                __syncthreads();
                if (wave == 0 && st_state[lane] == 2u) {
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

    // ---- write the rows (lane = query): kept blocks ascending, then -1
    if (wave == 0 && lane < rows_here) {
        int32_t* row = out + (int64_t)lane * k;
        int pos = 0;
        if constexpr (LISTS) {
            uint16_t* mine = lst + lane * kKeptList;
            const int c = min((int)lcnt[lane], min(k, kKeptList));
            for (int a = 1; a < c; ++a) {                 // insertion sort, ascending
                const uint16_t v = mine[a];
                int b = a - 1;
                for (; b >= 0 && mine[b] > v; --b) mine[b + 1] = mine[b];
                mine[b + 1] = v;
            }
            for (; pos < c; ++pos) row[pos] = mine[pos];
        } else {
            for (int w = 0; w < Wn; ++w) {
                uint32_t word = selm[lane * Wn + w];
                while (word) {
                    const int b = __ffs(word) - 1;
                    if (pos < k) row[pos] = 32 * w + b;
                    ++pos;
                    word &= word - 1;
                }
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

template <int D, bool LISTS>
static hipError_t topk_launch2(const Dims& s, const void* Q, const bf16_t* c3, int32_t* idx,
                               hipStream_t st)
{
    const int sps = (s.N + 63) / 64;
    const int64_t strips = (int64_t)sps * s.bh;
    const int Wn = ((s.n + 31) / 32) | 1;      // words per bit row, odd for the same reason
    const size_t lds = sizeof(uint32_t) * (size_t)(64 * kHistStride + 6 * 64 +
                                                   (LISTS ? 64 * kKeptList / 2 + 64 : 64 * Wn));
    hipError_t e = hipFuncSetAttribute((const void*)topk_mfma_kernel<D, LISTS>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfileScope timing(MOBA_PROFILE_TOPK, st);
    hipLaunchKernelGGL((topk_mfma_kernel<D, LISTS>), dim3((unsigned)strips), dim3(kTopkWaves * kWave), lds, st,
                       (const bf16_t*)Q, c3, (s.n + 15) / 16, idx, s.N, s.B, s.n, s.k, sps, Wn, s.G);
    return hipGetLastError();
}

template <int D>
static hipError_t topk_launch(const Dims& s, const void* Q, const bf16_t* c3, int32_t* idx,
                              hipStream_t st)
{
    return s.k <= kKeptList ? topk_launch2<D, true>(s, Q, c3, idx, st)
                            : topk_launch2<D, false>(s, Q, c3, idx, st);
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
