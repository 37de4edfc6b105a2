// bf16 MFMA helpers for gfx950 (v_mfma_f32_16x16x32_bf16) and the operand layouts the
// attention kernels share.
//
// One MFMA multiplies A (16 x 32) by B (32 x 16) into C (16 x 16), fp32 accumulate.
// With lane = 16*g + m (g = 0..3, m = 0..15):
//   A operand: lane holds row m,  contraction slots 8g .. 8g+7   (8 bf16 = 4 VGPRs)
//   B operand: lane holds col m,  contraction slots 8g .. 8g+7
//   C result : lane holds col m,  rows 4g .. 4g+3                (4 fp32)
//
// Keys are processed in groups of 32 consecutive keys.  Scores are computed transposed,
// S^T = K_group (32 keys x d) . Q^T (d x 16 queries), as two 16-key tiles; a lane then
// holds, for its query column, keys {4g+i} of tile 0 and {16+4g+i} of tile 1.  Packed to
// bf16 in that order these 8 values ARE a B operand whose contraction slot s of group g
// means key  slot_key(g, s)  -- so the other operand of the next product only has to use
// the same slot order, and P never moves between lanes.
#pragma once
#include "common.h"

namespace moba {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

union Frag {               // one A or B operand
    bf16x8_t v;
    uint4 q;
    u32x4_t n;             // the same four registers as one native vector (asm operands)
    uint32_t u[4];
};

__device__ __forceinline__ f32x4_t mfma16(const Frag& a, const Frag& b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

// key (0..31, inside its 32-key group) that contraction slot s of lane group g stands for
__host__ __device__ __forceinline__ constexpr int slot_key(int g, int s)
{
    return s < 4 ? 4 * g + s : 16 + 4 * g + (s - 4);
}

// channel that row m of M-tile mt of a (d x 16) product stands for.  Chosen so that the four
// lane groups of a result (rows 4g'..4g'+3) land D/4 channels apart: fp32 accumulators in
// LDS ([row][channel], odd row stride) then see the two lane groups that issue together on
// different halves of the banks.
template <int D>
__host__ __device__ __forceinline__ constexpr int tile_chan(int mt, int m)
{
    return (m >> 2) * (D / 4) + 4 * mt + (m & 3);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    // round to nearest even, two at a time
    return pack_bf16x2(lo, hi);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// exponent e with |x| * 2^-e <= 1 for every |x| <= vmax (vmax >= 0 given as fp32 bits)
__device__ __forceinline__ int scale_exponent(uint32_t vmax_bits)
{
    const int E = (int)((vmax_bits >> 23) & 0xffu);
    return E == 0 ? 0 : E - 127 + 1;
}

// maximum that hands a NaN on (v_maximum3_f32 on gfx950; fmaxf would drop it)
__device__ __forceinline__ float max_nan(float a, float b) { return __builtin_elementwise_maximum(a, b); }
// channel maximum (fp32 bits of a magnitude) of a tensor that holds an infinity or a NaN
__device__ __forceinline__ bool nonfinite_bits(uint32_t magnitude_bits) { return magnitude_bits >= 0x7f800000u; }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Element offset of the "slot-ordered transposed" copy of a [N, D] tensor X (keys or values):
// for 32-row group kap, M-tile mt, lane (g, m), slot s it holds X[32*kap + slot_key(g,s)][tile_chan(mt,m)],
// stored so that the 64 lanes of one (kap, mt) read 1 KB contiguously, 16 B per lane.
template <int D>
__host__ __device__ __forceinline__ constexpr int64_t slot_major_offset(int64_t kap, int mt, int lane)
{
    return (kap * (D / 16) + mt) * 512 + (int64_t)lane * 8;
}

// Ascending list of the non-empty blocks of a set of row lists (offs as built below):
// ulist[0 .. *count).  All NT threads; ends with a workgroup barrier.
template <int NT>
__device__ __forceinline__ void list_nonempty(const uint32_t* offs, int nb, uint16_t* ulist,
                                              int* count, uint32_t* wsum, int tid)
{
    const int lane = tid % kWave, wave = tid / kWave;
    int base = 0;
    for (int c = 0; c < nb; c += NT) {
        const int i = c + tid;
        const bool some = i < nb && offs[i + 1] > offs[i];
        const uint64_t b = __ballot(some);
        if (lane == 0) wsum[wave] = (uint32_t)__popcll(b);
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int wv = 0; wv < NT / kWave; ++wv) {
            const int n = (int)wsum[wv];
            if (wv < wave) before += n;
            total += n;
        }
        if (some) ulist[base + before + lanes_below(b)] = (uint16_t)i;
        base += total;
        __syncthreads();
    }
    if (tid == 0) *count = base;
    __syncthreads();
}

// Next entry of a work list shared by the waves of a workgroup (the same value in all lanes).
// Units differ in length and the memory system does not serve all waves alike, so a static
// deal leaves waves idle at the barrier that ends the list.
__device__ __forceinline__ int take_unit(int* counter, int lane)
{
    int e = 0;
    if (lane == 0) e = atomicAdd(counter, 1);
    return __builtin_amdgcn_readfirstlane(e);
}

// ---- per-tile block lists in LDS --------------------------------------------------------
// For a tile of TILE consecutive queries and the key blocks [lo, hi): a counting sort of the
// tile's (row, kept block) pairs by block.  Afterwards offs[j - lo] .. offs[j - lo + 1] is the
// piece of rows8[] holding the local rows (0 .. TILE-1, one byte each) that kept block j, in no
// particular order.  Built once per tile and range, by all NT threads; integer atomics only.
//   cur   [hi - lo + 1] words of scratch (counters, then insertion cursors)
//   offs  [hi - lo + 1] words
//   rows8 cap bytes; a routing without repeats has at most min(TILE * (hi - lo), TILE * k)
//         pairs, and pairs beyond cap are dropped rather than written
//   wsum  NT / 64 words of scratch
// `idx_tile` points at the tile's first topk_idx row; entries that are not past blocks of
// their row are ignored.  Ends with a workgroup barrier.
template <int TILE, int NT>
__device__ __forceinline__ void build_block_lists(const int32_t* __restrict__ idx_tile, int t0,
                                                  int rows_here, int k, int B, int lo, int hi,
                                                  uint32_t* cur, uint32_t* offs, uint8_t* rows8,
                                                  uint32_t cap, uint32_t* wsum, int tid)
{
    constexpr int TPR = NT / TILE;                 // threads per row
    const int nb = hi - lo;
    const int r = tid / TPR, part = tid % TPR;
    const int past = (t0 + r) / B;
    const int lane = tid % kWave, wave = tid / kWave;
    auto for_each_entry = [&](auto f) {
        if (r >= rows_here) return;
        const int32_t* row = idx_tile + (int64_t)r * k;
        auto one = [&](int b) { if (b >= lo && b < hi && b < past) f(b - lo); };
        if ((k & 3) == 0) {                        // 16-byte loads, several in flight
            const int4* row4 = reinterpret_cast<const int4*>(row);
            const int n4 = k >> 2;
            for (int e0 = part; e0 < n4; e0 += 4 * TPR) {
                int4 v[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    v[j] = e0 + j * TPR < n4 ? row4[e0 + j * TPR] : make_int4(-1, -1, -1, -1);
#pragma unroll
                for (int j = 0; j < 4; ++j) { one(v[j].x); one(v[j].y); one(v[j].z); one(v[j].w); }
            }
        } else {
            for (int e = part; e < k; e += TPR) one(row[e]);
        }
    };
    for (int i = tid; i <= nb; i += NT) cur[i] = 0u;
    __syncthreads();
    for_each_entry([&](int j) { atomicAdd(&cur[j], 1u); });
    __syncthreads();
    // exclusive scan of the counts: each thread takes EPT consecutive blocks
    constexpr int kMaxRange = 1024;
    constexpr int EPT = (kMaxRange + NT - 1) / NT;
    uint32_t v[EPT], sum = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid * EPT + e;
        v[e] = j < nb ? cur[j] : 0u;
        sum += v[e];
    }
    uint32_t incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t base = incl - sum;
    for (int wv = 0; wv < wave; ++wv) base += wsum[wv];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int j = tid * EPT + e;
        if (j < nb) { offs[j] = base; cur[j] = base; }
        base += v[e];
        if (j == nb - 1) offs[nb] = base;
    }
    __syncthreads();
    for_each_entry([&](int j) {
        const uint32_t pos = atomicAdd(&cur[j], 1u);
        if (pos < cap) rows8[pos] = (uint8_t)r;
    });
    __syncthreads();
}

// ---- prepared copies of K and V (prepare.hip) ------------------------------------------------
// "MFMA operand order": the 16 bytes lane (m, g) feeds to the MFMA as rows 16 mt + m, channels
// 32 ks + 8 g .. + 8 of 32-key group kap sit at ((kap * 2 + mt) * (D / 32) + ks) * 1024 + 16 * lane.
// One load instruction of a wave then covers 1 KB of consecutive bytes; reading the same operand
// from the row-major tensor (16 rows x 64 bytes per instruction) runs at a quarter of that rate on
// this chip.  "Slot-ordered transposed": slot_major_offset() above.
struct Prepared {
    uint32_t* kmax = nullptr;   // [bhk][D] largest magnitude per channel of K, fp32 bits
    uint32_t* vmax = nullptr;   //                                          of V
    void* Ka = nullptr;         // K in MFMA operand order
    void* Vt = nullptr;         // V slot-ordered transposed, scaled per channel
    void* Kt = nullptr;         // K slot-ordered transposed, scaled per channel
    void* Va = nullptr;         // V in MFMA operand order
};
constexpr unsigned kPrepKa = 1, kPrepVt = 2, kPrepKt = 4, kPrepVa = 8;
constexpr unsigned kPrepForward = kPrepKa | kPrepVt;             // what the query-tile forward reads
constexpr unsigned kPrepBackward = kPrepKa | kPrepKt | kPrepVa;  // what the query-tile dQ kernel reads
constexpr unsigned kPrepAll = kPrepForward | kPrepBackward;
size_t prepared_layout(const Dims& s, unsigned mask, void* base, Prepared* out);
// makes the parts of `p` that are not null (the maxima it needs first)
hipError_t launch_prepare(const Dims& kv, const void* K, const void* V, const Prepared& p, hipStream_t st);
bool shared_workspace(const Dims& s);

hipError_t launch_slot_major_copy(const Dims& s, const void* X, void* Xt, const uint32_t* vmax,
                                  hipStream_t st);
size_t forward_mfma_ws_bytes(const Dims& s);
hipError_t launch_forward_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                               void* ws, const int32_t* idx, const int32_t* off, const int32_t* ql,
                               void* O, float* lse, hipStream_t st);

size_t backward_mfma_ws_bytes(const Dims& s);
hipError_t launch_dq_mfma(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                          const float* lse, const int32_t* idx, const int32_t* off, const int32_t* ql,
                          void* dQ, void* ws, hipStream_t st);

// ld: per query (lse log2 e, -D), as the D kernel packs them; part: dkdv_heads_ws_bytes() of
// scratch for the per-query-head sums when key/value heads are shared (unused otherwise)
size_t dkdv_heads_ws_bytes(const Dims& s);
hipError_t launch_dkdv_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                            const void* dO, const float2* ld, const int32_t* off,
                            const int32_t* ql, void* dK, void* dV, float* part, hipStream_t st);

size_t topk_mfma_ws_bytes(const Dims& s);
bool topk_mfma_supported(const Dims& s);
hipError_t launch_topk_mfma(const Dims& s, const void* Q, const float* cent, int32_t* idx, void* ws,
                            hipStream_t st);

constexpr int kKeyMajorMaxTopk = 64;      // longest row of kept blocks the key-major kernels take

// keys a key-major workgroup holds in registers as MFMA operands: the whole block up to 128
// (d = 64) or 64 (d = 128) keys, else parts of that size
__host__ __device__ inline int km_part_keys(int B, int D)
{
    const int cap = D == 64 ? 128 : 64;
    return B <= cap ? B : cap;
}

// workspace parts start on 256-byte boundaries
inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

// (query, kept block or own block, part of the block) triples: the partial results of the
// key-major kernels, [bh][N][k+1][parts]
inline size_t km_partials(const Dims& s)
{
    return (size_t)s.bh * s.N * (size_t)(s.k + 1) * (size_t)(s.B / km_part_keys(s.B, s.D));
}

// shapes the MFMA kernels cover: bf16 I/O and key blocks made of whole 32-key groups
inline bool mfma_path(const Dims& s)
{
    return s.dtype == MOBA_BF16 && s.B % 32 == 0 && !(s.flags & MOBA_FLAG_REFERENCE_KERNELS);
}

// The query-tile forward accumulates the row sums and P V as 32-bit fixed point with
// F = 30 - bitlen(keys a query can attend) fraction bits, the 32 keys of a row and group per add
// (the channel sums of P V likewise): a partial sum below 2^-(F+1) is lost, so a row with one
// dominant logit beside very many tiny ones can lose up to keys * 2^-(F+6) of its denominator (the
// sum is biased: every term is positive).  With at most 4096 keys per query F is at least 17 and
// that loss at most 0.05 % in the worst case (16384 keys would allow 0.4 %, 32768 keys 1.6 %,
// which shows in the output); longer rows go to the key-major or the plain kernels, which keep
// their sums in floating point.
constexpr int64_t kTileForwardMaxKeys = 4096;
inline int64_t keys_per_query(const Dims& s)
{
    const int64_t kept = (int64_t)(s.k + 1) * s.B;
    return kept < s.N ? kept : s.N;
}
inline bool tile_forward_ok(const Dims& s) { return keys_per_query(s) <= kTileForwardMaxKeys; }

// shapes the key-major kernels cover: key blocks of one part or of whole parts
inline bool key_major_shape(const Dims& s)
{
    return mfma_path(s) && s.B % km_part_keys(s.B, s.D) == 0 && s.k <= kKeyMajorMaxTopk;
}

// Query-tile or key-major attention?  Both are priced per query from fits to measured times (ns
// per query and slice on the whole chip, forward and dQ averaged; a wrong pick near the line costs
// 10-20 %):
//   tiles      c0 + k (B / 32) (g0 + g1 / rows): a tile of T consecutive queries (256 for d = 64,
//              128 for d = 128) meets a past key block with rows = T k / n of its rows and pays
//              per 32-key group at least a 16-row MFMA tile and the group's operands;
//   key-major  c (k + 1) (1 + 0.7 (parts - 1)): the gathered row, the partial result written and
//              read back per (query, block) pair, whatever B, and again for every further part of
//              the block.
// With k = 8 of B = 128 key-major wins from N = 8K on; with k = 64 of B = 32 (many blocks per
// query, every pair a partial in memory) the tiles win up to N of a few hundred thousand.
inline bool key_major_path(const Dims& s)
{
    if (!key_major_shape(s) || (s.flags & MOBA_FLAG_QUERY_TILES)) return false;
    if (s.flags & MOBA_FLAG_KEY_MAJOR) return true;
    if (!tile_forward_ok(s)) return true;
    if (s.k <= 0) return false;
    const bool d64 = s.D == 64;
    const double T = d64 ? 256.0 : 128.0;
    const double rows = T * s.k * (double)s.B / (double)s.N;
    const double parts = (double)(s.B / km_part_keys(s.B, s.D));
    const double tiles = (d64 ? 0.6 : 1.1) + 0.0013 * s.B +
                         s.k * (s.B / 32.0) * (d64 ? 0.015 + 0.14 / rows : 0.033 + 0.272 / rows);
    const double keymajor = (d64 ? 0.115 : 0.17) * (s.k + 1) * (1.0 + 0.7 * (parts - 1.0));
    return keymajor < tiles;
}

// The caller gives forward and backward the same workspace and the forward call prepares for both:
// only where both run on the query-tile kernels.
inline bool shared_workspace(const Dims& s)
{
    return (s.flags & MOBA_FLAG_SHARED_WORKSPACE) && mfma_path(s) && tile_forward_ok(s) && !key_major_path(s);
}

size_t forward_km_ws_bytes(const Dims& s);
size_t backward_km_ws_bytes(const Dims& s);
hipError_t launch_dq_km(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                        const float2* ld, const int32_t* idx, const int32_t* off, const int32_t* ql,
                        void* dQ, void* ws, hipStream_t st);
hipError_t launch_forward_km(const Dims& s, const void* Q, const void* K, const void* V, void* ws,
                             const int32_t* idx, const int32_t* off, const int32_t* ql, void* O,
                             float* lse, hipStream_t st);

}  // namespace moba
