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

union Frag {               // one A or B operand
    bf16x8_t v;
    uint4 q;
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

// Bit matrix "which rows of this query tile go with which 32-key group", for the groups
// [lo, hi): mask[(kap - lo) * MW + r / 32] bit r % 32.  A row goes with every group of each
// block it kept (entries of its topk_idx row that are past blocks) and, when a block has several
// groups, with the groups of its own block that lie wholly before it.  `idx_tile` points at the
// tile's first topk_idx row.  The caller zeroes the mask before and synchronises after.
template <int TILE, int NT, int MW>
__device__ __forceinline__ void build_group_mask(uint32_t* mask, const int32_t* __restrict__ idx_tile,
                                                 int t0, int rows_here, int k, int B, int NG, int lo,
                                                 int hi, int tid)
{
    constexpr int TPR = NT / TILE;                 // threads per row
    const int r = tid / TPR, part = tid % TPR;
    if (r >= rows_here) return;
    const int past = (t0 + r) / B;
    const uint32_t bit = 1u << (r & 31);
    uint32_t* col = mask + (r >> 5);
    auto mark = [&](int b) {
        if (b >= 0 && b < past) {
            for (int gi = 0; gi < NG; ++gi) {
                const int kap = b * NG + gi - lo;
                if (kap >= 0 && kap < hi - lo) atomicOr(&col[kap * MW], bit);
            }
        }
    };
    const int32_t* row = idx_tile + (int64_t)r * k;
    if ((k & 3) == 0) {                            // 16-byte loads, several in flight
        const int4* row4 = reinterpret_cast<const int4*>(row);
        const int n4 = k >> 2;
        for (int e0 = part; e0 < n4; e0 += 4 * TPR) {
            int4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = e0 + j * TPR < n4 ? row4[e0 + j * TPR] : make_int4(-1, -1, -1, -1);
#pragma unroll
            for (int j = 0; j < 4; ++j) { mark(v[j].x); mark(v[j].y); mark(v[j].z); mark(v[j].w); }
        }
    } else {
        for (int e = part; e < k; e += TPR) mark(row[e]);
    }
    if (NG > 1 && part == 0) {
        const int t = t0 + r;
        for (int kap = (t / B) * NG; kap < (t >> 5); ++kap)
            if (kap >= lo && kap < hi) atomicOr(&col[(kap - lo) * MW], bit);
    }
}

hipError_t launch_absmax(const Dims& s, const void* X, uint32_t* vmax, hipStream_t st);
hipError_t launch_slot_major_copy(const Dims& s, const void* X, void* Xt, const uint32_t* vmax,
                                  hipStream_t st);
size_t forward_mfma_ws_bytes(const Dims& s);
hipError_t launch_forward_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                               void* ws, const int32_t* idx, const int32_t* off, const int32_t* ql,
                               const int32_t* chunk, void* O, float* lse, hipStream_t st);

size_t backward_mfma_ws_bytes(const Dims& s);
hipError_t launch_dq_mfma(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                          const float* lse, const int32_t* idx, const int32_t* off, const int32_t* ql,
                          const int32_t* chunk, void* dQ, void* ws, hipStream_t st);

hipError_t launch_dkdv_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                            const void* dO, const float* lse, const float* Dv, const int32_t* off,
                            const int32_t* ql, void* dK, void* dV, hipStream_t st);

size_t topk_mfma_ws_bytes(const Dims& s);
bool topk_mfma_supported(const Dims& s);
hipError_t launch_topk_mfma(const Dims& s, const void* Q, const float* cent, int32_t* idx, void* ws,
                            hipStream_t st);

// shapes the MFMA kernels cover: bf16 I/O and key blocks made of whole 32-key groups
inline bool mfma_path(const Dims& s)
{
    return s.dtype == MOBA_BF16 && s.B % 32 == 0 && !(s.flags & MOBA_FLAG_REFERENCE_KERNELS);
}

}  // namespace moba
