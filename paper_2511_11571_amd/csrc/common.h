// Shared device helpers of the MoBA kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moba.h"

namespace moba {

typedef uint16_t bf16_t;   // raw bfloat16 bits

constexpr int kWave = 64;
constexpr int kChunkQ = 256;   // queries per chunk of the list builder's per-(chunk, block) counts (= per workgroup there)

__device__ __forceinline__ float bf16_to_f32(bf16_t x)
{
    return __uint_as_float(((uint32_t)x) << 16);
}

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two fp32 -> two bf16 in one word, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t*>(&b);
}

// ---- 8-element vector access in the I/O type --------------------------------
template <typename T> struct Vec8;

template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[8])
    {
        float4 a = *reinterpret_cast<const float4*>(p);
        float4 b = *reinterpret_cast<const float4*>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[8])
    {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    // value after a round trip through the I/O type
    static __device__ __forceinline__ float round(float x) { return x; }
};

template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8])
    {
        uint4 a = *reinterpret_cast<const uint4*>(p);
        v[0] = __uint_as_float(a.x << 16); v[1] = __uint_as_float(a.x & 0xffff0000u);
        v[2] = __uint_as_float(a.y << 16); v[3] = __uint_as_float(a.y & 0xffff0000u);
        v[4] = __uint_as_float(a.z << 16); v[5] = __uint_as_float(a.z & 0xffff0000u);
        v[6] = __uint_as_float(a.w << 16); v[7] = __uint_as_float(a.w & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8])
    {
        uint4 a;
        a.x = pack_bf16x2(v[0], v[1]); a.y = pack_bf16x2(v[2], v[3]);
        a.z = pack_bf16x2(v[4], v[5]); a.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = a;
    }
    static __device__ __forceinline__ float round(float x) { return bf16_to_f32(f32_to_bf16(x)); }
};

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t x) { return bf16_to_f32(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f32_to_bf16(x); }

// ---- wave-level reductions (64 lanes) ------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
// number of set bits of `mask` below this lane
__device__ __forceinline__ int lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// monotone map of a gate score to uint32 (larger score <=> larger key); -0 is folded into +0
// first so that equal scores always have equal keys
__device__ __forceinline__ uint32_t order_key(float s)
{
    s += 0.0f;
    const uint32_t b = __float_as_uint(s);
    // negative: all bits flipped; else: sign bit set
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// ---- entries of the key-block-major query lists ------------------------------------------
// low 24 bits: the query; high byte: the position of the block in the query's row of kept blocks
// (filled in for top-k up to 64, see lists.hip)
constexpr int kListQueryMask = 0xffffff;
__device__ __forceinline__ int list_query(int entry) { return entry & kListQueryMask; }
__device__ __forceinline__ int list_slot(int entry) { return (int)((uint32_t)entry >> 24); }

// ---- workgroup -> (slice, position) ------------------------------------------------------
// Workgroups are dealt to the chip's 8 XCDs round robin (workgroup i runs on XCD i % 8) and
// every XCD has an L2 of its own.  The workgroups resident on one XCD at a time should
// therefore read the same K / V (or Q / dO) rows: with a multiple of 8 slices, XCD x works
// through the slices x, x + 8, ... one after the other; with 1, 2 or 4 slices, 8 / bh XCDs
// share the positions of a slice.  Anything else falls back to slice-interleaved order.
// A negative bh asks for the opposite: one slice after the other over the whole chip (slice
// -bh-major order).  Kernels that gather rows from all over a slice take it when the gathered
// tensors of eight slices at once would not fit the 256 MB cache behind the L2s (slice_major()
// below): the rows of the one slice in flight then stay there for their next reader.
constexpr int kXcds = 8;
__host__ __device__ inline int schedule_grid(int bh, int npos)
{
    if (bh < 0) return -bh * npos;
    if (bh % kXcds != 0 && kXcds % bh == 0) {
        const int X = kXcds / bh;
        return kXcds * ((npos + X - 1) / X);
    }
    return bh * npos;
}
// false: this workgroup has nothing to do
__device__ __forceinline__ bool schedule(int bid, int bh, int npos, int& s, int& pos)
{
    if (bh < 0) {                 // one slice after the other over the whole chip
        s = bid / npos;
        pos = bid - s * npos;
        return true;
    }
    const int xcd = bid % kXcds, local = bid / kXcds;
    if (bh % kXcds == 0) {
        s = xcd + kXcds * (local / npos);
        pos = local % npos;
        return true;
    }
    if (kXcds % bh == 0) {
        s = xcd % bh;
        pos = local * (kXcds / bh) + xcd / bh;
        return pos < npos;
    }
    s = bid % bh;
    pos = bid / bh;
    return true;
}

// ---- host-side view of a validated shape ------------------------------------------
struct Dims {
    // bh, heads: query heads.  G query heads share a key/value head (slice s reads key/value
    // slice s / G); bhk = bh / G key/value slices of hkv heads.
    int bh, heads, N, D, B, n, k, W;
    int G, bhk, hkv;
    int dtype;
    uint32_t flags;
    float scale;
    int64_t R;          // routes per slice
    int nchunk;         // ceil(N / kChunkQ)
    // Packed variable-length batches: first block of the sequence each key block belongs to
    // (device, [n]); the candidates of a query in block c are blocks blk_first[c] .. c - 1.
    // nullptr: one sequence, candidates 0 .. c - 1.
    const int32_t* blk_first = nullptr;
};

// the same shape as seen by kernels that walk key/value-shaped tensors only
inline Dims kv_view(const Dims& d)
{
    Dims v = d;
    v.bh = d.bhk;
    v.heads = d.hkv;
    v.G = 1;
    return v;
}

// +1 / -1: factor for the slice count handed to schedule() by a kernel whose workgroups gather rows
// of `tensors` query-shaped bf16 tensors from all over their slice: eight slices in flight (one per
// XCD) keep 8 * tensors * N * D * 2 bytes in use; beyond the 256 MB of the cache behind the L2s one
// slice at a time is the better order (measured: key-block-major forward, d = 64, 8 % slower at
// 16 MB per slice, 5 % faster at 32 MB, 13 % faster at 64 MB)
inline int slice_major(const Dims& d, int tensors)
{
    return d.bh > 1 && (int64_t)tensors * d.N * d.D * 2 >= ((int64_t)32 << 20) ? -1 : 1;
}

// hipFuncSetAttribute(MaxDynamicSharedMemorySize) for `kernel` on the current device, issued
// only when a launch needs more than was asked for before (the library remembers per kernel and
// device; thread-safe)
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes);

// kernel timing hooks (see moba_profile_begin): no-ops unless a session is open
void profile_mark(int kernel, bool start, hipStream_t st);
struct ProfileScope {
    int kernel;
    hipStream_t st;
    ProfileScope(int k, hipStream_t s) : kernel(k), st(s) { profile_mark(kernel, true, st); }
    ~ProfileScope() { profile_mark(kernel, false, st); }
};

// launchers (one translation unit each); every one returns a hipError_t
hipError_t launch_centroids(const Dims& s, const void* K, const float* w, void* Keff,
                            float* cent, hipStream_t st);
hipError_t launch_decode(const Dims& s, int q_len, const void* Q, const void* K, const void* V,
                         const float* cent, int cblocks, void* O, float* lse, int32_t* idx, hipStream_t st);
hipError_t launch_conv_backward(const Dims& s, const void* K, const float* w, const void* G, void* dK,
                                float* dw, void* ws, hipStream_t st);
size_t conv_bwd_ws_bytes(const Dims& s);
hipError_t launch_varlen_copy(bool pad, const int32_t* seq_off, const int32_t* pad_off, int num_seqs,
                              int64_t slices, int tokens, int padded_tokens, int row_bytes, const void* src,
                              void* dst, hipStream_t st);
hipError_t launch_varlen_block_first(const int32_t* pad_off, int num_seqs, int B, int nblocks, int32_t* first,
                                     hipStream_t st);
hipError_t launch_topk_reference(const Dims& s, const void* Q, const float* cent, int32_t* idx,
                                 hipStream_t st);
hipError_t launch_build_lists(const Dims& s, const int32_t* idx, int32_t* off, int32_t* ql,
                              int32_t* chunk_counts, hipStream_t st);
hipError_t launch_forward_reference(const Dims& s, const void* Q, const void* K, const void* V,
                                    const int32_t* idx, void* O, float* lse, hipStream_t st);
hipError_t launch_backward_reference(const Dims& s, const void* Q, const void* K, const void* V,
                                     const void* O, const float* lse, const void* dO,
                                     const int32_t* idx, const int32_t* off, const int32_t* ql,
                                     void* dQ, void* dK, void* dV, float* Dvec, uint32_t parts,
                                     float2* packed, hipStream_t st);


}  // namespace moba
