// Plain gate scoring + causal top-k (paper Section 2; Appendix C.1, top-k
// selection), one wave per query.  Scores are fp32 FMA dot products kept in LDS (one
// row of at most n values per wave, never written to memory); the k-th largest is
// found exactly by a 32-step bitwise search on order-preserving integer keys, and the
// kept blocks are emitted in ascending block order with ties resolved toward the
// lower block index.
#include "common.h"

namespace moba {

constexpr int kTopkMaxBlocks = 4096;   // LDS row length per wave

template <typename T, int D>
__global__ __launch_bounds__(256) void topk_reference_kernel(
    const T* __restrict__ Q, const float* __restrict__ cent, int32_t* __restrict__ idx,
    int N, int B, int n, int k, int64_t total_rows, int lds_row, int G,
    const int32_t* __restrict__ blk_first)
{
    extern __shared__ uint32_t smem[];
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    float* qs = reinterpret_cast<float*>(smem) + wave * D;                // [4][D]
    uint32_t* keys = smem + 4 * D + (size_t)wave * lds_row;               // [4][lds_row]
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    if (row >= total_rows) return;
    const int64_t s = row / N;
    const int t = (int)(row % N);
    // candidates: blocks first .. past - 1 (first > 0 in packed variable-length batches only)
    const int past = t / B;
    const int first = blk_first ? blk_first[past] : 0;
    int32_t* out = idx + row * k;

    if (past - first <= k) {              // keep every candidate
        for (int c = lane; c < k; c += kWave) out[c] = first + c < past ? first + c : -1;
        return;
    }
    for (int c = lane; c < D; c += kWave) qs[c] = to_f32<T>(Q[row * D + c]);
    __builtin_amdgcn_wave_barrier();

    const float* cs = cent + (s / G) * n * D;        // G query heads share the centroids
    for (int j = first + lane; j < past; j += kWave) {
        const float4* cj = reinterpret_cast<const float4*>(cs + (int64_t)j * D);
        float acc = 0.f;
#pragma unroll 4
        for (int c = 0; c < D / 4; ++c) {
            float4 v = cj[c];
            float4 q4 = *reinterpret_cast<const float4*>(qs + 4 * c);
            acc = fmaf(q4.x, v.x, acc); acc = fmaf(q4.y, v.y, acc);
            acc = fmaf(q4.z, v.z, acc); acc = fmaf(q4.w, v.w, acc);
        }
        keys[j] = order_key(acc);
    }
    __builtin_amdgcn_wave_barrier();

    // largest thr with count(key >= thr) >= k  ==  the k-th largest key
    uint32_t thr = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        int c = 0;
        for (int j = first + lane; j < past; j += kWave) c += keys[j] >= cand;
        if (wave_sum_i(c) >= k) thr = cand;
    }
    int g = 0;
    for (int j = first + lane; j < past; j += kWave) g += keys[j] > thr;
    const int need = k - wave_sum_i(g);     // how many of the blocks equal to thr to keep

    int pos = 0, eq_seen = 0;
    for (int j0 = first; j0 < past; j0 += kWave) {
        const int j = j0 + lane;
        const uint32_t key = j < past ? keys[j] : 0u;
        const bool eq = j < past && key == thr;
        const uint64_t eq_mask = __ballot(eq);
        const bool sel = j < past && (key > thr || (eq && eq_seen + lanes_below(eq_mask) < need));
        const uint64_t sel_mask = __ballot(sel);
        if (sel) out[pos + lanes_below(sel_mask)] = j;
        pos += __popcll(sel_mask);
        eq_seen += __popcll(eq_mask);
    }
}

template <typename T, int D>
static hipError_t launch_t(const Dims& s, const void* Q, const float* cent, int32_t* idx,
                           hipStream_t st)
{
    const int64_t rows = (int64_t)s.bh * s.N;
    if (rows == 0 || s.k == 0) return hipSuccess;
    const int lds_row = s.n;
    const size_t lds = sizeof(float) * 4 * D + sizeof(uint32_t) * 4 * (size_t)lds_row;
    dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (lds > 64 * 1024) {     // above the default dynamic LDS limit: opt in (gfx950 has 160 KB)
        hipError_t e = ensure_dynamic_lds((const void*)topk_reference_kernel<T, D>, (size_t)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((topk_reference_kernel<T, D>), grid, block, lds, st, (const T*)Q, cent, idx,
                       s.N, s.B, s.n, s.k, rows, lds_row, s.G, s.blk_first);
    return hipGetLastError();
}

hipError_t launch_topk_reference(const Dims& s, const void* Q, const float* cent, int32_t* idx,
                                 hipStream_t st)
{
    if (s.n > kTopkMaxBlocks) return hipErrorInvalidValue;
    if (s.dtype == MOBA_BF16)
        return s.D == 64 ? launch_t<bf16_t, 64>(s, Q, cent, idx, st)
                         : launch_t<bf16_t, 128>(s, Q, cent, idx, st);
    return s.D == 64 ? launch_t<float, 64>(s, Q, cent, idx, st)
                     : launch_t<float, 128>(s, Q, cent, idx, st);
}

}  // namespace moba
