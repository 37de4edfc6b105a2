// Key convolution (paper Appendix B) fused with the block centroids (Section 2;
// Appendix C.1, centroid algorithm).  One pass over K: a group of D/8 lanes walks a run of
// consecutive rows of one key block top to bottom, 8 channels per lane, keeps the W-1 previous
// rows in registers for the causal depthwise filter, writes the convolved key rounded to the
// I/O type, and sums those rounded rows.  A block is cut into RS such runs (lane groups next to
// each other in one wave, so that long blocks do not leave the chip idle); their sums are added
// by shuffles in a fixed order.
#include "common.h"

namespace moba {

template <typename T, int D, int W>
__global__ __launch_bounds__(256) void centroid_kernel(
    const T* __restrict__ K, const float* __restrict__ w, T* __restrict__ Keff,
    float* __restrict__ cent, int heads, int N, int B, int n, int64_t total_blocks, int RS)
{
    constexpr int G = D / 8;          // lanes per run of rows
    constexpr int BPW = 256 / G;      // runs per workgroup (a multiple of RS)
    constexpr int WW = W > 1 ? W - 1 : 1;
    const int64_t run = (int64_t)blockIdx.x * BPW + threadIdx.x / G;
    const int part = threadIdx.x % G;
    const bool live = run < total_blocks * RS;              // (idle lanes still take part in the shuffles)
    const int64_t blk = live ? run / RS : 0;
    const int sp = live ? (int)(run % RS) : 0;
    const int CH = B / RS;                                  // rows per run
    const int64_t s = blk / n;
    const int j = (int)(blk % n);
    const int first = j * B + sp * CH;                      // first row of the run inside the slice
    const int64_t row0 = s * N + first;
    const T* src = K + row0 * D + part * 8;
    T* dst = Keff ? Keff + row0 * D + part * 8 : nullptr;

    float wr[W > 0 ? W : 1][8];
    float win[WW][8];                  // win[l-1] = row t-l
    if constexpr (W > 0) {
        const float* wh = w + ((int64_t)(s % heads) * D + part * 8) * W;
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int l = 0; l < W; ++l) wr[l][e] = wh[e * W + l];
#pragma unroll
        for (int l = 1; l < W; ++l) {
            if (first - l >= 0) Vec8<T>::load(src - (int64_t)l * D, win[l - 1]);
            else {
#pragma unroll
                for (int e = 0; e < 8; ++e) win[l - 1][e] = 0.f;
            }
        }
    }

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int r = 0; r < (live ? CH : 0); ++r) {
        float x[8], y[8];
        Vec8<T>::load(src + (int64_t)r * D, x);
        if constexpr (W > 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float a = wr[0][e] * x[e];
#pragma unroll
                for (int l = 1; l < W; ++l) a = fmaf(wr[l][e], win[l - 1][e], a);
                y[e] = x[e] + a * __builtin_amdgcn_rcpf(1.f + __expf(-a));     // SiLU; sigmoid to ~1 ulp
            }
#pragma unroll
            for (int l = W - 1; l > 1; --l)
#pragma unroll
                for (int e = 0; e < 8; ++e) win[l - 1][e] = win[l - 2][e];
            if constexpr (W > 1) {
#pragma unroll
                for (int e = 0; e < 8; ++e) win[0][e] = x[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = x[e];
        }
        if (dst) Vec8<T>::store(dst + (int64_t)r * D, y);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += Vec8<T>::round(y[e]);
    }
    for (int o = G; o < G * RS; o <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
    if (live && sp == 0) {
        float out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = acc[e] / (float)B;
        Vec8<float>::store(cent + blk * D + part * 8, out);
    }
}

template <typename T, int D>
static hipError_t launch_w(const Dims& s, const void* K, const float* w, void* Keff, float* cent,
                           hipStream_t st)
{
    const int64_t total = (int64_t)s.bh * s.n;
    const int bpw = 256 / (D / 8);
    // runs per block: as many as fit a wave side by side, of at least 8 rows each
    int RS = 1;
    while (RS * 2 * (D / 8) <= kWave && s.B % (RS * 2) == 0 && s.B / (RS * 2) >= 8) RS *= 2;
    dim3 grid((unsigned)((total * RS + bpw - 1) / bpw)), block(256);
#define MOBA_CASE(WV)                                                                      \
    case WV:                                                                               \
        hipLaunchKernelGGL((centroid_kernel<T, D, WV>), grid, block, 0, st, (const T*)K, w, \
                           (T*)Keff, cent, s.heads, s.N, s.B, s.n, total, RS);             \
        break;
    switch (s.W) {
        MOBA_CASE(0) MOBA_CASE(1) MOBA_CASE(2) MOBA_CASE(3) MOBA_CASE(4)
        MOBA_CASE(5) MOBA_CASE(6) MOBA_CASE(7) MOBA_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef MOBA_CASE
    return hipGetLastError();
}

hipError_t launch_centroids(const Dims& s, const void* K, const float* w, void* Keff, float* cent,
                            hipStream_t st)
{
    if (s.dtype == MOBA_BF16)
        return s.D == 64 ? launch_w<bf16_t, 64>(s, K, w, Keff, cent, st)
                         : launch_w<bf16_t, 128>(s, K, w, Keff, cent, st);
    return s.D == 64 ? launch_w<float, 64>(s, K, w, Keff, cent, st)
                     : launch_w<float, 128>(s, K, w, Keff, cent, st);
}

}  // namespace moba
