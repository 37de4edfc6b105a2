// Backward of the key convolution (paper Appendix B: K' = K + SiLU(a), a_t = sum_l w_l K_{t-l};
// the gradients of routing and attention reach the token-level keys and the kernel weights
// through it).  With G = dL/dK' and g_t = G_t SiLU'(a_t):
//   dK_t = G_t + sum_{l<W, t+l<N} w_l g_{t+l},      dw_l = sum_{slices of the head} sum_t g_t K_{t-l}.
// One pass over K and G: a group of D/8 lanes walks a chunk of consecutive rows, 8 channels per
// lane.  Row u enters with K_u and G_u; a_u needs the W rows of K ending at u (a register
// window), and g_u adds w_l g_u to the unfinished dK rows u-l (a second window), so row
// u-W+1 is complete when row u has been seen.  A chunk runs W-1 rows past its end to finish its
// last rows; it adds to dw only for the rows it owns.  The dw sums of a workgroup's chunks are
// added up on chip, go to the workspace, and a second kernel adds those up, everything in a
// fixed order (bit-reproducible).
#include "common.h"

namespace moba {

constexpr int kConvRows = 128;     // rows per chunk

template <typename T, int D, int W>
__global__ __launch_bounds__(256) void conv_bwd_kernel(
    const T* __restrict__ K, const float* __restrict__ w, const T* __restrict__ G,
    T* __restrict__ dK, float* __restrict__ part, int heads, int N, int nck)
{
    constexpr int GL = D / 8;          // lanes per chunk
    constexpr int CPW = 256 / GL;      // chunks per workgroup
    __shared__ float red[4][D * W];    // the four waves' dw sums
    const int ck = blockIdx.x * CPW + threadIdx.x / GL;
    const int lane8 = threadIdx.x % GL;
    const int s = blockIdx.y;
    // a chunk past the end of the sequence has no rows: it only takes part in the dw sum
    const int r0 = min(N, ck * kConvRows), r1 = min(N, r0 + kConvRows);
    const int64_t base = (int64_t)s * N * D + lane8 * 8;

    float wr[W][8], kw[W][8], acc[W][8], dwa[W][8];    // kw[l] = K[u-l]; acc[l] = unfinished dK[u-l]
    const float* wh = w + ((int64_t)(s % heads) * D + lane8 * 8) * W;
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int l = 0; l < W; ++l) wr[l][e] = wh[e * W + l];
#pragma unroll
    for (int l = 0; l < W; ++l)
#pragma unroll
        for (int e = 0; e < 8; ++e) { acc[l][e] = 0.f; dwa[l][e] = 0.f; kw[l][e] = 0.f; }
    // rows r0-W+1 .. r0-1 of K: kw[l] must hold K[u-l] when u = r0 enters, i.e. after one shift
#pragma unroll
    for (int l = 1; l < W; ++l)
        if (r0 - l >= 0) Vec8<T>::load(K + base + (int64_t)(r0 - l) * D, kw[l - 1]);

#pragma unroll 4
    for (int u = r0; u < (r1 > r0 ? r1 + W - 1 : r0); ++u) {
        // shift the windows: slot 0 is row u
#pragma unroll
        for (int l = W - 1; l > 0; --l)
#pragma unroll
            for (int e = 0; e < 8; ++e) { kw[l][e] = kw[l - 1][e]; acc[l][e] = acc[l - 1][e]; }
        // unconditional loads (a load inside a branch is waited for at the end of the branch,
        // which would put a full memory latency on every row); rows past the end read as zero
        float gu[8], Gu[8];
        const int64_t ur = min(u, N - 1);
        Vec8<T>::load(K + base + ur * D, kw[0]);
        Vec8<T>::load(G + base + ur * D, Gu);
        if (u >= N) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { kw[0][e] = 0.f; Gu[e] = 0.f; }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = wr[0][e] * kw[0][e];
#pragma unroll
            for (int l = 1; l < W; ++l) a = fmaf(wr[l][e], kw[l][e], a);
            const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-a));     // sigmoid, ~1 ulp
            gu[e] = Gu[e] * sg * (1.f + a * (1.f - sg));
            acc[0][e] = Gu[e];
        }
        const bool own = u < r1;           // rows past the chunk belong to the next one
#pragma unroll
        for (int l = 0; l < W; ++l)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                acc[l][e] = fmaf(wr[l][e], gu[e], acc[l][e]);
                if (own) dwa[l][e] = fmaf(gu[e], kw[l][e], dwa[l][e]);
            }
        const int done = u - (W - 1);      // this row has now seen g of all its W successors
        if (done >= r0 && done < r1) Vec8<T>::store(dK + base + (int64_t)done * D, acc[W - 1]);
    }
    // dw of the workgroup: lane groups of a wave by shuffles, the four waves through LDS, all in
    // a fixed order
#pragma unroll
    for (int o = GL; o < kWave; o <<= 1)
#pragma unroll
        for (int l = 0; l < W; ++l)
#pragma unroll
            for (int e = 0; e < 8; ++e) dwa[l][e] += __shfl_xor(dwa[l][e], o, kWave);
    const int wave = threadIdx.x / kWave;
    if (threadIdx.x % kWave < GL) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int l = 0; l < W; ++l) red[wave][(lane8 * 8 + e) * W + l] = dwa[l][e];
    }
    __syncthreads();
    float* p = part + ((int64_t)s * gridDim.x + blockIdx.x) * (D * W);
    for (int i = threadIdx.x; i < D * W; i += 256) p[i] = (red[0][i] + red[1][i]) + (red[2][i] + red[3][i]);
}

// dw[h][c][l] = sum over the slices of head h (batch order) and over their workgroups (ascending)
__global__ __launch_bounds__(256) void conv_bwd_reduce_kernel(const float* __restrict__ part,
                                                              float* __restrict__ dw, int batch,
                                                              int heads, int nck, int DW)
{
    const int i = blockIdx.x * 256 + threadIdx.x;      // (c, l) of head blockIdx.y
    const int h = blockIdx.y;
    if (i >= DW) return;
    float sum = 0.f;
    for (int b = 0; b < batch; ++b) {
        const float* p = part + ((int64_t)(b * heads + h) * nck) * DW + i;
        for (int ck = 0; ck < nck; ++ck) sum += p[(int64_t)ck * DW];
    }
    dw[(int64_t)h * DW + i] = sum;
}

size_t conv_bwd_ws_bytes(const Dims& s)
{
    const int nck = (s.N + kConvRows - 1) / kConvRows;
    const int cpw = 256 / (s.D / 8);
    return sizeof(float) * (size_t)s.bh * ((nck + cpw - 1) / cpw) * s.D * (s.W > 0 ? s.W : 1);
}

template <typename T, int D>
static hipError_t launch_w(const Dims& s, const void* K, const float* w, const void* G, void* dK,
                           float* dw, float* part, hipStream_t st)
{
    const int nck = (s.N + kConvRows - 1) / kConvRows;
    const int cpw = 256 / (D / 8);
    dim3 grid((unsigned)((nck + cpw - 1) / cpw), (unsigned)s.bh), block(256);
#define MOBA_CASE(WV)                                                                       \
    case WV:                                                                                \
        hipLaunchKernelGGL((conv_bwd_kernel<T, D, WV>), grid, block, 0, st, (const T*)K, w, \
                           (const T*)G, (T*)dK, part, s.heads, s.N, nck);                   \
        break;
    switch (s.W) {
        MOBA_CASE(1) MOBA_CASE(2) MOBA_CASE(3) MOBA_CASE(4)
        MOBA_CASE(5) MOBA_CASE(6) MOBA_CASE(7) MOBA_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef MOBA_CASE
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int DW = D * s.W;
    hipLaunchKernelGGL(conv_bwd_reduce_kernel, dim3((unsigned)((DW + 255) / 256), (unsigned)s.heads),
                       dim3(256), 0, st, part, dw, s.bh / s.heads, s.heads, (int)grid.x, DW);
    return hipGetLastError();
}

hipError_t launch_conv_backward(const Dims& s, const void* K, const float* w, const void* G, void* dK,
                                float* dw, void* ws, hipStream_t st)
{
    if (s.bh == 0 || s.N == 0) return hipSuccess;
    float* part = static_cast<float*>(ws);
    if (s.dtype == MOBA_BF16)
        return s.D == 64 ? launch_w<bf16_t, 64>(s, K, w, G, dK, dw, part, st)
                         : launch_w<bf16_t, 128>(s, K, w, G, dK, dw, part, st);
    return s.D == 64 ? launch_w<float, 64>(s, K, w, G, dK, dw, part, st)
                     : launch_w<float, 128>(s, K, w, G, dK, dw, part, st);
}

}  // namespace moba
