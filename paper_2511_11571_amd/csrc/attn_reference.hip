// Plain (non-MFMA) MoBA attention, forward and backward, in fp32 arithmetic.
// These kernels serve the fp32 I/O type and every shape the MFMA kernels do not
// cover, and can be forced for any shape with MOBA_FLAG_REFERENCE_KERNELS.
//
// Forward (paper Section 2): one wave per query walks the keys of the kept past
// blocks and of the own block (keys u <= t) 64 at a time, one key per lane, with an
// online softmax; the weighted value sum is then taken with one channel per lane.
// Backward (paper Appendix C.3): D = rowsum(dO o O); dQ per query in the same
// layout as the forward; dK/dV per key block over that block's query list plus its
// own causally masked queries, everything held in registers.
#include "common.h"

namespace moba {

// Position -> key row for the concatenation "kept blocks, then own block prefix".
struct KeyWalk {
    const int32_t* sel;   // kept blocks of this query (k slots, -1 = unused)
    int k, B, t;
    int nsel;             // number of kept blocks (leading non-negative slots)
    int total;            // nsel*B + (t % B) + 1
    __device__ __forceinline__ int key(int i) const
    {
        const int slot = i / B, r = i - slot * B;
        return slot < nsel ? sel[slot] * B + r : (t / B) * B + r;
    }
};

template <typename T, int D>
__device__ __forceinline__ float dot_row(const T* __restrict__ row, const float* __restrict__ v)
{
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < D; c += 8) {
        float x[8];
        Vec8<T>::load(row + c, x);
        const float4 a = *reinterpret_cast<const float4*>(v + c);
        const float4 b = *reinterpret_cast<const float4*>(v + c + 4);
        acc = fmaf(x[0], a.x, acc); acc = fmaf(x[1], a.y, acc);
        acc = fmaf(x[2], a.z, acc); acc = fmaf(x[3], a.w, acc);
        acc = fmaf(x[4], b.x, acc); acc = fmaf(x[5], b.y, acc);
        acc = fmaf(x[6], b.z, acc); acc = fmaf(x[7], b.w, acc);
    }
    return acc;
}

// Compacts the kept blocks of row `sel_in` (entries may be -1 anywhere) into LDS.
__device__ __forceinline__ int compact_sel(const int32_t* sel_in, int32_t* sel_out, int k, int lane)
{
    int cnt = 0;
    for (int c0 = 0; c0 < k; c0 += kWave) {
        const int c = c0 + lane;
        const int v = c < k ? sel_in[c] : -1;
        const uint64_t m = __ballot(v >= 0);
        if (v >= 0) sel_out[cnt + lanes_below(m)] = v;
        cnt += __popcll(m);
    }
    return cnt;
}

// ---------------------------------------------------------------- forward
template <typename T, int D>
__global__ __launch_bounds__(256) void forward_reference_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ idx, T* __restrict__ O, float* __restrict__ lse,
    int N, int B, int k, float scale, int64_t total_rows, int G)
{
    extern __shared__ float smem[];
    constexpr int DP = D / kWave;                 // channels per lane
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    float* qs = smem + wave * (D + 2 * kWave);    // [D] query, [64] p, [64] key row
    float* ps = qs + D;
    int* us = reinterpret_cast<int*>(ps + kWave);
    int32_t* sel = reinterpret_cast<int32_t*>(smem + 4 * (D + 2 * kWave)) + (size_t)wave * k;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    if (row >= total_rows) return;
    const int64_t s = row / N;
    const int t = (int)(row % N);
    const T* Ks = K + (s / G) * N * D;            // G query heads share a key/value head
    const T* Vs = V + (s / G) * N * D;

    for (int c = lane; c < D; c += kWave) qs[c] = to_f32<T>(Q[row * D + c]);
    KeyWalk kw;
    kw.sel = sel; kw.k = k; kw.B = B; kw.t = t;
    kw.nsel = compact_sel(idx + row * k, sel, k, lane);
    kw.total = kw.nsel * B + (t % B) + 1;
    __builtin_amdgcn_wave_barrier();

    float m = -INFINITY, l = 0.f, acc[DP];
#pragma unroll
    for (int e = 0; e < DP; ++e) acc[e] = 0.f;
    for (int i0 = 0; i0 < kw.total; i0 += kWave) {
        const int i = i0 + lane;
        int u = 0;
        float z = -INFINITY;
        if (i < kw.total) {
            u = kw.key(i);
            z = scale * dot_row<T, D>(Ks + (int64_t)u * D, qs);
        }
        const float m_new = fmaxf(m, wave_max(z));
        const float p = __expf(z - m_new);        // exp(-inf) = 0 for idle lanes
        const float alpha = __expf(m - m_new);    // first chunk: exp(-inf) = 0
        l = l * alpha + wave_sum(p);
        m = m_new;
        ps[lane] = p; us[lane] = u;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int e = 0; e < DP; ++e) acc[e] *= alpha;
        const int cnt = min(kWave, kw.total - i0);
        for (int a = 0; a < cnt; ++a) {
            const float pa = ps[a];
            const T* vr = Vs + (int64_t)us[a] * D;
#pragma unroll
            for (int e = 0; e < DP; ++e) acc[e] = fmaf(pa, to_f32<T>(vr[lane + e * kWave]), acc[e]);
        }
        __builtin_amdgcn_wave_barrier();
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < DP; ++e) O[row * D + lane + e * kWave] = from_f32<T>(acc[e] * inv);
    if (lane == 0) lse[row] = m + __logf(l);
}

// ---------------------------------------------------------------- D = rowsum(dO o O)
// packed (may be null): per row (lse log2 e, -D), the two numbers the gathering backward kernels
// need of a query, side by side -- one 8-byte access per gathered row instead of two
template <typename T, int D>
__global__ __launch_bounds__(256) void rowdot_kernel(const T* __restrict__ dO,
                                                     const T* __restrict__ O,
                                                     float* __restrict__ Dv, int64_t total_rows,
                                                     const float* __restrict__ lse,
                                                     float2* __restrict__ packed)
{
    constexpr int G = D / 8;
    const int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;
    const int part = threadIdx.x % G;
    float acc = 0.f;
    if (row < total_rows) {
        float a[8], b[8];
        Vec8<T>::load(dO + row * D + part * 8, a);
        Vec8<T>::load(O + row * D + part * 8, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(a[e], b[e], acc);
    }
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (row < total_rows && part == 0) {
        Dv[row] = acc;
        if (packed) packed[row] = make_float2(lse[row] * 1.4426950408889634f, -acc);
    }
}

// ---------------------------------------------------------------- dQ
template <typename T, int D>
__global__ __launch_bounds__(256) void dq_reference_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ Dv,
    const int32_t* __restrict__ idx, T* __restrict__ dQ, int N, int B, int k, float scale,
    int64_t total_rows, int G)
{
    extern __shared__ float smem[];
    constexpr int DP = D / kWave;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    float* qs = smem + wave * (2 * D + 2 * kWave);    // [D] q, [D] dO, [64] dS, [64] key row
    float* gs = qs + D;
    float* ds = gs + D;
    int* us = reinterpret_cast<int*>(ds + kWave);
    int32_t* sel = reinterpret_cast<int32_t*>(smem + 4 * (2 * D + 2 * kWave)) + (size_t)wave * k;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    if (row >= total_rows) return;
    const int64_t s = row / N;
    const int t = (int)(row % N);
    const T* Ks = K + (s / G) * N * D;            // G query heads share a key/value head
    const T* Vs = V + (s / G) * N * D;
    for (int c = lane; c < D; c += kWave) {
        qs[c] = to_f32<T>(Q[row * D + c]);
        gs[c] = to_f32<T>(dO[row * D + c]);
    }
    KeyWalk kw;
    kw.sel = sel; kw.k = k; kw.B = B; kw.t = t;
    kw.nsel = compact_sel(idx + row * k, sel, k, lane);
    kw.total = kw.nsel * B + (t % B) + 1;
    __builtin_amdgcn_wave_barrier();
    const float L = lse[row], Dt = Dv[row];

    float acc[DP];
#pragma unroll
    for (int e = 0; e < DP; ++e) acc[e] = 0.f;
    for (int i0 = 0; i0 < kw.total; i0 += kWave) {
        const int i = i0 + lane;
        int u = 0;
        float dS = 0.f;
        if (i < kw.total) {
            u = kw.key(i);
            const float z = scale * dot_row<T, D>(Ks + (int64_t)u * D, qs);
            const float dp = dot_row<T, D>(Vs + (int64_t)u * D, gs);
            dS = __expf(z - L) * (dp - Dt);
        }
        ds[lane] = dS; us[lane] = u;
        __builtin_amdgcn_wave_barrier();
        const int cnt = min(kWave, kw.total - i0);
        for (int a = 0; a < cnt; ++a) {
            const float da = ds[a];
            const T* kr = Ks + (int64_t)us[a] * D;
#pragma unroll
            for (int e = 0; e < DP; ++e) acc[e] = fmaf(da, to_f32<T>(kr[lane + e * kWave]), acc[e]);
        }
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int e = 0; e < DP; ++e) dQ[row * D + lane + e * kWave] = from_f32<T>(scale * acc[e]);
}

// ---------------------------------------------------------------- dK, dV
// A workgroup owns 32 keys of one block: thread (u = tid/8, part = tid%8) holds D/8
// channels of key u and of value u, and the matching slices of dK_u and dV_u.  The
// block's queries are visited one at a time by the whole workgroup; the two dot
// products are completed across the 8 lanes of a key by xor shuffles.
template <typename T, int D>
__global__ __launch_bounds__(256) void dkdv_reference_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ Dv,
    const int32_t* __restrict__ off, const int32_t* __restrict__ ql,
    T* __restrict__ dK, T* __restrict__ dV, int N, int B, int n, float scale, int64_t R, int G)
{
    constexpr int C = D / 8;                       // channels per thread
    const int skv = blockIdx.z, j = blockIdx.x, sub = blockIdx.y;   // key/value slice
    const int ul = sub * 32 + threadIdx.x / 8;     // key inside the block
    const int part = threadIdx.x % 8;
    const bool live = ul < B;
    const int u = j * B + (live ? ul : 0);
    const int64_t kbase = (int64_t)skv * N;
    float kr[C], vr[C], dk[C], dv[C];
#pragma unroll
    for (int c = 0; c < C; c += 8) {
        float a[8], b[8];
        Vec8<T>::load(K + (kbase + u) * D + part * C + c, a);
        Vec8<T>::load(V + (kbase + u) * D + part * C + c, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) { kr[c + e] = a[e]; vr[c + e] = b[e]; dk[c + e] = 0.f; dv[c + e] = 0.f; }
    }
    // the query heads that share this key/value head, one after the other (fixed order)
    for (int s = skv * G; s < (skv + 1) * G; ++s) {
    const int64_t base = (int64_t)s * N;
    const int32_t* os = off + (int64_t)s * (n + 1);
    const int32_t* qs = ql + (int64_t)s * R;
    const int lo = os[j], nlist = os[j + 1] - lo;
    for (int a = 0; a < nlist + B; ++a) {
        const int t = a < nlist ? list_query(qs[lo + a]) : j * B + (a - nlist);
        const bool seen = live && (a < nlist || ul <= a - nlist);   // own block: keys <= query
        float q[C], g[C];
#pragma unroll
        for (int c = 0; c < C; c += 8) {
            float x[8], y[8];
            Vec8<T>::load(Q + (base + t) * D + part * C + c, x);
            Vec8<T>::load(dO + (base + t) * D + part * C + c, y);
#pragma unroll
            for (int e = 0; e < 8; ++e) { q[c + e] = x[e]; g[c + e] = y[e]; }
        }
        float z = 0.f, dp = 0.f;
#pragma unroll
        for (int e = 0; e < C; ++e) { z = fmaf(q[e], kr[e], z); dp = fmaf(g[e], vr[e], dp); }
#pragma unroll
        for (int o = 4; o > 0; o >>= 1) { z += __shfl_xor(z, o, 64); dp += __shfl_xor(dp, o, 64); }
        const float p = seen ? __expf(scale * z - lse[base + t]) : 0.f;
        const float dS = p * (dp - Dv[base + t]);
#pragma unroll
        for (int e = 0; e < C; ++e) { dv[e] = fmaf(p, g[e], dv[e]); dk[e] = fmaf(dS, q[e], dk[e]); }
    }
    }
    if (live) {
#pragma unroll
        for (int c = 0; c < C; c += 8) {
            float a[8], b[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) { a[e] = scale * dk[c + e]; b[e] = dv[c + e]; }
            Vec8<T>::store(dK + (kbase + u) * D + part * C + c, a);
            Vec8<T>::store(dV + (kbase + u) * D + part * C + c, b);
        }
    }
}

// ---------------------------------------------------------------- launchers
template <typename T, int D>
static hipError_t fwd_t(const Dims& s, const void* Q, const void* K, const void* V,
                        const int32_t* idx, void* O, float* lse, hipStream_t st)
{
    const int64_t rows = (int64_t)s.bh * s.N;
    if (rows == 0) return hipSuccess;
    const size_t lds = sizeof(float) * 4 * (D + 2 * kWave) + sizeof(int32_t) * 4 * (size_t)s.k;
    if (lds > 64 * 1024) {     // top-k in the thousands: above the default dynamic LDS limit, opt in
        hipError_t e = ensure_dynamic_lds((const void*)forward_reference_kernel<T, D>, (size_t)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((forward_reference_kernel<T, D>), dim3((unsigned)((rows + 3) / 4)), dim3(256),
                       lds, st, (const T*)Q, (const T*)K, (const T*)V, idx, (T*)O, lse, s.N, s.B, s.k,
                       s.scale, rows, s.G);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t bwd_t(const Dims& s, const void* Q, const void* K, const void* V, const void* O,
                        const float* lse, const void* dO, const int32_t* idx, const int32_t* off,
                        const int32_t* ql, void* dQ, void* dK, void* dV, float* Dvec, uint32_t parts,
                        float2* packed, hipStream_t st)
{
    const int64_t rows = (int64_t)s.bh * s.N;
    if (rows == 0) return hipSuccess;
    constexpr int RPB = 256 / (D / 8);
    if (parts & MOBA_BWD_PREPROCESS)
    hipLaunchKernelGGL((rowdot_kernel<T, D>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0,
                       st, (const T*)dO, (const T*)O, Dvec, rows, lse, packed);
    const size_t lds = sizeof(float) * 4 * (2 * D + 2 * kWave) + sizeof(int32_t) * 4 * (size_t)s.k;
    if ((parts & MOBA_BWD_DQ) && lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)dq_reference_kernel<T, D>, (size_t)lds);
        if (e != hipSuccess) return e;
    }
    if (parts & MOBA_BWD_DQ)
    hipLaunchKernelGGL((dq_reference_kernel<T, D>), dim3((unsigned)((rows + 3) / 4)), dim3(256), lds,
                       st, (const T*)Q, (const T*)K, (const T*)V, (const T*)dO, lse, Dvec, idx,
                       (T*)dQ, s.N, s.B, s.k, s.scale, rows, s.G);
    if (parts & MOBA_BWD_DKDV)
    hipLaunchKernelGGL((dkdv_reference_kernel<T, D>), dim3(s.n, (s.B + 31) / 32, s.bhk), dim3(256), 0,
                       st, (const T*)Q, (const T*)K, (const T*)V, (const T*)dO, lse, Dvec, off, ql,
                       (T*)dK, (T*)dV, s.N, s.B, s.n, s.scale, s.R, s.G);
    return hipGetLastError();
}

hipError_t launch_forward_reference(const Dims& s, const void* Q, const void* K, const void* V,
                                    const int32_t* idx, void* O, float* lse, hipStream_t st)
{
    if (s.dtype == MOBA_BF16)
        return s.D == 64 ? fwd_t<bf16_t, 64>(s, Q, K, V, idx, O, lse, st)
                         : fwd_t<bf16_t, 128>(s, Q, K, V, idx, O, lse, st);
    return s.D == 64 ? fwd_t<float, 64>(s, Q, K, V, idx, O, lse, st)
                     : fwd_t<float, 128>(s, Q, K, V, idx, O, lse, st);
}

hipError_t launch_backward_reference(const Dims& s, const void* Q, const void* K, const void* V,
                                     const void* O, const float* lse, const void* dO,
                                     const int32_t* idx, const int32_t* off, const int32_t* ql,
                                     void* dQ, void* dK, void* dV, float* Dvec, uint32_t parts,
                                     float2* packed, hipStream_t st)
{
    if (s.dtype == MOBA_BF16)
        return s.D == 64
                   ? bwd_t<bf16_t, 64>(s, Q, K, V, O, lse, dO, idx, off, ql, dQ, dK, dV, Dvec, parts, packed, st)
                   : bwd_t<bf16_t, 128>(s, Q, K, V, O, lse, dO, idx, off, ql, dQ, dK, dV, Dvec, parts, packed, st);
    return s.D == 64 ? bwd_t<float, 64>(s, Q, K, V, O, lse, dO, idx, off, ql, dQ, dK, dV, Dvec, parts, packed, st)
                     : bwd_t<float, 128>(s, Q, K, V, O, lse, dO, idx, off, ql, dQ, dK, dV, Dvec, parts, packed, st);
}

}  // namespace moba
