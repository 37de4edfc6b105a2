// Prepared copies of K and V for the query-tile attention kernels, made in two launches:
// the per-channel maxima of K and V (one kernel for both), then one pass that reads every
// 32-row group of K and V once and writes whichever of the four copies the caller asks for:
//   Ka, Va  K / V in MFMA operand order (see operand layout in mfma.h)
//   Kt, Vt  K / V slot-ordered transposed, each channel scaled by 2^-e to magnitude <= 1
// The forward needs Ka and Vt (+ the maxima of V), the dQ kernel Ka, Va and Kt (+ both maxima).
// A caller that hands the same workspace to forward and backward (MOBA_FLAG_SHARED_WORKSPACE)
// has all of it made once, in the forward call.
#include "mfma.h"

namespace moba {

__global__ void zero_words2_kernel(uint32_t* p, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// blockIdx.z = 0: K -> kmax, 1: V -> vmax; max_t |X[s][t][c]| as raw fp32 bits (non-negative
// floats order like integers)
template <int D>
__global__ __launch_bounds__(256) void absmax2_kernel(const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                                      uint32_t* __restrict__ kmax, uint32_t* __restrict__ vmax,
                                                      int N, int rows_per_wg, int first_z)
{
    __shared__ uint32_t red[256 / (D / 8)][D];
    constexpr int G = D / 8;
    const int z = blockIdx.z + first_z;
    const bf16_t* X = z == 0 ? K : V;
    uint32_t* out = z == 0 ? kmax : vmax;
    const int s = blockIdx.y, part = threadIdx.x % G, rr = threadIdx.x / G;
    const int r0 = blockIdx.x * rows_per_wg, r1 = min(N, r0 + rows_per_wg);
    // magnitudes compared as integers: infinities and NaNs come out on top instead of being dropped,
    // and the kernels that read the maxima turn them into NaN results
    uint32_t mx[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll 4
    for (int r = r0 + rr; r < r1; r += 256 / G) {
        float v[8];
        Vec8<bf16_t>::load(X + ((int64_t)s * N + r) * D + part * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) mx[e] = max(mx[e], __float_as_uint(v[e]) & 0x7fffffffu);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rr][part * 8 + e] = mx[e];
    __syncthreads();
    if (threadIdx.x < D) {
        uint32_t m = 0u;
        for (int i = 0; i < 256 / G; ++i) m = max(m, red[i][threadIdx.x]);
        atomicMax(&out[s * D + threadIdx.x], m);
    }
}

// one workgroup per 32-row group (over all key/value slices)
template <int D>
__global__ __launch_bounds__(256) void relayout_kernel(const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
                                                       const uint32_t* __restrict__ kmax,
                                                       const uint32_t* __restrict__ vmax, bf16_t* __restrict__ Ka,
                                                       bf16_t* __restrict__ Va, bf16_t* __restrict__ Kt,
                                                       bf16_t* __restrict__ Vt, int64_t groups_per_slice)
{
    constexpr int KS = D / 32, LD = D + 8;
    __shared__ __align__(16) bf16_t tile[2][32 * LD];
    const int64_t kap = blockIdx.x;            // group index over all slices
    const int s = (int)(kap / groups_per_slice);
    const bool needK = Ka || Kt, needV = Va || Vt;
    for (int i = threadIdx.x; i < 32 * D / 8; i += 256) {
        const int r = i / (D / 8), c = i % (D / 8);
        if (needK)
            *reinterpret_cast<uint4*>(&tile[0][r * LD + c * 8]) =
                *reinterpret_cast<const uint4*>(K + kap * 32 * D + r * D + c * 8);
        if (needV)
            *reinterpret_cast<uint4*>(&tile[1][r * LD + c * 8]) =
                *reinterpret_cast<const uint4*>(V + kap * 32 * D + r * D + c * 8);
    }
    __syncthreads();
    // operand order: the 16 bytes of lane (m, g) for rows 16 mt + m, channels 32 ks + 8 g .. + 8
    for (int i = threadIdx.x; i < 2 * KS * 64; i += 256) {
        const int lane = i % 64, ks = (i / 64) % KS, mt = i / (64 * KS);
        const int off = (16 * mt + (lane & 15)) * LD + 32 * ks + 8 * (lane >> 4);
        const int64_t dst = (kap * (2 * KS) + i / 64) * 512 + lane * 8;
        if (Ka) *reinterpret_cast<uint4*>(Ka + dst) = *reinterpret_cast<const uint4*>(&tile[0][off]);
        if (Va) *reinterpret_cast<uint4*>(Va + dst) = *reinterpret_cast<const uint4*>(&tile[1][off]);
    }
    // slot-ordered transposed and scaled: lane (g, m) of M-tile mt holds channel tile_chan(mt, m)
    // of the keys slot_key(g, 0 .. 7)
    for (int i = threadIdx.x; i < (D / 16) * 64; i += 256) {
        const int mt = i / 64, lane = i % 64, g = lane >> 4, m = lane & 15;
        const int ch = tile_chan<D>(mt, m);
        const int64_t dst = slot_major_offset<D>(kap, mt, lane);
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            bf16_t* out = which == 0 ? Kt : Vt;
            if (!out) continue;
            const int e = scale_exponent((which == 0 ? kmax : vmax)[s * D + ch]);
            float v[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) v[p] = ldexpf(bf16_to_f32(tile[which][slot_key(g, p) * LD + ch]), -e);
            Vec8<bf16_t>::store(out + dst, v);
        }
    }
}

// kv: the key/value-shaped view of the shape.  Null output pointers are skipped; kmax is needed
// for Kt, vmax for Vt (and by the kernels that undo the scaling).
hipError_t launch_prepare(const Dims& kv, const void* K, const void* V, const Prepared& p, hipStream_t st)
{
    if (kv.N == 0 || kv.bh == 0) return hipSuccess;
    const int cnt = kv.bh * kv.D;
    const bool wantK = p.kmax != nullptr, wantV = p.vmax != nullptr;
    if (wantK || wantV) {
        // (kmax and vmax are neighbours in the workspace: one launch clears both)
        uint32_t* first = wantK ? p.kmax : p.vmax;
        const int words = (int)((wantK && wantV ? (p.vmax - p.kmax) : 0) + cnt);
        hipLaunchKernelGGL(zero_words2_kernel, dim3((words + 255) / 256), dim3(256), 0, st, first, words);
        const int rows_per_wg = 256;                       // enough workgroups to keep all of HBM busy
        dim3 grid((kv.N + rows_per_wg - 1) / rows_per_wg, kv.bh, (wantK ? 1 : 0) + (wantV ? 1 : 0));
        const int first_z = wantK ? 0 : 1;
        if (kv.D == 64)
            hipLaunchKernelGGL(absmax2_kernel<64>, grid, dim3(256), 0, st, (const bf16_t*)K, (const bf16_t*)V,
                               p.kmax, p.vmax, kv.N, rows_per_wg, first_z);
        else
            hipLaunchKernelGGL(absmax2_kernel<128>, grid, dim3(256), 0, st, (const bf16_t*)K, (const bf16_t*)V,
                               p.kmax, p.vmax, kv.N, rows_per_wg, first_z);
    }
    const int64_t gps = kv.N / 32, groups = (int64_t)kv.bh * gps;
    if (groups == 0) return hipGetLastError();
    if (kv.D == 64)
        hipLaunchKernelGGL(relayout_kernel<64>, dim3((unsigned)groups), dim3(256), 0, st, (const bf16_t*)K,
                           (const bf16_t*)V, p.kmax, p.vmax, (bf16_t*)p.Ka, (bf16_t*)p.Va, (bf16_t*)p.Kt,
                           (bf16_t*)p.Vt, gps);
    else
        hipLaunchKernelGGL(relayout_kernel<128>, dim3((unsigned)groups), dim3(256), 0, st, (const bf16_t*)K,
                           (const bf16_t*)V, p.kmax, p.vmax, (bf16_t*)p.Ka, (bf16_t*)p.Va, (bf16_t*)p.Kt,
                           (bf16_t*)p.Vt, gps);
    return hipGetLastError();
}

// Places the parts named in `mask` one after the other from `base` on (maxima first); returns the
// bytes taken.  With base == nullptr only the size is computed.
size_t prepared_layout(const Dims& s, unsigned mask, void* base, Prepared* out)
{
    char* p = static_cast<char*>(base);
    size_t used = 0;
    Prepared r;
    auto take = [&](size_t bytes) { void* at = base ? p + used : nullptr; used += a256(bytes); return at; };
    const size_t maxima = sizeof(uint32_t) * (size_t)s.bhk * s.D, tensor = sizeof(bf16_t) * (size_t)s.bhk * s.N * s.D;
    // (kmax and vmax always both: they are small, and one launch clears them)
    r.kmax = static_cast<uint32_t*>(take(maxima));
    r.vmax = static_cast<uint32_t*>(take(maxima));
    r.Ka = mask & kPrepKa ? take(tensor) : nullptr;
    r.Vt = mask & kPrepVt ? take(tensor) : nullptr;
    r.Kt = mask & kPrepKt ? take(tensor) : nullptr;
    r.Va = mask & kPrepVa ? take(tensor) : nullptr;
    if (out) *out = r;
    return used;
}

}  // namespace moba
