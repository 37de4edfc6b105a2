// Decode-shaped MoBA forward (inference): the last q_len positions of a sequence of N keys, each
// query routed and attended on its own -- the operator of the paper's Section 2 for a few query
// rows and a long key sequence, where N need not be a multiple of the block size: a query's own
// block is then the ragged last block, attended causally like any own block (the centroid
// algorithm of Appendix C.1 treats the tail block the same way; here its centroid is never
// needed, because the own block is not a routing candidate).
//
// One workgroup of 16 waves per (query, batch*head): gate scores against the centroids of the
// complete past blocks (fp32, a thread per centroid), exact top-k by a four-pass radix select on
// order-preserving keys with ties to the lower block index, then attention over the kept blocks
// and the own block -- the waves take blocks in turn, each with its own running softmax, merged
// through LDS.  All arithmetic in
// fp32; nothing is written to global memory but O, lse and (optionally) the kept blocks.  The
// work per query is a few hundred KB of reads: the kernel is bound by latency, not by a pipe.
#include "common.h"

namespace moba {

// fp32 -> uint32 with the same order (negative numbers reversed, then below the positive ones)
__device__ __forceinline__ uint32_t decode_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <typename T, int D>
__device__ __forceinline__ float decode_dot(const T* __restrict__ row, const float* __restrict__ v)
{
    float acc = 0.f;
#pragma unroll
    for (int c0 = 0; c0 < D; c0 += 32) {                    // four independent loads at a time
        float x[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) Vec8<T>::load(row + c0 + 8 * i, x[i]);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf(x[i][e], v[c0 + 8 * i + e], acc);
    }
    return acc;
}

constexpr int kDecodeWaves = 16;
constexpr int kDecodeThreads = kDecodeWaves * kWave;

template <typename T, int D>
__global__ __launch_bounds__(kDecodeThreads) void decode_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const float* __restrict__ cent, T* __restrict__ O, float* __restrict__ lse,
    int32_t* __restrict__ idx_out, int N, int B, int k, int q_len, int cblocks, float scale, int G,
    int npast_max)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr int NT = kDecodeThreads, NW = kDecodeWaves;
    float* qs = reinterpret_cast<float*>(smem_raw);         // [D] the query
    float* sc = qs + D;                                     // [npast_max] gate scores
    uint32_t* hist = reinterpret_cast<uint32_t*>(sc + npast_max);   // [256]
    int* ctl = reinterpret_cast<int*>(hist + 256);          // prefix, need, number of kept blocks
    int* sel = ctl + 4;                                     // [k] kept blocks, ascending
    float* ps = reinterpret_cast<float*>(sel + k + 1);      // [NW][64] probabilities of a step
    float* mrg = ps + NW * kWave;                           // [NW][D + 2] the waves' (m, l, O)

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int r = blockIdx.x, s = blockIdx.y, skv = s / G;  // G query heads share a key/value head
    const int t = N - q_len + r;                            // position of the query
    const int past = t / B;                                 // complete blocks before its own block
    const int64_t qrow = (int64_t)s * q_len + r;

    for (int c = tid; c < D; c += NT) qs[c] = to_f32<T>(Q[qrow * D + c]);
    __syncthreads();

    // ---- gate scores q . centroid_j for the past blocks, a thread per centroid (all the loads of
    // a row are independent: one memory latency per row, not one per piece)
    if (k > 0) {
        for (int j = tid; j < past; j += NT) {
            const float4* c = reinterpret_cast<const float4*>(cent + ((int64_t)skv * cblocks + j) * D);
            float a = 0.f;
#pragma unroll
            for (int h = 0; h < D / 4; h += 8) {            // eight independent 16-byte loads at a time
                float4 x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = c[h + e];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float4 y = *reinterpret_cast<const float4*>(qs + 4 * (h + e));
                    a = fmaf(x[e].x, y.x, a); a = fmaf(x[e].y, y.y, a);
                    a = fmaf(x[e].z, y.z, a); a = fmaf(x[e].w, y.w, a);
                }
            }
            sc[j] = a;
        }
    }
    __syncthreads();

    // ---- the k largest scores, ties to the lower block (Section 2): radix select, 8 bits a pass
    const int want = min(k, past);
    if (past > k && k > 0) {
        if (tid == 0) { ctl[0] = 0; ctl[1] = k; }
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t prefix = (uint32_t)ctl[0];
            for (int j = tid; j < past; j += NT) {
                const uint32_t key = decode_key(sc[j]);
                if (shift == 24 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (wave == 0) {
                // the bin that holds the need-th largest key: lane l owns bins 4l .. 4l+3; above[l]
                // = keys in the bins of the lanes above it (suffix sum over the lanes)
                const int need = ctl[1];
                int c4[4], mine = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) { c4[i] = (int)hist[4 * lane + i]; mine += c4[i]; }
                int incl = mine;
#pragma unroll
                for (int o = 1; o < kWave; o <<= 1) {
                    const int v = __shfl_down(incl, o, kWave);
                    if (lane + o < kWave) incl += v;
                }
                const int above = incl - mine;
                // exactly one lane has above < need <= above + mine (the total is at least need);
                // should the counts ever fall short, lane 0 takes it with its lowest bin
                const bool here = (above < need && need <= incl) || (lane == 0 && incl < need);
                if (here) {
                    int left = need - above, b = 3;
                    for (; b > 0; --b) {
                        if (c4[b] >= left) break;
                        left -= c4[b];
                    }
                    ctl[0] = (int)((prefix << 8) | (uint32_t)(4 * lane + b));
                    ctl[1] = left;
                }
            }
            __syncthreads();
        }
        // kept: key above the k-th largest key T, and the first `need` blocks whose key equals T.
        // Wave 0, a contiguous chunk of blocks per lane, two passes around two prefix sums.
        if (wave == 0) {
            const uint32_t T0 = (uint32_t)ctl[0];
            const int need = ctl[1];
            const int chunk = (past + kWave - 1) / kWave;
            const int lo = min(lane * chunk, past), hi = min(lo + chunk, past);
            int gt = 0, eq = 0;
            for (int j = lo; j < hi; ++j) {
                const uint32_t key = decode_key(sc[j]);
                gt += key > T0;
                eq += key == T0;
            }
            int eq_before = eq, kept;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int v = __shfl_up(eq_before, o, kWave);
                if (lane >= o) eq_before += v;
            }
            eq_before -= eq;
            int quota = min(max(need - eq_before, 0), eq);
            kept = gt + quota;
            int pos = kept;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int v = __shfl_up(pos, o, kWave);
                if (lane >= o) pos += v;
            }
            pos -= kept;
            for (int j = lo; j < hi; ++j) {
                const uint32_t key = decode_key(sc[j]);
                bool take = key > T0;
                if (key == T0 && quota > 0) { take = true; --quota; }
                if (take && pos < k) sel[pos++] = j;
            }
        }
    } else {
        for (int j = tid; j < want; j += NT) sel[j] = j;    // fewer past blocks than k: keep them all
    }
    __syncthreads();
    if (idx_out)
        for (int c = tid; c < k; c += NT) idx_out[qrow * k + c] = c < want ? sel[c] : -1;

    // ---- attention over the kept blocks and the own block (keys own*B .. t), one block per wave
    // at a time, 64 keys a step.  Scores: a lane per key (the pieces of its K row are independent
    // loads).  P V: a lane per (key, 16-byte piece of its V row), KPI keys per load instruction,
    // all instructions of a step independent; the lanes that hold the same piece are summed at
    // the end.
    constexpr int PPR = D * (int)sizeof(T) / 16;            // 16-byte pieces per row
    constexpr int EPP = 16 / (int)sizeof(T);                // elements per piece
    constexpr int KPI = kWave / PPR;                        // keys per load instruction
    const int piece = lane % PPR, kslot = lane / PPR;
    const int nb = want + 1;
    float m = -INFINITY, l = 0.f, acc[EPP];
#pragma unroll
    for (int e = 0; e < EPP; ++e) acc[e] = 0.f;
    float* pw = ps + wave * kWave;
    for (int i = wave; i < nb; i += NW) {
        const int j = i < want ? sel[i] : past;
        const int nk = i < want ? B : t - past * B + 1;
        const int64_t base = (int64_t)skv * N + (int64_t)j * B;
        for (int u0 = 0; u0 < nk; u0 += kWave) {
            const int u = u0 + lane;
            // (a lane past the end reads the block's last key again and drops the result: the
            // loads stay unconditional)
            const float zz = scale * decode_dot<T, D>(K + (base + min(u, nk - 1)) * D, qs);
            const float z = u < nk ? zz : -INFINITY;
            const float m_new = fmaxf(m, wave_max(z));
            const float p = __expf(z - m_new);              // exp(-inf) = 0 for idle lanes
            const float alpha = __expf(m - m_new);          // first step: exp(-inf) = 0
            l = l * alpha + wave_sum(p);
            m = m_new;
            pw[lane] = p;
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < EPP; ++e) acc[e] *= alpha;
            const int cnt = min(kWave, nk - u0);
#pragma unroll 8
            for (int a0 = 0; a0 < kWave; a0 += KPI) {
                const int a = a0 + kslot;
                const float pa = a < cnt ? pw[a] : 0.f;
                const T* vr = V + (base + u0 + min(a, cnt - 1)) * D + piece * EPP;
                float v[EPP];
                if constexpr (sizeof(T) == 2) {
                    Vec8<T>::load(vr, v);
                } else {
                    const float4 x = *reinterpret_cast<const float4*>(vr);
                    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                }
#pragma unroll
                for (int e = 0; e < EPP; ++e) acc[e] = fmaf(pa, v[e], acc[e]);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    // the lanes of a wave that hold the same piece (every kslot)
#pragma unroll
    for (int o = PPR; o < kWave; o <<= 1)
#pragma unroll
        for (int e = 0; e < EPP; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
    // ---- merge the waves (a wave without a block has m = -inf, l = 0: weight 0)
    float* mw = mrg + wave * (D + 2);
    if (lane == 0) { mw[0] = m; mw[1] = l; }
    if (kslot == 0) {
#pragma unroll
        for (int e = 0; e < EPP; ++e) mw[2 + piece * EPP + e] = acc[e];
    }
    __syncthreads();
    float M = -INFINITY;
    for (int w = 0; w < NW; ++w) M = fmaxf(M, mrg[w * (D + 2)]);
    float L = 0.f;
    for (int w = 0; w < NW; ++w) L += mrg[w * (D + 2) + 1] * __expf(mrg[w * (D + 2)] - M);
    for (int c = tid; c < D; c += NT) {
        float o = 0.f;
        for (int w = 0; w < NW; ++w) o = fmaf(mrg[w * (D + 2) + 2 + c], __expf(mrg[w * (D + 2)] - M), o);
        O[qrow * D + c] = from_f32<T>(o / L);
    }
    if (tid == 0) lse[qrow] = M + __logf(L);
}

template <typename T, int D>
static hipError_t decode_t(const Dims& s, int q_len, const void* Q, const void* K, const void* V,
                           const float* cent, int cblocks, void* O, float* lse, int32_t* idx,
                           hipStream_t st)
{
    const int npast_max = (s.N - 1) / s.B;
    const size_t lds = sizeof(float) * (size_t)(D + npast_max + 256 + 4 + (s.k + 1) + kDecodeWaves * kWave +
                                                kDecodeWaves * (D + 2));
    if (lds > 64 * 1024) {
        hipError_t e = ensure_dynamic_lds((const void*)decode_kernel<T, D>, (size_t)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_kernel<T, D>), dim3((unsigned)q_len, (unsigned)s.bh), dim3(kDecodeThreads), lds, st,
                       (const T*)Q, (const T*)K, (const T*)V, cent, (T*)O, lse, idx, s.N, s.B, s.k, q_len,
                       cblocks, s.scale, s.G, npast_max);
    return hipGetLastError();
}

hipError_t launch_decode(const Dims& s, int q_len, const void* Q, const void* K, const void* V,
                         const float* cent, int cblocks, void* O, float* lse, int32_t* idx, hipStream_t st)
{
    if (s.dtype == MOBA_BF16)
        return s.D == 64 ? decode_t<bf16_t, 64>(s, q_len, Q, K, V, cent, cblocks, O, lse, idx, st)
                         : decode_t<bf16_t, 128>(s, q_len, Q, K, V, cent, cblocks, O, lse, idx, st);
    return s.D == 64 ? decode_t<float, 64>(s, q_len, Q, K, V, cent, cblocks, O, lse, idx, st)
                     : decode_t<float, 128>(s, q_len, Q, K, V, cent, cblocks, O, lse, idx, st);
}

}  // namespace moba
