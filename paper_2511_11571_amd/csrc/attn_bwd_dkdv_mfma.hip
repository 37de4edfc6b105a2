// dK and dV of the MoBA backward on bf16 MFMA (paper Section 4.2 backward and
// Appendix C.3: one workgroup per key block, queries gathered through the key-block-major
// lists, S recomputed, dV += P^T dO, dS = P o (dP - D), dK += dS^T Q).  Here a workgroup
// owns one 32-key group; its four waves split the group's query list (the routed
// queries of the block, then the block's own queries from this group on, the first 32
// of them causally masked) into steps of 32 queries.  dK^T and dV^T (channels x 32 keys)
// stay in MFMA accumulators for the whole list and are summed over the four waves
// through LDS at the end.
//
// Per step, with queries as the contraction index of the two accumulating products:
//   S  = Q_g K^T, dP = dO_g V^T          gathered rows straight from global memory as A
//                                        operands, K and V rows of the group as B operands;
//   P, dS                                in the result layout: a lane holds one key column
//                                        and query rows 4g..4g+3 of both 16-query tiles,
//                                        which packed to bf16 is already a B operand over
//                                        the 32 queries (slot order of mfma.h);
//   dV^T += dO_g^T P, dK^T += Q_g^T dS   the A operands need the gathered rows transposed:
//                                        they are parked in LDS and read back 16 bits at a
//                                        time in the same slot order.
#include "mfma.h"

namespace moba {

template <int D>
struct DkvCfg {
    static constexpr int NW = 4;
    static constexpr int NT = NW * kWave;
    static constexpr int SSTRIDE = D + 4;              // bf16 per staged row: 4 rows shift 8 banks
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int RSTRIDE = D + 4;              // floats per key row of the reduction buffer
    static constexpr size_t STAGE = (size_t)2 * 32 * SSTRIDE * 2;          // Q and dO, bytes per wave
    static constexpr size_t LDS = NW * (STAGE + 2 * 32 * 4) + (size_t)2 * 32 * RSTRIDE * 4;
};

template <int D>
__global__ __launch_bounds__(DkvCfg<D>::NT) void dkdv_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ lse, const float* __restrict__ Dv,
    const int32_t* __restrict__ off, const int32_t* __restrict__ ql, bf16_t* __restrict__ dK,
    bf16_t* __restrict__ dV, int N, int B, int n, float scale, int64_t R, int groups_per_slice)
{
    using C = DkvCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    bf16_t* stQ = reinterpret_cast<bf16_t*>(smem + wave * (C::STAGE + 256));
    bf16_t* stG = stQ + 32 * C::SSTRIDE;
    float* ls = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(stQ) + C::STAGE);
    float* Ds = ls + 32;
    float* red = reinterpret_cast<float*>(smem + C::NW * (C::STAGE + 256));    // [2][32][RSTRIDE]

    const int s = blockIdx.x / groups_per_slice;
    const int kap = blockIdx.x % groups_per_slice;          // 32-key group inside the slice
    const int NG = B / 32;
    const int j = kap / NG;
    const int64_t sbase = (int64_t)s * N;
    const float c2 = scale * kLog2e;
    const int32_t* os = off + (int64_t)s * (n + 1);
    const int32_t* qs = ql + (int64_t)s * R;
    const int lo = os[j], nlist = os[j + 1] - lo;
    const int own0 = 32 * kap;                              // first own query that sees this group
    const int total = nlist + (j + 1) * B - own0;

    // B operands: the group's keys and values (lane = key m16 of tile nt)
    Frag kb[2][C::KS], vb[2][C::KS];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const int64_t o = (sbase + 32 * kap + 16 * nt + m16) * D + 8 * g + 32 * ks;
            kb[nt][ks].q = *reinterpret_cast<const uint4*>(K + o);
            vb[nt][ks].q = *reinterpret_cast<const uint4*>(V + o);
        }
    f32x4_t dKT[C::MT][2], dVT[C::MT][2];
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            dKT[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            dVT[mt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }

    // The gathers are the long pole (two dependent global loads: list entry, then the row), so
    // they run ahead of the arithmetic: row ids two steps ahead, rows one step ahead.
    auto ids = [&](int a0, int (&t)[2], bool (&ok)[2]) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            const int a = a0 + 16 * qt + m16;
            ok[qt] = a < total;
            t[qt] = !ok[qt] ? own0 : (a < nlist ? qs[lo + a] : own0 + (a - nlist));
        }
    };
    auto fetch = [&](const int (&t)[2], const bool (&ok)[2], Frag (&qa)[2][C::KS], Frag (&ga)[2][C::KS],
                     float (&lv)[2], float (&dv)[2]) {
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                const int64_t o = (sbase + t[qt]) * D + 8 * g + 32 * ks;
                qa[qt][ks].q = *reinterpret_cast<const uint4*>(Q + o);
                ga[qt][ks].q = *reinterpret_cast<const uint4*>(dO + o);
            }
            lv[qt] = INFINITY;                        // rows past the list: P = 0
            dv[qt] = 0.f;
            if (g == 0 && ok[qt]) {
                lv[qt] = lse[sbase + t[qt]] * kLog2e;
                dv[qt] = Dv[sbase + t[qt]];
            }
        }
    };
    const int stride = 32 * C::NW;
    int tN[2];
    bool okN[2];
    Frag qa[2][C::KS], ga[2][C::KS], qaN[2][C::KS], gaN[2][C::KS];
    float lv[2], dv[2], lvN[2], dvN[2];
    {
        int t0[2];
        bool ok0[2];
        ids(32 * wave, t0, ok0);
        fetch(t0, ok0, qa, ga, lv, dv);
        ids(32 * wave + stride, tN, okN);
    }
    for (int a0 = 32 * wave; a0 < total; a0 += stride) {
        fetch(tN, okN, qaN, gaN, lvN, dvN);
        ids(a0 + 2 * stride, tN, okN);
        if (g == 0) {
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                ls[16 * qt + m16] = lv[qt];
                Ds[16 * qt + m16] = dv[qt];
            }
        }
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                const int o = (16 * qt + m16) * C::SSTRIDE + 8 * g + 32 * ks;
                *reinterpret_cast<uint2*>(stQ + o) = make_uint2(qa[qt][ks].u[0], qa[qt][ks].u[1]);
                *reinterpret_cast<uint2*>(stQ + o + 4) = make_uint2(qa[qt][ks].u[2], qa[qt][ks].u[3]);
                *reinterpret_cast<uint2*>(stG + o) = make_uint2(ga[qt][ks].u[0], ga[qt][ks].u[1]);
                *reinterpret_cast<uint2*>(stG + o + 4) = make_uint2(ga[qt][ks].u[2], ga[qt][ks].u[3]);
            }
        // S and dP
        f32x4_t sc[2][2], dp[2][2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                sc[qt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                dp[qt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    sc[qt][nt] = mfma16(qa[qt][ks], kb[nt][ks], sc[qt][nt]);
                    dp[qt][nt] = mfma16(ga[qt][ks], vb[nt][ks], dp[qt][nt]);
                }
            }
        __builtin_amdgcn_wave_barrier();
        // own queries of this very group are causal: key (16 nt + m16) must not exceed the query
        const bool causal = a0 + 32 > nlist && a0 < nlist + 32;    // the step touches own rows 0..31
        Frag pb[2], sb[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            float p[8], d[8];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const f32x4_t l4 = *reinterpret_cast<const f32x4_t*>(ls + 16 * qt + 4 * g);
                const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(Ds + 16 * qt + 4 * g);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float pv = fast_exp2(fmaf(sc[qt][nt][i], c2, -l4[i]));
                    if (causal) {
                        const int a = a0 + 16 * qt + 4 * g + i - nlist;     // own row index, if >= 0
                        if (a >= 0 && a < 32 && 16 * nt + m16 > a) pv = 0.f;
                    }
                    p[4 * qt + i] = pv;
                    d[4 * qt + i] = pv * (dp[qt][nt][i] - d4[i]);
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pb[nt].u[e] = pack2(p[2 * e], p[2 * e + 1]);
                sb[nt].u[e] = pack2(d[2 * e], d[2 * e + 1]);
            }
        }
        // transposed A operands from the staged rows, then the two accumulating products
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
            Frag qT, gT;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r0 = slot_key(g, 2 * e) * C::SSTRIDE + 16 * mt + m16;
                const int r1 = slot_key(g, 2 * e + 1) * C::SSTRIDE + 16 * mt + m16;
                qT.u[e] = (uint32_t)stQ[r0] | ((uint32_t)stQ[r1] << 16);
                gT.u[e] = (uint32_t)stG[r0] | ((uint32_t)stG[r1] << 16);
            }
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                dVT[mt][nt] = mfma16(gT, pb[nt], dVT[mt][nt]);
                dKT[mt][nt] = mfma16(qT, sb[nt], dKT[mt][nt]);
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) { qa[qt][ks] = qaN[qt][ks]; ga[qt][ks] = gaN[qt][ks]; }
            lv[qt] = lvN[qt];
            dv[qt] = dvN[qt];
        }
    }

    // sum the four waves' accumulators through LDS: red[tensor][key][channel]
    for (int w = 0; w < C::NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    float* pk = red + (16 * nt + m16) * C::RSTRIDE + 16 * mt + 4 * g;
                    float* pv = pk + 32 * C::RSTRIDE;
                    f32x4_t a = dKT[mt][nt], b = dVT[mt][nt];
                    if (w > 0) {
                        a += *reinterpret_cast<const f32x4_t*>(pk);
                        b += *reinterpret_cast<const f32x4_t*>(pv);
                    }
                    *reinterpret_cast<f32x4_t*>(pk) = a;
                    *reinterpret_cast<f32x4_t*>(pv) = b;
                }
        }
        __syncthreads();
    }
    for (int i = tid; i < 2 * 32 * (D / 8); i += C::NT) {
        const int which = i / (32 * (D / 8)), rem = i % (32 * (D / 8));
        const int key = rem / (D / 8), c = rem % (D / 8);
        const float* src = red + which * 32 * C::RSTRIDE + key * C::RSTRIDE + 8 * c;
        const float mul = which == 0 ? scale : 1.f;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[e] * mul;
        bf16_t* dst = (which == 0 ? dK : dV) + (sbase + 32 * kap + key) * D + 8 * c;
        Vec8<bf16_t>::store(dst, v);
    }
}

template <int D>
static hipError_t dkdv_launch(const Dims& s, const void* Q, const void* K, const void* V,
                              const void* dO, const float* lse, const float* Dv, const int32_t* off,
                              const int32_t* ql, void* dK, void* dV, hipStream_t st)
{
    using C = DkvCfg<D>;
    const int gps = s.N / 32;
    if (gps == 0) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void*)dkdv_mfma_kernel<D>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((dkdv_mfma_kernel<D>), dim3((unsigned)(gps * s.bh)), dim3(C::NT), C::LDS, st,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, lse, Dv,
                       off, ql, (bf16_t*)dK, (bf16_t*)dV, s.N, s.B, s.n, s.scale, s.R, gps);
    return hipGetLastError();
}

hipError_t launch_dkdv_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                            const void* dO, const float* lse, const float* Dv, const int32_t* off,
                            const int32_t* ql, void* dK, void* dV, hipStream_t st)
{
    return s.D == 64 ? dkdv_launch<64>(s, Q, K, V, dO, lse, Dv, off, ql, dK, dV, st)
                     : dkdv_launch<128>(s, Q, K, V, dO, lse, Dv, off, ql, dK, dV, st);
}

}  // namespace moba
