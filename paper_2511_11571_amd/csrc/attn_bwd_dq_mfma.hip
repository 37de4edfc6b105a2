// dQ of the MoBA backward on bf16 MFMA (paper Appendix C.3: P = exp(S - L),
// dP = dO V^T, dS = P o (dP - D), dQ = dS K), query-tile resident like the forward: a
// workgroup keeps the Q and dO rows of its tile and their dQ accumulators in LDS and
// walks the 32-key groups the rows were routed to.  The paper accumulates dQ with float
// atomics on a global buffer; measured on this chip those are two orders of magnitude
// too slow, and LDS float atomics one order, so dQ is accumulated here with LDS *integer*
// atomics in 32-bit fixed point, which is also order-independent (bit-reproducible).
//
// Scaling that makes fixed point safe: K is pre-scaled per channel to |k| <= 1 (slot-ordered
// transposed copy), and each row t carries a power of two 2^e_t >= sum_c |dO_tc| vmax_c + |D_t|
// >= |dP_tu - D_t| for every key u.  Then |dS_tu| 2^-e_t <= P_tu, and since the P of a row
// sum to one, |sum_u dS_tu k_u| 2^-e_t <= 1: the accumulator holds that sum times 2^30.
#include "mfma.h"

namespace moba {

template <int D>
struct DqCfg {
    static constexpr int TILE = D == 64 ? 256 : 128;
    static constexpr int NW = 8;
    static constexpr int NT = NW * kWave;
    static constexpr int QSTRIDE = D * 2 + 16;         // bytes per Q / dO row in LDS
    static constexpr int OSTRIDE = D + 1;              // words per accumulator row
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int MW = TILE / 32;
    static constexpr int RANGE = 256;                  // key groups per bit matrix
    static constexpr size_t LDS = (size_t)2 * TILE * QSTRIDE + 4 * TILE * OSTRIDE + 4 * 3 * TILE +
                                  4 * RANGE * MW + 2 * NW * TILE + 64;
};

constexpr float kDqBits = 30.f;

template <int D>
__global__ __launch_bounds__(DqCfg<D>::NT) void dq_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ Kt, const uint32_t* __restrict__ kmax,
    const uint32_t* __restrict__ vmax, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ Dv, const int32_t* __restrict__ idx, bf16_t* __restrict__ dQ, int N,
    int B, int k, float scale, int ntiles, int bh)
{
    using C = DqCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Qs = smem;
    unsigned char* Gs = Qs + (size_t)C::TILE * C::QSTRIDE;
    int* acc = reinterpret_cast<int*>(Gs + (size_t)C::TILE * C::QSTRIDE);
    float* pexp = reinterpret_cast<float*>(acc + C::TILE * C::OSTRIDE);   // lse*log2e - 30 + e_t
    float* Dr = pexp + C::TILE;
    int* esc = reinterpret_cast<int*>(Dr + C::TILE);
    uint32_t* mask = reinterpret_cast<uint32_t*>(esc + C::TILE);
    uint16_t* rlist = reinterpret_cast<uint16_t*>(mask + C::RANGE * C::MW);
    int* next = reinterpret_cast<int*>(rlist + C::NW * C::TILE);

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    const int s = blockIdx.x % bh;
    const int tile = ntiles - 1 - blockIdx.x / bh;
    const int t0 = tile * C::TILE;
    const int rows_here = min(C::TILE, N - t0);
    const int NG = B / 32;
    const float c2 = scale * kLog2e;
    const int64_t sbase = (int64_t)s * N;
    const bf16_t* Kg = K + sbase * D;
    const bf16_t* Vg = V + sbase * D;
    const bf16_t* Ktg = Kt + sbase * D;
    uint16_t* rl = rlist + wave * C::TILE;

    // 0. Q and dO tiles -> LDS; clear the accumulators
    for (int i = tid; i < C::TILE * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        uint4 q = make_uint4(0, 0, 0, 0), gq = q;
        if (r < rows_here) {
            q = *reinterpret_cast<const uint4*>(Q + (sbase + t0 + r) * D + c * 8);
            gq = *reinterpret_cast<const uint4*>(dO + (sbase + t0 + r) * D + c * 8);
        }
        *reinterpret_cast<uint4*>(Qs + (size_t)r * C::QSTRIDE + c * 16) = q;
        *reinterpret_cast<uint4*>(Gs + (size_t)r * C::QSTRIDE + c * 16) = gq;
    }
    for (int i = tid; i < C::TILE * C::OSTRIDE; i += C::NT) acc[i] = 0;
    __syncthreads();
    // per-row scale: 2^e_t >= sum_c |dO_tc| 2^ev_c + |D_t|
    for (int r = tid; r < C::TILE; r += C::NT) {
        float bound = 0.f, Dt = 0.f, L = 0.f;
        if (r < rows_here) {
            const bf16_t* grow = reinterpret_cast<const bf16_t*>(Gs + (size_t)r * C::QSTRIDE);
            for (int c = 0; c < D; ++c)
                bound += fabsf(bf16_to_f32(grow[c])) * ldexpf(1.f, scale_exponent(vmax[s * D + c]));
            Dt = Dv[sbase + t0 + r];
            L = lse[sbase + t0 + r];
            bound += fabsf(Dt);
        }
        const int e = max(scale_exponent(__float_as_uint(bound)), -60);   // keeps 2^(30-e) finite
        esc[r] = e;
        Dr[r] = Dt;
        pexp[r] = L * kLog2e - kDqBits + (float)e;
    }
    __syncthreads();

    // own 32-key groups, causal
    for (int p = wave; p < rows_here / 16; p += C::NW) {
        const int unit = p >> 1, st = p & 1;
        const int row = 32 * unit + 16 * st + m16;
        const int64_t kap = (t0 >> 5) + unit;
        Frag qb[C::KS], gb[C::KS];
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            qb[ks].q = *reinterpret_cast<const uint4*>(Qs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
            gb[ks].q = *reinterpret_cast<const uint4*>(Gs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
        }
        f32x4_t sc[2], dp[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            dp[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            if (mt <= st) {
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    Frag ka, va;
                    ka.q = *reinterpret_cast<const uint4*>(Kg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                    va.q = *reinterpret_cast<const uint4*>(Vg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                    sc[mt] = mfma16(ka, qb[ks], sc[mt]);
                    dp[mt] = mfma16(va, gb[ks], dp[mt]);
                }
            }
        }
        const float pe = pexp[row], Dt = Dr[row];
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool vis = 16 * (e >> 2) + 4 * g + (e & 3) <= 16 * st + m16;
            x[e] = vis ? fast_exp2(fmaf(sc[e >> 2][e & 3], c2, -pe)) * (dp[e >> 2][e & 3] - Dt) : 0.f;
        }
        Frag pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
            Frag kt;
            kt.q = *reinterpret_cast<const uint4*>(Ktg + slot_major_offset<D>(kap, mt, lane));
            f32x4_t o = mfma16(kt, pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int i = 0; i < 4; ++i)
                atomicAdd(&acc[row * C::OSTRIDE + tile_chan<D>(mt, 4 * g + i)], (int)o[i]);
        }
    }

    // routed groups (and, for B > 32, the earlier groups of the own block)
    const int gmax = (t0 + rows_here - 1) >> 5;
    for (int lo = 0; lo < gmax; lo += C::RANGE) {
        const int hi = min(gmax, lo + C::RANGE);
        __syncthreads();
        for (int i = tid; i < (hi - lo) * C::MW; i += C::NT) mask[i] = 0u;
        if (tid == 0) *next = 0;
        __syncthreads();
        for (int i = tid; i < rows_here * k; i += C::NT) {
            const int r = i / k, e = i - r * k;
            const int b = idx[(sbase + t0 + r) * k + e];
            if (b >= 0 && b < (t0 + r) / B) {
                for (int gi = 0; gi < NG; ++gi) {
                    const int kap = b * NG + gi - lo;
                    if (kap >= 0 && kap < hi - lo) atomicOr(&mask[kap * C::MW + (r >> 5)], 1u << (r & 31));
                }
            }
        }
        if (NG > 1) {
            for (int r = tid; r < rows_here; r += C::NT) {
                const int t = t0 + r;
                for (int kap = (t / B) * NG; kap < (t >> 5); ++kap)
                    if (kap >= lo && kap < hi) atomicOr(&mask[(kap - lo) * C::MW + (r >> 5)], 1u << (r & 31));
            }
        }
        __syncthreads();

        while (true) {
            int ui = 0;
            if (lane == 0) ui = atomicAdd(next, 1);
            ui = __builtin_amdgcn_readfirstlane(ui);
            if (ui >= hi - lo) break;
            uint32_t w[C::MW];
            int cnt = 0;
#pragma unroll
            for (int i = 0; i < C::MW; ++i) { w[i] = mask[ui * C::MW + i]; cnt += __popc(w[i]); }
            if (cnt == 0) continue;
            int base = 0;
#pragma unroll
            for (int r = 0; r < C::TILE / 64; ++r) {
                const uint64_t m64 = (uint64_t)w[2 * r] | ((uint64_t)w[2 * r + 1] << 32);
                if ((m64 >> lane) & 1ull) rl[base + __popcll(m64 & ((1ull << lane) - 1ull))] = (uint16_t)(64 * r + lane);
                base += __popcll(m64);
            }
            const int64_t kap = lo + ui;
            Frag ka[2][C::KS], va[2][C::KS], kt[C::MT];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    ka[mt][ks].q = *reinterpret_cast<const uint4*>(Kg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                    va[mt][ks].q = *reinterpret_cast<const uint4*>(Vg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                }
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
                kt[mt].q = *reinterpret_cast<const uint4*>(Ktg + slot_major_offset<D>(kap, mt, lane));
            __builtin_amdgcn_wave_barrier();

            for (int s0 = 0; s0 < cnt; s0 += 16) {
                const bool valid = s0 + m16 < cnt;
                const int row = rl[valid ? s0 + m16 : 0];
                Frag qb[C::KS], gb[C::KS];
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    qb[ks].q = *reinterpret_cast<const uint4*>(Qs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
                    gb[ks].q = *reinterpret_cast<const uint4*>(Gs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
                }
                f32x4_t sc[2], dp[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    dp[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) {
                        sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                        dp[mt] = mfma16(va[mt][ks], gb[ks], dp[mt]);
                    }
                }
                // rows beyond the list get an infinite exponent offset: their P is exactly 0
                const float pe = valid ? pexp[row] : INFINITY, Dt = Dr[row];
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[e] = fast_exp2(fmaf(sc[e >> 2][e & 3], c2, -pe)) * (dp[e >> 2][e & 3] - Dt);
                Frag pb;
#pragma unroll
                for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
                int oi[C::MT][4];
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    const f32x4_t o = mfma16(kt[mt], pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                    for (int i = 0; i < 4; ++i) oi[mt][i] = (int)o[i];   // toward zero; |o| ~ 2^12..2^20
                }
                if (valid) {
                    int* arow = acc + row * C::OSTRIDE + g * (D / 4);
#pragma unroll
                    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) atomicAdd(&arow[4 * mt + i], oi[mt][i]);
                }
            }
        }
    }
    __syncthreads();

    // dQ = scale * acc * 2^(e_t - 30) * 2^ek[c]
    bf16_t* dQg = dQ + (sbase + t0) * D;
    for (int i = tid; i < rows_here * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        const int et = esc[r] - 30;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = scale * ldexpf((float)acc[r * C::OSTRIDE + 8 * c + e], et + scale_exponent(kmax[s * D + 8 * c + e]));
        Vec8<bf16_t>::store(dQg + (int64_t)r * D + 8 * c, v);
    }
}

template <int D>
static hipError_t dq_launch(const Dims& s, const void* Q, const void* K, const void* V, const void* Kt,
                            const uint32_t* kmax, const uint32_t* vmax, const void* dO,
                            const float* lse, const float* Dv, const int32_t* idx, void* dQ,
                            hipStream_t st)
{
    using C = DqCfg<D>;
    const int ntiles = (s.N + C::TILE - 1) / C::TILE;
    hipError_t e = hipFuncSetAttribute((const void*)dq_mfma_kernel<D>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((dq_mfma_kernel<D>), dim3((unsigned)(ntiles * s.bh)), dim3(C::NT), C::LDS, st,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)Kt, kmax,
                       vmax, (const bf16_t*)dO, lse, Dv, idx, (bf16_t*)dQ, s.N, s.B, s.k, s.scale,
                       ntiles, s.bh);
    return hipGetLastError();
}

// Workspace of the MFMA backward: [D vector: bh*N fp32][slot-ordered scaled K: bh*N*D bf16]
// [kmax: bh*D words][vmax: bh*D words], each part 256-byte aligned.
static size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t backward_mfma_ws_bytes(const Dims& s)
{
    return a256(sizeof(float) * (size_t)s.bh * s.N) + a256(sizeof(bf16_t) * (size_t)s.bh * s.N * s.D) +
           2 * a256(sizeof(uint32_t) * (size_t)s.bh * s.D);
}

hipError_t launch_dq_mfma(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                          const float* lse, const int32_t* idx, const int32_t* off, const int32_t* ql,
                          const int32_t* chunk, void* dQ, void* ws, hipStream_t st)
{
    char* p = (char*)ws;
    const float* Dv = (const float*)p;
    p += a256(sizeof(float) * (size_t)s.bh * s.N);
    void* Kt = p;
    p += a256(sizeof(bf16_t) * (size_t)s.bh * s.N * s.D);
    uint32_t* kmax = (uint32_t*)p;
    p += a256(sizeof(uint32_t) * (size_t)s.bh * s.D);
    uint32_t* vmax = (uint32_t*)p;
    hipError_t e = launch_absmax(s, K, kmax, st);
    if (e != hipSuccess) return e;
    e = launch_absmax(s, V, vmax, st);
    if (e != hipSuccess) return e;
    e = launch_slot_major_copy(s, K, Kt, kmax, st);
    if (e != hipSuccess) return e;
    return s.D == 64 ? dq_launch<64>(s, Q, K, V, Kt, kmax, vmax, dO, lse, Dv, idx, dQ, st)
                     : dq_launch<128>(s, Q, K, V, Kt, kmax, vmax, dO, lse, Dv, idx, dQ, st);
}

}  // namespace moba
