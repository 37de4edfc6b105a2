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
//
// Structure, operand copies and workgroup schedule are the forward kernel's (see there): row
// lists per key block in LDS, K and V read in MFMA operand order, XCD-aware schedule.  The Q
// and dO tiles sit in LDS unpadded, with the 16-byte chunks of row r permuted by r & 7 so
// that a gather of arbitrary rows still spreads over the banks.
#include "mfma.h"

namespace moba {

#ifndef MOBA_DQ_NW64
#define MOBA_DQ_NW64 16
#endif

template <int D>
struct DqCfg {
    static constexpr int TILE = D == 64 ? 256 : 128;
    static constexpr int NW = D == 64 ? MOBA_DQ_NW64 : 8;
    static constexpr int NT = NW * kWave;
    static constexpr int ROWB = D * 2;                 // bytes per Q / dO row in LDS
    static constexpr int OSTRIDE = D + 1;              // words per accumulator row
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int RANGE = 1024;                 // key blocks per set of row lists (at most)
    static constexpr int LCAP = 16384;                 // (row, block) pairs per set of row lists
    static constexpr size_t LDS = (size_t)2 * TILE * ROWB + 4 * TILE * OSTRIDE + 4 * 3 * TILE +
                                  4 * 2 * (RANGE + 1) + 4 * NW + 8 + LCAP + 64;
};

constexpr float kDqBits = 30.f;
constexpr int kNanRow = 1 << 20;          // in place of a row's scale exponent: the row's dQ is NaN

template <int D>
__global__ __launch_bounds__(DqCfg<D>::NT) void dq_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Ka, const bf16_t* __restrict__ Va,
    const bf16_t* __restrict__ Kt, const uint32_t* __restrict__ kmax,
    const uint32_t* __restrict__ vmax, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
    const float* __restrict__ Dv, const int32_t* __restrict__ idx, bf16_t* __restrict__ dQ, int N,
    int B, int k, float scale, int ntiles, int bh, int G)
{
    using C = DqCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Qs = smem;
    unsigned char* Gs = Qs + (size_t)C::TILE * C::ROWB;
    int* acc = reinterpret_cast<int*>(Gs + (size_t)C::TILE * C::ROWB);
    float* pexp = reinterpret_cast<float*>(acc + C::TILE * C::OSTRIDE);   // lse*log2e - 30 + e_t
    float* Dr = pexp + C::TILE;                // -D_t
    int* esc = reinterpret_cast<int*>(Dr + C::TILE);
    uint32_t* cur = reinterpret_cast<uint32_t*>(esc + C::TILE);
    uint32_t* offs = cur + C::RANGE + 1;
    uint32_t* wsum = offs + C::RANGE + 1;
    int* next = reinterpret_cast<int*>(wsum + C::NW);
    int* take = next + 1;                                 // next unit of the list to hand to a wave
    uint8_t* rows8 = reinterpret_cast<uint8_t*>(take + 1);
    uint16_t* ulist = reinterpret_cast<uint16_t*>(cur);   // non-empty blocks of a range (over the builder's scratch)

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int m16 = lane & 15, g = lane >> 4;
    int s, pos;
    if (!schedule(blockIdx.x, bh, ntiles, s, pos)) return;
    const int tile = ntiles - 1 - pos;                 // late, long tiles first
    const int t0 = tile * C::TILE;
    const int rows_here = min(C::TILE, N - t0);
    const int NG = B / 32;
    const float c2 = scale * kLog2e;
    const int64_t sbase = (int64_t)s * N;
    const int skv = s / G;                             // G query heads share a key/value head
    const char* Kag = reinterpret_cast<const char*>(Ka + (int64_t)skv * N * D);
    const char* Vag = reinterpret_cast<const char*>(Va + (int64_t)skv * N * D);
    const char* Ktg = reinterpret_cast<const char*>(Kt + (int64_t)skv * N * D);
    const uint32_t vlane = (uint32_t)lane * 16u;       // this lane's bytes inside an operand

    // 0. Q and dO tiles -> LDS (chunk c of row r at chunk c ^ (r & 7)); clear the accumulators
    for (int i = tid; i < C::TILE * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        uint4 q = make_uint4(0, 0, 0, 0), gq = q;
        if (r < rows_here) {
            q = *reinterpret_cast<const uint4*>(Q + (sbase + t0 + r) * D + c * 8);
            gq = *reinterpret_cast<const uint4*>(dO + (sbase + t0 + r) * D + c * 8);
        }
        const uint32_t o = (uint32_t)r * C::ROWB + (uint32_t)((c ^ (r & 7)) << 4);
        *reinterpret_cast<uint4*>(Qs + o) = q;
        *reinterpret_cast<uint4*>(Gs + o) = gq;
    }
    for (int i = tid; i < C::TILE * C::OSTRIDE; i += C::NT) acc[i] = 0;
    __syncthreads();
    // per-row scale: 2^e_t >= sum_c |dO_tc| 2^ev_c + |D_t|.  NT / TILE neighbouring threads share a
    // row, a stretch of channels each, and add up by lane swaps of their neighbours.
    {
        constexpr int TPR = C::NT / C::TILE, CPT = D / TPR;       // threads per row, channels per thread
        static_assert(C::NT % C::TILE == 0 && (TPR == 4 || TPR == 8) && D % TPR == 0, "threads of a row are neighbours in a wave");
        const int r = tid / TPR, part = tid % TPR;
        float bound = 0.f, qsum = 0.f;
        bool finite = true;
        if (r < rows_here) {
            for (int c = part * CPT; c < (part + 1) * CPT; ++c) {
                const uint32_t o = (uint32_t)r * C::ROWB + ((((c >> 3) ^ (r & 7)) << 4) | ((c & 7) << 1));
                const bf16_t gv = *reinterpret_cast<const bf16_t*>(Gs + o);
                bound += fabsf(bf16_to_f32(gv)) * ldexpf(1.f, scale_exponent(vmax[skv * D + c]));
                qsum += fabsf(bf16_to_f32(*reinterpret_cast<const bf16_t*>(Qs + o)));
                finite = finite && !nonfinite_bits(kmax[skv * D + c]) && !nonfinite_bits(vmax[skv * D + c]);
            }
        }
#pragma unroll
        for (int o = 1; o < TPR; o <<= 1) {
            bound += __shfl_xor(bound, o, kWave);
            qsum += __shfl_xor(qsum, o, kWave);
            finite = __shfl_xor((int)finite, o, kWave) != 0 && finite;
        }
        if (part == 0) {
            float Dt = 0.f, L = 0.f;
            if (r < rows_here) {
                Dt = Dv[sbase + t0 + r];
                L = lse[sbase + t0 + r];
                bound += fabsf(Dt);
                // an infinity or a NaN in the row's dO, D, lse or Q, or anywhere in K or V: the integer
                // sums cannot carry it, the row's dQ is written as NaN
                finite = finite && fabsf(bound) < INFINITY && fabsf(L) < INFINITY && fabsf(qsum) < INFINITY;
            }
            const int e = finite ? max(scale_exponent(__float_as_uint(bound)), -60) : kNanRow;   // keeps 2^(30-e) finite
            esc[r] = e;
            Dr[r] = -Dt;                   // start value of the dP product: dP - D comes out of the MFMA
            pexp[r] = L * kLog2e - kDqBits + (float)e;
        }
    }
    __syncthreads();

    auto load_operand = [&](const char* base, int kap, Frag (&x)[2][C::KS]) {
        const char* b = base + (int64_t)kap * (64 * D);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
                x[mt][ks].q = *reinterpret_cast<const uint4*>(b + vlane + (mt * C::KS + ks) * 1024);
    };
    auto load_kt = [&](int kap, Frag (&kt)[C::MT]) {
        const char* b = Ktg + (int64_t)kap * (64 * D);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) kt[mt].q = *reinterpret_cast<const uint4*>(b + vlane + mt * 1024);
    };
    // this lane's chunks of Q and dO row `row`
    const uint32_t cg = (uint32_t)g << 4;
    auto gather = [&](int row, Frag (&qb)[C::KS], Frag (&gb)[C::KS]) {
        const uint32_t base = (uint32_t)row * C::ROWB, rx = ((uint32_t)row & 7u) << 4;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const uint32_t o = base + ((cg + 64u * ks) ^ rx);
            qb[ks].q = *reinterpret_cast<const uint4*>(Qs + o);
            gb[ks].q = *reinterpret_cast<const uint4*>(Gs + o);
        }
    };
    // x: dS^T (scaled) of this lane's row -> dQ accumulators
    auto accumulate = [&](int row, const float (&x)[8], const Frag (&kt)[C::MT], bool valid) {
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
            int* arow = acc + (uint32_t)row * C::OSTRIDE + g * (D / 4);
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) atomicAdd(&arow[4 * mt + i], oi[mt][i]);
        }
    };

    // own block: the row's own 32-key group under the causal mask and, for B > 32, the block's
    // earlier groups in full
    for (int p = wave; p < rows_here / 16; p += C::NW) {
        const int unit = p >> 1, st = p & 1;
        const int row = 32 * unit + 16 * st + m16;
        const int kown = (t0 >> 5) + unit;
        const int kfirst = NG == 1 ? kown : kown - kown % NG;
        Frag qb[C::KS], gb[C::KS];
        gather(row, qb, gb);
        const float pe = pexp[row], nD = Dr[row];
        for (int kap = kfirst; kap <= kown; ++kap) {
            const bool own = kap == kown;
            Frag ka[2][C::KS], va[2][C::KS], kt[C::MT];
            load_operand(Kag, kap, ka);
            load_operand(Vag, kap, va);
            load_kt(kap, kt);
            f32x4_t sc[2], dp[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                dp[mt] = f32x4_t{nD, nD, nD, nD};
                if (!own || mt <= st) {
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) {
                        sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                        dp[mt] = mfma16(va[mt][ks], gb[ks], dp[mt]);
                    }
                }
            }
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool vis = !own || 16 * (e >> 2) + 4 * g + (e & 3) <= 16 * st + m16;
                x[e] = vis ? fast_exp2(fmaf(sc[e >> 2][e & 3], c2, -pe)) * dp[e >> 2][e & 3] : 0.f;
            }
            accumulate(row, x, kt, true);
        }
    }

    // routed blocks
    const int pastmax = (t0 + rows_here - 1) / B;
    const int range = (int64_t)k * C::TILE <= C::LCAP ? C::RANGE : C::LCAP / C::TILE;
    for (int lo = 0; lo < pastmax; lo += range) {
        const int hi = min(pastmax, lo + range);
        __syncthreads();
        build_block_lists<C::TILE, C::NT>(idx + (sbase + t0) * k, t0, rows_here, k, B, lo, hi, cur, offs,
                                          rows8, C::LCAP, wsum, tid);
        if (tid == 0) *take = 0;
        list_nonempty<C::NT>(offs, hi - lo, ulist, next, wsum, tid);
        const int nblk = *next;

        // waves take the listed blocks as they get free; one unit = one 32-key group of a block
        int e = take_unit(take, lane);
        while (e < nblk) {
            const int en = take_unit(take, lane);     // asked for early: its latency hides behind this unit
            const int j = __builtin_amdgcn_readfirstlane((int)ulist[e]);
            const int beg = __builtin_amdgcn_readfirstlane((int)offs[j]);
            const int end = min(__builtin_amdgcn_readfirstlane((int)offs[j + 1]), (int)C::LCAP);
            for (int gi = 0; gi < NG; ++gi) {
                const int kap = (lo + j) * NG + gi;
                Frag ka[2][C::KS], va[2][C::KS], kt[C::MT];
                load_operand(Kag, kap, ka);
                load_operand(Vag, kap, va);
                load_kt(kap, kt);
                // sub-tiles of 16 listed rows; lanes beyond the list work on whatever row id
                // they read (always inside the tile) and add nothing
                for (int c0 = beg; c0 < end; c0 += 16) {
                    const bool valid = m16 < end - c0;
                    const int row = rows8[c0 + m16] & (C::TILE - 1);
                    Frag qb[C::KS], gb[C::KS];
                    gather(row, qb, gb);
                    const float pe = pexp[row], nD = Dr[row];
                    f32x4_t sc[2], dp[2];
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        dp[mt] = f32x4_t{nD, nD, nD, nD};
#pragma unroll
                        for (int ks = 0; ks < C::KS; ++ks) {
                            sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                            dp[mt] = mfma16(va[mt][ks], gb[ks], dp[mt]);
                        }
                    }
                    float x[8];
#pragma unroll
                    for (int e2 = 0; e2 < 8; ++e2)
                        x[e2] = fast_exp2(fmaf(sc[e2 >> 2][e2 & 3], c2, -pe)) * dp[e2 >> 2][e2 & 3];
                    accumulate(row, x, kt, valid);
                }
            }
            e = en;
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
            v[e] = esc[r] == kNanRow ? NAN
                 : scale * ldexpf((float)acc[r * C::OSTRIDE + 8 * c + e], et + scale_exponent(kmax[skv * D + 8 * c + e]));
        Vec8<bf16_t>::store(dQg + (int64_t)r * D + 8 * c, v);
    }
}

template <int D>
static hipError_t dq_launch(const Dims& s, const void* Q, const void* Ka, const void* Va, const void* Kt,
                            const uint32_t* kmax, const uint32_t* vmax, const void* dO,
                            const float* lse, const float* Dv, const int32_t* idx, void* dQ,
                            hipStream_t st)
{
    using C = DqCfg<D>;
    const int ntiles = (s.N + C::TILE - 1) / C::TILE;
    hipError_t e = ensure_dynamic_lds((const void*)dq_mfma_kernel<D>, (size_t)(C::LDS));
    if (e != hipSuccess) return e;
    ProfileScope timing(MOBA_PROFILE_DQ, st);
    hipLaunchKernelGGL((dq_mfma_kernel<D>), dim3((unsigned)schedule_grid(s.bh, ntiles)), dim3(C::NT), C::LDS, st,
                       (const bf16_t*)Q, (const bf16_t*)Ka, (const bf16_t*)Va, (const bf16_t*)Kt, kmax,
                       vmax, (const bf16_t*)dO, lse, Dv, idx, (bf16_t*)dQ, s.N, s.B, s.k, s.scale,
                       ntiles, s.bh, s.G);
    return hipGetLastError();
}

// Workspace of the MFMA backward: [D vector: bh*N fp32][prepared copies: maxima of K and V,
// operand-ordered K, slot-ordered scaled K, operand-ordered V], each part 256-byte aligned.  When
// the workspace is shared with the forward (MOBA_FLAG_SHARED_WORKSPACE) the forward's slot-ordered
// V lies among the copies too, and the forward call has made all of them.

size_t backward_mfma_ws_bytes(const Dims& s)
{
    return a256(sizeof(float) * (size_t)s.bh * s.N) +
           prepared_layout(s, shared_workspace(s) ? kPrepAll : kPrepBackward, nullptr, nullptr);
}

hipError_t launch_dq_mfma(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                          const float* lse, const int32_t* idx, const int32_t* off, const int32_t* ql,
                          void* dQ, void* ws, hipStream_t st)
{
    const float* Dv = (const float*)ws;
    Prepared p;
    prepared_layout(s, shared_workspace(s) ? kPrepAll : kPrepBackward,
                    (char*)ws + a256(sizeof(float) * (size_t)s.bh * s.N), &p);
    if (!shared_workspace(s)) {
        hipError_t e = launch_prepare(kv_view(s), K, V, p, st);
        if (e != hipSuccess) return e;
    }
    return s.D == 64 ? dq_launch<64>(s, Q, p.Ka, p.Va, p.Kt, p.kmax, p.vmax, dO, lse, Dv, idx, dQ, st)
                     : dq_launch<128>(s, Q, p.Ka, p.Va, p.Kt, p.kmax, p.vmax, dO, lse, Dv, idx, dQ, st);
}

}  // namespace moba
