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
//   gather                               the 32 rows of Q and dO come in with 8 (d = 64) lanes
//                                        per row, whole 128-byte lines per load instruction
//                                        (the rate of a lane-per-row gather is a quarter of
//                                        that on this chip), and are parked in LDS;
//   S  = Q_g K^T, dP = dO_g V^T          A operands read back from LDS row by row, K and V rows
//                                        of the group as B operands (registers, loaded once);
//   P, dS                                in the result layout: a lane holds one key column
//                                        and query rows 4g..4g+3 of both 16-query tiles,
//                                        which packed to bf16 is already a B operand over
//                                        the 32 queries (slot order of mfma.h);
//   dV^T += dO_g^T P, dK^T += Q_g^T dS   the A operands are the parked rows transposed, which
//                                        the LDS transpose read of gfx950 (ds_read_b64_tr_b16)
//                                        delivers four query slots per lane at a time.
#include <type_traits>

#include "mfma.h"

namespace moba {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int D>
struct DkvCfg {
    static constexpr int NW = 4;
    static constexpr int NT = NW * kWave;
    static constexpr int SB = D * 2 + 16;              // bytes per parked row
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row
    static constexpr int RPI = kWave / CPR;            // rows per gather instruction
    static constexpr int NI = 32 / RPI;                // gather instructions per tensor and step
    static constexpr int RSTRIDE = D + 4;              // floats per key row of the reduction buffer
    static constexpr size_t STAGE = (size_t)2 * 32 * SB;                   // Q and dO, bytes per wave
    static constexpr size_t LDS = NW * (STAGE + 2 * 32 * 4) + (size_t)2 * 32 * RSTRIDE * 4;
    // wide variant: two sets of four slots (the waves park one slot each, all read all four); at
    // the end every wave turns its accumulators over in 2 * 32 * RSTRIDE floats of its own
    static constexpr size_t WIDE_PARK = (size_t)2 * NW * (STAGE + 2 * 32 * 4);
    static constexpr size_t WIDE_OUT = (size_t)NW * 2 * 32 * RSTRIDE * 4;
    static constexpr size_t LDS_WIDE = WIDE_PARK > WIDE_OUT ? WIDE_PARK : WIDE_OUT;
};

// LDS transpose read: within each group of 16 lanes, lane i receives as element e the 16-bit
// element (i & 3) of the 8 bytes that lane 4 e + (i >> 2) of the group points at.
__device__ __forceinline__ uint2 lds_read_tr16(const unsigned char* p)
{
    typedef short v4s __attribute__((ext_vector_type(4)));
    const v4s r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) v4s*)(const_cast<unsigned char*>(p)));
    return *reinterpret_cast<const uint2*>(&r);
}

// GPW > 1 (key blocks of whole 64- or 128-key parts): a workgroup owns GPW = 2 or 4 consecutive
// 32-key groups of one block, wave w the group w mod GPW; a step covers 128 positions of the walk
// -- every wave gathers and parks 32 of them, and after a barrier every wave works through GPW of
// the four slots with its own keys (GPW = 4: all of them; GPW = 2: waves 0, 1 the first two,
// waves 2, 3 the others).  The block's list is then gathered once per 32 GPW keys instead of once
// per 32, and with GPW = 4 nothing has to be summed over the waves (GPW = 2: over two).
template <int D, int GPW>
__global__ __launch_bounds__(DkvCfg<D>::NT) __attribute__((amdgpu_waves_per_eu(D == 64 ? 2 : 1)))
void dkdv_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float2* __restrict__ ld,
    const int32_t* __restrict__ off, const int32_t* __restrict__ ql, bf16_t* __restrict__ dK,
    bf16_t* __restrict__ dV, int N, int B, int n, float scale, int64_t R, int groups_per_slice, int bhk,
    int G, float* __restrict__ part, int order)
{
    using C = DkvCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr bool WIDE = GPW > 1;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    constexpr size_t SLOT = C::STAGE + 256;                 // parked Q rows, dO rows, lse, -D of 32 positions
    float* red = reinterpret_cast<float*>(WIDE ? smem + (size_t)wave * 2 * 32 * C::RSTRIDE * 4
                                               : smem + C::NW * SLOT);        // [2][32][RSTRIDE]

    // part == nullptr: a workgroup per key/value slice and unit, the G query heads that share the
    // slice one after the other.  Otherwise (G > 1) a workgroup per QUERY head and unit, which
    // leaves its sums as fp32 in part[dK | dV][query slice][N][D] for dkdv_heads_kernel to add up:
    // the workgroups of an XCD then gather from one head's Q and dO at a time, as without sharing
    // (walking all G heads in every workgroup, the L2 hit rate of the gathers fell from 80 % to
    // 15 % with 16 heads on one key/value head).
    const int slices = part ? bhk * G : bhk;
    int slice, unit;                                        // slice; 32-key group or part of GPW groups
    if (!schedule(blockIdx.x, order * slices, groups_per_slice, slice, unit)) return;   // order -1: slice after slice
    const int skv = part ? slice / G : slice;               // key/value slice
    const int s_first = part ? slice : skv * G, s_last = part ? slice + 1 : (skv + 1) * G;
    const int kap = WIDE ? GPW * unit + wave % GPW : unit;  // this wave's 32-key group inside the slice
    const int NG = B / 32;
    const int j = kap / NG;
    const int64_t kvbase = (int64_t)skv * N;
    const float c2 = scale * kLog2e;
    const int own0 = WIDE ? 32 * GPW * unit : 32 * kap;     // first own query that sees the workgroup's keys
    const int kfirst = WIDE ? 32 * (wave % GPW) : 0;        // this wave's first key, counted from there
    int parity = 0;                                         // WIDE: which set of slots the next step parks in

    // B operands: the group's keys and values (lane = key m16 of tile nt)
    Frag kb[2][C::KS], vb[2][C::KS];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const int64_t o = (kvbase + 32 * kap + 16 * nt + m16) * D + 8 * g + 32 * ks;
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

    // The G query heads that share this key/value head (grouped-query attention, Appendix C, last
    // paragraph), one after the other: each has its own list for the block; dK and dV add up in
    // the same accumulators.
    for (int s = s_first; s < s_last; ++s) {
    const int64_t sbase = (int64_t)s * N;
    const int32_t* os = off + (int64_t)s * (n + 1);
    const int32_t* qs = ql + (int64_t)s * R;
    const int lo = os[j], nlist = os[j + 1] - lo;
    const int total = nlist + (j + 1) * B - own0;
    const char* Qg = reinterpret_cast<const char*>(Q + sbase * D);
    const char* Gg = reinterpret_cast<const char*>(dO + sbase * D);

    // position a of the walk -> query: the block's list, then its own queries from this group on;
    // positions past the end read as the first own query (a valid row; its P is forced to 0).
    // Every load below is unconditional (from an address that is always valid): a load inside a
    // branch would be waited for at the end of the branch, and with it all the row gathers
    // issued before it.
    const int32_t* lsrc = nlist > 0 ? qs + lo : os;          // an empty list reads os[0] and ignores it
    const int llast = max(nlist - 1, 0);
    auto query_at = [&](int a) {
        const int listed = list_query(lsrc[min(a, llast)]);
        const int t = a < nlist ? listed : own0 + (a - nlist);
        return a >= total ? own0 : t;
    };
    // The gathers are the long pole (two dependent global loads: list entry, then the row), so
    // they run ahead of the arithmetic: row ids two steps ahead, rows one step ahead.
    const int grow = lane / C::CPR;                          // row of this lane inside a gather instruction
    const uint32_t gcol = (uint32_t)(lane % C::CPR) * 16u;   // its bytes inside the row
    // `inside` (a compile-time flag): all 32 positions lie in the block's list -- the bulk of the
    // walk, which then needs no selects
    auto ids = [&](int a0, int (&t)[C::NI], int& tl, auto inside) {
        if constexpr (decltype(inside)::value) {
#pragma unroll
            for (int i = 0; i < C::NI; ++i) t[i] = list_query(lsrc[a0 + C::RPI * i + grow]);
            tl = list_query(lsrc[a0 + (lane & 31)]);
        } else {
#pragma unroll
            for (int i = 0; i < C::NI; ++i) t[i] = query_at(a0 + C::RPI * i + grow);
            tl = query_at(a0 + (lane & 31));
        }
    };
    // lv: lse in log2 units (+inf past the end: P = 0); dv: -D, the start value of the dP product
    auto fetch = [&](int a0, const int (&t)[C::NI], int tl, u32x4_t (&qr)[C::NI], u32x4_t (&gr)[C::NI],
                     float& lv, float& dv, auto inside) {
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            const uint32_t o = (uint32_t)t[i] * (uint32_t)(2 * D) + gcol;
            qr[i] = *reinterpret_cast<const u32x4_t*>(Qg + o);
            gr[i] = *reinterpret_cast<const u32x4_t*>(Gg + o);
        }
        const bool live = decltype(inside)::value || a0 + (lane & 31) < total;
        const float2 x = ld[sbase + tl];                  // (lse log2 e, -D) of the row
        lv = live ? x.x : INFINITY;
        dv = live ? x.y : 0.f;
    };
    const int stride = 32 * C::NW;
    int tN[C::NI], tlN;
    u32x4_t qr[C::NI], gr[C::NI];    // plain vectors: a struct type would be copied through scratch
    float lv, dv;
    {
        int t0[C::NI], tl0;
        ids(32 * wave, t0, tl0, std::false_type());
        fetch(32 * wave, t0, tl0, qr, gr, lv, dv, std::false_type());
        ids(32 * wave + stride, tN, tlN, std::false_type());
    }
    const uint32_t park = (uint32_t)grow * C::SB + gcol;                       // gather lane -> parked bytes
    const uint32_t arow = (uint32_t)m16 * C::SB + 16u * g;                     // row-major operand of this lane
    // transpose read: lanes 4 e + a of a 16-lane group point at query slot e (+4), channels 4 a ..
    const int te = (lane >> 2) & 3, ta = lane & 3;
    const uint32_t tr0 = (uint32_t)slot_key(g, te) * C::SB + 8u * ta;
    const uint32_t tr1 = (uint32_t)slot_key(g, te + 4) * C::SB + 8u * ta;
    // the arithmetic of 32 parked positions (walk positions p0 .. p0 + 31) against this wave's keys
    auto work = [&](unsigned char* stQ, int p0, auto inside) {
        unsigned char* stG = stQ + 32 * C::SB;
        const float* ls = reinterpret_cast<const float*>(stQ + C::STAGE);
        const float* Ds = ls + 32;
        // S and dP
        f32x4_t sc[2][2], dp[2][2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            Frag qa[C::KS], ga[C::KS];
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                qa[ks].q = *reinterpret_cast<const uint4*>(stQ + arow + qt * 16 * C::SB + 64 * ks);
                ga[ks].q = *reinterpret_cast<const uint4*>(stG + arow + qt * 16 * C::SB + 64 * ks);
            }
            const f32x4_t nd = *reinterpret_cast<const f32x4_t*>(Ds + 16 * qt + 4 * g);   // -D of the rows
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                sc[qt][nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                dp[qt][nt] = nd;                              // dP - D comes out of the MFMA
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks) {
                    sc[qt][nt] = mfma16(qa[ks], kb[nt][ks], sc[qt][nt]);
                    dp[qt][nt] = mfma16(ga[ks], vb[nt][ks], dp[qt][nt]);
                }
            }
        }
        // own queries are causal: the wave's key kfirst + 16 nt + m16 (counted from the first own
        // query's key) must not exceed the query
        const bool causal = !decltype(inside)::value && p0 + 32 > nlist && p0 < nlist + kfirst + 32;
        Frag pb[2], sb[2];
        f32x4_t l4[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) l4[qt] = *reinterpret_cast<const f32x4_t*>(ls + 16 * qt + 4 * g);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            float p[8], d[8];
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float pv = fast_exp2(fmaf(sc[qt][nt][i], c2, -l4[qt][i]));
                    if (causal) {
                        const int a = p0 + 16 * qt + 4 * g + i - nlist;     // own row index, if >= 0
                        if (a >= 0 && kfirst + 16 * nt + m16 > a) pv = 0.f;
                    }
                    p[4 * qt + i] = pv;
                    d[4 * qt + i] = pv * dp[qt][nt][i];
                }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pb[nt].u[e] = pack2(p[2 * e], p[2 * e + 1]);
                sb[nt].u[e] = pack2(d[2 * e], d[2 * e + 1]);
            }
        }
        // transposed A operands from the parked rows, then the two accumulating products
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
            Frag qT, gT;
            const uint2 q0 = lds_read_tr16(stQ + tr0 + 32 * mt), q1 = lds_read_tr16(stQ + tr1 + 32 * mt);
            const uint2 g0 = lds_read_tr16(stG + tr0 + 32 * mt), g1 = lds_read_tr16(stG + tr1 + 32 * mt);
            qT.u[0] = q0.x; qT.u[1] = q0.y; qT.u[2] = q1.x; qT.u[3] = q1.y;
            gT.u[0] = g0.x; gT.u[1] = g0.y; gT.u[2] = g1.x; gT.u[3] = g1.y;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                dVT[mt][nt] = mfma16(gT, pb[nt], dVT[mt][nt]);
                dKT[mt][nt] = mfma16(qT, sb[nt], dKT[mt][nt]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    // one step of this wave at walk position a0: park the 32 rows, put the next step's loads in
    // flight, then the arithmetic -- on the wave's own slot, or (WIDE) on the four slots of the
    // workgroup's 128 positions
    auto step = [&](int a0, auto inside) {
        unsigned char* mine = smem + (WIDE ? (size_t)(4 * parity + wave) * SLOT : (size_t)wave * SLOT);
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            *reinterpret_cast<u32x4_t*>(mine + park + i * C::RPI * C::SB) = qr[i];
            *reinterpret_cast<u32x4_t*>(mine + 32 * C::SB + park + i * C::RPI * C::SB) = gr[i];
        }
        if (lane < 32) {
            float* ls = reinterpret_cast<float*>(mine + C::STAGE);
            ls[lane] = lv;
            ls[32 + lane] = dv;
        }
        fetch(a0 + stride, tN, tlN, qr, gr, lv, dv, inside);
        ids(a0 + 2 * stride, tN, tlN, inside);
        if constexpr (WIDE) {
            // one barrier per step is enough: a slot set is parked again two steps later, and no
            // wave gets there before all have passed the barrier of the step in between
            __syncthreads();
            const int sl0 = wave / GPW * GPW;               // the GPW slots that waves with other keys do not share out among them
#pragma unroll 1
            for (int sl = sl0; sl < sl0 + GPW; ++sl) work(smem + (size_t)(4 * parity + sl) * SLOT, a0 - 32 * wave + 32 * sl, inside);
            parity ^= 1;
        } else {
            __builtin_amdgcn_wave_barrier();
            work(mine, a0, inside);
        }
    };
    // the bulk of the walk: this step, the rows fetched in it and the ids looked up in it all lie
    // inside the block's list; then the general steps (own rows, causal mask, end of the walk).
    // (WIDE: the same number of steps in every wave -- they meet at a barrier in each.)
    int a0 = 32 * wave;
    if constexpr (WIDE) {
        for (; a0 - 32 * wave + 3 * stride <= nlist; a0 += stride) step(a0, std::true_type());
        for (; a0 - 32 * wave < total; a0 += stride) step(a0, std::false_type());
    } else {
        for (; a0 + 2 * stride + 32 <= nlist; a0 += stride) step(a0, std::true_type());
        for (; a0 < total; a0 += stride) step(a0, std::false_type());
    }
    }

    if constexpr (WIDE) {
        __syncthreads();                                    // the slots are no longer read
        if constexpr (GPW < C::NW) {
            // waves w, w + GPW, ... hold parts of the sums of the same keys: the later ones leave
            // theirs in LDS, the first GPW waves add them up
            if (wave >= GPW) {
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        float* pk = red + (16 * nt + m16) * C::RSTRIDE + 16 * mt + 4 * g;
                        *reinterpret_cast<f32x4_t*>(pk) = dKT[mt][nt];
                        *reinterpret_cast<f32x4_t*>(pk + 32 * C::RSTRIDE) = dVT[mt][nt];
                    }
            }
            __syncthreads();
            if (wave >= GPW) return;                        // (no workgroup barrier follows)
            for (int w2 = wave + GPW; w2 < C::NW; w2 += GPW) {
                const float* other = reinterpret_cast<const float*>(smem + (size_t)w2 * 2 * 32 * C::RSTRIDE * 4);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt) {
                        const float* pk = other + (16 * nt + m16) * C::RSTRIDE + 16 * mt + 4 * g;
                        dKT[mt][nt] += *reinterpret_cast<const f32x4_t*>(pk);
                        dVT[mt][nt] += *reinterpret_cast<const f32x4_t*>(pk + 32 * C::RSTRIDE);
                    }
            }
        }
        // every wave (of the first GPW) has the whole sums of its own 32 keys: turn them over in
        // LDS (channels of a key side by side) and write them out
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                float* pk = red + (16 * nt + m16) * C::RSTRIDE + 16 * mt + 4 * g;
                *reinterpret_cast<f32x4_t*>(pk) = dKT[mt][nt];
                *reinterpret_cast<f32x4_t*>(pk + 32 * C::RSTRIDE) = dVT[mt][nt];
            }
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < 2 * 32 * (D / 8); i += kWave) {
            const int which = i / (32 * (D / 8)), rem = i % (32 * (D / 8));
            const int key = rem / (D / 8), c = rem % (D / 8);
            const float* src = red + which * 32 * C::RSTRIDE + key * C::RSTRIDE + 8 * c;
            const float mul = which == 0 ? scale : 1.f;
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = src[e] * mul;
            if (part) {
                Vec8<float>::store(part + (((int64_t)which * slices + slice) * N + 32 * kap + key) * D + 8 * c, v);
            } else {
                bf16_t* dst = (which == 0 ? dK : dV) + (kvbase + 32 * kap + key) * D + 8 * c;
                Vec8<bf16_t>::store(dst, v);
            }
        }
        return;
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
        if (part) {
            Vec8<float>::store(part + (((int64_t)which * slices + slice) * N + 32 * kap + key) * D + 8 * c, v);
        } else {
            bf16_t* dst = (which == 0 ? dK : dV) + (kvbase + 32 * kap + key) * D + 8 * c;
            Vec8<bf16_t>::store(dst, v);
        }
    }
}

// dK, dV of a key/value head = the sums over the G query heads that share it, added in head order
// (fixed: bit-reproducible); eight channels per thread
__global__ __launch_bounds__(256) void dkdv_heads_kernel(const float* __restrict__ part,
                                                         bf16_t* __restrict__ dK, bf16_t* __restrict__ dV,
                                                         int64_t chunks_per_slice, int bhk, int G)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;     // (tensor, key/value slice, 8-channel chunk)
    const int64_t per_tensor = chunks_per_slice * bhk;
    if (i >= 2 * per_tensor) return;
    const int which = (int)(i / per_tensor);
    const int64_t r = i % per_tensor, skv = r / chunks_per_slice, ch = r % chunks_per_slice;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int gq = 0; gq < G; ++gq) {
        float v[8];
        Vec8<float>::load(part + ((((int64_t)which * bhk + skv) * G + gq) * chunks_per_slice + ch) * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
    Vec8<bf16_t>::store((which == 0 ? dK : dV) + (skv * chunks_per_slice + ch) * 8, acc);
}

template <int D>
static hipError_t dkdv_launch(const Dims& s, const void* Q, const void* K, const void* V,
                              const void* dO, const float2* ld, const int32_t* off,
                              const int32_t* ql, void* dK, void* dV, float* part, hipStream_t st)
{
    using C = DkvCfg<D>;
    const int gps = s.N / 32;
    if (gps == 0) return hipSuccess;
    // 32-key groups of one block per workgroup: four, two or one
    const int gpw = s.B % 128 == 0 ? 4 : s.B % 64 == 0 ? 2 : 1;
    const size_t lds = gpw > 1 ? C::LDS_WIDE : C::LDS;
    const int units = gps / gpw;
    hipError_t e = gpw == 4   ? ensure_dynamic_lds((const void*)dkdv_mfma_kernel<D, 4>, (size_t)lds)
                   : gpw == 2 ? ensure_dynamic_lds((const void*)dkdv_mfma_kernel<D, 2>, (size_t)lds)
                              : ensure_dynamic_lds((const void*)dkdv_mfma_kernel<D, 1>, (size_t)lds);
    if (e != hipSuccess) return e;
    const int slices = part ? s.bh : s.bhk;
    const int order = slices > 1 ? slice_major(s, 2) : 1;       // (gathers Q and dO rows)
    ProfileScope timing(MOBA_PROFILE_DKDV, st);
    const dim3 grid((unsigned)schedule_grid(order * slices, units));
#define MOBA_DKDV_LAUNCH(GPW)                                                                                  \
    hipLaunchKernelGGL((dkdv_mfma_kernel<D, GPW>), grid, dim3(C::NT), lds, st, (const bf16_t*)Q,              \
                       (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, ld, off, ql, (bf16_t*)dK,       \
                       (bf16_t*)dV, s.N, s.B, s.n, s.scale, s.R, units, s.bhk, s.G, part, order)
    if (gpw == 4) MOBA_DKDV_LAUNCH(4);
    else if (gpw == 2) MOBA_DKDV_LAUNCH(2);
    else MOBA_DKDV_LAUNCH(1);
#undef MOBA_DKDV_LAUNCH
    if (part) {
        const int64_t cps = (int64_t)s.N * D / 8, total = 2 * cps * s.bhk;
        hipLaunchKernelGGL(dkdv_heads_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, part,
                           (bf16_t*)dK, (bf16_t*)dV, cps, s.bhk, s.G);
    }
    return hipGetLastError();
}

size_t dkdv_heads_ws_bytes(const Dims& s)
{
    return s.G > 1 ? a256(2 * sizeof(float) * (size_t)s.bh * s.N * s.D) : 0;
}

hipError_t launch_dkdv_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                            const void* dO, const float2* ld, const int32_t* off,
                            const int32_t* ql, void* dK, void* dV, float* part, hipStream_t st)
{
    if (s.G == 1) part = nullptr;
    return s.D == 64 ? dkdv_launch<64>(s, Q, K, V, dO, ld, off, ql, dK, dV, part, st)
                     : dkdv_launch<128>(s, Q, K, V, dO, ld, off, ql, dK, dV, part, st);
}

}  // namespace moba
