// MoBA forward on bf16 MFMA (paper Section 4.2, forward pass with gather-and-densify),
// re-cut for CDNA4: a workgroup owns a tile of consecutive queries and keeps their Q rows
// (bf16) and their output accumulators in LDS for the whole kernel -- the running output
// of the paper's forward algorithm never goes to HBM.  It walks the 32-key groups its
// queries were routed to; for each group one wave gathers the routed rows out of LDS
// sixteen at a time as a dense MFMA operand, computes S^T = K Q^T, turns it into
// probabilities and adds P V into the rows' accumulators.
//
// Several waves add to the same row concurrently, so the adds must be atomic.  On this
// chip LDS float atomics run ~30x slower than LDS integer atomics, so the accumulators are
// 32-bit fixed point:
//   pass 1  every routed (row, group) pair: S^T only, row maximum by integer atomic max on
//           order-preserving keys -> the exact softmax reference m of each row;
//   pass 2  the same walk again: p = exp(s - m) <= 1, so sum_u p_u <= (number of keys of the
//           row) and, with V pre-scaled per channel to |v| <= 1, |sum_u p_u v_u| has the same
//           bound; both sums are accumulated as integers scaled by 2^F, F chosen from that
//           bound (each 32-key partial of P V is cut toward zero, a relative shrink of ~1e-5,
//           two orders below the bf16 output's resolution; the row sums l round to nearest).  Integer adds commute exactly: the result does not depend on the order
//           in which waves arrive, so the output is bit-reproducible.
// Which rows go with which key group is a bit matrix in LDS (one row of TILE bits per
// group), built from the query-major routing, 1024 groups at a time.
#include "mfma.h"

namespace moba {

template <int D>
struct FwdCfg {
    static constexpr int TILE = D == 64 ? 256 : 128;   // queries per workgroup
    static constexpr int NW = 8;                       // waves per workgroup
    static constexpr int NT = NW * kWave;
    static constexpr int QSTRIDE = D * 2 + 16;         // bytes per Q row in LDS
    static constexpr int OSTRIDE = D + 1;              // words per accumulator row
    static constexpr int MT = D / 16;                  // 16-channel tiles of a row
    static constexpr int KS = D / 32;                  // contraction steps of q.k
    static constexpr int MW = TILE / 32;               // mask words per key group
    static constexpr int RANGE = 1024;                 // key groups per bit matrix
    static constexpr size_t LDS = (size_t)TILE * QSTRIDE + 4 * TILE * OSTRIDE + 4 * 2 * TILE +
                                  4 * RANGE * MW + 2 * NW * TILE + 4 * RANGE + 64;
};

// ---- per-channel scale of V and the slot-ordered transposed copy (see mfma.h) -----------

__global__ void zero_words_kernel(uint32_t* p, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// vmax[s][c] = max_t |X[s][t][c]| as raw fp32 bits (non-negative floats order like integers)
template <int D>
__global__ __launch_bounds__(256) void absmax_kernel(const bf16_t* __restrict__ X,
                                                     uint32_t* __restrict__ vmax, int N,
                                                     int rows_per_wg)
{
    __shared__ float red[256 / (D / 8)][D];
    constexpr int G = D / 8;
    const int s = blockIdx.y, part = threadIdx.x % G, rr = threadIdx.x / G;
    const int r0 = blockIdx.x * rows_per_wg, r1 = min(N, r0 + rows_per_wg);
    float mx[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r = r0 + rr; r < r1; r += 256 / G) {
        float v[8];
        Vec8<bf16_t>::load(X + ((int64_t)s * N + r) * D + part * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) mx[e] = fmaxf(mx[e], fabsf(v[e]));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rr][part * 8 + e] = mx[e];
    __syncthreads();
    if (threadIdx.x < D) {
        float m = 0.f;
        for (int i = 0; i < 256 / G; ++i) m = fmaxf(m, red[i][threadIdx.x]);
        atomicMax(&vmax[s * D + threadIdx.x], __float_as_uint(m));
    }
}

template <int D>
__global__ __launch_bounds__(256) void slot_major_copy_kernel(const bf16_t* __restrict__ X,
                                                              const uint32_t* __restrict__ vmax,
                                                              bf16_t* __restrict__ Xt,
                                                              int64_t groups_per_slice)
{
    __shared__ bf16_t tile[32 * (D + 8)];
    const int64_t kap = blockIdx.x;            // group index over all slices
    const int s = (int)(kap / groups_per_slice);
    const bf16_t* src = X + kap * 32 * D;
    for (int i = threadIdx.x; i < 32 * D / 8; i += 256) {
        const int r = i / (D / 8), c = i % (D / 8);
        float v[8];
        Vec8<bf16_t>::load(src + r * D + c * 8, v);
        if (vmax) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = ldexpf(v[e], -scale_exponent(vmax[s * D + c * 8 + e]));
        }
        Vec8<bf16_t>::store(&tile[r * (D + 8) + c * 8], v);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < (D / 16) * 64; i += 256) {
        const int mt = i / 64, lane = i % 64, g = lane >> 4, m = lane & 15;
        const int ch = tile_chan<D>(mt, m);
        uint32_t w[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t lo = tile[slot_key(g, 2 * p) * (D + 8) + ch];
            const uint32_t hi = tile[slot_key(g, 2 * p + 1) * (D + 8) + ch];
            w[p] = lo | (hi << 16);
        }
        *reinterpret_cast<uint4*>(Xt + slot_major_offset<D>(kap, mt, lane)) =
            make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// vmax[bh][D] <- largest magnitude of each channel of X, as fp32 bits
hipError_t launch_absmax(const Dims& s, const void* X, uint32_t* vmax, hipStream_t st)
{
    if (s.N == 0) return hipSuccess;
    const int cnt = s.bh * s.D, rows_per_wg = 1024;
    hipLaunchKernelGGL(zero_words_kernel, dim3((cnt + 255) / 256), dim3(256), 0, st, vmax, cnt);
    dim3 grid((s.N + rows_per_wg - 1) / rows_per_wg, s.bh);
    if (s.D == 64)
        hipLaunchKernelGGL(absmax_kernel<64>, grid, dim3(256), 0, st, (const bf16_t*)X, vmax, s.N,
                           rows_per_wg);
    else
        hipLaunchKernelGGL(absmax_kernel<128>, grid, dim3(256), 0, st, (const bf16_t*)X, vmax, s.N,
                           rows_per_wg);
    return hipGetLastError();
}

// Xt <- slot-ordered transposed copy of X, each channel scaled by 2^-e (e from its largest
// magnitude vmax[bh][D], fp32 bits); vmax == nullptr: plain copy.
hipError_t launch_slot_major_copy(const Dims& s, const void* X, void* Xt, const uint32_t* vmax,
                                  hipStream_t st)
{
    const int64_t gps = s.N / 32, groups = (int64_t)s.bh * gps;
    if (groups == 0) return hipSuccess;
    if (s.D == 64)
        hipLaunchKernelGGL(slot_major_copy_kernel<64>, dim3((unsigned)groups), dim3(256), 0, st,
                           (const bf16_t*)X, vmax, (bf16_t*)Xt, gps);
    else
        hipLaunchKernelGGL(slot_major_copy_kernel<128>, dim3((unsigned)groups), dim3(256), 0, st,
                           (const bf16_t*)X, vmax, (bf16_t*)Xt, gps);
    return hipGetLastError();
}

// ---- the tile kernel -------------------------------------------------------------------

// monotone map fp32 -> int32 (and back): larger float <=> larger int
__device__ __forceinline__ int float_key(float x)
{
    const int b = __float_as_int(x);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_float(int k)
{
    return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}

template <int D>
__global__ __launch_bounds__(FwdCfg<D>::NT) void forward_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ Vt,
    const uint32_t* __restrict__ vmax, const int32_t* __restrict__ idx, bf16_t* __restrict__ O,
    float* __restrict__ lse, int N, int B, int k, float scale, int ntiles, int bh)
{
    using C = FwdCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Qs = smem;
    int* Os = reinterpret_cast<int*>(Qs + (size_t)C::TILE * C::QSTRIDE);   // fixed point, 2^F
    int* mkey = Os + C::TILE * C::OSTRIDE;       // pass 1: key of the row max; then m (log2 units) as float bits
    int* lsum = mkey + C::TILE;                  // fixed point, 2^F
    uint32_t* mask = reinterpret_cast<uint32_t*>(lsum + C::TILE);
    uint16_t* rlist = reinterpret_cast<uint16_t*>(mask + C::RANGE * C::MW);
    uint32_t* ulist = reinterpret_cast<uint32_t*>(rlist + C::NW * C::TILE);   // non-empty groups of a range
    int* next = reinterpret_cast<int*>(ulist + C::RANGE);

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    // consecutive workgroups take different slices of the same tile index (late, long tiles first)
    const int s = blockIdx.x % bh;
    const int tile = ntiles - 1 - blockIdx.x / bh;
    const int t0 = tile * C::TILE;
    const int rows_here = min(C::TILE, N - t0);
    const int NG = B / 32;
    const float c2 = scale * kLog2e;
    const int64_t sbase = (int64_t)s * N;
    const bf16_t* Qg = Q + (sbase + t0) * D;
    const bf16_t* Kg = K + sbase * D;
    const bf16_t* Vtg = Vt + sbase * D;
    uint16_t* rl = rlist + wave * C::TILE;

    // Fixed-point scale: a row attends at most nkeys keys, so sum p <= nkeys < 2^(31-F).
    const int nkeys = min(t0 + rows_here, (k + 1) * B);
    const float Fbits = (float)(30 - (32 - __clz(nkeys)));

    // 0. Q tile -> LDS; clear the accumulators
    for (int i = tid; i < C::TILE * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < rows_here) v = *reinterpret_cast<const uint4*>(Qg + (int64_t)r * D + c * 8);
        *reinterpret_cast<uint4*>(Qs + (size_t)r * C::QSTRIDE + c * 16) = v;
    }
    for (int i = tid; i < C::TILE * C::OSTRIDE; i += C::NT) Os[i] = 0;
    for (int i = tid; i < C::TILE; i += C::NT) { mkey[i] = (int)0x80000000; lsum[i] = 0; }
    __syncthreads();

    const int gmax = (t0 + rows_here - 1) >> 5;        // groups below the last row's own group

    for (int pass = 0; pass < 2; ++pass) {
        // own 32-key groups, causal
        for (int p = wave; p < rows_here / 16; p += C::NW) {
            const int unit = p >> 1, st = p & 1;
            const int row = 32 * unit + 16 * st + m16;
            const int64_t kap = (t0 >> 5) + unit;
            Frag qb[C::KS];
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
                qb[ks].q = *reinterpret_cast<const uint4*>(Qs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
            f32x4_t sc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                if (mt <= st) {
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) {
                        Frag ka;
                        ka.q = *reinterpret_cast<const uint4*>(Kg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                        sc[mt] = mfma16(ka, qb[ks], sc[mt]);
                    }
                }
            }
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool vis = 16 * (e >> 2) + 4 * g + (e & 3) <= 16 * st + m16;
                x[e] = vis ? sc[e >> 2][e & 3] * c2 : -INFINITY;
            }
            if (pass == 0) {
                float mx = x[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) mx = fmaxf(mx, x[e]);
                atomicMax(&mkey[row], float_key(mx));
            } else {
                const float mr = __int_as_float(mkey[row]);
                float lp = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) { x[e] = fast_exp2(x[e] - mr); lp += x[e]; }
                atomicAdd(&lsum[row], __float2int_rn(lp));
                Frag pb;
#pragma unroll
                for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    Frag va;
                    va.q = *reinterpret_cast<const uint4*>(Vtg + slot_major_offset<D>(kap, mt, lane));
                    f32x4_t o = mfma16(va, pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        atomicAdd(&Os[row * C::OSTRIDE + tile_chan<D>(mt, 4 * g + i)], (int)o[i]);
                }
            }
        }

        // routed groups (and, for B > 32, the earlier groups of the own block)
        for (int lo = 0; lo < gmax; lo += C::RANGE) {
            const int hi = min(gmax, lo + C::RANGE);
            __syncthreads();
            for (int i = tid; i < (hi - lo) * C::MW; i += C::NT) mask[i] = 0u;
            if (tid == 0) *next = 0;
            __syncthreads();
            build_group_mask<C::TILE, C::NT, C::MW>(mask, idx + (sbase + t0) * k, t0, rows_here, k, B, NG, lo,
                                                     hi, tid);
            __syncthreads();
            // non-empty groups of this range -> ulist (count << 16 | group)
            for (int i = tid; i < hi - lo; i += C::NT) {
                int cnt = 0;
#pragma unroll
                for (int wd = 0; wd < C::MW; ++wd) cnt += __popc(mask[i * C::MW + wd]);
                if (cnt) ulist[atomicAdd(next, 1)] = (uint32_t)i | ((uint32_t)cnt << 16);
            }
            __syncthreads();
            const int nunits = *next;

            auto load_unit = [&](uint32_t entry, Frag (&ka)[2][C::KS], Frag (&va)[C::MT]) {
                const int64_t kap = lo + (int)(entry & 0xffffu);
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks)
                        ka[mt][ks].q = *reinterpret_cast<const uint4*>(Kg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
                if (pass == 1) {
#pragma unroll
                    for (int mt = 0; mt < C::MT; ++mt)
                        va[mt].q = *reinterpret_cast<const uint4*>(Vtg + slot_major_offset<D>(kap, mt, lane));
                }
            };
            auto run_unit = [&](uint32_t entry, const Frag (&ka)[2][C::KS], const Frag (&va)[C::MT]) {
                const int ui = (int)(entry & 0xffffu), cnt = (int)(entry >> 16);
                int base = 0;
#pragma unroll
                for (int r = 0; r < C::TILE / 64; ++r) {
                    const uint64_t m64 = (uint64_t)mask[ui * C::MW + 2 * r] | ((uint64_t)mask[ui * C::MW + 2 * r + 1] << 32);
                    if ((m64 >> lane) & 1ull) rl[base + __popcll(m64 & ((1ull << lane) - 1ull))] = (uint16_t)(64 * r + lane);
                    base += __popcll(m64);
                }
                __builtin_amdgcn_wave_barrier();
                // Sub-tiles of 16 rows.  The row ids of four sub-tiles are read at once, and the
                // LDS gather of the next sub-tile is issued before the arithmetic and the atomics
                // of the current one, so it never waits behind them.
                auto gather = [&](bool valid, int row, Frag (&qb)[C::KS], float& mr) {
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks)
                        qb[ks].q = *reinterpret_cast<const uint4*>(Qs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
                    // rows beyond the list get an infinite reference: their p is exactly 0
                    mr = (pass == 1 && valid) ? __int_as_float(mkey[row]) : INFINITY;
                };
                auto compute = [&](bool valid, int row, const Frag (&qb)[C::KS], float mr) {
                    f32x4_t sc[2];
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) {
                        sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < C::KS; ++ks) sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                    }
                    if (pass == 0) {
                        float mx = fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3]));
                        mx = fmaxf(mx, fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
                        if (valid) atomicMax(&mkey[row], float_key(mx * c2));
                    } else {
                        float x[8], lp = 0.f;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            x[e] = fast_exp2(fmaf(sc[e >> 2][e & 3], c2, -mr));
                            lp += x[e];
                        }
                        Frag pb;
#pragma unroll
                        for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
                        int oi[C::MT][4];
#pragma unroll
                        for (int mt = 0; mt < C::MT; ++mt) {
                            const f32x4_t o = mfma16(va[mt], pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                            for (int i = 0; i < 4; ++i) oi[mt][i] = (int)o[i];      // toward zero: see header
                        }
                        if (valid) {
                            atomicAdd(&lsum[row], __float2int_rn(lp));
                            int* orow = Os + row * C::OSTRIDE + g * (D / 4);
#pragma unroll
                            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                                for (int i = 0; i < 4; ++i) atomicAdd(&orow[4 * mt + i], oi[mt][i]);
                        }
                    }
                };
                for (int c0 = 0; c0 < cnt; c0 += 64) {
                    bool val[4];
                    int rows[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        val[j] = c0 + 16 * j + m16 < cnt;
                        rows[j] = rl[val[j] ? c0 + 16 * j + m16 : 0];
                    }
                    const int left = cnt - c0;          // > 0
                    Frag qA[C::KS], qB[C::KS];
                    float mA, mB;
                    gather(val[0], rows[0], qA, mA);
                    if (left > 16) gather(val[1], rows[1], qB, mB);
                    compute(val[0], rows[0], qA, mA);
                    if (left > 16) {
                        if (left > 32) gather(val[2], rows[2], qA, mA);
                        compute(val[1], rows[1], qB, mB);
                        if (left > 32) {
                            if (left > 48) gather(val[3], rows[3], qB, mB);
                            compute(val[2], rows[2], qA, mA);
                            if (left > 48) compute(val[3], rows[3], qB, mB);
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            };

            // waves take the units round robin; the operands of a wave's next unit are in flight
            // while it works on the current one
            Frag kaA[2][C::KS], vaA[C::MT], kaB[2][C::KS], vaB[C::MT];
            int u = wave;
            if (u < nunits) load_unit(ulist[u], kaA, vaA);
            while (u < nunits) {
                if (u + C::NW < nunits) load_unit(ulist[u + C::NW], kaB, vaB);
                run_unit(ulist[u], kaA, vaA);
                u += C::NW;
                if (u >= nunits) break;
                if (u + C::NW < nunits) load_unit(ulist[u + C::NW], kaA, vaA);
                run_unit(ulist[u], kaB, vaB);
                u += C::NW;
            }
        }
        __syncthreads();
        if (pass == 0) {      // keys -> reference values minus F (log2 units), in place
            for (int i = tid; i < C::TILE; i += C::NT) mkey[i] = __float_as_int(key_float(mkey[i]) - Fbits);
            __syncthreads();
        }
    }

    // normalise and write out: O = acc * 2^e[c] / l  (the 2^F of both cancels)
    bf16_t* Og = O + (sbase + t0) * D;
    for (int i = tid; i < rows_here * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        const float lf = (float)lsum[r];
        const float inv = 1.f / lf;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = ldexpf((float)Os[r * C::OSTRIDE + 8 * c + e] * inv, scale_exponent(vmax[s * D + 8 * c + e]));
        Vec8<bf16_t>::store(Og + (int64_t)r * D + 8 * c, v);
        if (c == 0) lse[sbase + t0 + r] = (__int_as_float(mkey[r]) + fast_log2(lf)) * kLn2;
    }
}

template <int D>
static hipError_t fwd_launch(const Dims& s, const void* Q, const void* K, const void* Vt,
                             const uint32_t* vmax, const int32_t* idx, void* O, float* lse,
                             hipStream_t st)
{
    using C = FwdCfg<D>;
    const int ntiles = (s.N + C::TILE - 1) / C::TILE;
    hipError_t e = hipFuncSetAttribute((const void*)forward_mfma_kernel<D>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((forward_mfma_kernel<D>), dim3((unsigned)(ntiles * s.bh)), dim3(C::NT), C::LDS,
                       st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)Vt, vmax, idx,
                       (bf16_t*)O, lse, s.N, s.B, s.k, s.scale, ntiles, s.bh);
    return hipGetLastError();
}

size_t forward_mfma_ws_bytes(const Dims& s)
{
    return sizeof(bf16_t) * (size_t)s.bh * s.N * s.D + 256 + sizeof(uint32_t) * (size_t)s.bh * s.D;
}

// ws: [bh*N*D bf16 slot-ordered scaled V][pad to 256][bh*D fp32 bits: channel maxima]
hipError_t launch_forward_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                               void* ws, const int32_t* idx, const int32_t* off, const int32_t* ql,
                               const int32_t* chunk, void* O, float* lse, hipStream_t st)
{
    const size_t vt_bytes = (sizeof(bf16_t) * (size_t)s.bh * s.N * s.D + 255) & ~(size_t)255;
    uint32_t* vmax = reinterpret_cast<uint32_t*>((char*)ws + vt_bytes);
    hipError_t e = launch_absmax(s, V, vmax, st);
    if (e != hipSuccess) return e;
    e = launch_slot_major_copy(s, V, ws, vmax, st);
    if (e != hipSuccess) return e;
    return s.D == 64 ? fwd_launch<64>(s, Q, K, ws, vmax, idx, O, lse, st)
                     : fwd_launch<128>(s, Q, K, ws, vmax, idx, O, lse, st);
}

}  // namespace moba
