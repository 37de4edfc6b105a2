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
//           bound (each 32-key partial of P V and of the row sum rounds to nearest: unbiased,
//           2^-(F+1) per add at most; F >= 17, see kTileForwardMaxKeys).
//           Integer adds commute exactly: the result does not depend on the order in which
//           waves arrive, so the output is bit-reproducible.
// Which rows go with which key block is a set of compact row lists in LDS (one byte per
// (row, block) pair, sorted by block), built once per tile from the query-major routing by a
// counting sort and used by both passes; the earlier 32-key groups of a row's own block
// (B > 32) are dense work and go with the own group.  With blocks of 64 keys and more (d = 64)
// a wave takes two 32-key groups of a block at a time: their operands stay in registers while
// the block's listed rows go by and a row's P V over both groups leaves the MFMA accumulators
// as one set of LDS adds (half the adds per key).
//
// What bounds the kernel is the operand traffic, not the arithmetic: with scattered routing a
// 256-query tile meets a key block with ~16 of its rows, so every 1-2 MFMA sub-tiles need a
// fresh 4 KB of K (both passes) and 4 KB of V.  Hence (a) K and V are read from copies laid
// out in MFMA operand order, 1 KB of consecutive bytes per load instruction (four times the
// rate of the row-major pattern on this chip), (b) the workgroups of one XCD work on the same
// slice and walk its blocks in ascending order, so these reads hit that XCD's L2, and (c) 16
// waves per workgroup keep loads, LDS traffic and MFMA work of different units overlapped.
#include <type_traits>

#include "mfma.h"

namespace moba {

template <int D>
struct FwdCfg {
    static constexpr int TILE = D == 64 ? 256 : 128;   // queries per workgroup
    static constexpr int NW = D == 64 ? 16 : 12;       // waves per workgroup (registers allow no more)
    static constexpr int NT = NW * kWave;
    static constexpr int QSTRIDE = D * 2 + 16;         // bytes per Q row in LDS
    static constexpr int OSTRIDE = D + 1;              // words per accumulator row
    static constexpr int MT = D / 16;                  // 16-channel tiles of a row
    static constexpr int KS = D / 32;                  // contraction steps of q.k
    static constexpr int RANGE = 1024;                 // key blocks per set of row lists (at most)
    static constexpr int LCAP = 16384;                 // (row, block) pairs per set of row lists
    static constexpr size_t LDS = (size_t)TILE * QSTRIDE + 4 * TILE * OSTRIDE + 4 * 2 * TILE +
                                  4 * 2 * (RANGE + 1) + 4 * NW + 8 + LCAP + 64;
};

// ---- the slot-ordered transposed copy alone (see mfma.h; the key-major kernels use it unscaled;
// the copies of the query-tile kernels are made in prepare.hip) -----------

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
    const int b = x != x ? 0x7fc00000 : __float_as_int(x);      // a NaN of either sign: above everything
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_float(int k)
{
    return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}
// sum / maximum (NaN-propagating) over the four lanes m16 + 16 g, g = 0 .. 3, in all of them:
// v_permlane32_swap / v_permlane16_swap exchange the halves / the odd and even quarters of a wave
__device__ __forceinline__ float sum_over_g(float x)
{
    const uint32_t b = __float_as_uint(x);
    const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    const uint32_t y = __float_as_uint(__uint_as_float(h[0]) + __uint_as_float(h[1]));
    const auto q = __builtin_amdgcn_permlane16_swap(y, y, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}
__device__ __forceinline__ float max_over_g(float x)
{
    const uint32_t b = __float_as_uint(x);
    const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    const uint32_t y = __float_as_uint(max_nan(__uint_as_float(h[0]), __uint_as_float(h[1])));
    const auto q = __builtin_amdgcn_permlane16_swap(y, y, false, false);
    return max_nan(__uint_as_float(q[0]), __uint_as_float(q[1]));
}

// GMAX: 32-key groups of a block that one unit takes together (2 needs B >= 64 and the registers
// of d = 64)
template <int D, int GMAX>
__global__ __launch_bounds__(FwdCfg<D>::NT) void forward_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Ka, const bf16_t* __restrict__ Vt,
    const uint32_t* __restrict__ vmax, const int32_t* __restrict__ idx, bf16_t* __restrict__ O,
    float* __restrict__ lse, int N, int B, int k, float scale, int ntiles, int bh, int G)
{
    using C = FwdCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Qs = smem;
    int* Os = reinterpret_cast<int*>(Qs + (size_t)C::TILE * C::QSTRIDE);   // fixed point, 2^F
    int* mkey = Os + C::TILE * C::OSTRIDE;       // pass 1: key of the row max; then m (log2 units) as float bits
    int* lsum = mkey + C::TILE;                  // fixed point, 2^F
    uint32_t* cur = reinterpret_cast<uint32_t*>(lsum + C::TILE);
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
    const bf16_t* Qg = Q + (sbase + t0) * D;
    const int skv = s / G;                                  // G query heads share a key/value head
    const char* Kg = reinterpret_cast<const char*>(Ka + (int64_t)skv * N * D);
    const char* Vtg = reinterpret_cast<const char*>(Vt + (int64_t)skv * N * D);
    const uint32_t vlane = (uint32_t)lane * 16u;   // this lane's bytes inside a K or V operand
    const uint32_t qlane = 16u * g;

    // Fixed-point scale: a row attends at most nkeys keys, so sum p <= nkeys < 2^(31-F).
    // (the library admits at most kTileForwardMaxKeys keys per query here: F >= 17)
    const int nkeys = (int)min((int64_t)(t0 + rows_here), (int64_t)(k + 1) * B);
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

    // blocks strictly before the own block of the tile's last row, taken `range` at a time so
    // that a range's (row, block) pairs fit rows8
    const int pastmax = (t0 + rows_here - 1) / B;
    const int range = (int64_t)k * C::TILE <= C::LCAP ? C::RANGE : C::LCAP / C::TILE;
    const bool one_range = pastmax <= range;

    auto load_k = [&](int kap, Frag (&ka)[2][C::KS]) {
        const char* kb = Kg + (int64_t)kap * (64 * D);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
                ka[mt][ks].q = *reinterpret_cast<const uint4*>(kb + vlane + (mt * C::KS + ks) * 1024);
    };
    auto load_v = [&](int kap, Frag (&va)[C::MT]) {
        const char* vb = Vtg + (int64_t)kap * (64 * D);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
            va[mt].q = *reinterpret_cast<const uint4*>(vb + vlane + mt * 1024);
    };
    auto gather_q = [&](int row, Frag (&qb)[C::KS]) {
        const unsigned char* qr = Qs + (uint32_t)row * C::QSTRIDE + qlane;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) qb[ks].q = *reinterpret_cast<const uint4*>(qr + 64 * ks);
    };
    // x: eight scores of this lane's row (log2 units, reference subtracted) -> probabilities;
    // their sum goes to lp and P V to the MFMA accumulators o, which a row's unit keeps over all
    // the 32-key groups it covers; flush() then adds them to the row's accumulators in LDS,
    // rounded to nearest once
    auto attend = [&](float (&x)[8], const Frag (&va)[C::MT], float& lp, f32x4_t (&o)[C::MT], bool fresh) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { x[e] = fast_exp2(x[e]); lp += x[e]; }
        Frag pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
            o[mt] = mfma16(va[mt], pb, fresh ? f32x4_t{0.f, 0.f, 0.f, 0.f} : o[mt]);
    };
    auto flush = [&](int row, float lp, const f32x4_t (&o)[C::MT], bool valid) {
        int oi[C::MT][4];
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) oi[mt][i] = __float2int_rn(o[mt][i]);
        lp = sum_over_g(lp);                       // the row's 32 (64) keys in one add, from one lane
        if (valid) {
            if (g == 0) atomicAdd(&lsum[row], __float2int_rn(lp));
            int* orow = Os + (uint32_t)row * C::OSTRIDE + g * (D / 4);
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) atomicAdd(&orow[4 * mt + i], oi[mt][i]);
        }
    };
    auto clear = [&](f32x4_t (&o)[C::MT]) {
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) o[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    };

    for (int pass = 0; pass < 2; ++pass) {
        // own block: the row's own 32-key group under the causal mask and, for B > 32, the
        // block's earlier groups in full
        for (int p = wave; p < rows_here / 16; p += C::NW) {
            const int unit = p >> 1, st = p & 1;
            const int row = 32 * unit + 16 * st + m16;
            const int kown = (t0 >> 5) + unit;
            const int kfirst = NG == 1 ? kown : kown - kown % NG;
            Frag qb[C::KS];
            gather_q(row, qb);
            const float mr = pass == 1 ? __int_as_float(mkey[row]) : 0.f;
            float mx = -INFINITY, lp = 0.f;
            f32x4_t o[C::MT];
            if (GMAX > 1) clear(o);
            for (int kap = kfirst; kap <= kown; ++kap) {
                const bool own = kap == kown;
                Frag ka[2][C::KS], va[C::MT];
                load_k(kap, ka);
                if (pass == 1) load_v(kap, va);
                f32x4_t sc[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    if (!own || mt <= st) {
#pragma unroll
                        for (int ks = 0; ks < C::KS; ++ks) sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                    }
                }
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool vis = !own || 16 * (e >> 2) + 4 * g + (e & 3) <= 16 * st + m16;
                    x[e] = vis ? fmaf(sc[e >> 2][e & 3], c2, -mr) : -INFINITY;
                }
                if (pass == 0) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) mx = max_nan(mx, x[e]);
                } else {
                    attend(x, va, lp, o, GMAX == 1);
                    if (GMAX == 1) {          // (no registers to keep the sums over the groups)
                        flush(row, lp, o, true);
                        lp = 0.f;
                    }
                }
            }
            if (pass == 0) {
                mx = max_over_g(mx);
                if (g == 0) atomicMax(&mkey[row], float_key(mx));
            }
            else if (GMAX > 1) flush(row, lp, o, true);
        }

        // routed blocks
        for (int lo = 0; lo < pastmax; lo += range) {
            const int hi = min(pastmax, lo + range);
            if (pass == 0 || !one_range) {
                __syncthreads();
                build_block_lists<C::TILE, C::NT>(idx + (sbase + t0) * k, t0, rows_here, k, B, lo, hi,
                                                  cur, offs, rows8, C::LCAP, wsum, tid);
                // Non-empty blocks of this range, ascending: the workgroups of an XCD then walk
                // K and V in the same order and find each other's blocks in the L2.
                if (tid == 0) *take = 0;
                list_nonempty<C::NT>(offs, hi - lo, ulist, next, wsum, tid);
            }
            const int nblk = *next;

            // one unit = one or two 32-key groups of a listed block: the operands of both stay in
            // registers while the block's rows go by, sixteen at a time, and a row's sums over
            // both groups reach LDS in one set of adds
            auto load_unit = [&](int e, int gi, auto gc, Frag (&ka)[GMAX][2][C::KS], Frag (&va)[GMAX][C::MT],
                                 int& beg, int& end) {
                const int j = __builtin_amdgcn_readfirstlane((int)ulist[e]);
                beg = offs[j];
                end = offs[j + 1];
#pragma unroll
                for (int u = 0; u < decltype(gc)::value; ++u) {
                    const int kap = (lo + j) * NG + gi + u;
                    load_k(kap, ka[u]);
                    if (pass == 1) load_v(kap, va[u]);
                }
            };
            auto run_unit = [&](int beg_v, int end_v, auto gc, const Frag (&ka)[GMAX][2][C::KS],
                                const Frag (&va)[GMAX][C::MT]) {
                constexpr int GC = decltype(gc)::value;
                const int beg = __builtin_amdgcn_readfirstlane(beg_v);
                const int end = min(__builtin_amdgcn_readfirstlane(end_v), (int)C::LCAP);
                // Sub-tiles of 16 listed rows.  Lanes beyond the list work on whatever row id they
                // read (always inside the tile) and add nothing.
                for (int c0 = beg; c0 < end; c0 += 16) {
                    const bool valid = m16 < end - c0;
                    const int row = rows8[c0 + m16] & (C::TILE - 1);
                    Frag qb[C::KS];
                    gather_q(row, qb);
                    const float mr = pass == 1 ? __int_as_float(mkey[row]) : 0.f;
                    auto scores = [&](int u, f32x4_t (&sc)[2]) {
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt) {
                            sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int ks = 0; ks < C::KS; ++ks) sc[mt] = mfma16(ka[u][mt][ks], qb[ks], sc[mt]);
                        }
                    };
                    if (pass == 0) {
                        // (a NaN score makes the row's reference, and with it the row, NaN)
                        float mx = -INFINITY;
#pragma unroll
                        for (int u = 0; u < GC; ++u) {
                            f32x4_t sc[2];
                            scores(u, sc);
#pragma unroll
                            for (int e = 0; e < 8; ++e) mx = max_nan(mx, sc[e >> 2][e & 3]);
                        }
                        // the four lanes of a row (g = 0 .. 3) hold different keys: their maximum by
                        // two lane swaps, so that one lane per row goes to LDS
                        mx = max_over_g(mx);
                        if (valid && g == 0) atomicMax(&mkey[row], float_key(mx * c2));
                    } else {
                        float lp = 0.f;
                        f32x4_t o[C::MT];
#pragma unroll
                        for (int u = 0; u < GC; ++u) {
                            f32x4_t sc[2];
                            scores(u, sc);
                            float x[8];
#pragma unroll
                            for (int e = 0; e < 8; ++e) x[e] = fmaf(sc[e >> 2][e & 3], c2, -mr);
                            attend(x, va[u], lp, o, u == 0);
                        }
                        flush(row, lp, o, valid);
                    }
                }
            };

            // waves take the listed blocks as they get free (other waves cover the operand latency)
            int e = take_unit(take, lane);
            while (e < nblk) {
                const int en = take_unit(take, lane);     // asked for early: its latency hides behind this unit
                for (int gi = 0; gi < NG; gi += GMAX) {
                    Frag ka[GMAX][2][C::KS], va[GMAX][C::MT];
                    int beg, end;
                    if (GMAX == 2 && gi + 1 < NG) {
                        load_unit(e, gi, std::integral_constant<int, GMAX>{}, ka, va, beg, end);
                        run_unit(beg, end, std::integral_constant<int, GMAX>{}, ka, va);
                    } else {
                        load_unit(e, gi, std::integral_constant<int, 1>{}, ka, va, beg, end);
                        run_unit(beg, end, std::integral_constant<int, 1>{}, ka, va);
                    }
                }
                e = en;
            }
        }
        __syncthreads();
        if (pass == 0) {      // keys -> reference values minus F (log2 units), in place
            for (int i = tid; i < C::TILE; i += C::NT) mkey[i] = __float_as_int(key_float(mkey[i]) - Fbits);
            if (tid == 0) *take = 0;
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
        for (int e = 0; e < 8; ++e) {
            const uint32_t vm = vmax[skv * D + 8 * c + e];
            v[e] = nonfinite_bits(vm) ? NAN          // V holds an infinity or a NaN in this channel
                                      : ldexpf((float)Os[r * C::OSTRIDE + 8 * c + e] * inv, scale_exponent(vm));
        }
        Vec8<bf16_t>::store(Og + (int64_t)r * D + 8 * c, v);
        if (c == 0) lse[sbase + t0 + r] = (__int_as_float(mkey[r]) + fast_log2(lf)) * kLn2;
    }
}

template <int D, int GMAX>
static hipError_t fwd_launch(const Dims& s, const void* Q, const void* K, const void* Vt,
                             const uint32_t* vmax, const int32_t* idx, void* O, float* lse,
                             hipStream_t st)
{
    using C = FwdCfg<D>;
    const int ntiles = (s.N + C::TILE - 1) / C::TILE;
    hipError_t e = ensure_dynamic_lds((const void*)forward_mfma_kernel<D, GMAX>, (size_t)(C::LDS));
    if (e != hipSuccess) return e;
    ProfileScope timing(MOBA_PROFILE_FORWARD, st);
    hipLaunchKernelGGL((forward_mfma_kernel<D, GMAX>), dim3((unsigned)schedule_grid(s.bh, ntiles)), dim3(C::NT), C::LDS,
                       st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)Vt, vmax, idx,
                       (bf16_t*)O, lse, s.N, s.B, s.k, s.scale, ntiles, s.bh, s.G);
    return hipGetLastError();
}

// ws: the prepared copies the forward reads (maxima of V, operand-ordered K, slot-ordered scaled V);
// with a workspace shared with the backward: behind the backward's D vector, and everything the
// backward reads as well
size_t forward_mfma_ws_bytes(const Dims& s)
{
    if (shared_workspace(s)) return backward_mfma_ws_bytes(s);
    return prepared_layout(s, kPrepForward, nullptr, nullptr);
}

hipError_t launch_forward_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                               void* ws, const int32_t* idx, const int32_t* off, const int32_t* ql,
                               void* O, float* lse, hipStream_t st)
{
    Prepared p;
    if (shared_workspace(s)) {
        prepared_layout(s, kPrepAll, (char*)ws + a256(sizeof(float) * (size_t)s.bh * s.N), &p);
    } else {
        prepared_layout(s, kPrepForward, ws, &p);
        p.kmax = nullptr;                                    // (only the dQ kernel scales K)
    }
    hipError_t e = launch_prepare(kv_view(s), K, V, p, st);  // K and V: one slice per key/value head
    if (e != hipSuccess) return e;
    if (s.D == 128) return fwd_launch<128, 1>(s, Q, p.Ka, p.Vt, p.vmax, idx, O, lse, st);
    return s.B >= 64 ? fwd_launch<64, 2>(s, Q, p.Ka, p.Vt, p.vmax, idx, O, lse, st)
                     : fwd_launch<64, 1>(s, Q, p.Ka, p.Vt, p.vmax, idx, O, lse, st);
}

}  // namespace moba
