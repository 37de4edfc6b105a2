// MoBA forward on bf16 MFMA (paper Section 4.2, forward pass with gather-and-densify),
// re-cut for CDNA4: a workgroup owns a tile of consecutive queries and keeps their
// Q rows (bf16) and their output accumulators (fp32) in LDS for the whole kernel -- the
// running output of the paper's forward algorithm never goes to HBM.  It walks the 32-key
// groups its queries were routed to; for each group one wave gathers the routed rows
// out of LDS sixteen at a time as a dense MFMA operand, computes S^T = K Q^T, turns it
// into probabilities and adds P V into the rows' accumulators with LDS float atomics.
//
// Softmax without rescaling: every row gets a fixed reference m_ref = the largest logit of
// its own (causal) 32-key group, computed first.  All later contributions are
// exp(s - m_ref), so they commute and any wave may add to any row in any order.  A logit
// more than 2^90 above its row's reference would overflow; such a row is flagged, left
// out of the fast path and recomputed at the end by a plain per-row online softmax.
//
// Which rows go with which key group is kept as a bit matrix in LDS (one 256-bit row per
// group), built from the query-major routing; 1024 groups are covered at a time.
#include "mfma.h"

namespace moba {

template <int D>
struct FwdCfg {
    static constexpr int TILE = D == 64 ? 256 : 128;   // queries per workgroup
    static constexpr int NW = 8;                       // waves per workgroup
    static constexpr int NT = NW * kWave;
    static constexpr int QSTRIDE = D * 2 + 16;         // bytes per Q row in LDS
    static constexpr int OSTRIDE = D + 1;              // floats per accumulator row
    static constexpr int MT = D / 16;                  // 16-channel tiles of a row
    static constexpr int KS = D / 32;                  // contraction steps of q.k
    static constexpr int MW = TILE / 32;               // mask words per key group
    static constexpr int RANGE = 1024;                 // key groups per bit matrix
    static constexpr size_t LDS = (size_t)TILE * QSTRIDE + sizeof(float) * TILE * OSTRIDE +
                                  sizeof(float) * 3 * TILE + sizeof(uint32_t) * RANGE * MW +
                                  sizeof(uint16_t) * NW * TILE + 64;
};

constexpr float kOverflowLog2 = 90.f;

// ---- slot-ordered transposed copy (see mfma.h) ---------------------------------------
template <int D>
__global__ __launch_bounds__(256) void slot_major_copy_kernel(const bf16_t* __restrict__ X,
                                                              bf16_t* __restrict__ Xt,
                                                              int64_t total_groups)
{
    __shared__ bf16_t tile[32 * (D + 8)];
    const int64_t kap = blockIdx.x;
    if (kap >= total_groups) return;
    const bf16_t* src = X + kap * 32 * D;
    for (int i = threadIdx.x; i < 32 * D / 8; i += 256) {
        const int r = i / (D / 8), c = i % (D / 8);
        *reinterpret_cast<uint4*>(&tile[r * (D + 8) + c * 8]) =
            *reinterpret_cast<const uint4*>(src + r * D + c * 8);
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

hipError_t launch_slot_major_copy(const Dims& s, const void* X, void* Xt, hipStream_t st)
{
    const int64_t groups = (int64_t)s.bh * s.N / 32;
    if (groups == 0) return hipSuccess;
    if (s.D == 64)
        hipLaunchKernelGGL(slot_major_copy_kernel<64>, dim3((unsigned)groups), dim3(256), 0, st,
                           (const bf16_t*)X, (bf16_t*)Xt, groups);
    else
        hipLaunchKernelGGL(slot_major_copy_kernel<128>, dim3((unsigned)groups), dim3(256), 0, st,
                           (const bf16_t*)X, (bf16_t*)Xt, groups);
    return hipGetLastError();
}

// ---- plain per-row attention for flagged rows (one wave) -----------------------------
// scratch: D + 128 floats of LDS private to the wave.
template <int D>
__device__ void forward_row_plain(const bf16_t* __restrict__ Qs_, const bf16_t* __restrict__ Ks,
                                  const bf16_t* __restrict__ Vs, const int32_t* __restrict__ sel,
                                  int t, int B, int k, float scale, float* scratch, int lane,
                                  bf16_t* __restrict__ Orow, float* __restrict__ lse_out)
{
    constexpr int DP = D / kWave;
    float* qs = scratch;
    float* ps = scratch + D;
    int* us = reinterpret_cast<int*>(ps + kWave);
    for (int c = lane; c < D; c += kWave) qs[c] = bf16_to_f32(Qs_[c]);
    __builtin_amdgcn_wave_barrier();
    const int own = t / B;
    const int total = k * B + (t % B) + 1;      // slot-major positions; empty slots are skipped
    float m = -INFINITY, l = 0.f, acc[DP];
#pragma unroll
    for (int e = 0; e < DP; ++e) acc[e] = 0.f;
    for (int i0 = 0; i0 < total; i0 += kWave) {
        const int i = i0 + lane;
        int u = -1;
        if (i < total) {
            const int slot = i / B, r = i - slot * B;
            const int blk = slot < k ? sel[slot] : own;
            if (blk >= 0 && (slot == k || blk < own)) u = blk * B + r;
        }
        float z = -INFINITY;
        if (u >= 0) {
            float a = 0.f;
            const bf16_t* kr = Ks + (int64_t)u * D;
            for (int c = 0; c < D; ++c) a = fmaf(bf16_to_f32(kr[c]), qs[c], a);
            z = scale * a;
        }
        const float cm = wave_max(z);
        if (cm == -INFINITY) continue;           // a whole chunk of empty slots
        const float m_new = fmaxf(m, cm);
        const float p = __expf(z - m_new);
        const float alpha = __expf(m - m_new);
        l = l * alpha + wave_sum(p);
        m = m_new;
        ps[lane] = p; us[lane] = u;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int e = 0; e < DP; ++e) acc[e] *= alpha;
        for (int a = 0; a < kWave; ++a) {
            const int ua = us[a];
            if (ua < 0) continue;
            const float pa = ps[a];
            const bf16_t* vr = Vs + (int64_t)ua * D;
#pragma unroll
            for (int e = 0; e < DP; ++e) acc[e] = fmaf(pa, bf16_to_f32(vr[lane + e * kWave]), acc[e]);
        }
        __builtin_amdgcn_wave_barrier();
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < DP; ++e) Orow[lane + e * kWave] = f32_to_bf16(acc[e] * inv);
    if (lane == 0) *lse_out = m + __logf(l);
}

// ---- the tile kernel -------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(FwdCfg<D>::NT) void forward_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ Vt, const int32_t* __restrict__ idx, bf16_t* __restrict__ O,
    float* __restrict__ lse, int N, int B, int k, float scale, int ntiles, int bh)
{
    using C = FwdCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* Qs = smem;
    float* Os = reinterpret_cast<float*>(Qs + (size_t)C::TILE * C::QSTRIDE);
    float* mref = Os + C::TILE * C::OSTRIDE;          // log2 units
    float* lsum = mref + C::TILE;
    int* bad = reinterpret_cast<int*>(lsum + C::TILE);
    uint32_t* mask = reinterpret_cast<uint32_t*>(bad + C::TILE);
    uint16_t* rlist = reinterpret_cast<uint16_t*>(mask + C::RANGE * C::MW);
    int* next = reinterpret_cast<int*>(rlist + C::NW * C::TILE);

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

    // 1. Q tile -> LDS
    for (int i = tid; i < C::TILE * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < rows_here) v = *reinterpret_cast<const uint4*>(Qg + (int64_t)r * D + c * 8);
        *reinterpret_cast<uint4*>(Qs + (size_t)r * C::QSTRIDE + c * 16) = v;
    }
    for (int i = tid; i < C::TILE; i += C::NT) bad[i] = 0;
    __syncthreads();

    // 2. own 32-key groups, causal: set m_ref, and store (not add) l and O
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
        float x[8], mx = -INFINITY;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool vis = 16 * mt + 4 * g + i <= 16 * st + m16;
                x[4 * mt + i] = vis ? sc[mt][i] * c2 : -INFINITY;
                mx = fmaxf(mx, x[4 * mt + i]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float lp = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { x[e] = fast_exp2(x[e] - mx); lp += x[e]; }
        lp += __shfl_xor(lp, 16, 64);
        lp += __shfl_xor(lp, 32, 64);
        if (g == 0) { mref[row] = mx; lsum[row] = lp; }
        Frag pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
            Frag va;
            va.q = *reinterpret_cast<const uint4*>(Vtg + slot_major_offset<D>(kap, mt, lane));
            f32x4_t o = mfma16(va, pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int i = 0; i < 4; ++i) Os[row * C::OSTRIDE + tile_chan<D>(mt, 4 * g + i)] = o[i];
        }
    }
    __syncthreads();

    // 3. routed groups (and, for B > 32, the earlier groups of the own block)
    const int gmax = (t0 + rows_here - 1) >> 5;        // groups below the last row's own group
    for (int lo = 0; lo < gmax; lo += C::RANGE) {
        const int hi = min(gmax, lo + C::RANGE);
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
            Frag ka[2][C::KS], va[C::MT];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks)
                    ka[mt][ks].q = *reinterpret_cast<const uint4*>(Kg + (kap * 32 + 16 * mt + m16) * D + 8 * g + 32 * ks);
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
                va[mt].q = *reinterpret_cast<const uint4*>(Vtg + slot_major_offset<D>(kap, mt, lane));
            __builtin_amdgcn_wave_barrier();

            for (int s0 = 0; s0 < cnt; s0 += 16) {
                const bool valid = s0 + m16 < cnt;
                const int row = rl[valid ? s0 + m16 : 0];
                Frag qb[C::KS];
#pragma unroll
                for (int ks = 0; ks < C::KS; ++ks)
                    qb[ks].q = *reinterpret_cast<const uint4*>(Qs + (size_t)row * C::QSTRIDE + 16 * g + 64 * ks);
                f32x4_t sc[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    sc[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) sc[mt] = mfma16(ka[mt][ks], qb[ks], sc[mt]);
                }
                const float mr = mref[row];
                float x[8], mx = -INFINITY;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    x[e] = fmaf(sc[e >> 2][e & 3], c2, -mr);
                    mx = fmaxf(mx, x[e]);
                }
                bool live = valid;
                if (__any(valid && !(mx <= kOverflowLog2))) {       // rare: flag the row, drop it here
                    if (valid && !(mx <= kOverflowLog2)) { bad[row] = 1; live = false; }
                }
                float lp = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) { x[e] = live ? fast_exp2(x[e]) : 0.f; lp += x[e]; }
                Frag pb;
#pragma unroll
                for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
                if (live) atomicAdd(&lsum[row], lp);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    f32x4_t o = mfma16(va[mt], pb, f32x4_t{0.f, 0.f, 0.f, 0.f});
                    if (live) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            atomicAdd(&Os[row * C::OSTRIDE + tile_chan<D>(mt, 4 * g + i)], o[i]);
                    }
                }
            }
        }
        __syncthreads();
    }

    // 4. normalise and write out; flagged rows are recomputed from scratch
    bf16_t* Og = O + (sbase + t0) * D;
    for (int i = tid; i < rows_here * (D / 8); i += C::NT) {
        const int r = i / (D / 8), c = i % (D / 8);
        if (bad[r]) continue;
        const float inv = 1.f / lsum[r];
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = Os[r * C::OSTRIDE + 8 * c + e] * inv;
        Vec8<bf16_t>::store(Og + (int64_t)r * D + 8 * c, v);
        if (c == 0) lse[sbase + t0 + r] = (mref[r] + fast_log2(lsum[r])) * kLn2;
    }
    float* scratch = reinterpret_cast<float*>(mask) + wave * (D + 2 * kWave);
    for (int r = wave; r < rows_here; r += C::NW) {
        if (!bad[r]) continue;
        forward_row_plain<D>(Qg + (int64_t)r * D, Kg, V + sbase * D, idx + (sbase + t0 + r) * k,
                             t0 + r, B, k, scale, scratch, lane, Og + (int64_t)r * D,
                             lse + sbase + t0 + r);
    }
}

template <int D>
static hipError_t fwd_launch(const Dims& s, const void* Q, const void* K, const void* V,
                             const void* Vt, const int32_t* idx, void* O, float* lse, hipStream_t st)
{
    using C = FwdCfg<D>;
    const int ntiles = (s.N + C::TILE - 1) / C::TILE;
    hipError_t e = hipFuncSetAttribute((const void*)forward_mfma_kernel<D>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((forward_mfma_kernel<D>), dim3((unsigned)(ntiles * s.bh)), dim3(C::NT), C::LDS,
                       st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)Vt,
                       idx, (bf16_t*)O, lse, s.N, s.B, s.k, s.scale, ntiles, s.bh);
    return hipGetLastError();
}

hipError_t launch_forward_mfma(const Dims& s, const void* Q, const void* K, const void* V,
                               void* Vt, const int32_t* idx, void* O, float* lse, hipStream_t st)
{
    hipError_t e = launch_slot_major_copy(s, V, Vt, st);
    if (e != hipSuccess) return e;
    return s.D == 64 ? fwd_launch<64>(s, Q, K, V, Vt, idx, O, lse, st)
                     : fwd_launch<128>(s, Q, K, V, Vt, idx, O, lse, st);
}

}  // namespace moba
