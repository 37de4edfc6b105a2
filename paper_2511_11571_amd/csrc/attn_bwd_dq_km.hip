// dQ of the MoBA backward, key-block major, for sparse routing (paper Section 4.2 backward and
// Appendix C.3: key blocks outermost, the queries routed to a block gathered into dense tiles,
// S recomputed, dS = P o (dP - D), dQ += scale dS K).  The companion of attn_fwd_km.hip: a
// workgroup owns up to 128 (d = 64) or 64 (d = 128) keys of one key block -- their MFMA operands
// stay on chip for the whole walk, K and V in LDS and K^T in registers -- and walks the block's
// query list, then the block's own queries (causally masked), 32 queries per step and wave.
//
// The paper's kernel adds each block's contribution to dQ with atomic additions into a
// high-precision buffer.  Here the contribution of (query t, kept block e, part c) is written
// once, as bf16, to [t][e][c], and a second kernel adds a query's contributions up in fp32 in a
// fixed order: no atomics, bit-reproducible, and the partial sums stream.
//
// Per 16-query tile (queries are the columns of every product, so a lane owns one query):
//   S^T  = K Q_g^T, dP^T = V dO_g^T - D      keys x queries; -D is the start value of the sum
//   dS^T = 2^(c S^T - lse) o dP^T            in the result layout, which packed to bf16 is the
//                                            B operand over the keys (slot order of mfma.h)
//   dQ^T += K^T dS^T                         channels x queries
#include <type_traits>

#include "mfma.h"

namespace moba {

typedef uint32_t dqvec4_t __attribute__((ext_vector_type(4)));

template <int D>
struct DqKmCfg {
    static constexpr int NW = 4;
    static constexpr int NT = NW * kWave;
    static constexpr int SB = D * 2 + 16;              // bytes per parked row: the row, then (t, e)
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row = lanes per gathered row
    static constexpr int RPI = kWave / CPR;            // rows per gather instruction
    static constexpr int NI = 32 / RPI;                // gather instructions per tensor and step
    static constexpr size_t WAVE = (size_t)2 * 32 * SB + 256;       // Q rows, dO rows, lse and -D
    static constexpr size_t PARK = NW * WAVE;
    static constexpr size_t lds(int ng) { return PARK + (size_t)2 * ng * 64 * D; }   // + the part's K and V
};

// NG: 32-key groups per workgroup
template <int D, int NG>
__global__ __launch_bounds__(DqKmCfg<D>::NT) void dq_km_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ dO, const bf16_t* __restrict__ K,
    const bf16_t* __restrict__ V, const bf16_t* __restrict__ Kt, const float2* __restrict__ ld,
    const int32_t* __restrict__ off,
    const int32_t* __restrict__ ql, bf16_t* __restrict__ PdQ, int N, int B, int n, int k, int nsub,
    float scale, int64_t R, int bh, int G)
{
    using C = DqKmCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    unsigned char* stQ = smem + (size_t)wave * C::WAVE;
    unsigned char* stG = stQ + 32 * C::SB;
    float* ls = reinterpret_cast<float*>(stG + 32 * C::SB);
    float* Ds = ls + 32;
    unsigned char* sK = smem + C::PARK;
    unsigned char* sV = sK + NG * 64 * D;

    int s, u;                                               // slice, (key block, part)
    if (!schedule(blockIdx.x, bh, n * nsub, s, u)) return;
    const int j = u / nsub, c = u - j * nsub;
    const int own_first = c * (32 * NG);                    // first key of the part inside the block
    const int64_t sbase = (int64_t)s * N;
    const int64_t kvbase = (int64_t)(s / G) * N;            // G query heads share a key/value head
    const float c2 = scale * kLog2e;
    const int32_t* os = off + (int64_t)s * (n + 1);
    const int32_t* qs = ql + (int64_t)s * R;
    const int lo = os[j], nlist = os[j + 1] - lo;
    const int own0 = j * B + own_first;                     // own queries that see keys of this part
    const int total = nlist + (B - own_first);
    const char* Qg = reinterpret_cast<const char*>(Q + sbase * D);
    const char* Gg = reinterpret_cast<const char*>(dO + sbase * D);
    const float2* ldq = ld + sbase;                         // per query (lse log2 e, -D)
    const uint32_t vlane = (uint32_t)lane * 16u;

    // The part's K and V rows go to LDS in MFMA operand order -- the 16 bytes lane (m, g) feeds as
    // rows 16 mt + m, channels 32 ks + 8 g .. + 8 of 32-key group gi sit at
    // ((gi * 2 + mt) * KS + ks) * 1024 + 16 * lane -- and are read from there in every step; K^T
    // (slot order) stays in registers for the whole walk.  (All three in registers would leave
    // room for one wave per SIMD only, and the walk needs a second one to fill the waits of the
    // first.)
    {
        const char* Kg = reinterpret_cast<const char*>(K + (kvbase + own0) * D);
        const char* Vg = reinterpret_cast<const char*>(V + (kvbase + own0) * D);
        for (int ch = tid; ch < NG * 32 * C::CPR; ch += C::NT) {
            const int row = ch / C::CPR, col = ch % C::CPR;             // key of the part, 16-byte piece
            const int gi = row >> 5, mt = (row >> 4) & 1, m = row & 15, ks = col >> 2, gg = col & 3;
            const int o = ((gi * 2 + mt) * C::KS + ks) * 1024 + (16 * gg + m) * 16;
            *reinterpret_cast<dqvec4_t*>(sK + o) = *reinterpret_cast<const dqvec4_t*>(Kg + (size_t)ch * 16);
            *reinterpret_cast<dqvec4_t*>(sV + o) = *reinterpret_cast<const dqvec4_t*>(Vg + (size_t)ch * 16);
        }
    }
    Frag kt[NG][C::MT];
    {
        const char* Ktg = reinterpret_cast<const char*>(Kt + (kvbase + own0) * D);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt)
                kt[gi][mt].q = *reinterpret_cast<const uint4*>(Ktg + gi * (64 * D) + vlane + mt * 1024);
    }
    __syncthreads();

    // every load of the walk is unconditional and from an address that is always valid (a load
    // inside a branch is waited for at the end of the branch)
    const int32_t* lsrc = nlist > 0 ? qs + lo : os;
    const int llast = max(nlist - 1, 0);
    // position a of the walk -> list entry (query, e: the place of this block in the query's row
    // of kept blocks, filed in the entry's high byte by the list builder); own rows and rows past
    // the end: e = k
    const int own_e = k << 24;
    auto query_at = [&](int a) {
        const int listed = lsrc[min(a, llast)];
        const int t = a < nlist ? listed : (own0 + (a - nlist)) | own_e;
        return a >= total ? own0 | own_e : t;
    };
    const int grow = lane / C::CPR, lcol = lane % C::CPR;
    const uint32_t gcol = (uint32_t)lcol * 16u;
    // t: the entries of the rows this lane gathers a piece of; tl: the row whose lse and D lane
    // (lane & 31) brings
    auto ids = [&](int a0, int (&t)[C::NI], int& tl) {
#pragma unroll
        for (int i = 0; i < C::NI; ++i) t[i] = query_at(a0 + C::RPI * i + grow);
        tl = list_query(query_at(a0 + (lane & 31)));
    };
    // one step's loads: the pieces of the Q and dO rows, lse in log2 units (+inf past the end:
    // P = 0) and -D
    auto fetch = [&](int a0, const int (&t)[C::NI], int tl, dqvec4_t (&qr)[C::NI], dqvec4_t (&gr)[C::NI],
                     float& lv, float& dv) {
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            const uint32_t o = (uint32_t)list_query(t[i]) * (uint32_t)(2 * D) + gcol;
            qr[i] = *reinterpret_cast<const dqvec4_t*>(Qg + o);
            gr[i] = *reinterpret_cast<const dqvec4_t*>(Gg + o);
        }
        const float2 x = ldq[tl];
        lv = a0 + (lane & 31) < total ? x.x : INFINITY;
        dv = x.y;
    };
    // The rows of the next step are in flight while one step is worked on; the row ids of the
    // step after that (tN, tlN) are loaded before that gather, so that waiting for them (loads
    // complete in order) leaves the gather in flight.
    const int stride = 32 * C::NW;
    int t0[C::NI], tN[C::NI], tl0, tlN;
    dqvec4_t qr0[C::NI], gr0[C::NI];
    float lv0, dv0;
    ids(32 * wave, t0, tl0);
    ids(32 * wave + stride, tN, tlN);
    fetch(32 * wave, t0, tl0, qr0, gr0, lv0, dv0);
    const uint32_t park = (uint32_t)grow * C::SB + gcol;
    const uint32_t arow = (uint32_t)m16 * C::SB + 16u * g;
    const int64_t slots = (int64_t)(k + 1) * nsub;          // partials per query

    auto step = [&](int a0, int (&tA)[C::NI], int& tlA, dqvec4_t (&qr)[C::NI], dqvec4_t (&gr)[C::NI],
                    float& lv, float& dv) {
        // park the gathered rows, the list entry (t, e) behind each Q row
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            *reinterpret_cast<dqvec4_t*>(stQ + park + i * C::RPI * C::SB) = qr[i];
            *reinterpret_cast<dqvec4_t*>(stG + park + i * C::RPI * C::SB) = gr[i];
            if (lcol == 0) *reinterpret_cast<int*>(stQ + (grow + i * C::RPI) * C::SB + 2 * D) = tA[i];
        }
        if (lane < 32) { ls[lane] = lv; Ds[lane] = dv; }
#pragma unroll
        for (int i = 0; i < C::NI; ++i) tA[i] = tN[i];
        tlA = tlN;
        ids(a0 + 2 * stride, tN, tlN);
        fetch(a0 + stride, tA, tlA, qr, gr, lv, dv);
        __builtin_amdgcn_wave_barrier();
        const bool masked = a0 + 32 > nlist;                       // the step holds own rows
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            Frag qb[C::KS], gb[C::KS];
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks) {
                qb[ks].q = *reinterpret_cast<const uint4*>(stQ + arow + qt * 16 * C::SB + 64 * ks);
                gb[ks].q = *reinterpret_cast<const uint4*>(stG + arow + qt * 16 * C::SB + 64 * ks);
            }
            const int te = *reinterpret_cast<const int*>(stQ + (16 * qt + m16) * C::SB + 2 * D);
            const float lq = ls[16 * qt + m16], nd = Ds[16 * qt + m16];
            const int av = a0 + 16 * qt + m16;                     // this lane's row of the walk
            const int r = av - nlist;                              // own row r sees keys 0 .. r of the part
            f32x4_t o[C::MT];
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) o[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                // x[4 mt + i]: dS of key 32 gi + 16 mt + 4 g + i of the part
                float x[8];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f}, dp = f32x4_t{nd, nd, nd, nd};
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) {
                        Frag ka, va;
                        const int o = ((gi * 2 + mt) * C::KS + ks) * 1024 + vlane;
                        ka.q = *reinterpret_cast<const uint4*>(sK + o);
                        va.q = *reinterpret_cast<const uint4*>(sV + o);
                        sc = mfma16(ka, qb[ks], sc);
                        dp = mfma16(va, gb[ks], dp);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float p = fast_exp2(fmaf(sc[i], c2, -lq));
                        if (masked && r >= 0 && 32 * gi + 16 * mt + 4 * g + i > r) p = 0.f;
                        x[4 * mt + i] = p * dp[i];
                    }
                }
                Frag pb;
#pragma unroll
                for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[2 * e], x[2 * e + 1]);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) o[mt] = mfma16(kt[gi][mt], pb, o[mt]);
            }
            // the partial: this lane holds D/4 consecutive channels of the row
            if (av < total) {
                // clamped: lists that do not match the rows of kept blocks give a wrong result,
                // never an address outside the partials
                const int e = min(list_slot(te), k);
                const int64_t prow = (sbase + min(list_query(te), N - 1)) * slots + (int64_t)e * nsub + c;
                uint32_t w[C::MT * 2];
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    w[2 * mt] = pack_bf16x2(o[mt][0] * scale, o[mt][1] * scale);
                    w[2 * mt + 1] = pack_bf16x2(o[mt][2] * scale, o[mt][3] * scale);
                }
                uint4* dst = reinterpret_cast<uint4*>(PdQ + prow * D + g * (D / 4));
#pragma unroll
                for (int q4 = 0; q4 < C::MT / 2; ++q4)
                    dst[q4] = make_uint4(w[4 * q4], w[4 * q4 + 1], w[4 * q4 + 2], w[4 * q4 + 3]);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    for (int a0 = 32 * wave; a0 < total; a0 += stride) step(a0, t0, tl0, qr0, gr0, lv0, dv0);
}

// dQ_t = sum of the query's partials, in the order [kept block][part], then the parts of its
// own block up to its own key.  D / 8 lanes per query; the partials of a query are consecutive
// and are loaded nine at a time, unconditionally (past the end: the last one again, ignored).
constexpr int kDqMergeChunk = 9;

template <int D>
__global__ __launch_bounds__(256) void dq_km_merge_kernel(
    const int32_t* __restrict__ idx, const bf16_t* __restrict__ PdQ, bf16_t* __restrict__ dQ, int N,
    int B, int k, int nsub, int64_t rows_total)
{
    constexpr int G = D / 8, CH = kDqMergeChunk;
    const int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;      // s * N + t
    const int part = threadIdx.x % G;
    if (row >= rows_total) return;
    const int t = (int)(row % N);
    const int own_parts = (t % B) / km_part_keys(B, D) + 1;
    const int slots = (k + 1) * nsub, klast = max(k - 1, 0);
    const int64_t p0 = row * slots;
    const char* orow = reinterpret_cast<const char*>(PdQ + p0 * D + part * 8);
    // (with k = 0 there is no row of kept blocks: any readable address serves the unused loads)
    const int32_t* irow = k > 0 ? idx + row * k : reinterpret_cast<const int32_t*>(orow);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0, e0 = 0, c0 = 0; i0 < slots; i0 += CH) {
        int jj[CH];
        dqvec4_t raw[CH];
#pragma unroll
        for (int i = 0, e = e0, c = c0; i < CH; ++i) {
            jj[i] = irow[min(e, klast)];
            raw[i] = *reinterpret_cast<const dqvec4_t*>(orow + (int64_t)min(i0 + i, slots - 1) * (2 * D));
            if (++c == nsub) { c = 0; ++e; }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            // the partial counts if it exists and its block was kept (own block: the parts up to
            // the query's own key); an unused slot holds whatever the workspace held
            const bool ok = i0 + i < slots && (e0 == k ? c0 < own_parts : jj[i] >= 0);
            if (++c0 == nsub) { c0 = 0; ++e0; }
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const float lo = __uint_as_float(raw[i][h] << 16), hi = __uint_as_float(raw[i][h] & 0xffff0000u);
                acc[2 * h] += ok ? lo : 0.f;
                acc[2 * h + 1] += ok ? hi : 0.f;
            }
        }
    }
    Vec8<bf16_t>::store(dQ + row * D + part * 8, acc);
}

// ---- workspace: [D: bh*N fp32][slot-ordered K][partial dQ: bh*N*(k+1)*parts*D bf16], each
// 256-byte aligned

size_t backward_km_ws_bytes(const Dims& s)
{
    const size_t tensor = a256(sizeof(bf16_t) * (size_t)s.bhk * s.N * s.D);
    return a256(sizeof(float) * (size_t)s.bh * s.N) + tensor + a256(sizeof(bf16_t) * km_partials(s) * s.D);
}

template <int D, int NG>
static hipError_t dq_launch2(const Dims& s, const void* Q, const void* dO, const void* K, const void* V,
                             const void* Kt, const float2* ld, const int32_t* idx,
                             const int32_t* off, const int32_t* ql, bf16_t* PdQ, void* dQ, hipStream_t st)
{
    using C = DqKmCfg<D>;
    const int nsub = s.B / km_part_keys(s.B, s.D);
    hipError_t e = ensure_dynamic_lds((const void*)dq_km_kernel<D, NG>, C::lds(NG));
    if (e != hipSuccess) return e;
    {
        ProfileScope timing(MOBA_PROFILE_DQ, st);
        const int bhs = slice_major(s, 2) * s.bh;           // (gathers Q and dO rows)
        hipLaunchKernelGGL((dq_km_kernel<D, NG>), dim3((unsigned)schedule_grid(bhs, s.n * nsub)),
                           dim3(C::NT), C::lds(NG), st, (const bf16_t*)Q, (const bf16_t*)dO, (const bf16_t*)K,
                           (const bf16_t*)V, (const bf16_t*)Kt, ld, off, ql, PdQ, s.N, s.B, s.n,
                           s.k, nsub, s.scale, s.R, bhs, s.G);
    }
    const int64_t rows = (int64_t)s.bh * s.N;
    const int rpw = 256 / (D / 8);
    hipLaunchKernelGGL((dq_km_merge_kernel<D>), dim3((unsigned)((rows + rpw - 1) / rpw)), dim3(256), 0, st,
                       idx, PdQ, (bf16_t*)dQ, s.N, s.B, s.k, nsub, rows);
    return hipGetLastError();
}

template <int D, typename... A>
static hipError_t dq_launch(const Dims& s, A... a)
{
    switch (km_part_keys(s.B, D) / 32) {
        case 1: return dq_launch2<D, 1>(s, a...);
        case 2: return dq_launch2<D, 2>(s, a...);
        case 3: if constexpr (D == 64) return dq_launch2<D, 3>(s, a...); else break;
        case 4: if constexpr (D == 64) return dq_launch2<D, 4>(s, a...); else break;
    }
    return hipErrorInvalidValue;
}

hipError_t launch_dq_km(const Dims& s, const void* Q, const void* K, const void* V, const void* dO,
                        const float2* ld, const int32_t* idx, const int32_t* off, const int32_t* ql,
                        void* dQ, void* ws, hipStream_t st)
{
    if (s.bh == 0 || s.N == 0) return hipSuccess;
    if (!key_major_shape(s)) return hipErrorInvalidValue;
    const size_t tensor = a256(sizeof(bf16_t) * (size_t)s.bhk * s.N * s.D);
    char* p = static_cast<char*>(ws);
    p += a256(sizeof(float) * (size_t)s.bh * s.N);         // D (not read here)
    void* Kt = p;
    p += tensor;
    bf16_t* PdQ = reinterpret_cast<bf16_t*>(p);
    hipError_t e = launch_slot_major_copy(kv_view(s), K, Kt, nullptr, st);
    if (e != hipSuccess) return e;
    return s.D == 64 ? dq_launch<64>(s, Q, dO, K, V, Kt, ld, idx, off, ql, PdQ, dQ, st)
                     : dq_launch<128>(s, Q, dO, K, V, Kt, ld, idx, off, ql, PdQ, dQ, st);
}

}  // namespace moba
