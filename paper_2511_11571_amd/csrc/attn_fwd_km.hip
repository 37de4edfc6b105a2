// MoBA forward, key-block major, for sparse routing (paper Section 4.2, forward pass with
// gather-and-densify: one logical key block at a time, the queries routed to it gathered into
// dense tiles).  The query-tile kernel of attn_fwd_mfma.hip needs a 256-query tile to meet a key
// block with many of its rows; with few kept blocks out of very many (long sequences) a tile
// meets a block with one or two rows and the work per (query, block) pair explodes.  Here a
// workgroup owns up to 128 (d = 64) or 64 (d = 128) keys of one key block -- their MFMA operands
// stay on chip for the whole walk, K in LDS and V^T in registers (d = 128: in LDS) -- and walks the list of ALL
// queries that kept the block (then the block's own queries, causally masked), 32 queries per
// step and wave: the tiles are dense whatever the sequence length, and nothing but the gathered
// query rows and their rows of kept blocks is read in the loop.
//
// A query's softmax spans several key blocks, i.e. several workgroups.  As in the paper's
// forward each (query, block) pair therefore produces a partial result -- the local softmax
// reference m, the sum l of exp(s - m), and sum p v / l rounded to bf16 -- and a second kernel
// merges a query's partials (Section 4.2: the partial outputs are combined with the
// log-sum-exp weights).  The partials of query t lie together, [t][e][c] for its e-th kept
// block (e = k: own block) and part c of the block's keys, so the merge streams them; e comes with
// the query in the block's list (the list builder files it in the entry's high byte).  No atomics anywhere; results are
// bit-reproducible.
#include <type_traits>

#include "mfma.h"

namespace moba {

typedef uint32_t kmvec4_t __attribute__((ext_vector_type(4)));

template <int D>
struct KmCfg {
    static constexpr int NW = 4;
    static constexpr int NT = NW * kWave;
    static constexpr int SB = D * 2 + 16;              // bytes per parked row: the row, then (t, e)
    static constexpr int MT = D / 16;
    static constexpr int KS = D / 32;
    static constexpr int CPR = D / 8;                  // 16-byte chunks per row = lanes per gathered row
    static constexpr int RPI = kWave / CPR;            // rows per gather instruction
    static constexpr int NI = 32 / RPI;                // gather instructions per step
    static constexpr size_t PARK = (size_t)NW * 32 * SB;                 // the waves' parked rows
    // d = 128: V^T goes to LDS as well -- in registers it leaves room for one wave per SIMD only
    static constexpr bool VLDS = D == 128;
    static constexpr size_t lds(int ng) { return PARK + (size_t)(VLDS ? 2 : 1) * ng * 64 * D; }   // + the part's keys (and values)
};

// NG: 32-key groups per workgroup
template <int D, int NG>
__global__ __launch_bounds__(KmCfg<D>::NT) __attribute__((amdgpu_waves_per_eu(D == 128 ? 2 : 1)))
void fwd_km_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ Vt,
    const int32_t* __restrict__ off, const int32_t* __restrict__ ql,
    bf16_t* __restrict__ PO, float* __restrict__ Pml, int N, int B, int n, int k, int nsub,
    float scale, int64_t R, int bh, int G)
{
    using C = KmCfg<D>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int m16 = lane & 15, g = lane >> 4;
    unsigned char* stQ = smem + (size_t)wave * 32 * C::SB;
    unsigned char* sK = smem + C::PARK;

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
    const uint32_t vlane = (uint32_t)lane * 16u;

    // The part's keys go to LDS in MFMA operand order -- the 16 bytes lane (m, g) feeds as rows
    // 16 mt + m, channels 32 ks + 8 g .. + 8 of 32-key group gi sit at
    // ((gi * 2 + mt) * KS + ks) * 1024 + 16 * lane -- and are read from there in every step; the
    // values (transposed, slot order) stay in registers for the whole walk.  (Keys in registers
    // as well would leave room for one wave per SIMD only, and the walk needs a second one to
    // fill the waits of the first.)
    {
        const char* Kg = reinterpret_cast<const char*>(K + (kvbase + own0) * D);
        for (int ch = tid; ch < NG * 32 * C::CPR; ch += C::NT) {
            const int row = ch / C::CPR, col = ch % C::CPR;             // key of the part, 16-byte piece
            const int gi = row >> 5, mt = (row >> 4) & 1, m = row & 15, ks = col >> 2, gg = col & 3;
            *reinterpret_cast<kmvec4_t*>(sK + ((gi * 2 + mt) * C::KS + ks) * 1024 + (16 * gg + m) * 16) =
                *reinterpret_cast<const kmvec4_t*>(Kg + (size_t)ch * 16);
        }
    }
    Frag va[C::VLDS ? 1 : NG][C::MT];
    unsigned char* sV = sK + (size_t)NG * 64 * D;
    {
        const char* Vtg = reinterpret_cast<const char*>(Vt + (kvbase + own0) * D);
        if constexpr (C::VLDS) {
            for (int ch = tid; ch < NG * 4 * D; ch += C::NT)          // NG * 64 * D bytes, as they are
                *reinterpret_cast<kmvec4_t*>(sV + (size_t)ch * 16) =
                    *reinterpret_cast<const kmvec4_t*>(Vtg + (size_t)ch * 16);
        } else {
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt)
                    va[gi][mt].q = *reinterpret_cast<const uint4*>(Vtg + gi * (64 * D) + vlane + mt * 1024);
        }
    }
    __syncthreads();

    // every load of the walk is unconditional and from an address that is always valid (a load
    // inside a branch is waited for at the end of the branch)
    const int32_t* lsrc = nlist > 0 ? qs + lo : os;
    const int llast = max(nlist - 1, 0);
    // position a of the walk -> list entry (query, e); own rows and rows past the end: e = k
    const int own_e = k << 24;
    auto query_at = [&](int a) {
        const int listed = lsrc[min(a, llast)];
        const int t = a < nlist ? listed : (own0 + (a - nlist)) | own_e;
        return a >= total ? own0 | own_e : t;
    };
    const int grow = lane / C::CPR, lcol = lane % C::CPR;
    const uint32_t gcol = (uint32_t)lcol * 16u;
    auto ids = [&](int a0, int (&t)[C::NI]) {
#pragma unroll
        for (int i = 0; i < C::NI; ++i) t[i] = query_at(a0 + C::RPI * i + grow);
    };
    auto fetch = [&](const int (&t)[C::NI], kmvec4_t (&qr)[C::NI]) {
#pragma unroll
        for (int i = 0; i < C::NI; ++i)
            qr[i] = *reinterpret_cast<const kmvec4_t*>(Qg + (uint32_t)list_query(t[i]) * (uint32_t)(2 * D) + gcol);
    };
    // Two steps of gathered rows are in flight while a third is worked on: t (the list entries)
    // and qr (the rows' 16-byte pieces) of step i sit in buffer i % 2, the entries of step i + 2
    // in tN.  The loads for tN go out before the gather of the step before it, so
    // that waiting for them (loads complete in order) leaves that gather in flight.
    const int stride = 32 * C::NW;
    int t0[C::NI], t1[C::NI], tN[C::NI];
    kmvec4_t qr0[C::NI], qr1[C::NI];
    ids(32 * wave, t0);
    ids(32 * wave + stride, t1);
    ids(32 * wave + 2 * stride, tN);
    fetch(t0, qr0);
    fetch(t1, qr1);
    const uint32_t park = (uint32_t)grow * C::SB + gcol;
    const uint32_t arow = (uint32_t)m16 * C::SB + 16u * g;
    const int64_t slots = (int64_t)(k + 1) * nsub;          // partials per query

    auto step = [&](int a0, int (&tA)[C::NI], kmvec4_t (&qr)[C::NI]) {
        // park the gathered rows, the list entry (t, e) behind each
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            *reinterpret_cast<kmvec4_t*>(stQ + park + i * C::RPI * C::SB) = qr[i];
            if (lcol == 0) *reinterpret_cast<int*>(stQ + (grow + i * C::RPI) * C::SB + 2 * D) = tA[i];
        }
#pragma unroll
        for (int i = 0; i < C::NI; ++i) tA[i] = tN[i];
        ids(a0 + 3 * stride, tN);
        fetch(tA, qr);
        __builtin_amdgcn_wave_barrier();
        const bool masked = a0 + 32 > nlist;                       // the step holds own rows
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            Frag qb[C::KS];
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
                qb[ks].q = *reinterpret_cast<const uint4*>(stQ + arow + qt * 16 * C::SB + 64 * ks);
            const int av = a0 + 16 * qt + m16;                     // this lane's row of the walk
            // raw scores of the row against the part's keys: x[gi][4 mt + i] is key
            // 32 gi + 16 mt + 4 g + i of the part
            float x[NG][8];
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < C::KS; ++ks) {
                        Frag ka;
                        ka.q = *reinterpret_cast<const uint4*>(sK + ((gi * 2 + mt) * C::KS + ks) * 1024 + vlane);
                        sc = mfma16(ka, qb[ks], sc);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[gi][4 * mt + i] = sc[i];
                }
            if (masked) {                                          // own row r sees keys 0 .. r of the part
                const int r = av - nlist;
#pragma unroll
                for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (r >= 0 && 32 * gi + 16 * (e >> 2) + 4 * g + (e & 3) > r) x[gi][e] = -INFINITY;
            }
            float mref = -INFINITY;
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                for (int e = 0; e < 8; ++e) mref = fmaxf(mref, x[gi][e]);
            mref = fmaxf(mref, __shfl_xor(mref, 16, kWave));
            mref = fmaxf(mref, __shfl_xor(mref, 32, kWave));
            mref *= c2;                                            // c2 > 0: the maximum commutes
            if (av >= total) mref = 0.f;                           // no such row: keep the arithmetic finite
            f32x4_t o[C::MT];
#pragma unroll
            for (int mt = 0; mt < C::MT; ++mt) o[mt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            float l = 0.f;
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    x[gi][e] = fast_exp2(fmaf(x[gi][e], c2, -mref));
                    l += x[gi][e];
                }
                Frag pb;
#pragma unroll
                for (int e = 0; e < 4; ++e) pb.u[e] = pack2(x[gi][2 * e], x[gi][2 * e + 1]);
#pragma unroll
                for (int mt = 0; mt < C::MT; ++mt) {
                    if constexpr (C::VLDS)
                        va[0][mt].q = *reinterpret_cast<const uint4*>(sV + gi * (64 * D) + vlane + mt * 1024);
                    o[mt] = mfma16(va[C::VLDS ? 0 : gi][mt], pb, o[mt]);
                }
            }
            l += __shfl_xor(l, 16, kWave);
            l += __shfl_xor(l, 32, kWave);
            // The partial: this lane holds D/4 consecutive channels of the row.  It goes back over
            // the row's parked bytes (the Q operands of these 16 rows are in registers by now),
            // (m, l) behind (t, e), and is then written out by whole rows -- CPR neighbouring
            // lanes store one row's 2 D consecutive bytes, so every line of the partials is
            // written by one instruction.
            {
                const float inv = 1.f / l;
                unsigned char* prk = stQ + (16 * qt + m16) * C::SB;
#pragma unroll
                for (int q4 = 0; q4 < C::MT / 2; ++q4) {
                    kmvec4_t w;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        w[2 * h] = pack_bf16x2(o[2 * q4 + h][0] * inv, o[2 * q4 + h][1] * inv);
                        w[2 * h + 1] = pack_bf16x2(o[2 * q4 + h][2] * inv, o[2 * q4 + h][3] * inv);
                    }
                    *reinterpret_cast<kmvec4_t*>(prk + g * (D / 2) + 16 * q4) = w;
                }
                if (g == 0) *reinterpret_cast<float2*>(prk + 2 * D + 8) = make_float2(mref, l);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int h = 0; h < 16 / C::RPI; ++h) {
                const int r = 16 * qt + C::RPI * h + grow;          // parked row of this lane
                const unsigned char* prk = stQ + r * C::SB;
                const kmvec4_t v = *reinterpret_cast<const kmvec4_t*>(prk + gcol);
                const int note = *reinterpret_cast<const int*>(prk + 2 * D);       // (t, e)
                if (a0 + r < total) {
                    // clamped: lists that do not match the rows of kept blocks give a wrong result,
                    // never an address outside the partials
                    const int e = min(list_slot(note), k);
                    const int64_t prow = (sbase + min(list_query(note), N - 1)) * slots + (int64_t)e * nsub + c;
                    kmvec4_t* dst = reinterpret_cast<kmvec4_t*>(reinterpret_cast<char*>(PO + prow * D) + gcol);
                    // d = 128: streaming stores -- the partials are read again only by the merge
                    // kernel, and not keeping their two lines per row in L2 measured -17 % there
                    // (d = 64: no difference)
                    if constexpr (D == 128) __builtin_nontemporal_store(v, dst);
                    else *dst = v;
                }
            }
        }
        // (m, l) of the step's 32 rows in one store instruction, a lane per row
        if (lane < 32 && a0 + lane < total) {
            const int4 note = *reinterpret_cast<const int4*>(stQ + lane * C::SB + 2 * D);    // (t, e), -, m, l
            const int e = min(list_slot(note.x), k);
            const int64_t prow = (sbase + min(list_query(note.x), N - 1)) * slots + (int64_t)e * nsub + c;
            float* pm = Pml + prow * 2;
            if constexpr (D == 128) {
                __builtin_nontemporal_store(__int_as_float(note.z), pm);
                __builtin_nontemporal_store(__int_as_float(note.w), pm + 1);
            } else {
                *reinterpret_cast<float2*>(pm) = make_float2(__int_as_float(note.z), __int_as_float(note.w));
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    for (int a0 = 32 * wave; a0 < total; a0 += 2 * stride) {
        step(a0, t0, qr0);
        if (a0 + stride >= total) break;
        step(a0 + stride, t1, qr1);
    }
}

// O_t = sum w O_p, w = l_p 2^(m_p - M) / L over the query's partials: all parts of its kept
// blocks, and the parts of its own block up to its own key; lse_t = (M + log2 L) ln 2.
// D / 8 lanes per query.  A query's partials are consecutive in memory; they are loaded nine at a
// time, every load unconditional (past the end: the last one again, ignored), so that a lane has
// up to nine independent 16-byte loads in flight.
constexpr int kMergeChunk = 9;

__device__ __forceinline__ void unpack_bf16x8(const kmvec4_t& r, float (&v)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(r[i] << 16);
        v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
}

template <int D>
__global__ __launch_bounds__(256) void fwd_km_merge_kernel(
    const int32_t* __restrict__ idx, const bf16_t* __restrict__ PO, const float* __restrict__ Pml,
    bf16_t* __restrict__ O, float* __restrict__ lse, int N, int B, int k, int nsub, int64_t rows_total)
{
    constexpr int G = D / 8, CH = kMergeChunk;
    const int64_t row = (int64_t)blockIdx.x * (256 / G) + threadIdx.x / G;      // s * N + t
    const int part = threadIdx.x % G;
    if (row >= rows_total) return;
    const int t = (int)(row % N);
    const int own_parts = (t % B) / km_part_keys(B, D) + 1;
    const int slots = (k + 1) * nsub, klast = max(k - 1, 0);
    const int64_t p0 = row * slots;
    // (with k = 0 there is no row of kept blocks: any readable address serves the unused loads)
    const int32_t* irow = k > 0 ? idx + row * k : reinterpret_cast<const int32_t*>(Pml + p0 * 2);
    const float2* mlrow = reinterpret_cast<const float2*>(Pml) + p0;
    const char* orow = reinterpret_cast<const char*>(PO + p0 * D + part * 8);
    // slot i0 + i is partial (e, c); it counts if it exists and its block was kept (own block:
    // the parts up to the query's own key)
    auto counts = [&](int si, int e, int c, int j) { return si < slots && (e == k ? c < own_parts : j >= 0); };
    float M = -INFINITY;
    for (int i0 = 0, e0 = 0, c0 = 0; i0 < slots; i0 += CH) {
        float m[CH];
        int jj[CH];
#pragma unroll
        for (int i = 0, e = e0, c = c0; i < CH; ++i) {
            jj[i] = irow[min(e, klast)];
            m[i] = mlrow[min(i0 + i, slots - 1)].x;
            if (++c == nsub) { c = 0; ++e; }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (counts(i0 + i, e0, c0, jj[i])) M = fmaxf(M, m[i]);
            if (++c0 == nsub) { c0 = 0; ++e0; }
        }
    }
    float L = 0.f, acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0, e0 = 0, c0 = 0; i0 < slots; i0 += CH) {
        float2 ml[CH];
        int jj[CH];
        kmvec4_t raw[CH];
#pragma unroll
        for (int i = 0, e = e0, c = c0; i < CH; ++i) {
            const int si = min(i0 + i, slots - 1);
            jj[i] = irow[min(e, klast)];
            ml[i] = mlrow[si];
            raw[i] = *reinterpret_cast<const kmvec4_t*>(orow + (int64_t)si * (2 * D));
            if (++c == nsub) { c = 0; ++e; }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool ok = counts(i0 + i, e0, c0, jj[i]);
            if (++c0 == nsub) { c0 = 0; ++e0; }
            // (an unused slot holds whatever the workspace held: select, do not multiply by 0)
            const float wgt = ok ? ml[i].y * fast_exp2(ml[i].x - M) : 0.f;
            float v[8];
            unpack_bf16x8(raw[i], v);
            L += wgt;
#pragma unroll
            for (int ch = 0; ch < 8; ++ch) acc[ch] = fmaf(wgt, ok ? v[ch] : 0.f, acc[ch]);
        }
    }
    const float inv = 1.f / L;
#pragma unroll
    for (int ch = 0; ch < 8; ++ch) acc[ch] *= inv;
    Vec8<bf16_t>::store(O + row * D + part * 8, acc);
    if (part == 0) lse[row] = (M + fast_log2(L)) * kLn2;
}

// ---- workspace: [slot-ordered V][partial O: bh*N*(k+1)*parts*D bf16][partial (m, l):
// bh*N*(k+1)*parts*2 fp32], each 256-byte aligned

size_t forward_km_ws_bytes(const Dims& s)
{
    const size_t tensor = a256(sizeof(bf16_t) * (size_t)s.bhk * s.N * s.D);
    return tensor + a256(sizeof(bf16_t) * km_partials(s) * s.D) + a256(sizeof(float) * km_partials(s) * 2);
}

template <int D, int NG>
static hipError_t km_launch2(const Dims& s, const void* Q, const void* K, const void* Vt,
                             const int32_t* idx, const int32_t* off, const int32_t* ql, bf16_t* PO,
                             float* Pml, void* O, float* lse, hipStream_t st)
{
    using C = KmCfg<D>;
    const int nsub = s.B / km_part_keys(s.B, s.D);
    hipError_t e = ensure_dynamic_lds((const void*)fwd_km_kernel<D, NG>, C::lds(NG));
    if (e != hipSuccess) return e;
    {
        ProfileScope timing(MOBA_PROFILE_FORWARD, st);
        const int bhs = slice_major(s, 1) * s.bh;           // (gathers Q rows)
        hipLaunchKernelGGL((fwd_km_kernel<D, NG>), dim3((unsigned)schedule_grid(bhs, s.n * nsub)),
                           dim3(C::NT), C::lds(NG), st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)Vt,
                           off, ql, PO, Pml, s.N, s.B, s.n, s.k, nsub, s.scale, s.R, bhs, s.G);
    }
    const int64_t rows = (int64_t)s.bh * s.N;
    const int rpw = 256 / (D / 8);
    hipLaunchKernelGGL((fwd_km_merge_kernel<D>), dim3((unsigned)((rows + rpw - 1) / rpw)), dim3(256), 0, st,
                       idx, PO, Pml, (bf16_t*)O, lse, s.N, s.B, s.k, nsub, rows);
    return hipGetLastError();
}

template <int D, typename... A>
static hipError_t km_launch(const Dims& s, A... a)
{
    switch (km_part_keys(s.B, D) / 32) {
        case 1: return km_launch2<D, 1>(s, a...);
        case 2: return km_launch2<D, 2>(s, a...);
        case 3: if constexpr (D == 64) return km_launch2<D, 3>(s, a...); else break;
        case 4: if constexpr (D == 64) return km_launch2<D, 4>(s, a...); else break;
    }
    return hipErrorInvalidValue;
}

hipError_t launch_forward_km(const Dims& s, const void* Q, const void* K, const void* V, void* ws,
                             const int32_t* idx, const int32_t* off, const int32_t* ql, void* O,
                             float* lse, hipStream_t st)
{
    if (s.bh == 0 || s.N == 0) return hipSuccess;
    if (!key_major_shape(s)) return hipErrorInvalidValue;
    const size_t tensor = a256(sizeof(bf16_t) * (size_t)s.bhk * s.N * s.D);
    char* p = static_cast<char*>(ws);
    void* Vt = p;
    p += tensor;
    bf16_t* PO = reinterpret_cast<bf16_t*>(p);
    p += a256(sizeof(bf16_t) * km_partials(s) * s.D);
    float* Pml = reinterpret_cast<float*>(p);
    hipError_t e = launch_slot_major_copy(kv_view(s), V, Vt, nullptr, st);
    if (e != hipSuccess) return e;
    return s.D == 64 ? km_launch<64>(s, Q, K, Vt, idx, off, ql, PO, Pml, O, lse, st)
                     : km_launch<128>(s, Q, K, Vt, idx, off, ql, PO, Pml, O, lse, st);
}

}  // namespace moba
