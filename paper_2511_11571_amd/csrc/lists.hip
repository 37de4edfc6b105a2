// Key-block-major query lists from query-major routing (paper Appendix C.1,
// "Reformatting Indices to Varlen Key-Block-Major").  The paper scatters with global
// atomics, which leaves the order inside a list to chance; here the lists come out
// ascending and bit-reproducible:
//   1. count: a workgroup takes a chunk of 256 consecutive queries and ORs one bit per
//      (query, kept block) into an LDS bit matrix [block][256 bits]; the population
//      count of a row is the number of queries of this chunk that kept that block.
//   2. scan: per key block an exclusive scan over chunks (start of each chunk's segment
//      inside the block's list), then an exclusive scan of the block totals (blk_off).
//   3. fill: the bit matrix is rebuilt and its rows are written out in ascending order at
//      blk_off[j] + chunk start, eight lanes per row.
// The bit matrix lives in LDS only and covers 1024 key blocks at a time (512 where a slice has more).
//
// A list entry holds the query in its low 24 bits (sequences are at most 2^24 long).  Where the
// key-block-major attention kernels will run (key_major_path() of the shape and its flags) the
// high byte holds the position e of the block in the query's row of kept blocks: those kernels
// file the partial result of (query, block) under (query, e) and would otherwise have to search
// the row for the block (10-15 % of their time); elsewhere it is zero.  The fill pass gets e by walking the
// routing rows a second time: entry e of row r names block b, whose place in b's run of this
// workgroup is the number of set bits below r in b's row of the bit matrix.
#include "mfma.h"

namespace moba {

constexpr int kRangeMax = 1024;                 // key blocks per LDS bit matrix at most (32 KB)
constexpr int kRangeLong = 512;                 // ... where a slice has more blocks than that
constexpr int kListQ = kChunkQ;                  // queries per workgroup: one chunk
constexpr int kWords = kListQ / 32;             // 8 words of 32 query bits per block
constexpr int kQueryBits = 24;                  // low bits of a list entry: the query

// f(r, b, e) for every entry b = row r's e-th of the routing rows r = 0 .. rows-1 of this workgroup
// (k entries per row, rows contiguous in memory), all 256 threads, 16-byte loads when the row length
// allows.  The row and place of a thread's entries advance by additions (one division per thread).
template <typename F>
__device__ __forceinline__ void for_each_entry_slot(const int32_t* __restrict__ rows0, int rows, int k,
                                                    int tid, F f)
{
    const int total = rows * k;
    if ((k & 3) == 0) {
        const int4* p4 = reinterpret_cast<const int4*>(rows0);
        const int n4 = total >> 2;
        const int dr = 1024 / k, de = 1024 % k;             // 256 pieces of four entries further on
        int r = 4 * tid / k, e = 4 * tid - r * k;           // a 16-byte piece never straddles rows
        for (int i0 = tid; i0 < n4; i0 += 4 * 256) {
            int4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = i0 + u * 256 < n4 ? p4[i0 + u * 256] : make_int4(-1, -1, -1, -1);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                f(r, v[u].x, e); f(r, v[u].y, e + 1); f(r, v[u].z, e + 2); f(r, v[u].w, e + 3);
                r += dr;
                e += de;
                if (e >= k) { e -= k; ++r; }
            }
        }
    } else {
        const int dr = 256 / k, de = 256 % k;
        int r = tid / k, e = tid - r * k;
        for (int i = tid; i < total; i += 256) {
            f(r, rows0[i], e);
            r += dr;
            e += de;
            if (e >= k) { e -= k; ++r; }
        }
    }
}

// the same without the place: f(r, b)
template <typename F>
__device__ __forceinline__ void for_each_entry(const int32_t* __restrict__ rows0, int rows, int k, int tid, F f)
{
    for_each_entry_slot(rows0, rows, k, tid, [&](int r, int b, int) { f(r, b); });
}

// kRange: key blocks per LDS bit matrix (blockIdx.y counts the ranges of a slice's blocks)
template <bool FILL, bool SLOTS, int kRange>
__global__ __launch_bounds__(256) void lists_chunk_kernel(
    const int32_t* __restrict__ idx, int32_t* __restrict__ cnt2, const int32_t* __restrict__ off,
    int32_t* __restrict__ ql, int N, int B, int n, int k, int nchunk, int64_t R, int bh)
{
    __shared__ __align__(16) uint32_t mask[kRange * kWords];
    __shared__ int32_t start[FILL ? kRange : 1];         // where this workgroup's queries start in each list
    __shared__ uint16_t lbase[SLOTS ? kRange : 1];       // where block b's run starts among this workgroup's entries
    extern __shared__ uint8_t slot[];                    // SLOTS: e of every entry, run by run (kListQ * k bytes)
    __shared__ int wsum[4];
    const int slot_last = kListQ * k - 1;
    // consecutive query chunks of a slice go to the same XCD: the 128-byte lines of a block's
    // list are completed by neighbouring chunks and should meet in one L2 before they are written back
    int c, s;
    if (!schedule(blockIdx.x, bh, nchunk, s, c)) return;
    const int lo = blockIdx.y * kRange;
    const int hi = min(n, lo + kRange);
    const int t0 = c * kListQ;
    const int rows = min(N - t0, kListQ);
    const int nblk = min(hi, (t0 + rows - 1) / B) - lo;   // kept blocks are < own block of the last query
    const int tid = threadIdx.x;
    int32_t* crow = cnt2 + ((int64_t)s * (nchunk + 1) + c) * n + lo;
    if (nblk <= 0) {
        if (!FILL)
            for (int j = tid; j < hi - lo; j += 256) crow[j] = 0;
        return;
    }
    for (int i = tid; i < nblk * kWords; i += 256) mask[i] = 0u;
    if (FILL) {
        const int32_t* orow = off + (int64_t)s * (n + 1) + lo;
        for (int j = tid; j < nblk; j += 256) {
            start[j] = orow[j] + crow[j];
        }
    }
    __syncthreads();
    const int32_t* rows0 = idx + ((int64_t)s * N + t0) * k;
    // only past blocks count: lists never exceed R
    for_each_entry(rows0, rows, k, tid, [&](int r, int b) {
        b -= lo;
        // (block b + lo lies before the own block of query t0 + r: its last key does)
        if (b >= 0 && b < nblk && (b + lo + 1) * B <= t0 + r) atomicOr(&mask[b * kWords + (r >> 5)], 1u << (r & 31));
    });
    __syncthreads();
    if (!FILL) {
        for (int j = tid; j < hi - lo; j += 256) {
            int c0 = 0;
            if (j < nblk) {
#pragma unroll
                for (int wd = 0; wd < kWords; ++wd) c0 += __popc(mask[j * kWords + wd]);
            }
            crow[j] = c0;
        }
    } else {
        if constexpr (SLOTS) {
            // runs of the blocks one after the other: exclusive scan of the rows' bit counts
            // (four consecutive blocks per thread, threads by shuffles, waves through LDS)
            int c4[4], mine = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int b = 4 * tid + u;
                int c = 0;
                if (b < nblk)
#pragma unroll
                    for (int wd = 0; wd < kWords; ++wd) c += __popc(mask[b * kWords + wd]);
                c4[u] = c;
                mine += c;
            }
            int incl = mine;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int up = __shfl_up(incl, o, kWave);
                if ((tid & (kWave - 1)) >= o) incl += up;
            }
            if ((tid & (kWave - 1)) == kWave - 1) wsum[tid / kWave] = incl;
            __syncthreads();
            int run = incl - mine;
            for (int wv = 0; wv < tid / kWave; ++wv) run += wsum[wv];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (4 * tid + u < nblk) lbase[4 * tid + u] = (uint16_t)run;
                run += c4[u];
            }
            __syncthreads();
            // a query keeps at most k blocks, so the runs hold at most kListQ * k entries
            for_each_entry_slot(rows0, rows, k, tid, [&](int r, int b, int e) {
                b -= lo;
                if (b >= 0 && b < nblk && (b + lo + 1) * B <= t0 + r) {
                    const uint32_t* mrow = mask + b * kWords;
                    int rank = __popc(mrow[r >> 5] & ((1u << (r & 31)) - 1u));
                    for (int wd = 0; wd < (r >> 5); ++wd) rank += __popc(mrow[wd]);
                    slot[min((int)lbase[b] + rank, slot_last)] = (uint8_t)e;
                }
            });
            __syncthreads();
        }
        // Eight lanes per block, one 32-query word each: a lane writes the queries of its word
        // after those of the lanes before it.  The 256 queries of this workgroup are neighbours
        // in every list, so a store instruction touches one short run of addresses per block.
        int32_t* qs = ql + (int64_t)s * R;
        const int lane8 = tid & 7;
        for (int b = tid >> 3; b < nblk; b += 256 / 8) {
            uint32_t word = mask[b * kWords + lane8];
            const int cnt = __popc(word);
            int incl = cnt;
#pragma unroll
            for (int o = 1; o < 8; o <<= 1) {
                const int up = __shfl_up(incl, o, 8);
                if (lane8 >= o) incl += up;
            }
            int64_t pos = (int64_t)start[b] + (incl - cnt);
            int local = SLOTS ? (int)lbase[b] + (incl - cnt) : 0;
            while (word) {
                int entry = t0 + 32 * lane8 + (__ffs(word) - 1);
                if constexpr (SLOTS) entry |= (int)slot[min(local++, slot_last)] << kQueryBits;
                // a routing that breaks the contract (repeats, too many kept blocks) must not
                // write outside the slice's lists
                if (pos < R) qs[pos] = entry;
                ++pos;
                word &= word - 1u;
            }
        }
    }
}

// per slice and key block: cnt2[c][j] <- sum_{c' < c} cnt2[c'][j] (row nchunk: the total).
// A workgroup takes 32 key blocks; 8 threads per block share the chunks.
__global__ __launch_bounds__(256) void lists_scan_kernel(int32_t* __restrict__ cnt2,
                                                         int32_t* __restrict__ off, int n,
                                                         int nchunk)
{
    __shared__ int part[8][33];
    const int s = blockIdx.y, tid = threadIdx.x;
    const int jj = tid & 31, seg = tid >> 5;
    const int j = blockIdx.x * 32 + jj;
    int32_t* cs = cnt2 + (int64_t)s * (nchunk + 1) * n;
    const int per = (nchunk + 7) / 8;
    const int c0 = min(nchunk, seg * per), c1 = min(nchunk, c0 + per);
    int sum = 0;
    if (j < n)
        for (int c = c0; c < c1; ++c) sum += cs[(int64_t)c * n + j];
    part[seg][jj] = sum;
    __syncthreads();
    int run = 0, total = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        const int v = part[g][jj];
        if (g < seg) run += v;
        total += v;
    }
    if (j < n) {
        for (int c = c0; c < c1; ++c) {
            const int v = cs[(int64_t)c * n + j];
            cs[(int64_t)c * n + j] = run;
            run += v;
        }
        if (seg == 0) {
            cs[(int64_t)nchunk * n + j] = total;
            off[(int64_t)s * (n + 1) + j + 1] = total;
        }
    }
}

// per slice: off[j] <- sum_{j' < j} total[j'] (off[j + 1] holds total[j] on entry)
__global__ __launch_bounds__(256) void lists_offsets_kernel(int32_t* __restrict__ off, int n)
{
    __shared__ int part[256];
    const int s = blockIdx.x, tid = threadIdx.x;
    int32_t* os = off + (int64_t)s * (n + 1);
    const int seg = (n + 255) / 256;
    const int a = min(n, tid * seg), b = min(n, a + seg);
    int sum = 0;
    for (int j = a; j < b; ++j) sum += os[j + 1];
    part[tid] = sum;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int i = 0; i < 256; ++i) { const int v = part[i]; part[i] = run; run += v; }
        os[0] = 0;
    }
    __syncthreads();
    int run = part[tid];
    for (int j = a; j < b; ++j) { run += os[j + 1]; os[j + 1] = run; }
}

template <int RANGE>
static hipError_t build_lists_launch(const Dims& s, const int32_t* idx, int32_t* off, int32_t* ql,
                                     int32_t* cnt2, hipStream_t st)
{
    const int nranges = (s.n + RANGE - 1) / RANGE;
    dim3 grid(schedule_grid(s.bh, s.nchunk), nranges), block(256);
    hipLaunchKernelGGL((lists_chunk_kernel<false, false, RANGE>), grid, block, 0, st, idx, cnt2,
                       (const int32_t*)off, ql, s.N, s.B, s.n, s.k, s.nchunk, s.R, s.bh);
    hipLaunchKernelGGL(lists_scan_kernel, dim3((s.n + 31) / 32, s.bh), block, 0, st, cnt2, off, s.n,
                       s.nchunk);
    hipLaunchKernelGGL(lists_offsets_kernel, dim3(s.bh), block, 0, st, off, s.n);
    if (s.R > 0) {
        static_assert(kKeyMajorMaxTopk <= 255 && kListQ * kKeyMajorMaxTopk <= 65535, "slot byte, 16-bit run starts");
        if (key_major_path(s))
            hipLaunchKernelGGL((lists_chunk_kernel<true, true, RANGE>), grid, block, (size_t)kListQ * s.k, st, idx,
                               cnt2, (const int32_t*)off, ql, s.N, s.B, s.n, s.k, s.nchunk, s.R, s.bh);
        else
            hipLaunchKernelGGL((lists_chunk_kernel<true, false, RANGE>), grid, block, 0, st, idx, cnt2,
                               (const int32_t*)off, ql, s.N, s.B, s.n, s.k, s.nchunk, s.R, s.bh);
    }
    return hipGetLastError();
}

// Up to kRangeMax blocks one range covers a slice and a workgroup reads its routing rows once.
// Beyond that the rows are read once per range anyway, and a workgroup's cost is that of walking
// its bit matrix, however few pairs fall into it: smaller ranges, more workgroups (N = 524288,
// B = 128, top-k 8: fill pass 3.9 ms with ranges of 1024 blocks, 2.6 ms with 512, 3.5 ms with 256).
hipError_t launch_build_lists(const Dims& s, const int32_t* idx, int32_t* off, int32_t* ql,
                              int32_t* cnt2, hipStream_t st)
{
    return s.n <= kRangeMax ? build_lists_launch<kRangeMax>(s, idx, off, ql, cnt2, st)
                            : build_lists_launch<kRangeLong>(s, idx, off, ql, cnt2, st);
}

}  // namespace moba
