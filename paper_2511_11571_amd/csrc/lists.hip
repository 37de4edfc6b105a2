// Key-block-major query lists from query-major routing (paper Appendix C.1,
// "Reformatting Indices to Varlen Key-Block-Major").  The paper scatters with global
// atomics, which leaves the order inside a list to chance; here the lists come out
// ascending and bit-reproducible:
//   1. count: a workgroup takes 256 consecutive queries (two chunks of 128) and ORs one bit per
//      (query, kept block) into an LDS bit matrix [block][256 bits]; the population
//      count of a row is the number of queries of this chunk that kept that block.
//   2. scan: per key block an exclusive scan over chunks (start of each chunk's segment
//      inside the block's list; kept as the blk_chunk output, which lets a query-tile kernel
//      find "its" rows of any block's list directly), then an exclusive scan of the block
//      totals (blk_off).
//   3. fill: the bit matrix is rebuilt and each row's set bits are written out in
//      ascending order at blk_off[j] + chunk start.
// The bit matrix lives in LDS only and covers 2048 key blocks at a time.
#include "common.h"

namespace moba {

constexpr int kRange = 2048;                    // key blocks per LDS bit matrix (64 KB)
constexpr int kListQ = 2 * kChunkQ;              // queries per workgroup: two chunks of 128
constexpr int kWords = kListQ / 32;             // 8 words of 32 query bits per block


template <bool FILL>
__global__ __launch_bounds__(256) void lists_chunk_kernel(
    const int32_t* __restrict__ idx, int32_t* __restrict__ cnt2, const int32_t* __restrict__ off,
    int32_t* __restrict__ ql, int N, int B, int n, int k, int nchunk, int64_t R)
{
    __shared__ uint32_t mask[kRange * kWords];
    const int c = blockIdx.x, s = blockIdx.z;
    const int lo = blockIdx.y * kRange;
    const int hi = min(n, lo + kRange);
    const int t_last = min(N, (c + 1) * kListQ) - 1;
    const int nblk = min(hi, t_last / B) - lo;          // kept blocks are < own block of t_last
    const int tid = threadIdx.x;
    // this workgroup covers chunks 2c and 2c+1 (the second may not exist)
    int32_t* crow = cnt2 + ((int64_t)s * (nchunk + 1) + 2 * c) * n + lo;
    const bool two = 2 * c + 1 < nchunk;
    if (nblk <= 0) {
        if (!FILL)
            for (int j = tid; j < hi - lo; j += 256) {
                crow[j] = 0;
                if (two) crow[n + j] = 0;
            }
        return;
    }
    for (int i = tid; i < nblk * kWords; i += 256) mask[i] = 0u;
    __syncthreads();
    const int t = c * kListQ + tid;
    if (t < N) {
        const int32_t* row = idx + ((int64_t)s * N + t) * k;
        const uint32_t bit = 1u << (tid & 31);
        const int word = tid >> 5;
        const int past = t / B;            // only past blocks count: lists never exceed R
        for (int e = 0; e < k; ++e) {
            const int b = row[e] - lo;
            if (b >= 0 && b < nblk && b + lo < past) atomicOr(&mask[b * kWords + word], bit);
        }
    }
    __syncthreads();
    if (!FILL) {
        for (int j = tid; j < hi - lo; j += 256) {
            int c0 = 0, c1 = 0;
            if (j < nblk) {
#pragma unroll
                for (int wd = 0; wd < kWords / 2; ++wd) {
                    c0 += __popc(mask[j * kWords + wd]);
                    c1 += __popc(mask[j * kWords + kWords / 2 + wd]);
                }
            }
            crow[j] = c0;
            if (two) crow[n + j] = c1;
        }
    } else {
        const int wave = tid / kWave, lane = tid % kWave;
        const int32_t* orow = off + (int64_t)s * (n + 1) + lo;
        int32_t* qs = ql + (int64_t)s * R;
        for (int j = wave; j < nblk; j += 4) {
            int base = orow[j] + crow[j];
#pragma unroll
            for (int r = 0; r < kListQ / kWave; ++r) {
                const int q = r * kWave + lane;
                const bool on = (mask[j * kWords + (q >> 5)] >> (q & 31)) & 1u;
                const uint64_t m = __ballot(on);
                if (on) qs[base + lanes_below(m)] = c * kListQ + q;
                base += __popcll(m);
            }
        }
    }
}

// per slice: cnt2[c][j] <- sum_{c' < c} cnt2[c'][j] (row nchunk: the total);  off[j] <- sum_{j' < j} total[j']
__global__ __launch_bounds__(256) void lists_scan_kernel(int32_t* __restrict__ cnt2,
                                                         int32_t* __restrict__ off, int n,
                                                         int nchunk)
{
    __shared__ int part[256];
    const int s = blockIdx.x, tid = threadIdx.x;
    int32_t* cs = cnt2 + (int64_t)s * (nchunk + 1) * n;
    int32_t* os = off + (int64_t)s * (n + 1);
    for (int j = tid; j < n; j += 256) {
        int run = 0;
        for (int c = 0; c < nchunk; ++c) {
            const int v = cs[(int64_t)c * n + j];
            cs[(int64_t)c * n + j] = run;
            run += v;
        }
        cs[(int64_t)nchunk * n + j] = run;
        os[j + 1] = run;
    }
    __syncthreads();
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

hipError_t launch_build_lists(const Dims& s, const int32_t* idx, int32_t* off, int32_t* ql,
                              int32_t* cnt2, hipStream_t st)
{
    const int nranges = (s.n + kRange - 1) / kRange;
    dim3 grid((s.nchunk + 1) / 2, nranges, s.bh), block(256);
    hipLaunchKernelGGL((lists_chunk_kernel<false>), grid, block, 0, st, idx, cnt2,
                       (const int32_t*)off, ql, s.N, s.B, s.n, s.k, s.nchunk, s.R);
    hipLaunchKernelGGL(lists_scan_kernel, dim3(s.bh), block, 0, st, cnt2, off, s.n, s.nchunk);
    if (s.R > 0)
        hipLaunchKernelGGL((lists_chunk_kernel<true>), grid, block, 0, st, idx, cnt2,
                           (const int32_t*)off, ql, s.N, s.B, s.n, s.k, s.nchunk, s.R);
    return hipGetLastError();
}

}  // namespace moba
