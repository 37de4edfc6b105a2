// Packed variable-length batches (paper Appendix C.1: a sequence of N keys is cut into
// ceil(N / B) blocks, the last one shorter; its index reformatting is "varlen" from the start).
//
// Several sequences lie one after the other along the token axis of [slices, T, row].  The
// attention kernels want every key block to start at a multiple of B, so the batch is brought
// into a padded layout first: every sequence is followed by zero rows up to the next multiple of
// B and the whole is treated as one sequence of T' tokens.  A query never sees a later key, so a
// real query never meets the zero rows of its own last block; the gate takes the candidates of a
// query from its own sequence only (blk_first); zero dO rows add nothing to dK and dV.  Rows of
// the padding carry no meaning and are dropped on the way back.
#include "common.h"

namespace moba {

// largest i with offs[i] <= x (offs ascending, offs[0] = 0, x < offs[num])
__device__ __forceinline__ int seq_of(const int32_t* __restrict__ offs, int num, int x)
{
    int lo = 0, hi = num;                   // answer in [lo, hi)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offs[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// PAD: Xp[s][p] <- X[s][row of token p] or zeros;  !PAD: X[s][r] <- Xp[s][padded place of r].
// One thread per element of type T (16 bytes where rows and pointers allow, else 4) of a row of
// the destination; blockIdx.y is the slice.
template <bool PAD, typename T>
__global__ __launch_bounds__(256) void varlen_copy_kernel(
    const int32_t* __restrict__ seq_off, const int32_t* __restrict__ pad_off, int num_seqs, int tokens,
    int padded_tokens, int row_elems, const T* __restrict__ src, T* __restrict__ dst)
{
    const int drows = PAD ? padded_tokens : tokens, srows = PAD ? tokens : padded_tokens;
    const int i = blockIdx.x * 256 + threadIdx.x;            // (rows * row_elems < 2^31: checked by the launcher)
    if (i >= drows * row_elems) return;
    const int r = i / row_elems, e = i - r * row_elems;
    const int64_t s = blockIdx.y;
    int from = -1;                                           // source row, -1: zeros
    if (PAD) {
        const int q = seq_of(pad_off, num_seqs, r);
        const int t = r - pad_off[q];
        if (t < seq_off[q + 1] - seq_off[q]) from = seq_off[q] + t;
    } else {
        const int q = seq_of(seq_off, num_seqs, r);
        from = pad_off[q] + (r - seq_off[q]);
    }
    T v{};
    if (from >= 0) v = src[(s * srows + from) * row_elems + e];
    dst[(s * drows + r) * row_elems + e] = v;
}

__global__ __launch_bounds__(256) void varlen_block_first_kernel(const int32_t* __restrict__ pad_off,
                                                                 int num_seqs, int B, int nblocks,
                                                                 int32_t* __restrict__ first)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= nblocks) return;
    first[c] = pad_off[seq_of(pad_off, num_seqs, c * B)] / B;
}

template <typename T>
static hipError_t varlen_copy_launch(bool pad, const int32_t* seq_off, const int32_t* pad_off, int num_seqs,
                                     int64_t slices, int tokens, int padded_tokens, int row_elems,
                                     const void* src, void* dst, hipStream_t st)
{
    const int64_t per_slice = (int64_t)(pad ? padded_tokens : tokens) * row_elems;
    if (per_slice == 0 || slices == 0) return hipSuccess;
    if (per_slice >= ((int64_t)1 << 31) || slices > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((per_slice + 255) / 256), (unsigned)slices);
    if (pad)
        hipLaunchKernelGGL((varlen_copy_kernel<true, T>), grid, dim3(256), 0, st, seq_off, pad_off, num_seqs,
                           tokens, padded_tokens, row_elems, (const T*)src, (T*)dst);
    else
        hipLaunchKernelGGL((varlen_copy_kernel<false, T>), grid, dim3(256), 0, st, seq_off, pad_off, num_seqs,
                           tokens, padded_tokens, row_elems, (const T*)src, (T*)dst);
    return hipGetLastError();
}

hipError_t launch_varlen_copy(bool pad, const int32_t* seq_off, const int32_t* pad_off, int num_seqs,
                              int64_t slices, int tokens, int padded_tokens, int row_bytes, const void* src,
                              void* dst, hipStream_t st)
{
    const bool wide = row_bytes % 16 == 0 && ((uintptr_t)src | (uintptr_t)dst) % 16 == 0;
    return wide ? varlen_copy_launch<uint4>(pad, seq_off, pad_off, num_seqs, slices, tokens, padded_tokens,
                                            row_bytes / 16, src, dst, st)
                : varlen_copy_launch<uint32_t>(pad, seq_off, pad_off, num_seqs, slices, tokens, padded_tokens,
                                               row_bytes / 4, src, dst, st);
}

hipError_t launch_varlen_block_first(const int32_t* pad_off, int num_seqs, int B, int nblocks, int32_t* first,
                                     hipStream_t st)
{
    if (nblocks == 0) return hipSuccess;
    hipLaunchKernelGGL(varlen_block_first_kernel, dim3((nblocks + 255) / 256), dim3(256), 0, st, pad_off,
                       num_seqs, B, nblocks, first);
    return hipGetLastError();
}

}  // namespace moba
