/*
 * moba.h -- C ABI of the MI355X (gfx950) Mixture of Block Attention library.
 *
 * The operator (paper "Optimizing Mixture of Block Attention", Section 2):
 * the N keys of one head are cut into n = N/B blocks; a block's gate score for a
 * query is q . mean(keys of the block); each query keeps its `topk` best *past*
 * blocks (ties: lower block index) and always attends its own block under a causal
 * mask; O = softmax(q K_S^T * scale) V_S over the kept tokens S.  An optional
 * depthwise causal convolution (Appendix B) replaces K by
 * K' = K + SiLU(conv(K)) before both the gate and attention.
 *
 * General rules for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps device memory.  `const moba_shape*` and the
 *     size_t* / int64_t* outputs are HOST pointers.
 *   - Tensors are contiguous, row-major [batch, heads, N, d]; element type is
 *     `shape->dtype` (fp32, or bf16 as raw 16-bit words) for Q, K, V, K_eff, O, dO,
 *     dQ, dK, dV.  Centroids, lse and conv weights are always fp32; indices int32.
 *   - Arguments are checked on the host before anything is enqueued; a call that
 *     returns MOBA_EINVAL, MOBA_EUNSUPPORTED or MOBA_EWORKSPACE has launched nothing (MOBA_EHIP:
 *     a launch failed; kernels enqueued before it may still run).  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns without synchronising.
 *   - Return value: MOBA_OK (0) or a negative moba_status.  No exceptions, no abort.
 *   - Supported: head_dim 64 or 128; seqlen a multiple of block; block >= 1;
 *     topk >= 0 (topk >= n-1 is full causal attention); conv_width 0 (none) or 1..8;
 *     at most 16384 key blocks per head for moba_topk with bf16 tensors, 4096 otherwise
 *     (and with MOBA_FLAG_REFERENCE_KERNELS); seqlen <= 2^24; batch * heads
 *     <= 65535; R < 2^31.
 *   - R below is the number of (query, kept past block) pairs of one [N, d]
 *     slice, R = B * sum_{c<n} min(c, topk); it depends on the shape only
 *     (moba_routes_per_slice).
 */
#ifndef MOBA_H_
#define MOBA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum moba_status {
    MOBA_OK = 0,
    MOBA_EINVAL = -1,       /* null pointer, non-positive size, N % B != 0, topk < 0, bad dtype */
    MOBA_EUNSUPPORTED = -2, /* legal but not built: head_dim, conv_width, sizes over the limits */
    MOBA_EWORKSPACE = -3,   /* workspace pointer null or smaller than moba_workspace_bytes    */
    MOBA_EHIP = -4          /* a HIP launch failed; see moba_last_hip_error                   */
} moba_status;

typedef enum moba_dtype { MOBA_F32 = 0, MOBA_BF16 = 1 } moba_dtype;

/* flags */
#define MOBA_FLAG_REFERENCE_KERNELS 1u /* use the plain (non-MFMA) kernels for every stage */
#define MOBA_FLAG_KEY_MAJOR 2u         /* attention forward and dQ by key block with one partial per
                                        * (query, block) pair and a merge kernel (paper Section 4.2):
                                        * force it where that path exists (bf16; B a multiple of 32
                                        * up to 128 (d = 64) / 64 (d = 128), or a multiple of that;
                                        * topk <= 64); elsewhere the flag is ignored              */
#define MOBA_FLAG_QUERY_TILES 4u       /* attention by query tile (suits dense routing): force it   */
#define MOBA_FLAG_GATE_EXACT_SEARCH 8u  /* moba_topk: skip the approximate first look of the selection and
                                        * search on exact scores from the start (slower, same result; the
                                        * path that queries with many equal scores take anyway)          */
#define MOBA_FLAG_SHARED_WORKSPACE 16u  /* the caller hands moba_forward and the following moba_backward /
                                        * moba_backward_parts of the same K_eff and V the SAME workspace
                                        * (then fwd_ws == bwd_ws in moba_workspace_bytes): the copies of K
                                        * and V that the query-tile kernels read are made once, by the
                                        * forward call, and the backward trusts what it finds there.
                                        * Without the flag every call prepares its own.  No effect where
                                        * the other kernels run.                                         */
/* With neither of KEY_MAJOR and QUERY_TILES the library picks by a cost estimate of both from the shape: key blocks
 * where a tile of consecutive queries would meet a key block with few of its rows (small topk,
 * long sequences, large blocks: e.g. topk 8 of B = 128 at any length), query tiles where a query
 * keeps many blocks (e.g. topk 64 of B = 32 up to a few hundred thousand keys).  KEY_MAJOR and
 * QUERY_TILES together are MOBA_EINVAL.  The workspace sizes depend on the choice: size and call
 * with the same flags. */

typedef struct moba_shape {
    int32_t batch, heads, seqlen, head_dim;
    int32_t block;         /* B: keys per block                                        */
    int32_t topk;          /* k: kept PAST blocks per query; the own block is extra    */
    int32_t conv_width;    /* W: 0 = no key convolution                                */
    int32_t dtype;         /* moba_dtype                                               */
    float   softmax_scale; /* <= 0 selects 1/sqrt(head_dim)                            */
    uint32_t flags;        /* MOBA_FLAG_*                                              */
    int32_t kv_heads;      /* grouped-query / multi-query attention (Appendix C, last paragraph):
                            * key/value heads; 0 = heads.  Must divide heads; query head h reads
                            * key/value head h / (heads / kv_heads).  Then K, V, K_eff, centroids,
                            * dK, dV and dK_eff are [b,kv_heads,..], conv_w and dconv_w
                            * [kv_heads,d,W]; Q, O, lse, dO, dQ and the routing stay [b,heads,..];
                            * dK and dV are summed over the query heads that share the head. */
} moba_shape;

/* In the argument tables below h stands for the query heads (shape.heads) and kv for the key/value
 * heads (shape.kv_heads, or heads when that is 0). */

/* Host-only helpers.  R and the byte counts are written to host memory. */
int moba_routes_per_slice(const moba_shape* shape, int64_t* R);
int moba_workspace_bytes(const moba_shape* shape, size_t* topk_ws, size_t* fwd_ws, size_t* bwd_ws);

/*
 * Key convolution (Appendix B, k'_t = k_t + SiLU(sum_l W_l * k_{t-l}), terms with
 * t-l < 0 dropped) followed by the block centroids (Section 2; Appendix C.1,
 * centroid algorithm).
 *   K         in   [b,kv,N,d] dtype
 *   conv_w    in   [kv,d,W] fp32, last axis = lag l; must be NULL iff conv_width == 0
 *   K_eff     out  [b,kv,N,d] dtype: the convolved keys rounded to dtype; required iff
 *                  conv_width > 0 (with conv_width == 0 it may be NULL; if given, K is copied);
 *                  with conv_width > 1 it must not be K itself (MOBA_EINVAL) nor overlap it
 *   centroids out  [b,kv,n,d] fp32: mean over each block of the (rounded) K_eff rows
 */
int moba_centroids(const moba_shape* shape, const void* K, const float* conv_w,
                   void* K_eff, float* centroids, void* stream);

/*
 * Backward of the key convolution (Appendix B: training sends the gradients through the
 * convolution to the token-level keys and to the kernel weights).  The rounding of K_eff to
 * dtype is taken as the identity.  With a_t = sum_l W_l * k_{t-l}, g_t = dK_eff_t * SiLU'(a_t):
 *   dK_t = dK_eff_t + sum_{l, t+l<N} W_l * g_{t+l},   dconv_w[h][c][l] = sum_{batch, t>=l} g_t k_{t-l}
 *   K        in   [b,kv,N,d] dtype: the keys the convolution was applied to
 *   conv_w   in   [kv,d,W] fp32
 *   dK_eff   in   [b,kv,N,d] dtype: gradient with respect to K_eff (dK of moba_backward)
 *   dK       out  [b,kv,N,d] dtype: gradient with respect to K; must not overlap dK_eff
 *   dconv_w  out  [kv,d,W] fp32, summed over the batch in a fixed order
 *   ws            at least moba_key_conv_backward_workspace bytes
 * conv_width must be at least 1.
 */
int moba_key_conv_backward_workspace(const moba_shape* shape, size_t* ws_bytes);
int moba_key_conv_backward(const moba_shape* shape, const void* K, const float* conv_w,
                           const void* dK_eff, void* dK, float* dconv_w, void* ws,
                           size_t ws_bytes, void* stream);

/*
 * Gate scores and causal top-k (Section 2; Appendix C.1, top-k selection algorithm)
 * followed by the key-block-major query lists (Appendix C.1, varlen reformatting).
 * The N x n score matrix is never written to memory.
 *   Q         in   [b,h,N,d] dtype
 *   centroids in   [b,kv,n,d] fp32
 *   topk_idx  out  [b,h,N,topk] int32: kept past blocks of each query in ascending
 *                  block order, -1 in unused trailing slots
 *   blk_off   out  [b,h,n+1] int32: exclusive prefix sums of the per-block list lengths
 *   blk_q     out  [b,h,R] int32: for each key block the queries that kept it,
 *                  ascending (deterministic); block j's list is
 *                  blk_q[blk_off[j] .. blk_off[j+1]).  Bits 0..23 of an entry are the
 *                  query's position in the sequence.  Bits 24..31 are for the library's
 *                  own use: where the shape and flags select the key-block-major
 *                  attention kernels they hold the position of block j in that query's
 *                  row of topk_idx, otherwise zero.  Lists MUST therefore be built (here or
 *                  by moba_build_lists) with the shape and flags they are used with: the
 *                  key-block-major kernels file their partial results by that position, and
 *                  lists built without it (e.g. with MOBA_FLAG_QUERY_TILES, then used with
 *                  MOBA_FLAG_KEY_MAJOR) give a wrong result that no status code reports.
 *   ws             at least topk_ws bytes from moba_workspace_bytes
 */
int moba_topk(const moba_shape* shape, const void* Q, const float* centroids,
              int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q,
              void* ws, size_t ws_bytes, void* stream);

/*
 * moba_topk for callers that cannot allocate device memory or hand over a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with
 * the workspace in a device array that is part of the library image, MOBA_TOPK_STATIC_MAX_BYTES
 * long, one copy per GPU, held until the process ends.  The call allocates nothing.  Same
 * arguments, outputs and checks as moba_topk without `ws`; a shape whose topk_ws (see
 * moba_workspace_bytes) exceeds MOBA_TOPK_STATIC_MAX_BYTES returns MOBA_EWORKSPACE and launches
 * nothing (batch 1, 16 heads, N = 32768, B = 32 needs 15 MiB).  All calls on one GPU share that
 * GPU's array: calls that may overlap in time on one GPU (different streams, different threads)
 * race and must be ordered by the caller.  Nothing in the array has to survive between calls.
 */
#define MOBA_TOPK_STATIC_MAX_BYTES (32u << 20)
int moba_topk_static(const moba_shape* shape, const void* Q, const float* centroids,
                     int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q, void* stream);

/*
 * Packed variable-length batches (Appendix C.1: a sequence of N keys has ceil(N / B) blocks, the last
 * one shorter).  The sequences of a batch lie one after the other along the token axis,
 * [1, heads, T, d] with sequence i in rows seq_offsets[i] .. seq_offsets[i+1]; each is the operator
 * on its own (blocks count from its first token, a query's candidates are the complete blocks before
 * its own block in its own sequence).  The kernels work on a PADDED layout in which every sequence
 * is followed by zero rows up to the next multiple of B and the whole is one sequence of T' tokens
 * (pad_offsets[i] = start of sequence i there):
 *   moba_varlen_layout       HOST ONLY: pad_offsets [num_seqs+1] and T' from seq_offsets
 *                            [num_seqs+1] (both host arrays; seq_offsets[0] = 0, ascending)
 *   moba_varlen_pad / _unpad [slices, T, row] <-> [slices, T', row] for rows of row_bytes bytes (a
 *                            multiple of 4: Q, K, V, O, dO, gradients, lse); padding rows are
 *                            written as zeros and dropped on the way back.  seq_offsets and
 *                            pad_offsets are DEVICE arrays here.  Source and destination differ.
 *                            At most 65535 slices and 2^31 - 1 four-byte words per padded slice
 *                            (MOBA_EUNSUPPORTED beyond, nothing launched).
 *   moba_varlen_block_first  block_first [T' / B] (device): first block of the sequence each block
 *                            of the padded layout belongs to
 *   moba_topk_varlen         moba_topk on the padded layout (shape.batch = 1, shape.seqlen = T'),
 *                            the candidates of a query in block c being blocks
 *                            block_first[c] .. c - 1.  topk_idx holds block numbers of the padded
 *                            layout.  blk_q is sized for R of that shape (moba_routes_per_slice),
 *                            an upper bound; the lists are blk_off[0] .. blk_off[T' / B].
 * moba_centroids, moba_forward and moba_backward run unchanged on the padded tensors with the
 * routing of moba_topk_varlen: no real query keeps a block of another sequence or sees a padding row,
 * and padding rows of dO are zero.
 */
int moba_varlen_layout(int32_t num_seqs, const int32_t* seq_offsets, int32_t block, int32_t* pad_offsets,
                       int32_t* padded_tokens);
int moba_varlen_pad(int32_t num_seqs, const int32_t* seq_offsets, const int32_t* pad_offsets, int32_t slices,
                    int32_t tokens, int32_t padded_tokens, int32_t row_bytes, const void* X, void* X_padded,
                    void* stream);
int moba_varlen_unpad(int32_t num_seqs, const int32_t* seq_offsets, const int32_t* pad_offsets, int32_t slices,
                      int32_t tokens, int32_t padded_tokens, int32_t row_bytes, const void* X_padded, void* X,
                      void* stream);
int moba_varlen_block_first(int32_t num_seqs, const int32_t* pad_offsets, int32_t block, int32_t padded_tokens,
                            int32_t* block_first, void* stream);
int moba_topk_varlen(const moba_shape* shape, const void* Q, const float* centroids,
                     const int32_t* block_first, int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * The list-building half of moba_topk alone (Appendix C.1, varlen reformatting), for a
 * routing supplied by the caller.  topk_idx rows may list their blocks in any order;
 * entries must be -1 or a past block of the query, without repeats, and every query of
 * block c must keep exactly min(c, topk) blocks (not checked on the device).
 */
int moba_build_lists(const moba_shape* shape, const int32_t* topk_idx,
                     int32_t* blk_off, int32_t* blk_q,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Attention over the kept blocks plus the causally masked own block
 * (Section 2; Section 4.2 forward algorithm).  Routing is an input.
 *   Q             in   [b,h,N,d] dtype
 *   K_eff, V      in   [b,kv,N,d] dtype (K_eff = K when there is no convolution)
 *   topk_idx, blk_off, blk_q   in   as produced by moba_topk / moba_build_lists for this shape and
 *                                   these flags (moba_backward takes the same three)
 *   O         out  [b,h,N,d] dtype
 *   lse       out  [b,h,N] fp32: natural log of sum_u exp(scale * q.k_u) over the kept keys
 *   ws             at least fwd_ws bytes
 */
int moba_forward(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                 const int32_t* topk_idx, const int32_t* blk_off, const int32_t* blk_q,
                 void* O, float* lse, void* ws, size_t ws_bytes,
                 void* stream);

/*
 * Backward at fixed routing (Section 4.2 backward; Appendix C.3):
 * D = rowsum(dO o O), P = exp(S - lse), dV = P^T dO, dS = P o (dO V^T - D),
 * dQ = scale * dS K, dK = scale * dS^T Q.  dK is the gradient with respect to K_eff.
 * No gradient flows through the gate (centroids / top-k).
 *   Q, O, dO             in   [b,h,N,d] dtype;   lse in [b,h,N] fp32 (from moba_forward)
 *   K_eff, V             in   [b,kv,N,d] dtype
 *   dQ                   out  [b,h,N,d] dtype
 *   dK, dV               out  [b,kv,N,d] dtype, summed over the query heads that share the head
 *   ws                        at least bwd_ws bytes
 */
int moba_backward(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                  const void* O, const float* lse, const void* dO,
                  const int32_t* topk_idx, const int32_t* blk_off, const int32_t* blk_q,
                  void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
                  void* stream);

/*
 * Decode-shaped forward (inference): the operator of Section 2 for the LAST q_len positions of a
 * sequence of seqlen keys -- query r stands at position t = seqlen - q_len + r, is scored against
 * the centroids of the complete blocks before its own block (j < t / B), keeps the topk best
 * (ties: lower block), and attends those blocks plus its own block up to itself.  Here seqlen
 * need NOT be a multiple of the block: the own block of a query may be the ragged last block
 * (Appendix C.1 treats the tail block of the centroid computation the same way; its centroid is
 * never used, the own block not being a candidate).  One kernel, no workspace, fp32 arithmetic.
 *   Q          in   [b,heads,q_len,d] dtype
 *   K_eff, V   in   [b,kv_heads,seqlen,d] dtype (key convolution, if any, already applied)
 *   centroids  in   [b,kv_heads,centroid_blocks,d] fp32: means of the complete blocks, e.g. a
 *                   cache kept by the caller; centroid_blocks >= (seqlen - 1) / B; may be NULL
 *                   when that is 0 or topk == 0
 *   O          out  [b,heads,q_len,d] dtype;  lse out [b,heads,q_len] fp32
 *   topk_idx   out  [b,heads,q_len,topk] int32 ascending, -1 padded; may be NULL
 * conv_width and flags of the shape are ignored.  At most 4096 complete blocks.
 */
int moba_decode_forward(const moba_shape* shape, int32_t q_len, const void* Q, const void* K_eff,
                        const void* V, const float* centroids, int32_t centroid_blocks, void* O,
                        float* lse, int32_t* topk_idx, void* stream);

/*
 * moba_backward split into its kernels, for callers that time or overlap them:
 * `parts` is a bit set of MOBA_BWD_PREPROCESS (D = rowsum(dO o O) into the workspace),
 * MOBA_BWD_DQ and MOBA_BWD_DKDV (both read D from the workspace, so PREPROCESS must have
 * run on the same workspace first).  Output pointers of parts not requested may be NULL.
 * moba_backward(...) is moba_backward_parts(..., MOBA_BWD_ALL).
 */
#define MOBA_BWD_PREPROCESS 1u
#define MOBA_BWD_DQ 2u
#define MOBA_BWD_DKDV 4u
#define MOBA_BWD_ALL 7u
int moba_backward_parts(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                        const void* O, const float* lse, const void* dO,
                        const int32_t* topk_idx, const int32_t* blk_off, const int32_t* blk_q,
                        void* dQ, void* dK, void* dV, void* ws,
                        size_t ws_bytes, void* stream, uint32_t parts);

/* Static, NUL-terminated description of a status code. */
const char* moba_strerror(int status);
/* hipError_t value of the most recent failed HIP call on the calling thread (0 if none). */
int moba_last_hip_error(void);

/*
 * Kernel timing for benchmarks (no part of the method).  Between moba_profile_begin and
 * moba_profile_end every launch of one of the main kernels is bracketed by a pair of HIP
 * events on the stream it is launched on.  moba_profile_end waits for those events and adds,
 * per kernel, the elapsed milliseconds to ms[kernel] and the launches to calls[kernel] (both
 * host arrays of MOBA_PROFILE_KERNELS entries, overwritten), then drops the events.  At most
 * 4096 launches are recorded per session; further ones go untimed.  One session per process at a
 * time (a second moba_profile_begin returns MOBA_EINVAL); launches from any thread are recorded.
 * Apart from an open timing session the library keeps no state that a call could observe: calls
 * on distinct streams and threads are independent.
 */
enum {
    MOBA_PROFILE_TOPK = 0,    /* gate scores + top-k selection                    */
    MOBA_PROFILE_FORWARD = 1, /* forward attention tile kernel                    */
    MOBA_PROFILE_DQ = 2,      /* backward dQ tile kernel                          */
    MOBA_PROFILE_DKDV = 3,    /* backward dK / dV kernel                          */
    MOBA_PROFILE_KERNELS = 4
};
int moba_profile_begin(void);
int moba_profile_end(float* ms, int32_t* calls);

/*
 * Measured ceilings for benchmarks (no part of the method).  Both calls time their own kernels with
 * a pair of HIP events on `stream` and wait for them.
 * moba_microbench_copy: a plain grid-stride copy of `bytes` (a multiple of 16) from src to dst
 *   (device buffers, not overlapping), `reps` launches after one warm-up; *ms = time per launch, so
 *   the HBM rate is 2 * bytes / *ms.
 * moba_microbench_mfma: a register-only loop of v_mfma_f32_16x16x32_bf16 (eight independent chains
 *   per wave, `iters` rounds) on waves_per_simd (1..8) waves per SIMD of every compute unit; `sink`
 *   is a device buffer of at least 1 KiB that is never written in practice; *ms = launch time,
 *   *flop = floating-point operations of the launch.
 */
int moba_microbench_copy(void* dst, const void* src, size_t bytes, int reps, float* ms, void* stream);
int moba_microbench_mfma(int waves_per_simd, int iters, void* sink, float* ms, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOBA_H_ */
