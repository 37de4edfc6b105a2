// C ABI of the library: host-side argument checks, workspace layout and dispatch.
// Every check happens before the first HIP call, so each error path can be
// exercised on a machine without a GPU.
#include <math.h>

#include <map>
#include <mutex>
#include <utility>

#include "mfma.h"

using namespace moba;

namespace {

thread_local int g_last_hip_error = 0;

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return MOBA_OK;
    g_last_hip_error = (int)e;
    return MOBA_EHIP;
}

constexpr int kMaxBlocks = 4096;   // key blocks per head the plain gate kernel and the decode kernel keep in LDS
constexpr int kMaxTopk = 4096;
constexpr int kMaxSeqlen = 1 << 24;       // the gathering kernels hold a row's byte offset inside its slice in 32 bits

// Fills `d` from `shape`; returns MOBA_OK or the status to hand back.
int make_dims(const moba_shape* sh, Dims& d, bool ragged_ok = false)
{
    if (!sh) return MOBA_EINVAL;
    if (sh->batch <= 0 || sh->heads <= 0 || sh->seqlen <= 0 || sh->head_dim <= 0) return MOBA_EINVAL;
    if (sh->block <= 0 || sh->topk < 0 || sh->conv_width < 0) return MOBA_EINVAL;
    if (!ragged_ok && sh->seqlen % sh->block != 0) return MOBA_EINVAL;
    if (sh->dtype != MOBA_F32 && sh->dtype != MOBA_BF16) return MOBA_EINVAL;
    if (sh->flags & ~(uint32_t)(MOBA_FLAG_REFERENCE_KERNELS | MOBA_FLAG_KEY_MAJOR | MOBA_FLAG_QUERY_TILES |
                                 MOBA_FLAG_GATE_EXACT_SEARCH | MOBA_FLAG_SHARED_WORKSPACE))
        return MOBA_EINVAL;
    if ((sh->flags & MOBA_FLAG_KEY_MAJOR) && (sh->flags & MOBA_FLAG_QUERY_TILES)) return MOBA_EINVAL;
    if (!(sh->softmax_scale == sh->softmax_scale) || isinf(sh->softmax_scale)) return MOBA_EINVAL;
    if (sh->head_dim != 64 && sh->head_dim != 128) return MOBA_EUNSUPPORTED;
    if (sh->conv_width > 8) return MOBA_EUNSUPPORTED;
    if (sh->topk > kMaxTopk) return MOBA_EUNSUPPORTED;
    if (sh->seqlen > kMaxSeqlen) return MOBA_EUNSUPPORTED;
    if ((int64_t)sh->batch * sh->heads > 65535) return MOBA_EUNSUPPORTED;
    if (sh->kv_heads < 0 || (sh->kv_heads > 0 && sh->heads % sh->kv_heads != 0)) return MOBA_EINVAL;
    d.bh = sh->batch * sh->heads;
    d.heads = sh->heads;
    d.hkv = sh->kv_heads > 0 ? sh->kv_heads : sh->heads;
    d.G = d.heads / d.hkv;
    d.bhk = sh->batch * d.hkv;
    d.N = sh->seqlen;
    d.D = sh->head_dim;
    d.B = sh->block;
    d.n = d.N / d.B;
    d.k = sh->topk;
    d.W = sh->conv_width;
    d.dtype = sh->dtype;
    d.flags = sh->flags;
    d.scale = sh->softmax_scale > 0.f ? sh->softmax_scale : 1.0f / sqrtf((float)d.D);
    d.nchunk = (d.N + kChunkQ - 1) / kChunkQ;
    // R = B * sum_{c<n} min(c, k) = B * (k*n - k(k+1)/2) for k < n, B * n(n-1)/2 otherwise
    const int64_t n = d.n, k = d.k;
    const int64_t blocks = k < n ? k * n - k * (k + 1) / 2 : n * (n - 1) / 2;
    d.R = blocks * d.B;
    if (d.R >= ((int64_t)1 << 31)) return MOBA_EUNSUPPORTED;   // list offsets are int32
    return MOBA_OK;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// top-k: the list builder's per-(256-query chunk, key block) counts, then the three bf16 terms
// of the centroids (MFMA scoring)
size_t chunk_counts_bytes(const Dims& d)
{
    return align256(sizeof(int32_t) * (size_t)d.bh * (d.nchunk + 1) * d.n);
}
size_t topk_ws_bytes(const Dims& d)
{
    return chunk_counts_bytes(d) + align256(topk_mfma_ws_bytes(d)) + 256;
}
int32_t* chunk_counts(const Dims&, void* ws) { return static_cast<int32_t*>(ws); }
void* topk_terms(const Dims& d, void* ws) { return static_cast<char*>(ws) + chunk_counts_bytes(d); }
size_t bwd_ws_bytes(const Dims& d);
// forward: operand copies of K and V (+ the per-pair partials of the key-major kernel)
size_t fwd_ws_bytes(const Dims& d)
{
    if (!mfma_path(d)) return 256;
    if (key_major_path(d)) return align256(forward_km_ws_bytes(d));
    if (!tile_forward_ok(d)) return 256;                                     // the plain kernel
    // one workspace for forward and backward: sized for the backward, which includes the forward's parts
    return shared_workspace(d) ? bwd_ws_bytes(d) : align256(forward_mfma_ws_bytes(d));
}
// backward: D first in every layout; on the MFMA path the per-query pairs (lse log2 e, -D) of
// the gathering kernels follow the layout, and with shared key/value heads the per-query-head sums
// of dK and dV come last
size_t bwd_packed_offset(const Dims& d)
{
    return align256(key_major_path(d) ? backward_km_ws_bytes(d) : backward_mfma_ws_bytes(d));
}
size_t bwd_ws_bytes(const Dims& d)
{
    if (!mfma_path(d)) return align256(sizeof(float) * (size_t)d.bh * d.N);
    return bwd_packed_offset(d) + align256(sizeof(float2) * (size_t)d.bh * d.N) + dkdv_heads_ws_bytes(d);
}

}  // namespace

// ---- kernel timing (benchmarks only) -------------------------------------------------------
namespace {
struct ProfileRec { int kernel; hipEvent_t a, b; };
constexpr int kProfileMax = 4096;
std::mutex g_profile_mutex;          // one timing session at a time, whichever threads launch
bool g_profile_on = false;
int g_profile_n = 0;
ProfileRec g_profile[kProfileMax];
}  // namespace

namespace moba {
hipError_t ensure_dynamic_lds(const void* kernel, size_t bytes)
{
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t& have = granted[std::make_pair(kernel, dev)];
    if (bytes <= have) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) have = bytes;
    return e;
}

void profile_mark(int kernel, bool start, hipStream_t st)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (!g_profile_on) return;
    if (start) {
        if (g_profile_n >= kProfileMax) return;
        ProfileRec& r = g_profile[g_profile_n];
        r.kernel = kernel;
        if (hipEventCreate(&r.a) != hipSuccess) return;
        if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
        (void)hipEventRecord(r.a, st);
        ++g_profile_n;
    } else if (g_profile_n > 0 && g_profile[g_profile_n - 1].kernel == kernel) {
        (void)hipEventRecord(g_profile[g_profile_n - 1].b, st);
    }
}

}  // namespace moba

// ---- scratch of the entry point that allocates nothing ------------------------------------------
// moba_topk_static keeps the workspace of moba_topk here.  Every GPU the library runs on holds its
// own copy of the array at its own address until the process ends; in host code the array's name
// is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticScratchBytes = (size_t)MOBA_TOPK_STATIC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once looked up

// device address of this GPU's copy of `scratch` (looked up once per device, with that device
// current); nullptr and *err set when HIP refuses
void* static_scratch(hipError_t* err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int moba_profile_begin(void)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (g_profile_on) return MOBA_EINVAL;
    g_profile_n = 0;
    g_profile_on = true;
    return MOBA_OK;
}

int moba_profile_end(float* ms, int32_t* calls)
{
    std::lock_guard<std::mutex> lock(g_profile_mutex);
    if (!g_profile_on || !ms || !calls) return MOBA_EINVAL;
    g_profile_on = false;
    for (int i = 0; i < MOBA_PROFILE_KERNELS; ++i) { ms[i] = 0.f; calls[i] = 0; }
    int status = MOBA_OK;
    for (int i = 0; i < g_profile_n; ++i) {
        ProfileRec& r = g_profile[i];
        float t = 0.f;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
        if (e == hipSuccess && r.kernel >= 0 && r.kernel < MOBA_PROFILE_KERNELS) {
            ms[r.kernel] += t;
            ++calls[r.kernel];
        } else if (e != hipSuccess) {
            status = MOBA_EHIP;
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_profile_n = 0;
    return status;
}

const char* moba_strerror(int status)
{
    switch (status) {
        case MOBA_OK: return "ok";
        case MOBA_EINVAL: return "invalid argument";
        case MOBA_EUNSUPPORTED: return "shape or option not supported by this build";
        case MOBA_EWORKSPACE: return "workspace missing or too small";
        case MOBA_EHIP: return "HIP call failed";
        default: return "unknown status";
    }
}

int moba_last_hip_error(void) { return g_last_hip_error; }

int moba_routes_per_slice(const moba_shape* shape, int64_t* R)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!R) return MOBA_EINVAL;
    *R = d.R;
    return MOBA_OK;
}

int moba_workspace_bytes(const moba_shape* shape, size_t* topk_ws, size_t* fwd_ws, size_t* bwd_ws)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (topk_ws) *topk_ws = topk_ws_bytes(d);
    if (fwd_ws) *fwd_ws = fwd_ws_bytes(d);
    if (bwd_ws) *bwd_ws = bwd_ws_bytes(d);
    return MOBA_OK;
}

int moba_centroids(const moba_shape* shape, const void* K, const float* conv_w, void* K_eff,
                   float* centroids, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!K || !centroids) return MOBA_EINVAL;
    if ((d.W > 0) != (conv_w != nullptr)) return MOBA_EINVAL;
    if (d.W > 0 && !K_eff) return MOBA_EINVAL;
    // the convolution reads the rows before a run of keys while other lanes already write theirs:
    // not in place
    if (d.W > 1 && K_eff == K) return MOBA_EINVAL;
    return hip_status(launch_centroids(kv_view(d), K, conv_w, K_eff, centroids, (hipStream_t)stream));
}

int moba_key_conv_backward_workspace(const moba_shape* shape, size_t* ws_bytes)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!ws_bytes || d.W < 1) return MOBA_EINVAL;
    *ws_bytes = align256(conv_bwd_ws_bytes(kv_view(d))) + 256;
    return MOBA_OK;
}

int moba_key_conv_backward(const moba_shape* shape, const void* K, const float* conv_w,
                           const void* dK_eff, void* dK, float* dconv_w, void* ws, size_t ws_bytes,
                           void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (d.W < 1 || !K || !conv_w || !dK_eff || !dK || !dconv_w || dK == dK_eff) return MOBA_EINVAL;
    if (!ws || ws_bytes < align256(conv_bwd_ws_bytes(kv_view(d))) + 256) return MOBA_EWORKSPACE;
    return hip_status(launch_conv_backward(kv_view(d), K, conv_w, dK_eff, dK, dconv_w, ws, (hipStream_t)stream));
}

int moba_build_lists(const moba_shape* shape, const int32_t* topk_idx, int32_t* blk_off,
                     int32_t* blk_q, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!blk_off) return MOBA_EINVAL;
    if (d.k > 0 && !topk_idx) return MOBA_EINVAL;
    if (d.R > 0 && !blk_q) return MOBA_EINVAL;
    if (!ws || ws_bytes < topk_ws_bytes(d)) return MOBA_EWORKSPACE;
    return hip_status(launch_build_lists(d, topk_idx, blk_off, blk_q, chunk_counts(d, ws), (hipStream_t)stream));
}

namespace {
int topk_call(const moba_shape* shape, const void* Q, const float* centroids, const int32_t* block_first,
              int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    d.blk_first = block_first;
    if (!Q || !centroids || !blk_off) return MOBA_EINVAL;
    if (d.k > 0 && !topk_idx) return MOBA_EINVAL;
    if (d.R > 0 && !blk_q) return MOBA_EINVAL;
    if (d.n > kMaxBlocks && !topk_mfma_supported(d)) return MOBA_EUNSUPPORTED;   // (the MFMA gate takes four times as many)
    if (!ws || ws_bytes < topk_ws_bytes(d)) return MOBA_EWORKSPACE;
    hipError_t e = topk_mfma_supported(d)
                       ? launch_topk_mfma(d, Q, centroids, topk_idx, topk_terms(d, ws), (hipStream_t)stream)
                       : launch_topk_reference(d, Q, centroids, topk_idx, (hipStream_t)stream);
    if (e != hipSuccess) return hip_status(e);
    return hip_status(launch_build_lists(d, topk_idx, blk_off, blk_q, chunk_counts(d, ws), (hipStream_t)stream));
}
}  // namespace

int moba_topk(const moba_shape* shape, const void* Q, const float* centroids, int32_t* topk_idx,
              int32_t* blk_off, int32_t* blk_q, void* ws, size_t ws_bytes, void* stream)
{
    return topk_call(shape, Q, centroids, nullptr, topk_idx, blk_off, blk_q, ws, ws_bytes, stream);
}

int moba_topk_varlen(const moba_shape* shape, const void* Q, const float* centroids,
                     const int32_t* block_first, int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q,
                     void* ws, size_t ws_bytes, void* stream)
{
    if (!block_first) return MOBA_EINVAL;
    if (shape && shape->batch != 1) return MOBA_EINVAL;          // the batch is folded into the sequences
    return topk_call(shape, Q, centroids, block_first, topk_idx, blk_off, blk_q, ws, ws_bytes, stream);
}

int moba_varlen_layout(int32_t num_seqs, const int32_t* seq_offsets, int32_t block, int32_t* pad_offsets,
                       int32_t* padded_tokens)
{
    if (num_seqs <= 0 || !seq_offsets || block <= 0 || !pad_offsets || !padded_tokens) return MOBA_EINVAL;
    if (seq_offsets[0] != 0) return MOBA_EINVAL;
    int64_t run = 0;
    for (int i = 0; i < num_seqs; ++i) {
        const int64_t len = (int64_t)seq_offsets[i + 1] - seq_offsets[i];
        if (len < 0) return MOBA_EINVAL;
        pad_offsets[i] = (int32_t)run;
        run += (len + block - 1) / block * block;
        if (run > kMaxSeqlen) return MOBA_EUNSUPPORTED;
    }
    pad_offsets[num_seqs] = (int32_t)run;
    *padded_tokens = (int32_t)run;
    return MOBA_OK;
}

namespace {
int varlen_copy(bool pad, int32_t num_seqs, const int32_t* seq_offsets, const int32_t* pad_offsets,
                int32_t slices, int32_t tokens, int32_t padded_tokens, int32_t row_bytes, const void* src,
                void* dst, void* stream)
{
    if (num_seqs <= 0 || !seq_offsets || !pad_offsets || slices <= 0 || tokens < 0 || padded_tokens < tokens)
        return MOBA_EINVAL;
    if (row_bytes <= 0 || (row_bytes & 3) || !src || !dst || src == dst) return MOBA_EINVAL;
    // (the slice is a grid axis of the copy; a slice's words are counted in 32 bits)
    if (slices > 65535 || (int64_t)padded_tokens * (row_bytes / 4) >= ((int64_t)1 << 31)) return MOBA_EUNSUPPORTED;
    return hip_status(launch_varlen_copy(pad, seq_offsets, pad_offsets, num_seqs, slices, tokens, padded_tokens,
                                         row_bytes, src, dst, (hipStream_t)stream));
}
}  // namespace

int moba_varlen_pad(int32_t num_seqs, const int32_t* seq_offsets, const int32_t* pad_offsets, int32_t slices,
                    int32_t tokens, int32_t padded_tokens, int32_t row_bytes, const void* X, void* X_padded,
                    void* stream)
{
    return varlen_copy(true, num_seqs, seq_offsets, pad_offsets, slices, tokens, padded_tokens, row_bytes, X,
                       X_padded, stream);
}

int moba_varlen_unpad(int32_t num_seqs, const int32_t* seq_offsets, const int32_t* pad_offsets, int32_t slices,
                      int32_t tokens, int32_t padded_tokens, int32_t row_bytes, const void* X_padded, void* X,
                      void* stream)
{
    return varlen_copy(false, num_seqs, seq_offsets, pad_offsets, slices, tokens, padded_tokens, row_bytes,
                       X_padded, X, stream);
}

int moba_varlen_block_first(int32_t num_seqs, const int32_t* pad_offsets, int32_t block, int32_t padded_tokens,
                            int32_t* block_first, void* stream)
{
    if (num_seqs <= 0 || !pad_offsets || block <= 0 || padded_tokens < 0 || padded_tokens % block != 0 ||
        !block_first)
        return MOBA_EINVAL;
    return hip_status(launch_varlen_block_first(pad_offsets, num_seqs, block, padded_tokens / block, block_first,
                                                (hipStream_t)stream));
}

int moba_topk_static(const moba_shape* shape, const void* Q, const float* centroids,
                     int32_t* topk_idx, int32_t* blk_off, int32_t* blk_q, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!Q || !centroids || !blk_off) return MOBA_EINVAL;
    if (d.k > 0 && !topk_idx) return MOBA_EINVAL;
    if (d.R > 0 && !blk_q) return MOBA_EINVAL;
    if (d.n > kMaxBlocks && !topk_mfma_supported(d)) return MOBA_EUNSUPPORTED;
    if (topk_ws_bytes(d) > kStaticScratchBytes) return MOBA_EWORKSPACE;
    hipError_t e = hipSuccess;
    void* ws = static_scratch(&e);
    if (!ws) return hip_status(e);
    return moba_topk(shape, Q, centroids, topk_idx, blk_off, blk_q, ws, kStaticScratchBytes, stream);
}

int moba_forward(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                 const int32_t* topk_idx, const int32_t* blk_off, const int32_t* blk_q,
                 void* O, float* lse, void* ws, size_t ws_bytes, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (!Q || !K_eff || !V || !O || !lse || !blk_off) return MOBA_EINVAL;
    if (d.k > 0 && !topk_idx) return MOBA_EINVAL;
    if (d.R > 0 && !blk_q) return MOBA_EINVAL;
    if (!ws || ws_bytes < fwd_ws_bytes(d)) return MOBA_EWORKSPACE;
    if (mfma_path(d) && key_major_path(d))
        return hip_status(launch_forward_km(d, Q, K_eff, V, ws, topk_idx, blk_off, blk_q, O, lse,
                                            (hipStream_t)stream));
    if (mfma_path(d) && tile_forward_ok(d))
        return hip_status(launch_forward_mfma(d, Q, K_eff, V, ws, topk_idx, blk_off, blk_q, O, lse,
                                              (hipStream_t)stream));
    return hip_status(
        launch_forward_reference(d, Q, K_eff, V, topk_idx, O, lse, (hipStream_t)stream));
}

int moba_decode_forward(const moba_shape* shape, int32_t q_len, const void* Q, const void* K_eff,
                        const void* V, const float* centroids, int32_t centroid_blocks, void* O,
                        float* lse, int32_t* topk_idx, void* stream)
{
    Dims d;
    const int st = make_dims(shape, d, true);              // any seqlen: the last block may be ragged
    if (st != MOBA_OK) return st;
    if (q_len <= 0 || q_len > d.N || centroid_blocks < 0) return MOBA_EINVAL;
    if (!Q || !K_eff || !V || !O || !lse) return MOBA_EINVAL;
    const int past_max = (d.N - 1) / d.B;                  // complete blocks before the last query's own
    if (d.k > 0 && past_max > 0 && (!centroids || centroid_blocks < past_max)) return MOBA_EINVAL;
    if (past_max > kMaxBlocks) return MOBA_EUNSUPPORTED;
    return hip_status(launch_decode(d, q_len, Q, K_eff, V, centroids, centroid_blocks, O, lse, topk_idx,
                                    (hipStream_t)stream));
}

int moba_backward_parts(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                        const void* O, const float* lse, const void* dO, const int32_t* topk_idx,
                        const int32_t* blk_off, const int32_t* blk_q,
                        void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes, void* stream,
                        uint32_t parts)
{
    Dims d;
    const int st = make_dims(shape, d);
    if (st != MOBA_OK) return st;
    if (parts == 0 || (parts & ~(uint32_t)MOBA_BWD_ALL)) return MOBA_EINVAL;
    if (!Q || !K_eff || !V || !lse || !dO || !blk_off) return MOBA_EINVAL;
    if ((parts & MOBA_BWD_PREPROCESS) && !O) return MOBA_EINVAL;
    if ((parts & MOBA_BWD_DQ) && !dQ) return MOBA_EINVAL;
    if ((parts & MOBA_BWD_DKDV) && (!dK || !dV)) return MOBA_EINVAL;
    if (d.k > 0 && !topk_idx) return MOBA_EINVAL;
    if (d.R > 0 && !blk_q) return MOBA_EINVAL;
    if (!ws || ws_bytes < bwd_ws_bytes(d)) return MOBA_EWORKSPACE;
    hipStream_t hs = (hipStream_t)stream;
    uint32_t plain = parts;
    if (mfma_path(d)) {
        // D first (plain row-dot kernel), then the MFMA kernels that exist; the rest stays plain
        float2* ld = reinterpret_cast<float2*>(static_cast<char*>(ws) + bwd_packed_offset(d));
        if (parts & MOBA_BWD_PREPROCESS) {
            hipError_t e = launch_backward_reference(d, Q, K_eff, V, O, lse, dO, topk_idx, blk_off, blk_q,
                                                     dQ, dK, dV, (float*)ws, MOBA_BWD_PREPROCESS, ld, hs);
            if (e != hipSuccess) return hip_status(e);
        }
        if (parts & MOBA_BWD_DQ) {
            hipError_t e = key_major_path(d)
                ? launch_dq_km(d, Q, K_eff, V, dO, ld, topk_idx, blk_off, blk_q, dQ, ws, hs)
                : launch_dq_mfma(d, Q, K_eff, V, dO, lse, topk_idx, blk_off, blk_q, dQ, ws, hs);
            if (e != hipSuccess) return hip_status(e);
        }
        if (parts & MOBA_BWD_DKDV) {
            float* part = reinterpret_cast<float*>(reinterpret_cast<char*>(ld) +
                                                   align256(sizeof(float2) * (size_t)d.bh * d.N));
            hipError_t e = launch_dkdv_mfma(d, Q, K_eff, V, dO, ld, blk_off, blk_q,
                                            dK, dV, part, hs);
            if (e != hipSuccess) return hip_status(e);
        }
        return MOBA_OK;
    }
    return hip_status(launch_backward_reference(d, Q, K_eff, V, O, lse, dO, topk_idx, blk_off, blk_q,
                                                dQ, dK, dV, (float*)ws, plain, nullptr, hs));
}

int moba_backward(const moba_shape* shape, const void* Q, const void* K_eff, const void* V,
                  const void* O, const float* lse, const void* dO, const int32_t* topk_idx,
                  const int32_t* blk_off, const int32_t* blk_q, void* dQ,
                  void* dK, void* dV, void* ws, size_t ws_bytes, void* stream)
{
    return moba_backward_parts(shape, Q, K_eff, V, O, lse, dO, topk_idx, blk_off, blk_q, dQ,
                               dK, dV, ws, ws_bytes, stream, MOBA_BWD_ALL);
}

}  // extern "C"
