// C ABI of the double-pruned 2:4 sparse linear layer (declared in include/slope.h):
// argument checks on the host, then the launchers.  No allocation, no synchronisation; the only
// state is the per-device address of the static scratch array of slope_spmm_fwd_static.
#include <atomic>

#include "pipeline.h"

namespace {

thread_local int g_last_hip_error = 0;

constexpr int64_t EXTENT_MAX = (int64_t)1 << 31;

inline bool misaligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

inline slope_status finish(hipError_t e) {
    if (e == hipSuccess) return SLOPE_OK;
    g_last_hip_error = (int)e;
    return SLOPE_ERR_HIP;
}

inline bool bad_extent(int64_t v, int64_t quantum) { return v <= 0 || v >= EXTENT_MAX || (v % quantum) != 0; }

// b tokens, a d_out x d_in layer: the extents every product call accepts
inline bool bad_layer(int64_t b, int64_t d_out, int64_t d_in) {
    return bad_extent(b, 1) || bad_extent(d_out, 8) || bad_extent(d_in, 8);
}

inline bool bad_rank(int64_t r) { return r % 32 != 0 || r > 512; }

inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// [ T | Lt | partial sums of X L ] when adapters are active, then the slab buffer of the split over K
size_t adapter_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r) {
    (void)d_out;
    if (r <= 0) return 0;
    size_t tiles = round256((size_t)b * r * 2) + round256((size_t)d_in * r * 2);
    // T = X L comes from a split over d_in whose partial sums also live here (none for many tokens)
    return tiles + round256(b <= XL_SMALL_MAX_TOKENS ? xl_small_scratch_bytes(b, d_in, r)
                                                     : dense_tn_plain_partial_bytes(b, r));
}

// T[n, r] = B[n, K] A^T for the skinny products of the adapters.  a_kmajor: A is [K][r] (the factor L as
// stored) instead of [r][K].  Whole k-steps of 64 go to the MFMA kernels, anything else to plain arithmetic.
hipError_t skinny_product(const bf16_t* B, int64_t n, int64_t K, const bf16_t* A, bool a_kmajor, int64_t r, bf16_t* T,
                          bf16_t* At_scratch, float* partial, hipStream_t s) {
    if (K % 64 != 0)
        return a_kmajor ? launch_plain_gemm(B, K, 1, A, 1, r, n, r, K, T, s)
                        : launch_plain_gemm(B, K, 1, A, K, 1, n, r, K, T, s);
    if (a_kmajor) return launch_lowrank_prepare(B, n, K, A, r, T, At_scratch, partial, s);
    return launch_dense_tn_plain(B, n, A, r, K, T, partial, s);
}

}  // namespace

void note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

extern "C" {

int slope_version(void) { return 200; }

int slope_last_hip_error(void) { return g_last_hip_error; }

const char* slope_status_string(int status) {
    switch (status) {
        case SLOPE_OK: return "ok";
        case SLOPE_ERR_NULL: return "a required pointer is NULL";
        case SLOPE_ERR_SHAPE: return "an extent is not positive, not a multiple of its quantum, or too large";
        case SLOPE_ERR_ALIGN: return "a pointer is not sufficiently aligned";
        case SLOPE_ERR_UNSUPPORTED: return "unsupported N:M pattern or adapter rank";
        case SLOPE_ERR_HIP: return "a HIP launch failed";
        case SLOPE_ERR_WORKSPACE: return "the call needs more scratch memory than the buffer it was given holds";
        default: return "unknown status";
    }
}

size_t slope_packed_vals_bytes(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0 || cols % 8) return 0;
    return (size_t)rows * (size_t)(cols / 2) * 2;
}

size_t slope_packed_meta_bytes(int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0 || cols % 8) return 0;
    return (size_t)rows * (size_t)(cols / 8);
}

size_t slope_mask_bytes(int64_t rows, int64_t cols) { return slope_packed_meta_bytes(rows, cols); }

size_t slope_spmm_fwd_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r) {
    if (b <= 0 || d_in <= 0 || d_out <= 0) return 0;
    // the slabs of mid-size batches or the slices of inference-size ones: never both
    return adapter_workspace_bytes(b, d_in, d_out, r) + round256(spmm_slab_bytes(b, d_out, d_in)) +
           round256(spmm_rows_partial_bytes(b, d_out, d_in));
}

size_t slope_token_copy_bytes(int64_t b, int64_t d) {
    if (b <= 0 || d <= 0) return 0;
    return round256(token_copy_bytes(b, d));
}

size_t slope_wgrad_t_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out) {
    if (b <= 0 || d_in <= 0 || d_out <= 0 || !wgrad_tn_fits(d_in)) return 0;
    return wgrad_tail_bytes(b, d_in, d_out);
}

size_t slope_wgrad_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out) {
    if (b <= 0 || d_in <= 0 || d_out <= 0) return 0;
    return slope_token_copy_bytes(b, d_in) + slope_token_copy_bytes(b, d_out) + slope_wgrad_t_workspace_bytes(b, d_in, d_out);
}

size_t slope_spmm_bwd_x_adapter_workspace_bytes(int64_t b, int64_t r) {
    if (b <= 0 || r <= 0) return 0;
    return round256((size_t)b * r * 2) + round256(dense_tn_plain_partial_bytes(b, r));
}

size_t slope_wgrad_adapter_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r) {
    if (b <= 0 || d_in <= 0 || d_out <= 0 || r <= 0) return 0;
    return round256(wgrad_adapter_workspace_bytes(b, d_in, d_out, r));
}

size_t slope_workspace_bytes(int call_id, int64_t b, int64_t d_in, int64_t d_out, int64_t r) {
    switch (call_id) {
        case SLOPE_CALL_SPMM_FWD: return slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r);
        case SLOPE_CALL_WGRAD_MASKED_WS: return slope_wgrad_workspace_bytes(b, d_in, d_out);
        case SLOPE_CALL_WGRAD_MASKED_T: return slope_wgrad_t_workspace_bytes(b, d_in, d_out);
        case SLOPE_CALL_SPMM_BWD_X_ADAPTER: return slope_spmm_bwd_x_adapter_workspace_bytes(b, r);
        case SLOPE_CALL_WGRAD_ADAPTER: return slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r);
        default: return 0;      // prune_rows, double_prune, spmm_bwd_x, wgrad_masked need no scratch; unknown ids
    }
}

slope_status slope_prune_rows(const void* W, int64_t d_out, int64_t d_in, int n, int m, void* Wr_vals, void* Wr_meta,
                              void* mask_or_null, void* stream) {
    if (!W || !Wr_vals || !Wr_meta) return SLOPE_ERR_NULL;
    if (n != 2 || m != 4) return SLOPE_ERR_UNSUPPORTED;
    if (bad_extent(d_out, 1) || bad_extent(d_in, 8)) return SLOPE_ERR_SHAPE;
    if (misaligned(W, 16) || misaligned(Wr_vals, 16) || misaligned(Wr_meta, 16) || misaligned(mask_or_null, 16))
        return SLOPE_ERR_ALIGN;
    return finish(launch_prune_rows((const bf16_t*)W, d_out, d_in, (bf16_t*)Wr_vals, (uint8_t*)Wr_meta,
                                    (uint8_t*)mask_or_null, (hipStream_t)stream));
}

slope_status slope_double_prune(const void* Wr_vals, const void* Wr_meta, int64_t d_out, int64_t d_in,
                                void* WrcT_vals, void* WrcT_meta, void* maskrc_or_null, void* stream) {
    if (!Wr_vals || !Wr_meta || !WrcT_vals || !WrcT_meta) return SLOPE_ERR_NULL;
    if (bad_extent(d_out, 8) || bad_extent(d_in, 8) || d_out > DP_EXTENT_MAX || d_in > DP_EXTENT_MAX)
        return SLOPE_ERR_SHAPE;
    if (misaligned(Wr_vals, 16) || misaligned(Wr_meta, 16) || misaligned(WrcT_vals, 16) ||
        misaligned(WrcT_meta, 16) || misaligned(maskrc_or_null, 16))
        return SLOPE_ERR_ALIGN;
    return finish(launch_double_prune((const bf16_t*)Wr_vals, (const uint8_t*)Wr_meta, d_out, d_in,
                                      (bf16_t*)WrcT_vals, (uint8_t*)WrcT_meta, (uint8_t*)maskrc_or_null,
                                      (hipStream_t)stream));
}

// Argument checks of the three forms of slope_spmm_fwd, up to the scratch buffer.
static slope_status spmm_fwd_check(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta, int64_t d_out,
                                   int64_t d_in, const void* L_or_null, const void* R_or_null, int64_t r, void* Y) {
    if (!X || !Wr_vals || !Wr_meta || !Y) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in)) return SLOPE_ERR_SHAPE;
    if (r < 0) return SLOPE_ERR_SHAPE;
    if (r > 0 && (L_or_null || R_or_null)) {
        if (!L_or_null || !R_or_null) return SLOPE_ERR_NULL;
        if (bad_rank(r)) return SLOPE_ERR_UNSUPPORTED;
        if (misaligned(L_or_null, 16) || misaligned(R_or_null, 16)) return SLOPE_ERR_ALIGN;
    }
    if (misaligned(X, 16) || misaligned(Wr_vals, 16) || misaligned(Wr_meta, 16) || misaligned(Y, 16))
        return SLOPE_ERR_ALIGN;
    return SLOPE_OK;
}

// The launches of slope_spmm_fwd; arguments are checked, `workspace` (if any) has
// slope_spmm_fwd_workspace_bytes(b, d_in, d_out, r) bytes.
static slope_status spmm_fwd_run(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta, int64_t d_out,
                                 int64_t d_in, const void* L_or_null, const void* R_or_null, int64_t r, void* Y,
                                 void* workspace, void* stream) {
    const bool adapter = r > 0 && (L_or_null || R_or_null);
    hipStream_t s = (hipStream_t)stream;
    const bf16_t* x = (const bf16_t*)X;
    const bf16_t* wv = (const bf16_t*)Wr_vals;
    const uint8_t* wm = (const uint8_t*)Wr_meta;
    uint8_t* ws = (uint8_t*)workspace;
    bf16_t* T = (bf16_t*)ws;
    if (adapter) {                                            // T = X L, rounded to bf16
        bf16_t* Lt = (bf16_t*)(ws + round256((size_t)b * r * 2));
        float* partial = (float*)((uint8_t*)Lt + round256((size_t)d_in * r * 2));
        hipError_t e;
        if (d_in % 64 == 0 && b <= XL_SMALL_MAX_TOKENS)       // too few tokens for the tile kernel to spread X L over the chip
            e = launch_xl_small(x, b, d_in, (const bf16_t*)L_or_null, r, partial, T, s);
        else
            e = skinny_product(x, b, d_in, (const bf16_t*)L_or_null, true, r, T, Lt,
                               b > XL_SMALL_MAX_TOKENS && dense_tn_plain_partial_bytes(b, r) ? partial : nullptr, s);
        if (e != hipSuccess) return finish(e);
    }
    if (spmm_stream_fits(b, d_in)) {                          // inference-size batch: one HBM-bound pass over the packed weight
        float* slices = workspace && spmm_rows_partial_bytes(b, d_out, d_in)
                            ? (float*)(ws + adapter_workspace_bytes(b, d_in, d_out, adapter ? r : 0)) : nullptr;
        return finish(launch_spmm_stream(x, b, wv, wm, d_out, d_in, adapter ? T : nullptr,
                                         adapter ? (const bf16_t*)R_or_null : nullptr, adapter ? r : 0, (bf16_t*)Y,
                                         slices, s));
    }
    // With scratch memory a batch of a few dozen to a few hundred tokens is split over K as well.
    float* slabs = workspace && spmm_slab_count(b, d_out, d_in) > 0
                       ? (float*)(ws + adapter_workspace_bytes(b, d_in, d_out, adapter ? r : 0)) : nullptr;
    const bf16_t* B2 = adapter ? T : nullptr;
    const bf16_t* A2 = adapter ? (const bf16_t*)R_or_null : nullptr;   // as stored, [r][d_out]: the kernels take it k-major
    const int64_t K2 = adapter ? -r : 0;
    if (slabs) return finish(launch_spmm_slabs(x, b, wv, wm, d_out, d_in, B2, A2, K2, (bf16_t*)Y, slabs, s));
    return finish(launch_spmm(x, b, wv, wm, d_out, d_in, B2, A2, K2, (bf16_t*)Y, s));
}

slope_status slope_spmm_fwd(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta, int64_t d_out,
                            int64_t d_in, const void* L_or_null, const void* R_or_null, int64_t r, void* Y,
                            void* workspace, void* stream) {
    slope_status st = spmm_fwd_check(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y);
    if (st != SLOPE_OK) return st;
    if (r > 0 && (L_or_null || R_or_null) && !workspace) return SLOPE_ERR_NULL;
    if (misaligned(workspace, 256)) return SLOPE_ERR_ALIGN;
    return spmm_fwd_run(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y, workspace, stream);
}

slope_status slope_spmm_fwd_ws(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta, int64_t d_out,
                               int64_t d_in, const void* L_or_null, const void* R_or_null, int64_t r, void* Y,
                               void* workspace, size_t workspace_bytes, void* stream) {
    slope_status st = spmm_fwd_check(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y);
    if (st != SLOPE_OK) return st;
    const bool adapter = r > 0 && (L_or_null || R_or_null);
    if (adapter && !workspace) return SLOPE_ERR_NULL;
    if (misaligned(workspace, 256)) return SLOPE_ERR_ALIGN;
    if (workspace && workspace_bytes < slope_spmm_fwd_workspace_bytes(b, d_in, d_out, adapter ? r : 0))
        return SLOPE_ERR_WORKSPACE;
    return spmm_fwd_run(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y, workspace, stream);
}

// ---- slope_spmm_fwd_static: the same call on a scratch buffer that lives in the library's image.
// `scratch` below is the host-side stand-in of the device array: its device address differs from
// GPU to GPU and is looked up once per device with hipGetSymbolAddress; only that address is ever
// handed to a kernel.
static __device__ __align__(256) unsigned char scratch[SLOPE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

// Device address of `scratch` on the current device (first call per device asks the runtime).
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // racing first calls store the same address
    }
    *out = p;
    return hipSuccess;
}
}  // namespace

slope_status slope_spmm_fwd_static(const void* X, int64_t b, const void* Wr_vals, const void* Wr_meta, int64_t d_out,
                                   int64_t d_in, const void* L_or_null, const void* R_or_null, int64_t r, void* Y,
                                   void* stream) {
    slope_status st = spmm_fwd_check(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y);
    if (st != SLOPE_OK) return st;
    const bool adapter = r > 0 && (L_or_null || R_or_null);
    const size_t need = slope_spmm_fwd_workspace_bytes(b, d_in, d_out, adapter ? r : 0);
    if (need > (size_t)SLOPE_STATIC_SCRATCH_BYTES) return SLOPE_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        hipError_t e = static_scratch(&ws);
        if (e != hipSuccess) return finish(e);
    }
    // Nothing in the buffer has to start at zero: every partial sum that is read was written by this
    // call's own kernels first.
    return spmm_fwd_run(X, b, Wr_vals, Wr_meta, d_out, d_in, L_or_null, R_or_null, r, Y, ws, stream);
}

slope_status slope_spmm_bwd_x(const void* dY, int64_t b, const void* WrcT_vals, const void* WrcT_meta, int64_t d_out,
                              int64_t d_in, void* dX, void* stream) {
    if (!dY || !WrcT_vals || !WrcT_meta || !dX) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in)) return SLOPE_ERR_SHAPE;
    if (misaligned(dY, 16) || misaligned(WrcT_vals, 16) || misaligned(WrcT_meta, 16) || misaligned(dX, 16))
        return SLOPE_ERR_ALIGN;
    // sparse rows = d_in, contraction over d_out
    if (spmm_stream_fits(b, d_out))
        return finish(launch_spmm_stream((const bf16_t*)dY, b, (const bf16_t*)WrcT_vals, (const uint8_t*)WrcT_meta,
                                         d_in, d_out, nullptr, nullptr, 0, (bf16_t*)dX, nullptr, (hipStream_t)stream));
    return finish(launch_spmm((const bf16_t*)dY, b, (const bf16_t*)WrcT_vals, (const uint8_t*)WrcT_meta, d_in, d_out,
                              nullptr, nullptr, 0, (bf16_t*)dX, (hipStream_t)stream));
}

slope_status slope_wgrad_masked(const void* dY, const void* X, int64_t b, const void* Wr_meta, int64_t d_out,
                                int64_t d_in, void* dW_vals, void* stream) {
    if (!dY || !X || !Wr_meta || !dW_vals) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in)) return SLOPE_ERR_SHAPE;
    if (misaligned(dY, 16) || misaligned(X, 16) || misaligned(Wr_meta, 16) || misaligned(dW_vals, 16))
        return SLOPE_ERR_ALIGN;
    return finish(launch_wgrad_masked((const bf16_t*)dY, (const bf16_t*)X, b, (const uint8_t*)Wr_meta, d_out, d_in,
                                      (bf16_t*)dW_vals, (hipStream_t)stream));
}

slope_status slope_wgrad_masked_ws(const void* dY, const void* X, int64_t b, const void* Wr_meta, int64_t d_out,
                                   int64_t d_in, void* dW_vals, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    if (!dY || !X || !Wr_meta || !dW_vals || !workspace) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in)) return SLOPE_ERR_SHAPE;
    if (misaligned(dY, 16) || misaligned(X, 16) || misaligned(Wr_meta, 16) || misaligned(dW_vals, 16) ||
        misaligned(workspace, 256))
        return SLOPE_ERR_ALIGN;
    if (workspace_bytes < slope_wgrad_workspace_bytes(b, d_in, d_out)) return SLOPE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    if (!wgrad_tn_fits(d_in))                                 // the packed epilogue of the tile kernels reads metadata by dwords
        return finish(launch_wgrad_masked((const bf16_t*)dY, (const bf16_t*)X, b, (const uint8_t*)Wr_meta, d_out, d_in,
                                          (bf16_t*)dW_vals, s));
    bf16_t* Xt = (bf16_t*)workspace;
    bf16_t* dYt = (bf16_t*)((uint8_t*)workspace + slope_token_copy_bytes(b, d_in));
    float* tail = slope_wgrad_t_workspace_bytes(b, d_in, d_out)
                      ? (float*)((uint8_t*)workspace + slope_token_copy_bytes(b, d_in) + slope_token_copy_bytes(b, d_out))
                      : nullptr;
    hipError_t e = launch_token_copies((const bf16_t*)X, d_in, Xt, (const bf16_t*)dY, d_out, dYt, b, s);
    if (e != hipSuccess) return finish(e);
    return finish(launch_wgrad_masked_t(dYt, Xt, b, (const uint8_t*)Wr_meta, d_out, d_in, (bf16_t*)dW_vals, tail, s));
}

slope_status slope_transpose_tokens(const void* A, int64_t b, int64_t d, void* At, size_t At_bytes, void* stream) {
    if (!A || !At) return SLOPE_ERR_NULL;
    if (bad_extent(b, 1) || bad_extent(d, 8)) return SLOPE_ERR_SHAPE;
    if (misaligned(A, 16) || misaligned(At, 256)) return SLOPE_ERR_ALIGN;
    if (At_bytes < slope_token_copy_bytes(b, d)) return SLOPE_ERR_WORKSPACE;
    return finish(launch_token_copies((const bf16_t*)A, d, (bf16_t*)At, nullptr, 0, nullptr, b, (hipStream_t)stream));
}

slope_status slope_wgrad_masked_t(const void* dYt, const void* Xt, int64_t b, const void* Wr_meta, int64_t d_out,
                                  int64_t d_in, void* dW_vals, void* workspace_or_null, size_t workspace_bytes,
                                  void* stream) {
    if (!dYt || !Xt || !Wr_meta || !dW_vals) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in) || !wgrad_tn_fits(d_in)) return SLOPE_ERR_SHAPE;
    if (misaligned(dYt, 256) || misaligned(Xt, 256) || misaligned(Wr_meta, 16) || misaligned(dW_vals, 16) ||
        misaligned(workspace_or_null, 256))
        return SLOPE_ERR_ALIGN;
    const size_t need = slope_wgrad_t_workspace_bytes(b, d_in, d_out);
    if (workspace_or_null && workspace_bytes < need) return SLOPE_ERR_WORKSPACE;
    return finish(launch_wgrad_masked_t((const bf16_t*)dYt, (const bf16_t*)Xt, b, (const uint8_t*)Wr_meta, d_out, d_in,
                                        (bf16_t*)dW_vals, need ? (float*)workspace_or_null : nullptr,
                                        (hipStream_t)stream));
}

slope_status slope_spmm_bwd_x_adapter(const void* dY, int64_t b, const void* WrcT_vals, const void* WrcT_meta,
                                      int64_t d_out, int64_t d_in, const void* L, const void* R, int64_t r, void* dX,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    if (!dY || !WrcT_vals || !WrcT_meta || !dX || !L || !R || !workspace) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in) || r <= 0) return SLOPE_ERR_SHAPE;
    if (bad_rank(r)) return SLOPE_ERR_UNSUPPORTED;
    if (misaligned(dY, 16) || misaligned(WrcT_vals, 16) || misaligned(WrcT_meta, 16) || misaligned(dX, 16) ||
        misaligned(L, 16) || misaligned(R, 16) || misaligned(workspace, 256))
        return SLOPE_ERR_ALIGN;
    if (workspace_bytes < slope_spmm_bwd_x_adapter_workspace_bytes(b, r)) return SLOPE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    bf16_t* T2 = (bf16_t*)workspace;                          // dY R^T, bf16[b, r]
    float* partial = dense_tn_plain_partial_bytes(b, r)
                         ? (float*)((uint8_t*)workspace + round256((size_t)b * r * 2)) : nullptr;
    hipError_t e = skinny_product((const bf16_t*)dY, b, d_out, (const bf16_t*)R, false, r, T2, nullptr, partial, s);
    if (e != hipSuccess) return finish(e);
    // sparse rows = d_in, contraction over d_out, then r more k-steps on T2 and L (K-contiguous as stored)
    return finish(launch_spmm((const bf16_t*)dY, b, (const bf16_t*)WrcT_vals, (const uint8_t*)WrcT_meta, d_in, d_out,
                              T2, (const bf16_t*)L, r, (bf16_t*)dX, s));
}

slope_status slope_wgrad_adapter(const void* dY, const void* X, int64_t b, const void* Wr_meta, int64_t d_out,
                                 int64_t d_in, const void* L, const void* R, int64_t r, void* dW_vals, void* dL,
                                 void* dR, void* workspace, size_t workspace_bytes, void* stream) {
    if (!dY || !X || !Wr_meta || !dW_vals || !L || !R || !dL || !dR || !workspace) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in) || r <= 0) return SLOPE_ERR_SHAPE;
    if (bad_rank(r)) return SLOPE_ERR_UNSUPPORTED;
    if (misaligned(dY, 16) || misaligned(X, 16) || misaligned(Wr_meta, 16) || misaligned(dW_vals, 16) ||
        misaligned(L, 16) || misaligned(R, 16) || misaligned(dL, 16) || misaligned(dR, 16) ||
        misaligned(workspace, 256))
        return SLOPE_ERR_ALIGN;
    if (workspace_bytes < slope_wgrad_adapter_workspace_bytes(b, d_in, d_out, r)) return SLOPE_ERR_WORKSPACE;
    return finish(launch_wgrad_adapter((const bf16_t*)dY, (const bf16_t*)X, b, (const uint8_t*)Wr_meta, d_out, d_in,
                                       (const bf16_t*)L, (const bf16_t*)R, r, (bf16_t*)dW_vals, (bf16_t*)dL,
                                       (bf16_t*)dR, workspace, (hipStream_t)stream));
}

slope_status slope_prune_mask(const void* W, int64_t rows, int64_t cols, int n, int m, int axis,
                              const void* candidates_or_null, void* mask_out, void* masked_out_or_null,
                              void* masked_t_out_or_null, void* stream) {
    if (!W || !mask_out) return SLOPE_ERR_NULL;
    if ((m != 2 && m != 4 && m != 8) || n < 1 || n > m || (axis != 0 && axis != 1)) return SLOPE_ERR_UNSUPPORTED;
    if (bad_extent(rows, axis == 1 ? m : 1) || bad_extent(cols, 8)) return SLOPE_ERR_SHAPE;
    if (misaligned(W, 16) || misaligned(masked_out_or_null, 16) || misaligned(masked_t_out_or_null, 16) ||
        misaligned(mask_out, 16) || misaligned(candidates_or_null, 16))
        return SLOPE_ERR_ALIGN;
    return finish(launch_nm_mask((const bf16_t*)W, rows, cols, n, m, axis, (const uint8_t*)candidates_or_null,
                                 (uint8_t*)mask_out, (bf16_t*)masked_out_or_null, (bf16_t*)masked_t_out_or_null,
                                 (hipStream_t)stream));
}

slope_status slope_gemm_tn(const void* B, int64_t n, const void* A, int64_t m, int64_t K, void* C, void* stream) {
    if (!B || !A || !C) return SLOPE_ERR_NULL;
    if (bad_extent(n, 1) || bad_extent(m, 4) || bad_extent(K, 64)) return SLOPE_ERR_SHAPE;
    if (misaligned(B, 16) || misaligned(A, 16) || misaligned(C, 16)) return SLOPE_ERR_ALIGN;
    return finish(launch_dense_tn_any((const bf16_t*)B, n, (const bf16_t*)A, m, K, (bf16_t*)C, (hipStream_t)stream));
}

slope_status slope_sparse_add(const void* A_vals, const void* B_vals, int64_t rows, int64_t cols, float beta,
                              float gamma, void* out_vals, void* stream) {
    if (!A_vals || !B_vals || !out_vals) return SLOPE_ERR_NULL;
    if (bad_extent(rows, 1) || bad_extent(cols, 8)) return SLOPE_ERR_SHAPE;
    if (misaligned(A_vals, 16) || misaligned(B_vals, 16) || misaligned(out_vals, 16)) return SLOPE_ERR_ALIGN;
    return finish(launch_sparse_add((const bf16_t*)A_vals, (const bf16_t*)B_vals, (size_t)rows * (size_t)(cols / 2),
                                    beta, gamma, (bf16_t*)out_vals, (hipStream_t)stream));
}

slope_status slope_update_sparse(const void* Wnew_vals, const void* Wr_meta, int64_t d_out, int64_t d_in,
                                 void* Wr_vals, const void* WrcT_meta, void* WrcT_vals, void* stream) {
    if (!Wnew_vals || !Wr_meta || !Wr_vals || !WrcT_meta || !WrcT_vals) return SLOPE_ERR_NULL;
    if (bad_extent(d_out, 8) || bad_extent(d_in, 8) || d_out > DP_EXTENT_MAX || d_in > DP_EXTENT_MAX)
        return SLOPE_ERR_SHAPE;
    if (misaligned(Wnew_vals, 16) || misaligned(Wr_meta, 16) || misaligned(Wr_vals, 16) ||
        misaligned(WrcT_meta, 16) || misaligned(WrcT_vals, 16))
        return SLOPE_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (Wr_vals != Wnew_vals) {
        hipError_t e = hipMemcpyAsync(Wr_vals, Wnew_vals, (size_t)d_out * (size_t)(d_in / 2) * 2,
                                      hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return finish(e);
    }
    return finish(launch_update_transposed((const bf16_t*)Wnew_vals, (const uint8_t*)Wr_meta, d_out, d_in,
                                           (const uint8_t*)WrcT_meta, (bf16_t*)WrcT_vals, s));
}

slope_status slope_spmm_fwd_plan(int64_t b, int64_t d_in, int64_t d_out, int64_t r, int with_workspace, int32_t* plan) {
    if (!plan) return SLOPE_ERR_NULL;
    if (bad_layer(b, d_out, d_in) || r < 0) return SLOPE_ERR_SHAPE;
    if (r > 0 && bad_rank(r)) return SLOPE_ERR_UNSUPPORTED;
    for (int i = 0; i < 6; ++i) plan[i] = 0;
    plan[3] = 1;
    if (spmm_stream_fits(b, d_in)) {
        const int slices = spmm_rows_slices(b, d_out, d_in, with_workspace != 0);
        plan[0] = slices > 0 ? 4 : 0;
        plan[1] = slices > 0 ? 48 : spmm_stream_rows(b, d_out, d_in);
        plan[2] = b <= 16 ? 16 : 32;
        if (slices > 0) plan[3] = slices;
    } else {
        const int slabs = with_workspace ? spmm_slab_count(b, d_out, d_in) : 0;
        int bm, bn;
        spmm_tile_choice(b, d_out, d_in, bm, bn);
        if (slabs > 0) { plan[0] = 1; plan[1] = 256; plan[2] = b <= 64 ? 64 : 128; plan[3] = slabs; }
        else if (bm == 0) { plan[0] = 3; plan[1] = plan[2] = 128; }
        else { plan[0] = 2; plan[1] = bm; plan[2] = bn; }
    }
    if (r > 0) {
        if (d_in % 64 != 0) {
            plan[4] = 4;
        } else if (b <= XL_SMALL_MAX_TOKENS) {
            plan[4] = 1;
            plan[5] = xl_subs(b, d_in, r);
        } else {
            plan[4] = dense_tn_plain_partial_bytes(b, r) ? 3 : 2;
        }
    }
    return SLOPE_OK;
}

int64_t slope_tile_order(int64_t tiles_m, int64_t tiles_n, int32_t* tm, int32_t* tn, int64_t capacity) {
    if (tiles_m <= 0 || tiles_n <= 0 || tiles_m > (1 << 20) || tiles_n > (1 << 20) || !tm || !tn) return -1;
    const int64_t grid = super_grid((int)tiles_m, (int)tiles_n);
    if (capacity < grid) return -1;
    for (int64_t w = 0; w < grid; ++w) {
        int a = -1, b = -1;
        if (!tile_of_index((int)w, (int)tiles_m, (int)tiles_n, a, b)) a = b = -1;
        tm[w] = a;
        tn[w] = b;
    }
    return grid;
}

}  // extern "C"
