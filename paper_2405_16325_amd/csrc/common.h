// Shared declarations of the gfx950 kernels behind the C ABI in include/slope.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "slope.h"

typedef uint16_t bf16_t;  // raw bf16 bit pattern

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// what slope_last_hip_error() reports for the calling thread
void note_hip_error(hipError_t e);

// Launchers (host side, one per kernel family).  Each returns the hipError_t of its launches.
hipError_t launch_prune_rows(const bf16_t* W, int64_t d_out, int64_t d_in, bf16_t* vals, uint8_t* meta,
                             uint8_t* mask, hipStream_t s);
// largest d_out and d_in of the two calls below: 128 rows of any of their arrays stay below 2^30 bytes, which the
// kernel's 32-bit offsets into a tile's rows rely on
constexpr int64_t DP_EXTENT_MAX = (int64_t)1 << 23;
hipError_t launch_double_prune(const bf16_t* vals, const uint8_t* meta, int64_t d_out, int64_t d_in,
                               bf16_t* valsT, uint8_t* metaT, uint8_t* maskrc, hipStream_t s);
hipError_t launch_update_transposed(const bf16_t* vals, const uint8_t* meta, int64_t d_out, int64_t d_in,
                                    const uint8_t* metaT, bf16_t* valsT, hipStream_t s);
hipError_t launch_sparse_add(const bf16_t* a, const bf16_t* b, size_t count, float beta, float gamma, bf16_t* out,
                             hipStream_t s);
// C[n, m] = B[n, K] * Asparse[m, K]^T  (+ B2[n, |K2|] * A2^T dense: K2 > 0 with A2 = [m][K2], k-contiguous;
// K2 < 0 with A2 = [-K2][m], k-major, the way the adapter factor R is stored)
hipError_t launch_spmm(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                       int64_t K, const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s);
// the choices behind it (pure functions of the shape): tile of the tile kernels (0 x 0 = the generic kernel),
// weight rows per workgroup of the small-batch kernel, chunks of 64 rows of L per workgroup of the X L split
void spmm_tile_choice(int64_t n, int64_t m, int64_t K, int& bm, int& bn);
int spmm_stream_rows(int64_t n, int64_t m, int64_t K);
int xl_subs(int64_t n, int64_t d_in, int64_t r);
// the same product for a few dozen to a few hundred tokens, split over K with fp32 partial sums in `slabs`
// (spmm_slab_bytes of them; 0 = this shape does not take the path)
int spmm_slab_count(int64_t n, int64_t m, int64_t K);
size_t spmm_slab_bytes(int64_t n, int64_t m, int64_t K);
hipError_t launch_spmm_slabs(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                             int64_t K, const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, float* slabs,
                             hipStream_t s);
// the same product for n <= 32 tokens (any K % 64 == 0, K >= 128); adapters as T[n, K2] and R[K2, m] as stored
constexpr int64_t STREAM_MAX_TOKENS = 32;
inline bool spmm_stream_fits(int64_t n, int64_t K) { return n <= STREAM_MAX_TOKENS && K >= 128 && K % 64 == 0; }
// (K % 1024 == 0 and enough rows: the row-split kernel, with the contraction cut into spmm_rows_slices slices when
// there is scratch for the partial sums, spmm_rows_partial_bytes of it; 0 slices = not this kernel)
int spmm_rows_slices(int64_t n, int64_t m, int64_t K, bool with_partial);
size_t spmm_rows_partial_bytes(int64_t n, int64_t m, int64_t K);
hipError_t launch_spmm_stream(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                              int64_t K, const bf16_t* T, const bf16_t* R, int64_t K2, bf16_t* C, float* partial_or_null,
                              hipStream_t s);
// T = X L for few tokens (n <= XL_SMALL_MAX_TOKENS), split over d_in with fp32 partial sums in `scratch`
constexpr int64_t XL_SMALL_MAX_TOKENS = 512;
size_t xl_small_scratch_bytes(int64_t n, int64_t d_in, int64_t r);
hipError_t launch_xl_small(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, float* scratch,
                           bf16_t* T, hipStream_t s);
// T[n, r] = X[n, K] * Lt[r, K]^T (dense tile kernel) for many tokens, with the k-contiguous copy Lt of L
hipError_t launch_lowrank_prepare(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, bf16_t* T,
                                  bf16_t* Lt, float* partial_or_null, hipStream_t s);
// C[n, m] = sum_k B[i sbn + k sbk] * A[j sam + k sak]: any strides and extents, plain fp32 arithmetic (the
// skinny adapter products of layers whose extents are not multiples of 64)
hipError_t launch_plain_gemm(const bf16_t* B, int64_t sbn, int64_t sbk, const bf16_t* A, int64_t sam, int64_t sak,
                             int64_t n, int64_t m, int64_t K, bf16_t* C, hipStream_t s);
hipError_t launch_wgrad_masked(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out,
                               int64_t d_in, bf16_t* gvals, hipStream_t s);
// the same result from token-contiguous copies Xt [d_in][ld], dYt [d_out][ld] (ld = the pitch behind
// token_copy_bytes); launch_token_copies writes one or two such copies (in1 == nullptr: one)
size_t token_copy_bytes(int64_t b, int64_t d);
hipError_t launch_token_copies(const bf16_t* in0, int64_t cols0, bf16_t* out0, const bf16_t* in1, int64_t cols1,
                               bf16_t* out1, int64_t b, hipStream_t s);
bool wgrad_tn_fits(int64_t d_in);
// tail_or_null: wgrad_tail_bytes(b, d_in, d_out) bytes of scratch for cutting the tiles a last partial round
// would hold along the tokens, or nullptr
size_t wgrad_tail_bytes(int64_t b, int64_t d_in, int64_t d_out);
hipError_t launch_wgrad_masked_t(const bf16_t* dYt, const bf16_t* Xt, int64_t b, const uint8_t* meta, int64_t d_out,
                                 int64_t d_in, bf16_t* gvals, float* tail_or_null, hipStream_t s);

// C[n, m] = B[n, K] * A[m, K]^T (dense bf16, fp32 accumulation), K % 64 == 0
size_t dense_tn_plain_partial_bytes(int64_t n, int64_t m);
hipError_t launch_dense_tn_plain(const bf16_t* B, int64_t n, const bf16_t* A, int64_t m, int64_t K, bf16_t* C,
                                 float* partial_or_null, hipStream_t s);
hipError_t launch_dense_tn_any(const bf16_t* B, int64_t n, const bf16_t* A, int64_t m, int64_t K, bf16_t* C,
                               hipStream_t s);
// general N:M magnitude mask (M in {2, 4, 8}); axis 0: groups inside a row, axis 1: inside a column
hipError_t launch_nm_mask(const bf16_t* W, int64_t rows, int64_t cols, int n, int m, int axis, const uint8_t* cand,
                          uint8_t* mask, bf16_t* masked, bf16_t* masked_t, hipStream_t s);
// dW (packed) + dL + dR of a layer with adapters, sharing the token-contiguous copies
size_t wgrad_adapter_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r);
hipError_t launch_wgrad_adapter(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out,
                                int64_t d_in, const bf16_t* L, const bf16_t* R, int64_t r, bf16_t* gvals, bf16_t* dL,
                                bf16_t* dR, void* workspace, hipStream_t s);

// Rank the four keys of a group by (key descending, index ascending) and return the 4-bit
// set of the two winners.  Keys are small non-negative integers.
__device__ __forceinline__ uint32_t top2_of_4(uint32_t k0, uint32_t k1, uint32_t k2, uint32_t k3) {
    // c_ij = 1 when j beats i (strictly larger key); ties leave the lower index in front
    uint32_t c01 = k1 > k0, c02 = k2 > k0, c03 = k3 > k0, c12 = k2 > k1, c13 = k3 > k1, c23 = k3 > k2;
    uint32_t r0 = c01 + c02 + c03;
    uint32_t r1 = (1u - c01) + c12 + c13;
    uint32_t r2 = (2u - c02 - c12) + c23;
    uint32_t r3 = 3u - c03 - c13 - c23;
    return (uint32_t)(r0 < 2u) | ((uint32_t)(r1 < 2u) << 1) | ((uint32_t)(r2 < 2u) << 2) | ((uint32_t)(r3 < 2u) << 3);
}

// Metadata nibble idx0 | idx1 << 2 of a 4-bit set with exactly two members, looked up in a
// 16 x 4-bit table: {0,1}->4 {0,2}->8 {1,2}->9 {0,3}->12 {1,3}->13 {2,3}->14.
__device__ __forceinline__ uint32_t nibble_of_pair(uint32_t set) {
    const uint64_t table = (4ull << 12) | (8ull << 20) | (9ull << 24) | (12ull << 36) | (13ull << 40) | (14ull << 48);
    return (uint32_t)(table >> (4u * set)) & 0xFu;
}
