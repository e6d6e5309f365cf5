// Adapter preparation for slope_spmm_fwd (Eq. 11) with many tokens: T = X L.
//
// The paper concatenates L to the sparse weight so that one vendor SpMM call yields [Y1 | Y2] and
// a second fused GEMM adds Y2 R.  Here the sparse kernel is simply extended by r more k-steps on
// dense MFMA (operands T and R as stored), so only the skinny product T = X L is a kernel of its
// own: the dense tile kernel with a plain epilogue on a k-contiguous copy of L, split over d_in
// while its tiles are too few to fill the chip; it is bound by reading X once.  With up to
// XL_SMALL_MAX_TOKENS tokens the split over d_in in spmm_stream.hip computes T instead, from L as
// stored.
#include "common.h"

namespace {

// out[c][r] = in[r][c] for a bf16 matrix in[rows][cols]; 64 x 64 tiles through LDS.
__global__ void __launch_bounds__(256) transpose_kernel(const bf16_t* __restrict__ in, int rows, int cols,
                                                        bf16_t* __restrict__ out) {
    __shared__ bf16_t tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
    for (int idx = t; idx < 64 * 64; idx += 256) {
        int r = idx >> 6, c = idx & 63;
        tile[r][c] = (r0 + r < rows && c0 + c < cols) ? in[(size_t)(r0 + r) * cols + c0 + c] : (bf16_t)0;
    }
    __syncthreads();
    for (int idx = t; idx < 64 * 64; idx += 256) {
        int c = idx >> 6, r = idx & 63;
        if (r0 + r < rows && c0 + c < cols) out[(size_t)(c0 + c) * rows + r0 + r] = tile[r][c];
    }
}

}  // namespace

hipError_t launch_lowrank_prepare(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, bf16_t* T,
                                  bf16_t* Lt, float* partial_or_null, hipStream_t s) {
    // L[d_in, r] -> Lt[r, d_in]
    transpose_kernel<<<dim3((unsigned)((r + 63) / 64), (unsigned)((d_in + 63) / 64)), dim3(256), 0, s>>>(
        L, (int)d_in, (int)r, Lt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_dense_tn_plain(X, n, Lt, r, d_in, T, partial_or_null, s);   // T[n, r] = X[n, d_in] * Lt[r, d_in]^T
}
