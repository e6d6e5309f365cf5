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

// C[i][j] = sum_k B[i * sbn + k * sbk] * A[j * sam + k * sak], bf16 operands with arbitrary element
// strides, fp32 accumulation, bf16 result, C row-major [n][m].  The fallback for the skinny products
// of the adapters when an extent is not a multiple of 64 (the MFMA tile kernels want whole k-steps
// and 16-byte rows): plain fp32 multiply-adds, 32 x 32 outputs per workgroup through LDS, 2 x 2 per
// thread.  Layer shapes of real models never come here.
__global__ void __launch_bounds__(256) plain_gemm_kernel(const bf16_t* __restrict__ B, int64_t sbn, int64_t sbk,
                                                         const bf16_t* __restrict__ A, int64_t sam, int64_t sak, int n,
                                                         int m, int K, bf16_t* __restrict__ C) {
    __shared__ float sB[32][33], sA[32][33];                  // [k][row]
    const int t = threadIdx.x, ti = t >> 4, tj = t & 15;
    const int tiles_m = (m + 31) / 32;
    const int i0 = (int)(blockIdx.x / tiles_m) * 32, j0 = (int)(blockIdx.x % tiles_m) * 32;
    float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    for (int k0 = 0; k0 < K; k0 += 32) {
        for (int idx = t; idx < 32 * 32; idx += 256) {
            // the fast index of the staging loop follows the operand's unit stride
            int a = idx >> 5, c = idx & 31;
            int rb = sbk == 1 ? a : c, kb = sbk == 1 ? c : a;
            int ra = sak == 1 ? a : c, ka = sak == 1 ? c : a;
            float vb = 0.f, va = 0.f;
            if (i0 + rb < n && k0 + kb < K)
                vb = __uint_as_float((uint32_t)B[(int64_t)(i0 + rb) * sbn + (int64_t)(k0 + kb) * sbk] << 16);
            if (j0 + ra < m && k0 + ka < K)
                va = __uint_as_float((uint32_t)A[(int64_t)(j0 + ra) * sam + (int64_t)(k0 + ka) * sak] << 16);
            sB[kb][rb] = vb;
            sA[ka][ra] = va;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            float b0 = sB[k][ti], b1 = sB[k][ti + 16], a0 = sA[k][tj], a1 = sA[k][tj + 16];
            acc[0][0] = __builtin_fmaf(b0, a0, acc[0][0]);
            acc[0][1] = __builtin_fmaf(b0, a1, acc[0][1]);
            acc[1][0] = __builtin_fmaf(b1, a0, acc[1][0]);
            acc[1][1] = __builtin_fmaf(b1, a1, acc[1][1]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 2; ++v) {
            int i = i0 + ti + 16 * u, j = j0 + tj + 16 * v;
            if (i < n && j < m) {
                union { __bf16 h; bf16_t b; } o;
                o.h = (__bf16)acc[u][v];
                C[(int64_t)i * m + j] = o.b;
            }
        }
}

}  // namespace

hipError_t launch_plain_gemm(const bf16_t* B, int64_t sbn, int64_t sbk, const bf16_t* A, int64_t sam, int64_t sak,
                             int64_t n, int64_t m, int64_t K, bf16_t* C, hipStream_t s) {
    const int64_t tiles = ((m + 31) / 32) * ((n + 31) / 32);
    if (tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    plain_gemm_kernel<<<dim3((unsigned)tiles), dim3(256), 0, s>>>(B, sbn, sbk, A, sam, sak, (int)n, (int)m, (int)K, C);
    return hipGetLastError();
}

hipError_t launch_lowrank_prepare(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, bf16_t* T,
                                  bf16_t* Lt, float* partial_or_null, hipStream_t s) {
    // L[d_in, r] -> Lt[r, d_in]
    transpose_kernel<<<dim3((unsigned)((r + 63) / 64), (unsigned)((d_in + 63) / 64)), dim3(256), 0, s>>>(
        L, (int)d_in, (int)r, Lt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_dense_tn_plain(X, n, Lt, r, d_in, T, partial_or_null, s);   // T[n, r] = X[n, d_in] * Lt[r, d_in]^T
}
