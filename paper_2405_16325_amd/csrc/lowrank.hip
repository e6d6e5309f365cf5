// Adapter preparation for slope_spmm_fwd (Eq. 11): T = X L, and K-contiguous copies of L and R.
//
// The paper concatenates L to the sparse weight so that one vendor SpMM call yields [Y1 | Y2] and
// a second fused GEMM adds Y2 R.  Here the sparse kernel's main loop is simply extended by r more
// k-steps on dense MFMA (operands T and R^T), so only the skinny product T = X L is a kernel of
// its own.  It is bound by reading X once: every wavefront owns 32 tokens and all r columns.
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

// T[n, r] = X[n, K] * Lt[r, K]^T.  One wavefront: 32 tokens x up to 128 columns of T;
// grid.y walks r in chunks of 128.  Operands go straight from global memory into the
// v_mfma_f32_16x16x32_bf16 layout (lane l: row l%16, k = 8*(l/16) .. +7).
__global__ void __launch_bounds__(256) xl_kernel(const bf16_t* __restrict__ X, int n, int K,
                                                 const bf16_t* __restrict__ Lt, int r, bf16_t* __restrict__ T) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int tok0 = (blockIdx.x * 4 + wave) * 32;
    const int c0 = blockIdx.y * 128;
    const int nf = (r - c0 < 128 ? r - c0 : 128) / 16;   // column fragments of this chunk
    if (tok0 >= n) return;
    f32x4 acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const bf16_t* xp[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int row = tok0 + 16 * i + l16;
        row = row < n ? row : n - 1;
        xp[i] = X + (size_t)row * K + lq * 8;
    }
    const bf16_t* lp = Lt + (size_t)(c0 + l16) * K + lq * 8;
    for (int k0 = 0; k0 < K; k0 += 32) {
        union U { uint4 u; bf16x8 v; };
        U x0, x1;
        x0.u = *(const uint4*)(xp[0] + k0);
        x1.u = *(const uint4*)(xp[1] + k0);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < nf) {
                U w;
                w.u = *(const uint4*)(lp + (size_t)(16 * j) * K + k0);
                // D rows = columns of T (so that a lane holds 4 consecutive columns), D columns = tokens
                acc[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.v, x0.v, acc[0][j], 0, 0, 0);
                acc[1][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.v, x1.v, acc[1][j], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int row = tok0 + 16 * i + l16;
        if (row >= n) continue;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < nf) {
                f32x4 v = acc[i][j];
                union { __bf16 h[4]; uint2 u; } o;
                o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
                *(uint2*)(T + (size_t)row * r + c0 + 16 * j + lq * 4) = o.u;
            }
        }
    }
}

}  // namespace

hipError_t launch_lowrank_prepare(const bf16_t* X, int64_t n, int64_t d_in, int64_t d_out, const bf16_t* L,
                                  const bf16_t* R, int64_t r, bf16_t* T, bf16_t* Lt, bf16_t* Rt, hipStream_t s) {
    // L[d_in, r] -> Lt[r, d_in];  R[r, d_out] -> Rt[d_out, r]
    transpose_kernel<<<dim3((unsigned)((r + 63) / 64), (unsigned)((d_in + 63) / 64)), dim3(256), 0, s>>>(
        L, (int)d_in, (int)r, Lt);
    transpose_kernel<<<dim3((unsigned)((d_out + 63) / 64), (unsigned)((r + 63) / 64)), dim3(256), 0, s>>>(
        R, (int)r, (int)d_out, Rt);
    xl_kernel<<<dim3((unsigned)((n + 127) / 128), (unsigned)((r + 127) / 128)), dim3(256), 0, s>>>(
        X, (int)n, (int)d_in, Lt, (int)r, T);
    return hipGetLastError();
}
