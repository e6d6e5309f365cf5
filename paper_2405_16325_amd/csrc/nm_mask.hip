// General N:M magnitude masks (Sec. 2.1; the paper's other patterns, e.g. 1:2 and 2:8 of Lemma 2.1)
// for M in {2, 4, 8} and any 1 <= N <= M.  Only 2:4 has a sparse MFMA, so these patterns run as
// masked dense weights ("emulation"): the kernels here emit the bit mask, the masked weight and,
// for the backward operand, its transpose; the products are plain dense tile kernels.
//
// Order inside a group: magnitude (bf16 bits with the sign cleared) descending, index ascending;
// positions outside the optional candidate mask never win and never count (double pruning:
// groups along the other axis, candidates = the first mask).
#include "common.h"

namespace {

// keep bits of one group: score[i] = candidate ? magnitude + 1 : 0
template <int M>
__device__ __forceinline__ uint32_t keep_of_group(const uint32_t (&score)[M], int n) {
    uint32_t keep = 0;
#pragma unroll
    for (int i = 0; i < M; ++i) {
        uint32_t rank = 0;
#pragma unroll
        for (int j = 0; j < M; ++j)
            if (j != i) rank += (score[j] > score[i]) || (score[j] == score[i] && j < i);
        keep |= (uint32_t)(score[i] != 0u && rank < (uint32_t)n) << i;
    }
    return keep;
}

__device__ __forceinline__ uint32_t half_of(const u32x4& v, int e) { return (v[e >> 1] >> (16 * (e & 1))) & 0xFFFFu; }

// groups of M consecutive elements inside a row; one lane = 8 consecutive elements of a row, the lanes of
// a workgroup on consecutive chunks (mask and masked weight only: fully contiguous accesses)
template <int M>
__global__ void __launch_bounds__(256) nm_mask_rows_kernel(const u32x4* __restrict__ W, size_t chunks, int n,
                                                           const uint8_t* __restrict__ cand,
                                                           uint8_t* __restrict__ mask, u32x4* __restrict__ masked) {
    for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += (size_t)gridDim.x * 256) {
        const u32x4 v = W[c];
        const uint32_t cb = cand ? cand[c] : 0xFFu;
        uint32_t keep = 0;
#pragma unroll
        for (int g = 0; g < 8 / M; ++g) {
            uint32_t score[M];
#pragma unroll
            for (int i = 0; i < M; ++i) {
                int e = g * M + i;
                score[i] = ((cb >> e) & 1u) ? (half_of(v, e) & 0x7FFFu) + 1u : 0u;
            }
            keep |= keep_of_group<M>(score, n) << (g * M);
        }
        mask[c] = (uint8_t)keep;
        u32x4 out;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            out[w] = (((keep >> (2 * w)) & 1u) ? (v[w] & 0xFFFFu) : 0u) | (((keep >> (2 * w + 1)) & 1u) ? (v[w] & 0xFFFF0000u) : 0u);
        if (masked) masked[c] = out;
    }
}

// The same with the transposed masked weight as a further output.
// A workgroup takes a tile of 64 columns x 128 rows (thread = chunk tx of 8 columns, rows ty + 32 i);
// the transposed masked weight, if asked for, leaves through LDS in runs of 128 rows per column.
template <int M>
__global__ void __launch_bounds__(256) nm_mask_rows_t_kernel(const bf16_t* __restrict__ W, int rows, int cols, int n,
                                                           const uint8_t* __restrict__ cand,
                                                           uint8_t* __restrict__ mask, bf16_t* __restrict__ masked,
                                                           bf16_t* __restrict__ masked_t) {
    constexpr int TR = 128, PITCH = TR + 2;
    __shared__ bf16_t tile[64 * PITCH];
    const size_t cpr = (size_t)cols / 8;
    const int tx = threadIdx.x & 7, ty = threadIdx.x >> 3;
    const size_t cc = (size_t)blockIdx.x * 8 + tx, r0 = (size_t)blockIdx.y * TR;
#pragma unroll
    for (int i = 0; i < TR / 32; ++i) {
        const size_t row = r0 + ty + 32 * i;
        if (cc >= cpr || row >= (size_t)rows) continue;
        const size_t c = row * cpr + cc;
        const u32x4 v = *(const u32x4*)(W + c * 8);
        const uint32_t cb = cand ? cand[c] : 0xFFu;
        uint32_t keep = 0;
#pragma unroll
        for (int g = 0; g < 8 / M; ++g) {
            uint32_t score[M];
#pragma unroll
            for (int q = 0; q < M; ++q) {
                int e = g * M + q;
                score[q] = ((cb >> e) & 1u) ? (half_of(v, e) & 0x7FFFu) + 1u : 0u;
            }
            keep |= keep_of_group<M>(score, n) << (g * M);
        }
        mask[c] = (uint8_t)keep;
        u32x4 out;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            out[w] = (((keep >> (2 * w)) & 1u) ? (v[w] & 0xFFFFu) : 0u) | (((keep >> (2 * w + 1)) & 1u) ? (v[w] & 0xFFFF0000u) : 0u);
        if (masked) *(u32x4*)(masked + c * 8) = out;
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[(tx * 8 + e) * PITCH + ty + 32 * i] = (bf16_t)half_of(out, e);
    }
    __syncthreads();
    const size_t c0 = (size_t)blockIdx.x * 64;
    for (int idx = threadIdx.x; idx < 64 * TR; idx += 256) {
        const int c = idx / TR, r = idx % TR;
        if (c0 + c >= (size_t)cols || r0 + r >= (size_t)rows) continue;
        masked_t[(c0 + c) * (size_t)rows + r0 + r] = tile[c * PITCH + r];
    }
}

// groups of M consecutive elements inside a column; one lane = 8 consecutive columns x the M rows of a group.
// A workgroup takes a tile of 64 columns x 32 row groups (thread = chunk tx of 8 columns, row group ty),
// so that the transposed masked weight leaves through LDS in runs of 32 M consecutive rows per column
// (lane-sized pieces of 2 M bytes scattered over eight rows of the output made this kernel 3-8 x slower).
template <int M>
__global__ void __launch_bounds__(256) nm_mask_cols_kernel(const bf16_t* __restrict__ W, int rows, int cols, int n,
                                                           const uint8_t* __restrict__ cand,
                                                           uint8_t* __restrict__ mask, bf16_t* __restrict__ masked,
                                                           bf16_t* __restrict__ masked_t) {
    constexpr int TR = 32 * M;                                // rows of a tile
    constexpr int PITCH = TR + 2;                             // elements per column of the transposed tile
    __shared__ bf16_t tile[64 * PITCH];
    const size_t cpr = (size_t)cols / 8;                      // 8-column chunks per row
    const int tx = threadIdx.x & 7, ty = threadIdx.x >> 3;
    const size_t cc = (size_t)blockIdx.x * 8 + tx;            // chunk of 8 columns
    const size_t row0 = ((size_t)blockIdx.y * 32 + ty) * M;   // first row of the group
    const bool live = cc < cpr && row0 < (size_t)rows;        // rows % M == 0: a group is whole or absent
    u32x4 v[M];
    if (live) {
        uint32_t cb[M], keep[M];
#pragma unroll
        for (int k = 0; k < M; ++k) {
            v[k] = *(const u32x4*)(W + (row0 + k) * (size_t)cols + cc * 8);
            cb[k] = cand ? cand[(row0 + k) * cpr + cc] : 0xFFu;
            keep[k] = 0;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t score[M];
#pragma unroll
            for (int k = 0; k < M; ++k) score[k] = ((cb[k] >> e) & 1u) ? (half_of(v[k], e) & 0x7FFFu) + 1u : 0u;
            const uint32_t kg = keep_of_group<M>(score, n);
#pragma unroll
            for (int k = 0; k < M; ++k) keep[k] |= ((kg >> k) & 1u) << e;
        }
#pragma unroll
        for (int k = 0; k < M; ++k) {
            mask[(row0 + k) * cpr + cc] = (uint8_t)keep[k];
            u32x4 out;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                out[w] = (((keep[k] >> (2 * w)) & 1u) ? (v[k][w] & 0xFFFFu) : 0u) |
                         (((keep[k] >> (2 * w + 1)) & 1u) ? (v[k][w] & 0xFFFF0000u) : 0u);
            v[k] = out;
            if (masked) *(u32x4*)(masked + (row0 + k) * (size_t)cols + cc * 8) = out;
        }
    }
    if (!masked_t) return;                                    // uniform
    if (live) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int k = 0; k < M; ++k) tile[(tx * 8 + e) * PITCH + ty * M + k] = (bf16_t)half_of(v[k], e);
    }
    __syncthreads();
    // column c of the tile = TR consecutive elements of row (c0 + c) of the transposed output, two per lane
    const size_t c0 = (size_t)blockIdx.x * 64, r0 = (size_t)blockIdx.y * TR;
    for (int idx = threadIdx.x; idx < 64 * (TR / 2); idx += 256) {
        const int c = idx / (TR / 2), p = idx % (TR / 2);
        if (c0 + c >= (size_t)cols || r0 + 2 * p >= (size_t)rows) continue;      // rows is even
        const uint32_t pair = (uint32_t)tile[c * PITCH + 2 * p] | ((uint32_t)tile[c * PITCH + 2 * p + 1] << 16);
        *(uint32_t*)(masked_t + (c0 + c) * (size_t)rows + r0 + 2 * p) = pair;
    }
}

template <int M>
hipError_t launch_m(const bf16_t* W, int64_t rows, int64_t cols, int n, int axis, const uint8_t* cand, uint8_t* mask,
                    bf16_t* masked, bf16_t* masked_t, hipStream_t s) {
    if (axis == 0 && masked_t)
        nm_mask_rows_t_kernel<M><<<dim3((unsigned)((cols + 63) / 64), (unsigned)((rows + 127) / 128)), dim3(256), 0, s>>>(
            W, (int)rows, (int)cols, n, cand, mask, masked, masked_t);
    else if (axis == 0) {
        const size_t chunks = (size_t)rows * (size_t)(cols / 8);
        size_t blocks = (chunks + 255) / 256;
        if (blocks > 256 * 32) blocks = 256 * 32;
        nm_mask_rows_kernel<M><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const u32x4*)W, chunks, n, cand, mask,
                                                                          (u32x4*)masked);
    } else
        nm_mask_cols_kernel<M><<<dim3((unsigned)((cols + 63) / 64), (unsigned)((rows / M + 31) / 32)), dim3(256), 0, s>>>(
            W, (int)rows, (int)cols, n, cand, mask, masked, masked_t);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_nm_mask(const bf16_t* W, int64_t rows, int64_t cols, int n, int m, int axis, const uint8_t* cand,
                          uint8_t* mask, bf16_t* masked, bf16_t* masked_t, hipStream_t s) {
    if (m == 2) return launch_m<2>(W, rows, cols, n, axis, cand, mask, masked, masked_t, s);
    if (m == 4) return launch_m<4>(W, rows, cols, n, axis, cand, mask, masked, masked_t, s);
    return launch_m<8>(W, rows, cols, n, axis, cand, mask, masked, masked_t, s);
}
