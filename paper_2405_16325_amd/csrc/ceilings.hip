// Micro-benchmarks behind slope_ceiling: what the chip delivers to the simplest possible kernel of
// each kind, measured in the same run and under the same power management as the library's kernels.
//   MFMA loops: operands stay in registers, every wavefront issues independent matrix instructions
//   back to back (16 accumulators), so nothing but the matrix pipe and the clock it is allowed
//   bounds them.  The operands are read once from the caller's buffer: with random data the pipe
//   draws the power it draws in a real product, with zeros far less, and the clock follows.
//   Streams: a read-only pass (one 16-byte load per lane per step, a sum kept alive by one store per
//   lane at the end) and a copy of the first half of the buffer onto the second half.
#include "pipeline.h"

namespace {

constexpr int CEIL_ACC = 16;          // independent accumulators per wavefront

typedef __attribute__((ext_vector_type(16))) float f32x16;

// the 32 x 32 forms of the same instructions (four independent 16-register accumulators per wavefront):
// kind 0: v_smfmac_f32_32x32x32_bf16 (2 * 32 * 32 * 32 dense-equivalent flops each)
// kind 1: v_mfma_f32_32x32x16_bf16   (2 * 32 * 32 * 16 flops each)
template <int KIND>
__global__ void __launch_bounds__(256) mfma32_loop_kernel(const u32x4* __restrict__ src, int iters, float* __restrict__ sink) {
    const int t = threadIdx.x, g = blockIdx.x * 256 + t;
    AFrag a[4];
    BFrag b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = src[(size_t)g * 12 + i];
        b[i].u[0] = src[(size_t)g * 12 + 4 + 2 * i];
        b[i].u[1] = src[(size_t)g * 12 + 5 + 2 * i];
    }
    const int idx = 0xD8E4;
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (KIND == 0) {
                    acc[i] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a[(i + r) & 3].v, b[i].v, acc[i], idx, 0, 0);
                } else {
                    AFrag bb;
                    bb.u = b[i].u[r];
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + r) & 3].v, bb.v, acc[i], 0, 0, 0);
                }
            }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    sink[g] = s;
}

// kind 0: v_smfmac_f32_16x16x64_bf16 (2 * 16 * 16 * 64 dense-equivalent flops each)
// kind 1: v_mfma_f32_16x16x32_bf16   (2 * 16 * 16 * 32 flops each)
template <int KIND>
__global__ void __launch_bounds__(256) mfma_loop_kernel(const u32x4* __restrict__ src, int iters, float* __restrict__ sink) {
    const int t = threadIdx.x, g = blockIdx.x * 256 + t;
    AFrag a[4];
    BFrag b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = src[(size_t)g * 12 + i];
        b[i].u[0] = src[(size_t)g * 12 + 4 + 2 * i];
        b[i].u[1] = src[(size_t)g * 12 + 5 + 2 * i];
    }
    // metadata nibbles that name two distinct ascending positions whatever the data: 0x4 (0, 1), 0xE (2, 3), 0x8 (0, 2), 0xD (1, 3)
    const int idx = 0xD8E4;
    f32x4 acc[CEIL_ACC];
#pragma unroll
    for (int i = 0; i < CEIL_ACC; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < CEIL_ACC; ++i) {
            if (KIND == 0) {
                acc[i] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a[i & 3].v, b[i >> 2].v, acc[i], idx, 0, 0);
            } else {
                AFrag bb;
                bb.u = b[i >> 2].u[0];
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3].v, bb.v, acc[i], 0, 0, 0);
            }
        }
    }
    f32x4 s = acc[0];
#pragma unroll
    for (int i = 1; i < CEIL_ACC; ++i) { s[0] += acc[i][0]; s[1] += acc[i][1]; s[2] += acc[i][2]; s[3] += acc[i][3]; }
    sink[g] = s[0] + s[1] + s[2] + s[3];
}

// One 16-byte vector per lane and no loop: workgroups that come and go in address order keep the accesses in
// flight close together, which is what the memory likes best (a grid-stride loop over the same data, every lane
// walking through windows far apart, reads 5.6 instead of 7.0 TB/s and copies 4.5 instead of 6.5).
__global__ void __launch_bounds__(256) read_stream_kernel(const u32x4* __restrict__ src, size_t nvec, uint32_t* __restrict__ sink) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= nvec) return;
    const u32x4 v = __builtin_nontemporal_load(src + i);
    if ((v[0] ^ v[1] ^ v[2] ^ v[3]) == 0x9E3779B9u) sink[threadIdx.x] = v[0];   // keeps the load; (almost) never taken
}

__global__ void __launch_bounds__(256) copy_stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t nvec) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

constexpr int CEIL_BLOCKS = 256 * 4;  // four workgroups of four wavefronts per compute unit

}  // namespace

extern "C" {

// bytes the buffer must have for the MFMA kinds: operands of every lane plus one float per lane
size_t slope_ceiling_min_bytes(void) { return (size_t)CEIL_BLOCKS * 256 * (12 * 16 + 4); }

slope_status slope_ceiling(int kind, void* buf, size_t bytes, int iters, double* work, void* stream) {
    if (!buf || !work) return SLOPE_ERR_NULL;
    if (((uintptr_t)buf & 255) != 0) return SLOPE_ERR_ALIGN;
    if (iters <= 0 || bytes < slope_ceiling_min_bytes()) return SLOPE_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    const size_t lanes = (size_t)CEIL_BLOCKS * 256;
    float* sink = (float*)((uint8_t*)buf + lanes * 12 * 16);
    switch (kind) {
        case SLOPE_CEILING_SPARSE_MFMA:
            mfma_loop_kernel<0><<<dim3(CEIL_BLOCKS), dim3(256), 0, s>>>((const u32x4*)buf, iters, sink);
            *work = (double)(lanes / 64) * iters * CEIL_ACC * 2.0 * 16 * 16 * 64;
            break;
        case SLOPE_CEILING_DENSE_MFMA:
            mfma_loop_kernel<1><<<dim3(CEIL_BLOCKS), dim3(256), 0, s>>>((const u32x4*)buf, iters, sink);
            *work = (double)(lanes / 64) * iters * CEIL_ACC * 2.0 * 16 * 16 * 32;
            break;
        case SLOPE_CEILING_SPARSE_MFMA_32:
            mfma32_loop_kernel<0><<<dim3(CEIL_BLOCKS), dim3(256), 0, s>>>((const u32x4*)buf, iters, sink);
            *work = (double)(lanes / 64) * iters * 8 * 2.0 * 32 * 32 * 32;
            break;
        case SLOPE_CEILING_DENSE_MFMA_32:
            mfma32_loop_kernel<1><<<dim3(CEIL_BLOCKS), dim3(256), 0, s>>>((const u32x4*)buf, iters, sink);
            *work = (double)(lanes / 64) * iters * 8 * 2.0 * 32 * 32 * 16;
            break;
        case SLOPE_CEILING_READ: {
            const size_t sink_bytes = 4096;                   // past the data
            if (bytes < 2 * sink_bytes) return SLOPE_ERR_SHAPE;
            const size_t nvec = (bytes - sink_bytes) / 16;
            if ((nvec + 255) / 256 > 0x7FFFFFFFu) return SLOPE_ERR_SHAPE;
            read_stream_kernel<<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>(
                (const u32x4*)buf, nvec, (uint32_t*)((uint8_t*)buf + nvec * 16));
            *work = (double)nvec * 16;
            break;
        }
        case SLOPE_CEILING_COPY: {
            const size_t nvec = bytes / 32;
            if ((nvec + 255) / 256 > 0x7FFFFFFFu) return SLOPE_ERR_SHAPE;
            copy_stream_kernel<<<dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s>>>((const u32x4*)buf,
                                                                                         (u32x4*)buf + nvec, nvec);
            *work = (double)nvec * 32;                        // read + written
            break;
        }
        default: return SLOPE_ERR_UNSUPPORTED;
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return SLOPE_OK;
    note_hip_error(e);
    return SLOPE_ERR_HIP;
}

}  // extern "C"
