// Small-batch form of the 2:4 sparse product (inference-size token counts, n <= 32):
//     C[n, m] = sum_k B[n, k] * A[m, k]   (+ T[n, K2] * R[K2, m] for the adapters of Eq. 11)
// With so few tokens the product is one pass over the packed weight (1.125 bytes per element) and
// HBM bounds it, so the kernel is built to keep reads in flight rather than to share operands:
//   - a workgroup owns 32 weight rows and all tokens; its 8 wavefronts take the k-steps of 64 in
//     turn (wavefront w: the pairs of steps w, w + 8, ...), each accumulating a partial 32 x n tile, so even a
//     9216-row weight gives 288 workgroups and every row of the weight is read in 128-byte pieces
//     by neighbouring wavefronts at about the same time;
//   - operands go from global memory into registers, several steps ahead, four lanes per row
//     segment of 64 bytes, and reach the lane order of v_smfmac_f32_16x16x64_bf16 (lane = row
//     l%16, chunk l/16) by ds_bpermute; no LDS buffers, no barriers in the main loop;
//   - the 8 partial tiles are summed in a fixed order through LDS (bit-identical runs), and the
//     adapter term is added there with plain fp32 FMAs on T = X L and the factor R as stored.
// T itself comes from a split over d_in (xl_partial_kernel, fp32 partial sums in the workspace)
// followed by a fixed-order reduction that rounds to bf16 (xl_reduce_kernel).
#include "common.h"

namespace {

constexpr int ST_BM = 32;           // weight rows per workgroup
constexpr int ST_WAVES = 8;
#ifndef ST_DEPTH_PAIRS
#define ST_DEPTH_PAIRS 2
#endif
#ifdef ST_NONTEMPORAL
#define ST_LOAD(p) __builtin_nontemporal_load(p)
#else
#define ST_LOAD(p) (*(p))
#endif
constexpr int ST_DEPTH = ST_DEPTH_PAIRS;   // pairs of k-steps each wavefront keeps in flight
constexpr int XL_CHUNK = 128;       // rows of L per workgroup of xl_partial_kernel

union StB { u32x4 u[2]; bf16x16 v; };
union StA { u32x4 u; bf16x8 v; };

// One pair of k-steps as loaded: every load instruction fetches 8 rows x 128 contiguous bytes
// (8 lanes per row), which for the packed weight is both steps of the pair and for the token
// operand one step.
template <int NF>
struct StStage {
    u32x4 a[2][2];          // [fragment][rows 0-7 | rows 8-15]: 128 bytes per row = 2 steps x 64
    uint32_t mt[2];         // [fragment]: 16 bytes of metadata per row (4 lanes per row)
    u32x4 b[2][NF][2];      // [step][fragment][tokens 0-7 | 8-15]: 128 bytes per token
};

template <int NF>
__global__ void __launch_bounds__(ST_WAVES * 64) spmm_stream_kernel(const bf16_t* __restrict__ B, int n,
                                                                  const bf16_t* __restrict__ Av,
                                                                  const uint8_t* __restrict__ Am, int m, int K,
                                                                  const bf16_t* __restrict__ T,
                                                                  const bf16_t* __restrict__ R, int K2,
                                                                  bf16_t* __restrict__ C) {
    constexpr int MF = ST_BM / 16, NC = NF * 16, PITCH = NC + 1;
    __shared__ float part[ST_WAVES][ST_BM][PITCH];

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int m0 = blockIdx.x * ST_BM;
    const int ksteps = K / 64, kpairs = (ksteps + 1) / 2;
    const bool odd_tail = (ksteps & 1) != 0;                 // the last pair has one step only

    // Loader lanes: lane = 8 * row + chunk.  The MFMA wants row l%16 and 16-byte chunk l/16 of the
    // step in lane l: multiply() fetches them from the loader lanes with ds_bpermute.
    const int ld_row = lane >> 3, ld_chunk = lane & 7;
    const uint8_t* a_ptr[MF][2];
    const uint8_t* m_ptr[MF];
#pragma unroll
    for (int i = 0; i < MF; ++i) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int row = m0 + 16 * i + 8 * h + ld_row;
            row = row < m ? row : m - 1;
            a_ptr[i][h] = (const uint8_t*)Av + (size_t)row * K + 16 * ld_chunk;   // K bytes of packed values per row
        }
        int row = m0 + 16 * i + (lane >> 2);
        row = row < m ? row : m - 1;
        m_ptr[i] = Am + (size_t)row * (K / 8) + 4 * (lane & 3);
    }
    const uint8_t* b_ptr[NF][2];
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int tok = 16 * j + 8 * h + ld_row;
            tok = tok < n ? tok : n - 1;
            b_ptr[j][h] = (const uint8_t*)B + (size_t)tok * K * 2 + 16 * ld_chunk;
        }
    const int src_lo = ((l16 & 7) * 8 + lq) * 4;              // ds_bpermute byte address: chunk lq of row l16 % 8
    const bool upper = l16 >= 8;                              // which of the two 8-row loads holds row l16
    const int src_meta = (4 * l16 + (lq >> 1)) * 4;           // dword lq / 2 of row l16's metadata of a step

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    StStage<NF> st[ST_DEPTH];
    auto load = [&](StStage<NF>& s, int kp) {                 // pair kp, clamped: a late load is never used
        const size_t pc = kp < kpairs ? kp : kpairs - 1;
        // an odd number of steps: the last pair is read as steps (ksteps - 2, ksteps - 1) and only
        // its second half is used, so that no load runs past the row
        const size_t s0 = (odd_tail && pc == (size_t)kpairs - 1) ? (size_t)ksteps - 2 : 2 * pc;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            s.a[i][0] = ST_LOAD((const u32x4*)(a_ptr[i][0] + s0 * 64));
            s.a[i][1] = ST_LOAD((const u32x4*)(a_ptr[i][1] + s0 * 64));
            s.mt[i] = *(const uint32_t*)(m_ptr[i] + s0 * 8);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                s.b[e][j][0] = *(const u32x4*)(b_ptr[j][0] + (s0 + e) * 128);
                s.b[e][j][1] = *(const u32x4*)(b_ptr[j][1] + (s0 + e) * 128);
            }
    };
    // chunk c (0..7) of row l16 out of the pair of 8-row loads
    auto gather = [&](const u32x4 (&v)[2], int c) {
        u32x4 r;
        const int addr = src_lo + c * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)v[0][e]);
            uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(addr, (int)v[1][e]);
            r[e] = upper ? hi : lo;
        }
        return r;
    };
    auto multiply = [&](const StStage<NF>& s, int e) {       // step e (0 or 1) of the pair
        StB b[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            b[j].u[0] = gather(s.b[e][j], 0);
            b[j].u[1] = gather(s.b[e][j], 4);
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            uint32_t w = (uint32_t)__builtin_amdgcn_ds_bpermute(src_meta + e * 8, (int)s.mt[i]);
            int idx = (int)((w >> (16 * (lq & 1))) & 0xFFFFu);
            StA a;
            a.u = gather(s.a[i], 4 * e);
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, b[j].v, acc[i][j], idx, 0, 0);
        }
    };

    // Workgroups start at different places of the k range and wrap around, so that at any moment
    // the chip reads many different column bands of the weight rather than one (all rows have the
    // same pitch, and one band maps to few memory channels).
    const int rot = (int)((blockIdx.x * 37u) % (unsigned)kpairs);
    auto pair_of = [&](int q) { int p = q + rot; return p >= kpairs ? p - kpairs : p; };   // q < kpairs
#pragma unroll
    for (int d = 0; d < ST_DEPTH; ++d) {
        const int q = wave + ST_WAVES * d;
        load(st[d], q < kpairs ? pair_of(q) : kpairs - 1);
    }
    for (int kq = wave; kq < kpairs; kq += ST_WAVES * ST_DEPTH) {
#pragma unroll
        for (int d = 0; d < ST_DEPTH; ++d) {
            const int q = kq + ST_WAVES * d;                  // wave-uniform
            if (q < kpairs) {
                const int p = pair_of(q);
                if (!(odd_tail && p == kpairs - 1)) multiply(st[d], 0);
                multiply(st[d], 1);
            }
            const int qn = q + ST_WAVES * ST_DEPTH;
            load(st[d], qn < kpairs ? pair_of(qn) : kpairs - 1);
        }
    }

    // partial tiles: lane (l16, lq) holds token 16 j + l16, rows 16 i + 4 lq .. + 3
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) part[wave][16 * i + 4 * lq + e][16 * j + l16] = acc[i][j][e];
    __syncthreads();

    // fixed-order sum, adapter term, store: thread = (feature o, token tok)
    const int o = t & 31;
    for (int tok = t >> 5; tok < n; tok += ST_WAVES * 2) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < ST_WAVES; ++w) v += part[w][o][tok];
        if (m0 + o < m) {
            if (K2 > 0) {
                float low = 0.f;
                const bf16_t* tp = T + (size_t)tok * K2;
                const bf16_t* rp = R + m0 + o;
#pragma unroll 8
                for (int k = 0; k < K2; ++k)
                    low = __builtin_fmaf(__uint_as_float((uint32_t)tp[k] << 16),
                                         __uint_as_float((uint32_t)rp[(size_t)k * m] << 16), low);
                v += low;
            }
            union { __bf16 h; bf16_t u; } r;
            r.h = (__bf16)v;
            C[(size_t)tok * m + m0 + o] = r.u;
        }
    }
}

// P[c][t][k] = sum over the rows i of chunk c of X[t][i] * L[i][k]   (fp32; c = blockIdx.x)
// thread = column k of L: its loads of a row of L are contiguous across the wavefront; the token
// values are the same for all lanes and come through scalar loads.
template <int NT>
__global__ void __launch_bounds__(256) xl_partial_kernel(const bf16_t* __restrict__ X, int n, int d_in,
                                                         const bf16_t* __restrict__ L, int r,
                                                         float* __restrict__ P) {
    const int c = blockIdx.x, i0 = c * XL_CHUNK;
    const int k = blockIdx.y * 256 + threadIdx.x;
    const int rows = d_in - i0 < XL_CHUNK ? d_in - i0 : XL_CHUNK;       // a multiple of 64
    const int kc = k < r ? k : r - 1;
    float acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = 0.f;
    for (int i = 0; i < rows; i += 2) {
        float l0 = __uint_as_float((uint32_t)L[(size_t)(i0 + i) * r + kc] << 16);
        float l1 = __uint_as_float((uint32_t)L[(size_t)(i0 + i + 1) * r + kc] << 16);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            int tt = t < n ? t : n - 1;                                        // uniform
            uint32_t w = *(const uint32_t*)(X + (size_t)tt * d_in + i0 + i);   // uniform address: two tokens' worth of k
            acc[t] = __builtin_fmaf(__uint_as_float(w << 16), l0, acc[t]);
            acc[t] = __builtin_fmaf(__uint_as_float(w & 0xFFFF0000u), l1, acc[t]);
        }
    }
    if (k < r)
#pragma unroll
        for (int t = 0; t < NT; ++t)
            if (t < n) P[((size_t)c * n + t) * r + k] = acc[t];
}

// T[t][k] = bf16( sum over chunks, in order, of P[c][t][k] )
__global__ void __launch_bounds__(256) xl_reduce_kernel(const float* __restrict__ P, int chunks, int count,
                                                        bf16_t* __restrict__ T) {
    int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= count) return;
    float v = 0.f;
    for (int c = 0; c < chunks; ++c) v += P[(size_t)c * count + idx];
    union { __bf16 h; bf16_t u; } o;
    o.h = (__bf16)v;
    T[idx] = o.u;
}

}  // namespace

// n <= 32, K % 64 == 0, K >= 128; T (bf16[n][K2]) and R (bf16[K2][m]) only when K2 > 0
hipError_t launch_spmm_stream(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                              int64_t K, const bf16_t* T, const bf16_t* R, int64_t K2, bf16_t* C, hipStream_t s) {
    dim3 grid((unsigned)((m + ST_BM - 1) / ST_BM)), block(ST_WAVES * 64);
    if (n <= 16)
        spmm_stream_kernel<1><<<grid, block, 0, s>>>(B, (int)n, A_vals, A_meta, (int)m, (int)K, T, R, (int)K2, C);
    else
        spmm_stream_kernel<2><<<grid, block, 0, s>>>(B, (int)n, A_vals, A_meta, (int)m, (int)K, T, R, (int)K2, C);
    return hipGetLastError();
}

// T = X L for n <= 32 tokens; scratch holds ceil(d_in / 128) * n * r floats
size_t xl_small_scratch_bytes(int64_t n, int64_t d_in, int64_t r) {
    return (size_t)((d_in + XL_CHUNK - 1) / XL_CHUNK) * (size_t)n * (size_t)r * 4;
}

hipError_t launch_xl_small(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, float* scratch,
                           bf16_t* T, hipStream_t s) {
    const int chunks = (int)((d_in + XL_CHUNK - 1) / XL_CHUNK);
    dim3 grid((unsigned)chunks, (unsigned)((r + 255) / 256));
    if (n <= 16)
        xl_partial_kernel<16><<<grid, dim3(256), 0, s>>>(X, (int)n, (int)d_in, L, (int)r, scratch);
    else
        xl_partial_kernel<32><<<grid, dim3(256), 0, s>>>(X, (int)n, (int)d_in, L, (int)r, scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int count = (int)(n * r);
    xl_reduce_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s>>>(scratch, chunks, count, T);
    return hipGetLastError();
}
