// 2:4 sparse x dense product on CDNA4's structured-sparse MFMA, shared by
// slope_spmm_fwd (Eq. 4, with the low-rank K-extension of Eq. 11) and slope_spmm_bwd_x (Eq. 6).
//
//     C[n, m] = sum_k B[n, k] * A[m, k]        A: packed 2:4 along k (vals + 4-bit metadata)
//             + sum_k2 B2[n, k2] * A2[m, k2]   dense bf16, K2 = adapter rank (optional)
//
// fwd  : A = W^R        (m = d_out, k = d_in ), B = X,  C = Y,  A2 = R^T, B2 = X L
// bwd_x: A = (W^{R,C})^T (m = d_in,  k = d_out), B = dY, C = dX
//
// The instruction is v_smfmac_f32_16x16x64_bf16 (D[16 x 16] += Asparse[16 x 64] * B[64 x 16]):
//   A   lane l holds row l%16 and the 8 packed values of logical k = 16*(l/16) .. +15
//   idx lane l holds the 4 metadata nibbles of those 16 k in bits 0..15 (idx0 | idx1 << 2 each)
//   B   lane l holds column l%16; registers 0-3 = k 8*(l/16) .. +7, registers 4-7 = 32 + the same
//   D   lane l holds column l%16, rows 4*(l/16) .. +3
// so the sparse operand is the weight, rows of D are output features, and a lane's four
// accumulators are four consecutive features of one token: an 8-byte store into row-major C.
//
// LDS holds operands in fragment order (the 16 bytes a lane feeds to the instruction sit at
// 16 * lane inside a 1 KiB fragment), so every ds_read_b128 is a linear, conflict-free read and
// every global load instruction fetches exactly one fragment (16 rows x 64 contiguous bytes).
#include "common.h"

namespace {

constexpr int XCDS = 8;

// blockIdx -> tile, so that the 32 tiles resident on one XCD form a compact 4 x 8 patch and
// share operand panels in that XCD's L2.
__device__ __forceinline__ void tile_of_block(int nblocks, int tiles_m, int tiles_n, int& tm, int& tn) {
    int b = blockIdx.x;
    int xcd = b % XCDS, pos = b / XCDS;
    int q = nblocks / XCDS, rem = nblocks % XCDS;
    int id = xcd * q + (xcd < rem ? xcd : rem) + pos;
    constexpr int GM = 4;
    int per_group = GM * tiles_n;
    int g = id / per_group, first_m = g * GM;
    int gsize = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    int in_group = id - g * per_group;
    tm = first_m + in_group % gsize;
    tn = in_group / gsize;
}

template <int BM, int BN>
struct SpmmSmem {
    static constexpr int A_BYTES = BM * 64;     // packed values of a BM x 64 (logical k) slab
    static constexpr int B_BYTES = BN * 128;    // dense BN x 64 slab
    static constexpr int M_BYTES = BM * 8;      // metadata: 16 nibbles per row
    static constexpr int STAGE = A_BYTES + B_BYTES + M_BYTES;
};

// One workgroup = 4 wavefronts in a 2 x 2 grid; each wavefront owns (BM/2) x (BN/2) of C.
template <int BM, int BN>
__global__ void __launch_bounds__(256) spmm_kernel(const bf16_t* __restrict__ B, int n, const bf16_t* __restrict__ Av,
                                                   const uint8_t* __restrict__ Am, int m, int K,
                                                   const bf16_t* __restrict__ B2, const bf16_t* __restrict__ A2,
                                                   int K2, bf16_t* __restrict__ C, int tiles_m, int tiles_n) {
    using S = SpmmSmem<BM, BN>;
    constexpr int MF = BM / 32, NF = BN / 32;            // fragments per wavefront
    constexpr int A_LD = BM / 64, B_LD = BN / 32;        // 16-byte global loads per lane per stage
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    tile_of_block(tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- global -> register staging addresses (rows clamped: out-of-range rows are never stored)
    const size_t a_pitch = (size_t)K / 2, m_pitch = (size_t)K / 8, b_pitch = (size_t)K;
    const bf16_t* a_src[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int frag = wave * A_LD + i;                       // 16-row fragment of the A slab
        int row = m0 + frag * 16 + l16;
        row = row < m ? row : m - 1;
        a_src[i] = Av + (size_t)row * a_pitch + lq * 8;   // 8 packed values = logical k 16*lq..
    }
    const bf16_t* b_src[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int slot = wave * B_LD + i;                       // (fragment, half) pair
        int frag = slot >> 1, half = slot & 1;
        int row = n0 + frag * 16 + l16;
        row = row < n ? row : n - 1;
        b_src[i] = B + (size_t)row * b_pitch + half * 32 + lq * 8;
    }
    const uint8_t* m_src;
    {
        int row = m0 + t;
        row = row < m ? row : m - 1;
        m_src = Am + (size_t)row * m_pitch;
    }
    constexpr bool META_ALL = BM >= 256;                  // otherwise only the first BM lanes load metadata

    u32x4 a_reg[A_LD], b_reg[B_LD];
    u32x2 m_reg = (u32x2){0u, 0u};
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) a_reg[i] = *(const u32x4*)(a_src[i] + k0 / 2);
#pragma unroll
        for (int i = 0; i < B_LD; ++i) b_reg[i] = *(const u32x4*)(b_src[i] + k0);
        if (META_ALL || t < BM) m_reg = *(const u32x2*)(m_src + k0 / 8);
    };
    auto store_lds = [&](int stage) {
        uint8_t* base = smem + stage * S::STAGE;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) *(u32x4*)(base + (wave * A_LD + i) * 1024 + lane * 16) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_LD; ++i) *(u32x4*)(base + S::A_BYTES + (wave * B_LD + i) * 1024 + lane * 16) = b_reg[i];
        if (META_ALL || t < BM) *(u32x2*)(base + S::A_BYTES + S::B_BYTES + t * 8) = m_reg;
    };

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int ksteps = K / 64;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int stage = ks & 1;
        // prefetch the next slab into registers; the last step re-reads its own slab (unused)
        load_global((ks + 1 < ksteps ? ks + 1 : ks) * 64);
        const uint8_t* base = smem + stage * S::STAGE;
        const uint8_t* sa = base + (wm * MF) * 1024 + lane * 16;
        const uint8_t* sb = base + S::A_BYTES + (wn * NF) * 2048 + lane * 16;
        const uint8_t* sm = base + S::A_BYTES + S::B_BYTES + (wm * MF * 16 + l16) * 8 + lq * 2;
        bf16x16 bf[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            union { uint4 u[2]; bf16x16 v; } x;
            x.u[0] = *(const uint4*)(sb + j * 2048);
            x.u[1] = *(const uint4*)(sb + j * 2048 + 1024);
            bf[j] = x.v;
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            union { uint4 u; bf16x8 v; } a;
            a.u = *(const uint4*)(sa + i * 1024);
            int idx = *(const uint16_t*)(sm + i * 128);
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, bf[j], acc[i][j], idx, 0, 0);
        }
        store_lds(stage ^ 1);
        __syncthreads();
    }

    // ---- dense K-extension: C += B2 * A2^T with v_mfma_f32_16x16x32_bf16, operands straight
    //      from global memory (lane l: row l%16, k = 8*(l/16) .. +7, for A and B alike)
    for (int k0 = 0; k0 < K2; k0 += 32) {
        bf16x8 af[MF], bfr[NF];
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int row = m0 + (wm * MF + i) * 16 + l16;
            row = row < m ? row : m - 1;
            union { uint4 u; bf16x8 v; } x;
            x.u = *(const uint4*)(A2 + (size_t)row * K2 + k0 + lq * 8);
            af[i] = x.v;
        }
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            int row = n0 + (wn * NF + j) * 16 + l16;
            row = row < n ? row : n - 1;
            union { uint4 u; bf16x8 v; } x;
            x.u = *(const uint4*)(B2 + (size_t)row * K2 + k0 + lq * 8);
            bfr[j] = x.v;
        }
#pragma unroll
        for (int i = 0; i < MF; ++i)
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }

    // ---- epilogue: four consecutive features of one token per lane
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        int row = n0 + (wn * NF + j) * 16 + l16;          // token
        if (row >= n) continue;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int col = m0 + (wm * MF + i) * 16 + lq * 4;   // feature
            if (col >= m) continue;
            f32x4 v = acc[i][j];
            union { __bf16 h[4]; uint2 u; } o;
            o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
            *(uint2*)(C + (size_t)row * m + col) = o.u;
        }
    }
}

template <int BM, int BN>
hipError_t launch_tile(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    using S = SpmmSmem<BM, BN>;
    int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    size_t smem = 2 * S::STAGE;
    auto kern = spmm_kernel<BM, BN>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), smem, s>>>(B, (int)n, Av, Am, (int)m, (int)K, B2, A2,
                                                                       (int)K2, C, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_spmm(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    // big tiles once they fill the 256 compute units, small tiles otherwise
    int64_t big = ((m + 255) / 256) * ((n + 255) / 256);
    if (big >= 256) return launch_tile<256, 256>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
    return launch_tile<128, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
}
