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
// Data movement.  A workgroup owns a BM x BN tile of C and walks k in steps of 64.  It has 8
// wavefronts (2 x 4 over the tile, two per SIMD) in two groups that run half a step apart: while
// one group issues its MFMAs the other reads its fragments from LDS and queues global loads, then
// they swap (two barriers per step), so each SIMD's matrix pipe always has a wavefront feeding it.
// Operands travel global -> LDS with global_load_lds (no registers in between) into a ring of three
// stages, two steps ahead of their use.  LDS holds them in fragment order: the 16 bytes a lane
// feeds to the instruction sit at 16 * lane inside a 1 KiB fragment, so every global load
// instruction fetches one fragment (16 rows x 64 contiguous bytes) and every ds_read_b128 is a
// linear, conflict-free read.
#include "common.h"

namespace {

constexpr int XCDS = 8;
constexpr int SUPER = 16;                 // tiles per edge of the chip-wide patch of 256 resident tiles

// s_waitcnt immediate (gfx9 encoding): vmcnt <= vm, lgkmcnt <= lgkm, expcnt unconstrained.
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (lgkm << 8); }

// blockIdx -> tile.  Workgroups are dealt round-robin to the 8 XCDs, 32 resident per XCD.  The 256
// resident tiles form one 16 x 16 patch (so the whole chip shares 16 + 16 operand panels in the
// last-level cache) and each XCD owns an 8 x 4 corner of it (sharing 8 + 4 panels in its L2).
__device__ __forceinline__ bool tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
    int b = blockIdx.x;
    int xcd = b % XCDS, slot = b / XCDS;
    int round = slot / 32, w = slot % 32;
    int supers_n = (tiles_n + SUPER - 1) / SUPER;
    int sm = round / supers_n, sn = round % supers_n;
    tm = sm * SUPER + (xcd & 1) * 8 + (w & 7);
    tn = sn * SUPER + (xcd >> 1) * 4 + (w >> 3);
    return tm < tiles_m && tn < tiles_n;
}

template <int BM, int BN>
struct SpmmSmem {
    static constexpr int A_BYTES = BM * 64;     // packed values of a BM x 64 (logical k) slab
    static constexpr int B_BYTES = BN * 128;    // dense BN x 64 slab
    static constexpr int M_BYTES = BM * 8;      // metadata: 16 nibbles per row
    static constexpr int STAGE = A_BYTES + B_BYTES + M_BYTES;
    static constexpr int NST = 3;
    static constexpr int DUMMY = NST * STAGE;   // landing zone for metadata loads of idle wavefronts
    static constexpr int TOTAL = DUMMY + 8 * 256;
};

// 64 lanes x 16 (or 4) bytes: lane l's bytes land at lds_dst + 16 (4) * l; lds_dst is wave-uniform
__device__ __forceinline__ void dma16(const void* gsrc, uint8_t* lds_dst) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gsrc,
                                     (void __attribute__((address_space(3)))*)lds_dst, 16, 0, 0);
}
__device__ __forceinline__ void dma4(const void* gsrc, uint8_t* lds_dst) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gsrc,
                                     (void __attribute__((address_space(3)))*)lds_dst, 4, 0, 0);
}

constexpr int SPMM_THREADS = 512;

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for every
// outstanding global -> LDS load (vmcnt(0)), which is exactly what the ring is there to avoid.
// Visibility of those loads is handled by explicit s_waitcnt vmcnt(n) before the barrier; LDS reads
// are kept on their side of the barrier by the compiler-level clobbers.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
#ifndef SLOPE_LOOSE_PHASES
    __builtin_amdgcn_sched_barrier(0);   // nothing is scheduled across: phases stay phases
#endif
    __builtin_amdgcn_s_barrier();
#ifndef SLOPE_LOOSE_PHASES
    __builtin_amdgcn_sched_barrier(0);
#endif
    asm volatile("" ::: "memory");
}

template <int BM, int BN>
__global__ void __launch_bounds__(SPMM_THREADS) spmm_kernel(const bf16_t* __restrict__ B, int n,
                                                            const bf16_t* __restrict__ Av,
                                                            const uint8_t* __restrict__ Am, int m, int K,
                                                            const bf16_t* __restrict__ B2,
                                                            const bf16_t* __restrict__ A2, int K2,
                                                            bf16_t* __restrict__ C, int tiles_m, int tiles_n) {
    using S = SpmmSmem<BM, BN>;
    constexpr int MF = BM / 32, NF = BN / 64;                // 16 x 16 fragments per wavefront
    constexpr int A_LD = BM / 128, B_LD = BN / 64;           // fragment loads per wavefront per step
    constexpr int NLD = A_LD + B_LD + 1;                     // + one metadata load
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    if (!tile_of_block(tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;                             // the two wavefronts of a SIMD differ here
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- per-lane global sources (rows clamped: results of out-of-range rows are never stored)
    const size_t a_pitch = (size_t)K / 2, m_pitch = (size_t)K / 8, b_pitch = (size_t)K;
    const bf16_t* a_src[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int row = m0 + (wave * A_LD + i) * 16 + l16;
        row = row < m ? row : m - 1;
        a_src[i] = Av + (size_t)row * a_pitch + lq * 8;       // 8 packed values = logical k 16*lq ..
    }
    const bf16_t* b_src[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int slot = wave * B_LD + i;                           // (fragment, half) pair
        int row = n0 + (slot >> 1) * 16 + l16;
        row = row < n ? row : n - 1;
        b_src[i] = B + (size_t)row * b_pitch + (slot & 1) * 32 + lq * 8;
    }
    // metadata: 32 rows per wavefront, two lanes (4 bytes each) per row
    const bool meta_wave = wave * 32 < BM;
    const uint8_t* m_src;
    {
        int row = m0 + (meta_wave ? wave * 32 : 0) + (lane >> 1);
        row = row < m ? row : m - 1;
        m_src = Am + (size_t)row * m_pitch + (lane & 1) * 4;
    }
    const int m_dst = meta_wave ? S::A_BYTES + S::B_BYTES + wave * 256 : -1;

    const int ksteps = K / 64;
    // queue this wavefront's share of k-step `ks` (clamped to the last one) into ring stage ks % 3
    auto issue = [&](int ks) {
        int kc = ks < ksteps ? ks : ksteps - 1;
        uint8_t* st = smem + (ks % S::NST) * S::STAGE;
        dma4(m_src + kc * 8, m_dst >= 0 ? st + m_dst : smem + S::DUMMY + wave * 256);
#pragma unroll
        for (int i = 0; i < A_LD; ++i) dma16(a_src[i] + kc * 32, st + (wave * A_LD + i) * 1024);
#pragma unroll
        for (int i = 0; i < B_LD; ++i) dma16(b_src[i] + kc * 64, st + S::A_BYTES + (wave * B_LD + i) * 1024);
    };

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    union BFrag { u32x4 u[2]; bf16x16 v; };
    union AFrag { u32x4 u; bf16x8 v; };

    const int a_rd = (wm * MF) * 1024 + lane * 16;
    const int b_rd = S::A_BYTES + (wn * NF) * 2048 + lane * 16;
    const int m_rd = S::A_BYTES + S::B_BYTES + (wm * MF * 16 + l16) * 8 + lq * 2;

    // ---- prologue: two steps in flight; the second group starts half a step late
    issue(0);
    issue(1);
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(NLD, 15));         // step 0 has landed (this wave's share)
    wg_barrier();

    // One step of one wavefront.  The wait for the wavefront's own share of step ks + 1 sits at the
    // end of the compute phase for group 0 and at the end of the memory phase for group 1: either
    // way it precedes the barrier after which group 0 starts reading that step.
#define SPMM_STEP(G)                                                                                   \
    {                                                                                                  \
        const uint8_t* st = smem + (ks % S::NST) * S::STAGE;                                           \
        BFrag bf[NF];                                                                                  \
        AFrag af[MF];                                                                                  \
        int ai[MF];                                                                                    \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(st + b_rd + j * 2048);                                        \
            bf[j].u[1] = *(const u32x4*)(st + b_rd + j * 2048 + 1024);                                 \
        }                                                                                              \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u = *(const u32x4*)(st + a_rd + i * 1024);                                           \
            ai[i] = *(const uint16_t*)(st + m_rd + i * 128);                                           \
        }                                                                                              \
        issue(ks + 2);                                                                                 \
        if (G == 1) __builtin_amdgcn_s_waitcnt(waitcnt_imm(NLD, 15));                                  \
        wg_barrier();                                                                                  \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) _Pragma("unroll") for (int j = 0; j < NF; ++j)  \
            acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(af[i].v, bf[j].v, acc[i][j], ai[i], 0, 0); \
        if (G == 0) __builtin_amdgcn_s_waitcnt(waitcnt_imm(NLD, 15));                                  \
        wg_barrier();                                                                                  \
    }
    if (group == 0) {
        for (int ks = 0; ks < ksteps; ++ks) SPMM_STEP(0)
        wg_barrier();
    } else {
        wg_barrier();
        for (int ks = 0; ks < ksteps; ++ks) SPMM_STEP(1)
    }
#undef SPMM_STEP
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 15));           // drain the clamped look-ahead loads

    // ---- dense K-extension: C += B2 * A2^T with v_mfma_f32_16x16x32_bf16, operands straight
    //      from global memory (lane l: row l%16, k = 8*(l/16) .. +7, for A and B alike)
    for (int k0 = 0; k0 < K2; k0 += 32) {
        bf16x8 a2[MF], b2[NF];
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int row = m0 + (wm * MF + i) * 16 + l16;
            row = row < m ? row : m - 1;
            AFrag x;
            x.u = *(const u32x4*)(A2 + (size_t)row * K2 + k0 + lq * 8);
            a2[i] = x.v;
        }
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            int row = n0 + (wn * NF + j) * 16 + l16;
            row = row < n ? row : n - 1;
            AFrag x;
            x.u = *(const u32x4*)(B2 + (size_t)row * K2 + k0 + lq * 8);
            b2[j] = x.v;
        }
#pragma unroll
        for (int i = 0; i < MF; ++i)
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2[i], b2[j], acc[i][j], 0, 0, 0);
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
            union { __bf16 h[4]; u32x2 u; } o;
            o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
            *(u32x2*)(C + (size_t)row * m + col) = o.u;
        }
    }
}

template <int BM, int BN>
hipError_t launch_tile(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    using S = SpmmSmem<BM, BN>;
    int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    int supers = ((tiles_m + SUPER - 1) / SUPER) * ((tiles_n + SUPER - 1) / SUPER);
    auto kern = spmm_kernel<BM, BN>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, S::TOTAL);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)(supers * SUPER * SUPER)), dim3(SPMM_THREADS), S::TOTAL, s>>>(B, (int)n, Av, Am, (int)m, (int)K, B2,
                                                                               A2, (int)K2, C, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_spmm(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    // big tiles once they fill the 256 compute units, small tiles otherwise
    int64_t big = ((m + 255) / 256) * ((n + 255) / 256);
    if (big >= 192) return launch_tile<256, 256>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
    return launch_tile<128, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
}
