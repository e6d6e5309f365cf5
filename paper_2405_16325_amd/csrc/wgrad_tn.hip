// slope_wgrad_masked with a workspace: dW = dY^T X (Eq. 5) as a token-contiguous dense MFMA
// product, with the prune-and-compress step of Algorithm 1 line 13 folded into the epilogue.
//
// The contraction runs over the b tokens, the slow index of both operands in memory.  Feeding the
// MFMA straight from [token][feature] slabs needs the transposing LDS read, which delivers only a
// quarter of the LDS bandwidth of ds_read_b128 and caps the kernel near half the MFMA peak.  So
// the operands are first copied once into token-contiguous form in the caller's workspace
//     Xt [d_in ][bp],  dYt[d_out][bp],   bp = b rounded up to 64, the tail zero-filled
// (two HBM streams, a few percent of the product's time at LLM layer sizes), and the product
//     D[i, j] = sum_t Xt[i, t] * dYt[j, t]
// runs with the same machinery as the sparse kernels: 8 wavefronts in two groups half a k-step
// apart, global -> LDS loads of full 128-byte lines (8 rows x 128 B per instruction, 16-byte chunks
// rotated by (row / 2) % 8), conflict-free ds_read_b128 in MFMA order, v_mfma_f32_16x16x32_bf16.
// D rows are d_in and D columns d_out, so a lane's four accumulators (column l%16, rows
// 4*(l/16) .. +3) are exactly one group of four of W^R's row: the epilogue picks two of them with
// the group's metadata nibble and stores one 4-byte pair of the packed gradient.
#include "pipeline.h"

namespace {

// out[c][r] = in[r][c] for r < rows, zero for rows <= r < rows_pad; in is [rows][cols] bf16,
// out is [cols][rows_pad].  64 x 64 tiles through LDS, 16-byte global accesses on both sides.
__global__ void __launch_bounds__(256) transpose_pad_kernel(const bf16_t* __restrict__ in, int rows, int cols,
                                                            int rows_pad, bf16_t* __restrict__ out) {
    __shared__ bf16_t tile[64][66];
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64, t = threadIdx.x;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        int r = (t >> 3) + 32 * p, c8 = (t & 7) * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r0 + r < rows) v = *(const u32x4*)(in + (size_t)(r0 + r) * cols + c0 + c8);
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[c8 + e][r] = (bf16_t)(v[e >> 1] >> (16 * (e & 1)));
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        int c = (t >> 3) + 32 * p, r8 = (t & 7) * 8;
        const uint32_t* src = (const uint32_t*)&tile[c][r8];
        u32x4 v = {src[0], src[1], src[2], src[3]};
        *(u32x4*)(out + (size_t)(c0 + c) * rows_pad + r0 + r8) = v;
    }
}

struct TnSmem {
    static constexpr int BM = 256, BN = 256;
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;   // one k-step of 64 tokens
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int TOTAL = 2 * STAGE;
};

constexpr int TN_THREADS = 512;

// At: [m][kp] (d_in rows), Bt: [n][kp] (d_out rows), kp % 64 == 0.  G: packed gradient [n][m/2].
__global__ void __launch_bounds__(TN_THREADS) wgrad_tn_kernel(const bf16_t* __restrict__ At, int m,
                                                              const bf16_t* __restrict__ Bt, int n, int kp,
                                                              const uint8_t* __restrict__ meta,
                                                              bf16_t* __restrict__ G, int tiles_m, int tiles_n) {
    using S = TnSmem;
    constexpr int MF = 8, NF = 4;                            // wavefront tile 128 (d_in) x 64 (d_out)
    constexpr int LD = 4;                                    // 1 KiB loads per wavefront per operand per step
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    if (!tile_of_block(tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * S::BM, n0 = tn * S::BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // loader lanes: 8 lanes per row, chunk rotated by (row / 2) % 8 (rows clamped, never stored)
    const uint8_t* a_src[LD];
    const uint8_t* b_src[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        int rl = (wave * LD + i) * 8 + (lane >> 3);
        int chunk = ((lane & 7) ^ ((rl >> 1) & 7)) * 16;
        int ra = m0 + rl < m ? m0 + rl : m - 1;
        int rb = n0 + rl < n ? n0 + rl : n - 1;
        a_src[i] = (const uint8_t*)At + (size_t)ra * kp * 2 + chunk;
        b_src[i] = (const uint8_t*)Bt + (size_t)rb * kp * 2 + chunk;
    }
    const int ksteps = kp / 64;
    auto issue = [&](int ks) {                               // k-step ks (clamped) into stage ks % 2
        int kc = ks < ksteps ? ks : ksteps - 1;
        uint8_t* st = smem + (ks & 1) * S::STAGE + wave * LD * 1024;
#pragma unroll
        for (int i = 0; i < LD; ++i) dma16(a_src[i] + (size_t)kc * 128, st + i * 1024);
#pragma unroll
        for (int i = 0; i < LD; ++i) dma16(b_src[i] + (size_t)kc * 128, st + S::A_BYTES + i * 1024);
    };

    // reader lanes: fragment f = rows 16f .. 16f+15 = 2 KiB; lane (l16, lq) wants chunk 4h + lq
    const int sw = (l16 >> 1) & 7;
    const int rd0 = l16 * 128 + ((lq ^ sw) * 16);
    const int rd1 = l16 * 128 + (((4 + lq) ^ sw) * 16);
    const int a_rd = (wm * MF) * 2048;
    const int b_rd = S::A_BYTES + (wn * NF) * 2048;

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // One k-step.  Loads of step s + 1 are queued in the even phase in which stage (s + 1) % 2 has
    // just been released: group 0 is then in its memory phase of step s, group 1 in its compute
    // phase of step s - 1.  Every wavefront waits for its own loads one phase later, before the
    // barrier after which group 0 reads them.
#define TN_STEP(G)                                                                                     \
    {                                                                                                  \
        const uint8_t* st = smem + (ks & 1) * S::STAGE;                                                \
        BFrag af[MF], bf[NF];                                                                          \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u[0] = *(const u32x4*)(st + a_rd + i * 2048 + rd0);                                  \
            af[i].u[1] = *(const u32x4*)(st + a_rd + i * 2048 + rd1);                                  \
        }                                                                                              \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(st + b_rd + j * 2048 + rd0);                                  \
            bf[j].u[1] = *(const u32x4*)(st + b_rd + j * 2048 + rd1);                                  \
        }                                                                                              \
        if (G == 0) issue(ks + 1);                                                                     \
        /* all LDS reads of this stage have returned before anybody may overwrite it */                \
        WAIT_HERE(waitcnt_imm(G == 1 ? 0 : 63, 0));                                   \
        wg_barrier();                                                                                  \
        if (G == 1) issue(ks + 2);                                                                     \
        _Pragma("unroll") for (int h = 0; h < 2; ++h)                                                  \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) _Pragma("unroll") for (int j = 0; j < NF; ++j) { \
            AFrag a, b;                                                                                \
            a.u = af[i].u[h]; b.u = bf[j].u[h];                                                        \
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc[i][j], 0, 0, 0);         \
        }                                                                                              \
        if (G == 0) WAIT_HERE(waitcnt_imm(0, 15));                                    \
        wg_barrier();                                                                                  \
    }
    issue(0);
    WAIT_HERE(waitcnt_imm(0, 15));
    wg_barrier();
    if (group == 0) {
        for (int ks = 0; ks < ksteps; ++ks) TN_STEP(0)
        wg_barrier();
    } else {
        issue(1);
        wg_barrier();
        for (int ks = 0; ks < ksteps; ++ks) TN_STEP(1)
    }
#undef TN_STEP
    WAIT_HERE(waitcnt_imm(0, 15));           // drain the clamped look-ahead loads

    // epilogue: a lane's four accumulators are one group of four along d_in of row o
    const size_t mpitch = (size_t)m / 8, gpitch = (size_t)m / 2;
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        int o = n0 + (wn * NF + j) * 16 + l16;
        if (o >= n) continue;
        // metadata of the wavefront's 128 d_in columns of row o: 32 groups = 16 bytes
        int c0 = m0 + wm * (S::BM / 2);
        u32x4 mw = {0u, 0u, 0u, 0u};
        if (c0 + 128 <= m) {
            mw = *(const u32x4*)(meta + (size_t)o * mpitch + c0 / 8);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (c0 + 32 * q < m) mw[q] = *(const uint32_t*)(meta + (size_t)o * mpitch + c0 / 8 + 4 * q);
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int col = c0 + i * 16 + lq * 4;               // first d_in index of the group
            if (col >= m) continue;
            int gl = i * 4 + lq;                          // group index inside the 128 columns
            uint32_t nib = (mw[gl >> 3] >> (4 * (gl & 7))) & 0xFu;
            uint32_t a = nib & 3u, c = nib >> 2;
            f32x4 v = acc[i][j];
            float v0 = a == 0 ? v[0] : (a == 1 ? v[1] : v[2]);
            float v1 = c == 1 ? v[1] : (c == 2 ? v[2] : v[3]);
            union { __bf16 h[2]; uint32_t u; } out;
            out.h[0] = (__bf16)v0;
            out.h[1] = (__bf16)v1;
            *(uint32_t*)(G + (size_t)o * gpitch + (col >> 1)) = out.u;
        }
    }
}

}  // namespace

size_t wgrad_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out) {
    size_t bp = ((size_t)b + 63) / 64 * 64;
    return (size_t)(d_in + d_out) * bp * 2;
}

hipError_t launch_wgrad_masked_ws(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out,
                                  int64_t d_in, bf16_t* gvals, void* workspace, hipStream_t s) {
    int bp = (int)((b + 63) / 64 * 64);
    bf16_t* Xt = (bf16_t*)workspace;
    bf16_t* dYt = Xt + (size_t)d_in * bp;
    transpose_pad_kernel<<<dim3((unsigned)(bp / 64), (unsigned)(d_in / 64)), dim3(256), 0, s>>>(X, (int)b, (int)d_in, bp, Xt);
    transpose_pad_kernel<<<dim3((unsigned)(bp / 64), (unsigned)(d_out / 64)), dim3(256), 0, s>>>(dY, (int)b, (int)d_out, bp, dYt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int tiles_m = (int)((d_in + 255) / 256), tiles_n = (int)((d_out + 255) / 256);
    e = hipFuncSetAttribute((const void*)wgrad_tn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, TnSmem::TOTAL);
    if (e != hipSuccess) return e;
    wgrad_tn_kernel<<<dim3((unsigned)super_grid(tiles_m, tiles_n)), dim3(TN_THREADS), TnSmem::TOTAL, s>>>(
        Xt, (int)d_in, dYt, (int)d_out, bp, meta, gvals, tiles_m, tiles_n);
    return hipGetLastError();
}
