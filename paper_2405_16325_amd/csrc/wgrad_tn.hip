// slope_wgrad_masked with a workspace: dW = dY^T X (Eq. 5) as a token-contiguous dense MFMA
// product, with the prune-and-compress step of Algorithm 1 line 13 folded into the epilogue.
//
// The contraction runs over the b tokens, the slow index of both operands in memory.  Feeding the
// MFMA straight from [token][feature] slabs needs the transposing LDS read, which delivers only a
// quarter of the LDS bandwidth of ds_read_b128 and caps the kernel near half the MFMA peak.  So
// the operands are first copied once into token-contiguous form in the caller's workspace
//     Xt [d_in ][ld],  dYt[d_out][ld],   bp = b rounded up to 64, the tail zero-filled,
//     ld = row pitch: bp, plus one 128-byte line where bp * 2 is a multiple of 4 KiB (rows that
//     far apart crowd the same L2 channels: the padded pitch is 2-3 % faster at b = 16384)
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

// out[c][r] = in[r][c] for r < rows, zero for rows <= r < rows_pad; in is [rows][cols] bf16 with
// cols % 8 == 0, out is [cols] rows of pitch ld >= rows_pad, rows_pad % 64 == 0, ld % 8 == 0.
// Tiles of TP_ROWS rows x 64 columns through LDS, 16-byte global accesses on both sides, non-temporal (116.9 -> 99.4 us
// for 16384 x 9216 alone, 8 % inside a training step); consecutive workgroups go down the rows, so that every output
// row is written front to back.
// blockIdx.z picks one of two matrices of the same row count (one launch for both operands of a product).
constexpr int TP_ROWS = 64;                                   // 128 and 256 measured the same
__global__ void __launch_bounds__(256) transpose_pad_kernel(const bf16_t* __restrict__ in0, int cols0,
                                                            bf16_t* __restrict__ out0, const bf16_t* __restrict__ in1,
                                                            int cols1, bf16_t* __restrict__ out1, int rows,
                                                            int rows_pad, int ld) {
    __shared__ bf16_t tile[64][TP_ROWS + 2];
    const bf16_t* __restrict__ in = blockIdx.z ? in1 : in0;
    bf16_t* __restrict__ out = blockIdx.z ? out1 : out0;
    const int cols = blockIdx.z ? cols1 : cols0;
    const int r0 = blockIdx.x * TP_ROWS, c0 = blockIdx.y * 64, t = threadIdx.x;
    if (c0 >= cols) return;                                   // uniform: the other matrix is wider
#pragma unroll
    for (int p = 0; p < TP_ROWS / 32; ++p) {
        int r = (t >> 3) + 32 * p, c8 = (t & 7) * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r0 + r < rows && c0 + c8 < cols) v = __builtin_nontemporal_load((const u32x4*)(in + (size_t)(r0 + r) * cols + c0 + c8));
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[c8 + e][r] = (bf16_t)(v[e >> 1] >> (16 * (e & 1)));
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < TP_ROWS / 32; ++p) {
        int idx = t + 256 * p, c = idx / (TP_ROWS / 8), r8 = (idx % (TP_ROWS / 8)) * 8;
        if (c0 + c >= cols || r0 + r8 >= rows_pad) continue;
        const uint32_t* src = (const uint32_t*)&tile[c][r8];
        u32x4 v = {src[0], src[1], src[2], src[3]};
        __builtin_nontemporal_store(v, (u32x4*)(out + (size_t)(c0 + c) * ld + r0 + r8));
    }
}

inline void launch_transpose_pad(const bf16_t* in, int64_t rows, int64_t cols, int64_t rows_pad, int64_t ld,
                                 bf16_t* out, hipStream_t s) {
    transpose_pad_kernel<<<dim3((unsigned)((rows_pad + TP_ROWS - 1) / TP_ROWS), (unsigned)((cols + 63) / 64), 1), dim3(256), 0, s>>>(
        in, (int)cols, out, nullptr, 0, nullptr, (int)rows, (int)rows_pad, (int)ld);
}

// two matrices with the same rows, rows_pad and ld in one launch
inline void launch_transpose_pad2(const bf16_t* in0, int64_t cols0, bf16_t* out0, const bf16_t* in1, int64_t cols1,
                                  bf16_t* out1, int64_t rows, int64_t rows_pad, int64_t ld, hipStream_t s) {
    const int64_t cmax = cols0 > cols1 ? cols0 : cols1;
    transpose_pad_kernel<<<dim3((unsigned)((rows_pad + TP_ROWS - 1) / TP_ROWS), (unsigned)((cmax + 63) / 64), 2), dim3(256), 0, s>>>(
        in0, (int)cols0, out0, in1, (int)cols1, out1, (int)rows, (int)rows_pad, (int)ld);
}

// pitch (elements) of a token-contiguous copy with bp tokens per row
inline int64_t token_pitch(int64_t bp) { return (bp * 2) % 4096 == 0 ? bp + 64 : bp; }

template <int BM, int BN, int NS>
struct TnSmem {
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;   // one k-step of 64
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int TOTAL = NS * STAGE;                       // ring of NS stages
};

constexpr int TN_THREADS = 512;
enum { EPI_MASKED_PACKED = 0, EPI_PLAIN = 1 };

// Masked, packed epilogue: acc[i][j] of a wavefront is the 16 x 16 fragment at D rows c0 + 16 i (d_in) and D
// columns o0 + 16 j (d_out).  A lane's four accumulators are one group of four along d_in of row o: the
// group's metadata nibble picks the two that W^R keeps.  Stored straight from the registers a pair is a
// 4-byte piece and an instruction touches sixteen rows; so the workgroup's tile of pairs goes through LDS
// (the rings are idle) as [d_out row][pair] and leaves in whole rows, 16 bytes per lane.
// BMT x BNT = the workgroup's tile (d_in x d_out) at (tile_c0, tile_o0); every thread must make the call.
template <int MF, int NF, int BMT, int BNT>
__device__ __forceinline__ void store_masked_packed(const f32x4 (&acc)[MF][NF], int m, int n, int c0, int o0,
                                                    int tile_c0, int tile_o0, int l16, int lq,
                                                    const uint8_t* __restrict__ meta, bf16_t* __restrict__ out,
                                                    uint8_t* smem) {
    constexpr int WM = MF * 16;
    constexpr int CP = BMT + 16;                              // bytes per staged row of pairs: 16 rows x 4 lanes x 4 B
                                                              // of one store fall on 64 different banks
    constexpr int LPR = BMT / 8;                              // 8-byte pieces per row
    const size_t mpitch = (size_t)m / 8, gpitch = (size_t)m / 2;
    __syncthreads();                                          // every wavefront is done with the rings
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        int o = o0 + j * 16 + l16;
        // metadata of the wavefront's WM d_in columns of row o: WM / 4 groups = WM / 8 bytes
        uint32_t mw[WM / 32];
#pragma unroll
        for (int q = 0; q < WM / 32; ++q)
            mw[q] = o < n && c0 + 32 * q < m ? *(const uint32_t*)(meta + (size_t)o * mpitch + c0 / 8 + 4 * q) : 0u;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int gl = i * 4 + lq;                              // group index inside the WM columns
            uint32_t nib = (mw[i >> 1] >> (4 * (gl & 7))) & 0xFu;
            uint32_t a = nib & 3u, c = nib >> 2;
            f32x4 v = acc[i][j];
            float v0 = a == 0 ? v[0] : (a == 1 ? v[1] : v[2]);
            float v1 = c == 1 ? v[1] : (c == 2 ? v[2] : v[3]);
            union { __bf16 h[2]; uint32_t u; } pr;
            pr.h[0] = (__bf16)v0;
            pr.h[1] = (__bf16)v1;
            *(uint32_t*)(smem + (o - tile_o0) * CP + ((c0 - tile_c0) / 4 + gl) * 4) = pr.u;
        }
    }
    __syncthreads();
    // 16-byte pieces (four pairs = sixteen columns of W), all read from LDS before the first is stored; the layers
    // that come here have d_in % 32 == 0, so a piece is inside the row or outside as a whole
    constexpr int PPR = BMT / 16, PER_THREAD = BNT * PPR / TN_THREADS;
    static_assert(BNT * PPR % TN_THREADS == 0 && LPR == 2 * PPR, "whole pieces per thread");
    u32x4 piece[PER_THREAD];
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const int idx = (int)threadIdx.x + u * TN_THREADS;
        piece[u] = *(const u32x4*)(smem + (idx / PPR) * CP + (idx % PPR) * 16);
    }
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const int idx = (int)threadIdx.x + u * TN_THREADS;
        const int o = tile_o0 + idx / PPR, col = tile_c0 + (idx % PPR) * 16;
        if (o < n && col < m) *(u32x4*)(out + (size_t)o * gpitch + (col >> 1)) = piece[u];
    }
}

// Plain epilogue of one wavefront: out[j][i] bf16 row-major [n][m] (row j, four consecutive i per lane), or
// the fp32 accumulators into partial[n][m] for a later reduction.
template <int MF, int NF>
__device__ __forceinline__ void store_plain(const f32x4 (&acc)[MF][NF], int m, int n, int c0, int o0, int l16, int lq,
                                            bf16_t* __restrict__ out, float* __restrict__ partial) {
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        int row = o0 + j * 16 + l16;
        if (row >= n) continue;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int col = c0 + i * 16 + lq * 4;
            if (col >= m) continue;
            f32x4 v = acc[i][j];
            if (partial) {
                *(f32x4*)(partial + (size_t)row * m + col) = v;
                continue;
            }
            union { __bf16 h[4]; u32x2 u; } o;
            o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
            *(u32x2*)(out + (size_t)row * m + col) = o.u;
        }
    }
}

// D[i, j] = sum_k At[i, k] * Bt[j, k];  At: m rows, Bt: n rows, both of pitch ld elements; kp % 64 == 0.
//   EPI_MASKED_PACKED: out = packed gradient [n][m/2] selected by meta (u8[n][m/8])
//   EPI_PLAIN        : out = bf16 [n][m]  (row j, four consecutive i per lane)
// NS = ring depth: loads run NS - 1 k-steps ahead.  Two stages are all that fits beside a 256 x 256
// tile; small tiles (memory-bound skinny products) take a deeper ring to cover the HBM latency.
template <int BM, int BN, int EPI, int NS>
__global__ void __launch_bounds__(TN_THREADS) dense_tn_kernel(const bf16_t* __restrict__ At, int m,
                                                              const bf16_t* __restrict__ Bt, int n, int kp,
                                                              int ld, const uint8_t* __restrict__ meta,
                                                              bf16_t* __restrict__ out, int tiles_m, int tiles_n,
                                                              int slab_steps, float* __restrict__ partial) {
    using S = TnSmem<BM, BN, NS>;
    constexpr int MF = BM / 32, NF = BN / 64;                // 16 x 16 fragments per wavefront (2 x 4 waves)
    constexpr int LD_A = BM / 64, LD_B = BN / 64;            // 1 KiB loads per wavefront per step
    constexpr int WM = BM / 2;                               // rows of D per wavefront
    constexpr int AHEAD = (NS - 2) * (LD_A + LD_B);          // loads that may stay in flight at a wait
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    if (!tile_of_block(tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // loader lanes: 8 lanes per row, chunk rotated by (row / 2) % 8 (rows past the end wrapped, never stored)
    const uint8_t* a_src[LD_A];
    const uint8_t* b_src[LD_B];
#pragma unroll
    for (int i = 0; i < LD_A; ++i) {
        int rl = (wave * LD_A + i) * 8 + (lane >> 3);
        int ra = wrap_row(m0 + rl, m);
        a_src[i] = (const uint8_t*)At + (size_t)ra * ld * 2 + (((lane & 7) ^ ((rl >> 1) & 7)) * 16);
    }
#pragma unroll
    for (int i = 0; i < LD_B; ++i) {
        int rl = (wave * LD_B + i) * 8 + (lane >> 3);
        int rb = wrap_row(n0 + rl, n);
        b_src[i] = (const uint8_t*)Bt + (size_t)rb * ld * 2 + (((lane & 7) ^ ((rl >> 1) & 7)) * 16);
    }
    const int ksteps = kp / 64;
    // with `partial` the k range is cut into slabs of slab_steps k-steps, one per blockIdx.y, each
    // leaving fp32 sums; the look-ahead past a slab's end reads real (unused) data
    const int k_begin = partial ? (int)blockIdx.y * slab_steps : 0;
    const int k_end = partial && k_begin + slab_steps < ksteps ? k_begin + slab_steps : ksteps;
    auto issue = [&](int ks) {                               // k-step ks (clamped) into stage ks % NS
        int kc = ks < ksteps ? ks : ksteps - 1;
        uint8_t* st = smem + (ks % NS) * S::STAGE;
#pragma unroll
        for (int i = 0; i < LD_A; ++i) dma16(a_src[i] + (size_t)kc * 128, st + (wave * LD_A + i) * 1024);
#pragma unroll
        for (int i = 0; i < LD_B; ++i)
            dma16(b_src[i] + (size_t)kc * 128, st + S::A_BYTES + (wave * LD_B + i) * 1024);
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

    // One k-step.  Loads of step s + NS - 1 are queued in the even phase in which their stage, last
    // read for step s - 1, has just been released: group 0 is then in its memory phase of step s,
    // group 1 in its compute phase of step s - 1.  One phase later every wavefront waits until only
    // the loads of steps beyond s + 1 are outstanding, before the barrier after which group 0 reads
    // step s + 1.
#define TN_STEP(G)                                                                                     \
    {                                                                                                  \
        const uint8_t* st = smem + (ks % NS) * S::STAGE;                                               \
        BFrag af[MF], bf[NF];                                                                          \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u[0] = *(const u32x4*)(st + a_rd + i * 2048 + rd0);                                  \
            af[i].u[1] = *(const u32x4*)(st + a_rd + i * 2048 + rd1);                                  \
        }                                                                                              \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(st + b_rd + j * 2048 + rd0);                                  \
            bf[j].u[1] = *(const u32x4*)(st + b_rd + j * 2048 + rd1);                                  \
        }                                                                                              \
        if (G == 0) issue(ks + NS - 1);                                                                \
        /* all LDS reads of this stage have returned before anybody may overwrite it */                \
        WAIT_HERE(waitcnt_imm(G == 1 ? AHEAD : 63, 0));                                                \
        wg_barrier();                                                                                  \
        if (G == 1) issue(ks + NS);                                                                    \
        _Pragma("unroll") for (int h = 0; h < 2; ++h)                                                  \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) _Pragma("unroll") for (int jj = 0; jj < NF; ++jj) { \
            const int j = (i & 1) ? NF - 1 - jj : jj;         /* back and forth: one operand changes per MFMA */ \
            AFrag a, b;                                                                                \
            a.u = af[i].u[h]; b.u = bf[j].u[h];                                                        \
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc[i][j], 0, 0, 0);         \
        }                                                                                              \
        if (G == 0) WAIT_HERE(waitcnt_imm(AHEAD, 15));                                                 \
        wg_barrier();                                                                                  \
    }
#pragma unroll
    for (int p = 0; p < NS - 1; ++p) issue(k_begin + p);
    WAIT_HERE(waitcnt_imm(AHEAD, 15));                        // the first step has landed (this wave's share)
    wg_barrier();
    if (group == 0) {
        for (int ks = k_begin; ks < k_end; ++ks) TN_STEP(0)
        wg_barrier();
    } else {
        issue(k_begin + NS - 1);
        wg_barrier();
        for (int ks = k_begin; ks < k_end; ++ks) TN_STEP(1)
    }
#undef TN_STEP
    WAIT_HERE(waitcnt_imm(0, 15));                            // drain the clamped look-ahead loads

    if (EPI == EPI_PLAIN) {
        store_plain<MF, NF>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, l16, lq, out,
                            partial ? partial + (size_t)blockIdx.y * n * m : nullptr);
        return;
    }
    static_assert(BN * (BM + 16) <= S::TOTAL, "the staged tile of pairs fits in the ring");
    store_masked_packed<MF, NF, BM, BN>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, m0, n0, l16, lq, meta, out, smem);
}

// out = sum over the slabs (in slab order: runs are bit-identical), rounded to bf16; four elements per lane
__global__ void __launch_bounds__(256) partial_reduce_kernel(const f32x4* __restrict__ P, int nslabs, size_t count4,
                                                             u32x2* __restrict__ out) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count4) return;
    f32x4 v = P[idx];
    for (int sl = 1; sl < nslabs; ++sl) {
        f32x4 w = P[(size_t)sl * count4 + idx];
        v[0] += w[0]; v[1] += w[1]; v[2] += w[2]; v[3] += w[3];
    }
    union { __bf16 h[4]; u32x2 u; } o;
    o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
    out[idx] = o.u;
}

// The 256 x 256 tile of the weight gradient with split rings.  A plain two-stage ring (all that
// fits beside such a tile) makes every k-step a burst: nothing may be queued for a stage before
// both groups have read it, and everything queued must have landed one k-step later, so the load
// path runs dry at every step.  Here the two groups take the two column halves of the tile, which
// makes each half of the B panel private to one group, free again as soon as that group has read
// it, while the A panel, read by both, gets a ring of three:
//     A ring  3 x 32 KiB | B half of group 0  2 x 16 KiB | B half of group 1  2 x 16 KiB  = 160 KiB
// Every phase (half a k-step) each wavefront queues four 1 KiB loads
//     even phase 2k  :  B1(k+1), lower half of A(k+2)        odd phase 2k+1 :  upper half of A(k+2), B0(k+2)
// and at the end of every phase waits only for what it queued two or more phases ago (at most
// eight loads stay in flight), which is what the next phase reads.  A stage is always rewritten in
// the first phase after its last reader's barrier.
struct SplitSmem {
    static constexpr int BM = 256, BN = 256;
    static constexpr int A_STAGE = BM * 128, B_HALF = BN / 2 * 128;
    static constexpr int B_OFF = 3 * A_STAGE;                 // then [group][stage] halves of B
    static constexpr int TOTAL = 3 * A_STAGE + 4 * B_HALF;
};

// TAIL: the tiles left over after the last full round of 256.  Run as a round of their own they would
// keep a few compute units busy for a whole tile's time while the rest of the chip idles.  Instead each
// of them (positions first_tile .. first_tile + tail_tiles - 1 of the tile order) is cut along k into
// slabs of slab_steps k-steps; workgroup w takes tile w % tail_tiles, slab w / tail_tiles, and leaves its
// fp32 accumulators in partial[w] in register order; tail_reduce_kernel adds the slabs and stores.
template <int EPI, bool TAIL>
__global__ void __launch_bounds__(TN_THREADS) dense_tn_split_kernel(const bf16_t* __restrict__ At, int m,
                                                                    const bf16_t* __restrict__ Bt, int n, int kp,
                                                                    int ld, const uint8_t* __restrict__ meta,
                                                                    bf16_t* __restrict__ out, int tiles_m,
                                                                    int tiles_n, int first_tile, int tail_tiles,
                                                                    int slab_steps, f32x4* __restrict__ partial) {
    using S = SplitSmem;
    constexpr int MF = 8, NF = 4, WM = 128;                  // wavefront tile 128 x 64, 2 x 4 wavefronts
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn, k_first = 0;
    if (TAIL) {
        tile_of_position(first_tile + (int)blockIdx.x % tail_tiles, tiles_m, tiles_n, tm, tn);
        k_first = ((int)blockIdx.x / tail_tiles) * slab_steps;
    } else if (!tile_of_block(tiles_m, tiles_n, tm, tn)) {
        return;
    }
    const int m0 = tm * S::BM, n0 = tn * S::BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;                             // = column half of the tile
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // loader lanes: 8 lanes per row, chunk rotated by (row / 2) % 8 (rows past the end wrapped, never stored).
    // Each load set (half of A, half of B) is 16 loads of 8 rows: two per wavefront.
    const uint8_t* a_src[4];                                 // [half * 2 + i]
    const uint8_t* b_src[4];                                 // [group * 2 + i]
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int rl = ((q >> 1) * 16 + wave * 2 + (q & 1)) * 8 + (lane >> 3);     // row inside the tile
        int sw16 = ((lane & 7) ^ ((rl >> 1) & 7)) * 16;
        int ra = wrap_row(m0 + rl, m);
        int rb = wrap_row(n0 + rl, n);
        a_src[q] = (const uint8_t*)At + (size_t)ra * ld * 2 + sw16 + (size_t)k_first * 128;
        b_src[q] = (const uint8_t*)Bt + (size_t)rb * ld * 2 + sw16 + (size_t)k_first * 128;
    }
    // k-steps of this workgroup (the host leaves no slab empty)
    const int ksteps = TAIL ? (kp / 64 - k_first < slab_steps ? kp / 64 - k_first : slab_steps) : kp / 64;
    // the four loads a wavefront queues per phase, one at a time (ks clamped: the look-ahead of the
    // last steps re-reads the last one)
    auto issue_a = [&](int half, int ks, int i) {            // 8 rows of rows 128 half .. +127 of A(ks)
        int kc = ks < ksteps ? ks : ksteps - 1;
        dma16(a_src[half * 2 + i] + (size_t)kc * 128, smem + (ks % 3) * S::A_STAGE + (half * 16 + wave * 2 + i) * 1024);
    };
    auto issue_b = [&](int g, int ks, int i) {               // 8 rows of the B half of group g, step ks
        int kc = ks < ksteps ? ks : ksteps - 1;
        dma16(b_src[g * 2 + i] + (size_t)kc * 128, smem + S::B_OFF + (g * 2 + (ks & 1)) * S::B_HALF + (wave * 2 + i) * 1024);
    };
    auto even_load = [&](int k, int idx) { if (idx < 2) issue_b(1, k + 1, idx); else issue_a(0, k + 2, idx - 2); };
    auto odd_load = [&](int k, int idx) { if (idx < 2) issue_a(1, k + 2, idx); else issue_b(0, k + 2, idx - 2); };

    // reader lanes: fragment f = rows 16f .. 16f+15 = 2 KiB; lane (l16, lq) wants chunk 4h + lq
    const int sw = (l16 >> 1) & 7;
    const int rd0 = l16 * 128 + ((lq ^ sw) * 16);
    const int rd1 = l16 * 128 + (((4 + lq) ^ sw) * 16);
    const int a_rd = (wm * MF) * 2048;
    const int b_rd = S::B_OFF + group * 2 * S::B_HALF + ((wn & 1) * NF) * 2048;

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    constexpr int KEEP = 8;                                  // loads of the last two phases
#define SPLIT_READ(ks)                                                                                 \
        const uint8_t* sa = smem + ((ks) % 3) * S::A_STAGE + a_rd;                                     \
        const uint8_t* sb = smem + b_rd + ((ks) & 1) * S::B_HALF;                                      \
        BFrag af[MF], bf[NF];                                                                          \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u[0] = *(const u32x4*)(sa + i * 2048 + rd0);                                         \
            af[i].u[1] = *(const u32x4*)(sa + i * 2048 + rd1);                                         \
        }                                                                                              \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(sb + j * 2048 + rd0);                                         \
            bf[j].u[1] = *(const u32x4*)(sb + j * 2048 + rd1);                                         \
        }
// the compute phase: 64 MFMAs with the phase's four loads spread between them (queued in one burst
// at the start of the phase they cost 2 % more).  The B fragments are taken back and forth, so that only
// one operand changes from one MFMA to the next: the kernel runs at the clock the chip's power limit
// allows, and that order draws measurably less (1.7 % faster than always restarting at fragment 0).
#define SPLIT_MFMA(LOAD, k)                                                                            \
        _Pragma("unroll") for (int h = 0; h < 2; ++h)                                                  \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            _Pragma("unroll") for (int jj = 0; jj < NF; ++jj) {                                        \
                const int j = (i & 1) ? NF - 1 - jj : jj;                                              \
                AFrag a, b;                                                                            \
                a.u = af[i].u[h]; b.u = bf[j].u[h];                                                    \
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc[i][j], 0, 0, 0);     \
            }                                                                                          \
            if (h == 0 && (i & 1) == 1) LOAD(k, i >> 1);                                               \
            __builtin_amdgcn_sched_barrier(0);                                                         \
        }
#define EVEN_LOADS(k) { even_load(k, 0); even_load(k, 1); even_load(k, 2); even_load(k, 3); }
#define ODD_LOADS(k)  { odd_load(k, 0); odd_load(k, 1); odd_load(k, 2); odd_load(k, 3); }

    // steps 0 and 1 as far as the schedule would have queued them before phase 0
    issue_a(0, 0, 0); issue_a(0, 0, 1); issue_a(1, 0, 0); issue_a(1, 0, 1); issue_b(0, 0, 0); issue_b(0, 0, 1);
    issue_b(1, 0, 0); issue_b(1, 0, 1); issue_a(0, 1, 0); issue_a(0, 1, 1);
    issue_a(1, 1, 0); issue_a(1, 1, 1); issue_b(0, 1, 0); issue_b(0, 1, 1);
    WAIT_HERE(waitcnt_imm(KEEP, 15));                         // A(0) and B0(0) have landed
    wg_barrier();
    if (group == 0) {
        for (int ks = 0; ks < ksteps; ++ks) {
            SPLIT_READ(ks)                                    // phase 2 ks
            EVEN_LOADS(ks)
            WAIT_HERE(waitcnt_imm(KEEP, 0));
            wg_barrier();
            SPLIT_MFMA(odd_load, ks)                          // phase 2 ks + 1
            WAIT_HERE(waitcnt_imm(KEEP, 15));
            wg_barrier();
        }
        wg_barrier();                                         // group 1's last compute phase
    } else {
        EVEN_LOADS(0)                                         // phase 0: nothing to compute yet
        WAIT_HERE(waitcnt_imm(KEEP, 15));
        wg_barrier();
        for (int ks = 0; ks < ksteps; ++ks) {
            SPLIT_READ(ks)                                    // phase 2 ks + 1
            ODD_LOADS(ks)
            WAIT_HERE(waitcnt_imm(KEEP, 0));
            wg_barrier();
            SPLIT_MFMA(even_load, ks + 1)                     // phase 2 ks + 2
            WAIT_HERE(waitcnt_imm(KEEP, 15));
            wg_barrier();
        }
    }
#undef SPLIT_READ
#undef SPLIT_MFMA
#undef EVEN_LOADS
#undef ODD_LOADS
    WAIT_HERE(waitcnt_imm(0, 15));                            // drain the clamped look-ahead loads
    if (TAIL) {
        f32x4* dst = partial + (size_t)blockIdx.x * (MF * NF * TN_THREADS) + t;
#pragma unroll
        for (int i = 0; i < MF; ++i)
#pragma unroll
            for (int j = 0; j < NF; ++j) dst[(i * NF + j) * TN_THREADS] = acc[i][j];
        return;
    }
    if (EPI == EPI_PLAIN) store_plain<MF, NF>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, l16, lq, out, nullptr);
    else store_masked_packed<MF, NF, S::BM, S::BN>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, m0, n0, l16, lq, meta, out,
                                                   smem);
}

// Second pass of the tail, in two kernels.  tail_sum_kernel adds the slabs element by element in slab
// order into slab 0 (slab sl of a tile lies tail_tiles tiles further on in `partial`); it has a workgroup
// per 256 elements, because the few workgroups of tail_reduce_kernel alone would read the partial sums at
// a small fraction of the chip's bandwidth.  tail_reduce_kernel then loads a tile's sums in the register
// layout dense_tn_split_kernel left them in and stores the tile through that kernel's epilogue.
__global__ void __launch_bounds__(256) tail_sum_kernel(f32x4* __restrict__ partial, int nslabs, size_t slab_stride4,
                                                       size_t count4) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count4) return;
    f32x4 v = partial[idx];
    for (int sl = 1; sl < nslabs; ++sl) {
        f32x4 w = partial[(size_t)sl * slab_stride4 + idx];
        v[0] += w[0]; v[1] += w[1]; v[2] += w[2]; v[3] += w[3];
    }
    partial[idx] = v;
}

constexpr int TAIL_REDUCE_LDS = SplitSmem::BN * (SplitSmem::BM + 16);
template <int EPI>
__global__ void __launch_bounds__(TN_THREADS) tail_reduce_kernel(const f32x4* __restrict__ partial, int m, int n,
                                                                 const uint8_t* __restrict__ meta,
                                                                 bf16_t* __restrict__ out, int tiles_m, int tiles_n,
                                                                 int first_tile) {
    using S = SplitSmem;
    constexpr int MF = 8, NF = 4, WM = 128;
    extern __shared__ __align__(16) uint8_t smem[];
    int tm, tn;
    tile_of_position(first_tile + (int)blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int m0 = tm * S::BM, n0 = tn * S::BN;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave & 1, wn = wave >> 1, l16 = lane & 15, lq = lane >> 4;
    f32x4 acc[MF][NF];
    const f32x4* src = partial + (size_t)blockIdx.x * (MF * NF * TN_THREADS) + t;
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = src[(i * NF + j) * TN_THREADS];
    if (EPI == EPI_PLAIN) store_plain<MF, NF>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, l16, lq, out, nullptr);
    else store_masked_packed<MF, NF, S::BM, S::BN>(acc, m, n, m0 + wm * WM, n0 + wn * NF * 16, m0, n0, l16, lq, meta, out,
                                                   smem);
}

template <int BM, int BN, int EPI, int NS>
hipError_t launch_dense_tn(const bf16_t* At, int64_t m, const bf16_t* Bt, int64_t n, int64_t kp, int64_t ld,
                           const uint8_t* meta, bf16_t* out, hipStream_t s, int nslabs = 1, int slab_steps = 0,
                           float* partial = nullptr) {
    using S = TnSmem<BM, BN, NS>;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    auto kern = dense_tn_kernel<BM, BN, EPI, NS>;
    hipError_t e = allow_dynamic_lds<dense_tn_kernel<BM, BN, EPI, NS>>(S::TOTAL);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)super_grid(tiles_m, tiles_n), (unsigned)nslabs), dim3(TN_THREADS), S::TOTAL, s>>>(
        At, (int)m, Bt, (int)n, (int)kp, (int)ld, meta, out, tiles_m, tiles_n, slab_steps, partial);
    return hipGetLastError();
}

// How the tiles left over after the last full round are cut: tail tiles (0 = none worth cutting), slabs
// per tile, k-steps per slab.  Only wide grids (the tile order has positions there), only leftovers of at
// most half a round (more would be cut into too few slabs to gain), at least eight k-steps per slab.
struct TailPlan { int first_tile, tiles, slabs, slab_steps; };
inline TailPlan tail_plan(int64_t tiles_m, int64_t tiles_n, int64_t ksteps) {
    TailPlan p = {0, 0, 0, 0};
    const int64_t tiles = tiles_m * tiles_n;
    if (!wide_grid((int)tiles_m, (int)tiles_n) || tiles < RESIDENT || tiles > (1 << 30)) return p;
    const int64_t rem = tiles % RESIDENT;
    if (rem == 0 || rem > RESIDENT / 2) return p;
    int64_t slabs = RESIDENT / rem;
    if (slabs > ksteps / 8) slabs = ksteps / 8;
    if (slabs < 2) return p;
    const int64_t steps = (ksteps + slabs - 1) / slabs;
    p.first_tile = (int)(tiles - rem);
    p.tiles = (int)rem;
    p.slab_steps = (int)steps;
    p.slabs = (int)((ksteps + steps - 1) / steps);
    return p;
}

template <int EPI>
hipError_t launch_dense_tn_split(const bf16_t* At, int64_t m, const bf16_t* Bt, int64_t n, int64_t kp, int64_t ld,
                                 const uint8_t* meta, bf16_t* out, hipStream_t s, float* tail = nullptr) {
    using S = SplitSmem;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    int tiles_m = (int)((m + S::BM - 1) / S::BM), tiles_n = (int)((n + S::BN - 1) / S::BN);
    hipError_t e = allow_dynamic_lds<dense_tn_split_kernel<EPI, false>>(S::TOTAL);
    if (e != hipSuccess) return e;
    const TailPlan p = tail ? tail_plan(tiles_m, tiles_n, kp / 64) : TailPlan{0, 0, 0, 0};
    // with a tail the first launch is whole rounds only: workgroups 0 .. first_tile - 1 are exactly the
    // positions 0 .. first_tile - 1 of the order
    const int grid = p.tiles ? p.first_tile : super_grid(tiles_m, tiles_n);
    dense_tn_split_kernel<EPI, false><<<dim3((unsigned)grid), dim3(TN_THREADS), S::TOTAL, s>>>(
        At, (int)m, Bt, (int)n, (int)kp, (int)ld, meta, out, tiles_m, tiles_n, 0, 0, 0, nullptr);
    if ((e = hipGetLastError()) != hipSuccess || !p.tiles) return e;
    if ((e = allow_dynamic_lds<dense_tn_split_kernel<EPI, true>>(S::TOTAL)) != hipSuccess) return e;
    if ((e = allow_dynamic_lds<tail_reduce_kernel<EPI>>(TAIL_REDUCE_LDS)) != hipSuccess) return e;
    dense_tn_split_kernel<EPI, true><<<dim3((unsigned)(p.tiles * p.slabs)), dim3(TN_THREADS), S::TOTAL, s>>>(
        At, (int)m, Bt, (int)n, (int)kp, (int)ld, meta, out, tiles_m, tiles_n, p.first_tile, p.tiles, p.slab_steps,
        (f32x4*)tail);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const size_t count4 = (size_t)p.tiles * (S::BM * S::BN / 4);
    tail_sum_kernel<<<dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s>>>((f32x4*)tail, p.slabs, count4, count4);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tail_reduce_kernel<EPI><<<dim3((unsigned)p.tiles), dim3(TN_THREADS), TAIL_REDUCE_LDS, s>>>(
        (const f32x4*)tail, (int)m, (int)n, meta, out, tiles_m, tiles_n, p.first_tile);
    return hipGetLastError();
}

}  // namespace

namespace {
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }
}  // namespace

// Token-contiguous copy of a [b][d] activation: d rows of token_pitch(b rounded up to 64) elements.
size_t token_copy_bytes(int64_t b, int64_t d) { return (size_t)d * (size_t)token_pitch((b + 63) / 64 * 64) * 2; }

// One or two copies (in1 == nullptr: one) of matrices with b rows in one launch.
hipError_t launch_token_copies(const bf16_t* in0, int64_t cols0, bf16_t* out0, const bf16_t* in1, int64_t cols1,
                               bf16_t* out1, int64_t b, hipStream_t s) {
    const int64_t bp = (b + 63) / 64 * 64, ld = token_pitch(bp);
    if (in1) launch_transpose_pad2(in0, cols0, out0, in1, cols1, out1, b, bp, ld, s);
    else launch_transpose_pad(in0, b, cols0, bp, ld, out0, s);
    return hipGetLastError();
}

// The packed epilogue reads the metadata of 32 columns of W^R as one dword: rows of d_in / 8 bytes must
// keep those dwords aligned.  Other layers take the in-place kernel.
bool wgrad_tn_fits(int64_t d_in) { return d_in % 32 == 0; }

// Tile shape of the weight gradient: 0 = 256 x 256 (split rings), 1 = 256 x 128, 2 = 128 x 128, 3 = 128 x 64.
// The kernels run at the rate their compute units pull operands from L2: a launch costs about (rounds of
// 256 resident tiles) x (rows per tile).  Take the cheapest shape, the larger on ties.  With scratch memory
// the 256 x 256 kernel cuts the tiles left over after its last full round along the tokens
// (launch_dense_tn_split): they then cost about 1 / slabs of a round, plus a quarter for the second pass.
static int wgrad_tile_choice(int64_t d_in, int64_t d_out, int64_t ksteps, bool with_tail) {
    const int bms[4] = {256, 256, 128, 128}, bns[4] = {256, 128, 128, 64};
    int best = 0;
    int64_t best_cost = INT64_MAX;
    for (int c = 0; c < 4; ++c) {
        const int64_t tm = (d_in + bms[c] - 1) / bms[c], tn = (d_out + bns[c] - 1) / bns[c], tiles = tm * tn;
        int64_t cost = ((tiles + RESIDENT - 1) / RESIDENT) * (bms[c] + bns[c]) * 100;
        if (c == 0 && with_tail) {
            const TailPlan p = tail_plan(tm, tn, ksteps);
            if (p.tiles) cost = (tiles / RESIDENT) * 512 * 100 + 512 * (100 / p.slabs + 25);
        }
        if (cost < best_cost) { best_cost = cost; best = c; }
    }
    return best;
}

// scratch bytes of launch_wgrad_masked_t's tail pass (0: the shape has none)
size_t wgrad_tail_bytes(int64_t b, int64_t d_in, int64_t d_out) {
    const int64_t ksteps = (b + 63) / 64;
    if (wgrad_tile_choice(d_in, d_out, ksteps, true) != 0) return 0;
    const TailPlan p = tail_plan((d_in + 255) / 256, (d_out + 255) / 256, ksteps);
    return (size_t)p.tiles * (size_t)p.slabs * (256 * 256 * 4);
}

// dW (masked, packed) from token-contiguous copies Xt [d_in][ld], dYt [d_out][ld]; tail_or_null: scratch of
// wgrad_tail_bytes(b, d_in, d_out) bytes, or nullptr (then a last partial round of tiles runs as it is)
hipError_t launch_wgrad_masked_t(const bf16_t* dYt, const bf16_t* Xt, int64_t b, const uint8_t* meta, int64_t d_out,
                                 int64_t d_in, bf16_t* gvals, float* tail_or_null, hipStream_t s) {
    const int64_t bp = (b + 63) / 64 * 64, ld = token_pitch(bp);
    const int best = wgrad_tile_choice(d_in, d_out, bp / 64, tail_or_null != nullptr);
    if (best == 0)
        return launch_dense_tn_split<EPI_MASKED_PACKED>(Xt, d_in, dYt, d_out, bp, ld, meta, gvals, s, tail_or_null);
    if (best == 1) return launch_dense_tn<256, 128, EPI_MASKED_PACKED, 3>(Xt, d_in, dYt, d_out, bp, ld, meta, gvals, s);
    if (best == 2) return launch_dense_tn<128, 128, EPI_MASKED_PACKED, 4>(Xt, d_in, dYt, d_out, bp, ld, meta, gvals, s);
    return launch_dense_tn<128, 64, EPI_MASKED_PACKED, 6>(Xt, d_in, dYt, d_out, bp, ld, meta, gvals, s);
}

// C[n, m] = B[n, K] * A[m, K]^T, all bf16 row-major, K % 64 == 0 (the skinny product T = X L of the
// adapter: m = rank).  The product is bound by streaming B once: narrow token tiles so that even
// m = 128 gives every compute unit a tile, and a six-deep ring to keep enough reads in flight.
//
// A few hundred to a few thousand tokens give that product only a handful of tiles with a long
// contraction each.  With scratch memory (`partial`, dense_tn_plain_partial_bytes(n, m) bytes) the
// contraction is then cut into slabs that run as separate workgroups, about 256 in all, and leave
// fp32 sums that a second kernel adds in slab order.
size_t dense_tn_plain_partial_bytes(int64_t n, int64_t m) {
    const int64_t tiles = ((m + 127) / 128) * ((n + 63) / 64);
    if (tiles >= RESIDENT / 2) return 0;
    return (size_t)((RESIDENT + tiles - 1) / tiles) * (size_t)n * (size_t)m * 4;
}

hipError_t launch_dense_tn_plain(const bf16_t* B, int64_t n, const bf16_t* A, int64_t m, int64_t K, bf16_t* C,
                                 float* partial, hipStream_t s) {
    const int64_t tiles = ((m + 127) / 128) * ((n + 63) / 64), ksteps = K / 64;
    int64_t nslabs = partial && tiles < RESIDENT / 2 ? (RESIDENT + tiles - 1) / tiles : 1;
    if (nslabs > ksteps / 8) nslabs = ksteps / 8;            // at least eight k-steps per slab
    if (nslabs <= 1) return launch_dense_tn<128, 64, EPI_PLAIN, 6>(A, m, B, n, K, K, nullptr, C, s);
    const int64_t slab_steps = (ksteps + nslabs - 1) / nslabs;
    nslabs = (ksteps + slab_steps - 1) / slab_steps;
    hipError_t e = launch_dense_tn<128, 64, EPI_PLAIN, 6>(A, m, B, n, K, K, nullptr, C, s, (int)nslabs, (int)slab_steps,
                                                          partial);
    if (e != hipSuccess) return e;
    const size_t count4 = (size_t)n * (size_t)m / 4;
    partial_reduce_kernel<<<dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s>>>((const f32x4*)partial, (int)nslabs,
                                                                                     count4, (u32x2*)C);
    return hipGetLastError();
}

// The same product for any shape (dense weights with a general N:M mask, where no sparse MFMA
// applies): tile by the rounds x operand-rows estimate of the other tile kernels.
hipError_t launch_dense_tn_any(const bf16_t* B, int64_t n, const bf16_t* A, int64_t m, int64_t K, bf16_t* C,
                               hipStream_t s) {
    const int bms[4] = {256, 256, 128, 128}, bns[4] = {256, 128, 128, 64};
    int best = 0;
    int64_t best_cost = INT64_MAX;
    for (int c = 0; c < 4; ++c) {
        int64_t tiles = ((m + bms[c] - 1) / bms[c]) * ((n + bns[c] - 1) / bns[c]);
        int64_t cost = ((tiles + RESIDENT - 1) / RESIDENT) * (bms[c] + bns[c]);
        if (cost < best_cost) { best_cost = cost; best = c; }
    }
    switch (best) {
        case 0: return launch_dense_tn_split<EPI_PLAIN>(A, m, B, n, K, K, nullptr, C, s);
        case 1: return launch_dense_tn<256, 128, EPI_PLAIN, 3>(A, m, B, n, K, K, nullptr, C, s);
        case 2: return launch_dense_tn<128, 128, EPI_PLAIN, 4>(A, m, B, n, K, K, nullptr, C, s);
        default: return launch_dense_tn<128, 64, EPI_PLAIN, 6>(A, m, B, n, K, K, nullptr, C, s);
    }
}

// ------------------------------------------------------------------------------------------
// Weight gradient of a layer with adapters: the packed dW as above plus the adapter gradients
// (chain rule of Eq. 11)   dL = X^T (dY R^T)  [d_in, r],   dR = (X L)^T dY  [r, d_out],
// all three contractions over the tokens sharing the token-contiguous copies of X and dY.
// Workspace: Xt | dYt | Lt [r][d_in] | T = X L [b][r] | T2 = dY R^T [b][r] | Tt [r][ld] | T2t [r][ld] | the
// scratch of launch_wgrad_masked_t.
size_t wgrad_adapter_workspace_bytes(int64_t b, int64_t d_in, int64_t d_out, int64_t r) {
    size_t ld = (size_t)token_pitch((b + 63) / 64 * 64);
    return round256(token_copy_bytes(b, d_in)) + round256(token_copy_bytes(b, d_out)) + round256((size_t)r * d_in * 2) +
           2 * round256((size_t)b * r * 2) + 2 * round256((size_t)r * ld * 2) + wgrad_tail_bytes(b, d_in, d_out);
}

hipError_t launch_wgrad_adapter(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out,
                                int64_t d_in, const bf16_t* L, const bf16_t* R, int64_t r, bf16_t* gvals, bf16_t* dL,
                                bf16_t* dR, void* workspace, hipStream_t s) {
    const int64_t bp = (b + 63) / 64 * 64, ld = token_pitch(bp);
    uint8_t* w = (uint8_t*)workspace;
    bf16_t* Xt = (bf16_t*)w;   w += round256(token_copy_bytes(b, d_in));
    bf16_t* dYt = (bf16_t*)w;  w += round256(token_copy_bytes(b, d_out));
    bf16_t* Lt = (bf16_t*)w;   w += round256((size_t)r * d_in * 2);
    bf16_t* T = (bf16_t*)w;    w += round256((size_t)b * r * 2);
    bf16_t* T2 = (bf16_t*)w;   w += round256((size_t)b * r * 2);
    bf16_t* Tt = (bf16_t*)w;   w += round256((size_t)r * ld * 2);
    bf16_t* T2t = (bf16_t*)w;  w += round256((size_t)r * ld * 2);
    float* tail = wgrad_tail_bytes(b, d_in, d_out) ? (float*)w : nullptr;

    hipError_t e;
    if (d_in % 64 != 0 || d_out % 64 != 0) {
        // Extents that are not whole k-steps of the MFMA kernels: the in-place kernel for dW and plain
        // arithmetic for the four skinny products (T and T2 rounded to bf16 as on the fast path).
        if ((e = launch_wgrad_masked(dY, X, b, meta, d_out, d_in, gvals, s)) != hipSuccess) return e;
        if ((e = launch_plain_gemm(X, d_in, 1, L, 1, r, b, r, d_in, T, s)) != hipSuccess) return e;        // T  = X L
        if ((e = launch_plain_gemm(dY, d_out, 1, R, d_out, 1, b, r, d_out, T2, s)) != hipSuccess) return e; // T2 = dY R^T
        if ((e = launch_plain_gemm(X, 1, d_in, T2, 1, r, d_in, r, b, dL, s)) != hipSuccess) return e;       // dL = X^T T2
        return launch_plain_gemm(T, 1, r, dY, 1, d_out, r, d_out, b, dR, s);                               // dR = T^T dY
    }
    if ((e = launch_token_copies(X, d_in, Xt, dY, d_out, dYt, b, s)) != hipSuccess) return e;
    if ((e = launch_wgrad_masked_t(dYt, Xt, b, meta, d_out, d_in, gvals, tail, s)) != hipSuccess) return e;
    launch_transpose_pad(L, d_in, r, d_in, d_in, Lt, s);                          // Lt[r][d_in]
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = launch_dense_tn_plain(X, b, Lt, r, d_in, T, nullptr, s)) != hipSuccess) return e;      // T  = X L
    if ((e = launch_dense_tn_plain(dY, b, R, r, d_out, T2, nullptr, s)) != hipSuccess) return e;    // T2 = dY R^T
    launch_transpose_pad2(T, r, Tt, T2, r, T2t, b, bp, ld, s);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    e = launch_dense_tn<128, 64, EPI_PLAIN, 6>(T2t, r, Xt, d_in, bp, ld, nullptr, dL, s);   // dL[d_in][r]
    if (e != hipSuccess) return e;
    return launch_dense_tn<128, 64, EPI_PLAIN, 6>(dYt, d_out, Tt, r, bp, ld, nullptr, dR, s);   // dR[r][d_out]
}
