// 2:4 sparse x dense product on CDNA4's structured-sparse MFMA, shared by
// slope_spmm_fwd (Eq. 4, with the low-rank K-extension of Eq. 11) and slope_spmm_bwd_x (Eq. 6).
//
//     C[n, m] = sum_k B[n, k] * A[m, k]        A: packed 2:4 along k (vals + 4-bit metadata)
//             + sum_k2 B2[n, k2] * A2[m, k2]   dense bf16, K2 = adapter rank (optional)
//
// fwd  : A = W^R        (m = d_out, k = d_in ), B = X,  C = Y,  B2 = X L, A2 = R^T given as R (k-major)
// bwd_x: A = (W^{R,C})^T (m = d_in,  k = d_out), B = dY, C = dX (with adapters: B2 = dY R^T, A2 = L)
//
// The instruction is v_smfmac_f32_16x16x64_bf16 (D[16 x 16] += Asparse[16 x 64] * B[64 x 16]):
//   A   lane l holds row l%16 and the 8 packed values of logical k = 16*(l/16) .. +15
//   idx lane l holds the 4 metadata nibbles of those 16 k in bits 0..15 (idx0 | idx1 << 2 each)
//   B   lane l holds column l%16; registers 0-3 = k 8*(l/16) .. +7, registers 4-7 = 32 + the same
//   D   lane l holds column l%16, rows 4*(l/16) .. +3
// so the sparse operand is the weight, rows of D are output features, and a lane's four
// accumulators are four consecutive features of one token: an 8-byte store into row-major C.
//
// Three kernels here (launch_spmm picks; the forms for very few tokens are in spmm_stream.hip):
// spmm_kernel<BM, BN> and spmm_split_kernel (the 256 x 256 tile) are the fast ones and need
// K % 256 == 0; spmm_generic_kernel takes any K % 64 == 0 with a plain register-staged pipeline.
//
// spmm_kernel.  What a compute unit can pull from L2 per unit of time matters as much as the matrix
// pipe (whose clock the power management lowers well below nominal under this load), so the data
// path is built around full 128-byte lines:
//   - every global -> LDS load instruction (global_load_lds_dwordx4, no registers in between)
//     fetches 8 rows x 128 contiguous bytes, 8 consecutive lanes per row;
//   - a row of the token operand has 128 bytes per k-step of 64, so B sits in a ring of three
//     k-step stages; a row of the packed weight has only 64, so A is fetched for two k-steps at
//     a time into two alternating pair buffers, and its metadata for four k-steps at a time;
//   - inside a row the eight 16-byte chunks are rotated by (row / 2) % 8, which makes the
//     ds_read_b128 of the MFMA layout (16 lanes = 16 rows, same chunk) hit 16 different bank groups.
// A workgroup owns a BM x BN tile of C with 8 wavefronts (2 x 4, two per SIMD) in two groups that
// run half a k-step apart: while one group issues its MFMAs the other reads its fragments from
// LDS and queues global loads, then they swap (two barriers per k-step), so every SIMD's matrix
// pipe always has a wavefront feeding it.  Loads run two k-steps ahead of their use.
#include "pipeline.h"

namespace {

// Tail shared by the tile kernels, for one wavefront whose acc[i][j] is the 16 x 16 fragment at
// features f0 + 16 i, tokens t0 + 16 j.
//  - dense K-extension: C += B2 * A2^T with v_mfma_f32_16x16x32_bf16.  K2 > 0: A2 is [m][K2],
//    k-contiguous like B2, and both operands come straight from global memory (lane l: row l%16,
//    k = 8*(l/16) .. +7).  K2 < 0: A2 is k-major, [-K2][m] (the adapter factor R as stored): the
//    workgroup stages the tile's BMT columns of 128 rows at a time in LDS (the rings are idle by
//    then) and the wavefronts read their fragments back with the transposing LDS read; every
//    thread of the workgroup must make the call (it contains barriers);
//  - epilogue: a lane holds four consecutive features of one token.  Stored straight from the registers that
//    is 8 bytes per lane in pieces of 32 contiguous bytes: sixteen rows per instruction, each a partial
//    line.  So the workgroup's tile goes through LDS (the rings are idle by then) as [token][feature] rows
//    and leaves in whole rows: 16 bytes per lane, up to 512 contiguous bytes per half wavefront.
//    BNT = tokens of the workgroup's tile, tile_t0 its first token; every thread must make the call.
//  - with a slab buffer (a split over k, see launch_spmm_slabs): the fp32 accumulators go to
//    partial[token][feature] instead, 16 bytes per lane, and a reduction kernel finishes.
template <int MF, int NF, int BMT, int BNT, int THREADS>
__device__ __forceinline__ void extend_and_store(f32x4 (&acc)[MF][NF], int f0, int t0, int m, int n, int l16, int lq,
                                                 const bf16_t* __restrict__ B2, const bf16_t* __restrict__ A2,
                                                 int K2, bf16_t* __restrict__ C, uint8_t* smem, int tile_f0,
                                                 int tile_t0, float* __restrict__ partial = nullptr) {
    if (K2 < 0) {
        constexpr int PITCH = BMT * 2 + 32;                   // pitch % 128 == 32: the four rows of a transposing
                                                              // read fall on distinct banks
        constexpr int SEG = BMT / 8;                          // 16-byte pieces per staged row
        const int KR = -K2, tid = (int)threadIdx.x;
        const bf16_t* b_row[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) b_row[j] = B2 + (size_t)wrap_row(t0 + j * 16 + l16, n) * KR + lq * 8;
        // lane (s = l16, q = lq) points at staged row 8 q + 4 h + s / 4, column 4 (s % 4) of a fragment
        const uint8_t* tr = smem + (8 * lq + (l16 >> 2)) * PITCH + 2 * (f0 - tile_f0 + 4 * (l16 & 3));
        // pieces of the staged chunk per thread: a compile-time count, so that all of a thread's global loads are
        // in flight together (a loop of load, wait, LDS store per piece pays the L2 latency once per piece)
        constexpr int PER = 128 * SEG / THREADS;
        static_assert(128 * SEG % THREADS == 0, "whole pieces per thread");
        for (int kc = 0; kc < KR; kc += 128) {
            const int kn = KR - kc < 128 ? KR - kc : 128;     // a multiple of 32
            // the token-side fragments of the whole chunk come straight from global memory: requested first
            // (steps past the chunk's end re-read the first, unused)
            AFrag b2[4][NF];
#pragma unroll
            for (int st = 0; st < 2; ++st)
#pragma unroll
                for (int j = 0; j < NF; ++j) b2[st][j].u = *(const u32x4*)(b_row[j] + kc + (32 * st < kn ? 32 * st : 0));
            u32x4 piece[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int idx = tid + u * THREADS, k = idx / SEG, col = tile_f0 + 8 * (idx % SEG);
                piece[u] = (u32x4){0u, 0u, 0u, 0u};
                if (k < kn && col < m) piece[u] = *(const u32x4*)(A2 + (size_t)(kc + k) * m + col);
            }
            __syncthreads();                                  // the rings are drained / the last chunk is consumed
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int idx = tid + u * THREADS;
                *(u32x4*)(smem + (idx / SEG) * PITCH + (idx % SEG) * 16) = piece[u];
            }
#pragma unroll
            for (int st = 2; st < 4; ++st)                    // in the registers the staged pieces have left
#pragma unroll
                for (int j = 0; j < NF; ++j) b2[st][j].u = *(const u32x4*)(b_row[j] + kc + (32 * st < kn ? 32 * st : 0));
            __syncthreads();
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const int kk = 32 * st;
                if (kk >= kn) break;                          // uniform
#pragma unroll
                for (int i = 0; i < MF; ++i) {
                    union { s16x4 hh[2]; bf16x8 v; } a;
                    a.hh[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(tr + kk * PITCH + 32 * i));
                    a.hh[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(tr + (kk + 4) * PITCH + 32 * i));
#pragma unroll
                    for (int j = 0; j < NF; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b2[st][j].v, acc[i][j], 0, 0, 0);
                }
            }
        }
    }
    if (K2 > 0) {
        // operands of step k0 + 32 are requested before the MFMAs of step k0 are issued
        const bf16_t* a_row[MF];
        const bf16_t* b_row[NF];
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int row = f0 + i * 16 + l16;
            a_row[i] = A2 + (size_t)wrap_row(row, m) * K2 + lq * 8;
        }
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            int row = t0 + j * 16 + l16;
            b_row[j] = B2 + (size_t)wrap_row(row, n) * K2 + lq * 8;
        }
        AFrag a2[2][MF], b2[2][NF];
#pragma unroll
        for (int i = 0; i < MF; ++i) a2[0][i].u = *(const u32x4*)(a_row[i]);
#pragma unroll
        for (int j = 0; j < NF; ++j) b2[0][j].u = *(const u32x4*)(b_row[j]);
        for (int k0 = 0; k0 < K2; k0 += 64) {                 // K2 % 32 == 0: two steps per trip, the second maybe absent
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kk = k0 + 32 * h;                   // uniform
                if (kk >= K2) break;
                const int kn = kk + 32 < K2 ? kk + 32 : kk;   // the last step re-reads itself (unused)
#pragma unroll
                for (int i = 0; i < MF; ++i) a2[h ^ 1][i].u = *(const u32x4*)(a_row[i] + kn);
#pragma unroll
                for (int j = 0; j < NF; ++j) b2[h ^ 1][j].u = *(const u32x4*)(b_row[j] + kn);
#pragma unroll
                for (int i = 0; i < MF; ++i)
#pragma unroll
                    for (int j = 0; j < NF; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a2[h][i].v, b2[h][j].v, acc[i][j], 0, 0, 0);
            }
        }
    }
    if (partial) {
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            int row = t0 + j * 16 + l16;                      // token
            if (row >= n) continue;
#pragma unroll
            for (int i = 0; i < MF; ++i) {
                int col = f0 + i * 16 + lq * 4;               // feature
                if (col < m) *(f32x4*)(partial + (size_t)row * m + col) = acc[i][j];
            }
        }
        return;
    }
    constexpr int CP = BMT * 2 + 16;                          // bytes per staged token row: 16 rows x 4 lanes x 8 B
                                                              // of one store fall on 64 different banks
    constexpr int LPR = BMT / 4;                              // 8-byte pieces per row
    __syncthreads();                                          // every wavefront is done with the rings / the staged factor
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            f32x4 v = acc[i][j];
            union { __bf16 h[4]; u32x2 u; } o;
            o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
            *(u32x2*)(smem + (t0 - tile_t0 + j * 16 + l16) * CP + (f0 - tile_f0 + i * 16 + lq * 4) * 2) = o.u;
        }
    __syncthreads();
    // 16-byte pieces, all read from LDS before the first is stored (a loop of read, wait, store per piece took
    // 2.5 us of every tile); m is a multiple of 8, so a piece is inside the row or outside as a whole
    constexpr int PPR = BMT / 8, PER_THREAD = BNT * PPR / THREADS;   // THREADS = the workgroup's size
    static_assert(BNT * PPR % THREADS == 0 && LPR == 2 * PPR, "whole pieces per thread");
    u32x4 piece[PER_THREAD];
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const int idx = (int)threadIdx.x + u * THREADS;
        piece[u] = *(const u32x4*)(smem + (idx / PPR) * CP + (idx % PPR) * 16);
    }
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const int idx = (int)threadIdx.x + u * THREADS;
        const int tok = tile_t0 + idx / PPR, col = tile_f0 + (idx % PPR) * 8;
        if (tok < n && col < m) *(u32x4*)(C + (size_t)tok * m + col) = piece[u];
    }
}

template <int BM, int BN>
struct SpmmSmem {
    static constexpr int A_PAIR = BM * 128;     // packed values of BM rows x 2 k-steps
    static constexpr int B_STAGE = BN * 128;    // BN token rows x 1 k-step
    static constexpr int M_QUAD = BM * 32;      // metadata of BM rows x 4 k-steps
    static constexpr int B_OFF = 2 * A_PAIR;
    static constexpr int M_OFF = B_OFF + 3 * B_STAGE;
    static constexpr int DUMMY = M_OFF + 2 * M_QUAD;   // landing zone for the metadata load of idle wavefronts
    static constexpr int TOTAL = DUMMY + 1024;
};

constexpr int SPMM_THREADS = 512;

template <int BM, int BN>
__global__ void __launch_bounds__(SPMM_THREADS) spmm_kernel(const bf16_t* __restrict__ B, int n,
                                                            const bf16_t* __restrict__ Av,
                                                            const uint8_t* __restrict__ Am, int m, int K,
                                                            const bf16_t* __restrict__ B2,
                                                            const bf16_t* __restrict__ A2, int K2,
                                                            bf16_t* __restrict__ C, int tiles_m, int tiles_n,
                                                            int slab_steps, float* __restrict__ slabs) {
    using S = SpmmSmem<BM, BN>;
    constexpr int MF = BM / 32, NF = BN / 64;                // 16 x 16 fragments per wavefront
    constexpr int A_LD = BM / 64, B_LD = BN / 64;            // 1 KiB loads per wavefront: per pair, per step
    constexpr int M_WAVES = BM / 32;                         // wavefronts that load metadata (32 rows each)
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    if (!tile_of_block(tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;                             // the two wavefronts of a SIMD differ here
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- loader lanes: 8 lanes per row, chunk rotated by (row / 2) % 8
    const uint8_t* a_src[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int rl = (wave * A_LD + i) * 8 + (lane >> 3);         // row inside the tile
        int row = wrap_row(m0 + rl, m);
        a_src[i] = (const uint8_t*)Av + (size_t)row * K + (((lane & 7) ^ ((rl >> 1) & 7)) * 16);
    }
    const uint8_t* b_src[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int rl = (wave * B_LD + i) * 8 + (lane >> 3);
        int row = wrap_row(n0 + rl, n);
        b_src[i] = (const uint8_t*)B + (size_t)row * K * 2 + (((lane & 7) ^ ((rl >> 1) & 7)) * 16);
    }
    const bool meta_wave = wave < M_WAVES;                    // wave-uniform
    const uint8_t* m_src;
    {
        // 32 rows = two fragments per instruction; lane l brings the 16-byte half (l >> 4) & 1 of row
        // 16 (l >> 5) + (l & 15), so that LDS holds each fragment as [half][row]: the sixteen rows of a
        // 2-byte metadata read then fall on sixteen different bank groups ([row][half] made rows r and r + 8
        // collide: over a third of the LDS-active cycles of the 256 x 256 kernel were bank conflicts)
        int rl = (meta_wave ? wave : 0) * 32 + (lane >> 5) * 16 + (lane & 15);
        int row = wrap_row(m0 + rl, m);
        m_src = Am + (size_t)row * (K / 8) + ((lane >> 4) & 1) * 16;
    }
    uint8_t* const m_dst0 = smem + (meta_wave ? S::M_OFF + wave * 1024 : S::DUMMY);
    const int m_dst_step = meta_wave ? S::M_QUAD : 0;

    // ---- reader lanes: fragment f = rows 16f .. 16f+15 = 2 KiB; lane (l16, lq) wants chunk 4h + lq
    const int sw = (l16 >> 1) & 7;
    const int rd0 = l16 * 128 + ((lq ^ sw) * 16);             // h = 0
    const int rd1 = l16 * 128 + (((4 + lq) ^ sw) * 16);       // h = 1
    const int a_rd = (wm * MF) * 2048;
    const int b_rd = S::B_OFF + (wn * NF) * 2048;
    const int m_rd = S::M_OFF + wm * MF * 512 + l16 * 16 + lq * 2;

    // A split over k: workgroup row blockIdx.y takes k-steps [k_first, k_first + ksteps) and leaves
    // fp32 partial sums in its slab; without a slab buffer there is one row and it takes all of K.
    const int k_first = blockIdx.y * slab_steps;              // a multiple of 4
    const int ksteps = K / 64 - k_first < slab_steps ? K / 64 - k_first : slab_steps;   // a multiple of 4
#pragma unroll
    for (int i = 0; i < A_LD; ++i) a_src[i] += (size_t)k_first * 64;
#pragma unroll
    for (int i = 0; i < B_LD; ++i) b_src[i] += (size_t)k_first * 128;
    m_src += (size_t)k_first * 8;
    auto issue_b = [&](int ks, int stage) {                   // token rows of k-step ks (clamped)
        int kc = ks < ksteps ? ks : ksteps - 1;
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            dma16(b_src[i] + (size_t)kc * 128, smem + S::B_OFF + stage * S::B_STAGE + (wave * B_LD + i) * 1024);
    };
    auto issue_a = [&](int pair, int buf) {                   // weight rows of k-steps 2 pair, 2 pair + 1
        int pc = 2 * pair < ksteps ? pair : ksteps / 2 - 1;
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            dma16(a_src[i] + (size_t)pc * 128, smem + buf * S::A_PAIR + (wave * A_LD + i) * 1024);
    };
    auto issue_m = [&](int quad, int buf) {                   // metadata of k-steps 4 quad .. 4 quad + 3
        int qc = 4 * quad < ksteps ? quad : ksteps / 4 - 1;
        dma16(m_src + (size_t)qc * 32, m_dst0 + buf * m_dst_step);
    };

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // ---- prologue: k-steps 0 and 1 in flight; the second group starts half a step late
    issue_m(0, 0);
    issue_a(0, 0);
    issue_b(0, 0);
    issue_b(1, 1);
    WAIT_HERE(waitcnt_imm(B_LD, 15));        // everything but B of step 1 has landed
    wg_barrier();

    // One k-step of one wavefront; S4 = ks % 4 is a literal so that the number of loads queued in
    // this step, which the wait below has to leave outstanding, is a constant.  The wait for the
    // wavefront's own share of step ks + 1 sits at the end of the compute phase for group 0 and at
    // the end of the memory phase for group 1: either way it precedes the barrier after which
    // group 0 starts reading that step.
#define SPMM_STEP(G, S4)                                                                               \
    {                                                                                                  \
        const int ks = ks0 + S4;                                                                       \
        constexpr int QUEUED = B_LD + ((S4 & 1) == 0 ? A_LD : 0) + (S4 == 0 ? 1 : 0);                  \
        const uint8_t* pa = smem + ((S4 >> 1) & 1) * S::A_PAIR + a_rd + ((S4 & 1) ? rd1 : rd0);        \
        const uint8_t* pb = smem + b_rd + bst * S::B_STAGE;                                            \
        const uint8_t* pm = smem + m_rd + ((ks0 >> 2) & 1) * S::M_QUAD + (S4 >> 1) * 256 + (S4 & 1) * 8; \
        BFrag bf[NF];                                                                                  \
        AFrag af[MF];                                                                                  \
        int ai[MF];                                                                                    \
        issue_b(ks + 2, bst >= 1 ? bst - 1 : 2);                                                       \
        if ((S4 & 1) == 0) issue_a((ks >> 1) + 1, ((S4 >> 1) + 1) & 1);                                \
        if (S4 == 0) issue_m((ks >> 2) + 1, ((ks0 >> 2) + 1) & 1);                                     \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(pb + j * 2048 + rd0);                                         \
            bf[j].u[1] = *(const u32x4*)(pb + j * 2048 + rd1);                                         \
        }                                                                                              \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u = *(const u32x4*)(pa + i * 2048);                                                  \
            ai[i] = *(const uint16_t*)(pm + i * 512);                                                  \
        }                                                                                              \
        bst = bst == 2 ? 0 : bst + 1;                                                                  \
        /* all LDS reads of this stage have returned before anybody may overwrite it */                \
        WAIT_HERE(waitcnt_imm(G == 1 ? QUEUED : 63, 0));                              \
        wg_barrier();                                                                                  \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) _Pragma("unroll") for (int j = 0; j < NF; ++j)  \
            acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(af[i].v, bf[j].v, acc[i][j], ai[i], 0, 0); \
        if (G == 0) WAIT_HERE(waitcnt_imm(QUEUED, 15));                               \
        wg_barrier();                                                                                  \
    }
    int bst = 0;                                              // ring stage of the current k-step
    if (group == 0) {
        for (int ks0 = 0; ks0 < ksteps; ks0 += 4) { SPMM_STEP(0, 0) SPMM_STEP(0, 1) SPMM_STEP(0, 2) SPMM_STEP(0, 3) }
        wg_barrier();
    } else {
        wg_barrier();
        for (int ks0 = 0; ks0 < ksteps; ks0 += 4) { SPMM_STEP(1, 0) SPMM_STEP(1, 1) SPMM_STEP(1, 2) SPMM_STEP(1, 3) }
    }
#undef SPMM_STEP
    WAIT_HERE(waitcnt_imm(0, 15));           // drain the clamped look-ahead loads

    // the dense extension is added once, by the first slab
    static_assert(BN * (BM * 2 + 16) <= S::TOTAL, "the staged output tile fits in the rings");
    extend_and_store<MF, NF, BM, BN, SPMM_THREADS>(acc, m0 + wm * MF * 16, n0 + wn * NF * 16, m, n, l16, lq, B2, A2,
                                     blockIdx.y == 0 ? K2 : 0, C, smem, m0, n0,
                                     slabs ? slabs + (size_t)blockIdx.y * (size_t)n * (size_t)m : nullptr);
}

// ------------------------------------------------------------------------------------------
// spmm_split_kernel: the 256 x 256 tile.  A fifth fewer operand bytes per flop than the
// 192 x 256 tile, but a ring of three B stages no longer fits beside it.  The two wavefront groups
// own the two token halves of the tile, so each half of a B stage is private to one group and free
// again as soon as that group has read it; two stages per half then give every load the same two
// to three phases (half k-steps) of flight that the shared ring of three gave:
//     A pair buffers 2 x 32 KiB | B half of group 0  2 x 16 KiB | of group 1  2 x 16 KiB | metadata 2 x 8 KiB
// Queued by every wavefront, k = k-step, phases 2k (group 0 reads step k) and 2k + 1 (group 1 does):
//     phase 2k     : B1(k+1);  lower half of A pair k/2 + 1 if k is even;  metadata quad (k+3)/4 if k % 4 == 1
//     phase 2k + 1 : B0(k+2);  upper half of A pair k/2 + 1 if k is even
// and at the end of each phase a wavefront waits for everything it queued two or more phases ago,
// which covers all that the next phase reads.  Every buffer is rewritten in the first phase after
// the barrier that ends its last reader's phase.
struct SplitSmem {
    static constexpr int BM = 256, BN = 256;
    static constexpr int A_PAIR = BM * 128, B_HALF = BN / 2 * 128, M_QUAD = BM * 32;
    static constexpr int B_OFF = 2 * A_PAIR;                  // then [group][stage] halves of B
    static constexpr int M_OFF = B_OFF + 4 * B_HALF;
    static constexpr int TOTAL = M_OFF + 2 * M_QUAD;
};

// loads one wavefront queues in the even / odd phase of k-step k (k taken mod 4)
constexpr int split_even(int k) { return 2 + ((k & 1) == 0 ? 2 : 0) + ((k & 3) == 1 ? 1 : 0); }
constexpr int split_odd(int k) { return 2 + ((k & 1) == 0 ? 2 : 0); }

template <bool PREFETCH>
__global__ void __launch_bounds__(SPMM_THREADS) spmm_split_kernel(const bf16_t* __restrict__ B, int n,
                                                                  const bf16_t* __restrict__ Av,
                                                                  const uint8_t* __restrict__ Am, int m, int K,
                                                                  const bf16_t* __restrict__ B2,
                                                                  const bf16_t* __restrict__ A2, int K2,
                                                                  bf16_t* __restrict__ C, int tiles_m, int tiles_n) {
    using S = SplitSmem;
    constexpr int MF = 8, NF = 4;                            // wavefront tile 128 features x 64 tokens
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    if (!tile_of_block(tiles_m, tiles_n, tm, tn)) return;
    const int m0 = tm * S::BM, n0 = tn * S::BN;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int group = wave >> 2;                             // = token half of the tile
    const int wm = wave & 1, wn = wave >> 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- loader lanes: 8 lanes per row, chunk rotated by (row / 2) % 8.  A half of A and a half of
    //      B are 16 loads of 8 rows each: two per wavefront.
    const uint8_t* a_src[4];                                 // [half * 2 + i]
    const uint8_t* b_src[4];                                 // [group * 2 + i]
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int rl = ((q >> 1) * 16 + wave * 2 + (q & 1)) * 8 + (lane >> 3);     // row inside the tile
        int sw16 = ((lane & 7) ^ ((rl >> 1) & 7)) * 16;
        int ra = wrap_row(m0 + rl, m);
        int rb = wrap_row(n0 + rl, n);
        a_src[q] = (const uint8_t*)Av + (size_t)ra * K + sw16;
        b_src[q] = (const uint8_t*)B + (size_t)rb * K * 2 + sw16;
    }
    const uint8_t* m_src;                                    // 32 rows per wavefront
    {
        int rl = wave * 32 + (lane >> 5) * 16 + (lane & 15);  // fragments land as [half][row], see spmm_kernel
        int row = wrap_row(m0 + rl, m);
        m_src = Am + (size_t)row * (K / 8) + ((lane >> 4) & 1) * 16;
    }

    // ---- L2 prefetch of the token panel through the scalar cache.  A compute unit holds about 128 vector-memory
    //      requests of 128 bytes in flight, so its operand feed is that many lines per mean latency, and the
    //      latency is set by the lines that miss the XCD's L2 (a sixth of them, compulsory: each operand panel
    //      enters the L2 once per chunk of 8 x 4 tiles), on which all tiles that share the panel wait together.
    //      Scalar loads take another path into the same L2.  The 8 tiles of a chunk that share a token panel
    //      each touch an eighth of its rows PF_AHEAD k-steps ahead (4 rows per wavefront, both 64-byte halves of
    //      a row's 128 bytes: the L2 fills halves), so the vector loads of the token panel hit: 3-6 % on the
    //      whole product at OPT-66B sizes.  The scalar path takes about 70 such requests per microsecond and compute unit, which
    //      these 64 per k-step use up; touching only part of the panel, or the weight panels instead, gained
    //      nothing.  The loaded dwords are not used; they stay allocated until the wavefront's next
    //      s_waitcnt lgkmcnt(0), since a scalar load may return any time before that.
    constexpr int PF_AHEAD = 6, PF_ROWS = S::BN / CHUNK_M / 8;
    const uint8_t* pf_row[PF_ROWS];
#pragma unroll
    for (int r = 0; r < PF_ROWS; ++r) {
        int row = wrap_row(n0 + (tm % CHUNK_M) * (S::BN / CHUNK_M) + wave * PF_ROWS + r, n);
        pf_row[r] = (const uint8_t*)B + (size_t)row * K * 2;
    }
    // PREFETCH is the host's choice (launch_split): only for grids in the chunked order, and only if the tokens do
    // not fit into the last-level cache: lines that come from there rather than from HBM arrive soon enough anyway,
    // and the scalar loads then cost more than they gain (measured: 1-5 % faster with 16384 tokens of 9216 features
    // or more, 3-12 % slower with 8192 tokens or fewer).  It is a template parameter because a branch around the
    // loads inside the k-loop cost what they gain.  Tiles outside whole chunks touch rows as if they were in one:
    // harmless, and they are few.
    uint32_t pf[2 * PF_ROWS];
#pragma unroll
    for (int r = 0; r < 2 * PF_ROWS; ++r) pf[r] = 0;
    // to be placed right after an s_waitcnt lgkmcnt(0): retires the previous k-step's loads, issues the next
#define PF_ISSUE(ks)                                                                                   \
    {                                                                                                  \
        _Pragma("unroll") for (int r = 0; r < 2 * PF_ROWS; ++r) asm volatile("" ::"s"(pf[r]));         \
        const int kpf = (ks) + PF_AHEAD < ksteps ? (ks) + PF_AHEAD : ksteps - 1;                       \
        const uint32_t off = (uint32_t)kpf * 128u;            /* inside the row: K * 2 bytes, K < 2^31 */ \
        if (PREFETCH) {                                                                                \
            _Pragma("unroll") for (int r = 0; r < PF_ROWS; ++r) {                                      \
                asm volatile("s_load_dword %0, %1, %2" : "=s"(pf[2 * r]) : "s"(pf_row[r]), "s"(off));   \
                asm volatile("s_load_dword %0, %1, %2" : "=s"(pf[2 * r + 1]) : "s"(pf_row[r]), "s"(off + 64u)); \
            }                                                                                          \
        }                                                                                              \
    }
    // ---- reader lanes: fragment f = rows 16f .. 16f+15 = 2 KiB; lane (l16, lq) wants chunk 4h + lq
    const int sw = (l16 >> 1) & 7;
    const int rd0 = l16 * 128 + ((lq ^ sw) * 16);             // h = 0
    const int rd1 = l16 * 128 + (((4 + lq) ^ sw) * 16);       // h = 1
    const int a_rd = (wm * MF) * 2048;
    const int b_rd = S::B_OFF + group * 2 * S::B_HALF + ((wn & 1) * NF) * 2048;
    const int m_rd = S::M_OFF + wm * MF * 512 + l16 * 16 + lq * 2;

    const int ksteps = K / 64;                                // a multiple of 4
    auto issue_b = [&](int g, int ks) {                       // token half g of k-step ks (clamped)
        int kc = ks < ksteps ? ks : ksteps - 1;
        uint8_t* st = smem + S::B_OFF + (g * 2 + (ks & 1)) * S::B_HALF + (wave * 2) * 1024;
        dma16(b_src[g * 2] + (size_t)kc * 128, st);
        dma16(b_src[g * 2 + 1] + (size_t)kc * 128, st + 1024);
    };
    auto issue_a = [&](int half, int pair) {                  // weight rows 128 half .. +127, k-steps 2 pair, 2 pair + 1
        int pc = 2 * pair < ksteps ? pair : ksteps / 2 - 1;
        uint8_t* st = smem + (pair & 1) * S::A_PAIR + (half * 16 + wave * 2) * 1024;
        dma16(a_src[half * 2] + (size_t)pc * 128, st);
        dma16(a_src[half * 2 + 1] + (size_t)pc * 128, st + 1024);
    };
    auto issue_m = [&](int quad) {                            // metadata of k-steps 4 quad .. 4 quad + 3
        int qc = 4 * quad < ksteps ? quad : ksteps / 4 - 1;
        dma16(m_src + (size_t)qc * 32, smem + S::M_OFF + (quad & 1) * S::M_QUAD + wave * 1024);
    };

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // S4 = k % 4 is a literal, so the number of loads a wait may leave in flight is a constant.
#define EVEN_LOADS(k, S4)                                                                              \
    {                                                                                                  \
        issue_b(1, (k) + 1);                                                                           \
        if (((S4) & 1) == 0) issue_a(0, ((k) >> 1) + 1);                                               \
        if (((S4) & 3) == 1) issue_m(((k) + 3) >> 2);                                                  \
    }
#define ODD_LOADS(k, S4)                                                                               \
    {                                                                                                  \
        issue_b(0, (k) + 2);                                                                           \
        if (((S4) & 1) == 0) issue_a(1, ((k) >> 1) + 1);                                               \
    }
#define SPLIT_READ(S4)                                                                                 \
        const uint8_t* pa = smem + (((S4) >> 1) & 1) * S::A_PAIR + a_rd + (((S4) & 1) ? rd1 : rd0);    \
        const uint8_t* pb = smem + b_rd + ((S4) & 1) * S::B_HALF;                                      \
        const uint8_t* pm = smem + m_rd + ((ks0 >> 2) & 1) * S::M_QUAD + ((S4) >> 1) * 256 + ((S4) & 1) * 8; \
        BFrag bf[NF];                                                                                  \
        AFrag af[MF];                                                                                  \
        int ai[MF];                                                                                    \
        _Pragma("unroll") for (int j = 0; j < NF; ++j) {                                               \
            bf[j].u[0] = *(const u32x4*)(pb + j * 2048 + rd0);                                         \
            bf[j].u[1] = *(const u32x4*)(pb + j * 2048 + rd1);                                         \
        }                                                                                              \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) {                                               \
            af[i].u = *(const u32x4*)(pa + i * 2048);                                                  \
            ai[i] = *(const uint16_t*)(pm + i * 512);                                                  \
        }
#define SPLIT_MFMA                                                                                     \
        _Pragma("unroll") for (int i = 0; i < MF; ++i) _Pragma("unroll") for (int j = 0; j < NF; ++j)  \
            acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(af[i].v, bf[j].v, acc[i][j], ai[i], 0, 0);
    // group 0: phase 2k reads step k, phase 2k + 1 multiplies it
#define SPLIT_STEP0(S4)                                                                                \
    {                                                                                                  \
        const int ks = ks0 + (S4);                                                                     \
        SPLIT_READ(S4)                                                                                 \
        EVEN_LOADS(ks, S4)                                                                             \
        WAIT_HERE(waitcnt_imm(split_even(S4) + split_odd((S4) + 3), 0));                               \
        PF_ISSUE(ks)                                                                                   \
        wg_barrier();                                                                                  \
        ODD_LOADS(ks, S4)                                                                              \
        SPLIT_MFMA                                                                                     \
        WAIT_HERE(waitcnt_imm(split_odd(S4) + split_even(S4), 15));                                    \
        wg_barrier();                                                                                  \
    }
    // group 1: phase 2k + 1 reads step k, phase 2k + 2 multiplies it
#define SPLIT_STEP1(S4)                                                                                \
    {                                                                                                  \
        const int ks = ks0 + (S4);                                                                     \
        SPLIT_READ(S4)                                                                                 \
        ODD_LOADS(ks, S4)                                                                              \
        WAIT_HERE(waitcnt_imm(split_odd(S4) + split_even(S4), 0));                                     \
        PF_ISSUE(ks)                                                                                   \
        wg_barrier();                                                                                  \
        EVEN_LOADS(ks + 1, (S4) + 1)                                                                   \
        SPLIT_MFMA                                                                                     \
        WAIT_HERE(waitcnt_imm(split_even((S4) + 1) + split_odd(S4), 15));                              \
        wg_barrier();                                                                                  \
    }

    // ---- prologue: what the schedule would have queued in the phases before phase 0
    issue_m(0);
    issue_a(0, 0); issue_a(1, 0); issue_b(0, 0);
    issue_b(1, 0);
    issue_b(0, 1);                                            // = the odd phase of step -1
    WAIT_HERE(waitcnt_imm(4, 15));                            // metadata, A pair 0 and B0(0) have landed
    wg_barrier();
    if (group == 0) {
        for (int ks0 = 0; ks0 < ksteps; ks0 += 4) { SPLIT_STEP0(0) SPLIT_STEP0(1) SPLIT_STEP0(2) SPLIT_STEP0(3) }
        wg_barrier();                                         // group 1's last compute phase
    } else {
        EVEN_LOADS(0, 0)                                      // phase 0: nothing to multiply yet
        WAIT_HERE(waitcnt_imm(split_even(0) + split_odd(3), 15));
        wg_barrier();
        for (int ks0 = 0; ks0 < ksteps; ks0 += 4) { SPLIT_STEP1(0) SPLIT_STEP1(1) SPLIT_STEP1(2) SPLIT_STEP1(3) }
    }
#undef EVEN_LOADS
#undef ODD_LOADS
#undef SPLIT_READ
#undef SPLIT_MFMA
#undef SPLIT_STEP0
#undef SPLIT_STEP1
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");        // the last scalar prefetches have returned
#pragma unroll
    for (int r = 0; r < 2 * PF_ROWS; ++r) asm volatile("" ::"s"(pf[r]));
#undef PF_ISSUE
    WAIT_HERE(waitcnt_imm(0, 15));                            // drain the clamped look-ahead loads
    static_assert(S::BN * (S::BM * 2 + 16) <= S::TOTAL, "the staged output tile fits in the rings");
    extend_and_store<MF, NF, S::BM, S::BN, SPMM_THREADS>(acc, m0 + wm * MF * 16, n0 + wn * NF * 16, m, n, l16, lq, B2, A2, K2, C, smem,
                                           m0, n0);
}

// ------------------------------------------------------------------------------------------
// Generic kernel (any K % 8 == 0): 128 x 128 tile, 4 wavefronts (2 x 2), operands staged through
// registers into two LDS buffers in fragment order (the 16 bytes a lane feeds to the MFMA sit at
// 16 * lane inside a 1 KiB fragment), one barrier per k-step.
// RAGGED (K not a multiple of 64): the last k-step is partly past the end of the rows, and rows of
// the packed weight are only 8-byte, rows of the metadata only 1-byte aligned.  Loads then come in
// pieces of 8 logical k (8 bytes of packed values, 16 bytes of tokens, 1 byte of metadata), each
// either wholly inside the row or replaced: zeros for values and tokens, the nibble pair 0x44
// (positions 0, 1: a legal encoding) for metadata, so the tail contributes exact zeros.
struct GenSmem {
    static constexpr int A_BYTES = 128 * 64, B_BYTES = 128 * 128, M_BYTES = 128 * 8;
    static constexpr int STAGE = A_BYTES + B_BYTES + M_BYTES;
};

template <bool RAGGED>
__global__ void __launch_bounds__(256) spmm_generic_kernel(const bf16_t* __restrict__ B, int n,
                                                           const bf16_t* __restrict__ Av,
                                                           const uint8_t* __restrict__ Am, int m, int K,
                                                           const bf16_t* __restrict__ B2,
                                                           const bf16_t* __restrict__ A2, int K2,
                                                           bf16_t* __restrict__ C, int tiles_m) {
    using S = GenSmem;
    constexpr int MF = 4, NF = 4, A_LD = 2, B_LD = 4;
    __shared__ __align__(16) uint8_t smem[2 * S::STAGE];
    const int m0 = (blockIdx.x % tiles_m) * 128, n0 = (blockIdx.x / tiles_m) * 128;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;
    const size_t a_pitch = (size_t)K / 2, m_pitch = (size_t)K / 8, b_pitch = (size_t)K;
    const bf16_t* a_src[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int row = m0 + (wave * A_LD + i) * 16 + l16;
        row = wrap_row(row, m);
        a_src[i] = Av + (size_t)row * a_pitch + lq * 8;
    }
    const bf16_t* b_src[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        int slot = wave * B_LD + i;
        int row = n0 + (slot >> 1) * 16 + l16;
        row = wrap_row(row, n);
        b_src[i] = B + (size_t)row * b_pitch + (slot & 1) * 32 + lq * 8;
    }
    const uint8_t* m_src;
    {
        int row = m0 + (t & 127);
        row = wrap_row(row, m);
        m_src = Am + (size_t)row * m_pitch;
    }
    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int ksteps = (K + 63) / 64;
    u32x4 a_reg[A_LD], b_reg[B_LD];
    u32x2 m_reg;
    // first logical k of the lane's 16 of the sparse operand, and of its two token pieces, in k-step 0
    const int a_k = lq * 16;
    int b_k[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) b_k[i] = ((wave * B_LD + i) & 1) * 32 + lq * 8;
    auto load_ragged = [&](int kk) {
        const int k0 = kk * 64;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            u32x2 lo = {0u, 0u}, hi = {0u, 0u};
            if (k0 + a_k < K) lo = *(const u32x2*)(a_src[i] + kk * 32);
            if (k0 + a_k + 8 < K) hi = *(const u32x2*)(a_src[i] + kk * 32 + 4);
            a_reg[i] = (u32x4){lo[0], lo[1], hi[0], hi[1]};
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            b_reg[i] = (u32x4){0u, 0u, 0u, 0u};
            if (k0 + b_k[i] < K) b_reg[i] = *(const u32x4*)(b_src[i] + kk * 64);
        }
        uint32_t w[2] = {0x44444444u, 0x44444444u};
        const int have = K / 8 - kk * 8;                      // metadata bytes of this k-step inside the row
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < have) w[e >> 2] = (w[e >> 2] & ~(0xFFu << (8 * (e & 3)))) | ((uint32_t)m_src[kk * 8 + e] << (8 * (e & 3)));
        m_reg = (u32x2){w[0], w[1]};
    };
#define GEN_LOAD(kk)                                                                                   \
    if (RAGGED) {                                                                                      \
        load_ragged(kk);                                                                               \
    } else {                                                                                           \
        _Pragma("unroll") for (int i = 0; i < A_LD; ++i) a_reg[i] = *(const u32x4*)(a_src[i] + (kk) * 32); \
        _Pragma("unroll") for (int i = 0; i < B_LD; ++i) b_reg[i] = *(const u32x4*)(b_src[i] + (kk) * 64); \
        m_reg = *(const u32x2*)(m_src + (kk) * 8);                                                     \
    }
#define GEN_STORE(stage)                                                                               \
    {                                                                                                  \
        uint8_t* base = smem + (stage) * S::STAGE;                                                     \
        _Pragma("unroll") for (int i = 0; i < A_LD; ++i) *(u32x4*)(base + (wave * A_LD + i) * 1024 + lane * 16) = a_reg[i]; \
        _Pragma("unroll") for (int i = 0; i < B_LD; ++i)                                               \
            *(u32x4*)(base + S::A_BYTES + (wave * B_LD + i) * 1024 + lane * 16) = b_reg[i];            \
        if (t < 128) *(u32x2*)(base + S::A_BYTES + S::B_BYTES + t * 8) = m_reg;                        \
    }
    GEN_LOAD(0)
    GEN_STORE(0)
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int stage = ks & 1;
        GEN_LOAD(ks + 1 < ksteps ? ks + 1 : ks)               // the last step re-reads its own slab (unused)
        const uint8_t* base = smem + stage * S::STAGE;
        const uint8_t* sa = base + (wm * MF) * 1024 + lane * 16;
        const uint8_t* sb = base + S::A_BYTES + (wn * NF) * 2048 + lane * 16;
        const uint8_t* sm = base + S::A_BYTES + S::B_BYTES + (wm * MF * 16 + l16) * 8 + lq * 2;
        BFrag bf[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            bf[j].u[0] = *(const u32x4*)(sb + j * 2048);
            bf[j].u[1] = *(const u32x4*)(sb + j * 2048 + 1024);
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            AFrag a;
            a.u = *(const u32x4*)(sa + i * 1024);
            int idx = *(const uint16_t*)(sm + i * 128);
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, bf[j].v, acc[i][j], idx, 0, 0);
        }
        GEN_STORE(stage ^ 1)
        __syncthreads();
    }
#undef GEN_LOAD
#undef GEN_STORE
    static_assert(128 * (128 * 2 + 16) <= 2 * S::STAGE, "the staged output tile fits in the stages");
    extend_and_store<MF, NF, 128, 128, 256>(acc, m0 + wm * MF * 16, n0 + wn * NF * 16, m, n, l16, lq, B2, A2, K2, C, smem, m0,
                                       n0);
}

template <int BM, int BN>
hipError_t launch_tile(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s, int nslabs = 1,
                       int slab_steps = 0, float* slabs = nullptr) {
    using S = SpmmSmem<BM, BN>;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    int tiles_m = (int)((m + BM - 1) / BM), tiles_n = (int)((n + BN - 1) / BN);
    auto kern = spmm_kernel<BM, BN>;
    hipError_t e = allow_dynamic_lds<spmm_kernel<BM, BN>>(S::TOTAL);
    if (e != hipSuccess) return e;
    if (!slabs) { nslabs = 1; slab_steps = (int)(K / 64); }
    kern<<<dim3((unsigned)super_grid(tiles_m, tiles_n), (unsigned)nslabs), dim3(SPMM_THREADS), S::TOTAL, s>>>(
        B, (int)n, Av, Am, (int)m, (int)K, B2, A2, (int)K2, C, tiles_m, tiles_n, slab_steps, slabs);
    return hipGetLastError();
}

// C[idx] = bf16( sum over slabs, in order, of P[s][idx] ), four elements per thread
__global__ void __launch_bounds__(256) slab_reduce_kernel(const f32x4* __restrict__ P, int nslabs, size_t count4,
                                                          u32x2* __restrict__ C) {
    size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count4) return;
    f32x4 v = P[idx];
    for (int sl = 1; sl < nslabs; ++sl) {
        f32x4 w = P[(size_t)sl * count4 + idx];
        v[0] += w[0]; v[1] += w[1]; v[2] += w[2]; v[3] += w[3];
    }
    union { __bf16 h[4]; u32x2 u; } o;
    o.h[0] = (__bf16)v[0]; o.h[1] = (__bf16)v[1]; o.h[2] = (__bf16)v[2]; o.h[3] = (__bf16)v[3];
    C[idx] = o.u;
}

hipError_t launch_split(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                        const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    using S = SplitSmem;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    int tiles_m = (int)((m + S::BM - 1) / S::BM), tiles_n = (int)((n + S::BN - 1) / S::BN);
    const bool prefetch = wide_grid(tiles_m, tiles_n) && (size_t)n * (size_t)K * 2 > LAST_LEVEL_CACHE_BYTES;
    hipError_t e = prefetch ? allow_dynamic_lds<spmm_split_kernel<true>>(S::TOTAL)
                            : allow_dynamic_lds<spmm_split_kernel<false>>(S::TOTAL);
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)super_grid(tiles_m, tiles_n));
    if (prefetch)
        spmm_split_kernel<true><<<grid, dim3(SPMM_THREADS), S::TOTAL, s>>>(B, (int)n, Av, Am, (int)m, (int)K, B2, A2,
                                                                           (int)K2, C, tiles_m, tiles_n);
    else
        spmm_split_kernel<false><<<grid, dim3(SPMM_THREADS), S::TOTAL, s>>>(B, (int)n, Av, Am, (int)m, (int)K, B2, A2,
                                                                            (int)K2, C, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

// A few dozen to a thousand tokens: the token tile is so narrow that small weight tiles would
// re-read it from L2 for every few weight rows (the tile kernels run at the L2 -> LDS rate), and
// tall weight tiles alone are too few to fill the chip.  So: 256-row weight tiles, the k range
// cut into slabs that run as separate workgroups and leave fp32 partial sums in `slabs`, and a
// short reduction kernel (fixed order: bit-identical runs) that rounds to bf16.
constexpr int64_t SLAB_MAX_TOKENS = 1024;

int spmm_slab_count(int64_t n, int64_t m, int64_t K) {
    if (n <= STREAM_MAX_TOKENS || n > SLAB_MAX_TOKENS || K % 256 != 0) return 0;
    const int64_t tiles = ((m + 255) / 256) * ((n + 127) / 128);
    if (tiles >= RESIDENT) return 0;                          // the chip is full without a split (measured: slabs lose)
    const int64_t quads = K / 256;                            // slabs are whole quads of k-steps
    // Estimate per slab count: the rounds of 256 workgroups, each pulling its share of the packed
    // weight at what one compute unit sustains with this tile (about 24 B/ns of weight bytes), plus
    // writing and re-reading the partial sums at HBM speed.  One slab means: not worth it.
    const double weight = 1.125 * (double)m * (double)K, cu = 24.0, hbm = 5.0e3;   // bytes, bytes per ns
    int best = 1;
    double best_ns = 1e300;
    // (a round is counted full at 7/8 of the compute units: on a 9216 x 36864 layer at 128 tokens 7 slabs, 252
    // workgroups, took 180 us where 6 slabs, 216 workgroups, take 138 us, and 8, 9 and 12 slabs 172, 170 and 149 us;
    // the cut tail of the weight gradient shows no such step between 224 and 256 workgroups)
    const int64_t fit = RESIDENT - RESIDENT / 8;
    for (int sl = 1; sl <= 16 && sl * 4 <= quads; ++sl) {
        const double rounds = (double)((tiles * sl + fit - 1) / fit);
        const double ns = rounds * weight / (double)(tiles * sl) / cu
                          + (sl > 1 ? 2.0 * sl * (double)n * (double)m * 4.0 / hbm : 0.0);
        if (ns < best_ns) { best_ns = ns; best = sl; }
    }
    return best < 2 ? 0 : best;
}

size_t spmm_slab_bytes(int64_t n, int64_t m, int64_t K) {
    return (size_t)spmm_slab_count(n, m, K) * (size_t)n * (size_t)m * 4;
}

hipError_t launch_spmm_slabs(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                             int64_t K, const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, float* slabs,
                             hipStream_t s) {
    const int want = spmm_slab_count(n, m, K);
    const int64_t quads = K / 256;
    const int slab_steps = (int)((quads + want - 1) / want) * 4;
    const int nslabs = (int)((K / 64 + slab_steps - 1) / slab_steps);       // <= want
    hipError_t e = n <= 64 ? launch_tile<256, 64>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s, nslabs, slab_steps, slabs)
                           : launch_tile<256, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s, nslabs, slab_steps, slabs);
    if (e != hipSuccess) return e;
    const size_t count4 = (size_t)n * (size_t)m / 4;
    slab_reduce_kernel<<<dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s>>>((const f32x4*)slabs, nslabs, count4,
                                                                                   (u32x2*)C);
    return hipGetLastError();
}

// Tile of the product for n tokens, m sparse rows, contraction K: bm = bn = 0 means the generic kernel.
void spmm_tile_choice(int64_t n, int64_t m, int64_t K, int& bm, int& bn) {
    bm = bn = 0;
    if (K % 256 != 0) return;
    // Few tokens (inference): the product is a single pass over the packed weight, bound by HBM.
    // Narrow token tiles, and weight tiles small enough that every compute unit streams its share.
    if (n <= 128) {
        const bool many = (m + 127) / 128 >= 200;
        bm = many ? 128 : 64;
        bn = n <= 64 ? 64 : 128;
        return;
    }
    // The tile kernels run at the rate their compute units pull operands from L2, so a launch costs
    // about (rounds of 256 resident tiles) x (operand bytes per tile and k-step: 72 per weight row,
    // 128 per token row).  Take the tile shape for which that is least; ties go to the larger tile.
    const int bms[6] = {256, 192, 256, 128, 128, 64}, bns[6] = {256, 256, 128, 128, 64, 128};
    int64_t best_cost = INT64_MAX;
    for (int c = 0; c < 6; ++c) {
        int64_t tiles = ((m + bms[c] - 1) / bms[c]) * ((n + bns[c] - 1) / bns[c]);
        int64_t cost = ((tiles + RESIDENT - 1) / RESIDENT) * (72 * bms[c] + 128 * bns[c]);
        if (cost < best_cost) { best_cost = cost; bm = bms[c]; bn = bns[c]; }
    }
}

hipError_t launch_spmm(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m, int64_t K,
                       const bf16_t* B2, const bf16_t* A2, int64_t K2, bf16_t* C, hipStream_t s) {
    int bm, bn;
    spmm_tile_choice(n, m, K, bm, bn);
    if (bm == 0) {
        int tiles_m = (int)((m + 127) / 128), tiles_n = (int)((n + 127) / 128);
        if (K % 64 == 0)
            spmm_generic_kernel<false><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, s>>>(
                B, (int)n, A_vals, A_meta, (int)m, (int)K, B2, A2, (int)K2, C, tiles_m);
        else
            spmm_generic_kernel<true><<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, s>>>(
                B, (int)n, A_vals, A_meta, (int)m, (int)K, B2, A2, (int)K2, C, tiles_m);
        return hipGetLastError();
    }
    switch (bm * 1000 + bn) {
        case 256256: return launch_split(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        case 192256: return launch_tile<192, 256>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        case 256128: return launch_tile<256, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        case 128128: return launch_tile<128, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        case 128064: return launch_tile<128, 64>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        case 64064: return launch_tile<64, 64>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
        default: return launch_tile<64, 128>(B, n, A_vals, A_meta, m, K, B2, A2, K2, C, s);
    }
}
