// Small-batch form of the 2:4 sparse product (inference-size token counts, n <= 32):
//     C[n, m] = sum_k B[n, k] * A[m, k]   (+ T[n, K2] * R[K2, m] for the adapters of Eq. 11)
// With so few tokens the product is one pass over the packed weight (1.125 bytes per element) and
// HBM bounds it, so the kernel is built to keep reads in flight rather than to share operands:
//   - a workgroup owns 32 to 64 weight rows and all tokens; its wavefronts take the pairs of
//     k-steps in turn (wavefront w: pairs w, w + W, ...), each accumulating a partial tile;
//   - every operand goes through a ring in LDS that is private to the wavefront, fed by
//     global -> LDS loads of full 128-byte lines and read back with ds_read_b128 in MFMA order:
//     no barrier in the main loop, only the wavefront's own s_waitcnt;
//   - the partial tiles are summed in a fixed order through LDS (bit-identical runs); before that
//     the adapter term is added on dense MFMA from T = X L and the factor R as stored.
// T itself comes from a split over d_in (xl_mfma_kernel, fp32 partial sums in the workspace)
// followed by a fixed-order reduction that rounds to bf16 (xl_reduce_kernel).
// (A first version kept the operands in registers and moved them into MFMA order with ds_bpermute;
// the permutes capped a compute unit near 23 B/ns, against 44 B/ns with the LDS rings.)
#include "pipeline.h"

namespace {

constexpr int XL_CHUNK = 64;        // rows of L per chunk of the X L split

union StB { u32x4 u[2]; bf16x16 v; };
union StA { u32x4 u; bf16x8 v; };

// The ring is two pairs of k-steps deep.  One workgroup per compute unit is resident and about 140
// of them saturate HBM.  NF token fragments of 16: one (up to 16 tokens, 8 to 4 wavefronts) or
// two (up to 32 tokens, 4 wavefronts).  Ring stage of one wavefront:
//     A: MF fragments x (16 rows x 128 B: both steps of the pair) | B: 2 steps x NF x (16 tokens x 128 B)
//     | metadata: 16 MF rows x 16 B
template <int MF, int WAVES, int NF>
struct StreamLds {
    static constexpr int BM = 16 * MF;
    static constexpr int A_BYTES = MF * 2048, B_BYTES = 2 * NF * 2048, M_BYTES = MF * 256;
    static constexpr int STAGE = A_BYTES + B_BYTES + M_BYTES;
    static constexpr int OPS = 2 * MF + 4 * NF + 1;           // loads per wavefront and pair
    static constexpr int RING = WAVES * 2 * STAGE;
    static constexpr int PART_PITCH = 16 * NF + 1;
    static constexpr int TOTAL = RING + WAVES * BM * PART_PITCH * 4;
};

template <int MF, int WAVES, int NF>
__global__ void __launch_bounds__(WAVES * 64) spmm_stream_lds_kernel(const bf16_t* __restrict__ B, int n,
                                                                   const bf16_t* __restrict__ Av,
                                                                   const uint8_t* __restrict__ Am, int m, int K,
                                                                   const bf16_t* __restrict__ T,
                                                                   const bf16_t* __restrict__ R, int K2,
                                                                   bf16_t* __restrict__ C) {
    using S = StreamLds<MF, WAVES, NF>;
    extern __shared__ __align__(16) uint8_t smem[];
    float* part = (float*)(smem + S::RING);                   // [wave][row][PART_PITCH]

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int m0 = blockIdx.x * S::BM;
    const int ksteps = K / 64, kpairs = (ksteps + 1) / 2;
    const bool odd_tail = (ksteps & 1) != 0;                 // the last pair has one step only
    uint8_t* const ring = smem + wave * 2 * S::STAGE;

    // loader lanes: 8 lanes per row, the 16-byte chunks of a row rotated by (row / 2) % 8
    const int ld_row = lane >> 3, ld_slot = lane & 7;
    const uint8_t* a_src[MF][2];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int rl = 8 * h + ld_row;
            int row = m0 + 16 * i + rl;
            row = row < m ? row : m - 1;
            a_src[i][h] = (const uint8_t*)Av + (size_t)row * K + ((ld_slot ^ ((rl >> 1) & 7)) * 16);
        }
    const uint8_t* b_src[NF][2];
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int rl = 8 * h + ld_row;
            int tok = 16 * j + rl < n ? 16 * j + rl : n - 1;
            b_src[j][h] = (const uint8_t*)B + (size_t)tok * K * 2 + ((ld_slot ^ ((rl >> 1) & 7)) * 16);
        }
    const bool meta_lane = lane < 16 * MF;
    const uint8_t* m_src;
    {
        int row = m0 + (meta_lane ? lane : 0);
        row = row < m ? row : m - 1;
        m_src = Am + (size_t)row * (K / 8);
    }
    auto issue = [&](int stage, int p) {                      // pair p (valid) into ring stage `stage`
        // an odd number of steps: the last pair is read as steps (ksteps - 2, ksteps - 1) and only
        // its second half is used, so that no load runs past the row
        const size_t s0 = (odd_tail && p == kpairs - 1) ? (size_t)ksteps - 2 : (size_t)2 * p;
        uint8_t* st = ring + stage * S::STAGE;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            dma16(a_src[i][0] + s0 * 64, st + i * 2048);
            dma16(a_src[i][1] + s0 * 64, st + i * 2048 + 1024);
        }
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                dma16(b_src[j][0] + (s0 + e) * 128, st + S::A_BYTES + (e * NF + j) * 2048);
                dma16(b_src[j][1] + (s0 + e) * 128, st + S::A_BYTES + (e * NF + j) * 2048 + 1024);
            }
        if (meta_lane) dma16(m_src + s0 * 8, st + S::A_BYTES + S::B_BYTES);
    };

    const int sw = (l16 >> 1) & 7;
    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](int stage, int e) {                   // step e (0 or 1) of the pair in `stage`
        const uint8_t* st = ring + stage * S::STAGE;
        StB b[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            b[j].u[0] = *(const u32x4*)(st + S::A_BYTES + (e * NF + j) * 2048 + l16 * 128 + ((lq ^ sw) * 16));
            b[j].u[1] = *(const u32x4*)(st + S::A_BYTES + (e * NF + j) * 2048 + l16 * 128 + (((4 + lq) ^ sw) * 16));
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            StA a;
            a.u = *(const u32x4*)(st + i * 2048 + l16 * 128 + (((4 * e + lq) ^ sw) * 16));
            int idx = *(const uint16_t*)(st + S::A_BYTES + S::B_BYTES + (16 * i + l16) * 16 + 8 * e + 2 * lq);
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, b[j].v, acc[i][j], idx, 0, 0);
        }
    };

    // workgroups start at different places of the k range and wrap around
    const int rot = (int)((blockIdx.x * 37u) % (unsigned)kpairs);
    auto pair_of = [&](int q) {                               // q-th pair of this workgroup; late ones clamped
        if (q >= kpairs) return kpairs - 1;
        int p = q + rot;
        return p >= kpairs ? p - kpairs : p;
    };
    issue(0, pair_of(wave));
    issue(1, pair_of(wave + WAVES));
    for (int q = wave; q < kpairs; q += 2 * WAVES) {
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            const int qq = q + d * WAVES;                     // wave-uniform
            WAIT_HERE(waitcnt_imm(S::OPS, 15));               // the older of the two pairs in flight has landed
            if (qq < kpairs) {
                const int p = pair_of(qq);
                if (!(odd_tail && p == kpairs - 1)) multiply(d, 0);
                multiply(d, 1);
            }
            // the MFMAs above consumed every LDS read of this stage: it may be refilled
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            issue(d, pair_of(qq + 2 * WAVES));
        }
    }
    WAIT_HERE(waitcnt_imm(0, 15));                            // drain the clamped look-ahead loads

    // partial tiles: lane (l16, lq) holds token 16 j + l16, rows 16 i + 4 lq .. + 3
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                part[(wave * S::BM + 16 * i + 4 * lq + e) * S::PART_PITCH + 16 * j + l16] = acc[i][j][e];
    __syncthreads();

    // Adapter term T R on dense MFMA, in chunks of 128 of the rank, from operands staged in the ring
    // (free now).  T[tok][k] is k-contiguous as stored; the tile of R[k][m0 .. m0 + BM) is k-major
    // and is read with the transposing LDS read (lane s of a 16-lane block gets four consecutive k of
    // column s; a row pitch of 160 bytes keeps its four rows on distinct banks).  Every wavefront
    // adds the fragments it owns to its own partial tile, so the sum below stays in a fixed order.
    if (K2 > 0) {
        constexpr int TP = 128 * 2 + 16, RP = 160;            // bytes per staged row of T and of R's tile
        constexpr int FR = (MF * NF + WAVES - 1) / WAVES;     // fragments per wavefront
        constexpr int SEG = S::BM / 8;                        // 16-byte segments per row of R's tile
        static_assert(16 * NF * TP + 128 * RP <= S::RING, "adapter operands fit in the ring");
        uint8_t* const t_lds = smem;                          // [16 NF tokens][TP]
        uint8_t* const r_lds = smem + 16 * NF * TP;           // [128 k][RP]
        f32x4 low[FR];
#pragma unroll
        for (int q = 0; q < FR; ++q) low[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int kc = 0; kc < K2; kc += 128) {
            const int kn = K2 - kc < 128 ? K2 - kc : 128;     // a multiple of 32
            for (int idx = t; idx < 16 * NF * 16; idx += WAVES * 64) {
                int tok = idx >> 4, pc = idx & 15;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (tok < n && pc * 8 < kn) v = *(const u32x4*)(T + (size_t)tok * K2 + kc + pc * 8);
                *(u32x4*)(t_lds + tok * TP + pc * 16) = v;
            }
            for (int idx = t; idx < 128 * SEG; idx += WAVES * 64) {
                int k = idx / SEG, sg = idx % SEG;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (k < kn && m0 + 8 * sg < m) v = *(const u32x4*)(R + (size_t)(kc + k) * m + m0 + 8 * sg);
                *(u32x4*)(r_lds + k * RP + sg * 16) = v;
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < FR; ++q) {
                const int fi = wave + WAVES * q;              // wave-uniform
                if (fi < MF * NF) {
                    const int i = fi / NF, j = fi % NF;
                    const uint8_t* ra = r_lds + (8 * lq + (l16 >> 2)) * RP + 2 * (16 * i + 4 * (l16 & 3));
                    const uint8_t* tb = t_lds + (16 * j + l16) * TP + lq * 16;
                    for (int ks = 0; ks * 32 < kn; ++ks) {
                        union { s16x4 h[2]; bf16x8 v; } a;
                        a.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(ra + ks * 32 * RP));
                        a.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(ra + (ks * 32 + 4) * RP));
                        StA b;
                        b.u = *(const u32x4*)(tb + ks * 64);
                        low[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, low[q], 0, 0, 0);
                    }
                }
            }
            __syncthreads();                                  // before the next chunk overwrites the operands
        }
#pragma unroll
        for (int q = 0; q < FR; ++q) {
            const int fi = wave + WAVES * q;
            if (fi < MF * NF) {
                const int i = fi / NF, j = fi % NF;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    part[(wave * S::BM + 16 * i + 4 * lq + e) * S::PART_PITCH + 16 * j + l16] += low[q][e];
            }
        }
        __syncthreads();
    }

    // fixed-order sum and store: thread = (feature o, token tok)
    constexpr int TOK_GROUPS = WAVES * 64 / S::BM;            // whole groups of BM threads
    const int o = t % S::BM;
    for (int tok = t < TOK_GROUPS * S::BM ? t / S::BM : n; tok < n; tok += TOK_GROUPS) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) v += part[(w * S::BM + o) * S::PART_PITCH + tok];
        if (m0 + o < m) {
            union { __bf16 h; bf16_t u; } r;
            r.h = (__bf16)v;
            C[(size_t)tok * m + m0 + o] = r.u;
        }
    }
}

template <int MF, int WAVES, int NF>
hipError_t launch_stream_lds(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                             const bf16_t* T, const bf16_t* R, int64_t K2, bf16_t* C, hipStream_t s) {
    using S = StreamLds<MF, WAVES, NF>;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    auto kern = spmm_stream_lds_kernel<MF, WAVES, NF>;
    hipError_t e = allow_dynamic_lds<spmm_stream_lds_kernel<MF, WAVES, NF>>(S::TOTAL);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)((m + S::BM - 1) / S::BM)), dim3(WAVES * 64), S::TOTAL, s>>>(B, (int)n, Av, Am, (int)m, (int)K,
                                                                                     T, R, (int)K2, C);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// The row-split form of the same product, for contractions that are whole multiples of 1024 (16 k-steps: the
// metadata of a row then comes in whole 128-byte lines).  What the kernel above pays for beyond the weight's own
// bytes is the rest of its load mix: every wavefront loads its own copy of the token operand (two thirds as many
// requests as the values) and a 16-byte piece of metadata per row and pair of k-steps (as many requests again, each
// for an eighth of a line).  Here a workgroup of three wavefronts owns 48 weight rows, every wavefront its own 16 of
// them over the workgroup's whole share of the contraction, so that
//   - the token operand of a pair of k-steps is loaded once per workgroup into a shared ring (the wavefronts deal
//     its loads among themselves; one barrier per pair),
//   - metadata is loaded a whole line per row at a time, for 8 pairs,
//   - a wavefront's accumulators are complete sums: no reduction across wavefronts,
//   - the rings are 3 pairs deep and small (42 KiB per workgroup for up to 16 tokens), so three workgroups share a
//     compute unit and cover each other's first loads and epilogues.  (The loads alone stream fastest with a ring of
//     8 pairs, 62 us against 65 us at 36864 x 9216, and 73 us for the mix of the kernel above; but then one workgroup
//     fills a compute unit, and the whole kernel took 83 us where this takes 76 us.)
// Few weight rows would leave most compute units without a workgroup; then the contraction is cut into slices
// (blockIdx.y) of whole chunks of 8 pairs, each leaving fp32 partial sums that rows_sum_kernel adds in slice order.
// About 768 workgroups, one round of three per compute unit, measured best (512: +10 % time, 1024 and more: +5-10 %).
// 36864 x 9216 at 16 tokens, rank-128 adapters: 91 -> 78 us; 9216 x 36864: 107 -> 85 us; without adapters 67 and 72 us
// (5.7 and 5.3 TB/s of packed weight).
constexpr int ROWS_WAVES = 3, ROWS_DEPTH = 3, ROWS_BM = 16 * ROWS_WAVES;
template <int NF>
struct RowsLds {
    static constexpr int A_STAGE = 2048;                      // 16 rows x 128 B: both steps of a pair
    static constexpr int M_SLOT = 2048;                       // 16 rows x 128 B: the metadata of 8 pairs
    static constexpr int WAVE_BYTES = ROWS_DEPTH * A_STAGE + 2 * M_SLOT;
    static constexpr int X_OPS = 4 * NF;                      // 1 KiB loads per pair: 2 steps x NF fragments x 2 halves
    static constexpr int X_STAGE = X_OPS * 1024;
    static constexpr int TOTAL = ROWS_WAVES * WAVE_BYTES + ROWS_DEPTH * X_STAGE;
};

// The main loop of one wavefront.  XW = how many of the pair's X_OPS token loads this wavefront issues, so that the
// number of its loads per pair, 2 + XW, is a constant the s_waitcnt immediates can be built from.
template <int NF, int XW>
__device__ __forceinline__ void rows_main_loop(const uint8_t* const (&a_src)[2], const uint8_t* const (&m_src)[2],
                                               const uint8_t* const (&b_src)[NF][2], int wave, uint8_t* mine,
                                               uint8_t* xring, int pair0, int npairs, int l16, int lq,
                                               f32x4 (&acc)[NF]) {
    using S = RowsLds<NF>;
    constexpr int L = 2 + XW;                                 // loads per pair (the metadata loads come on top, every 8th pair)
    const int sw = (l16 >> 1) & 7;
    // pair q of this slice (late ones clamped to the last, so that every call issues its L loads) into stage q % DEPTH
    auto issue = [&](int q) {
        const int p = pair0 + (q < npairs ? q : npairs - 1);
        uint8_t* st = mine + (q % ROWS_DEPTH) * S::A_STAGE;
        dma16(a_src[0] + (size_t)p * 128, st);
        dma16(a_src[1] + (size_t)p * 128, st + 1024);
        uint8_t* xs = xring + (q % ROWS_DEPTH) * S::X_STAGE;
#pragma unroll
        for (int x = 0; x < S::X_OPS; ++x)                    // load x = (step e, fragment j, half h), dealt in turn
            if (x % ROWS_WAVES == wave) {
                const int e = x / (2 * NF), j = (x / 2) % NF, h = x & 1;
                dma16(b_src[j][h] + ((size_t)2 * p + e) * 128, xs + x * 1024);
            }
    };
    auto issue_meta = [&](int c) {                            // chunk c of 8 pairs of this slice (clamped) into slot c & 1
        const int chunks = npairs / 8;
        const int pc = pair0 / 8 + (c < chunks ? c : chunks - 1);
        uint8_t* ms = mine + ROWS_DEPTH * S::A_STAGE + (c & 1) * S::M_SLOT;
        dma16(m_src[0] + (size_t)pc * 128, ms);
        dma16(m_src[1] + (size_t)pc * 128, ms + 1024);
    };
    issue_meta(0);
#pragma unroll
    for (int q = 0; q < ROWS_DEPTH - 1; ++q) issue(q);
    for (int q = 0; q < npairs; ++q) {
        // Pair q has landed (and the metadata chunk it needs, which is older) once at most the loads of the
        // DEPTH - 2 younger pairs are outstanding; a metadata load among those only makes the wait stricter.
        WAIT_HERE(waitcnt_imm((ROWS_DEPTH - 2) * L, 15));
        wg_barrier();                                         // everybody's share of the pair's tokens has landed, and
                                                              // everybody is done reading the stage refilled next
        issue(q + ROWS_DEPTH - 1);
        if ((q & 7) == 0) issue_meta(q / 8 + 1);
        const uint8_t* st = mine + (q % ROWS_DEPTH) * S::A_STAGE;
        const uint8_t* xs = xring + (q % ROWS_DEPTH) * S::X_STAGE;
        const uint8_t* ms = mine + ROWS_DEPTH * S::A_STAGE + ((q >> 3) & 1) * S::M_SLOT;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            StB b[NF];
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                b[j].u[0] = *(const u32x4*)(xs + (e * NF + j) * 2048 + l16 * 128 + ((lq ^ sw) * 16));
                b[j].u[1] = *(const u32x4*)(xs + (e * NF + j) * 2048 + l16 * 128 + (((4 + lq) ^ sw) * 16));
            }
            StA a;
            a.u = *(const u32x4*)(st + l16 * 128 + (((4 * e + lq) ^ sw) * 16));
            const int idx = *(const uint16_t*)(ms + l16 * 128 + (((q & 7) ^ sw) * 16) + 8 * e + 2 * lq);
#pragma unroll
            for (int j = 0; j < NF; ++j) acc[j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(a.v, b[j].v, acc[j], idx, 0, 0);
        }
    }
    WAIT_HERE(waitcnt_imm(0, 15));                            // drain the clamped look-ahead loads
}

// K % 1024 == 0.  blockIdx.x: block of 48 weight rows; blockIdx.y: slice of slice_pairs pairs of k-steps (a multiple of
// 8).  partial == nullptr (one slice): C bf16[n][m]; else fp32 sums into partial[slice][n][m].  The adapter term is
// added by slice 0.
template <int NF>
__global__ void __launch_bounds__(ROWS_WAVES * 64) spmm_rows_kernel(const bf16_t* __restrict__ B, int n,
                                                                   const bf16_t* __restrict__ Av,
                                                                   const uint8_t* __restrict__ Am, int m, int K,
                                                                   const bf16_t* __restrict__ T,
                                                                   const bf16_t* __restrict__ R, int K2,
                                                                   bf16_t* __restrict__ C, float* __restrict__ partial,
                                                                   int slice_pairs) {
    using S = RowsLds<NF>;
    extern __shared__ __align__(16) uint8_t smem[];
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int m0 = blockIdx.x * ROWS_BM, mw = m0 + 16 * wave;   // the workgroup's and the wavefront's first row
    const int kpairs = K / 128;
    const int pair0 = blockIdx.y * slice_pairs;
    const int npairs = kpairs - pair0 < slice_pairs ? kpairs - pair0 : slice_pairs;   // > 0 by the launch's grid
    uint8_t* const mine = smem + wave * S::WAVE_BYTES;
    uint8_t* const xring = smem + ROWS_WAVES * S::WAVE_BYTES;

    // loader lanes: 8 lanes per row, the 16-byte pieces of a line rotated by (row / 2) % 8; rows and tokens past
    // the end are read from the last one and never stored
    const int ld_row = lane >> 3, ld_slot = lane & 7;
    const uint8_t* a_src[2];
    const uint8_t* m_src[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int rl = 8 * h + ld_row;
        const int row = mw + rl < m ? mw + rl : m - 1;
        a_src[h] = (const uint8_t*)Av + (size_t)row * K + ((ld_slot ^ ((rl >> 1) & 7)) * 16);
        m_src[h] = Am + (size_t)row * (K / 8) + ((ld_slot ^ ((rl >> 1) & 7)) * 16);
    }
    const uint8_t* b_src[NF][2];
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int rl = 8 * h + ld_row;
            const int tok = 16 * j + rl < n ? 16 * j + rl : n - 1;
            b_src[j][h] = (const uint8_t*)B + (size_t)tok * K * 2 + ((ld_slot ^ ((rl >> 1) & 7)) * 16);
        }
    f32x4 acc[NF];
#pragma unroll
    for (int j = 0; j < NF; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // the token loads of a pair go to the wavefronts in turn: wavefront w issues those with x % 3 == w
    constexpr int XW0 = (S::X_OPS + 2) / 3, XW1 = (S::X_OPS + 1) / 3, XW2 = S::X_OPS / 3;
    if (wave == 0) rows_main_loop<NF, XW0>(a_src, m_src, b_src, 0, mine, xring, pair0, npairs, l16, lq, acc);
    else if (wave == 1) rows_main_loop<NF, XW1>(a_src, m_src, b_src, 1, mine, xring, pair0, npairs, l16, lq, acc);
    else rows_main_loop<NF, XW2>(a_src, m_src, b_src, 2, mine, xring, pair0, npairs, l16, lq, acc);
    __syncthreads();                                          // the rings are free

    // Adapter term T R on dense MFMA, as in the kernel above: chunks of 128 of the rank, T and the workgroup's
    // tile of R (as stored, k-major) staged in the rings, R read back with the transposing LDS read.  Wavefront w
    // owns the fragments of its 16 rows and adds them to its accumulators.
    if (K2 > 0 && blockIdx.y == 0) {
        constexpr int TP = 128 * 2 + 16, RP = 160;            // bytes per staged row of T and of R's tile
        constexpr int SEG = ROWS_BM / 8;                      // 16-byte segments per row of R's tile
        static_assert(16 * NF * TP + 128 * RP <= S::TOTAL, "adapter operands fit in the rings");
        uint8_t* const t_lds = smem;                          // [16 NF tokens][TP]
        uint8_t* const r_lds = smem + 16 * NF * TP;           // [128 k][RP]
        for (int kc = 0; kc < K2; kc += 128) {
            const int kn = K2 - kc < 128 ? K2 - kc : 128;     // a multiple of 32
            for (int idx = t; idx < 16 * NF * 16; idx += ROWS_WAVES * 64) {
                int tok = idx >> 4, pc = idx & 15;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (tok < n && pc * 8 < kn) v = *(const u32x4*)(T + (size_t)tok * K2 + kc + pc * 8);
                *(u32x4*)(t_lds + tok * TP + pc * 16) = v;
            }
            for (int idx = t; idx < 128 * SEG; idx += ROWS_WAVES * 64) {
                int k = idx / SEG, sg = idx % SEG;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (k < kn && m0 + 8 * sg < m) v = *(const u32x4*)(R + (size_t)(kc + k) * m + m0 + 8 * sg);
                *(u32x4*)(r_lds + k * RP + sg * 16) = v;
            }
            __syncthreads();
            const uint8_t* ra = r_lds + (8 * lq + (l16 >> 2)) * RP + 2 * (16 * wave + 4 * (l16 & 3));
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const uint8_t* tb = t_lds + (16 * j + l16) * TP + lq * 16;
                for (int ks = 0; ks * 32 < kn; ++ks) {
                    union { s16x4 h[2]; bf16x8 v; } a;
                    a.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(ra + ks * 32 * RP));
                    a.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(ra + (ks * 32 + 4) * RP));
                    StA b;
                    b.u = *(const u32x4*)(tb + ks * 64);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, acc[j], 0, 0, 0);
                }
            }
            __syncthreads();                                  // before the next chunk overwrites the operands
        }
    }

    // lane (l16, lq) holds token 16 j + l16, rows mw + 4 lq .. + 3 (m is a multiple of 8: the four are inside or outside together)
    const int row = mw + 4 * lq;
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        const int tok = 16 * j + l16;
        if (tok >= n || row >= m) continue;
        if (partial) {
            *(f32x4*)(partial + ((size_t)blockIdx.y * n + tok) * m + row) = acc[j];
        } else {
            union { __bf16 h[4]; u32x2 u; } o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o.h[e] = (__bf16)acc[j][e];
            *(u32x2*)(C + (size_t)tok * m + row) = o.u;
        }
    }
}

// C = the slices' partial sums added in slice order (bit-identical runs), rounded to bf16; four elements per lane
__global__ void __launch_bounds__(256) rows_sum_kernel(const f32x4* __restrict__ P, int slices, size_t count4,
                                                       u32x2* __restrict__ C) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= count4) return;
    f32x4 v = P[idx];
    for (int sl = 1; sl < slices; ++sl) {
        const f32x4 w = P[(size_t)sl * count4 + idx];
        v[0] += w[0]; v[1] += w[1]; v[2] += w[2]; v[3] += w[3];
    }
    union { __bf16 h[4]; u32x2 u; } o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o.h[e] = (__bf16)v[e];
    C[idx] = o.u;
}

// P[c][t][j] = sum over the rows i of slab c of X[t][i] * L[i][j]   (fp32 partial sums of T = X L for
// up to XL_SMALL_MAX_TOKENS tokens, on MFMA).  L is k-major (rows = d_in), the wrong way round for an
// MFMA operand, so a slab of it is staged in LDS as stored and read back with the transposing read
// ds_read_b64_tr_b16: in each block of 16 lanes, lane s receives four consecutive rows (k) of
// column s.  (A first version with fp32 multiply-adds and token values broadcast from LDS took
// 24 us where this takes 6, at 9216 x 128 and 64 tokens, and was 2 us slower even for one token.)  D rows are the
// columns of L, D columns the tokens: a lane ends up with four consecutive columns of one token.
//   workgroup = slab c of 64 * subs rows x 128 columns (blockIdx.y) x 128 tokens (blockIdx.z);
//   wavefront w takes columns 32 w .. 32 w + 31; token rows come straight from global memory
//   (k-contiguous).
constexpr int XLM_PITCH = 128 * 2 + 32;      // bytes per staged row of L: pitch % 128 == 32 keeps the
                                             // four rows of a transposing read on distinct banks
__global__ void __launch_bounds__(256) xl_mfma_kernel(const bf16_t* __restrict__ X, int n, int d_in,
                                                      const bf16_t* __restrict__ L, int r, int subs,
                                                      float* __restrict__ P) {
    extern __shared__ __align__(16) uint8_t smem[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int c = blockIdx.x, j0 = blockIdx.y * 128;
    const int k0 = c * XL_CHUNK * subs;
    int rows = d_in - k0;                                    // d_in % 64 == 0: whole chunks
    if (rows > XL_CHUNK * subs) rows = XL_CHUNK * subs;
    if (rows <= 0) return;                                   // uniform

    // stage the slab: 16 pieces of 16 bytes per row, 16 rows per pass of the workgroup
    {
        const int pc = t & 15, col = j0 + pc * 8;
        u32x4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int row = u * 16 + (t >> 4);
            v[u] = (u32x4){0u, 0u, 0u, 0u};
            if (row < rows && col < r) v[u] = *(const u32x4*)(L + (size_t)(k0 + row) * r + col);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            int row = u * 16 + (t >> 4);
            if (row < rows) *(u32x4*)(smem + row * XLM_PITCH + pc * 16) = v[u];
        }
    }
    __syncthreads();

    const int t0 = blockIdx.z * 128;
    const int ntf = ((n - t0 < 128 ? n - t0 : 128) + 15) / 16;   // token fragments of this workgroup, at most 8
    const bf16_t* x_row[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int tok = t0 + 16 * j + l16;
        x_row[j] = X + (size_t)(tok < n ? tok : t0) * d_in + k0 + lq * 8;
    }
    f32x4 acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // lane (s = l16, q = lq) points at slab row 8 q + 4 h + s / 4, column 4 (s % 4) of a 16-column
    // fragment; it receives k = 8 q + 4 h .. + 3 of column s
    const uint8_t* tr = smem + (8 * lq + (l16 >> 2)) * XLM_PITCH + 2 * (32 * wave + 4 * (l16 & 3));
    const int steps = rows / 32;
    u32x4 xb[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (j < ntf) xb[j] = *(const u32x4*)x_row[j];
    for (int st = 0; st < steps; ++st) {
        StA af[2], bf[8];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            union { s16x4 h[2]; bf16x8 v; } x;
            x.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(tr + st * 32 * XLM_PITCH + 32 * i));
            x.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3)))*)(tr + (st * 32 + 4) * XLM_PITCH + 32 * i));
            af[i].v = x.v;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) bf[j].u = xb[j];
        if (st + 1 < steps) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (j < ntf) xb[j] = *(const u32x4*)(x_row[j] + (st + 1) * 32);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (j < ntf) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i].v, bf[j].v, acc[i][j], 0, 0, 0);
            }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int tok = t0 + 16 * j + l16;
        if (tok >= n) continue;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int col = j0 + 32 * wave + 16 * i + 4 * lq;
            if (col < r) *(f32x4*)(P + ((size_t)c * n + tok) * r + col) = acc[i][j];
        }
    }
}

// T[idx] = bf16( sum over chunks of P[c][idx] ), idx = t * r + k, in a fixed order: a workgroup
// takes 32 outputs; its 8 wavefront-halves each sum every 8th chunk, then the 8 sums are added
// in order through LDS.
__global__ void __launch_bounds__(256) xl_reduce_kernel(const float* __restrict__ P, int chunks, int count,
                                                        bf16_t* __restrict__ T) {
    __shared__ float red[8][33];
    const int o = threadIdx.x & 31, cl = threadIdx.x >> 5;
    const int idx = blockIdx.x * 32 + o;
    float v = 0.f;
    if (idx < count) {
        int c = cl;
        for (; c + 56 < chunks; c += 64) {                    // 8 loads in flight
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = P[(size_t)(c + 8 * u) * count + idx];
#pragma unroll
            for (int u = 0; u < 8; ++u) v += x[u];
        }
        for (; c < chunks; c += 8) v += P[(size_t)c * count + idx];
    }
    red[cl][o] = v;
    __syncthreads();
    if (cl == 0 && idx < count) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) sum += red[w][o];
        union { __bf16 h; bf16_t u; } out;
        out.h = (__bf16)sum;
        T[idx] = out.u;
    }
}

}  // namespace

// Weight rows per workgroup of the small-batch kernel for n <= 32 tokens.
int spmm_stream_rows(int64_t n, int64_t m, int64_t K) {
    if (n <= 16) {
        // Workgroups of 32, 48 or 64 weight rows (8, 6, 4 wavefronts: what fits in LDS).  One per
        // compute unit is resident; a round of 256 of them is bound by HBM, a thin last round by
        // what one workgroup can pull (measured per shape).  Take the shape with the least estimate.
        const double hbm = 5.8e3, cap[3] = {44.0, 36.0, 29.0};   // bytes per ns: the chip, one workgroup
        const int rows[3] = {32, 48, 64};
        int best = 0;
        double best_t = 1e300;
        for (int c = 0; c < 3; ++c) {
            const double bytes = 1.125 * (double)rows[c] * (double)K;
            const int64_t blocks = (m + rows[c] - 1) / rows[c];
            const int64_t full = blocks / RESIDENT, rest = blocks % RESIDENT;
            auto round_ns = [&](int64_t nb) { double a = nb * bytes / hbm, b = bytes / cap[c]; return a > b ? a : b; };
            const double est = full * round_ns(RESIDENT) + (rest ? round_ns(rest) : 0.0);
            if (est < best_t) { best_t = est; best = c; }
        }
        return rows[best];
    }
    // 17 to 32 tokens: two token fragments per wavefront leave room for four wavefronts only
    const int64_t b32 = (m + 31) / 32, b48 = (m + 47) / 48;
    auto last_round = [](int64_t blocks) { int64_t r = blocks % RESIDENT; return r == 0 ? RESIDENT : r; };
    return last_round(b48) > last_round(b32) || b48 % RESIDENT == 0 ? 48 : 32;
}

// Slices of the row-split kernel for n <= 32 tokens (0: the shape stays with the kernel whose wavefronts split the
// contraction).  Its workgroups are 48 rows each; about three per compute unit keep the chip busy.  With scratch
// for partial sums (with_partial) a short matrix is cut along the contraction, in whole chunks of 8 pairs of k-steps.
int spmm_rows_slices(int64_t n, int64_t m, int64_t K, bool with_partial) {
    if (n > STREAM_MAX_TOKENS || K % 1024 != 0) return 0;
    const int64_t blocks = (m + ROWS_BM - 1) / ROWS_BM, chunks = K / 1024;
    int64_t slices = 1;
    if (with_partial && blocks < 3 * RESIDENT) {
        slices = (3 * RESIDENT + blocks - 1) / blocks;
        if (slices > chunks) slices = chunks;
        const int64_t per = (chunks + slices - 1) / slices;    // chunks per slice; then no slice is empty
        slices = (chunks + per - 1) / per;
    }
    // slices cost a second launch: worth it only for long contractions (9216 x 36864 at 16 tokens: 107 -> 85 us;
    // 9216 x 9216 gains nothing in 3 slices and loses 1.4 us when its weight comes from the last-level cache)
    if (slices > 1 && chunks < 16) slices = 1;
    if (blocks * slices < 2 * RESIDENT) return 0;
    // 17 to 32 tokens: the token operand is then the larger half of what a workgroup loads, and the kernel above
    // holds its own except where a long contraction over few rows leaves it with too few workgroups
    // (measured at 32 tokens: 9216 x 36864 121 -> 114 us, but 36864 x 9216 104 -> 108 us and 9216 x 9216 40 -> 43 us)
    if (n > 16 && slices < 4) return 0;
    return (int)slices;
}

size_t spmm_rows_partial_bytes(int64_t n, int64_t m, int64_t K) {
    const int slices = spmm_rows_slices(n, m, K, true);
    return slices > 1 ? (size_t)slices * (size_t)n * (size_t)m * 4 : 0;
}

template <int NF>
static hipError_t launch_rows(const bf16_t* B, int64_t n, const bf16_t* Av, const uint8_t* Am, int64_t m, int64_t K,
                              const bf16_t* T, const bf16_t* R, int64_t K2, bf16_t* C, float* partial, int slices,
                              hipStream_t s) {
    using S = RowsLds<NF>;
    static_assert(S::TOTAL <= 160 * 1024, "LDS budget");
    hipError_t e = allow_dynamic_lds<spmm_rows_kernel<NF>>(S::TOTAL);
    if (e != hipSuccess) return e;
    const int64_t chunks = K / 1024, per = (chunks + slices - 1) / slices;
    spmm_rows_kernel<NF><<<dim3((unsigned)((m + ROWS_BM - 1) / ROWS_BM), (unsigned)slices), dim3(ROWS_WAVES * 64), S::TOTAL, s>>>(
        B, (int)n, Av, Am, (int)m, (int)K, T, R, (int)K2, C, slices > 1 ? partial : nullptr, (int)(per * 8));
    if ((e = hipGetLastError()) != hipSuccess || slices == 1) return e;
    const size_t count4 = (size_t)n * (size_t)m / 4;
    rows_sum_kernel<<<dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, s>>>((const f32x4*)partial, slices, count4, (u32x2*)C);
    return hipGetLastError();
}

// n <= 32, K % 64 == 0, K >= 128; T (bf16[n][K2]) and R (bf16[K2][m]) only when K2 > 0; partial_or_null: scratch of
// spmm_rows_partial_bytes(n, m, K) bytes
hipError_t launch_spmm_stream(const bf16_t* B, int64_t n, const bf16_t* A_vals, const uint8_t* A_meta, int64_t m,
                              int64_t K, const bf16_t* T, const bf16_t* R, int64_t K2, bf16_t* C, float* partial_or_null,
                              hipStream_t s) {
    const int slices = spmm_rows_slices(n, m, K, partial_or_null != nullptr);
    if (slices > 0)
        return n <= 16 ? launch_rows<1>(B, n, A_vals, A_meta, m, K, T, R, K2, C, partial_or_null, slices, s)
                       : launch_rows<2>(B, n, A_vals, A_meta, m, K, T, R, K2, C, partial_or_null, slices, s);
    const int rows = spmm_stream_rows(n, m, K);
    if (n <= 16) {
        if (rows == 32) return launch_stream_lds<2, 8, 1>(B, n, A_vals, A_meta, m, K, T, R, K2, C, s);
        if (rows == 48) return launch_stream_lds<3, 6, 1>(B, n, A_vals, A_meta, m, K, T, R, K2, C, s);
        return launch_stream_lds<4, 4, 1>(B, n, A_vals, A_meta, m, K, T, R, K2, C, s);
    }
    if (rows == 48) return launch_stream_lds<3, 4, 2>(B, n, A_vals, A_meta, m, K, T, R, K2, C, s);
    return launch_stream_lds<2, 4, 2>(B, n, A_vals, A_meta, m, K, T, R, K2, C, s);
}

// T = X L for few tokens (up to XL_SMALL_MAX_TOKENS), split over d_in; scratch holds xl_small_scratch_bytes.
// Slabs of L per workgroup: up to four chunks of 64 rows (smaller partial sums) as long as the launch
// still has a workgroup for every compute unit.
int xl_subs(int64_t n, int64_t d_in, int64_t r) {
    const int64_t per_slab = ((r + 127) / 128) * ((n + 127) / 128);   // workgroups per slab
    for (int subs = 4; subs > 1; subs /= 2)
        if ((d_in + XL_CHUNK * subs - 1) / (XL_CHUNK * subs) * per_slab >= RESIDENT) return subs;
    return 1;
}

size_t xl_small_scratch_bytes(int64_t n, int64_t d_in, int64_t r) {
    const int64_t rows = (int64_t)XL_CHUNK * xl_subs(n, d_in, r);
    return (size_t)((d_in + rows - 1) / rows) * (size_t)n * (size_t)r * 4;
}

hipError_t launch_xl_small(const bf16_t* X, int64_t n, int64_t d_in, const bf16_t* L, int64_t r, float* scratch,
                           bf16_t* T, hipStream_t s) {
    const int subs = xl_subs(n, d_in, r);
    const int slabs = (int)((d_in + XL_CHUNK * subs - 1) / (XL_CHUNK * subs));
    const int lds = XL_CHUNK * subs * XLM_PITCH;
    hipError_t e = allow_dynamic_lds<xl_mfma_kernel>(XL_CHUNK * 4 * XLM_PITCH);   // the largest slab (subs <= 4)
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)slabs, (unsigned)((r + 127) / 128), (unsigned)((n + 127) / 128));
    xl_mfma_kernel<<<grid, dim3(256), lds, s>>>(X, (int)n, (int)d_in, L, (int)r, subs, scratch);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int count = (int)(n * r);
    xl_reduce_kernel<<<dim3((unsigned)((count + 31) / 32)), dim3(256), 0, s>>>(scratch, slabs, count, T);
    return hipGetLastError();
}
