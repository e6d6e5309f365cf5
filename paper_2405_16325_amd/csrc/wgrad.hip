// slope_wgrad_masked: dW = dY^T X (Eq. 5) on dense MFMA, with the prune-and-compress step of
// Algorithm 1 line 13 folded into the epilogue.
//
// The contraction runs over the b tokens, which is the slow index of both operands, so both are
// staged in LDS as [token][feature] slabs (the same order as in memory: fully coalesced loads) and
// read back with ds_read_b64_tr_b16, CDNA4's transposing LDS read: inside each block of 16 lanes,
// lane r receives element r of four consecutive slab rows, i.e. four consecutive k of one feature.
//
// The MFMA is v_mfma_f32_16x16x32_bf16 with D rows = d_in and D columns = d_out:
//   D lane l holds column (d_out) l%16 and rows (d_in) 4*(l/16) .. +3 = exactly one group of four
//   of W^R's row, so the epilogue picks two of a lane's four accumulators with the group's
//   metadata nibble and stores them as one 4-byte pair of the packed gradient.
#include "pipeline.h"

namespace {

constexpr int WG_KS = 32;                      // tokens per LDS stage

__device__ __forceinline__ void wgrad_tile_of_block(int nblocks, int tiles_m, int tiles_n, int& tm, int& tn) {
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

// BM: tile extent along d_in (MFMA rows), BN: along d_out (MFMA columns).
template <int BM, int BN>
struct WgSmem {
    static constexpr int PITCH_A = BM * 2 + 32;     // bytes per token row; pitch % 128 == 32 keeps the
    static constexpr int PITCH_B = BN * 2 + 32;     // four rows of a transposing read on distinct banks
    static constexpr int A_BYTES = WG_KS * PITCH_A;
    static constexpr int B_BYTES = WG_KS * PITCH_B;
    static constexpr int STAGE = A_BYTES + B_BYTES;
};

__device__ __forceinline__ s16x4 lds_read_tr(const uint8_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

template <int BM, int BN>
__global__ void __launch_bounds__(256) wgrad_kernel(const bf16_t* __restrict__ dY, const bf16_t* __restrict__ X, int b,
                                                    const uint8_t* __restrict__ meta, int d_out, int d_in,
                                                    bf16_t* __restrict__ G, int tiles_m, int tiles_n) {
    using S = WgSmem<BM, BN>;
    constexpr int MF = BM / 32, NF = BN / 32;           // 16 x 16 fragments per wavefront (2 x 2 waves)
    constexpr int A_LD = BM / 64, B_LD = BN / 64;       // 16-byte loads per lane per stage (32 rows)
    extern __shared__ __align__(16) uint8_t smem[];

    int tm, tn;
    wgrad_tile_of_block(tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
    const int i0 = tm * BM, o0 = tn * BN;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, lq = lane >> 4;

    // global -> register staging: lane owns 16-byte pieces (8 features) of token rows
    constexpr int A_PER_ROW = BM / 8, B_PER_ROW = BN / 8;
    uint4 a_reg[A_LD], b_reg[B_LD];
    auto load_global = [&](int t0) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            int idx = t + 256 * i, row = idx / A_PER_ROW, c = idx % A_PER_ROW;
            int tok = t0 + row, col = i0 + 8 * c;
            a_reg[i] = (tok < b && col < d_in) ? *(const uint4*)(X + (size_t)tok * d_in + col) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int idx = t + 256 * i, row = idx / B_PER_ROW, c = idx % B_PER_ROW;
            int tok = t0 + row, col = o0 + 8 * c;
            b_reg[i] = (tok < b && col < d_out) ? *(const uint4*)(dY + (size_t)tok * d_out + col) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int stage) {
        uint8_t* base = smem + stage * S::STAGE;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            int idx = t + 256 * i, row = idx / A_PER_ROW, c = idx % A_PER_ROW;
            *(uint4*)(base + row * S::PITCH_A + 16 * c) = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            int idx = t + 256 * i, row = idx / B_PER_ROW, c = idx % B_PER_ROW;
            *(uint4*)(base + S::A_BYTES + row * S::PITCH_B + 16 * c) = b_reg[i];
        }
    };

    f32x4 acc[MF][NF];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < NF; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // transposing-read addresses: lane (s = l%16, q = l/16) points at slab row 8q + 4h + s/4,
    // feature 4*(s%4); it receives k = 8q + 4h .. +3 of feature s
    const int tr_row = 8 * lq + (l16 >> 2), tr_col = 4 * (l16 & 3);
    const int a_off = tr_row * S::PITCH_A + 2 * (wm * (BM / 2) + tr_col);
    const int b_off = tr_row * S::PITCH_B + 2 * (wn * (BN / 2) + tr_col);

    const int ksteps = (b + WG_KS - 1) / WG_KS;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < ksteps; ++ks) {
        const int stage = ks & 1;
        if (ks + 1 < ksteps) load_global((ks + 1) * WG_KS);
        const uint8_t* sa = smem + stage * S::STAGE + a_off;
        const uint8_t* sb = smem + stage * S::STAGE + S::A_BYTES + b_off;
        bf16x8 bf[NF];
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            union { s16x4 h[2]; bf16x8 v; } x;
            x.h[0] = lds_read_tr(sb + 32 * j);
            x.h[1] = lds_read_tr(sb + 32 * j + 4 * S::PITCH_B);
            bf[j] = x.v;
        }
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            union { s16x4 h[2]; bf16x8 v; } a;
            a.h[0] = lds_read_tr(sa + 32 * i);
            a.h[1] = lds_read_tr(sa + 32 * i + 4 * S::PITCH_A);
#pragma unroll
            for (int j = 0; j < NF; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, bf[j], acc[i][j], 0, 0, 0);
        }
        if (ks + 1 < ksteps) store_lds(stage ^ 1);
        __syncthreads();
    }

    // epilogue: a lane's four accumulators are one group of four along d_in of row o
    const size_t mpitch = (size_t)d_in / 8, gpitch = (size_t)d_in / 2;
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        int o = o0 + (wn * NF + j) * 16 + l16;
        if (o >= d_out) continue;
#pragma unroll
        for (int i = 0; i < MF; ++i) {
            int col = i0 + (wm * MF + i) * 16 + lq * 4;   // first d_in index of the group
            if (col >= d_in) continue;
            int g = col >> 2;
            uint32_t nib = (meta[(size_t)o * mpitch + (g >> 1)] >> (4 * (g & 1))) & 0xFu;
            uint32_t a = nib & 3u, c = nib >> 2;
            f32x4 v = acc[i][j];
            float v0 = a == 0 ? v[0] : (a == 1 ? v[1] : v[2]);
            float v1 = c == 1 ? v[1] : (c == 2 ? v[2] : v[3]);
            union { __bf16 h[2]; uint32_t u; } out;
            out.h[0] = (__bf16)v0;
            out.h[1] = (__bf16)v1;
            *(uint32_t*)(G + (size_t)o * gpitch + 2 * g) = out.u;
        }
    }
}

template <int BM, int BN>
hipError_t launch_tile(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out, int64_t d_in,
                       bf16_t* G, hipStream_t s) {
    using S = WgSmem<BM, BN>;
    int tiles_m = (int)((d_in + BM - 1) / BM), tiles_n = (int)((d_out + BN - 1) / BN);
    size_t smem = 2 * S::STAGE;
    auto kern = wgrad_kernel<BM, BN>;
    hipError_t e = allow_dynamic_lds<wgrad_kernel<BM, BN>>((int)smem);
    if (e != hipSuccess) return e;
    kern<<<dim3((unsigned)(tiles_m * tiles_n)), dim3(256), smem, s>>>(dY, X, (int)b, meta, (int)d_out, (int)d_in, G,
                                                                       tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_wgrad_masked(const bf16_t* dY, const bf16_t* X, int64_t b, const uint8_t* meta, int64_t d_out,
                               int64_t d_in, bf16_t* gvals, hipStream_t s) {
    int64_t big = ((d_in + 255) / 256) * ((d_out + 255) / 256);
    if (big >= 256) return launch_tile<256, 256>(dY, X, b, meta, d_out, d_in, gvals, s);
    return launch_tile<128, 128>(dY, X, b, meta, d_out, d_in, gvals, s);
}
