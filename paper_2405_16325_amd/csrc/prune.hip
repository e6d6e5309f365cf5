// slope_prune_rows and slope_double_prune: HBM-bound streams (Sec. 2.1; App. B "setup").
//
// prune_rows   : one lane owns 8 consecutive weights (one 16-byte load = two groups of four),
//                ranks each group with a branch-free comparison network and writes 8 bytes of
//                kept values, one metadata byte and (optionally) one mask byte.  A wavefront
//                reads 1 KiB and writes 512 + 64 (+ 64) contiguous bytes.
// double_prune : a workgroup takes a 128 x 128 tile of W^R; every lane reads 4 rows x 8 columns of it
//                (packed, whole lines per 16 lanes), decompresses them in registers, ranks each column's
//                group of four along d_out among the surviving positions, and the tile is written out
//                transposed through an LDS stage so that the write is coalesced as well.
#include "common.h"

// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void prune_chunk(u32x4 w, u32x2& packed, uint32_t& meta_byte, uint32_t& mask_byte) {
    uint32_t lo[2] = {w.x, w.z}, hi[2] = {w.y, w.w}, pk[2], nib[2], set[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        uint32_t k0 = lo[g] & 0x7FFFu, k1 = (lo[g] >> 16) & 0x7FFFu;
        uint32_t k2 = hi[g] & 0x7FFFu, k3 = (hi[g] >> 16) & 0x7FFFu;
        set[g] = top2_of_4(k0, k1, k2, k3);
        nib[g] = nibble_of_pair(set[g]);
        uint64_t q = (uint64_t)lo[g] | ((uint64_t)hi[g] << 32);
        uint32_t v0 = (uint32_t)(q >> (16u * (nib[g] & 3u))) & 0xFFFFu;
        uint32_t v1 = (uint32_t)(q >> (16u * (nib[g] >> 2))) & 0xFFFFu;
        pk[g] = v0 | (v1 << 16);
    }
    packed = (u32x2){pk[0], pk[1]};
    meta_byte = nib[0] | (nib[1] << 4);
    mask_byte = set[0] | (set[1] << 4);
}

// Four neighbouring lanes hold four consecutive output bytes: gather them into lane 4q.
__device__ __forceinline__ uint32_t gather_quad_bytes(uint32_t b) {
    b |= (uint32_t)__shfl_down((int)b, 1, 64) << 8;
    b |= (uint32_t)__shfl_down((int)b, 2, 64) << 16;
    return b;
}

// A workgroup takes PR_UNROLL x 256 consecutive 16-byte chunks of W, lane t the chunks t, t + 256, ...
// of them, and the workgroups follow each other in address order.  Many short-lived workgroups, each with all of
// its loads issued at once, stream measurably faster on this chip than a few thousand that loop over the array with
// the stride of the grid (a plain copy: 6.6 against 4.5 TB/s).
constexpr int PR_UNROLL = 2;        // 8 KiB of W per workgroup: 0.118 -> 0.087 ms per OPT-66B layer (6.1 TB/s); 1: 0.101, 4: 0.089, 8: 0.094

__global__ void __launch_bounds__(256) prune_rows_kernel(const u32x4* __restrict__ W, size_t nchunks,
                                                         u32x2* __restrict__ vals, uint8_t* __restrict__ meta,
                                                         uint8_t* __restrict__ mask) {
    const size_t first = (size_t)blockIdx.x * (256 * PR_UNROLL) + threadIdx.x;
    const int sub = threadIdx.x & 3;
    u32x4 w[PR_UNROLL];
#pragma unroll
    for (int u = 0; u < PR_UNROLL; ++u) {
        size_t c = first + u * 256;
        w[u] = c < nchunks ? __builtin_nontemporal_load(W + c) : (u32x4){0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < PR_UNROLL; ++u) {
        size_t c = first + u * 256;
        u32x2 pk;
        uint32_t mb, kb;
        prune_chunk(w[u], pk, mb, kb);
        bool ok = c < nchunks;
        bool quad_ok = (c - sub) + 3 < nchunks;  // all four lanes of the quad are in range
        if (ok) __builtin_nontemporal_store(pk, vals + c);
        uint32_t m4 = gather_quad_bytes(mb);
        if (quad_ok) {
            if (sub == 0) __builtin_nontemporal_store(m4, (uint32_t*)(meta + c));
        } else if (ok) {
            meta[c] = (uint8_t)mb;
        }
        if (mask) {
            uint32_t k4 = gather_quad_bytes(kb);
            if (quad_ok) {
                if (sub == 0) __builtin_nontemporal_store(k4, (uint32_t*)(mask + c));
            } else if (ok) {
                mask[c] = (uint8_t)kb;
            }
        }
    }
}

hipError_t launch_prune_rows(const bf16_t* W, int64_t d_out, int64_t d_in, bf16_t* vals, uint8_t* meta,
                             uint8_t* mask, hipStream_t s) {
    size_t nchunks = (size_t)d_out * (size_t)d_in / 8;
    size_t per_block = 256 * PR_UNROLL;
    size_t blocks = (nchunks + per_block - 1) / per_block;    // extents below 2^31: fewer than 2^31 workgroups
    if (blocks == 0) blocks = 1;
    prune_rows_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const u32x4*)W, nchunks, (u32x2*)vals, meta, mask);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
constexpr int DP_TILE = 128;        // logical tile edge along d_out and d_in
constexpr int DP_THREADS = 512;     // a lane ranks 4 rows x 8 columns of the tile
constexpr int DP_CHUNK = 8;         // an XCD takes chunks of 8 x 8 neighbouring tiles
constexpr int DP_OPITCH = 33;       // dwords per output row [i][og] (32 + 1: conflict-free columns)
constexpr int DP_NPITCH = 36;       // bytes per nibble row [i][og]

// A raw buffer descriptor over `bytes` bytes from `base` (the same for all lanes of a workgroup): loads at offsets
// beyond it return 0 and stores there are dropped, which replaces every bounds branch of the kernel below.
typedef __amdgpu_buffer_rsrc_t buffer_t;
__device__ __forceinline__ buffer_t tile_buffer(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
constexpr uint32_t NOWHERE = 0x80000000u;   // an offset outside every descriptor (they cover less than 2^31 bytes)

// Per 16-bit half: 1 where kj > ki, else 0 (saturating subtract, then min with 1).  Written as instructions
// because the compiler turns the portable form back into one compare and one select per half.
__device__ __forceinline__ uint32_t pk_beats(uint32_t kj, uint32_t ki, uint32_t ones) {
    uint32_t d, c;
    asm("v_pk_sub_u16 %0, %1, %2 clamp" : "=v"(d) : "v"(kj), "v"(ki));
    asm("v_pk_min_u16 %0, %1, %2" : "=v"(c) : "v"(d), "v"(ones));
    return c;
}

// GIVEN = false: slope_double_prune, the pairs are chosen here by magnitude among the survivors
//                 and their metadata is written.
// GIVEN = true : slope_update_sparse, the pairs are the ones metaT_in already names (static
//                 masks, Alg. 1 line 18); only the values of the transposed copy are rewritten.
//                 A slot that names a position outside W^R's mask reads the zero that the
//                 decompression left there, so padding stays +0.0.
// RAGGED: d_out is not a multiple of 32: rows of the transposed arrays are then only 8-byte (values) and
//                 1-byte (metadata) aligned and may end inside a lane's piece, so they are written in pieces
//                 of 8 logical elements (8 bytes of values, 1 byte of metadata), each wholly inside the row
//                 or skipped.  The input needs no such care: a lane reads 8 logical columns of a row at a
//                 time (8 bytes of values, 1 byte of metadata), and d_in is a multiple of 8.
//
// A lane ranks 4 rows x 8 columns (one group of four along d_out per column).  It reads exactly those pieces of
// packed W^R itself: 16 neighbouring lanes cover 128 contiguous bytes of a row, so the loads are whole lines
// without a stage in LDS (an earlier version decompressed the tile into LDS first: 15 % more vector instructions
// and two more barriers for nothing).  512 lanes of 43 registers rather than 256 lanes with two pieces each: 8
// waves per SIMD hide the loads; walking several tiles per workgroup with the next tile's loads in flight was
// slower than one tile per short-lived workgroup (175 -> 185 us with two tiles, 192 with four).
template <bool GIVEN, bool MASK, bool RAGGED>
__global__ void __launch_bounds__(DP_THREADS) double_prune_kernel(const bf16_t* __restrict__ vals,
                                                           const uint8_t* __restrict__ meta, int d_out, int d_in,
                                                           bf16_t* __restrict__ valsT, uint8_t* __restrict__ metaT,
                                                           uint8_t* __restrict__ maskrc,
                                                           const uint8_t* __restrict__ metaT_in, int tiles_x,
                                                           int tiles_y) {
    // the output tile: kept value pairs [i][og] and metadata nibbles [i][og]; given metadata (GIVEN) has its own
    __shared__ __align__(16) uint8_t sbuf[DP_TILE * DP_OPITCH * 4 + DP_TILE * DP_NPITCH];
    __shared__ __align__(4) uint8_t sG[GIVEN ? DP_TILE * DP_NPITCH : 4];
    uint32_t* const sO = (uint32_t*)sbuf;                      // kept value pairs [i][og]
    uint8_t* const sN = sbuf + DP_TILE * DP_OPITCH * 4;        // metadata nibbles [i][og]
    // Decompression by table: a packed dword (the values at positions a < b of a group of four) becomes the two
    // dwords of the group's four columns through two byte permutes, whose selectors depend on the metadata nibble
    // alone: bytes 0, 1 for position a, bytes 2, 3 for position b, the constant zero (selector 12) elsewhere.
    __shared__ uint2 sSel[16];
    // Ranking by table: the six comparisons of a group's four keys (bit 0: 1 beats 0, then 2 beats 0, 3 beats 0,
    // 2 beats 1, 3 beats 1, 3 beats 2) decide which two rows are kept.  Entry: .x = the byte-permute selector that
    // picks the kept pair out of the four rows' values (bytes 2 idx, 2 idx + 1 of the eight), .y = the metadata
    // nibble | the 4-bit set of kept rows << 8.  sNib: the same selector by metadata nibble, for given metadata.
    __shared__ uint2 sRank[64];
    __shared__ uint32_t sNib[16];

    const int t = threadIdx.x;
    // Workgroup -> tile.  A tile's rows of metadata are 16-byte pieces of 128-byte lines, which 8 neighbours along
    // d_in share on the input side and 8 along d_out on the output side.  Workgroups go to the 8 XCDs in turn and
    // each XCD has its own L2, so with neighbouring tiles on neighbouring workgroup numbers every XCD fetched every
    // such line: as many bytes again as the values.  Instead an XCD takes chunks of 8 x 8 neighbouring tiles, whose
    // rows are 1 KB runs of values in both arrays (measured: 171 -> 157 us at 36864 x 9216; 8 x 4 163, 16 x 8 166,
    // 8 x 16 161, 8 x 1 180; chunk after chunk along d_out instead of d_in: 161).
    const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    const uint32_t chunk = (slot / (DP_CHUNK * DP_CHUNK)) * 8 + xcd, within = slot % (DP_CHUNK * DP_CHUNK);
    const uint32_t chunks_x = ((uint32_t)tiles_x + DP_CHUNK - 1) / DP_CHUNK;
    const int tile_x = (int)((chunk % chunks_x) * DP_CHUNK + within % DP_CHUNK);
    const int tile_y = (int)((chunk / chunks_x) * DP_CHUNK + within / DP_CHUNK);
    if (tile_x >= tiles_x || tile_y >= tiles_y) return;         // the whole workgroup: padding of the chunked order
    const int o0 = tile_y * DP_TILE;
    // Bytes per row: packed W^R values d_in, its metadata (and the mask) d_in / 8; transposed values d_out,
    // transposed metadata d_out / 8.  Every access goes through a buffer descriptor that covers the tile's rows
    // of its array: rows past the end of the matrix fall outside the descriptor (loads return 0, stores are
    // dropped), and a lane whose columns lie past the end of a row gets an offset that no descriptor covers.
    // No access is under a branch, so the compiler knows how many are in flight at any point.
    const uint32_t vrow = (uint32_t)d_in, mrow = (uint32_t)d_in / 8, vtrow = (uint32_t)d_out, mtrow = (uint32_t)d_out / 8;
    const uint32_t rows_o = (uint32_t)min(DP_TILE, d_out - o0);
    const buffer_t bV = tile_buffer((const uint8_t*)vals + (size_t)o0 * vrow, rows_o * vrow);
    const buffer_t bM = tile_buffer(meta + (size_t)o0 * mrow, rows_o * mrow);
    const buffer_t bK = tile_buffer(MASK ? maskrc + (size_t)o0 * mrow : nullptr, MASK ? rows_o * mrow : 0u);

    // A lane's 4 rows x 8 columns of packed W^R: 8 bytes of values and the metadata byte per row.
    const uint32_t og = t >> 4, i8 = t & 15;
    const int i0 = tile_x * DP_TILE;
    const uint32_t rows_i = (uint32_t)min(DP_TILE, d_in - i0);
    const bool col_ok = i0 + 8 * (int)i8 < d_in;
    u32x2 pk[4];
    uint32_t mb[4];
    {
        const uint32_t voff = col_ok ? 4u * og * vrow + (uint32_t)i0 + 8u * i8 : NOWHERE;
        const uint32_t moff = col_ok ? 4u * og * mrow + (uint32_t)i0 / 8 + i8 : NOWHERE;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            pk[k] = __builtin_amdgcn_raw_buffer_load_b64(bV, voff + k * vrow, 0, 0);
            mb[k] = __builtin_amdgcn_raw_buffer_load_b8(bM, moff + k * mrow, 0, 0);
        }
    }
    // (the table is filled while the loads are in flight)
    if (t < 16) {
        const uint32_t a = t & 3u, b = t >> 2;
        uint32_t src[4];
#pragma unroll
        for (uint32_t p = 0; p < 4; ++p) src[p] = p == a ? 0x0100u : (p == b ? 0x0302u : 0x0C0Cu);
        sSel[t] = make_uint2(src[0] | (src[1] << 16), src[2] | (src[3] << 16));
        sNib[t] = 0x01000100u + a * 0x0202u + ((b * 0x0202u) << 16);
    }
    if (!GIVEN && t >= 64 && t < 128) {
        const uint32_t c = t - 64;
        const uint32_t c01 = c & 1u, c02 = (c >> 1) & 1u, c03 = (c >> 2) & 1u, c12 = (c >> 3) & 1u, c13 = (c >> 4) & 1u,
                       c23 = (c >> 5) & 1u;
        // rank = how many of the others come first (larger key, or equal key and lower index); ranks 0 and 1 stay
        const uint32_t r0 = c01 + c02 + c03, r1 = (1u - c01) + c12 + c13, r2 = (2u - c02 - c12) + c23,
                       r3 = 3u - c03 - c13 - c23;
        const uint32_t set = (uint32_t)(r0 < 2u) | ((uint32_t)(r1 < 2u) << 1) | ((uint32_t)(r2 < 2u) << 2) |
                             ((uint32_t)(r3 < 2u) << 3);
        const uint32_t nib = nibble_of_pair(set);              // (comparisons that contradict each other: never looked up)
        sRank[c] = make_uint2(0x01000100u + (nib & 3u) * 0x0202u + (((nib >> 2) * 0x0202u) << 16), nib | (set << 8));
    }
    __syncthreads();
    if (GIVEN) {   // the tile of the given metadata, one nibble per byte: 128 rows (d_in) x 32 groups along d_out
        const buffer_t bG = tile_buffer(metaT_in + (size_t)i0 * mtrow, rows_i * mtrow);
        const uint32_t row = t >> 2, quarter = t & 3;
        const int o = o0 + 32 * quarter;
        const uint32_t off = row * mtrow + (uint32_t)o / 8;
        uint32_t x = 0;
        if (!RAGGED) {
            x = __builtin_amdgcn_raw_buffer_load_b32(bG, o < d_out ? off : NOWHERE, 0, 0);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t byte = __builtin_amdgcn_raw_buffer_load_b8(bG, o + 8 * q < d_out ? off + q : NOWHERE, 0, 0);
                x |= byte << (8 * q);
            }
        }
        uint8_t* dst = sG + row * DP_NPITCH + 8 * quarter;
#pragma unroll
        for (int q = 0; q < 8; ++q) dst[q] = (uint8_t)((x >> (4 * q)) & 0xFu);
        __syncthreads();
    }
    // r[k][q] = the values of columns 2q, 2q + 1 of row k as one dword (zeros where W^R has none);
    // ky[k][q] = their ranking keys in the same places: magnitude + 1 for a survivor of the row prune, 0 for a
    // pruned slot, so that survivors outrank every pruned slot, zeros included.  Both come out of the same two
    // permutes; the keys' source is the packed dword with the signs cleared and 1 added to both halves.  Rows and
    // columns outside the matrix read as zeros with metadata 0; what is ranked there is never stored (d_out is a
    // multiple of 4, so a group of four rows is inside or outside as a whole).
    uint32_t r[4][4], ky[4][4], cb[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t m = mb[k];
        uint32_t cand = 0;
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const uint32_t w = pk[k][g], nib = (m >> (4 * g)) & 0xFu;
            const uint2 sel = sSel[nib];
            r[k][2 * g] = __builtin_amdgcn_perm(0u, w, sel.x);
            r[k][2 * g + 1] = __builtin_amdgcn_perm(0u, w, sel.y);
            if (!GIVEN) {
                const uint32_t kw = (w & 0x7FFF7FFFu) + 0x00010001u;
                ky[k][2 * g] = __builtin_amdgcn_perm(0u, kw, sel.x);
                ky[k][2 * g + 1] = __builtin_amdgcn_perm(0u, kw, sel.y);
            }
            if (MASK) cand |= ((1u << (nib & 3u)) | (1u << (nib >> 2))) << (4 * g);
        }
        cb[k] = cand;                                             // only the mask output needs the candidate bits
    }
    // Two neighbouring columns are ranked at once in the two 16-bit halves of a register: a row's dword already
    // holds the pair, keys are at most 0x8000, and "j beats i" is min(k_j -sat k_i, 1).
    const uint32_t ones = 0x00010001u;
    const uint32_t swz = (i8 >> 3) << 2;                           // = ((column >> 6) << 2)
    uint32_t keep[4] = {0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < 4; ++q) {                                  // columns 8 i8 + 2 q (low halves) and + 1 (high halves)
        uint32_t x[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) x[k] = r[k][q];
        uint2 picked[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};   // the table's entries of the two columns
        if (!GIVEN) {
            uint32_t key[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) key[k] = ky[k][q];
            const uint32_t c01 = pk_beats(key[1], key[0], ones), c02 = pk_beats(key[2], key[0], ones),
                           c03 = pk_beats(key[3], key[0], ones), c12 = pk_beats(key[2], key[1], ones),
                           c13 = pk_beats(key[3], key[1], ones), c23 = pk_beats(key[3], key[2], ones);
            // the six outcomes of either column as the byte offset of its table entry (8 bytes each)
            const uint32_t code = (c01 << 3) | (c02 << 4) | (c03 << 5) | (c12 << 6) | (c13 << 7) | (c23 << 8);
            picked[0] = *(const uint2*)((const uint8_t*)sRank + (code & 0x1F8u));
            picked[1] = *(const uint2*)((const uint8_t*)sRank + (code >> 16));
        }
        // the four rows' values of either column as one 64-bit word
        const uint32_t qlo[2] = {__builtin_amdgcn_perm(x[1], x[0], 0x05040100u), __builtin_amdgcn_perm(x[3], x[2], 0x05040100u)};
        const uint32_t qhi[2] = {__builtin_amdgcn_perm(x[1], x[0], 0x07060302u), __builtin_amdgcn_perm(x[3], x[2], 0x07060302u)};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = 2 * q + h;
            const uint32_t col = 8 * i8 + j;
            // the values of rows idx0 = nib & 3 and idx1 = nib >> 2
            const uint32_t sel = GIVEN ? sNib[sG[col * DP_NPITCH + og]] : picked[h].x;
            // a wave's 16 columns x 4 row groups: columns 64 apart would share banks, so the upper 64 swap
            // neighbouring fours of row groups
            sO[col * DP_OPITCH + (og ^ swz)] = h ? __builtin_amdgcn_perm(qhi[1], qhi[0], sel) : __builtin_amdgcn_perm(qlo[1], qlo[0], sel);
            if (!GIVEN) sN[col * DP_NPITCH + (og ^ swz)] = (uint8_t)picked[h].y;   // the low byte: the nibble
            if (MASK) {
                const uint32_t set = picked[h].y >> 8;
#pragma unroll
                for (int k = 0; k < 4; ++k) keep[k] |= (((set >> k) & 1u) & ((cb[k] >> j) & 1u)) << j;
            }
        }
    }
    if (MASK) {
        const uint32_t off = col_ok ? 4u * og * mrow + (uint32_t)i0 / 8 + i8 : NOWHERE;
#pragma unroll
        for (int k = 0; k < 4; ++k) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)keep[k], bK, off + k * mrow, 0, 0);
    }
    __syncthreads();

    // coalesced write of packed (W^{R,C})^T rows
    const buffer_t bVT = tile_buffer((uint8_t*)valsT + (size_t)i0 * vtrow, rows_i * vtrow);
#pragma unroll
    for (int n = 0; n < 2; ++n) {
        const uint32_t idx = t + DP_THREADS * n, row = idx >> 3, c = idx & 7;
        const int o = o0 + 16 * c;
        const uint32_t* src = sO + row * DP_OPITCH + 4 * (c ^ (row >> 6));
        const uint32_t off = row * vtrow + (uint32_t)o;
        if (!RAGGED) {
            __builtin_amdgcn_raw_buffer_store_b128((u32x4){src[0], src[1], src[2], src[3]}, bVT, o < d_out ? off : NOWHERE, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b64((u32x2){src[0], src[1]}, bVT, o < d_out ? off : NOWHERE, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b64((u32x2){src[2], src[3]}, bVT, o + 8 < d_out ? off + 8 : NOWHERE, 0, 0);
        }
    }
    if (!GIVEN) {
        const buffer_t bMT = tile_buffer(metaT + (size_t)i0 * mtrow, rows_i * mtrow);
        const uint32_t row = t >> 2, c = t & 3;
        const int o = o0 + 32 * c;
        const uint32_t* src = (const uint32_t*)(sN + row * DP_NPITCH + 8 * c);
        const uint32_t x = src[row >> 6], y = src[1 - (row >> 6)];
        const uint32_t lo = (x & 0xFu) | ((x >> 4) & 0xF0u) | ((x >> 8) & 0xF00u) | ((x >> 12) & 0xF000u);
        const uint32_t hi = (y & 0xFu) | ((y >> 4) & 0xF0u) | ((y >> 8) & 0xF00u) | ((y >> 12) & 0xF000u);
        const uint32_t word = lo | (hi << 16);
        const uint32_t off = row * mtrow + (uint32_t)o / 8;
        if (!RAGGED) {
            __builtin_amdgcn_raw_buffer_store_b32(word, bMT, o < d_out ? off : NOWHERE, 0, 0);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(word >> (8 * q)), bMT, o + 8 * q < d_out ? off + q : NOWHERE, 0, 0);
        }
    }
}

// Grid of the chunked tile order: whole chunks of 8 x 8 tiles, a multiple of 8 chunks (one per XCD); workgroups
// whose tile lies outside the matrix leave at once.
static dim3 double_prune_grid(int64_t tiles_x, int64_t tiles_y) {
    const int64_t chunks = ((tiles_x + DP_CHUNK - 1) / DP_CHUNK) * ((tiles_y + DP_CHUNK - 1) / DP_CHUNK);
    return dim3((unsigned)(((chunks + 7) / 8) * 8 * DP_CHUNK * DP_CHUNK));
}

hipError_t launch_double_prune(const bf16_t* vals, const uint8_t* meta, int64_t d_out, int64_t d_in, bf16_t* valsT,
                               uint8_t* metaT, uint8_t* maskrc, hipStream_t s) {
    const int64_t tiles_x = (d_in + DP_TILE - 1) / DP_TILE, tiles_y = (d_out + DP_TILE - 1) / DP_TILE;
    const dim3 grid = double_prune_grid(tiles_x, tiles_y);
    if (d_in > DP_EXTENT_MAX || d_out > DP_EXTENT_MAX) return hipErrorInvalidValue;
    const bool ragged = d_out % 32 != 0;
    if (ragged && maskrc)
        double_prune_kernel<false, true, true><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                          metaT, maskrc, nullptr, (int)tiles_x, (int)tiles_y);
    else if (ragged)
        double_prune_kernel<false, false, true><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                           metaT, nullptr, nullptr, (int)tiles_x, (int)tiles_y);
    else if (maskrc)
        double_prune_kernel<false, true, false><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                           metaT, maskrc, nullptr, (int)tiles_x, (int)tiles_y);
    else
        double_prune_kernel<false, false, false><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                            metaT, nullptr, nullptr, (int)tiles_x, (int)tiles_y);
    return hipGetLastError();
}

// Values of packed (W^{R,C})^T from new packed values of W^R, metadata of both unchanged.
hipError_t launch_update_transposed(const bf16_t* vals, const uint8_t* meta, int64_t d_out, int64_t d_in,
                                    const uint8_t* metaT, bf16_t* valsT, hipStream_t s) {
    const int64_t tiles_x = (d_in + DP_TILE - 1) / DP_TILE, tiles_y = (d_out + DP_TILE - 1) / DP_TILE;
    const dim3 grid = double_prune_grid(tiles_x, tiles_y);
    if (d_in > DP_EXTENT_MAX || d_out > DP_EXTENT_MAX) return hipErrorInvalidValue;
    if (d_in % 16 != 0 || d_out % 64 != 0)
        double_prune_kernel<true, false, true><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                          nullptr, nullptr, metaT, (int)tiles_x, (int)tiles_y);
    else
        double_prune_kernel<true, false, false><<<grid, dim3(DP_THREADS), 0, s>>>(vals, meta, (int)d_out, (int)d_in, valsT,
                                                                           nullptr, nullptr, metaT, (int)tiles_x, (int)tiles_y);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// out = beta * a + gamma * b on packed values (App. K, sparse matrix addition): one fp32 fused
// multiply-add per element on top of the fp32 product gamma * b, rounded to bf16 (nearest even).
// A plain stream: 16 bytes of each operand per lane, 6 bytes of traffic per element.
constexpr int SA_UNROLL = 2;       // vectors per lane; a workgroup takes SA_UNROLL x 256 consecutive ones (see prune_rows_kernel)

__device__ __forceinline__ uint32_t sparse_add_pair(uint32_t wa, uint32_t wb, float beta, float gamma) {
    float a0 = __uint_as_float(wa << 16), a1 = __uint_as_float(wa & 0xFFFF0000u);
    float b0 = __uint_as_float(wb << 16), b1 = __uint_as_float(wb & 0xFFFF0000u);
    union { __bf16 h[2]; uint32_t x; } o;
    o.h[0] = (__bf16)__builtin_fmaf(beta, a0, gamma * b0);
    o.h[1] = (__bf16)__builtin_fmaf(beta, a1, gamma * b1);
    return o.x;
}

// tail4: four more elements follow the nvec whole vectors of eight (a layer whose rows x cols / 2 is odd in eights)
__global__ void __launch_bounds__(256) sparse_add_kernel(const u32x4* __restrict__ a, const u32x4* __restrict__ b,
                                                         size_t nvec, bool tail4, float beta, float gamma,
                                                         u32x4* __restrict__ out) {
    if (tail4 && blockIdx.x == 0 && threadIdx.x == 0) {
        const u32x2 ta = *(const u32x2*)(a + nvec), tb = *(const u32x2*)(b + nvec);
        *(u32x2*)(out + nvec) = (u32x2){sparse_add_pair(ta[0], tb[0], beta, gamma), sparse_add_pair(ta[1], tb[1], beta, gamma)};
    }
    const size_t first = (size_t)blockIdx.x * (256 * SA_UNROLL) + threadIdx.x;
    u32x4 va[SA_UNROLL], vb[SA_UNROLL];
#pragma unroll
    for (int u = 0; u < SA_UNROLL; ++u) {
        size_t i = first + u * 256;
        if (i < nvec) {
            va[u] = __builtin_nontemporal_load(a + i);
            vb[u] = __builtin_nontemporal_load(b + i);
        }
    }
#pragma unroll
    for (int u = 0; u < SA_UNROLL; ++u) {
        size_t i = first + u * 256;
        if (i >= nvec) continue;
        u32x4 r;
#pragma unroll
        for (int w = 0; w < 4; ++w) r[w] = sparse_add_pair(va[u][w], vb[u][w], beta, gamma);
        __builtin_nontemporal_store(r, out + i);
    }
}

hipError_t launch_sparse_add(const bf16_t* a, const bf16_t* b, size_t count, float beta, float gamma, bf16_t* out,
                             hipStream_t s) {
    size_t nvec = count / 8;                                  // count is a multiple of 4
    size_t blocks = (nvec + 256 * SA_UNROLL - 1) / (256 * SA_UNROLL);
    if (blocks > 0x7FFFFFFFu) return hipErrorInvalidValue;   // cannot happen for extents below 2^31
    if (blocks == 0) blocks = 1;
    sparse_add_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const u32x4*)a, (const u32x4*)b, nvec, count % 8 != 0,
                                                                   beta, gamma, (u32x4*)out);
    return hipGetLastError();
}
