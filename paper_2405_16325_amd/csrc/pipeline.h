// Building blocks shared by the MFMA kernels: tile order, global -> LDS loads, barriers.
#pragma once
#include <atomic>

#include "common.h"

// Dynamic LDS beyond the default limit has to be enabled per kernel; once per device is enough, and the
// call is not free (it is what made 20 us launches of small layers measurably slower).
template <auto Kernel>
inline hipError_t allow_dynamic_lds(int bytes) {
    static std::atomic<uint64_t> done{0};                     // one bit per device
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

constexpr int XCDS = 8;
constexpr int RESIDENT = 256;             // tiles in flight on the chip: one per compute unit
constexpr size_t LAST_LEVEL_CACHE_BYTES = (size_t)256 << 20;   // the memory-side cache in front of HBM
// s_waitcnt immediate (gfx9 encoding): vmcnt <= vm, lgkmcnt <= lgkm, expcnt unconstrained.
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | ((vm >> 4) << 14) | (7 << 4) | (lgkm << 8); }

// blockIdx -> tile.  Workgroups are dealt round-robin to the 8 XCDs, 32 resident per XCD.
//  * A grid of at least 8 x 4 tiles that fills the chip: the tiles are put in an order without gaps, and the 32
//    tiles an XCD holds at a time are 32 consecutive positions of it (group g of 32 goes to XCD
//    g % 8), so every XCD gets the same number of tiles, give or take one group, whatever the
//    grid's shape.  The order: first the part of the grid that whole chunks of 8 x 4 tiles cover
//    (a chunk's tiles share 8 + 4 operand panels in the XCD's L2), chunk after chunk, numbered so
//    that eight consecutive chunks form a 16 x 16 patch (2 x 4 chunks; the chip then shares 16 + 16
//    panels in the last-level cache), patch after patch along n, then along m; then the rows that
//    are left below it, column by column (32 positions: their few rows of 8 or more columns); then
//    the columns left beside it, row by row.  What is left of the order after the last whole round of 256 is dealt
//    out in eight equal runs.
//  * A narrow grid (skinny products, inference-size batches): tiles are numbered short axis first
//    and each XCD takes runs of consecutive tiles: at most 32, sized so that all 8 XCDs get equal
//    shares in every round, also when there are fewer than 256 tiles.
constexpr int CHUNK_M = 8, CHUNK_N = 4;

__host__ __device__ inline int narrow_run(int tiles) {
    int rounds = (tiles + RESIDENT - 1) / RESIDENT;        // even shares in every round, the last included
    return (tiles + XCDS * rounds - 1) / (XCDS * rounds);
}

// a grid has the chunked order if it holds at least one whole chunk and fills the chip at least once
__host__ __device__ inline bool wide_grid(int tiles_m, int tiles_n) {
    return tiles_m >= CHUNK_M && tiles_n >= CHUNK_N && (int64_t)tiles_m * tiles_n >= RESIDENT;
}
// the tile belongs to a whole 8 x 4 chunk of a wide grid: then the 32 tiles its XCD holds with it are that chunk
__host__ __device__ inline bool in_whole_chunk(int tm, int tn, int tiles_m, int tiles_n) {
    return wide_grid(tiles_m, tiles_n) && tm < tiles_m / CHUNK_M * CHUNK_M && tn < tiles_n / CHUNK_N * CHUNK_N;
}

// position q (0 <= q < tiles_m * tiles_n) in the order of a wide grid -> tile
__host__ __device__ inline void tile_of_position(int q, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int m8 = tiles_m / CHUNK_M * CHUNK_M, n4 = tiles_n / CHUNK_N * CHUNK_N;
    if (q < m8 * n4) {
        const int c = q / 32, w = q % 32;
        const int chunks_m = m8 / CHUNK_M, chunks_n = n4 / CHUNK_N;
        int sm = c / (2 * chunks_n), rem = c - sm * 2 * chunks_n;   // patch row: 2 chunk rows (1 in a ragged last)
        int hm = chunks_m - 2 * sm < 2 ? 1 : 2;
        int sn = rem / (4 * hm), r2 = rem - sn * 4 * hm;            // patch: 4 chunk columns (fewer at the edge)
        int wn = chunks_n - 4 * sn < 4 ? chunks_n - 4 * sn : 4;
        tm = (2 * sm + r2 / wn) * CHUNK_M + (w & 7);
        tn = (4 * sn + r2 % wn) * CHUNK_N + (w >> 3);
        return;
    }
    q -= m8 * n4;
    const int below = tiles_m - m8;
    if (q < below * tiles_n) { tn = q / below; tm = m8 + q % below; return; }
    q -= below * tiles_n;
    const int beside = tiles_n - n4;
    tm = q / beside;
    tn = n4 + q % beside;
}

// workgroup b of a launch over a wide grid -> its position in the order (XCD b % 8, 32 positions at a time)
__host__ __device__ inline int position_of_block(int b) {
    const int xcd = b % XCDS, slot = b / XCDS;
    return ((slot / 32) * XCDS + xcd) * 32 + slot % 32;
}

__host__ __device__ inline bool tile_of_index(int b, int tiles_m, int tiles_n, int& tm, int& tn) {
    int xcd = b % XCDS, slot = b / XCDS;
    if (wide_grid(tiles_m, tiles_n)) {
        // whole rounds of 256: 32 consecutive positions per XCD; the tiles left for a last, partial round are
        // dealt out in equal runs, so that all 8 XCDs (their L2s, their links to memory) share them
        const int tiles = tiles_m * tiles_n, whole = tiles / RESIDENT * RESIDENT;
        int q;
        if (b < whole) {
            q = position_of_block(b);
        } else {
            const int run = (tiles - whole + XCDS - 1) / XCDS;
            slot -= whole / XCDS;
            q = whole + xcd * run + slot;
            if (slot >= run || q >= tiles) return false;
        }
        tile_of_position(q, tiles_m, tiles_n, tm, tn);
        return true;
    }
    int run = narrow_run(tiles_m * tiles_n);
    int t = ((slot / run) * XCDS + xcd) * run + slot % run;
    if (tiles_m <= tiles_n) { tm = t % tiles_m; tn = t / tiles_m; }
    else { tn = t % tiles_n; tm = t / tiles_n; }
    return tm < tiles_m && tn < tiles_n;
}

__device__ __forceinline__ bool tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
    return tile_of_index((int)blockIdx.x, tiles_m, tiles_n, tm, tn);
}

inline int super_grid(int tiles_m, int tiles_n) {
    int tiles = tiles_m * tiles_n;
    if (wide_grid(tiles_m, tiles_n)) {
        const int whole = tiles / RESIDENT * RESIDENT;
        return whole + (tiles - whole + XCDS - 1) / XCDS * XCDS;
    }
    int chunk = XCDS * narrow_run(tiles);
    return (tiles + chunk - 1) / chunk * chunk;
}

// Row that a loader lane reads for tile row `row` of an operand with `rows` rows.  Rows past the
// end only feed accumulators that are never stored, so any valid row will do; they are spread over
// the operand (row % rows) rather than clamped to the last row, which would make that one row's
// lines a hot spot of the L2 channel they live in (a ragged token tile ran 25 % slower that way).
__device__ __forceinline__ int wrap_row(int row, int rows) { return row < rows ? row : row % rows; }

// 64 lanes x 16 bytes: lane l's bytes land at lds_dst + 16 * l; lds_dst is wave-uniform
__device__ __forceinline__ void dma16(const void* gsrc, uint8_t* lds_dst) {
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gsrc,
                                     (void __attribute__((address_space(3)))*)lds_dst, 16, 0, 0);
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for every
// outstanding global -> LDS load (vmcnt(0)), which is exactly what the load rings are there to
// avoid.  Visibility of those loads is handled by explicit s_waitcnt vmcnt(n) before the barrier;
// nothing is scheduled across it, so the two phases of a k-step stay phases.
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// s_waitcnt that stays where it is written: without the fences the scheduler is free to sink the
// MFMAs of a compute phase below the wait that ends it.
#define WAIT_HERE(imm)                          \
    do {                                        \
        __builtin_amdgcn_sched_barrier(0);      \
        __builtin_amdgcn_s_waitcnt(imm);        \
        __builtin_amdgcn_sched_barrier(0);      \
    } while (0)

union BFrag { u32x4 u[2]; bf16x16 v; };
union AFrag { u32x4 u; bf16x8 v; };
