// Pieces shared by the expert-FFN translation units: K-stage size, the packed weight layout, the tile schedule.
#pragma once
#include "kernels.hpp"

namespace lexi {

constexpr int BK = 64;         // K elements per LDS stage
constexpr int LDS_PAD = 8;     // bf16 elements of padding per LDS row (16 B): spreads the 16-byte operand reads over banks
constexpr int LDS_LD = BK + LDS_PAD;

// Expert weight matrices W[R][K] (R output features, K inputs) are stored in the MFMA-native "packed" layout:
// the matrix is cut into blocks of 16 rows x 32 K elements; a block is 64 runs of 8 consecutive K elements, run
// (q, i) = (K-octet q of the block, row i of the block) at position q*16 + i; blocks follow each other along K, then
// along R.  A wave-wide 16-byte-per-lane load of one block is therefore 1 KB of contiguous memory and is, as it
// stands, the A operand of v_mfma_f32_16x16x32_bf16 (lane = q*16 + i).
__host__ __device__ __forceinline__ size_t packed_index(int r, int k, int K) {
    return ((((size_t)(r >> 4) * (K >> 5) + (k >> 5)) * 64 + ((k & 31) >> 3) * 16 + (r & 15)) << 3) + (k & 7);
}

struct TileInfo {
    int expert, row0, rows;
};

// Tile schedule written by the scan kernel: one entry of kSchedStride ints per token tile,
//   (expert, first permuted row of the expert, rows of the expert, index of the tile inside its expert, tiles of the
//   expert, 0, 0, 0),
// tiles sorted by expert; sched_count[0] = number of tiles.  Every entry carries its expert's whole extent, so any tile
// of the expert can be derived from any of its entries with one load.  sched == null: one dense group of M rows.
constexpr int kSchedStride = 8;

__device__ __forceinline__ bool fetch_tile(const int32_t* sched, const int32_t* sched_count, int tile, int M,
                                           int tile_tokens, TileInfo& ti) {
    if (sched != nullptr) {
        if (tile >= sched_count[0]) return false;
        const int32_t* s = sched + (size_t)tile * kSchedStride;
        ti.expert = s[0];
        ti.row0 = s[1] + s[3] * tile_tokens;
        ti.rows = min(tile_tokens, s[2] - s[3] * tile_tokens);
        return true;
    }
    ti.expert = 0;
    ti.row0 = tile * tile_tokens;
    ti.rows = min(tile_tokens, M - ti.row0);
    return ti.rows > 0;
}

// XCD-aware work order for the tile kernels.  Workgroup ids are handed to the 8 XCDs round-robin (id % 8), each XCD
// with its own L2, and a CU holds two workgroups, so 64 consecutive work items of an XCD are resident together.
// Work items are (token tile, column block).  They are ordered expert by expert; inside an expert by groups of
// kCbGroup column blocks; inside a group tile-major.  A window of 64 items then holds few distinct weight slabs,
// each read by ALL token tiles of its expert at the same time, whatever the number of column blocks is (sharing the
// weight stream is what pays: groups of 1 or 2 column blocks measured 10 to 40 % faster than groups of 8 or more,
// which favour sharing the much smaller token tile).  The item list is cut into 8 contiguous parts, XCD x takes
// the x-th.
// The grid is 1-D: 8 * ceil(ncb * max_tiles / 8) workgroups.
constexpr int kXcds = 8;
constexpr int kCbGroup = 2;
inline unsigned xcd_grid(int ncb, int max_tiles, int ksplit = 1) {
    const long long total = (long long)ncb * max_tiles * ksplit;
    return (unsigned)(((total + kXcds - 1) / kXcds) * kXcds);
}

// With ksplit > 1 every item appears ksplit times in a row, once per part of the reduction dimension.
__device__ __forceinline__ bool fetch_item(const int32_t* sched, const int32_t* sched_count, int ncb, int M,
                                           int tile_tokens, TileInfo& ti, int& cb, int ksplit = 1, int* part = nullptr) {
    const int ntiles = sched != nullptr ? sched_count[0] : (M + tile_tokens - 1) / tile_tokens;
    const int total = ntiles * ncb;
    const int pieces = total * ksplit;
    const int per = (pieces + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int piece = xcd * per + slot;
    if (slot >= per || piece >= pieces) return false;
    const int item = piece / ksplit;
    if (part != nullptr) *part = piece - item * ksplit;
    // an expert with n tiles owns n * ncb consecutive items, so tile (item / ncb) belongs to the item's expert
    int first = 0, n = ntiles, erow0 = 0, erows = M;
    ti.expert = 0;
    if (sched != nullptr) {
        const int tq = item / ncb;
        const int32_t* s = sched + (size_t)tq * kSchedStride;
        ti.expert = s[0];
        erow0 = s[1];
        erows = s[2];
        first = tq - s[3];
        n = s[4];
    }
    const int j = item - first * ncb;
    const int gsz = n * kCbGroup;
    const int g = j / gsz, r = j - g * gsz;
    const int gw = min(kCbGroup, ncb - g * kCbGroup);   // the last group of an expert may be narrower
    const int t = r / gw;
    cb = g * kCbGroup + (r - t * gw);
    ti.row0 = erow0 + t * tile_tokens;
    ti.rows = min(tile_tokens, erows - t * tile_tokens);
    return true;
}

hipError_t launch_gateup_stream(const FfnArgs& a, hipStream_t s);
hipError_t launch_down_stream(const FfnArgs& a, hipStream_t s);

}  // namespace lexi
