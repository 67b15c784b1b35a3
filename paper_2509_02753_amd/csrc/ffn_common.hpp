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

__device__ __forceinline__ bool fetch_tile(const int32_t* sched, const int32_t* sched_count, int tile, int M,
                                           int tile_tokens, TileInfo& ti) {
    if (sched != nullptr) {
        if (tile >= sched_count[0]) return false;
        const int32_t* s = sched + (size_t)tile * 4;
        ti.expert = s[0];
        ti.row0 = s[1];
        ti.rows = s[2];
        return true;
    }
    ti.expert = 0;
    ti.row0 = tile * tile_tokens;
    ti.rows = min(tile_tokens, M - ti.row0);
    return ti.rows > 0;
}


hipError_t launch_gateup_stream(const FfnArgs& a, hipStream_t s);
hipError_t launch_down_stream(const FfnArgs& a, hipStream_t s);

}  // namespace lexi
