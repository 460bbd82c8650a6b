// Tile kernel (16 chains per workgroup, MFMA gradient) - interface used by the host API.
#pragma once
#include <vector>

#include "nuts_dev.h"

namespace nuts {

constexpr int kTileMaxDim = 32;
constexpr int kTileMaxDepth = 12;

struct TileData {
    double* base = nullptr;  // device: packed operands
};

struct TileLaunch {
    int blocks = 0;
    size_t block_bytes = 0, workspace_bytes = 0;
};

inline bool tile_supports_shape(int64_t) { return false; }
inline void tile_pack_operands(const double*, const double*, int64_t, int64_t, TileData*, std::vector<double>*) {}
inline void tile_plan(const TileData&, long, int, TileLaunch*) {}
inline void tile_launch(const TileData&, const DevSample&, double, const TileLaunch&, hipStream_t) {}

}  // namespace nuts
