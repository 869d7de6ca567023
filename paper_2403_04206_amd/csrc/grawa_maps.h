// Host-side index maps of a GRAWA plan: how the flat parameter vector is cut into tiles (norm
// pass, scored local step) and 256-column cells (center+pull pass).  Plain C++ with no GPU
// dependency, so that it can be built and run under the host sanitizers on its own.
#ifndef GRAWA_MAPS_H
#define GRAWA_MAPS_H

#include <stddef.h>
#include <stdint.h>

#include <vector>

// One tile of the flat vector.  A tile never crosses a layer boundary, so its sum of squares
// belongs to one layer.  16 bytes: fetched with one scalar load.
struct GrawaTile {
    int64_t start; // first element (index into a row)
    int32_t len;   // 1 .. tile length
    int32_t layer; // layer the tile lies in
};

#define GRAWA_ROW_TILE 1024 // columns per tile of the scored local step
#define GRAWA_CELL_COLS 256 // columns per cell of the center+pull pass
#define GRAWA_MAX_TILES ((int64_t)1 << 24) // keeps grid.x * 256 below 2^32

struct GrawaHostMaps {
    std::vector<GrawaTile> tiles;       // norm pass: layers cut at the multiples of tile_elems
    std::vector<int32_t> layer_tile0;   // [L+1] first tile of every layer
    std::vector<GrawaTile> rtiles;      // scored local step: layers cut at the multiples of 1024
    std::vector<int32_t> layer_rtile0;  // [L+1]
    std::vector<int32_t> block_rtile0;  // [ceil(P/1024)+1] first short tile of every aligned block of 1024 columns
    std::vector<int32_t> cell_layer;    // [ceil(P/256)] layer of a cell, or ~(first layer) if it holds a boundary
};

// Norm-pass tile length for a problem: as long as possible while leaving ~8192 blocks.
int grawa_default_tile_elems(int K, int64_t P);

// 0: offsets are valid (off[0] = 0, strictly increasing, off[L] = P, 1 <= L <= P); 1 otherwise.
int grawa_offsets_invalid(int64_t P, int L, const int64_t *off);

// Fills `m` for valid offsets.  Returns 0, or 1 when the problem needs more than
// GRAWA_MAX_TILES tiles or cells (nothing useful is left in `m` then).
int grawa_build_maps(int64_t P, int L, const int64_t *off, int tile_elems, GrawaHostMaps &m);

#endif
