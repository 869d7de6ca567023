// Construction of the plan's index maps (see grawa_maps.h).  Host code only.
#include "grawa_maps.h"

// As long as possible (fewer partials, less per-block overhead) while leaving at least ~8192
// blocks to fill the chip; 2048 is the shortest tile that gives every lane of a block one
// 16-byte load of bf16.
int grawa_default_tile_elems(int K, int64_t P)
{
    const int64_t per_block = (int64_t)K * P / 8192;
    int t = 16384;
    while (t > 2048 && t > per_block) t >>= 1;
    return t;
}

int grawa_offsets_invalid(int64_t P, int L, const int64_t *off)
{
    if (!off || L < 1 || P < 1 || (int64_t)L > P) return 1;
    if (off[0] != 0 || off[L] != P) return 1;
    for (int l = 0; l < L; ++l)
        if (off[l + 1] <= off[l]) return 1;
    return 0;
}

// Cut every layer at the multiples of `len` of the flat index: tile starts are either a
// multiple of `len` or a layer start, and no tile crosses a layer boundary.
static void cut_layers(int64_t P, int L, const int64_t *off, int len, std::vector<GrawaTile> &out,
                       std::vector<int32_t> &first)
{
    out.clear();
    out.reserve((size_t)(P / len + L + 1));
    first.assign((size_t)L + 1, 0);
    for (int l = 0; l < L; ++l) {
        first[(size_t)l] = (int32_t)out.size();
        int64_t s = off[l];
        const int64_t e = off[l + 1];
        while (s < e) {
            int64_t stop = (s / len + 1) * len;
            if (stop > e) stop = e;
            out.push_back(GrawaTile{s, (int32_t)(stop - s), (int32_t)l});
            s = stop;
        }
    }
    first[(size_t)L] = (int32_t)out.size();
}

int grawa_build_maps(int64_t P, int L, const int64_t *off, int tile_elems, GrawaHostMaps &m)
{
    const int TR = GRAWA_ROW_TILE;
    if (P / tile_elems + L > GRAWA_MAX_TILES || P / TR + L > GRAWA_MAX_TILES) return 1;
    const int64_t cell = GRAWA_CELL_COLS;
    const int64_t nc = (P + cell - 1) / cell;
    if (nc >= GRAWA_MAX_TILES) return 1;

    cut_layers(P, L, off, tile_elems, m.tiles, m.layer_tile0);
    cut_layers(P, L, off, TR, m.rtiles, m.layer_rtile0);

    // Short tiles never cross a multiple of TR: index them by aligned block.
    const int64_t nrt = (int64_t)m.rtiles.size();
    const int64_t nrb = (P + TR - 1) / TR;
    m.block_rtile0.assign((size_t)nrb + 1, 0);
    int64_t r = 0;
    for (int64_t b = 0; b < nrb; ++b) {
        m.block_rtile0[(size_t)b] = (int32_t)r;
        while (r < nrt && m.rtiles[(size_t)r].start < (b + 1) * TR) ++r;
    }
    m.block_rtile0[(size_t)nrb] = (int32_t)nrt;

    // Cell c covers columns [256 c, 256 c + 256).
    m.cell_layer.assign((size_t)nc, 0);
    int l = 0;
    for (int64_t c = 0; c < nc; ++c) {
        const int64_t first = c * cell;
        const int64_t last = (first + cell < P ? first + cell : P) - 1;
        while (off[l + 1] <= first) ++l;
        m.cell_layer[(size_t)c] = (off[l + 1] > last) ? (int32_t)l : ~(int32_t)l;
    }
    return 0;
}
