// Builds the plan's host-side index maps (paper_2403_04206_amd/csrc/grawa_maps.cpp, compiled into
// this program with -fsanitize=address,undefined and no GPU toolchain) for layer offsets read from a
// file and checks what the kernels rely on:
//   * the tiles of a layer cover it exactly, in order, without gaps; no tile crosses a layer boundary or a
//     multiple of the tile length; 1 <= len <= tile length; layer_tile0 brackets each layer's tiles;
//   * the short (1024-column) tiles likewise, and block_rtile0[b] .. block_rtile0[b+1] are exactly the
//     short tiles inside aligned block b;
//   * cell_layer[c] is the layer of a cell that lies in one layer, or the complement of the layer of its
//     first column when the cell holds a boundary.
// Input file: int64 P, L, tile_elems (0 = the library's choice for K), K ; int64 off[L+1].
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "grawa_maps.h"

static void die(const char *what, long long a = 0, long long b = 0)
{
    std::fprintf(stderr, "maps_sanitizer_driver: %s (%lld, %lld)\n", what, a, b);
    std::exit(2);
}

static void check_cut(const std::vector<GrawaTile> &tiles, const std::vector<int32_t> &first, int64_t P, int L,
                      const int64_t *off, int len)
{
    if ((int)first.size() != L + 1 || first[0] != 0 || first[(size_t)L] != (int32_t)tiles.size()) die("first[] ends");
    for (int l = 0; l < L; ++l) {
        int64_t at = off[l];
        if (first[(size_t)l + 1] <= first[(size_t)l]) die("layer without tiles", l);
        for (int32_t t = first[(size_t)l]; t < first[(size_t)l + 1]; ++t) {
            const GrawaTile &q = tiles[(size_t)t];
            if (q.layer != l) die("tile in the wrong layer", t, l);
            if (q.start != at) die("gap or overlap", t, at);
            if (q.len < 1 || q.len > len) die("tile length", t, q.len);
            if (q.start / len != (q.start + q.len - 1) / len) die("tile crosses a multiple of its length", t);
            at += q.len;
        }
        if (at != off[l + 1]) die("layer not covered", l, at);
    }
    if (off[L] != P) die("offsets");
}

int main(int argc, char **argv)
{
    if (argc != 2) die("usage: driver <input>");
    std::FILE *in = std::fopen(argv[1], "rb");
    if (!in) die("cannot open input");
    int64_t h[4];
    if (std::fread(h, sizeof h, 1, in) != 1) die("short header");
    const int64_t P = h[0];
    const int L = (int)h[1];
    std::vector<int64_t> off((size_t)L + 1);
    if (std::fread(off.data(), sizeof(int64_t), off.size(), in) != off.size()) die("short offsets");
    std::fclose(in);
    if (grawa_offsets_invalid(P, L, off.data())) {
        std::puts("invalid offsets");
        return 3;
    }
    const int T = h[2] ? (int)h[2] : grawa_default_tile_elems((int)h[3], P);
    if (T < 2048 || T > 16384 || (T & (T - 1))) die("tile length", T);
    GrawaHostMaps m;
    if (grawa_build_maps(P, L, off.data(), T, m)) {
        std::puts("too many tiles");
        return 4;
    }
    check_cut(m.tiles, m.layer_tile0, P, L, off.data(), T);
    check_cut(m.rtiles, m.layer_rtile0, P, L, off.data(), GRAWA_ROW_TILE);

    const int64_t nrb = (P + GRAWA_ROW_TILE - 1) / GRAWA_ROW_TILE;
    if ((int64_t)m.block_rtile0.size() != nrb + 1 || m.block_rtile0[0] != 0 ||
        m.block_rtile0[(size_t)nrb] != (int32_t)m.rtiles.size())
        die("block_rtile0 ends");
    for (int64_t b = 0; b < nrb; ++b) {
        if (m.block_rtile0[(size_t)b + 1] <= m.block_rtile0[(size_t)b]) die("block without tiles", b);
        for (int32_t t = m.block_rtile0[(size_t)b]; t < m.block_rtile0[(size_t)b + 1]; ++t)
            if (m.rtiles[(size_t)t].start / GRAWA_ROW_TILE != b) die("short tile in the wrong block", t, b);
    }

    const int64_t nc = (P + GRAWA_CELL_COLS - 1) / GRAWA_CELL_COLS;
    if ((int64_t)m.cell_layer.size() != nc) die("cell count");
    int l = 0;
    for (int64_t c = 0; c < nc; ++c) {
        const int64_t first = c * GRAWA_CELL_COLS, last = (first + GRAWA_CELL_COLS < P ? first + GRAWA_CELL_COLS : P) - 1;
        while (off[(size_t)l + 1] <= first) ++l;                 // layer of the first column
        int le = l;
        while (off[(size_t)le + 1] <= last) ++le;                // layer of the last column
        const int32_t want = (le == l) ? (int32_t)l : ~(int32_t)l;
        if (m.cell_layer[(size_t)c] != want) die("cell layer", c, m.cell_layer[(size_t)c]);
    }
    std::printf("ok tiles=%zu rtiles=%zu cells=%zu T=%d\n", m.tiles.size(), m.rtiles.size(), m.cell_layer.size(), T);
    return 0;
}
