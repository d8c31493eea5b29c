// Workgroup -> output tile for the tiled products, in a form the host compiler can build too (a CPU
// test enumerates it and checks that every tile is produced exactly once).
#pragma once

#if defined(__HIPCC__)
#define HBMM_HOST_DEVICE __host__ __device__
#else
#define HBMM_HOST_DEVICE
#endif

namespace hbmm {

constexpr int kMapXcds = 8;           // workgroup i is dispatched to XCD i % 8
constexpr int kMapSuperTiles = 128;   // popcount product: tiles per super-tile (about the workgroups resident on one XCD: 32 CUs x 3..4)

// Workgroups to launch for `tiles` tiles under xcd_map_tile (at most 7 of them get no tile).
HBMM_HOST_DEVICE inline long long xcd_map_blocks(long long tiles)
{
    return (tiles + kMapXcds - 1) / kMapXcds * kMapXcds;
}

// The tile of workgroup `block`, or false when the workgroup has none.
// Every XCD has its own L2.  The tiles are put in one sequence, super-tile after super-tile
// (sup_p x sup_q tiles: bands of sup_q tiles along Q, in a band groups of sup_p tiles along P, ragged
// at the edges, P fastest inside a group), and XCD x takes the x-th eighth of that sequence in order:
// every XCD gets the same number of tiles (+-1) whatever the shape, and its resident workgroups sit in
// one or two super-tiles, so a P tile is fetched into that L2 once for sup_q workgroups and a Q tile
// once for sup_p of them.
HBMM_HOST_DEVICE inline bool xcd_map_tile(int block, int tiles_p, int tiles_q, int sup_p, int sup_q, int &tile_p, int &tile_q)
{
    const int xcd = block % kMapXcds, in_xcd = block / kMapXcds;
    const int tiles = tiles_p * tiles_q;
    const int share = tiles / kMapXcds, extra = tiles % kMapXcds;
    if (in_xcd >= share + (xcd < extra ? 1 : 0)) return false;
    const int i = xcd * share + (xcd < extra ? xcd : extra) + in_xcd;
    const int band_tiles = tiles_p * sup_q;
    const int band = i / band_tiles, in_band = i - band * band_tiles;
    const int left_q = tiles_q - band * sup_q;
    const int band_q = left_q < sup_q ? left_q : sup_q;          // the last band may be narrower
    const int group_tiles = sup_p * band_q;
    const int group = in_band / group_tiles, r = in_band - group * group_tiles;
    const int left_p = tiles_p - group * sup_p;
    const int group_p = left_p < sup_p ? left_p : sup_p;         // the last group may be shorter
    tile_p = group * sup_p + r % group_p;
    tile_q = band * sup_q + r / group_p;
    return true;
}

// The popcount product: super-tiles of sup_p x (128 / sup_p) tiles; sup_p == 0 (small grids) maps
// plainly, P fastest.
HBMM_HOST_DEVICE inline long long popcount_map_blocks(int tiles_p, int tiles_q, int sup_p)
{
    const long long tiles = (long long)tiles_p * tiles_q;
    return sup_p == 0 ? tiles : xcd_map_blocks(tiles);
}
HBMM_HOST_DEVICE inline bool popcount_map_tile(int block, int tiles_p, int tiles_q, int sup_p, int &tile_p, int &tile_q)
{
    if (sup_p == 0) {
        tile_p = block % tiles_p;
        tile_q = block / tiles_p;
        return true;
    }
    return xcd_map_tile(block, tiles_p, tiles_q, sup_p, kMapSuperTiles / sup_p, tile_p, tile_q);
}

}  // namespace hbmm
