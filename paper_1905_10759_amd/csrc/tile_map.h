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
// at the edges, P fastest inside a group).  The sequence is cut into pieces of one super-tile's
// length; in every round the 8 XCDs take 8 consecutive pieces, so that at any time each XCD works
// inside one or two super-tiles (a P tile is fetched into its L2 once for sup_q workgroups and a Q
// tile once for sup_p of them) and the 8 XCDs together work on neighbouring super-tiles (which
// share their Q band: what one XCD has fetched from HBM, the others find in the memory-side cache
// while it is still there).  What is left after the last full round is dealt in 8 equal slices:
// every XCD gets the same number of tiles (+-1) whatever the shape.
HBMM_HOST_DEVICE inline bool xcd_map_tile(int block, int tiles_p, int tiles_q, int sup_p, int sup_q, int &tile_p, int &tile_q)
{
    const int xcd = block % kMapXcds, in_xcd = block / kMapXcds;
    const int tiles = tiles_p * tiles_q;
    const int piece = sup_p * sup_q, round = piece * kMapXcds;
    const int full = tiles / round;                              // rounds in which every XCD takes a whole piece
    int i;
    if (in_xcd < full * piece) {
        i = (in_xcd / piece) * round + xcd * piece + in_xcd % piece;
    } else {
        const int left = tiles - full * round, j = in_xcd - full * piece;
        const int share = left / kMapXcds, extra = left % kMapXcds;
        if (j >= share + (xcd < extra ? 1 : 0)) return false;
        i = full * round + xcd * share + (xcd < extra ? xcd : extra) + j;
    }
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
