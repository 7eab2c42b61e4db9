// Internal layout tables of the MG-WFBP library (not part of the C ABI).
//
// Arena picture (Sec. 5.3: one pre-allocated contiguous buffer per group, members dense, in the
// order their gradients arrive):
//
//   arena:  | group 0 .......... pad | group 1 .... pad | group 2 ...
//           ^ tile 0   ^ tile 1 ...   ^ first tile of group 1 (group bases are tile-aligned)
//   group:  | tensor hi | tensor hi-1 | ... | tensor lo |        <- "segments", zero-element
//                                                                   tensors have no segment
// A tile is MGWFBP_TILE_ELEMS consecutive arena elements and is processed by one workgroup.
// Each tile carries a header that tells the workgroup which segments it intersects.
#ifndef MGWFBP_TABLES_H
#define MGWFBP_TABLES_H

#include <cstdint>
#include <vector>

#ifndef MGWFBP_TILE_VECS
#define MGWFBP_TILE_VECS 1          // 16-byte vectors per lane per tile
#endif
#ifndef MGWFBP_BLOCK
#define MGWFBP_BLOCK 64             // lanes per workgroup (a multiple of 64): one wavefront per tile
#endif
#define MGWFBP_VEC 4                // elements per lane-vector
#define MGWFBP_TILE_ELEMS (MGWFBP_BLOCK * MGWFBP_VEC * MGWFBP_TILE_VECS)
#define MGWFBP_MAX_P 64

struct TileHdr {          // 32 bytes, read with two 16-byte loads
    int64_t first_start;  // (arena start of segment seg0) - (arena start of the tile); <= 0
    int32_t first_end;    // tile-local end of segment seg0, clipped to `valid`
    int32_t seg0;         // first segment that intersects the tile
    int32_t nseg;         // segments that intersect the tile, >= 1
    int32_t valid;        // leading elements of the tile that belong to the group, 1..TILE
    int32_t layer0;       // tensor index of segment seg0
    int32_t flags;        // bit 0: weights and momenta of this tile are kept cacheable (see kernels.hip)
};
static_assert(sizeof(TileHdr) == 32, "TileHdr must stay 32 bytes");

struct HostTables {
    int32_t L = 0, G = 0;
    uint64_t arena_elems = 0;
    // per tensor
    std::vector<uint64_t> tensor_off;     // [L] element offset inside the group's slice
    std::vector<int32_t> tensor_group;    // [L]
    std::vector<uint64_t> tensor_n;       // [L] element count
    // per group (arrival order)
    std::vector<uint64_t> group_base;     // [G] arena element
    std::vector<uint64_t> group_elems;    // [G]
    std::vector<int32_t> group_tile;      // [G+1] first tile of each group
    // per segment (arena order)
    std::vector<uint64_t> seg_off;        // [S+1] arena element of the segment start; seg_off[S] = arena_elems
    std::vector<uint32_t> seg_n;          // [S] elements, saturated at 2^32-1
    std::vector<int32_t> seg_layer;       // [S] tensor index
    // per tile
    std::vector<TileHdr> tiles;           // [T]
};

// Records a failed HIP call for mgwfbp_last_hip_error() on this thread and returns MGWFBP_EHIP; returns
// MGWFBP_OK for code 0 (hipSuccess).  Defined next to the device entry points.
int mgwfbp_note_hip_result(int hip_error_code);

// Returns 0 or a negative mgwfbp_status.  Pure host code.
int mgwfbp_build_tables(const uint64_t* n_elems, int32_t L, const uint8_t* merged, HostTables& out);

#endif
