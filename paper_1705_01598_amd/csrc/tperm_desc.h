// Kernel descriptors: plain structs filled by the host planner and passed BY VALUE as
// kernel arguments (no device allocation, no host-to-device copy at plan time), plus the
// index arithmetic that both the kernels and the host-side self check evaluate.
//
// Notation follows Section 2 of the paper: a tile is the sub-volume M_mk staged through
// LDS; the remaining dimensions (M-bar_mk, here together with the chunk counters of split
// dimensions) are enumerated by the tile index b; "major" offsets depend on b only
// (Eqs. (2),(3)), "minor" offsets on the position k inside the tile (Eqs. (4)-(6)).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__) || defined(__HIP__)
#define TPERM_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define TPERM_HD inline
#endif

#define TPERM_DESC_MAX_DIMS 16   // canonical rank limit = lanes of one DPP row
#define TPERM_MAX_THREADS 256    // largest workgroup of the tile kernels (4 wavefronts)
#define TPERM_NO_REM 0xFFFFu     // "no split on this side": every real coordinate is below it
// Tensors of 4 GiB and more: bytes one buffer description covers, counted from a tile's origin
// (every position inside a tile must lie below it); also the lane offset of a masked slot.
#define TPERM_BIG_RANGE 0xFFFFFF00u

namespace tperm {

// Division of a 31-bit unsigned n by a constant d >= 1 as multiply + shift:
// with l = ceil(log2 d), magic = ceil(2^(31+l) / d) < 2^32 and
// floor(n / d) = (n * magic) >> (31 + l) for every n < 2^31 (Granlund-Montgomery).
struct FastDiv {
    uint32_t magic;
    uint32_t shift;
};

TPERM_HD uint32_t fdiv(uint32_t n, FastDiv f) {
    return (uint32_t)(((uint64_t)n * (uint64_t)f.magic) >> f.shift);
}

// One dimension of the tile, as seen from one side (input order or output order).
struct TileDim {
    uint32_t ext;      // tile extent t_z (>= 2)
    FastDiv div;       // division by ext
    uint32_t gstride;  // element stride of this dim in global memory on this side
    uint32_t ostride;  // element stride of this dim in global memory on the other side
    uint32_t lstride;  // element stride of this dim in the LDS image of the tile
    uint32_t sel;      // 0: whole dim is in the tile; 1: split dim A; 2: split dim B
    uint32_t xshift;   // 1 if this entry counts pairs of elements (vec2 plans), else 0: the
                       // coordinate compared with the remaining extent is x << xshift
};

// One term of the major-offset sums (Eqs. (2),(3)): lane j of every 16-lane row holds
// term j.  coordinate = (b / cum) % ext.
struct MajorDims {
    FastDiv cum[TPERM_DESC_MAX_DIMS];   // division by the cumulative volume c_j
    FastDiv ext_div[TPERM_DESC_MAX_DIMS];
    uint32_t ext[TPERM_DESC_MAX_DIMS];
    uint32_t stride_in[TPERM_DESC_MAX_DIMS];   // elements
    uint32_t stride_out[TPERM_DESC_MAX_DIMS];  // elements
};

// A major dimension whose counter is split into a low part of `width` values (placed early
// in the tile order, so that tiles running at the same time are neighbours along that
// dimension) and a high part: counter = c[lane_lo] + width * c[lane_hi].  Combinations with
// counter >= count do not exist and are skipped.  count == 0: pair unused.
struct SplitPair {
    uint32_t lane_lo, lane_hi, width, count;
};

// Line-aligned output windows.  When the rows of the output are not aligned to 128-byte lines,
// a tile that writes the same index range [c t, (c+1) t) of the output's leading dimension in
// every row starts and ends each row piece inside a line, and partially written lines are what
// the memory system handles worst.  In this mode every row writes the window
// [c t - s, (c+1) t - s) instead, with s in [0, line_elems) chosen per row so that the window
// starts on a line boundary; t is a multiple of line_elems, so it ends on one too, and the
// windows of consecutive chunks still tile the row.  The data for the shifted windows comes
// from a halo: on the read side the tile covers line_elems extra coordinates in front,
// [c t - line_elems, (c+1) t), which the neighbouring tile reads as well (from cache, mostly).
// That dimension is always split dim B here; its tile coordinate x stands for the output
// coordinate c t - line_elems + x, valid when lo <= x < remaining (see tile_remaining).
struct OutAlign {
    uint32_t enabled;
    uint32_t line_elems;     // elements per 128-byte line (the halo width)
    uint32_t total_slots;    // write-side slots of a tile: rows * t
    uint32_t lstride_b;      // LDS stride of the shifted dimension
    uint32_t in_halo_elems;  // input elements between the tensor base and the halo origin
};

// Descriptor of the generic tile kernel (Tiled, Packed, PackedSplit and the LDS-free
// row-copy all reduce to it).
struct TileDesc {
    uint32_t num_tiles;     // vol(M-bar_mk) times the chunk counts of the split dims
    uint32_t tile_vol;      // vol(M_mk) with split dims at their tile extent
    uint32_t n_tile_dims;
    uint32_t n_major;       // terms in use in `major` (the rest are neutral)
    uint32_t split_ext[2];  // full extent d of split dim A / B (0 if none)
    uint32_t split_tile[2]; // tile extent of split dim A / B
    uint32_t split_step[2]; // distance of consecutive chunk origins (= split_tile unless the
                            // tiles overlap: line-aligned output windows)
    uint32_t split_halo[2]; // leading coordinates of the dim that do not exist (the halo in
                            // front of the first chunk); 0 normally
    uint32_t lds_elems;     // size of one LDS image (with padding), elements
    uint32_t lds_buffers;   // 1, or 2: tiles alternate between two images (one barrier per tile)
    uint32_t vec2;          // 1: 4-byte elements move in pairs (8-byte global accesses): entry 0
                            // of in_order counts pairs along input dim 0, entry 0 of out_order
                            // pairs along output dim 0; tile_vol is in pairs
    uint32_t pair_lstride;  // vec2: LDS distance of the two elements of an output-side pair
    uint32_t pair_a_split;  // vec2 in line-aligned windows: 1 if input dim 0, along which the read
                            // pairs run, is split dim A (its remaining extent may then be odd)
    uint32_t grid_mode;     // how workgroups walk the tiles, see tile_of()
    uint32_t tiles_per_xcd; // grid_mode 1: ceil(num_tiles / 8)
    uint32_t group_log2;    // grid_mode 2: log2 of the tile group dealt to one XCD
    uint32_t lane_a;        // lane of `major` holding the chunk counter of split A (if any)
    uint32_t lane_b;        // same for split B
    uint32_t chunk_pair[2]; // index of the SplitPair that carries the chunk counter of split
                            // A / B instead of a single lane; >= 2: none
    SplitPair pair[2];
    TileDim in_order[TPERM_DESC_MAX_DIMS];   // tile dims, input order (k enumerates these)
    TileDim out_order[TPERM_DESC_MAX_DIMS];  // the same dims, output order
    MajorDims major;
    OutAlign oa;
};

// The fields of TileDesc that say which tile comes next and what is left of the split dims in
// it (tile_of, tile_remaining), under the same names.  The kernel copies them out of the
// kernel-argument segment once, in one batch of scalar loads, and keeps them in scalar
// registers: read where they are used, each of them is a scalar load of its own with a wait
// behind it, a dozen round trips in a row before the first tile's loads can leave and again
// for every tile.
struct TileWalk {
    uint32_t num_tiles;
    uint32_t split_ext[2], split_tile[2], split_step[2], split_halo[2];
    uint32_t grid_mode, tiles_per_xcd, group_log2;
    uint32_t lane_a, lane_b;
    uint32_t chunk_pair[2];
    SplitPair pair[2];
};

template <typename D>
TPERM_HD TileWalk tile_walk_of(const D& d) {
    TileWalk w;
    w.num_tiles = d.num_tiles;
    for (int s = 0; s < 2; ++s) {
        w.split_ext[s] = d.split_ext[s];
        w.split_tile[s] = d.split_tile[s];
        w.split_step[s] = d.split_step[s];
        w.split_halo[s] = d.split_halo[s];
        w.chunk_pair[s] = d.chunk_pair[s];
        w.pair[s] = d.pair[s];
    }
    w.grid_mode = d.grid_mode;
    w.tiles_per_xcd = d.tiles_per_xcd;
    w.group_log2 = d.group_log2;
    w.lane_a = d.lane_a;
    w.lane_b = d.lane_b;
    return w;
}

// Per-thread, per-slot minor position for the read side (Eq. (4) and the LDS store slot).
// k is the position inside the tile in input order.  xa/xb are the coordinates along the
// split dims, used to mask ragged edge tiles.
struct Slot {
    uint32_t goff;   // element offset in global memory relative to the tile's major offset
    uint32_t ooff;   // the same element's offset on the other side (LDS-free kernels)
    uint32_t loff;   // element index in the LDS image
    uint32_t xa, xb;
};

TPERM_HD Slot tile_slot(const TileDim* dims, uint32_t n, uint32_t k) {
    Slot s;
    s.goff = 0; s.ooff = 0; s.loff = 0; s.xa = 0; s.xb = 0;
    uint32_t rem = k;
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t q = fdiv(rem, dims[i].div);
        const uint32_t x = rem - q * dims[i].ext;
        rem = q;
        s.goff += x * dims[i].gstride;
        s.ooff += x * dims[i].ostride;
        s.loff += x * dims[i].lstride;
        if (dims[i].sel == 1u) s.xa = x << dims[i].xshift;
        if (dims[i].sel == 2u) s.xb = x << dims[i].xshift;
    }
    return s;
}

// Term `lane` of the major sums for tile b: coordinate along that major dim.
TPERM_HD uint32_t major_coord(const MajorDims& m, uint32_t lane, uint32_t b) {
    const uint32_t q = fdiv(b, m.cum[lane]);
    return q - fdiv(q, m.ext_div[lane]) * m.ext[lane];
}

// Remaining extent of a split dim in the chunk with counter `chunk` (ragged last chunk).
TPERM_HD uint32_t split_remaining(uint32_t full_ext, uint32_t tile_ext, uint32_t step, uint32_t chunk) {
    if (full_ext == 0u) return TPERM_NO_REM;
    const uint32_t start = chunk * step;
    if (start >= full_ext) return 0u;
    const uint32_t left = full_ext - start;
    return left < tile_ext ? left : tile_ext;
}

// From the per-lane coordinates of a tile (coord(l) returns lane l's coordinate): does the
// tile exist, and what is left of the split dims in it.  A tile that does not exist gets
// remaining extents of 0, which masks every slot.  lo_b: first valid coordinate of split dim B
// in this tile (non-zero only in the first chunk of a dim with a halo).
// D: the descriptor, or a copy of its tile-walk fields (see TileWalk).
template <typename D, typename CoordFn>
TPERM_HD void tile_remaining(const D& d, CoordFn coord, uint32_t* rem_a, uint32_t* rem_b,
                             uint32_t* lo_b) {
    bool exists = true;
    uint32_t counter[2] = {0u, 0u};
    for (int p = 0; p < 2; ++p)
        if (d.pair[p].count != 0u) {
            counter[p] = coord(d.pair[p].lane_lo) + d.pair[p].width * coord(d.pair[p].lane_hi);
            exists = exists && counter[p] < d.pair[p].count;
        }
    const uint32_t chunk_a = d.chunk_pair[0] < 2u ? counter[d.chunk_pair[0]] : coord(d.lane_a);
    const uint32_t chunk_b = d.chunk_pair[1] < 2u ? counter[d.chunk_pair[1]] : coord(d.lane_b);
    *rem_a = exists ? split_remaining(d.split_ext[0], d.split_tile[0], d.split_step[0], chunk_a) : 0u;
    *rem_b = exists ? split_remaining(d.split_ext[1], d.split_tile[1], d.split_step[1], chunk_b) : 0u;
    const uint32_t start_b = chunk_b * d.split_step[1];
    *lo_b = d.split_halo[1] > start_b ? d.split_halo[1] - start_b : 0u;
}

// Tile visited by workgroup `block` of `grid` on its i-th iteration, or num_tiles if done.
// Workgroups are dealt round-robin to the 8 XCDs (workgroup w runs on XCD w % 8), each with
// its own L2.  grid_mode 0 walks the tiles in launch order, so neighbouring tiles run on
// different XCDs.  grid_mode 1 gives each XCD one contiguous eighth of the tiles.
// grid_mode 2 deals groups of 2^group_log2 consecutive tiles to the XCDs in turn: tiles
// that share cache lines at their edges meet in one L2, while all XCDs still work on the
// same neighbourhood of the tensors.  Modes 1 and 2 need grid % 8 == 0.
template <typename D>
TPERM_HD uint32_t tile_of(const D& d, uint32_t block, uint32_t grid, uint32_t i) {
    if (d.grid_mode == 1u) {
        const uint32_t xcd = block & 7u, slot = block >> 3, per = grid >> 3;
        const uint32_t local = slot + i * per;
        if (local >= d.tiles_per_xcd) return d.num_tiles;
        const uint32_t b = xcd * d.tiles_per_xcd + local;
        return b < d.num_tiles ? b : d.num_tiles;
    }
    if (d.grid_mode == 2u) {
        const uint32_t xcd = block & 7u, slot = block >> 3, per = grid >> 3;
        const uint64_t local = (uint64_t)slot + (uint64_t)i * per;
        const uint64_t group = local >> d.group_log2;
        const uint64_t b = (((group << 3) + xcd) << d.group_log2) + (local & ((1u << d.group_log2) - 1u));
        return b < d.num_tiles ? (uint32_t)b : d.num_tiles;
    }
    const uint64_t b = (uint64_t)block + (uint64_t)i * grid;
    return b < d.num_tiles ? (uint32_t)b : d.num_tiles;
}

// Descriptor of the naive gather kernel: one thread per output element.
struct NaiveDesc {
    uint32_t rank;
    uint32_t volume;
    FastDiv out_ext_div[TPERM_DESC_MAX_DIMS];  // division by output extent j
    uint32_t out_ext[TPERM_DESC_MAX_DIMS];
    uint32_t in_stride[TPERM_DESC_MAX_DIMS];   // input stride of the dim at output position j
};

TPERM_HD uint32_t naive_input_offset(const NaiveDesc& d, uint32_t o) {
    uint32_t rem = o, p = 0;
    for (uint32_t j = 0; j < d.rank; ++j) {
        const uint32_t q = fdiv(rem, d.out_ext_div[j]);
        p += (rem - q * d.out_ext[j]) * d.in_stride[j];
        rem = q;
    }
    return p;
}

}  // namespace tperm
