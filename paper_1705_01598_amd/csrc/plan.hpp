// Host-side planner: validate, canonicalise, enumerate candidate tiles, score them and
// fill the kernel descriptor.  Pure C++ with no HIP calls, so it runs on a GPU-less host.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/tperm_tuning.h"
#include "tperm_desc.h"

namespace tperm {

// Largest tile the tile kernels accept: NREG_MAX slots per thread, and an LDS image that
// fits the 64 KiB a workgroup may take without opting in to more.
constexpr int kMaxNreg = 32;
constexpr int64_t kMaxTileVol = (int64_t)kMaxNreg * TPERM_MAX_THREADS;  // 8192 elements
constexpr int64_t kMaxLdsBytes = 64 * 1024;
// Tiles that run at the same time can be grouped into windows of this many neighbours along
// the input side and along the output side (1 = no window; on the input side 0 = automatic:
// only the chunk counter of a few ragged chunks of the input run, see build_tile_plan).
constexpr int kDefaultWindow = 1;
constexpr int kDefaultWindowIn = 0;
constexpr int kDefaultThreads = 256;
constexpr int kDefaultLdsBuffers = 1;
// Groups of 32 consecutive tiles are dealt to the XCDs in turn: tiles that are neighbours
// along the output run then share an L2, which merges the cache lines they both write
// part of (+4 % measured on shapes whose runs are not line-aligned, neutral otherwise).
constexpr int kDefaultGridMode = 2 + 5;
constexpr int kDefaultTileOrder = 1;  // output-major: +1-4 % measured over input-major
// Score of a candidate with line-aligned output windows, fitted to the measured times of all
// candidates of 82 ragged benchmark cases that have such candidates (both halves of the sample
// give the same constants; picks land at 97.6 % of the best candidate against 94.9 % without
// this form): input runs keep paying off longer than in plain tiles (overhead worth 64 bytes
// instead of 16: the rows it reads are the misaligned side now), the halo makes the reads cost
// (1 + 3 (line / chunk)^1.5) as much, an output run costs a fixed 32 bytes on top of its
// length, and the whole is 15 % cheaper than those terms say.
constexpr double kAlignInOverhead = 64.0;
constexpr double kAlignOutOverhead = 32.0;
constexpr double kAlignHaloWeight = 3.0;
constexpr double kAlignHaloPower = 1.5;
constexpr double kAlignWeight = 0.85;
// The same for 4-byte elements, which such tiles move in pairs; fitted to all candidates of 110
// ragged 4-byte cases of rank 2 to 4 (picks at 93.6 % of the best candidate against 87.4 %
// without this form; both halves of the sample agree): input rows want to be longer still
// (overhead worth 256 bytes: a 256-byte row beats a 128-byte one by 12 % at equal tile
// volume), the halo weighs less (1 + (line / chunk)^2), the whole is 30 % cheaper.
constexpr double kAlign4InOverhead = 256.0;
constexpr double kAlign4OutOverhead = 64.0;
constexpr double kAlign4HaloWeight = 1.0;
constexpr double kAlign4HaloPower = 2.0;
constexpr double kAlign4Weight = 0.7;

// The per-thread slot counts the tile kernel is instantiated for, by workgroup size.
// Returns the smallest instantiated count >= need, or -1.
int pick_nreg(int64_t tile_vol, int threads);

struct Canonical {
    int rank = 0;
    int64_t dims[TPERM_MAX_RANK] = {0};
    int perm[TPERM_MAX_RANK] = {0};
    int64_t volume = 0;
};

// A candidate tile: extents per canonical dim (1 = dim is enumerated by the tile index).
struct Candidate {
    int kclass = 0;   // ROWCOPY / TILED / PACKED
    bool use_lds = true;
    bool align = false;        // line-aligned output windows (see OutAlign)
    int m = 0, k = 0;
    int64_t t[TPERM_MAX_RANK] = {0};
    int64_t tile_vol = 0, run_in = 0, run_out = 0, num_tiles = 0;
    bool aligned = false;      // every run starts and ends on a 128-byte line boundary
    bool out_aligned = false;  // output runs start and end on line boundaries
    bool load_nt = false;      // every input run starts and ends on a 128-byte line boundary
    bool store_nt = false;     // every written piece starts and ends on a 32-byte sector
    double utilisation = 1.0;  // useful fraction of the slots of all tiles (ragged edges)
    double score = 0.0;        // relative cost estimate, lower is better
};

struct Plan {
    int rank = 0;
    int64_t dims[TPERM_MAX_RANK] = {0};
    int perm[TPERM_MAX_RANK] = {0};
    int elem = 0;
    Canonical c;
    int kclass = 0;
    Candidate cand;
    bool use_lds = false;
    int nreg = 0;
    int threads = TPERM_MAX_THREADS;  // workgroup size: 256 (four wavefronts) or 64 (one)
    int lds_pad = 0;
    int lds_bytes = 0;
    bool align_out = false;  // the plan writes line-aligned output windows
    int grid_mode = 0;
    int blocks_per_cu = 0;   // cap on resident workgroups per compute unit (0 = none)
    bool vec2 = false;         // 4-byte elements move in pairs; needs 8-byte aligned pointers
    bool loads_first = false;  // next tile's loads are issued before this tile's stores
    int cache_policy = 1;    // 1 = cached, 2 = nontemporal loads and stores, 3 = nontemporal stores, 4 = nontemporal loads
    bool big = false;        // tensor of 4 GiB or more: tiles describe their buffers from their own origin
    TileDesc tile;
    NaiveDesc naive;
    // launch geometry, resolved on first execute (needs the device); 0 = not yet
    int max_blocks = 0;
};

tperm_status_t validate(int rank, const int64_t* dims, const int* perm, size_t elem);
void canonicalise(int rank, const int64_t* dims, const int* perm, Canonical* out);
FastDiv make_fastdiv(uint32_t d);

// All candidate tiles for a canonical problem, each scored; sorted best first.
std::vector<Candidate> enumerate_candidates(const Canonical& c, int elem);

// Build a candidate from explicit (m, tile_in, k, tile_out); false if it cannot run.
bool make_candidate(const Canonical& c, int elem, int m, int64_t tile_in, int k,
                    int64_t tile_out, bool use_lds, Candidate* out, bool align = false);

// Fill plan->tile (and nreg, lds size, padding) from a candidate.
struct TileBuildOpts {
    int lds_pad = -1;       // -1: search
    int grid_mode = kDefaultGridMode;
    int window_in = kDefaultWindowIn, window_out = kDefaultWindow;
    int threads = kDefaultThreads;
    int lds_buffers = kDefaultLdsBuffers;
    int align_out = 0;      // line-aligned output windows: 0 = as the candidate says, 1 = off, 2 = on where the tile allows
    int tile_order = kDefaultTileOrder;  // 0: input-major, 1: output-major
    int vec2 = 0;           // elements in pairs: 0 = off, 1 = where possible and worth it, 2 = wherever possible
    bool big = false;       // tensor of 4 GiB or more: plain LDS-staged tiles of 256 threads whose positions stay below TPERM_BIG_RANGE
};
tperm_status_t build_tile_plan(Plan* plan, const Candidate& cand, const TileBuildOpts& opts);
void build_naive_desc(Plan* plan);

// Plan creation proper.
tperm_status_t create_plan(Plan** out, int rank, const int64_t* dims, const int* perm,
                           size_t elem, const tperm_plan_opts_t* opts);

// Plan for one explicit candidate (measurement-based selection tries them one by one).
// vec2: move 4-byte elements in pairs where the candidate allows (the plan then needs 8-byte
// aligned pointers; plan->vec2 tells whether it does).
tperm_status_t create_plan_with_candidate(Plan** out, int rank, const int64_t* dims,
                                          const int* perm, size_t elem, const Candidate& cand,
                                          bool vec2 = false);

// Host evaluation of the plan's index maps (see tperm_plan_index_map).
tperm_status_t index_map(const Plan& plan, int64_t* out_to_in);

// Estimated LDS cycles of the first accesses of a workgroup for a given descriptor
// (bank-conflict count evaluated from the slot positions, as Section 2.3 does for the
// shared-memory term of its model).
double lds_conflict_cost(const TileDesc& d, int elem, int nreg, int threads);
// The same as a ratio: LDS passes per wave-wide access, 1 = conflict-free (the TPR_shmem of
// Section 2.3).
double lds_conflict_ratio(const TileDesc& d, int elem, int nreg, int threads);

// Analytical estimate of a tile plan's run time (model.cpp): Eqs. (10)-(13) of Section 2.3 with
// exact line counts from a sample of tiles and constants for MI355X.
tperm_status_t model_plan(const Plan& plan, tperm_model_t* out);

}  // namespace tperm
