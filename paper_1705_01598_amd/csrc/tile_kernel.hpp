// HIP device code for gfx950 (MI355X): the tile kernel that every staged transpose class
// runs through.
//
// Tile kernel, per workgroup (256 threads = 4 wavefronts of 64):
//   prologue  every thread evaluates, once, the minor positions (Eqs. (4)-(6)) of the
//             NREG tile slots it owns and keeps them in registers;
//   per tile  the major offsets (Eqs. (2),(3)) are evaluated lane-parallel: lane j of a
//             16-lane DPP row holds term j, a row_shr scan adds them, v_readlane moves the
//             sum into scalar registers (the wave64 form of the paper's Algorithm 1);
//             global -> registers -> LDS (input order), barrier, LDS (output order) ->
//             registers -> global.  The loads of the next tile are issued back to back
//             with the stores of the current one, so reads are in flight while the tile
//             is finished; which of the two goes first is a plan choice (see the loop).
// This header holds the device code; tile_inst_*.hip instantiate it per element type and
// workgroup size so that the units compile in parallel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "tperm_desc.h"

namespace tperm {

// ---------------------------------------------------------------------------------------
// wave-level helpers
// ---------------------------------------------------------------------------------------

// Inclusive add-scan inside each row of 16 lanes with DPP row shifts; lane 15 of a row
// ends up with the sum of the row.  Lanes shifted in from outside the row read 0.
__device__ __forceinline__ uint32_t row_scan_add(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, true);  // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, true);  // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);  // row_shr:8
    return v;
}

__device__ __forceinline__ uint32_t read_lane(uint32_t v, uint32_t lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)lane);
}

// Keeps a wave-uniform value in a scalar register from here on: the compiler may not go back
// to the kernel-argument segment for it (it would otherwise reload such values where they are
// used, one scalar load and one wait each).
__device__ __forceinline__ void keep_scalar(uint32_t& v) { asm volatile("" : "+s"(v)); }

__device__ __forceinline__ void keep_tile_dim(TileDim& t) {
    keep_scalar(t.ext);
    keep_scalar(t.div.magic);
    keep_scalar(t.div.shift);
    keep_scalar(t.gstride);
    keep_scalar(t.ostride);
    keep_scalar(t.lstride);
    keep_scalar(t.sel);
    keep_scalar(t.xshift);
}

__device__ __forceinline__ TileWalk pinned_tile_walk(const TileDesc& d) {
    TileWalk w = tile_walk_of(d);
    keep_scalar(w.num_tiles);
    for (int s = 0; s < 2; ++s) {
        keep_scalar(w.split_ext[s]);
        keep_scalar(w.split_tile[s]);
        keep_scalar(w.split_step[s]);
        keep_scalar(w.split_halo[s]);
        keep_scalar(w.chunk_pair[s]);
        keep_scalar(w.pair[s].lane_lo);
        keep_scalar(w.pair[s].lane_hi);
        keep_scalar(w.pair[s].width);
        keep_scalar(w.pair[s].count);
    }
    keep_scalar(w.grid_mode);
    keep_scalar(w.tiles_per_xcd);
    keep_scalar(w.group_log2);
    keep_scalar(w.lane_a);
    keep_scalar(w.lane_b);
    return w;
}

// The tile-walk fields as the kernel uses them: a pinned copy, or the descriptor itself.
template <bool PIN>
__device__ __forceinline__ typename std::conditional<PIN, TileWalk, const TileDesc&>::type tile_walk_source(const TileDesc& d) {
    if constexpr (PIN) return pinned_tile_walk(d);
    else return d;
}

struct MajorPos {
    uint32_t in, out;        // element offsets of the tile (wave-uniform)
    uint32_t rem_a, rem_b;   // remaining extent of the split dims in this tile
    uint32_t lo_b, span_b;   // line-aligned windows: coordinates lo_b <= x < lo_b + span_b
                             // of split dim B exist in this tile
};

// One lane's term of the major sums, kept in registers for the whole kernel.
struct MajorLane {
    FastDiv cum, ext_div;
    uint32_t ext, stride_in, stride_out;
};

template <typename D>
__device__ __forceinline__ MajorPos major_position(const D& d, const MajorLane& ml, uint32_t b) {
    const uint32_t q = fdiv(b, ml.cum);
    const uint32_t c = q - fdiv(q, ml.ext_div) * ml.ext;
    const uint32_t sum_in = row_scan_add(c * ml.stride_in);
    const uint32_t sum_out = row_scan_add(c * ml.stride_out);
    MajorPos p;
    p.in = read_lane(sum_in, 15);
    p.out = read_lane(sum_out, 15);
    tile_remaining(d, [&](uint32_t lane) { return read_lane(c, lane); }, &p.rem_a, &p.rem_b, &p.lo_b);
    p.span_b = p.rem_b > p.lo_b ? p.rem_b - p.lo_b : 0u;
    return p;
}

__device__ __forceinline__ bool slot_valid(uint32_t packed, uint32_t rem_a, uint32_t rem_b) {
    return ((packed & 0xFFFFu) < rem_a) && ((packed >> 16) < rem_b);
}

// The same with a lower bound on the coordinate along split dim B: lo_b <= x < lo_b + span_b.
__device__ __forceinline__ bool slot_valid_from(uint32_t packed, uint32_t rem_a, uint32_t lo_b,
                                                uint32_t span_b) {
    return ((packed & 0xFFFFu) < rem_a) && (((packed >> 16) - lo_b) < span_b);
}

// ---------------------------------------------------------------------------------------
// buffer addressing
// ---------------------------------------------------------------------------------------
// Global accesses of the tile kernel go through buffer instructions: a 128-bit resource in
// scalar registers describes the whole tensor, the tile's major offset rides in the scalar
// offset operand and each lane supplies only its 32-bit minor byte offset.  One VGPR per
// address instead of two, no 64-bit vector adds, and the hardware drops any access past
// the end of the tensor.  NT selects the cache policy: 0 = cached, 1 = nontemporal stores
// (written lines are not worth a place in the caches once they are complete), 2 =
// nontemporal loads as well (every byte is touched exactly once), 3 = nontemporal loads only
// (line-aligned input, output pieces that end inside lines and want them kept in L2).

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T, int NT> struct Elem;
template <int NT> struct Elem<uint32_t, NT> {
    typedef uint32_t reg;
    // accumulate: the 4-byte element is an IEEE binary32 number
    static __device__ __forceinline__ reg add(reg a, reg b) {
        return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
    }
    static __device__ __forceinline__ reg load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        return __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, (NT == 2 || NT == 3) ? 2 : 0);
    }
    static __device__ __forceinline__ void store(reg v, __amdgpu_buffer_rsrc_t r, uint32_t voff,
                                                 uint32_t soff) {
        __builtin_amdgcn_raw_buffer_store_b32(v, r, (int)voff, (int)soff, (NT == 1 || NT == 2) ? 2 : 0);
    }
};
template <int NT> struct Elem<uint64_t, NT> {
    typedef u32x2 reg;
    // accumulate: the 8-byte element is an IEEE binary64 number
    static __device__ __forceinline__ reg add(reg a, reg b) {
        const double s = __hiloint2double((int)a.y, (int)a.x) + __hiloint2double((int)b.y, (int)b.x);
        reg r;
        r.x = (uint32_t)__double2loint(s);
        r.y = (uint32_t)__double2hiint(s);
        return r;
    }
    static __device__ __forceinline__ reg load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        return __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, (NT == 2 || NT == 3) ? 2 : 0);
    }
    static __device__ __forceinline__ void store(reg v, __amdgpu_buffer_rsrc_t r, uint32_t voff,
                                                 uint32_t soff) {
        __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)voff, (int)soff, (NT == 1 || NT == 2) ? 2 : 0);
    }
};

// Lane offset of a slot that must not touch memory in this tile (ragged edge, tile that
// does not exist).  It lies beyond every tensor the planner accepts (volume * elem_size <
// 2^32 - 256), so the buffer range check, which looks at the lane offset only, drops the
// access: loads return zero, stores are discarded.  Issuing every memory instruction
// unconditionally keeps their number per tile fixed, which lets the loads of the next tile
// be waited for with a partial vmcnt while this tile's stores are still in flight; with
// branches around them the only safe wait is for everything, stores included.
constexpr uint32_t kDroppedOffset = 0xFFFFFF00u;

// 16-byte accesses: two 8-byte elements at once (vec2 plans of 8-byte problems); never
// accumulated.
struct Pair64 {};
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int NT> struct Elem<Pair64, NT> {
    typedef u32x4 reg;
    static __device__ __forceinline__ reg add(reg a, reg) { return a; }
    static __device__ __forceinline__ reg load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, (NT == 2 || NT == 3) ? 2 : 0);
    }
    static __device__ __forceinline__ void store(reg v, __amdgpu_buffer_rsrc_t r, uint32_t voff,
                                                 uint32_t soff) {
        __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voff, (int)soff, (NT == 1 || NT == 2) ? 2 : 0);
    }
};

// Raw (untyped, unstrided) buffer resource over `bytes` bytes starting at p.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// ---------------------------------------------------------------------------------------
// the tile kernel
// ---------------------------------------------------------------------------------------

// BIG: tensors of 4 GiB and more.  A tile's origin (its major offset) no longer fits the 32-bit
// scalar offset of a buffer access, so it goes into the base address instead: every tile
// describes its buffers anew, starting at its own origin, and the scalar offset stays zero.  The
// lane offsets (positions inside the tile, which the planner keeps below TPERM_BIG_RANGE bytes)
// and the dropped-offset masking work as before; nbytes is then TPERM_BIG_RANGE, the range one
// such description covers.  With line-aligned windows the halo origin in front of the tensors
// moves along with the tile's.  LDS-staged tiles in every form, stores first.
template <typename T, int NREG, int THREADS, bool USE_LDS, int NT, bool ALIGN, bool ACC, bool LOADS_FIRST, bool VEC2, bool BIG = false>
__global__ void __launch_bounds__(THREADS)
tile_kernel(const TileDesc d, const T* __restrict__ in_arg, T* __restrict__ out_arg, uint32_t nbytes_arg) {
    static_assert(!BIG || (USE_LDS && !LOADS_FIRST), "large tensors: LDS-staged tiles, stores first");
    const T* in = in_arg;
    T* out = out_arg;
    uint32_t nbytes = nbytes_arg;
    // VEC2: a slot is a pair of elements, moved through global memory with one access of
    // twice the element size; the LDS image stays in single elements.
    static_assert(!VEC2 || (USE_LDS && !ACC), "vec2 is an LDS-staged, non-accumulating form");
    static_assert(!(VEC2 && ALIGN) || sizeof(T) == 4, "pairs in line-aligned windows: 4-byte elements");
    // PAIRWIN: pairs of 4-byte elements in line-aligned output windows.  Read pairs run along
    // input dim 0 (8-byte loads from 4-byte aligned addresses when rows have odd lengths),
    // written pairs along the window, where they are always 8-byte aligned.  A tile that
    // holds the odd end of an input row, or a window clipped by the ends of an output row,
    // moves that side element by element instead (a wave-uniform choice per tile and side).
    constexpr bool PAIRWIN = VEC2 && ALIGN;
    typedef typename std::conditional<sizeof(T) == 4, uint64_t, Pair64>::type pair_t;
    typedef Elem<typename std::conditional<VEC2, pair_t, T>::type, NT> io;
    typedef Elem<T, NT> io1;  // single elements
    typedef typename io::reg reg_t;
    typedef typename Elem<T, NT>::reg lds_t;  // one element
    extern __shared__ __align__(16) unsigned char smem_raw[];
    lds_t* lds = reinterpret_cast<lds_t*>(smem_raw);
    const uint32_t tid = threadIdx.x;
    // This lane's term of the major sums.  The descriptor sits in the kernel-argument segment and
    // a per-lane index into it becomes vector loads from there, which take a good half
    // microsecond to come back: they are issued first, so that they travel while the prologue
    // below computes.
    const uint32_t lane16 = tid & 15u;
    MajorLane ml;
    ml.cum = d.major.cum[lane16];
    ml.ext_div = d.major.ext_div[lane16];
    ml.ext = d.major.ext[lane16];
    ml.stride_in = d.major.stride_in[lane16];
    ml.stride_out = d.major.stride_out[lane16];

    // What the tile loop needs of the descriptor, and the constants of the first two tile dims,
    // fetched now in one batch of scalar loads (one round trip to the kernel-argument segment
    // instead of one per use) and kept in scalar registers.  Not in the kernels with
    // line-aligned windows: their loop keeps so many scalars alive that pinned ones end up
    // spilled into vector lanes, which costs the pairs-in-windows form 7 %; there the compiler
    // reads the descriptor where it needs it.
    constexpr bool PIN = !ALIGN;
    TileDim first_out[2] = {d.out_order[0], d.out_order[1]};
    TileDim first_in[2] = {d.in_order[0], d.in_order[1]};
    typename std::conditional<PIN, const TileWalk, const TileDesc&>::type walk = tile_walk_source<PIN>(d);
    uint32_t n_tile_dims = d.n_tile_dims, tile_vol = d.tile_vol, lds_elems = d.lds_elems;
    uint32_t lds_buffers = d.lds_buffers, pair_lstride = d.pair_lstride, pair_a_split = d.pair_a_split;
    if constexpr (PIN) {
        for (int i = 0; i < 2; ++i) {
            keep_tile_dim(first_out[i]);
            if (USE_LDS) keep_tile_dim(first_in[i]);
        }
        asm volatile("" : "+s"(in), "+s"(out), "+s"(nbytes));  // the same batch
        keep_scalar(n_tile_dims);
        keep_scalar(tile_vol);
        if (USE_LDS) {
            keep_scalar(lds_elems);
            keep_scalar(lds_buffers);
        }
        if (VEC2) {
            keep_scalar(pair_lstride);
            keep_scalar(pair_a_split);
        }
    }
    const OutAlign oa = d.oa;

    // ALIGN (line-aligned output windows): tile coordinates along the shifted dimension count
    // from a halo origin one line's worth of elements in front of the chunk, so both buffers
    // are described from that far in front of the tensors; the slots that would fall before
    // a tensor's first element are masked (lo_b).
    const uint32_t halo_in = ALIGN ? oa.in_halo_elems * (uint32_t)sizeof(T) : 0u;
    const uint32_t halo_out = ALIGN ? oa.line_elems * (uint32_t)sizeof(T) : 0u;
    // (BIG: nbytes is already the whole range of a description, counted from a tile's origin)
    const char* const in_origin = reinterpret_cast<const char*>(in) - halo_in;
    char* const out_origin = reinterpret_cast<char*>(out) - halo_out;
    const __amdgpu_buffer_rsrc_t rsrc_in_whole = make_rsrc(in_origin, BIG ? nbytes : nbytes + halo_in);
    const __amdgpu_buffer_rsrc_t rsrc_out_whole = make_rsrc(out_origin, BIG ? nbytes : nbytes + halo_out);

    // minor positions of this thread's slots; global offsets are kept in BYTES
    uint32_t rd_off[NREG], wr_off[NREG], rd_mask[NREG], wr_mask[NREG];
    uint32_t lds_pos[NREG];  // low half: slot written on the read side; high half: slot
                             // read on the write side
    uint32_t wr_aux[NREG];   // ALIGN: unshifted tile coordinate along the shifted dim |
                             // phase of the row start << 16
    {
        // Slots walk the tile dims in groups of up to four: each dim's constants are fetched
        // once per group (scalar loads) and the group's independent digit steps overlap,
        // instead of one dependent chain per slot that waits for the same loads again.
        // Larger groups would raise the register peak of the kernel above the main loop's.
        constexpr int G = NREG <= 4 ? NREG : (NREG % 4 == 0 ? 4 : 3);
        static_assert(NREG % G == 0, "slot groups must tile the slots");
        // ALIGN: the write side has fewer slots than the read side (no halo)
        const uint32_t write_slots = ALIGN ? oa.total_slots : tile_vol;
#pragma unroll
        for (int g0 = 0; g0 < NREG; g0 += G) {
            uint32_t rem_o[G], rem_i[G], loff_o[G], loff_i[G];
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                rem_o[jj] = rem_i[jj] = tid + (uint32_t)(g0 + jj) * THREADS;
                wr_off[g0 + jj] = 0;
                rd_off[g0 + jj] = 0;
                wr_mask[g0 + jj] = 0;
                rd_mask[g0 + jj] = 0;
                loff_o[jj] = 0;
                loff_i[jj] = 0;
            }
            // Entry i of both orders in one pass: the write side (output order; LDS-free
            // kernels read the same slots through ostride) and, with an LDS stage, the read
            // side (input order).
            auto digit_step = [&](const TileDim& to, const TileDim& ti) {
                const uint32_t shift_o = to.sel == 2u ? 16u + to.xshift : to.xshift;
#pragma unroll
                for (int jj = 0; jj < G; ++jj) {
                    const int j = g0 + jj;
                    const uint32_t q = fdiv(rem_o[jj], to.div);
                    const uint32_t x = rem_o[jj] - q * to.ext;
                    rem_o[jj] = q;
                    wr_off[j] += x * to.gstride;
                    if (USE_LDS) loff_o[jj] += x * to.lstride;
                    else rd_off[j] += x * to.ostride;
                    if (to.sel != 0u) wr_mask[j] |= x << shift_o;
                }
                if (USE_LDS) {
                    const uint32_t shift_i = ti.sel == 2u ? 16u + ti.xshift : ti.xshift;
#pragma unroll
                    for (int jj = 0; jj < G; ++jj) {
                        const int j = g0 + jj;
                        const uint32_t q = fdiv(rem_i[jj], ti.div);
                        const uint32_t x = rem_i[jj] - q * ti.ext;
                        rem_i[jj] = q;
                        rd_off[j] += x * ti.gstride;
                        loff_i[jj] += x * ti.lstride;
                        if (ti.sel != 0u) rd_mask[j] |= x << shift_i;
                    }
                }
            };
            // The first two entries are taken unconditionally, from the copies fetched at the top of
            // the kernel; every turn of the loop below costs one more round trip to the descriptor.  (An entry beyond n_tile_dims is all
            // zero, which is neutral here: quotient 0, no stride, no mask.)
            if constexpr (PIN) {
                digit_step(first_out[0], first_in[0]);
                digit_step(first_out[1], first_in[1]);
            }
            for (uint32_t i = PIN ? 2u : 0u; i < n_tile_dims; ++i) {
                // whole entries at once: one round trip per turn, not one per field
                TileDim to = d.out_order[i], ti = d.in_order[i];
                if constexpr (PIN) {
                    keep_tile_dim(to);
                    if (USE_LDS) keep_tile_dim(ti);
                }
                digit_step(to, ti);
            }
#pragma unroll
            for (int jj = 0; jj < G; ++jj) {
                const int j = g0 + jj;
                const uint32_t k = tid + (uint32_t)j * THREADS;
                const bool used_r = k < tile_vol, used_w = k < write_slots;
                wr_aux[j] = 0;
                if (ALIGN) {
                    // p = position in the chunk (output stride 1); the slot reads the tile
                    // coordinate p + line_elems - shift and stores that many elements on
                    // from the halo origin, where shift is this row's phase in the tile
                    const uint32_t p = wr_mask[j] >> 16;
                    const uint32_t rho = (wr_off[j] - p) & (oa.line_elems - 1u);
                    wr_aux[j] = used_w ? ((p + oa.line_elems) | (rho << 16)) : 0u;
                    wr_off[j] += oa.line_elems;
                    loff_o[jj] += oa.line_elems * oa.lstride_b;
                }
                wr_off[j] = used_w ? wr_off[j] * (uint32_t)sizeof(T) : 0u;
                rd_off[j] = used_r ? rd_off[j] * (uint32_t)sizeof(T) : 0u;
                wr_mask[j] = used_w ? wr_mask[j] : 0xFFFFFFFFu;  // coordinates no remaining
                if (USE_LDS) {                                    // extent exceeds: unused
                    rd_mask[j] = used_r ? rd_mask[j] : 0xFFFFFFFFu;
                    lds_pos[j] = (used_r ? loff_i[jj] : 0u) | ((used_w ? loff_o[jj] : 0u) << 16);
                } else {
                    rd_mask[j] = wr_mask[j];
                }
            }
        }
    }

    const uint32_t grid = gridDim.x, block = blockIdx.x;
    uint32_t it = 0;
    uint32_t b = tile_of(walk, block, grid, it);
    reg_t v[NREG];
    MajorPos pos, nxt;
    pos.in = pos.out = pos.rem_a = pos.rem_b = pos.lo_b = pos.span_b = 0;
    nxt = pos;
    // does read-side slot j exist in tile t
    auto read_ok = [&](int j, const MajorPos& t) {
        return ALIGN ? slot_valid_from(rd_mask[j], t.rem_a, t.lo_b, t.span_b)
                     : slot_valid(rd_mask[j], t.rem_a, t.rem_b);
    };
    // PAIRWIN: the second element of read-side pair j exists in tile t / the tile holds the odd
    // end of an input row (remaining extent of split dim A is odd)
    auto read_ok_second = [&](int j, const MajorPos& t) {
        return read_ok(j, t) && slot_valid_from(rd_mask[j] + 1u, t.rem_a, t.lo_b, t.span_b);
    };
    auto odd_row_end = [&](const MajorPos& t) { return PAIRWIN && pair_a_split != 0u && (t.rem_a & 1u) != 0u; };
    // the buffer description and scalar offset that reach element `origin` of a tensor
    auto reach = [&](const __amdgpu_buffer_rsrc_t& whole, const void* base, uint32_t origin, uint32_t* soff) {
        if constexpr (BIG) {
            *soff = 0u;
            return make_rsrc(reinterpret_cast<const char*>(base) + (uint64_t)origin * sizeof(T), nbytes);
        } else {
            *soff = origin * (uint32_t)sizeof(T);
            return whole;
        }
    };
    auto load_tile = [&](const MajorPos& t) {
        uint32_t soff;
        const __amdgpu_buffer_rsrc_t rsrc_in = reach(rsrc_in_whole, in_origin, t.in, &soff);
        if constexpr (PAIRWIN) {
            if (odd_row_end(t)) {
#pragma unroll
                for (int j = 0; j < NREG; ++j) {
                    v[j].x = io1::load(rsrc_in, read_ok(j, t) ? rd_off[j] : kDroppedOffset, soff);
                    v[j].y = io1::load(rsrc_in, read_ok_second(j, t) ? rd_off[j] + 4u : kDroppedOffset, soff);
                }
                return;
            }
        }
#pragma unroll
        for (int j = 0; j < NREG; ++j)
            v[j] = io::load(rsrc_in, read_ok(j, t) ? rd_off[j] : kDroppedOffset, soff);
    };
    if (b < walk.num_tiles) {
        pos = major_position(walk, ml, b);
        load_tile(pos);
    }
    // As many dropped stores as a tile has real ones: every pass through the loop below then
    // starts with the same queue of memory operations behind it (one tile of loads, one of
    // stores), which is what lets the compiler wait for the loads alone.
    {
        const reg_t nothing = {};
#pragma unroll
        for (int j = 0; j < NREG; ++j)  // distinct offsets, or the compiler folds them into one
            io::store(nothing, rsrc_out_whole, kDroppedOffset + (LOADS_FIRST ? 0u : 4u * (uint32_t)j), 0u);
    }
    // the position of the tile after this one is worked out while the loads are in flight
    uint32_t bn = tile_of(walk, block, grid, it + 1);
    const MajorPos no_tile = nxt;  // all zero: no slot is valid
    if (bn < walk.num_tiles) nxt = major_position(walk, ml, bn);
    const bool two_buffers = lds_buffers == 2u;
    // line-aligned windows: phase of the output base pointer within a 128-byte line
    const uint32_t line_mask = ALIGN ? oa.line_elems - 1u : 0u;
    const uint32_t out_phase =
        ALIGN ? (uint32_t)(reinterpret_cast<uintptr_t>(out) / sizeof(T)) & line_mask : 0u;
    while (b < walk.num_tiles) {
        reg_t w[NREG];
        // Write side of this tile: byte offset of every slot, or kDroppedOffset.  ALIGN: the
        // slot's row starts `shift` elements past a line boundary (phase of the tile origin +
        // phase of the row within the tile), so the slot moves down by that much, in the
        // output and in the LDS image alike.
        const uint32_t phi = ALIGN ? (out_phase + pos.out) & line_mask : 0u;
        auto row_shift = [&](int j) { return (phi + (wr_aux[j] >> 16)) & line_mask; };
        auto write_at = [&](int j) -> uint32_t {
            if (ALIGN) {
                const uint32_t sh = row_shift(j);
                const uint32_t xb = (wr_aux[j] & 0xFFFFu) - sh;
                const bool ok = ((wr_mask[j] & 0xFFFFu) < pos.rem_a) && ((xb - pos.lo_b) < pos.span_b);
                return ok ? wr_off[j] - sh * (uint32_t)sizeof(T) : kDroppedOffset;
            }
            return slot_valid(wr_mask[j], pos.rem_a, pos.rem_b) ? wr_off[j] : kDroppedOffset;
        };
        // The reads of the next tile and the stores of this one are issued back to back after
        // the barrier and the LDS reads, so that all waves of the workgroup ask for their
        // rows together (issuing the reads before the barrier, each wave on its own, measured
        // 2-8 % slower).  Which of the two goes first is the plan's choice:
        //   stores first  (default) the tile's registers are freed at once; every memory
        //                 instruction is issued unconditionally, so the compiler knows how
        //                 many are in flight and waits for exactly what it needs.  Best for
        //                 large or ragged tiles (+5-19 % over the other form).
        //   LOADS_FIRST   the loads sit in a conditional block ahead of the stores (without
        //                 the branch the compiler sinks them below the stores: nothing ties
        //                 the two together), and the workgroup ends up waiting for most of
        //                 its previous stores before it touches the next tile.  That
        //                 throttle is worth +3-5 % on small line-aligned tiles whose
        //                 neighbours read other lines of the same rows (measured on the
        //                 96^4 set); explicit waits in the other form did not reproduce it.
        // After the last tile the stores-first form issues the reads all the same, with
        // every lane dropped (nxt then has remaining extents 0).
        auto issue_next_loads = [&]() { load_tile(nxt); };
        if (USE_LDS) {
            // with two LDS images the tiles alternate between them and one barrier per
            // tile is enough: a wave can only overwrite an image two tiles later, after
            // the barrier of the tile in between
            lds_t* img = lds + ((two_buffers && (it & 1u)) ? lds_elems : 0u);
#pragma unroll
            for (int j = 0; j < NREG; ++j)
                if (read_ok(j, pos)) {
                    if constexpr (VEC2) {
                        // neighbours along input dim 0 are neighbours in the image
                        if constexpr (sizeof(T) == 4) {
                            img[lds_pos[j] & 0xFFFFu] = v[j].x;
                            if (!odd_row_end(pos) || read_ok_second(j, pos))
                                img[(lds_pos[j] & 0xFFFFu) + 1u] = v[j].y;
                        } else {
                            img[lds_pos[j] & 0xFFFFu] = lds_t{v[j].x, v[j].y};
                            img[(lds_pos[j] & 0xFFFFu) + 1u] = lds_t{v[j].z, v[j].w};
                        }
                    } else {
                        img[lds_pos[j] & 0xFFFFu] = v[j];
                    }
                }
            __syncthreads();
            if (ALIGN) {
#pragma unroll
                for (int j = 0; j < NREG; ++j) {
                    const uint32_t at = (lds_pos[j] >> 16) - row_shift(j) * oa.lstride_b;
                    if constexpr (PAIRWIN) {
                        // both elements of the pair lie inside the image whenever the row does
                        if ((wr_mask[j] & 0xFFFFu) < pos.rem_a) {
                            w[j].x = img[at];
                            w[j].y = img[at + oa.lstride_b];
                        }
                    } else if constexpr (!VEC2) {
                        if (write_at(j) != kDroppedOffset) w[j] = img[at];
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < NREG; ++j)
                    if (write_at(j) != kDroppedOffset) {
                        if constexpr (VEC2) {
                            // neighbours along output dim 0 are pair_lstride apart
                            if constexpr (sizeof(T) == 4) {
                                w[j].x = img[lds_pos[j] >> 16];
                                w[j].y = img[(lds_pos[j] >> 16) + pair_lstride];
                            } else {
                                const lds_t lo = img[lds_pos[j] >> 16];
                                const lds_t hi = img[(lds_pos[j] >> 16) + pair_lstride];
                                w[j] = reg_t{lo.x, lo.y, hi.x, hi.y};
                            }
                        } else {
                            w[j] = img[lds_pos[j] >> 16];
                        }
                    }
            }
        } else {
#pragma unroll
            for (int j = 0; j < NREG; ++j) w[j] = v[j];
        }
        if (LOADS_FIRST) {
            // under a branch on purpose: a conditional block is what keeps the compiler from
            // sinking these loads below the stores
            if (bn < walk.num_tiles) issue_next_loads();
        }
        uint32_t soff_out;
        const __amdgpu_buffer_rsrc_t rsrc_out = reach(rsrc_out_whole, out_origin, pos.out, &soff_out);
        if (ACC) {
            // out = out + transposed in: fetch the old output values (all loads first), add
            reg_t old[NREG];
#pragma unroll
            for (int j = 0; j < NREG; ++j)
                old[j] = io::load(rsrc_out, write_at(j), soff_out);
#pragma unroll
            for (int j = 0; j < NREG; ++j) w[j] = io::add(old[j], w[j]);
        }
        bool stored = false;
        if constexpr (PAIRWIN) {
            // a window clipped by the ends of its output row: element by element
            if (pos.lo_b != 0u || pos.rem_b != walk.split_tile[1]) {
#pragma unroll
                for (int j = 0; j < NREG; ++j) {
                    const uint32_t sh = row_shift(j);
                    const uint32_t xb = (wr_aux[j] & 0xFFFFu) - sh;
                    const bool row_ok = (wr_mask[j] & 0xFFFFu) < pos.rem_a;
                    const uint32_t at = wr_off[j] - sh * (uint32_t)sizeof(T);
                    io1::store(w[j].x, rsrc_out, row_ok && (xb - pos.lo_b) < pos.span_b ? at : kDroppedOffset, soff_out);
                    io1::store(w[j].y, rsrc_out, row_ok && (xb + 1u - pos.lo_b) < pos.span_b ? at + 4u : kDroppedOffset, soff_out);
                }
                stored = true;
            }
        }
        if (!stored) {
#pragma unroll
            for (int j = 0; j < NREG; ++j) io::store(w[j], rsrc_out, write_at(j), soff_out);
        }
        if (!LOADS_FIRST) issue_next_loads();
        b = bn;
        pos = nxt;
        ++it;
        bn = tile_of(walk, block, grid, it + 1);
        nxt = no_tile;
        if (bn < walk.num_tiles) nxt = major_position(walk, ml, bn);
        if (USE_LDS && !two_buffers) __syncthreads();  // all waves are done reading the image
    }
}

// Kernel pointer for one element type and workgroup size; nullptr if the combination is
// not instantiated.  Accumulating kernels (ACC) exist for 256 threads, cached policy.
template <typename T, int THREADS, bool USE_LDS, int NT, bool ALIGN, bool ACC, bool LOADS_FIRST = false, bool VEC2 = false, bool BIG = false>
static const void* tile_kernel_ptr(int nreg) {
    switch (nreg) {
#define TPERM_CASE(N) \
    case N:           \
        return reinterpret_cast<const void*>(&tile_kernel<T, N, THREADS, USE_LDS, NT, ALIGN, ACC, LOADS_FIRST, VEC2, BIG>);
        TPERM_CASE(4)
        TPERM_CASE(8)
        TPERM_CASE(12)
        TPERM_CASE(16)
        TPERM_CASE(24)
        TPERM_CASE(32)
        default:
            break;
    }
    if constexpr (THREADS == 256) {
        switch (nreg) {
            TPERM_CASE(1)
            TPERM_CASE(2)
            TPERM_CASE(3)
            TPERM_CASE(6)
            default:
                break;
        }
    }
#undef TPERM_CASE
    return nullptr;
}

// nt: 0 = cached, 1 = nontemporal stores, 2 = nontemporal loads and stores, 3 = nontemporal
// loads.  The 64-thread variants exist for policies 0 and 2 only (1 runs as 2).
// loads_first: order of the next tile's loads and this tile's stores (see the kernel); both
// orders exist for the plain 256-thread kernels, elsewhere stores go first.
template <typename T, int THREADS>
static const void* tile_kernel_select(int nreg, bool use_lds, int nt, bool align, bool acc,
                                      bool loads_first, bool vec2) {
    if constexpr (THREADS == 256) {
        if (vec2 && align) {
            // pairs of 4-byte elements in line-aligned windows
            if constexpr (sizeof(T) == 4) {
                if (!use_lds || acc) return nullptr;
                switch (nt) {
                    case 0: return tile_kernel_ptr<T, 256, true, 0, true, false, false, true>(nreg);
                    case 1: return tile_kernel_ptr<T, 256, true, 1, true, false, false, true>(nreg);
                    case 2: return tile_kernel_ptr<T, 256, true, 2, true, false, false, true>(nreg);
                    default: return tile_kernel_ptr<T, 256, true, 3, true, false, false, true>(nreg);
                }
            } else {
                return nullptr;
            }
        }
        if (nt == 3) {
            // nontemporal loads only: plain stores-first forms
            if (acc || loads_first) return nullptr;
            if (vec2) return use_lds && !align ? tile_kernel_ptr<T, 256, true, 3, false, false, false, true>(nreg) : nullptr;
            if (align) return use_lds ? tile_kernel_ptr<T, 256, true, 3, true, false>(nreg) : nullptr;
            return use_lds ? tile_kernel_ptr<T, 256, true, 3, false, false>(nreg)
                           : tile_kernel_ptr<T, 256, false, 3, false, false>(nreg);
        }
        // pairs of elements: LDS-staged, stores first
        if (vec2) {
            if (!use_lds || align || acc) return nullptr;
            if (nt == 1) return tile_kernel_ptr<T, 256, true, 1, false, false, false, true>(nreg);
            return nt != 0 ? tile_kernel_ptr<T, 256, true, 2, false, false, false, true>(nreg)
                           : tile_kernel_ptr<T, 256, true, 0, false, false, false, true>(nreg);
        }
    }
    if (vec2) return nullptr;
    if constexpr (THREADS == 256) {
        if (align && !use_lds) return nullptr;
        if (acc) {
            if (nt != 0) return nullptr;
            if (align) return tile_kernel_ptr<T, 256, true, 0, true, true>(nreg);
            return use_lds ? tile_kernel_ptr<T, 256, true, 0, false, true>(nreg)
                           : tile_kernel_ptr<T, 256, false, 0, false, true>(nreg);
        }
        if (align) {
            if (nt == 1) return tile_kernel_ptr<T, 256, true, 1, true, false>(nreg);
            return nt != 0 ? tile_kernel_ptr<T, 256, true, 2, true, false>(nreg)
                           : tile_kernel_ptr<T, 256, true, 0, true, false>(nreg);
        }
        if (loads_first) {
            if (nt == 1)
                return use_lds ? tile_kernel_ptr<T, 256, true, 1, false, false, true>(nreg)
                               : tile_kernel_ptr<T, 256, false, 1, false, false, true>(nreg);
            if (use_lds)
                return nt != 0 ? tile_kernel_ptr<T, 256, true, 2, false, false, true>(nreg)
                               : tile_kernel_ptr<T, 256, true, 0, false, false, true>(nreg);
            return nt != 0 ? tile_kernel_ptr<T, 256, false, 2, false, false, true>(nreg)
                           : tile_kernel_ptr<T, 256, false, 0, false, false, true>(nreg);
        }
        if (nt == 1)
            return use_lds ? tile_kernel_ptr<T, 256, true, 1, false, false>(nreg)
                           : tile_kernel_ptr<T, 256, false, 1, false, false>(nreg);
    } else {
        if (acc || align) return nullptr;
    }
    if (use_lds)
        return nt != 0 ? tile_kernel_ptr<T, THREADS, true, 2, false, false>(nreg)
                       : tile_kernel_ptr<T, THREADS, true, 0, false, false>(nreg);
    return nt != 0 ? tile_kernel_ptr<T, THREADS, false, 2, false, false>(nreg)
                   : tile_kernel_ptr<T, THREADS, false, 0, false, false>(nreg);
}

}  // namespace tperm
