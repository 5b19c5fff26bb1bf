// Analytical performance estimate of a tile plan: the structure of the paper's Section 2.3
// (Eqs. (10)-(13): cycles = (cycles_mem + cycles_shmem + cycles_ac) * N_iter, with the
// memory term driven by the number of transactions per request and stores to partially
// written cache lines counted double), evaluated with constants for MI355X instead of the
// paper's NVIDIA ones.
//
// The counts are exact, not fitted: a sample of tiles is walked with the very index
// arithmetic the kernel runs (tperm_desc.h), every element a tile reads or writes is mapped to
// its 128-byte line, and the distinct lines, and for the write side the bytes each line
// receives, are tallied.  Pure host code.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "plan.hpp"

namespace tperm {

namespace {

// MI355X (gfx950) parameters of the model, the counterpart of the paper's Table I.
// Published: 256 compute units, 2.4 GHz, 8 TB/s.  Measured on the chip with the pointer-chasing
// probe that ships beside this file (latency_probe.hip): a wave-wide load of lines that sit in
// HBM returns after 1080 cycles on an idle machine; a single wave gets a further independent
// four-line request under way every 40 cycles, and a whole compute unit with 32 KiB or more in
// flight takes a line every 5 cycles (26 bytes per cycle), which is the departure delay of a
// compute unit; a dependent LDS load takes 64-68 cycles.  Estimated: ~300 cycles of address
// arithmetic, waits and barriers per tile.
constexpr double kFreq = 2.4e9;
constexpr double kNumCU = 256.0;
constexpr double kMemBW = 8.0e12;
constexpr double kBaseLat = 1080.0;
constexpr double kDelta = 5.0;
constexpr double kLdsLat = 66.0;
constexpr double kCyclesAc = 300.0;
constexpr double kLine = 128.0;
constexpr uint32_t kModelSamples = 16;

// Bytes each touched line receives: a small open-addressing table keyed by line number.
struct LineTally {
    std::vector<uint64_t> key;
    std::vector<uint32_t> bytes;
    uint32_t mask;
    explicit LineTally(uint32_t capacity_log2) : key(1u << capacity_log2, ~0ull), bytes(1u << capacity_log2, 0), mask((1u << capacity_log2) - 1u) {}
    void clear() {
        std::fill(key.begin(), key.end(), ~0ull);
        std::fill(bytes.begin(), bytes.end(), 0u);
    }
    void add(uint64_t byte_begin, uint32_t nbytes) {
        while (nbytes > 0) {
            const uint64_t line = byte_begin / 128u;
            const uint32_t room = (uint32_t)((line + 1) * 128u - byte_begin);
            const uint32_t take = nbytes < room ? nbytes : room;
            uint32_t h = (uint32_t)((line * 0x9E3779B97F4A7C15ull) >> 40) & mask;
            while (key[h] != ~0ull && key[h] != line) h = (h + 1) & mask;
            key[h] = line;
            bytes[h] += take;
            byte_begin += take;
            nbytes -= take;
        }
    }
    bool has(uint64_t line) const {
        uint32_t h = (uint32_t)((line * 0x9E3779B97F4A7C15ull) >> 40) & mask;
        while (key[h] != ~0ull) {
            if (key[h] == line) return true;
            h = (h + 1) & mask;
        }
        return false;
    }
    // runs: maximal ranges of consecutive touched lines
    void count(double* lines, double* full, double* part, double* runs) const {
        for (size_t i = 0; i < key.size(); ++i)
            if (key[i] != ~0ull) {
                *lines += 1.0;
                if (bytes[i] >= 128u) *full += 1.0;
                else *part += 1.0;
                if (key[i] == 0 || !has(key[i] - 1)) *runs += 1.0;
            }
    }
};

}  // namespace

tperm_status_t model_plan(const Plan& plan, tperm_model_t* out) {
    std::memset(out, 0, sizeof(*out));
    if (plan.kclass != TPERM_KERNEL_ROWCOPY && plan.kclass != TPERM_KERNEL_TILED && plan.kclass != TPERM_KERNEL_PACKED)
        return TPERM_ERR_KERNEL;
    const TileDesc& d = plan.tile;
    const uint32_t elem = (uint32_t)plan.elem;
    const uint32_t per_slot = d.vec2 ? 2u : 1u;  // elements moved by one slot
    const OutAlign& oa = d.oa;
    const bool windows = plan.use_lds && oa.enabled != 0u;
    LineTally rd(15), wr(15);  // up to 8192 slots of up to 16 bytes: at most 2 lines each
    // Tiles are sampled, as in the paper; one per equal stretch of the tile index, at a position
    // inside the stretch that moves by the golden ratio from one stretch to the next, so the
    // samples do not fall in step with the period of any tile counter.
    const uint32_t n_samples = std::min<uint32_t>(d.num_tiles, kModelSamples);
    double ld_lines = 0, st_lines = 0, st_full = 0, st_part = 0, useful = 0, existing = 0, dummy1 = 0, dummy2 = 0, ld_runs = 0, st_runs = 0;
    for (uint32_t s = 0; s < n_samples; ++s) {
        uint32_t b = s;
        if (d.num_tiles > n_samples) {
            const double inside = std::fmod(0.5 + 0.6180339887498949 * (double)s, 1.0);
            b = std::min<uint32_t>(d.num_tiles - 1u, (uint32_t)(((double)s + inside) * (double)d.num_tiles / (double)n_samples));
        }
        uint64_t maj_in = 0, maj_out = 0;
        uint32_t coord[TPERM_DESC_MAX_DIMS];
        for (uint32_t l = 0; l < TPERM_DESC_MAX_DIMS; ++l) {
            coord[l] = major_coord(d.major, l, b);
            maj_in += (uint64_t)coord[l] * d.major.stride_in[l];
            maj_out += (uint64_t)coord[l] * d.major.stride_out[l];
        }
        uint32_t rem_a = 0, rem_b = 0, lo_b = 0;
        tile_remaining(d, [&](uint32_t l) { return coord[l]; }, &rem_a, &rem_b, &lo_b);
        if (rem_a == 0u || rem_b == 0u) continue;  // a combination of split counters that does not exist
        existing += 1.0;
        const uint32_t span_b = rem_b > lo_b ? rem_b - lo_b : 0u;
        rd.clear();
        wr.clear();
        double elems = 0;
        if (plan.use_lds) {
            for (uint32_t k = 0; k < d.tile_vol; ++k) {
                const Slot sl = tile_slot(d.in_order, d.n_tile_dims, k);
                const bool ok = windows ? (sl.xa < rem_a && (sl.xb - lo_b) < span_b) : (sl.xa < rem_a && sl.xb < rem_b);
                if (!ok) continue;
                const int64_t gi = (int64_t)maj_in + (int64_t)sl.goff - (windows ? (int64_t)oa.in_halo_elems : 0);
                if (gi < 0) continue;
                rd.add((uint64_t)gi * elem, per_slot * elem);
            }
            const uint32_t wslots = windows ? oa.total_slots : d.tile_vol;
            for (uint32_t k = 0; k < wslots; ++k) {
                const Slot so = tile_slot(d.out_order, d.n_tile_dims, k);
                if (windows) {
                    // every row writes a window shifted down to a line boundary (output base
                    // pointer taken as line-aligned): the same bytes, moved by the row's phase
                    const uint32_t p = so.xb;
                    const uint32_t rho = (so.goff - p) & (oa.line_elems - 1u);
                    const uint32_t shift = (uint32_t)((maj_out + rho) & (oa.line_elems - 1u));
                    const uint32_t xb = p + oa.line_elems - shift;
                    if (!(so.xa < rem_a && (xb - lo_b) < span_b)) continue;
                    const int64_t go = (int64_t)maj_out + (int64_t)so.goff - (int64_t)shift;
                    if (go < 0) continue;
                    wr.add((uint64_t)go * elem, per_slot * elem);
                    elems += per_slot;
                } else {
                    if (!(so.xa < rem_a && so.xb < rem_b)) continue;
                    wr.add((maj_out + so.goff) * elem, per_slot * elem);
                    elems += per_slot;
                }
            }
        } else {
            for (uint32_t k = 0; k < d.tile_vol; ++k) {
                const Slot so = tile_slot(d.out_order, d.n_tile_dims, k);
                if (!(so.xa < rem_a && so.xb < rem_b)) continue;
                rd.add((maj_in + so.ooff) * elem, elem);
                wr.add((maj_out + so.goff) * elem, elem);
                elems += 1.0;
            }
        }
        rd.count(&ld_lines, &dummy1, &dummy2, &ld_runs);
        wr.count(&st_lines, &st_full, &st_part, &st_runs);
        useful += elems * elem;
    }
    if (existing == 0.0 || useful == 0.0) return TPERM_ERR_INTERNAL;
    const double waves = (double)plan.threads / 64.0;
    // Ratio estimate: the sample gives lines per useful byte; the bytes an average tile index
    // carries are known exactly (all tile indices together write the tensor once, the
    // combinations of split counters that do not exist write nothing).  Ragged tiles that the
    // sample over- or under-represents then do not shift the totals.
    double volume = 1.0;
    for (int i = 0; i < plan.rank; ++i) volume *= (double)plan.dims[i];
    const double bytes_per_tile = volume * (double)elem / (double)d.num_tiles;
    const double per_byte = bytes_per_tile / useful;
    out->ld_tran = ld_lines * per_byte;
    out->st_tran = st_lines * per_byte;
    out->cl_full = st_full * per_byte;
    out->cl_part = st_part * per_byte;
    out->useful_bytes_per_tile = bytes_per_tile;
    // one request = one wave-wide memory instruction; a thread issues nreg loads and nreg stores per tile
    out->ld_req = out->st_req = (double)plan.nreg * waves;
    const double part_frac = out->cl_part / std::max(1.0, out->cl_full + out->cl_part);
    out->ld_runs = ld_runs * per_byte;
    out->st_runs = st_runs * per_byte;
    out->tpr_mem = (out->ld_tran + out->st_tran * (1.0 + part_frac)) / (out->ld_req + out->st_req);  // Eq. (13)
    out->mem_lat = kBaseLat + std::max(0.0, out->tpr_mem - 1.0) * kDelta;
    out->mlp = (double)plan.nreg;  // independent requests per wave per iteration (the paper's nReg for Packed)
    // resident workgroups per compute unit: the plan's cap (the occupancy limit is not known on the host)
    const double wg_per_cu = (double)std::max(1, plan.blocks_per_cu);
    const double waves_per_cu = waves * wg_per_cu;
    const double bytes_req = out->tpr_mem * kLine;  // streamed once: no cache hits assumed
    const double bw_wave = kFreq * bytes_req / out->mem_lat;
    const double mwp_peak = kMemBW / (bw_wave * kNumCU);
    const double mwp_mem = out->mem_lat / kDelta;
    // A wave keeps all its nreg requests of a tile in flight at once (the hardware counts up to
    // 63 outstanding vector memory instructions per wave), so the occupancy cap is in requests,
    // waves * MLP, where the paper has the number of resident warps.
    out->mwp = std::min(std::min(mwp_mem * out->mlp, mwp_peak), waves_per_cu * out->mlp);
    // all resident workgroups of a compute unit advance one tile each per iteration
    out->cycles_mem = 2.0 * out->mem_lat * out->mlp * waves_per_cu / std::max(out->mwp, 1e-9);  // Eq. (11)
    out->tpr_lds = 1.0;
    if (plan.use_lds) {
        // bank conflicts of the first wave-wide accesses, from the slot positions of Eq. (6)
        out->tpr_lds = std::max(1.0, lds_conflict_ratio(d, plan.elem, plan.nreg, plan.threads));
        out->cycles_lds = 2.0 * out->tpr_lds * kLdsLat * out->mlp;
    }
    out->cycles_ac = kCyclesAc;
    out->n_iter = std::ceil((double)d.num_tiles / (kNumCU * wg_per_cu));
    out->cycles_total = (out->cycles_mem + out->cycles_lds + out->cycles_ac) * out->n_iter;  // Eq. (10)
    out->microseconds = out->cycles_total / kFreq * 1e6;
    return TPERM_OK;
}

}  // namespace tperm
