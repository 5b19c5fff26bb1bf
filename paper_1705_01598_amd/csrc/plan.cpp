// Host-side planner.  See plan.hpp.
#include "plan.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

namespace tperm {

// keep in step with the instantiation lists in kernels.hip
static const int kNregSet256[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
static const int kNregSet64[] = {4, 8, 12, 16, 24, 32};

int pick_nreg(int64_t tile_vol, int threads) {
    const int64_t need = (tile_vol + threads - 1) / threads;
    const int* set = threads == 64 ? kNregSet64 : kNregSet256;
    const int n = threads == 64 ? (int)(sizeof(kNregSet64) / sizeof(int))
                                : (int)(sizeof(kNregSet256) / sizeof(int));
    for (int i = 0; i < n; ++i)
        if (set[i] >= need) return set[i];
    return -1;
}

// ---------------------------------------------------------------------------------------
// validation and canonical form
// ---------------------------------------------------------------------------------------

tperm_status_t validate(int rank, const int64_t* dims, const int* perm, size_t elem) {
    if (dims == nullptr || perm == nullptr) return TPERM_ERR_NULL;
    if (rank < 1 || rank > TPERM_MAX_RANK) return TPERM_ERR_RANK;
    if (elem != 4 && elem != 8) return TPERM_ERR_ELEM_SIZE;
    bool seen[TPERM_MAX_RANK] = {false};
    for (int j = 0; j < rank; ++j) {
        if (perm[j] < 0 || perm[j] >= rank || seen[perm[j]]) return TPERM_ERR_PERM;
        seen[perm[j]] = true;
    }
    int64_t vol = 1;
    for (int z = 0; z < rank; ++z) {
        if (dims[z] < 1) return TPERM_ERR_DIMS;
    }
    for (int z = 0; z < rank; ++z) {
        if (dims[z] >= ((int64_t)1 << 31)) return TPERM_ERR_TOO_LARGE;
        vol *= dims[z];
        if (vol >= ((int64_t)1 << 31)) return TPERM_ERR_TOO_LARGE;
    }
    return TPERM_OK;
}

// Drop extent-1 dims, then fuse input dims z, z+1 that sit next to each other and in the
// same order in the output: such a pair moves as one dimension of extent d(z)*d(z+1).
// Neither step changes where any element goes.
void canonicalise(int rank, const int64_t* dims, const int* perm, Canonical* out) {
    // output order without extent-1 dims
    int ord[TPERM_MAX_RANK];
    int n = 0;
    for (int j = 0; j < rank; ++j)
        if (dims[perm[j]] > 1) ord[n++] = perm[j];
    Canonical c;
    c.volume = 1;
    for (int z = 0; z < rank; ++z) c.volume *= dims[z];
    if (n == 0) {
        c.rank = 1;
        c.dims[0] = 1;
        c.perm[0] = 0;
        *out = c;
        return;
    }
    // groups of output positions whose input dims are consecutive among the kept dims
    // (kept dims are consecutive if no kept dim lies strictly between them)
    bool kept[TPERM_MAX_RANK] = {false};
    for (int j = 0; j < n; ++j) kept[ord[j]] = true;
    auto next_kept = [&](int z) {
        for (int t = z + 1; t < rank; ++t)
            if (kept[t]) return t;
        return -1;
    };
    int group_first[TPERM_MAX_RANK];  // first input dim of each group, in output order
    int64_t group_ext[TPERM_MAX_RANK];
    int g = 0;
    for (int j = 0; j < n;) {
        int first = ord[j];
        int64_t ext = dims[first];
        int last = first;
        int jj = j + 1;
        while (jj < n && ord[jj] == next_kept(last)) {
            last = ord[jj];
            ext *= dims[last];
            ++jj;
        }
        group_first[g] = first;
        group_ext[g] = ext;
        ++g;
        j = jj;
    }
    // new input order = groups sorted by their first input dim
    int idx[TPERM_MAX_RANK];
    for (int i = 0; i < g; ++i) idx[i] = i;
    std::sort(idx, idx + g, [&](int a, int b) { return group_first[a] < group_first[b]; });
    int new_id[TPERM_MAX_RANK];  // group (output order) -> canonical input dim
    for (int z = 0; z < g; ++z) {
        new_id[idx[z]] = z;
        c.dims[z] = group_ext[idx[z]];
    }
    for (int j = 0; j < g; ++j) c.perm[j] = new_id[j];
    c.rank = g;
    *out = c;
}

FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    if (d == 0) d = 1;
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    f.shift = 31 + l;
    const uint64_t pow = (uint64_t)1 << f.shift;
    f.magic = (uint32_t)((pow + d - 1) / d);
    return f;
}

// ---------------------------------------------------------------------------------------
// candidate tiles
// ---------------------------------------------------------------------------------------

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

static int64_t gcd64(int64_t a, int64_t b) {
    while (b) {
        int64_t t = a % b;
        a = b;
        b = t;
    }
    return a;
}


// Fill the derived fields of a candidate from its tile extents; false if unusable.
static bool finish_candidate(const Canonical& c, int elem, Candidate* cd) {
    const int r = c.rank;
    int inv[TPERM_MAX_RANK];
    for (int j = 0; j < r; ++j) inv[c.perm[j]] = j;
    int64_t sI[TPERM_MAX_RANK], sO[TPERM_MAX_RANK];
    sI[0] = 1;
    for (int z = 1; z < r; ++z) sI[z] = sI[z - 1] * c.dims[z - 1];
    sO[0] = 1;
    for (int j = 1; j < r; ++j) sO[j] = sO[j - 1] * c.dims[c.perm[j - 1]];

    int splits = 0;
    int64_t vol = 1, tiles = 1;
    double util = 1.0;
    int n_tile_dims = 0, n_outer = 0;
    for (int z = 0; z < r; ++z) {
        const int64_t t = cd->t[z], d = c.dims[z];
        if (t < 1 || t > d) return false;
        if (t > 1) {
            vol *= t;
            ++n_tile_dims;
        }
        if (t < d) {
            const int64_t n = ceil_div(d, t);
            tiles *= n;
            util *= (double)d / (double)(n * t);
            if (t > 1) ++splits; else ++n_outer;
        }
        if (t > 0x7FFF) return false;
    }
    if (n_tile_dims == 0) return false;
    if (splits > 2) return false;
    if (splits + n_outer > TPERM_DESC_MAX_DIMS) return false;
    if (vol > kMaxTileVol) return false;
    if (tiles >= ((int64_t)1 << 31)) return false;
    // contiguous run on the input side: leading dims, all but the last at full extent
    int64_t run_in = 1;
    for (int z = 0; z < r; ++z) {
        run_in *= cd->t[z];
        if (cd->t[z] < c.dims[z]) break;
    }
    int64_t run_out = 1;
    for (int j = 0; j < r; ++j) {
        const int z = c.perm[j];
        run_out *= cd->t[z];
        if (cd->t[z] < c.dims[z]) break;
    }
    cd->tile_vol = vol;
    cd->num_tiles = tiles;
    cd->run_in = run_in;
    cd->run_out = run_out;
    cd->utilisation = util;
    // the LDS image must fit with room left for the bank-conflict padding
    if (cd->use_lds && vol * elem > kMaxLdsBytes - 8192) return false;

    // Alignment granule of run starts on each side: every stride that separates two runs
    // (the strides of all dims other than the run's own leading dims, and the chunk step
    // of a split leading dim) is a multiple of it.
    auto granule = [&](bool input) {
        int64_t g = 128;
        bool in_run = true;
        for (int p = 0; p < r; ++p) {
            const int z = input ? p : c.perm[p];
            const int64_t stride = (input ? sI[p] : sO[p]) * elem;
            if (in_run) {
                if (cd->t[z] < c.dims[z]) {
                    // split (or outer) dim ends the run; its chunks start t*stride apart
                    g = gcd64(g, stride * cd->t[z]);
                    in_run = false;
                }
            } else {
                g = gcd64(g, stride);
            }
        }
        return (double)g;
    };
    const double rin = (double)(cd->use_lds ? run_in : cd->t[0]) * elem;
    const double rout = (double)run_out * elem;
    double gin = granule(true), gout = granule(false);
    // Line-aligned output windows: the leading output dim is cut into chunks of whole lines
    // and every row shifts its window to line boundaries, at the price of a halo of one
    // line's worth of coordinates on the read side.  Only where rows are misaligned.
    const int q0 = c.perm[0];
    const int64_t line_elems = 128 / elem;
    int64_t read_vol = vol;
    if (cd->align) {
        // Not when the shifted dim is itself part of the input run (the halo then lengthens
        // the rows read; measured: such candidates win in 5 % of the cases, by 5 %).
        bool q0_in_input_run = true;  // all dims in front of it are taken whole
        for (int z = 0; z < q0; ++z) q0_in_input_run = q0_in_input_run && cd->t[z] == c.dims[z];
        if (!cd->use_lds || q0 == 0 || q0_in_input_run || cd->k != 1 || cd->t[q0] >= c.dims[q0] ||
            cd->t[q0] % line_elems != 0 || gout >= 128.0)
            return false;
        // 4-byte elements only where the kernel can move them in pairs (see build_tile_plan),
        // and not when the input rows are line-aligned: plain tiles with nontemporal loads
        // then win 8 times out of 10, by 15 % on average (measured on every candidate of 14 such
        // shapes; 8-byte elements are undecided there: windows win on large matrices, lose on
        // shapes with a short leading output dim, and stay as they are)
        if (elem == 4 && !(cd->t[0] % 2 == 0 && (c.dims[0] % 2 == 0 || cd->t[0] < c.dims[0]))) return false;
        if (elem == 4 && gin >= 128.0 && std::fmod(rin, 128.0) == 0.0) return false;
        read_vol = vol / cd->t[q0] * (cd->t[q0] + line_elems);
        // the shifted windows need chunks for d + L - 1 coordinates, not d: with a short leading
        // output dim that is one chunk more out of a few
        util *= (double)ceil_div(c.dims[q0], cd->t[q0]) /
                (double)ceil_div(c.dims[q0] + line_elems - 1, cd->t[q0]);
        // beyond 16 slots (of pairs, for 4-byte elements, as long as the single-element form
        // still exists) the kernel's registers allow one workgroup per CU only
        if (read_vol > (elem == 4 ? 24 : 16) * TPERM_MAX_THREADS) return false;
        if (read_vol * elem > kMaxLdsBytes - 8192) return false;
        gout = 128.0;
    }
    if (!cd->use_lds) {
        // rows are read in output-lane order: contiguous only along dim 0
        gin = (double)gcd64(128, (r > 1 ? sI[1] : 1) * elem);
        if (cd->t[0] < c.dims[0]) gin = (double)gcd64((int64_t)gin, cd->t[0] * elem);
    }
    // Cost per useful byte on each side: 128-byte lines touched per line's worth of useful
    // data, plus a fixed per-run overhead.  The constants were fitted on MI355X to the
    // measured times of every candidate of ~220 benchmark cases (half held out: the fit
    // picks plans within 2 % of the best candidate on average on the held-out half):
    // output runs keep paying off up to a few KiB (overhead worth 128 bytes, misalignment
    // weighted 2x: a partially written line costs more than a partially read one, cf.
    // Eq. (13)), input runs are flat from 128 bytes on (overhead worth 16 bytes).
    // (the LDS-free row copy reads its rows one by one: misaligned short rows weigh double
    // there; measured over all candidates of the 125 benchmark cases that keep dim 0 in front)
    const bool al4 = cd->align && elem == 4;
    double cost_in = (rin + (cd->align ? (al4 ? kAlign4InOverhead : kAlignInOverhead) : 16.0) + (cd->use_lds ? 0.5 : 1.0) * (128.0 - gin)) / rin;
    if (rin < 128.0) cost_in += (128.0 - rin) / 64.0;  // below one line per run reads collapse
    if (cd->align)
        cost_in *= 1.0 + (al4 ? kAlign4HaloWeight : kAlignHaloWeight) *
                             std::pow((double)line_elems / (double)cd->t[q0], al4 ? kAlign4HaloPower : kAlignHaloPower);
    const double cost_out = (rout + (cd->align ? (al4 ? kAlign4OutOverhead : kAlignOutOverhead) : 128.0) + 2.0 * (128.0 - gout)) / rout;
    double cost = (cost_in + cost_out) / util;
    // Tile size, by slots per thread of a 256-thread workgroup: a table fitted with the rest.
    // Three to eight slots are the sweet spot (enough loads in flight per wave, several
    // workgroups per compute unit); a single slot cannot keep enough bytes in flight, and
    // beyond twelve slots fewer workgroups fit and LDS padding runs out of room.  4-byte
    // elements moved singly want more slots: their tiles are half the bytes (table smoothed
    // by hand from a fit over every candidate of 230 4-byte cases; both halves of the sample
    // gain 1 % over the flatter table used before).
    static const int kSlots[10] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32};
    static const double kWeight8[10] = {1.4, 1.05, 0.95, 0.95, 1.1, 1.0, 1.06, 1.1, 1.16, 1.2};
    static const double kWeight4[10] = {1.4, 1.2, 0.85, 0.85, 0.8, 0.85, 0.9, 1.0, 1.1, 1.2};
    // The LDS-free row copy keeps few registers per slot and has no barrier: four to six
    // slots do better there than the LDS-staged table says when they come from more rows
    // (measured on every candidate of the benchmark cases that keep dim 0 in front; making a
    // single row longer instead loses 1-5 %).
    static const double kWeightRc[10] = {1.4, 1.05, 0.95, 0.9, 0.9, 1.0, 1.06, 1.1, 1.16, 1.2};
    // A 4-byte candidate that can move its elements in pairs (see build_tile_plan) has half
    // the slots and behaves like the 8-byte kernel of the same tile bytes.
    const bool pairable = cd->use_lds && !cd->align && q0 != 0 && c.dims[0] % 2 == 0 &&
                          c.dims[q0] % 2 == 0 && cd->t[0] % 2 == 0 && cd->t[q0] % 2 == 0;
    const bool pairs = elem == 4 && pairable;
    // 8-byte elements in pairs (16-byte accesses) where every run starts and ends on a line
    // boundary: half the memory instructions per byte, and the sweet spot moves to tiles of
    // 16 KiB (four pair slots per thread).  Table fitted to the measured times of every
    // candidate of 50 line-aligned 8-byte problems of 16 MiB to 680 MiB (squares, cubes,
    // power-of-two and 48^4 / 96^4 tensors), with and without pairs: picks +3 % on the
    // mid-size ones, +0.4 % on the 96^4 set; ragged shapes keep single elements in the score
    // (their pairs run where possible, measured neutral).
    const bool line_aligned = gin >= 128.0 && gout >= 128.0 && std::fmod(rin, 128.0) == 0.0 &&
                              std::fmod(rout, 128.0) == 0.0;
    const bool pairs8 = elem == 8 && pairable && line_aligned;
    static const double kWeight8Pairs[10] = {1.4, 0.85, 0.9, 0.8, 1.0, 1.0, 1.06, 1.1, 1.16, 1.2};
    const bool window_pairs = elem == 4 && cd->align;
    const int64_t slots_needed = (pairs || pairs8) ? vol / 2 : (window_pairs ? read_vol / 2 : read_vol);
    const int64_t need = (slots_needed + TPERM_MAX_THREADS - 1) / TPERM_MAX_THREADS;
    int bucket = 9;
    for (int i = 0; i < 10; ++i)
        if (kSlots[i] >= need) {
            bucket = i;
            break;
        }
    cost *= (!cd->use_lds && n_tile_dims >= 2 ? kWeightRc : (pairs8 ? kWeight8Pairs : (elem == 4 && !pairs && !window_pairs ? kWeight4 : kWeight8)))[bucket];
    // A tile that does not fill the 256 lanes of its workgroup wastes the rest of them.
    if (need == 1) cost /= std::pow((double)slots_needed / TPERM_MAX_THREADS, 0.75);
    // Pipeline fill and drain: a persistent workgroup spends about four tile times without
    // overlap, which matters when it only gets a few tiles.
    const double bytes = (double)vol * elem;
    const double wg_per_cu =
        std::max(2.0, std::min(8.0, std::round((cd->use_lds ? 20480.0 : 14336.0) / bytes)));
    const double rounds = (double)tiles / (256.0 * wg_per_cu);
    cost *= 1.0 + 4.0 / std::max(rounds, 4.0);
    // Rows a large power of two apart land in the same memory channels: when the pitch of the
    // rows a tile reads (the input stride of its first dim beyond the input run) is a multiple
    // of 8 KiB, more than 32 of them per tile cost.  A rule about the pitch, whatever the
    // tensor: with it the 96^4 permutations (pitches 2^13 * 9 and 2^18 * 27 bytes) run 1.7 %
    // faster as a set (32 x 32 tiles replace 32 x 96 ones there although their output runs are
    // short), the power-of-two fp32 set and the ragged rank sweep are unchanged (same-box A/B).
    if (cd->use_lds && !cd->align) {
        int z = 0;
        while (z < r) {  // skip the input run
            const bool cut = cd->t[z] < c.dims[z];
            ++z;
            if (cut) break;
        }
        int64_t rows = 1, pitch = 0;
        for (; z < r; ++z)
            if (cd->t[z] > 1) {
                rows *= cd->t[z];
                if (pitch == 0) pitch = sI[z] * elem;
            }
        if (pitch != 0 && pitch % 8192 == 0 && rows > 32) cost *= 1.0 + 0.15 * std::log2((double)rows / 32.0);
    }
    // The LDS stage itself is not free.
    if (cd->use_lds) cost *= 1.1;
    if (cd->align) cost *= al4 ? kAlign4Weight : kAlignWeight;
    // Tiny tensors (a few rounds of tiles at most) are bound by latency, not bandwidth: what
    // counts is how long one workgroup needs for its tiles, a good half microsecond per slot
    // of a thread and a little more per tile dim (the prologue evaluates every slot's
    // position), spread over the rounds that overlap.  Expressed in the units of `cost` (1 =
    // the time 9 MB take), so that it fades out as the tensor grows.  Fitted to the measured
    // times of all candidates of 100 problems of 8 Ki to 2 Mi elements (picks went from 66 %
    // to 92 % of the best candidate there) and rescaled by 0.6 after the kernel's start-up
    // path got shorter (52 problems of 0.25 to 128 MiB: 91.9 % -> 92.7 % of the best candidate).
    double total_bytes = (double)elem;
    for (int z = 0; z < r; ++z) total_bytes *= (double)c.dims[z];
    cost += (double)need * (1.0 + 0.2 * n_tile_dims) / std::max(1.0, rounds) * (9.0e6 / total_bytes);
    // Nontemporal loads and stores when every run starts and ends on a line boundary.
    cd->aligned = (gin >= 128.0 && gout >= 128.0 && std::fmod(rin, 128.0) == 0.0 &&
                   std::fmod(rout, 128.0) == 0.0);
    // Otherwise nontemporal stores alone pay off when every piece a tile writes starts and
    // ends on a 64-byte boundary, or on a 32-byte sector boundary if the pieces are longer
    // than 1 KiB (measured over 330 ragged shapes: median +3-9 % there; with 32-byte
    // granules and short pieces -4 to -8 %, below 32 bytes -1-2 % with swings to -20 %):
    // whole sectors can go straight out, while pieces that end inside a sector want the
    // line kept in L2 until the neighbouring tile has written the rest of it.
    cd->store_nt = gout >= 64.0 || (gout >= 32.0 && rout > 1024.0);
    // Nontemporal loads alone pay off when the input side is line-aligned and the output is
    // not (measured on 2-D transposes with a power-of-two leading extent: +3 to +21 % over the
    // cached policy; on ragged inputs they lose 10-25 %).
    cd->load_nt = gin >= 128.0 && std::fmod(rin, 128.0) == 0.0;
    cd->out_aligned = (gout >= 128.0 && std::fmod(rout, 128.0) == 0.0);
    cd->score = cost;
    return true;
}

// Tile extents proposed for one side: take the first `count` dims of `order` whole except
// the last, which gets extent `last`.
struct SideChoice {
    int count;
    int64_t last;
};

static std::vector<SideChoice> side_choices(const Canonical& c, const int* order) {
    static const int64_t targets[] = {4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048};
    std::vector<SideChoice> v;
    int64_t prefix = 1;
    for (int n = 1; n <= c.rank; ++n) {
        const int64_t d = c.dims[order[n - 1]];
        for (int64_t target : targets) {
            if (prefix >= target) continue;
            int64_t t = std::min(d, ceil_div(target, prefix));
            const int64_t chunks = ceil_div(d, t);
            t = ceil_div(d, chunks);  // balance the chunks
            if (prefix * t > kMaxTileVol) continue;
            bool dup = false;
            for (const auto& s : v) dup |= (s.count == n && s.last == t);
            if (!dup) v.push_back({n, t});
            // also the unbalanced power-of-two-ish chunk (keeps chunk starts aligned)
            const int64_t t2 = std::min(d, ceil_div(target, prefix));
            if (t2 != t && prefix * t2 <= kMaxTileVol) {
                dup = false;
                for (const auto& s : v) dup |= (s.count == n && s.last == t2);
                if (!dup) v.push_back({n, t2});
            }
        }
        if (prefix * d <= kMaxTileVol) {
            bool dup = false;
            for (const auto& s : v) dup |= (s.count == n && s.last == d);
            if (!dup) v.push_back({n, d});
        }
        prefix *= d;
        if (prefix >= 2048) break;
    }
    return v;
}

bool make_candidate(const Canonical& c, int elem, int m, int64_t tile_in, int k,
                    int64_t tile_out, bool use_lds, Candidate* out, bool align) {
    const int r = c.rank;
    if (m < 1 || m > r || k < 1 || k > r) return false;
    Candidate cd;
    cd.m = m;
    cd.k = k;
    cd.use_lds = use_lds;
    cd.align = align;
    for (int z = 0; z < r; ++z) cd.t[z] = 1;
    for (int z = 0; z < m - 1; ++z) cd.t[z] = c.dims[z];
    const int za = m - 1;
    if (tile_in <= 0 || tile_in > c.dims[za]) tile_in = c.dims[za];
    cd.t[za] = std::max(cd.t[za], tile_in);
    for (int j = 0; j < k - 1; ++j) cd.t[c.perm[j]] = c.dims[c.perm[j]];
    const int zb = c.perm[k - 1];
    if (tile_out <= 0 || tile_out > c.dims[zb]) tile_out = c.dims[zb];
    cd.t[zb] = std::max(cd.t[zb], tile_out);
    if (!use_lds && c.perm[0] != 0) return false;  // LDS-free only when dim 0 stays first
    if (!finish_candidate(c, elem, &cd)) return false;
    if (!use_lds)
        cd.kclass = TPERM_KERNEL_ROWCOPY;
    else if (m == 1 && k == 1 && c.perm[0] != 0)
        cd.kclass = TPERM_KERNEL_TILED;
    else
        cd.kclass = TPERM_KERNEL_PACKED;
    *out = cd;
    return true;
}

std::vector<Candidate> enumerate_candidates(const Canonical& c, int elem) {
    std::vector<Candidate> out;
    if (c.rank < 2) return out;
    int in_order[TPERM_MAX_RANK];
    for (int z = 0; z < c.rank; ++z) in_order[z] = z;
    const auto ins = side_choices(c, in_order);
    const auto outs = side_choices(c, c.perm);
    auto push = [&](const Candidate& cd) {
        for (const auto& o : out) {
            if (o.use_lds != cd.use_lds || o.align != cd.align) continue;
            bool same = true;
            for (int z = 0; z < c.rank; ++z) same &= (o.t[z] == cd.t[z]);
            if (same) return;
        }
        out.push_back(cd);
    };
    for (const auto& a : ins)
        for (const auto& b : outs) {
            Candidate cd;
            if (make_candidate(c, elem, a.count, a.last, b.count, b.last, true, &cd)) push(cd);
            // the same tile with line-aligned output windows, where that form applies: the
            // chunk is rounded down to whole lines
            if (b.count == 1) {
                const int64_t line = 128 / elem;
                const int64_t tb = std::max(line, b.last / line * line);
                if (make_candidate(c, elem, a.count, a.last, b.count, tb, true, &cd, true)) push(cd);
            }
        }
    if (c.perm[0] == 0) {
        // LDS-free row copy: the tile is taken in output order only
        for (const auto& b : outs) {
            Candidate cd;
            if (make_candidate(c, elem, 1, b.count == 1 ? b.last : 0, b.count, b.last, false, &cd))
                push(cd);
        }
    }
    std::stable_sort(out.begin(), out.end(),
                     [](const Candidate& x, const Candidate& y) { return x.score < y.score; });
    return out;
}

// ---------------------------------------------------------------------------------------
// descriptor construction
// ---------------------------------------------------------------------------------------


// LDS cost of the first slots of each wavefront: for every wavefront-wide access, the
// largest number of distinct addresses that fall into one bank (64 banks of 4 bytes; an
// 8-byte access is served per half wavefront and occupies two banks).  The slot positions
// are affine in the row padding, so they are sampled once (padding 0 and 1) and the cost
// of any padding follows without walking the tile dims again.
namespace {

struct ConflictSampler {
    struct Group {
        int n;
        uint32_t base[64];   // LDS element index at padding 0
        uint32_t slope[64];  // increase per unit of padding
    };
    std::vector<Group> groups;
    int elem = 8;

    // d0 / d1: the descriptor with LDS strides set for padding 0 / padding 1
    ConflictSampler(const TileDesc& d0, const TileDesc& d1, int elem_, int nreg, int threads)
        : elem(elem_) {
        const int slots = std::min(nreg, 4);
        const int per = elem == 8 ? 32 : 64;  // lanes served together
        for (int side = 0; side < 2; ++side) {
            const TileDim* a = side == 0 ? d0.in_order : d0.out_order;
            const TileDim* b = side == 0 ? d1.in_order : d1.out_order;
            for (int w = 0; w < threads / 64; ++w)
                for (int j = 0; j < slots; ++j)
                    for (int g = 0; g < 64 / per; ++g) {
                        Group gr;
                        gr.n = 0;
                        for (int l = 0; l < per; ++l) {
                            const uint32_t k = (uint32_t)(w * 64 + g * per + l + j * threads);
                            if (k >= d0.tile_vol) continue;
                            const uint32_t l0 = tile_slot(a, d0.n_tile_dims, k).loff;
                            const uint32_t l1 = tile_slot(b, d1.n_tile_dims, k).loff;
                            gr.base[gr.n] = l0;
                            gr.slope[gr.n] = l1 - l0;
                            ++gr.n;
                        }
                        if (gr.n > 0) groups.push_back(gr);
                    }
        }
    }

    double cost(uint32_t pad) const {
        const uint32_t kBanks = 64;
        const uint32_t words = (uint32_t)(elem / 4);
        double total = 0.0;
        for (const Group& gr : groups) {
            uint32_t addr[64];
            for (int i = 0; i < gr.n; ++i) addr[i] = gr.base[i] + pad * gr.slope[i];
            std::sort(addr, addr + gr.n);
            int per_bank[64] = {0};
            int worst = 0;
            for (int i = 0; i < gr.n; ++i) {
                if (i > 0 && addr[i] == addr[i - 1]) continue;  // same address: one access
                const uint32_t bank = (addr[i] * words) % kBanks;
                worst = std::max(worst, ++per_bank[bank]);
            }
            total += worst;
        }
        return total;
    }
};

}  // namespace

double lds_conflict_cost(const TileDesc& d, int elem, int nreg, int threads) {
    return ConflictSampler(d, d, elem, nreg, threads).cost(0);
}

double lds_conflict_ratio(const TileDesc& d, int elem, int nreg, int threads) {
    const ConflictSampler s(d, d, elem, nreg, threads);
    return s.groups.empty() ? 1.0 : s.cost(0) / (double)s.groups.size();
}

// Fill the LDS strides of both dim lists for a given row padding; returns LDS elements.
static uint32_t set_lds_strides(TileDesc* d, const int* dim_of_in, const int* dim_of_out,
                                int run_dims, uint32_t pad) {
    uint32_t lstride[TPERM_DESC_MAX_DIMS];
    uint32_t cum = 1;
    const uint32_t n = d->n_tile_dims;
    for (uint32_t i = 0; i < n; ++i) {
        if ((int)i == run_dims && run_dims > 0 && i < n) cum += pad;  // pitch after the run
        lstride[i] = cum;
        cum *= d->in_order[i].ext;
        d->in_order[i].lstride = lstride[i];
    }
    for (uint32_t j = 0; j < n; ++j)
        for (uint32_t i = 0; i < n; ++i)
            if (dim_of_out[j] == dim_of_in[i]) d->out_order[j].lstride = lstride[i];
    return cum;
}

tperm_status_t build_tile_plan(Plan* plan, const Candidate& cand, const TileBuildOpts& opts) {
    const int lds_pad = opts.lds_pad, grid_mode = opts.grid_mode, window_in = opts.window_in,
              window_out = opts.window_out, threads = opts.threads, lds_buffers = opts.lds_buffers;
    if (threads != 64 && threads != 256) return TPERM_ERR_KERNEL;
    // large tensors run plain LDS-staged tiles of 256 threads (the forms instantiated for them)
    if (opts.big && (!cand.use_lds || threads != 256)) return TPERM_ERR_KERNEL;
    const Canonical& c = plan->c;
    const int r = c.rank;
    const int elem = plan->elem;
    int inv[TPERM_MAX_RANK];
    for (int j = 0; j < r; ++j) inv[c.perm[j]] = j;
    int64_t sI[TPERM_MAX_RANK], sO[TPERM_MAX_RANK];
    sI[0] = 1;
    for (int z = 1; z < r; ++z) sI[z] = sI[z - 1] * c.dims[z - 1];
    sO[0] = 1;
    for (int j = 1; j < r; ++j) sO[j] = sO[j - 1] * c.dims[c.perm[j - 1]];

    TileDesc d;
    std::memset(&d, 0, sizeof(d));
    // split dims: A = first split dim in input order, B = the second
    int split_dim[2] = {-1, -1};
    for (int z = 0, s = 0; z < r; ++z)
        if (cand.t[z] > 1 && cand.t[z] < c.dims[z]) {
            if (s >= 2) return TPERM_ERR_KERNEL;
            split_dim[s++] = z;
        }
    // Line-aligned output windows (see OutAlign): the output's leading dimension q0 is cut
    // into chunks of whole lines, every row shifts its window down to a line boundary, and the
    // read side covers a halo of one line's worth of coordinates in front of the chunk.
    const int q0 = c.perm[0];
    const int64_t line_elems = 128 / elem;
    bool align_out = false;
    // the halo in front of the tensors has to fit the 32-bit byte offsets: with the whole tensor
    // behind it, or, for large tensors, within the range of one buffer description
    const bool halo_fits = opts.big ? line_elems * sI[q0] * elem < (int64_t)TPERM_BIG_RANGE / 2
                                    : (c.volume + line_elems * sI[q0]) * elem + 512 < ((int64_t)1 << 32) - 256;
    if ((opts.align_out == 2 || (opts.align_out == 0 && cand.align)) && cand.use_lds && threads == 256 &&
        q0 != 0 && cand.k == 1 && cand.t[q0] < c.dims[q0] &&
        cand.t[q0] >= line_elems && cand.t[q0] % line_elems == 0 &&
        cand.t[q0] + line_elems <= 0x7FFF && halo_fits) {
        align_out = true;
        // the shifted dimension is always split dim B
        if (split_dim[0] == q0) std::swap(split_dim[0], split_dim[1]);
    }
    auto sel_of = [&](int z) -> uint32_t {
        return z == split_dim[0] ? 1u : (z == split_dim[1] ? 2u : 0u);
    };
    // tile dims in input order and in output order; with aligned windows the read side sees
    // the shifted dimension with its halo, the write side without
    int dim_of_in[TPERM_DESC_MAX_DIMS], dim_of_out[TPERM_DESC_MAX_DIMS];
    uint32_t n = 0;
    for (int z = 0; z < r; ++z)
        if (cand.t[z] > 1) {
            TileDim& td = d.in_order[n];
            td.ext = (uint32_t)(cand.t[z] + (align_out && z == q0 ? line_elems : 0));
            td.div = make_fastdiv(td.ext);
            td.gstride = (uint32_t)sI[z];
            td.ostride = (uint32_t)sO[inv[z]];
            td.sel = sel_of(z);
            dim_of_in[n++] = z;
        }
    uint32_t n2 = 0;
    for (int j = 0; j < r; ++j) {
        const int z = c.perm[j];
        if (cand.t[z] > 1) {
            TileDim& td = d.out_order[n2];
            td.ext = (uint32_t)cand.t[z];
            td.div = make_fastdiv(td.ext);
            td.gstride = (uint32_t)sO[j];
            td.ostride = (uint32_t)sI[z];
            td.sel = sel_of(z);
            dim_of_out[n2++] = z;
        }
    }
    d.n_tile_dims = n;
    // read-side slots (with the halo); the write side has cand.tile_vol slots
    const int64_t read_vol = align_out ? cand.tile_vol / cand.t[q0] * (cand.t[q0] + line_elems) : cand.tile_vol;
    if (read_vol > kMaxTileVol) return TPERM_ERR_KERNEL;
    d.tile_vol = (uint32_t)read_vol;
    for (int s = 0; s < 2; ++s) {
        d.split_ext[s] = split_dim[s] >= 0 ? (uint32_t)c.dims[split_dim[s]] : 0u;
        d.split_tile[s] = split_dim[s] >= 0 ? (uint32_t)cand.t[split_dim[s]] : 0u;
        d.split_step[s] = d.split_tile[s];
        d.split_halo[s] = 0;
    }
    if (align_out) {
        // coordinates of the shifted dimension are counted from the halo origin: the first
        // line_elems of them do not exist, tiles are t + line_elems wide and t apart
        d.split_ext[1] = (uint32_t)(c.dims[q0] + line_elems);
        d.split_tile[1] = (uint32_t)(cand.t[q0] + line_elems);
        d.split_step[1] = (uint32_t)cand.t[q0];
        d.split_halo[1] = (uint32_t)line_elems;
    }
    // Major terms.  The order of the lanes is the order in which the tile index b walks the
    // tiles, and with it which tiles run at the same time.  A "window" of up to window_in
    // tiles that are neighbours on the input side (smallest input strides) comes first,
    // then a window of up to window_out tiles that are neighbours on the output side, then
    // everything else in input order: the few hundred tiles in flight at any moment then
    // cover a compact region of both tensors instead of a thin slab of one.
    for (int l = 0; l < TPERM_DESC_MAX_DIMS; ++l) {
        d.major.cum[l] = make_fastdiv(1);
        d.major.ext_div[l] = make_fastdiv(1);
        d.major.ext[l] = 1;
        d.major.stride_in[l] = 0;
        d.major.stride_out[l] = 0;
    }
    struct MDim {
        int z;             // canonical dim
        uint32_t count;    // chunks (split dim) or extent (outer dim)
        uint64_t sin, sout;
        int split;         // 0 / 1: chunk counter of split A / B; -1: outer dim
        uint32_t lo = 0;   // > 0: counter split into lo (window) and hi parts
        int window = -1;   // 0: in the input window, 1: in the output window, -1: neither
    };
    std::vector<MDim> md;
    for (int z = 0; z < r; ++z) {
        if (cand.t[z] >= c.dims[z]) continue;
        MDim m;
        m.z = z;
        // shifted windows reach up to line_elems - 1 short of the chunk's nominal end
        m.count = (uint32_t)ceil_div(c.dims[z] + (align_out && z == q0 ? line_elems - 1 : 0), cand.t[z]);
        m.sin = (uint64_t)cand.t[z] * sI[z];
        m.sout = (uint64_t)cand.t[z] * sO[inv[z]];
        m.split = z == split_dim[0] ? 0 : (z == split_dim[1] ? 1 : -1);
        md.push_back(m);
    }
    if (md.size() > TPERM_DESC_MAX_DIMS) return TPERM_ERR_KERNEL;
    int n_pairs = 0;
    auto take_window = [&](int side, uint32_t budget) {
        // walk the major dims by increasing stride on this side
        std::vector<int> order(md.size());
        for (size_t i = 0; i < md.size(); ++i) order[i] = (int)i;
        std::sort(order.begin(), order.end(), [&](int a, int b) {
            return side == 0 ? md[a].sin < md[b].sin : md[a].sout < md[b].sout;
        });
        for (int i : order) {
            if (budget < 2) break;
            MDim& m = md[i];
            if (m.window >= 0) continue;  // already taken by the other window
            if (m.count <= budget) {
                m.window = side;
                budget /= m.count;
            } else {
                if (n_pairs >= 2 || md.size() + (size_t)n_pairs + 1 > TPERM_DESC_MAX_DIMS) break;
                const uint32_t hi = (uint32_t)ceil_div(m.count, budget);
                m.lo = (uint32_t)ceil_div(m.count, hi);  // balanced: few non-existent tiles
                m.window = side;
                ++n_pairs;
                break;
            }
        }
    };
    if (window_in <= 0 && opts.tile_order == 1) {
        // Automatic input window.  Tiles that are neighbours along the input run read parts of
        // the same 128-byte lines whenever the pieces they read do not start and end on line
        // boundaries; in output-major order they would run far apart in time, or at the same
        // time on different XCDs, and each fetch those lines again (measured: up to 2x the
        // algorithmic read traffic).  When the counter that steps along the input run has at
        // most 8 values it is walked first, which puts those neighbours next to each other in
        // the tile order and so into one group of tiles dealt to one XCD, where the second
        // reader finds the line in L2.  Two cases: the run is cut inside a dimension (the
        // counter is that dimension's chunk counter), or it ends at a dimension boundary and
        // is at most 1 KiB long (the counter is the next dimension's index).  Measured over
        // 438 ragged cases (rank sweep, rank-6 set, held-out shapes): the second case changes
        // 40 of them by +4 to +23 % and none by more than -2 %.  Counters with more values
        // would have to be split into a low and a high part; that was measured too and loses
        // as often as it wins (-15 to +13 %), so they are left alone.
        int zr = -1;
        for (int z = 0; z < r; ++z)
            if (cand.t[z] < c.dims[z]) {
                zr = z;
                break;
            }
        bool steps_along_run = false;
        if (zr >= 0 && cand.t[zr] > 1) steps_along_run = ((cand.t[zr] * sI[zr] * elem) % 128) != 0;
        else if (zr >= 0 && window_in == 0 && cand.use_lds)
            steps_along_run = ((sI[zr] * elem) % 128) != 0 && sI[zr] * elem <= 1024;
        if (steps_along_run)
            for (auto& m : md)
                if (m.z == zr && m.count <= 8) m.window = 0;
    }
    if (window_in > 1) take_window(0, (uint32_t)window_in);
    if (window_out > 1) take_window(1, (uint32_t)window_out);

    uint32_t lane = 0;
    uint64_t cum = 1;
    auto add_major = [&](uint32_t ext, uint64_t sin, uint64_t sout) {
        d.major.cum[lane] = make_fastdiv((uint32_t)cum);
        d.major.ext_div[lane] = make_fastdiv(ext);
        d.major.ext[lane] = ext;
        d.major.stride_in[lane] = (uint32_t)sin;
        d.major.stride_out[lane] = (uint32_t)sout;
        cum *= ext;
        return lane++;
    };
    d.lane_a = d.lane_b = 0;
    d.chunk_pair[0] = d.chunk_pair[1] = 2;
    for (int p = 0; p < 2; ++p) d.pair[p] = SplitPair{0, 0, 0, 0};
    int pair_of[TPERM_DESC_MAX_DIMS];
    int next_pair = 0;
    // passes 0 and 1: the two windows (low parts), pass 2: the rest.  In input-major order
    // the input window comes first and the rest follows by increasing input stride; in
    // output-major order the roles are swapped, which makes the write stream the more
    // sequential one (measured: HBM tolerates scattered reads better than scattered writes).
    std::vector<size_t> walk(md.size());
    for (size_t i = 0; i < md.size(); ++i) walk[i] = i;
    if (opts.tile_order == 1)
        std::sort(walk.begin(), walk.end(), [&](size_t a, size_t b) { return md[a].sout < md[b].sout; });
    for (int pass = 0; pass < 3; ++pass)
        for (size_t wi = 0; wi < md.size(); ++wi) {
            const size_t i = walk[wi];
            MDim& m = md[i];
            if (pass < 2) {
                if (m.window != (opts.tile_order == 1 ? 1 - pass : pass)) continue;
                if (m.lo > 0) {
                    pair_of[i] = next_pair++;
                    SplitPair& sp = d.pair[pair_of[i]];
                    sp.width = m.lo;
                    sp.count = m.count;
                    sp.lane_lo = add_major(m.lo, m.sin, m.sout);
                    if (m.split >= 0) d.chunk_pair[m.split] = (uint32_t)pair_of[i];
                } else {
                    const uint32_t l = add_major(m.count, m.sin, m.sout);
                    if (m.split == 0) d.lane_a = l;
                    if (m.split == 1) d.lane_b = l;
                }
            } else {
                if (m.window >= 0 && m.lo == 0) continue;  // placed whole in a window
                if (m.lo > 0) {
                    d.pair[pair_of[i]].lane_hi = add_major((uint32_t)ceil_div(m.count, m.lo),
                                                           m.sin * m.lo, m.sout * m.lo);
                } else {
                    const uint32_t l = add_major(m.count, m.sin, m.sout);
                    if (m.split == 0) d.lane_a = l;
                    if (m.split == 1) d.lane_b = l;
                }
            }
        }
    d.n_major = lane;
    if (cum >= ((uint64_t)1 << 31)) return TPERM_ERR_KERNEL;
    d.num_tiles = (uint32_t)cum;  // includes the non-existent combinations of split counters

    std::memset(&d.oa, 0, sizeof(d.oa));
    if (align_out) {
        d.oa.enabled = 1;
        d.oa.line_elems = (uint32_t)line_elems;
        d.oa.total_slots = (uint32_t)cand.tile_vol;
        d.oa.in_halo_elems = (uint32_t)(line_elems * sI[q0]);
    }
    const int nreg = pick_nreg(read_vol, threads);
    if (nreg < 0) return TPERM_ERR_KERNEL;

    // LDS image: tile in input order, rows of the contiguous input run separated by a padded
    // pitch.  The pad is chosen to minimise the bank conflicts of the strided side.
    int run_dims = 0;
    for (uint32_t i = 0; i < n; ++i) {
        // dims of the run are the leading canonical dims 0,1,..: tile dim i belongs to
        // the run if it is canonical dim i and all earlier ones were taken whole
        if (dim_of_in[i] != (int)i) break;
        ++run_dims;
        if (cand.t[i] < c.dims[i]) break;
    }
    // A tile that is one contiguous piece of the input (every tile dim belongs to the run) needs
    // a padded pitch all the same: the write side walks the image across the run's last dim,
    // with a power-of-two stride if the dims in front are powers of two (measured on 16 x 2^20
    // fp32: 16-way bank conflicts, 3.6 TB/s against 5.1 with a padded pitch).  The pad then
    // goes in front of the tile's last dim.
    if (run_dims >= (int)n && n >= 2) run_dims = (int)n - 1;
    auto lay = [&](uint32_t p) { return set_lds_strides(&d, dim_of_in, dim_of_out, run_dims, p); };
    const int layout_run_dims = run_dims;
    int pad = 0;
    uint32_t lds_elems = 0;
    if (cand.use_lds) {
        if (lds_pad >= 0) {
            pad = lds_pad;
            lds_elems = lay((uint32_t)pad);
        } else if (layout_run_dims >= (int)n) {
            pad = 0;
            lds_elems = lay(0);
        } else {
            double best = 1e300;
            int best_pad = 0;
            const int max_pad = elem == 8 ? 16 : 32;
            const uint32_t le0 = lay(0);
            const TileDesc d0 = d;
            const uint32_t le1 = lay(1);
            const ConflictSampler sampler(d0, d, elem, nreg, threads);
            for (int p = 0; p <= max_pad; ++p) {
                const int64_t le = (int64_t)le0 + (int64_t)p * ((int64_t)le1 - (int64_t)le0);
                if (le * elem > kMaxLdsBytes) break;
                const double cost = sampler.cost((uint32_t)p);
                if (cost < best - 1e-9) {
                    best = cost;
                    best_pad = p;
                }
            }
            pad = best_pad;
            lds_elems = lay((uint32_t)pad);
        }
        if ((int64_t)lds_elems * elem > kMaxLdsBytes) return TPERM_ERR_KERNEL;
        if (lds_elems + 64u > 0xFFFFu) return TPERM_ERR_KERNEL;  // LDS slots are kept in 16 bits
    }
    d.lds_elems = lds_elems;
    if (align_out) d.oa.lstride_b = d.out_order[0].lstride;
    d.lds_buffers = (cand.use_lds && lds_buffers == 2 && (int64_t)lds_elems * elem * 2 <= kMaxLdsBytes) ? 2u : 1u;
    // grid_mode values >= 2 carry the group size: mode 2 + log2(group) (2 -> groups of 1)
    d.grid_mode = grid_mode >= 2 ? 2u : (uint32_t)grid_mode;
    d.group_log2 = grid_mode >= 2 ? (uint32_t)(grid_mode - 2) : 0u;
    if (d.group_log2 > 20u) return TPERM_ERR_KERNEL;
    // every XCD should get at least 8 groups, or the XCDs run out of balance
    while (d.grid_mode == 2u && d.group_log2 > 0u && d.num_tiles < ((64u << d.group_log2)))
        --d.group_log2;
    d.tiles_per_xcd = (uint32_t)ceil_div((int64_t)d.num_tiles, 8);

    // Pairs of 4-byte elements (vec2).  A transposing tile of 4-byte elements can read two
    // neighbours along input dim 0 with one 8-byte load and write two neighbours along output
    // dim 0 with one 8-byte store when every pair is whole and 8-byte aligned: even extents
    // and even tile extents along both dims (all other strides are then even too).  Half
    // the global memory instructions per byte; the LDS image and its padding stay as laid
    // out above, in single elements.
    int nreg_final = nreg;
    plan->vec2 = false;
    {
        const int q = c.perm[0];
        const int nreg2 = pick_nreg(cand.tile_vol / 2, threads);
        // 8-byte elements in 16-byte accesses wherever the shape allows: measured neutral to
        // +1 % on ragged shapes, +3 to +14 % on line-aligned tensors once the selector sizes such
        // tiles by pair slots (see finish_candidate).
        const bool worth_it = true;
        // In line-aligned windows (4-byte elements only) the written pairs are 8-byte aligned
        // whatever the extents, and an odd row length on the read side is allowed as long as
        // dim 0 is chunked: the tile that holds the odd end reads element by element.
        const int nreg2w = pick_nreg(read_vol / 2, threads);
        const bool pair_windows = align_out && elem == 4 && nreg2w > 0 && cand.t[0] % 2 == 0 &&
                                  (c.dims[0] % 2 == 0 || cand.t[0] < c.dims[0]) &&
                                  (split_dim[0] == 0 || cand.t[0] == c.dims[0]);
        const bool pair_plain = !align_out && worth_it && nreg2 > 0 && c.dims[0] % 2 == 0 &&
                                c.dims[q] % 2 == 0 && cand.t[0] % 2 == 0 && cand.t[q] % 2 == 0;
        if (opts.vec2 >= 1 && cand.use_lds && threads == 256 && q != 0 && (pair_plain || pair_windows) &&
            dim_of_in[0] == 0 && dim_of_out[0] == q) {
            TileDim& a = d.in_order[0];
            a.ext /= 2;
            a.div = make_fastdiv(a.ext);
            a.gstride *= 2;
            a.lstride *= 2;
            a.xshift = 1;
            TileDim& o = d.out_order[0];
            d.pair_lstride = o.lstride;
            o.ext /= 2;
            o.div = make_fastdiv(o.ext);
            o.gstride *= 2;
            o.lstride *= 2;
            o.xshift = 1;
            d.tile_vol /= 2;
            if (align_out) {
                d.oa.total_slots /= 2;
                d.pair_a_split = split_dim[0] == 0 ? 1u : 0u;
            }
            d.vec2 = 1;
            nreg_final = align_out ? nreg2w : nreg2;
            plan->vec2 = true;
        }
    }

    plan->big = opts.big;
    if (opts.big) {
        // every position inside a tile, on either side, within the range of one buffer description
        uint64_t span_in = 0, span_out = 0;
        for (uint32_t i = 0; i < d.n_tile_dims; ++i) {
            span_in += (uint64_t)(d.in_order[i].ext - 1u) * d.in_order[i].gstride;
            span_out += (uint64_t)(d.out_order[i].ext - 1u) * d.out_order[i].gstride;
        }
        // (+ 2: the last access may be a pair of elements; + one line: written windows are
        // placed from a halo origin one line in front of the tile)
        if ((std::max(span_in, span_out) + 2u + (uint64_t)line_elems) * (uint64_t)elem > (uint64_t)TPERM_BIG_RANGE)
            return TPERM_ERR_KERNEL;
    }
    plan->tile = d;
    plan->cand = cand;
    plan->kclass = cand.kclass;
    plan->use_lds = cand.use_lds;
    plan->nreg = nreg_final;
    plan->threads = threads;
    {
        // resident workgroups per compute unit: aim at ~20 KiB of tile data per CU for the
        // LDS-staged kernels and ~14 KiB for the LDS-free row copy, whose tiles turn round
        // faster (measured optimum over the row-copy cases of all benchmark sets: two
        // workgroups from 6 KiB tiles up, three below)
        const double tile_bytes = (double)cand.tile_vol * elem;
        int bpc = (int)std::lround((cand.use_lds ? 20480.0 : 14336.0) / tile_bytes);
        plan->blocks_per_cu = std::max(2, std::min(8, bpc));
        // aligned windows write whole lines, whatever the granule of the rows
        const bool store_nt = cand.store_nt || align_out;
        plan->cache_policy = cand.aligned ? 2 : (store_nt ? (cand.load_nt ? 2 : 3) : (cand.load_nt ? 4 : 1));
        // loads before stores pays on line-aligned shapes with small LDS-staged tiles only
        // (measured per case over all benchmark sets; see tile_kernel)
        plan->loads_first = cand.aligned && cand.use_lds && nreg <= 6 && !plan->vec2 && !align_out && !opts.big;
    }
    plan->lds_pad = pad;
    plan->align_out = align_out;
    plan->lds_bytes = (int)((int64_t)lds_elems * elem);
    plan->grid_mode = grid_mode;
    return TPERM_OK;
}

void build_naive_desc(Plan* plan) {
    const Canonical& c = plan->c;
    NaiveDesc nd;
    std::memset(&nd, 0, sizeof(nd));
    nd.rank = (uint32_t)c.rank;
    nd.volume = (uint32_t)c.volume;
    int64_t sI[TPERM_MAX_RANK];
    sI[0] = 1;
    for (int z = 1; z < c.rank; ++z) sI[z] = sI[z - 1] * c.dims[z - 1];
    for (int j = 0; j < c.rank; ++j) {
        nd.out_ext[j] = (uint32_t)c.dims[c.perm[j]];
        nd.out_ext_div[j] = make_fastdiv(nd.out_ext[j]);
        nd.in_stride[j] = (uint32_t)sI[c.perm[j]];
    }
    plan->naive = nd;
}

// ---------------------------------------------------------------------------------------
// plan creation
// ---------------------------------------------------------------------------------------

// Tensors whose byte offsets do not fit the 32-bit operands of buffer addressing.
static bool is_big(const Canonical& c, int elem) {
    return (uint64_t)c.volume * (uint64_t)elem >= ((uint64_t)1 << 32) - 256u;
}

tperm_status_t create_plan(Plan** out, int rank, const int64_t* dims, const int* perm,
                           size_t elem, const tperm_plan_opts_t* opts) {
    if (out == nullptr) return TPERM_ERR_NULL;
    *out = nullptr;
    tperm_status_t st = validate(rank, dims, perm, elem);
    if (st != TPERM_OK) return st;
    Plan* p = new (std::nothrow) Plan();
    if (p == nullptr) return TPERM_ERR_NOMEM;
    p->rank = rank;
    for (int z = 0; z < rank; ++z) {
        p->dims[z] = dims[z];
        p->perm[z] = perm[z];
    }
    p->elem = (int)elem;
    canonicalise(rank, dims, perm, &p->c);
    std::memset(&p->tile, 0, sizeof(p->tile));
    build_naive_desc(p);

    tperm_plan_opts_t o;
    std::memset(&o, 0, sizeof(o));
    o.lds_pad = -1;
    if (opts) o = *opts;
    const int want = o.kernel_class;
    const bool identity = (p->c.rank == 1);
    p->big = is_big(p->c, p->elem) || o.large == 1;

    auto fail = [&](tperm_status_t s) {
        delete p;
        return s;
    };

    if (want == TPERM_KERNEL_NAIVE) {
        p->kclass = TPERM_KERNEL_NAIVE;
        *out = p;
        return TPERM_OK;
    }
    if (identity) {
        if (want != TPERM_KERNEL_AUTO && want != TPERM_KERNEL_COPY) return fail(TPERM_ERR_KERNEL);
        p->kclass = TPERM_KERNEL_COPY;
        *out = p;
        return TPERM_OK;
    }
    if (want == TPERM_KERNEL_COPY) return fail(TPERM_ERR_KERNEL);
    if (want < 0 || want > TPERM_KERNEL_NAIVE) return fail(TPERM_ERR_KERNEL);

    TileBuildOpts bo;
    bo.lds_pad = o.lds_pad;
    bo.grid_mode = o.grid_mode == 0 ? kDefaultGridMode : (o.grid_mode < 0 ? 0 : o.grid_mode);
    if (o.window_in != 0) bo.window_in = o.window_in;  // -1: the narrower automatic window (whole chunk counters of at most 8 values)
    if (o.window_out > 0) bo.window_out = o.window_out;
    if (o.threads > 0) bo.threads = o.threads;
    if (o.lds_buffers > 0) bo.lds_buffers = o.lds_buffers;
    bo.align_out = o.align_out;
    bo.tile_order = o.tile_order > 0 ? o.tile_order - 1 : kDefaultTileOrder;
    bo.vec2 = o.vec2 == 2 ? 2 : 0;
    bo.big = p->big;
    if (bo.big) {
        // options that large tensors have no kernels for are ignored
        bo.threads = kDefaultThreads;
        o.loads_first = 0;
    }
    if (bo.big && want == TPERM_KERNEL_ROWCOPY) return fail(TPERM_ERR_KERNEL);
    // can this candidate run the problem as given (large tensors: a tile whose positions fit)
    auto runnable = [&](const Candidate& cd) {
        if (!bo.big) return true;
        Plan tmp = *p;
        return build_tile_plan(&tmp, cd, bo) == TPERM_OK;
    };
    Candidate chosen;
    bool have = false;
    if (o.m > 0 || o.k > 0) {
        const int m = o.m > 0 ? o.m : 1, k = o.k > 0 ? o.k : 1;
        const bool use_lds = (want != TPERM_KERNEL_ROWCOPY);
        if (!make_candidate(p->c, p->elem, m, o.tile_in, k, o.tile_out, use_lds, &chosen))
            return fail(TPERM_ERR_KERNEL);
        if (want != TPERM_KERNEL_AUTO && want != chosen.kclass) {
            // an explicit tile may be run under the PACKED label whatever its shape
            if (!(want == TPERM_KERNEL_PACKED && chosen.use_lds)) return fail(TPERM_ERR_KERNEL);
            chosen.kclass = TPERM_KERNEL_PACKED;
        }
        have = true;
    } else {
        const auto cands = enumerate_candidates(p->c, p->elem);
        if (o.selector == 1) {
            // Section 2.3's way: build the plans (here: of the 24 best-scored candidates) and
            // keep the one the analytical model expects to finish first
            double best_us = 0.0;
            int tried = 0;
            for (const auto& cd : cands) {
                if (want != TPERM_KERNEL_AUTO && cd.kclass != want) continue;
                if (o.align_out == 1 && cd.align) continue;
                if (tried++ >= 24) break;
                Plan tmp = *p;
                tperm_model_t m;
                if (build_tile_plan(&tmp, cd, bo) != TPERM_OK || model_plan(tmp, &m) != TPERM_OK) continue;
                if (!have || m.microseconds < best_us) {
                    chosen = cd;
                    best_us = m.microseconds;
                    have = true;
                }
            }
        } else {
            for (const auto& cd : cands) {
                if (want != TPERM_KERNEL_AUTO && cd.kclass != want) continue;
                // windows switched off: a candidate scored and flagged for them is not this plan
                if (o.align_out == 1 && cd.align) continue;
                if (!runnable(cd)) continue;
                chosen = cd;
                have = true;
                break;
            }
        }
    }
    if (!have) {
        // a large tensor none of whose tiles fits the range of a buffer description: the gather
        // kernel, which computes whole addresses, moves it
        if (bo.big && want == TPERM_KERNEL_AUTO) {
            p->kclass = TPERM_KERNEL_NAIVE;
            *out = p;
            return TPERM_OK;
        }
        return fail(TPERM_ERR_KERNEL);
    }
    st = build_tile_plan(p, chosen, bo);
    if (st != TPERM_OK) return fail(st);
    if (o.blocks_per_cu > 0) p->blocks_per_cu = o.blocks_per_cu;
    if (o.cache_policy >= 1 && o.cache_policy <= 4) p->cache_policy = o.cache_policy;
    if (o.loads_first == 1 || o.loads_first == 2) p->loads_first = o.loads_first == 2;
    *out = p;
    return TPERM_OK;
}

tperm_status_t create_plan_with_candidate(Plan** out, int rank, const int64_t* dims,
                                          const int* perm, size_t elem, const Candidate& cand,
                                          bool vec2) {
    if (out == nullptr) return TPERM_ERR_NULL;
    *out = nullptr;
    tperm_status_t st = validate(rank, dims, perm, elem);
    if (st != TPERM_OK) return st;
    Plan* p = new (std::nothrow) Plan();
    if (p == nullptr) return TPERM_ERR_NOMEM;
    p->rank = rank;
    for (int z = 0; z < rank; ++z) {
        p->dims[z] = dims[z];
        p->perm[z] = perm[z];
    }
    p->elem = (int)elem;
    canonicalise(rank, dims, perm, &p->c);
    std::memset(&p->tile, 0, sizeof(p->tile));
    build_naive_desc(p);
    TileBuildOpts bo;
    bo.vec2 = vec2 ? 1 : 0;
    bo.big = is_big(p->c, p->elem);
    st = build_tile_plan(p, cand, bo);
    if (st != TPERM_OK) {
        delete p;
        return st;
    }
    *out = p;
    return TPERM_OK;
}

// ---------------------------------------------------------------------------------------
// host evaluation of a plan's index maps
// ---------------------------------------------------------------------------------------

// out_phase: what the kernel would see as (output pointer / element size) mod line_elems; only
// plans with line-aligned output windows look at it.
static tperm_status_t index_map_at_phase(const Plan& plan, int64_t* out_to_in, uint32_t out_phase) {
    const int64_t vol = plan.c.volume;
    for (int64_t i = 0; i < vol; ++i) out_to_in[i] = -1;
    if (plan.kclass == TPERM_KERNEL_COPY) {
        for (int64_t i = 0; i < vol; ++i) out_to_in[i] = i;
        return TPERM_OK;
    }
    if (plan.kclass == TPERM_KERNEL_NAIVE) {
        for (int64_t o = 0; o < vol; ++o)
            out_to_in[o] = (int64_t)naive_input_offset(plan.naive, (uint32_t)o);
        return TPERM_OK;
    }
    const TileDesc& d = plan.tile;
    std::vector<int64_t> lds(plan.use_lds ? d.lds_elems : 1, -1);
    const uint32_t slots = (uint32_t)plan.nreg * (uint32_t)plan.threads;
    if (slots < d.tile_vol) return TPERM_ERR_INTERNAL;
    // visit tiles the way a launch with `grid` workgroups would; any grid gives the same
    // set of tiles, use a small one that still exercises the iteration arithmetic
    const uint32_t grid = d.grid_mode != 0u ? 16u : 7u;
    std::vector<char> tile_seen(d.num_tiles, 0);
    for (uint32_t block = 0; block < grid; ++block)
        for (uint32_t it = 0;; ++it) {
            const uint32_t b = tile_of(d, block, grid, it);
            if (b >= d.num_tiles) break;
            if (tile_seen[b]) return TPERM_ERR_INTERNAL;
            tile_seen[b] = 1;
            // major offsets: sum of the per-lane terms (Eqs. (2),(3))
            uint64_t maj_in = 0, maj_out = 0;
            uint32_t coord[TPERM_DESC_MAX_DIMS];
            for (uint32_t l = 0; l < TPERM_DESC_MAX_DIMS; ++l) {
                coord[l] = major_coord(d.major, l, b);
                maj_in += (uint64_t)coord[l] * d.major.stride_in[l];
                maj_out += (uint64_t)coord[l] * d.major.stride_out[l];
            }
            uint32_t rem_a = 0, rem_b = 0, lo_b = 0;
            tile_remaining(d, [&](uint32_t l) { return coord[l]; }, &rem_a, &rem_b, &lo_b);
            if (plan.use_lds && d.vec2 && d.oa.enabled) {
                // pairs of 4-byte elements in line-aligned windows: read pairs along input dim
                // 0 (halo included), written pairs along the shifted window
                const OutAlign& oa = d.oa;
                const uint32_t span_b = rem_b > lo_b ? rem_b - lo_b : 0u;
                std::fill(lds.begin(), lds.end(), -1);
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.in_order, d.n_tile_dims, k);
                    for (uint32_t e = 0; e < 2; ++e) {
                        const uint32_t xa = d.pair_a_split ? s.xa + e : s.xa;
                        if (!(xa < rem_a && (s.xb - lo_b) < span_b)) continue;
                        const int64_t gi = (int64_t)maj_in + (int64_t)s.goff + e - (int64_t)oa.in_halo_elems;
                        if (gi < 0 || gi >= vol || s.loff + e >= d.lds_elems) return TPERM_ERR_INTERNAL;
                        if (lds[s.loff + e] != -1) return TPERM_ERR_INTERNAL;
                        lds[s.loff + e] = gi;
                    }
                }
                const uint32_t phi = (uint32_t)((maj_out + out_phase) & (oa.line_elems - 1u));
                for (uint32_t k = 0; k < oa.total_slots; ++k) {
                    const Slot so = tile_slot(d.out_order, d.n_tile_dims, k);
                    const uint32_t p = so.xb;  // even position in the chunk
                    const uint32_t rho = (so.goff - p) & (oa.line_elems - 1u);
                    const uint32_t shift = (phi + rho) & (oa.line_elems - 1u);
                    for (uint32_t e = 0; e < 2; ++e) {
                        const uint32_t xb = p + e + oa.line_elems - shift;
                        if (!(so.xa < rem_a && (xb - lo_b) < span_b)) continue;
                        const int64_t go = (int64_t)maj_out + (int64_t)so.goff + e - (int64_t)shift;
                        const int64_t li = (int64_t)so.loff + (int64_t)(oa.line_elems - shift + e) * oa.lstride_b;
                        if (go < 0 || go >= vol || li < 0 || li >= (int64_t)d.lds_elems) return TPERM_ERR_INTERNAL;
                        if (lds[li] == -1) return TPERM_ERR_INTERNAL;
                        if (out_to_in[go] != -1) return TPERM_ERR_INTERNAL;
                        out_to_in[go] = lds[li];
                    }
                }
            } else if (plan.use_lds && d.vec2) {
                // pairs: two neighbours along input dim 0 in, two along output dim 0 out
                std::fill(lds.begin(), lds.end(), -1);
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.in_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && s.xb < rem_b)) continue;
                    for (uint32_t e = 0; e < 2; ++e) {
                        const uint64_t gi = maj_in + s.goff + e;
                        if (gi >= (uint64_t)vol || s.loff + e >= d.lds_elems) return TPERM_ERR_INTERNAL;
                        if (lds[s.loff + e] != -1) return TPERM_ERR_INTERNAL;
                        lds[s.loff + e] = (int64_t)gi;
                    }
                }
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.out_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && s.xb < rem_b)) continue;
                    for (uint32_t e = 0; e < 2; ++e) {
                        const uint64_t go = maj_out + s.goff + e;
                        const uint32_t li = s.loff + e * d.pair_lstride;
                        if (go >= (uint64_t)vol || li >= d.lds_elems) return TPERM_ERR_INTERNAL;
                        if (lds[li] == -1) return TPERM_ERR_INTERNAL;
                        if (out_to_in[go] != -1) return TPERM_ERR_INTERNAL;
                        out_to_in[go] = lds[li];
                    }
                }
            } else if (plan.use_lds && d.oa.enabled) {
                // line-aligned output windows: the read side covers the halo, every row of
                // the write side shifts its window by its own phase
                const OutAlign& oa = d.oa;
                const uint32_t span_b = rem_b > lo_b ? rem_b - lo_b : 0u;
                std::fill(lds.begin(), lds.end(), -1);
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.in_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && (s.xb - lo_b) < span_b)) continue;
                    const int64_t gi = (int64_t)maj_in + (int64_t)s.goff - (int64_t)oa.in_halo_elems;
                    if (gi < 0 || gi >= vol || s.loff >= d.lds_elems) return TPERM_ERR_INTERNAL;
                    if (lds[s.loff] != -1) return TPERM_ERR_INTERNAL;
                    lds[s.loff] = gi;
                }
                const uint32_t phi = (uint32_t)((maj_out + out_phase) & (oa.line_elems - 1u));
                for (uint32_t k = 0; k < oa.total_slots; ++k) {
                    const Slot so = tile_slot(d.out_order, d.n_tile_dims, k);
                    const uint32_t p = so.xb;                       // position in the chunk
                    const uint32_t rho = (so.goff - p) & (oa.line_elems - 1u);
                    const uint32_t shift = (phi + rho) & (oa.line_elems - 1u);
                    const uint32_t xb = p + oa.line_elems - shift;  // tile coordinate written
                    if (!(so.xa < rem_a && (xb - lo_b) < span_b)) continue;
                    const int64_t go = (int64_t)maj_out + (int64_t)so.goff - (int64_t)shift;
                    const int64_t li = (int64_t)so.loff + (int64_t)(oa.line_elems - shift) * oa.lstride_b;
                    if (go < 0 || go >= vol || li < 0 || li >= (int64_t)d.lds_elems) return TPERM_ERR_INTERNAL;
                    if (lds[li] == -1) return TPERM_ERR_INTERNAL;
                    if (out_to_in[go] != -1) return TPERM_ERR_INTERNAL;
                    out_to_in[go] = lds[li];
                }
            } else if (plan.use_lds) {
                std::fill(lds.begin(), lds.end(), -1);
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.in_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && s.xb < rem_b)) continue;
                    const uint64_t gi = maj_in + s.goff;
                    if (gi >= (uint64_t)vol || s.loff >= d.lds_elems) return TPERM_ERR_INTERNAL;
                    if (lds[s.loff] != -1) return TPERM_ERR_INTERNAL;
                    lds[s.loff] = (int64_t)gi;
                }
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.out_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && s.xb < rem_b)) continue;
                    const uint64_t go = maj_out + s.goff;
                    if (go >= (uint64_t)vol || s.loff >= d.lds_elems) return TPERM_ERR_INTERNAL;
                    if (lds[s.loff] == -1) return TPERM_ERR_INTERNAL;
                    if (out_to_in[go] != -1) return TPERM_ERR_INTERNAL;
                    out_to_in[go] = lds[s.loff];
                }
            } else {
                for (uint32_t k = 0; k < d.tile_vol; ++k) {
                    const Slot s = tile_slot(d.out_order, d.n_tile_dims, k);
                    if (!(s.xa < rem_a && s.xb < rem_b)) continue;
                    const uint64_t go = maj_out + s.goff, gi = maj_in + s.ooff;
                    if (go >= (uint64_t)vol || gi >= (uint64_t)vol) return TPERM_ERR_INTERNAL;
                    if (out_to_in[go] != -1) return TPERM_ERR_INTERNAL;
                    out_to_in[go] = (int64_t)gi;
                }
            }
        }
    for (uint32_t b = 0; b < d.num_tiles; ++b)
        if (!tile_seen[b]) return TPERM_ERR_INTERNAL;
    // The map is in canonical coordinates; canonicalisation leaves scalar positions
    // unchanged, so it is also the map of the problem as given.
    return TPERM_OK;
}

tperm_status_t index_map(const Plan& plan, int64_t* out_to_in) {
    const tperm_status_t st = index_map_at_phase(plan, out_to_in, 0u);
    if (st != TPERM_OK) return st;
    if (plan.kclass != TPERM_KERNEL_COPY && plan.kclass != TPERM_KERNEL_NAIVE && plan.tile.oa.enabled) {
        // which tile writes an element depends on the phase of the output pointer; the
        // element map must not
        std::vector<int64_t> other((size_t)plan.c.volume);
        const tperm_status_t st2 = index_map_at_phase(plan, other.data(), 5u);
        if (st2 != TPERM_OK) return st2;
        for (int64_t i = 0; i < plan.c.volume; ++i)
            if (other[(size_t)i] != out_to_in[i]) return TPERM_ERR_INTERNAL;
    }
    return TPERM_OK;
}

}  // namespace tperm
