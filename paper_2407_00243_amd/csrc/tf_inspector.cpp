// Inspector: the tile fusion scheduler (paper Section 3.1, Algorithm 1) for one GPU.
//
// Step 1 forms uniform tiles of t consecutive rows and fuses a row of the second operation
// into the tile that produces the same row range exactly when every column index of that row
// of A lies inside the range.  Step 2 halves every tile whose fast-memory footprint exceeds
// the budget.  The GPU additions are the spill set (D1 rows that a second-wavefront row
// reads and that therefore must also reach device memory) and the work-balanced units of the
// second wavefront (the `balance` routine of Algorithm 1, read as: spread the leftover rows
// over units of about equal work; rows too long for one unit get a workgroup of their own).
//
// Pure host code: no HIP calls.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <thread>

#include "tf_internal.h"

// Section timings on stderr, for profiling the inspector on its own (compile with -DTF_TIMING).
#ifdef TF_TIMING
#include <cstdio>
#define TF_TICK(label)                                                                          \
    do {                                                                                        \
        const auto tf_now = std::chrono::steady_clock::now();                                   \
        std::fprintf(stderr, "  [inspector] %-28s %8.2f ms\n", label,                           \
                     std::chrono::duration<double>(tf_now - tf_tick).count() * 1e3);            \
        tf_tick = tf_now;                                                                       \
    } while (0)
#else
#define TF_TICK(label)
#endif

namespace tf {

namespace {

struct Range {
    int64_t i0, i1;
};

int64_t tile_footprint(const Schedule &s, int64_t rows) {
    return s.lds_fixed_bytes + round_up(rows, s.lds_row_granule) * s.lds_bytes_per_row;
}

// Step 2 for one coarse tile: halve (left half gets floor(rows / 2)) until the footprint fits.
void split_tile(const Schedule &s, Range r, bool allow_split, std::vector<Range> &out) {
    const int64_t rows = r.i1 - r.i0;
    if (!allow_split || rows <= 1 || tile_footprint(s, rows) <= s.fast_mem_bytes) {
        out.push_back(r);
        return;
    }
    const int64_t mid = r.i0 + rows / 2;
    split_tile(s, Range{r.i0, mid}, allow_split, out);
    split_tile(s, Range{mid, r.i1}, allow_split, out);
}

}  // namespace

namespace {

struct PackRules {
    int max_rows;        // most rows per unit
    int64_t max_slots;   // most padded entries per unit
    int split_groups;    // lane groups available for splitting long rows; 0 = never split
};

int pow2_at_least(int64_t x) {
    int g = 1;
    while (g < x) g *= 2;
    return g;
}

// Host threads for per-tile or per-unit work: one for small matrices, else up to 16.
int host_threads(int64_t nnz, int64_t n_items, int64_t min_items_per_thread) {
    if (nnz < ((int64_t)1 << 18) || n_items < 4 * min_items_per_thread) return 1;
    unsigned hw = std::min(16u, std::max(1u, std::thread::hardware_concurrency()));
    if (const char *e = std::getenv("TF_HOST_THREADS")) {      // a cap set by the caller's environment
        const long k = std::strtol(e, nullptr, 10);
        if (k >= 1) hw = (unsigned)std::min<long>(k, 16);
    }
    return (int)std::min<int64_t>(hw, n_items / min_items_per_thread);
}

// Runs fn(v) for v in [0, count) on `nthreads` host threads, each with a contiguous range (fn
// writes to places of its own v only, so the outcome does not depend on the thread count).
template <typename Fn> void for_each_item(int64_t count, int nthreads, Fn fn) {
    if (nthreads <= 1) {
        for (int64_t v = 0; v < count; ++v) fn(v);
        return;
    }
    std::atomic<bool> failed{false};
    std::vector<std::thread> pool;
    for (int th = 0; th < nthreads; ++th)
        pool.emplace_back([&, th] {
            try {
                for (int64_t v = count * th / nthreads; v < count * (th + 1) / nthreads; ++v) fn(v);
            } catch (...) {
                failed = true;
            }
        });
    for (std::thread &t : pool) t.join();
    if (failed) throw std::bad_alloc();
}

// Re-packs the rows `list` of the CSR matrix into units of uniform padded length and appends
// them to `out` (see RowPack).  local(c) maps a column index to what the kernel should index
// its operand with.  First the units are cut (row lengths only), then their entries are filled
// in, unit by unit on the host threads: a unit's place in the arrays follows from the cuts.
template <typename LocalFn>
void pack_rows(const int32_t *rowptr, const int32_t *colidx, const unsigned char *vals, int es,
               std::vector<int32_t> list, const PackRules &rules, bool may_sort, LocalFn local,
               RowPack &out) {
    auto len = [&](int32_t j) { return (int64_t)rowptr[j + 1] - rowptr[j]; };
    const int64_t count = (int64_t)list.size();
    // empty rows last, so that no unit mixes them with rows that need padding entries
    std::stable_partition(list.begin(), list.end(), [&](int32_t j) { return len(j) > 0; });
    int64_t real = 0;
    for (int32_t j : list) real += len(j);
    if (may_sort && count > 0) {
        // padded size in the given order; re-order by length when padding would cost over 15 %
        int64_t padded = 0;
        for (int64_t p0 = 0; p0 < count; p0 += rules.max_rows) {
            const int64_t p1 = std::min(count, p0 + rules.max_rows);
            int64_t mx = 0;
            for (int64_t q = p0; q < p1; ++q) mx = std::max(mx, len(list[q]));
            padded += mx * (p1 - p0);
        }
        if (padded > real + real * 15 / 100) {
            // longest first, rows of one length in their given order: by counting when the
            // lengths are a small range, else by comparison
            int64_t longest = 0;
            for (int32_t j : list) longest = std::max(longest, len(j));
            if (longest <= 4 * count + 1024) {
                std::vector<int64_t> start((size_t)longest + 2, 0);
                for (int32_t j : list) ++start[(size_t)(longest - len(j)) + 1];
                for (size_t b = 1; b < start.size(); ++b) start[b] += start[b - 1];
                std::vector<int32_t> sorted((size_t)count);
                for (int32_t j : list) sorted[(size_t)start[(size_t)(longest - len(j))]++] = j;
                list.swap(sorted);
            } else {
                std::stable_sort(list.begin(), list.end(),
                                 [&](int32_t a, int32_t b) { return len(a) > len(b); });
            }
            out.sorted = true;
        }
    }
    const int64_t list_base = (int64_t)out.rows.size();
    out.rows.insert(out.rows.end(), list.begin(), list.end());
    const size_t first_unit = out.units.size();
    // every unit starts at a multiple of four entries (16-byte aligned pieces for the kernels'
    // bulk copies, which may also read up to three entries past a unit's end)
    int64_t at = (int64_t)out.idx32.size();
    int64_t pos = 0;
    while (pos < count) {
        UnitDesc u{};
        u.row_begin = (int32_t)(list_base + pos);
        u.entry_base = at;
        const int64_t len0 = len(list[pos]);
        int64_t L = len0;
        int64_t take = 1;
        if (rules.split_groups > 1 && len0 >= kSplitMinSlots) {
            int split = pow2_at_least((len0 + kSplitPartSlots - 1) / kSplitPartSlots);
            split = std::min(split, rules.split_groups);
            const int cap = rules.split_groups / split;
            while (take < cap && pos + take < count && len(list[pos + take]) >= kSplitMinSlots) {
                L = std::max(L, len(list[pos + take]));
                ++take;
            }
            u.split = split;
        } else {
            u.split = 1;
            while (take < rules.max_rows && pos + take < count) {
                const int64_t ln = len(list[pos + take]);
                if ((ln == 0) != (len0 == 0)) break;
                if (rules.split_groups > 1 && ln >= kSplitMinSlots) break;
                const int64_t nl = std::max(L, ln);
                if (nl * (take + 1) > rules.max_slots) break;
                L = nl;
                ++take;
            }
        }
        u.n_rows = (int32_t)take;
        u.slots = (int32_t)L;
        out.units.push_back(u);
        at = (at + take * L + 3) / 4 * 4;
        pos += take;
    }
    const int64_t end = at + kPackSpareSlots;         // spare zero entries behind the last unit
    out.idx32.resize((size_t)end);
    out.vals.resize((size_t)end * es);
    const int64_t n_new = (int64_t)(out.units.size() - first_unit);
    if (n_new == 0) {
        std::memset(out.idx32.data() + at, 0, (size_t)kPackSpareSlots * 4);
        std::memset(out.vals.data() + (size_t)at * es, 0, (size_t)kPackSpareSlots * es);
    }
    for_each_item(n_new, host_threads(real, n_new, 64), [&](int64_t k) {
        const UnitDesc &u = out.units[first_unit + (size_t)k];
        const int64_t next = k + 1 < n_new ? out.units[first_unit + (size_t)k + 1].entry_base : end;
        const int64_t L = u.slots;
        int32_t *ip = out.idx32.data() + u.entry_base;
        unsigned char *vp = out.vals.data() + (size_t)u.entry_base * es;
        for (int64_t q = 0; q < u.n_rows; ++q) {
            const int32_t j = out.rows[(size_t)u.row_begin + (size_t)q];
            const int64_t k0 = rowptr[j], ln = len(j);
            for (int64_t sl = 0; sl < ln; ++sl) *ip++ = (int32_t)local(colidx[k0 + sl]);
            std::memcpy(vp, vals + (size_t)k0 * es, (size_t)ln * es);
            // padding repeats the last entry's index with value 0 (units of empty rows have L = 0)
            for (int64_t sl = ln; sl < L; ++sl) *ip++ = (int32_t)local(colidx[k0 + ln - 1]);
            std::memset(vp + (size_t)ln * es, 0, (size_t)(L - ln) * es);
            vp += (size_t)L * es;
        }
        const int64_t filled = u.entry_base + (int64_t)u.n_rows * L;
        std::memset(out.idx32.data() + filled, 0, (size_t)(next - filled) * 4);
        std::memset(out.vals.data() + (size_t)filled * es, 0, (size_t)(next - filled) * es);
    });
}

}  // namespace

namespace {

// Second-phase block of one tile (see TileDesc): the fused rows, longest first, cut into units
// of one padded length each.  A unit ends when the next row is shorter and the unit already
// has 64 rows, or when the next row would be padded by more than a quarter.  The padded length
// (stride) is even so that value pairs are aligned; padding entries repeat the row's last
// column with value 0.  local(c) is what the kernel finds the D1 row of column c with.
struct TileBlock {
    std::vector<unsigned char> bytes;
    std::vector<int32_t> rows;      // fused rows in block order
    int32_t n_units = 0, n_entries = 0;
};

template <typename LocalFn>
TileBlock pack_tile(const int32_t *rowptr, const int32_t *colidx, const unsigned char *vals, int es,
                    std::vector<int32_t> list, LocalFn local) {
    auto len = [&](int32_t j) { return (int64_t)rowptr[j + 1] - rowptr[j]; };
    auto align16 = [](size_t x) { return (x + 15) / 16 * 16; };
    TileBlock tb;
    std::stable_sort(list.begin(), list.end(), [&](int32_t a, int32_t b) { return len(a) > len(b); });
    tb.rows = list;
    std::vector<TileUnit> units;
    std::vector<uint16_t> idx;
    std::vector<unsigned char> val;
    const int64_t count = (int64_t)list.size();
    int64_t pos = 0;
    while (pos < count) {
        const int64_t L = len(list[pos]);
        const int64_t stride = (L + 1) / 2 * 2;
        int64_t take = 1;
        while (pos + take < count) {
            const int64_t ln = len(list[pos + take]);
            if (ln == L) {
                ++take;
                continue;
            }
            if (take >= 64 || ln * 4 < L * 3 || ln == 0) break;
            ++take;
        }
        TileUnit u{};
        u.entry_base = (int32_t)idx.size();
        u.row_begin = (int32_t)pos;
        u.n_rows = (int32_t)take;
        u.slots = (int32_t)(stride | (L << 16));
        {
            const size_t at0 = idx.size();
            idx.resize(at0 + (size_t)(take * stride), 0);
            val.resize(idx.size() * es, 0);
            uint16_t *ip = idx.data() + at0;
            unsigned char *vp = val.data() + at0 * es;
            for (int64_t q = pos; q < pos + take; ++q) {
                const int32_t j = list[q];
                const int64_t k0 = rowptr[j], ln = len(j);
                for (int64_t sl = 0; sl < ln; ++sl) *ip++ = (uint16_t)local(colidx[k0 + sl]);
                std::memcpy(vp, vals + (size_t)k0 * es, (size_t)ln * es);
                if (ln > 0)
                    for (int64_t sl = ln; sl < stride; ++sl) *ip++ = (uint16_t)local(colidx[k0 + ln - 1]);
                else
                    ip += stride;
                vp += (size_t)stride * es;
            }
        }
        units.push_back(u);
        pos += take;
    }
    const size_t off_rows2 = align16(units.size() * sizeof(TileUnit));
    const size_t off_idx = align16(off_rows2 + list.size() * 4);
    const size_t off_val = align16(off_idx + idx.size() * 2);
    tb.bytes.assign(align16(off_val + val.size()), 0);
    if (!units.empty()) std::memcpy(tb.bytes.data(), units.data(), units.size() * sizeof(TileUnit));
    if (!list.empty()) std::memcpy(tb.bytes.data() + off_rows2, list.data(), list.size() * 4);
    // operand positions: the even slots of all rows first, then the odd slots, so that the two
    // positions of a pair come from different arrays, by two plain 16-bit reads (one 32-bit read
    // of both would have to be taken apart again by the vector ALU, the scarce unit there)
    uint16_t *ip = reinterpret_cast<uint16_t *>(tb.bytes.data() + off_idx);
    const size_t pairs = idx.size() / 2;
    for (size_t q = 0; q < pairs; ++q) {
        ip[q] = idx[2 * q];
        ip[pairs + q] = idx[2 * q + 1];
    }
    if (!val.empty()) std::memcpy(tb.bytes.data() + off_val, val.data(), val.size());
    tb.n_units = (int32_t)units.size();
    tb.n_entries = (int32_t)idx.size();
    return tb;
}

}  // namespace

// Units of a packed row list of `count` rows: a unit is one workgroup; short lists are cut into
// smaller units (down to one row per lane group) so that they still spread over the machine.
static PackRules pack_rules(const InspectorInput &in, int64_t count, int sw) {
    const int v = vec_elems(in.dtype);
    const int vv = in.ccol % v == 0 ? v : 1;
    const int groups = kSpmmThreads / lane_group(sw, vv);
    const int64_t want = (count + 1023) / 1024;
    return PackRules{(int)std::min<int64_t>(kUnitRows, std::max<int64_t>(groups, want)), kUnitSlots,
                     groups};
}

// The gather kernel stages the entries of a unit whose rows are not split in LDS arrays of
// kUnitSlots entries; a unit beyond that would write past them.  pack_rows never cuts one (rows that
// long are split), this is the check behind that.
static bool units_fit_staging(const RowPack &pk) {
    for (const UnitDesc &u : pk.units)
        if (u.split <= 1 && (int64_t)u.n_rows * u.slots > kUnitSlots) return false;
    return true;
}

tf_status build_schedule(const InspectorInput &in, Schedule &s, std::string &err) {
    const int64_t n = in.n;
    const int es = elem_size(in.dtype);
#ifdef TF_TIMING
    auto tf_tick = std::chrono::steady_clock::now();
#endif
    s = Schedule();
    s.n = n;
    s.nnz = in.nnz;

    // ---- column slice -------------------------------------------------------------------
    const int v = vec_elems(in.dtype);
    int64_t max_cs = in.b_is_sparse ? 64 * v : kMaxMfmaSliceCols;
    if (in.ccol % v != 0) max_cs = 64;                 // scalar lanes: one column per lane
    int64_t cs = in.col_slice > 0 ? in.col_slice : in.ccol;
    if (in.col_slice < 0) {
        err = "col_slice must be >= 0";
        return TF_EINVAL;
    }
    cs = std::min<int64_t>(cs, in.ccol);
    if (cs > max_cs) {
        if (in.col_slice > 0) {
            err = "col_slice is wider than the kernels cover for this shape";
            return TF_EUNSUPPORTED;
        }
        cs = max_cs;
    }
    if (in.ccol % v == 0 && cs % v != 0 && cs != in.ccol) {
        err = "col_slice must be a multiple of 16 bytes of elements";
        return TF_EINVAL;
    }
    // ---- fast-memory model --------------------------------------------------------------
    // Per D1 row: the row itself, its id in two buffers (this tile's and the next one's), and an
    // estimate of its share of the second-phase block (row id, packed entries of an average row).
    // The C slice of a dense B takes LDS for good only when the waves read their operands from it.
    const int64_t avg_nnz = n > 0 ? (in.nnz + n - 1) / n : 0;
    s.lds_meta_bytes_per_row = 8 + 4 + avg_nnz * (2 + es);
    const int64_t b_stage = in.b_is_sparse ? lds_sparse_b_bytes_per_row(in.dtype) : 0;
    s.lds_row_granule = lds_row_granule(in.b_is_sparse);
    s.fast_mem_bytes = in.fast_mem_bytes;
    auto model = [&](int64_t width) {
        const bool c_regs = !in.b_is_sparse &&
                            c_in_registers(in.dtype, mfma_blocks((int)width),
                                           mfma_ksteps_special(in.dtype, (int)in.bcol, (int)in.ccol, (int)width));
        s.lds_fixed_bytes =
            (c_regs ? 0 : lds_fixed_bytes(in.dtype, in.b_is_sparse, (int)in.bcol, (int)width)) + 256;
        s.lds_bytes_per_row =
            lds_ldl(in.dtype, in.b_is_sparse, (int)width) * es + s.lds_meta_bytes_per_row + b_stage;
    };
    model(cs);
    // ---- the caller left the tiling to the library ----------------------------------------
    // (no tile size, no tile count, no flag that fixes the kind of tiles).  Then: a quarter of the
    // compute units as the wanted number of tiles (with all of them a small matrix gets tiles of a
    // handful of rows, which fuse nothing); for a dense B whose C operands sit in registers, half
    // of the LDS per tile when that still holds kWantedTileRows rows, so that two workgroups share
    // a compute unit; consecutive or graph-grown tiles, whichever moves fewer bytes; and fused rows
    // that would keep the whole tile machinery alive for next to no work are left to the second
    // wavefront (see below).
    const bool automatic = in.ct_size == 0 && in.p == 0 &&
                           !(in.flags & (TF_FLAG_REORDER | TF_FLAG_NO_SPLIT));
    s.automatic = automatic;
    if (automatic && !in.b_is_sparse && in.fast_mem_bytes >= 128 * 1024) {
        const bool c_regs = c_in_registers(in.dtype, mfma_blocks((int)cs),
                                           mfma_ksteps_special(in.dtype, (int)in.bcol, (int)in.ccol, (int)cs));
        const int64_t half = in.fast_mem_bytes / 2;
        if (c_regs && s.lds_fixed_bytes + kWantedTileRows * s.lds_bytes_per_row <= half)
            s.fast_mem_bytes = half;
    }
    // ---- step 1: tile size --------------------------------------------------------------
    const int64_t ct = in.ct_size > 0 ? in.ct_size : 2048;
    const int64_t p = in.p > 0 ? in.p : (automatic ? std::max(1, in.n_cu / 4) : 32);
    int64_t t = ct;
    if (n > 0 && (n + ct - 1) / ct < p) t = (n + p - 1) / p;
    if (t < 1) t = 1;
    s.t = (int32_t)std::min<int64_t>(t, INT32_MAX);

    // A default slice is narrowed (cCol / 2, / 4, ... rounded up to 16 columns; thirds leave a
    // ragged last slice and measured worse than either neighbour) until the fast
    // memory holds a tile of t rows, or of kWantedTileRows if t is larger: a C slice that fills
    // the LDS leaves tiles of a few rows, which fuse nothing.  If no width gets there the one
    // with the most rows is taken.  A slice the caller asked for is taken as given.
    if (in.col_slice == 0) {
        auto capacity = [&]() -> int64_t {
            const int64_t room = s.fast_mem_bytes - s.lds_fixed_bytes;
            if (room < s.lds_bytes_per_row) return 0;
            return room / s.lds_bytes_per_row / s.lds_row_granule * s.lds_row_granule;
        };
        const int64_t want = round_up(std::min<int64_t>(std::max<int64_t>(t, 1), kWantedTileRows),
                                      s.lds_row_granule);
        const int64_t widest = cs;
        int64_t best_cs = cs, best_rows = capacity();
        for (int64_t k = 2; best_rows < want && cs > 16; k *= 2) {
            const int64_t c = round_up((widest + k - 1) / k, 16);
            if (c >= cs) continue;
            cs = c;
            model(cs);
            if (capacity() > best_rows) {
                best_rows = capacity();
                best_cs = cs;
            }
        }
        cs = best_cs;
        model(cs);
    }
    if (tile_footprint(s, 1) > s.fast_mem_bytes) {
        err = "fast_mem_bytes cannot hold one D1 row of the chosen column slice (plus the C slice)";
        return TF_EUNSUPPORTED;
    }
    s.col_slice = (int32_t)cs;
    s.n_slices = (int32_t)((in.ccol + cs - 1) / cs);

    // ---- tiles: lists of first-operation rows -------------------------------------------
    // first_rows holds the rows tile after tile; tile_first_ptr delimits the tiles.
    const bool allow_split = !(in.flags & TF_FLAG_NO_SPLIT);
    struct Tiling {
        std::vector<int32_t> first_rows, tile_first_ptr;
        int64_t n_coarse = 0;
        bool grown = false;
    };
    auto make_grown = [&](Tiling &tl) {
        // Tiles grown along the dependence graph: as many rows as fit the fast memory (and at
        // most t), collected breadth first from the lowest row not yet in a tile by following
        // each row's column indices; when a search runs dry the tile goes on from the next
        // free row.  Rows inside a tile are kept in ascending order.
        tl.grown = true;
        tl.first_rows.resize((size_t)n);
        tl.tile_first_ptr.assign(1, 0);
        int64_t cap = std::min<int64_t>(automatic ? 65536 : t, 65536);
        while (cap > 1 && tile_footprint(s, cap) > s.fast_mem_bytes) --cap;
        cap = std::max<int64_t>(1, cap / s.lds_row_granule * s.lds_row_granule);
        if (tile_footprint(s, cap) > s.fast_mem_bytes) cap = 1;
        // One workgroup per compute unit walks the tiles of its column slice, so a tile count that
        // is not a multiple of the workgroups per slice leaves most of them waiting for the few
        // that got one tile more (304 tiles on 256 units: two rounds for the work of 1.2).  The
        // tiles are made smaller (by less than half) so that the count becomes such a multiple.
        // With fewer tiles than workgroups there is nothing to balance.
        if (n > 0 && in.n_cu > 0) {
            const int64_t per_slice = std::max<int64_t>(1, in.n_cu / s.n_slices);
            const int64_t count0 = (n + cap - 1) / cap;
            if (count0 >= per_slice) {
                const int64_t count = round_up(count0, per_slice);
                const int64_t even = round_up((n + count - 1) / count, s.lds_row_granule);
                if (even >= 1 && even < cap) cap = even;
            }
        }
        // (Growing the tiles of several row ranges at once on the host threads was measured: tiles
        // cut off at the end of a range fuse less -- 80.6 % of config 2's rows with four ranges, 74 %
        // with ranges of one tile height, against 82 % -- which costs every execution more than the
        // millisecond of inspector time it saves.)
        // tile_no[row]: number of the row's tile, -1 while the row is free
        std::vector<int32_t> tile_no((size_t)n, -1), queue;
        queue.reserve((size_t)cap);
        int64_t seed = 0, filled = 0;
        int32_t vt = 0;
        while (filled < n) {
            queue.clear();
            size_t head = 0;
            while ((int64_t)queue.size() < cap && filled + (int64_t)queue.size() < n) {
                if (head == queue.size()) {               // start (or restart) from a free row
                    while (tile_no[seed] >= 0) ++seed;
                    tile_no[seed] = vt;
                    queue.push_back((int32_t)seed);
                    continue;
                }
                const int32_t j = queue[head++];
                for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) {
                    const int32_t c = in.colidx[q];
                    if (tile_no[c] < 0 && (int64_t)queue.size() < cap) {
                        tile_no[c] = vt;
                        queue.push_back(c);
                    }
                }
            }
            filled += (int64_t)queue.size();
            tl.tile_first_ptr.push_back((int32_t)filled);
            ++vt;
        }
        // the rows of every tile in ascending order: one pass over the rows instead of a sort per tile
        std::vector<int32_t> cursor(tl.tile_first_ptr.begin(), tl.tile_first_ptr.end() - 1);
        for (int64_t row = 0; row < n; ++row)
            tl.first_rows[(size_t)cursor[(size_t)tile_no[(size_t)row]]++] = (int32_t)row;
        tl.n_coarse = (int64_t)tl.tile_first_ptr.size() - 1;
    };
    auto make_consecutive = [&](Tiling &tl) {
        // Algorithm 1: uniform tiles of t consecutive rows (step 1), halved until they fit (step 2)
        tl.first_rows.resize((size_t)n);
        tl.tile_first_ptr.assign(1, 0);
        std::vector<Range> tiles;
        for (int64_t i0 = 0; i0 < n; i0 += t) {
            ++tl.n_coarse;
            split_tile(s, Range{i0, std::min(n, i0 + t)}, allow_split, tiles);
        }
        std::iota(tl.first_rows.begin(), tl.first_rows.end(), 0);
        for (const Range &r : tiles) tl.tile_first_ptr.push_back((int32_t)r.i1);
    };
    // What a tiling is worth, without packing anything: the stored entries of the rows it fuses
    // (all of them, and those of rows that are not direct rows) and the number of D1 rows it spills.
    struct Worth {
        int64_t fused_nnz = 0, lds_nnz = 0, lds_rows = 0, spill_rows = 0;
        std::vector<uint8_t> spilled;      // the spill set of the tiling (before any row is demoted)
    };
    auto evaluate = [&](const Tiling &tl) {
        const int64_t ntl = (int64_t)tl.tile_first_ptr.size() - 1;
        std::vector<int32_t> tile_of((size_t)n);
        for (int64_t vt = 0; vt < ntl; ++vt)
            for (int64_t q = tl.tile_first_ptr[vt]; q < tl.tile_first_ptr[vt + 1]; ++q)
                tile_of[tl.first_rows[q]] = (int32_t)vt;
        std::vector<uint8_t> spilled((size_t)n, 0);
        std::vector<Worth> part((size_t)ntl);
        for_each_item(ntl, host_threads(in.nnz, ntl, 16), [&](int64_t vt) {
            Worth &w = part[(size_t)vt];
            for (int64_t fq = tl.tile_first_ptr[vt]; fq < tl.tile_first_ptr[vt + 1]; ++fq) {
                const int64_t j = tl.first_rows[fq];
                const int64_t k0 = in.rowptr[j], k1 = in.rowptr[j + 1];
                bool inside = k1 - k0 < 32768;
                for (int64_t q = k0; inside && q < k1; ++q) inside = tile_of[in.colidx[q]] == (int32_t)vt;
                if (inside) {
                    w.fused_nnz += k1 - k0;
                    if (!(k1 == k0 || (k1 - k0 == 1 && in.colidx[k0] == (int32_t)j))) {
                        w.lds_nnz += k1 - k0;
                        ++w.lds_rows;
                    }
                } else {
                    for (int64_t q = k0; q < k1; ++q) {
                        uint8_t *m = &spilled[(size_t)in.colidx[q]];
                        if (!__atomic_load_n(m, __ATOMIC_RELAXED)) __atomic_store_n(m, (uint8_t)1, __ATOMIC_RELAXED);
                    }
                }
            }
        });
        Worth w;
        for (const Worth &pw : part) {
            w.fused_nnz += pw.fused_nnz;
            w.lds_nnz += pw.lds_nnz;
            w.lds_rows += pw.lds_rows;
        }
        w.spill_rows = std::accumulate(spilled.begin(), spilled.end(), (int64_t)0);
        w.spilled = std::move(spilled);
        return w;
    };
    // Rows that reach far (graphs): mean distance, over a sample of the entries, between a row and
    // the columns it holds, in bytes of D1 rows, against the 4 MiB of one XCD's L2.
    bool far_rows = false;
    if (n > 0 && in.nnz > 0) {
        // the sample: 64 runs of up to 1024 consecutive rows, evenly spread (runs, not single rows:
        // their entries are read as a stream)
        const int64_t run = std::min<int64_t>(1024, std::max<int64_t>(1, n / 64));
        double dist = 0.0;
        int64_t cnt = 0;
        for (int64_t k = 0; k < 64; ++k) {
            const int64_t j0 = std::min(n - run, n * k / 64);
            for (int64_t j = j0; j < j0 + run; ++j)
                for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) {
                    dist += std::abs((double)in.colidx[q] - (double)j);
                    ++cnt;
                }
        }
        far_rows = cnt > 0 && dist / (double)cnt * (double)in.ccol * es > 4.0 * 1048576.0;
    }
    s.far_rows = far_rows;
    bool demote_lds_rows = false;
    std::vector<uint8_t> known_spill;      // spill set of the chosen tiling, when it was evaluated
    Tiling tiling;
    TF_TICK("setup, far-row sample");
    if (in.flags & TF_FLAG_REORDER) {
        make_grown(tiling);
        TF_TICK("grown tiles");
    } else {
        make_consecutive(tiling);
        if (automatic && in.nnz > 0) {
            Worth w = evaluate(tiling);
            TF_TICK("consecutive tiles + worth");
            // consecutive tiles that fuse less than half of the work of a matrix whose rows stay
            // near the diagonal (a stencil in natural ordering): try tiles grown along the graph
            // and keep them if they spill fewer D1 rows, i.e. move fewer bytes
            if (!far_rows && 2 * w.fused_nnz < in.nnz) {
                Tiling grown;
                make_grown(grown);
                TF_TICK("grown tiles");
                Worth wg = evaluate(grown);
                TF_TICK("worth of grown tiles");
                if (wg.spill_rows < w.spill_rows) {
                    tiling = std::move(grown);
                    w = std::move(wg);
                }
            }
            // Fused rows that read the LDS tile make every workgroup keep a tile in LDS and pass
            // two barriers per tile.  When they hold under 2 % of the entries that machinery costs
            // more than the D1 round trip it saves (measured on the graph configurations: a
            // handful of such rows, first wavefront 0.44 ms with tiles against 0.31 ms without):
            // they are left to the second wavefront and the first wavefront streams.
            demote_lds_rows = w.lds_rows > 0 && 50 * w.lds_nnz < in.nnz;
            known_spill = std::move(w.spilled);
        }
    }
    s.first_rows = std::move(tiling.first_rows);
    s.tile_first_ptr = std::move(tiling.tile_first_ptr);
    s.n_coarse_tiles = tiling.n_coarse;
    s.grown_tiles = tiling.grown;
    const int64_t nt = (int64_t)s.tile_first_ptr.size() - 1;
    for (int64_t vt = 0; vt < nt; ++vt) {
        const int64_t rows = s.tile_first_ptr[vt + 1] - s.tile_first_ptr[vt];
        if (tile_footprint(s, rows) > s.fast_mem_bytes) {
            err = "a tile does not fit the fast memory and splitting is disabled";
            return TF_EUNSUPPORTED;
        }
        s.max_tile_rows = std::max(s.max_tile_rows, rows);
    }

    // ---- classification: a row is fused when every column it refers to is produced by the
    // tile that produces its own row; fused rows are packed with tile-local column indices ----
    s.tile_second_ptr.resize(nt + 1);
    s.spill.assign((size_t)n, 0);
    const unsigned char *vals = static_cast<const unsigned char *>(in.vals);
    std::vector<TileBlock> blocks((size_t)nt);
    // the packed entries of a tile name their D1 operand by its position in the LDS tile, in units of
    // 16 bytes (16 bits: enough for 1 MiB of tile)
    const int32_t pitch16 = (int32_t)(lds_ldl(in.dtype, in.b_is_sparse, (int)cs) * es / 16);
    if (s.max_tile_rows * pitch16 > 65536) {
        err = "a tile is larger than 1 MiB (tile-local operand offsets are 16 bit)";
        return TF_EUNSUPPORTED;
    }
    std::vector<int32_t> wf1;
    int64_t lds_nonempty = 0;          // fused rows that read the LDS tile and have entries
    // A row belongs to one tile: there it is a candidate for fusion and there its D1 row is
    // produced.  With TF_FLAG_SKIP_UNREAD the D1 rows that no row of A reads are not produced at
    // all: they leave the tiles' first lists (a tile keeps at least one row) and get no place in LDS.
    // (member_*: the tiles' rows before any are taken out; the lists themselves when none are)
    const bool skip_rows = (in.flags & TF_FLAG_SKIP_UNREAD) != 0;
    std::vector<int32_t> all_ptr, all_rows;
    if (skip_rows) {
        all_ptr = s.tile_first_ptr;
        all_rows = s.first_rows;
    }
    const std::vector<int32_t> &member_ptr = skip_rows ? all_ptr : s.tile_first_ptr;
    const std::vector<int32_t> &member_rows = skip_rows ? all_rows : s.first_rows;
    if (skip_rows) {
        std::vector<uint8_t> read((size_t)n, 0);
        for (int64_t q = 0; q < in.nnz; ++q) read[in.colidx[q]] = 1;
        int64_t kept = 0;
        s.max_tile_rows = 0;
        for (int64_t vt = 0; vt < nt; ++vt) {
            const int64_t before = kept;
            for (int64_t q = member_ptr[vt]; q < member_ptr[vt + 1]; ++q)
                if (read[member_rows[q]]) s.first_rows[kept++] = member_rows[q];
            if (kept == before && member_ptr[vt + 1] > member_ptr[vt])
                s.first_rows[kept++] = member_rows[member_ptr[vt]];
            s.tile_first_ptr[vt + 1] = (int32_t)kept;
            s.max_tile_rows = std::max(s.max_tile_rows, kept - before);
        }
        s.first_rows.resize((size_t)kept);
    }
    std::vector<int32_t> tile_of((size_t)n), local_of((size_t)n, 0);
    // kept[row]: the tile produces the D1 row (always, unless unread rows are skipped);
    // direct_kind[row]: 1 = the row of D is the D1 row times its only entry, the diagonal one;
    // 2 = the row of D is empty; both leave from the registers that hold the D1 row
    std::vector<uint8_t> kept((size_t)n, 0), direct_kind((size_t)n, 0);
    // (every row is in one tile: the threads write to places of their own tiles only)
    for_each_item(nt, host_threads(in.nnz, nt, 16), [&](int64_t vt) {
        for (int64_t q = member_ptr[vt]; q < member_ptr[vt + 1]; ++q)
            tile_of[member_rows[q]] = (int32_t)vt;
        for (int64_t q = s.tile_first_ptr[vt]; q < s.tile_first_ptr[vt + 1]; ++q) {
            local_of[s.first_rows[q]] = (int32_t)(q - s.tile_first_ptr[vt]);
            kept[s.first_rows[q]] = 1;
        }
    });
    std::vector<int32_t> seen((size_t)n, -1);      // Eq. 2: distinct columns per tile
    // Per tile: which of its rows are fused, and their packed block.  Tiles are independent (a fused
    // row only names columns of its own tile, so even `seen` is written at disjoint places), which
    // lets several host threads share the tiles of a large matrix; the results are put together
    // in tile order afterwards, so the schedule does not depend on the number of threads.
    struct TileResult {
        std::vector<int32_t> wf1, direct, demoted_rows;
        int64_t tile_nnz = 0, uc = 0, nj = 0, demoted = 0, lds_nonempty = 0;
    };
    std::vector<TileResult> res((size_t)nt);
    auto classify = [&](int64_t vt) {
        TileResult &tr = res[(size_t)vt];
        std::vector<int32_t> tile_rows;
        for (int64_t fq = member_ptr[vt]; fq < member_ptr[vt + 1]; ++fq) {
            const int64_t j = member_rows[fq];
            // (a row of 32768 entries or more, possible only with duplicates, is left to the second
            // wavefront: the tile units store lengths in 15 bits)
            bool inside = in.rowptr[j + 1] - in.rowptr[j] < 32768;
            for (int64_t q = in.rowptr[j]; inside && q < in.rowptr[j + 1]; ++q) {
                if (tile_of[in.colidx[q]] != (int32_t)vt) {
                    inside = false;
                    break;
                }
            }
            const int64_t ln = in.rowptr[j + 1] - in.rowptr[j];
            const bool direct = kept[j] && (ln == 0 || (ln == 1 && in.colidx[in.rowptr[j]] == (int32_t)j));
            if (inside && demote_lds_rows && !direct && ln > 0) {       // (a row without entries reads no tile)
                inside = false;
                ++tr.demoted;
                tr.demoted_rows.push_back((int32_t)j);
            }
            if (inside) {
                if (direct) {
                    direct_kind[j] = ln == 0 ? 2 : 1;
                    tr.direct.push_back((int32_t)j);
                } else {
                    tile_rows.push_back((int32_t)j);
                    direct_kind[j] = 3;          // fused through the LDS tile
                    if (ln > 0) ++tr.lds_nonempty;
                }
                for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) {
                    const int32_t c = in.colidx[q];
                    if (seen[c] != (int32_t)vt) {
                        seen[c] = (int32_t)vt;
                        ++tr.uc;
                    }
                }
                tr.tile_nnz += in.rowptr[j + 1] - in.rowptr[j];
            } else {
                tr.wf1.push_back((int32_t)j);
            }
        }
        tr.nj = (int64_t)(tile_rows.size() + tr.direct.size());
        blocks[(size_t)vt] = pack_tile(in.rowptr, in.colidx, vals, es, tile_rows,
                                       [&](int32_t c) { return local_of[c] * pitch16; });
    };
    TF_TICK("tile maps");
    for_each_item(nt, host_threads(in.nnz, nt, 16), classify);
    TF_TICK("classify + pack tiles");
    for (int64_t vt = 0; vt < nt; ++vt) {
        const TileResult &tr = res[(size_t)vt];
        const int64_t rows = s.tile_first_ptr[vt + 1] - s.tile_first_ptr[vt];
        wf1.insert(wf1.end(), tr.wf1.begin(), tr.wf1.end());
        s.tile_second_ptr[vt] = (int32_t)s.second_rows.size();
        s.second_rows.insert(s.second_rows.end(), blocks[(size_t)vt].rows.begin(),
                             blocks[(size_t)vt].rows.end());
        s.second_rows.insert(s.second_rows.end(), tr.direct.begin(), tr.direct.end());
        s.n_demoted_rows += tr.demoted;
        lds_nonempty += tr.lds_nonempty;
        s.n_lds_rows += (int64_t)blocks[(size_t)vt].rows.size();
        s.n_direct_rows += (int64_t)tr.direct.size();
        // Eq. 2 (diagnostic): (nz + uc + t + |J|) * cCol + idx, counted in elements; for a dense B
        // the tile's rows x bCol block of B is added to nz, a sparse B is unknown here.
        const double nz = (double)tr.tile_nnz + (in.b_is_sparse ? 0.0 : (double)rows * in.bcol);
        const double idx = (double)(rows + 1) + (double)tr.tile_nnz;
        s.eq2_cost_max = std::max(s.eq2_cost_max, (nz + tr.uc + rows + tr.nj) * (double)in.ccol + idx);
        s.fused_nnz += tr.tile_nnz;
    }
    s.tile_second_ptr[nt] = (int32_t)s.second_rows.size();
    s.n_fused_rows = (int64_t)s.second_rows.size();
    if (!s.grown_tiles && !std::is_sorted(wf1.begin(), wf1.end())) std::sort(wf1.begin(), wf1.end());

    TF_TICK("collect tiles");
    // ---- spill set ----------------------------------------------------------------------
    if (!known_spill.empty() && !(in.flags & TF_FLAG_SKIP_UNREAD)) {
        // the tiling was evaluated: its spill set is known; rows left to the second wavefront since
        // then add the rows they read
        s.spill = std::move(known_spill);
        for (const TileResult &tr : res)
            for (int32_t j : tr.demoted_rows)
                for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) s.spill[(size_t)in.colidx[q]] = 1;
    } else {
        // (several threads may mark the same row: every one of them stores the same byte)
        for_each_item((int64_t)wf1.size(), host_threads(in.nnz, (int64_t)wf1.size(), 4096), [&](int64_t k) {
            const int32_t j = wf1[(size_t)k];
            for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) {
                // (a marked row is not written again: the columns of hub rows would otherwise keep
                // their cache lines travelling between the threads)
                uint8_t *m = &s.spill[(size_t)in.colidx[q]];
                if (!__atomic_load_n(m, __ATOMIC_RELAXED)) __atomic_store_n(m, (uint8_t)1, __ATOMIC_RELAXED);
            }
        });
    }
    s.n_spill_rows = std::accumulate(s.spill.begin(), s.spill.end(), (int64_t)0);
    if (s.n_spill_rows > (int64_t)kInfoSlotMask) {
        err = "more than 2^28 D1 rows cross tiles";
        return TF_EUNSUPPORTED;
    }
    // Only the rows in the spill set reach device memory (one barrier: nothing else crosses tiles),
    // so the workspace has one slot per such row, in row order.
    s.spill_slot.assign((size_t)n, -1);
    {
        int32_t slot = 0;
        for (int64_t i = 0; i < n; ++i)
            if (s.spill[(size_t)i]) s.spill_slot[(size_t)i] = slot++;
    }
    // ---- layout of the workspace = column slices of the gather kernel ---------------------
    // On a matrix whose rows reach far (a graph) every XCD's L2 sees the same hot rows of D1 and
    // holds them all, whole: the eight caches together are worth one.  With n_sl slices each XCD
    // gathers sw-wide pieces of the rows, so the hot set is spread over the caches, at the price of
    // reading the packed entries of A once per slice.  Matrices whose rows stay near the diagonal
    // (stencils, bands) keep one slice: their operands are in the L2 anyway.
    {
        const int vv = in.ccol % v == 0 ? v : 1;
        int n_sl = 1;
        auto usable = [&](int k) {
            if (k == 1) return true;
            if (vv == 1 || in.ccol % k) return false;
            // (the MFMA phase stores 16-column blocks that start at multiples of the fused column
            // slice: they must not straddle a slice of the workspace)
            if (s.n_slices > 1 && cs % 16 != 0) return false;
            const int64_t sw = in.ccol / k;
            return sw % 16 == 0 && (sw & (sw - 1)) == 0 && sw * es >= 64;
        };
        if (in.gather_slices > 0) {
            if ((in.gather_slices != 1 && in.gather_slices != 2 && in.gather_slices != 4 &&
                 in.gather_slices != 8) || !usable(in.gather_slices)) {
                err = "gather_slices must be 1, 2, 4 or 8 and leave slices of a power of two of columns, "
                      "at least 16 and at least 64 bytes";
                return TF_EINVAL;
            }
            n_sl = in.gather_slices;
        } else if (!wf1.empty()) {
            const double row_bytes = (double)in.ccol * es;
            const bool large = (double)s.n_spill_rows * row_bytes > 64.0 * 1048576.0;
            if (far_rows && large)
                for (int k = 8; k > 1; k /= 2)
                    if (usable(k) && in.ccol / k * es >= kGatherSliceBytes) {
                        n_sl = k;
                        break;
                    }
        }
        s.d1.n_sl = n_sl;
        s.d1.sw = (int32_t)(in.ccol / n_sl);
        s.d1.rows = std::max<int64_t>(1, s.n_spill_rows);
        const int groups = kSpmmThreads / lane_group(s.d1.sw, vv);
        s.gather_r = groups >= 64 ? 1 : groups >= 32 ? 2 : 4;
    }
    TF_TICK("spill set, slots, layout");
    // ---- per-tile blocks (see TileDesc) ---------------------------------------------------
    s.tile_desc.resize((size_t)nt);
    s.first_stride = (int32_t)round_up(std::max<int64_t>(s.max_tile_rows, 1), 16);
    s.tile_first.assign((size_t)nt * s.first_stride, 0);
    s.tile_info.assign((size_t)nt * s.first_stride, 0u);
    if (s.n_direct_rows > 0) {
        s.tile_scale.resize((size_t)nt * s.first_stride * es);
        std::memset(s.tile_scale.data(), 0, s.tile_scale.size());
    }
    {
        int64_t total = 0;
        for (int64_t vt = 0; vt < nt; ++vt) {
            s.tile_desc[(size_t)vt].meta_off = total;
            total += (int64_t)blocks[(size_t)vt].bytes.size();
            s.second_block_cap = std::max<int64_t>(s.second_block_cap, (int64_t)blocks[(size_t)vt].bytes.size());
        }
        s.tile_meta_bytes = (size_t)total + 64;           // the kernels may read one piece past an empty block
        s.tile_meta.reset(new unsigned char[s.tile_meta_bytes]);
        std::memset(s.tile_meta.get() + total, 0, 64);
    }
    for_each_item(nt, host_threads(in.nnz, nt, 16), [&](int64_t vt) {
        const int64_t f0 = s.tile_first_ptr[vt], f1 = s.tile_first_ptr[vt + 1];
        TileBlock &tb = blocks[(size_t)vt];
        TileDesc &d = s.tile_desc[(size_t)vt];
        d.n_rows = (int32_t)(f1 - f0);
        d.n_units = tb.n_units;
        d.n_second = (int32_t)tb.rows.size();
        d.n_entries = tb.n_entries;
        d.s_bytes = (int32_t)tb.bytes.size();
        d.reserved = 0;
        int32_t *first = s.tile_first.data() + (size_t)vt * s.first_stride;
        uint32_t *info = s.tile_info.data() + (size_t)vt * s.first_stride;
        for (int64_t q = f0; q < f1; ++q) {
            const int32_t row = s.first_rows[q];
            first[q - f0] = row;
            uint32_t w = s.spill[row] ? (kInfoSpill | (uint32_t)s.spill_slot[row]) : 0u;
            if (direct_kind[row] == 1) {
                w |= kInfoDirect;
                std::memcpy(s.tile_scale.data() + ((size_t)vt * s.first_stride + (size_t)(q - f0)) * es,
                            vals + (size_t)in.rowptr[row] * es, (size_t)es);
            } else if (direct_kind[row] == 2) {
                w |= kInfoZero;
            }
            info[q - f0] = w;
        }
        // (padding repeats the last row, with an empty info word)
        for (int64_t q = f1 - f0; q < s.first_stride; ++q) first[q] = s.first_rows[f1 - 1];
        if (!tb.bytes.empty()) std::memcpy(s.tile_meta.get() + d.meta_off, tb.bytes.data(), tb.bytes.size());
        TileBlock().bytes.swap(tb.bytes);
    });
    // A plan none of whose fused rows reads the LDS tile needs no tiles at execution: the first
    // wavefront streams through the rows, and what happens to each finished D1 row is told by a word
    // per row.  (Fused rows without entries read nothing: where unread D1 rows are skipped some of
    // them have no D1 row of their own to leave with and sit in the tiles' second lists; by row they
    // are zero rows like the others.)  With TF_FLAG_SKIP_UNREAD only a CSR B streams: its kernel
    // leaves out single rows (kInfoSkip), the dense product works on blocks of sixteen.
    const bool skip_unread = in.flags & TF_FLAG_SKIP_UNREAD;
    s.streaming = n > 0 && lds_nonempty == 0 && (!skip_unread || in.b_is_sparse);
    if (s.streaming) {
        s.row_info.assign((size_t)n, 0u);
        const bool scales = s.n_direct_rows > 0;
        if (scales) {
            s.row_scale.resize((size_t)n * es);
            std::memset(s.row_scale.data(), 0, s.row_scale.size());
        }
        for_each_item(nt, host_threads(in.nnz, nt, 16), [&](int64_t vt) {
            for (int64_t q = member_ptr[vt]; q < member_ptr[vt + 1]; ++q) {
                const int32_t row = member_rows[q];
                uint32_t w = s.spill[row] ? (kInfoSpill | (uint32_t)s.spill_slot[row]) : 0u;
                if (direct_kind[row] == 1) {
                    w |= kInfoDirect;
                    std::memcpy(s.row_scale.data() + (size_t)row * es, vals + (size_t)in.rowptr[row] * es, (size_t)es);
                } else if (direct_kind[row] == 2 || direct_kind[row] == 3) {
                    w |= kInfoZero;
                }
                if (skip_unread && !kept[row]) w |= kInfoSkip;
                s.row_info[(size_t)row] = w;
            }
        });
    }
    {
        // LDS actually needed with the second-phase blocks staged: everything but the estimate
        const int64_t rows_cap = round_up(s.max_tile_rows, s.lds_row_granule);
        const int64_t need = s.lds_fixed_bytes + s.second_block_cap +
                             rows_cap * (s.lds_bytes_per_row - s.lds_meta_bytes_per_row + 8);
        s.second_block_in_lds = need <= s.fast_mem_bytes;
    }

    TF_TICK("tile blocks, row arrays");
    // ---- balance: units of the second wavefront --------------------------------------------
    const PackRules wf1_rules = pack_rules(in, (int64_t)wf1.size(), s.d1.sw);
    auto slot_of = [&](int32_t c) { return s.spill_slot[(size_t)c]; };
    pack_rows(in.rowptr, in.colidx, vals, es, wf1, wf1_rules, true, slot_of, s.wf1);
    if (!units_fit_staging(s.wf1)) {
        err = "internal: a unit of the second wavefront exceeds the staging arrays of the gather kernel";
        return TF_EUNSUPPORTED;
    }
    s.wf1_rows = s.wf1.rows;
    s.wf1_unit_ptr.clear();
    for (const UnitDesc &u : s.wf1.units) s.wf1_unit_ptr.push_back(u.row_begin);
    s.wf1_unit_ptr.push_back((int32_t)s.wf1_rows.size());
    TF_TICK("second-wavefront units");
    return TF_OK;
}

bool build_baseline_pack(const InspectorInput &in, Schedule &s) {
    std::vector<int32_t> all((size_t)in.n);
    std::iota(all.begin(), all.end(), 0);
    auto ident = [](int32_t c) { return c; };
    pack_rows(in.rowptr, in.colidx, static_cast<const unsigned char *>(in.vals), elem_size(in.dtype),
              all, pack_rules(in, in.n, s.d1.sw), true, ident, s.all);
    return units_fit_staging(s.all);
}

}  // namespace tf
