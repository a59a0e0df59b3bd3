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
    const int64_t end = at + 4;                       // four spare entries behind the last unit
    out.idx32.resize((size_t)end);
    out.vals.resize((size_t)end * es);
    const int64_t n_new = (int64_t)(out.units.size() - first_unit);
    if (n_new == 0) {
        std::memset(out.idx32.data() + at, 0, 4 * 4);
        std::memset(out.vals.data() + (size_t)at * es, 0, (size_t)4 * es);
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
static PackRules pack_rules(const InspectorInput &in, int64_t count) {
    const int v = vec_elems(in.dtype);
    const int vv = in.ccol % v == 0 ? v : 1;
    const int groups = kSpmmThreads / lane_group((int)in.ccol, vv);
    const int64_t want = (count + 1023) / 1024;
    return PackRules{(int)std::min<int64_t>(kUnitRows, std::max<int64_t>(groups, want)), kUnitSlots,
                     groups};
}

tf_status build_schedule(const InspectorInput &in, Schedule &s, std::string &err) {
    const int64_t n = in.n;
    const int es = elem_size(in.dtype);
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
    // ---- step 1: tile size --------------------------------------------------------------
    const int64_t ct = in.ct_size > 0 ? in.ct_size : 2048;
    const int64_t p = in.p > 0 ? in.p : 32;
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
    s.first_rows.resize((size_t)n);
    s.tile_first_ptr.assign(1, 0);
    if (in.flags & TF_FLAG_REORDER) {
        // Tiles grown along the dependence graph: as many rows as fit the fast memory (and at
        // most t), collected breadth first from the lowest row not yet in a tile by following
        // each row's column indices; when a search runs dry the tile goes on from the next
        // free row.  Rows inside a tile are kept in ascending order.
        int64_t cap = std::min<int64_t>(t, 65536);
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
        std::vector<uint8_t> taken((size_t)n, 0);
        std::vector<int32_t> queue;
        queue.reserve((size_t)cap);
        int64_t seed = 0, filled = 0;
        while (filled < n) {
            queue.clear();
            size_t head = 0;
            while ((int64_t)queue.size() < cap && filled + (int64_t)queue.size() < n) {
                if (head == queue.size()) {               // start (or restart) from a free row
                    while (taken[seed]) ++seed;
                    taken[seed] = 1;
                    queue.push_back((int32_t)seed);
                    continue;
                }
                const int32_t j = queue[head++];
                for (int64_t q = in.rowptr[j]; q < in.rowptr[j + 1]; ++q) {
                    const int32_t c = in.colidx[q];
                    if (!taken[c] && (int64_t)queue.size() < cap) {
                        taken[c] = 1;
                        queue.push_back(c);
                    }
                }
            }
            std::copy(queue.begin(), queue.end(), s.first_rows.begin() + filled);
            filled += (int64_t)queue.size();
            s.tile_first_ptr.push_back((int32_t)filled);
        }
        s.n_coarse_tiles = (int64_t)s.tile_first_ptr.size() - 1;
        for_each_item(s.n_coarse_tiles, host_threads(in.nnz, s.n_coarse_tiles, 16), [&](int64_t vt) {
            std::sort(s.first_rows.begin() + s.tile_first_ptr[vt], s.first_rows.begin() + s.tile_first_ptr[vt + 1]);
        });
    } else {
        // Algorithm 1: uniform tiles of t consecutive rows (step 1), halved until they fit (step 2)
        std::vector<Range> tiles;
        for (int64_t i0 = 0; i0 < n; i0 += t) {
            ++s.n_coarse_tiles;
            split_tile(s, Range{i0, std::min(n, i0 + t)}, allow_split, tiles);
        }
        std::iota(s.first_rows.begin(), s.first_rows.end(), 0);
        for (const Range &r : tiles) s.tile_first_ptr.push_back((int32_t)r.i1);
    }
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
    // A row belongs to one tile: there it is a candidate for fusion and there its D1 row is
    // produced.  With TF_FLAG_SKIP_UNREAD the D1 rows that no row of A reads are not produced at
    // all: they leave the tiles' first lists (a tile keeps at least one row) and get no place in LDS.
    std::vector<int32_t> member_ptr = s.tile_first_ptr, member_rows = s.first_rows;
    if (in.flags & TF_FLAG_SKIP_UNREAD) {
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
    for (int64_t vt = 0; vt < nt; ++vt) {
        for (int64_t q = member_ptr[vt]; q < member_ptr[vt + 1]; ++q)
            tile_of[member_rows[q]] = (int32_t)vt;
        for (int64_t q = s.tile_first_ptr[vt]; q < s.tile_first_ptr[vt + 1]; ++q)
            local_of[s.first_rows[q]] = (int32_t)(q - s.tile_first_ptr[vt]);
    }
    std::vector<int32_t> seen((size_t)n, -1);      // Eq. 2: distinct columns per tile
    // Per tile: which of its rows are fused, and their packed block.  Tiles are independent (a fused
    // row only names columns of its own tile, so even `seen` is written at disjoint places), which
    // lets several host threads share the tiles of a large matrix; the results are put together
    // in tile order afterwards, so the schedule does not depend on the number of threads.
    struct TileResult {
        std::vector<int32_t> wf1;
        int64_t tile_nnz = 0, uc = 0, nj = 0;
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
            if (inside) {
                tile_rows.push_back((int32_t)j);
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
        tr.nj = (int64_t)tile_rows.size();
        blocks[(size_t)vt] = pack_tile(in.rowptr, in.colidx, vals, es, tile_rows,
                                       [&](int32_t c) { return local_of[c] * pitch16; });
    };
    for_each_item(nt, host_threads(in.nnz, nt, 16), classify);
    for (int64_t vt = 0; vt < nt; ++vt) {
        const TileResult &tr = res[(size_t)vt];
        const int64_t rows = s.tile_first_ptr[vt + 1] - s.tile_first_ptr[vt];
        wf1.insert(wf1.end(), tr.wf1.begin(), tr.wf1.end());
        s.tile_second_ptr[vt] = (int32_t)s.second_rows.size();
        s.second_rows.insert(s.second_rows.end(), blocks[(size_t)vt].rows.begin(),
                             blocks[(size_t)vt].rows.end());
        // Eq. 2 (diagnostic): (nz + uc + t + |J|) * cCol + idx, counted in elements; for a dense B
        // the tile's rows x bCol block of B is added to nz, a sparse B is unknown here.
        const double nz = (double)tr.tile_nnz + (in.b_is_sparse ? 0.0 : (double)rows * in.bcol);
        const double idx = (double)(rows + 1) + (double)tr.tile_nnz;
        s.eq2_cost_max = std::max(s.eq2_cost_max, (nz + tr.uc + rows + tr.nj) * (double)in.ccol + idx);
        s.fused_nnz += tr.tile_nnz;
    }
    s.tile_second_ptr[nt] = (int32_t)s.second_rows.size();
    s.n_fused_rows = (int64_t)s.second_rows.size();
    if (!(in.flags & TF_FLAG_REORDER) && !std::is_sorted(wf1.begin(), wf1.end())) std::sort(wf1.begin(), wf1.end());

    // ---- spill set ----------------------------------------------------------------------
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
    s.n_spill_rows = std::accumulate(s.spill.begin(), s.spill.end(), (int64_t)0);
    // ---- per-tile blocks (see TileDesc) ---------------------------------------------------
    s.tile_desc.resize((size_t)nt);
    s.first_stride = (int32_t)round_up(std::max<int64_t>(s.max_tile_rows, 1), 16);
    s.tile_first.assign((size_t)nt * s.first_stride, 0);
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
        for (int64_t q = f0; q < f1; ++q) {
            const int32_t row = s.first_rows[q];
            first[q - f0] = (int32_t)((uint32_t)row | (s.spill[row] ? kSpillBit : 0u));
        }
        for (int64_t q = f1 - f0; q < s.first_stride; ++q) first[q] = s.first_rows[f1 - 1];
        if (!tb.bytes.empty()) std::memcpy(s.tile_meta.get() + d.meta_off, tb.bytes.data(), tb.bytes.size());
        TileBlock().bytes.swap(tb.bytes);
    });
    {
        // LDS actually needed with the second-phase blocks staged: everything but the estimate
        const int64_t rows_cap = round_up(s.max_tile_rows, s.lds_row_granule);
        const int64_t need = s.lds_fixed_bytes + s.second_block_cap +
                             rows_cap * (s.lds_bytes_per_row - s.lds_meta_bytes_per_row + 8);
        s.second_block_in_lds = need <= s.fast_mem_bytes;
    }

    // ---- balance: units of the second wavefront --------------------------------------------
    const PackRules wf1_rules = pack_rules(in, (int64_t)wf1.size());
    auto ident = [](int32_t c) { return c; };
    pack_rows(in.rowptr, in.colidx, vals, es, wf1, wf1_rules, true, ident, s.wf1);
    s.wf1_rows = s.wf1.rows;
    s.wf1_unit_ptr.clear();
    for (const UnitDesc &u : s.wf1.units) s.wf1_unit_ptr.push_back(u.row_begin);
    s.wf1_unit_ptr.push_back((int32_t)s.wf1_rows.size());
    return TF_OK;
}

void build_baseline_pack(const InspectorInput &in, Schedule &s) {
    std::vector<int32_t> all((size_t)in.n);
    std::iota(all.begin(), all.end(), 0);
    auto ident = [](int32_t c) { return c; };
    pack_rows(in.rowptr, in.colidx, static_cast<const unsigned char *>(in.vals), elem_size(in.dtype),
              all, pack_rules(in, in.n), true, ident, s.all);
}

}  // namespace tf
