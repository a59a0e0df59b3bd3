// Internal declarations shared by the inspector (host), the kernels (device) and the C ABI.
#pragma once
#include <cstdint>
#include <memory>
#include <new>
#include <utility>
#include <string>
#include <vector>

#include "../../include/tilefusion.h"

namespace tf {

// Limits of the kernels.
constexpr int kMaxMfmaSliceCols = 128;   // one wave holds at most 8 accumulator blocks of 16 columns
constexpr int kRowGranuleDense = 16;     // dense-B tiles are produced in blocks of 16 rows (MFMA M/N)
constexpr int kXcds = 8;                 // XCDs of the device: consecutive workgroup ids are dealt to them round robin,
                                         // each has its own L2 (the kernels' work-to-workgroup maps and the grid sizes use it)
constexpr int kFusedThreads = 512;       // workgroup size of the fused kernels
constexpr int kSpmmThreads = 256;        // workgroup size of the row-list SpMM kernel
constexpr int kWantedTileRows = 256;     // a default column slice is narrowed until tiles this large fit
constexpr int kUnitRows = 64;            // most rows in one unit of a packed row list
constexpr int kUnitSlots = 2048;         // most padded entries (rows x slots) in one such unit (they are staged in LDS)
constexpr int kPackSpareSlots = 8 * 64 + 8;  // zero entries behind the last unit of a packed row list: the gather kernel
                                         // fetches the entries of split rows in windows of 8 slots per lane of a lane
                                         // group (64 lanes at most), which may reach that far past the last row
constexpr int kSplitMinSlots = 128;      // rows at least this long are split over several lane groups
constexpr int kSplitPartSlots = 96;      // target slots per part of a split row
// a row long enough to be split gets at least two parts: units whose rows are not split are staged
// in LDS whole (kUnitSlots entries at most), so a row that long must never end up in one
static_assert(kSplitMinSlots > kSplitPartSlots && kSplitMinSlots <= kUnitSlots,
              "rows of kSplitMinSlots entries or more must be split");
constexpr int kGatherSliceBytes = 128;    // narrowest column slice of the gather kernel chosen by default, bytes

// Per D1 row of a tile, beside its row id: one info word.  kInfoSpill: the row is also stored to
// the D1 workspace, at the slot in the low bits (a row that the second wavefront reads).
// kInfoDirect: the row of D with the same id is fused and has exactly one stored entry, on the
// diagonal, so it is the D1 row times that entry (tile_scale) and leaves from the registers that
// hold the D1 row; kInfoZero: the row of D with the same id is empty and is stored as zeros.
// 0 for padding rows.
constexpr uint32_t kInfoSpill = 0x80000000u;
constexpr uint32_t kInfoDirect = 0x40000000u;
constexpr uint32_t kInfoZero = 0x20000000u;
// kInfoSkip (streaming first wavefront of a CSR-B plan with TF_FLAG_SKIP_UNREAD only): no row of A
// reads this D1 row, it is not computed.
constexpr uint32_t kInfoSkip = 0x10000000u;
constexpr uint32_t kInfoSlotMask = 0x0fffffffu;

// Where the D1 rows that cross tiles live in device memory: `n_sl` column slices of `sw` columns
// each (the last may be narrower in use, never in storage), slice after slice, each slice a dense
// array of `rows` rows of sw elements.  Element (slot, col) is at
// (col / sw) * rows * sw + slot * sw + col % sw.  One slice = plain row-major.  Slices are what one
// XCD of the gather kernel works on: its L2 then holds sw-wide pieces of the rows instead of whole
// rows, and the hot rows of an irregular matrix are not replicated in all eight L2 caches.
struct D1Layout {
    int32_t sw = 0, n_sl = 1;
    int64_t rows = 0;
    int64_t slice_stride() const { return rows * sw; }
    int64_t elements() const { return (int64_t)n_sl * rows * sw; }
};

// Lanes that share one row in the gather kernels: each lane owns vv columns (vv = elements per
// 16 bytes when rows are 16-byte aligned, else 1); the group is the smallest power of two of
// lanes that covers `cols` columns, at most one wave.
inline int lane_group(int cols, int vv) {
    int g = 1;
    while (g * vv < cols && g < 64) g *= 2;
    return g;
}

inline int elem_size(int dtype) { return dtype == TF_F64 ? 8 : 4; }
inline int vec_elems(int dtype) { return dtype == TF_F64 ? 2 : 4; }   // elements per 16 bytes

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// LDS layout of a fused workgroup, shared by the inspector (tile fitting) and the kernels.
//   dense B : [C slice in MFMA operand order: bcol_pad x cs16] [D1 tile: rows_pad16 x ldl]
//   sparse B: [D1 tile: rows x ldl]
// ldl is the leading dimension of the D1 tile in elements; dense-B tiles are as wide as the
// MFMA blocks that produce them and carry 16 bytes of padding per row so that the 16 rows written
// by one MFMA block start in different banks.
// Number of 16-column accumulator blocks the MFMA phase runs for a slice of cs columns
// (instantiated for 1, 2, 4 and 8 blocks) and the padded slice width that goes with it.
inline int mfma_blocks(int cs) {
    int nb = 1;
    while (nb * 16 < cs) nb *= 2;
    return nb;
}
inline int mfma_cols(int cs) { return 16 * mfma_blocks(cs); }
inline int64_t lds_ldl(int dtype, int b_is_sparse, int cs) {
    const int v = vec_elems(dtype);
    return b_is_sparse ? round_up(cs, v) : mfma_cols(cs) + v;
}
inline int64_t lds_fixed_bytes(int dtype, int b_is_sparse, int bcol, int cs) {
    if (b_is_sparse) return 0;
    const int kc = 4 * vec_elems(dtype);
    return round_up(bcol, kc) * mfma_cols(cs) * elem_size(dtype);
}
inline int lds_row_granule(int b_is_sparse) { return b_is_sparse ? 1 : kRowGranuleDense; }
// A CSR B: the workgroup first copies the extents of the tile's rows of B and up to
// kSparseEntryCap entries of each into LDS (two loads per row for the whole tile instead of a
// chain of dependent loads per row); bytes of LDS per tile row that this takes.
constexpr int kSparseEntryCap = 8;
constexpr int kCsrRowsPerWg = 64;        // rows of one workgroup of the unfused CSR SpMM
inline int64_t lds_sparse_b_bytes_per_row(int dtype) {
    return 2 * 8 + kSparseEntryCap * (4 + (int64_t)elem_size(dtype));    // extents of two tiles
}

// Whether a wave of the dense-B kernels keeps its operands of the C slice in registers: only for
// the specialised shallow depths (ks = bCol / (4 * elements per 16 bytes) steps, nb accumulator
// blocks) and at most 64 registers' worth (32 for fp64, whose B buffers are twice as large).
// The C slice then needs no LDS.
constexpr bool c_in_registers(int dtype, int nb, int ks) {
    return (ks == 2 || ks == 4) &&
           ks * (dtype == TF_F64 ? 2 : 4) * nb * (dtype == TF_F64 ? 2 : 1) <= (dtype == TF_F64 ? 32 : 64);
}
// ks as the kernels specialise it: 0 = generic loop over k.
inline int mfma_ksteps_special(int dtype, int bcol, int ccol, int cs) {
    const int v = dtype == TF_F64 ? 2 : 4;
    if (bcol % v || ccol % v || cs % v || bcol % (4 * v)) return 0;
    const int ks = bcol / (4 * v);
    return (ks == 2 || ks == 4 || ks == 8 || ks == 16) ? ks : 0;
}

// What a fused workgroup needs to know about one tile: the ids of its D1 rows, one info word per
// row (kInfo*: spill slot, direct, zero) and the diagonal entry of direct rows, in three arrays with
// the same stride for every tile, so that their addresses follow from the tile's number alone
// (the first loads of a workgroup do not wait for a descriptor); padding up to the stride repeats
// the last row, with an empty info word.  And, so that nothing in the tile waits for a
// chain of dependent loads (row list -> unit -> entries), this fixed-size descriptor plus one
// contiguous, 16-byte aligned second-phase block of s_bytes bytes (each array padded to 16 bytes):
//   TileUnit units[n_units]
//   int32    rows2[n_second]               row ids of the fused rows of D, unit after unit
//   uint16   idx[n_entries]                where the D1 row of every packed entry sits in the LDS tile,
//                                          in units of 16 bytes: the even slots of all rows first
//                                          (n_entries / 2 of them), then the odd slots
//   T        val[n_entries]
struct TileDesc {
    int64_t meta_off;      // byte offset of the block
    int32_t n_rows;        // D1 rows the tile produces
    int32_t n_units;
    int32_t n_second;      // fused rows of D that read the LDS tile (direct rows are not among them)
    int32_t n_entries;     // padded entries over all units
    int32_t s_bytes;       // size of the second-phase block
    int32_t reserved;
};
struct TileUnit {          // n_rows rows of `stride` entry slots each, from entry_base on
    int32_t entry_base;    // even
    int32_t row_begin;     // position of the unit's first row in rows2
    int32_t n_rows;
    int32_t slots;         // stride (even, low 16 bits) | real length of the longest row (high 16 bits)
};

// Dynamic LDS of a fused workgroup: two buffers of row ids (this tile's and the next one's),
// the staged second-phase block (s_lds bytes, 0 when it is read in place), the staged rows of a
// CSR B, the C slice of a dense B unless the waves hold it in registers, the D1 tile.
struct FusedLdsLayout {
    int64_t first0, first1, second, bext, bidx, bval, cslice, tile, total;
};
inline FusedLdsLayout fused_lds_layout(int dtype, int b_is_sparse, int bcol, int ccol, int cs,
                                       int max_tile_rows, int s_lds, bool need_tile = true) {
    FusedLdsLayout l{};
    const int es = elem_size(dtype);
    const int64_t rows16 = round_up(max_tile_rows, 16);       // the row id buffers are padded
    const int64_t rows_cap = round_up(max_tile_rows, lds_row_granule(b_is_sparse));
    l.first0 = 0;
    l.first1 = rows16 * 4;
    l.second = 2 * rows16 * 4;
    // staged rows of a CSR B: (first entry, length) per row for this tile and for the next one,
    // then the column indices, then the values
    l.bext = l.second + round_up(s_lds, 16);
    l.bidx = l.bext + (b_is_sparse ? 2 * round_up(rows_cap * 8, 16) : 0);
    l.bval = l.bidx + (b_is_sparse ? round_up(rows_cap * kSparseEntryCap * 4, 16) : 0);
    l.cslice = l.bval + (b_is_sparse ? round_up(rows_cap * kSparseEntryCap * es, 16) : 0);
    const int64_t cbytes = lds_fixed_bytes(dtype, b_is_sparse, bcol, cs);
    const bool c_regs = !b_is_sparse && c_in_registers(dtype, mfma_blocks(cs),
                                                       mfma_ksteps_special(dtype, bcol, ccol, cs));
    l.tile = l.cslice + (c_regs ? 0 : cbytes);
    // (a plan none of whose fused rows reads the tile keeps no tile at all)
    l.total = l.tile + (need_tile ? rows_cap * lds_ldl(dtype, b_is_sparse, cs) * es : 0);
    return l;
}
inline int64_t fused_lds_bytes(int dtype, int b_is_sparse, int bcol, int ccol, int cs,
                               int max_tile_rows, int s_lds, bool need_tile = true) {
    return fused_lds_layout(dtype, b_is_sparse, bcol, ccol, cs, max_tile_rows, s_lds, need_tile).total;
}

// One unit of a packed row list: n_rows rows, all padded to `slots` entries, stored row after
// row from entry_base on.  split > 1: every row is shared by `split` lane groups, each summing
// a contiguous part of the slots.
struct UnitDesc {
    int64_t entry_base;
    int32_t row_begin;    // position of the unit's first row in the list
    int32_t n_rows;
    int32_t slots;
    int32_t split;
};

// A list of rows of A re-packed for the gather kernels: per unit a uniform padded row length,
// so the kernels need no row pointers and no per-row bounds.  Padding repeats the row's last
// column index with value 0.
// A vector whose resize() leaves the new elements uninitialised: the packed arrays are sized once
// and then written in full by the host threads, which are also the first to touch their pages.
template <typename T> struct NoInitAlloc : std::allocator<T> {
    template <typename U> struct rebind {
        using other = NoInitAlloc<U>;
    };
    template <typename U> void construct(U *p) noexcept { ::new (static_cast<void *>(p)) U; }
    template <typename U, typename... A> void construct(U *p, A &&...a) {
        ::new (static_cast<void *>(p)) U(std::forward<A>(a)...);
    }
};
template <typename T> using RawVec = std::vector<T, NoInitAlloc<T>>;

struct RowPack {
    std::vector<UnitDesc> units;
    std::vector<int32_t> rows;           // row ids, list order
    RawVec<int32_t> idx32;               // column indices
    RawVec<unsigned char> vals;          // packed values, element size of the plan's dtype
    bool sorted = false;                 // rows were re-ordered by length
    int64_t entries() const { return (int64_t)idx32.size(); }
};

// Host-side schedule produced by the inspector.
struct Schedule {
    int64_t n = 0, nnz = 0;
    int32_t t = 0;                 // step-1 uniform tile size
    int32_t col_slice = 0, n_slices = 1;
    int64_t n_coarse_tiles = 0;
    std::vector<int32_t> tile_first_ptr, first_rows;      // first_rows: plain row ids
    std::vector<int32_t> tile_second_ptr, second_rows;
    std::vector<int32_t> wf1_unit_ptr, wf1_rows;
    std::vector<uint8_t> spill;
    std::vector<TileDesc> tile_desc;                      // one per tile, see TileDesc
    // the tiles' second-phase blocks, back to back (not zero-filled on allocation: the host threads
    // that copy the blocks in are the first to touch its pages)
    std::unique_ptr<unsigned char[]> tile_meta;
    size_t tile_meta_bytes = 0;
    std::vector<int32_t> tile_first;                      // the tiles' row ids, first_stride ints per tile
    std::vector<uint32_t> tile_info;                      // info word per D1 row of a tile (kInfo*), same stride
    RawVec<unsigned char> tile_scale;                     // diagonal entry of the direct rows (plan's dtype), same stride; empty when there are none
    std::vector<int32_t> spill_slot;                      // per row: its slot in the D1 workspace, -1 when not spilled
    D1Layout d1;                                          // workspace of the fused path (rows = spilled rows)
    int64_t n_direct_rows = 0;                            // fused rows that leave from registers (diagonal-only or empty)
    int64_t n_lds_rows = 0;                               // fused rows computed out of the LDS tile
    int32_t gather_r = 4;                                 // rows per lane group and pass of the gather kernel
    // When no fused row reads the LDS tile the first wavefront streams through the rows without
    // tiles: the info words and diagonal entries again, indexed by row (empty otherwise).
    std::vector<uint32_t> row_info;
    RawVec<unsigned char> row_scale;
    bool streaming = false;
    bool automatic = false;        // the caller left the tiling to the library
    bool far_rows = false;         // rows reach far from the diagonal (a graph), see build_schedule
    bool grown_tiles = false;      // tiles grown along the dependence graph
    int64_t n_demoted_rows = 0;    // rows that a tile could have fused but that were left to the second wavefront
    int32_t first_stride = 0;                             // largest tile, in rows, rounded up to 16
    int64_t second_block_cap = 0;                         // largest second-phase block, bytes
    bool second_block_in_lds = true;                      // it fits beside the largest tile
    int64_t lds_meta_bytes_per_row = 0;                   // part of lds_bytes_per_row: row ids + estimate of the second-phase block
    RowPack wf1;                   // wf1_rows re-packed
    RowPack all;                   // all rows re-packed (unfused baseline)
    int64_t n_fused_rows = 0, n_spill_rows = 0, fused_nnz = 0;
    int64_t max_tile_rows = 0;
    int64_t lds_fixed_bytes = 0, lds_bytes_per_row = 0, fast_mem_bytes = 0;
    int32_t lds_row_granule = 1;
    double eq2_cost_max = 0.0;
};

struct InspectorInput {
    int64_t n, nnz;
    const int32_t *rowptr, *colidx;   // host
    const void *vals;                 // host, element size of dtype
    int64_t bcol, ccol;
    int32_t b_is_sparse;
    int32_t dtype;
    int32_t ct_size, p;
    int64_t fast_mem_bytes;
    int32_t col_slice;
    uint32_t flags;
    int32_t gather_slices;            // column slices of the D1 workspace and of the gather kernel; 0 = chosen here
    int32_t n_cu;                     // compute units of the device the plan will run on
};

// Builds the schedule; returns TF_OK or an error with a message in `err`.
tf_status build_schedule(const InspectorInput &in, Schedule &out, std::string &err);
// The packed copy of all rows of A that the unfused baseline's second operation runs on
// (Schedule::all).  Not part of the fused schedule and not counted in its time.
// (false: a unit exceeds the gather kernel's staging arrays; never expected)
bool build_baseline_pack(const InspectorInput &in, Schedule &s);


// ---------------------------------------------------------------- device launch interface

struct CsrDev {
    const int32_t *rowptr = nullptr;
    const int32_t *colidx = nullptr;
    const void *vals = nullptr;
};

struct PackDev {
    const UnitDesc *units = nullptr;
    const int32_t *rows = nullptr;
    const void *idx = nullptr;        // int32 or uint16
    const void *vals = nullptr;
};

struct FusedLaunch {
    int32_t dtype;
    int32_t n_tiles, n_slices, cs, ccol, bcol;
    int32_t rows_cap;                 // largest tile, in rows, rounded up to 16
    int32_t tile_rows;                // largest tile, in rows, rounded up to the tile's row granule
    int32_t s_cap;                    // largest second-phase block, bytes (multiple of 16)
    int32_t s_in_lds;                 // 1: second-phase blocks are staged in LDS, 0: read in place
    int64_t lds_bytes;                // dynamic LDS of the launch
    const TileDesc *tile_desc;
    const unsigned char *tile_meta;
    const int32_t *tile_first;        // row ids of tile v at tile_first + v * first_stride
    const uint32_t *tile_info;        // info words (kInfo*), same indexing
    const void *tile_scale;           // diagonal entries of direct rows, same indexing; nullptr: no direct rows
    int32_t first_stride;
    int32_t need_tile;                // 0: no tile of the plan has fused rows that read the LDS tile
    int32_t n_cu;                     // compute units of the device
    const void *B;                    // dense B (gemm) or nullptr
    CsrDev Bs;                        // sparse B (spmm)
    const void *C;
    int32_t c_ldk, c_ldc;             // dense B: element (k, c) of the multiplier is C[k c_ldk + c c_ldc]
    void *D;
    void *D1;
    int32_t d1_sw_shift, d1_sw_mask;  // column -> (slice, offset) of the D1 workspace (one slice: 31, 0x7fffffff)
    int32_t d1_sw;
    int64_t d1_slice_stride;          // elements
};

// Y[row] = sum over the packed entries of the row of val * X[idx]; one unit per workgroup.
struct PackedSpmmLaunch {
    int32_t dtype;
    int64_t n_units;
    int32_t contiguous;               // 1: neighbouring units share an XCD; 0: round robin (one slice only)
    int32_t wide;                     // 1: X spans 4 GiB or more (64-bit operand offsets)
    PackDev pack;                     // int32 indices: rows (slots) of X
    const void *X;                    // D1 workspace in the layout below
    int32_t n_xs, sw;                 // column slices (1, 2, 4 or 8; each handled by 8 / n_xs XCDs) of sw columns
    int64_t x_slice_stride;           // elements between the slices of X
    int32_t rows_per_pass;            // R of the kernel instantiation: 1, 2 or 4
    void *Y;                          // row-major, ccol columns
    int32_t ccol;
};

// Y[j] = S[j, :] X for a caller-supplied CSR matrix S, `rows_per_wg` consecutive rows per workgroup.
struct CsrSpmmLaunch {
    int32_t dtype;
    int64_t n_rows;
    int32_t rows_per_wg;
    CsrDev S;
    const void *X;
    void *Y;                          // D1 workspace layout: slices of y_sw columns
    int32_t ccol;
    int32_t y_sw_shift, y_sw_mask, y_sw;
    int64_t y_slice_stride;
    const uint32_t *row_info;         // as in GemmLaunch
    const void *row_scale;
    void *D;
};

struct GemmLaunch {
    int32_t dtype;
    int64_t n;
    int32_t bcol, ccol, cs, n_slices;
    const void *B, *C;
    int32_t c_ldk, c_ldc;             // element (k, c) of the multiplier is C[k c_ldk + c c_ldc]
    void *D1;                         // workspace layout: slices of d1_sw columns
    int32_t d1_sw_shift, d1_sw_mask, d1_sw;
    int64_t d1_slice_stride;
    // first wavefront of a plan without an LDS tile (else nullptr): info word per row (kInfo*),
    // diagonal entry of the direct rows (nullptr: none), and D
    const uint32_t *row_info;
    const void *row_scale;
    void *D;
};

// Each returns hipError_t as int (0 = success).  `stream` is a hipStream_t.
int launch_fused_gemm_spmm(const FusedLaunch &a, void *stream);
int launch_fused_spmm_spmm(const FusedLaunch &a, void *stream);
int launch_packed_spmm(const PackedSpmmLaunch &a, void *stream);
int launch_csr_spmm(const CsrSpmmLaunch &a, void *stream);
int launch_gemm(const GemmLaunch &a, void *stream);

}  // namespace tf
