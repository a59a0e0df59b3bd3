// Internal declarations shared by the inspector (host), the kernels (device) and the C ABI.
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/tilefusion.h"

namespace tf {

// Limits of the kernels.
constexpr int kMaxMfmaSliceCols = 128;   // one wave holds at most 8 accumulator blocks of 16 columns
constexpr int kRowGranuleDense = 16;     // dense-B tiles are produced in blocks of 16 rows (MFMA M/N)
constexpr int kFusedThreads = 512;       // workgroup size of the fused kernels
constexpr int kSpmmThreads = 256;        // workgroup size of the row-list SpMM kernel
constexpr int kLongRowNnz = 2048;        // a second-wavefront row this long gets a workgroup of its own
constexpr int kUnitWork = 1024;          // target work (nnz + 8 per row) of one second-wavefront unit
constexpr uint32_t kSpillBit = 0x80000000u;

inline int elem_size(int dtype) { return dtype == TF_F64 ? 8 : 4; }
inline int vec_elems(int dtype) { return dtype == TF_F64 ? 2 : 4; }   // elements per 16 bytes

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// LDS layout of a fused workgroup, shared by the inspector (tile fitting) and the kernels.
//   dense B : [C slice in MFMA operand order: bcol_pad x cs16] [D1 tile: rows_pad16 x ldl]
//   sparse B: [D1 tile: rows x ldl]
// ldl is the leading dimension of the D1 tile in elements; dense-B tiles carry 16 bytes of
// padding per row so that the 16 rows written by one MFMA block start in different banks.
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
    return b_is_sparse ? round_up(cs, v) : round_up(cs, v) + v;
}
inline int64_t lds_fixed_bytes(int dtype, int b_is_sparse, int bcol, int cs) {
    if (b_is_sparse) return 0;
    const int kc = 4 * vec_elems(dtype);
    return round_up(bcol, kc) * mfma_cols(cs) * elem_size(dtype);
}
inline int lds_row_granule(int b_is_sparse) { return b_is_sparse ? 1 : kRowGranuleDense; }

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
    std::vector<uint16_t> lcol;    // per stored entry of A: tile-local index of its column (fused rows only)
    std::vector<int32_t> all_unit_ptr, all_rows;          // balanced units over all rows (unfused baseline)
    int64_t n_fused_rows = 0, n_spill_rows = 0, fused_nnz = 0;
    int64_t max_tile_rows = 0;
    int64_t lds_fixed_bytes = 0, lds_bytes_per_row = 0, fast_mem_bytes = 0;
    int32_t lds_row_granule = 1;
    double eq2_cost_max = 0.0;
};

struct InspectorInput {
    int64_t n, nnz;
    const int32_t *rowptr, *colidx;   // host
    int64_t bcol, ccol;
    int32_t b_is_sparse;
    int32_t dtype;
    int32_t ct_size, p;
    int64_t fast_mem_bytes;
    int32_t col_slice;
    uint32_t flags;
};

// Builds the schedule; returns TF_OK or an error with a message in `err`.
tf_status build_schedule(const InspectorInput &in, Schedule &out, std::string &err);

// Balanced partition of a row list into units of about equal work (host helper).
void balance_units(const int32_t *rowptr, const std::vector<int32_t> &rows, bool long_first,
                   std::vector<int32_t> &rows_out, std::vector<int32_t> &unit_ptr);

// ---------------------------------------------------------------- device launch interface

struct CsrDev {
    const int32_t *rowptr = nullptr;
    const int32_t *colidx = nullptr;
    const void *vals = nullptr;
};

struct FusedLaunch {
    int32_t dtype;
    int32_t n_tiles, n_slices, cs, ccol, bcol;
    int32_t max_tile_rows;            // largest tile, in rows
    int64_t lds_bytes;                // dynamic LDS of the launch
    const int32_t *tile_first_ptr, *first_rows_enc;   // first_rows with kSpillBit
    const int32_t *tile_second_ptr, *second_rows;
    const int32_t *a_rowptr;
    const uint16_t *lcol;
    const void *a_vals;
    const void *B;                    // dense B (gemm) or nullptr
    CsrDev Bs;                        // sparse B (spmm)
    const void *C;
    void *D;
    void *D1;
};

struct SpmmLaunch {
    int32_t dtype;
    int64_t n_units;
    const int32_t *unit_ptr;          // nullptr: uniform units of `uniform_rows` consecutive rows
    const int32_t *rows;              // nullptr: identity
    int64_t n_rows;                   // used with uniform units
    int32_t uniform_rows;
    CsrDev S;
    const void *X;                    // [*, ccol]
    void *Y;                          // [*, ccol]
    int32_t ccol;
};

struct GemmLaunch {
    int32_t dtype;
    int64_t n;
    int32_t bcol, ccol, cs, n_slices;
    const void *B, *C;
    void *D1;
};

// Each returns hipError_t as int (0 = success).  `stream` is a hipStream_t.
int launch_fused_gemm_spmm(const FusedLaunch &a, void *stream);
int launch_fused_spmm_spmm(const FusedLaunch &a, void *stream);
int launch_spmm_units(const SpmmLaunch &a, void *stream);
int launch_gemm(const GemmLaunch &a, void *stream);
int prepare_kernels(int64_t max_dynamic_lds);                 // raises the dynamic-LDS limit of the kernels

}  // namespace tf
