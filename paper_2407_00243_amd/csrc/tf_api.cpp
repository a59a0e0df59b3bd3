// C ABI of the tile-fusion library: argument checks, device memory owned by a plan, and the
// two-launch execution (first wavefront, then second wavefront, in stream order).
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "tf_internal.h"

namespace {

thread_local std::string g_err;

tf_status fail(tf_status st, const std::string &msg) {
    g_err = msg;
    return st;
}

tf_status hip_fail(hipError_t e, const char *what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return e == hipErrorOutOfMemory ? TF_ENOMEM : TF_EHIP;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Device buffers owned by a plan.
struct DevBuf {
    void *p = nullptr;
    ~DevBuf() {
        if (p) (void)hipFree(p);
    }
    hipError_t upload(const void *src, size_t bytes) {
        hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
        if (e != hipSuccess) return e;
        if (bytes) e = hipMemcpy(p, src, bytes, hipMemcpyHostToDevice);
        return e;
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 16); }
};

}  // namespace

struct tf_plan {
    int64_t n = 0, nnz = 0, bcol = 0, ccol = 0;
    int32_t dtype = 0, b_is_sparse = 0;
    int device = 0;
    int64_t lds_per_cu = 160 * 1024;
    bool schedule_only = false;
    bool c_transposed = false;             // dense-B calls take C as cCol x bCol (D = A (B C^T))
    tf::Schedule s;
    double plan_seconds = 0.0;
    struct PackBufs {
        DevBuf units, rows, idx, vals;
        int64_t n_units = 0;
        bool sorted = false;
        tf::PackDev dev() const {
            tf::PackDev d;
            d.units = static_cast<const tf::UnitDesc *>(units.p);
            d.rows = static_cast<const int32_t *>(rows.p);
            d.idx = idx.p;
            d.vals = vals.p;
            return d;
        }
    };
    DevBuf tile_desc, tile_meta, tile_first, tile_info, tile_scale, row_info, row_scale;
    PackBufs wf1, all;
    DevBuf d1;                             // fused path: one slot per spilled D1 row
    bool has_baseline = false;             // the packed copy of all rows of A exists
    int n_cu = 256;
    // unfused baseline: all n rows of D1, allocated by the first unfused call (or tf_plan_prepare_unfused)
    mutable std::mutex unf_mutex;
    mutable DevBuf d1_unf;
    tf::D1Layout unf_layout() const {
        tf::D1Layout l = s.d1;
        l.rows = n > 0 ? n : 1;
        return l;
    }
};

namespace {

tf_status check_csr_host(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                         const int32_t *colidx) {
    if (rowptr[0] != 0) return fail(TF_EBADCSR, "rowptr[0] != 0");
    for (int64_t i = 0; i < n_rows; ++i)
        if (rowptr[i + 1] < rowptr[i]) return fail(TF_EBADCSR, "rowptr is not monotone");
    if (rowptr[n_rows] != nnz) return fail(TF_EBADCSR, "rowptr[n_rows] != nnz");
    for (int64_t q = 0; q < nnz; ++q)
        if (colidx[q] < 0 || colidx[q] >= n_cols)
            return fail(TF_EBADCSR, "column index out of range");
    return TF_OK;
}

template <typename V, typename A> hipError_t up(DevBuf &b, const std::vector<V, A> &v) {
    return b.upload(v.data(), v.size() * sizeof(V));
}

hipError_t upload_pack(tf_plan::PackBufs &b, tf::RowPack &pk) {
    hipError_t e = up(b.units, pk.units);
    if (e == hipSuccess) e = up(b.rows, pk.rows);
    if (e == hipSuccess) e = up(b.idx, pk.idx32);
    if (e == hipSuccess) e = up(b.vals, pk.vals);
    b.n_units = (int64_t)pk.units.size();
    b.sorted = pk.sorted;
    // the packed entries live on the device from here on; the row lists stay for the schedule view
    tf::RawVec<int32_t>().swap(pk.idx32);
    tf::RawVec<unsigned char>().swap(pk.vals);
    return e;
}

// column -> (slice, offset inside the slice) of a workspace: a shift and a mask; with one slice the
// shift empties the column number and the mask keeps it
int32_t sw_shift(const tf::D1Layout &l) {
    if (l.n_sl == 1) return 31;
    int32_t sh = 0;
    while ((1 << sh) < l.sw) ++sh;
    return sh;
}
int32_t sw_mask(const tf::D1Layout &l) { return l.n_sl == 1 ? 0x7fffffff : l.sw - 1; }

tf::FusedLaunch fused_args(const tf_plan *p, const void *C, void *D) {
    tf::FusedLaunch a{};
    a.dtype = p->dtype;
    a.n_tiles = (int32_t)(p->s.tile_first_ptr.size() - 1);
    a.n_slices = p->s.n_slices;
    a.cs = p->s.col_slice;
    a.ccol = (int32_t)p->ccol;
    a.bcol = (int32_t)p->bcol;
    a.rows_cap = (int32_t)tf::round_up(p->s.max_tile_rows, 16);     // size of a row id buffer
    a.tile_rows = (int32_t)tf::round_up(p->s.max_tile_rows, tf::lds_row_granule(p->b_is_sparse));
    a.s_cap = (int32_t)p->s.second_block_cap;
    a.s_in_lds = p->s.second_block_in_lds ? 1 : 0;
    a.need_tile = p->s.n_lds_rows > 0 ? 1 : 0;
    a.lds_bytes = tf::fused_lds_bytes(p->dtype, p->b_is_sparse, a.bcol, a.ccol, a.cs,
                                      (int)p->s.max_tile_rows, a.s_in_lds ? a.s_cap : 0, a.need_tile);
    a.tile_desc = static_cast<const tf::TileDesc *>(p->tile_desc.p);
    a.tile_meta = static_cast<const unsigned char *>(p->tile_meta.p);
    a.tile_first = static_cast<const int32_t *>(p->tile_first.p);
    a.tile_info = static_cast<const uint32_t *>(p->tile_info.p);
    a.tile_scale = p->s.n_direct_rows > 0 ? p->tile_scale.p : nullptr;
    a.first_stride = p->s.first_stride;
    a.n_cu = p->n_cu;
    a.C = C;
    a.c_ldk = p->c_transposed ? 1 : a.ccol;
    a.c_ldc = p->c_transposed ? a.bcol : 1;
    a.D = D;
    a.D1 = p->d1.p;
    a.d1_sw = p->s.d1.sw;
    a.d1_sw_shift = sw_shift(p->s.d1);
    a.d1_sw_mask = sw_mask(p->s.d1);
    a.d1_slice_stride = p->s.d1.slice_stride();
    return a;
}

tf::PackedSpmmLaunch packed_args(const tf_plan *p, const tf_plan::PackBufs &b, const void *X,
                                 const tf::D1Layout &lay, void *D) {
    tf::PackedSpmmLaunch w{};
    w.dtype = p->dtype;
    w.n_units = b.n_units;
    w.contiguous = b.sorted ? 0 : 1;
    // operand offsets inside a slice are formed in 32 bits unless the slice spans 4 GiB or more
    w.wide = (double)lay.slice_stride() * tf::elem_size(p->dtype) >= 4294967296.0 ? 1 : 0;
    w.pack = b.dev();
    w.X = X;
    w.n_xs = lay.n_sl;
    w.sw = lay.sw;
    w.x_slice_stride = lay.slice_stride();
    w.rows_per_pass = p->s.gather_r;
    w.Y = D;
    w.ccol = (int32_t)p->ccol;
    return w;
}

tf::PackedSpmmLaunch second_wavefront_args(const tf_plan *p, void *D) {
    return packed_args(p, p->wf1, p->d1.p, p->s.d1, D);
}

tf::PackedSpmmLaunch all_rows_args(const tf_plan *p, void *D) {
    return packed_args(p, p->all, p->d1_unf.p, p->unf_layout(), D);
}

// The unfused baseline's workspace holds all n rows of D1; it is allocated when first needed.
tf_status prepare_unfused(const tf_plan *p) {
    if (!p->has_baseline)
        return fail(TF_EINVAL, "the plan was built with TF_FLAG_NO_BASELINE");
    std::lock_guard<std::mutex> lock(p->unf_mutex);
    if (p->d1_unf.p) return TF_OK;
    hipError_t e = p->d1_unf.alloc((size_t)p->unf_layout().elements() * tf::elem_size(p->dtype));
    if (e != hipSuccess) return hip_fail(e, "allocating the workspace of the unfused baseline");
    return TF_OK;
}

tf_status check_exec(const tf_plan *p, int want_sparse, const void *C, const void *D) {
    if (!p || !C || !D) return fail(TF_EINVAL, "null argument");
    if (p->schedule_only) return fail(TF_EINVAL, "the plan was built with TF_FLAG_SCHEDULE_ONLY");
    if (p->b_is_sparse != want_sparse)
        return fail(TF_EMISMATCH, want_sparse ? "plan was built for a dense B"
                                              : "plan was built for a sparse B");
    if (!aligned16(C) || !aligned16(D)) return fail(TF_EINVAL, "C and D must be 16-byte aligned");
    return TF_OK;
}

tf_status check_sparse_b(const tf_plan *p, const tf_csr *B) {
    if (!B || !B->rowptr || (B->nnz > 0 && (!B->colidx || !B->vals)))
        return fail(TF_EINVAL, "null argument");
    if (!B->on_device) return fail(TF_EINVAL, "B must be on the device for execution");
    if (B->dtype != p->dtype) return fail(TF_EMISMATCH, "B has a different element type than A");
    if (B->n_rows != p->n || B->n_cols != p->bcol)
        return fail(TF_EMISMATCH, "B is not n x bCol for this plan");
    return TF_OK;
}

// Shape of the plain product D1 = B C (k_gemm): the column slice is as wide as one wave's
// accumulators allow, narrowed until the C slice fits the LDS.  False if it never does.
bool gemm_shape(const tf_plan *p, tf::GemmLaunch &g) {
    g.dtype = p->dtype;
    g.n = p->n;
    g.bcol = (int32_t)p->bcol;
    g.ccol = (int32_t)p->ccol;
    g.cs = p->ccol > tf::kMaxMfmaSliceCols ? tf::kMaxMfmaSliceCols : (int32_t)p->ccol;
    while (g.cs > 16 && tf::lds_fixed_bytes(p->dtype, 0, g.bcol, g.cs) > p->lds_per_cu)
        g.cs = (g.cs - 1) / 16 * 16;
    if (tf::lds_fixed_bytes(p->dtype, 0, g.bcol, g.cs) > p->lds_per_cu) return false;
    g.n_slices = (int32_t)((p->ccol + g.cs - 1) / g.cs);
    g.c_ldk = p->c_transposed ? 1 : g.ccol;
    g.c_ldc = p->c_transposed ? g.bcol : 1;
    return true;
}
void gemm_workspace(tf::GemmLaunch &g, void *ws, const tf::D1Layout &lay) {
    g.D1 = ws;
    g.d1_sw = lay.sw;
    g.d1_sw_shift = sw_shift(lay);
    g.d1_sw_mask = sw_mask(lay);
    g.d1_slice_stride = lay.slice_stride();
}
tf::CsrSpmmLaunch csr_spmm_args(const tf_plan *p, const tf_csr *B, const void *C, void *ws,
                                const tf::D1Layout &lay) {
    tf::CsrSpmmLaunch f{};
    f.dtype = p->dtype;
    f.rows_per_wg = tf::kCsrRowsPerWg;
    f.n_rows = p->n;
    f.S.rowptr = B->rowptr;
    f.S.colidx = B->colidx;
    f.S.vals = B->vals;
    f.X = C;
    f.Y = ws;
    f.ccol = (int32_t)p->ccol;
    f.y_sw = lay.sw;
    f.y_sw_shift = sw_shift(lay);
    f.y_sw_mask = sw_mask(lay);
    f.y_slice_stride = lay.slice_stride();
    return f;
}

// First wavefront into the workspace `ws` (the plan's own, or the static one).  A plan none of
// whose fused rows reads the LDS tile runs it without tiles, as the plain first operation whose
// rows go where their info words say; every other plan runs the tiled fused kernel.
tf_status first_wavefront_dense(const tf_plan *p, const void *B, const void *C, void *D, void *ws,
                                void *stream) {
    tf::GemmLaunch g{};
    if (p->s.streaming && gemm_shape(p, g)) {
        g.B = B;
        g.C = C;
        gemm_workspace(g, ws, p->s.d1);
        g.row_info = static_cast<const uint32_t *>(p->row_info.p);
        g.row_scale = p->s.n_direct_rows > 0 ? p->row_scale.p : nullptr;
        g.D = D;
        const int e = tf::launch_gemm(g, stream);
        if (e) return hip_fail((hipError_t)e, "launching the first wavefront");
        return TF_OK;
    }
    tf::FusedLaunch a = fused_args(p, C, D);
    a.B = B;
    a.D1 = ws;
    const int e = tf::launch_fused_gemm_spmm(a, stream);
    if (e) return hip_fail((hipError_t)e, "launching the first wavefront");
    return TF_OK;
}
tf_status first_wavefront_sparse(const tf_plan *p, const tf_csr *B, const void *C, void *D, void *ws,
                                 void *stream) {
    int e;
    if (p->s.streaming) {
        tf::CsrSpmmLaunch f = csr_spmm_args(p, B, C, ws, p->s.d1);
        f.row_info = static_cast<const uint32_t *>(p->row_info.p);
        f.row_scale = p->s.n_direct_rows > 0 ? p->row_scale.p : nullptr;
        f.D = D;
        e = tf::launch_csr_spmm(f, stream);
    } else {
        tf::FusedLaunch a = fused_args(p, C, D);
        a.Bs.rowptr = B->rowptr;
        a.Bs.colidx = B->colidx;
        a.Bs.vals = B->vals;
        a.D1 = ws;
        e = tf::launch_fused_spmm_spmm(a, stream);
    }
    if (e) return hip_fail((hipError_t)e, "launching the first wavefront");
    return TF_OK;
}
tf_status second_wavefront(const tf_plan *p, void *D, void *ws, void *stream) {
    tf::PackedSpmmLaunch w = second_wavefront_args(p, D);
    w.X = ws;
    const int e = tf::launch_packed_spmm(w, stream);
    if (e) return hip_fail((hipError_t)e, "launching the second wavefront");
    return TF_OK;
}

// Workspace of tf_gemm_spmm_static: one array per GPU, part of the loaded code object, so that
// the call needs no allocation at all.  In host code the array's name is only a handle; its
// device address is looked up once per device and used from then on.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
tf_status static_scratch(void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(TF_EUNSUPPORTED, "device ordinal out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!ptr) return fail(TF_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TF_OK;
}

int device_compute_units() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0)
        return 256;
    return cus;
}

int device_lds_limit() {
    int dev = 0, lds = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 64 * 1024;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
        lds <= 0)
        return 64 * 1024;
    return lds;
}

}  // namespace

extern "C" {

const char *tf_last_error(void) { return g_err.c_str(); }

const char *tf_version(void) { return "0.1"; }

tf_status tf_plan_create(const tf_csr *A, int64_t bCol, int64_t cCol, int32_t b_is_sparse,
                         const tf_tile_params *tp, tf_plan **out) {
    if (out) *out = nullptr;
    if (!A || !out) return fail(TF_EINVAL, "null argument");
    if (A->n_rows < 0 || A->nnz < 0 || !A->rowptr || (A->nnz > 0 && (!A->colidx || !A->vals)))
        return fail(TF_EINVAL, "A is missing an array or has a negative size");
    if (A->n_rows != A->n_cols) return fail(TF_EINVAL, "A must be square");
    if (A->nnz >= (int64_t(1) << 31) || A->n_rows >= (int64_t(1) << 31) - 1)
        return fail(TF_EUNSUPPORTED, "indices are 32 bit: n and nnz must be below 2^31");
    if (A->dtype != TF_F32 && A->dtype != TF_F64) return fail(TF_EINVAL, "unknown dtype");
    if (bCol <= 0 || cCol <= 0) return fail(TF_EINVAL, "bCol and cCol must be positive");
    if (bCol >= (int64_t(1) << 31) || cCol > (1 << 20))
        return fail(TF_EUNSUPPORTED, "bCol or cCol too large");
    if (tp && (tp->ct_size < 0 || tp->p < 0 || tp->fast_mem_bytes < 0 || tp->gather_slices < 0))
        return fail(TF_EINVAL, "negative tile parameter");

    const bool schedule_only = tp && (tp->flags & TF_FLAG_SCHEDULE_ONLY);
    if (tp && (tp->flags & TF_FLAG_C_TRANSPOSED) && b_is_sparse)
        return fail(TF_EUNSUPPORTED, "TF_FLAG_C_TRANSPOSED needs a dense B: a sparse B gathers rows of C");
    if (schedule_only && A->on_device)
        return fail(TF_EINVAL, "TF_FLAG_SCHEDULE_ONLY needs A in host memory");
    const int64_t n = A->n_rows, nnz = A->nnz;
    const int es = tf::elem_size(A->dtype);
    const auto t_start = std::chrono::steady_clock::now();

    // Host view of A's pattern (the scheduler runs on the host).
    std::vector<int32_t> h_rowptr, h_colidx;
    std::vector<unsigned char> h_vals;
    const int32_t *rowptr = A->rowptr, *colidx = A->colidx;
    const void *vals = A->vals;
    try {
        if (A->on_device) {
            h_rowptr.resize((size_t)n + 1);
            h_colidx.resize((size_t)nnz);
            h_vals.resize((size_t)nnz * es);
            hipError_t e = hipMemcpy(h_rowptr.data(), A->rowptr, (n + 1) * 4, hipMemcpyDeviceToHost);
            if (e == hipSuccess && nnz)
                e = hipMemcpy(h_colidx.data(), A->colidx, nnz * 4, hipMemcpyDeviceToHost);
            if (e == hipSuccess && nnz)
                e = hipMemcpy(h_vals.data(), A->vals, nnz * es, hipMemcpyDeviceToHost);
            if (e != hipSuccess) return hip_fail(e, "copying A to the host");
            rowptr = h_rowptr.data();
            colidx = h_colidx.data();
            vals = h_vals.data();
        }
        tf_status st = check_csr_host(n, n, nnz, rowptr, colidx);
        if (st != TF_OK) return st;

        tf_plan *p = new (std::nothrow) tf_plan();
        if (!p) return fail(TF_ENOMEM, "out of host memory");
        struct Guard {
            tf_plan *p;
            ~Guard() { delete p; }
        } guard{p};
        p->n = n;
        p->nnz = nnz;
        p->bcol = bCol;
        p->ccol = cCol;
        p->dtype = A->dtype;
        p->b_is_sparse = b_is_sparse ? 1 : 0;
        p->schedule_only = schedule_only;
        p->c_transposed = tp && (tp->flags & TF_FLAG_C_TRANSPOSED);
        if (!schedule_only) (void)hipGetDevice(&p->device);

        tf::InspectorInput in{};
        in.n = n;
        in.nnz = nnz;
        in.rowptr = rowptr;
        in.colidx = colidx;
        in.vals = vals;
        in.bcol = bCol;
        in.ccol = cCol;
        in.b_is_sparse = p->b_is_sparse;
        in.dtype = A->dtype;
        in.ct_size = tp ? tp->ct_size : 0;
        in.p = tp ? tp->p : 0;
        in.col_slice = tp ? tp->col_slice : 0;
        in.flags = tp ? tp->flags : 0;
        in.gather_slices = tp ? tp->gather_slices : 0;
        in.n_cu = schedule_only ? 256 : device_compute_units();
        p->n_cu = in.n_cu;
        const int64_t lds_limit = schedule_only ? 160 * 1024 : device_lds_limit();
        in.fast_mem_bytes = (tp && tp->fast_mem_bytes > 0) ? tp->fast_mem_bytes : lds_limit;
        if (!schedule_only && in.fast_mem_bytes > lds_limit) in.fast_mem_bytes = lds_limit;
        std::string err;
        st = tf::build_schedule(in, p->s, err);
        if (st != TF_OK) return fail(st, err);
        p->plan_seconds =
            std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count();

        if (schedule_only) {
            guard.p = nullptr;
            *out = p;
            return TF_OK;
        }
        p->has_baseline = !(tp && (tp->flags & TF_FLAG_NO_BASELINE));
        if (p->has_baseline && !tf::build_baseline_pack(in, p->s))
            return fail(TF_EUNSUPPORTED, "internal: a unit of the baseline exceeds the staging arrays of the gather kernel");
        p->lds_per_cu = lds_limit;
        // the launch must fit the device whatever the schedule's own estimate said
        auto launch_lds = [&]() {
            return tf::fused_lds_bytes(p->dtype, p->b_is_sparse, (int)bCol, (int)cCol, p->s.col_slice,
                                       (int)p->s.max_tile_rows,
                                       p->s.second_block_in_lds ? (int)p->s.second_block_cap : 0,
                                       p->s.n_lds_rows > 0);
        };
        if (launch_lds() > lds_limit) p->s.second_block_in_lds = false;
        if (launch_lds() > lds_limit)
            return fail(TF_EUNSUPPORTED, "a tile does not fit the LDS of this device");
        hipError_t e = hipSuccess;
        auto ok = [&](hipError_t r) {
            if (e == hipSuccess) e = r;
        };
        ok(up(p->tile_desc, p->s.tile_desc));
        if (e == hipSuccess) e = p->tile_meta.upload(p->s.tile_meta.get(), p->s.tile_meta_bytes);
        p->s.tile_meta.reset();
        ok(up(p->tile_first, p->s.tile_first));
        std::vector<int32_t>().swap(p->s.tile_first);
        ok(up(p->tile_info, p->s.tile_info));
        std::vector<uint32_t>().swap(p->s.tile_info);
        ok(up(p->tile_scale, p->s.tile_scale));
        tf::RawVec<unsigned char>().swap(p->s.tile_scale);
        if (p->s.streaming) {
            ok(up(p->row_info, p->s.row_info));
            std::vector<uint32_t>().swap(p->s.row_info);
            ok(up(p->row_scale, p->s.row_scale));
            tf::RawVec<unsigned char>().swap(p->s.row_scale);
        }
        ok(upload_pack(p->wf1, p->s.wf1));
        if (p->has_baseline) ok(upload_pack(p->all, p->s.all));
        ok(p->d1.alloc((size_t)p->s.d1.elements() * es));
        if (e != hipSuccess) return hip_fail(e, "allocating the plan's device memory");
        guard.p = nullptr;
        *out = p;
        return TF_OK;
    } catch (const std::bad_alloc &) {
        return fail(TF_ENOMEM, "out of host memory");
    }
}

tf_status tf_csr_validate(const tf_csr *M) {
    if (!M || !M->rowptr || M->n_rows < 0 || M->n_cols < 0 || M->nnz < 0 ||
        (M->nnz > 0 && !M->colidx))
        return fail(TF_EINVAL, "null argument or negative size");
    if (M->nnz >= (int64_t(1) << 31)) return fail(TF_EUNSUPPORTED, "indices are 32 bit");
    try {
        std::vector<int32_t> h_rowptr, h_colidx;
        const int32_t *rowptr = M->rowptr, *colidx = M->colidx;
        if (M->on_device) {
            h_rowptr.resize((size_t)M->n_rows + 1);
            h_colidx.resize((size_t)M->nnz);
            hipError_t e = hipMemcpy(h_rowptr.data(), M->rowptr, (M->n_rows + 1) * 4, hipMemcpyDeviceToHost);
            if (e == hipSuccess && M->nnz)
                e = hipMemcpy(h_colidx.data(), M->colidx, M->nnz * 4, hipMemcpyDeviceToHost);
            if (e != hipSuccess) return hip_fail(e, "copying the matrix to the host");
            rowptr = h_rowptr.data();
            colidx = h_colidx.data();
        }
        return check_csr_host(M->n_rows, M->n_cols, M->nnz, rowptr, colidx);
    } catch (const std::bad_alloc &) {
        return fail(TF_ENOMEM, "out of host memory");
    }
}

tf_status tf_plan_destroy(tf_plan *plan) {
    delete plan;
    return TF_OK;
}

tf_status tf_plan_schedule(const tf_plan *p, tf_schedule_view *v) {
    if (!p || !v) return fail(TF_EINVAL, "null argument");
    std::memset(v, 0, sizeof(*v));
    const tf::Schedule &s = p->s;
    const int es = tf::elem_size(p->dtype);
    v->n = p->n;
    v->nnz = p->nnz;
    v->t = s.t;
    v->col_slice = s.col_slice;
    v->n_slices = s.n_slices;
    v->dtype = p->dtype;
    v->b_is_sparse = p->b_is_sparse;
    v->n_coarse_tiles = s.n_coarse_tiles;
    v->n_tiles = (int64_t)s.tile_first_ptr.size() - 1;
    v->tile_first_ptr = s.tile_first_ptr.data();
    v->first_rows = s.first_rows.data();
    v->tile_second_ptr = s.tile_second_ptr.data();
    v->second_rows = s.second_rows.data();
    v->n_wf1_units = (int64_t)s.wf1_unit_ptr.size() - 1;
    v->wf1_unit_ptr = s.wf1_unit_ptr.data();
    v->wf1_rows = s.wf1_rows.data();
    v->spill = s.spill.data();
    v->n_fused_rows = s.n_fused_rows;
    v->n_wf1_rows = (int64_t)s.wf1_rows.size();
    v->n_spill_rows = s.n_spill_rows;
    v->fused_nnz = s.fused_nnz;
    v->fused_ratio_eq3 = p->n ? (double)s.n_fused_rows / (2.0 * (double)p->n) : 0.0;
    v->fused_ratio_rows = p->n ? (double)s.n_fused_rows / (double)p->n : 0.0;
    v->fused_ratio_nnz = p->nnz ? (double)s.fused_nnz / (double)p->nnz : 0.0;
    v->fast_mem_bytes = s.fast_mem_bytes;
    v->lds_fixed_bytes = s.lds_fixed_bytes;
    v->lds_bytes_per_row = s.lds_bytes_per_row;
    v->lds_row_granule = s.lds_row_granule;
    v->eq2_cost_max = s.eq2_cost_max;
    v->plan_seconds = p->plan_seconds;
    // algorithmic bytes: A once, B once (dense; a sparse B is not known to the plan and is left
    // out), C once, D once, and every spilled D1 row written once and read once
    const int64_t a_bytes = 4 * (p->n + 1) + p->nnz * (4 + es);
    const int64_t b_bytes = p->b_is_sparse ? 0 : p->n * p->bcol * es;
    const int64_t b_read = p->b_is_sparse ? 0 : (int64_t)s.first_rows.size() * p->bcol * es;
    const int64_t c_bytes = p->bcol * p->ccol * es;
    const int64_t d_bytes = p->n * p->ccol * es;
    v->n_first_rows = (int64_t)s.first_rows.size();
    v->alg_bytes = a_bytes + b_read + c_bytes + d_bytes + 2 * s.n_spill_rows * p->ccol * es;
    v->alg_bytes_unfused = a_bytes + b_bytes + c_bytes + 3 * d_bytes;
    v->second_block_in_lds = s.second_block_in_lds ? 1 : 0;
    v->second_block_bytes = s.second_block_cap;
    v->lds_launch_bytes =
        p->schedule_only
            ? 0
            : tf::fused_lds_bytes(p->dtype, p->b_is_sparse, (int)p->bcol, (int)p->ccol, s.col_slice,
                                  (int)s.max_tile_rows, s.second_block_in_lds ? (int)s.second_block_cap : 0,
                                  s.n_lds_rows > 0);
    v->spill_slot = s.spill_slot.data();
    v->n_direct_rows = s.n_direct_rows;
    v->d1_slices = s.d1.n_sl;
    v->d1_slice_cols = s.d1.sw;
    v->d1_rows = s.d1.rows;
    v->first_wavefront_streams = s.streaming ? 1 : 0;
    v->grown_tiles = s.grown_tiles ? 1 : 0;
    v->n_demoted_rows = s.n_demoted_rows;
    v->far_rows = s.far_rows ? 1 : 0;
    v->automatic = s.automatic ? 1 : 0;
    return TF_OK;
}

tf_status tf_plan_workspace(const tf_plan *p, void **d1_device) {
    if (!p || !d1_device) return fail(TF_EINVAL, "null argument");
    *d1_device = p->d1.p;
    return TF_OK;
}

tf_status tf_plan_prepare_unfused(const tf_plan *p) {
    if (!p) return fail(TF_EINVAL, "null argument");
    if (p->schedule_only) return fail(TF_EINVAL, "the plan was built with TF_FLAG_SCHEDULE_ONLY");
    return prepare_unfused(p);
}

tf_status tf_plan_workspace_unfused(const tf_plan *p, void **d1_device) {
    if (!p || !d1_device) return fail(TF_EINVAL, "null argument");
    *d1_device = p->d1_unf.p;
    return TF_OK;
}

tf_status tf_gemm_spmm(const tf_plan *p, const void *B, const void *C, void *D, void *stream) {
    tf_status st = check_exec(p, 0, C, D);
    if (st != TF_OK) return st;
    if (!B || !aligned16(B)) return fail(TF_EINVAL, "B must be a 16-byte aligned device pointer");
    st = first_wavefront_dense(p, B, C, D, p->d1.p, stream);
    if (st != TF_OK) return st;
    return second_wavefront(p, D, p->d1.p, stream);
}

tf_status tf_gemm_spmm_static(const tf_plan *p, const void *B, const void *C, void *D, void *stream) {
    tf_status st = check_exec(p, 0, C, D);
    if (st != TF_OK) return st;
    if (!B || !aligned16(B)) return fail(TF_EINVAL, "B must be a 16-byte aligned device pointer");
    const size_t need = (size_t)p->s.d1.elements() * (size_t)tf::elem_size(p->dtype);
    if (need > kStaticScratchBytes)
        return fail(TF_EUNSUPPORTED, "the plan's D1 workspace (" + std::to_string(need) +
                                         " bytes) exceeds the static workspace of " +
                                         std::to_string(kStaticScratchBytes) + " bytes");
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != TF_OK) return st;
    // every spilled row is written by the first wavefront before the second one reads it: nothing
    // in the array has to start at zero
    st = first_wavefront_dense(p, B, C, D, ws, stream);
    if (st != TF_OK) return st;
    return second_wavefront(p, D, ws, stream);
}

tf_status tf_spmm_spmm(const tf_plan *p, const tf_csr *B, const void *C, void *D, void *stream) {
    tf_status st = check_exec(p, 1, C, D);
    if (st != TF_OK) return st;
    st = check_sparse_b(p, B);
    if (st != TF_OK) return st;
    st = first_wavefront_sparse(p, B, C, D, p->d1.p, stream);
    if (st != TF_OK) return st;
    return second_wavefront(p, D, p->d1.p, stream);
}

tf_status tf_run_wavefront(const tf_plan *p, int32_t wavefront, const void *B_dense,
                           const tf_csr *B_csr, const void *C, void *D, void *stream) {
    if (!p) return fail(TF_EINVAL, "null argument");
    tf_status st = check_exec(p, p->b_is_sparse, C, D);
    if (st != TF_OK) return st;
    if (wavefront == 1) return second_wavefront(p, D, p->d1.p, stream);
    if (wavefront != 0) return fail(TF_EINVAL, "wavefront must be 0 or 1");
    if (p->b_is_sparse) {
        st = check_sparse_b(p, B_csr);
        if (st != TF_OK) return st;
        return first_wavefront_sparse(p, B_csr, C, D, p->d1.p, stream);
    }
    if (!B_dense || !aligned16(B_dense))
        return fail(TF_EINVAL, "B must be a 16-byte aligned device pointer");
    return first_wavefront_dense(p, B_dense, C, D, p->d1.p, stream);
}

tf_status tf_unfused_gemm_spmm(const tf_plan *p, const void *B, const void *C, void *D,
                               void *stream) {
    tf_status st = check_exec(p, 0, C, D);
    if (st != TF_OK) return st;
    if (!B || !aligned16(B)) return fail(TF_EINVAL, "B must be a 16-byte aligned device pointer");
    tf::GemmLaunch g{};
    if (!gemm_shape(p, g))
        return fail(TF_EUNSUPPORTED, "bCol is too large for the C slice of the unfused GeMM to fit LDS");
    st = prepare_unfused(p);
    if (st != TF_OK) return st;
    g.B = B;
    g.C = C;
    gemm_workspace(g, p->d1_unf.p, p->unf_layout());
    int e = tf::launch_gemm(g, stream);
    if (e) return hip_fail((hipError_t)e, "launching the GeMM");
    e = tf::launch_packed_spmm(all_rows_args(p, D), stream);
    if (e) return hip_fail((hipError_t)e, "launching the SpMM");
    return TF_OK;
}

tf_status tf_unfused_spmm_spmm(const tf_plan *p, const tf_csr *B, const void *C, void *D,
                               void *stream) {
    tf_status st = check_exec(p, 1, C, D);
    if (st != TF_OK) return st;
    st = check_sparse_b(p, B);
    if (st != TF_OK) return st;
    st = prepare_unfused(p);
    if (st != TF_OK) return st;
    tf::CsrSpmmLaunch f = csr_spmm_args(p, B, C, p->d1_unf.p, p->unf_layout());
    int e = tf::launch_csr_spmm(f, stream);
    if (e) return hip_fail((hipError_t)e, "launching the first SpMM");
    e = tf::launch_packed_spmm(all_rows_args(p, D), stream);
    if (e) return hip_fail((hipError_t)e, "launching the second SpMM");
    return TF_OK;
}

}  // extern "C"
