// gfx950 kernels of the tile-fusion path  D = A (B C).
//
//   k_fused_gemm_spmm   first wavefront, dense B   (paper Section 3.2, fused GeMM-SpMM listing)
//   k_fused_spmm_spmm   first wavefront, CSR B     (Section 3.2, fused SpMM-SpMM listing)
//   k_packed_spmm       second wavefront (rows whose D1 rows come from device memory); also the
//                       SpMM of the unfused baseline
//   k_gemm              D1 = B C for all rows: the GeMM of the unfused baseline, and the first
//                       wavefront of a dense-B plan that needs no tile in LDS
//   k_csr_spmm          D1 = B C for a CSR B, likewise
//
// A fused workgroup owns one tile (a list of D1 rows) and one column slice.  It produces the
// tile's D1 rows into LDS -- by MFMA for a dense B, by a row gather over C for a CSR B -- stores
// the rows flagged "spill" to the D1 workspace as well, and after one workgroup barrier computes
// the tile's fused rows of D straight out of LDS.  Fused rows of D that are a multiple of their
// own D1 row (only a diagonal entry) or empty leave from the registers that hold the D1 row.
// Nothing is accumulated with atomics: every output element is written by exactly one lane.
//
// Wave size is 64.  Lanes run across columns (16 bytes per lane where alignment allows), row
// groups across the rest of the wave.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <type_traits>

#include "tf_internal.h"

namespace tf {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef double doublex4 __attribute__((ext_vector_type(4)));

template <typename T> struct Tr;
// D(16x16) += A(16x4) * B(4x16), one wave.  Lane l supplies A[l % 16][l / 16] and
// B[l / 16][l % 16].  Afterwards lane l = 16 g + r holds, in component v, D[4 g + v][r] for
// fp32 but D[4 v + g][r] for fp64 (measured on gfx950).  `col_of_m` maps the M index that a
// lane feeds to the column of the C slice it stands for, chosen so that in both precisions
// lane (g, r) ends up with the four consecutive columns 4 g .. 4 g + 3 of row r.
template <> struct Tr<float> {
    static constexpr int V = 4;
    typedef floatx4 Acc;
    __device__ static __forceinline__ int col_of_m(int m) { return m; }
};
template <> struct Tr<double> {
    static constexpr int V = 2;
    typedef doublex4 Acc;
    __device__ static __forceinline__ int col_of_m(int m) { return 4 * (m & 3) + (m >> 2); }
};

__device__ __forceinline__ floatx4 mfma16(float a, float b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ doublex4 mfma16(double a, double b, doublex4 c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

template <typename T, int N> struct alignas(sizeof(T) * N) Pack {
    T x[N];
};

template <typename T, int N> __device__ __forceinline__ void load_pack(T (&dst)[N], const T *p) {
    const Pack<T, N> v = *reinterpret_cast<const Pack<T, N> *>(p);
#pragma unroll
    for (int i = 0; i < N; ++i) dst[i] = v.x[i];
}
template <typename T, int N> __device__ __forceinline__ void store_pack(T *p, const T (&src)[N]) {
    Pack<T, N> v;
#pragma unroll
    for (int i = 0; i < N; ++i) v.x[i] = src[i];
    *reinterpret_cast<Pack<T, N> *>(p) = v;
}

__device__ __forceinline__ int pow2_at_least(int x) {
    int g = 1;
    while (g < x) g <<= 1;
    return g;
}

// Consecutive workgroup ids are dealt round-robin to the eight XCDs, each with its own L2.
// Work items that touch neighbouring rows (adjacent tiles, the column slices of one tile, adjacent
// units of the second wavefront) should share an L2, so item ids are handed out in eight
// contiguous ranges, one per XCD: workgroup b works on item (b % 8) * ceil(total / 8) + b / 8.
__device__ __forceinline__ int64_t xcd_contiguous(int64_t bid, int64_t total) {
    const int64_t per = (total + kXcds - 1) / kXcds;
    return (bid % kXcds) * per + bid / kXcds;
}

// ------------------------------------------------------------------------------------------
// MFMA phase: stages the C slice in LDS in operand order and multiplies 16-row blocks of B.
//
// k is visited in a permuted order so that each lane can fetch 16 contiguous bytes of its B row:
// with V = elements per 16 bytes and KC = 4 V, MFMA number (s, q) pairs, in lane group g = l / 16,
// the element k = KC s + V g + q of the row with row k of C.  The C slice is laid out so that
// MFMA (s, q, nb) reads 64 consecutive elements: Cl[((s V + q) NB + nb) 64 + l] =
// C[KC s + V (l / 16) + q][c0 + 16 nb + col_of_m(l % 16)], zero beyond bCol or the slice width.
//
// The product is formed transposed (C^T in the first operand, B^T in the second), which leaves
// lane (g, r) with D1[row r][16 nb + 4 g .. + 3]: four contiguous columns, one vector store.
template <typename T, int NB>
__device__ __forceinline__ void stage_c_slice(T *Cl, const T *__restrict__ C, int bcol, int ldk,
                                              int ldc, int c0, int w) {
    constexpr int V = Tr<T>::V, KC = 4 * V;
    const int ksteps = (bcol + KC - 1) / KC;
    const int total = ksteps * V * NB * 64;
    constexpr int U = 8;                                  // loads in flight per thread
    for (int e0 = threadIdx.x; e0 < total; e0 += U * (int)blockDim.x) {
        T tmp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (int)blockDim.x;
            const int l = e & 63;
            const int rest = e >> 6;
            const int nb = rest % NB;
            const int sq = rest / NB;
            const int k = KC * (sq / V) + V * (l >> 4) + (sq % V);
            const int col = 16 * nb + Tr<T>::col_of_m(l & 15);
            const bool in = e < total && k < bcol && col < w;
            tmp[u] = C[in ? (int64_t)k * ldk + (int64_t)(c0 + col) * ldc : 0];
            if (!in) tmp[u] = T(0);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (int)blockDim.x;
            if (e < total) Cl[e] = tmp[u];
        }
    }
}

// The operands of the C slice that one lane feeds to the MFMAs, straight from device memory
// (what stage_c_slice would put at Cl[i * 64 + lane]); bCol = KC * KS exactly.  Element (k, c) of
// the multiplier is C[k ldk + c ldc] (ldc = 1 for C as given, ldk = 1 for its transpose).
template <typename T, int NB, int KS>
__device__ __forceinline__ void load_c_regs(T (&creg)[KS * Tr<T>::V * NB], const T *__restrict__ C,
                                            int ldk, int ldc, int c0, int w, int lane) {
    constexpr int V = Tr<T>::V, KC = 4 * V;
    // element (k, col) with k = V (lane / 16) + [KC (sq / V) + sq % V] and col = col_of_m(lane % 16)
    // + [16 nb]: a per-lane offset plus a wave-uniform one (the bracketed parts)
    const int lcol = Tr<T>::col_of_m(lane & 15);
    const uint32_t lane_off = (uint32_t)(V * (lane >> 4) * ldk + lcol * ldc);
    const T *base = C + (int64_t)c0 * ldc;
#pragma unroll
    for (int i = 0; i < KS * V * NB; ++i) {
        const int nb = i % NB, sq = i / NB;
        const int ku = KC * (sq / V) + (sq % V);
        const bool in = 16 * nb + lcol < w;
        creg[i] = (base + (ku * ldk + 16 * nb * ldc))[in ? lane_off : 0u];
        if (!in) creg[i] = T(0);
    }
}

template <typename T, int NB, bool FAST>
__device__ __forceinline__ void mfma_row_block(typename Tr<T>::Acc (&acc)[NB], const T *Cl,
                                               const T *__restrict__ brow, bool valid, int bcol,
                                               int lane) {
    constexpr int V = Tr<T>::V, KC = 4 * V;
    const int g = lane >> 4;
    const int ksteps = (bcol + KC - 1) / KC;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = typename Tr<T>::Acc{0, 0, 0, 0};
    for (int s = 0; s < ksteps; ++s) {
        const int kb = KC * s + V * g;
        T av[V];
        if (FAST) {
            if (valid && kb < bcol) {
                load_pack<T, V>(av, brow + kb);
            } else {
#pragma unroll
                for (int q = 0; q < V; ++q) av[q] = T(0);
            }
        } else {
#pragma unroll
            for (int q = 0; q < V; ++q) av[q] = (valid && kb + q < bcol) ? brow[kb + q] : T(0);
        }
#pragma unroll
        for (int q = 0; q < V; ++q) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = mfma16(Cl[((s * V + q) * NB + nb) * 64 + lane], av[q], acc[nb]);
        }
    }
}

// Stores the four columns a lane holds of accumulator block nb to `dst` (which points at the
// lane's first column), keeping to columns below w.
template <typename T, bool FAST>
__device__ __forceinline__ void store_acc4(T *dst, const typename Tr<T>::Acc &a, int col, int w) {
    constexpr int V = Tr<T>::V;
    if (FAST) {
#pragma unroll
        for (int h = 0; h < 4 / V; ++h) {
            if (col + V * h < w) {
                T tmp[V];
#pragma unroll
                for (int i = 0; i < V; ++i) tmp[i] = a[V * h + i];
                store_pack<T, V>(dst + V * h, tmp);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (col + i < w) dst[i] = a[i];
    }
}

// Gathers for R rows at once by one lane group: acc[r][0..N) += sum_k val[k] * X[idx[k] * ldx + ..]
// over k in [kb[r], ke[r]), k ascending per row.  E entries of every row are fetched per pass, so
// R * E independent gathers are in flight per lane; this is what hides the latency of the
// dependent index -> operand loads for short rows.  Slots beyond a row's end repeat a valid
// entry (so every load is unconditional and nothing waits on a branch) and are masked out of
// the sum; `k_any` is any valid entry index, used for rows that are empty.
template <typename T, int N, typename IdxT, int R, int E>
__device__ __forceinline__ void rows_dot(T (&acc)[R][N], const IdxT *__restrict__ idx,
                                         const T *__restrict__ val, const int (&kb)[R],
                                         const int (&ke)[R], const T *X, int64_t ldx) {
    int maxlen = 0, k_any = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (ke[r] - kb[r] > maxlen) {
            maxlen = ke[r] - kb[r];
            k_any = kb[r];
        }
    }
    for (int off = 0; off < maxlen; off += E) {
        int64_t c[R][E];
        T v[R][E];
        bool ok[R][E];
        T x[R][E][N];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int last = ke[r] > kb[r] ? ke[r] - 1 : k_any;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const int k = kb[r] + off + e;
                ok[r][e] = k < ke[r];
                const int kc = ok[r][e] ? k : last;
                c[r][e] = (int64_t)idx[kc];
                v[r][e] = val[kc];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < E; ++e) load_pack<T, N>(x[r][e], X + c[r][e] * ldx);
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const T vv = ok[r][e] ? v[r][e] : T(0);
#pragma unroll
                for (int i = 0; i < N; ++i) acc[r][i] += vv * (ok[r][e] ? x[r][e][i] : T(0));
            }
        }
    }
}

constexpr int kRowsPerPass = 4;     // R: rows a lane group works on at once
constexpr int kEntriesPerPass = 4;  // E: entries of each of those rows fetched per pass

// ------------------------------------------------------------------------------------------
// Packed row lists (see RowPack): every row of a unit has `slots` entries, so the gather loop has
// a wave-uniform trip count and needs neither row pointers nor bounds on individual entries.
//
// X is addressed as  base + idx * ldx + lane offset.  For operands below 4 GiB (and for LDS)
// the offset is formed in 32 bits, which lets the load use a scalar base plus a 32-bit lane
// offset; WIDE selects 64-bit arithmetic for larger operands.
template <typename T, int N, bool WIDE>
__device__ __forceinline__ void load_x(T (&x)[N], const T *X, uint32_t c, uint32_t ldx,
                                       uint32_t lane_off) {
    if (WIDE) {
        load_pack<T, N>(x, X + ((uint64_t)c * ldx + lane_off));
    } else {
        const uint32_t off = (c * ldx + lane_off) * (uint32_t)sizeof(T);
        load_pack<T, N>(x, reinterpret_cast<const T *>(reinterpret_cast<const char *>(X) + off));
    }
}

// One unit, rows not split: lane group `grp` of `ngrp` takes rows grp, grp + ngrp, ..., R at a
// time, E slots of each per pass (R * E gathers in flight per lane).  out(row id, acc).
template <typename T, int N, typename IdxT, int R, int E, bool WIDE, typename OutFn>
__device__ __forceinline__ void unit_rows(const UnitDesc d, const int32_t *__restrict__ rows,
                                          const IdxT *__restrict__ idx,
                                          const T *__restrict__ val, const T *X, uint32_t ldx,
                                          uint32_t lane_off, int grp, int ngrp, OutFn out) {
    const int L = d.slots;
    for (int i0 = grp; i0 < d.n_rows; i0 += ngrp * R) {
        const IdxT *ip[R];
        const T *vp[R];
        int32_t rid[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = i0 + r * ngrp;
            const int ic = i < d.n_rows ? i : i0;
            const int64_t at = d.entry_base + (int64_t)ic * L;
            ip[r] = idx + at;
            vp[r] = val + at;
            rid[r] = rows[d.row_begin + ic];
        }
        T acc[R][N];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int i = 0; i < N; ++i) acc[r][i] = T(0);
        int s = 0;
        for (; s + E <= L; s += E) {
            uint32_t c[R][E];
            T v[R][E];
            T x[R][E][N];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    c[r][e] = (uint32_t)ip[r][s + e];
                    v[r][e] = vp[r][s + e];
                }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < E; ++e) load_x<T, N, WIDE>(x[r][e], X, c[r][e], ldx, lane_off);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < E; ++e)
#pragma unroll
                    for (int i = 0; i < N; ++i) acc[r][i] += v[r][e] * x[r][e][i];
        }
        for (; s < L; ++s) {
            uint32_t c[R];
            T v[R];
            T x[R][N];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                c[r] = (uint32_t)ip[r][s];
                v[r] = vp[r][s];
            }
#pragma unroll
            for (int r = 0; r < R; ++r) load_x<T, N, WIDE>(x[r], X, c[r], ldx, lane_off);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < N; ++i) acc[r][i] += v[r] * x[r][i];
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (i0 + r * ngrp < d.n_rows) out(rid[r], acc[r]);
    }
}

extern __shared__ __align__(16) unsigned char tf_smem[];

// B operand of one 16-row block, all k: KS vectors of V elements per lane.
template <typename T, int KS> struct BFrag {
    T v[KS][Tr<T>::V];
};

// Loads are unconditional (the caller passes a row that exists): a lane whose row is padding
// computes garbage that is never stored, and each output row depends on its own lane only.
template <typename T, int KS>
__device__ __forceinline__ void load_b_frag(BFrag<T, KS> &f, const T *__restrict__ brow, int g) {
    constexpr int V = Tr<T>::V, KC = 4 * V;
#pragma unroll
    for (int s = 0; s < KS; ++s) load_pack<T, V>(f.v[s], brow + KC * s + V * g);
}

template <typename T, int NB, int KS>
__device__ __forceinline__ void mfma_frag(typename Tr<T>::Acc (&acc)[NB], const T *Cl,
                                          const BFrag<T, KS> &f, int lane) {
    constexpr int V = Tr<T>::V;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = typename Tr<T>::Acc{0, 0, 0, 0};
    // the C operands of step i + 1 are read from LDS before the MFMAs of step i are issued
    T c[2][NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) c[0][nb] = Cl[nb * 64 + lane];
#pragma unroll
    for (int i = 0; i < KS * V; ++i) {
        if (i + 1 < KS * V) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) c[(i + 1) & 1][nb] = Cl[((i + 1) * NB + nb) * 64 + lane];
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma16(c[i & 1][nb], f.v[i / V][i % V], acc[nb]);
    }
}

// The same with the lane's C operands already in registers (creg[(s V + q) NB + nb]).
template <typename T, int NB, int KS>
__device__ __forceinline__ void mfma_frag_reg(typename Tr<T>::Acc (&acc)[NB],
                                              const T (&creg)[KS * Tr<T>::V * NB],
                                              const BFrag<T, KS> &f) {
    constexpr int V = Tr<T>::V;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = typename Tr<T>::Acc{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int q = 0; q < V; ++q)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb] = mfma16(creg[(s * V + q) * NB + nb], f.v[s][q], acc[nb]);
}

template <typename T> constexpr int dtype_of() { return sizeof(T) == 8 ? TF_F64 : TF_F32; }

// Which tiles a fused workgroup works on.  Workgroups are persistent: workgroup b sits on XCD
// b % 8 (consecutive ids are dealt round-robin to the XCDs), keeps one column slice for its
// whole life (so the C slice is staged once) and walks through that XCD's contiguous range of
// tiles with a fixed stride.  The slices of a tile belong to neighbouring workgroups of one XCD.
struct TileWalk {
    int slice, tile, tile_end, step;
};
__device__ __forceinline__ TileWalk tile_walk(int n_tiles, int n_slices) {
    const int per = (n_tiles + kXcds - 1) / kXcds;
    const int k = blockIdx.x / kXcds, wg_per_xcd = gridDim.x / kXcds;
    TileWalk t;
    t.slice = k % n_slices;
    t.step = wg_per_xcd / n_slices;
    t.tile = (int)(blockIdx.x % kXcds) * per + k / n_slices;
    t.tile_end = min(n_tiles, ((int)(blockIdx.x % kXcds) + 1) * per);
    return t;
}

// LDS of a fused workgroup, as laid out by fused_lds_layout.
struct FusedSmem {
    int32_t *first[2];            // row ids of the current and of the next tile
    unsigned char *second;        // staged second-phase block (or unused)
    int32_t *bext, *bidx;         // CSR B: (first entry, length) of the rows of B of this tile and of the
    unsigned char *bval;          //        next (bext_stride ints apart), column indices and values
    int bext_stride;              //        (kSparseEntryCap slots per row)
    unsigned char *cslice;
    unsigned char *tile;
};
// sparse_es: element size for a CSR B (its staged rows take LDS), 0 for a dense B
__device__ __forceinline__ FusedSmem fused_smem(const FusedLaunch &a, bool c_regs, int64_t cbytes,
                                                int sparse_es) {
    auto up16 = [](int64_t x) { return (x + 15) & ~(int64_t)15; };
    FusedSmem m;
    m.first[0] = reinterpret_cast<int32_t *>(tf_smem);
    m.first[1] = m.first[0] + a.rows_cap;
    m.second = tf_smem + 2 * (int64_t)a.rows_cap * 4;
    unsigned char *p = m.second + (a.s_in_lds ? a.s_cap : 0);
    m.bext = reinterpret_cast<int32_t *>(p);
    m.bext_stride = (int)(up16((int64_t)a.tile_rows * 8) / 4);
    if (sparse_es) p += 2 * up16((int64_t)a.tile_rows * 8);
    m.bidx = reinterpret_cast<int32_t *>(p);
    if (sparse_es) p += up16((int64_t)a.tile_rows * kSparseEntryCap * 4);
    m.bval = p;
    if (sparse_es) p += up16((int64_t)a.tile_rows * kSparseEntryCap * sparse_es);
    m.cslice = p;
    m.tile = m.cslice + (c_regs ? 0 : cbytes);
    return m;
}

// Copies of a tile's block on their way from device memory to LDS: issued early, written late.
// NS 16-byte pieces per thread cover 16 NS bytes per thread of the workgroup; what is beyond that is
// copied by a plain loop at the time of writing.
typedef int32_t Piece __attribute__((ext_vector_type(4)));
template <int NS> struct Staged {
    Piece v[NS];
};
// (tid, nt): index of the calling thread among the nt threads that do the copy; tid < 0: not one of them
template <int NS>
__device__ __forceinline__ void stage_issue(Staged<NS> &st, const unsigned char *src, int bytes,
                                            int tid, int nt) {
    const Piece *p = reinterpret_cast<const Piece *>(src);
    const int n = bytes >> 4;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = tid + i * nt;
        st.v[i] = p[(tid >= 0 && e < n) ? e : 0];      // unconditional: the values stay in registers
    }
}
template <int NS>
__device__ __forceinline__ void stage_write(const Staged<NS> &st, unsigned char *dst,
                                            const unsigned char *src, int bytes, int tid, int nt) {
    if (tid < 0) return;
    Piece *q = reinterpret_cast<Piece *>(dst);
    const Piece *p = reinterpret_cast<const Piece *>(src);
    const int n = bytes >> 4;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = tid + i * nt;
        if (e < n) q[e] = st.v[i];
    }
    for (int e = tid + NS * nt; e < n; e += nt) q[e] = p[e];
}

// The arrays of a second-phase block.
template <typename T> struct SecondBlock {
    const TileUnit *units;
    const int32_t *rows2;
    const uint16_t *idx_a, *idx_b;      // operand positions of the even and of the odd slots, per pair
    const T *val;
};
template <typename T>
__device__ __forceinline__ SecondBlock<T> second_block(const unsigned char *sb, const TileDesc &d) {
    SecondBlock<T> b;
    const int off_rows2 = (d.n_units * (int)sizeof(TileUnit) + 15) & ~15;
    const int off_idx = (off_rows2 + d.n_second * 4 + 15) & ~15;
    const int off_val = (off_idx + d.n_entries * 2 + 15) & ~15;
    b.units = reinterpret_cast<const TileUnit *>(sb);
    b.rows2 = reinterpret_cast<const int32_t *>(sb + off_rows2);
    b.idx_a = reinterpret_cast<const uint16_t *>(sb + off_idx);
    b.idx_b = b.idx_a + (d.n_entries >> 1);
    b.val = reinterpret_cast<const T *>(sb + off_val);
    return b;
}

// After the tile's D1 rows are complete in LDS: computes the tile's fused rows of D, all
// operands out of LDS.  Lane group grp of ngrp owns
// the rows grp, grp + ngrp, ...; lane gl of the group owns VV columns from VV gl on.
//
// A unit's rows all have `stride` entry slots (even; the real length `len` may be one less)
// and are walked R rows at a time, two slots per step.  Nothing but LDS latency limits this
// loop, so the entries (index pair, value pair) of the next step are read while the operands of
// the current step are on their way.
// (The spilled rows of the tile have been stored during the first phase, by the waves or lane
// groups that produced them.)
template <typename T, int VV, int R, int W = 1>
__device__ __forceinline__ void fused_tail(const FusedLaunch &a, const TileDesc &d,
                                           const unsigned char *sb,
                                           const T *tileD1, int ldl, int c0, int gl, int grp,
                                           int ngrp) {
    const int ccol = a.ccol;
    const uint32_t lane_off = (uint32_t)(W * VV * gl);      // W packs of VV columns per lane
    const SecondBlock<T> b = second_block<T>(sb, d);
    T *__restrict__ D = static_cast<T *>(a.D);
    typedef Pack<T, 2> ValPair;
    const unsigned char *tile_lane = reinterpret_cast<const unsigned char *>(tileD1 + lane_off);
    for (int u = 0; u < d.n_units; ++u) {
        const TileUnit un = b.units[u];
        const int stride = un.slots & 0xffff, len = un.slots >> 16;
        const int S = stride >> 1;                                   // steps per row
        const int KB = (un.n_rows + ngrp * R - 1) / (ngrp * R);      // row blocks, wave-uniform
        const uint16_t *ia = b.idx_a + (un.entry_base >> 1), *ib = b.idx_b + (un.entry_base >> 1);
        const ValPair *vp = reinterpret_cast<const ValPair *>(b.val + un.entry_base);
        // rows past the unit's end re-read its last row
        auto row_at = [&](int kb, int r) {
            const int i = grp + (kb * R + r) * ngrp;
            return i < un.n_rows ? i : un.n_rows - 1;
        };
        // entries of step sp of the rows whose first entries sit at rb[]: operand offsets (16-byte
        // units) and values.  The step offset is kept as a scalar the compiler cannot fold into
        // the per-row positions, which would cost one vector add per array and row in every step.
        uint32_t cn[R][2];
        ValPair vn[R];
        struct RowEntries {           // where the entries of a row start in the three arrays
            const uint16_t *a, *b;
            const ValPair *v;
        };
        auto first_entries = [&](RowEntries (&rb)[R], int kb) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int at = row_at(kb, r) * S;
                rb[r].a = ia + at;
                rb[r].b = ib + at;
                rb[r].v = vp + at;
            }
        };
        auto read_entries = [&](const RowEntries (&rb)[R], int sp) {
            int so = sp;
            asm volatile("" : "+s"(so));
#pragma unroll
            for (int r = 0; r < R; ++r) {
                cn[r][0] = rb[r].a[so];
                cn[r][1] = rb[r].b[so];
                vn[r] = rb[r].v[so];
            }
        };
        RowEntries rb[R], rbn[R];
        first_entries(rb, 0);
        if (S > 0) read_entries(rb, 0);
        // all steps of a row but the last have two entries; the last has two when the longest
        // row's length is even.  `more`: entries are read ahead for the following step.
        const bool last_two = 2 * S - 1 < len;
        for (int kb = 0; kb < KB; ++kb) {
            int32_t rid[R];
#pragma unroll
            for (int r = 0; r < R; ++r) rid[r] = b.rows2[un.row_begin + row_at(kb, r)];
            T acc[R][W][VV];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int wq = 0; wq < W; ++wq)
#pragma unroll
                    for (int i = 0; i < VV; ++i) acc[r][wq][i] = T(0);
            auto step = [&](auto two_c, const RowEntries (&next_rb)[R], int nsp, bool more) {
                constexpr bool TWO = decltype(two_c)::value;
                ValPair v[R];
                T x[R][2][W][VV];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    v[r] = vn[r];
#pragma unroll
                    for (int wq = 0; wq < W; ++wq) {
                        load_pack<T, VV>(x[r][0][wq],
                                         reinterpret_cast<const T *>(tile_lane + (cn[r][0] << 4)) + wq * VV);
                        if (TWO)
                            load_pack<T, VV>(x[r][1][wq],
                                             reinterpret_cast<const T *>(tile_lane + (cn[r][1] << 4)) + wq * VV);
                    }
                }
                if (more) read_entries(next_rb, nsp);
#pragma unroll
                for (int r = 0; r < R; ++r) {
#pragma unroll
                    for (int wq = 0; wq < W; ++wq) {
#pragma unroll
                        for (int i = 0; i < VV; ++i) acc[r][wq][i] += v[r].x[0] * x[r][0][wq][i];
                        if (TWO) {
#pragma unroll
                            for (int i = 0; i < VV; ++i) acc[r][wq][i] += v[r].x[1] * x[r][1][wq][i];
                        }
                    }
                }
            };
            for (int sp = 0; sp + 1 < S; ++sp) step(std::true_type(), rb, sp + 1, true);
            if (S > 0) {
                // the step after the last one is the first of the next row block
                const bool more = kb + 1 < KB;
                if (more) first_entries(rbn, kb + 1);
                if (last_two) step(std::true_type(), rbn, 0, more);
                else step(std::false_type(), rbn, 0, more);
                if (more) {
#pragma unroll
                    for (int r = 0; r < R; ++r) rb[r] = rbn[r];
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (grp + (kb * R + r) * ngrp < un.n_rows) {
#pragma unroll
                    for (int wq = 0; wq < W; ++wq)
                        store_pack<T, VV>(D + (int64_t)rid[r] * ccol + c0 + lane_off + wq * VV, acc[r][wq]);
                }
        }
    }
}

constexpr int kStagePieces = 3;     // 16-byte pieces of a second-phase block in flight per thread

// First wavefront, dense B.  A workgroup walks through its tiles; per tile
//   phase 1  multiplies the tile's rows of B by the C slice with MFMA into the LDS tile (spilled
//            rows also go to the D1 workspace, straight from the accumulators), while the
//            tile's second-phase block and the next tile's row ids travel to LDS;
//   barrier;
//   phase 2  starts the loads of the next tile's first rows of B and computes the tile's fused
//            rows of D out of LDS;
//   barrier (the LDS tile is rewritten by the next tile).
// KS > 0: bCol = 4 V KS exactly and the B rows of the next two 16-row blocks of a wave are in
// flight while the current block is multiplied; KS = 0: any bCol, no prefetch.
// SLDS: the second-phase blocks are staged in LDS (else they are read where they are).
template <typename T, int NB, int KS, bool FAST, bool SLDS>
__global__ __launch_bounds__(kFusedThreads) void k_fused_gemm_spmm(const FusedLaunch a) {
    constexpr int V = Tr<T>::V, KC = 4 * V;
    constexpr int VV = FAST ? V : 1;
    constexpr int KSF = KS > 0 ? KS : 1;
    constexpr bool CREG = c_in_registers(dtype_of<T>(), NB, KS);
    TileWalk tw = tile_walk(a.n_tiles, a.n_slices);
    if (tw.tile >= tw.tile_end) return;
    const int c0 = tw.slice * a.cs;
    const int w = min(a.cs, a.ccol - c0);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = (int)blockDim.x >> 6;
    const int g = lane >> 4, r = lane & 15;
    const int bcol_pad = (a.bcol + KC - 1) / KC * KC;
    const int ldl = 16 * NB + V;
    const FusedSmem sm = fused_smem(a, CREG, (int64_t)bcol_pad * 16 * NB * (int64_t)sizeof(T), 0);
    T *Cl = reinterpret_cast<T *>(sm.cslice);
    T *tileD1 = reinterpret_cast<T *>(sm.tile);
    const T *__restrict__ B = static_cast<const T *>(a.B);
    const int G = pow2_at_least((a.cs + VV - 1) / VV);
    const int gl = threadIdx.x % G, grp = threadIdx.x / G, ngrp = (int)blockDim.x / G;

    // row of B behind lane r of block lb; blocks past the end of the tile name its last row, so
    // that every load is unconditional (first[] is padded to a multiple of 16 rows)
    auto row_of = [&](const int32_t *first, int rows, int lb) -> int64_t {
        const int lr = lb * 16 + r;
        return (int64_t)first[lr < rows ? lr : rows - 1];
    };

    TileDesc d = a.tile_desc[tw.tile];
    int par = 0;
    // nmw waves run the matrix cores (measured: all of them is best; one per SIMD with deeper
    // prefetch, the rest copying metadata, is slower); the threads that do not copy the tile's
    // second-phase block and the next tile's row ids into LDS meanwhile.
    const int nmw = nwaves;
    const bool is_mfma = wave < nmw;
    const int snt = nwaves > nmw ? (int)blockDim.x - 64 * nmw : (int)blockDim.x;
    const int stid = nwaves > nmw ? (int)threadIdx.x - 64 * nmw : (int)threadIdx.x;
    // B buffers per wave, ND - 1 blocks ahead (measured: 3 is better than 4); two when a block of B
    // rows is 64 registers per lane, three of which would not leave room for the rest
    constexpr int ND = KSF * Tr<T>::V * (int)(sizeof(T) / 4) >= 64 ? 2 : 3;
    BFrag<T, KSF> fb[ND];
    T creg[CREG ? KSF * V * NB : 1];
    {
        // Start-up, ordered so that the longest chain (row ids -> rows of B) begins first: each
        // lane fetches the ids of its own first rows straight from device memory, at an address
        // that follows from the tile's number (no wait for the descriptor; ids past the tile's
        // last row repeat it up to the stride); the C operands and the copy of all row ids to LDS
        // follow, then the B loads go out.
        const int32_t *src = a.tile_first + (int64_t)tw.tile * a.first_stride;
        int64_t row0[ND - 1];
        if constexpr (KS > 0) {
#pragma unroll
            for (int i = 0; i < ND - 1; ++i) row0[i] = row_of(src, a.first_stride, wave + i * nmw);
        }
        const int n16 = (d.n_rows + 15) & ~15;
        for (int e = threadIdx.x; e < n16; e += (int)blockDim.x) sm.first[0][e] = src[e];
        if constexpr (KS > 0) {
            if (is_mfma) {
#pragma unroll
                for (int i = 0; i < ND - 1; ++i) load_b_frag<T, KSF>(fb[i], B + row0[i] * a.bcol, g);
            }
        }
        const T *Cg = static_cast<const T *>(a.C);
        if constexpr (CREG) load_c_regs<T, NB, KSF>(creg, Cg, a.c_ldk, a.c_ldc, c0, w, lane);
        else stage_c_slice<T, NB>(Cl, Cg, a.bcol, a.c_ldk, a.c_ldc, c0, w);
        __syncthreads();
    }

    for (;;) {
        const int rows = d.n_rows;
        const int32_t *first = sm.first[0] + par * a.rows_cap;
        int32_t *next_first = sm.first[0] + (par ^ 1) * a.rows_cap;
        const int nblk = (rows + 15) >> 4;
        const int ntile = tw.tile + tw.step;
        const bool has_next = ntile < tw.tile_end;
        const TileDesc nd = a.tile_desc[has_next ? ntile : tw.tile];
        const unsigned char *blk = a.tile_meta + d.meta_off;
        const Piece *nsrc = reinterpret_cast<const Piece *>(
            a.tile_first + (int64_t)(has_next ? ntile : tw.tile) * a.first_stride);

        // on their way during phase 1: this tile's second-phase block, the next tile's row ids
        Staged<kStagePieces> st;
        const int nfirst_pieces = has_next ? ((nd.n_rows + 15) >> 4) * 4 : 0;
        if constexpr (SLDS) stage_issue<kStagePieces>(st, blk, d.s_bytes, stid, snt);
        const Piece nfirst = nsrc[(stid >= 0 && stid < nfirst_pieces) ? stid : 0];

        // all 16 NB columns of a block's rows are written (the tile's rows are that wide)
        auto write_block = [&](int lb, typename Tr<T>::Acc(&acc)[NB]) {
            T *dst = tileD1 + (lb * 16 + r) * ldl + 4 * g;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int h = 0; h < 4 / V; ++h) {
                    T tmp[V];
#pragma unroll
                    for (int i = 0; i < V; ++i) tmp[i] = acc[nb][V * h + i];
                    store_pack<T, V>(dst + 16 * nb + V * h, tmp);
                }
            }
        };
        // Rows that leave from the accumulators of the wave that produced them (as the unfused
        // product stores its rows): lane (g, r) holds columns 16 nb + 4 g .. + 3 of row r, so the four
        // lanes of a row store 64 contiguous bytes per block of columns.  `info` is the lane's info
        // word (0 past the tile's end), fetched from device memory before the multiplications.
        //  - spilled rows go to their slot of the D1 workspace (column slices of d1_sw columns);
        //  - direct rows of D (the D1 row times the diagonal entry `sc`) and empty rows of D go to D.
        // (Reading the rows back from the LDS tile, whole rows per store, cost a chain of two LDS
        // round trips per pass of four rows.)
        const int64_t info_base = (int64_t)tw.tile * a.first_stride;
        auto row_info = [&](int lb) -> uint32_t { return a.tile_info[info_base + lb * 16 + r]; };
        auto row_scale = [&](int lb) -> T {
            return a.tile_scale ? static_cast<const T *>(a.tile_scale)[info_base + lb * 16 + r] : T(0);
        };
        auto store_cols = [&](T *dst, int nb, const T (&x)[4]) {      // dst: the lane's first column of block nb
#pragma unroll
            for (int h = 0; h < 4 / V; ++h) {
                const int col = 16 * nb + 4 * g + V * h;
                if (FAST) {
                    if (col < w) {
                        T tmp[V];
#pragma unroll
                        for (int i = 0; i < V; ++i) tmp[i] = x[V * h + i];
                        store_pack<T, V>(dst + V * h, tmp);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < V; ++i)
                        if (col + i < w) dst[V * h + i] = x[V * h + i];
                }
            }
        };
        auto spill_block = [&](uint32_t info, typename Tr<T>::Acc(&acc)[NB]) {
            if (!(info & kInfoSpill)) return;
            T *slot = static_cast<T *>(a.D1) + (int64_t)(info & kInfoSlotMask) * a.d1_sw + 4 * g;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int cb = c0 + 16 * nb;                        // wave-uniform
                T x[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = acc[nb][i];
                store_cols(slot + (int64_t)(cb >> a.d1_sw_shift) * a.d1_slice_stride + (cb & a.d1_sw_mask),
                           nb, x);
            }
        };
        auto direct_block = [&](uint32_t info, T sc, int64_t row, typename Tr<T>::Acc(&acc)[NB]) {
            if (!(info & (kInfoDirect | kInfoZero))) return;
            T *dst = static_cast<T *>(a.D) + row * a.ccol + c0 + 4 * g;
            if (info & kInfoZero) sc = T(0);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                T x[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) x[i] = (info & kInfoZero) ? T(0) : sc * acc[nb][i];
                store_cols(dst + 16 * nb, nb, x);
            }
        };
        const bool has2 = d.n_second > 0;       // fused rows that read the LDS tile
        if constexpr (KS > 0) {
            // One block per step: start the loads of the block ND - 1 steps ahead, multiply,
            // write the results to the LDS tile.  The B buffers rotate by name (the loop is
            // unrolled ND times), never by copying: a copy of a buffer would have to wait for
            // the loads that fill it.
            auto step = [&](auto fi, int lb) {
                constexpr int FI = decltype(fi)::value;
                load_b_frag<T, KSF>(fb[(FI + ND - 1) % ND],
                                    B + row_of(first, rows, lb + (ND - 1) * nmw) * a.bcol, g);
                // the loads go out before the multiplications, not after them: left alone the
                // compiler reuses the accumulators' registers for the buffer being filled and
                // sinks the loads to the end of the step, which halves the distance they run ahead
                const uint32_t info = row_info(lb);
                const T sc = row_scale(lb);
                __builtin_amdgcn_sched_barrier(0);
                typename Tr<T>::Acc acc[NB];
                if constexpr (CREG) {
                    mfma_frag_reg<T, NB, KSF>(acc, creg, fb[FI]);
                } else {
                    // the C slice is loop invariant: without this the compiler keeps all of it
                    // in registers, which the rest of the kernel cannot spare
                    asm volatile("" ::: "memory");
                    mfma_frag<T, NB, KSF>(acc, Cl, fb[FI], lane);
                }
                if (has2) write_block(lb, acc);
                spill_block(info, acc);
                direct_block(info, sc, row_of(first, rows, lb), acc);
            };
            if (is_mfma) {
                for (int lb = wave; lb < nblk; lb += ND * nmw) {
                    step(std::integral_constant<int, 0>(), lb);
                    if (lb + nmw >= nblk) break;
                    step(std::integral_constant<int, 1>(), lb + nmw);
                    static_assert(ND >= 2 && ND <= 4, "the loop is unrolled once per B buffer");
                    if constexpr (ND >= 3) {
                        if (lb + 2 * nmw >= nblk) break;
                        step(std::integral_constant<int, 2>(), lb + 2 * nmw);
                    }
                    if constexpr (ND == 4) {
                        if (lb + 3 * nmw >= nblk) break;
                        step(std::integral_constant<int, 3>(), lb + 3 * nmw);
                    }
                }
            }
        } else {
            for (int lb = wave; lb < nblk; lb += nwaves) {
                const uint32_t info = row_info(lb);
                const T sc = row_scale(lb);
                typename Tr<T>::Acc acc[NB];
                mfma_row_block<T, NB, FAST>(acc, Cl, B + row_of(first, rows, lb) * a.bcol, true,
                                            a.bcol, lane);
                if (has2) write_block(lb, acc);
                spill_block(info, acc);
                direct_block(info, sc, row_of(first, rows, lb), acc);
            }
        }
        if constexpr (SLDS) stage_write<kStagePieces>(st, sm.second, blk, d.s_bytes, stid, snt);
        if (stid >= 0) {
            if (stid < nfirst_pieces) reinterpret_cast<Piece *>(next_first)[stid] = nfirst;
            for (int e = snt + stid; e < nfirst_pieces; e += snt)
                reinterpret_cast<Piece *>(next_first)[e] = nsrc[e];
        }
        __syncthreads();
        if constexpr (KS > 0) {
            if (has_next && is_mfma) {
                // first blocks of the next tile: on their way during this tile's second phase
#pragma unroll
                for (int i = 0; i < ND - 1; ++i)
                    load_b_frag<T, KSF>(fb[i], B + row_of(next_first, nd.n_rows, wave + i * nmw) * a.bcol, g);
            }
        }
        // (three rows per lane group at a time: with four the kernel no longer fits the 256
        // registers of a wave at this occupancy and spills)
        // When the slice is a whole number of double packs each lane takes two packs of a row
        // (half as many lanes per row, twice as many rows per wave): the index and address work of
        // a step is shared by twice as many columns.
        if (!has2) {
            // nothing reads the LDS tile: the workgroup streams on
        } else if (FAST && G >= 2 && w % (2 * VV) == 0) {
            const int G2 = G / 2;
            const int gl2 = (int)threadIdx.x % G2;
            if (2 * VV * gl2 < w)
                fused_tail<T, VV, 2, 2>(a, d, SLDS ? sm.second : blk, tileD1, ldl, c0, gl2,
                                        (int)threadIdx.x / G2, (int)blockDim.x / G2);
        } else if (VV * gl < w) {
            fused_tail<T, VV, 3>(a, d, SLDS ? sm.second : blk, tileD1, ldl, c0, gl, grp, ngrp);
        }
        if (!has_next) break;
        // (the next tile rewrites the LDS tile and the staged block; its row ids are in the other buffer)
        if (has2) __syncthreads();
        d = nd;
        tw.tile = ntile;
        par ^= 1;
    }
}

constexpr int kEntriesPerPassLong = 4;   // entries in flight per lane for a row too long to stage

// Y[pos] = S[row_of(pos), :] X for a list of `rows` rows of a CSR matrix S handled by one workgroup.
// Per row the chain row id -> extent -> entries -> rows of X is three dependent loads; walked row
// by row it leaves the memory pipe idle most of the time.  Here the whole workgroup takes each
// link of the chain for all rows of the list at once, handing over through LDS:
// stage_extents      (1) extents of all rows;
// stage_entries      (2) up to kSparseEntryCap entries of every row (padding slots repeat the
//                    row's last entry, or column 0 for an empty row, so that the gathers need no
//                    bounds);
// gather_staged_rows (3) the gathers, RP rows of kSparseEntryCap slots each in flight per lane;
//                    out(pos, acc) takes a finished row.  A row with more entries than the cap
//                    is gathered from device memory entry by entry.
// ext holds 2 ints per row, eidx and eval kSparseEntryCap slots per row (LDS, 16-byte aligned).
template <typename RowFn>
__device__ __forceinline__ void stage_extents(int rows, int32_t *ext,
                                              const int32_t *__restrict__ rowptr, RowFn row_of) {
    for (int i = threadIdx.x; i < rows; i += (int)blockDim.x) {
        const int64_t rid = row_of(i);
        const int kb = rowptr[rid], ke = rowptr[rid + 1];
        ext[2 * i] = kb;
        ext[2 * i + 1] = ke - kb;
    }
}
// (the extents must be visible to the workgroup; ends with a barrier)
template <typename T>
__device__ __forceinline__ void stage_entries(int rows, const int32_t *ext, int32_t *eidx, T *eval,
                                              const int32_t *__restrict__ colidx,
                                              const T *__restrict__ vals) {
    constexpr int CAP = kSparseEntryCap;
    constexpr int SW = 4;                                  // slots per thread whose loads go out together
    const int total = rows * CAP;
    for (int s0 = threadIdx.x; s0 < total; s0 += SW * (int)blockDim.x) {
        int32_t ci[SW];
        T v[SW];
#pragma unroll
        for (int u = 0; u < SW; ++u) {
            const int s = s0 + u * (int)blockDim.x;
            const int i = (s < total ? s : s0) / CAP, e = s % CAP;
            const int kb = ext[2 * i], len = ext[2 * i + 1];
            ci[u] = 0;
            v[u] = T(0);
            if (len > 0 && len <= CAP) {
                const int k = kb + (e < len ? e : len - 1);
                ci[u] = colidx[k];
                v[u] = vals[k];
            }
        }
#pragma unroll
        for (int u = 0; u < SW; ++u) {
            const int s = s0 + u * (int)blockDim.x;
            if (s < total) {
                eidx[s] = ci[u];
                eval[s] = v[u];
            }
        }
    }
    __syncthreads();
}

// pre(pos) is called before the gathers of a row go out and its result handed to out(pos, pre, acc):
// what a finished row needs to know from device memory is then fetched along with the operands.
template <typename T, int VV, int RP, typename PreFn, typename OutFn>
__device__ __forceinline__ void gather_staged_rows(int rows, const int32_t *ext, const int32_t *eidx,
                                                   const T *eval,
                                                   const int32_t *__restrict__ colidx,
                                                   const T *__restrict__ vals, const T *Xl,
                                                   int64_t ldx, bool active, int grp, int ngrp,
                                                   PreFn pre, OutFn out) {
    constexpr int CAP = kSparseEntryCap;
    typedef int32_t Idx4 __attribute__((ext_vector_type(4)));
    for (int base = grp; base < rows; base += ngrp * RP) {
        int pos[RP], len[RP];
        bool ok[RP];
#pragma unroll
        for (int r = 0; r < RP; ++r) {
            pos[r] = base + r * ngrp;
            ok[r] = pos[r] < rows;
            if (!ok[r]) pos[r] = base;
            len[r] = ok[r] ? ext[2 * pos[r] + 1] : 0;
        }
        if (!active) continue;
        T acc[RP][VV];
        int32_t ci[RP][CAP];
        decltype(pre(0)) pr[RP];
#pragma unroll
        for (int r = 0; r < RP; ++r) {
            pr[r] = pre(pos[r]);
#pragma unroll
            for (int i = 0; i < VV; ++i) acc[r][i] = T(0);
            const Idx4 *p = reinterpret_cast<const Idx4 *>(eidx + pos[r] * CAP);
#pragma unroll
            for (int q = 0; q < CAP / 4; ++q) {
                const Idx4 c4 = p[q];
#pragma unroll
                for (int j = 0; j < 4; ++j) ci[r][4 * q + j] = c4[j];
            }
        }
        // All loads of a half (four slots) go out back to back, unconditionally: every slot names a
        // valid row of X.  The second half is skipped when no row of the wave reaches into it (a
        // wave-uniform branch; a branch per slot made the compiler wait for each load in turn).
        static_assert(CAP == 8, "the slots are fetched in two halves of four");
        T x[RP][CAP][VV];
        bool far = false;
#pragma unroll
        for (int r = 0; r < RP; ++r) far = far || (len[r] > CAP / 2 && len[r] <= CAP);
        const bool second_half = __builtin_amdgcn_ballot_w64(far) != 0;
#pragma unroll
        for (int e = 0; e < CAP / 2; ++e)
#pragma unroll
            for (int r = 0; r < RP; ++r) load_pack<T, VV>(x[r][e], Xl + (int64_t)ci[r][e] * ldx);
        if (second_half) {
#pragma unroll
            for (int e = CAP / 2; e < CAP; ++e)
#pragma unroll
                for (int r = 0; r < RP; ++r) load_pack<T, VV>(x[r][e], Xl + (int64_t)ci[r][e] * ldx);
        }
        auto sum_slots = [&](int r, const T(&v)[CAP], int e0) {
#pragma unroll
            for (int e = e0; e < e0 + CAP / 2; ++e) {
                const bool use = e < len[r] && len[r] <= CAP;
                const T vv = use ? v[e] : T(0);
#pragma unroll
                for (int i = 0; i < VV; ++i) acc[r][i] += vv * (use ? x[r][e][i] : T(0));
            }
        };
#pragma unroll
        for (int r = 0; r < RP; ++r) {
            T v[CAP];
            const T *vp = eval + pos[r] * CAP;
#pragma unroll
            for (int q = 0; q < CAP; q += Tr<T>::V)
                load_pack<T, Tr<T>::V>(*reinterpret_cast<T(*)[Tr<T>::V]>(&v[q]), vp + q);
            sum_slots(r, v, 0);
            if (second_half) sum_slots(r, v, CAP / 2);
        }
#pragma unroll
        for (int r = 0; r < RP; ++r) {
            if (len[r] > CAP) {
                const int kb1[1] = {ext[2 * pos[r]]};
                const int ke1[1] = {kb1[0] + len[r]};
                T a1[1][VV];
#pragma unroll
                for (int i = 0; i < VV; ++i) a1[0][i] = T(0);
                rows_dot<T, VV, int32_t, 1, kEntriesPerPassLong>(a1, colidx, vals, kb1, ke1, Xl, ldx);
#pragma unroll
                for (int i = 0; i < VV; ++i) acc[r][i] = a1[0][i];
            }
            if (ok[r]) out(pos[r], pr[r], acc[r]);
        }
    }
}

// First wavefront, CSR B: phase 1 gathers rows of C for the tile's rows of B into the LDS tile.
// Gathers hide their latency with waves: the workgroup is as large as the machine allows (16
// waves) and each lane group keeps one row (kSparseEntryCap gathers) in flight, so that a wave
// fits 128 registers.
constexpr int kFusedSparseThreads = 1024;
template <typename T, bool FAST, bool SLDS>
__global__ __launch_bounds__(kFusedSparseThreads) void k_fused_spmm_spmm(const FusedLaunch a) {
    constexpr int VV = FAST ? Tr<T>::V : 1;
    TileWalk tw = tile_walk(a.n_tiles, a.n_slices);
    if (tw.tile >= tw.tile_end) return;
    const int c0 = tw.slice * a.cs;
    const int w = min(a.cs, a.ccol - c0);
    const int ldl = (a.cs + Tr<T>::V - 1) / Tr<T>::V * Tr<T>::V;
    const FusedSmem sm = fused_smem(a, true, 0, (int)sizeof(T));
    T *tileD1 = reinterpret_cast<T *>(sm.tile);
    const int G = pow2_at_least((a.cs + VV - 1) / VV);
    const int gl = threadIdx.x % G, grp = threadIdx.x / G, ngrp = (int)blockDim.x / G;
    const T *__restrict__ bvals = static_cast<const T *>(a.Bs.vals);
    const T *__restrict__ C = static_cast<const T *>(a.C);
    const int ccol = a.ccol;

    TileDesc d = a.tile_desc[tw.tile];
    int par = 0;
    {
        const int n16 = (d.n_rows + 15) & ~15;
        const int32_t *src = a.tile_first + (int64_t)tw.tile * a.first_stride;
        for (int e = threadIdx.x; e < n16; e += (int)blockDim.x) sm.first[0][e] = src[e];
    }
    __syncthreads();
    // extents of the first tile's rows of B; those of every later tile are fetched during the
    // second phase of the tile before it
    auto row_id = [](const int32_t *ids, int i) { return (int64_t)ids[i]; };
    stage_extents(d.n_rows, sm.bext, a.Bs.rowptr, [&](int i) { return row_id(sm.first[0], i); });
    __syncthreads();
    for (;;) {
        const int rows = d.n_rows;
        const int32_t *first = sm.first[0] + par * a.rows_cap;
        const int ntile = tw.tile + tw.step;
        const bool has_next = ntile < tw.tile_end;
        const TileDesc nd = a.tile_desc[has_next ? ntile : tw.tile];
        const unsigned char *blk = a.tile_meta + d.meta_off;
        Staged<kStagePieces> st;
        const bool has2 = d.n_second > 0;       // fused rows that read the LDS tile
        const int nfirst_pieces = has_next ? ((nd.n_rows + 15) >> 4) * 4 : 0;
        if constexpr (SLDS) stage_issue<kStagePieces>(st, blk, d.s_bytes, threadIdx.x, blockDim.x);
        const Piece *nsrc = reinterpret_cast<const Piece *>(
            a.tile_first + (int64_t)(has_next ? ntile : tw.tile) * a.first_stride);
        const Piece nfirst = nsrc[(int)threadIdx.x < nfirst_pieces ? threadIdx.x : 0];

        // D1[pos] = B[row(pos), :] C for the tile's rows, into the LDS tile; a row that the second
        // wavefront reads also goes to the D1 workspace, from the registers of its lane group
        {
            T *eval = reinterpret_cast<T *>(sm.bval);
            const int32_t *ext_cur = sm.bext + par * sm.bext_stride;
            stage_entries<T>(rows, ext_cur, sm.bidx, eval, a.Bs.colidx, bvals);
            T *tile_lane = tileD1 + VV * gl;
            // the lane's columns of a workspace row (slices of d1_sw columns) and of a row of D
            const int colg = c0 + VV * gl;
            T *D1l = static_cast<T *>(a.D1) + (int64_t)(colg >> a.d1_sw_shift) * a.d1_slice_stride +
                     (colg & a.d1_sw_mask);
            T *Dl = static_cast<T *>(a.D) + colg;
            const uint32_t *info_t = a.tile_info + (int64_t)tw.tile * a.first_stride;
            const T *scale_t = a.tile_scale
                                   ? static_cast<const T *>(a.tile_scale) + (int64_t)tw.tile * a.first_stride
                                   : nullptr;
            struct RowInfo {
                uint32_t info;
                T sc;
            };
            gather_staged_rows<T, VV, 1>(
                rows, ext_cur, sm.bidx, eval, a.Bs.colidx, bvals, C + c0 + VV * gl, ccol,
                VV * gl < w, grp, ngrp,
                [&](int pos) { return RowInfo{info_t[pos], scale_t ? scale_t[pos] : T(0)}; },
                [&](int pos, const RowInfo &ri, const T(&acc)[VV]) {
                    if (has2) store_pack<T, VV>(tile_lane + (int64_t)pos * ldl, acc);
                    if (ri.info & kInfoSpill)
                        store_pack<T, VV>(D1l + (int64_t)(ri.info & kInfoSlotMask) * a.d1_sw, acc);
                    if (ri.info & (kInfoDirect | kInfoZero)) {
                        T x[VV];
#pragma unroll
                        for (int i = 0; i < VV; ++i) x[i] = (ri.info & kInfoZero) ? T(0) : ri.sc * acc[i];
                        store_pack<T, VV>(Dl + (int64_t)first[pos] * ccol, x);
                    }
                });
        }

        if constexpr (SLDS) stage_write<kStagePieces>(st, sm.second, blk, d.s_bytes, threadIdx.x, blockDim.x);
        if ((int)threadIdx.x < nfirst_pieces)
            reinterpret_cast<Piece *>((sm.first[0] + (par ^ 1) * a.rows_cap))[threadIdx.x] = nfirst;
        for (int e = (int)blockDim.x + threadIdx.x; e < nfirst_pieces; e += (int)blockDim.x)
            reinterpret_cast<Piece *>((sm.first[0] + (par ^ 1) * a.rows_cap))[e] =
                nsrc[e];
        __syncthreads();
        // the extents of the next tile's rows of B are on their way during the second phase
        constexpr int NE = 1;                               // rows per thread fetched that way
        const int32_t *next_first = sm.first[0] + (par ^ 1) * a.rows_cap;
        int nb0[NE], nb1[NE];
        if (has_next) {
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const int i = (int)threadIdx.x + e * (int)blockDim.x;
                if (i < nd.n_rows) {
                    const int64_t rid = row_id(next_first, i);
                    nb0[e] = a.Bs.rowptr[rid];
                    nb1[e] = a.Bs.rowptr[rid + 1];
                }
            }
        }
        // (two packs of one row per lane when the slice allows, else one pack of two rows: the same
        // registers, half the index and address work per column)
        if (!has2) {
            // nothing reads the LDS tile
        } else if (FAST && G >= 2 && w % (2 * VV) == 0) {
            const int G2 = G / 2;
            const int gl2 = (int)threadIdx.x % G2;
            if (2 * VV * gl2 < w)
                fused_tail<T, VV, 1, 2>(a, d, SLDS ? sm.second : blk, tileD1, ldl, c0, gl2,
                                        (int)threadIdx.x / G2, (int)blockDim.x / G2);
        } else if (VV * gl < w) {
            fused_tail<T, VV, 2>(a, d, SLDS ? sm.second : blk, tileD1, ldl, c0, gl, grp, ngrp);
        }
        if (!has_next) break;
        {
            int32_t *ext = sm.bext + (par ^ 1) * sm.bext_stride;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const int i = (int)threadIdx.x + e * (int)blockDim.x;
                if (i < nd.n_rows) {
                    ext[2 * i] = nb0[e];
                    ext[2 * i + 1] = nb1[e] - nb0[e];
                }
            }
            // (a tile of more rows than that: the rest the plain way)
            for (int i = NE * (int)blockDim.x + (int)threadIdx.x; i < nd.n_rows; i += (int)blockDim.x) {
                const int64_t rid = row_id(next_first, i);
                const int kb = a.Bs.rowptr[rid];
                ext[2 * i] = kb;
                ext[2 * i + 1] = a.Bs.rowptr[rid + 1] - kb;
            }
        }
        __syncthreads();
        d = nd;
        tw.tile = ntile;
        par ^= 1;
    }
}

// Packed-row SpMM: Y[row][:] = sum over the row's packed entries of val * X[idx][:], one unit
// (and one column slice) per workgroup: the second wavefront, and the second operation of the
// unfused baseline.  X is the D1 workspace: n_xs column slices of sw columns, idx is a row (slot)
// of it.
//
// With one slice a workgroup handles whole rows.  With n_xs = 2, 4 or 8 slices, workgroup b (which
// the hardware places on XCD b % 8) handles slice (b % 8) % n_xs of unit (b / 8) (8 / n_xs) +
// (b % 8) / n_xs: an XCD only ever touches one slice of X, so its L2 holds sw-wide pieces of the
// hot rows instead of whole rows, and the eight caches hold different data.
//
// The entries of a unit are contiguous (n_rows x slots): the workgroup first copies them to LDS
// with coalesced 16-byte loads, then every lane group reads the entries of its rows from there
// (an LDS broadcast) instead of fetching each index and value through the vector memory path
// once per lane.  A lane group works on R rows at a time and keeps E entries of each in flight.
// Units whose rows are split hand their partial sums through LDS and add them in a fixed order.
template <typename T, bool FAST, bool WIDE, int R>
__global__ __launch_bounds__(kSpmmThreads) void k_packed_spmm(const PackedSpmmLaunch a) {
    constexpr int VV = FAST ? Tr<T>::V : 1;
    constexpr int E = R >= 4 ? 4 : 8;
    __shared__ __align__(16) int32_t idx_s[kUnitSlots + 4];
    __shared__ __align__(16) T val_s[kUnitSlots + 4];
    T *red = val_s;                                     // split units do not stage their entries
    int64_t u;
    int slice = 0;
    if (a.n_xs == 1) {
        u = a.contiguous ? xcd_contiguous(blockIdx.x, a.n_units) : (int64_t)blockIdx.x;
    } else {
        const int x = blockIdx.x % kXcds, per = kXcds / a.n_xs;
        slice = x % a.n_xs;
        u = (int64_t)(blockIdx.x / kXcds) * per + x / a.n_xs;
    }
    if (u >= a.n_units) return;
    const UnitDesc d = a.pack.units[u];
    const int ccol = a.ccol;
    const int c0 = slice * a.sw;
    const int w = min(a.sw, ccol - c0);                 // columns of this slice
    const int G = min(64, pow2_at_least((a.sw + VV - 1) / VV));
    const int gl = threadIdx.x % G, grp = threadIdx.x / G, ngrp = blockDim.x / G;
    const int32_t *__restrict__ rows = a.pack.rows;
    const int32_t *__restrict__ idx = static_cast<const int32_t *>(a.pack.idx);
    const T *__restrict__ val = static_cast<const T *>(a.pack.vals);
    const T *__restrict__ X = static_cast<const T *>(a.X) + (int64_t)slice * a.x_slice_stride;
    const uint32_t ldx = (uint32_t)a.sw;
    T *__restrict__ Y = static_cast<T *>(a.Y) + c0;
    if (d.split <= 1) {
        const int n_ent = d.n_rows * d.slots;
        {
            // unit bases are multiples of four entries; the copy may run up to three entries over
            const Piece *src_i = reinterpret_cast<const Piece *>(idx + d.entry_base);
            Piece *dst_i = reinterpret_cast<Piece *>(idx_s);
            for (int e = threadIdx.x; e < (n_ent + 3) / 4; e += blockDim.x) dst_i[e] = src_i[e];
            constexpr int PV = 16 / (int)sizeof(T);
            const Piece *src_v = reinterpret_cast<const Piece *>(val + d.entry_base);
            Piece *dst_v = reinterpret_cast<Piece *>(val_s);
            for (int e = threadIdx.x; e < (n_ent + PV - 1) / PV; e += blockDim.x) dst_v[e] = src_v[e];
        }
        int32_t rid[R];
        {
            // row ids of this group's first rows, on their way while the entries are copied
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int i = grp + r * ngrp;
                rid[r] = rows[d.row_begin + (i < d.n_rows ? i : 0)];
            }
        }
        __syncthreads();
        const int L = d.slots;
        for (int cb = 0; cb < w; cb += G * VV) {
            const int col = cb + VV * gl;
            const bool active = col < w;
            const uint32_t lane_off = active ? (uint32_t)col : 0u;      // idle lanes read column 0
            for (int i0 = grp; i0 < d.n_rows; i0 += ngrp * R) {
                int at[R];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int i = i0 + r * ngrp;
                    at[r] = (i < d.n_rows ? i : i0) * L;
                }
                if (i0 != grp || cb != 0) {
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const int i = i0 + r * ngrp;
                        rid[r] = rows[d.row_begin + (i < d.n_rows ? i : i0)];
                    }
                }
                T acc[R][VV];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int i = 0; i < VV; ++i) acc[r][i] = T(0);
                // E entries of each of the R rows per pass, from slot sl on.  The last pass of a row
                // may reach past the row's end: its surplus slots re-read the last entry (same
                // address: no extra traffic) with a zero value, so that the whole remainder is one
                // round trip to memory instead of one per entry (most rows of a graph are short).
                auto pass = [&](auto masked_c, int sl) {
                    constexpr bool MASKED = decltype(masked_c)::value;
                    uint32_t c[R][E];
                    T v[R][E];
                    T x[R][E][VV];
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            const bool in = !MASKED || sl + e < L;
                            const int at_e = at[r] + (in ? sl + e : L - 1);
                            c[r][e] = (uint32_t)idx_s[at_e];
                            v[r][e] = in ? val_s[at_e] : T(0);
                        }
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int e = 0; e < E; ++e) load_x<T, VV, WIDE>(x[r][e], X, c[r][e], ldx, lane_off);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            // (a surplus slot adds nothing, whatever the operand holds)
                            if (MASKED && sl + e >= L) continue;
#pragma unroll
                            for (int i = 0; i < VV; ++i) acc[r][i] += v[r][e] * x[r][e][i];
                        }
                };
                int sl = 0;
                for (; sl + E <= L; sl += E) pass(std::false_type(), sl);
                if (sl < L) pass(std::true_type(), sl);
                if (active) {
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        if (i0 + r * ngrp < d.n_rows)
                            store_pack<T, VV>(Y + (int64_t)rid[r] * ccol + col, acc[r]);
                }
            }
        }
        return;
    }
    for (int cb = 0; cb < w; cb += G * VV) {
        const int col = cb + VV * gl;
        const bool active = col < w;
        const uint32_t lane_off = active ? (uint32_t)col : 0u;      // idle lanes read column 0
        {
            // group -> (row, part); `split` groups share a row, each takes a range of the slots
            const int row_i = grp / d.split, part = grp % d.split;
            const int chunk = (d.slots + d.split - 1) / d.split;
            const int s0 = min(d.slots, part * chunk), s1 = min(d.slots, s0 + chunk);
            T acc[VV];
#pragma unroll
            for (int i = 0; i < VV; ++i) acc[i] = T(0);
            // The entries of the group's part travel through LDS as well, a window of 8 G slots at a
            // time: the G lanes fetch them with coalesced loads (one word per lane and load instead of
            // the same word for every lane), put them into the group's piece of the staging arrays,
            // and read them back as broadcasts, 8 per pass.  The next window's entries are in flight
            // while the current window is gathered.  A group is part of one wave and LDS operations
            // of a wave complete in order, so no workgroup barrier is involved.
            const int WS = 8 * G;
            int32_t *gi = idx_s + grp * WS;
            T *gv = val_s + grp * WS;
            const bool has_row = row_i < d.n_rows;
            const int64_t at = d.entry_base + (int64_t)(has_row ? row_i : 0) * d.slots;
            const int32_t *__restrict__ ip = idx + at;
            const T *__restrict__ vp = val + at;
            // Lane gl fetches the eight consecutive slots 8 gl .. 8 gl + 7 of a window (one address,
            // eight immediate offsets).  A window may reach past the end of the part, of the row and,
            // for the last row of the list, of the packed arrays, which therefore end with
            // kPackSpareSlots zero entries: whatever index is read there names a valid row, and
            // slots past the part's end are left out of the sum.
            int32_t ci[8];
            T vi[8];
            const int32_t *__restrict__ ipl = ip + 8 * gl;
            const T *__restrict__ vpl = vp + 8 * gl;
            auto fetch_window = [&](int w0) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    ci[k] = ipl[w0 + k];
                    vi[k] = vpl[w0 + k];
                }
            };
            if (has_row && s0 < s1) {
                fetch_window(s0);
                for (int w0 = s0; w0 < s1; w0 += WS) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        gi[8 * gl + k] = ci[k];
                        gv[8 * gl + k] = vi[k];
                    }
                    if (w0 + WS < s1) fetch_window(w0 + WS);
                    __builtin_amdgcn_wave_barrier();
                    asm volatile("" ::: "memory");
                    const int n_here = min(WS, s1 - w0);
                    for (int p0 = 0; p0 < n_here; p0 += 8) {
                        uint32_t c[8];
                        T v[8];
                        T x[8][VV];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            c[e] = (uint32_t)gi[p0 + e];
                            v[e] = gv[p0 + e];
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) load_x<T, VV, WIDE>(x[e], X, c[e], ldx, lane_off);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            if (p0 + e >= n_here) continue;      // (a surplus slot adds nothing)
#pragma unroll
                            for (int i = 0; i < VV; ++i) acc[i] += v[e] * x[e][i];
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                    asm volatile("" ::: "memory");
                }
            }
            __syncthreads();          // the staging arrays become the partial sums
#pragma unroll
            for (int i = 0; i < VV; ++i) red[(grp * G + gl) * VV + i] = acc[i];
            __syncthreads();
            if (part == 0 && row_i < d.n_rows && active) {
                T sum[VV];
#pragma unroll
                for (int i = 0; i < VV; ++i) sum[i] = T(0);
                for (int pp = 0; pp < d.split; ++pp)
#pragma unroll
                    for (int i = 0; i < VV; ++i) sum[i] += red[((grp + pp) * G + gl) * VV + i];
                store_pack<T, VV>(Y + (int64_t)rows[d.row_begin + row_i] * ccol + col, sum);
            }
            __syncthreads();
        }
    }
}

// CSR SpMM over a caller-supplied matrix: Y[j][:] = sum_k S.vals[k] X[S.colidx[k]][:], consecutive
// rows per workgroup.  The first operation of the unfused SpMM-SpMM baseline (row_info = nullptr:
// every row goes to the workspace, slot = row), and the first wavefront of a CSR-B plan that needs
// no tile in LDS (row_info set, see k_gemm).
template <typename T, bool FAST>
__global__ __launch_bounds__(kSpmmThreads) void k_csr_spmm(const CsrSpmmLaunch a) {
    constexpr int VV = FAST ? Tr<T>::V : 1;
    const int64_t n_wg = (a.n_rows + a.rows_per_wg - 1) / a.rows_per_wg;
    const int64_t u = xcd_contiguous(blockIdx.x, n_wg);
    if (u >= n_wg) return;
    const int64_t r0 = u * a.rows_per_wg;
    const int64_t r1 = r0 + a.rows_per_wg < a.n_rows ? r0 + a.rows_per_wg : a.n_rows;
    const int ccol = a.ccol;
    const int G = min(64, pow2_at_least((ccol + VV - 1) / VV));
    const int gl = threadIdx.x % G, grp = threadIdx.x / G, ngrp = blockDim.x / G;
    const T *__restrict__ vals = static_cast<const T *>(a.S.vals);
    const T *__restrict__ X = static_cast<const T *>(a.X);
    T *__restrict__ Y = static_cast<T *>(a.Y);
    // the rows of the workgroup are staged once (see stage_extents), then gathered per column block
    __shared__ __align__(16) int32_t ext_s[2 * kCsrRowsPerWg];
    __shared__ __align__(16) int32_t idx_s[kSparseEntryCap * kCsrRowsPerWg];
    __shared__ __align__(16) T val_s[kSparseEntryCap * kCsrRowsPerWg];
    const int rows = (int)(r1 - r0);
    if (!a.row_info) {
        stage_extents(rows, ext_s, a.S.rowptr, [&](int i) { return r0 + i; });
    } else {
        // a row whose D1 row nobody reads and that the plan leaves out counts as empty here: nothing
        // of it is fetched (its gathers name row 0 of X with a zero value)
        for (int i = threadIdx.x; i < rows; i += (int)blockDim.x) {
            const int64_t rid = r0 + i;
            const int kb = a.S.rowptr[rid], ke = a.S.rowptr[rid + 1];
            ext_s[2 * i] = kb;
            ext_s[2 * i + 1] = (a.row_info[rid] & kInfoSkip) ? 0 : ke - kb;
        }
    }
    __syncthreads();
    stage_entries<T>(rows, ext_s, idx_s, val_s, a.S.colidx, vals);
    for (int cb = 0; cb < ccol; cb += G * VV) {
        const int col = cb + VV * gl;
        // the lane's columns of a row of the workspace (slices of y_sw columns)
        T *Yl = Y + (int64_t)(col >> a.y_sw_shift) * a.y_slice_stride + (col & a.y_sw_mask);
        if (!a.row_info) {
            gather_staged_rows<T, VV, 2>(rows, ext_s, idx_s, val_s, a.S.colidx, vals, X + col, ccol,
                                         col < ccol, grp, ngrp, [](int) { return 0; },
                                         [&](int pos, int, const T(&acc)[VV]) {
                                             store_pack<T, VV>(Yl + (r0 + pos) * a.y_sw, acc);
                                         });
        } else {
            // first wavefront of a plan without an LDS tile: what happens to a finished D1 row is
            // told by its info word (see k_gemm)
            struct RowInfo {
                uint32_t info;
                T sc;
            };
            const T *scale = static_cast<const T *>(a.row_scale);
            T *Dl = static_cast<T *>(a.D) + col;
            gather_staged_rows<T, VV, 2>(
                rows, ext_s, idx_s, val_s, a.S.colidx, vals, X + col, ccol, col < ccol, grp, ngrp,
                [&](int pos) { return RowInfo{a.row_info[r0 + pos], scale ? scale[r0 + pos] : T(0)}; },
                [&](int pos, const RowInfo &ri, const T(&acc)[VV]) {
                    if (ri.info & kInfoSpill)
                        store_pack<T, VV>(Yl + (int64_t)(ri.info & kInfoSlotMask) * a.y_sw, acc);
                    if (ri.info & (kInfoDirect | kInfoZero)) {
                        T x[VV];
#pragma unroll
                        for (int i = 0; i < VV; ++i) x[i] = (ri.info & kInfoZero) ? T(0) : ri.sc * acc[i];
                        store_pack<T, VV>(Dl + (r0 + pos) * ccol, x);
                    }
                });
        }
    }
}

// D1 = B C for all rows, one 16-row block per wave at a time, the next block's rows of B in
// flight while the current one is multiplied (KS > 0, as above).
// INFO = false: the GeMM of the unfused baseline; every row goes to the workspace, slot = row.
// INFO = true: the first wavefront of a plan none of whose fused rows reads the LDS tile (a graph:
// the only rows that fuse hold just a diagonal entry, or nothing).  Then no tile has to sit in LDS
// and the workgroups stream through the rows like the plain product; what happens to a finished
// D1 row is told by its info word (kInfo*): stored to its workspace slot when the second wavefront
// reads it, stored to D times the diagonal entry (or as zeros) when the row of D is fused.
template <typename T, int NB, int KS, bool FAST, bool INFO>
__global__ __launch_bounds__(kFusedThreads) void k_gemm(const GemmLaunch a) {
    const int slice = blockIdx.y;
    const int c0 = slice * a.cs;
    const int w = min(a.cs, a.ccol - c0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int g = lane >> 4, r = lane & 15;
    T *Cl = reinterpret_cast<T *>(tf_smem);
    stage_c_slice<T, NB>(Cl, static_cast<const T *>(a.C), a.bcol, a.c_ldk, a.c_ldc, c0,
                         w);
    __syncthreads();
    const int64_t nblk = (a.n + 15) >> 4;
    const T *__restrict__ B = static_cast<const T *>(a.B);
    T *__restrict__ D1 = static_cast<T *>(a.D1);
    // contiguous range of row blocks per workgroup, waves interleaved inside it
    const int64_t per_wg = (nblk + gridDim.x - 1) / gridDim.x;
    const int64_t lb0 = (int64_t)blockIdx.x * per_wg;
    const int64_t lb1 = lb0 + per_wg < nblk ? lb0 + per_wg : nblk;
    struct RowInfo {
        uint32_t info;
        T sc;
    };
    // (fetched before the multiplications of the block, used after them)
    auto row_info = [&](int64_t lb) -> RowInfo {
        RowInfo ri{0u, T(0)};
        if constexpr (INFO) {
            const int64_t row = lb * 16 + r;
            const int64_t rc = row < a.n ? row : a.n - 1;
            ri.info = row < a.n ? a.row_info[rc] : 0u;
            if (a.row_scale) ri.sc = static_cast<const T *>(a.row_scale)[rc];
        }
        return ri;
    };
    auto write_block = [&](int64_t lb, const RowInfo &ri, typename Tr<T>::Acc(&acc)[NB]) {
        const int64_t row = lb * 16 + r;
        if (row >= a.n) return;
        if constexpr (!INFO) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int col = 16 * nb + 4 * g;
                const int cb = c0 + 16 * nb;        // the workspace is cut into slices of d1_sw columns
                store_acc4<T, FAST>(D1 + (int64_t)(cb >> a.d1_sw_shift) * a.d1_slice_stride +
                                        row * a.d1_sw + (cb & a.d1_sw_mask) + 4 * g,
                                    acc[nb], col, w);
            }
        } else {
            if (ri.info & kInfoSpill) {
                const int64_t slot = (int64_t)(ri.info & kInfoSlotMask);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int col = 16 * nb + 4 * g;
                    const int cb = c0 + 16 * nb;
                    store_acc4<T, FAST>(D1 + (int64_t)(cb >> a.d1_sw_shift) * a.d1_slice_stride +
                                            slot * a.d1_sw + (cb & a.d1_sw_mask) + 4 * g,
                                        acc[nb], col, w);
                }
            }
            if (ri.info & (kInfoDirect | kInfoZero)) {
                T *dst = static_cast<T *>(a.D) + row * a.ccol + c0 + 4 * g;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    typename Tr<T>::Acc x;
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[i] = (ri.info & kInfoZero) ? T(0) : ri.sc * acc[nb][i];
                    store_acc4<T, FAST>(dst + 16 * nb, x, 16 * nb + 4 * g, w);
                }
            }
        }
    };
    if constexpr (KS > 0) {
        constexpr int KSF = KS;
        BFrag<T, KSF> cur, nxt;
        int64_t lb = lb0 + wave;
        {
            const int64_t row = lb * 16 + r;
            load_b_frag<T, KSF>(cur, B + (row < a.n ? row : a.n - 1) * a.bcol, g);
        }
        for (; lb < lb1; lb += nwaves) {
            // The C slice is loop invariant; keeping all of it in registers only pays while it
            // is small, so for larger slices the LDS reads are pinned inside the loop.
            if constexpr (KSF * Tr<T>::V * NB * (sizeof(T) / 4) > 64) asm volatile("" ::: "memory");
            const int64_t nrow = (lb + nwaves) * 16 + r;
            load_b_frag<T, KSF>(nxt, B + (nrow < a.n ? nrow : a.n - 1) * a.bcol, g);
            const RowInfo ri = row_info(lb);
            __builtin_amdgcn_sched_barrier(0);      // keep the prefetch ahead of the MFMAs
            typename Tr<T>::Acc acc[NB];
            mfma_frag<T, NB, KSF>(acc, Cl, cur, lane);
            write_block(lb, ri, acc);
            cur = nxt;
        }
    } else {
        for (int64_t lb = lb0 + wave; lb < lb1; lb += nwaves) {
            const int64_t row = lb * 16 + r;
            const bool valid = row < a.n;
            const RowInfo ri = row_info(lb);
            typename Tr<T>::Acc acc[NB];
            mfma_row_block<T, NB, FAST>(acc, Cl, B + (valid ? row : 0) * a.bcol, valid, a.bcol, lane);
            write_block(lb, ri, acc);
        }
    }
}

// ------------------------------------------------------------------------------------------ host

template <typename K> int raise_lds_limit(K kernel, int64_t bytes) {
    return (int)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// Workgroups of a fused kernel that one compute unit holds at once (registers and LDS), 1..4.
template <typename K> int resident_per_cu(K kernel, int threads, int64_t lds_bytes) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, reinterpret_cast<const void *>(kernel),
                                                     threads, (size_t)lds_bytes) != hipSuccess)
        nb = 1;
    return nb < 1 ? 1 : (nb > 4 ? 4 : nb);
}

// Launch shape of a fused kernel: the number of waves per compute unit stays the same whatever
// the tile size.  When the tiles are small enough for the LDS of two workgroups (or more), the
// kernel runs with half-size workgroups, as many to a compute unit as fit, so that small tiles
// do not leave half of the waves of a large workgroup without a 16-row block or a row to work on.
// (Measured on config 2: two half-size workgroups on half-size tiles are as fast as one full one;
// their phases do not overlap usefully because fp32 MFMA and vector ALU work of one SIMD serialise.)
struct FusedShape {
    int threads = kFusedThreads, wg_per_cu = 1;
};
template <typename K> FusedShape fused_shape(K kernel, int64_t lds_bytes, int max_threads) {
    FusedShape s;
    s.threads = max_threads;
    if (resident_per_cu(kernel, max_threads / 2, lds_bytes) >= 2) s.threads = max_threads / 2;
    s.wg_per_cu = resident_per_cu(kernel, s.threads, lds_bytes);
    return s;
}

// Persistent workgroups of the fused kernels: as many per XCD as its CUs (an eighth of the
// device's) hold at once (one or more per CU, by LDS and registers), a multiple of the number of
// slices, no more than there are (tile, slice) pairs.
int64_t fused_grid(const FusedLaunch &a, int wg_per_cu) {
    const int64_t per = (a.n_tiles + kXcds - 1) / kXcds;
    const int64_t cu_per_xcd = std::max(1, a.n_cu / kXcds);
    int64_t wg_per_xcd = std::min<int64_t>(per * a.n_slices, cu_per_xcd * (int64_t)wg_per_cu);
    wg_per_xcd = std::max<int64_t>(a.n_slices, wg_per_xcd / a.n_slices * a.n_slices);
    return kXcds * wg_per_xcd;
}

// Per kernel instantiation: the dynamic-LDS limit raised so far (it only ever grows: lowering it
// would break a launch of another plan) and the launch shape last worked out.  Calls may come
// from several host threads, so both sit behind a mutex.
struct KernelSetup {
    std::mutex m;
    int64_t raised = -1, occ_lds = -1;
    FusedShape shape;
};
template <typename K>
int fused_setup(KernelSetup &ks, K kernel, int64_t lds_bytes, int max_threads, FusedShape &shape) {
    std::lock_guard<std::mutex> lock(ks.m);
    if (lds_bytes > ks.raised) {
        const int e = raise_lds_limit(kernel, lds_bytes);
        if (e) return e;
        ks.raised = lds_bytes;
    }
    if (lds_bytes != ks.occ_lds) {
        ks.shape = fused_shape(kernel, lds_bytes, max_threads);
        ks.occ_lds = lds_bytes;
    }
    shape = ks.shape;
    return 0;
}

template <typename T, int NB, int KS, bool FAST, bool SLDS>
int run_fused_gemm2(const FusedLaunch &a, hipStream_t st) {
    static KernelSetup ks;
    FusedShape shape;
    if (int e = fused_setup(ks, k_fused_gemm_spmm<T, NB, KS, FAST, SLDS>, a.lds_bytes, kFusedThreads, shape))
        return e;
    (void)hipGetLastError();      // an error left by an earlier, unrelated call is not this launch's
    k_fused_gemm_spmm<T, NB, KS, FAST, SLDS>
        <<<dim3((unsigned)fused_grid(a, shape.wg_per_cu)), dim3(shape.threads), a.lds_bytes, st>>>(a);
    return (int)hipGetLastError();
}
template <typename T, int NB, int KS, bool FAST>
int run_fused_gemm(const FusedLaunch &a, hipStream_t st) {
    return a.s_in_lds ? run_fused_gemm2<T, NB, KS, FAST, true>(a, st)
                      : run_fused_gemm2<T, NB, KS, FAST, false>(a, st);
}

template <typename T, bool FAST, bool SLDS> int run_fused_spmm2(const FusedLaunch &a, hipStream_t st) {
    static KernelSetup ks;
    FusedShape shape;
    if (int e = fused_setup(ks, k_fused_spmm_spmm<T, FAST, SLDS>, a.lds_bytes, kFusedSparseThreads, shape))
        return e;
    (void)hipGetLastError();
    k_fused_spmm_spmm<T, FAST, SLDS>
        <<<dim3((unsigned)fused_grid(a, shape.wg_per_cu)), dim3(shape.threads), a.lds_bytes, st>>>(a);
    return (int)hipGetLastError();
}
template <typename T, bool FAST> int run_fused_spmm(const FusedLaunch &a, hipStream_t st) {
    return a.s_in_lds ? run_fused_spmm2<T, FAST, true>(a, st) : run_fused_spmm2<T, FAST, false>(a, st);
}

template <typename T, int NB, int KS, bool FAST, bool INFO>
int run_gemm2(const GemmLaunch &a, hipStream_t st) {
    const int64_t lds = lds_fixed_bytes(a.dtype, 0, a.bcol, a.cs);
    static std::mutex m;
    static int64_t raised = -1;
    {
        std::lock_guard<std::mutex> lock(m);
        if (lds > raised) {
            const int e = raise_lds_limit(k_gemm<T, NB, KS, FAST, INFO>, lds);
            if (e) return e;
            raised = lds;
        }
    }
    const int nwaves = kFusedThreads / 64;
    const int64_t nblk = (a.n + 15) / 16;
    int64_t gx = (nblk + nwaves - 1) / nwaves;
    gx = gx < 1 ? 1 : (gx > 1024 ? 1024 : gx);
    (void)hipGetLastError();
    k_gemm<T, NB, KS, FAST, INFO>
        <<<dim3((unsigned)gx, (unsigned)a.n_slices), dim3(kFusedThreads), lds, st>>>(a);
    return (int)hipGetLastError();
}
template <typename T, int NB, int KS, bool FAST> int run_gemm(const GemmLaunch &a, hipStream_t st) {
    return a.row_info ? run_gemm2<T, NB, KS, FAST, true>(a, st) : run_gemm2<T, NB, KS, FAST, false>(a, st);
}

// Calls f(NB, KS) with compile-time constants: NB accumulator blocks for the slice width, and
// KS = bCol / (4 V) when that is one of the specialised depths, else 0 (generic k loop).
template <typename L> int dispatch_shape(int dtype, int cs, int bcol, bool fast, L &&f) {
    const int kc = 4 * vec_elems(dtype);
    int ks = (fast && bcol % kc == 0) ? bcol / kc : 0;
    if (ks != 2 && ks != 4 && ks != 8 && ks != 16) ks = 0;
#define TF_KS(NBV)                                                                        \
    switch (ks) {                                                                         \
        case 2: return f(std::integral_constant<int, NBV>(), std::integral_constant<int, 2>());   \
        case 4: return f(std::integral_constant<int, NBV>(), std::integral_constant<int, 4>());   \
        case 8: return f(std::integral_constant<int, NBV>(), std::integral_constant<int, 8>());   \
        case 16: return f(std::integral_constant<int, NBV>(), std::integral_constant<int, 16>()); \
        default: return f(std::integral_constant<int, NBV>(), std::integral_constant<int, 0>());  \
    }
    switch (mfma_blocks(cs)) {
        case 1: TF_KS(1)
        case 2: TF_KS(2)
        case 4: TF_KS(4)
        case 8: TF_KS(8)
    }
#undef TF_KS
    return (int)hipErrorInvalidValue;
}

template <typename L> int dispatch_nb(int cs, L &&f) {
    switch (mfma_blocks(cs)) {
        case 1: return f(std::integral_constant<int, 1>());
        case 2: return f(std::integral_constant<int, 2>());
        case 4: return f(std::integral_constant<int, 4>());
        case 8: return f(std::integral_constant<int, 8>());
    }
    return (int)hipErrorInvalidValue;
}

bool gemm_fast(int dtype, int bcol, int ccol, int cs) {
    const int v = vec_elems(dtype);
    return bcol % v == 0 && ccol % v == 0 && (cs % v == 0);
}
bool spmm_fast(int dtype, int ccol, int cs) {
    const int v = vec_elems(dtype);
    return ccol % v == 0 && cs % v == 0;
}

}  // namespace

int launch_fused_gemm_spmm(const FusedLaunch &a, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n_tiles == 0) return 0;
    const bool fast = gemm_fast(a.dtype, a.bcol, a.ccol, a.cs);
    if (!fast) {
        return dispatch_nb(a.cs, [&](auto nb) {
            constexpr int NB = decltype(nb)::value;
            return a.dtype == TF_F32 ? run_fused_gemm<float, NB, 0, false>(a, st)
                                     : run_fused_gemm<double, NB, 0, false>(a, st);
        });
    }
    return dispatch_shape(a.dtype, a.cs, a.bcol, fast, [&](auto nb, auto ks) {
        constexpr int NB = decltype(nb)::value, KS = decltype(ks)::value;
        return a.dtype == TF_F32 ? run_fused_gemm<float, NB, KS, true>(a, st)
                                 : run_fused_gemm<double, NB, KS, true>(a, st);
    });
}

int launch_fused_spmm_spmm(const FusedLaunch &a, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n_tiles == 0) return 0;
    const bool fast = spmm_fast(a.dtype, a.ccol, a.cs);
    if (a.dtype == TF_F32)
        return fast ? run_fused_spmm<float, true>(a, st) : run_fused_spmm<float, false>(a, st);
    return fast ? run_fused_spmm<double, true>(a, st) : run_fused_spmm<double, false>(a, st);
}

int launch_packed_spmm(const PackedSpmmLaunch &a, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n_units == 0) return 0;
    if (a.n_xs != 1 && a.n_xs != 2 && a.n_xs != 4 && a.n_xs != 8) return (int)hipErrorInvalidValue;
    const bool fast = spmm_fast(a.dtype, a.ccol, a.sw);
    // one workgroup per unit and slice; with slices, 8 / n_xs units per round of eight workgroups
    const int64_t rounds = (a.n_units * a.n_xs + kXcds - 1) / kXcds;
    const dim3 grid((unsigned)(rounds * kXcds)), block(kSpmmThreads);
    (void)hipGetLastError();
#define TF_GO2(T, W)                                                                     \
    do {                                                                                 \
        if (!fast) k_packed_spmm<T, false, W, 4><<<grid, block, 0, st>>>(a);             \
        else if (a.rows_per_pass == 1) k_packed_spmm<T, true, W, 1><<<grid, block, 0, st>>>(a); \
        else if (a.rows_per_pass == 2) k_packed_spmm<T, true, W, 2><<<grid, block, 0, st>>>(a); \
        else k_packed_spmm<T, true, W, 4><<<grid, block, 0, st>>>(a);                    \
    } while (0)
#define TF_GO(T)                                                                         \
    do {                                                                                 \
        if (a.wide) TF_GO2(T, true); else TF_GO2(T, false);                              \
    } while (0)
    if (a.dtype == TF_F32) TF_GO(float); else TF_GO(double);
#undef TF_GO
#undef TF_GO2
    return (int)hipGetLastError();
}

int launch_csr_spmm(const CsrSpmmLaunch &a, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n_rows == 0) return 0;
    // the kernel stages the rows of a workgroup in LDS arrays of this many rows
    if (a.rows_per_wg < 1 || a.rows_per_wg > kCsrRowsPerWg) return (int)hipErrorInvalidValue;
    const bool fast = spmm_fast(a.dtype, a.ccol, a.ccol);
    const int64_t n_wg = (a.n_rows + a.rows_per_wg - 1) / a.rows_per_wg;
    const dim3 grid((unsigned)((n_wg + kXcds - 1) / kXcds * kXcds)), block(kSpmmThreads);
    (void)hipGetLastError();
    if (a.dtype == TF_F32) {
        if (fast) k_csr_spmm<float, true><<<grid, block, 0, st>>>(a);
        else k_csr_spmm<float, false><<<grid, block, 0, st>>>(a);
    } else {
        if (fast) k_csr_spmm<double, true><<<grid, block, 0, st>>>(a);
        else k_csr_spmm<double, false><<<grid, block, 0, st>>>(a);
    }
    return (int)hipGetLastError();
}

int launch_gemm(const GemmLaunch &a, void *stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (a.n == 0) return 0;
    const bool fast = gemm_fast(a.dtype, a.bcol, a.ccol, a.cs);
    if (!fast) {
        return dispatch_nb(a.cs, [&](auto nb) {
            constexpr int NB = decltype(nb)::value;
            return a.dtype == TF_F32 ? run_gemm<float, NB, 0, false>(a, st)
                                     : run_gemm<double, NB, 0, false>(a, st);
        });
    }
    return dispatch_shape(a.dtype, a.cs, a.bcol, fast, [&](auto nb, auto ks) {
        constexpr int NB = decltype(nb)::value, KS = decltype(ks)::value;
        return a.dtype == TF_F32 ? run_gemm<float, NB, KS, true>(a, st)
                                 : run_gemm<double, NB, KS, true>(a, st);
    });
}

}  // namespace tf
