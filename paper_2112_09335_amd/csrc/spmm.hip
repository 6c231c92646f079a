// Community-blocked sparse aggregation  Y = A~ X  on gfx950 (paper, Section 2, Problem 3: row block m
// is A~_{m,m} X_m + sum_{r in N_m} A~_{m,r} X_r; Appendix A: the same sum restricted to one
// neighbour community per output row, the "segments").
//
// Layout: a row list (the CSR rows, or the (row, community) segments with several entries) laid out by the host
// for this kernel: rows grouped into length classes, the longest class first and community-contiguous inside a
// class, with a copy of the column indices and values in that order and the output row of every list row.
// Features are row-major fp32.
//
// Mapping: a group of LPR lanes (a power of two, up to the 64-lane wavefront) reads one gathered
// neighbour row with one fully coalesced VEC*4-byte load per lane and keeps VEC*R accumulators per lane.
// GPR such groups share one output row and take its entries round-robin, eight (or four) entries in flight per
// group; their partial sums are added by a wavefront-level xor-shuffle reduction.  GPR is chosen per length
// class so that one trip of the entry loop covers the class's longest row: short rows pack many rows into a
// wavefront, long rows spread over it, and the rows of a wavefront need the same number of trips.
// Rows beyond a length threshold (power-law hubs) are cut into parts that run first in the same launch, into a
// side buffer; a small kernel adds a row's parts in order.  Segments with a single entry are scaled copies of a
// gathered row and have a kernel of their own.  Everything is order-fixed: no atomics, results are reproducible.
// The bound is the L2 / fabric traffic of the gathers.  Inside a class XCD k (blockIdx mod 8) walks the k-th
// contiguous eighth of the rows (a few communities), so that the rows it gathers stay in its L2.
#include "kernels.h"

namespace cadmm {

namespace {

template <int VEC> struct VecT;
template <> struct VecT<4> { using type = float4; };
template <> struct VecT<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void load_vec(float (&dst)[VEC], const float* p) {
    if constexpr (VEC == 4) {
        float4 v = *reinterpret_cast<const float4*>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else {
        dst[0] = *p;
    }
}

typedef float float_x4 __attribute__((ext_vector_type(4)));

// results are written once and read by a later kernel: streamed past the L2's resident lines
template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&src)[VEC]) {
    if constexpr (VEC == 4) {
        float_x4 v = {src[0], src[1], src[2], src[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<float_x4*>(p));
    } else {
        __builtin_nontemporal_store(src[0], p);
    }
}

// Which rows a workgroup takes: class j covers the rows [row_start[j], row_start[j+1]) with 2^g[j] lane groups per
// row, in the workgroups [block_start[j], block_start[j+1]) after those of the parts.
struct ClassMap {
    int n;
    int part_g;
    int g[kSpmmClasses];
    long long row_start[kSpmmClasses + 1];
    long long block_start[kSpmmClasses + 1];
};

template <int VEC, int R, int EPI, int U>
__global__ __launch_bounds__(256) void spmm_rows_kernel(
    const int64_t* __restrict__ lo, const int64_t* __restrict__ hi, const int64_t* __restrict__ part_lo,
    const int64_t* __restrict__ part_hi, int64_t nrows, int64_t nparts, const int32_t* __restrict__ col,
    const float* __restrict__ val, const float* __restrict__ X, float* __restrict__ Y, float* __restrict__ side,
    int width, int lpr_log2, ClassMap cm, int col0, int col1, int max_len, int xcd_remap,
    const float* __restrict__ Zl, const float* __restrict__ Tl, float nu, const int32_t* __restrict__ out_index,
    int64_t part_blocks) {
    // The first part_blocks workgroups (a multiple of 8) take the parts of split rows, the longest pieces of work,
    // so that they do not form the tail of the launch; then come the workgroups of each length class in turn (each
    // count a multiple of 8).  Optional XCD-aware renumbering inside a class: XCD k (blockIdx mod 8) walks the
    // k-th contiguous eighth of its rows.
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int gpr_log2;
    int64_t vrow;
    if ((int64_t)blockIdx.x < part_blocks) {
        gpr_log2 = cm.part_g;
        const int span_log2 = lpr_log2 + gpr_log2;      // lanes that share one output row
        vrow = (((int64_t)blockIdx.x * 4 + wave) << (6 - span_log2)) + (lane >> span_log2);
        if (vrow >= nparts) return;
        vrow += nrows;
    } else {
        const int64_t b = (int64_t)blockIdx.x - part_blocks;
        int j = 0;
        while (j + 1 < cm.n && b >= cm.block_start[j + 1]) ++j;
        gpr_log2 = cm.g[j];
        const int span_log2 = lpr_log2 + gpr_log2;
        int64_t lb = b - cm.block_start[j];
        if (xcd_remap) lb = (lb & 7) * ((cm.block_start[j + 1] - cm.block_start[j]) >> 3) + (lb >> 3);
        vrow = cm.row_start[j] + (((lb * 4 + wave) << (6 - span_log2)) + (lane >> span_log2));
        if (vrow >= cm.row_start[j + 1]) return;        // uniform over the row's lane span
    }
    const int lpr = 1 << lpr_log2;
    const int gpr = 1 << gpr_log2;
    const int grp = (lane >> lpr_log2) & (gpr - 1);
    const int sub = lane & (lpr - 1);
    const int cbase = col0 + sub * VEC;                 // first column of repeat 0
    const int cstride = lpr * VEC;                      // columns between repeats

    int64_t p, e;
    float* dst;
    bool is_part = vrow >= nrows;
    if (!is_part) {
        p = lo[vrow];
        e = hi[vrow];
        if (max_len > 0 && e - p > max_len) return;     // split row: the first workgroups take its parts
        dst = Y + (out_index ? (int64_t)out_index[vrow] : vrow) * (int64_t)width;
    } else {
        p = part_lo[vrow - nrows];
        e = part_hi[vrow - nrows];
        dst = side + (vrow - nrows) * (int64_t)width;
    }

    float acc[R][VEC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[r][v] = 0.f;

    // the groups of a row take entries p+grp, p+grp+gpr, ...; U of them in flight per group.  Every load is
    // unconditional: a slot past the end of the row reads the row's last entry again with weight zero, and a lane
    // past the last column reads the last columns again without storing them.  (Loads under a branch would make
    // the compiler wait for each gather before it issues the next.)
    int ccl[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int cc = cbase + r * cstride;
        ccl[r] = cc < col1 ? cc : col1 - VEC;
    }
    for (int64_t q = p + grp; q < e; q += U * gpr) {
        int32_t c[U];
        float a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t qu = q + u * gpr;
            const bool ok = qu < e;
            const int64_t qc = ok ? qu : e - 1;
            c[u] = col[qc];
            const float av = val[qc];
            a[u] = ok ? av : 0.f;
        }
        float x[U][R][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r) load_vec<VEC>(x[u][r], X + (int64_t)c[u] * width + ccl[r]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[r][v] = fmaf(a[u], x[u][r][v], acc[r][v]);
    }
    // wavefront-level reduction across the groups of the row
    for (int off = lpr; off < (lpr << gpr_log2); off <<= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[r][v] += __shfl_xor(acc[r][v], off, 64);
    }
    if (grp != 0) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int cc = cbase + r * cstride;
        if (cc < col1) {
            if constexpr (EPI == 1) {
                if (!is_part) {
                    const int64_t o = (out_index ? (int64_t)out_index[vrow] : vrow) * (int64_t)width + cc;
                    float z[VEC], t[VEC];
                    load_vec<VEC>(z, Zl + o);
                    load_vec<VEC>(t, Tl + o);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[r][v] = nu * (z[v] - fmaxf(t[v], 0.f)) + acc[r][v];
                }
            }
            store_vec<VEC>(dst + cc, acc[r]);
        }
    }
}

// Output rows with a single entry (most (row, neighbour community) segments of a sparse graph): row pos[k] of Y is
// val[k] times row col[k] of X.  A lane group takes kSingleBatch consecutive k, so that their index loads, their
// gathers and their stores are in flight together; the lists are read front to back.
constexpr int kSingleBatch = 4;
template <int VEC>
__global__ __launch_bounds__(256) void spmm_single_kernel(const int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ col,
                                                          const float* __restrict__ val, const float* __restrict__ X,
                                                          float* __restrict__ Y, int64_t n, int width, int lpr_log2) {
    const int lpr = 1 << lpr_log2;
    const int sub = threadIdx.x & (lpr - 1);
    const int64_t group = (int64_t)blockIdx.x * (256 >> lpr_log2) + (threadIdx.x >> lpr_log2);
    const int64_t k0 = group * kSingleBatch;
    if (k0 >= n) return;
    int32_t o[kSingleBatch], c[kSingleBatch];
    float a[kSingleBatch];
#pragma unroll
    for (int j = 0; j < kSingleBatch; ++j) {
        const int64_t k = k0 + j < n ? k0 + j : n - 1;
        o[j] = pos[k];
        c[j] = col[k];
        a[j] = val[k];
    }
    for (int cc = sub * VEC; cc < width; cc += lpr * VEC) {
        float x[kSingleBatch][VEC];
#pragma unroll
        for (int j = 0; j < kSingleBatch; ++j) load_vec<VEC>(x[j], X + (int64_t)c[j] * width + cc);
#pragma unroll
        for (int j = 0; j < kSingleBatch; ++j) {
            if (k0 + j >= n) break;
#pragma unroll
            for (int v = 0; v < VEC; ++v) x[j][v] *= a[j];
            store_vec<VEC>(Y + (int64_t)o[j] * width + cc, x[j]);
        }
    }
}

int g_tile_cols = 0;
int g_xcd_remap = 1;
int g_gpr_log2 = -1;      // -1: chosen from the mean row length
int g_unroll = 8;

// Adds the parts of every split row and applies the epilogue.  One wavefront per row: 2^lpr_log2 lanes cover the
// columns of the tile; where that leaves lanes over, the 64 >> lpr_log2 lane groups take the parts round-robin and
// their sums are added by xor-shuffles, so that a hub with a hundred parts is not one chain of dependent loads.
// The order of the additions is fixed by the part count alone.
template <int VEC, int EPI>
__global__ __launch_bounds__(64) void spmm_combine_kernel(const float* __restrict__ side,
                                                          const int32_t* __restrict__ long_row,
                                                          const int32_t* __restrict__ long_part_ptr, int64_t n_long,
                                                          float* __restrict__ Y, int width, int col0, int col1,
                                                          const float* __restrict__ Zl, const float* __restrict__ Tl,
                                                          float nu, int lpr_log2) {
    const int64_t i = blockIdx.x;
    if (i >= n_long) return;
    const int64_t row = long_row[i];
    const int p0 = long_part_ptr[i], p1 = long_part_ptr[i + 1];
    const int lpr = 1 << lpr_log2, groups = 64 >> lpr_log2;
    const int sub = threadIdx.x & (lpr - 1), grp = threadIdx.x >> lpr_log2;
    for (int cb = col0; cb < col1; cb += lpr * VEC) {           // same trip count in every lane
        const int c = cb + sub * VEC;
        const bool ok = c < col1;
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        if (ok) {
            for (int p = p0 + grp; p < p1; p += groups) {
                float x[VEC];
                load_vec<VEC>(x, side + (int64_t)p * width + c);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] += x[v];
            }
        }
        for (int off = lpr; off < 64; off <<= 1) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
        }
        if (!ok || grp != 0) continue;
        const int64_t o = row * (int64_t)width + c;
        if constexpr (EPI == 1) {
            float z[VEC], t[VEC];
            load_vec<VEC>(z, Zl + o);
            load_vec<VEC>(t, Tl + o);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = nu * (z[v] - fmaxf(t[v], 0.f)) + acc[v];
        }
        store_vec<VEC>(Y + o, acc);
    }
}

template <int VEC, int R>
void launch_cfg(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                const float* X, float* Y, int64_t nrows, int width, int lpr_log2, int gpr_log2, int col0, int col1,
                const SpmmEpilogue& epi, const SpmmLong& lg, bool split, const int32_t* out_index) {
    const int64_t nparts = split ? lg.n_parts : 0;
    constexpr int U = (R == 1) ? 8 : 4;              // gathers in flight per lane group when g_unroll allows
    const bool deep = g_unroll == 8 && R == 1;
    const int in_flight = deep ? U : 4;
    const int g_max = 6 - lpr_log2;
    ClassMap cm;
    if (lg.class_start && g_gpr_log2 < 0) {
        // class j holds rows of at most 4 * 2^(kSpmmClasses-1-j) entries (j = 0: up to the split threshold): the
        // fewest lane groups whose gathers in flight cover such a row in one trip of the entry loop
        cm.n = kSpmmClasses;
        for (int j = 0; j < kSpmmClasses; ++j) {
            int g = 0;
            if (j == 0) g = g_max;
            else while (g < g_max && (in_flight << g) < (4 << (kSpmmClasses - 1 - j))) ++g;
            cm.g[j] = g;
            cm.row_start[j] = lg.class_start[j];
        }
        cm.row_start[kSpmmClasses] = lg.class_start[kSpmmClasses];
    } else {
        cm.n = 1;
        cm.g[0] = gpr_log2;
        cm.row_start[0] = 0;
        cm.row_start[1] = nrows;
    }
    cm.part_g = (g_gpr_log2 >= 0) ? gpr_log2 : g_max;
    cm.block_start[0] = 0;
    for (int j = 0; j < cm.n; ++j) {
        const int64_t per_block = 4 * (64 >> (lpr_log2 + cm.g[j]));
        const int64_t n = cm.row_start[j + 1] - cm.row_start[j];
        cm.block_start[j + 1] = cm.block_start[j] + ((n + per_block - 1) / per_block + 7) / 8 * 8;
    }
    for (int j = cm.n; j < kSpmmClasses; ++j) {
        cm.g[j] = 0;
        cm.row_start[j + 1] = cm.row_start[cm.n];
        cm.block_start[j + 1] = cm.block_start[cm.n];
    }
    const int64_t part_per_block = 4 * (64 >> (lpr_log2 + cm.part_g));
    const int64_t part_blocks = ((nparts + part_per_block - 1) / part_per_block + 7) / 8 * 8;
    const int64_t nb = part_blocks + cm.block_start[cm.n];
    if (nb <= 0) return;
    dim3 grid((unsigned)nb), block(256);
    const int xcd_remap = (lg.xcd_remap >= 0) ? lg.xcd_remap : g_xcd_remap;
    const int max_len = split ? lg.max_len : 0;
#define CADMM_SPMM(E_, U_, Z_, T_, NU_) hipLaunchKernelGGL((spmm_rows_kernel<VEC, R, E_, U_>), grid, block, 0, s, lo, hi, lg.part_lo, lg.part_hi, nrows, nparts, col, val, X, Y, lg.side, width, lpr_log2, cm, col0, col1, max_len, xcd_remap, Z_, T_, NU_, out_index, part_blocks)
    if (epi.kind == 1) { if (deep) CADMM_SPMM(1, 8, epi.Zl, epi.Tl, epi.nu); else CADMM_SPMM(1, 4, epi.Zl, epi.Tl, epi.nu); }
    else { if (deep) CADMM_SPMM(0, 8, nullptr, nullptr, 0.f); else CADMM_SPMM(0, 4, nullptr, nullptr, 0.f); }
#undef CADMM_SPMM
}

template <int VEC>
void launch_vec(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                const float* X, float* Y, int64_t nrows, int width, const SpmmEpilogue& epi, const SpmmLong& lg,
                const int32_t* out_index) {
    // column tiles of at most 64 lanes * VEC * 4 repeats; a smaller tile can be requested
    int tile = 64 * VEC * 4;
    if (g_tile_cols > 0 && g_tile_cols < tile) tile = (g_tile_cols + VEC - 1) / VEC * VEC;
    const bool split = lg.max_len > 0 && lg.n_long > 0;
    for (int col0 = 0; col0 < width; col0 += tile) {
        const int col1 = (width - col0 < tile) ? width : col0 + tile;
        const int lanes_needed = (col1 - col0 + VEC - 1) / VEC;
        int lpr_log2 = 0;
        while ((1 << lpr_log2) < lanes_needed && lpr_log2 < 6) ++lpr_log2;
        const int reps = (lanes_needed + (1 << lpr_log2) - 1) >> lpr_log2;
        // lane groups per row: as many as the wavefront allows, but only until one trip of the entry loop
        // (groups x gathers in flight per group) covers a row of mean length
        int gpr_log2 = 0;
        const int mean_len = lg.mean_len > 0 ? lg.mean_len : 1;
        const int in_flight = (reps <= 1) ? g_unroll : 4;
        while (lpr_log2 + gpr_log2 < 6 && (in_flight << gpr_log2) < mean_len) ++gpr_log2;
        if (g_gpr_log2 >= 0) gpr_log2 = (lpr_log2 + g_gpr_log2 <= 6) ? g_gpr_log2 : 6 - lpr_log2;
        if (reps <= 1) launch_cfg<VEC, 1>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, gpr_log2, col0, col1, epi, lg, split, out_index);
        else if (reps <= 2) launch_cfg<VEC, 2>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, gpr_log2, col0, col1, epi, lg, split, out_index);
        else launch_cfg<VEC, 4>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, gpr_log2, col0, col1, epi, lg, split, out_index);
        if (split) {
            dim3 grid((unsigned)lg.n_long), block(64);
            if (epi.kind == 1)
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 1>), grid, block, 0, s, lg.side, lg.long_row,
                                   lg.long_part_ptr, lg.n_long, Y, width, col0, col1, epi.Zl, epi.Tl, epi.nu, lpr_log2);
            else
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 0>), grid, block, 0, s, lg.side, lg.long_row,
                                   lg.long_part_ptr, lg.n_long, Y, width, col0, col1, nullptr, nullptr, 0.f, lpr_log2);
        }
    }
}

}  // namespace

void set_spmm_tile_cols(int cols) { g_tile_cols = cols > 0 ? cols : 0; }
void set_spmm_xcd_remap(int on) { g_xcd_remap = on ? 1 : 0; }
void set_spmm_groups_log2(int v) { g_gpr_log2 = v; }
void set_spmm_unroll(int v) { g_unroll = (v == 8) ? 8 : 4; }

void launch_spmm(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                 const float* X, float* Y, int64_t nrows, int width, const SpmmEpilogue& epi, const SpmmLong& lg,
                 const int32_t* out_index) {
    if ((nrows <= 0 && lg.n_parts <= 0) || width <= 0) return;
    if (width % 4 == 0) launch_vec<4>(s, lo, hi, col, val, X, Y, nrows, width, epi, lg, out_index);
    else launch_vec<1>(s, lo, hi, col, val, X, Y, nrows, width, epi, lg, out_index);
}

void launch_spmm_single(hipStream_t s, const int32_t* pos, const int32_t* col, const float* val, const float* X,
                        float* Y, int64_t n, int width) {
    if (n <= 0 || width <= 0) return;
    const int vec = (width % 4 == 0) ? 4 : 1;
    const int lanes_needed = (width + vec - 1) / vec;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < lanes_needed && lpr_log2 < 6) ++lpr_log2;
    const int64_t groups = (n + kSingleBatch - 1) / kSingleBatch;
    const int64_t per_block = 256 >> lpr_log2;
    const int64_t nb = (groups + per_block - 1) / per_block;
    if (vec == 4) hipLaunchKernelGGL((spmm_single_kernel<4>), dim3((unsigned)nb), dim3(256), 0, s, pos, col, val, X, Y, n, width, lpr_log2);
    else hipLaunchKernelGGL((spmm_single_kernel<1>), dim3((unsigned)nb), dim3(256), 0, s, pos, col, val, X, Y, n, width, lpr_log2);
}

}  // namespace cadmm
