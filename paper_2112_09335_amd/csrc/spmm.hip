// Community-blocked sparse aggregation  Y = A~ X  on gfx950 (paper, Section 2, Problem 3: row block m
// is A~_{m,m} X_m + sum_{r in N_m} A~_{m,r} X_r; Appendix A: the same sum restricted to one
// neighbour community per output row, the "segments").
//
// Layout: CSR with sorted columns in the community-contiguous numbering, so one row's entries are
// grouped by community and a (row, community) segment is a contiguous entry range [lo, hi).
// Features are row-major fp32.
//
// Mapping: a group of LPR lanes (a power of two, up to the 64-lane wavefront) owns one output row;
// every lane keeps VEC*R accumulators, so a gathered neighbour row is read by the group with one
// fully coalesced VEC*4-byte load per lane and no cross-lane reduction is needed.  The entry loop is
// unrolled by four so that four independent row gathers are in flight per group.  The bound is HBM
// / L2 traffic of the gathers.  Blocks are renumbered so that each XCD (blockIdx mod 8) walks one
// contiguous eighth of the rows: neighbours are mostly in the same community, i.e. in the same
// row range, and stay in that XCD's L2.
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

template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&src)[VEC]) {
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(src[0], src[1], src[2], src[3]);
    } else {
        *p = src[0];
    }
}

template <int VEC, int R, int EPI>
__global__ __launch_bounds__(256) void spmm_rows_kernel(
    const int64_t* __restrict__ lo, const int64_t* __restrict__ hi, const int32_t* __restrict__ col,
    const float* __restrict__ val, const float* __restrict__ X, float* __restrict__ Y, int64_t nrows,
    int width, int lpr_log2, int col0, int col1, int max_len, int xcd_remap, const float* __restrict__ Zl,
    const float* __restrict__ Tl, float nu) {
    // XCD-aware renumbering: gridDim.x is a multiple of 8
    const int per_xcd = gridDim.x >> 3;
    const int64_t lb = xcd_remap ? (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3) : (int64_t)blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int rows_per_wave = 64 >> lpr_log2;
    const int64_t row = (lb * 4 + wave) * rows_per_wave + (lane >> lpr_log2);
    if (row >= nrows) return;
    const int lpr = 1 << lpr_log2;
    const int sub = lane & (lpr - 1);
    const int cbase = col0 + sub * VEC;       // first column of repeat 0
    const int cstride = lpr * VEC;            // columns between repeats

    float acc[R][VEC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[r][v] = 0.f;

    int64_t p = lo[row];
    const int64_t e = hi[row];
    if (max_len > 0 && e - p > max_len) return;     // split row: its parts are handled separately
    for (; p + 4 <= e; p += 4) {
        int32_t c[4];
        float a[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) { c[u] = col[p + u]; a[u] = val[p + u]; }
        float x[4][R][VEC];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float* xr = X + (int64_t)c[u] * width;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int cc = cbase + r * cstride;
                if (cc < col1) load_vec<VEC>(x[u][r], xr + cc);
                else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) x[u][r][v] = 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[r][v] = fmaf(a[u], x[u][r][v], acc[r][v]);
    }
    for (; p < e; ++p) {
        const int32_t c = col[p];
        const float a = val[p];
        const float* xr = X + (int64_t)c * width;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int cc = cbase + r * cstride;
            if (cc < col1) {
                float x[VEC];
                load_vec<VEC>(x, xr + cc);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[r][v] = fmaf(a, x[v], acc[r][v]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int cc = cbase + r * cstride;
        if (cc < col1) {
            const int64_t o = row * (int64_t)width + cc;
            if constexpr (EPI == 1) {
                float z[VEC], t[VEC];
                load_vec<VEC>(z, Zl + o);
                load_vec<VEC>(t, Tl + o);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[r][v] = nu * (z[v] - fmaxf(t[v], 0.f)) + acc[r][v];
            }
            store_vec<VEC>(Y + o, acc[r]);
        }
    }
}

int g_tile_cols = 0;
int g_xcd_remap = 1;

// Adds the parts of every split row in part order and applies the epilogue.  One lane group per row.
template <int VEC, int EPI>
__global__ __launch_bounds__(256) void spmm_combine_kernel(const float* __restrict__ side,
                                                           const int32_t* __restrict__ long_row,
                                                           const int32_t* __restrict__ long_part_ptr, int64_t n_long,
                                                           float* __restrict__ Y, int width, int col0, int col1,
                                                           const float* __restrict__ Zl, const float* __restrict__ Tl,
                                                           float nu) {
    const int64_t i = blockIdx.x;
    if (i >= n_long) return;
    const int64_t row = long_row[i];
    const int p0 = long_part_ptr[i], p1 = long_part_ptr[i + 1];
    for (int c = col0 + threadIdx.x * VEC; c < col1; c += blockDim.x * VEC) {
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        for (int p = p0; p < p1; ++p) {
            float x[VEC];
            load_vec<VEC>(x, side + (int64_t)p * width + c);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] += x[v];
        }
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
                const float* X, float* Y, int64_t nrows, int width, int lpr_log2, int col0, int col1, int max_len,
                const SpmmEpilogue& epi) {
    const int rows_per_block = 4 * (64 >> lpr_log2);
    int64_t nb = (nrows + rows_per_block - 1) / rows_per_block;
    nb = (nb + 7) / 8 * 8;
    dim3 grid((unsigned)nb), block(256);
    if (epi.kind == 1)
        hipLaunchKernelGGL((spmm_rows_kernel<VEC, R, 1>), grid, block, 0, s, lo, hi, col, val, X, Y, nrows, width,
                           lpr_log2, col0, col1, max_len, g_xcd_remap, epi.Zl, epi.Tl, epi.nu);
    else
        hipLaunchKernelGGL((spmm_rows_kernel<VEC, R, 0>), grid, block, 0, s, lo, hi, col, val, X, Y, nrows, width,
                           lpr_log2, col0, col1, max_len, g_xcd_remap, nullptr, nullptr, 0.f);
}


template <int VEC>
void launch_tile(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                 const float* X, float* Y, int64_t nrows, int width, int col0, int col1, int max_len,
                 const SpmmEpilogue& epi) {
    const int lanes_needed = (col1 - col0 + VEC - 1) / VEC;
    int lpr_log2 = 0;
    while ((1 << lpr_log2) < lanes_needed && lpr_log2 < 6) ++lpr_log2;
    const int reps = (lanes_needed + (1 << lpr_log2) - 1) >> lpr_log2;
    if (reps <= 1) launch_cfg<VEC, 1>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, col0, col1, max_len, epi);
    else if (reps <= 2) launch_cfg<VEC, 2>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, col0, col1, max_len, epi);
    else launch_cfg<VEC, 4>(s, lo, hi, col, val, X, Y, nrows, width, lpr_log2, col0, col1, max_len, epi);
}

template <int VEC>
void launch_vec(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                const float* X, float* Y, int64_t nrows, int width, const SpmmEpilogue& epi, const SpmmLong& lg) {
    // column tiles of at most 64 lanes * VEC * 4 repeats; a smaller tile can be requested
    int tile = 64 * VEC * 4;
    if (g_tile_cols > 0 && g_tile_cols < tile) tile = (g_tile_cols + VEC - 1) / VEC * VEC;
    const bool split = lg.max_len > 0 && lg.n_long > 0;
    for (int col0 = 0; col0 < width; col0 += tile) {
        const int col1 = (width - col0 < tile) ? width : col0 + tile;
        launch_tile<VEC>(s, lo, hi, col, val, X, Y, nrows, width, col0, col1, split ? lg.max_len : 0, epi);
        if (split) {
            launch_tile<VEC>(s, lg.part_lo, lg.part_hi, col, val, X, lg.side, lg.n_parts, width, col0, col1, 0,
                             SpmmEpilogue());
            dim3 grid((unsigned)lg.n_long), block(64);
            if (epi.kind == 1)
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 1>), grid, block, 0, s, lg.side, lg.long_row,
                                   lg.long_part_ptr, lg.n_long, Y, width, col0, col1, epi.Zl, epi.Tl, epi.nu);
            else
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 0>), grid, block, 0, s, lg.side, lg.long_row,
                                   lg.long_part_ptr, lg.n_long, Y, width, col0, col1, nullptr, nullptr, 0.f);
        }
    }
}

}  // namespace

void set_spmm_tile_cols(int cols) { g_tile_cols = cols > 0 ? cols : 0; }
void set_spmm_xcd_remap(int on) { g_xcd_remap = on ? 1 : 0; }

void launch_spmm(hipStream_t s, const int64_t* lo, const int64_t* hi, const int32_t* col, const float* val,
                 const float* X, float* Y, int64_t nrows, int width, const SpmmEpilogue& epi, const SpmmLong& lg) {
    if (nrows <= 0 || width <= 0) return;
    if (width % 4 == 0) launch_vec<4>(s, lo, hi, col, val, X, Y, nrows, width, epi, lg);
    else launch_vec<1>(s, lo, hi, col, val, X, Y, nrows, width, epi, lg);
}

}  // namespace cadmm
