// Community-blocked sparse aggregation  Y = A~ X  on gfx950 (paper, Section 2, Problem 3: row block m
// is A~_{m,m} X_m + sum_{r in N_m} A~_{m,r} X_r; Appendix A: the same sum restricted to one
// neighbour community per output row, the "segments").
//
// Layout: a row list (the CSR rows, or the (row, community) segments with several entries) laid out by the host
// for these kernels: rows sorted by (community, length class); one 16-byte record per row (its chunk range and
// output row); the entries as (column, value) pairs in chunks of eight, padded with weight zero; and a table that
// names the rows of every workgroup.  Features are row-major fp32.
//
// Mapping: a group of LPR lanes (a power of two, up to the 64-lane wavefront) reads one gathered
// neighbour row with one fully coalesced VEC*4-byte load per lane and keeps VEC*R accumulators per lane.
// GPR such groups share one output row and take its chunks round-robin, one chunk = eight gathers in flight per
// group and trip; their partial sums are added by a wavefront-level xor-shuffle reduction.  GPR is chosen per run
// of one length class so that one trip covers the class's longest row: short rows pack many rows into a
// wavefront, long rows spread over it, and the rows of a wavefront need the same number of trips.
// What bounds the narrow shapes (rows of up to 64 bytes) is the rate at which the L2s take 64-byte requests from the
// L1s, one per gathered row (measured with gather_calibration_kernel below); everything around the gathers is kept
// out of their way: a lane group fetches its chunk with one load of 64 bytes spread over its lanes (one instruction
// per 128 entries at 16 columns) and hands the pairs round by lane exchanges, instead of one load of four bytes per
// entry and array.
// Rows beyond a length threshold (power-law hubs) are cut into parts that run first in the same launch, into a
// side buffer; a small kernel adds a row's parts in order.  Segments with a single entry are scaled copies of a
// gathered row and have a kernel of their own.  Everything is order-fixed: no atomics, results are reproducible.
// XCD k (blockIdx mod 8) walks the k-th slice of the workgroup table, whole communities one after the other with
// all their length classes, so that the rows of the gathered matrix a community reads are fetched into that XCD's
// L2 once.
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

// Slice k of the workgroup table (the workgroups of XCD k) is [start[k], start[k+1]).
struct XcdMap {
    long long start[9];
};

template <int S>
__device__ __forceinline__ int quad_bcast(int v) {       // lane j of every quad gets lane S's value
    return __builtin_amdgcn_mov_dpp(v, S * 0x55, 0xF, 0xF, true);
}

// The eight (column, value) pairs of chunk `chunk` for every lane of a lane group of 2^LPRL lanes (LPRL = 3 stands
// for 8 and more lanes, lpr_log2 then says how many).  The group's lanes share the chunk's 64 bytes among them in
// as few load instructions as possible and exchange the pairs afterwards.
template <int LPRL>
__device__ __forceinline__ void load_chunk(const int2* __restrict__ ent, int64_t chunk, int lpr_log2, int lane,
                                           int32_t (&c)[8], float (&a)[8]) {
    const int4* e4 = reinterpret_cast<const int4*>(ent) + chunk * 4;      // a chunk is four 16-byte pieces
    if constexpr (LPRL == 0) {
        const int4 q0 = e4[0], q1 = e4[1], q2 = e4[2], q3 = e4[3];
        c[0] = q0.x; c[1] = q0.z; c[2] = q1.x; c[3] = q1.z; c[4] = q2.x; c[5] = q2.z; c[6] = q3.x; c[7] = q3.z;
        a[0] = __int_as_float(q0.y); a[1] = __int_as_float(q0.w); a[2] = __int_as_float(q1.y); a[3] = __int_as_float(q1.w);
        a[4] = __int_as_float(q2.y); a[5] = __int_as_float(q2.w); a[6] = __int_as_float(q3.y); a[7] = __int_as_float(q3.w);
    } else if constexpr (LPRL == 1) {
        const int sub = lane & 1;
        const int4 q0 = e4[2 * sub], q1 = e4[2 * sub + 1];                // pairs 4 sub .. 4 sub + 3
        const int mine[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int src = (lane & ~1) | (u >> 2);
            c[u] = __shfl(mine[2 * (u & 3)], src, 64);
            a[u] = __int_as_float(__shfl(mine[2 * (u & 3) + 1], src, 64));
        }
    } else if constexpr (LPRL == 2) {
        const int4 q = e4[lane & 3];                                      // pairs 2 sub, 2 sub + 1
        c[0] = quad_bcast<0>(q.x); a[0] = __int_as_float(quad_bcast<0>(q.y));
        c[1] = quad_bcast<0>(q.z); a[1] = __int_as_float(quad_bcast<0>(q.w));
        c[2] = quad_bcast<1>(q.x); a[2] = __int_as_float(quad_bcast<1>(q.y));
        c[3] = quad_bcast<1>(q.z); a[3] = __int_as_float(quad_bcast<1>(q.w));
        c[4] = quad_bcast<2>(q.x); a[4] = __int_as_float(quad_bcast<2>(q.y));
        c[5] = quad_bcast<2>(q.z); a[5] = __int_as_float(quad_bcast<2>(q.w));
        c[6] = quad_bcast<3>(q.x); a[6] = __int_as_float(quad_bcast<3>(q.y));
        c[7] = quad_bcast<3>(q.z); a[7] = __int_as_float(quad_bcast<3>(q.w));
    } else {
        const int base = lane & ~((1 << lpr_log2) - 1);
        const int2 q = ent[chunk * 8 + (lane & 7)];                       // lane j of the group holds pair j mod 8
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            c[u] = __shfl(q.x, base + u, 64);
            a[u] = __int_as_float(__shfl(q.y, base + u, 64));
        }
    }
}

// LPRL: lanes per gathered row as a power of two (3 stands for 8 and more, lpr_log2_arg then says how many); R column
// repeats per lane (more than one only for more than 256 columns, a whole wavefront per gathered row).
template <int VEC, int R, int EPI, int LPRL>
__global__ __launch_bounds__(256) void spmm_rows_kernel(
    const int4* __restrict__ rec, int64_t nrows, const int2* __restrict__ ent, const float* __restrict__ X,
    float* __restrict__ Y, float* __restrict__ side, int width, int lpr_log2_arg, const int4* __restrict__ blocks,
    XcdMap xm, int col0, int col1, int xcd_remap, const float* __restrict__ Zl, const float* __restrict__ Tl, float nu) {
    // Workgroup b belongs to XCD b mod 8 and takes the (b / 8)-th entry of that XCD's slice of the table (or, without
    // the XCD-aware numbering, simply entry b).  Records from nrows on are the parts of split rows.
    const int lpr_log2 = LPRL < 3 ? LPRL : lpr_log2_arg;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    int64_t idx;
    if (xcd_remap) {
        const int k = (int)(blockIdx.x & 7);
        idx = xm.start[k] + (blockIdx.x >> 3);
        if (idx >= xm.start[k + 1]) return;
    } else {
        idx = blockIdx.x;
        if (idx >= xm.start[8]) return;
    }
    const int4 d = blocks[idx];                         // rows [d.x, d.y), 2^d.z lane groups per row
    const int gpr_log2 = d.z;
    const int span_log2 = lpr_log2 + gpr_log2;          // lanes that share one output row
    const int64_t vrow = (int64_t)d.x + ((wave << (6 - span_log2)) + (lane >> span_log2));
    if (vrow >= d.y) return;                            // uniform over the row's lane span
    const int4 r = rec[vrow];                           // chunks [r.x, r.y), output row r.z
    const bool is_part = vrow >= nrows;
    float* const dst = (is_part ? side : Y) + (int64_t)r.z * (int64_t)width;
    const int lpr = 1 << lpr_log2;
    const int gpr = 1 << gpr_log2;
    const int grp = (lane >> lpr_log2) & (gpr - 1);
    const int sub = lane & (lpr - 1);
    const int cbase = col0 + sub * VEC;                 // first column of repeat 0
    const int cstride = lpr * VEC;                      // columns between repeats

    float acc[R][VEC];
#pragma unroll
    for (int q = 0; q < R; ++q)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[q][v] = 0.f;
    // a lane past the last column reads the last columns again without storing them
    int ccl[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
        const int cc = cbase + q * cstride;
        ccl[q] = cc < col1 ? cc : col1 - VEC;
    }
    // the epilogue's operands (rows of Z_l and T_l at the output row) are asked for before the gathers, so that their
    // latency is not added at the end of every row
    float ez[R][VEC], et[R][VEC];
    if constexpr (EPI == 1) {
        if (!is_part && grp == 0) {
#pragma unroll
            for (int q = 0; q < R; ++q) {
                const int64_t o = (int64_t)r.z * (int64_t)width + ccl[q];
                load_vec<VEC>(ez[q], Zl + o);
                load_vec<VEC>(et[q], Tl + o);
            }
        }
    }
    // the groups of a row take its chunks grp, grp + gpr, ...: eight gathers in flight per group (four per column
    // repeat for the wide shapes); the padding of a chunk carries weight zero, so no entry is masked
    constexpr int UH = (R == 1) ? 8 : 4;
    for (int ch = r.x + grp; ch < r.y; ch += gpr) {
        int32_t c[8];
        float a[8];
        load_chunk<LPRL>(ent, ch, lpr_log2, lane, c, a);
#pragma unroll
        for (int h = 0; h < 8 / UH; ++h) {
            float x[UH][R][VEC];
#pragma unroll
            for (int u = 0; u < UH; ++u)
#pragma unroll
                for (int q = 0; q < R; ++q) load_vec<VEC>(x[u][q], X + (int64_t)c[UH * h + u] * width + ccl[q]);
#pragma unroll
            for (int u = 0; u < UH; ++u)
#pragma unroll
                for (int q = 0; q < R; ++q)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[q][v] = fmaf(a[UH * h + u], x[u][q][v], acc[q][v]);
        }
    }
    // wavefront-level reduction across the groups of the row
    for (int off = lpr; off < (lpr << gpr_log2); off <<= 1) {
#pragma unroll
        for (int q = 0; q < R; ++q)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[q][v] += __shfl_xor(acc[q][v], off, 64);
    }
    if (grp != 0) return;
#pragma unroll
    for (int q = 0; q < R; ++q) {
        const int cc = cbase + q * cstride;
        if (cc < col1) {
            if constexpr (EPI == 1) {
                if (!is_part) {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[q][v] = nu * (ez[q][v] - fmaxf(et[q][v], 0.f)) + acc[q][v];
                }
            }
            store_vec<VEC>(dst + cc, acc[q]);
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

// Machine calibration for the aggregation: the gathers of a row list and nothing else.  Every lane group takes one
// chunk of the entry array (the real column stream, in the order the aggregation reads it: XCD k, the workgroups with
// blockIdx mod 8 = k, walks the k-th eighth front to back), gathers the eight rows the chunk names and adds them up;
// there are no row records, no reduction across lanes and no result rows (a lane stores only if its sum is a value
// that does not occur, which keeps the loads alive).  What this reaches is the rate at which the memory system serves
// this column stream's gathers of 4 * VEC * 2^lpr_log2 bytes.
template <int LPRL>
__global__ __launch_bounds__(256) void gather_calibration_kernel(const int2* __restrict__ ent, int64_t n_chunks,
                                                                 const float* __restrict__ X, int width, int lpr_log2_arg,
                                                                 float* __restrict__ out) {
    const int lpr_log2 = LPRL < 3 ? LPRL : lpr_log2_arg;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int k = blockIdx.x & 7;
    const int64_t per_xcd = (n_chunks + 7) / 8;
    const int64_t lo = 1 + k * per_xcd, hi = lo + per_xcd < n_chunks ? lo + per_xcd : n_chunks;   // chunk 0 is padding
    const int groups = 64 >> lpr_log2;
    const int64_t ch = lo + ((int64_t)(blockIdx.x >> 3) * 4 + wave) * groups + (lane >> lpr_log2);
    if (ch >= hi) return;                               // uniform over a lane group
    const int cc = (lane & ((1 << lpr_log2) - 1)) * 4;
    int32_t c[8];
    float a[8];
    load_chunk<LPRL>(ent, ch, lpr_log2, lane, c, a);
    float x[8][4];
#pragma unroll
    for (int u = 0; u < 8; ++u) load_vec<4>(x[u], X + (int64_t)c[u] * width + cc);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = fmaf(a[u], x[u][v], acc[v]);
    const float sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (sum == 1.2345678e33f) out[threadIdx.x] = sum;
}

int g_tile_cols = 0;
int g_xcd_remap = 1;

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
void launch_cfg(hipStream_t s, const SpmmSchedule& sc, const float* X, float* Y, int width, int lpr_log2, int col0,
                int col1, const SpmmEpilogue& epi) {
    XcdMap xm;
    int64_t longest = 0;
    for (int k = 0; k <= 8; ++k) xm.start[k] = sc.xcd_start[lpr_log2][k];
    for (int k = 0; k < 8; ++k) longest = xm.start[k + 1] - xm.start[k] > longest ? xm.start[k + 1] - xm.start[k] : longest;
    const int64_t nb = g_xcd_remap ? 8 * longest : (sc.n_blocks[lpr_log2] + 7) / 8 * 8;
    if (nb <= 0) return;
    dim3 grid((unsigned)nb), block(256);
#define CADMM_ROWS(L_) do { \
        if (epi.kind == 1) hipLaunchKernelGGL((spmm_rows_kernel<VEC, R, 1, L_>), grid, block, 0, s, sc.rec, sc.n_rows, sc.ent, X, Y, \
                                              sc.side, width, lpr_log2, sc.blocks[lpr_log2], xm, col0, col1, g_xcd_remap, epi.Zl, epi.Tl, epi.nu); \
        else hipLaunchKernelGGL((spmm_rows_kernel<VEC, R, 0, L_>), grid, block, 0, s, sc.rec, sc.n_rows, sc.ent, X, Y, sc.side, width, \
                                lpr_log2, sc.blocks[lpr_log2], xm, col0, col1, g_xcd_remap, nullptr, nullptr, 0.f); } while (0)
    if constexpr (R == 1) {
        if (lpr_log2 == 0) CADMM_ROWS(0);
        else if (lpr_log2 == 1) CADMM_ROWS(1);
        else if (lpr_log2 == 2) CADMM_ROWS(2);
        else CADMM_ROWS(3);
    } else {
        CADMM_ROWS(3);                                   // column repeats only occur with a whole wavefront per row
    }
#undef CADMM_ROWS
}

template <int VEC>
void launch_vec(hipStream_t s, const SpmmSchedule& sc, const float* X, float* Y, int width, const SpmmEpilogue& epi) {
    // column tiles of at most 64 lanes * VEC * 4 repeats; a smaller tile can be requested
    int tile = 64 * VEC * 4;
    if (g_tile_cols > 0 && g_tile_cols < tile) tile = (g_tile_cols + VEC - 1) / VEC * VEC;
    for (int col0 = 0; col0 < width; col0 += tile) {
        const int col1 = (width - col0 < tile) ? width : col0 + tile;
        const int lanes_needed = (col1 - col0 + VEC - 1) / VEC;
        int lpr_log2 = 0;
        while ((1 << lpr_log2) < lanes_needed && lpr_log2 < 6) ++lpr_log2;
        const int reps = (lanes_needed + (1 << lpr_log2) - 1) >> lpr_log2;
        if (reps <= 1) launch_cfg<VEC, 1>(s, sc, X, Y, width, lpr_log2, col0, col1, epi);
        else if (reps <= 2) launch_cfg<VEC, 2>(s, sc, X, Y, width, lpr_log2, col0, col1, epi);
        else launch_cfg<VEC, 4>(s, sc, X, Y, width, lpr_log2, col0, col1, epi);
        if (sc.n_long > 0) {
            dim3 grid((unsigned)sc.n_long), block(64);
            if (epi.kind == 1)
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 1>), grid, block, 0, s, sc.side, sc.long_row,
                                   sc.long_part_ptr, sc.n_long, Y, width, col0, col1, epi.Zl, epi.Tl, epi.nu, lpr_log2);
            else
                hipLaunchKernelGGL((spmm_combine_kernel<VEC, 0>), grid, block, 0, s, sc.side, sc.long_row,
                                   sc.long_part_ptr, sc.n_long, Y, width, col0, col1, nullptr, nullptr, 0.f, lpr_log2);
        }
    }
}

}  // namespace

void set_spmm_tile_cols(int cols) { g_tile_cols = cols > 0 ? cols : 0; }
void set_spmm_xcd_remap(int on) { g_xcd_remap = on ? 1 : 0; }

double launch_gather_calibration(hipStream_t s, const SpmmSchedule& sc, int64_t n_chunks, const float* X, int width,
                                 float* out) {
    int lpr_log2 = 0;
    while ((4 << lpr_log2) < width) ++lpr_log2;
    const int64_t per_xcd = (n_chunks + 7) / 8, per_block = 4 * (64 >> lpr_log2);
    dim3 grid((unsigned)(8 * ((per_xcd + per_block - 1) / per_block))), block(256);
    if (lpr_log2 == 0) hipLaunchKernelGGL((gather_calibration_kernel<0>), grid, block, 0, s, sc.ent, n_chunks, X, width, lpr_log2, out);
    else if (lpr_log2 == 1) hipLaunchKernelGGL((gather_calibration_kernel<1>), grid, block, 0, s, sc.ent, n_chunks, X, width, lpr_log2, out);
    else if (lpr_log2 == 2) hipLaunchKernelGGL((gather_calibration_kernel<2>), grid, block, 0, s, sc.ent, n_chunks, X, width, lpr_log2, out);
    else hipLaunchKernelGGL((gather_calibration_kernel<3>), grid, block, 0, s, sc.ent, n_chunks, X, width, lpr_log2, out);
    return (double)(n_chunks - 1) * 8.0 * (8.0 + 4.0 * width);       // the pairs and the rows they name
}

void launch_spmm(hipStream_t s, const SpmmSchedule& sched, const float* X, float* Y, int width, const SpmmEpilogue& epi) {
    if ((sched.n_rows <= 0 && sched.n_parts <= 0) || width <= 0) return;
    if (width % 4 == 0) launch_vec<4>(s, sched, X, Y, width, epi);
    else launch_vec<1>(s, sched, X, Y, width, epi);
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
