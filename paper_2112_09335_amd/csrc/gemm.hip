// Dense fp32 contractions of the sweep on the gfx950 matrix cores: v_mfma_f32_32x32x2_f32, or (default for results
// wider than 32 columns, the *_split_kernel variants) v_mfma_f32_32x32x16_bf16 on operands split exactly into
// three bf16 parts each, which gives the same accuracy at a fraction of the matrix-core time:
//   gemm_nn : out[n x C] = A[n x K] B[K x C]     (T_l = H_l W_l, Q = H_l gradW, G W^T, gradZ W;
//                                                 paper Section 3.1 and Appendix A)
//   gemm_tn : out[K x C] = A[n x K]^T G[n x C]   (gradient of phi with respect to W_l: a sum over all
//                                                 nodes of all communities, Section 3.1)
// n is the number of nodes (huge), K and C are layer widths (3..512).
//
// Tiling: 256 threads = 4 wavefronts; block tile 128 x BN (BN = 128: 2x2 waves of 64x64; BN = 32: 4x1
// waves of 32x32), K-step 16, operands staged through LDS, next tile prefetched into registers while
// the current one feeds the MFMAs.  MFMA operand layout for 32x32x2 (64 lanes): lane holds
// A[i = lane%32][k = lane/32] and B[k = lane/32][j = lane%32]; accumulator register r of a lane is
// C[8*(r/4) + 4*(lane/32) + r%4][lane%32].
// gemm_tn splits n into chunks, each block reduces one chunk for one 128 x BN output tile into a
// partial matrix; a second kernel adds the partials in chunk order in fp64 (deterministic).
#include "kernels.h"

namespace cadmm {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BK = 16;

__device__ __forceinline__ float4 ld4_guard(const float* base, int64_t off, bool ok, bool aligned, int valid) {
    // valid: number of in-range elements (0..4) starting at off
    if (!ok || valid <= 0) return make_float4(0.f, 0.f, 0.f, 0.f);
    if (aligned && valid >= 4) return *reinterpret_cast<const float4*>(base + off);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    v.x = base[off];
    if (valid > 1) v.y = base[off + 1];
    if (valid > 2) v.z = base[off + 2];
    if (valid > 3) v.w = base[off + 3];
    return v;
}

// Consecutive workgroups go round-robin to the eight XCDs, each with an L2 of its own.  Workgroups that read the
// same operand tile (the `inner` column tiles of one row tile, the tiles of one row chunk) are therefore given
// indices 8 apart, so that they run at about the same time on ONE XCD and the shared tile comes from its L2.
// The last, incomplete set of 8 * inner workgroups keeps the plain order.  (outer, in) is a bijection of blockIdx.
__device__ __forceinline__ void xcd_group(unsigned b, unsigned nb, unsigned inner, int64_t& outer, int& in) {
    const unsigned set = 8u * inner;
    if (b < nb / set * set) {
        const unsigned w = b % set;
        outer = (int64_t)(b / set) * 8 + (w & 7u);
        in = (int)(w >> 3);
    } else {
        outer = b / inner;
        in = (int)(b % inner);
    }
}

// Epilogue of a 128 x 128 result tile held as 2 x 2 accumulators per wavefront (2 x 2 wavefronts).
// The accumulators hold 32 consecutive columns per row and lane group; passing each 32-row slab of the tile
// through LDS (Cs: 32 x 132 floats, the operand buffer reused) turns every global access of the epilogue into
// float4 pieces of a 512-byte row.
// EPI 0: out = acc.  EPI 1: out = nu (Zl - relu(Tl)) + acc.  EPI 2: first candidate of the W search and the step
// on Tio ahead of the decision, see GemmEpilogue.
template <int EPI>
__device__ __forceinline__ void tile128_epilogue(floatx16 (&acc)[2][2], float* Cs, int64_t m0, int c0, int64_t n, int C,
                                                 float* __restrict__ out, const float* __restrict__ Zl,
                                                 const float* __restrict__ Tl, float nu, float* __restrict__ Tio,
                                                 const Unit* unit, double* __restrict__ partials) {
    constexpr int LDC = 128 + 4;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lk = lane >> 5;
    const bool c_al = (C % 4) == 0;
    double inv0 = 0.0, dsum = 0.0;
    bool take = false;
    if constexpr (EPI == 2) {
        inv0 = unit->skip ? 0.0 : 1.0 / unit->step0;
        take = unit->spec != 0 && !unit->skip;
    }
    // one result element: returns what goes to out, updates t (EPI 2) and the candidate's sum
    auto finish = [&](float v, float z, float& t) -> float {
        if constexpr (EPI == 1) v = nu * (z - fmaxf(t, 0.f)) + v;
        if constexpr (EPI == 2) {
            const double t0 = (double)t, zd = (double)z;
            const double t1 = t0 - (double)v * inv0;
            const double e0 = fmax(t0, 0.0) - zd, e1 = fmax(t1, 0.0) - zd;
            dsum += (e1 - e0) * (e1 + e0);
            t = (float)t1;
        }
        return v;
    };
    const float* tin = (EPI == 2) ? Tio : Tl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        __syncthreads();
        if (wm == q / 2) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    Cs[(8 * (r >> 2) + 4 * lk + (r & 3)) * LDC + wn * 64 + j * 32 + li] = acc[q % 2][j][r];
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int f = tid + 256 * u;
            const int rl = f >> 5, cq = f & 31;
            const int64_t row = m0 + 32 * q + rl;
            const int c = c0 + 4 * cq;
            if (row >= n || c >= C) continue;
            const float4 v4 = *reinterpret_cast<const float4*>(Cs + rl * LDC + 4 * cq);
            float v[4] = {v4.x, v4.y, v4.z, v4.w};
            const int64_t o = row * C + c;
            if (c_al) {
                float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f), t4 = z4;
                if constexpr (EPI != 0) {
                    z4 = *reinterpret_cast<const float4*>(Zl + o);
                    t4 = *reinterpret_cast<const float4*>(tin + o);
                }
                v[0] = finish(v[0], z4.x, t4.x);
                v[1] = finish(v[1], z4.y, t4.y);
                v[2] = finish(v[2], z4.z, t4.z);
                v[3] = finish(v[3], z4.w, t4.w);
                if constexpr (EPI == 2) {
                    if (take) *reinterpret_cast<float4*>(Tio + o) = t4;
                    else *reinterpret_cast<float4*>(out + o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    *reinterpret_cast<float4*>(out + o) = make_float4(v[0], v[1], v[2], v[3]);
                }
            } else {
                for (int e = 0; e < 4 && c + e < C; ++e) {
                    float z = 0.f, t = 0.f;
                    if constexpr (EPI != 0) { z = Zl[o + e]; t = tin[o + e]; }
                    const float w = finish(v[e], z, t);
                    if constexpr (EPI == 2) {
                        if (take) Tio[o + e] = t;
                        else out[o + e] = w;
                    } else {
                        out[o + e] = w;
                    }
                }
            }
        }
    }
    if constexpr (EPI == 2) {
        __shared__ double red[4];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if (lane == 0) red[wave] = dsum;
        __syncthreads();
        if (tid == 0) partials[blockIdx.x] = 0.5 * (double)nu * (red[0] + red[1] + red[2] + red[3]);
    }
}

// ------------------------------------------------------------------------------------------------ NN
// EPI 1: out = nu * (Zl - relu(Tl)) + A B   (gradient of the Z subproblem, Appendix A)
// EPI 2: out = Q = A B; first candidate of the W search and speculative step on Tio (Section 3.1), see kernels.h
template <int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_nn_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                      float* __restrict__ out, int64_t n, int K, int C,
                                                      const float* __restrict__ Zl, const float* __restrict__ Tl,
                                                      float nu, float* __restrict__ Tio, const Unit* unit,
                                                      double* __restrict__ partials) {
    constexpr int WN = (BN == 128) ? 2 : 1;       // waves along columns
    constexpr int WM = 4 / WN;                    // waves along rows
    constexpr int TM = BM / (WM * 32);            // 32x32 tiles per wave along rows
    constexpr int TN = BN / (WN * 32);
    // columns of A per step: the narrow variant is bound by reading A, and takes a whole 128-byte line of a
    // row per step so that no half line has to survive in the L2 until the next step
    constexpr int BKK = (BN == 32) ? 32 : BK;
    constexpr int LDA = BKK + 1;
    constexpr int LDB = BN + 4;
    constexpr int A_Q = BKK / 4;                  // float4 per row of the A tile
    constexpr int A_PER_T = BM * A_Q / 256;
    constexpr int B_F4 = BKK * BN / 4;            // float4 loads for the B tile
    constexpr int B_PER_T = (B_F4 + 255) / 256;

    // one buffer: the operand tiles during the product, a 32-row slab of the result tile afterwards
    __shared__ __align__(16) float smem[BM * LDA + BKK * LDB];
    float* const As = smem;
    float* const Bs = smem + BM * LDA;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int ctiles = (C + BN - 1) / BN;
    if constexpr (EPI == 0) {
        // gated plain product: Q again for a W search whose speculative step (epilogue 2, Q not stored) was rejected
        if (unit != nullptr && (!unit->spec || unit->skip || (unit->done && unit->step == unit->step0))) return;
    }
    int64_t mtile;
    int ctile;
    xcd_group(blockIdx.x, gridDim.x, (unsigned)ctiles, mtile, ctile);
    const int64_t m0 = mtile * BM;
    const int c0 = ctile * BN;
    const bool a_al = (K % 4) == 0;
    const bool b_al = (C % 4) == 0;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[A_PER_T], rb[B_PER_T];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int f = tid + 256 * i;
            const int row = f / A_Q, kq = f % A_Q;
            const int64_t gr = m0 + row;
            const int k = k0 + 4 * kq;
            ra[i] = ld4_guard(A, gr * K + k, gr < n, a_al, K - k);
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int f = tid + 256 * i;
            if (f < B_F4) {
                const int kr = f / (BN / 4), cq = f % (BN / 4);
                const int k = k0 + kr, c = c0 + 4 * cq;
                rb[i] = ld4_guard(B, (int64_t)k * C + c, k < K, b_al, C - c);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            const int f = tid + 256 * i;
            const int row = f / A_Q, kq = f % A_Q;
            float* d = As + row * LDA + 4 * kq;
            d[0] = ra[i].x; d[1] = ra[i].y; d[2] = ra[i].z; d[3] = ra[i].w;
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            const int f = tid + 256 * i;
            if (f < B_F4) {
                const int kr = f / (BN / 4), cq = f % (BN / 4);
                *reinterpret_cast<float4*>(Bs + kr * LDB + 4 * cq) = rb[i];
            }
        }
    };

    const int nk = (K + BKK - 1) / BKK;
    fetch(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();            // previous tile fully consumed
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * BKK);
        const int li = lane & 31, lk = lane >> 5;
#pragma unroll
        for (int kk = 0; kk < BKK; kk += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = As[(wm * TM * 32 + i * 32 + li) * LDA + kk + lk];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bs[(kk + lk) * LDB + wn * TN * 32 + j * 32 + li];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    if constexpr (BN == 128) {
        static_assert(32 * (BN + 4) <= BM * LDA + BKK * LDB, "result slab must fit the operand buffer");
        tile128_epilogue<EPI>(acc, smem, m0, c0, n, C, out, Zl, Tl, nu, Tio, unit, partials);
    } else {
        static_assert(BN == 128 || EPI != 2, "the search epilogue exists for the wide tile only");
        const int li = lane & 31, lk = lane >> 5;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c = c0 + wn * TN * 32 + j * 32 + li;
                if (c >= C) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = m0 + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                    if (row < n) {
                        float v = acc[i][j][r];
                        if constexpr (EPI == 1) v = nu * (Zl[row * C + c] - fmaxf(Tl[row * C + c], 0.f)) + v;
                        out[row * C + c] = v;
                    }
                }
            }
    }
}

// The same product out[n x C] = A[n x K] B[K x C] on the bf16 matrix cores, fp32-exact in its inputs: an fp32 number is the
// exact sum of three bf16 numbers (8 + 8 + 8 significand bits, each part the truncated remainder of the one before), and of the
// nine cross products the six largest are accumulated in fp32 (hi*hi, hi*mid, mid*hi, mid*mid, hi*lo, lo*hi; the three
// that are left out are below 2^-24 of |a||b|).  Six v_mfma_f32_32x32x16_bf16 per 16 columns of K replace 32
// v_mfma_f32_32x32x2_f32, at a sixteenth of the cycles per flop.  Operand layout of 32x32x16 (64 lanes): a lane holds
// A[i = lane%32][k = 8*(lane/32) .. +7] and B[k = 8*(lane/32) .. +7][j = lane%32]; the accumulator as for 32x32x2.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef int intx4 __attribute__((ext_vector_type(4)));        // eight bf16 carried as plain bits

// two fp32 numbers -> their three bf16 parts, each pair packed into one dword (low half = first number)
__device__ __forceinline__ void split3_pair(float x0, float x1, unsigned& h, unsigned& m, unsigned& l) {
    const unsigned u0 = __float_as_uint(x0), u1 = __float_as_uint(x1);
    h = __builtin_amdgcn_perm(u1, u0, 0x07060302u);             // upper halves of u1 and u0
    const float r0 = x0 - __uint_as_float(u0 & 0xFFFF0000u);    // exact
    const float r1 = x1 - __uint_as_float(u1 & 0xFFFF0000u);
    const unsigned v0 = __float_as_uint(r0), v1 = __float_as_uint(r1);
    m = __builtin_amdgcn_perm(v1, v0, 0x07060302u);
    const float s0 = r0 - __uint_as_float(v0 & 0xFFFF0000u);    // exact, at most 8 significant bits left
    const float s1 = r1 - __uint_as_float(v1 & 0xFFFF0000u);
    l = __builtin_amdgcn_perm(__float_as_uint(s1), __float_as_uint(s0), 0x07060302u);
}

// (four wavefronts per SIMD asked for: the few registers that spill cost less than the fourth wavefront gains)
template <int EPI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void gemm_nn_split_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                            float* __restrict__ out, int64_t n, int K, int C,
                                                            const float* __restrict__ Zl, const float* __restrict__ Tl,
                                                            float nu, float* __restrict__ Tio, const Unit* unit,
                                                            double* __restrict__ partials) {
    constexpr int BN = 128;
    if constexpr (EPI == 0) {
        // gated plain product, as in gemm_nn_kernel
        if (unit != nullptr && (!unit->spec || unit->skip || (unit->done && unit->step == unit->step0))) return;
    }
    constexpr int LDH = BK + 8;                   // bf16 per tile row: rows start 16-byte aligned
    constexpr int PLANE = BM * LDH;               // BM == BN
    __shared__ __align__(16) unsigned short smem[6 * PLANE];
    unsigned short* const As = smem;              // [3][BM][LDH]: A tile, k contiguous per row
    unsigned short* const Bs = smem + 3 * PLANE;  // [3][BN][LDH]: B tile transposed, k contiguous per column
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lk = lane >> 5;
    const int ctiles = (C + BN - 1) / BN;
    int64_t mtile;
    int ctile;
    xcd_group(blockIdx.x, gridDim.x, (unsigned)ctiles, mtile, ctile);
    const int64_t m0 = mtile * BM;
    const int c0 = ctile * BN;
    const bool a_al = (K % 4) == 0;
    const bool b_al = (C % 4) == 0;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // A: thread takes 4 consecutive k of two rows; B: 8 consecutive k of one column (coalesced across the columns)
    float4 ra[2];
    float rb[8];
    const int bc = tid & 127, bkg = tid >> 7;
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int f = tid + 256 * i;
            const int row = f >> 2, kq = f & 3;
            const int64_t gr = m0 + row;
            const int k = k0 + 4 * kq;
            ra[i] = ld4_guard(A, gr * K + k, gr < n, a_al, K - k);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = k0 + 8 * bkg + e;
            rb[e] = (k < K && c0 + bc < C) ? B[(int64_t)k * C + c0 + bc] : 0.f;
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int f = tid + 256 * i;
            const int row = f >> 2, kq = f & 3;
            unsigned h0, m0_, l0, h1, m1, l1;
            split3_pair(ra[i].x, ra[i].y, h0, m0_, l0);
            split3_pair(ra[i].z, ra[i].w, h1, m1, l1);
            const int o = row * LDH + 4 * kq;
            *reinterpret_cast<uint2*>(As + o) = make_uint2(h0, h1);
            *reinterpret_cast<uint2*>(As + PLANE + o) = make_uint2(m0_, m1);
            *reinterpret_cast<uint2*>(As + 2 * PLANE + o) = make_uint2(l0, l1);
        }
        {
            unsigned h[4], m[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) split3_pair(rb[2 * e], rb[2 * e + 1], h[e], m[e], l[e]);
            const int o = bc * LDH + 8 * bkg;
            *reinterpret_cast<uint4*>(Bs + o) = make_uint4(h[0], h[1], h[2], h[3]);
            *reinterpret_cast<uint4*>(Bs + PLANE + o) = make_uint4(m[0], m[1], m[2], m[3]);
            *reinterpret_cast<uint4*>(Bs + 2 * PLANE + o) = make_uint4(l[0], l[1], l[2], l[3]);
        }
    };

    auto multiply = [&]() {
        bf16x8 a[3][2];
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[p][i] = *reinterpret_cast<const bf16x8*>(As + p * PLANE + (wm * 64 + i * 32 + li) * LDH + 8 * lk);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            bf16x8 b[3];                             // one column tile's parts at a time keeps the register count down
#pragma unroll
            for (int p = 0; p < 3; ++p)
                b[p] = *reinterpret_cast<const bf16x8*>(Bs + p * PLANE + (wn * 64 + j * 32 + li) * LDH + 8 * lk);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                floatx16 c = acc[i][j];
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2][i], b[0], c, 0, 0, 0);   // small terms first
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[2], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[1], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[0], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[1], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0], c, 0, 0, 0);
                acc[i][j] = c;
            }
        }
    };
    // (fetching two steps ahead was tried: the second register set costs more occupancy than the latency it hides)
    const int nk = (K + BK - 1) / BK;
    fetch(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * BK);
        multiply();
    }
    static_assert(32 * (BN + 4) * 4 <= 6 * PLANE * 2, "result slab must fit the operand buffer");
    tile128_epilogue<EPI>(acc, reinterpret_cast<float*>(smem), m0, c0, n, C, out, Zl, Tl, nu, Tio, unit, partials);
}

// out[n x C] = [ nu (Z - relu(T)) | SG ] * Bcat  with Bcat = [ W (K1 x C) ; S (K2 x C) ],  C <= 32.
// This is (grad_Z psi) W for grad = nu (Z - relu(T)) + SG W^T and S = W^T W, without ever storing the gradient:
// the left operand is formed while its tile is loaded.  K1 and K2 are multiples of four.
__global__ __launch_bounds__(256) void gemm_nn_gradz_kernel(const float* __restrict__ Zl, const float* __restrict__ Tl,
                                                            const float* __restrict__ SG, const float* __restrict__ Bcat,
                                                            float* __restrict__ out, int64_t n, int K1, int K2, int C,
                                                            float nu) {
    constexpr int BN = 32;
    // 32 columns of Z_l and T_l per step: every row then gives a whole 128-byte line of each matrix to one step.
    // With half lines the second half had left the L2 before its step came (twice the traffic, measured).
    constexpr int GBK = 32;
    constexpr int LDA = GBK + 1;
    constexpr int LDB = BN + 4;
    __shared__ __align__(16) float As[BM * LDA];
    __shared__ __align__(16) float Bs[GBK * LDB];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wm = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.x * BM;
    const int K = K1 + K2;
    const bool b_al = (C % 4) == 0;
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float4 ra[4], rb;
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = tid + 256 * i;
            const int row = f >> 3, kq = f & 7;
            const int64_t gr = m0 + row;
            const int k = k0 + 4 * kq;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (gr < n) {
                if (k < K1) {
                    const float4 z = *reinterpret_cast<const float4*>(Zl + gr * K1 + k);
                    const float4 t = *reinterpret_cast<const float4*>(Tl + gr * K1 + k);
                    v.x = nu * (z.x - fmaxf(t.x, 0.f));
                    v.y = nu * (z.y - fmaxf(t.y, 0.f));
                    v.z = nu * (z.z - fmaxf(t.z, 0.f));
                    v.w = nu * (z.w - fmaxf(t.w, 0.f));
                } else if (k < K) {
                    v = *reinterpret_cast<const float4*>(SG + gr * K2 + (k - K1));
                }
            }
            ra[i] = v;
        }
        {
            const int kr = tid / (BN / 4), cq = tid % (BN / 4);      // 32 x 8 float4, one per thread
            const int k = k0 + kr, c = 4 * cq;
            rb = ld4_guard(Bcat, (int64_t)k * C + c, k < K, b_al, C - c);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int f = tid + 256 * i;
            const int row = f >> 3, kq = f & 7;
            float* d = As + row * LDA + 4 * kq;
            d[0] = ra[i].x; d[1] = ra[i].y; d[2] = ra[i].z; d[3] = ra[i].w;
        }
        {
            const int kr = tid / (BN / 4), cq = tid % (BN / 4);
            *reinterpret_cast<float4*>(Bs + kr * LDB + 4 * cq) = rb;
        }
    };
    const int nk = (K + GBK - 1) / GBK;
    const int li = lane & 31, lk = lane >> 5;
    fetch(0);
    for (int kt = 0; kt < nk; ++kt) {
        __syncthreads();
        stash();
        __syncthreads();
        if (kt + 1 < nk) fetch((kt + 1) * GBK);
#pragma unroll
        for (int kk = 0; kk < GBK; kk += 2) {
            const float a = As[(wm * 32 + li) * LDA + kk + lk];
            const float b = Bs[(kk + lk) * LDB + li];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
    }
    if (li < C) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + wm * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
            if (row < n) out[row * C + li] = acc[r];
        }
    }
}

// ------------------------------------------------------------------------------------------------ TN
// Block (chunk, ktile, ctile): partial[chunk][k][c] = sum_{rows of chunk} A[row][k] G[row][c].
// PRO 1: the right operand is the hidden-layer pre-activation gradient nu (relu(T) - Z) 1[T > 0], formed from
// T (passed as G) and Z while the tile is loaded, so that it is never stored.
template <int BN, int PRO>
__global__ __launch_bounds__(256) void gemm_tn_kernel(const float* __restrict__ A, const float* __restrict__ G,
                                                      const float* __restrict__ Zl, float nu,
                                                      float* __restrict__ partial, int64_t n, int K, int C,
                                                      int64_t rows_per_chunk) {
    constexpr int WN = (BN == 128) ? 2 : 1;
    constexpr int WM = 4 / WN;
    constexpr int TM = BM / (WM * 32);
    constexpr int TN = BN / (WN * 32);
    constexpr int LDA = BM + 4;
    constexpr int LDG = BN + 4;
    constexpr int G_F4 = BK * BN / 4;
    constexpr int G_PER_T = (G_F4 + 255) / 256;

    __shared__ __align__(16) float As[BK * LDA];
    __shared__ __align__(16) float Gs[BK * LDG];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int ktiles = (K + BM - 1) / BM;
    const int ctiles = (C + BN - 1) / BN;
    int tile;
    int64_t chunk;
    xcd_group(blockIdx.x, gridDim.x, (unsigned)(ktiles * ctiles), chunk, tile);
    const int k0 = (tile / ctiles) * BM;
    const int c0 = (tile % ctiles) * BN;
    const int64_t r_begin = chunk * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < n) ? (r_begin + rows_per_chunk) : n;
    const bool a_al = (K % 4) == 0;
    const bool g_al = (C % 4) == 0;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    float4 ra[2], rg[G_PER_T];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {              // A tile: 16 rows x 128 k = 512 float4
            const int f = tid + 256 * i;
            const int rr = f >> 5, kq = f & 31;
            const int64_t gr = r0 + rr;
            const int k = k0 + 4 * kq;
            ra[i] = ld4_guard(A, gr * K + k, gr < r_end, a_al, K - k);
        }
#pragma unroll
        for (int i = 0; i < G_PER_T; ++i) {
            const int f = tid + 256 * i;
            if (f < G_F4) {
                const int rr = f / (BN / 4), cq = f % (BN / 4);
                const int64_t gr = r0 + rr;
                const int c = c0 + 4 * cq;
                rg[i] = ld4_guard(G, gr * C + c, gr < r_end, g_al, C - c);
                if constexpr (PRO == 1) {
                    const float4 t = rg[i];
                    const float4 z = ld4_guard(Zl, gr * C + c, gr < r_end, g_al, C - c);
                    rg[i].x = (t.x > 0.f) ? nu * (t.x - z.x) : 0.f;
                    rg[i].y = (t.y > 0.f) ? nu * (t.y - z.y) : 0.f;
                    rg[i].z = (t.z > 0.f) ? nu * (t.z - z.z) : 0.f;
                    rg[i].w = (t.w > 0.f) ? nu * (t.w - z.w) : 0.f;
                }
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int f = tid + 256 * i;
            const int rr = f >> 5, kq = f & 31;
            *reinterpret_cast<float4*>(As + rr * LDA + 4 * kq) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < G_PER_T; ++i) {
            const int f = tid + 256 * i;
            if (f < G_F4) {
                const int rr = f / (BN / 4), cq = f % (BN / 4);
                *reinterpret_cast<float4*>(Gs + rr * LDG + 4 * cq) = rg[i];
            }
        }
    };

    const int li = lane & 31, lk = lane >> 5;
    if (r_begin < r_end) fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += BK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (r0 + BK < r_end) fetch(r0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = As[(kk + lk) * LDA + wm * TM * 32 + i * 32 + li];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Gs[(kk + lk) * LDG + wn * TN * 32 + j * 32 + li];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
    float* dst = partial + chunk * (int64_t)K * C;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int c = c0 + wn * TN * 32 + j * 32 + li;
            if (c >= C) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + wm * TM * 32 + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                if (k < K) dst[(int64_t)k * C + c] = acc[i][j][r];
            }
        }
}

// gemm_tn on the bf16 matrix cores, same three-way split as gemm_nn_split_kernel.  Both operands are contracted
// over the rows, so both tiles are stored transposed (8 consecutive rows of one column per lane and MFMA): a thread
// loads 8 rows of one column, which is coalesced across the threads of a wavefront (consecutive columns).
// PRO 1 forms G = nu (relu(T) - Z) 1[T > 0] from T (passed as G) and Zl while loading.  128 x 128 result tile.
template <int PRO>
__global__ __launch_bounds__(256) void gemm_tn_split_kernel(const float* __restrict__ A, const float* __restrict__ G,
                                                            const float* __restrict__ Zl, float nu,
                                                            float* __restrict__ partial, int64_t n, int K, int C,
                                                            int64_t rows_per_chunk) {
    constexpr int LDH = BK + 8;
    constexpr int PLANE = 128 * LDH;
    __shared__ __align__(16) unsigned short smem[6 * PLANE];
    unsigned short* const As = smem;              // [3][128 columns of A][LDH rows]
    unsigned short* const Gs = smem + 3 * PLANE;  // [3][128 columns of G][LDH rows]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int li = lane & 31, lk = lane >> 5;
    const int ktiles = (K + 127) / 128;
    const int ctiles = (C + 127) / 128;
    int tile;
    int64_t chunk;
    xcd_group(blockIdx.x, gridDim.x, (unsigned)(ktiles * ctiles), chunk, tile);
    const int k0 = (tile / ctiles) * 128;
    const int c0 = (tile % ctiles) * 128;
    const int64_t r_begin = chunk * rows_per_chunk;
    const int64_t r_end = (r_begin + rows_per_chunk < n) ? (r_begin + rows_per_chunk) : n;

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int col = tid & 127, rg = tid >> 7;     // this thread: column `col` of both tiles, rows 8 rg .. 8 rg + 7
    const bool a_on = k0 + col < K, g_on = c0 + col < C;
    float ra[8], rgv[8];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t r = r0 + 8 * rg + e;
            const bool on = r < r_end;
            ra[e] = (on && a_on) ? A[r * K + k0 + col] : 0.f;
            float g = (on && g_on) ? G[r * C + c0 + col] : 0.f;
            if constexpr (PRO == 1) {
                const float z = (on && g_on) ? Zl[r * C + c0 + col] : 0.f;
                g = (g > 0.f) ? nu * (g - z) : 0.f;
            }
            rgv[e] = g;
        }
    };
    auto stash = [&]() {
        unsigned h[4], m[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split3_pair(ra[2 * e], ra[2 * e + 1], h[e], m[e], l[e]);
        const int o = col * LDH + 8 * rg;
        *reinterpret_cast<uint4*>(As + o) = make_uint4(h[0], h[1], h[2], h[3]);
        *reinterpret_cast<uint4*>(As + PLANE + o) = make_uint4(m[0], m[1], m[2], m[3]);
        *reinterpret_cast<uint4*>(As + 2 * PLANE + o) = make_uint4(l[0], l[1], l[2], l[3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) split3_pair(rgv[2 * e], rgv[2 * e + 1], h[e], m[e], l[e]);
        *reinterpret_cast<uint4*>(Gs + o) = make_uint4(h[0], h[1], h[2], h[3]);
        *reinterpret_cast<uint4*>(Gs + PLANE + o) = make_uint4(m[0], m[1], m[2], m[3]);
        *reinterpret_cast<uint4*>(Gs + 2 * PLANE + o) = make_uint4(l[0], l[1], l[2], l[3]);
    };

    auto multiply = [&]() {
        bf16x8 a[3][2];
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[p][i] = *reinterpret_cast<const bf16x8*>(As + p * PLANE + (wm * 64 + i * 32 + li) * LDH + 8 * lk);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            bf16x8 b[3];                             // one column tile's parts at a time keeps the register count down
#pragma unroll
            for (int p = 0; p < 3; ++p)
                b[p] = *reinterpret_cast<const bf16x8*>(Gs + p * PLANE + (wn * 64 + j * 32 + li) * LDH + 8 * lk);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                floatx16 c = acc[i][j];
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2][i], b[0], c, 0, 0, 0);   // small terms first
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[2], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[1], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[0], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[1], c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0], c, 0, 0, 0);
                acc[i][j] = c;
            }
        }
    };
    if (r_begin < r_end) fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += BK) {
        __syncthreads();
        stash();
        __syncthreads();
        if (r0 + BK < r_end) fetch(r0 + BK);
        multiply();
    }
    float* dst = partial + chunk * (int64_t)K * C;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = c0 + wn * 64 + j * 32 + li;
            if (c >= C) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = k0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
                if (k < K) dst[(int64_t)k * C + c] = acc[i][j][r];
            }
        }
}

// Eight lanes share one output entry: lane j adds chunks j, j+8, ... in order, then the eight partial
// sums are added in lane order by a shuffle tree (fixed order, so the result is reproducible).
__global__ __launch_bounds__(256) void gemm_tn_reduce_kernel(const float* __restrict__ partial,
                                                             float* __restrict__ out, int64_t count, int nchunks) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t i = t >> 3;
    const int j = (int)(t & 7);
    double acc = 0.0;
    if (i < count)
        for (int c = j; c < nchunks; c += 8) acc += (double)partial[(int64_t)c * count + i];
    acc += __shfl_xor(acc, 1, 64);
    acc += __shfl_xor(acc, 2, 64);
    acc += __shfl_xor(acc, 4, 64);
    if (i < count && j == 0) out[i] = (float)acc;
}

__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                        int K, int C) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K * C) return;
    const int k = i / C, c = i % C;
    out[c * K + k] = in[i];
}

// Machine calibration: nothing but dependent chains of fp32 MFMAs on registers, four chains per wavefront.
__global__ __launch_bounds__(256) void mfma_chain_kernel(float* __restrict__ out, int iters, float seed) {
    floatx16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    const float a = seed + (float)(threadIdx.x & 7), b = 0.5f * seed;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Machine calibration: chains of bf16 MFMAs (32x32x16) on registers, four chains per wavefront.  With VALU > 0, that
// many independent vector instructions (fused multiply-adds on registers of their own) follow every matrix
// instruction: whether the vector ALU runs beside the matrix cores, and how many instructions fit per matrix instruction.
template <int VALU>
__global__ __launch_bounds__(256) void mfma_bf16_chain_kernel(float* __restrict__ out, int iters, float seed) {
    floatx16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    intx4 a, b;
    a.x = a.y = a.z = a.w = 0x3F803F80 + (int)(threadIdx.x & 7);      // pairs of bf16 near 1
    b.x = b.y = b.z = b.w = 0x3F003F00;
    float v[VALU > 0 ? VALU : 1];
#pragma unroll
    for (int q = 0; q < (VALU > 0 ? VALU : 1); ++q) v[q] = seed + (float)q;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc[j],
                                                             0, 0, 0);
#pragma unroll
            for (int q = 0; q < VALU; ++q) v[q] = __builtin_fmaf(v[q], 0.999f, seed);
            if constexpr (VALU > 0) {
                // keep each matrix instruction and its vector instructions together in the schedule
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, VALU, 0);     // VALU instructions
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
#pragma unroll
    for (int q = 0; q < (VALU > 0 ? VALU : 1); ++q) s += v[q];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Machine calibration: dst = src, one float4 per thread and step.
__global__ __launch_bounds__(256) void stream_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                          int64_t n4) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

// Machine calibration: dst = 0.999 dst + src in place, one float4 per thread and step: two arrays read, one of them
// written back to where it was read, the memory mix of the step kernels.
__global__ __launch_bounds__(256) void stream_update_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                            int64_t n4) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const float4 a = src[i];
        float4 d = dst[i];
        d.x = 0.999f * d.x + a.x; d.y = 0.999f * d.y + a.y; d.z = 0.999f * d.z + a.z; d.w = 0.999f * d.w + a.w;
        dst[i] = d;
    }
}

int g_split = 1;      // 1: wide products run on the bf16 matrix cores with three-way split operands, 0: fp32 MFMA

struct TnPlan {
    int nchunks;
    int64_t rows_per_chunk;
    int bn;
    int tiles;
};

TnPlan tn_plan(int64_t n, int K, int C) {
    TnPlan p;
    p.bn = (C > 32) ? 128 : 32;
    const int ktiles = (K + BM - 1) / BM;
    const int ctiles = (C + p.bn - 1) / p.bn;
    p.tiles = ktiles * ctiles;
    int64_t want = (1024 + p.tiles - 1) / p.tiles;          // about 1024 blocks, four per compute unit
    int64_t max_chunks = (n + 255) / 256;                   // at least 256 rows per chunk
    int64_t nch = want < max_chunks ? want : max_chunks;
    if (nch < 1) nch = 1;
    int64_t rpc = (n + nch - 1) / nch;
    rpc = (rpc + BK - 1) / BK * BK;
    p.rows_per_chunk = rpc;
    p.nchunks = (int)((n + rpc - 1) / rpc);
    if (p.nchunks < 1) p.nchunks = 1;
    return p;
}

}  // namespace

void set_gemm_split(int on) { g_split = on ? 1 : 0; }
int get_gemm_split() { return g_split; }

void launch_gemm_nn(hipStream_t s, const float* A, const float* B, float* out, int64_t n, int K, int C,
                    const GemmEpilogue& epi) {
    if (n <= 0 || C <= 0) return;
    const int64_t mt = (n + BM - 1) / BM;
    if (C > 32) {
        const int ct = (C + 127) / 128;
        dim3 grid((unsigned)(mt * ct));
#define CADMM_NN128(K2_, K1_, K0_) \
        if (epi.kind == 2) \
            hipLaunchKernelGGL(K2_, grid, dim3(256), 0, s, A, B, out, n, K, C, epi.Zl, nullptr, epi.nu, epi.Tio, epi.unit, \
                               epi.partials); \
        else if (epi.kind == 1) \
            hipLaunchKernelGGL(K1_, grid, dim3(256), 0, s, A, B, out, n, K, C, epi.Zl, epi.Tl, epi.nu, nullptr, nullptr, \
                               nullptr); \
        else \
            hipLaunchKernelGGL(K0_, grid, dim3(256), 0, s, A, B, out, n, K, C, nullptr, nullptr, 0.f, nullptr, epi.unit, \
                               nullptr)
        if (g_split) {
            CADMM_NN128((gemm_nn_split_kernel<2>), (gemm_nn_split_kernel<1>), (gemm_nn_split_kernel<0>));
        } else {
            CADMM_NN128((gemm_nn_kernel<128, 2>), (gemm_nn_kernel<128, 1>), (gemm_nn_kernel<128, 0>));
        }
#undef CADMM_NN128
    } else {
        dim3 grid((unsigned)mt);
        if (epi.kind == 1)
            hipLaunchKernelGGL((gemm_nn_kernel<32, 1>), grid, dim3(256), 0, s, A, B, out, n, K, C, epi.Zl, epi.Tl, epi.nu,
                               nullptr, nullptr, nullptr);
        else
            hipLaunchKernelGGL((gemm_nn_kernel<32, 0>), grid, dim3(256), 0, s, A, B, out, n, K, C, nullptr, nullptr, 0.f,
                               nullptr, nullptr, nullptr);
    }
}

void launch_gemm_nn_gradz(hipStream_t s, const float* Zl, const float* Tl, const float* SG, const float* Bcat,
                          float* out, int64_t n, int K1, int K2, int C, float nu) {
    if (n <= 0) return;
    hipLaunchKernelGGL(gemm_nn_gradz_kernel, dim3((unsigned)((n + BM - 1) / BM)), dim3(256), 0, s, Zl, Tl, SG, Bcat, out,
                       n, K1, K2, C, nu);
}

int64_t gemm_nn_blocks(int64_t n, int C) {
    const int64_t mt = (n + BM - 1) / BM;
    return C > 32 ? mt * ((C + 127) / 128) : mt;
}

size_t gemm_tn_scratch_floats(int64_t n, int K, int C) {
    TnPlan p = tn_plan(n, K, C);
    return (size_t)p.nchunks * K * C;
}

void launch_gemm_tn(hipStream_t s, const float* A, const float* G, float* out, int64_t n, int K, int C,
                    float* partial, const float* Zl, float nu) {
    if (K <= 0 || C <= 0) return;
    TnPlan p = tn_plan(n, K, C);
    const dim3 grid((unsigned)((int64_t)p.nchunks * p.tiles)), block(256);
    if (g_split && p.bn == 128) {
        if (Zl) hipLaunchKernelGGL((gemm_tn_split_kernel<1>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
        else hipLaunchKernelGGL((gemm_tn_split_kernel<0>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
    } else if (Zl) {
        if (p.bn == 128)
            hipLaunchKernelGGL((gemm_tn_kernel<128, 1>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
        else
            hipLaunchKernelGGL((gemm_tn_kernel<32, 1>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
    } else {
        if (p.bn == 128)
            hipLaunchKernelGGL((gemm_tn_kernel<128, 0>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
        else
            hipLaunchKernelGGL((gemm_tn_kernel<32, 0>), grid, block, 0, s, A, G, Zl, nu, partial, n, K, C, p.rows_per_chunk);
    }
    const int64_t count = (int64_t)K * C;
    hipLaunchKernelGGL(gemm_tn_reduce_kernel, dim3((unsigned)((count * 8 + 255) / 256)), dim3(256), 0, s, partial, out,
                       count, p.nchunks);
}

double launch_mfma_chain(hipStream_t s, float* out, int blocks, int iters) {
    hipLaunchKernelGGL(mfma_chain_kernel, dim3((unsigned)blocks), dim3(256), 0, s, out, iters, 1.0f);
    return (double)blocks * 4.0 * iters * 4.0 * (32.0 * 32.0 * 2.0 * 2.0);      // flops
}

double launch_mfma_bf16_chain(hipStream_t s, float* out, int blocks, int iters, int valu) {
    if (valu <= 0) hipLaunchKernelGGL((mfma_bf16_chain_kernel<0>), dim3((unsigned)blocks), dim3(256), 0, s, out, iters, 1.0f);
    else if (valu <= 4) hipLaunchKernelGGL((mfma_bf16_chain_kernel<4>), dim3((unsigned)blocks), dim3(256), 0, s, out, iters, 1.0f);
    else if (valu <= 6) hipLaunchKernelGGL((mfma_bf16_chain_kernel<6>), dim3((unsigned)blocks), dim3(256), 0, s, out, iters, 1.0f);
    else hipLaunchKernelGGL((mfma_bf16_chain_kernel<8>), dim3((unsigned)blocks), dim3(256), 0, s, out, iters, 1.0f);
    return (double)blocks * 4.0 * iters * 4.0 * (32.0 * 32.0 * 16.0 * 2.0);      // flops
}

void launch_stream_copy(hipStream_t s, const float* src, float* dst, int64_t count) {
    const int64_t n4 = count / 4;
    hipLaunchKernelGGL(stream_copy_kernel, dim3(8192), dim3(256), 0, s, reinterpret_cast<const float4*>(src),
                       reinterpret_cast<float4*>(dst), n4);
}

void launch_stream_update(hipStream_t s, const float* src, float* dst, int64_t count) {
    hipLaunchKernelGGL(stream_update_kernel, dim3(8192), dim3(256), 0, s, reinterpret_cast<const float4*>(src),
                       reinterpret_cast<float4*>(dst), count / 4);
}

void launch_transpose(hipStream_t s, const float* in, float* out, int K, int C) {
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)((K * C + 255) / 256)), dim3(256), 0, s, in, out, K, C);
}

}  // namespace cadmm
