// Fused elementwise kernels and reductions of the ADMM sweep (gfx950): subproblem values phi / psi and
// their pre-activation gradients, the step-size searches for tau_l (Section 3.1) and theta_{l,m}
// (Appendix A) run entirely on the device, the last-layer solver fused with the dual step (Eq. 5, Eq. 2).
//
// All of these are bound by HBM traffic.  State is fp32; every sum and every quantity that decides a
// step-size test is formed in fp64 from the fp32 inputs (the fp64 vector rate of the chip is far above
// what these memory-bound passes need).  Reductions are two-stage and order-fixed: each block writes its
// partial sums, a finishing kernel adds them in index order, so results are reproducible run to run.
//
// A step-size search is a sequence of passes enqueued by the host without reading anything back: a pass
// evaluates up to kMaxCand candidates step*eta^j in one sweep over memory, the finishing kernel picks the
// first that passes the test  value(step) - value(0) <= -||grad||^2 / (2 step)  and marks the search
// done; later passes see the flag and return at once.
#include "kernels.h"

namespace cadmm {

namespace {

constexpr double kStepFloor = 1e-12;   // a step that moves the block by less than this fraction is not taken

// VEC consecutive floats per lane: 16-byte accesses when the element count allows (VEC = 4), else scalar
template <int VEC>
__device__ __forceinline__ void ldv(float (&d)[VEC], const float* p) {
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    } else {
        d[0] = *p;
    }
}
template <int VEC>
__device__ __forceinline__ void stv(float* p, const float (&d)[VEC]) {
    if constexpr (VEC == 4) *reinterpret_cast<float4*>(p) = make_float4(d[0], d[1], d[2], d[3]);
    else *p = d[0];
}

__device__ __forceinline__ double block_sum(double v, double* sm) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) t += sm[w];
    return t;
}

// slack: the test accepts up to this much above the bound (0 for the tau and theta searches)
__device__ __forceinline__ void decide(Unit* u, const double* D, int ncand, SearchParams sp, int32_t* status,
                                       double slack = 0.0) {
    double step = u->step;
    const double g = u->g;
    int nt = u->ntrials;
    for (int j = 0; j < ncand; ++j) {
        ++nt;
        const double d = D[j];
        if (!(d == d) || fabs(d) > 1.7e308) atomicOr(status, 2);
        if (d <= -g / (2.0 * step) + slack) { u->step = step; u->ntrials = nt; u->done = 1; return; }
        if (nt > sp.max_backtrack) {
            u->step = step; u->ntrials = nt; u->done = 1;
            atomicOr(status, 1);
            return;
        }
        step *= (double)sp.eta;
    }
    u->step = step;
    u->ntrials = nt;
}

// Start of a search, before its first trial: the first candidate is the last accepted value, or that divided by
// eta if the parameters may shrink again.
__device__ __forceinline__ void begin_search(Unit* u, SearchParams sp) {
    u->spec = (u->ntrials == 1) ? 1 : 0;     // last search: first candidate accepted
    u->ntrials = 0;
    u->keep = u->step;
    if (sp.relax) u->step = u->step / (double)sp.eta;
    u->step0 = u->step;
    u->done = 0;
    u->skip = 0;
}

// A step below resolution is not taken: the block and its step parameter stay as they were.
__device__ __forceinline__ void floor_test(Unit* u, double g, double bnorm) {
    u->g = g;
    u->bnorm = bnorm;
    const double lim = kStepFloor * u->step;
    if (g <= lim * lim * bnorm) { u->done = 1; u->skip = 1; u->step = u->keep; }
}

// ------------------------------------------------------------------------------------------ phi and G
// hidden layer:  e = relu(t) - z,  phi += e^2 (scaled nu/2 at the end),  G = nu e 1[t>0]
// last layer:    r = z - t,        phi += u r + rho/2 r^2,               G = -(u + rho r)
// apply_dual (last layer only): first take the dual ascent step U += rho (Z_L - T) on the iterate just
// reached, then evaluate phi and G with the new U.
template <int LAST, int VEC>
__global__ __launch_bounds__(256) void phi_G_kernel(const float* __restrict__ T, const float* __restrict__ Z,
                                                    float* __restrict__ U, float* __restrict__ G,
                                                    float* __restrict__ Tprev, int have_prev, int apply_dual,
                                                    int64_t count, float nu, float rho,
                                                    double* __restrict__ partials) {
    __shared__ double sm[4];
    double s_phi = 0.0, s_res = 0.0, s_dt = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * VEC;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; i < count; i += stride) {
        float t[VEC], z[VEC], g[VEC];
        ldv<VEC>(t, T + i);
        ldv<VEC>(z, Z + i);
        if (LAST) {
            float u[VEC], tp[VEC];
            ldv<VEC>(u, U + i);
            if (Tprev && have_prev) ldv<VEC>(tp, Tprev + i);
            if (apply_dual) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) u[v] = u[v] + rho * (z[v] - t[v]);
                stv<VEC>(U + i, u);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const double r = (double)z[v] - (double)t[v];
                s_phi += (double)u[v] * r + 0.5 * (double)rho * r * r;
                s_res += r * r;
                g[v] = -(u[v] + rho * (z[v] - t[v]));
                if (Tprev && have_prev) { const double d = (double)t[v] - (double)tp[v]; s_dt += d * d; }
            }
            if (Tprev) stv<VEC>(Tprev + i, t);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const double e = (double)fmaxf(t[v], 0.f) - (double)z[v];
                s_phi += e * e;
                g[v] = (t[v] > 0.f) ? nu * (float)e : 0.f;
            }
        }
        if (G) stv<VEC>(G + i, g);
    }
    s_phi = block_sum(s_phi, sm);
    if (LAST) { s_res = block_sum(s_res, sm); s_dt = block_sum(s_dt, sm); }
    if (threadIdx.x == 0) {
        partials[blockIdx.x * 3 + 0] = s_phi;
        partials[blockIdx.x * 3 + 1] = s_res;
        partials[blockIdx.x * 3 + 2] = s_dt;
    }
}

__global__ __launch_bounds__(256) void phi_G_finish_kernel(const double* __restrict__ partials, int nblocks, int last,
                                                           float nu, LayerScalars* out) {
    __shared__ double sm[4];
    double a = 0.0, b = 0.0, c = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += blockDim.x) {
        a += partials[i * 3 + 0];
        b += partials[i * 3 + 1];
        c += partials[i * 3 + 2];
    }
    a = block_sum(a, sm);
    b = block_sum(b, sm);
    c = block_sum(c, sm);
    if (threadIdx.x == 0) {
        out->phi = last ? a : 0.5 * (double)nu * a;
        out->res2 = b;
        out->dT2 = c;
    }
}

template <int LAST, int VEC>
__global__ __launch_bounds__(256) void G_only_kernel(const float* __restrict__ T, const float* __restrict__ Z,
                                                     const float* __restrict__ U, float* __restrict__ G,
                                                     int64_t count, float nu, float rho) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * VEC;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; i < count; i += stride) {
        float t[VEC], z[VEC], g[VEC];
        ldv<VEC>(t, T + i);
        ldv<VEC>(z, Z + i);
        if (LAST) {
            float u[VEC];
            ldv<VEC>(u, U + i);
#pragma unroll
            for (int v = 0; v < VEC; ++v) g[v] = -(u[v] + rho * (z[v] - t[v]));
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) g[v] = (t[v] > 0.f) ? nu * (float)((double)t[v] - (double)z[v]) : 0.f;
        }
        stv<VEC>(G + i, g);
    }
}

// ------------------------------------------------------------------------------------------ risk
__global__ __launch_bounds__(256) void risk_kernel(const float* __restrict__ ZL, const int32_t* __restrict__ labels,
                                                   int64_t N, int CL, int risk, double* __restrict__ partials) {
    __shared__ double sm[4];
    double s = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N; i += stride) {
        const int y = labels[i];
        if (y < 0) continue;
        const float* z = ZL + i * CL;
        if (risk == 0) {
            double mx = (double)z[0];
            for (int c = 1; c < CL; ++c) mx = fmax(mx, (double)z[c]);
            double se = 0.0;
            for (int c = 0; c < CL; ++c) se += exp((double)z[c] - mx);
            s += mx + log(se) - (double)z[y];
        } else {
            for (int c = 0; c < CL; ++c) {
                const double d = (double)z[c] - (c == y ? 1.0 : 0.0);
                s += 0.5 * d * d;
            }
        }
    }
    s = block_sum(s, sm);
    if (threadIdx.x == 0) partials[blockIdx.x] = s;
}

__global__ __launch_bounds__(256) void risk_finish_kernel(const double* __restrict__ partials, int nblocks,
                                                          LayerScalars* out) {
    __shared__ double sm[4];
    double a = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += blockDim.x) a += partials[i];
    a = block_sum(a, sm);
    if (threadIdx.x == 0) out->risk = a;
}

// ------------------------------------------------------------------------------------------ W search
// ||gradW||^2 and ||W||^2: per-block partial sums, then one block adds them in order and starts the search.
__global__ __launch_bounds__(256) void w_norms_kernel(const float* __restrict__ gradW, const float* __restrict__ W,
                                                      int count, double* __restrict__ partials) {
    __shared__ double sm[4];
    double g = 0.0, b = 0.0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) {
        const double x = (double)gradW[i], w = (double)W[i];
        g += x * x;
        b += w * w;
    }
    g = block_sum(g, sm);
    b = block_sum(b, sm);
    if (threadIdx.x == 0) { partials[2 * blockIdx.x] = g; partials[2 * blockIdx.x + 1] = b; }
}

__global__ __launch_bounds__(64) void w_norms_finish_kernel(const double* __restrict__ partials, int nblocks,
                                                            Unit* unit, SearchParams sp) {
    if (threadIdx.x != 0) return;
    double g = 0.0, b = 0.0;
    for (int i = 0; i < nblocks; ++i) { g += partials[2 * i]; b += partials[2 * i + 1]; }
    begin_search(unit, sp);
    floor_test(unit, g, b);
}

template <int LAST, int NC, int VEC>
__global__ __launch_bounds__(256) void w_trial_kernel(const float* __restrict__ T0, const float* __restrict__ Q,
                                                      const float* __restrict__ Z, const float* __restrict__ U,
                                                      int64_t count, SearchParams sp, const Unit* unit,
                                                      double* __restrict__ partials, int speculated) {
    __shared__ double sm[4];
    if (unit->done) return;
    const double spec_inv = (speculated && unit->spec) ? 1.0 / unit->step0 : 0.0;      // T0 holds T0 - Q/step0: undo
    double inv[NC];
    {
        double step = unit->step;
#pragma unroll
        for (int j = 0; j < NC; ++j) { inv[j] = 1.0 / step; step *= (double)sp.eta; }
    }
    double D[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) D[j] = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * VEC;
    for (int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC; i < count; i += stride) {
        float t0v[VEC], qv[VEC], zv[VEC], uv[VEC];
        ldv<VEC>(t0v, T0 + i);
        ldv<VEC>(qv, Q + i);
        ldv<VEC>(zv, Z + i);
        if (LAST) ldv<VEC>(uv, U + i);
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const double q = (double)qv[v], z = (double)zv[v];
            const double t0 = (double)t0v[v] + q * spec_inv;
            if (LAST) {
                const double u = (double)uv[v];
                const double r0 = z - t0;
#pragma unroll
                for (int j = 0; j < NC; ++j) {
                    const double dq = q * inv[j];          // r_new - r_old
                    D[j] += dq * (u + 0.5 * (double)sp.rho * (2.0 * r0 + dq));
                }
            } else {
                const double e0 = fmax(t0, 0.0) - z;
#pragma unroll
                for (int j = 0; j < NC; ++j) {
                    const double e1 = fmax(t0 - q * inv[j], 0.0) - z;
                    D[j] += (e1 - e0) * (e1 + e0);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const double s = block_sum(D[j], sm);
        if (threadIdx.x == 0) partials[blockIdx.x * kMaxCand + j] = LAST ? s : 0.5 * (double)sp.nu * s;
    }
}

__global__ __launch_bounds__(256) void w_trial_finish_kernel(const double* __restrict__ partials, int nblocks,
                                                             int stride, int ncand, SearchParams sp, Unit* unit,
                                                             int32_t* status) {
    __shared__ double sm[4];
    __shared__ double D[kMaxCand];
    if (unit->done) return;
    for (int j = 0; j < ncand; ++j) {
        double a = 0.0, b = 0.0, c = 0.0, d = 0.0;     // four independent loads in flight per thread
        int i = threadIdx.x;
        for (; i + 768 < nblocks; i += 1024) {
            a += partials[(int64_t)i * stride + j];
            b += partials[(int64_t)(i + 256) * stride + j];
            c += partials[(int64_t)(i + 512) * stride + j];
            d += partials[(int64_t)(i + 768) * stride + j];
        }
        for (; i < nblocks; i += 256) a += partials[(int64_t)i * stride + j];
        a = (a + b) + (c + d);
        a = block_sum(a, sm);
        if (threadIdx.x == 0) D[j] = a;
    }
    __syncthreads();
    if (threadIdx.x == 0) decide(unit, D, ncand, sp, status);
}

template <int VEC>
__global__ __launch_bounds__(256) void w_step_kernel(float* __restrict__ W, const float* __restrict__ gradW,
                                                     int count_w, float* __restrict__ T, const float* __restrict__ Q,
                                                     int64_t count_t, const Unit* unit, int speculated) {
    if (unit->skip) return;
    const double inv = 1.0 / unit->step;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t nthreads = (int64_t)gridDim.x * blockDim.x;
    // T already holds T0 - Q/step0 when the step was taken speculatively: nothing to do if step0 was accepted,
    // otherwise T0 - Q/step = T + Q (1/step0 - 1/step)
    const bool spec = speculated && unit->spec;
    const double tinv = spec ? inv - 1.0 / unit->step0 : inv;
    const bool t_done = spec && unit->step == unit->step0;
    for (int64_t i = gtid * VEC; !t_done && i < count_t; i += nthreads * VEC) {
        float t[VEC], q[VEC];
        ldv<VEC>(t, T + i);
        ldv<VEC>(q, Q + i);
#pragma unroll
        for (int v = 0; v < VEC; ++v) t[v] = (float)((double)t[v] - (double)q[v] * tinv);
        stv<VEC>(T + i, t);
    }
    for (int64_t i = gtid; i < count_w; i += nthreads) W[i] = (float)((double)W[i] - (double)gradW[i] * inv);
}

// ------------------------------------------------------------------------------------------ Z search
// One block per chunk.  kind 0: rows [begin,end) of community `unit`, own term
//     nu/2 ||Z - relu(T_l)||^2  under  Z -> Z - gradZ/theta;
// kind 1: segments [begin,end) (community,row order) of the next layer's term, whose pre-activation
//     row T_{l+1,i} moves by -P_s/theta as seen from this community.
// grad[v] = nu (z[v] - relu(t[v])) + sum_k sg[k] wt[k][v], always in this order (the step kernel must
// reproduce the very same values the search saw).  The rows of W_{l+1}^T are read from LDS (wcol: this lane's four
// columns of row 0, wv float4 per row): the kernels that rebuild the gradient stream N x C_l matrices and need the
// wavefronts in flight that 64 registers per lane for these rows would cost them.
__device__ __forceinline__ void lowrank_grad_lds(float (&g)[4], const float (&z)[4], const float (&t)[4],
                                                 const float (&sg)[kLowRankMax], const float4* wcol, int wv, int Cn, float nu) {
#pragma unroll
    for (int v = 0; v < 4; ++v) g[v] = nu * (z[v] - fmaxf(t[v], 0.f));
#pragma unroll
    for (int k = 0; k < kLowRankMax; ++k) {
        if (k < Cn) {
            const float4 w4 = wcol[k * wv];
            g[0] = fmaf(sg[k], w4.x, g[0]); g[1] = fmaf(sg[k], w4.y, g[1]);
            g[2] = fmaf(sg[k], w4.z, g[2]); g[3] = fmaf(sg[k], w4.w, g[3]);
        }
    }
}

// s_wt: LDS room for W_{l+1}^T (LR only); wt_loaded: whether this workgroup has filled it already.
template <int NC, int VEC, int LR>
__device__ __forceinline__ void z_trial_chunk(const ZTrialArgs& a, int ch, double* sm, float* s_wt, bool& wt_loaded) {
    const int unit = a.chunk_unit[ch];
    const Unit* u = a.units + unit;
    if (u->done) return;
    const int kind = a.chunk_kind[ch];
    if (LR == 1 && kind == 0 && !wt_loaded) {           // (uniform over the workgroup)
        for (int i = threadIdx.x; i < a.Cn * a.Cl; i += 256) s_wt[i] = a.Wt[i];
        __syncthreads();
        wt_loaded = true;
    }
    const int begin = a.chunk_begin[ch], end = a.chunk_end[ch];
    double inv[NC];
    {
        double step = u->step;
#pragma unroll
        for (int j = 0; j < NC; ++j) { inv[j] = 1.0 / step; step *= (double)a.sp.eta; }
    }
    double D[NC];
#pragma unroll
    for (int j = 0; j < NC; ++j) D[j] = 0.0;
    double sg = 0.0, sb = 0.0;
    const int width = kind == 0 ? a.Cl : a.Cn;
    const int wv = (width + VEC - 1) / VEC;       // lane slots per row
    int cshift = 0;
    while ((1 << cshift) < wv && cshift < 8) ++cshift;
    const int cp = 1 << cshift;
    const int c_first = threadIdx.x & (cp - 1);
    const int r_first = threadIdx.x >> cshift;
    const int r_step = 256 >> cshift;
    const double hnu = 0.5 * (double)a.sp.nu, hrho = 0.5 * (double)a.sp.rho;
    if (kind == 0) {
        // low-rank gradient: this thread's four columns of W_{l+1}^T, read from LDS (one column slot per thread)
        const float4* const wcol = reinterpret_cast<const float4*>(s_wt) + (c_first < wv ? c_first : 0);
        for (int r = begin + r_first; r < end; r += r_step) {
            const int64_t base = (int64_t)r * width;
            float srow[LR ? kLowRankMax : 1];      // this row of the N x Cn factor
            if constexpr (LR == 1) {
#pragma unroll
                for (int k4 = 0; k4 < kLowRankMax / 4; ++k4) {
                    float q[4] = {0.f, 0.f, 0.f, 0.f};
                    if (4 * k4 < a.Cn) ldv<4>(q, a.SG + (int64_t)r * a.Cn + 4 * k4);
                    srow[4 * k4] = q[0]; srow[4 * k4 + 1] = q[1]; srow[4 * k4 + 2] = q[2]; srow[4 * k4 + 3] = q[3];
                }
            }
            for (int cv = c_first; cv < wv; cv += cp) {
                float zv[VEC], gv[VEC], tv[VEC];
                ldv<VEC>(zv, a.Zl + base + cv * VEC);
                ldv<VEC>(tv, a.Tl + base + cv * VEC);
                if constexpr (LR == 1) lowrank_grad_lds(gv, zv, tv, srow, wcol, wv, a.Cn, a.sp.nu);
                else ldv<VEC>(gv, a.gradZ + base + cv * VEC);
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double z = (double)zv[v], gz = (double)gv[v], t = (double)tv[v];
                    const double e0 = z - fmax(t, 0.0);
                    if (a.first_pass) { sg += gz * gz; sb += z * z; }
#pragma unroll
                    for (int j = 0; j < NC; ++j) {
                        const double dz = -gz * inv[j];
                        D[j] += hnu * dz * (2.0 * e0 + dz);
                    }
                }
            }
        }
    } else {
        for (int s = begin + r_first; s < end; s += r_step) {
            const int64_t row = a.segc_row[s];
            const int64_t base = row * width, pbase = (int64_t)s * width;
            for (int cv = c_first; cv < wv; cv += cp) {
                float tv[VEC], zv[VEC], pv[VEC];
                ldv<VEC>(pv, a.P + pbase + cv * VEC);
                if (a.next_is_last) {
                    // the change of <U, Z_L - T> + rho/2 |Z_L - T|^2 under T -> T - p/theta is
                    // (p/theta) (u + rho (z - t)) + rho/2 (p/theta)^2, and u + rho (z - t) = -G_L is at hand
                    ldv<VEC>(tv, a.Gn + base + cv * VEC);
                } else {
                    ldv<VEC>(tv, a.Tn + base + cv * VEC);
                    ldv<VEC>(zv, a.Zn + base + cv * VEC);
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const double t0 = (double)tv[v], z = (double)zv[v], p = (double)pv[v];
                    if (a.next_is_last) {
#pragma unroll
                        for (int j = 0; j < NC; ++j) {
                            const double dq = p * inv[j];
                            D[j] += dq * (hrho * dq - t0);
                        }
                    } else {
                        const double e0 = fmax(t0, 0.0) - z;
#pragma unroll
                        for (int j = 0; j < NC; ++j) {
                            const double e1 = fmax(t0 - p * inv[j], 0.0) - z;
                            D[j] += hnu * (e1 - e0) * (e1 + e0);
                        }
                    }
                }
            }
        }
    }
    double* out = a.partials + (int64_t)ch * (kMaxCand + 2);
#pragma unroll
    for (int j = 0; j < NC; ++j) {
        const double s = block_sum(D[j], sm);
        if (threadIdx.x == 0) out[j] = s;
    }
    if (a.first_pass) {
        sg = block_sum(sg, sm);
        sb = block_sum(sb, sm);
        if (threadIdx.x == 0) { out[kMaxCand] = sg; out[kMaxCand + 1] = sb; }
    }
}

// The first pass (one candidate) runs one block per chunk.  A later pass (NC candidates) usually finds every
// community done: each block first looks at all the done flags at once and leaves if nothing is pending,
// otherwise a small grid strides over the chunks.
template <int NC, int VEC, int LR>
__global__ __launch_bounds__(256) void z_trial_kernel(ZTrialArgs a) {
    __shared__ double sm[4];
    extern __shared__ __align__(16) float s_wt[];       // [Cn][Cl] with the low-rank gradient, else nothing
    bool wt_loaded = false;
    if constexpr (NC == 1) {
        z_trial_chunk<NC, VEC, LR>(a, blockIdx.x, sm, s_wt, wt_loaded);
    } else {
        int pending = 0;
        for (int i = threadIdx.x; i < a.M; i += 256) pending |= (a.units[i].done == 0);
        if (!__syncthreads_or(pending)) return;
        for (int ch = blockIdx.x; ch < a.n_chunks; ch += gridDim.x) z_trial_chunk<NC, VEC, LR>(a, ch, sm, s_wt, wt_loaded);
    }
}

__global__ __launch_bounds__(256) void z_trial_finish_kernel(ZTrialArgs a) {
    __shared__ double sm[4];
    __shared__ double D[kMaxCand + 2];
    const int unit = blockIdx.x;
    Unit* u = a.units + unit;
    if (u->done) return;
    const int c0 = a.unit_chunk_ptr[unit], c1 = a.unit_chunk_ptr[unit + 1];
    const int nq = a.first_pass ? kMaxCand + 2 : a.ncand;
    for (int q = 0; q < nq; ++q) {
        if (q >= a.ncand && q < kMaxCand) continue;
        double s = 0.0;
        for (int i = c0 + threadIdx.x; i < c1; i += blockDim.x) s += a.partials[(int64_t)i * (kMaxCand + 2) + q];
        s = block_sum(s, sm);
        if (threadIdx.x == 0) D[q] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (a.first_pass) {
            floor_test(u, D[kMaxCand], D[kMaxCand + 1]);      // the search began in reset_units_kernel
            if (u->done) return;
        }
        decide(u, D, a.ncand, a.sp, a.status);
    }
}

constexpr int kStepUnits = 1024;       // communities whose 1/theta a workgroup keeps in LDS
// Z_{l,m} <- Z_{l,m} - grad / theta_{l,m}.  LDSU: 1/theta of every community (0 where no step is taken) is copied
// to LDS first and the loads of a row are issued before its community is known: the row's community, then its step
// parameter, then the data used to be three dependent round trips per row.
template <int VEC, bool LDSU>
__global__ __launch_bounds__(256) void z_step_kernel(float* __restrict__ Zl, const float* __restrict__ gradZ,
                                                     const int32_t* __restrict__ row_comm, int64_t N, int Cl,
                                                     const Unit* __restrict__ units, int M) {
    __shared__ double s_inv[LDSU ? kStepUnits : 1];
    if constexpr (LDSU) {
        for (int i = threadIdx.x; i < M; i += 256) s_inv[i] = units[i].skip ? 0.0 : 1.0 / units[i].step;
        __syncthreads();
    }
    const int wv = (Cl + VEC - 1) / VEC;
    int cshift = 0;
    while ((1 << cshift) < wv && cshift < 8) ++cshift;
    const int cp = 1 << cshift;
    const int c_first = threadIdx.x & (cp - 1);
    const int64_t r_step = (int64_t)gridDim.x * (256 >> cshift);
    for (int64_t r = (int64_t)blockIdx.x * (256 >> cshift) + (threadIdx.x >> cshift); r < N; r += r_step) {
        const int cm = row_comm[r];
        const int64_t base = r * Cl;
        for (int cv = c_first; cv < wv; cv += cp) {
            float z[VEC], g[VEC];
            ldv<VEC>(z, Zl + base + cv * VEC);
            ldv<VEC>(g, gradZ + base + cv * VEC);
            double inv;
            if constexpr (LDSU) inv = s_inv[cm];
            else inv = units[cm].skip ? 0.0 : 1.0 / units[cm].step;
            if (inv == 0.0) break;                   // no step for this row's community
#pragma unroll
            for (int v = 0; v < VEC; ++v) z[v] = (float)((double)z[v] - (double)g[v] * inv);
            stv<VEC>(Zl + base + cv * VEC, z);
        }
    }
}

// The same step with the gradient rebuilt from its low-rank form (see lowrank_grad_lds: the same operations in the
// same order); a lane group handles two rows per trip with every load issued before the first use.  The rows of W_{l+1}^T
// live in LDS, not in 64 registers per lane: the kernel is a plain in-place update of Z_l and needs the wavefronts in
// flight that a small register footprint allows (5 TB/s against 4.4 with the rows in registers).
template <bool LDSU>
__global__ __launch_bounds__(256) void z_step_lowrank_kernel(float* __restrict__ Zl, const float* __restrict__ Tl,
                                                             const float* __restrict__ SG, const float* __restrict__ Wt,
                                                             float nu, const int32_t* __restrict__ row_comm, int64_t N,
                                                             int Cl, int Cn, const Unit* __restrict__ units, int M) {
    __shared__ double s_inv[LDSU ? kStepUnits : 1];
    extern __shared__ __align__(16) float s_wt[];        // [Cn][Cl]
    if constexpr (LDSU) {
        for (int i = threadIdx.x; i < M; i += 256) s_inv[i] = units[i].skip ? 0.0 : 1.0 / units[i].step;
    }
    for (int i = threadIdx.x; i < Cn * Cl; i += 256) s_wt[i] = Wt[i];
    __syncthreads();
    const int wv = Cl / 4;
    int cshift = 0;
    while ((1 << cshift) < wv && cshift < 8) ++cshift;
    const int c_first = threadIdx.x & ((1 << cshift) - 1);
    if (c_first >= wv) return;                       // (after the barrier)
    const float4* const wcol = reinterpret_cast<const float4*>(s_wt) + c_first;      // row k: wcol[k * wv]
    constexpr int R = 2;
    const int64_t rows_per_block = 256 >> cshift;
    const int64_t r_step = (int64_t)gridDim.x * rows_per_block * R;
    for (int64_t r0 = ((int64_t)blockIdx.x * R) * rows_per_block + (threadIdx.x >> cshift); r0 < N; r0 += r_step) {
        int cm[R];
        float z[R][4], t[R][4], sg[R][kLowRankMax];
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int64_t r = r0 + q * rows_per_block;
            const int64_t rr = r < N ? r : N - 1;    // a row past the end repeats the last one and is not stored
            cm[q] = row_comm[rr];
            const int64_t o = rr * Cl + c_first * 4;
            ldv<4>(z[q], Zl + o);
            ldv<4>(t[q], Tl + o);
#pragma unroll
            for (int k4 = 0; k4 < kLowRankMax / 4; ++k4) {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if (4 * k4 < Cn) ldv<4>(v, SG + rr * Cn + 4 * k4);
                sg[q][4 * k4] = v[0]; sg[q][4 * k4 + 1] = v[1]; sg[q][4 * k4 + 2] = v[2]; sg[q][4 * k4 + 3] = v[3];
            }
        }
        float g[R][4];
#pragma unroll
        for (int q = 0; q < R; ++q)
#pragma unroll
            for (int v = 0; v < 4; ++v) g[q][v] = nu * (z[q][v] - fmaxf(t[q][v], 0.f));
#pragma unroll
        for (int k = 0; k < kLowRankMax; ++k) {
            if (k < Cn) {
                const float4 w4 = wcol[k * wv];
                const float w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                for (int q = 0; q < R; ++q)
#pragma unroll
                    for (int v = 0; v < 4; ++v) g[q][v] = fmaf(sg[q][k], w[v], g[q][v]);
            }
        }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int64_t r = r0 + q * rows_per_block;
            double inv;
            if constexpr (LDSU) inv = s_inv[cm[q]];
            else inv = units[cm[q]].skip ? 0.0 : 1.0 / units[cm[q]].step;
            if (r >= N || inv == 0.0) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) z[q][v] = (float)((double)z[q][v] - (double)g[q][v] * inv);
            stv<4>(Zl + r * Cl + c_first * 4, z[q]);
        }
    }
}

// After Z_{l,m} <- Z_{l,m} - grad/theta_{l,m} the next layer's pre-activation A~ Z_l W_{l+1} of row i changes by
// - sum over the segments (i, c) of P_{(i,c)} / theta_{l,c}  (P = A~_{., c} grad W_{l+1}, already formed for the
// search).  Applying that keeps T_{l+1} valid for the next iteration without a new aggregation and product.
constexpr int kCarryBatch = 4;
constexpr int kCarryUnits = 1024;      // communities whose 1/theta a workgroup keeps in LDS
// LDSU: the workgroup first copies 1/theta of every community (0 for a skipped step) into LDS, which takes the
// lookup of a segment's step parameter out of the chain of dependent global loads (row -> segment -> unit).
template <int VEC, bool LDSU>
__global__ __launch_bounds__(256) void t_carry_kernel(float* __restrict__ Tn, const float* __restrict__ P,
                                                      const int64_t* __restrict__ row_seg_ptr,
                                                      const int32_t* __restrict__ seg_comm,
                                                      const int32_t* __restrict__ seg_pos, int64_t N, int Cn,
                                                      const Unit* __restrict__ units, int M) {
    __shared__ double s_inv[LDSU ? kCarryUnits : 1];
    if constexpr (LDSU) {
        for (int i = threadIdx.x; i < M; i += 256) s_inv[i] = units[i].skip ? 0.0 : 1.0 / units[i].step;
        __syncthreads();
    }
    const int wv = (Cn + VEC - 1) / VEC;
    int cshift = 0;
    while ((1 << cshift) < wv && cshift < 8) ++cshift;
    const int cp = 1 << cshift;
    const int c_first = threadIdx.x & (cp - 1);
    const int64_t r_step = (int64_t)gridDim.x * (256 >> cshift);
    for (int64_t r = (int64_t)blockIdx.x * (256 >> cshift) + (threadIdx.x >> cshift); r < N; r += r_step) {
        const int64_t s0 = row_seg_ptr[r], s1 = row_seg_ptr[r + 1];
        for (int cv = c_first; cv < wv; cv += cp) {
            double acc[VEC];
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = 0.0;
            bool any = false;
            // kCarryBatch segments at a time: their index, unit and row loads do not depend on each other, so they
            // are in flight together; the sums are still taken in segment order.
            for (int64_t sgm = s0; sgm < s1; sgm += kCarryBatch) {
                int cm[kCarryBatch], ps[kCarryBatch];
#pragma unroll
                for (int j = 0; j < kCarryBatch; ++j) {
                    const int64_t sj = sgm + j < s1 ? sgm + j : s1 - 1;
                    cm[j] = seg_comm[sj];
                    ps[j] = seg_pos[sj];
                }
                double inv[kCarryBatch];
                float p[kCarryBatch][VEC];
#pragma unroll
                for (int j = 0; j < kCarryBatch; ++j) {
                    if constexpr (LDSU) {
                        inv[j] = s_inv[cm[j]];
                    } else {
                        const Unit* u = units + cm[j];
                        inv[j] = u->skip ? 0.0 : 1.0 / u->step;
                    }
                    if (sgm + j >= s1) inv[j] = 0.0;
                    ldv<VEC>(p[j], P + (int64_t)ps[j] * Cn + cv * VEC);
                }
#pragma unroll
                for (int j = 0; j < kCarryBatch; ++j) {
                    if (inv[j] == 0.0) continue;          // past the row's end, or a step that was not taken
                    any = true;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[v] += (double)p[j][v] * inv[j];
                }
            }
            if (!any) continue;
            float t[VEC];
            ldv<VEC>(t, Tn + r * Cn + cv * VEC);
#pragma unroll
            for (int v = 0; v < VEC; ++v) t[v] = (float)((double)t[v] - acc[v]);
            stv<VEC>(Tn + r * Cn + cv * VEC, t);
        }
    }
}

// ------------------------------------------------------------------------------------------ last layer + dual
// 2^LPLOG lanes share one node row, four classes per lane, so a wavefront reads whole 64-byte-aligned
// pieces of consecutive rows with 16-byte accesses; the row maximum and the softmax denominator are
// formed by xor-shuffles inside the lane group.  FISTA on
//   R(z, y_i) + <u, z - c> + rho/2 ||z - c||^2,   c = row of A~ Z_{L-1}^k W_L^{k+1},
// whose smooth part is the whole objective: x_j = y_j - grad(y_j)/Lip, Lip = rho + (1/2 | 1).
template <int LPLOG>
__global__ __launch_bounds__(256) void last_layer_kernel(float* __restrict__ ZL, float* __restrict__ U,
                                                         const float* __restrict__ TL,
                                                         const int32_t* __restrict__ labels, int64_t N, int CL,
                                                         int risk, float rho, int J, int update_u) {
    constexpr int LP = 1 << LPLOG;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = t >> LPLOG;
    const int j0 = (int)(t & (LP - 1)) * 4;
    const bool act = row < N;                       // uniform over the lane group of a row
    const int64_t base = (act ? row : 0) * CL + j0;
    const bool vec = (CL % 4) == 0;
    bool ok[4];
    float c[4], u[4], xp[4], y[4], x[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) ok[v] = act && (j0 + v < CL);
    if (vec && ok[0]) {
        const float4 a = *reinterpret_cast<const float4*>(TL + base);
        const float4 b = *reinterpret_cast<const float4*>(U + base);
        const float4 d = *reinterpret_cast<const float4*>(ZL + base);
        c[0] = a.x; c[1] = a.y; c[2] = a.z; c[3] = a.w;
        u[0] = b.x; u[1] = b.y; u[2] = b.z; u[3] = b.w;
        xp[0] = d.x; xp[1] = d.y; xp[2] = d.z; xp[3] = d.w;
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            c[v] = ok[v] ? TL[base + v] : 0.f;
            u[v] = ok[v] ? U[base + v] : 0.f;
            xp[v] = ok[v] ? ZL[base + v] : 0.f;
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) { y[v] = xp[v]; x[v] = xp[v]; }
    // dual step with the iterates as printed in Eq. 2: Z_L^k and the aggregation with W_L^{k+1}
    float un[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) un[v] = u[v] + rho * (xp[v] - c[v]);
    const int lab = act ? labels[row] : -1;
    if (lab < 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = c[v] - u[v] / rho;       // exact minimiser of the quadratic
    } else {
        const float inv_lip = 1.0f / (rho + (risk == 0 ? 0.5f : 1.0f));
        float tk = 1.0f;
        for (int it = 0; it < J; ++it) {
            float g[4];
            if (risk == 0) {
                float mx = -3.0e38f;
#pragma unroll
                for (int v = 0; v < 4; ++v) mx = ok[v] ? fmaxf(mx, y[v]) : mx;
#pragma unroll
                for (int o = 1; o < LP; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
                float se = 0.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) { g[v] = ok[v] ? __expf(y[v] - mx) : 0.f; se += g[v]; }
#pragma unroll
                for (int o = 1; o < LP; o <<= 1) se += __shfl_xor(se, o, 64);
                const float inv_se = 1.0f / se;
#pragma unroll
                for (int v = 0; v < 4; ++v) g[v] = g[v] * inv_se - ((j0 + v) == lab ? 1.f : 0.f);
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v) g[v] = y[v] - ((j0 + v) == lab ? 1.f : 0.f);
            }
            const float tn = 0.5f * (1.0f + sqrtf(1.0f + 4.0f * tk * tk));
            const float mom = (tk - 1.0f) / tn;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float grad = g[v] + u[v] + rho * (y[v] - c[v]);
                x[v] = y[v] - grad * inv_lip;
                y[v] = x[v] + mom * (x[v] - xp[v]);
                xp[v] = x[v];
            }
            tk = tn;
        }
    }
    if (vec && ok[0]) {
        if (update_u) *reinterpret_cast<float4*>(U + base) = make_float4(un[0], un[1], un[2], un[3]);
        *reinterpret_cast<float4*>(ZL + base) = make_float4(x[0], x[1], x[2], x[3]);
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (ok[v]) {
                if (update_u) U[base + v] = un[v];
                ZL[base + v] = x[v];
            }
    }
}

__global__ __launch_bounds__(256) void relu_kernel(const float* __restrict__ T, float* __restrict__ Z, int64_t count,
                                                   int apply_relu) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
        Z[i] = apply_relu ? fmaxf(T[i], 0.f) : T[i];
}

// class of every node: index of the largest entry of its row (the first one on equal values)
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float* __restrict__ T, int32_t* __restrict__ pred,
                                                          int64_t N, int C) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const float* t = T + i * C;
    int best = 0;
    float bv = t[0];
    for (int c = 1; c < C; ++c)
        if (t[c] > bv) { bv = t[c]; best = c; }
    pred[i] = best;
}

// ------------------------------------------------------------------------------------------ last layer, FISTA with backtracking
// See FistaArgs.  2^LPLOG lanes share a node row, four classes per lane, as in last_layer_kernel; a workgroup takes one
// chunk of rows of one community.  Everything that enters a decision is formed in fp64 from the fp32 state: the
// gradient g of F(z) = R(z, y) + <u, z - c> + rho/2 ||z - c||^2 at y, and for a candidate L the difference
// F(y - g/L) - F(y), term by term (the log-sum-exp of both points, the linear and the quadratic terms through
// x - y = -g/L), so that nothing is lost to the cancellation of two nearly equal values of F.
constexpr int kFistaStride = kMaxCand + 3;        // per chunk: candidate differences, ||g||^2, ||y||^2, F(y)
constexpr double kFistaSlack = 1e-12;             // the test accepts up to this relative rounding of F(y)

template <int LPLOG>
__device__ __forceinline__ double group_sum(double v) {
#pragma unroll
    for (int o = 1; o < (1 << LPLOG); o <<= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int LPLOG>
__device__ __forceinline__ double group_max(double v) {
#pragma unroll
    for (int o = 1; o < (1 << LPLOG); o <<= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}

// log-sum-exp over the row (the lanes of the group hold four entries each; entries past CL are off)
template <int LPLOG>
__device__ __forceinline__ double row_lse(const double (&z)[4], const bool (&ok)[4], double (&e)[4], double& se) {
    double mx = -1.0e300;
#pragma unroll
    for (int v = 0; v < 4; ++v) mx = ok[v] ? fmax(mx, z[v]) : mx;
    mx = group_max<LPLOG>(mx);
    double s = 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) { e[v] = ok[v] ? exp(z[v] - mx) : 0.0; s += e[v]; }
    se = group_sum<LPLOG>(s);
    return mx + log(se);
}

template <int LPLOG, int NC>
__global__ __launch_bounds__(256) void fista_stage_kernel(FistaArgs a, int stage, int more, float mom) {
    __shared__ double sm[4];
    constexpr int LP = 1 << LPLOG;
    if (more) {                                        // a pass of further candidates: only if some search is pending
        int pending = 0;
        for (int i = threadIdx.x; i < a.M; i += 256) pending |= (a.units[i].done == 0);
        if (!__syncthreads_or(pending)) return;
    }
    for (int ch = blockIdx.x; ch < a.n_chunks; ch += gridDim.x) {
        if (a.chunk_kind[ch] != 0) continue;           // only the chunks of rows
        const Unit* u = a.units + a.chunk_unit[ch];
        if (more && u->done) continue;
        const double Lcur = (stage == 0 && !more) ? (double)a.rho : u->step;       // every solve starts from L = rho
        const bool skipped = stage > 0 && !more && u->skip;
        const int r0 = a.chunk_begin[ch], r1 = a.chunk_end[ch];
        double D[NC], sgg = 0.0, syy = 0.0, sF = 0.0;
#pragma unroll
        for (int q = 0; q < NC; ++q) D[q] = 0.0;
        for (int rb = r0; rb < r1; rb += 256 >> LPLOG) {
            const int row = rb + (threadIdx.x >> LPLOG);
            const int j0 = (threadIdx.x & (LP - 1)) * 4;
            const bool act = row < r1;
            const int64_t base = (int64_t)(act ? row : r0) * a.CL + j0;
            bool ok[4];
            double c[4], uu[4], y[4], xo[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                ok[v] = act && (j0 + v < a.CL);
                c[v] = ok[v] ? (double)a.TL[base + v] : 0.0;
                uu[v] = ok[v] ? (double)a.U[base + v] : 0.0;
                // y_{stage-1} and x_{stage-1}; both are Z_L before the first step
                y[v] = ok[v] ? (double)((stage <= 1 && !more) || stage == 0 ? a.ZL[base + v] : a.Yb[base + v]) : 0.0;
                xo[v] = ok[v] ? (double)(stage <= 1 ? a.ZL[base + v] : a.Xb[base + v]) : 0.0;
            }
            const int lab = act ? a.labels[row] : -1;
            const bool on = lab >= 0;                  // uniform over the lane group; rows without label are no part of F
            double e[4], se, g[4];
            auto gradient = [&](const double (&z)[4], double& lse) {
                lse = 0.0;
                if (a.risk == 0) {
                    lse = row_lse<LPLOG>(z, ok, e, se);
#pragma unroll
                    for (int v = 0; v < 4; ++v) g[v] = ok[v] ? e[v] / se - ((j0 + v) == lab ? 1.0 : 0.0) : 0.0;
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v) g[v] = ok[v] ? z[v] - ((j0 + v) == lab ? 1.0 : 0.0) : 0.0;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) g[v] = ok[v] ? g[v] + uu[v] + (double)a.rho * (z[v] - c[v]) : 0.0;
            };
            double lse_y;
            if (stage > 0 && !more) {
                // take step stage-1 from y with the L its search ended with, then the momentum point
                gradient(y, lse_y);
                const double invL = skipped ? 0.0 : 1.0 / Lcur;
                float xn[4], yn[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    xn[v] = (float)(y[v] - g[v] * invL);
                    yn[v] = xn[v] + mom * (xn[v] - (float)xo[v]);
                }
                if (stage < a.J) {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (ok[v]) { a.Xb[base + v] = xn[v]; a.Yb[base + v] = yn[v]; }
                } else {
                    // last stage: the result, and the dual step of Eq. 2 with the old Z_L
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (ok[v]) {
                            const float zold = a.ZL[base + v];
                            a.ZL[base + v] = on ? xn[v] : (float)c[v] - (float)uu[v] / a.rho;
                            if (a.update_u) a.U[base + v] = (float)uu[v] + a.rho * (zold - (float)c[v]);
                        }
                    continue;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v) y[v] = (double)yn[v];
            }
            // the search at y: ||g||^2, ||y||^2, F(y), and F(y - g/L) - F(y) for the candidates L = Lcur eta^q
            gradient(y, lse_y);
            if (!on) continue;                         // (its lanes still took part in the group reductions above)
            double gg = 0.0, yy = 0.0, Fy = 0.0, ug = 0.0, gd = 0.0;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                gg += g[v] * g[v];
                yy += y[v] * y[v];
                ug += uu[v] * g[v];
                gd += g[v] * (y[v] - c[v]);
                const double lin = (j0 + v) == lab ? 1.0 : 0.0;
                Fy += ok[v] ? uu[v] * (y[v] - c[v]) + 0.5 * (double)a.rho * (y[v] - c[v]) * (y[v] - c[v]) +
                                  (a.risk == 0 ? -lin * y[v] : 0.5 * (y[v] - lin) * (y[v] - lin)) : 0.0;
            }
            const bool lead = (threadIdx.x & (LP - 1)) == 0;
            if (a.risk == 0 && lead) Fy += lse_y;
            double gl = 0.0;
#pragma unroll
            for (int v = 0; v < 4; ++v) gl += (j0 + v) == lab ? g[v] : 0.0;
            const double glab = group_sum<LPLOG>(gl);
            const double gg_row = group_sum<LPLOG>(gg), ug_row = group_sum<LPLOG>(ug), gd_row = group_sum<LPLOG>(gd);
            sgg += gg; syy += yy; sF += Fy;
            double Lq = more ? u->step : Lcur;
#pragma unroll
            for (int q = 0; q < NC; ++q) {
                const double inv = 1.0 / Lq;
                // x - y = -g/L:  <u, x - y> + rho/2 (||x - c||^2 - ||y - c||^2)
                double d = -inv * ug_row + 0.5 * (double)a.rho * (-2.0 * inv * gd_row + inv * inv * gg_row);
                if (a.risk == 0) {
                    double x[4], e2[4], se2;
#pragma unroll
                    for (int v = 0; v < 4; ++v) x[v] = y[v] - g[v] * inv;
                    const double lse_x = row_lse<LPLOG>(x, ok, e2, se2);
                    d += (lse_x - lse_y) + inv * glab;     // R(x) - R(y), with -(x - y)_label = g_label / L
                } else {
                    // 1/2 (||x - e||^2 - ||y - e||^2) = sum (x - y) (y - e) + 1/2 ||x - y||^2
                    double t = 0.0;
#pragma unroll
                    for (int v = 0; v < 4; ++v) t += ok[v] ? g[v] * (y[v] - ((j0 + v) == lab ? 1.0 : 0.0)) : 0.0;
                    d += -inv * group_sum<LPLOG>(t) + 0.5 * inv * inv * gg_row;
                }
                if (lead) D[q] += d;
                Lq *= (double)a.sp.eta;
            }
        }
        if (stage == a.J && !more) continue;
        double* out = a.partials + (int64_t)ch * kFistaStride;
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const double t = block_sum(D[q], sm);
            if (threadIdx.x == 0) out[q] = t;
        }
        if (!more) {
            const double t0 = block_sum(sgg, sm), t1 = block_sum(syy, sm), t2 = block_sum(sF, sm);
            if (threadIdx.x == 0) { out[kMaxCand] = t0; out[kMaxCand + 1] = t1; out[kMaxCand + 2] = t2; }
        }
    }
}

// Takes the decisions of a pass.  first_pass: the searches of stage `stage` begin here (the counters of the finished
// stage are added up, every solve starts from L = rho), the step floor is applied, then the first candidates are judged.
__global__ __launch_bounds__(256) void fista_finish_kernel(FistaArgs a, int ncand, int first_pass, int stage) {
    __shared__ double sm[4];
    __shared__ double D[kFistaStride];
    const int unit = blockIdx.x;
    Unit* u = a.units + unit;
    if (!first_pass && u->done) return;
    const int c0 = a.unit_chunk_ptr[unit], c1 = a.unit_chunk_ptr[unit + 1];
    for (int q = 0; q < kFistaStride; ++q) {
        if ((q < kMaxCand && q >= ncand) || (q >= kMaxCand && !first_pass)) continue;
        double s = 0.0;
        for (int i = c0 + threadIdx.x; i < c1; i += blockDim.x)
            if (a.chunk_kind[i] == 0) s += a.partials[(int64_t)i * kFistaStride + q];
        s = block_sum(s, sm);
        if (threadIdx.x == 0) D[q] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (first_pass) {
            if (stage == 0) { u->step = (double)a.rho; u->total = 0; }
            else u->total += u->ntrials;
            u->ntrials = 0; u->done = 0; u->skip = 0; u->keep = u->step;
            floor_test(u, D[kMaxCand], D[kMaxCand + 1]);
            u->step0 = kFistaSlack * fabs(D[kMaxCand + 2]);       // kept for the passes of further candidates
            if (u->done) return;
        }
        decide(u, D, ncand, a.sp, a.status, u->step0);
    }
}

__global__ void fill_units_kernel(Unit* units, int n, double step) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    Unit u;
    u.step = step; u.step0 = step; u.keep = step; u.g = 0.0; u.bnorm = 0.0; u.done = 0; u.skip = 0; u.ntrials = 0;
    u.spec = 0; u.total = 0; u.pad = 0;
    units[i] = u;
}

__global__ void reset_units_kernel(Unit* units, int n, SearchParams sp) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    begin_search(units + i, sp);
}

__global__ __launch_bounds__(256) void permute_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                           const int32_t* __restrict__ idx, int64_t N, int C,
                                                           int scatter) {
    const int64_t total = N * (int64_t)C;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int64_t r = e / C;
        const int c = (int)(e - r * C);
        const int64_t o = (int64_t)idx[r] * C + c;
        if (scatter) dst[o] = src[e];
        else dst[e] = src[o];
    }
}

inline int flat_grid(int64_t count) {
    int64_t nb = (count + 1023) / 1024;     // about four elements per thread at least
    if (nb < 1) nb = 1;
    if (nb > kReduceBlocks) nb = kReduceBlocks;
    return (int)nb;
}

}  // namespace

void launch_phi_G(hipStream_t s, const float* T, const float* Z, float* U, float* G, float* Tprev,
                  int have_prev, int apply_dual, int64_t count, int last, float nu, float rho, double* partials,
                  LayerScalars* out) {
    const int nb = flat_grid(count);
    const bool v4 = (count % 4) == 0;
#define CADMM_PHI_G(L_, V_) hipLaunchKernelGGL((phi_G_kernel<L_, V_>), dim3(nb), dim3(256), 0, s, T, Z, U, G, Tprev, have_prev, apply_dual, count, nu, rho, partials)
    if (last) { if (v4) CADMM_PHI_G(1, 4); else CADMM_PHI_G(1, 1); }
    else { if (v4) CADMM_PHI_G(0, 4); else CADMM_PHI_G(0, 1); }
#undef CADMM_PHI_G
    hipLaunchKernelGGL(phi_G_finish_kernel, dim3(1), dim3(256), 0, s, partials, nb, last, nu, out);
}

void launch_G_only(hipStream_t s, const float* T, const float* Z, const float* U, float* G, int64_t count,
                   int last, float nu, float rho) {
    const int nb = flat_grid(count);
    const bool v4 = (count % 4) == 0;
#define CADMM_G_ONLY(L_, V_) hipLaunchKernelGGL((G_only_kernel<L_, V_>), dim3(nb), dim3(256), 0, s, T, Z, U, G, count, nu, rho)
    if (last) { if (v4) CADMM_G_ONLY(1, 4); else CADMM_G_ONLY(1, 1); }
    else { if (v4) CADMM_G_ONLY(0, 4); else CADMM_G_ONLY(0, 1); }
#undef CADMM_G_ONLY
}

void launch_risk(hipStream_t s, const float* ZL, const int32_t* labels, int64_t N, int CL, int risk,
                 double* partials, LayerScalars* out) {
    const int nb = flat_grid(N * 4);
    hipLaunchKernelGGL(risk_kernel, dim3(nb), dim3(256), 0, s, ZL, labels, N, CL, risk, partials);
    hipLaunchKernelGGL(risk_finish_kernel, dim3(1), dim3(256), 0, s, partials, nb, out);
}

void launch_w_norms(hipStream_t s, const float* gradW, const float* W, int count, Unit* unit, double* partials,
                    SearchParams sp) {
    int nb = (count + 2047) / 2048;
    if (nb > 64) nb = 64;
    if (nb < 1) nb = 1;
    hipLaunchKernelGGL(w_norms_kernel, dim3(nb), dim3(256), 0, s, gradW, W, count, partials);
    hipLaunchKernelGGL(w_norms_finish_kernel, dim3(1), dim3(64), 0, s, partials, nb, unit, sp);
}

void launch_w_trial_finish(hipStream_t s, double* partials, int n_partials, SearchParams sp, Unit* unit,
                           int32_t* status) {
    hipLaunchKernelGGL(w_trial_finish_kernel, dim3(1), dim3(256), 0, s, partials, n_partials, 1, 1, sp, unit, status);
}

void launch_w_trial(hipStream_t s, const float* T0, const float* Q, const float* Z, const float* U,
                    int64_t count, int last, int ncand, SearchParams sp, Unit* unit, double* partials,
                    int32_t* status, int speculated) {
    const int nb = flat_grid(count);
    const bool v4 = (count % 4) == 0;
#define CADMM_W_TRIAL(L_, N_, V_) hipLaunchKernelGGL((w_trial_kernel<L_, N_, V_>), dim3(nb), dim3(256), 0, s, T0, Q, Z, U, count, sp, unit, partials, speculated)
    if (ncand == 1) {
        if (last) { if (v4) CADMM_W_TRIAL(1, 1, 4); else CADMM_W_TRIAL(1, 1, 1); }
        else { if (v4) CADMM_W_TRIAL(0, 1, 4); else CADMM_W_TRIAL(0, 1, 1); }
    } else {
        ncand = kMaxCand;
        if (last) { if (v4) CADMM_W_TRIAL(1, kMaxCand, 4); else CADMM_W_TRIAL(1, kMaxCand, 1); }
        else { if (v4) CADMM_W_TRIAL(0, kMaxCand, 4); else CADMM_W_TRIAL(0, kMaxCand, 1); }
    }
#undef CADMM_W_TRIAL
    hipLaunchKernelGGL(w_trial_finish_kernel, dim3(1), dim3(256), 0, s, partials, nb, kMaxCand, ncand, sp, unit, status);
}

void launch_w_step(hipStream_t s, float* W, const float* gradW, int count_w, float* T, const float* Q,
                   int64_t count_t, const Unit* unit, int speculated) {
    const int nb = flat_grid(count_t > count_w ? count_t : count_w);
    if (count_t % 4 == 0) hipLaunchKernelGGL((w_step_kernel<4>), dim3(nb), dim3(256), 0, s, W, gradW, count_w, T, Q, count_t, unit, speculated);
    else hipLaunchKernelGGL((w_step_kernel<1>), dim3(nb), dim3(256), 0, s, W, gradW, count_w, T, Q, count_t, unit, speculated);
}

void launch_z_trial(hipStream_t s, const ZTrialArgs& a0) {
    ZTrialArgs a = a0;
    if (a.n_chunks > 0) {
        const bool v4 = (a.Cl % 4) == 0 && (a.Cn % 4) == 0;
        const bool lr = a.gradZ == nullptr;           // low-rank gradient (the caller checked the shape limits)
        const size_t lds = lr ? (size_t)a.Cn * a.Cl * sizeof(float) : 0;      // W_{l+1}^T: at most 16 x 1024 floats
        if (a.ncand == 1) {
            if (lr) hipLaunchKernelGGL((z_trial_kernel<1, 4, 1>), dim3(a.n_chunks), dim3(256), lds, s, a);
            else if (v4) hipLaunchKernelGGL((z_trial_kernel<1, 4, 0>), dim3(a.n_chunks), dim3(256), 0, s, a);
            else hipLaunchKernelGGL((z_trial_kernel<1, 1, 0>), dim3(a.n_chunks), dim3(256), 0, s, a);
        } else {
            a.ncand = kMaxCand;
            // a small grid: such a pass nearly always finds every community done and only has to notice it
            const int nb = a.n_chunks < kReduceBlocks / 4 ? a.n_chunks : kReduceBlocks / 4;
            if (lr) hipLaunchKernelGGL((z_trial_kernel<kMaxCand, 4, 1>), dim3(nb), dim3(256), lds, s, a);
            else if (v4) hipLaunchKernelGGL((z_trial_kernel<kMaxCand, 4, 0>), dim3(nb), dim3(256), 0, s, a);
            else hipLaunchKernelGGL((z_trial_kernel<kMaxCand, 1, 0>), dim3(nb), dim3(256), 0, s, a);
        }
    }
    hipLaunchKernelGGL(z_trial_finish_kernel, dim3(a.M), dim3(256), 0, s, a);
}

void launch_z_step(hipStream_t s, float* Zl, const float* gradZ, const int32_t* row_comm, int64_t N, int Cl,
                   const Unit* units, int M) {
    const int nb = flat_grid(N * (int64_t)Cl);
#define CADMM_ZSTEP(V_, L_) hipLaunchKernelGGL((z_step_kernel<V_, L_>), dim3(nb), dim3(256), 0, s, Zl, gradZ, row_comm, N, Cl, units, M)
    if (M <= kStepUnits) { if (Cl % 4 == 0) CADMM_ZSTEP(4, true); else CADMM_ZSTEP(1, true); }
    else { if (Cl % 4 == 0) CADMM_ZSTEP(4, false); else CADMM_ZSTEP(1, false); }
#undef CADMM_ZSTEP
}

void launch_z_step_lowrank(hipStream_t s, float* Zl, const float* Tl, const float* SG, const float* Wt, float nu,
                           const int32_t* row_comm, int64_t N, int Cl, int Cn, const Unit* units, int M) {
    // more and smaller workgroups than the reducing kernels use: nothing is reduced here
    int64_t nb = (N * (int64_t)Cl + 2047) / 2048;
    nb = nb < 1 ? 1 : (nb > 4 * kReduceBlocks ? 4 * kReduceBlocks : nb);
    const size_t lds = (size_t)Cn * Cl * sizeof(float);                 // at most 16 x 1024 floats (the low-rank limit)
    if (M <= kStepUnits)
        hipLaunchKernelGGL((z_step_lowrank_kernel<true>), dim3((unsigned)nb), dim3(256), lds, s, Zl, Tl, SG, Wt, nu, row_comm, N, Cl, Cn, units, M);
    else
        hipLaunchKernelGGL((z_step_lowrank_kernel<false>), dim3((unsigned)nb), dim3(256), lds, s, Zl, Tl, SG, Wt, nu, row_comm, N, Cl, Cn, units, M);
}

void launch_t_carry(hipStream_t s, float* Tn, const float* P, const int64_t* row_seg_ptr, const int32_t* seg_comm,
                    const int32_t* seg_pos, int64_t N, int Cn, const Unit* units, int M) {
    const int nb = flat_grid(N * (int64_t)Cn * 4);
#define CADMM_CARRY(V_, L_) hipLaunchKernelGGL((t_carry_kernel<V_, L_>), dim3(nb), dim3(256), 0, s, Tn, P, row_seg_ptr, seg_comm, seg_pos, N, Cn, units, M)
    if (M <= kCarryUnits) { if (Cn % 4 == 0) CADMM_CARRY(4, true); else CADMM_CARRY(1, true); }
    else { if (Cn % 4 == 0) CADMM_CARRY(4, false); else CADMM_CARRY(1, false); }
#undef CADMM_CARRY
}

void launch_last_layer(hipStream_t s, float* ZL, float* U, const float* TL, const int32_t* labels, int64_t N,
                       int CL, int risk, float rho, int J, int update_u) {
#define CADMM_LAST(LG_) hipLaunchKernelGGL((last_layer_kernel<LG_>), dim3((unsigned)(((N << LG_) + 255) / 256)), dim3(256), 0, s, ZL, U, TL, labels, N, CL, risk, rho, J, update_u)
    if (CL <= 4) CADMM_LAST(0);
    else if (CL <= 8) CADMM_LAST(1);
    else if (CL <= 16) CADMM_LAST(2);
    else if (CL <= 32) CADMM_LAST(3);
    else CADMM_LAST(4);
#undef CADMM_LAST
}

void launch_relu(hipStream_t s, const float* T, float* Z, int64_t count, int apply_relu) {
    hipLaunchKernelGGL(relu_kernel, dim3(flat_grid(count)), dim3(256), 0, s, T, Z, count, apply_relu);
}

void launch_argmax_rows(hipStream_t s, const float* T, int32_t* pred, int64_t N, int C) {
    hipLaunchKernelGGL(argmax_rows_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, T, pred, N, C);
}

void launch_fista_stage(hipStream_t s, const FistaArgs& a, int stage, int more, float mom) {
    if (a.n_chunks <= 0) return;
    // more = 0: the pass that takes the step and tries the first candidate (sixteen at once in stage 0, where L climbs
    // from rho); more = 1: four further candidates on a full grid (a step usually needs one or two doublings, in many
    // communities at once); more = 2: sixteen further candidates on a small grid, which usually finds nothing pending
    const int nc = more == 0 ? (stage == 0 ? kMaxCand : 1) : (more == 1 ? 4 : kMaxCand);
    const int cap = more == 0 ? a.n_chunks : (more == 1 ? kReduceBlocks : kReduceBlocks / 4);
    const int nb = a.n_chunks < cap ? a.n_chunks : cap;
#define CADMM_FISTA(LG_) do { \
        if (nc == kMaxCand) hipLaunchKernelGGL((fista_stage_kernel<LG_, kMaxCand>), dim3(nb), dim3(256), 0, s, a, stage, more, mom); \
        else if (nc == 4) hipLaunchKernelGGL((fista_stage_kernel<LG_, 4>), dim3(nb), dim3(256), 0, s, a, stage, more, mom); \
        else hipLaunchKernelGGL((fista_stage_kernel<LG_, 1>), dim3(nb), dim3(256), 0, s, a, stage, more, mom); } while (0)
    if (a.CL <= 4) CADMM_FISTA(0);
    else if (a.CL <= 8) CADMM_FISTA(1);
    else if (a.CL <= 16) CADMM_FISTA(2);
    else if (a.CL <= 32) CADMM_FISTA(3);
    else CADMM_FISTA(4);
#undef CADMM_FISTA
    if (stage < a.J) hipLaunchKernelGGL(fista_finish_kernel, dim3(a.M), dim3(256), 0, s, a, nc, more ? 0 : 1, stage);
}

void launch_fill_units(hipStream_t s, Unit* units, int n, double step) {
    hipLaunchKernelGGL(fill_units_kernel, dim3((n + 255) / 256), dim3(256), 0, s, units, n, step);
}

void launch_reset_units(hipStream_t s, Unit* units, int n, SearchParams sp) {
    hipLaunchKernelGGL(reset_units_kernel, dim3((n + 255) / 256), dim3(256), 0, s, units, n, sp);
}

void launch_permute_rows(hipStream_t s, const float* src, float* dst, const int32_t* idx, int64_t N, int C,
                         int scatter) {
    hipLaunchKernelGGL(permute_rows_kernel, dim3(flat_grid(N * (int64_t)C)), dim3(256), 0, s, src, dst, idx, N, C, scatter);
}

}  // namespace cadmm
