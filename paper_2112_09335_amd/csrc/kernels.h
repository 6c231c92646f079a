// Launch wrappers of the HIP kernels (gfx950).  All pointers are device pointers; all work is
// enqueued on `s`.  Row-major fp32 matrices whose leading dimension equals their width.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace cadmm {

// ---------------------------------------------------------------- sparse aggregation (spmm.hip)
// Y[r,:] = sum_{p in [lo[r], hi[r])} val[p] * X[col[p],:]   for r < nrows.
// epilogue 0: store;  1: Y = nu * (Zl - relu(Tl)) + sum  (gradient of the Z subproblem).
struct SpmmEpilogue {
    int kind = 0;
    const float* Zl = nullptr;
    const float* Tl = nullptr;
    float nu = 0.f;
};
// Device view of a row list laid out for the aggregation (RowSchedule on the host).  rec[i] = (first chunk, one past
// the last chunk, output row, 0) of scheduled row i; a chunk is 8 (column, value) pairs of 8 bytes, padded with
// weight zero, chunk 0 all padding.  Records from n_rows on are the parts of rows that were too long for one lane
// group: their output row is a row of `side` (n_parts x width), and a combine kernel adds a split row's parts in
// order and applies the epilogue.
// blocks[l] / n_blocks[l] / xcd_start[l]: the workgroup -> rows table for 2^l lanes per gathered row (BlockTable).
struct SpmmSchedule {
    int64_t n_rows = 0;
    int64_t n_parts = 0;
    const int4* rec = nullptr;
    const int2* ent = nullptr;
    int64_t n_long = 0;
    const int32_t* long_row = nullptr;
    const int32_t* long_part_ptr = nullptr;
    float* side = nullptr;
    const int4* blocks[7] = {};
    int64_t n_blocks[7] = {};
    int64_t xcd_start[7][9] = {};
};
void launch_spmm(hipStream_t s, const SpmmSchedule& sched, const float* X, float* Y, int width, const SpmmEpilogue& epi);
// Y[pos[k], :] = val[k] * X[col[k], :] for k < n: the output rows that have a single entry.
// calibration: only the gathers of the row list's column stream, rows of `width` floats (4, 8, 16, ... 256) of X;
// out: 256 floats (never written in practice); returns the bytes the launch asks the memory system for
double launch_gather_calibration(hipStream_t s, const SpmmSchedule& sc, int64_t n_chunks, const float* X, int width,
                                 float* out);
void launch_spmm_single(hipStream_t s, const int32_t* pos, const int32_t* col, const float* val, const float* X,
                        float* Y, int64_t n, int width);
// columns of the feature matrix handled per launch (0 = all); smaller tiles keep a community's share of
// the gathered matrix inside one XCD's L2 at the price of re-reading the entries once per tile
void set_spmm_tile_cols(int cols);
// 1: every XCD walks one contiguous slice of the workgroup table, whole communities one after the other (default);
// 0: workgroups in plain table order, which deals consecutive row blocks round-robin to the XCDs
void set_spmm_xcd_remap(int on);

// ---------------------------------------------------------------- dense contractions (gemm.hip)
struct Unit;
// out[n x C] = A[n x K] * B[K x C];  epilogue 1: out = nu * (Zl - relu(Tl)) + A B.
// epilogue 2 (hidden layer, W search): with Q = A B, t0 = Tio, t1 = t0 - Q / unit->step0 the first candidate of
// the search is evaluated in the same pass, partials[block] = nu/2 sum ((relu(t1) - Zl)^2 - (relu(t0) - Zl)^2), and
// either the step is taken ahead of the decision (unit->spec: Tio = t1, Q is not stored) or out = Q is stored.
// If the search then rejects the first candidate, a plain product with kind 0 and `unit` set forms Q after all
// (its workgroups leave at once otherwise) and w_step repairs Tio from it.  The step is only taken ahead of the
// decision when the previous search accepted its first candidate: then Q/step0 is small against Tio and
// undoing it costs one rounding; with a step0 far too small (first iterations) it would wipe out Tio.
struct GemmEpilogue {
    int kind = 0;
    const float* Zl = nullptr;
    const float* Tl = nullptr;
    float nu = 0.f;
    float* Tio = nullptr;
    const Unit* unit = nullptr;
    double* partials = nullptr;
};
void launch_gemm_nn(hipStream_t s, const float* A, const float* B, float* out, int64_t n, int K, int C,
                    const GemmEpilogue& epi = GemmEpilogue());
// 1: plain products wider than 32 columns use three-way bf16 splits of both operands on the bf16 matrix cores
void set_gemm_split(int on);
int get_gemm_split();
// calibration kernels: chains of fp32 MFMAs on registers (returns the flops of the launch; out: blocks * 256 floats),
// and a plain copy of count floats (count % 4 == 0)
double launch_mfma_chain(hipStream_t s, float* out, int blocks, int iters);
// the same with bf16 32x32x16 MFMAs, each followed by `valu` (0, 4, 6, 8) independent vector instructions
double launch_mfma_bf16_chain(hipStream_t s, float* out, int blocks, int iters, int valu);
void launch_stream_copy(hipStream_t s, const float* src, float* dst, int64_t count);
// dst = 0.999 dst + src in place (count % 4 == 0): two reads and one write-back per element
void launch_stream_update(hipStream_t s, const float* src, float* dst, int64_t count);
int64_t gemm_nn_blocks(int64_t n, int C);      // grid size of that launch (= block results of epilogue 2)
// out[n x C] = [nu (Zl - relu(Tl)) | SG] * Bcat, Bcat = [W (K1 x C); S (K2 x C)], C <= 32, K1 % 4 == K2 % 4 == 0:
// the product (grad_Z psi) W with grad = nu (Zl - relu(Tl)) + SG W^T, S = W^T W, the gradient never stored.
void launch_gemm_nn_gradz(hipStream_t s, const float* Zl, const float* Tl, const float* SG, const float* Bcat,
                          float* out, int64_t n, int K1, int K2, int C, float nu);
// out[K x C] = A[n x K]^T * G[n x C]; partial: scratch of gemm_tn_scratch_floats(n,K,C) floats.
size_t gemm_tn_scratch_floats(int64_t n, int K, int C);
// With Zl != nullptr, G holds the pre-activation T of a hidden layer and the right operand is
// nu (relu(T) - Zl) 1[T > 0], formed on the fly.
void launch_gemm_tn(hipStream_t s, const float* A, const float* G, float* out, int64_t n, int K, int C,
                    float* partial, const float* Zl = nullptr, float nu = 0.f);
// out[C x K] = in[K x C]^T (small)
void launch_transpose(hipStream_t s, const float* in, float* out, int K, int C);

// ---------------------------------------------------------------- fused elementwise + reductions (elementwise.hip)
constexpr int kReduceBlocks = 2048;      // grid of the flat reducing kernels
constexpr int kMaxCand = 16;             // step-size candidates evaluated per pass
constexpr int kLowRankMax = 16;          // widest next layer for which the Z gradient is kept in low-rank form
constexpr int kChunkRows = 128;          // rows / segments per reduction chunk of the Z search

// One step-size search ("unit"): a layer's tau, or a (layer, community)'s theta.
struct Unit {
    double step;       // current first candidate / accepted value
    double step0;      // first candidate of this iteration's search (the value the speculative step used)
    double keep;       // value accepted by the previous search (restored if this one takes no step)
    double g;          // squared gradient norm
    double bnorm;      // squared norm of the block that moves
    int32_t done;      // search finished
    int32_t skip;      // step below resolution: block stays
    int32_t ntrials;   // candidates tested this iteration
    int32_t spec;      // the previous search accepted its first candidate: a speculative step with step0 is safe
    int32_t total;     // candidates tested since the counter was cleared (the last-layer solve adds up its steps)
    int32_t pad;
};

// Readout scalars of one layer's base evaluation.
struct LayerScalars {
    double phi;        // phi_l at the base point
    double res2;       // ||Z_L - T_L||^2           (last layer only)
    double dT2;        // ||T_L - T_L(previous)||^2 (last layer only)
    double risk;       // R(Z_L, Y)                 (last layer only)
};

struct SearchParams {
    float nu, rho, eta;
    int32_t max_backtrack;
    int32_t relax;       // 1: a search starts from (last accepted value) / eta, 0: from the last accepted value
};

// phi_l and G_l at T (hidden: G = nu (relu(T)-Z) 1[T>0]; last: G = -(U + rho (Z - T))).
// last != 0 additionally accumulates ||Z-T||^2, ||T-Tprev||^2 (if have_prev) and writes Tprev = T.
// apply_dual (last layer): U += rho (Z - T) is applied first (dual ascent on the iterate just reached).
void launch_phi_G(hipStream_t s, const float* T, const float* Z, float* U, float* G, float* Tprev,
                  int have_prev, int apply_dual, int64_t count, int last, float nu, float rho, double* partials,
                  LayerScalars* out);
// G only (no reduction), same formulas.
void launch_G_only(hipStream_t s, const float* T, const float* Z, const float* U, float* G, int64_t count,
                   int last, float nu, float rho);
// R(Z_L, Y) summed over labelled rows -> out->risk
void launch_risk(hipStream_t s, const float* ZL, const int32_t* labels, int64_t N, int CL, int risk,
                 double* partials, LayerScalars* out);
// unit.g = ||gradW||^2, unit.bnorm = ||W||^2, applies the step floor, resets the search state.
void launch_w_norms(hipStream_t s, const float* gradW, const float* W, int count, Unit* unit, double* partials,
                    SearchParams sp);
// One pass of the W search: candidates step*eta^j, j < ncand, on phi_l(T0 - Q/step).
// speculated != 0: T0 already holds the speculative step T0 - Q/step0; the pass rebuilds T0 = T0 + Q/step0.
void launch_w_trial(hipStream_t s, const float* T0, const float* Q, const float* Z, const float* U,
                    int64_t count, int last, int ncand, SearchParams sp, Unit* unit, double* partials,
                    int32_t* status, int speculated = 0);
// Sums n_partials block results of an epilogue-2 product (candidate 0 only) and takes the search decision.
void launch_w_trial_finish(hipStream_t s, double* partials, int n_partials, SearchParams sp, Unit* unit,
                           int32_t* status);
// W -= gradW/step (count_w entries), T = T0 - Q/step (count_t entries); no-op if unit.skip.
// speculated != 0: T already holds T0 - Q/step0 and is only repaired if the accepted step differs.
void launch_w_step(hipStream_t s, float* W, const float* gradW, int count_w, float* T, const float* Q,
                   int64_t count_t, const Unit* unit, int speculated = 0);

// Z search, layer l (widths Cl, Cn = C_{l+1}).  Device arrays of the graph:
struct ZTrialArgs {
    const int32_t* chunk_unit; const int32_t* chunk_kind; const int32_t* chunk_begin; const int32_t* chunk_end;
    int32_t n_chunks;
    const int32_t* unit_chunk_ptr; int32_t M;
    const int32_t* segc_row;
    const float* Zl; const float* gradZ; const float* Tl; int Cl;       // own term, rows of the community
    // low-rank form of the gradient (gradZ == nullptr): grad = nu (Zl - relu(Tl)) + SG Wt, SG is N x Cn with
    // Cn <= kLowRankMax, Wt is Cn x Cl; it is recomputed per element instead of being read
    const float* SG = nullptr; const float* Wt = nullptr;
    const float* Tn; const float* Zn; const float* U; const float* P; int Cn;   // next layer, per segment
    const float* Gn = nullptr;   // last next layer: G_L = -(U + rho (Z_L - T_L)), read in place of Tn, Zn and U
    int next_is_last;
    int first_pass;        // also accumulate ||gradZ_m||^2 and ||Z_m||^2, apply the step floor
    int ncand;
    SearchParams sp;
    Unit* units;           // [M]
    double* partials;      // [n_chunks * (kMaxCand + 2)]
    int32_t* status;
};
void launch_z_trial(hipStream_t s, const ZTrialArgs& a);
// Z_l[i,:] -= gradZ[i,:] / theta[comm(i)]
void launch_z_step(hipStream_t s, float* Zl, const float* gradZ, const int32_t* row_comm, int64_t N, int Cl,
                   const Unit* units, int M);
// the same step with the gradient in its low-rank form nu (Zl - relu(Tl)) + SG Wt (SG: N x Cn, Wt: Cn x Cl)
void launch_z_step_lowrank(hipStream_t s, float* Zl, const float* Tl, const float* SG, const float* Wt, float nu,
                           const int32_t* row_comm, int64_t N, int Cl, int Cn, const Unit* units, int M);
// Tn[i,:] -= sum over the segments (i,c) of row i of P[(i,c),:] / theta_c  (communities whose step was skipped
// contribute nothing): the pre-activation of the next layer after the Z step, without a new aggregation.
void launch_t_carry(hipStream_t s, float* Tn, const float* P, const int64_t* row_seg_ptr, const int32_t* seg_comm,
                    const int32_t* seg_pos, int64_t N, int Cn, const Unit* units, int M);
// Last layer (Appendix A, Eq. 5) by J FISTA steps per row, fused with the dual step (Eq. 2):
//   U_new = U + rho (Z_L - T_L),  Z_L_new = FISTA(start Z_L; c = T_L, U, rho)
// update_u = 0 leaves U alone (the dual step is then taken on the new iterates by the next phi_G)
void launch_last_layer(hipStream_t s, float* ZL, float* U, const float* TL, const int32_t* labels, int64_t N,
                       int CL, int risk, float rho, int J, int update_u);
// Last layer by FISTA with backtracking on the block subproblem of Z_{L,m} (Appendix A, Eq. 5): one L per community
// and step, found by the device-side search over the rows of the community (chunk tables of the graph, kind 0).
// Stage `stage` of `J` steps: stage 0 evaluates 16 candidates L = rho eta^q at y_0 = Z_L; stage j = 1..J-1 takes step
// j-1 with the L found (x_j = y_{j-1} - grad / L, y_j = x_j + mom (x_j - x_{j-1})) and evaluates the current L at
// y_j; stage J takes the last step, writes Z_L (rows without label: their exact minimiser) and, with update_u, the dual
// step of Eq. 2 with the old Z_L.  more = 1 launches a pass of 16 further candidates for the searches not yet done
// (it returns at once otherwise).  Every stage is followed by the finishing kernel that takes the decisions.
struct FistaArgs {
    float* ZL; float* U; const float* TL; float* Xb; float* Yb;      // Xb, Yb: N x CL scratch (x_j and y_j)
    const int32_t* labels;
    const int32_t* chunk_unit; const int32_t* chunk_kind; const int32_t* chunk_begin; const int32_t* chunk_end;
    int32_t n_chunks; const int32_t* unit_chunk_ptr; int32_t M;
    int CL, risk, J, update_u;
    float rho;
    SearchParams sp;
    Unit* units;           // [M]
    double* partials;      // [n_chunks * (kMaxCand + 3)]
    int32_t* status;
};
void launch_fista_stage(hipStream_t s, const FistaArgs& a, int stage, int more, float mom);
void launch_relu(hipStream_t s, const float* T, float* Z, int64_t count, int apply_relu);
void launch_argmax_rows(hipStream_t s, const float* T, int32_t* pred, int64_t N, int C);
void launch_fill_units(hipStream_t s, Unit* units, int n, double step);
void launch_reset_units(hipStream_t s, Unit* units, int n, SearchParams sp);
// gather / scatter rows between caller order and internal order: dst[r,:] = src[idx[r],:] or dst[idx[r],:] = src[r,:]
void launch_permute_rows(hipStream_t s, const float* src, float* dst, const int32_t* idx, int64_t N, int C,
                         int scatter);

}  // namespace cadmm
