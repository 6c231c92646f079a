/*
 * cadmm.h - C ABI of the community-blocked ADMM sweep for GCN training on one MI355X (gfx950).
 *
 * The calls follow the inputs and outputs of the paper's Algorithm 1 (REQUIRE Y, Z_0, nu, rho;
 * ENSURE W_l, Z_{l,m}) and its Problems 1-3 (Section 2): build the graph and its communities,
 * set model and data, initialise W/Z/U, run k ADMM iterations, read the objective and residuals.
 *
 * General conventions
 *   - Every call returns CADMM_OK (0) or a negative CADMM_E* code; nothing throws, aborts or
 *     prints.  cadmm_last_error() gives a text for the last failure on that context.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on the
 *     context's GPU.  The caller owns every buffer it passes.  Inputs are copied; outputs are
 *     written into caller memory.
 *   - All device memory the library uses comes from ONE caller-provided workspace
 *     (cadmm_workspace_bytes / cadmm_set_workspace).  The library never calls hipMalloc for
 *     device memory; it allocates only small host buffers (readouts, the host copy of the graph).
 *   - Node order at the boundary is the caller's.  Internally nodes are renumbered so that
 *     every community is a contiguous row range (stable sort on (community, id)); that
 *     numbering is visible through cadmm_get_graph and is the row order of the cadmm_op_*
 *     kernel-level calls.
 *   - Matrices are dense row-major fp32.  Layer widths C_0..C_L as in the paper's notation
 *     table (C_l = number of neurons of layer l, C_0 = input features, C_L = classes).
 *   - All work is enqueued on the HIP stream given at creation.  cadmm_run does not
 *     synchronise; the cadmm_get_*, cadmm_eval calls do.
 *   - Call order: create -> build_graph -> set_model -> workspace_bytes -> set_workspace ->
 *     set_data -> init -> { run | eval | get_* | set_state }*.  A call out of order returns
 *     CADMM_EORDER.
 */
#ifndef CADMM_H
#define CADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CADMM_OK          0
#define CADMM_EINVAL     -1   /* bad argument (null pointer, id out of range, size mismatch)   */
#define CADMM_EORDER     -2   /* call out of order                                              */
#define CADMM_ENOMEM     -3   /* workspace too small / host allocation failed                   */
#define CADMM_EHIP       -4   /* a HIP runtime call failed                                      */
#define CADMM_EUNSUPPORTED -5 /* valid request this build does not implement                    */

#define CADMM_STATUS_BACKTRACK_CAP 1  /* a step-size search used all max_backtrack multiplications */
#define CADMM_STATUS_NONFINITE     2  /* a non-finite value was seen in a reduction                 */

typedef struct cadmm_ctx cadmm_ctx;   /* opaque */

/* Create a context on GPU `device`.  hip_stream: a hipStream_t (NULL = the default stream).
 * device = -1 gives a host-only context: graph construction, its getters, set_model and
 * workspace_bytes work; every call that needs the GPU returns CADMM_EUNSUPPORTED / CADMM_EORDER. */
int  cadmm_create(cadmm_ctx** out, int device, void* hip_stream);
void cadmm_destroy(cadmm_ctx* ctx);
const char* cadmm_last_error(cadmm_ctx* ctx);

/*
 * Communities for a graph that comes without them (paper, Section 2: the graph is divided into M
 * communities; the paper uses METIS there, this is the library's own deterministic stand-in).
 *   src,dst  host int32[n_edges] as for cadmm_build_graph (repeats, both orientations and self pairs
 *            are normalised away);  comm  host int32[N], out: community of every node, in [0,M).
 * Size-capped label propagation from one cluster per node, merging of clusters along the connection
 * with the most edges until M are left, propagation on the original graph until it rests; every tie is broken by node
 * or cluster number, so the result depends on the input only.  No community exceeds
 * ceil(N/M) + floor(N/M)/20 + 1 nodes unless clusters had to be merged regardless of size; some
 * communities may stay empty.  Host work only: valid on a context created with device = -1.
 */
int  cadmm_partition(cadmm_ctx* ctx, int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst,
                     int32_t M, int32_t* comm);

/*
 * Graph and communities (paper, Section 2: undirected unweighted graph G(V,E), normalised
 * adjacency A~ = (D+I)^(-1/2)(A+I)(D+I)^(-1/2), partition into M communities V_m, neighbour
 * sets N_m, blocks A~_{m,r}).
 *   src,dst  host int32[n_edges], endpoints in [0,N); any order, both orientations, repeats and
 *            self pairs are tolerated and normalised away.
 *   comm     host int32[N], values in [0,M); NULL = contiguous chunks of ceil(N/M) nodes.
 * Builds a CSR of A~ in the internal numbering (sorted columns, so each row's entries are
 * grouped by community), the per-row community segments, and uploads it to the workspace once
 * that is set.  Values: (float)(1.0 / sqrt((double)d_i * (double)d_j)), d_i = 1 + degree.
 */
int  cadmm_build_graph(cadmm_ctx* ctx, int64_t N, int64_t n_edges, const int32_t* src,
                       const int32_t* dst, int32_t M, const int32_t* comm);
/* nnz = 2E + N stored entries; n_segments = number of (row, community) pairs that occur;
 * n_halo_rows = rows with at least one neighbour in another community. */
int  cadmm_graph_sizes(cadmm_ctx* ctx, int64_t* nnz, int64_t* n_segments, int64_t* n_halo_rows);
/*
 * Copy the graph out (host pointers, any may be NULL to skip):
 *   perm[N]            internal row -> caller's node id
 *   row_ptr[N+1], col[nnz], val[nnz]        CSR of A~, internal numbering
 *   seg_ptr[n_segments+1], seg_row[n_segments], seg_comm[n_segments]
 *                      segments in (row, community) order; seg_ptr indexes col/val
 *   comm_row_ptr[M+1]  first internal row of every community
 *   neighbour[M*M]     neighbour[m*M+r] = 1 iff r is in N_m
 */
int  cadmm_get_graph(cadmm_ctx* ctx, int32_t* perm, int64_t* row_ptr, int32_t* col, float* val,
                     int64_t* seg_ptr, int32_t* seg_row, int32_t* seg_comm, int64_t* comm_row_ptr,
                     uint8_t* neighbour);
/* Order in which cadmm_op_aggregate_segments writes its rows: segments sorted by
 * (community, row).  order[j] = index of that segment in the (row, community) order above. */
int  cadmm_get_segment_order(cadmm_ctx* ctx, int64_t* order /* host [n_segments] */);

/*
 * Model and hyper-parameters (Problem 2: nu; Eq. 1: rho; Section 3.1 / Appendix A: the step
 * parameters tau_l, theta_{l,m} and their conditions).
 *   L >= 2 layers, C[0..L] widths.  risk: 0 = softmax cross-entropy summed over labelled
 *   rows, 1 = 1/2 ||Z_L - Y||^2 over labelled rows.
 *   tau0/theta0: first candidates at k = 0; eta > 1: growth factor of the search;
 *   max_backtrack: multiplications allowed per search (<= 64); fista_iters: J steps of the
 *   last-layer solver (Appendix A, Eq. 5); dual_form: 0 = dual step with the superscripts as
 *   printed in Eq. 2 (Z_L^k, W_L^{k+1}); 1 = dual ascent on the new iterates,
 *   U^{k+1} = U^k + rho (Z_L^{k+1} - A~ Z_{L-1}^{k+1} W_L^{k+1}).
 *   schedule: 0 = Algorithm 1 (every W_l, then every Z_{l,m}, all from the values of iteration k);
 *   1 = the serial baseline of Section 4.1, layers one after the other: for l = 1..L first W_l, then
 *   Z_l (its communities together), each from the newest values of everything else.
 *   step_policy: 0 = a search for tau_l / theta_{l,m} starts from the value accepted last time, so the
 *   parameters never shrink; 1 = it starts from that value divided by eta, so they can.
 *   fista_mode: how Z_{L,m} is solved (Appendix A, Eq. 5, "via FISTA"): 0 = fista_iters steps of constant length
 *   1 / (rho + c_R), c_R = 1/2 (cross-entropy) or 1 (least squares), row by row; 1 = FISTA with backtracking on the block
 *   Z_{L,m}: one L per community and step, started at rho in every iteration, multiplied by eta until
 *   F(y - grad/L) <= F(y) - ||grad||^2 / (2L) holds over the labelled rows of the community (at most max_backtrack
 *   multiplications per step), kept for the later steps of the solve.
 */
typedef struct {
    int32_t L;
    const int32_t* C;
    int32_t risk;
    float nu, rho, tau0, theta0, eta;
    int32_t max_backtrack, fista_iters, dual_form;
    int32_t schedule;
    int32_t step_policy;
    int32_t fista_mode;
} cadmm_model;
int  cadmm_set_model(cadmm_ctx* ctx, const cadmm_model* model);

/* Device bytes needed for graph + state + scratch (valid after build_graph and set_model). */
int  cadmm_workspace_bytes(cadmm_ctx* ctx, size_t* bytes);
/* Hand over the workspace: device pointer, 256-byte aligned, at least workspace_bytes long.
 * It must stay valid until cadmm_destroy.  Uploads the graph. */
int  cadmm_set_workspace(cadmm_ctx* ctx, void* dev_ptr, size_t bytes);

/* Z_0 = X (N x C_0, row-major, caller's node order; host pointer, or device pointer if
 * x_on_device != 0) and the label matrix Y as class ids: labels host int32[N], -1 = unlabelled. */
int  cadmm_set_data(cadmm_ctx* ctx, const float* X, const int32_t* labels, int x_on_device);

/* W0: L host pointers, W0[l-1] is C_{l-1} x C_l.  Sets Z_l to the forward pass of Problem 1's
 * constraints (Z_l = relu(A~ Z_{l-1} W_l), Z_L = A~ Z_{L-1} W_L), U = 0, tau = tau0,
 * theta = theta0, iteration counter 0. */
int  cadmm_init(cadmm_ctx* ctx, const float* const* W0);

/* k iterations of Algorithm 1 (W-update, Z-update, U-update), enqueued on the stream.  On a
 * non-default stream an iteration is captured once as a HIP graph and replayed (same kernels, same
 * results); the library records no memset nodes. */
int  cadmm_run(cadmm_ctx* ctx, int32_t k);

/*
 * Readout at the current iterate (synchronises).  objective = R(Z_L,Y) + sum_{l<L} nu/2
 * ||Z_l - relu(A~ Z_{l-1} W_l)||^2 (Problem 2); lagrangian = Eq. 1; primal_res =
 * ||Z_L - A~ Z_{L-1} W_L||_F; dual_res = rho ||A~ Z_{L-1}^k W_L^k - A~ Z_{L-1}^{k-1} W_L^{k-1}||_F
 * (0 before the first iteration).  layer_penalty: host double[L-1] or NULL.
 */
typedef struct {
    double objective, lagrangian, risk, primal_res, dual_res;
    int32_t iter, status;
} cadmm_stats;
int  cadmm_eval(cadmm_ctx* ctx, cadmm_stats* out, double* layer_penalty);

/*
 * Inference with the current weights (paper, Section 4.2: training / test accuracy): the forward pass
 * Z_l = relu(A~ Z_{l-1} W_l), logits = A~ Z_{L-1} W_L from Z_0, class = argmax of a row (lowest index on
 * ties).  pred: host int32[N] or NULL; logits: host N x C_L or NULL (both in the caller's node order);
 * accuracy: fraction of labelled nodes whose class equals their label.  Synchronises.  Does not change
 * W, Z, U.
 */
int  cadmm_predict(cadmm_ctx* ctx, int32_t* pred, float* logits, double* accuracy);

/* State readout, host pointers, caller's node order.  l in 1..L for W, 0..L for Z. */
int  cadmm_get_W(cadmm_ctx* ctx, int32_t l, float* dst);
int  cadmm_get_Z(cadmm_ctx* ctx, int32_t l, float* dst);
int  cadmm_get_U(cadmm_ctx* ctx, float* dst);
/* tau[L], theta[(L-1)*M] (layer-major), n_trials[L + (L-1)*M] and sq_grad[L + (L-1)*M]
 * (squared gradient norms) of the last iteration.  Any pointer may be NULL. */
int  cadmm_get_steps(cadmm_ctx* ctx, double* tau, double* theta, int32_t* n_trials, double* sq_grad);
/* fista_mode 1: L[M] = the constant every community's last solve of Z_{L,m} ended with, n_trials[M] = candidates it
 * tested over all its steps.  Any pointer may be NULL. */
int  cadmm_get_fista(cadmm_ctx* ctx, double* L, int32_t* n_trials);
/* Overwrite state (resume / tests).  Any pointer may be NULL (= keep).  W: L host pointers;
 * Z: L host pointers for layers 1..L (caller's node order); U: N x C_L. */
int  cadmm_set_state(cadmm_ctx* ctx, const float* const* W, const float* const* Z, const float* U,
                     const double* tau, const double* theta);

/*
 * Kernel-level calls on device buffers in the INTERNAL row order (for tests and profiling).
 * They run the same kernels the sweep uses.
 *   aggregate:           Y = A~ X                         X,Y device N x width    (Problem 3's
 *                        blocked sum A~_{m,m} X_m + sum_{r in N_m} A~_{m,r} X_r for every m)
 *   aggregate_segments:  P[(i,c)] = sum_{j in V_c} A~_ij V_j   one row per segment, written in
 *                        the order of cadmm_get_segment_order (Appendix A: A~_{r,m} applied to
 *                        a change of Z_{l,m}, for every r in N_m or r = m)
 *   transform:           out = A B        A device n x K, B device K x C, out n x C
 *   wgrad:               out = A^T G      A device n x K, G device n x C, out K x C
 */
int  cadmm_op_aggregate(cadmm_ctx* ctx, const float* X, int32_t width, float* Y);
int  cadmm_op_aggregate_segments(cadmm_ctx* ctx, const float* V, int32_t width, float* P);
int  cadmm_op_transform(cadmm_ctx* ctx, const float* A, int64_t n, int32_t K, const float* B,
                        int32_t C, float* out);
int  cadmm_op_wgrad(cadmm_ctx* ctx, const float* A, const float* G, int64_t n, int32_t K,
                    int32_t C, float* out);

/*
 * cadmm_op_wgrad for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same result bit for bit as
 * cadmm_op_wgrad (out = A^T G, A device n x K, G device n x C, out device K x C, enqueued on the context's stream),
 * but the per-chunk partial matrices of the product live in a static device array inside the library (72 MiB on every
 * GPU the library runs on, held until the process ends) instead of the workspace, so the call works on a context
 * that has no graph, model or workspace yet and calls no allocating routine.  Shapes whose partial matrices need more
 * than 18 * 2^20 floats (about (1024 + tiles) * 16384 floats for tiles = ceil(K/128) * ceil(C/128) result tiles when
 * C > 32; all widths up to 1024 x 1024 fit) return CADMM_ENOMEM.  All calls on one GPU share that array: two calls
 * that overlap on one GPU (different streams or contexts) race; calls on one stream are ordered and safe.  Nothing in
 * the array has to be cleared between calls: the product writes every entry the reduction reads.
 */
int  cadmm_op_wgrad_noalloc(cadmm_ctx* ctx, const float* A, const float* G, int64_t n, int32_t K, int32_t C,
                            float* out);

/*
 * Machine calibration for the rooflines the benchmarks quote (no counterpart in the paper).  Runs `reps` timed
 * launches (after one untimed) on the context's stream, synchronises, and returns the rate.
 *   kind 0: plain copy of `count` floats (multiple of 4) from src to dst, both device; rate = GB/s read + written.
 *   kind 1: dependent chains of fp32 MFMAs on registers, `count` steps of four 32x32x2 MFMAs per wavefront,
 *           2048 workgroups of four wavefronts; dst: device scratch of at least 2048 * 256 floats (src unused);
 *           rate = TFLOP/s.
 *   kind 2 / 3: the gathers of the aggregation and nothing else, driven by the column stream of the graph's rows (2) or
 *           of its (row, community) segments with several entries (3), in the order the aggregation reads it: every
 *           eight-entry chunk is loaded and the eight rows of `count` floats (4, 8, ... 256) it names are gathered from
 *           src (device, N x count) and added up; no row bounds, no reduction, no result rows.  dst as for kind 1.
 *           rate = GB/s of entry pairs plus gathered rows: what the memory system serves to this access pattern, the
 *           ceiling for cadmm_op_aggregate / _aggregate_segments at that width.  Needs the workspace.
 *   kind 4: as kind 1 with bf16 MFMAs (32x32x16), the instruction the split products issue; rate = TFLOP/s.
 *   kind 5 / 6 / 7: as kind 4 with 4 / 6 / 8 independent fp32 vector instructions after every MFMA (the rate still
 *           counts the MFMA flops only): how much vector work runs beside the matrix cores.
 *   kind 8: dst = 0.999 dst + src in place over `count` floats (multiple of 4), both device: two arrays read, one
 *           written back where it was read, the memory mix of the step kernels; rate = GB/s of the 12 bytes per element.
 */
int  cadmm_op_calibrate(cadmm_ctx* ctx, int32_t kind, const float* src, float* dst, int64_t count, int32_t reps,
                        double* rate);

/*
 * Per-kernel-class timing for benchmarks (no counterpart in the paper).  cadmm_profile(ctx, 1) clears
 * the counters and makes every later launch group be bracketed by a pair of HIP events on the
 * context's stream; cadmm_profile(ctx, 0) stops that.  cadmm_get_profile synchronises and returns,
 * per class (host arrays of CADMM_PROFILE_CLASSES entries, any may be NULL): elapsed milliseconds,
 * number of timed launch groups, and the algorithmic bytes and flops booked for them (what the
 * operation must move / compute: operands read once, results written once).
 */
#define CADMM_PROFILE_CLASSES 19
int  cadmm_profile(cadmm_ctx* ctx, int enable);
int  cadmm_get_profile(cadmm_ctx* ctx, double* ms, int64_t* records, double* bytes, double* flops);
const char* cadmm_profile_class_name(int32_t cls);

/* Tuning knobs for experiments.  "use_graph" (per context): 1 = cadmm_run replays one iteration as a
 * captured HIP graph when the context's stream is not the default stream (default), 0 = plain launches.
 * "use_lowrank" (per context): 1 = with a next layer of at most 16 units the Z gradient is kept as
 * nu (Z_l - relu(T_l)) + (A~ G_{l+1}) W_{l+1}^T and rebuilt per element by its consumers (default), 0 = stored.
 * "use_speculative" (per context): 1 = in a wide hidden layer the product Q = A~ Z_{l-1} grad W also evaluates the
 * first candidate of the tau search and takes the step on the pre-activation speculatively (default), 0 = separate passes.
 * "t1_refresh" (per context): the pre-activations A~ Z_{l-1} W_l are carried from one iteration to the
 * next (through the W step, and through the segment products of the Z step) and formed anew every
 * this many iterations (default 16; 0 = always form them anew).
 * Process-wide: "spmm_tile_cols": feature columns handled per
 * aggregation launch (0 = all at once); "spmm_xcd_remap": 1 = each XCD walks one contiguous slice of the aggregation's
 * work list, whole communities one after the other (default), 0 = workgroups in plain order;
 * "gemm_split": 1 = products with more than 32 result columns run on the bf16 matrix
 * cores, both operands split exactly into three bf16 parts and the six largest cross products accumulated in fp32
 * (default), 0 = on the fp32 matrix cores. */
int  cadmm_tune(cadmm_ctx* ctx, const char* key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* CADMM_H */
