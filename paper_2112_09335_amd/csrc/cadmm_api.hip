// C ABI of the community-blocked ADMM sweep: context, workspace layout, and the schedule of one
// iteration of the paper's Algorithm 1 (W-update, Z-update, U-update) as a fixed sequence of kernel
// launches on one HIP stream.  Nothing is read back from the device inside cadmm_run.
#include "../../include/cadmm.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "host_graph.h"
#include "host_partition.h"
#include "kernels.h"

using namespace cadmm;

// Scratch of cadmm_op_wgrad_noalloc: the per-chunk partial matrices of the W-gradient product, for callers that cannot
// allocate.  Every GPU the library runs on holds its own copy of this array until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the per-device address looked up below.
constexpr size_t kStaticScratchFloats = (size_t)18 << 20;          // 72 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices] = {};                     // device address of `scratch` on GPU d, once looked up
static std::mutex g_scratch_mutex;

struct cadmm_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    HostGraph hg;
    bool has_graph = false, has_model = false, has_ws = false, has_data = false, has_init = false;
    // model
    int L = 0;
    std::vector<int> C;
    // agg_first[l]: layer l forms T_l as A~ (Z_{l-1} W_l), aggregating on the narrow side C_l, instead of
    // (A~ Z_{l-1}) W_l.  Its W-update then needs three aggregations of width C_l, so it pays if
    // 3 C_l < C_{l-1}.  In those layers the slot H[l] holds A~ G_l (N x C_l).
    std::vector<char> agg_first;
    int risk = 0, max_bt = 60, J = 10, dual_form = 0, schedule = 0, step_policy = 0, fista_mode = 0;
    bool u_pending = false;      // dual_form 1: the dual step of the last sweep is still to be applied
    float nu = 0, rho = 0, tau0 = 0, theta0 = 0, eta = 2;
    // workspace
    char* ws = nullptr;
    size_t ws_bytes = 0;
    // graph on the device
    int32_t* d_row_comm = nullptr;
    int32_t* d_perm = nullptr;
    int32_t* d_seg1_pos = nullptr; int32_t* d_seg1_col = nullptr; float* d_seg1_val = nullptr;
    int32_t* d_segc_row = nullptr;
    // reduction chunk tables of the Z search: [0] many segments per chunk (narrow next layer), [1] few (wide)
    struct DevChunks { int32_t *unit = nullptr, *kind = nullptr, *begin = nullptr, *end = nullptr, *unit_ptr = nullptr; int32_t n = 0; };
    DevChunks d_chunks[2];
    int32_t* d_labels = nullptr;
    int32_t* d_pred = nullptr;
    int64_t* d_row_seg_ptr = nullptr;
    int32_t* d_seg_comm = nullptr;
    int32_t* d_seg_pos = nullptr;
    std::vector<int32_t> h_labels;     // internal row order
    // split rows of the CSR row list and of the segment list; side buffer for their parts
    struct DevSchedule {               // device copy of a RowSchedule
        int4* rec = nullptr; int2* ent = nullptr; int32_t* long_row = nullptr; int32_t* long_ptr = nullptr;
        int4* blocks[7] = {};          // workgroup -> rows table per lane count of a gathered row
        int64_t n_blocks[7] = {};
        int64_t xcd_start[7][9] = {};
    };
    DevSchedule d_rows, d_segs;
    float* side = nullptr;
    // state and per-layer buffers, index l = 0..L (unused slots stay null)
    std::vector<float*> Z, W, H, T, G;
    float* U = nullptr;
    float* TLprev = nullptr;
    float* tmpA = nullptr;      // N x max width: staging, G W^T
    float* tmpB = nullptr;      // N x max hidden width: gradient of the Z subproblem
    float* tmpV = nullptr;      // N x max next width
    float* P = nullptr;         // n_seg x max next width, the buffer of the layer being searched
    float* Pbuf[2] = {nullptr, nullptr};   // layers alternate: P of layer l stays until layer l+1 is done
    float* gradW = nullptr;
    float* Wt = nullptr;
    float* Bcat = nullptr;      // [W_{l+1}; W_{l+1}^T W_{l+1}] for the low-rank form of the Z gradient
    float* tn_partial = nullptr;
    size_t tn_partial_floats = 0;
    double* partials = nullptr;
    Unit* unitsW = nullptr;     // [L]
    Unit* unitsZ = nullptr;     // [(L-1) * M]
    Unit* unitsF = nullptr;     // [M]: the L of the last-layer solve with backtracking (fista_mode 1)
    float* fistaX = nullptr;    // N x C_L each: x_j and y_j of that solve
    float* fistaY = nullptr;
    LayerScalars* scalars = nullptr;   // [L+1]
    int32_t* status = nullptr;
    bool base_valid = false, have_prev = false, dual_valid = false;
    bool phi_valid = false;      // the penalties of the hidden layers whose gradient is not stored are evaluated too
    int iter = 0;
    // The pre-activations T_l = A~ Z_{l-1} W_l are carried from one iteration to the next instead of being
    // formed anew: the W step leaves T_l - Q/tau = A~ Z_{l-1}^k W_l^{k+1}, and the Z step of layer l-1 changes
    // it by - sum_c P_(i,c) / theta_c (T_1 does not depend on any Z at all).  t1_age counts such updates since
    // the last exact evaluation (-1: the T buffers are not images of the state); after t1_refresh of them
    // everything is formed again, which bounds the rounding drift.
    int t1_age = -1;
    int t1_refresh = 16;
    // One iteration captured as a HIP graph, per variant of the launch sequence (base evaluation already
    // done or not; previous T_L available or not).  Replayed by cadmm_run when the stream is not the
    // default stream; launch-bound problem sizes gain most.
    bool use_graph = true;
    bool use_lowrank = true;
    bool use_speculative = true;
    struct GraphSlot { hipGraphExec_t exec = nullptr; bool tried = false; };
    GraphSlot graphs[2][2][2][2];
    // optional per-kernel-class timing with HIP events on the context's stream
    bool prof_on = false;
    struct ProfRec { int cls; hipEvent_t a, b; };
    std::vector<ProfRec> prof_recs;
    std::vector<hipEvent_t> prof_pool;
    double prof_ms[CADMM_PROFILE_CLASSES] = {0};
    int64_t prof_launches[CADMM_PROFILE_CLASSES] = {0};
    double prof_bytes[CADMM_PROFILE_CLASSES] = {0};
    double prof_flops[CADMM_PROFILE_CLASSES] = {0};
};

namespace {

int fail(cadmm_ctx* c, int code, const std::string& msg) {
    if (c) c->err = msg;
    return code;
}

int hip_fail(cadmm_ctx* c, hipError_t e, const char* what) {
    return fail(c, CADMM_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define HIP_TRY(ctx, call)                                        \
    do {                                                          \
        hipError_t e_ = (call);                                   \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, #call);    \
    } while (0)

struct Bump {
    char* base;
    size_t off = 0;
    template <class T>
    T* take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

int max_of(const std::vector<int>& v, int lo, int hi) {
    int m = 0;
    for (int i = lo; i <= hi; ++i) m = v[i] > m ? v[i] : m;
    return m;
}

// Assign every device buffer inside the workspace; with base == nullptr only the size is computed.
size_t layout(cadmm_ctx* c, char* base) {
    const HostGraph& g = c->hg;
    const int L = c->L;
    const int64_t N = g.N;
    Bump b{base};
    c->d_row_comm = b.take<int32_t>(N);
    c->d_perm = b.take<int32_t>(N);
    auto take_schedule = [&](cadmm_ctx::DevSchedule& d, const RowSchedule& rs) {
        d.rec = b.take<int4>(rs.rec.size());
        d.ent = b.take<int2>(rs.ent.size());
        d.long_row = b.take<int32_t>(rs.n_long());
        d.long_ptr = b.take<int32_t>(rs.n_long() + 1);
        for (int l = 0; l < 7; ++l) {
            d.n_blocks[l] = count_blocks(rs, l);
            d.blocks[l] = b.take<int4>((size_t)d.n_blocks[l]);
        }
    };
    take_schedule(c->d_rows, g.row_sched);
    take_schedule(c->d_segs, g.seg_sched);
    c->d_seg1_pos = b.take<int32_t>(g.seg1_pos.size());
    c->d_seg1_col = b.take<int32_t>(g.seg1_pos.size());
    c->d_seg1_val = b.take<float>(g.seg1_pos.size());
    c->d_segc_row = b.take<int32_t>(g.n_seg);
    const size_t nch = g.chunks.size() > g.chunks_wide.size() ? g.chunks.size() : g.chunks_wide.size();
    for (int t = 0; t < 2; ++t) {
        const size_t nt = t == 0 ? g.chunks.size() : g.chunks_wide.size();
        c->d_chunks[t].unit = b.take<int32_t>(nt);
        c->d_chunks[t].kind = b.take<int32_t>(nt);
        c->d_chunks[t].begin = b.take<int32_t>(nt);
        c->d_chunks[t].end = b.take<int32_t>(nt);
        c->d_chunks[t].unit_ptr = b.take<int32_t>(g.M + 1);
        c->d_chunks[t].n = (int32_t)nt;
    }
    c->d_labels = b.take<int32_t>(N);
    c->d_pred = b.take<int32_t>(N);
    c->d_row_seg_ptr = b.take<int64_t>(N + 1);
    c->d_seg_comm = b.take<int32_t>(g.n_seg);
    c->d_seg_pos = b.take<int32_t>(g.n_seg);
    {
        const int64_t np_ = g.row_sched.n_parts() > g.seg_sched.n_parts() ? g.row_sched.n_parts() : g.seg_sched.n_parts();
        c->side = b.take<float>((size_t)np_ * max_of(c->C, 0, L));
    }
    c->Z.assign(L + 1, nullptr);
    c->W.assign(L + 1, nullptr);
    c->H.assign(L + 1, nullptr);
    c->T.assign(L + 1, nullptr);
    c->G.assign(L + 1, nullptr);
    for (int l = 0; l <= L; ++l) c->Z[l] = b.take<float>(N * c->C[l]);
    for (int l = 1; l <= L; ++l) {
        c->W[l] = b.take<float>((size_t)c->C[l - 1] * c->C[l]);
        c->H[l] = b.take<float>(N * (c->agg_first[l] ? c->C[l] : c->C[l - 1]));
        c->T[l] = b.take<float>(N * c->C[l]);
        c->G[l] = b.take<float>(N * c->C[l]);
    }
    c->U = b.take<float>(N * c->C[L]);
    c->TLprev = b.take<float>(N * c->C[L]);
    c->tmpA = b.take<float>(N * max_of(c->C, 0, L));
    c->tmpB = b.take<float>(N * max_of(c->C, 1, L - 1));
    c->tmpV = b.take<float>(N * max_of(c->C, 2, L));
    c->Pbuf[0] = b.take<float>(g.n_seg * max_of(c->C, 2, L));
    c->Pbuf[1] = L > 2 ? b.take<float>(g.n_seg * max_of(c->C, 2, L)) : c->Pbuf[0];
    c->P = c->Pbuf[0];
    size_t wmax = 0, tnmax = 0;
    for (int l = 1; l <= L; ++l) {
        size_t w = (size_t)c->C[l - 1] * c->C[l];
        wmax = w > wmax ? w : wmax;
        size_t t = gemm_tn_scratch_floats(N, c->C[l - 1], c->C[l]);
        tnmax = t > tnmax ? t : tnmax;
    }
    c->gradW = b.take<float>(wmax);
    c->Wt = b.take<float>(wmax);
    c->Bcat = b.take<float>((size_t)(max_of(c->C, 0, L) + kLowRankMax) * kLowRankMax);
    c->tn_partial = b.take<float>(tnmax);
    c->tn_partial_floats = tnmax;
    size_t np = (size_t)kReduceBlocks * kMaxCand;
    const size_t np2 = nch * (kMaxCand + 3);
    np = np > np2 ? np : np2;
    for (int l = 1; l <= L; ++l) {               // block results of the products that also evaluate a candidate
        const size_t np3 = (size_t)gemm_nn_blocks(N, c->C[l]) * kMaxCand;
        np = np > np3 ? np : np3;
    }
    c->partials = b.take<double>(np);
    c->unitsW = b.take<Unit>(L);
    c->unitsZ = b.take<Unit>((size_t)(L - 1) * g.M);
    c->unitsF = b.take<Unit>((size_t)g.M);
    if (c->fista_mode == 1) {
        c->fistaX = b.take<float>(N * c->C[L]);
        c->fistaY = b.take<float>(N * c->C[L]);
    }
    c->scalars = b.take<LayerScalars>(L + 1);
    c->status = b.take<int32_t>(4);
    return (b.off + 255) & ~(size_t)255;
}

template <class T>
hipError_t upload(hipStream_t s, T* dst, const std::vector<T>& src) {
    if (src.empty()) return hipSuccess;
    return hipMemcpyAsync(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice, s);
}

// One class per kernel symbol (and role, where one symbol serves two), so that the live timings can be
// set beside a profiler's per-kernel averages.
enum ProfClass {
    P_SPMM = 0, P_SPMM_GRADZ, P_SPMM_SEG, P_GEMM_NN_128, P_GEMM_NN_128_GRADZ, P_GEMM_NN_128_TRIAL, P_GEMM_NN_32, P_GEMM_TN, P_GEMM_TN_32, P_PHI_G,
    P_G_ONLY, P_W_TRIAL, P_Z_TRIAL, P_W_STEP, P_Z_STEP, P_LAST_LAYER, P_T_CARRY, P_GEMM_GRADZ, P_OTHER
};
const char* kProfNames[CADMM_PROFILE_CLASSES] = {
    "spmm_rows_kernel[rows]", "spmm_rows_kernel[rows,gradz]", "spmm_rows_kernel[segments]", "gemm_nn_kernel<128,0>",
    "gemm_nn_kernel<128,1>", "gemm_nn_kernel<128,2>+finish", "gemm_nn_kernel<32>", "gemm_tn_kernel<128>+reduce", "gemm_tn_kernel<32>+reduce",
    "phi_G_kernel", "G_only_kernel",
    "w_trial_kernel", "z_trial_kernel", "w_step_kernel", "z_step_kernel", "last_layer_kernel", "t_carry_kernel",
    "gemm_nn_gradz_kernel", "other"};

hipEvent_t prof_event(cadmm_ctx* c) {
    if (!c->prof_pool.empty()) {
        hipEvent_t e = c->prof_pool.back();
        c->prof_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Times the launches enqueued by `body` as one record of class `cls` and books its algorithmic work.
template <class F>
void timed(cadmm_ctx* c, int cls, double bytes, double flops, F body) {
    if (!c->prof_on) { body(); return; }
    hipEvent_t a = prof_event(c), b = prof_event(c);
    if (a && b) (void)hipEventRecord(a, c->stream);
    body();
    if (a && b) {
        (void)hipEventRecord(b, c->stream);
        c->prof_recs.push_back({cls, a, b});
        c->prof_bytes[cls] += bytes;
        c->prof_flops[cls] += flops;
    }
}

SpmmSchedule schedule_of(const cadmm_ctx* c, const cadmm_ctx::DevSchedule& d, const RowSchedule& rs) {
    SpmmSchedule sc;
    sc.n_rows = rs.n_rows();
    sc.n_parts = rs.n_parts();
    sc.rec = d.rec; sc.ent = d.ent;
    sc.n_long = rs.n_long(); sc.long_row = d.long_row; sc.long_part_ptr = d.long_ptr;
    sc.side = c->side;
    for (int l = 0; l < 7; ++l) {
        sc.blocks[l] = d.blocks[l];
        sc.n_blocks[l] = d.n_blocks[l];
        for (int k = 0; k <= 8; ++k) sc.xcd_start[l][k] = d.xcd_start[l][k];
    }
    return sc;
}

double spmm_bytes(const cadmm_ctx* c, int64_t out_rows, int width, int extra_reads) {
    // entries (column id + value), row bounds, one read of the gathered matrix, one write of the result
    return 8.0 * (double)c->hg.nnz + 16.0 * (double)out_rows + 4.0 * (double)c->hg.N * width +
           4.0 * (double)out_rows * width * (1 + extra_reads);
}

void gemm_nn(cadmm_ctx* c, const float* A, const float* B, float* out, int64_t n, int K, int C,
             const GemmEpilogue& epi = GemmEpilogue()) {
    timed(c, C > 32 ? (epi.kind ? P_GEMM_NN_128_GRADZ : P_GEMM_NN_128) : P_GEMM_NN_32,
          4.0 * ((double)n * K + (double)K * C + (double)n * C * (epi.kind ? 3 : 1)), 2.0 * (double)n * K * C,
          [&] { launch_gemm_nn(c->stream, A, B, out, n, K, C, epi); });
}

SearchParams search_params(const cadmm_ctx* c) {
    SearchParams sp;
    sp.nu = c->nu;
    sp.rho = c->rho;
    sp.eta = c->eta;
    sp.max_backtrack = c->max_bt;
    sp.relax = c->step_policy == 1 ? 1 : 0;
    return sp;
}

void aggregate(cadmm_ctx* c, const float* X, float* Y, int width, const SpmmEpilogue& epi) {
    timed(c, epi.kind ? P_SPMM_GRADZ : P_SPMM, spmm_bytes(c, c->hg.N, width, epi.kind ? 2 : 0),
          2.0 * (double)c->hg.nnz * width, [&] {
              launch_spmm(c->stream, schedule_of(c, c->d_rows, c->hg.row_sched), X, Y, width, epi);
          });
}

// P_{(i,c)} = sum over the entries of row i in community c of A~_ij V_j, one output row per segment, in the
// (community, row) order: the segments with several entries as a row list, those with one entry as scaled copies.
void aggregate_segments(cadmm_ctx* c, const float* V, float* P, int width) {
    timed(c, P_SPMM_SEG, spmm_bytes(c, c->hg.n_seg, width, 0), 2.0 * (double)c->hg.nnz * width, [&] {
        launch_spmm(c->stream, schedule_of(c, c->d_segs, c->hg.seg_sched), V, P, width, SpmmEpilogue());
        launch_spmm_single(c->stream, c->d_seg1_pos, c->d_seg1_col, c->d_seg1_val, V, P, (int64_t)c->hg.seg1_pos.size(),
                           width);
    });
}

bool t1_reusable(const cadmm_ctx* c) { return c->t1_age >= 0 && c->t1_age < c->t1_refresh; }

// T_l = A~ Z_{l-1} W_l in the association chosen for the layer.  Used by the initial forward pass and
// by every base evaluation, so that re-evaluating an unchanged point reproduces T_l bit for bit.
void compute_T(cadmm_ctx* c, int l, bool force = false) {
    const int64_t N = c->hg.N;
    const bool carried = !force && t1_reusable(c);     // T[l] already holds A~ Z_{l-1} W_l for the current state
    if (c->agg_first[l]) {
        if (carried) return;
        gemm_nn(c, c->Z[l - 1], c->W[l], c->tmpV, N, c->C[l - 1], c->C[l]);
        aggregate(c, c->tmpV, c->T[l], c->C[l], SpmmEpilogue());
    } else {
        if (l >= 2) aggregate(c, c->Z[l - 1], c->H[l], c->C[l - 1], SpmmEpilogue());   // the W step needs H_l itself
        if (carried) return;
        gemm_nn(c, c->H[l], c->W[l], c->T[l], N, c->C[l - 1], c->C[l]);
    }
}

// A hidden layer in the (A~ Z) W association feeds its pre-activation gradient to the W gradient only, where
// it is formed on the fly from T_l and Z_l; a sweep therefore skips phi_G for it (phi_l is a readout).
bool gradient_on_the_fly(const cadmm_ctx* c, int l) { return l < c->L && !c->agg_first[l]; }

// H_l, T_l = H_l W_l, phi_l and G_l at the current iterate.  This is both the start of a sweep and the readout of
// the previous one, so it is computed once per iterate (need_phi: also the penalties a sweep does not need).
void base_eval(cadmm_ctx* c, bool need_phi) {
    const int L = c->L;
    const int64_t N = c->hg.N;
    auto run_phi_G = [&](int l) {
        const double cnt = (double)N * c->C[l];
        timed(c, P_PHI_G, 4.0 * cnt * (l == L ? 6 : 3), 0.0, [&] {
            launch_phi_G(c->stream, c->T[l], c->Z[l], c->U, c->G[l], l == L ? c->TLprev : nullptr,
                         c->have_prev ? 1 : 0, (l == L && c->u_pending) ? 1 : 0, N * c->C[l], l == L, c->nu, c->rho,
                         c->partials, c->scalars + l);
        });
    };
    if (!c->base_valid) {
        for (int l = 1; l <= L; ++l) {
            compute_T(c, l);
            if (!gradient_on_the_fly(c, l) || need_phi) run_phi_G(l);
        }
        if (!t1_reusable(c)) c->t1_age = 0;                // every T_l was just formed exactly
        c->u_pending = false;
        c->dual_valid = c->have_prev;
        c->have_prev = true;
        c->base_valid = true;
        c->phi_valid = need_phi;
    } else if (need_phi && !c->phi_valid) {
        for (int l = 1; l <= L; ++l)
            if (gradient_on_the_fly(c, l)) run_phi_G(l);
        c->phi_valid = true;
    }
}

// T_l <- A~ Z_{l-1}^{k+1} W_l^{k+1}, from the segment products P of layer l-1 and its accepted theta.
void carry_T(cadmm_ctx* c, int l) {
    if (c->t1_refresh <= 0) return;
    const int64_t N = c->hg.N;
    const int Cl = c->C[l];
    timed(c, P_T_CARRY, 4.0 * ((double)c->hg.n_seg * Cl + 2.0 * (double)N * Cl) + 8.0 * (double)c->hg.n_seg, 0.0, [&] {
        launch_t_carry(c->stream, c->T[l], c->Pbuf[(l - 1) & 1], c->d_row_seg_ptr, c->d_seg_comm, c->d_seg_pos, N, Cl,
                       c->unitsZ + (size_t)(l - 2) * c->hg.M, c->hg.M);
    });
}

// W_l <- W_l - grad phi_l / tau_l with backtracking on tau_l (Section 3.1), from the T_l, H_l (or Z_{l-1}) and G_l
// in memory; leaves T_l = A~ Z_{l-1} W_l^{new}.
void w_update(cadmm_ctx* c, int l) {
    const int L = c->L;
    const int64_t N = c->hg.N;
    hipStream_t s = c->stream;
    const SearchParams sp = search_params(c);
    const int more_passes = (c->max_bt + kMaxCand - 1) / kMaxCand;
    {
        const int K = c->C[l - 1], Cl = c->C[l];
        const int64_t count = N * Cl;
        const int last = (l == L);
        Unit* unit = c->unitsW + (l - 1);
        // grad phi = (A~ Z_{l-1})^T G_l = Z_{l-1}^T (A~ G_l)   (A~ is symmetric)
        const float* left = c->H[l];
        const float* right = c->G[l];
        if (c->agg_first[l]) {
            aggregate(c, c->G[l], c->H[l], Cl, SpmmEpilogue());
            left = c->Z[l - 1];
            right = c->H[l];
        }
        const bool fly = gradient_on_the_fly(c, l);    // G_l = nu (relu(T_l) - Z_l) 1[T_l > 0] formed inside the product
        timed(c, Cl > 32 ? P_GEMM_TN : P_GEMM_TN_32,
              4.0 * ((double)N * K + (double)N * Cl * (fly ? 2 : 1) + (double)K * Cl), 2.0 * (double)N * K * Cl,
              [&] {
                  if (fly) launch_gemm_tn(s, left, c->T[l], c->gradW, N, K, Cl, c->tn_partial, c->Z[l], c->nu);
                  else launch_gemm_tn(s, left, right, c->gradW, N, K, Cl, c->tn_partial);
              });
        timed(c, P_OTHER, 8.0 * K * Cl, 0.0, [&] { launch_w_norms(s, c->gradW, c->W[l], K * Cl, unit, c->partials, sp); });
        float* Q = c->G[l];                                                          // G_l is no longer needed
        // T(W - g/tau) = T - Q/tau with Q = A~ Z_{l-1} gradW
        // In a wide hidden layer the product that forms Q also evaluates the first candidate of the search and
        // takes the step on T_l speculatively (tau rarely changes once found); later kernels repair it if needed.
        const bool spec = c->use_speculative && !c->agg_first[l] && !last && Cl > 32;
        if (c->agg_first[l]) {
            gemm_nn(c, c->Z[l - 1], c->gradW, c->tmpV, N, K, Cl);
            aggregate(c, c->tmpV, Q, Cl, SpmmEpilogue());
        } else if (spec) {
            GemmEpilogue ge;
            ge.kind = 2; ge.Zl = c->Z[l]; ge.nu = c->nu; ge.Tio = c->T[l]; ge.unit = unit; ge.partials = c->partials;
            timed(c, P_GEMM_NN_128_TRIAL, 4.0 * ((double)N * K + (double)K * Cl + 3.0 * (double)count), 2.0 * (double)N * K * Cl,
                  [&] {
                      launch_gemm_nn(s, c->H[l], c->gradW, Q, N, K, Cl, ge);
                      launch_w_trial_finish(s, c->partials, (int)gemm_nn_blocks(N, Cl), sp, unit, c->status);
                      GemmEpilogue again;          // Q itself, only if the step was taken ahead and then rejected
                      again.unit = unit;
                      launch_gemm_nn(s, c->H[l], c->gradW, Q, N, K, Cl, again);
                  });
        } else {
            gemm_nn(c, c->H[l], c->gradW, Q, N, K, Cl);
        }
        // one pass reads T0, Q, Z_l (and U for the last layer); passes after an accepted one return at once
        timed(c, P_W_TRIAL, spec ? 0.0 : 4.0 * (double)count * (last ? 4 : 3), 0.0, [&] {
            if (!spec) launch_w_trial(s, c->T[l], Q, c->Z[l], c->U, count, last, 1, sp, unit, c->partials, c->status);
            for (int p = 0; p < more_passes; ++p)
                launch_w_trial(s, c->T[l], Q, c->Z[l], c->U, count, last, kMaxCand, sp, unit, c->partials, c->status,
                               spec ? 1 : 0);
        });
        timed(c, P_W_STEP, 4.0 * ((spec ? 0.0 : 3.0) * (double)count + 3.0 * K * Cl), 0.0, [&] {
            // W^{k+1}; T_l = A~ Z^k W^{k+1}
            launch_w_step(s, c->W[l], c->gradW, K * Cl, c->T[l], Q, count, unit, spec ? 1 : 0);
        });
    }
}

// Z_{l,m} <- Z_{l,m} - grad psi_{l,m} / theta_{l,m} for every community of hidden layer l (Appendix A, Eqs. 3, 4, 6-8),
// from T_l, T_{l+1}, Z_{l+1}, U, W_{l+1} in memory.  Leaves the segment products in Pbuf[l & 1].
void z_update_hidden(cadmm_ctx* c, int l) {
    const int L = c->L;
    const int64_t N = c->hg.N;
    const int M = c->hg.M;
    hipStream_t s = c->stream;
    const SearchParams sp = search_params(c);
    const int more_passes = (c->max_bt + kMaxCand - 1) / kMaxCand;
    {
        const int Cl = c->C[l], Cn = c->C[l + 1];
        const int next_last = (l + 1 == L);
        Unit* units = c->unitsZ + (size_t)(l - 1) * M;
        c->P = c->Pbuf[l & 1];
        timed(c, P_G_ONLY, 4.0 * (double)N * Cn * (next_last ? 4 : 3), 0.0, [&] {
            launch_G_only(s, c->T[l + 1], c->Z[l + 1], c->U, c->G[l + 1], N * Cn, next_last, c->nu, c->rho);
        });
        timed(c, P_OTHER, 8.0 * Cl * Cn, 0.0, [&] { launch_transpose(s, c->W[l + 1], c->Wt, Cl, Cn); });
        // grad psi (all communities at once) = nu (Z_l - relu(T_l)) + A~ G_{l+1} W_{l+1}^T; aggregate on the
        // narrower of the two widths, the penalty term rides in the epilogue of whichever kernel comes last.
        // With a very narrow next layer the gradient is never stored: its consumers (the product with
        // W_{l+1}, the search, the step) rebuild it per element from Z_l, T_l and the N x C_{l+1} factor
        // A~ G_{l+1}, which removes a full write and two full reads of an N x C_l matrix.
        const bool lowrank = c->use_lowrank && Cn <= kLowRankMax && Cn < Cl && Cn % 4 == 0 && Cl % 4 == 0 && Cl <= 1024;
        if (lowrank) {
            aggregate(c, c->G[l + 1], c->tmpA, Cn, SpmmEpilogue());                  // A~ G_{l+1}
            timed(c, P_OTHER, 8.0 * Cl * Cn, 0.0, [&] {
                launch_relu(s, c->W[l + 1], c->Bcat, (int64_t)Cl * Cn, 0);             // rows 0..Cl: W_{l+1}
                launch_gemm_nn(s, c->Wt, c->W[l + 1], c->Bcat + (size_t)Cl * Cn, Cn, Cl, Cn);   // then W^T W
            });
        } else if (Cn < Cl) {
            aggregate(c, c->G[l + 1], c->tmpA, Cn, SpmmEpilogue());                  // A~ G_{l+1}
            GemmEpilogue ge;
            ge.kind = 1; ge.Zl = c->Z[l]; ge.Tl = c->T[l]; ge.nu = c->nu;
            gemm_nn(c, c->tmpA, c->Wt, c->tmpB, N, Cn, Cl, ge);
        } else {
            gemm_nn(c, c->G[l + 1], c->Wt, c->tmpA, N, Cn, Cl);                      // G_{l+1} W_{l+1}^T
            SpmmEpilogue epi;
            epi.kind = 1; epi.Zl = c->Z[l]; epi.Tl = c->T[l]; epi.nu = c->nu;
            aggregate(c, c->tmpA, c->tmpB, Cl, epi);
        }
        if (lowrank)
            timed(c, P_GEMM_GRADZ, 4.0 * (2.0 * (double)N * Cl + 2.0 * (double)N * Cn), 2.0 * (double)N * (Cl + Cn) * Cn, [&] {
                launch_gemm_nn_gradz(s, c->Z[l], c->T[l], c->tmpA, c->Bcat, c->tmpV, N, Cl, Cn, Cn, c->nu);
            });
        else
            gemm_nn(c, c->tmpB, c->W[l + 1], c->tmpV, N, Cl, Cn);                    // grad W_{l+1}
        aggregate_segments(c, c->tmpV, c->P, Cn);                                    // A~_{r,m} (grad W) per segment
        launch_reset_units(s, units, M, sp);
        ZTrialArgs a;
        const cadmm_ctx::DevChunks& ct = c->d_chunks[Cn > 32 ? 1 : 0];        // a segment's row of P and T_{l+1} has Cn columns
        a.chunk_unit = ct.unit; a.chunk_kind = ct.kind;
        a.chunk_begin = ct.begin; a.chunk_end = ct.end;
        a.n_chunks = ct.n;
        a.unit_chunk_ptr = ct.unit_ptr; a.M = M;
        a.segc_row = c->d_segc_row;
        a.Zl = c->Z[l]; a.gradZ = lowrank ? nullptr : c->tmpB; a.Tl = c->T[l]; a.Cl = Cl;
        a.SG = c->tmpA; a.Wt = c->Wt;
        a.Tn = c->T[l + 1]; a.Zn = c->Z[l + 1]; a.U = c->U; a.P = c->P; a.Cn = Cn;
        a.Gn = c->G[l + 1];
        a.next_is_last = next_last;
        a.sp = sp; a.units = units; a.partials = c->partials; a.status = c->status;
        // one pass reads Z_l, grad, T_l over the rows and P with T_{l+1}, Z_{l+1} (or G_L alone) over the segments
        const double zt_bytes = 4.0 * ((lowrank ? 2.0 : 3.0) * (double)N * Cl + (lowrank ? (double)N * Cn : 0.0) +
                                       (next_last ? 2.0 : 3.0) * (double)c->hg.n_seg * Cn) + 4.0 * (double)c->hg.n_seg;
        timed(c, P_Z_TRIAL, zt_bytes, 0.0, [&] {
            a.first_pass = 1; a.ncand = 1;
            launch_z_trial(s, a);
            a.first_pass = 0; a.ncand = kMaxCand;
            for (int p = 0; p < more_passes; ++p) launch_z_trial(s, a);
        });
        timed(c, P_Z_STEP, 4.0 * (3.0 * (double)N * Cl + (double)N + (lowrank ? (double)N * Cn : 0.0)), 0.0, [&] {
            if (lowrank)
                launch_z_step_lowrank(s, c->Z[l], c->T[l], c->tmpA, c->Wt, c->nu, c->d_row_comm, N, Cl, Cn, units, c->hg.M);
            else
                launch_z_step(s, c->Z[l], c->tmpB, c->d_row_comm, N, Cl, units, c->hg.M);
        });
    }
}

// last layer Z_L (Eq. 5) and, for dual_form 0, the dual step (Eq. 2), both from Z_L^k, U^k and the T_L in memory
void last_layer_update(cadmm_ctx* c) {
    const int L = c->L;
    const int64_t N = c->hg.N;
    if (c->fista_mode == 1 && c->J > 0) {
        // FISTA with backtracking on the blocks Z_{L,m}: J + 1 passes over the rows, a device-side search per step
        FistaArgs a;
        a.ZL = c->Z[L]; a.U = c->U; a.TL = c->T[L]; a.Xb = c->fistaX; a.Yb = c->fistaY; a.labels = c->d_labels;
        const cadmm_ctx::DevChunks& ct = c->d_chunks[0];                      // only the chunks of rows are used here
        a.chunk_unit = ct.unit; a.chunk_kind = ct.kind; a.chunk_begin = ct.begin; a.chunk_end = ct.end;
        a.n_chunks = ct.n; a.unit_chunk_ptr = ct.unit_ptr; a.M = c->hg.M;
        a.CL = c->C[L]; a.risk = c->risk; a.J = c->J; a.update_u = c->dual_form == 0 ? 1 : 0; a.rho = c->rho;
        a.sp = search_params(c); a.units = c->unitsF; a.partials = c->partials; a.status = c->status;
        // candidates per step: 1 (16 in stage 0), then a pass of 4, then passes of 16 until max_backtrack + 1 are covered
        const int wide_passes = (c->max_bt + kMaxCand - 1) / kMaxCand;
        timed(c, P_LAST_LAYER, 4.0 * (double)N * c->C[L] * (3.0 + 7.0 * (c->J - 1) + 6.0) + 4.0 * (double)N * (c->J + 1), 0.0, [&] {
            double t = 1.0;
            for (int stage = 0; stage <= c->J; ++stage) {
                float mom = 0.f;
                if (stage > 0) {                        // the step taken in this stage is step stage-1
                    const double tn = 0.5 * (1.0 + std::sqrt(1.0 + 4.0 * t * t));
                    mom = (float)((t - 1.0) / tn);
                    t = tn;
                }
                launch_fista_stage(c->stream, a, stage, 0, mom);
                if (stage < c->J) {
                    if (stage > 0) launch_fista_stage(c->stream, a, stage, 1, 0.f);
                    for (int p = stage == 0 ? 1 : 0; p < wide_passes; ++p) launch_fista_stage(c->stream, a, stage, 2, 0.f);
                }
            }
        });
        return;
    }
    timed(c, P_LAST_LAYER, 4.0 * (5.0 * (double)N * c->C[L] + (double)N), 0.0, [&] {
        launch_last_layer(c->stream, c->Z[L], c->U, c->T[L], c->d_labels, N, c->C[L], c->risk, c->rho, c->J,
                          c->dual_form == 0 ? 1 : 0);
    });
}

// Serial baseline of Section 4.1 read as a Gauss-Seidel pass: for l = 1..L first W_l, then Z_l, each from the newest
// values.  T_l is formed anew once Z_{l-1} has changed; T_{l+1} = A~ Z_l^k W_{l+1}^k comes from the base evaluation.
void sweep_layer_by_layer(cadmm_ctx* c) {
    const int L = c->L;
    const int64_t N = c->hg.N;
    base_eval(c, false);
    for (int l = 1; l <= L; ++l) {
        if (l >= 2) {
            compute_T(c, l, true);
            if (!gradient_on_the_fly(c, l))
                timed(c, P_G_ONLY, 4.0 * (double)N * c->C[l] * (l == L ? 4 : 3), 0.0, [&] {
                    launch_G_only(c->stream, c->T[l], c->Z[l], c->U, c->G[l], N * c->C[l], l == L, c->nu, c->rho);
                });
        }
        w_update(c, l);
        if (l < L) z_update_hidden(c, l);
        else last_layer_update(c);
    }
    if (c->t1_age >= 0) c->t1_age++;
    if (c->dual_form == 1) c->u_pending = true;
    c->iter++;
    c->base_valid = false;
}

// Algorithm 1: every W_l from (W^k, Z^k, U^k), then every Z_{l,m} from (W^{k+1}, Z^k, U^k), then U.
void sweep(cadmm_ctx* c) {
    if (c->schedule == 1) { sweep_layer_by_layer(c); return; }
    const int L = c->L;
    base_eval(c, false);
    for (int l = 1; l <= L; ++l) w_update(c, l);
    // Ascending l keeps the Z update Jacobi although Z_l is overwritten in place: layer l reads Z_{l+1}^k
    // (not yet touched) and T_l, T_{l+1}, which were formed from Z^k before any Z changed.
    for (int l = 1; l <= L - 1; ++l) {
        z_update_hidden(c, l);
        // T_l is not read again in this sweep: bring it to the new Z_{l-1} (P and theta of layer l-1)
        if (l >= 2) carry_T(c, l);
    }
    last_layer_update(c);
    carry_T(c, L);
    if (c->t1_age >= 0) c->t1_age++;
    if (c->dual_form == 1) c->u_pending = true;      // applied by the next base evaluation, on the new iterates
    c->iter++;
    c->base_valid = false;
}

int check_launch(cadmm_ctx* c, const char* where) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(c, e, where);
    return CADMM_OK;
}

// copy an N x C matrix out in the caller's node order
int download_rows(cadmm_ctx* c, const float* src_internal, int C, float* dst_host) {
    const int64_t N = c->hg.N;
    launch_permute_rows(c->stream, src_internal, c->tmpA, c->d_perm, N, C, 1);   // tmpA[perm[r]] = src[r]
    HIP_TRY(c, hipMemcpyAsync(dst_host, c->tmpA, (size_t)N * C * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return check_launch(c, "download_rows");
}

int upload_rows(cadmm_ctx* c, const float* src, int on_device, int C, float* dst_internal) {
    const int64_t N = c->hg.N;
    HIP_TRY(c, hipMemcpyAsync(c->tmpA, src, (size_t)N * C * sizeof(float),
                              on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c->stream));
    launch_permute_rows(c->stream, c->tmpA, dst_internal, c->d_perm, N, C, 0);   // dst[r] = tmpA[perm[r]]
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return check_launch(c, "upload_rows");
}

void drop_graphs(cadmm_ctx* c) {
    for (auto& cube : c->graphs)
        for (auto& plane : cube)
            for (auto& row : plane)
                for (auto& slot : row) {
                    if (slot.exec) (void)hipGraphExecDestroy(slot.exec);
                    slot.exec = nullptr;
                    slot.tried = false;
                }
}

}  // namespace

extern "C" {

int cadmm_create(cadmm_ctx** out, int device, void* hip_stream) {
    if (!out) return CADMM_EINVAL;
    *out = nullptr;
    if (device >= 0) {
        int ndev = 0;
        if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return CADMM_EHIP;
        if (hipSetDevice(device) != hipSuccess) return CADMM_EHIP;
    }
    cadmm_ctx* c = new (std::nothrow) cadmm_ctx();
    if (!c) return CADMM_ENOMEM;
    c->device = device;
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    *out = c;
    return CADMM_OK;
}

void cadmm_destroy(cadmm_ctx* ctx) {
    if (!ctx) return;
    if (ctx->device >= 0) {
        (void)hipStreamSynchronize(ctx->stream);
        for (auto& r : ctx->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
        for (auto e : ctx->prof_pool) (void)hipEventDestroy(e);
        drop_graphs(ctx);
    }
    delete ctx;
}

const char* cadmm_last_error(cadmm_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int cadmm_partition(cadmm_ctx* c, int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst, int32_t M,
                    int32_t* comm) {
    if (!c) return CADMM_EINVAL;
    std::string e = partition_graph(N, n_edges, src, dst, M, comm);
    if (!e.empty()) return fail(c, CADMM_EINVAL, e);
    return CADMM_OK;
}

int cadmm_build_graph(cadmm_ctx* c, int64_t N, int64_t n_edges, const int32_t* src, const int32_t* dst, int32_t M,
                      const int32_t* comm) {
    if (!c) return CADMM_EINVAL;
    if (c->has_ws) return fail(c, CADMM_EORDER, "graph cannot change after the workspace is set");
    std::string e = build_host_graph(c->hg, N, n_edges, src, dst, M, comm, kChunkRows);
    if (!e.empty()) { c->has_graph = false; return fail(c, CADMM_EINVAL, e); }
    c->has_graph = true;
    return CADMM_OK;
}

int cadmm_graph_sizes(cadmm_ctx* c, int64_t* nnz, int64_t* n_segments, int64_t* n_halo_rows) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_graph) return fail(c, CADMM_EORDER, "build_graph first");
    if (nnz) *nnz = c->hg.nnz;
    if (n_segments) *n_segments = c->hg.n_seg;
    if (n_halo_rows) *n_halo_rows = c->hg.n_halo_rows;
    return CADMM_OK;
}

int cadmm_get_graph(cadmm_ctx* c, int32_t* perm, int64_t* row_ptr, int32_t* col, float* val, int64_t* seg_ptr,
                    int32_t* seg_row, int32_t* seg_comm, int64_t* comm_row_ptr, uint8_t* neighbour) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_graph) return fail(c, CADMM_EORDER, "build_graph first");
    const HostGraph& g = c->hg;
    auto cp = [](auto* dst, const auto& v) { if (dst && !v.empty()) std::memcpy(dst, v.data(), v.size() * sizeof(v[0])); };
    cp(perm, g.perm); cp(row_ptr, g.row_ptr); cp(col, g.col); cp(val, g.val);
    cp(seg_ptr, g.seg_ptr); cp(seg_row, g.seg_row); cp(seg_comm, g.seg_comm);
    cp(comm_row_ptr, g.comm_row_ptr); cp(neighbour, g.neighbour);
    return CADMM_OK;
}

int cadmm_get_segment_order(cadmm_ctx* c, int64_t* order) {
    if (!c || !order) return CADMM_EINVAL;
    if (!c->has_graph) return fail(c, CADMM_EORDER, "build_graph first");
    if (!c->hg.segc_order.empty()) std::memcpy(order, c->hg.segc_order.data(), c->hg.segc_order.size() * sizeof(int64_t));
    return CADMM_OK;
}

int cadmm_set_model(cadmm_ctx* c, const cadmm_model* m) {
    if (!c || !m || !m->C) return CADMM_EINVAL;
    if (c->has_ws) return fail(c, CADMM_EORDER, "model cannot change after the workspace is set");
    if (m->L < 2 || m->L > 64) return fail(c, CADMM_EINVAL, "L must be in [2, 64]");
    for (int l = 0; l <= m->L; ++l)
        if (m->C[l] < 1 || m->C[l] > 4096) return fail(c, CADMM_EINVAL, "layer width must be in [1, 4096]");
    if (m->C[m->L] > 64) return fail(c, CADMM_EUNSUPPORTED, "at most 64 classes");
    if (m->risk != 0 && m->risk != 1) return fail(c, CADMM_EINVAL, "risk must be 0 or 1");
    if (!(m->nu > 0) || !(m->rho > 0) || !(m->tau0 > 0) || !(m->theta0 > 0) || !(m->eta > 1))
        return fail(c, CADMM_EINVAL, "nu, rho, tau0, theta0 must be positive and eta > 1");
    if (m->max_backtrack < 0 || m->max_backtrack > 64) return fail(c, CADMM_EINVAL, "max_backtrack must be in [0, 64]");
    if (m->fista_iters < 0) return fail(c, CADMM_EINVAL, "fista_iters must be non-negative");
    if (m->dual_form != 0 && m->dual_form != 1) return fail(c, CADMM_EINVAL, "dual_form must be 0 or 1");
    if (m->schedule != 0 && m->schedule != 1) return fail(c, CADMM_EINVAL, "schedule must be 0 or 1");
    if (m->step_policy != 0 && m->step_policy != 1) return fail(c, CADMM_EINVAL, "step_policy must be 0 or 1");
    if (m->fista_mode != 0 && m->fista_mode != 1) return fail(c, CADMM_EINVAL, "fista_mode must be 0 or 1");
    c->L = m->L;
    c->C.assign(m->C, m->C + m->L + 1);
    c->risk = m->risk;
    c->nu = m->nu; c->rho = m->rho; c->tau0 = m->tau0; c->theta0 = m->theta0; c->eta = m->eta;
    c->max_bt = m->max_backtrack;
    c->J = m->fista_iters;
    c->dual_form = m->dual_form;
    c->schedule = m->schedule;
    c->step_policy = m->step_policy;
    c->fista_mode = m->fista_mode;
    c->agg_first.assign(c->L + 1, 0);
    for (int l = 2; l <= c->L; ++l) c->agg_first[l] = (3 * c->C[l] < c->C[l - 1]) ? 1 : 0;
    c->has_model = true;
    return CADMM_OK;
}

int cadmm_workspace_bytes(cadmm_ctx* c, size_t* bytes) {
    if (!c || !bytes) return CADMM_EINVAL;
    if (!c->has_graph || !c->has_model) return fail(c, CADMM_EORDER, "build_graph and set_model first");
    if (c->has_ws) { *bytes = c->ws_bytes; return CADMM_OK; }
    *bytes = layout(c, nullptr);
    return CADMM_OK;
}

int cadmm_set_workspace(cadmm_ctx* c, void* dev_ptr, size_t bytes) {
    if (!c || !dev_ptr) return CADMM_EINVAL;
    if (!c->has_graph || !c->has_model) return fail(c, CADMM_EORDER, "build_graph and set_model first");
    if (c->has_ws) return fail(c, CADMM_EORDER, "workspace already set");
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context (device -1) has no device path");
    if ((reinterpret_cast<uintptr_t>(dev_ptr) & 255) != 0) return fail(c, CADMM_EINVAL, "workspace must be 256-byte aligned");
    const size_t need = layout(c, nullptr);
    if (bytes < need) return fail(c, CADMM_ENOMEM, "workspace too small");
    HIP_TRY(c, hipSetDevice(c->device));
    layout(c, static_cast<char*>(dev_ptr));
    c->ws = static_cast<char*>(dev_ptr);
    c->ws_bytes = need;
    const HostGraph& g = c->hg;
    hipStream_t s = c->stream;
    HIP_TRY(c, upload(s, c->d_row_comm, g.row_comm));
    HIP_TRY(c, upload(s, c->d_perm, g.perm));
    auto upload_schedule = [&](cadmm_ctx::DevSchedule& d, const RowSchedule& rs) -> hipError_t {
        hipError_t e;
        for (int l = 0; l < 7; ++l) {
            BlockTable bt;
            build_block_table(rs, l, bt);
            static_assert(sizeof(BlockRows) == sizeof(int4), "table entries are read as int4");
            if ((int64_t)bt.blocks.size() != d.n_blocks[l] || !block_table_ok(rs, l, bt)) return hipErrorInvalidValue;
            for (int k = 0; k <= 8; ++k) d.xcd_start[l][k] = bt.xcd_start[k];
            if (!bt.blocks.empty()) {
                // synchronous with respect to the host buffer: the table is a temporary
                if ((e = hipMemcpyAsync(d.blocks[l], bt.blocks.data(), bt.blocks.size() * sizeof(BlockRows),
                                        hipMemcpyHostToDevice, s)) != hipSuccess) return e;
                if ((e = hipStreamSynchronize(s)) != hipSuccess) return e;
            }
        }
        static_assert(sizeof(RowRecord) == sizeof(int4) && sizeof(EntryPair) == sizeof(int2), "records are read as int4, pairs as int2");
        if (!rs.rec.empty() && (e = hipMemcpyAsync(d.rec, rs.rec.data(), rs.rec.size() * sizeof(RowRecord), hipMemcpyHostToDevice, s)) != hipSuccess) return e;
        if ((e = hipMemcpyAsync(d.ent, rs.ent.data(), rs.ent.size() * sizeof(EntryPair), hipMemcpyHostToDevice, s)) != hipSuccess) return e;
        if ((e = upload(s, d.long_row, rs.long_row)) != hipSuccess) return e;
        return upload(s, d.long_ptr, rs.long_part_ptr);
    };
    HIP_TRY(c, upload_schedule(c->d_rows, g.row_sched));
    HIP_TRY(c, upload_schedule(c->d_segs, g.seg_sched));
    HIP_TRY(c, upload(s, c->d_seg1_pos, g.seg1_pos));
    HIP_TRY(c, upload(s, c->d_seg1_col, g.seg1_col));
    HIP_TRY(c, upload(s, c->d_seg1_val, g.seg1_val));
    HIP_TRY(c, upload(s, c->d_segc_row, g.segc_row));
    for (int t = 0; t < 2; ++t) {
        std::vector<int32_t> cu, ck, cb, ce;
        for (const Chunk& ch : (t == 0 ? g.chunks : g.chunks_wide)) { cu.push_back(ch.unit); ck.push_back(ch.kind); cb.push_back(ch.begin); ce.push_back(ch.end); }
        HIP_TRY(c, upload(s, c->d_chunks[t].unit, cu));
        HIP_TRY(c, upload(s, c->d_chunks[t].kind, ck));
        HIP_TRY(c, upload(s, c->d_chunks[t].begin, cb));
        HIP_TRY(c, upload(s, c->d_chunks[t].end, ce));
        HIP_TRY(c, upload(s, c->d_chunks[t].unit_ptr, t == 0 ? g.unit_chunk_ptr : g.unit_chunk_ptr_wide));
    }
    HIP_TRY(c, upload(s, c->d_row_seg_ptr, g.row_seg_ptr));
    HIP_TRY(c, upload(s, c->d_seg_comm, g.seg_comm));
    HIP_TRY(c, upload(s, c->d_seg_pos, g.seg_pos));
    HIP_TRY(c, hipMemsetAsync(c->status, 0, 4 * sizeof(int32_t), s));
    HIP_TRY(c, hipStreamSynchronize(s));     // the host vectors above must outlive the copies
    c->has_ws = true;
    return CADMM_OK;
}

int cadmm_set_data(cadmm_ctx* c, const float* X, const int32_t* labels, int x_on_device) {
    if (!c || !X || !labels) return CADMM_EINVAL;
    if (!c->has_ws) return fail(c, CADMM_EORDER, "set_workspace first");
    const int64_t N = c->hg.N;
    std::vector<int32_t> lab(N);
    for (int64_t r = 0; r < N; ++r) {
        int32_t y = labels[c->hg.perm[r]];
        if (y < -1 || y >= c->C[c->L]) return fail(c, CADMM_EINVAL, "label out of range");
        lab[r] = y;
    }
    HIP_TRY(c, hipMemcpyAsync(c->d_labels, lab.data(), N * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    int rc = upload_rows(c, X, x_on_device, c->C[0], c->Z[0]);     // synchronises
    if (rc != CADMM_OK) return rc;
    c->h_labels.swap(lab);
    c->has_data = true;
    c->has_init = false;
    return CADMM_OK;
}

int cadmm_init(cadmm_ctx* c, const float* const* W0) {
    if (!c || !W0) return CADMM_EINVAL;
    if (!c->has_data) return fail(c, CADMM_EORDER, "set_data first");
    const int L = c->L;
    const int64_t N = c->hg.N;
    hipStream_t s = c->stream;
    for (int l = 1; l <= L; ++l) {
        if (!W0[l - 1]) return fail(c, CADMM_EINVAL, "null weight pointer");
        HIP_TRY(c, hipMemcpyAsync(c->W[l], W0[l - 1], (size_t)c->C[l - 1] * c->C[l] * sizeof(float),
                                  hipMemcpyHostToDevice, s));
    }
    c->t1_age = -1;
    aggregate(c, c->Z[0], c->H[1], c->C[0], SpmmEpilogue());      // A~ Z_0 never changes
    for (int l = 1; l <= L; ++l) {
        compute_T(c, l);
        launch_relu(s, c->T[l], c->Z[l], N * c->C[l], l < L);
    }
    HIP_TRY(c, hipMemsetAsync(c->U, 0, (size_t)N * c->C[L] * sizeof(float), s));
    HIP_TRY(c, hipMemsetAsync(c->status, 0, 4 * sizeof(int32_t), s));
    launch_fill_units(s, c->unitsW, L, (double)c->tau0);
    launch_fill_units(s, c->unitsZ, (L - 1) * c->hg.M, (double)c->theta0);
    launch_fill_units(s, c->unitsF, c->hg.M, (double)c->rho);
    HIP_TRY(c, hipStreamSynchronize(s));                           // W0 host buffers may be freed by the caller
    c->iter = 0;
    c->base_valid = false;
    c->have_prev = false;
    c->dual_valid = false;
    c->u_pending = false;
    c->has_init = true;
    return check_launch(c, "init");
}

int cadmm_run(cadmm_ctx* c, int32_t k) {
    if (!c || k < 0) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    for (int i = 0; i < k; ++i) {
        const bool graphable = c->use_graph && c->stream != nullptr && !c->prof_on;
        if (!graphable) { sweep(c); continue; }
        const bool t1_skip = !c->base_valid && t1_reusable(c);
        cadmm_ctx::GraphSlot& slot =
            c->graphs[c->base_valid ? 1 : 0][c->have_prev ? 1 : 0][c->u_pending ? 1 : 0][t1_skip ? 1 : 0];
        if (!slot.tried) {
            // capture this variant once; the capture enqueues nothing, sweep() only advances the host flags
            slot.tried = true;
            const bool bv = c->base_valid, hp = c->have_prev, dv = c->dual_valid, up = c->u_pending;
            const int it = c->iter, age = c->t1_age;
            if (hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed) == hipSuccess) {
                sweep(c);
                hipGraph_t graph = nullptr;
                hipError_t e = hipStreamEndCapture(c->stream, &graph);
                if (e == hipSuccess && graph) {
                    if (hipGraphInstantiate(&slot.exec, graph, nullptr, nullptr, 0) != hipSuccess) slot.exec = nullptr;
                    (void)hipGraphDestroy(graph);
                }
                c->base_valid = bv; c->have_prev = hp; c->dual_valid = dv; c->u_pending = up; c->iter = it;
                c->t1_age = age;
            }
            (void)hipGetLastError();
        }
        if (slot.exec && hipGraphLaunch(slot.exec, c->stream) == hipSuccess) {
            // the host-side bookkeeping sweep() would have done
            if (!c->base_valid) {
                c->dual_valid = c->have_prev;
                c->have_prev = true;
                if (!t1_skip) c->t1_age = 0;
            }
            if (c->t1_age >= 0) c->t1_age++;
            c->base_valid = false;
            c->u_pending = c->dual_form == 1;
            c->iter++;
        } else {
            sweep(c);
        }
    }
    return check_launch(c, "run");
}

int cadmm_eval(cadmm_ctx* c, cadmm_stats* out, double* layer_penalty) {
    if (!c || !out) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    const int L = c->L;
    base_eval(c, true);
    launch_risk(c->stream, c->Z[L], c->d_labels, c->hg.N, c->C[L], c->risk, c->partials, c->scalars + L);
    std::vector<LayerScalars> sc(L + 1);
    int32_t st[4] = {0, 0, 0, 0};
    HIP_TRY(c, hipMemcpyAsync(sc.data(), c->scalars, (L + 1) * sizeof(LayerScalars), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipMemcpyAsync(st, c->status, sizeof(st), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    double pen = 0.0;
    for (int l = 1; l < L; ++l) {
        pen += sc[l].phi;
        if (layer_penalty) layer_penalty[l - 1] = sc[l].phi;
    }
    out->risk = sc[L].risk;
    out->objective = sc[L].risk + pen;
    out->lagrangian = out->objective + sc[L].phi;
    out->primal_res = std::sqrt(sc[L].res2);
    out->dual_res = c->dual_valid ? (double)c->rho * std::sqrt(sc[L].dT2) : 0.0;
    out->iter = c->iter;
    out->status = st[0];
    if (!std::isfinite(out->lagrangian)) out->status |= CADMM_STATUS_NONFINITE;
    return check_launch(c, "eval");
}

int cadmm_predict(cadmm_ctx* c, int32_t* pred, float* logits, double* accuracy) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    const int L = c->L;
    const int64_t N = c->hg.N;
    hipStream_t s = c->stream;
    // forward pass of Problem 1's constraints with the current weights; the per-layer scratch of the
    // sweep is reused, so the next sweep or readout recomputes its base evaluation
    const float* in = c->Z[0];
    for (int l = 1; l <= L; ++l) {
        if (c->agg_first[l]) {
            gemm_nn(c, in, c->W[l], c->tmpV, N, c->C[l - 1], c->C[l]);
            aggregate(c, c->tmpV, c->T[l], c->C[l], SpmmEpilogue());
        } else {
            if (l >= 2) aggregate(c, in, c->H[l], c->C[l - 1], SpmmEpilogue());
            gemm_nn(c, c->H[l], c->W[l], c->T[l], N, c->C[l - 1], c->C[l]);
        }
        if (l < L) {
            launch_relu(s, c->T[l], c->G[l], N * c->C[l], 1);
            in = c->G[l];
        }
    }
    c->base_valid = false;
    c->t1_age = -1;                 // the T buffers now hold the forward pass, not images of the state
    launch_argmax_rows(s, c->T[L], c->d_pred, N, c->C[L]);
    std::vector<int32_t> p((size_t)N);
    HIP_TRY(c, hipMemcpyAsync(p.data(), c->d_pred, N * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    int64_t labelled = 0, hit = 0;
    for (int64_t r = 0; r < N; ++r) {
        if (pred) pred[c->hg.perm[r]] = p[r];
        if (c->h_labels[r] >= 0) { ++labelled; hit += (p[r] == c->h_labels[r]); }
    }
    if (accuracy) *accuracy = labelled ? (double)hit / (double)labelled : 0.0;
    if (logits) {
        int rc = download_rows(c, c->T[L], c->C[L], logits);
        if (rc != CADMM_OK) return rc;
    }
    return check_launch(c, "predict");
}

int cadmm_get_W(cadmm_ctx* c, int32_t l, float* dst) {
    if (!c || !dst) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    if (l < 1 || l > c->L) return fail(c, CADMM_EINVAL, "layer out of range");
    HIP_TRY(c, hipMemcpyAsync(dst, c->W[l], (size_t)c->C[l - 1] * c->C[l] * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return CADMM_OK;
}

int cadmm_get_Z(cadmm_ctx* c, int32_t l, float* dst) {
    if (!c || !dst) return CADMM_EINVAL;
    if (!c->has_data) return fail(c, CADMM_EORDER, "set_data first");
    if (l < 0 || l > c->L) return fail(c, CADMM_EINVAL, "layer out of range");
    if (l > 0 && !c->has_init) return fail(c, CADMM_EORDER, "init first");
    return download_rows(c, c->Z[l], c->C[l], dst);
}

int cadmm_get_U(cadmm_ctx* c, float* dst) {
    if (!c || !dst) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    if (c->u_pending) base_eval(c, false);   // dual_form 1: the step of the last sweep rides on the base evaluation
    return download_rows(c, c->U, c->C[c->L], dst);
}

int cadmm_get_steps(cadmm_ctx* c, double* tau, double* theta, int32_t* n_trials, double* sq_grad) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    const int L = c->L, M = c->hg.M;
    const int nz = (L - 1) * M;
    std::vector<Unit> uw(L), uz(nz);
    HIP_TRY(c, hipMemcpyAsync(uw.data(), c->unitsW, L * sizeof(Unit), hipMemcpyDeviceToHost, c->stream));
    if (nz) HIP_TRY(c, hipMemcpyAsync(uz.data(), c->unitsZ, nz * sizeof(Unit), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int l = 0; l < L; ++l) {
        if (tau) tau[l] = uw[l].step;
        if (n_trials) n_trials[l] = uw[l].ntrials;
        if (sq_grad) sq_grad[l] = uw[l].g;
    }
    for (int i = 0; i < nz; ++i) {
        if (theta) theta[i] = uz[i].step;
        if (n_trials) n_trials[L + i] = uz[i].ntrials;
        if (sq_grad) sq_grad[L + i] = uz[i].g;
    }
    return CADMM_OK;
}

int cadmm_get_fista(cadmm_ctx* c, double* L, int32_t* n_trials) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    const int M = c->hg.M;
    std::vector<Unit> u(M);
    HIP_TRY(c, hipMemcpyAsync(u.data(), c->unitsF, M * sizeof(Unit), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (int m = 0; m < M; ++m) {
        if (L) L[m] = u[m].step;
        if (n_trials) n_trials[m] = u[m].total + u[m].ntrials;     // the last step's count is not yet added up
    }
    return CADMM_OK;
}

int cadmm_set_state(cadmm_ctx* c, const float* const* W, const float* const* Z, const float* U, const double* tau,
                    const double* theta) {
    if (!c) return CADMM_EINVAL;
    if (!c->has_init) return fail(c, CADMM_EORDER, "init first");
    const int L = c->L, M = c->hg.M;
    hipStream_t s = c->stream;
    if (c->u_pending) base_eval(c, false);   // finish the pending dual step before anything is overwritten
    c->t1_age = -1;
    if (W)
        for (int l = 1; l <= L; ++l)
            if (W[l - 1])
                HIP_TRY(c, hipMemcpyAsync(c->W[l], W[l - 1], (size_t)c->C[l - 1] * c->C[l] * sizeof(float), hipMemcpyHostToDevice, s));
    if (Z)
        for (int l = 1; l <= L; ++l)
            if (Z[l - 1]) {
                int rc = upload_rows(c, Z[l - 1], 0, c->C[l], c->Z[l]);
                if (rc != CADMM_OK) return rc;
            }
    if (U) {
        int rc = upload_rows(c, U, 0, c->C[L], c->U);
        if (rc != CADMM_OK) return rc;
    }
    if (tau || theta) {
        const int nz = (L - 1) * M;
        std::vector<Unit> uw(L), uz(nz);
        HIP_TRY(c, hipMemcpyAsync(uw.data(), c->unitsW, L * sizeof(Unit), hipMemcpyDeviceToHost, s));
        if (nz) HIP_TRY(c, hipMemcpyAsync(uz.data(), c->unitsZ, nz * sizeof(Unit), hipMemcpyDeviceToHost, s));
        HIP_TRY(c, hipStreamSynchronize(s));
        if (tau) for (int l = 0; l < L; ++l) { if (!(tau[l] > 0)) return fail(c, CADMM_EINVAL, "tau must be positive"); uw[l].step = tau[l]; }
        if (theta) for (int i = 0; i < nz; ++i) { if (!(theta[i] > 0)) return fail(c, CADMM_EINVAL, "theta must be positive"); uz[i].step = theta[i]; }
        HIP_TRY(c, hipMemcpyAsync(c->unitsW, uw.data(), L * sizeof(Unit), hipMemcpyHostToDevice, s));
        if (nz) HIP_TRY(c, hipMemcpyAsync(c->unitsZ, uz.data(), nz * sizeof(Unit), hipMemcpyHostToDevice, s));
    }
    HIP_TRY(c, hipStreamSynchronize(s));
    c->base_valid = false;
    c->have_prev = false;
    c->dual_valid = false;
    return CADMM_OK;
}

int cadmm_profile(cadmm_ctx* c, int enable) {
    if (!c) return CADMM_EINVAL;
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context");
    c->prof_on = enable != 0;
    if (enable) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        for (auto& r : c->prof_recs) { c->prof_pool.push_back(r.a); c->prof_pool.push_back(r.b); }
        c->prof_recs.clear();
        for (int i = 0; i < CADMM_PROFILE_CLASSES; ++i) {
            c->prof_ms[i] = 0; c->prof_launches[i] = 0; c->prof_bytes[i] = 0; c->prof_flops[i] = 0;
        }
    }
    return CADMM_OK;
}

int cadmm_get_profile(cadmm_ctx* c, double* ms, int64_t* records, double* bytes, double* flops) {
    if (!c) return CADMM_EINVAL;
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context");
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    for (auto& r : c->prof_recs) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
            c->prof_ms[r.cls] += (double)t;
            c->prof_launches[r.cls] += 1;
        }
        c->prof_pool.push_back(r.a);
        c->prof_pool.push_back(r.b);
    }
    c->prof_recs.clear();
    for (int i = 0; i < CADMM_PROFILE_CLASSES; ++i) {
        if (ms) ms[i] = c->prof_ms[i];
        if (records) records[i] = c->prof_launches[i];
        if (bytes) bytes[i] = c->prof_bytes[i];
        if (flops) flops[i] = c->prof_flops[i];
    }
    return CADMM_OK;
}

const char* cadmm_profile_class_name(int32_t cls) {
    if (cls < 0 || cls >= CADMM_PROFILE_CLASSES) return "";
    if (get_gemm_split()) {                      // the wide products run as the bf16-split kernel: name that symbol
        if (cls == P_GEMM_NN_128) return "gemm_nn_split_kernel<0>";
        if (cls == P_GEMM_NN_128_GRADZ) return "gemm_nn_split_kernel<1>";
        if (cls == P_GEMM_NN_128_TRIAL) return "gemm_nn_split_kernel<2>+finish";
        if (cls == P_GEMM_TN) return "gemm_tn_split_kernel+reduce";
    }
    return kProfNames[cls];
}

int cadmm_tune(cadmm_ctx* c, const char* key, int32_t value) {
    if (!c || !key) return CADMM_EINVAL;
    if (std::strcmp(key, "use_graph") == 0) { c->use_graph = value != 0; return CADMM_OK; }
    const bool k_lowrank = std::strcmp(key, "use_lowrank") == 0, k_spec = std::strcmp(key, "use_speculative") == 0;
    const bool k_split = std::strcmp(key, "gemm_split") == 0, k_refresh = std::strcmp(key, "t1_refresh") == 0;
    if (k_lowrank || k_spec || k_split || k_refresh) {
        // each of these changes the launch sequence of an iteration: captured iterations of this context are dropped
        if (k_lowrank) c->use_lowrank = value != 0;
        else if (k_spec) c->use_speculative = value != 0;
        else if (k_refresh) { c->t1_refresh = value; c->t1_age = -1; }
        else set_gemm_split(value);                  // process-wide
        drop_graphs(c);
        return CADMM_OK;
    }
    if (std::strcmp(key, "spmm_tile_cols") == 0) { set_spmm_tile_cols(value); return CADMM_OK; }
    if (std::strcmp(key, "spmm_xcd_remap") == 0) { set_spmm_xcd_remap(value); drop_graphs(c); return CADMM_OK; }
    return fail(c, CADMM_EINVAL, "unknown tuning key");
}

int cadmm_op_aggregate(cadmm_ctx* c, const float* X, int32_t width, float* Y) {
    if (!c || !X || !Y || width < 1) return CADMM_EINVAL;
    if (!c->has_ws) return fail(c, CADMM_EORDER, "set_workspace first");
    if (width > max_of(c->C, 0, c->L)) return fail(c, CADMM_ENOMEM, "width exceeds the widest layer the workspace was sized for");
    aggregate(c, X, Y, width, SpmmEpilogue());
    return check_launch(c, "op_aggregate");
}

int cadmm_op_aggregate_segments(cadmm_ctx* c, const float* V, int32_t width, float* P) {
    if (!c || !V || !P || width < 1) return CADMM_EINVAL;
    if (!c->has_ws) return fail(c, CADMM_EORDER, "set_workspace first");
    if (width > max_of(c->C, 0, c->L)) return fail(c, CADMM_ENOMEM, "width exceeds the widest layer the workspace was sized for");
    aggregate_segments(c, V, P, width);
    return check_launch(c, "op_aggregate_segments");
}

int cadmm_op_transform(cadmm_ctx* c, const float* A, int64_t n, int32_t K, const float* B, int32_t C, float* out) {
    if (!c || !A || !B || !out || n < 1 || K < 1 || C < 1) return CADMM_EINVAL;
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context (device -1) has no device path");
    gemm_nn(c, A, B, out, n, K, C);
    return check_launch(c, "op_transform");
}

int cadmm_op_wgrad(cadmm_ctx* c, const float* A, const float* G, int64_t n, int32_t K, int32_t C, float* out) {
    if (!c || !A || !G || !out || n < 1 || K < 1 || C < 1) return CADMM_EINVAL;
    if (!c->has_ws) return fail(c, CADMM_EORDER, "set_workspace first");
    if (gemm_tn_scratch_floats(n, K, C) > c->tn_partial_floats) return fail(c, CADMM_ENOMEM, "shape needs more scratch than the model reserved");
    timed(c, C > 32 ? P_GEMM_TN : P_GEMM_TN_32, 4.0 * ((double)n * K + (double)n * C + (double)K * C),
          2.0 * (double)n * K * C, [&] { launch_gemm_tn(c->stream, A, G, out, n, K, C, c->tn_partial); });
    return check_launch(c, "op_wgrad");
}

int cadmm_op_wgrad_noalloc(cadmm_ctx* c, const float* A, const float* G, int64_t n, int32_t K, int32_t C, float* out) {
    if (!c || !A || !G || !out || n < 1 || K < 1 || C < 1) return CADMM_EINVAL;
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context (device -1) has no device path");
    if (c->device >= kMaxDevices) return fail(c, CADMM_EUNSUPPORTED, "device index beyond the static scratch table");
    const size_t need = gemm_tn_scratch_floats(n, K, C);
    if (need > kStaticScratchFloats)
        return fail(c, CADMM_ENOMEM, "shape needs " + std::to_string(need) + " floats of scratch, the static scratch holds " +
                                         std::to_string(kStaticScratchFloats) + "; use cadmm_op_wgrad with a workspace");
    int current = -1;
    HIP_TRY(c, hipGetDevice(&current));
    if (current != c->device) HIP_TRY(c, hipSetDevice(c->device));
    float* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[c->device]) {
            // once per device, with that device current: every GPU has its own copy of the array at its own address
            void* p = nullptr;
            hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) {
                if (current != c->device) (void)hipSetDevice(current);
                return hip_fail(c, e, "hipGetSymbolAddress(scratch)");
            }
            g_scratch_ptr[c->device] = static_cast<float*>(p);
        }
        ptr = g_scratch_ptr[c->device];
    }
    // every entry of the partial matrices that the reduction reads is written by the product first: nothing to clear
    launch_gemm_tn(c->stream, A, G, out, n, K, C, ptr);
    int rc = check_launch(c, "op_wgrad_noalloc");
    if (current != c->device) (void)hipSetDevice(current);
    return rc;
}

int cadmm_op_calibrate(cadmm_ctx* c, int32_t kind, const float* src, float* dst, int64_t count, int32_t reps,
                       double* rate) {
    if (!c || !dst || !rate || count < 4 || reps < 1 || kind < 0 || kind > 8) return CADMM_EINVAL;
    if (c->device < 0) return fail(c, CADMM_EUNSUPPORTED, "host-only context");
    const int blocks = 2048;
    if ((kind == 0 || kind == 8) && (!src || count % 4 != 0)) return fail(c, CADMM_EINVAL, "copy needs src and a multiple of four floats");
    if ((kind == 1 || (kind >= 4 && kind <= 7)) && count > (1 << 24)) return fail(c, CADMM_EINVAL, "at most 2^24 MFMA steps per launch");
    if (kind == 2 || kind == 3) {
        if (!c->has_ws) return fail(c, CADMM_EORDER, "set_workspace first");
        if (!src || (count != 4 && count != 8 && count != 16 && count != 32 && count != 64 && count != 128 && count != 256))
            return fail(c, CADMM_EINVAL, "gather calibration needs src and a row width of 4, 8, ... 256 floats");
    }
    hipEvent_t a = nullptr, b = nullptr;
    HIP_TRY(c, hipEventCreate(&a));
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(c, CADMM_EHIP, "hipEventCreate"); }
    double work = 0.0;
    auto once = [&] {
        if (kind == 0) { launch_stream_copy(c->stream, src, dst, count); work += 8.0 * (double)count; }
        else if (kind == 8) { launch_stream_update(c->stream, src, dst, count); work += 12.0 * (double)count; }
        else if (kind == 1) work += launch_mfma_chain(c->stream, dst, blocks, (int)count);
        else if (kind >= 4 && kind <= 7) work += launch_mfma_bf16_chain(c->stream, dst, blocks, (int)count, kind == 4 ? 0 : kind == 5 ? 4 : kind == 6 ? 6 : 8);
        else {
            const RowSchedule& rs = kind == 2 ? c->hg.row_sched : c->hg.seg_sched;
            work += launch_gather_calibration(c->stream, schedule_of(c, kind == 2 ? c->d_rows : c->d_segs, rs), rs.n_chunks(), src,
                                              (int)count, dst);
        }
    };
    once();                                     // untimed first launch
    work = 0.0;
    (void)hipEventRecord(a, c->stream);
    for (int i = 0; i < reps; ++i) once();
    (void)hipEventRecord(b, c->stream);
    hipError_t e = hipEventSynchronize(b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (e != hipSuccess) return hip_fail(c, e, "op_calibrate");
    *rate = ms > 0.f ? work / ((double)ms * 1e-3) / ((kind == 1 || (kind >= 4 && kind <= 7)) ? 1e12 : 1e9) : 0.0;
    return check_launch(c, "op_calibrate");
}

}  // extern "C"
