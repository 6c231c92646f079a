"""ctypes binding over the C ABI in include/cadmm.h: argument marshalling only.

Every step of the ADMM sweep runs inside libcadmm.so (HIP, gfx950).  PyTorch is used
for one thing: it allocates the device workspace and owns the stream the library
enqueues on.  If the library has not been built this module raises; there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcadmm.so")
_lib = None

EXPORTS = [
    "cadmm_create", "cadmm_destroy", "cadmm_last_error", "cadmm_build_graph", "cadmm_graph_sizes",
    "cadmm_get_graph", "cadmm_get_segment_order", "cadmm_set_model", "cadmm_workspace_bytes",
    "cadmm_set_workspace", "cadmm_set_data", "cadmm_init", "cadmm_run", "cadmm_eval", "cadmm_get_W",
    "cadmm_get_Z", "cadmm_get_U", "cadmm_get_steps", "cadmm_set_state", "cadmm_op_aggregate",
    "cadmm_op_aggregate_segments", "cadmm_op_transform", "cadmm_op_wgrad",
    "cadmm_profile", "cadmm_get_profile", "cadmm_profile_class_name", "cadmm_tune", "cadmm_predict",
    "cadmm_partition", "cadmm_op_calibrate", "cadmm_op_wgrad_noalloc", "cadmm_get_fista",
]
PROFILE_CLASSES = 19


class CadmmError(RuntimeError):
    pass


class _Model(C.Structure):
    _fields_ = [("L", C.c_int32), ("C", C.POINTER(C.c_int32)), ("risk", C.c_int32),
                ("nu", C.c_float), ("rho", C.c_float), ("tau0", C.c_float), ("theta0", C.c_float),
                ("eta", C.c_float), ("max_backtrack", C.c_int32), ("fista_iters", C.c_int32),
                ("dual_form", C.c_int32), ("schedule", C.c_int32), ("step_policy", C.c_int32),
                ("fista_mode", C.c_int32)]


class _Stats(C.Structure):
    _fields_ = [("objective", C.c_double), ("lagrangian", C.c_double), ("risk", C.c_double),
                ("primal_res", C.c_double), ("dual_res", C.c_double), ("iter", C.c_int32),
                ("status", C.c_int32)]


def load_library():
    """dlopen libcadmm.so and check that every declared entry point is exported."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise CadmmError(f"{_LIB_PATH} is missing: run `python __graft_entry__.py` (build) first; "
                         "there is no fallback path")
    # PyTorch ships its own copy of the HIP runtime.  Load it first so that this library binds to the
    # same runtime instance: two HIP runtimes in one process do not both see the GPU.
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise CadmmError(f"libcadmm.so does not export {name}")
    lib.cadmm_last_error.restype = C.c_char_p
    lib.cadmm_last_error.argtypes = [C.c_void_p]
    lib.cadmm_destroy.restype = None
    lib.cadmm_destroy.argtypes = [C.c_void_p]
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.cadmm_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.cadmm_build_graph.argtypes = [vp, i64, i64, vp, vp, i32, vp]
    lib.cadmm_partition.argtypes = [vp, i64, i64, vp, vp, i32, vp]
    lib.cadmm_graph_sizes.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.cadmm_get_graph.argtypes = [vp] * 10
    lib.cadmm_get_segment_order.argtypes = [vp, vp]
    lib.cadmm_set_model.argtypes = [vp, C.POINTER(_Model)]
    lib.cadmm_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.cadmm_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.cadmm_set_data.argtypes = [vp, vp, vp, C.c_int]
    lib.cadmm_init.argtypes = [vp, vp]
    lib.cadmm_run.argtypes = [vp, i32]
    lib.cadmm_eval.argtypes = [vp, C.POINTER(_Stats), vp]
    lib.cadmm_get_W.argtypes = [vp, i32, vp]
    lib.cadmm_get_Z.argtypes = [vp, i32, vp]
    lib.cadmm_get_U.argtypes = [vp, vp]
    lib.cadmm_get_steps.argtypes = [vp, vp, vp, vp, vp]
    lib.cadmm_set_state.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.cadmm_get_fista.argtypes = [vp, vp, vp]
    lib.cadmm_op_aggregate.argtypes = [vp, vp, i32, vp]
    lib.cadmm_op_aggregate_segments.argtypes = [vp, vp, i32, vp]
    lib.cadmm_op_transform.argtypes = [vp, vp, i64, i32, vp, i32, vp]
    lib.cadmm_op_wgrad.argtypes = [vp, vp, vp, i64, i32, i32, vp]
    lib.cadmm_op_wgrad_noalloc.argtypes = [vp, vp, vp, i64, i32, i32, vp]
    lib.cadmm_op_calibrate.argtypes = [vp, i32, vp, vp, i64, i32, C.POINTER(C.c_double)]
    lib.cadmm_tune.argtypes = [vp, C.c_char_p, i32]
    lib.cadmm_predict.argtypes = [vp, vp, vp, C.POINTER(C.c_double)]
    lib.cadmm_profile.argtypes = [vp, C.c_int]
    lib.cadmm_get_profile.argtypes = [vp, vp, vp, vp, vp]
    lib.cadmm_profile_class_name.argtypes = [i32]
    lib.cadmm_profile_class_name.restype = C.c_char_p
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _ptr_array(arrs):
    """Array of L host pointers (None entries stay null)."""
    out = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


class Solver:
    """One problem instance on one GPU.  Method names mirror the C entry points."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.device = device
        stream_handle = None
        if device >= 0:
            import torch
            if not torch.cuda.is_available():
                raise CadmmError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
            self._torch = torch
            torch.cuda.set_device(device)
            # a stream of its own (default priority): the library can then replay an iteration as a HIP graph
            self.stream = torch.cuda.Stream(device=device)
            stream_handle = self.stream.cuda_stream
        h = C.c_void_p()
        rc = self.lib.cadmm_create(C.byref(h), device, C.c_void_p(stream_handle))
        if rc != 0:
            raise CadmmError(f"cadmm_create failed ({rc})")
        self.h = h
        self.workspace = None
        self.N = self.M = self.L = 0
        self.dims: List[int] = []

    def close(self):
        if getattr(self, "h", None):
            self.lib.cadmm_destroy(self.h)
            self.h = None
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != 0:
            msg = self.lib.cadmm_last_error(self.h)
            raise CadmmError(f"{what} failed ({rc}): {msg.decode() if msg else ''}")

    # ---- graph
    def partition(self, N, src, dst, M):
        """Communities for a graph without them: int32 [N] in [0, M) (host work, any context)."""
        src = np.ascontiguousarray(src, dtype=np.int32)
        dst = np.ascontiguousarray(dst, dtype=np.int32)
        if src.shape != dst.shape:
            raise CadmmError("edge array size mismatch")
        comm = np.empty(int(N), np.int32)
        self._check(self.lib.cadmm_partition(self.h, N, src.shape[0], _ptr(src), _ptr(dst), M, _ptr(comm)),
                    "cadmm_partition")
        return comm

    def build_graph(self, N, src, dst, M, comm=None):
        src = np.ascontiguousarray(src, dtype=np.int32)
        dst = np.ascontiguousarray(dst, dtype=np.int32)
        comm = None if comm is None else np.ascontiguousarray(comm, dtype=np.int32)
        if src.shape != dst.shape or (comm is not None and comm.shape[0] != N):
            raise CadmmError("edge / community array size mismatch")
        self._check(self.lib.cadmm_build_graph(self.h, N, src.shape[0], _ptr(src), _ptr(dst), M, _ptr(comm)),
                    "cadmm_build_graph")
        self.N, self.M = int(N), int(M)

    def graph_sizes(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        self._check(self.lib.cadmm_graph_sizes(self.h, C.byref(a), C.byref(b), C.byref(c)), "cadmm_graph_sizes")
        return int(a.value), int(b.value), int(c.value)

    def get_graph(self):
        nnz, nseg, _ = self.graph_sizes()
        N, M = self.N, self.M
        out = dict(perm=np.empty(N, np.int32), row_ptr=np.empty(N + 1, np.int64), col=np.empty(nnz, np.int32),
                   val=np.empty(nnz, np.float32), seg_ptr=np.empty(nseg + 1, np.int64),
                   seg_row=np.empty(nseg, np.int32), seg_comm=np.empty(nseg, np.int32),
                   comm_row_ptr=np.empty(M + 1, np.int64), neighbour=np.empty(M * M, np.uint8))
        self._check(self.lib.cadmm_get_graph(self.h, *[_ptr(out[k]) for k in
                                                       ("perm", "row_ptr", "col", "val", "seg_ptr", "seg_row",
                                                        "seg_comm", "comm_row_ptr", "neighbour")]), "cadmm_get_graph")
        out["neighbour"] = out["neighbour"].reshape(M, M).astype(bool)
        return out

    def get_segment_order(self):
        _, nseg, _ = self.graph_sizes()
        order = np.empty(nseg, np.int64)
        self._check(self.lib.cadmm_get_segment_order(self.h, _ptr(order)), "cadmm_get_segment_order")
        return order

    # ---- model / workspace / data
    def set_model(self, dims, *, nu, rho, tau0, theta0, eta, max_backtrack, fista_iters, risk=0, dual_form=0,
                  schedule=0, step_policy=0, fista_mode=0):
        self.dims = [int(d) for d in dims]
        self.L = len(self.dims) - 1
        arr = (C.c_int32 * len(self.dims))(*self.dims)
        m = _Model(self.L, arr, risk, nu, rho, tau0, theta0, eta, max_backtrack, fista_iters, dual_form, schedule,
                   step_policy, fista_mode)
        self._check(self.lib.cadmm_set_model(self.h, C.byref(m)), "cadmm_set_model")

    def workspace_bytes(self):
        b = C.c_size_t()
        self._check(self.lib.cadmm_workspace_bytes(self.h, C.byref(b)), "cadmm_workspace_bytes")
        return int(b.value)

    def set_workspace(self):
        torch = self._torch
        nbytes = self.workspace_bytes()
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=f"cuda:{self.device}")
        base = self.workspace.data_ptr()
        aligned = (base + 255) & ~255
        self._check(self.lib.cadmm_set_workspace(self.h, C.c_void_p(aligned), nbytes), "cadmm_set_workspace")
        return nbytes

    def set_data(self, X, labels):
        X = np.ascontiguousarray(X, dtype=np.float32)
        labels = np.ascontiguousarray(labels, dtype=np.int32)
        if X.shape != (self.N, self.dims[0]) or labels.shape != (self.N,):
            raise CadmmError("X / labels shape mismatch")
        self._check(self.lib.cadmm_set_data(self.h, _ptr(X), _ptr(labels), 0), "cadmm_set_data")

    def init(self, W0):
        W0 = [np.ascontiguousarray(w, dtype=np.float32) for w in W0]
        for l, w in enumerate(W0, 1):
            if w.shape != (self.dims[l - 1], self.dims[l]):
                raise CadmmError("W0 shape mismatch")
        self._check(self.lib.cadmm_init(self.h, _ptr_array(W0)), "cadmm_init")

    # ---- iterate / read
    def run(self, k=1):
        self._check(self.lib.cadmm_run(self.h, k), "cadmm_run")

    def eval(self):
        st = _Stats()
        pen = np.zeros(max(self.L - 1, 1), np.float64)
        self._check(self.lib.cadmm_eval(self.h, C.byref(st), _ptr(pen)), "cadmm_eval")
        return dict(objective=st.objective, lagrangian=st.lagrangian, risk=st.risk, primal_res=st.primal_res,
                    dual_res=st.dual_res, iter=st.iter, status=st.status, layer_penalty=list(pen[:self.L - 1]))

    def predict(self):
        """(classes [N], logits [N, C_L], accuracy over labelled nodes) with the current weights."""
        pred = np.empty(self.N, np.int32)
        logits = np.empty((self.N, self.dims[-1]), np.float32)
        acc = C.c_double()
        self._check(self.lib.cadmm_predict(self.h, _ptr(pred), _ptr(logits), C.byref(acc)), "cadmm_predict")
        return pred, logits, float(acc.value)

    def get_W(self, l):
        out = np.empty((self.dims[l - 1], self.dims[l]), np.float32)
        self._check(self.lib.cadmm_get_W(self.h, l, _ptr(out)), "cadmm_get_W")
        return out

    def get_Z(self, l):
        out = np.empty((self.N, self.dims[l]), np.float32)
        self._check(self.lib.cadmm_get_Z(self.h, l, _ptr(out)), "cadmm_get_Z")
        return out

    def get_U(self):
        out = np.empty((self.N, self.dims[-1]), np.float32)
        self._check(self.lib.cadmm_get_U(self.h, _ptr(out)), "cadmm_get_U")
        return out

    def get_steps(self):
        nz = (self.L - 1) * self.M
        tau = np.empty(self.L, np.float64)
        theta = np.empty(nz, np.float64)
        trials = np.empty(self.L + nz, np.int32)
        sq = np.empty(self.L + nz, np.float64)
        self._check(self.lib.cadmm_get_steps(self.h, _ptr(tau), _ptr(theta), _ptr(trials), _ptr(sq)),
                    "cadmm_get_steps")
        return tau, theta, trials, sq

    def get_fista(self):
        """(L [M], candidates tested [M]) of the last solve of Z_L with backtracking (fista_mode 1)."""
        L = np.empty(self.M, np.float64)
        trials = np.empty(self.M, np.int32)
        self._check(self.lib.cadmm_get_fista(self.h, _ptr(L), _ptr(trials)), "cadmm_get_fista")
        return L, trials

    def set_state(self, W=None, Z=None, U=None, tau=None, theta=None):
        keep = []

        def prep(lst):
            if lst is None:
                return None
            arrs = [None if a is None else np.ascontiguousarray(a, dtype=np.float32) for a in lst]
            keep.append(arrs)
            return _ptr_array(arrs)
        Wp, Zp = prep(W), prep(Z)
        U = None if U is None else np.ascontiguousarray(U, dtype=np.float32)
        tau = None if tau is None else np.ascontiguousarray(tau, dtype=np.float64)
        theta = None if theta is None else np.ascontiguousarray(theta, dtype=np.float64)
        self._check(self.lib.cadmm_set_state(self.h, Wp, Zp, _ptr(U), _ptr(tau), _ptr(theta)), "cadmm_set_state")

    # ---- kernel-level calls on torch device tensors (internal row order)
    def _enter(self):
        """Tensors come from torch's current stream; the library runs on its own."""
        self.stream.wait_stream(self._torch.cuda.current_stream(self.device))

    def _leave(self):
        self._torch.cuda.current_stream(self.device).wait_stream(self.stream)

    def op_aggregate(self, X):
        torch = self._torch
        assert X.is_cuda and X.dtype == torch.float32 and X.is_contiguous() and X.shape[0] == self.N
        Y = torch.empty_like(X)
        self._enter()
        self._check(self.lib.cadmm_op_aggregate(self.h, C.c_void_p(X.data_ptr()), X.shape[1],
                                                C.c_void_p(Y.data_ptr())), "cadmm_op_aggregate")
        self._leave()
        return Y

    def op_aggregate_segments(self, V):
        torch = self._torch
        assert V.is_cuda and V.dtype == torch.float32 and V.is_contiguous() and V.shape[0] == self.N
        nseg = self.graph_sizes()[1]
        P = torch.empty((nseg, V.shape[1]), dtype=torch.float32, device=V.device)
        self._enter()
        self._check(self.lib.cadmm_op_aggregate_segments(self.h, C.c_void_p(V.data_ptr()), V.shape[1],
                                                         C.c_void_p(P.data_ptr())), "cadmm_op_aggregate_segments")
        self._leave()
        return P

    def op_transform(self, A, B):
        torch = self._torch
        assert A.is_cuda and B.is_cuda and A.is_contiguous() and B.is_contiguous() and A.shape[1] == B.shape[0]
        out = torch.empty((A.shape[0], B.shape[1]), dtype=torch.float32, device=A.device)
        self._enter()
        self._check(self.lib.cadmm_op_transform(self.h, C.c_void_p(A.data_ptr()), A.shape[0], A.shape[1],
                                                C.c_void_p(B.data_ptr()), B.shape[1], C.c_void_p(out.data_ptr())),
                    "cadmm_op_transform")
        self._leave()
        return out

    def op_calibrate(self, kind, count, reps=5):
        """'copy': GB/s of a plain device copy of `count` floats; 'update': GB/s of dst = 0.999 dst + src in place; 'mfma': TFLOP/s of register-only fp32 MFMA chains;
        'mfma_bf16': the same with bf16 MFMAs, 'mfma_bf16_valu4/6/8': with that many vector instructions after each;
        'gather' / 'gather_segments': GB/s of the aggregation's gathers alone at a row width of `count` floats."""
        torch = self._torch
        rate = C.c_double()
        self._enter()
        if kind in ("copy", "update"):
            src = torch.ones(count, dtype=torch.float32, device=f"cuda:{self.device}")
            dst = torch.zeros_like(src)
            torch.cuda.current_stream().synchronize()
            rc = self.lib.cadmm_op_calibrate(self.h, 0 if kind == "copy" else 8, C.c_void_p(src.data_ptr()),
                                             C.c_void_p(dst.data_ptr()), count, reps, C.byref(rate))
        elif kind == "mfma":
            dst = torch.empty(2048 * 256, dtype=torch.float32, device=f"cuda:{self.device}")
            rc = self.lib.cadmm_op_calibrate(self.h, 1, None, C.c_void_p(dst.data_ptr()), count, reps, C.byref(rate))
        elif kind in ("mfma_bf16", "mfma_bf16_valu4", "mfma_bf16_valu6", "mfma_bf16_valu8"):
            dst = torch.empty(2048 * 256, dtype=torch.float32, device=f"cuda:{self.device}")
            code = {"mfma_bf16": 4, "mfma_bf16_valu4": 5, "mfma_bf16_valu6": 6, "mfma_bf16_valu8": 7}[kind]
            rc = self.lib.cadmm_op_calibrate(self.h, code, None, C.c_void_p(dst.data_ptr()), count, reps, C.byref(rate))
        elif kind in ("gather", "gather_segments"):
            src = torch.randn(self.N, count, dtype=torch.float32, device=f"cuda:{self.device}")
            dst = torch.empty(2048 * 256, dtype=torch.float32, device=f"cuda:{self.device}")
            torch.cuda.current_stream().synchronize()
            rc = self.lib.cadmm_op_calibrate(self.h, 2 if kind == "gather" else 3, C.c_void_p(src.data_ptr()),
                                             C.c_void_p(dst.data_ptr()), count, reps, C.byref(rate))
        else:
            raise CadmmError(f"unknown calibration {kind}")
        self._check(rc, "cadmm_op_calibrate")
        self._leave()
        return float(rate.value)

    def op_wgrad(self, A, G):
        torch = self._torch
        assert A.is_cuda and G.is_cuda and A.is_contiguous() and G.is_contiguous() and A.shape[0] == G.shape[0]
        out = torch.empty((A.shape[1], G.shape[1]), dtype=torch.float32, device=A.device)
        self._enter()
        self._check(self.lib.cadmm_op_wgrad(self.h, C.c_void_p(A.data_ptr()), C.c_void_p(G.data_ptr()), A.shape[0],
                                            A.shape[1], G.shape[1], C.c_void_p(out.data_ptr())), "cadmm_op_wgrad")
        self._leave()
        return out

    def op_wgrad_noalloc(self, A, G, out=None):
        """out = A^T G through the entry point that allocates nothing; `out` may be a preallocated tensor."""
        torch = self._torch
        assert A.is_cuda and G.is_cuda and A.is_contiguous() and G.is_contiguous() and A.shape[0] == G.shape[0]
        if out is None:
            out = torch.empty((A.shape[1], G.shape[1]), dtype=torch.float32, device=A.device)
        self._enter()
        self._check(self.lib.cadmm_op_wgrad_noalloc(self.h, C.c_void_p(A.data_ptr()), C.c_void_p(G.data_ptr()),
                                                    A.shape[0], A.shape[1], G.shape[1], C.c_void_p(out.data_ptr())),
                    "cadmm_op_wgrad_noalloc")
        self._leave()
        return out

    def tune(self, key, value):
        self._check(self.lib.cadmm_tune(self.h, key.encode(), int(value)), "cadmm_tune")

    # ---- per-kernel-class timing
    def profile(self, enable=True):
        self._check(self.lib.cadmm_profile(self.h, 1 if enable else 0), "cadmm_profile")

    def get_profile(self):
        n = PROFILE_CLASSES
        ms, rec = np.zeros(n, np.float64), np.zeros(n, np.int64)
        by, fl = np.zeros(n, np.float64), np.zeros(n, np.float64)
        self._check(self.lib.cadmm_get_profile(self.h, _ptr(ms), _ptr(rec), _ptr(by), _ptr(fl)), "cadmm_get_profile")
        out = {}
        for i in range(n):
            name = self.lib.cadmm_profile_class_name(i).decode()
            out[name] = dict(ms=float(ms[i]), records=int(rec[i]), bytes=float(by[i]), flops=float(fl[i]))
        return out

    # ---- convenience
    @classmethod
    def from_workload(cls, w, device=0):
        s = cls(device)
        s.build_graph(w.N, w.src, w.dst, w.M, w.comm)
        h = w.hyper
        s.set_model(w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                    max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"],
                    dual_form=h["dual_form"], schedule=h.get("schedule", 0),
                    step_policy=h.get("step_policy", 0), fista_mode=h.get("fista_mode", 0))
        s.set_workspace()
        s.set_data(w.X, w.labels)
        s.init(w.W0)
        return s
