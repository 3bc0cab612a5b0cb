"""ctypes binding of libdash.so (include/dash.h).

Argument marshalling only: tensors are checked (CUDA/HIP device, float32, contiguous,
shape [N,B,B]) and their device pointers handed to the C ABI.  torch is used for device
memory and for the stream; every arithmetic step runs in the library's HIP kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdash.so")

# enums of dash.h
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(5)
NEWTON_DB, CHEBYSHEV, COUPLED_NEWTON = 0, 1, 2
SCALE_FROBENIUS, SCALE_TRACE, SCALE_NONE, SCALE_POWER_ITERATION = 0, 1, 2, 3
FP32, BF16_ACC32, FP16_ACC32, BF16X3, BF16X6, FP16X3 = 0, 1, 2, 3, 4, 5

_METHODS = {"newton_db": NEWTON_DB, "ndb": NEWTON_DB, "chebyshev": CHEBYSHEV, "cheb": CHEBYSHEV,
            "coupled_newton": COUPLED_NEWTON, "cn": COUPLED_NEWTON}
_SCALINGS = {"frobenius": SCALE_FROBENIUS, "trace": SCALE_TRACE, "none": SCALE_NONE,
             "power_iteration": SCALE_POWER_ITERATION, "pi": SCALE_POWER_ITERATION}
_PRECISIONS = {"fp32": FP32, "bf16": BF16_ACC32, "fp16": FP16_ACC32, "bf16x3": BF16X3, "bf16x6": BF16X6, "fp16x3": FP16X3}


class DashError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dash status {status}: {message}")
        self.status = status


class _Stats(C.Structure):
    _fields_ = [("matmul_products", C.c_int64), ("matmul_launches", C.c_int64),
                ("matmul_block_products", C.c_double), ("matmul_ms", C.c_double),
                ("variant_launches", C.c_int64 * 4), ("variant_block_products", C.c_double * 4),
                ("variant_ms", C.c_double * 4), ("matmul_flops", C.c_double), ("variant_flops", C.c_double * 4)]


class _StepArgs(C.Structure):
    _fields_ = [
        ("G", C.c_void_p), ("S", C.c_void_p), ("X", C.c_void_p), ("U", C.c_void_p),
        ("N", C.c_int64), ("B", C.c_int32),
        ("beta", C.c_float), ("alpha", C.c_float), ("eps", C.c_float),
        ("method", C.c_int32), ("p", C.c_int32), ("iters", C.c_int32),
        ("scaling", C.c_int32), ("precision", C.c_int32), ("refresh", C.c_int32),
        ("cheb_coeffs", C.POINTER(C.c_double)), ("cheb_a", C.c_double), ("cheb_b", C.c_double),
        ("nonfinite_out", C.c_void_p),
        ("graft", C.c_int32), ("graft_acc", C.c_void_p), ("theta", C.c_void_p),
        ("beta_g", C.c_float), ("eps_g", C.c_float), ("lr", C.c_float),
    ]


class _LayerShape(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64)]


class _ModelInfo(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_buckets", C.c_int32), ("n_stacks", C.c_int32), ("B", C.c_int32),
                ("n_gradient_blocks", C.c_int64), ("n_factor_blocks", C.c_int64), ("arena_bytes", C.c_int64)]


class _ModelStepArgs(C.Structure):
    _fields_ = [("grads", C.POINTER(C.c_void_p)), ("updates", C.POINTER(C.c_void_p)),
                ("beta", C.c_float), ("alpha", C.c_float), ("eps", C.c_float),
                ("method", C.c_int32), ("iters", C.c_int32), ("scaling", C.c_int32), ("precision", C.c_int32),
                ("refresh", C.c_int32),
                ("cheb_coeffs", C.POINTER(C.c_double)), ("cheb_a", C.c_double), ("cheb_b", C.c_double),
                ("nonfinite_out", C.c_void_p),
                ("graft", C.c_int32), ("beta_g", C.c_float), ("eps_g", C.c_float),
                ("thetas", C.POINTER(C.c_void_p)), ("lr", C.c_float)]


_lib = None


def load_library(path: str = LIB_PATH):
    """Loads libdash.so and declares the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise DashError(ERR_HIP, f"{path} not found: build it first (python -m paper_2602_02016_amd.build)")
    # torch ships its own HIP runtime; if libdash.so were loaded first it would pull in the system one and
    # the process would end up with two (dash_create then fails with a HIP error).  Load torch's first.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp, i32, i64, f32, f64 = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_double
    lib.dash_create.argtypes = [C.POINTER(vp), i32, vp]
    lib.dash_destroy.argtypes = [vp]
    lib.dash_set_stream.argtypes = [vp, vp]
    lib.dash_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
    lib.dash_workspace_bytes.restype = C.c_size_t
    lib.dash_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.dash_last_error.argtypes = [vp]
    lib.dash_last_error.restype = C.c_char_p
    lib.dash_status_string.argtypes = [i32]
    lib.dash_status_string.restype = C.c_char_p
    lib.dash_reset_stats.argtypes = [vp]
    lib.dash_set_timing.argtypes = [vp, i32]
    lib.dash_set_symmetric.argtypes = [vp, i32]
    lib.dash_set_lanes.argtypes = [vp, i32]
    lib.dash_set_power_iteration.argtypes = [vp, i32, i32, vp, i32]
    lib.dash_get_stats.argtypes = [vp, C.POINTER(_Stats)]
    lib.dash_gemm_batched.argtypes = [vp, i32, i32, vp, vp, vp, vp, i64, i32, f32, f32, f32, i32]
    lib.dash_accumulate_factors.argtypes = [vp, vp, vp, vp, i64, i32, f32, f32]
    lib.dash_accumulate_factors_rect.argtypes = [vp, vp, vp, vp, i64, i32, i32, f32, f32]
    lib.dash_precondition_rect.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32]
    lib.dash_accumulate_vector.argtypes = [vp, vp, vp, i64, i32, f32, f32]
    lib.dash_precondition_vector.argtypes = [vp, vp, vp, vp, i64, i32]
    lib.dash_block_layer.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.dash_unblock_layer.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp, vp]
    lib.dash_block_layer_padded.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.dash_unblock_layer_padded.argtypes = [vp, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    lib.dash_model_create.argtypes = [vp, C.POINTER(_LayerShape), i32, i32, i32, i32, C.POINTER(vp)]
    lib.dash_model_destroy.argtypes = [vp]
    lib.dash_model_last_error.argtypes = [vp]
    lib.dash_model_last_error.restype = C.c_char_p
    lib.dash_model_get_info.argtypes = [vp, C.POINTER(_ModelInfo)]
    lib.dash_model_get_bucket.argtypes = [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(i64)]
    lib.dash_model_get_stack.argtypes = [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(i64),
                                         C.POINTER(vp), C.POINTER(vp)]
    lib.dash_model_workspace_bytes.argtypes = [vp, i32, i32]
    lib.dash_model_workspace_bytes.restype = C.c_size_t
    lib.dash_model_set_arena.argtypes = [vp, vp, C.c_size_t]
    lib.dash_model_step.argtypes = [vp, C.POINTER(_ModelStepArgs)]
    lib.dash_block_norms.argtypes = [vp, vp, i64, i32, f32, i32, vp]
    lib.dash_block_norms_static.argtypes = [vp, vp, i64, i32, f32, i32, vp]
    lib.dash_inverse_root.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, f32, i32, i32,
                                      C.POINTER(f64), f64, f64, vp, vp]
    lib.dash_chebyshev_fit.argtypes = [i32, i32, f64, f64, i32, C.POINTER(f64)]
    lib.dash_precondition.argtypes = [vp, vp, vp, vp, vp, i64, i32]
    lib.dash_graft_update.argtypes = [vp, vp, vp, vp, vp, i64, i32, f32, f32, f32, vp]
    lib.dash_step.argtypes = [vp, C.POINTER(_StepArgs)]
    lib.dash_graft_scale.argtypes = [vp, vp, vp, vp, i64, i64, f32, f32, vp, vp]
    lib.dash_apply_update.argtypes = [vp, vp, vp, i64, f32]
    for name in ("dash_create", "dash_destroy", "dash_set_stream", "dash_set_workspace", "dash_reset_stats", "dash_set_timing",
                 "dash_set_symmetric", "dash_set_lanes", "dash_set_power_iteration", "dash_accumulate_factors_rect",
                 "dash_block_layer", "dash_unblock_layer", "dash_block_layer_padded", "dash_unblock_layer_padded", "dash_graft_scale", "dash_apply_update", "dash_model_create", "dash_model_destroy",
                 "dash_model_get_info", "dash_model_get_bucket", "dash_model_get_stack", "dash_model_set_arena",
                 "dash_model_step",
                 "dash_precondition_rect", "dash_accumulate_vector", "dash_precondition_vector",
                 "dash_get_stats", "dash_gemm_batched", "dash_accumulate_factors", "dash_block_norms",
                 "dash_block_norms_static",
                 "dash_inverse_root", "dash_chebyshev_fit", "dash_precondition", "dash_graft_update", "dash_step"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def chebyshev_fit(p: int, degree: int, a: float, b: float, n_points: int = 10000):
    """Host-side coefficient fit of the library (double precision); returns a list."""
    lib = load_library()
    out = (C.c_double * (degree + 1))()
    st = lib.dash_chebyshev_fit(p, degree, a, b, n_points, out)
    if st != OK:
        raise DashError(st, lib.dash_status_string(st).decode())
    return list(out)


def layer_plan(m: int, n: int, B: int, pad_m: int = 1, pad_n: int = 1) -> dict:
    """Stack shapes block() gives for a [m, n] layer (host arithmetic only; see dash_block_layer and, for
    pad_m, pad_n > 1, dash_block_layer_padded: the rest extents are rounded up inside the stacks)."""
    Nm, Nn, rm, rn = m // B, n // B, m % B, n % B
    pm, pn = -(-rm // pad_m) * pad_m, -(-rn // pad_n) * pad_n
    return dict(full=(Nm * Nn, B, B), row_rest=(Nn if rm else 0, pm, B), col_rest=(Nm if rn else 0, B, pn),
                corner=(1 if rm and rn else 0, pm, pn))


def _enum(table, v):
    return table[v] if isinstance(v, str) else int(v)


class Dash:
    """One library context bound to a device and to torch's current stream on it."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        self._torch = torch
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise DashError(ERR_HIP, "no GPU visible; the HIP path has no CPU fallback")
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        h = C.c_void_p()
        st = self.lib.dash_create(C.byref(h), device, C.c_void_p(stream.cuda_stream))
        if st != OK:
            raise DashError(st, "dash_create failed: " + self.lib.dash_status_string(st).decode())
        self.h = h
        self._ws = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.dash_destroy(self.h)
            self.h = None

    def set_stream(self, stream):
        """Later calls enqueue on this torch stream (kept alive by this object)."""
        self.stream = stream
        self._check(self.lib.dash_set_stream(self.h, C.c_void_p(stream.cuda_stream)))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- helpers -----------------------------------------------------------------------
    def _check(self, st: int):
        if st != OK:
            raise DashError(st, self.lib.dash_last_error(self.h).decode() or self.lib.dash_status_string(st).decode())

    def _stack(self, t, name: str, n: Optional[int] = None, b: Optional[int] = None):
        torch = self._torch
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
                and t.dim() == 3 and t.shape[1] == t.shape[2]):
            raise DashError(ERR_INVALID_ARG, f"{name}: need a contiguous float32 device tensor of shape [N,B,B]")
        if n is not None and (t.shape[0] != n or t.shape[1] != b):
            raise DashError(ERR_INVALID_ARG, f"{name}: shape {tuple(t.shape)} does not match [{n},{b},{b}]")
        return C.c_void_p(t.data_ptr())

    def _dense(self, t, name: str, shape):
        torch = self._torch
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
                and tuple(t.shape) == tuple(shape)):
            raise DashError(ERR_INVALID_ARG, f"{name}: need a contiguous float32 device tensor of shape {list(shape)}")
        return C.c_void_p(t.data_ptr())

    def _vec(self, t, name: str, n: int, dtype):
        torch = self._torch
        if t is None:
            return C.c_void_p(None)
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous() and t.numel() == n):
            raise DashError(ERR_INVALID_ARG, f"{name}: need a contiguous {dtype} device tensor of {n} elements")
        return C.c_void_p(t.data_ptr())

    def workspace_bytes(self, n_blocks: int, B: int, method="newton_db", p: int = 4, precision="fp32") -> int:
        return int(self.lib.dash_workspace_bytes(n_blocks, B, _enum(_METHODS, method), p, _enum(_PRECISIONS, precision)))

    def set_workspace_bytes(self, nbytes: int):
        """Gives the context a torch-allocated scratch tensor of at least nbytes."""
        torch = self._torch
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = None
            self._ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=self.device)
        self._check(self.lib.dash_set_workspace(self.h, C.c_void_p(self._ws.data_ptr()), self._ws.numel()))

    def ensure_workspace(self, n_blocks: int, B: int, method="newton_db", p: int = 4, precision="fp32",
                         max_bytes: Optional[int] = None):
        """Sizes the workspace for n_blocks in one chunk (capped by max_bytes: the library then chunks)."""
        need = self.workspace_bytes(n_blocks, B, method, p, precision)
        if max_bytes is not None:
            need = min(need, int(max_bytes))
        if self._ws is None or self._ws.numel() < need:
            self.set_workspace_bytes(need)

    # ---- statistics --------------------------------------------------------------------
    def reset_stats(self):
        self._check(self.lib.dash_reset_stats(self.h))

    def set_timing(self, on: bool):
        self._check(self.lib.dash_set_timing(self.h, 1 if on else 0))

    def get_stats(self) -> dict:
        s = _Stats()
        self._check(self.lib.dash_get_stats(self.h, C.byref(s)))
        return dict(matmul_products=s.matmul_products, matmul_launches=s.matmul_launches,
                    matmul_block_products=s.matmul_block_products, matmul_ms=s.matmul_ms,
                    variant_launches=list(s.variant_launches),
                    variant_block_products=list(s.variant_block_products), variant_ms=list(s.variant_ms),
                    matmul_flops=s.matmul_flops, variant_flops=list(s.variant_flops))

    def set_power_iteration(self, start_vectors, sweeps: int):
        """Configures multi-Power-Iteration scaling: start_vectors is a contiguous float32 device
        tensor [rows, pool]; it is kept alive by this object."""
        torch = self._torch
        v = start_vectors
        if not (isinstance(v, torch.Tensor) and v.is_cuda and v.dtype == torch.float32 and v.is_contiguous() and v.dim() == 2):
            raise DashError(ERR_INVALID_ARG, "start_vectors: need a contiguous float32 device tensor [rows, pool]")
        self._pi_v0 = v
        self._check(self.lib.dash_set_power_iteration(self.h, v.shape[1], sweeps, C.c_void_p(v.data_ptr()), v.shape[0]))

    def set_lanes(self, on: bool):
        """Two-stream lanes for stacks of small blocks (see dash_set_lanes in dash.h); default on."""
        self._check(self.lib.dash_set_lanes(self.h, 1 if on else 0))

    def set_symmetric(self, on: bool):
        """Symmetric mode of the library (see dash_set_symmetric in dash.h); default on."""
        self._check(self.lib.dash_set_symmetric(self.h, 1 if on else 0))

    # ---- the calls of dash.h -------------------------------------------------------------
    def gemm_batched(self, A, Bm, C_out, D=None, transA=False, transB=False, alpha=1.0, beta=0.0, gamma=0.0,
                     precision="fp32"):
        n, b = A.shape[0], A.shape[1]
        if _enum(_PRECISIONS, precision) != FP32 and n > 0:
            need = n * b * b * 8                      # up to four 16-bit operand planes
            if self._ws is None or self._ws.numel() < need:
                self.set_workspace_bytes(need)
        self._check(self.lib.dash_gemm_batched(
            self.h, int(transA), int(transB), self._stack(A, "A"), self._stack(Bm, "B", n, b),
            self._stack(D, "D", n, b) if D is not None else C.c_void_p(None), self._stack(C_out, "C", n, b),
            n, b, alpha, beta, gamma, _enum(_PRECISIONS, precision)))
        return C_out

    def accumulate_factors(self, G, L, R, beta: float, alpha: Optional[float] = None):
        if alpha is None:
            alpha = 1.0 - beta
        n, b = G.shape[0], G.shape[1]
        self._check(self.lib.dash_accumulate_factors(self.h, self._stack(G, "G"), self._stack(L, "L", n, b),
                                                     self._stack(R, "R", n, b), n, b, beta, alpha))

    def block_layer(self, W, B: int, pad_m: int = 1, pad_n: int = 1):
        """block() of a [m, n] layer: returns dict(full, row_rest, col_rest, corner) of device stacks
        (None for an empty group).  pad_m, pad_n > 1: rest extents rounded up, padding zero filled."""
        torch = self._torch
        m, n = W.shape
        shapes = layer_plan(m, n, B, pad_m, pad_n)
        out = {k: (torch.empty(sh, dtype=torch.float32, device=self.device) if sh[0] * sh[1] * sh[2] > 0 else None)
               for k, sh in shapes.items()}
        ptr = lambda t: C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)
        self._check(self.lib.dash_block_layer_padded(self.h, self._dense(W, "W", (m, n)), m, n, B, pad_m, pad_n,
                                                     ptr(out["full"]), ptr(out["row_rest"]), ptr(out["col_rest"]),
                                                     ptr(out["corner"])))
        return out

    def unblock_layer(self, W, B: int, groups: dict, pad_m: int = 1, pad_n: int = 1):
        m, n = W.shape
        shapes = layer_plan(m, n, B, pad_m, pad_n)
        ptrs = []
        for k in ("full", "row_rest", "col_rest", "corner"):
            sh, t = shapes[k], groups.get(k)
            ptrs.append(self._dense(t, k, sh) if sh[0] * sh[1] * sh[2] > 0 else C.c_void_p(None))
        self._check(self.lib.dash_unblock_layer_padded(self.h, self._dense(W, "W", (m, n)), m, n, B, pad_m, pad_n, *ptrs))
        return W

    def accumulate_factors_rect(self, G, L, R, beta: float, alpha: Optional[float] = None):
        """Ragged blocks: G [N,Bm,Bn], L [N,Bm,Bm], R [N,Bn,Bn]."""
        if alpha is None:
            alpha = 1.0 - beta
        n, bm, bn = G.shape
        self._check(self.lib.dash_accumulate_factors_rect(
            self.h, self._dense(G, "G", (n, bm, bn)), self._dense(L, "L", (n, bm, bm)), self._dense(R, "R", (n, bn, bn)),
            n, bm, bn, beta, alpha))

    def precondition_rect(self, Linv, G, Rinv, U=None):
        torch = self._torch
        n, bm, bn = G.shape
        if U is None:
            U = torch.empty_like(G)
        if n > 0 and (self._ws is None or self._ws.numel() < n * bm * bn * 4):
            self.set_workspace_bytes(n * bm * bn * 4)
        self._check(self.lib.dash_precondition_rect(
            self.h, self._dense(Linv, "Linv", (n, bm, bm)), self._dense(G, "G", (n, bm, bn)),
            self._dense(Rinv, "Rinv", (n, bn, bn)), self._dense(U, "U", (n, bm, bn)), n, bm, bn))
        return U

    def accumulate_vector(self, g, L, beta: float, alpha: Optional[float] = None):
        """1-D parameters: g [N,B], L [N,B,B]."""
        if alpha is None:
            alpha = 1.0 - beta
        n, b = g.shape
        self._check(self.lib.dash_accumulate_vector(self.h, self._dense(g, "g", (n, b)), self._dense(L, "L", (n, b, b)),
                                                    n, b, beta, alpha))

    def precondition_vector(self, Linv, g, u=None):
        torch = self._torch
        n, b = g.shape
        if u is None:
            u = torch.empty_like(g)
        self._check(self.lib.dash_precondition_vector(self.h, self._dense(Linv, "Linv", (n, b, b)),
                                                      self._dense(g, "g", (n, b)), self._dense(u, "u", (n, b)), n, b))
        return u

    def block_norms(self, A, eps: float = 0.0, scaling="frobenius", out=None):
        torch = self._torch
        n, b = A.shape[0], A.shape[1]
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=self.device)
        self.ensure_workspace(max(n, 1), b, "chebyshev")
        self._check(self.lib.dash_block_norms(self.h, self._stack(A, "A"), n, b, eps, _enum(_SCALINGS, scaling),
                                              self._vec(out, "s_out", n, torch.float32)))
        return out

    def block_norms_static(self, A, out, eps: float = 0.0, scaling="frobenius"):
        """dash_block_norms_static: as block_norms, on the library's static scratch; `out` is the caller's
        [N] float32 device tensor (nothing is allocated here either)."""
        n, b = A.shape[0], A.shape[1]
        self._check(self.lib.dash_block_norms_static(self.h, self._stack(A, "A"), n, b, eps, _enum(_SCALINGS, scaling),
                                                     self._vec(out, "s_out", n, self._torch.float32)))
        return out

    def inverse_root(self, A, X=None, method="newton_db", p: int = 4, iters: int = 10, eps: float = 0.0,
                     scaling="frobenius", precision="fp32", cheb_coeffs: Optional[Sequence[float]] = None,
                     cheb_a: float = 0.0, cheb_b: float = 1.0, scale_out=None, nonfinite_out=None,
                     workspace_max_bytes: Optional[int] = None):
        torch = self._torch
        n, b = A.shape[0], A.shape[1]
        if X is None:
            X = torch.empty_like(A)
        coeffs = None
        if cheb_coeffs is not None:
            coeffs = (C.c_double * len(cheb_coeffs))(*[float(v) for v in cheb_coeffs])
            if _enum(_METHODS, method) == CHEBYSHEV and len(cheb_coeffs) != iters + 1:
                raise DashError(ERR_INVALID_ARG, "Chebyshev: need degree+1 coefficients")
        if n > 0:
            self.ensure_workspace(n, b, method, p, precision, workspace_max_bytes)
        self._check(self.lib.dash_inverse_root(
            self.h, self._stack(A, "A"), self._stack(X, "X", n, b), n, b, _enum(_METHODS, method), p, iters, eps,
            _enum(_SCALINGS, scaling), _enum(_PRECISIONS, precision), coeffs, cheb_a, cheb_b,
            self._vec(scale_out, "scale_out", n, torch.float32), self._vec(nonfinite_out, "nonfinite_out", n, torch.int32)))
        return X

    def precondition(self, Linv, G, Rinv, U=None):
        torch = self._torch
        n, b = G.shape[0], G.shape[1]
        if U is None:
            U = torch.empty_like(G)
        if n > 0 and (self._ws is None or self._ws.numel() < n * b * b * 4):
            self.set_workspace_bytes(n * b * b * 4)
        self._check(self.lib.dash_precondition(self.h, self._stack(Linv, "Linv", n, b), self._stack(G, "G"),
                                               self._stack(Rinv, "Rinv", n, b), self._stack(U, "U", n, b), n, b))
        return U

    def graft_update(self, G, U, Acc, theta=None, beta_g: float = 0.999, eps_g: float = 1e-8, lr: float = 0.0,
                     s_out=None):
        torch = self._torch
        n, b = G.shape[0], G.shape[1]
        if n > 0 and (self._ws is None or self._ws.numel() < 512 * n):
            self.set_workspace_bytes(512 * n)
        self._check(self.lib.dash_graft_update(
            self.h, self._stack(G, "G"), self._stack(U, "U", n, b), self._stack(Acc, "Acc", n, b),
            self._stack(theta, "theta", n, b) if theta is not None else C.c_void_p(None), n, b, beta_g, eps_g, lr,
            self._vec(s_out, "s_out", n, torch.float32)))

    def graft_scale(self, G, U, Acc, U_scaled=None, beta_g: float = 0.999, eps_g: float = 1e-8, s_out=None):
        """Grafting on a stack of blocks of any shape [N, ...]: Acc updated, U_scaled = s_b U_b (default: in place)."""
        torch = self._torch
        n = G.shape[0]
        elems = G[0].numel() if n else 4
        if U_scaled is None:
            U_scaled = U
        for t, name in ((G, "G"), (U, "U"), (Acc, "Acc"), (U_scaled, "U_scaled")):
            self._dense(t, name, tuple(G.shape))
        if n > 0 and (self._ws is None or self._ws.numel() < 512 * n):
            self.set_workspace_bytes(512 * n)
        self._check(self.lib.dash_graft_scale(self.h, C.c_void_p(G.data_ptr()), C.c_void_p(U.data_ptr()),
                                              C.c_void_p(Acc.data_ptr()), n, elems, beta_g, eps_g,
                                              C.c_void_p(U_scaled.data_ptr()), self._vec(s_out, "s_out", n, torch.float32)))
        return U_scaled

    def apply_update(self, theta, update, lr: float):
        self._dense(update, "update", tuple(theta.shape))
        self._dense(theta, "theta", tuple(theta.shape))
        self._check(self.lib.dash_apply_update(self.h, C.c_void_p(theta.data_ptr()), C.c_void_p(update.data_ptr()),
                                               theta.numel(), lr))
        return theta

    def step(self, G, S, X, U, beta: float, eps: float, alpha: Optional[float] = None, method="newton_db", p: int = 4,
             iters: int = 10, scaling="frobenius", precision="fp32", refresh: bool = True,
             cheb_coeffs: Optional[Sequence[float]] = None, cheb_a: float = 0.0, cheb_b: float = 1.0,
             nonfinite_out=None, graft_acc=None, theta=None, beta_g: float = 0.999, eps_g: float = 1e-8,
             lr: float = 0.0, workspace_max_bytes: Optional[int] = None):
        torch = self._torch
        n, b = G.shape[0], G.shape[1]
        if alpha is None:
            alpha = 1.0 - beta
        a = _StepArgs()
        a.G = self._stack(G, "G").value
        a.S = self._stack(S, "S", 2 * n, b).value
        a.X = self._stack(X, "X", 2 * n, b).value
        a.U = self._stack(U, "U", n, b).value
        a.N, a.B = n, b
        a.beta, a.alpha, a.eps = beta, alpha, eps
        a.method, a.p, a.iters = _enum(_METHODS, method), p, iters
        a.scaling, a.precision, a.refresh = _enum(_SCALINGS, scaling), _enum(_PRECISIONS, precision), int(refresh)
        keep = None
        if cheb_coeffs is not None:
            keep = (C.c_double * len(cheb_coeffs))(*[float(v) for v in cheb_coeffs])
            a.cheb_coeffs = C.cast(keep, C.POINTER(C.c_double))
        a.cheb_a, a.cheb_b = cheb_a, cheb_b
        a.nonfinite_out = self._vec(nonfinite_out, "nonfinite_out", 2 * n, torch.int32).value
        a.graft = int(graft_acc is not None)
        a.graft_acc = self._stack(graft_acc, "graft_acc", n, b).value if graft_acc is not None else None
        a.theta = self._stack(theta, "theta", n, b).value if theta is not None else None
        a.beta_g, a.eps_g, a.lr = beta_g, eps_g, lr
        if n > 0:
            self.ensure_workspace(2 * n, b, method, p, precision, workspace_max_bytes)
        self._check(self.lib.dash_step(self.h, C.byref(a)))
        return U


def model_plan(layers, B: int, p: int = 4, p_vec: int = 2, ctx_handle=None):
    """Host-side plan of dash_model_create for a list of layer shapes ((m, n), or (m,) / (m, 0) for a
    1-D parameter): dict(info=..., buckets=[(bm, bn, count)], stacks=[(size, p, count)]).  Needs no GPU
    when ctx_handle is None (planning never touches the context)."""
    lib = load_library()
    arr = (_LayerShape * len(layers))(*[_LayerShape(int(s[0]), int(s[1]) if len(s) > 1 else 0) for s in layers])
    h = C.c_void_p()
    st = lib.dash_model_create(ctx_handle, arr, len(layers), B, p, p_vec, C.byref(h))     # NULL context: planning only
    if st != OK:
        raise DashError(st, "dash_model_create: " + lib.dash_status_string(st).decode())
    try:
        return _describe_model(lib, h)
    finally:
        lib.dash_model_destroy(h)


def _describe_model(lib, h):
    info = _ModelInfo()
    lib.dash_model_get_info(h, C.byref(info))
    buckets, stacks = [], []
    for i in range(info.n_buckets):
        bm, bn, cnt = C.c_int32(), C.c_int32(), C.c_int64()
        lib.dash_model_get_bucket(h, i, C.byref(bm), C.byref(bn), C.byref(cnt))
        buckets.append((bm.value, bn.value, cnt.value))
    for i in range(info.n_stacks):
        size, p, cnt = C.c_int32(), C.c_int32(), C.c_int64()
        lib.dash_model_get_stack(h, i, C.byref(size), C.byref(p), C.byref(cnt), None, None)
        stacks.append((size.value, p.value, cnt.value))
    return dict(info={k: getattr(info, k) for k, _ in _ModelInfo._fields_}, buckets=buckets, stacks=stacks)


class DashModel:
    """All layers of a model in shared stacks (dash_model_* of dash.h).  The arena (optimizer state) is a
    torch tensor owned by this object, zero-initialised."""

    def __init__(self, dash: Dash, layers, B: int, p: int = 4, p_vec: int = 2):
        import torch
        self.dash, self.lib = dash, dash.lib
        self.shapes = [(int(s[0]), int(s[1]) if len(s) > 1 else 0) for s in layers]
        arr = (_LayerShape * len(self.shapes))(*[_LayerShape(m, n) for m, n in self.shapes])
        h = C.c_void_p()
        st = self.lib.dash_model_create(dash.h, arr, len(self.shapes), B, p, p_vec, C.byref(h))
        if st != OK:
            raise DashError(st, "dash_model_create: " + self.lib.dash_status_string(st).decode())
        self.h = h
        self.plan = _describe_model(self.lib, h)
        self.arena = torch.zeros(max(self.plan["info"]["arena_bytes"], 256), dtype=torch.uint8, device=dash.device)
        self._check(self.lib.dash_model_set_arena(h, C.c_void_p(self.arena.data_ptr()), self.arena.numel()))

    def _check(self, st: int):
        if st != OK:
            raise DashError(st, self.lib.dash_model_last_error(self.h).decode() or self.lib.dash_status_string(st).decode())

    def close(self):
        if getattr(self, "h", None):
            self.lib.dash_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def stack(self, i: int):
        """(S, X) of factor stack i as torch views [count, size, size] into the arena."""
        import torch
        size, p, cnt = self.plan["stacks"][i]
        S, X = C.c_void_p(), C.c_void_p()
        self._check(self.lib.dash_model_get_stack(self.h, i, None, None, None, C.byref(S), C.byref(X)))
        base = self.arena.data_ptr()
        n = cnt * size * size
        f = self.arena.view(torch.float32)
        return (f[(S.value - base) // 4:(S.value - base) // 4 + n].view(cnt, size, size),
                f[(X.value - base) // 4:(X.value - base) // 4 + n].view(cnt, size, size))

    def step(self, grads, updates, beta: float, eps: float, alpha: Optional[float] = None, method="newton_db",
             iters: int = 10, scaling="frobenius", precision="fp32", refresh: bool = True,
             cheb_coeffs: Optional[Sequence[float]] = None, cheb_a: float = 0.0, cheb_b: float = 1.0,
             nonfinite_out=None, workspace_max_bytes: Optional[int] = None, graft: bool = False,
             beta_g: float = 0.999, eps_g: float = 1e-8, thetas=None, lr: float = 0.0):
        import torch
        if len(grads) != len(self.shapes) or len(updates) != len(self.shapes):
            raise DashError(ERR_INVALID_ARG, "one gradient and one update tensor per layer")
        for t, (m, n) in zip(list(grads) + list(updates), self.shapes * 2):
            self.dash._dense(t, "layer tensor", (m, n) if n else (m,))
        a = _ModelStepArgs()
        gp = (C.c_void_p * len(grads))(*[t.data_ptr() for t in grads])
        up = (C.c_void_p * len(updates))(*[t.data_ptr() for t in updates])
        a.grads, a.updates = gp, up
        a.beta, a.alpha, a.eps = beta, (1.0 - beta) if alpha is None else alpha, eps
        a.method, a.iters = _enum(_METHODS, method), iters
        a.scaling, a.precision, a.refresh = _enum(_SCALINGS, scaling), _enum(_PRECISIONS, precision), int(refresh)
        keep = None
        if cheb_coeffs is not None:
            keep = (C.c_double * len(cheb_coeffs))(*[float(v) for v in cheb_coeffs])
            a.cheb_coeffs = C.cast(keep, C.POINTER(C.c_double))
        a.cheb_a, a.cheb_b = cheb_a, cheb_b
        a.nonfinite_out = self.dash._vec(nonfinite_out, "nonfinite_out", self.plan["info"]["n_factor_blocks"],
                                         torch.int32).value
        a.graft, a.beta_g, a.eps_g, a.lr = int(graft), beta_g, eps_g, lr
        tp = None
        if thetas is not None:
            if len(thetas) != len(self.shapes):
                raise DashError(ERR_INVALID_ARG, "one parameter tensor per layer")
            for t, (m, n) in zip(thetas, self.shapes):
                self.dash._dense(t, "theta", (m, n) if n else (m,))
            tp = (C.c_void_p * len(thetas))(*[t.data_ptr() for t in thetas])
            a.thetas = tp
        need = int(self.lib.dash_model_workspace_bytes(self.h, a.method, a.precision))
        if workspace_max_bytes is not None:
            need = min(need, int(workspace_max_bytes))
        if self.dash._ws is None or self.dash._ws.numel() < need:
            self.dash.set_workspace_bytes(need)
        self._check(self.lib.dash_model_step(self.h, C.byref(a)))
        return updates
