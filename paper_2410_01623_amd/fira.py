"""Thin Python binding over the C ABI of include/fira.h (argument marshalling only).

Every step of the optimizer runs in the HIP library; this module converts torch tensors to raw
device pointers, owns the device slab as a torch byte tensor, and forwards the calls.  PyTorch is
used for device memory and the stream, nothing else.  There is no CPU fallback: if libfira.so is
missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch  # must be imported before the library so that both share one HIP runtime

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libfira.so")

FIRA_OK = 0
FIRA_ERR_INVALID_ARG = -1
FIRA_ERR_SHAPE = -2
FIRA_ERR_NO_PROJECTOR = -3
FIRA_ERR_DTYPE = -4
FIRA_ERR_WORKSPACE = -5
FIRA_ERR_HIP = -6
FIRA_F32, FIRA_BF16 = 0, 1
FIRA_SCALE_COLUMN, FIRA_SCALE_MATRIX, FIRA_SCALE_NONE = 0, 1, 2
FIRA_VARIANT_FULL, FIRA_VARIANT_ONLY_SCALING = 0, 1
FIRA_NORM_RESIDUAL, FIRA_NORM_GRAM = 0, 1
FIRA_NUM_KERNELS = 6
FIRA_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = (
    "fira_method_state_numel", "fira_state_bytes", "fira_init_state", "fira_set_projector", "fira_set_projectors", "fira_step",
    "fira_set_hparams", "fira_set_options", "fira_set_variant", "fira_set_fusion", "fira_last_step_fused", "fira_set_z_planes",
    "fira_get_state", "fira_set_state", "fira_get_diag", "fira_get_gate", "fira_set_gate",
    "fira_get_factors", "fira_get_lowrank", "fira_get_projector", "fira_refresh_workspace_bytes",
    "fira_refresh_projectors", "fira_refresh_projectors_static", "fira_profile_begin", "fira_profile_end", "fira_kernel_name",
    "fira_last_error", "fira_destroy",
)


class fira_hparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("alpha", ctypes.c_double), ("gamma", ctypes.c_double)]


class fira_matrix_desc(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("ld", ctypes.c_int64),
                ("r", ctypes.c_int32), ("wg_dtype", ctypes.c_int32)]


class FiraError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"fira status {status}: {message}")
        self.status = status


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libfira.so (built in-tree by paper_2410_01623_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(
            f"{p} not found: build it with `python -m paper_2410_01623_amd.build` "
            "(the Fira step has no fallback path)")
    lib = ctypes.CDLL(p)
    vp, ci, cd = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
    lib.fira_method_state_numel.restype = ctypes.c_int64
    lib.fira_method_state_numel.argtypes = [ctypes.POINTER(fira_matrix_desc)]
    lib.fira_state_bytes.restype = ctypes.c_size_t
    lib.fira_state_bytes.argtypes = [ctypes.POINTER(fira_matrix_desc), ci]
    lib.fira_init_state.restype = ci
    lib.fira_init_state.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(fira_matrix_desc), ci,
                                    ctypes.POINTER(fira_hparams), vp, ctypes.c_size_t, vp]
    lib.fira_set_projector.restype = ci
    lib.fira_set_projector.argtypes = [vp, ci, vp, ci]
    lib.fira_set_projectors.restype = ci
    lib.fira_set_projectors.argtypes = [vp, ci, ctypes.POINTER(ci), ctypes.POINTER(vp), ci]
    lib.fira_step.restype = ci
    lib.fira_step.argtypes = [vp, ci, ctypes.POINTER(ci), ctypes.POINTER(vp), ctypes.POINTER(vp)]
    lib.fira_set_hparams.restype = ci
    lib.fira_set_hparams.argtypes = [vp, ctypes.POINTER(fira_hparams)]
    lib.fira_set_options.restype = ci
    lib.fira_set_options.argtypes = [vp, ci, ci]
    lib.fira_set_variant.restype = ci
    lib.fira_set_variant.argtypes = [vp, ci]
    lib.fira_set_fusion.restype = ci
    lib.fira_set_fusion.argtypes = [vp, ci]
    lib.fira_set_z_planes.restype = ci
    lib.fira_set_z_planes.argtypes = [vp, ci]
    lib.fira_last_step_fused.restype = ci
    lib.fira_last_step_fused.argtypes = [vp]
    lib.fira_get_state.restype = ci
    lib.fira_get_state.argtypes = [vp, ci, vp, vp, ctypes.POINTER(cd), ctypes.POINTER(ctypes.c_int64)]
    lib.fira_set_state.restype = ci
    lib.fira_set_state.argtypes = [vp, ci, vp, vp, cd, ctypes.c_int64]
    lib.fira_get_diag.restype = ci
    lib.fira_get_diag.argtypes = [vp, ci, ctypes.POINTER(cd), ctypes.POINTER(cd), ctypes.POINTER(cd)]
    lib.fira_get_gate.restype = ci
    lib.fira_get_gate.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ci)]
    lib.fira_set_gate.restype = ci
    lib.fira_set_gate.argtypes = [vp, ci, ctypes.c_float, ctypes.c_float]
    lib.fira_get_factors.restype = ci
    lib.fira_get_factors.argtypes = [vp, ci, vp]
    lib.fira_get_lowrank.restype = ci
    lib.fira_get_lowrank.argtypes = [vp, ci, vp]
    lib.fira_get_projector.restype = ci
    lib.fira_get_projector.argtypes = [vp, ci, vp]
    lib.fira_refresh_workspace_bytes.restype = ctypes.c_size_t
    lib.fira_refresh_workspace_bytes.argtypes = [vp, ci, ctypes.POINTER(ci)]
    lib.fira_refresh_projectors.restype = ci
    lib.fira_refresh_projectors.argtypes = [vp, ci, ctypes.POINTER(ci), ctypes.POINTER(vp), ci, ctypes.c_uint64, vp,
                                            ctypes.c_size_t]
    lib.fira_refresh_projectors_static.restype = ci
    lib.fira_refresh_projectors_static.argtypes = [vp, ci, ctypes.POINTER(ci), ctypes.POINTER(vp), ci, ctypes.c_uint64]
    lib.fira_profile_begin.restype = ci
    lib.fira_profile_begin.argtypes = [vp, ci]
    lib.fira_profile_end.restype = ci
    lib.fira_profile_end.argtypes = [vp, ctypes.POINTER(cd), ctypes.POINTER(ci)]
    lib.fira_kernel_name.restype = ctypes.c_char_p
    lib.fira_kernel_name.argtypes = [ci]
    lib.fira_last_error.restype = ctypes.c_char_p
    lib.fira_last_error.argtypes = [vp]
    lib.fira_destroy.restype = None
    lib.fira_destroy.argtypes = [vp]
    if path is None:
        _lib = lib
    return lib


def _check(lib, ctx, status: int):
    if status != FIRA_OK:
        msg = lib.fira_last_error(ctx)
        raise FiraError(status, msg.decode() if msg else "")


def make_descs(shapes: Sequence[Tuple[int, int]], rank, dtype, lds: Optional[Sequence[int]] = None):
    """(m, n) list -> ctypes array of fira_matrix_desc.  rank/dtype may be scalars or per-matrix."""
    n = len(shapes)
    arr = (fira_matrix_desc * n)()
    for i, (m, nn) in enumerate(shapes):
        r = rank[i] if isinstance(rank, (list, tuple)) else rank
        dt = dtype[i] if isinstance(dtype, (list, tuple)) else dtype
        arr[i] = fira_matrix_desc(m, nn, lds[i] if lds is not None else nn, r, dt)
    return arr


def make_hparams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, alpha=1.0, gamma=1.01) -> fira_hparams:
    return fira_hparams(lr, beta1, beta2, eps, alpha, gamma)


def fira_method_state_numel(desc: fira_matrix_desc) -> int:
    return int(load_library().fira_method_state_numel(ctypes.byref(desc)))


def fira_state_bytes(descs) -> int:
    return int(load_library().fira_state_bytes(descs, len(descs)))


_TORCH_DTYPE = {FIRA_F32: torch.float32, FIRA_BF16: torch.bfloat16}


class PreparedList:
    """Host arrays of one fira_step call, marshalled once (idx, W pointers, G pointers)."""

    def __init__(self, idx: Sequence[int], Ws: Sequence[torch.Tensor], Gs: Sequence[torch.Tensor]):
        n = len(idx)
        self.count = n
        self.idx = (ctypes.c_int * n)(*idx)
        self.W = (ctypes.c_void_p * n)(*[w.data_ptr() for w in Ws])
        self.G = (ctypes.c_void_p * n)(*[g.data_ptr() for g in Gs])
        self._keep = (list(Ws), list(Gs))


class FiraContext:
    """Owns a fira_ctx and its device slab.  Methods carry the names of the C entry points."""

    def __init__(self, shapes: Sequence[Tuple[int, int]], rank, dtype=FIRA_BF16, hp: Optional[fira_hparams] = None,
                 device: str = "cuda:0", lds: Optional[Sequence[int]] = None, stream: Optional[torch.cuda.Stream] = None):
        self.lib = load_library()
        self.descs = make_descs(shapes, rank, dtype, lds)
        self.shapes = list(shapes)
        self.hp = hp or make_hparams()
        self.device = torch.device(device)
        nbytes = fira_state_bytes(self.descs)
        if nbytes == 0:
            raise FiraError(FIRA_ERR_SHAPE, (self.lib.fira_last_error(None) or b"").decode())
        self.state_bytes = nbytes
        self.slab = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.stream = stream or torch.cuda.current_stream(self.device)
        self.ctx = ctypes.c_void_p()
        st = self.lib.fira_init_state(ctypes.byref(self.ctx), self.descs, len(self.descs), ctypes.byref(self.hp),
                                      ctypes.c_void_p(self.slab.data_ptr()), nbytes,
                                      ctypes.c_void_p(self.stream.cuda_stream))
        _check(self.lib, None, st)

    # -- calls ------------------------------------------------------------------------------
    def fira_set_projector(self, idx: int, P: torch.Tensor):
        assert P.is_contiguous() and P.device == self.slab.device
        dt = {torch.float32: FIRA_F32, torch.bfloat16: FIRA_BF16}[P.dtype]
        m, n = self.shapes[idx]
        assert tuple(P.shape) == (min(m, n), self.descs[idx].r), "P must be min(m,n) x r"
        _check(self.lib, self.ctx, self.lib.fira_set_projector(self.ctx, idx, ctypes.c_void_p(P.data_ptr()), dt))

    def fira_set_projectors(self, idx, Ps):
        """Projectors of several matrices in one call (all of one dtype)."""
        idx = list(idx)
        assert len(idx) == len(Ps)
        dts = {P.dtype for P in Ps}
        assert len(dts) <= 1, "one dtype per call"
        dt = {torch.float32: FIRA_F32, torch.bfloat16: FIRA_BF16}[Ps[0].dtype] if Ps else FIRA_F32
        for i, P in zip(idx, Ps):
            assert P.is_contiguous() and P.device == self.slab.device
            if 0 <= i < len(self.descs):   # the library reports bad indices
                m, n = self.shapes[i]
                assert tuple(P.shape) == (min(m, n), self.descs[i].r), "P must be min(m,n) x r"
        c_idx = (ctypes.c_int * len(idx))(*idx)
        c_P = (ctypes.c_void_p * len(idx))(*[P.data_ptr() for P in Ps])
        _check(self.lib, self.ctx, self.lib.fira_set_projectors(self.ctx, len(idx), c_idx, c_P, dt))

    def prepare(self, idx, Ws, Gs) -> PreparedList:
        for i, w, g in zip(idx, Ws, Gs):
            if not 0 <= i < len(self.descs):
                continue   # the library reports bad indices
            d = self.descs[i]
            want = _TORCH_DTYPE[d.wg_dtype]
            assert w.dtype == want and g.dtype == want, "W/G dtype must match the descriptor"
            assert tuple(w.shape) == (d.m, d.n) and tuple(g.shape) == (d.m, d.n)
            assert w.stride(1) == 1 and g.stride(1) == 1 and w.stride(0) == d.ld and g.stride(0) == d.ld
        return PreparedList(idx, Ws, Gs)

    def fira_step(self, idx=None, Ws=None, Gs=None, prepared: Optional[PreparedList] = None):
        p = prepared if prepared is not None else self.prepare(idx, Ws, Gs)
        _check(self.lib, self.ctx, self.lib.fira_step(self.ctx, p.count, p.idx, p.W, p.G))

    def fira_set_hparams(self, hp: fira_hparams):
        self.hp = hp
        _check(self.lib, self.ctx, self.lib.fira_set_hparams(self.ctx, ctypes.byref(hp)))

    def fira_set_options(self, scaling=FIRA_SCALE_COLUMN, norm_mode=FIRA_NORM_GRAM):
        _check(self.lib, self.ctx, self.lib.fira_set_options(self.ctx, scaling, norm_mode))

    def fira_set_variant(self, variant: int):
        _check(self.lib, self.ctx, self.lib.fira_set_variant(self.ctx, variant))

    def fira_set_fusion(self, enable: bool):
        _check(self.lib, self.ctx, self.lib.fira_set_fusion(self.ctx, 1 if enable else 0))

    def fira_set_z_planes(self, planes: int):
        _check(self.lib, self.ctx, self.lib.fira_set_z_planes(self.ctx, planes))

    def fira_last_step_fused(self) -> bool:
        return bool(self.lib.fira_last_step_fused(self.ctx))

    def fira_get_state(self, idx: int):
        m, n = self.shapes[idx]
        r = self.descs[idx].r
        shape = (r, n) if m <= n else (m, r)
        M = torch.empty(shape, dtype=torch.float32)
        V = torch.empty(shape, dtype=torch.float32)
        s_prev, t = ctypes.c_double(), ctypes.c_int64()
        _check(self.lib, self.ctx, self.lib.fira_get_state(self.ctx, idx, ctypes.c_void_p(M.data_ptr()),
                                                        ctypes.c_void_p(V.data_ptr()), ctypes.byref(s_prev),
                                                        ctypes.byref(t)))
        return M, V, s_prev.value, t.value

    def fira_set_state(self, idx: int, M: torch.Tensor, V: torch.Tensor, s_prev: float, t: int):
        M = M.contiguous().to(torch.float32).cpu()
        V = V.contiguous().to(torch.float32).cpu()
        _check(self.lib, self.ctx, self.lib.fira_set_state(self.ctx, idx, ctypes.c_void_p(M.data_ptr()),
                                                        ctypes.c_void_p(V.data_ptr()), float(s_prev), int(t)))

    def fira_get_diag(self, idx: int):
        a, b, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        _check(self.lib, self.ctx, self.lib.fira_get_diag(self.ctx, idx, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return a.value, b.value, c.value

    def fira_get_gate(self, idx: int):
        """-> (ortho_err, gram_err, route of the last step: 0 residual, 1 Gram, 2 Gram with the fused kernel)"""
        a, b, r = ctypes.c_float(), ctypes.c_float(), ctypes.c_int()
        _check(self.lib, self.ctx, self.lib.fira_get_gate(self.ctx, idx, ctypes.byref(a), ctypes.byref(b), ctypes.byref(r)))
        return a.value, b.value, int(r.value)

    def fira_set_gate(self, idx: int, ortho_err: float, gram_err: float):
        _check(self.lib, self.ctx, self.lib.fira_set_gate(self.ctx, idx, ortho_err, gram_err))

    def fira_get_factors(self, idx: int) -> torch.Tensor:
        m, n = self.shapes[idx]
        k = torch.empty(max(m, n), dtype=torch.float32)
        _check(self.lib, self.ctx, self.lib.fira_get_factors(self.ctx, idx, ctypes.c_void_p(k.data_ptr())))
        return k

    def fira_get_lowrank(self, idx: int) -> torch.Tensor:
        m, n = self.shapes[idx]
        r = self.descs[idx].r
        R = torch.empty((r, n) if m <= n else (m, r), dtype=torch.float32)
        _check(self.lib, self.ctx, self.lib.fira_get_lowrank(self.ctx, idx, ctypes.c_void_p(R.data_ptr())))
        return R

    def fira_get_projector(self, idx: int) -> torch.Tensor:
        m, n = self.shapes[idx]
        P = torch.empty((min(m, n), self.descs[idx].r), dtype=torch.float32)
        _check(self.lib, self.ctx, self.lib.fira_get_projector(self.ctx, idx, ctypes.c_void_p(P.data_ptr())))
        return P

    def fira_refresh_workspace_bytes(self, idx: Sequence[int]) -> int:
        arr = (ctypes.c_int * len(idx))(*idx)
        return int(self.lib.fira_refresh_workspace_bytes(self.ctx, len(idx), arr))

    def fira_refresh_projectors(self, idx: Sequence[int], G: Sequence[torch.Tensor], iters: int = 2, seed: int = 0,
                                workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Recomputes and installs the projectors of the listed matrices from their gradients on the
        device.  Returns the workspace tensor (keep it until the stream has passed the call)."""
        count = len(idx)
        assert len(G) == count
        need = self.fira_refresh_workspace_bytes(idx)
        if workspace is None or workspace.numel() < need:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=self.slab.device)
        assert workspace.data_ptr() % 256 == 0
        for e, i in enumerate(idx):
            m, n = self.shapes[i]
            g = G[e]
            d = self.descs[i]
            assert g.device == self.slab.device and g.dtype == _TORCH_DTYPE[d.wg_dtype] and tuple(g.shape) == (m, n)
            assert g.stride(1) == 1 and g.stride(0) == d.ld
        ci = (ctypes.c_int * count)(*idx)
        cg = (ctypes.c_void_p * count)(*[g.data_ptr() for g in G])
        _check(self.lib, self.ctx, self.lib.fira_refresh_projectors(self.ctx, count, ci, cg, iters, seed,
                                                                    ctypes.c_void_p(workspace.data_ptr()), need))
        return workspace

    def fira_refresh_projectors_static(self, idx: Sequence[int], G: Sequence[torch.Tensor], iters: int = 2, seed: int = 0):
        """fira_refresh_projectors on the library's static scratch: no workspace, no device allocation."""
        count = len(idx)
        assert len(G) == count
        ci = (ctypes.c_int * count)(*idx)
        cg = (ctypes.c_void_p * count)(*[g.data_ptr() for g in G])
        _check(self.lib, self.ctx, self.lib.fira_refresh_projectors_static(self.ctx, count, ci, cg, iters, seed))

    def fira_profile_begin(self, max_steps: int):
        _check(self.lib, self.ctx, self.lib.fira_profile_begin(self.ctx, max_steps))

    def fira_profile_end(self):
        """-> ({kernel name: total milliseconds}, recorded steps)"""
        ms = (ctypes.c_double * FIRA_NUM_KERNELS)()
        steps = ctypes.c_int()
        _check(self.lib, self.ctx, self.lib.fira_profile_end(self.ctx, ms, ctypes.byref(steps)))
        names = [self.lib.fira_kernel_name(k).decode() for k in range(FIRA_NUM_KERNELS)]
        return dict(zip(names, list(ms))), steps.value

    def fira_destroy(self):
        if self.ctx:
            self.lib.fira_destroy(self.ctx)
            self.ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.fira_destroy()
        except Exception:
            pass
