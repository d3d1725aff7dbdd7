"""ctypes binding of include/snlp.h: argument marshalling only.

Every step of the path (norms, GEMMs, rotary embedding, attention, correction scan, probe) runs in the
HIP library; PyTorch supplies device memory and the stream.  There is no CPU fallback: if the library
is missing or fails to load, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

IDN, HCN = 0, 1
F32, BF16 = 0, 1
INIT_H0, INIT_FWD = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SnlpError(RuntimeError):
    pass


class _Config(C.Structure):
    _fields_ = [("L", C.c_int), ("d", C.c_int), ("n_heads", C.c_int), ("head_dim", C.c_int), ("d_mlp", C.c_int),
                ("n_streams", C.c_int), ("B", C.c_int), ("T", C.c_int), ("P", C.c_int),
                ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int)]


# name -> (restype, argtypes); exactly the entry points include/snlp.h declares
_SIGNATURES = {
    "snlp_create": (C.c_int, [C.POINTER(_Config), C.POINTER(C.c_void_p)]),
    "snlp_destroy": (None, [C.c_void_p]),
    "snlp_last_error": (C.c_char_p, [C.c_void_p]),
    "snlp_workspace_bytes": (C.c_size_t, [C.c_void_p]),
    "snlp_bind_workspace": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "snlp_bind_weights": (C.c_int, [C.c_void_p] + [C.c_void_p] * 4 + [C.c_void_p]),
    "snlp_bind_kv_prefix": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_set_hc": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_bind_trace": (C.c_int, [C.c_void_p, C.c_void_p]),
    "snlp_init_trace": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_set_prefix": (C.c_int, [C.c_void_p, C.c_int]),
    "snlp_set_fusion": (C.c_int, [C.c_void_p, C.c_int]),
    "snlp_init_trace_ex": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "snlp_iterate": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "snlp_sequential_forward": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_residual_norm": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
    "snlp_evaluate_branches": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_correction_scan": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_correction_scan_static": (C.c_int, [C.c_int] * 5 + [C.c_void_p] * 6),
    "snlp_correction_scan_diag": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_iterate_diag": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]),
    "snlp_set_skip_converged": (C.c_int, [C.c_void_p, C.c_int]),
    "snlp_stage_buffer": (C.c_int, [C.c_void_p, C.c_char_p, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]),
    "snlp_profile_stages": (C.c_int, [C.c_void_p, C.c_uint]),
    "snlp_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int)]),
}

N_STAGES = 9
STAGE_NAMES = ("premix_rmsnorm", "gemm_qkv", "rope_qknorm", "attention", "gemm_o", "mid_rmsnorm", "gemm_fc",
               "gemm_proj", "correction_scan")


def library_path() -> str:
    return os.path.join(_HERE, "libsnlp_hip.so")


def load_library():
    """dlopen libsnlp_hip.so (built in-tree by build.py) and declare its signatures.  Raises if absent."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise SnlpError("HIP library %s is not built; run `python -m paper_2605_17842_amd.build` "
                            "(or __graft_entry__.build()) first" % path)
        lib = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _LIB = lib
    return _LIB


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def correction_scan_static(mode, trace, g, Hres=None, post=None, probe=None):
    """snlp_correction_scan_static: the correction scan on caller-owned device tensors, no context and no workspace.
    trace [L+1, M, n, d], g [L, M, d], Hres [L, n, n] / post [L, n] (device tensors, n > 1), probe [2, L] or None."""
    lib = load_library()
    for t in (trace, g, Hres, post, probe):
        if t is not None and (t.dtype != torch.float32 or not t.is_contiguous() or t.device != trace.device):
            raise SnlpError("arguments must be contiguous fp32 tensors on one device")
    L1, M, n, d = trace.shape
    with torch.cuda.device(trace.device):
        rc = lib.snlp_correction_scan_static(mode, L1 - 1, M, n, d, _ptr(trace), _ptr(g), _ptr(Hres), _ptr(post), _ptr(probe),
                                             C.c_void_p(torch.cuda.current_stream(trace.device).cuda_stream))
    if rc != 0:
        raise SnlpError("snlp_correction_scan_static: %s (%d)" % (lib.snlp_last_error(None).decode(), rc))


class Snlp:
    """One model + batch shape bound to device buffers.  Methods mirror the C entry points."""

    def __init__(self, *, L, d, n_heads, head_dim, d_mlp, B, T, P=0, n_streams=1, rope_base=1.0e4, rms_eps=1.0e-6,
                 dtype=BF16, device="cuda:0"):
        self.lib = load_library()
        self.cfg = _Config(L, d, n_heads, head_dim, d_mlp, n_streams, B, T, P, rope_base, rms_eps, dtype)
        self.device = torch.device(device)
        self.L, self.d, self.M, self.n, self.dtype = L, d, B * T, n_streams, dtype
        self.units = L
        self._h = C.c_void_p()
        rc = self.lib.snlp_create(C.byref(self.cfg), C.byref(self._h))
        if rc != 0:
            raise SnlpError("snlp_create: %s (%d)" % (self.lib.snlp_last_error(None).decode(), rc))
        self._keep = {}
        with torch.cuda.device(self.device):
            nbytes = self.lib.snlp_workspace_bytes(self._h)
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            self._check(self.lib.snlp_bind_workspace(self._h, C.c_void_p(self._ws_ptr), nbytes), "snlp_bind_workspace")
        self.trace = None

    # -- plumbing
    def _check(self, rc, what):
        if rc != 0:
            raise SnlpError("%s: %s (%d)" % (what, self.lib.snlp_last_error(self._h).decode(), rc))

    def _stream(self):
        return C.c_void_p(torch.cuda.current_stream(self.device).cuda_stream)

    def _dev(self, t: torch.Tensor, dtype, what) -> torch.Tensor:
        if t.device != self.device or t.dtype != dtype or not t.is_contiguous():
            raise SnlpError("%s must be a contiguous %s tensor on %s" % (what, dtype, self.device))
        return t

    @property
    def _wdtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32

    def close(self):
        if self._h:
            self.lib.snlp_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- binding
    def bind_weights(self, Wqkv, Wo, Wfc, Wproj):
        ws = [self._dev(w, self._wdtype, "weights") for w in (Wqkv, Wo, Wfc, Wproj)]
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_bind_weights(self._h, *[_ptr(w) for w in ws], self._stream()), "snlp_bind_weights")
        self._keep["w"] = ws

    def bind_kv_prefix(self, Kpre, Vpre):
        k, v = self._dev(Kpre, self._wdtype, "Kpre"), self._dev(Vpre, self._wdtype, "Vpre")
        self._check(self.lib.snlp_bind_kv_prefix(self._h, _ptr(k), _ptr(v)), "snlp_bind_kv_prefix")
        self._keep["kv"] = (k, v)

    def set_hc(self, Hres, pre, post):
        hs = [torch.as_tensor(x, dtype=torch.float32, device="cpu").contiguous() for x in (Hres, pre, post)]
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_set_hc(self._h, *[_ptr(x) for x in hs]), "snlp_set_hc")

    def bind_trace(self, trace=None):
        if trace is None:
            trace = torch.empty((self.units + 1, self.M, self.n, self.d), dtype=torch.float32, device=self.device)
        self.trace = self._dev(trace, torch.float32, "trace")
        self._check(self.lib.snlp_bind_trace(self._h, _ptr(self.trace)), "snlp_bind_trace")
        return self.trace

    # -- the path
    def init_trace(self, h0):
        h0 = self._dev(h0, torch.float32, "h0")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_init_trace(self._h, _ptr(h0), self._stream()), "snlp_init_trace")

    def set_fusion(self, F: int):
        """Group the layers into chunks of F; all calls then work in chunk units (trace [L/F + 1, M, 1, d])."""
        self._check(self.lib.snlp_set_fusion(self._h, F), "snlp_set_fusion")
        self.units = self.L // F

    def set_prefix(self, S: int):
        self._check(self.lib.snlp_set_prefix(self._h, S), "snlp_set_prefix")

    def init_trace_ex(self, mode, init, h0):
        h0 = self._dev(h0, torch.float32, "h0")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_init_trace_ex(self._h, mode, init, _ptr(h0), self._stream()), "snlp_init_trace_ex")

    def iterate(self, mode, K, probe=None):
        if probe is not None:
            self._dev(probe, torch.float32, "probe")
            if probe.numel() < K * 2 * self.units:
                raise SnlpError("probe needs K * 2 * L floats (L / F when fused)")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_iterate(self._h, mode, K, _ptr(probe), self._stream()), "snlp_iterate")

    def sequential_forward(self, mode, h0, trace_out=None):
        h0 = self._dev(h0, torch.float32, "h0")
        if trace_out is None:
            trace_out = torch.empty((self.units + 1, self.M, self.n, self.d), dtype=torch.float32, device=self.device)
        self._dev(trace_out, torch.float32, "trace_out")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_sequential_forward(self._h, mode, _ptr(h0), _ptr(trace_out), self._stream()),
                        "snlp_sequential_forward")
        return trace_out

    def residual_norm(self, mode, out=None):
        if out is None:
            out = torch.empty(self.units, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_residual_norm(self._h, mode, _ptr(self._dev(out, torch.float32, "out")), self._stream()),
                        "snlp_residual_norm")
        return out

    def evaluate_branches(self, g_out=None):
        if g_out is None:
            g_out = torch.empty((self.units, self.M, self.d), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_evaluate_branches(self._h, _ptr(self._dev(g_out, torch.float32, "g_out")), self._stream()),
                        "snlp_evaluate_branches")
        return g_out

    def correction_scan(self, mode, g, probe=None):
        g = self._dev(g, torch.float32, "g")
        if g.numel() != self.units * self.M * self.d:
            raise SnlpError("g must be [L, M, d] ([L / F, M, d] when fused)")
        if probe is not None:
            self._dev(probe, torch.float32, "probe")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_correction_scan(self._h, mode, _ptr(g), _ptr(probe), self._stream()),
                        "snlp_correction_scan")

    def correction_scan_diag(self, g, diag, probe=None):
        g, diag = self._dev(g, torch.float32, "g"), self._dev(diag, torch.float32, "diag")
        if g.numel() != self.units * self.M * self.d or diag.numel() != g.numel():
            raise SnlpError("g and diag must be [L, M, d]")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_correction_scan_diag(self._h, _ptr(g), _ptr(diag), _ptr(probe), self._stream()),
                        "snlp_correction_scan_diag")

    def iterate_diag(self, K, diag, probe=None):
        diag = self._dev(diag, torch.float32, "diag")
        if diag.numel() != self.units * self.M * self.d:
            raise SnlpError("diag must be [L, M, d]")
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_iterate_diag(self._h, K, _ptr(diag), _ptr(probe), self._stream()), "snlp_iterate_diag")

    def set_skip_converged(self, on: bool):
        """Leave layers that are already exact out of later rounds (same results, less work)."""
        self._check(self.lib.snlp_set_skip_converged(self._h, 1 if on else 0), "snlp_set_skip_converged")

    def profile_stages(self, mask: int):
        self._check(self.lib.snlp_profile_stages(self._h, mask), "snlp_profile_stages")

    def profile_read(self):
        """(milliseconds, launches) per stage since the last read."""
        ms = (C.c_float * N_STAGES)()
        cnt = (C.c_int * N_STAGES)()
        with torch.cuda.device(self.device):
            self._check(self.lib.snlp_profile_read(self._h, ms, cnt), "snlp_profile_read")
        return list(ms), list(cnt)

    def stage_buffer(self, name: str) -> torch.Tensor:
        """Diagnostic copy of a stage buffer as a flat tensor (fp32, or bf16 for bf16 operand buffers)."""
        p, n = C.c_void_p(), C.c_size_t()
        self._check(self.lib.snlp_stage_buffer(self._h, name.encode(), C.byref(p), C.byref(n)), "snlp_stage_buffer")
        off = p.value - self.workspace.data_ptr()
        raw = self.workspace[off: off + n.value]
        dt = torch.float32 if (name in ("a", "g", "u") or self.dtype == F32) else torch.bfloat16
        return raw.view(dt).clone()
