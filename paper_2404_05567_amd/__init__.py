"""Thin Python binding of libdsmoe (the MI355X / gfx950 DS-MoE expert layer).

Argument marshalling only: every step of the layer runs in the HIP kernels behind the C ABI declared in
`include/dsmoe.h`.  PyTorch is used for device memory and streams.  There is no CPU fallback: if the
shared library has not been built, importing the binding's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_int64, c_size_t, c_void_p

_PKG = os.path.dirname(os.path.abspath(__file__))
# DSMOE_LIBRARY names another build of the same sources to load instead (the conservative-waits build that a GPU test
# compares the library with); by default the in-tree libdsmoe.so.
LIB_PATH = os.environ.get("DSMOE_LIBRARY") or os.path.join(_PKG, "libdsmoe.so")
LIB_CHECKED_PATH = os.path.join(_PKG, "libdsmoe_checked.so")

F32, BF16 = 0, 1
SEL_TOPK, SEL_THRESHOLD, SEL_THRESHOLD_TOPK = 0, 1, 2
SEL_NORMALISED = 0x100   # OR into a threshold mode: eps is the paper's normalised threshold (N * S_i > eps)
SEL_ALL = -1          # attention layer only: every expert
EXPERT_SWIGLU, EXPERT_GELU = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_CAPACITY, ERR_HIP, ERR_NOT_IMPL = 0, -1, -2, -3, -4, -5, -6
ERR_INTERNAL = -7

EXPORTS = [
    "dsmoe_create", "dsmoe_destroy", "dsmoe_last_error", "dsmoe_set_expert_kind", "dsmoe_workspace_bytes",
    "dsmoe_set_workspace", "dsmoe_set_sync_spin_limit",
    "dsmoe_poll_error", "dsmoe_route", "dsmoe_select", "dsmoe_dispatch", "dsmoe_dispatch_static", "dsmoe_expert_ffn",
    "dsmoe_combine",
    "dsmoe_sparse_fwd", "dsmoe_sparse_fwd_routing", "dsmoe_sparse_fwd_uses_persistent_kernel", "dsmoe_sparse_fwd_path", "dsmoe_dense_saved_bytes", "dsmoe_dense_fwd",
    "dsmoe_dense_bwd_scratch_bytes", "dsmoe_dense_bwd", "dsmoe_mi_loss", "dsmoe_dense_bwd_mi",
    "dsmoe_profile_enable", "dsmoe_profile_read", "dsmoe_bench_mfma", "dsmoe_bench_stream", "dsmoe_bench_xcc_ids",
    "dsmoe_moa_create", "dsmoe_moa_destroy", "dsmoe_moa_last_error", "dsmoe_moa_workspace_bytes",
    "dsmoe_moa_set_workspace", "dsmoe_moa_fwd", "dsmoe_moa_routing", "dsmoe_moa_bwd_scratch_bytes", "dsmoe_moa_bwd",
]


class MoaDesc(ctypes.Structure):
    _fields_ = [("d_model", c_int32), ("n_experts", c_int32), ("n_head", c_int32), ("d_head", c_int32),
                ("dtype", c_int32), ("max_tokens", c_int32)]


class Desc(ctypes.Structure):
    _fields_ = [("d_model", c_int32), ("d_ff", c_int32), ("n_experts", c_int32), ("dtype", c_int32),
                ("max_tokens", c_int32), ("max_rows", c_int64)]


class DsmoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libdsmoe status {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libdsmoe.so (built in-tree by `paper_2404_05567_amd/build.py`); fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2404_05567_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    P = c_void_p
    sig = {
        "dsmoe_create": (c_int32, [POINTER(Desc), POINTER(c_void_p)]),
        "dsmoe_destroy": (c_int32, [P]),
        "dsmoe_last_error": (c_char_p, [P]),
        "dsmoe_set_expert_kind": (c_int32, [P, c_int32]),
        "dsmoe_workspace_bytes": (c_int32, [P, POINTER(c_size_t)]),
        "dsmoe_set_workspace": (c_int32, [P, P, c_size_t]),
        "dsmoe_set_sync_spin_limit": (c_int32, [P, c_int32]),
        "dsmoe_poll_error": (c_int32, [P, P]),
        "dsmoe_route": (c_int32, [P, P, P, P, c_int32, P, P]),
        "dsmoe_select": (c_int32, [P, P, c_int32, c_int32, c_int32, c_float, P, P, P]),
        "dsmoe_dispatch": (c_int32, [P, P, P, P, c_int32, P, P, P, P, P, P, P, P]),
        "dsmoe_dispatch_static": (c_int32, [P, P, P, P, c_int32, P, P, P, P, P, P, P, P]),
        "dsmoe_expert_ffn": (c_int32, [P] * 10),
        "dsmoe_combine": (c_int32, [P, P, P, P, P, c_int32, P, P]),
        "dsmoe_sparse_fwd": (c_int32, [P, P, P, P, P, P, P, c_int32, c_int32, c_int32, c_float, P, P]),
        "dsmoe_sparse_fwd_routing": (c_int32, [P, c_int32, P, P, P, P, P]),
        "dsmoe_sparse_fwd_uses_persistent_kernel": (c_int32, [P, c_int32, c_int32, c_int32, c_float]),
        "dsmoe_sparse_fwd_path": (c_int32, [P, c_int32, c_int32, c_int32, c_float]),
        "dsmoe_dense_saved_bytes": (c_int32, [P, c_int32, POINTER(c_size_t)]),
        "dsmoe_dense_fwd": (c_int32, [P, P, P, P, P, P, P, c_int32, P, P, P, P]),
        "dsmoe_dense_bwd_scratch_bytes": (c_int32, [P, c_int32, POINTER(c_size_t)]),
        "dsmoe_dense_bwd": (c_int32, [P, P, P, P, P, P, P, P, c_int32, P, P, P, P, P, P, P, P]),
        "dsmoe_mi_loss": (c_int32, [P, P, c_int32, P, P, P]),
        "dsmoe_dense_bwd_mi": (c_int32, [P, P, P, P, P, P, P, P, c_int32, P, P, P, P, P, P, P, c_float, P]),
        "dsmoe_profile_enable": (c_int32, [P, c_int32]),
        "dsmoe_profile_read": (c_int32, [P, POINTER(c_int32), POINTER(c_float), POINTER(c_float)]),
        "dsmoe_bench_mfma": (c_int32, [P, P, c_int32, c_int32, POINTER(c_float), POINTER(ctypes.c_double), P]),
        "dsmoe_bench_stream": (c_int32, [P, c_size_t, c_int32, c_int32, P, POINTER(c_float), POINTER(c_size_t), P]),
        "dsmoe_bench_xcc_ids": (c_int32, [P, c_int32, P]),
        "dsmoe_moa_create": (c_int32, [POINTER(MoaDesc), POINTER(c_void_p)]),
        "dsmoe_moa_destroy": (c_int32, [P]),
        "dsmoe_moa_last_error": (c_char_p, [P]),
        "dsmoe_moa_workspace_bytes": (c_int32, [P, POINTER(c_size_t)]),
        "dsmoe_moa_set_workspace": (c_int32, [P, P, c_size_t]),
        "dsmoe_moa_fwd": (c_int32, [P, P, P, P, P, P, P, P, c_int32, c_int32, c_int32, c_int32, c_float, c_float, P, P]),
        "dsmoe_moa_routing": (c_int32, [P, c_int32, P, P, P]),
        "dsmoe_moa_bwd_scratch_bytes": (c_int32, [P, c_int32, c_int32, POINTER(c_size_t)]),
        "dsmoe_moa_bwd": (c_int32, [P, P, P, P, P, P, P, P, c_int32, c_int32, c_float, P, P, P, P, P, P, P, P, P]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _ptr(t):
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to libdsmoe must be contiguous device tensors")
    return c_void_p(t.data_ptr())


def _stream():
    import torch
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def bench_mfma(random_operands: bool, blocks: int = 1024, iters: int = 20000):
    """TFLOP/s of a bare bf16 MFMA loop (dsmoe_bench_mfma) on zero or random register operands."""
    import torch
    lib = load_library()
    seed = (torch.randn(8192, device="cuda:0") if random_operands else torch.zeros(8192, device="cuda:0")).to(torch.bfloat16)
    sink = torch.empty(blocks * 512, dtype=torch.float32, device="cuda:0")
    ms, flop = c_float(), ctypes.c_double()
    rc = lib.dsmoe_bench_mfma(_ptr(seed), _ptr(sink), blocks, iters, byref(ms), byref(flop), _stream())
    if rc != OK:
        raise DsmoeError(rc, "dsmoe_bench_mfma")
    return flop.value / (ms.value * 1e-3) / 1e12


def bench_stream(buf, offset: int, nbytes: int, write: bool, blocks: int = 2048):
    """GB/s of one streaming pass (dsmoe_bench_stream) over bytes [offset, offset + nbytes) of the uint8 tensor buf."""
    import torch
    lib = load_library()
    sink = torch.zeros(4, dtype=torch.float32, device=buf.device)
    ms, moved = c_float(), c_size_t()
    rc = lib.dsmoe_bench_stream(c_void_p(buf.data_ptr() + offset), c_size_t(nbytes), int(write), blocks, _ptr(sink),
                                byref(ms), byref(moved), _stream())
    if rc != OK:
        raise DsmoeError(rc, "dsmoe_bench_stream")
    return moved.value / (ms.value * 1e-3) / 1e9


def dense_decode_applies(layer, T: int, mode: int, k: int, eps: float) -> bool:
    """Whether dsmoe_sparse_fwd serves this call with the persistent all-expert decode kernel (what the library
    decides from the batch size and the selection rule; reported by the benchmark)."""
    lib = load_library()
    return bool(lib.dsmoe_sparse_fwd_uses_persistent_kernel(layer.ctx, T, mode, k, c_float(eps)))


PATH_GROUPED, PATH_STREAMING, PATH_ALL_EXPERTS, PATH_FEW_TOKENS = 0, 1, 2, 3


def sparse_fwd_path(layer, T: int, mode: int, k: int, eps: float) -> int:
    """Which kernels dsmoe_sparse_fwd runs for such a call (one of the PATH_* values)."""
    return int(load_library().dsmoe_sparse_fwd_path(layer.ctx, T, mode, k, c_float(eps)))


def xcc_ids(blocks: int = 256):
    """Hardware XCD id of every block of a `blocks`-block launch (torch int32 tensor on the host)."""
    import torch
    lib = load_library()
    out = torch.full((blocks,), -1, dtype=torch.int32, device="cuda:0")
    rc = lib.dsmoe_bench_xcc_ids(_ptr(out), blocks, _stream())
    if rc != OK:
        raise DsmoeError(rc, "dsmoe_bench_xcc_ids")
    torch.cuda.synchronize()
    return out.cpu()


class Layer:
    """One `dsmoe_ctx` plus its workspace.  Method names and argument order mirror the C ABI."""

    def __init__(self, d_model: int, d_ff: int, n_experts: int, dtype: str, max_tokens: int,
                 max_rows: int | None = None, device="cuda:0", expert: str = "swiglu", workspace: bool = True):
        import torch
        self.lib = load_library()
        self.torch = torch
        self.device = torch.device(device)
        self.d, self.f, self.E = d_model, d_ff, n_experts
        self.dtype_code = {"f32": F32, "bf16": BF16}[dtype]
        self.tdtype = torch.float32 if dtype == "f32" else torch.bfloat16
        self.max_tokens = max_tokens
        self.max_rows = max_tokens * n_experts if max_rows is None else max_rows
        desc = Desc(d_model, d_ff, n_experts, self.dtype_code, max_tokens, self.max_rows)
        self.ctx = c_void_p()
        rc = self.lib.dsmoe_create(byref(desc), byref(self.ctx))
        if rc != OK:
            raise DsmoeError(rc, "dsmoe_create rejected the descriptor")
        self.expert = expert
        self._check(self.lib.dsmoe_set_expert_kind(self.ctx, {"swiglu": EXPERT_SWIGLU, "gelu": EXPERT_GELU}[expert]))
        nbytes = c_size_t()
        self._check(self.lib.dsmoe_workspace_bytes(self.ctx, byref(nbytes)))
        self.workspace_bytes = nbytes.value
        self.workspace = None
        if workspace:       # workspace=False: only the calls that need none (e.g. dsmoe_dispatch_static) work
            with torch.cuda.device(self.device):
                self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.device)
                base = (self.workspace.data_ptr() + 255) // 256 * 256
                self._check(self.lib.dsmoe_set_workspace(self.ctx, c_void_p(base), c_size_t(nbytes.value)))

    def __del__(self):
        try:
            if getattr(self, "ctx", None):
                self.lib.dsmoe_destroy(self.ctx)
                self.ctx = None
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != OK:
            raise DsmoeError(rc, self.lib.dsmoe_last_error(self.ctx).decode())

    def _empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device=self.device)

    # ---- staged calls ---------------------------------------------------------------------------
    def route(self, x, w_r, b_r=None):
        T = x.shape[0]
        probs = self._empty((T, self.E), self.torch.float32)
        self._check(self.lib.dsmoe_route(self.ctx, _ptr(x), _ptr(w_r), _ptr(b_r), T, _ptr(probs), _stream()))
        return probs

    def select(self, probs, mode: int, k: int = 0, eps: float = 0.0):
        T = probs.shape[0]
        mask = self._empty((T,), self.torch.int64)
        cnt = self._empty((T,), self.torch.int32)
        self._check(self.lib.dsmoe_select(self.ctx, _ptr(probs), T, mode, k, eps, _ptr(mask), _ptr(cnt), _stream()))
        return mask, cnt

    def dispatch(self, x, probs, mask, materialize: bool = False, static: bool = False, out=None):
        """static: dsmoe_dispatch_static (the library's own scratch array instead of the workspace);
        out: a dict of buffers from an earlier call to write into (nothing is allocated then)."""
        T = probs.shape[0]
        t = self.torch
        cap = max(self.max_rows, 1)
        r = out if out is not None else dict(
            expert_off=self._empty((self.E + 1,), t.int32), row_token=self._empty((cap,), t.int32),
            row_weight=self._empty((cap,), t.float32), tok_off=self._empty((T + 1,), t.int32),
            tok_rows=self._empty((cap,), t.int32), nnz=self._empty((4,), t.int32),
            x_perm=self._empty((cap, self.d), self.tdtype) if materialize else None)
        fn = self.lib.dsmoe_dispatch_static if static else self.lib.dsmoe_dispatch
        self._check(fn(self.ctx, _ptr(x), _ptr(probs), _ptr(mask), T, _ptr(r["expert_off"]),
                    _ptr(r["row_token"]), _ptr(r["row_weight"]), _ptr(r["tok_off"]),
                    _ptr(r["tok_rows"]), _ptr(r["nnz"]), _ptr(r["x_perm"]), _stream()))
        return r

    def expert_ffn(self, x, r, w_gate, w_up, w_down):
        y = self._empty((max(self.max_rows, 1), self.d), self.tdtype)
        self._check(self.lib.dsmoe_expert_ffn(self.ctx, _ptr(x), _ptr(r.get("x_perm")), _ptr(r["row_token"]),
                                              _ptr(r["expert_off"]), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                              _ptr(y), _stream()))
        return y

    def combine(self, y_perm, r, T: int):
        out = self._empty((T, self.d), self.tdtype)
        self._check(self.lib.dsmoe_combine(self.ctx, _ptr(y_perm), _ptr(r["row_weight"]), _ptr(r["tok_off"]),
                                           _ptr(r["tok_rows"]), T, _ptr(out), _stream()))
        return out

    # ---- fused calls ----------------------------------------------------------------------------
    def sparse_fwd(self, x, w_r, b_r, w_gate, w_up, w_down, mode: int, k: int = 0, eps: float = 0.0, out=None):
        T = x.shape[0]
        if out is None:
            out = self._empty((T, self.d), self.tdtype)
        self._check(self.lib.dsmoe_sparse_fwd(self.ctx, _ptr(x), _ptr(w_r), _ptr(b_r), _ptr(w_gate), _ptr(w_up),
                                              _ptr(w_down), T, mode, k, eps, _ptr(out), _stream()))
        return out

    def sparse_fwd_routing(self, T: int):
        t = self.torch
        probs = self._empty((T, self.E), t.float32)
        mask = self._empty((T,), t.int64)
        expert_off = self._empty((self.E + 1,), t.int32)
        row_token = self._empty((max(self.max_rows, 1),), t.int32)
        self._check(self.lib.dsmoe_sparse_fwd_routing(self.ctx, T, _ptr(probs), _ptr(mask), _ptr(expert_off),
                                                      _ptr(row_token), _stream()))
        return probs, mask, expert_off, row_token

    def profile_enable(self, max_calls: int):
        self._check(self.lib.dsmoe_profile_enable(self.ctx, max_calls))

    def profile_read(self):
        """(calls, summed gate/up kernel ms, summed down kernel ms) since the last read."""
        n, a, b = c_int32(), c_float(), c_float()
        self._check(self.lib.dsmoe_profile_read(self.ctx, byref(n), byref(a), byref(b)))
        return n.value, a.value, b.value

    def set_sync_spin_limit(self, polls: int):
        self._check(self.lib.dsmoe_set_sync_spin_limit(self.ctx, polls))

    def poll_error(self) -> int:
        return self.lib.dsmoe_poll_error(self.ctx, _stream())

    def dense_buffers(self, T: int, with_bias_grad: bool = False):
        """Every output and scratch buffer of one dense forward + backward, allocated once."""
        t = self.torch
        n1, n2 = c_size_t(), c_size_t()
        self._check(self.lib.dsmoe_dense_saved_bytes(self.ctx, T, byref(n1)))
        self._check(self.lib.dsmoe_dense_bwd_scratch_bytes(self.ctx, T, byref(n2)))
        return dict(out=self._empty((T, self.d), self.tdtype), probs=self._empty((T, self.E), t.float32),
                    saved=self._empty((max(n1.value, 16),), t.uint8),
                    scratch=self._empty((max(n2.value, 16),), t.uint8),
                    dx=self._empty((T, self.d), self.tdtype), dw_r=self._empty((self.d, self.E), t.float32),
                    db_r=self._empty((self.E,), t.float32) if with_bias_grad else None,
                    dw_gate=self._empty((self.E, self.d, self.f), t.float32),
                    dw_up=self._empty((self.E, self.d, self.f), t.float32) if self.expert == "swiglu" else None,
                    dw_down=self._empty((self.E, self.f, self.d), t.float32))

    def dense_fwd(self, x, w_r, b_r, w_gate, w_up, w_down, want_probs=False, save=False, buffers=None):
        T = x.shape[0]
        t = self.torch
        if buffers is not None:
            out, probs, saved = buffers["out"], buffers["probs"], buffers["saved"]
        else:
            out = self._empty((T, self.d), self.tdtype)
            probs = self._empty((T, self.E), t.float32) if want_probs else None
            saved = None
            if save:
                n = c_size_t()
                self._check(self.lib.dsmoe_dense_saved_bytes(self.ctx, T, byref(n)))
                saved = self._empty((max(n.value, 16),), t.uint8)
        self._check(self.lib.dsmoe_dense_fwd(self.ctx, _ptr(x), _ptr(w_r), _ptr(b_r), _ptr(w_gate), _ptr(w_up),
                                             _ptr(w_down), T, _ptr(out), _ptr(probs), _ptr(saved), _stream()))
        return out, probs, saved

    def mi_loss(self, probs):
        """(loss fp32 [1], p_mean fp32 [E]) of the router scores probs [T,E], both on the device."""
        t = self.torch
        loss, p_mean = self._empty((1,), t.float32), self._empty((self.E,), t.float32)
        self._check(self.lib.dsmoe_mi_loss(self.ctx, _ptr(probs), probs.shape[0], _ptr(loss), _ptr(p_mean), _stream()))
        return loss, p_mean

    def dense_bwd(self, x, w_r, w_gate, w_up, w_down, saved, d_out, with_bias_grad=False, buffers=None,
                  mi_alpha: float = 0.0):
        T = x.shape[0]
        t = self.torch
        if buffers is not None:
            scratch, g = buffers["scratch"], buffers
        else:
            n = c_size_t()
            self._check(self.lib.dsmoe_dense_bwd_scratch_bytes(self.ctx, T, byref(n)))
            scratch = self._empty((max(n.value, 16),), t.uint8)
            g = dict(dx=self._empty((T, self.d), self.tdtype), dw_r=self._empty((self.d, self.E), t.float32),
                     db_r=self._empty((self.E,), t.float32) if with_bias_grad else None,
                     dw_gate=self._empty((self.E, self.d, self.f), t.float32),
                     dw_up=self._empty((self.E, self.d, self.f), t.float32) if self.expert == "swiglu" else None,
                     dw_down=self._empty((self.E, self.f, self.d), t.float32))
        args = (self.ctx, _ptr(x), _ptr(w_r), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(saved), _ptr(d_out), T,
                _ptr(scratch), _ptr(g["dx"]), _ptr(g["dw_r"]), _ptr(g["db_r"]), _ptr(g["dw_gate"]), _ptr(g["dw_up"]),
                _ptr(g["dw_down"]))
        if mi_alpha != 0.0:
            self._check(self.lib.dsmoe_dense_bwd_mi(*args, c_float(mi_alpha), _stream()))
        else:
            self._check(self.lib.dsmoe_dense_bwd(*args, _stream()))
        return g


class MoaLayer:
    """One `dsmoe_moa_ctx` plus its workspace (Mixture-of-Attention-heads layer, bf16)."""

    def __init__(self, d_model: int, n_experts: int, n_head: int, d_head: int, max_tokens: int, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.torch = torch
        self.device = torch.device(device)
        self.d, self.E, self.n_head, self.d_head = d_model, n_experts, n_head, d_head
        self.max_tokens = max_tokens
        desc = MoaDesc(d_model, n_experts, n_head, d_head, BF16, max_tokens)
        self.ctx = c_void_p()
        rc = self.lib.dsmoe_moa_create(byref(desc), byref(self.ctx))
        if rc != OK:
            raise DsmoeError(rc, "dsmoe_moa_create rejected the descriptor")
        nbytes = c_size_t()
        self._check(self.lib.dsmoe_moa_workspace_bytes(self.ctx, byref(nbytes)))
        self.workspace_bytes = nbytes.value
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes.value + 256, dtype=torch.uint8, device=self.device)
            base = (self.workspace.data_ptr() + 255) // 256 * 256
            self._check(self.lib.dsmoe_moa_set_workspace(self.ctx, c_void_p(base), c_size_t(nbytes.value)))

    def __del__(self):
        try:
            if getattr(self, "ctx", None):
                self.lib.dsmoe_moa_destroy(self.ctx)
                self.ctx = None
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != OK:
            raise DsmoeError(rc, self.lib.dsmoe_moa_last_error(self.ctx).decode())

    def fwd(self, x, w_r, b_r, w_q, k_cache, v_cache, w_o, mode: int, k: int = 0, eps: float = 0.0,
            scale: float = 1.0, out=None):
        T, L = x.shape[0], k_cache.shape[1]
        if out is None:
            out = self.torch.empty((T, self.d), dtype=self.torch.bfloat16, device=self.device)
        self._check(self.lib.dsmoe_moa_fwd(self.ctx, _ptr(x), _ptr(w_r), _ptr(b_r), _ptr(w_q), _ptr(k_cache),
                                           _ptr(v_cache), _ptr(w_o), T, L, mode, k, eps, scale, _ptr(out), _stream()))
        return out

    def routing(self, T: int):
        t = self.torch
        probs = t.empty((T, self.E), dtype=t.float32, device=self.device)
        mask = t.empty((T,), dtype=t.int64, device=self.device)
        self._check(self.lib.dsmoe_moa_routing(self.ctx, T, _ptr(probs), _ptr(mask), _stream()))
        return probs, mask

    def bwd_scratch_bytes(self, T: int, L: int) -> int:
        n = c_size_t()
        self._check(self.lib.dsmoe_moa_bwd_scratch_bytes(self.ctx, T, L, byref(n)))
        return n.value

    def bwd(self, x, w_r, w_q, k_cache, v_cache, w_o, d_out, scale: float = 1.0, scratch=None, grads=None,
            want_db_r: bool = True):
        """Gradients of the dense-training forward (`fwd` with mode SEL_ALL, called right before with the same
        arguments).  Returns a dict dx, dw_r, db_r, dw_q, dw_o, dk, dv; `scratch` / `grads` may be reused."""
        t = self.torch
        T, L = x.shape[0], k_cache.shape[1]
        hd = self.n_head * self.d_head
        if scratch is None:
            scratch = t.empty(self.bwd_scratch_bytes(T, L) + 256, dtype=t.uint8, device=self.device)
        base = (scratch.data_ptr() + 255) // 256 * 256
        if grads is None:
            f = dict(dtype=t.float32, device=self.device)
            grads = dict(dx=t.empty((T, self.d), dtype=t.bfloat16, device=self.device),
                         dw_r=t.empty((self.d, self.E), **f), db_r=t.empty((self.E,), **f) if want_db_r else None,
                         dw_q=t.empty((self.E, self.d, hd), **f), dw_o=t.empty((self.E, hd, self.d), **f),
                         dk=t.empty((self.n_head, L, self.d_head), **f), dv=t.empty((self.n_head, L, self.d_head), **f))
        g = grads
        self._check(self.lib.dsmoe_moa_bwd(self.ctx, _ptr(x), _ptr(w_r), _ptr(w_q), _ptr(k_cache), _ptr(v_cache),
                                           _ptr(w_o), _ptr(d_out), T, L, scale, c_void_p(base), _ptr(g["dx"]),
                                           _ptr(g["dw_r"]), _ptr(g["db_r"]), _ptr(g["dw_q"]), _ptr(g["dw_o"]),
                                           _ptr(g["dk"]), _ptr(g["dv"]), _stream()))
        return grads
