"""ctypes binding of libtrispec.so: argument marshalling only.

Every step of the verification pass runs in the HIP kernels behind the C ABI
(include/trispec.h).  torch is used for device memory and the stream, nothing
else.  There is no CPU fallback: if the shared library is missing, importing
the binding's entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtrispec.so")

TRISPEC_F32, TRISPEC_BF16 = 0, 1
CRIT_MARGIN, CRIT_TOP1, CRIT_ENTROPY = 0, 1, 2
RESAMPLE_RESIDUAL, RESAMPLE_DIRECT = 0, 1
MAX_NODES, MAX_BATCH, MAX_ROWS, PATH_STRIDE = 128, 8, 256, 128

EXPORTS = [
    "trispec_model_create", "trispec_model_destroy", "trispec_kv_bytes", "trispec_kv_create",
    "trispec_kv_set_len", "trispec_kv_destroy", "trispec_workspace_bytes",
    "trispec_workspace_region", "trispec_pass_bytes", "trispec_verify", "trispec_decide",
    "trispec_strerror", "trispec_timer_create", "trispec_timer_reset", "trispec_timer_read",
    "trispec_timer_destroy", "trispec_model_pack_bytes", "trispec_model_pack", "trispec_copy_probe",
    "trispec_kv_commit", "trispec_sample_scratch_bytes", "trispec_sample_decide",
    "trispec_sample_decide_static", "trispec_debug_set_spin_limit", "trispec_wait_probe",
    "trispec_prune_reroot", "trispec_draft_ranks", "trispec_pack_matrix_bytes", "trispec_pack_matrix",
    "trispec_kv_get_len", "trispec_kv_paged_bytes", "trispec_kv_create_paged", "trispec_ternary_create", "trispec_ternary_destroy", "trispec_ternary_start",
    "trispec_ternary_resume", "trispec_ternary_round", "trispec_ternary_sequence", "trispec_ternary_round_sample",
]
K_GEMM, K_HEAD, K_ATTN = 0, 1, 2
LAUNCH_PER_MATMUL, LAUNCH_PER_LAYER = 0, 1


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("qk_norm", C.c_int32)]


_PP = C.POINTER(C.c_void_p)
TERNARY_SCRATCH_INTS = 1024


class TernaryConfig(C.Structure):
    _fields_ = [("proxy", C.c_void_p), ("target", C.c_void_p), ("kv_proxy", C.c_void_p), ("kv_target", C.c_void_p),
                ("workspace_proxy", C.c_void_p), ("workspace_target", C.c_void_p),
                ("workspace_proxy_bytes", C.c_size_t), ("workspace_target_bytes", C.c_size_t),
                ("scratch_dev", C.c_void_p), ("criterion", C.c_int32), ("max_nodes", C.c_int32),
                ("stream", C.c_void_p)]


class PassResult(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("accepted_len", "token", "escalate", "status", "path_len")] + \
               [("path", C.c_int32 * PATH_STRIDE)]


class SampleRound(C.Structure):
    _fields_ = [("temperature", C.c_float), ("resample", C.c_int32), ("p_draft_dev", C.c_void_p),
                ("u_accept_proxy_host", C.POINTER(C.c_float)), ("u_accept_target_host", C.POINTER(C.c_float)),
                ("u_sample_proxy", C.c_float), ("u_sample_target", C.c_float),
                ("logits_dev", C.c_void_p), ("p_draft_work_dev", C.c_void_p)]


class RoundInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("escalate", "catch_up", "target_nodes", "n_forced_target", "n_emitted",
                                         "ctx_len_proxy", "ctx_len_target")] + \
               [("proxy", PassResult), ("target", PassResult)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, _PP) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn",
                                   "q_norm", "k_norm")]


class VerifyOpts(C.Structure):
    _fields_ = [("criterion", C.c_int32), ("n_forced", C.c_int32), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("debug_logits", C.c_void_p), ("stream", C.c_void_p),
                ("timer", C.c_void_p), ("hidden_out", C.c_void_p), ("launch_mode", C.c_int32),
                ("feature_layers", C.POINTER(C.c_int32)), ("n_feature_layers", C.c_int32),
                ("features_out", C.c_void_p), ("adapter_w", C.c_void_p), ("adapter_bias", C.c_void_p),
                ("adapter_dim", C.c_int32), ("adapter_out", C.c_void_p),
                ("draft_ranks", C.c_void_p), ("accept_top_k", C.c_int32), ("stamps", C.c_void_p)]


class VerifyOut(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("accepted_len", "token", "escalate", "path", "argmax", "confidence", "margin", "entropy", "status")]


class SampleOpts(C.Structure):
    _fields_ = [("temperature", C.c_float), ("resample", C.c_int32), ("criterion", C.c_int32),
                ("n_forced", C.c_int32), ("p_draft", C.c_void_p), ("u_accept", C.c_void_p),
                ("u_sample", C.c_void_p), ("scratch", C.c_void_p), ("scratch_bytes", C.c_size_t),
                ("stream", C.c_void_p)]


class TriSpecError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"trispec error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (python -m paper_2601_23180_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2601_23180_amd.build` "
                "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        l.trispec_strerror.restype = C.c_char_p
        l.trispec_strerror.argtypes = [C.c_int]
        for name in EXPORTS:
            if name != "trispec_strerror":
                getattr(l, name).restype = C.c_int
        l.trispec_model_create.argtypes = [C.POINTER(ModelConfig), C.POINTER(Weights), C.POINTER(C.c_void_p)]
        l.trispec_model_destroy.argtypes = [C.c_void_p]
        l.trispec_model_pack_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
        l.trispec_model_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        l.trispec_kv_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        l.trispec_kv_create.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                        C.POINTER(C.c_void_p)]
        l.trispec_kv_set_len.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        l.trispec_kv_get_len.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        l.trispec_kv_paged_bytes.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
        l.trispec_kv_create_paged.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                              C.c_int32, C.POINTER(C.c_void_p)]
        l.trispec_ternary_create.argtypes = [C.POINTER(TernaryConfig), C.POINTER(C.c_void_p)]
        l.trispec_ternary_destroy.argtypes = [C.c_void_p]
        l.trispec_ternary_start.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        l.trispec_ternary_resume.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32]
        l.trispec_ternary_round.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
                                            C.c_float, C.POINTER(RoundInfo)]
        l.trispec_ternary_round_sample.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_float,
                                                   C.POINTER(SampleRound), C.POINTER(RoundInfo)]
        l.trispec_ternary_sequence.argtypes = [C.c_void_p, C.POINTER(C.POINTER(C.c_int32)), C.POINTER(C.c_int32)]
        l.trispec_kv_destroy.argtypes = [C.c_void_p]
        l.trispec_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        l.trispec_workspace_region.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_char_p,
                                               C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        l.trispec_kv_commit.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_void_p]
        l.trispec_copy_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.trispec_pass_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                         C.POINTER(C.c_double)]
        l.trispec_verify.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_void_p,
                                     C.c_int32, C.c_float, C.POINTER(VerifyOpts), C.POINTER(VerifyOut)]
        l.trispec_decide.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_int32), C.c_int32,
                                     C.c_float, C.POINTER(VerifyOpts), C.POINTER(VerifyOut)]
        l.trispec_sample_scratch_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        l.trispec_sample_decide.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                            C.POINTER(SampleOpts), C.POINTER(VerifyOut)]
        l.trispec_sample_decide_static.argtypes = l.trispec_sample_decide.argtypes
        l.trispec_debug_set_spin_limit.argtypes = [C.c_uint64]
        l.trispec_wait_probe.argtypes = [C.c_void_p, C.c_int32, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        _pi = C.POINTER(C.c_int32)
        l.trispec_prune_reroot.argtypes = [_pi, _pi, _pi, C.c_int32, _pi, C.c_int32, _pi, C.c_int32, C.c_int32,
                                           _pi, _pi, _pi, _pi, _pi, _pi]
        l.trispec_pack_matrix_bytes.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        l.trispec_pack_matrix.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        l.trispec_draft_ranks.argtypes = [C.c_void_p, C.c_void_p, _pi, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                          C.c_void_p]
        l.trispec_timer_create.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        l.trispec_timer_reset.argtypes = [C.c_void_p]
        l.trispec_timer_read.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                         C.POINTER(C.c_double)]
        l.trispec_timer_destroy.argtypes = [C.c_void_p]
        _lib = l
    return _lib


def check(rc: int) -> None:
    if rc != 0:
        raise TriSpecError(rc, lib().trispec_strerror(rc).decode())


def _torch_dtype(dtype: int):
    return torch.float32 if dtype == TRISPEC_F32 else torch.bfloat16


_LAYER_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")


class Model:
    """trispec_model over device tensors the caller supplies.

    tensors: {"embed", "lm_head", "final_norm": tensor, "wq".. : list of n_layers tensors}
    (row-major [out, in], on the GPU, dtype matching `dtype`).  The object keeps them alive.
    """

    def __init__(self, *, n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, dtype,
                 rms_eps, rope_base, tensors: Dict[str, object], qk_norm: bool = False):
        self.cfg = ModelConfig(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, dtype,
                               rms_eps, rope_base, 1 if qk_norm else 0)
        self.tensors = tensors
        self.dtype = dtype
        w = Weights()
        w.embed = tensors["embed"].data_ptr()
        w.lm_head = tensors["lm_head"].data_ptr()
        w.final_norm = tensors["final_norm"].data_ptr()
        self._tables = []
        for n in _LAYER_NAMES + (("q_norm", "k_norm") if qk_norm else ()):
            arr = (C.c_void_p * n_layers)(*[t.data_ptr() for t in tensors[n]])
            self._tables.append(arr)
            setattr(w, n, C.cast(arr, _PP))
        self.handle = C.c_void_p()
        check(lib().trispec_model_create(C.byref(self.cfg), C.byref(w), C.byref(self.handle)))
        self.packed = None

    def pack(self, release_originals: bool = False, device="cuda") -> None:
        """Repack the matrices for the streaming kernels (bf16 models; a no-op for fp32).
        release_originals drops this object's references to wq..w_down / lm_head afterwards."""
        n = C.c_size_t()
        check(lib().trispec_model_pack_bytes(self.handle, C.byref(n)))
        if n.value:
            self.packed = torch.empty(n.value + 256, dtype=torch.uint8, device=device)
            ptr = self.packed.data_ptr() + (-self.packed.data_ptr()) % 256
        else:
            ptr = None
        check(lib().trispec_model_pack(self.handle, ptr, torch.cuda.current_stream().cuda_stream))
        if release_originals and n.value:
            torch.cuda.current_stream().synchronize()
            for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                self.tensors[name] = None
            if self.tensors["lm_head"] is not self.tensors["embed"]:
                self.tensors["lm_head"] = None

    def workspace_bytes(self, batch: int, max_nodes: int) -> int:
        n = C.c_size_t()
        check(lib().trispec_workspace_bytes(self.handle, batch, max_nodes, C.byref(n)))
        return n.value

    def workspace_region(self, batch: int, n_nodes: int, name: str):
        off, n = C.c_size_t(), C.c_size_t()
        check(lib().trispec_workspace_region(self.handle, batch, n_nodes, name.encode(), C.byref(off), C.byref(n)))
        return off.value, n.value

    def pass_bytes(self, batch: int, n_nodes: int, ctx_len: Sequence[int]) -> float:
        arr = (C.c_int32 * batch)(*ctx_len)
        out = C.c_double()
        check(lib().trispec_pass_bytes(self.handle, batch, n_nodes, arr, C.byref(out)))
        return out.value

    def close(self):
        if self.handle:
            lib().trispec_model_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KVCache:
    """trispec_kv over two device tensors:
    K [L, B, n_kv, capacity, d] (post-rotary keys) and V [L, B, n_kv, d, capacity] (transposed)."""

    def __init__(self, model: Model, batch: int, capacity: int, k: Optional[torch.Tensor] = None,
                 v: Optional[torch.Tensor] = None, device="cuda"):
        c = model.cfg
        n = C.c_size_t()
        check(lib().trispec_kv_bytes(model.handle, batch, capacity, C.byref(n)))
        dt = _torch_dtype(c.dtype)
        self.k = k if k is not None else torch.zeros((c.n_layers, batch, c.n_kv_heads, capacity, c.head_dim),
                                                      dtype=dt, device=device)
        self.v = v if v is not None else torch.zeros((c.n_layers, batch, c.n_kv_heads, c.head_dim, capacity),
                                                      dtype=dt, device=device)
        assert self.k.is_contiguous() and self.v.is_contiguous()
        assert self.k.numel() * self.k.element_size() == n.value == self.v.numel() * self.v.element_size()
        self.model, self.batch, self.capacity = model, batch, capacity
        self.handle = C.c_void_p()
        check(lib().trispec_kv_create(model.handle, self.k.data_ptr(), self.v.data_ptr(), batch, capacity,
                                      C.byref(self.handle)))
        self.ctx_len = [0] * batch

    def set_len(self, ctx_len: Sequence[int]) -> None:
        arr = (C.c_int32 * self.batch)(*ctx_len)
        check(lib().trispec_kv_set_len(self.handle, arr))
        self.ctx_len = list(ctx_len)

    def load_dense(self, k: torch.Tensor, v: torch.Tensor) -> None:
        """k [L, B, n_kv, capacity, d], v [L, B, n_kv, d, capacity] (the layout of self.k / self.v)."""
        self.k.copy_(k)
        self.v.copy_(v)

    def write_layer(self, layer: int, k: torch.Tensor, v: torch.Tensor) -> None:
        """The first C slots of one layer: k, v [B, n_kv, C, d] (V is stored transposed)."""
        C_ = k.shape[2]
        self.k[layer, :, :, :C_, :] = k.to(self.k.dtype)
        self.v[layer, :, :, :, :C_] = v.to(self.v.dtype).transpose(-1, -2)

    def sync_len(self) -> None:
        """Re-read the context lengths from the library (after calls that commit inside it)."""
        arr = (C.c_int32 * self.batch)()
        check(lib().trispec_kv_get_len(self.handle, arr))
        self.ctx_len = list(arr)

    def commit(self, nodes: Sequence[Sequence[int]], stream=None) -> None:
        """trispec_kv_commit: nodes[b] = node ids of sequence b's verified path, root first."""
        arr = (C.c_int32 * (self.batch * PATH_STRIDE))()
        cnt = (C.c_int32 * self.batch)()
        for b, p in enumerate(nodes):
            cnt[b] = len(p)
            for i, v in enumerate(p):
                arr[b * PATH_STRIDE + i] = int(v)
        st = (stream if stream is not None else torch.cuda.current_stream()).cuda_stream
        check(lib().trispec_kv_commit(self.handle, arr, cnt, st))
        self.ctx_len = [c + len(p) for c, p in zip(self.ctx_len, nodes)]

    def close(self):
        if self.handle:
            lib().trispec_kv_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


KV_PAGE = 256


class PagedKVCache(KVCache):
    """trispec_kv over two page pools and a device page table (trispec_kv_create_paged):
    K pool [L, n_pages, n_kv, KV_PAGE, d], V pool [L, n_pages, n_kv, d, KV_PAGE]; slot s of sequence b is
    slot s % KV_PAGE of page table[b, s // KV_PAGE].  `table` (int array [batch, max_pages]) defaults to a
    seeded shuffle of the pool with `spare_pages` pages left unmapped.  `k` and `v` READ the cache as
    dense tensors in the contiguous layout (copies); `load_dense` writes such tensors into the pages."""

    def __init__(self, model: Model, batch: int, capacity: int, table=None, spare_pages: int = 3, seed: int = 0,
                 device="cuda"):
        c = model.cfg
        self.max_pages = (capacity + KV_PAGE - 1) // KV_PAGE
        if table is None:
            self.n_pages = batch * self.max_pages + spare_pages
            g = torch.Generator().manual_seed(seed)
            table = torch.randperm(self.n_pages, generator=g)[: batch * self.max_pages].reshape(batch, self.max_pages)
        else:
            table = torch.as_tensor(table).reshape(batch, self.max_pages)
            self.n_pages = int(table.max()) + 1 + spare_pages
        self.table = table.to(torch.int32).to(device).contiguous()
        n = C.c_size_t()
        check(lib().trispec_kv_paged_bytes(model.handle, self.n_pages, C.byref(n)))
        dt = _torch_dtype(c.dtype)
        self.k_pool = torch.zeros((c.n_layers, self.n_pages, c.n_kv_heads, KV_PAGE, c.head_dim), dtype=dt, device=device)
        self.v_pool = torch.zeros((c.n_layers, self.n_pages, c.n_kv_heads, c.head_dim, KV_PAGE), dtype=dt, device=device)
        assert self.k_pool.numel() * self.k_pool.element_size() == n.value
        self.model, self.batch, self.capacity = model, batch, self.max_pages * KV_PAGE
        self.handle = C.c_void_p()
        check(lib().trispec_kv_create_paged(model.handle, self.k_pool.data_ptr(), self.v_pool.data_ptr(),
                                            self.table.data_ptr(), batch, self.max_pages, self.n_pages,
                                            C.byref(self.handle)))
        self.ctx_len = [0] * batch

    @property
    def k(self) -> torch.Tensor:          # [L, B, n_kv, capacity, d]
        t = self.k_pool[:, self.table.long()]                      # [L, B, P, n_kv, page, d]
        L, B, P, H, S, D = t.shape
        return t.permute(0, 1, 3, 2, 4, 5).reshape(L, B, H, P * S, D)

    @property
    def v(self) -> torch.Tensor:          # [L, B, n_kv, d, capacity]
        t = self.v_pool[:, self.table.long()]                      # [L, B, P, n_kv, d, page]
        L, B, P, H, D, S = t.shape
        return t.permute(0, 1, 3, 4, 2, 5).reshape(L, B, H, D, P * S)

    def load_dense(self, k: torch.Tensor, v: torch.Tensor) -> None:
        """k [L, B, n_kv, capacity, d], v [L, B, n_kv, d, capacity] -> the mapped pages."""
        L, B, H, Cc, D = k.shape
        P, S = self.max_pages, KV_PAGE
        assert Cc == self.capacity
        kp = k.reshape(L, B, H, P, S, D).permute(0, 1, 3, 2, 4, 5)  # [L, B, P, H, S, D]
        vp = v.reshape(L, B, H, D, P, S).permute(0, 1, 4, 2, 3, 5)  # [L, B, P, H, D, S]
        idx = self.table.long()
        self.k_pool[:, idx] = kp.to(self.k_pool.dtype)
        self.v_pool[:, idx] = vp.to(self.v_pool.dtype)

    def write_layer(self, layer: int, k: torch.Tensor, v: torch.Tensor) -> None:
        C_ = k.shape[2]
        for p0 in range(0, C_, KV_PAGE):
            n = min(KV_PAGE, C_ - p0)
            pages = self.table[:, p0 // KV_PAGE].long()                                  # [B]
            self.k_pool[layer, pages, :, :n, :] = k[:, :, p0:p0 + n, :].to(self.k_pool.dtype)
            self.v_pool[layer, pages, :, :, :n] = v[:, :, p0:p0 + n, :].to(self.v_pool.dtype).transpose(-1, -2)


class KernelTimer:
    """HIP-event timer around every launch of one kernel class (measurement only)."""

    def __init__(self, kernel_class: int, capacity: int):
        self.handle = C.c_void_p()
        check(lib().trispec_timer_create(kernel_class, capacity, C.byref(self.handle)))

    def reset(self):
        check(lib().trispec_timer_reset(self.handle))

    def read(self):
        """(launches, total ms, total algorithmic bytes); synchronise the stream first."""
        n, ms, by = C.c_int32(), C.c_double(), C.c_double()
        check(lib().trispec_timer_read(self.handle, C.byref(n), C.byref(ms), C.byref(by)))
        return n.value, ms.value, by.value

    def __del__(self):
        try:
            if self.handle:
                lib().trispec_timer_destroy(self.handle)
                self.handle = C.c_void_p()
        except Exception:
            pass


def copy_probe(dst, src, stream=None) -> None:
    """trispec_copy_probe on two device tensors of equal byte size (argument marshalling only)."""
    import torch
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("copy_probe: sizes differ")
    st = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    check(lib().trispec_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, st))


def prune_reroot(tokens, parents, positions, path, prefix_tokens=(), prefix_pos0: int = 0) -> Dict[str, object]:
    """trispec_prune_reroot on host integer sequences (argument marshalling only)."""
    def arr(v):
        v = [int(x) for x in v]
        return (C.c_int32 * max(len(v), 1))(*v), len(v)
    tok, n = arr(tokens)
    par, _ = arr(parents)
    pos, _ = arr(positions)
    pth, n_path = arr(path)
    pre, n_pre = arr(prefix_tokens)
    out = [(C.c_int32 * MAX_NODES)() for _ in range(4)]
    n_out, n_forced = C.c_int32(), C.c_int32()
    check(lib().trispec_prune_reroot(tok, par, pos, n, pth, n_path, pre if n_pre else None, n_pre, int(prefix_pos0),
                                     out[0], out[1], out[2], out[3], C.byref(n_out), C.byref(n_forced)))
    m = n_out.value
    return {"tokens": list(out[0][:m]), "parents": list(out[1][:m]), "positions": list(out[2][:m]),
            "old_id": list(out[3][:m]), "n_forced": n_forced.value}


class SampleDecider:
    """Pre-allocated scratch and output buffers for repeated trispec_sample_decide calls on
    [batch, n_nodes, vocab] logits."""

    def __init__(self, batch: int, n_nodes: int, vocab: int, device="cuda", static_scratch: bool = False):
        """static_scratch: call trispec_sample_decide_static (the library's own scratch area; no
        scratch tensor is allocated here) instead of trispec_sample_decide."""
        self.batch, self.n_nodes, self.vocab = batch, n_nodes, vocab
        n = C.c_size_t()
        check(lib().trispec_sample_scratch_bytes(batch, n_nodes, vocab, C.byref(n)))
        self.scratch_bytes = n.value
        self.static_scratch = static_scratch
        if static_scratch:
            self.scratch, self._sptr = None, None
        else:
            self.scratch = torch.empty(n.value + 256, dtype=torch.uint8, device=device)
            self._sptr = self.scratch.data_ptr() + (-self.scratch.data_ptr()) % 256
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.out = {
            "accepted_len": torch.zeros(batch, **i32), "token": torch.zeros(batch, **i32),
            "escalate": torch.zeros(batch, **i32), "path": torch.zeros((batch, PATH_STRIDE), **i32),
            "argmax": torch.zeros((batch, n_nodes), **i32), "confidence": torch.zeros((batch, n_nodes), **f32),
            "margin": torch.zeros((batch, n_nodes), **f32), "entropy": torch.zeros((batch, n_nodes), **f32),
            "status": torch.zeros(1, **i32),
        }
        self._out = VerifyOut(*[self.out[k].data_ptr() for k, _ in VerifyOut._fields_])

    def decide(self, logits, draft_tokens, p_draft, u_accept, u_sample, temperature: float, threshold: float,
               criterion: int = CRIT_MARGIN, n_forced: int = 1, resample: int = RESAMPLE_RESIDUAL,
               stream=None) -> Dict[str, torch.Tensor]:
        """logits [batch, n_nodes, vocab] fp32, draft_tokens [batch, n_nodes] int32, p_draft
        [batch, n_nodes - 1, vocab] fp32, u_accept [batch, n_nodes] fp32, u_sample [batch] fp32,
        all contiguous device tensors.  Marshals and returns the (reused) output tensors."""
        batch, n_nodes, vocab = self.batch, self.n_nodes, self.vocab
        for t, dt, shape in ((logits, torch.float32, (batch, n_nodes, vocab)),
                             (draft_tokens, torch.int32, (batch, n_nodes)),
                             (u_accept, torch.float32, (batch, n_nodes)), (u_sample, torch.float32, (batch,))):
            if t.dtype != dt or tuple(t.shape) != shape or not t.is_contiguous() or not t.is_cuda:
                raise ValueError("sample_decide: tensor of the wrong dtype, shape, layout or device")
        if n_nodes > 1 and (p_draft.dtype != torch.float32 or tuple(p_draft.shape) != (batch, n_nodes - 1, vocab)
                            or not p_draft.is_contiguous() or not p_draft.is_cuda):
            raise ValueError("sample_decide: p_draft of the wrong dtype, shape, layout or device")
        st = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        opts = SampleOpts(float(temperature), int(resample), int(criterion), int(n_forced),
                          p_draft.data_ptr() if n_nodes > 1 else None, u_accept.data_ptr(), u_sample.data_ptr(),
                          self._sptr, self.scratch_bytes if not self.static_scratch else 0, st)
        fn = lib().trispec_sample_decide_static if self.static_scratch else lib().trispec_sample_decide
        check(fn(logits.data_ptr(), draft_tokens.data_ptr(), batch, n_nodes, vocab, float(threshold),
                 C.byref(opts), C.byref(self._out)))
        return self.out


def sample_decide(logits, draft_tokens, p_draft, u_accept, u_sample, temperature: float, threshold: float,
                  criterion: int = CRIT_MARGIN, n_forced: int = 1, resample: int = RESAMPLE_RESIDUAL,
                  stream=None) -> Dict[str, torch.Tensor]:
    """One-off form of SampleDecider.decide (allocates its buffers on every call)."""
    batch, n_nodes, vocab = logits.shape
    dec = SampleDecider(batch, n_nodes, vocab, logits.device)
    res = dict(dec.decide(logits, draft_tokens, p_draft, u_accept, u_sample, temperature, threshold, criterion,
                          n_forced, resample, stream))
    res["_decider"] = dec   # keeps scratch and outputs alive until the caller drops the result
    return res


class Verifier:
    """Pre-allocated workspace and output buffers for repeated trispec_verify calls."""

    def __init__(self, model: Model, batch: int, max_nodes: int, debug_logits: bool = False, device="cuda",
                 export_hidden: bool = False):
        self.model, self.batch, self.max_nodes = model, batch, max_nodes
        self.ws_bytes = model.workspace_bytes(batch, max_nodes)
        self.workspace = torch.zeros(self.ws_bytes + 256, dtype=torch.uint8, device=device)
        pad = (-self.workspace.data_ptr()) % 256
        self._ws_ptr = self.workspace.data_ptr() + pad
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.out = {
            "accepted_len": torch.zeros(batch, **i32), "token": torch.zeros(batch, **i32),
            "escalate": torch.zeros(batch, **i32), "path": torch.zeros((batch, PATH_STRIDE), **i32),
            "argmax": torch.zeros((batch, max_nodes), **i32), "confidence": torch.zeros((batch, max_nodes), **f32),
            "margin": torch.zeros((batch, max_nodes), **f32), "entropy": torch.zeros((batch, max_nodes), **f32),
            "status": torch.zeros(1, **i32),
        }
        self.logits = torch.zeros((batch, max_nodes, model.cfg.vocab), **f32) if debug_logits else None
        self.hidden = torch.zeros((batch, max_nodes, model.cfg.hidden), **f32) if export_hidden else None
        self.timer = None   # optional KernelTimer attached to every verify call
        self.feature_layers: List[int] = []   # layers whose residual stream is exported to self.features
        self.features = None                  # fp32 [n_feature_layers, batch, max_nodes, hidden]
        self._adapter = None                  # (weights as the kernels read them, bias or None, dim, out)
        self.ranks = None   # int32 [batch, max_nodes], filled by draft_ranks()
        self.accept_top_k = 0
        self.launch_mode = LAUNCH_PER_MATMUL
        self.stamps = None  # optional int64 device tensor [n_layers, 16] (phase time stamps of the layer launches)

    def _opts(self, criterion, n_forced, stream, want_logits):
        o = VerifyOpts()
        o.criterion, o.n_forced = criterion, n_forced
        o.workspace, o.workspace_bytes = self._ws_ptr, self.ws_bytes
        o.debug_logits = self.logits.data_ptr() if (want_logits and self.logits is not None) else None
        s = stream if stream is not None else torch.cuda.current_stream()
        o.stream = s.cuda_stream
        o.timer = self.timer.handle if self.timer is not None else None
        o.hidden_out = self.hidden.data_ptr() if self.hidden is not None else None
        o.launch_mode = self.launch_mode
        if self.feature_layers:
            if self.features is None or self.features.shape[0] != len(self.feature_layers):
                self.features = torch.zeros((len(self.feature_layers), self.batch, self.max_nodes, self.model.cfg.hidden),
                                            dtype=torch.float32, device=self.workspace.device)
            self._fl = (C.c_int32 * len(self.feature_layers))(*self.feature_layers)
            o.feature_layers, o.n_feature_layers = self._fl, len(self.feature_layers)
            o.features_out = self.features.data_ptr()
        if self._adapter is not None:
            w, b, dim, out = self._adapter
            packed = self.model.dtype == TRISPEC_BF16      # the packed copy sits at the next 256-byte boundary
            o.adapter_w = w.data_ptr() + ((-w.data_ptr()) % 256 if packed else 0)
            o.adapter_dim, o.adapter_out = dim, out.data_ptr()
            o.adapter_bias = b.data_ptr() if b is not None else None
        o.draft_ranks = self.ranks.data_ptr() if (self.ranks is not None and self.accept_top_k > 1) else None
        o.accept_top_k = self.accept_top_k if self.ranks is not None else 0
        o.stamps = self.stamps.data_ptr() if self.stamps is not None else None
        return o

    def _out(self, n_nodes):
        o = VerifyOut()
        for name, t in self.out.items():
            setattr(o, name, t.data_ptr())
        return o

    def verify(self, kv: KVCache, draft_tokens: torch.Tensor, tree_parents: np.ndarray,
               positions: torch.Tensor, threshold: float, criterion: int = CRIT_MARGIN, n_forced: int = 1,
               stream=None, want_logits: bool = True) -> Dict[str, torch.Tensor]:
        """draft_tokens / positions: int32 device tensors [batch, n_nodes]; tree_parents: host int32
        [batch, n_nodes].  n_nodes must equal max_nodes (the output buffers are laid out for it)."""
        n_nodes = draft_tokens.shape[-1]
        assert n_nodes == self.max_nodes and draft_tokens.dtype == torch.int32 and positions.dtype == torch.int32
        par = np.ascontiguousarray(tree_parents, dtype=np.int32)
        opts, out = self._opts(criterion, n_forced, stream, want_logits), self._out(n_nodes)
        check(lib().trispec_verify(self.model.handle, kv.handle, draft_tokens.data_ptr(),
                                   par.ctypes.data_as(C.POINTER(C.c_int32)), positions.data_ptr(), n_nodes,
                                   float(threshold), C.byref(opts), C.byref(out)))
        return self.out

    def decide(self, draft_tokens: torch.Tensor, tree_parents: np.ndarray, threshold: float,
               criterion: int = CRIT_MARGIN, n_forced: int = 1, stream=None) -> Dict[str, torch.Tensor]:
        n_nodes = draft_tokens.shape[-1]
        par = np.ascontiguousarray(tree_parents, dtype=np.int32)
        opts, out = self._opts(criterion, n_forced, stream, False), self._out(n_nodes)
        check(lib().trispec_decide(self.model.handle, self.batch, draft_tokens.data_ptr(),
                                   par.ctypes.data_as(C.POINTER(C.c_int32)), n_nodes, float(threshold),
                                   C.byref(opts), C.byref(out)))
        return self.out

    def set_adapter(self, weight: torch.Tensor, bias: Optional[torch.Tensor] = None) -> torch.Tensor:
        """weight: [adapter_dim, hidden] device tensor in the model's dtype; bias: fp32 [adapter_dim] or None.
        bf16 models: the matrix is repacked once (trispec_pack_matrix).  Returns the output tensor
        [batch, max_nodes, adapter_dim] that every later verify call fills."""
        dim, hid = weight.shape
        assert hid == self.model.cfg.hidden and weight.is_contiguous()
        if self.model.dtype == TRISPEC_BF16:
            n = C.c_size_t()
            check(lib().trispec_pack_matrix_bytes(dim, hid, C.byref(n)))
            w = torch.empty(n.value + 256, dtype=torch.uint8, device=weight.device)
            check(lib().trispec_pack_matrix(weight.data_ptr(), dim, hid, w.data_ptr() + (-w.data_ptr()) % 256,
                                            torch.cuda.current_stream().cuda_stream))
            torch.cuda.current_stream().synchronize()
        else:
            w = weight
        out = torch.zeros((self.batch, self.max_nodes, dim), dtype=torch.float32, device=weight.device)
        self._adapter = (w, bias, dim, out)
        return out

    def draft_ranks(self, draft_tokens: torch.Tensor, tree_parents: np.ndarray, stream=None) -> torch.Tensor:
        """trispec_draft_ranks on the logits of the last verify call (needs debug_logits=True)."""
        assert self.logits is not None, "draft_ranks needs the materialised logits (debug_logits=True)"
        if self.ranks is None:
            self.ranks = torch.zeros((self.batch, self.max_nodes), dtype=torch.int32, device=self.logits.device)
        par = np.ascontiguousarray(tree_parents, dtype=np.int32)
        s = stream if stream is not None else torch.cuda.current_stream()
        check(lib().trispec_draft_ranks(self.logits.data_ptr(), draft_tokens.data_ptr(),
                                        par.ctypes.data_as(C.POINTER(C.c_int32)), self.batch, self.max_nodes,
                                        self.model.cfg.vocab, self.ranks.data_ptr(), s.cuda_stream))
        return self.ranks

    def region(self, name: str, n_nodes: Optional[int] = None) -> torch.Tensor:
        """Raw bytes of a named workspace region (test hook)."""
        off, n = self.model.workspace_region(self.batch, n_nodes or self.max_nodes, name)
        base = self._ws_ptr - self.workspace.data_ptr()
        return self.workspace[base + off: base + off + n]
