"""Host arrays -> device tensors in the layouts the C ABI expects.  Data movement only."""
from __future__ import annotations

from typing import Callable

import numpy as np
import torch

from .binding import TRISPEC_BF16, TRISPEC_F32, KVCache, Model

_LAYER_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn")


def _to_device(a: np.ndarray, bf16: bool, device) -> torch.Tensor:
    """float32 values (exactly representable in the target dtype) or uint16 bf16 bit patterns."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16) if bf16 else t


def model_from_arrays(shape, get: Callable[[str, int], np.ndarray], device="cuda",
                      release_originals: bool = True) -> Model:
    """shape: any object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
    dtype ("f32" | "bf16"), rms_eps, rope_base.  get(name, layer) returns the tensor as float32
    values or (bf16 models) as uint16 bit patterns."""
    bf16 = shape.dtype == "bf16"
    tensors = {n: _to_device(get(n, 0), bf16, device) for n in ("embed", "lm_head", "final_norm")}
    qk_norm = bool(getattr(shape, "qk_norm", False))
    for n in _LAYER_NAMES + (("q_norm", "k_norm") if qk_norm else ()):
        tensors[n] = [_to_device(get(n, l), bf16, device) for l in range(shape.n_layers)]
    m = Model(n_layers=shape.n_layers, hidden=shape.hidden, n_q_heads=shape.n_q_heads,
                 n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, vocab=shape.vocab,
                 dtype=TRISPEC_BF16 if bf16 else TRISPEC_F32, rms_eps=shape.rms_eps,
                 rope_base=shape.rope_base, tensors=tensors, qk_norm=qk_norm)
    m.pack(release_originals=release_originals)
    return m


def fill_kv_layer(kv: KVCache, layer: int, k: np.ndarray, v: np.ndarray) -> None:
    """k, v: [batch, n_kv, C, d] values of the first C cache slots of one layer
    (keys after the rotary embedding).  V is stored transposed."""
    dev = kv.table.device if hasattr(kv, "table") else kv.k.device
    kt = torch.from_numpy(np.ascontiguousarray(k, dtype=np.float32)).to(dev)
    vt = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(dev)
    kv.write_layer(layer, kt, vt)
