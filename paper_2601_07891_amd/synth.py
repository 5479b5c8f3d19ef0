"""Seeded synthetic inputs shaped like the paper's workloads.

Generators only: this module holds none of the method's arithmetic (no scorer,
no mask, no gather).  Both the CPU oracle's tests and the HIP path's tests and
benchmark draw their inputs from here, so the two sides see identical bf16 bit
patterns.  Shapes come from the paper's overhead table (App. B: H = 8 KV heads,
D = 128, D_h = 4096 or 5120, MLP width D_h/8) and Sec. 3.3 (window 128).

All tensors are torch tensors on `device`; weights are stored output-major
([out, in], as a PyTorch linear module stores them).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    L: int            # layers
    B: int            # sequences
    T: int            # tokens per sequence
    Dh: int           # hidden size
    H: int = 8        # KV heads
    D: int = 128      # head dim
    scorer: str = "mlp"          # "mlp" | "linear"
    window: int = 128
    keep_fraction: float = 0.5   # of non-window tokens; tau is derived from it
    seed: int = 0
    token_scale_sigma: float = 0.0   # >0: per-token log-normal scale on hidden
    bias_std: float = 0.0            # 0: biases are exactly zero

    @property
    def M(self) -> int:
        return self.Dh // 8 if self.scorer == "mlp" else 0

    def layer_seed(self, layer: int) -> int:
        return self.seed * 1000 + layer if self.L > 1 else self.seed


# The five benchmark configurations (sizes and distributions as named in the
# task's baseline description; tau is always derived from the oracle's scores).
CONFIGS: Dict[str, Workload] = {
    "c1_t1k_linear": Workload("c1_t1k_linear", L=1, B=1, T=1024, Dh=4096,
                              scorer="linear", keep_fraction=0.5, seed=0),
    "c2_llama8b_32k_mlp": Workload("c2_llama8b_32k_mlp", L=1, B=1, T=32768, Dh=4096,
                                   scorer="mlp", keep_fraction=0.5, seed=0,
                                   bias_std=0.1),
    "c3_qwen8b_128k_mlp": Workload("c3_qwen8b_128k_mlp", L=36, B=1, T=131072, Dh=4096,
                                   scorer="mlp", keep_fraction=0.25, seed=3,
                                   token_scale_sigma=0.5, bias_std=0.1),
    "c4_qwen32b_4x64k_mlp": Workload("c4_qwen32b_4x64k_mlp", L=64, B=4, T=65536, Dh=5120,
                                     scorer="mlp", keep_fraction=0.5, seed=4,
                                     bias_std=0.1),
    "c4_qwen32b_4x64k_linear": Workload("c4_qwen32b_4x64k_linear", L=64, B=4, T=65536,
                                        Dh=5120, scorer="linear", keep_fraction=0.5,
                                        seed=4),
    "c5_qwen8b_decode": Workload("c5_qwen8b_decode", L=36, B=64, T=1, Dh=4096,
                                 scorer="mlp", seed=7, bias_std=0.1),
}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_bf16(shape, g, device, scale: float = 1.0) -> torch.Tensor:
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if scale != 1.0:
        x = x * scale
    return x.to(torch.bfloat16)


def make_weights(wl: Workload, layer: int = 0, device="cpu") -> Dict[str, Optional[torch.Tensor]]:
    """Surrogate parameters ~ N(0, 1/fan_in), rounded to bf16, output-major."""
    g = _gen(device, wl.layer_seed(layer) * 7 + 1)
    out: Dict[str, Optional[torch.Tensor]] = {}
    if wl.scorer == "mlp":
        M = wl.M
        out["W1"] = _randn_bf16((M, wl.Dh), g, device, wl.Dh ** -0.5)
        out["W2"] = _randn_bf16((wl.H, M), g, device, M ** -0.5)
        if wl.bias_std > 0:
            out["b1"] = _randn_bf16((M,), g, device, wl.bias_std)
            out["b2"] = _randn_bf16((wl.H,), g, device, wl.bias_std)
        else:
            out["b1"] = None
            out["b2"] = None
    else:
        out["W1"] = _randn_bf16((wl.H, wl.Dh), g, device, wl.Dh ** -0.5)
        out["b1"] = _randn_bf16((wl.H,), g, device, wl.bias_std) if wl.bias_std > 0 else None
        out["W2"] = None
        out["b2"] = None
    return out


def make_hidden(wl: Workload, layer: int = 0, device="cpu",
                B: Optional[int] = None, T: Optional[int] = None) -> torch.Tensor:
    """Hidden states bf16 [B, T, Dh] ~ N(0,1), optionally times a per-token
    log-normal scale exp(sigma * z_t)."""
    B = wl.B if B is None else B
    T = wl.T if T is None else T
    g = _gen(device, wl.layer_seed(layer) * 7 + 2)
    if wl.token_scale_sigma > 0:
        x = torch.randn((B, T, wl.Dh), generator=g, device=device, dtype=torch.float32)
        z = torch.randn((B, T, 1), generator=g, device=device, dtype=torch.float32)
        x.mul_(torch.exp(wl.token_scale_sigma * z))
        return x.to(torch.bfloat16)
    return _randn_bf16((B, T, wl.Dh), g, device)


def make_kv(wl: Workload, layer: int = 0, device="cpu",
            B: Optional[int] = None, T: Optional[int] = None):
    """K and V bf16 [B, H, T, D] ~ N(0,1)."""
    B = wl.B if B is None else B
    T = wl.T if T is None else T
    g = _gen(device, wl.layer_seed(layer) * 7 + 3)
    K = _randn_bf16((B, wl.H, T, wl.D), g, device)
    V = _randn_bf16((B, wl.H, T, wl.D), g, device)
    return K, V


def make_attend_inputs(B: int, H: int, HQ: int, D: int, total_rows: int, window: int,
                       seed: int, device="cpu", q_gain: float = 1.0):
    """Inputs of one decode-attention step: q bf16 [B,HQ,D] ~ q_gain*N(0,1), row store
    K_rows/V_rows bf16 [total_rows,D] ~ N(0,1) and ring K/V bf16 [B,H,max(window,1),D]
    ~ N(0,1).  With scale = 1/sqrt(D) the logits are ~ N(0, q_gain^2): q_gain = 1 gives
    a spread softmax, larger gains a peaked one."""
    g = _gen(device, seed * 13 + 5)
    q = _randn_bf16((B, HQ, D), g, device, q_gain)
    K_rows = _randn_bf16((max(total_rows, 1), D), g, device)
    V_rows = _randn_bf16((max(total_rows, 1), D), g, device)
    K_ring = _randn_bf16((B, H, max(window, 1), D), g, device)
    V_ring = _randn_bf16((B, H, max(window, 1), D), g, device)
    return q, K_rows, V_rows, K_ring, V_ring


def make_exact_case(T: int, Dh: int, H: int, M: int, seed: int, device="cpu"):
    """Inputs on which every partial sum of the linear surrogate (M == 0) is an
    exactly representable small integer in fp32, in any summation order:
    hidden in {-4..4}, weights in {-1, 0, 1}, integer biases.  For M > 0 the
    same recipe is used for W1/W2 (then only the first projection is exact)."""
    g = _gen(device, seed)
    hid = torch.randint(-4, 5, (1, T, Dh), generator=g, device=device).to(torch.bfloat16)
    rows = M if M > 0 else H
    W1 = torch.randint(-1, 2, (rows, Dh), generator=g, device=device).to(torch.bfloat16)
    b1 = torch.randint(-3, 4, (rows,), generator=g, device=device).to(torch.bfloat16)
    out = {"W1": W1, "b1": b1, "W2": None, "b2": None}
    if M > 0:
        out["W2"] = torch.randint(-1, 2, (H, M), generator=g, device=device).to(torch.bfloat16)
        out["b2"] = torch.randint(-3, 4, (H,), generator=g, device=device).to(torch.bfloat16)
    return hid, out


def make_scores(B: int, H: int, T: int, seed: int, device="cpu",
                ties: bool = False) -> torch.Tensor:
    """fp32 scores for mask/compact tests that bypass the scorer.  With `ties`
    the values are drawn from a small grid so that many equal tau exactly."""
    g = _gen(device, seed)
    if ties:
        return (torch.randint(-8, 9, (B, H, T), generator=g, device=device)
                .to(torch.float32) * 0.25)
    return torch.randn((B, H, T), generator=g, device=device, dtype=torch.float32)


# ---- views for the CPU oracle (bit patterns and paper-orientation weights) ----
def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 numpy array of the same shape (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """Exact float64 copy of a bf16/fp32 tensor (None passes through)."""
    if t is None:
        return None
    return t.detach().cpu().to(torch.float64).numpy()


def oracle_weights(w: Dict[str, Optional[torch.Tensor]]) -> Dict[str, Optional[np.ndarray]]:
    """Storage layout [out, in] -> the paper's orientation [in, out], float64."""
    if w.get("W2") is not None:
        return {"W1": f64(w["W1"]).T, "b1": f64(w["b1"]),
                "W2": f64(w["W2"]).T, "b2": f64(w["b2"])}
    return {"W": f64(w["W1"]).T, "b": f64(w["b1"])}


def with_size(wl: Workload, **kw) -> Workload:
    return replace(wl, **kw)
