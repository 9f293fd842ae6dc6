"""Seeded synthetic attention blocks (weights + calibration activations).

Input generation only: nothing of the quantization method is computed here.  The same
tensors are handed to the HIP library and (as host copies) to whatever checks it.
The distributions stand in for a real calibration set pushed through real weights:
Gaussian activations with a few outlier channels, Gaussian weights of std 0.02.
"""
from __future__ import annotations

import dataclasses
import math

import torch


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    name: str
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_seqs: int
    seq_len: int
    dtype: str = "bf16"              # storage type of X and W: "fp32" | "bf16"
    outlier: str = "student_t"       # "scale": fixed x20 channels | "student_t": t_3 x c_out channels
    n_outlier: int = 0               # 0 -> 1% of d_model
    outlier_scale: float = 20.0
    noise: float = 0.05              # X = X_fp + noise * rms(X_fp) * N(0,1)
    rotate: bool = False             # config 5: the block comes with random signs; X_fp <- X_fp diag(signs) H / sqrt(d) is a step
                                     # of the method (the library's tboa_hadamard_rotate) applied by the pipeline
    act_bits: int = 0                # config 5: X is the per-token fake-quant of X_fp (done by the library)
    bits: int = 2
    block: int = 32
    group: int = 0
    d_ff: int = 0                    # width of the gated MLP of the same transformer block (make_mlp)

    @property
    def d_q(self):
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self):
        return self.n_kv_heads * self.head_dim

    @property
    def n_tokens(self):
        return self.n_seqs * self.seq_len


CONFIGS = {
    "tiny": BlockConfig("tiny", 256, 4, 4, 64, 8, 128, dtype="fp32", outlier="scale", n_outlier=4,
                        bits=2, block=4, d_ff=512),
    "llama2-7b": BlockConfig("llama2-7b", 4096, 32, 32, 128, 128, 2048, bits=2, block=32, d_ff=11008),
    "llama2-13b": BlockConfig("llama2-13b", 5120, 40, 40, 128, 128, 2048, bits=3, block=32, group=128, d_ff=13824),
    "llama2-70b": BlockConfig("llama2-70b", 8192, 64, 8, 128, 128, 2048, bits=2, block=64, d_ff=28672),
    "llama2-7b-w4a4": BlockConfig("llama2-7b-w4a4", 4096, 32, 32, 128, 128, 2048, rotate=True, act_bits=4,
                                  bits=4, block=32, d_ff=11008),
}


def scaled(cfg: BlockConfig, **kw) -> BlockConfig:
    """A config of the same family with some fields replaced (smaller test cases)."""
    return dataclasses.replace(cfg, **kw)


def _torch_dtype(name):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def make_block(cfg: BlockConfig, seed: int = 0, device="cpu"):
    """Weights and calibration activations of one attention block.

    Returns dict(Wq [Hq*dh,d], Wk, Wv [Hkv*dh,d], Wo [d,Hq*dh], X_fp [S,L,d], X [S,L,d] or None, signs [d] or None).
    X is None when cfg.act_bits > 0: then the quantized-path input is the fake-quantized X_fp,
    which is a step of the method and is left to the library.  signs (+-1, fp32) is given when
    cfg.rotate: X_fp is then the activation BEFORE the randomised Hadamard rotation."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(1000003 * seed + 17)
    dt = _torch_dtype(cfg.dtype)
    d = cfg.d_model

    def normal(*shape, std=1.0):
        return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32) * std

    out = {}
    out["Wq"] = normal(cfg.d_q, d, std=0.02).to(dt)
    out["Wk"] = normal(cfg.d_kv, d, std=0.02).to(dt)
    out["Wv"] = normal(cfg.d_kv, d, std=0.02).to(dt)
    out["Wo"] = normal(d, cfg.d_q, std=0.02).to(dt)

    n_out = cfg.n_outlier or max(1, round(0.01 * d))
    perm = torch.randperm(d, generator=g, device=dev)
    ch = perm[:n_out]
    signs = (torch.randint(0, 2, (d,), generator=g, device=dev).float() * 2 - 1) if cfg.rotate else None

    X_fp = torch.empty(cfg.n_seqs, cfg.seq_len, d, device=dev, dtype=dt)
    X = None if cfg.act_bits else torch.empty_like(X_fp)
    for s in range(cfg.n_seqs):                       # per sequence: bounds the fp32 temporaries
        x = normal(cfg.seq_len, d)
        if cfg.outlier == "scale":
            x[:, ch] *= cfg.outlier_scale
        else:                                         # Student-t, nu = 3: N(0,1) / sqrt(chi2_3 / 3)
            num = normal(cfg.seq_len, n_out)
            den = (normal(cfg.seq_len, n_out, 3) ** 2).sum(-1).div(3.0).sqrt()
            x[:, ch] = cfg.outlier_scale * num / den
        X_fp[s] = x.to(dt)
        if X is not None:
            rms = x.pow(2).mean().sqrt()
            X[s] = (x + cfg.noise * rms * normal(cfg.seq_len, d)).to(dt)
    out["X_fp"] = X_fp
    out["X"] = X
    out["signs"] = signs
    return out


def make_mlp(cfg: BlockConfig, seed: int = 0, device="cpu"):
    """Weights and calibration inputs of the gated MLP of the block: Wg, Wu [d_ff, d], Wd [d, d_ff] ~ N(0, 0.02^2),
    M_fp [S, L, d] with the same activation recipe as make_block (Gaussian, outlier channels), M = M_fp + noise."""
    sub = make_block(dataclasses.replace(cfg, rotate=False, act_bits=0), seed=seed + 7919, device=device)
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(1000003 * seed + 31)
    dt = _torch_dtype(cfg.dtype)
    w = lambda *shape: (torch.randn(*shape, generator=g, device=dev, dtype=torch.float32) * 0.02).to(dt)
    return {"Wg": w(cfg.d_ff, cfg.d_model), "Wu": w(cfg.d_ff, cfg.d_model), "Wd": w(cfg.d_model, cfg.d_ff),
            "M_fp": sub["X_fp"], "M": sub["X"]}


def correlated_mix(d, rank=8, strength=0.3, seed=0, device="cpu"):
    """M = I + strength * low-rank: X <- X M gives correlated channels (a harder H_in)."""
    g = torch.Generator(device=torch.device(device))
    g.manual_seed(7919 * seed + 5)
    a = torch.randn(d, rank, generator=g, device=device)
    b = torch.randn(rank, d, generator=g, device=device)
    return torch.eye(d, device=device) + strength * (a @ b) / math.sqrt(rank)


def apply_mix(blk, M):
    """X_fp <- X_fp M and X <- X M in place, one sequence at a time (fp32 product, rounded back to the block's dtype)."""
    for key in ("X_fp", "X"):
        t = blk.get(key)
        if t is None:
            continue
        for s in range(t.shape[0]):
            t[s] = (t[s].float() @ M).to(t.dtype)
    return blk
