"""Seeded synthetic inputs for the MoE-layer hot path.

This module only draws random numbers and rounds them to the storage type.  It
holds none of the method's arithmetic (no routing, no expert FFN, no combine)
and is the one piece that both the CPU oracle's tests and the GPU path's tests
and benchmark may share: each side receives the very same arrays.

Recipe.  Every tensor is drawn from its own NumPy ``Generator(PCG64(sub_seed))``
with ``sub_seed = seed*10**6 + layer*10**3 + tensor_id`` where ``tensor_id`` is
0 for the activations X, 1 for the gate matrix Wg and ``2 + 3*e + {0,1,2}`` for
W1, W3, W2 of expert ``e`` (shared experts follow the routed ones: e = E..E+S-1).
Values are float32 normal draws, scaled, then (for bf16 workloads) rounded to
bfloat16 with round-to-nearest-even; the rounded values are what both sides see.

Shapes follow the paper's evaluated model family (Section 9.1: Mixtral-8x7B and
Mixtral-8x22B, prompt 512 tokens, batch sizes 4-64) and the skewed expert
popularity it reports (Section 3.3); the paper's datasets and trained weights are
not available, these inputs stand in for them.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np
import torch

TID_X = 0
TID_WG = 1


def tid_expert(e: int, which: int) -> int:
    """tensor_id of W1 (which=0), W3 (1) or W2 (2) of expert ``e``."""
    return 2 + 3 * e + which


@dataclass(frozen=True)
class Workload:
    """One MoE-layer workload: shapes, batch structure and distributions."""
    name: str
    dtype: str            # "f32" or "bf16"
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    n_shared: int = 0
    n_layers: int = 1
    batch_tokens: tuple = (16, 16, 16, 16)   # tokens per batch of the batch group
    streamed: bool = False
    window_layers: int = 0
    zipf_s: float = 0.0                      # >0: skewed router targets
    corr: float = 0.0                        # layer-to-layer routing correlation
    seed: int = 0
    token_seed: int = -1      # >= 0: tokens (activations, routing noise) drawn from this seed, weights from `seed`
    w_std: float = 0.02

    @property
    def n_tokens(self) -> int:
        return int(sum(self.batch_tokens))

    @property
    def n_batches(self) -> int:
        return len(self.batch_tokens)

    @property
    def batch_offsets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.batch_tokens)]).astype(np.int32)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def expert_bytes(self) -> int:
        return 3 * self.d_model * self.d_ff * self.elt_bytes


# The five workloads the build is measured and checked on.
WORKLOADS: Dict[str, Workload] = {
    "tiny_f32": Workload("tiny_f32", "f32", 256, 512, 8, 2, batch_tokens=(16,) * 4),
    "mixtral8x7b_decode": Workload("mixtral8x7b_decode", "bf16", 4096, 14336, 8, 2,
                                   batch_tokens=(64,) * 8),
    "mixtral8x7b_prefill": Workload("mixtral8x7b_prefill", "bf16", 4096, 14336, 8, 2,
                                    batch_tokens=(8 * 512,) * 4),
    "mixtral8x22b_stream": Workload("mixtral8x22b_stream", "bf16", 6144, 16384, 8, 2,
                                    n_layers=8, batch_tokens=(32,) * 16, streamed=True,
                                    window_layers=2),
    "finegrained_stream": Workload("finegrained_stream", "bf16", 2048, 1408, 64, 6,
                                   n_shared=2, n_layers=12, batch_tokens=(16,) * 32,
                                   streamed=True, window_layers=2, zipf_s=1.1, corr=0.6),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of ``w`` with some fields replaced (smaller shapes for tests)."""
    return replace(w, **kw)


def _sub_seed(seed: int, layer: int, tid: int) -> int:
    return seed * 10**6 + layer * 10**3 + tid


def _normal(seed: int, layer: int, tid: int, shape, std: float) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(_sub_seed(seed, layer, tid)))
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def to_storage(a: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 array -> CPU torch tensor in the workload's storage type (RNE for bf16)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t if dtype == "f32" else t.to(torch.bfloat16)


def as_f32(t: torch.Tensor) -> np.ndarray:
    """Exact float32 view of a stored tensor (bf16 widens exactly)."""
    return t.detach().cpu().to(torch.float32).numpy()


def as_raw(t: torch.Tensor) -> np.ndarray:
    """Raw storage as NumPy: float32 array, or uint16 bit patterns for bf16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


@dataclass
class LayerData:
    """All tensors of one MoE layer, as CPU torch tensors in storage dtype."""
    x: torch.Tensor                       # [N, d]
    wg: torch.Tensor                      # [E, d]
    w1: List[torch.Tensor] = field(default_factory=list)   # E+S tensors [f, d]
    w3: List[torch.Tensor] = field(default_factory=list)   # E+S tensors [f, d]
    w2: List[torch.Tensor] = field(default_factory=list)   # E+S tensors [d, f]


def gen_gate(w: Workload, layer: int = 0) -> torch.Tensor:
    return to_storage(_normal(w.seed, layer, TID_WG, (w.n_experts, w.d_model), w.w_std), w.dtype)


def gen_expert(w: Workload, layer: int, e: int):
    """(W1 [f,d], W3 [f,d], W2 [d,f]) of expert e (e >= E: shared expert)."""
    w1 = to_storage(_normal(w.seed, layer, tid_expert(e, 0), (w.d_ff, w.d_model), w.w_std), w.dtype)
    w3 = to_storage(_normal(w.seed, layer, tid_expert(e, 1), (w.d_ff, w.d_model), w.w_std), w.dtype)
    w2 = to_storage(_normal(w.seed, layer, tid_expert(e, 2), (w.d_model, w.d_ff), w.w_std), w.dtype)
    return w1, w3, w2


def gen_expert_q4(w: Workload, layer: int, e: int, group: int = 64):
    """A 4-bit group-quantised expert as random inputs: for each of W1, W3 ([f, d]) and W2
    ([d, f]) a triple (codes uint8 [rows, cols/2] with the even column in the low nibble,
    scales bf16 [rows, cols/group], zero points bf16 [rows, cols/group]).  Codes are uniform on
    0..15, zero points uniform on [6, 9], scales uniform on [0.5, 1.5] x w_std / 4.6, so that the
    weights s * (code - z) have a standard deviation near w_std."""
    out = []
    for j, (rows, cols) in enumerate(((w.d_ff, w.d_model), (w.d_ff, w.d_model), (w.d_model, w.d_ff))):
        g = np.random.Generator(np.random.PCG64(_sub_seed(w.seed, layer, 500 + tid_expert(e, j))))
        codes = g.integers(0, 256, size=(rows, cols // 2), dtype=np.uint8)   # two uniform nibbles
        s = (g.uniform(0.5, 1.5, size=(rows, cols // group)) * (w.w_std / 4.6)).astype(np.float32)
        z = g.uniform(6.0, 9.0, size=(rows, cols // group)).astype(np.float32)
        out.append((torch.from_numpy(codes), torch.from_numpy(s).to(torch.bfloat16),
                    torch.from_numpy(z).to(torch.bfloat16)))
    return tuple(out)


def gen_x_gaussian(w: Workload, layer: int = 0) -> torch.Tensor:
    return to_storage(_normal(w.token_seed if w.token_seed >= 0 else w.seed, layer, TID_X,
                              (w.n_tokens, w.d_model), 1.0), w.dtype)


def zipf_target_logits(w: Workload, layer: int, prev_noise: Optional[np.ndarray]):
    """Target router logits with Zipf-skewed expert popularity and layer correlation.

    Rank r (1..E) gets log-popularity -s*ln r; a seeded permutation maps ranks to
    experts per layer.  Per token a Gumbel(0,1) noise vector is added (so the
    top-k of the targets is a Zipf sample without replacement).  With probability
    ``corr`` a token re-uses its noise vector of the previous layer, which keeps
    its rank set and so ties its expert set to the previous layer's.
    Returns (targets [N,E] float64, noise [N,E] float64).
    """
    E, N = w.n_experts, w.n_tokens
    g = np.random.Generator(np.random.PCG64(_sub_seed(w.seed, layer, 900)))
    rank_to_expert = g.permutation(E)
    if w.token_seed >= 0:  # another batch group for the same model: same popularity map, new tokens
        g = np.random.Generator(np.random.PCG64(_sub_seed(w.token_seed, layer, 901)))
    u = g.random((N, E))
    noise = -np.log(-np.log(np.clip(u, 1e-12, 1.0 - 1e-12)))
    if prev_noise is not None and w.corr > 0:
        keep = g.random(N) < w.corr
        noise[keep] = prev_noise[keep]
    base = -w.zipf_s * np.log(np.arange(1, E + 1, dtype=np.float64))
    by_rank = base[None, :] + noise
    targets = np.empty_like(by_rank)
    targets[:, rank_to_expert] = by_rank
    return targets, noise


def gen_x_for_targets(w: Workload, layer: int, wg: torch.Tensor, targets: np.ndarray) -> torch.Tensor:
    """Activations whose gate logits come out as ``targets`` (up to storage rounding).

    x = z - Wg^T (Wg Wg^T)^-1 (Wg z - target): the minimum-norm correction of a
    Gaussian draw z onto the affine set {x : Wg x = target}.
    """
    z = _normal(w.token_seed if w.token_seed >= 0 else w.seed, layer, TID_X,
                (w.n_tokens, w.d_model), 1.0).astype(np.float64)
    g = as_f32(wg).astype(np.float64)
    resid = z @ g.T - targets                       # [N, E]
    corr = np.linalg.solve(g @ g.T, resid.T).T @ g  # [N, d]
    return to_storage((z - corr).astype(np.float32), w.dtype)


def gen_layer(w: Workload, layer: int = 0, prev_noise: Optional[np.ndarray] = None,
              threads: int = 8, with_experts: bool = True):
    """Generate one layer.  Returns (LayerData, noise) — noise feeds the next layer."""
    wg = gen_gate(w, layer)
    noise = None
    if w.zipf_s > 0:
        targets, noise = zipf_target_logits(w, layer, prev_noise)
        x = gen_x_for_targets(w, layer, wg, targets)
    else:
        x = gen_x_gaussian(w, layer)
    data = LayerData(x=x, wg=wg)
    if with_experts:
        n_all = w.n_experts + w.n_shared
        with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
            trip = list(pool.map(lambda e: gen_expert(w, layer, e), range(n_all)))
        for w1, w3, w2 in trip:
            data.w1.append(w1)
            data.w3.append(w3)
            data.w2.append(w2)
    return data, noise


# ---- attention (non-expert) layer of the pipeline --------------------------------------------

@dataclass(frozen=True)
class AttnWorkload:
    """One decoding step of the attention layer over a batch group (Algorithm 1, non-expert
    branch): every batch brings its hidden state and its key-value cache."""
    name: str
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch_seqs: tuple          # sequences per batch of the group
    batch_pos: tuple           # cached positions per batch (all sequences of a batch alike)
    max_len: int               # capacity of the caches, in positions
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-5
    kv_on_host: bool = True    # caches in pinned host memory, streamed batch by batch
    seed: int = 0
    w_std: float = 0.02

    @property
    def n_batches(self) -> int:
        return len(self.batch_seqs)

    @property
    def n_tokens(self) -> int:
        return int(sum(self.batch_seqs))

    def kv_bytes(self, b: int) -> int:
        """Bytes of valid K and V of batch b before the step."""
        return 2 * self.batch_seqs[b] * self.n_kv_heads * self.batch_pos[b] * self.head_dim * 2


# Mixtral-8x7B attention shape; 8 batches x 64 sequences after a 512-token prompt (Section 9.1).
ATTN_WORKLOADS: Dict[str, AttnWorkload] = {
    "attn_tiny": AttnWorkload("attn_tiny", 256, 8, 2, 32, (5, 3, 8), (17, 0, 40), 48, kv_on_host=True),
    "attn_mixtral8x7b_decode": AttnWorkload("attn_mixtral8x7b_decode", 4096, 32, 8, 128, (64,) * 8,
                                            (512,) * 8, 576, kv_on_host=True),
    "attn_mixtral8x7b_decode_hbm": AttnWorkload("attn_mixtral8x7b_decode_hbm", 4096, 32, 8, 128,
                                                (64,) * 8, (512,) * 8, 576, kv_on_host=False),
}

_TID_ATTN = {"norm": 700, "wq": 701, "wk": 702, "wv": 703, "wo": 704}


def gen_attn_weights(w: AttnWorkload, layer: int = 0) -> Dict[str, torch.Tensor]:
    """bf16 tensors: norm [d] ~ 1 + N(0, 0.1), wq [Hq*hd, d], wk / wv [Hkv*hd, d], wo [d, Hq*hd]."""
    dq, dkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    out = {"norm": to_storage(1.0 + _normal(w.seed, layer, _TID_ATTN["norm"], (w.d_model,), 0.1), "bf16")}
    for name, shape in (("wq", (dq, w.d_model)), ("wk", (dkv, w.d_model)), ("wv", (dkv, w.d_model)),
                        ("wo", (w.d_model, dq))):
        out[name] = to_storage(_normal(w.seed, layer, _TID_ATTN[name], shape, w.w_std), "bf16")
    return out


def gen_attn_hidden(w: AttnWorkload, layer: int, b: int) -> torch.Tensor:
    """Hidden state of batch b entering the layer: bf16 [n_seq, d], N(0, 1)."""
    return to_storage(_normal(w.seed, layer, 710 + b, (w.batch_seqs[b], w.d_model), 1.0), "bf16")


def gen_kv_cache(w: AttnWorkload, layer: int, b: int, pin: bool = False):
    """(K, V) caches of batch b: bf16 [n_seq, Hkv, max_len, hd]; the first batch_pos[b] positions
    hold N(0, 1) draws, the rest zeros."""
    shape = (w.batch_seqs[b], w.n_kv_heads, w.max_len, w.head_dim)
    out = []
    for j in range(2):
        t = torch.zeros(shape, dtype=torch.bfloat16, pin_memory=pin)
        if w.batch_pos[b] > 0:
            g = np.random.Generator(np.random.PCG64(_sub_seed(w.seed, layer, 800 + 2 * b + j)))
            a = g.standard_normal((shape[0], shape[1], w.batch_pos[b], shape[3]), dtype=np.float32)
            t[:, :, :w.batch_pos[b], :] = torch.from_numpy(a).to(torch.bfloat16)
        out.append(t)
    return out[0], out[1]
