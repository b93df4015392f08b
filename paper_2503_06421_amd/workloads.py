"""Seeded synthetic workloads: tensor lists, host tensors and LoRA adapters.

This module only *describes* and *draws* inputs.  It contains none of the
method's arithmetic (no bf16 rounding, no merge), imports neither the HIP
binding nor the CPU oracle, and is the one piece both of them are fed from.

The shapes are those of the models the paper evaluates (Sec. 7.1: Llama-family
decoder stacks, with and without LoRA adapters); the paper's checkpoints and
adapters are replaced by seeded random tensors with the same shapes, host
dtypes and value distributions, which is sufficient because the path is
data-oblivious.  Each tensor has its own counter-based stream
Philox(key = [workload id, stream id]), so tensors can be drawn in any order
or in parallel and always come out identical.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

F32, F16, BF16 = 0, 1, 2                      # host dtype codes (same numbering as the C-ABI)
NP_DTYPE = {F32: np.float32, F16: np.float16, BF16: np.uint16}   # bf16 travels as raw uint16
ITEMSIZE = {F32: 4, F16: 2, BF16: 2}

_BLOCK = 1 << 22                               # elements drawn per temporary buffer


@dataclass(frozen=True)
class TensorSpec:
    name: str
    rows: int
    cols: int
    dist: str = "normal"                       # "normal": N(0, scale); "uniform": U[-scale, scale]
    scale: float = 0.02

    @property
    def numel(self) -> int:
        return self.rows * self.cols


@dataclass
class Workload:
    name: str
    wid: int                                   # workload id, first half of every Philox key
    host_dtype: int
    tensors: list                              # TensorSpec, in access (= slot) order
    lora_slots: list = field(default_factory=list)   # slot indices that carry LoRA
    rank: int = 0
    alpha: float = 0.0
    adapter_scale: float = 0.01                # A, B ~ N(0, adapter_scale)

    @property
    def shapes(self):
        return [(t.rows, t.cols) for t in self.tensors]

    @property
    def source_bytes(self) -> int:
        return sum(t.numel for t in self.tensors) * ITEMSIZE[self.host_dtype]

    @property
    def lora_w_elements(self) -> int:
        return sum(self.tensors[s].numel for s in self.lora_slots)


# ----------------------------------------------------------------------------
# drawing
# ----------------------------------------------------------------------------

def _rng(wid: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(wid), np.uint64(stream)]))


def _store(dst: np.ndarray, vals: np.ndarray, dtype: int) -> None:
    """Put float32 samples into a host tensor of the workload's dtype.  fp16 uses numpy's
    cast; bf16 host data keeps the upper half of the fp32 pattern (truncation), which is
    a choice of input data, not the method's rounding."""
    if dtype == BF16:
        np.copyto(dst, (vals.view(np.uint32) >> 16).astype(np.uint16))
    else:
        np.copyto(dst, vals, casting="same_kind")


def draw_into(dst: np.ndarray, wid: int, stream: int, dist: str, scale: float, dtype: int) -> None:
    """Fill the flat host array ``dst`` (dtype NP_DTYPE[dtype]) from stream (wid, stream)."""
    flat = dst.reshape(-1)
    g = _rng(wid, stream)
    tmp = np.empty(min(_BLOCK, flat.size), dtype=np.float32)
    for lo in range(0, flat.size, _BLOCK):
        hi = min(lo + _BLOCK, flat.size)
        t = tmp[: hi - lo]
        if dist == "normal":
            g.standard_normal(out=t, dtype=np.float32)
            t *= np.float32(scale)
        elif dist == "uniform":
            g.random(out=t, dtype=np.float32)
            t *= np.float32(2.0 * scale)
            t -= np.float32(scale)
        else:
            raise ValueError(dist)
        _store(flat[lo:hi], t, dtype)


def draw_tensor(wl: Workload, idx: int, out: np.ndarray | None = None) -> np.ndarray:
    """Host tensor ``idx`` of the workload, shape (rows, cols), dtype NP_DTYPE[wl.host_dtype]."""
    t = wl.tensors[idx]
    if out is None:
        out = np.empty((t.rows, t.cols), dtype=NP_DTYPE[wl.host_dtype])
    assert out.size == t.numel
    draw_into(out, wl.wid, idx, t.dist, t.scale, wl.host_dtype)
    return out


def draw_all(wl: Workload, outs: list, threads: int = 8) -> None:
    """Draw every tensor of the workload into the given host arrays, in parallel."""
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(lambda i: draw_tensor(wl, i, outs[i]), range(len(wl.tensors))))


def draw_adapter(wl: Workload, adapter_id: int, slot: int, rank: int | None = None):
    """LoRA factors for one target: A (r, in), B (out, r), host dtype of the workload.
    Stream ids start at 2**32 so they never collide with tensor streams."""
    t = wl.tensors[slot]
    r = wl.rank if rank is None else rank
    base = (1 << 32) + (adapter_id << 20) + 2 * slot
    A = np.empty((r, t.cols), dtype=NP_DTYPE[wl.host_dtype])
    B = np.empty((t.rows, r), dtype=NP_DTYPE[wl.host_dtype])
    if r:
        draw_into(A, wl.wid, base, "normal", wl.adapter_scale, wl.host_dtype)
        draw_into(B, wl.wid, base + 1, "normal", wl.adapter_scale, wl.host_dtype)
    return A, B


# ----------------------------------------------------------------------------
# the configurations
# ----------------------------------------------------------------------------

def single_linear(n: int = 4096, rank: int = 8, alpha: float = 16.0) -> Workload:
    """One linear layer, fp32 host U[-0.02, 0.02]; one adapter attached, then swapped for
    a second one (adapter ids 0 and 1)."""
    return Workload(name=f"single_linear_{n}", wid=1, host_dtype=F32,
                    tensors=[TensorSpec("w", n, n, "uniform", 0.02)],
                    lora_slots=[0], rank=rank, alpha=alpha)


_PROJ = ("q", "k", "v", "o", "gate", "up", "down")


def llama_stack(name: str, wid: int, layers: int, hidden: int, ffn: int, vocab: int,
                host_dtype: int, lora_on=("q", "v"), rank: int = 16, alpha: float = 32.0,
                kv_dim: int | None = None, with_norms: bool = False) -> Workload:
    """Decoder-only stack in access order: embed, per layer q,k,v,o,gate,up,down, lm_head.
    ``kv_dim`` < hidden gives grouped-query k/v projections.  ``with_norms`` adds the small
    RMSNorm vectors (two per layer and a final one), which exercises chunk coalescing."""
    kv = hidden if kv_dim is None else kv_dim
    shape = {"q": (hidden, hidden), "k": (kv, hidden), "v": (kv, hidden), "o": (hidden, hidden),
             "gate": (ffn, hidden), "up": (ffn, hidden), "down": (hidden, ffn)}
    tensors = [TensorSpec("embed", vocab, hidden)]
    lora_slots = []
    for l in range(layers):
        if with_norms:
            tensors.append(TensorSpec(f"l{l}.attn_norm", 1, hidden))
        for p in _PROJ:
            if with_norms and p == "gate":
                tensors.append(TensorSpec(f"l{l}.ffn_norm", 1, hidden))
            if p in lora_on:
                lora_slots.append(len(tensors))
            tensors.append(TensorSpec(f"l{l}.{p}", *shape[p]))
    if with_norms:
        tensors.append(TensorSpec("final_norm", 1, hidden))
    tensors.append(TensorSpec("lm_head", vocab, hidden))
    return Workload(name=name, wid=wid, host_dtype=host_dtype, tensors=tensors,
                    lora_slots=lora_slots, rank=rank, alpha=alpha)


def llama2_7b(layers: int = 32, **kw) -> Workload:
    return llama_stack("llama2_7b_shaped", 2, layers, 4096, 11008, 32000, F16,
                       lora_on=("q", "v"), rank=16, alpha=32.0, **kw)


def llama2_13b(layers: int = 40, **kw) -> Workload:
    return llama_stack("llama2_13b_shaped", 3, layers, 5120, 13824, 32000, F16,
                       lora_on=_PROJ, rank=64, alpha=128.0, **kw)


def llama3_70b(layers: int = 80, **kw) -> Workload:
    return llama_stack("llama3_70b_shaped", 5, layers, 8192, 28672, 128256, BF16,
                       lora_on=_PROJ, rank=16, alpha=32.0, kv_dim=1024, **kw)


def llama70b_tp8_shard_many_tensors(layers: int = 80) -> Workload:
    """One tensor-parallel rank's share (1/8) of a Llama2-70B-shaped stack as a framework would
    initialise it: 15 tensors per layer -- the seven projection shards, two norm vectors and six
    tiny per-layer buffers -- i.e. 1,200 tensors for 80 layers, the count the paper quotes for
    Llama2-70B on 8 GPUs in its tensor-merging experiment (Sec. 7.4)."""
    h, ffn, kv, tp = 8192, 28672, 1024, 8
    tensors = [TensorSpec("embed_shard", 32000 // tp, h)]
    for l in range(layers):
        tensors += [TensorSpec(f"l{l}.attn_norm", 1, h), TensorSpec(f"l{l}.q", h // tp, h),
                    TensorSpec(f"l{l}.k", kv // tp, h), TensorSpec(f"l{l}.v", kv // tp, h),
                    TensorSpec(f"l{l}.o", h, h // tp), TensorSpec(f"l{l}.ffn_norm", 1, h),
                    TensorSpec(f"l{l}.gate", ffn // tp, h), TensorSpec(f"l{l}.up", ffn // tp, h),
                    TensorSpec(f"l{l}.down", h, ffn // tp)]
        tensors += [TensorSpec(f"l{l}.buf{b}", 1, 128) for b in range(6)]
    tensors.append(TensorSpec("lm_head_shard", 32000 // tp, h))
    return Workload(name="llama70b_tp8_shard_1200_tensors", wid=6, host_dtype=F16, tensors=tensors)


def tiny_stack(host_dtype: int = F16, layers: int = 2, hidden: int = 192, ffn: int = 520,
               vocab: int = 1000, kv_dim: int | None = None, lora_on=("q", "v"), rank: int = 16,
               alpha: float = 32.0, with_norms: bool = False, wid: int = 9) -> Workload:
    """Same structure at a size the CPU oracle finishes in well under a second."""
    return llama_stack("tiny_stack", wid, layers, hidden, ffn, vocab, host_dtype, lora_on=lora_on,
                       rank=rank, alpha=alpha, kv_dim=kv_dim, with_norms=with_norms)


# ----------------------------------------------------------------------------
# multi-tenant adapter churn
# ----------------------------------------------------------------------------

@dataclass
class Churn:
    base: Workload                              # lora_slots = q,k,v,o of every layer
    ranks: list                                 # rank of each pooled adapter
    alphas: list                                # alpha = 2 * rank
    schedule: list                              # adapter index per invocation


def adapter_churn(base: Workload | None = None, pool: int = 32, steps: int = 200,
                  zipf_s: float = 1.1, seed: int = 4) -> Churn:
    """Pool of adapters with rank ~ U{8,16,32,64}; invocations pick adapter i (1-based
    popularity rank) with probability proportional to i**-s."""
    if base is None:
        base = llama_stack("llama2_7b_shaped_churn", 4, 32, 4096, 11008, 32000, F16,
                           lora_on=("q", "k", "v", "o"))
    g = _rng(seed, 0)
    ranks = [int(x) for x in g.choice([8, 16, 32, 64], size=pool)]
    p = 1.0 / np.arange(1, pool + 1, dtype=np.float64) ** zipf_s
    p /= p.sum()
    schedule = [int(x) for x in g.choice(pool, size=steps, p=p)]
    return Churn(base=base, ranks=ranks, alphas=[2.0 * r for r in ranks], schedule=schedule)
