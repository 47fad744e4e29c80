"""Seeded synthetic inputs for the Tier-2 attention step.

This module only *draws data*: context lengths, slot permutations and the
16-bit tensors.  It holds none of the method's arithmetic and imports neither
the HIP binding nor the CPU oracle; tests and the benchmark hand the very same
bytes to both sides.

The five workloads stand in for the paper's evaluation traffic (Section 5.1:
Llama-2 models in FP16 serving prompts whose prompt/completion lengths follow a
public chat data set).  That data set is not used here; its only role for the
attention step -- a batch whose sequences have different context lengths -- is
kept through the length distributions below.
"""
from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f16" | "bf16"
    lengths: tuple        # ("const", L) | ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi)
    seed: int
    outlier_key_frac: float = 0.0   # fraction of cached key rows multiplied by 8
    note: str = ""


WORKLOADS = {
    "c1": Workload("c1", 4, 8, 8, 128, "f16", ("const", 512), 1001,
                   note="tiny MHA decode step"),
    "c2": Workload("c2", 64, 32, 32, 128, "f16", ("uniform", 512, 2048), 1002,
                   note="Llama-2-7B-shaped MHA layer"),
    "c3": Workload("c3", 256, 32, 8, 128, "bf16", ("uniform", 1024, 4096), 1003,
                   note="Llama-3-8B-shaped GQA layer"),
    "c4": Workload("c4", 1024, 64, 8, 128, "bf16", ("uniform", 256, 4096), 1004,
                   note="Llama-3-70B-shaped GQA layer, large offline batch"),
    "c5": Workload("c5", 32, 64, 8, 128, "bf16", ("lognormal", 16384, 0.5, 4096, 32768), 1005,
                   outlier_key_frac=0.01, note="long-sequence GQA with 1% of key rows x8"),
}

TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_CODE = {"f16": 0, "bf16": 1}
ELEM_BYTES = 2


def draw_lengths(w: Workload) -> np.ndarray:
    """Rows cached per sequence *before* the step (the new row lands at this index)."""
    rng = np.random.default_rng(w.seed)
    kind = w.lengths[0]
    if kind == "const":
        L = np.full(w.batch, w.lengths[1], dtype=np.int64)
    elif kind == "uniform":
        L = rng.integers(w.lengths[1], w.lengths[2], size=w.batch, endpoint=True)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = w.lengths
        z = rng.standard_normal(w.batch)
        L = np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi).astype(np.int64)
    else:
        raise ValueError(kind)
    return L.astype(np.int32)


def draw_slots(w: Workload, n_slots: int) -> np.ndarray:
    """A seeded assignment of distinct slots to the batch (never the identity for B > 1)."""
    rng = np.random.default_rng(w.seed + 7919)
    return rng.permutation(n_slots)[: w.batch].astype(np.int32)


def cache_shape_and_strides(n_slots, n_kv_heads, capacity, head_dim, layout="head_major",
                            block_rows=0):
    """Tensor shape of one cache and its (slot, head, row) strides in elements."""
    if layout == "head_major":      # [slot][kv head][row][d]
        shape = (n_slots, n_kv_heads, capacity, head_dim)
        strides = (n_kv_heads * capacity * head_dim, capacity * head_dim, head_dim)
    elif layout == "token_major":   # [slot][row][kv head][d]
        shape = (n_slots, capacity, n_kv_heads, head_dim)
        strides = (capacity * n_kv_heads * head_dim, head_dim, n_kv_heads * head_dim)
    elif layout == "head_blocked":  # [slot][block][kv head][row in block][d]
        assert block_rows > 0 and capacity % block_rows == 0
        shape = (n_slots, capacity // block_rows, n_kv_heads, block_rows, head_dim)
        strides = (capacity * n_kv_heads * head_dim, block_rows * head_dim, head_dim)
    else:
        raise ValueError(layout)
    return shape, strides


def _randn16(shape, dtype, gen, device, chunk_elems=1 << 28):
    """N(0,1) rounded to a 16-bit dtype, drawn in bounded fp32 pieces along dim 0."""
    out = torch.empty(shape, dtype=dtype, device=device)
    per0 = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    step = max(1, chunk_elems // max(per0, 1))
    for i in range(0, shape[0], step):
        j = min(shape[0], i + step)
        out[i:j] = torch.randn((j - i,) + tuple(shape[1:]), generator=gen, device=device,
                               dtype=torch.float32).to(dtype)
    return out


def make_inputs(w: Workload, device="cpu", lengths=None, n_slots=None, capacity=None,
                layout="head_major", poison=True, slots=None, block_rows=0):
    """Build one step's inputs on `device`.

    Returns a dict of torch tensors plus the scalar geometry:
      q [B,H,d], k_new/v_new [B,H_kv,d], k_cache/v_cache (layout-dependent),
      slot_id, pos, ctx_len (int32 [B]; ctx_len = pos + 1), strides, capacity.
    Rows at index >= pos[b] of a sequence's slot, and every row of unused
    slots, hold a NaN bit pattern when `poison` is set, so that a read outside
    the problem shows up in the output.

    layout "head_blocked" stores blocks of `block_rows` rows, [slot][block][kv head][row][d]; the
    capacity is rounded up to whole blocks and the dict carries "block" = (block_rows, elements
    between a head's consecutive blocks).

    `slots` overrides the seeded slot assignment; entries may then share a slot
    (the tokens of a prefill chunk: same slot, consecutive `lengths`), in which
    case the slot's cached rows end at the smallest of their lengths.
    """
    dt = TORCH_DTYPE[w.dtype]
    L = draw_lengths(w) if lengths is None else np.asarray(lengths, dtype=np.int32)
    assert L.shape == (w.batch,)
    n_slots = w.batch if n_slots is None else n_slots
    capacity = int(L.max()) + 1 if capacity is None else capacity
    assert capacity >= int(L.max()) + 1
    if layout == "head_blocked":
        capacity = -(-capacity // block_rows) * block_rows
    if slots is None:
        assert n_slots >= w.batch
        slot = draw_slots(w, n_slots)
    else:
        slot = np.asarray(slots, dtype=np.int32)
        assert slot.shape == (w.batch,) and slot.min() >= 0 and slot.max() < n_slots
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed)
    B, H, Hkv, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    shape, strides = cache_shape_and_strides(n_slots, Hkv, capacity, d, layout, block_rows)

    q = _randn16((B, H, d), dt, gen, device)
    k_new = _randn16((B, Hkv, d), dt, gen, device)
    v_new = _randn16((B, Hkv, d), dt, gen, device)
    k_cache = _randn16(shape, dt, gen, device)
    v_cache = _randn16(shape, dt, gen, device)

    rows_np = np.full(n_slots, np.iinfo(np.int64).max, dtype=np.int64)
    np.minimum.at(rows_np, slot.astype(np.int64), L.astype(np.int64))
    rows_np[rows_np == np.iinfo(np.int64).max] = 0
    rows_of_slot = torch.from_numpy(rows_np).to(device)
    row_idx = torch.arange(capacity, device=device)
    live = row_idx[None, :] < rows_of_slot[:, None]                 # [slot, row]
    if layout == "head_major":
        live4 = live[:, None, :, None]
    elif layout == "head_blocked":
        live4 = live.reshape(n_slots, capacity // block_rows, 1, block_rows, 1)
    else:
        live4 = live[:, :, None, None]

    if w.outlier_key_frac > 0.0:
        # i.i.d. Bernoulli per (slot, kv head, row); the whole key row is scaled by 8,
        # which is exact in both 16-bit formats for N(0,1) magnitudes.
        mshape = shape[:-1]
        hit = torch.rand(mshape, generator=gen, device=device) < w.outlier_key_frac
        k_cache = torch.where(hit[..., None], k_cache * 8, k_cache)

    if poison:
        nan = torch.tensor(float("nan"), dtype=dt, device=device)
        k_cache = torch.where(live4, k_cache, nan)
        v_cache = torch.where(live4, v_cache, nan)

    pos = torch.from_numpy(L.copy()).to(device)
    return {
        "workload": w, "q": q, "k_new": k_new, "v_new": v_new,
        "k_cache": k_cache.contiguous(), "v_cache": v_cache.contiguous(),
        "slot_id": torch.from_numpy(slot.copy()).to(device), "pos": pos,
        "ctx_len": (pos + 1).to(torch.int32),
        "lengths": L, "slots": slot, "n_slots": n_slots, "capacity": capacity,
        "strides": strides, "layout": layout, "scale": float(np.float32(1.0 / np.sqrt(d))),
        "block": (block_rows, block_rows * Hkv * d) if layout == "head_blocked" else (0, 0),
    }


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a half/bfloat16 tensor as a numpy uint16 array (host copy)."""
    assert t.dtype in (torch.float16, torch.bfloat16)
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16).copy()


def from_bits(a: np.ndarray, dtype: str, device="cpu") -> torch.Tensor:
    """Inverse of bits()."""
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy())
    return t.view(TORCH_DTYPE[dtype]).to(device)


def round_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64/float32 values to the 16-bit dtype (nearest even), returned as bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(TORCH_DTYPE[dtype])
    return bits(t)


def algorithmic_bytes(w: Workload, ctx_len: np.ndarray) -> int:
    """Bytes the method itself must move for one step (Appendix A, Table 5, minus the score
    traffic that a fused kernel never materialises): K and V rows once per KV head, q read,
    fp32 output written, and the appended rows read and written."""
    e, d = ELEM_BYTES, w.head_dim
    n = np.asarray(ctx_len, dtype=np.int64)
    per_seq = 2 * n * w.n_kv_heads * d * e + w.n_q_heads * d * e + w.n_q_heads * d * 4 \
        + 2 * (2 * w.n_kv_heads * d * e)
    return int(per_seq.sum())


def attention_bytes(w: Workload, ctx_len: np.ndarray) -> int:
    """Algorithmic bytes of the attention kernel alone: K/V rows and q read (partials and the
    final output belong to the merge and are not counted here)."""
    e, d = ELEM_BYTES, w.head_dim
    n = np.asarray(ctx_len, dtype=np.int64)
    return int((2 * n * w.n_kv_heads * d * e + w.n_q_heads * d * e).sum())


def algorithmic_flops(w: Workload, ctx_len: np.ndarray) -> int:
    """4*H*d*n_b flops per sequence-step (Table 5: 2*S*B*D multiply-accumulates)."""
    n = np.asarray(ctx_len, dtype=np.int64)
    return int((4 * w.n_q_heads * w.head_dim * n).sum())
