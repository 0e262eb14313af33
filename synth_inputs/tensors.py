"""Array generation and number-format conversion for the synthetic inputs.

Nothing here evaluates the method: values are drawn, rounded to the storage
format and laid out.  The only "sampling" done is picking the draft tree's
sibling tokens, which belongs to the (absent) draft model, not to verification.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

RULE_GREEDY = 0
RULE_DETERMINISTIC = 1
RULE_DRAFT_WOR = 2
RULE_DRAFT_WR = 3
RULE_SAMPLE_MATCH = 4


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns.
    Inputs are finite here, so NaN handling is not needed."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class AttnInputs:
    """One batched verify-attention call.  `q`, `k_pool`, `v_pool` are in storage
    format: float32 arrays for dtype 'f32', uint16 bf16 bit patterns for 'bf16'.
    The pool holds, for sequence b, rows kv_offset[b] .. kv_offset[b]+prefix_len[b]+M-1:
    the cached prefix (its first soft_len rows are the soft-prompt slots) followed by
    this step's M new rows."""
    dtype: str
    B: int
    M: int
    Hq: int
    Hkv: int
    D: int
    soft_len: int
    scale: float
    prefix_len: np.ndarray          # int32 [B]
    kv_offset: np.ndarray           # int64 [B]
    q: np.ndarray                   # [B, M, Hq, D]
    k_pool: np.ndarray              # [tokens, Hkv, D]
    v_pool: np.ndarray              # [tokens, Hkv, D]
    parent: np.ndarray              # int32 [B, M]
    kind: np.ndarray                # uint8 [B, M]

    def _wide(self, a: np.ndarray) -> np.ndarray:
        if self.dtype == "bf16":
            return bf16_bits_to_f32(a).astype(np.float64)
        return a.astype(np.float64)

    def q_f64(self, b: int) -> np.ndarray:
        return self._wide(self.q[b])

    def _rows(self, b: int) -> slice:
        o = int(self.kv_offset[b])
        return slice(o, o + int(self.prefix_len[b]) + self.M)

    def k_f64(self, b: int) -> np.ndarray:
        return self._wide(self.k_pool[self._rows(b)])

    def v_f64(self, b: int) -> np.ndarray:
        return self._wide(self.v_pool[self._rows(b)])


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def make_attention_inputs(
    rng: np.random.Generator,
    *,
    dtype: str,
    Hq: int,
    Hkv: int,
    D: int,
    prefix_len,
    parent: np.ndarray,
    kind: np.ndarray,
    soft_len: int = 0,
    q_std: float = 1.0,
    kv_std: float = 1.0,
    scale: Optional[float] = None,
    pool_pad_tokens: int = 0,
) -> AttnInputs:
    """Draws Q ~ N(0, q_std), K,V ~ N(0, kv_std) and packs the sequences back to back
    into one pool (with `pool_pad_tokens` unused rows between sequences, so that a
    kernel reading past a sequence's end shows up as a wrong result)."""
    prefix_len = np.atleast_1d(np.asarray(prefix_len, dtype=np.int32))
    B = len(prefix_len)
    parent = np.asarray(parent, dtype=np.int32)
    kind = np.asarray(kind, dtype=np.uint8)
    if parent.ndim == 1:
        parent = np.broadcast_to(parent, (B, len(parent))).copy()
        kind = np.broadcast_to(kind, (B, len(kind))).copy()
    M = parent.shape[1]
    lens = prefix_len.astype(np.int64) + M
    kv_offset = np.zeros(B, dtype=np.int64)
    for b in range(1, B):
        kv_offset[b] = kv_offset[b - 1] + lens[b - 1] + pool_pad_tokens
    total = int(kv_offset[-1] + lens[-1] + pool_pad_tokens)
    q = _store(rng.standard_normal((B, M, Hq, D), dtype=np.float32) * q_std, dtype)
    k = _store(rng.standard_normal((total, Hkv, D), dtype=np.float32) * kv_std, dtype)
    v = _store(rng.standard_normal((total, Hkv, D), dtype=np.float32) * kv_std, dtype)
    return AttnInputs(
        dtype=dtype, B=B, M=M, Hq=Hq, Hkv=Hkv, D=D, soft_len=soft_len,
        scale=float(scale if scale is not None else 1.0 / np.sqrt(D)),
        prefix_len=prefix_len, kv_offset=kv_offset, q=q, k_pool=k, v_pool=v,
        parent=parent, kind=kind,
    )


@dataclass
class AcceptInputs:
    """One batched tree_accept call (parent/token index the T draft nodes only)."""
    B: int
    T: int
    V: int
    C: int
    temperature: float
    rule: int
    target_logits: np.ndarray               # float32 [B, T, V]
    draft_logits: Optional[np.ndarray]      # float32 [B, T, V] or None
    token: np.ndarray                       # int32 [B, T]
    parent: np.ndarray                      # int32 [B, T]
    uniforms: np.ndarray                    # float32 [B, 2T]
    con_anchor: Optional[np.ndarray] = None  # int32 [B, C]
    notes: dict = field(default_factory=dict)


def _children_lists(parent: np.ndarray):
    ch = [[] for _ in range(len(parent))]
    for i in range(1, len(parent)):
        ch[int(parent[i])].append(i)
    return ch


def make_accept_inputs(
    rng: np.random.Generator,
    *,
    parent: np.ndarray,
    V: int,
    temperature: float,
    rule: int,
    logit_std: float,
    con_anchor: Optional[np.ndarray] = None,
    draft_target_corr: float = 0.0,
    proposal_noise_std: float = 1.0,
    child_boost: float = 0.0,
) -> AcceptInputs:
    """parent: int32 [B, T] (or [T]).  Logits ~ N(0, logit_std) in float32.

    Sibling tokens: with draft logits (DRAFT_* rules) the children of a node are drawn
    without replacement from the draft distribution at that node's row, in draw order
    (Gumbel top-k on logits / temperature; for DRAFT_WR each child is drawn independently).
    Without draft logits the children are the top-k entries, best first, of a hidden
    proposal row = target row + N(0, proposal_noise_std) noise.
    `draft_target_corr` rho makes draft = rho*target + sqrt(1-rho^2)*noise.
    `child_boost` is added, after the tokens are picked, to the target (and draft) logit of every
    drafted token in its parent's row: a knob that lengthens the accepted walks (Gaussian logits
    over a large vocabulary are nearly flat, so most walks would stop at the root).
    """
    parent = np.asarray(parent, dtype=np.int32)
    if parent.ndim == 1:
        parent = parent[None, :]
    B, T = parent.shape
    target = (rng.standard_normal((B, T, V), dtype=np.float32) * np.float32(logit_std)).astype(np.float32)
    draft = None
    if rule in (RULE_DRAFT_WOR, RULE_DRAFT_WR):
        noise = rng.standard_normal((B, T, V), dtype=np.float32) * np.float32(logit_std)
        rho = np.float32(draft_target_corr)
        draft = (rho * target + np.sqrt(np.float32(1) - rho * rho) * noise).astype(np.float32)
    token = np.zeros((B, T), dtype=np.int32)
    for b in range(B):
        token[b, 0] = int(rng.integers(0, V))
        ch = _children_lists(parent[b])
        for u in range(T):
            k = len(ch[u])
            if k == 0:
                continue
            if draft is not None and temperature > 0:
                z = draft[b, u].astype(np.float64) / temperature
                if rule == RULE_DRAFT_WR:
                    picks = [int(np.argmax(z + rng.gumbel(size=V))) for _ in range(k)]
                else:
                    pert = z + rng.gumbel(size=V)
                    top = np.argpartition(-pert, k - 1)[:k]
                    picks = top[np.argsort(-pert[top])].tolist()
            else:
                prop = target[b, u].astype(np.float64) + rng.standard_normal(V) * proposal_noise_std
                top = np.argpartition(-prop, k - 1)[:k]
                picks = top[np.argsort(-prop[top])].tolist()
            for c, x in zip(ch[u], picks):
                token[b, c] = int(x)
                if child_boost:
                    target[b, u, int(x)] += np.float32(child_boost)
                    if draft is not None:
                        draft[b, u, int(x)] += np.float32(child_boost)
    uniforms = rng.random((B, 2 * T), dtype=np.float32)
    C = 0 if con_anchor is None else int(np.asarray(con_anchor).shape[-1])
    if con_anchor is not None:
        con_anchor = np.asarray(con_anchor, dtype=np.int32)
        if con_anchor.ndim == 1:
            con_anchor = np.broadcast_to(con_anchor, (B, C)).copy()
    return AcceptInputs(
        B=B, T=T, V=V, C=C, temperature=float(temperature), rule=int(rule),
        target_logits=target, draft_logits=draft, token=token, parent=parent.copy(),
        uniforms=uniforms, con_anchor=con_anchor,
    )
