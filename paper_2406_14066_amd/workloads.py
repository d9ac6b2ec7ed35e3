"""Seeded synthetic inputs of the speculative-verification step.

This module only draws random numbers and lays bytes out.  It holds none of
the method's arithmetic (no softmax, no accept rule, no attention) so that the
CPU oracle and the HIP library can both be fed from it without sharing any of
what is being checked.

The five named workloads stand in for the paper's serving traces: head shapes
of Llama-2-7B / Llama-3-70B class models, context lengths in the range of the
paper's datasets (its Table 2) and of its long-context runs, draft/target
agreement tuned to the acceptance rates it reports (0.5 / 0.7 / 0.9 in the
micro-benchmarks of Section 5.1, 0.53-0.92 in its Table 3), speculation lengths
0..8 (its sweeps use 1..7).

Canonical KV layout produced here: token-major pages
``[num_blocks, Hkv, block_size, d]``; logical token ``t`` of request ``b`` is
in page ``block_table[b, t // block_size]`` at slot ``t % block_size``.  Slots
past ``kv_len`` in a request's last page and all spare pages hold a large
finite filler value that must never influence a result.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

BLOCK_SIZE = 16
FILLER = 1.0e4  # value of never-visible KV slots

# Standard deviation of (target - draft) logit noise per acceptance level.
# For Gaussian logits and a large vocabulary the per-token acceptance
# probability is close to 2*Phi(-sigma/2); the values below were then refined
# against the measured sum_v min(p_v, q_v) of generated rows by
# tests/golden/calibrate_sigma.py (which uses only the CPU oracle).
SIGMA_FOR_ALPHA = {
    # (vocab, draft_std): {alpha: sigma}
    (1024, 2.0): {0.6: 1.0},   # fixed by the workload's statement: N(0,1) noise
    (32000, 3.0): {0.5: 1.353, 0.6: 1.051, 0.7: 0.773, 0.9: 0.254},
    (128256, 3.0): {0.75: 0.643},
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class VerifyWorkload:
    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    V: int
    dtype: str                      # "f32" or "bf16" (Q/K/V storage; logits are always fp32)
    block_size: int
    kv_len: np.ndarray              # [B] int32, includes this step's q_len new tokens
    q_len: np.ndarray               # [B] int32 = k_b + 1
    cu_q_len: np.ndarray            # [B+1] int32
    block_table: np.ndarray         # [B, max_blocks_per_req] int32 (unused entries 0)
    q: np.ndarray                   # [T, Hq, d] float32 or uint16 (bf16 bits)
    k_pages: np.ndarray             # [num_blocks, Hkv, bs, d]
    v_pages: np.ndarray
    target_logits: np.ndarray       # [T, V] float32
    draft_logits: np.ndarray        # [T-B, V] float32
    draft_tokens: np.ndarray        # [T-B] int32
    philox_seed: int
    philox_step: int
    sigma: float = 0.0
    meta: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return int(self.cu_q_len[-1])

    @property
    def num_blocks(self) -> int:
        return int(self.k_pages.shape[0])

    @property
    def k(self) -> np.ndarray:
        return self.q_len - 1

    def attn_algorithmic_bytes(self) -> int:
        """Bytes the attention must move: every K and V element of every request
        once, Q in, O (fp32) out, and the block-table entries walked."""
        esz = 4 if self.dtype == "f32" else 2
        kv = int(self.kv_len.astype(np.int64).sum()) * self.Hkv * self.d * 2 * esz
        qo = self.T * self.Hq * self.d * (esz + 4)
        bt = 4 * int(((self.kv_len.astype(np.int64) + self.block_size - 1) // self.block_size).sum())
        return kv + qo + bt

    def reject_algorithmic_bytes(self) -> int:
        """Every target row and every draft row once."""
        return (self.T + (self.T - self.B)) * self.V * 4

    def verified_tokens(self) -> int:
        return self.T


def make_logits(rng: np.random.Generator, q_len: np.ndarray, V: int, draft_std: float, sigma: float):
    """Draft rows ~ N(0, draft_std^2); target row = draft row + N(0, sigma^2).
    Every request gets q_len rows of each; the last draft row of a request has
    no draft token (it only seeds the extra target row) and is dropped.
    Draft tokens are drawn from softmax(draft row) by the Gumbel-max trick."""
    T = int(q_len.sum())
    B = len(q_len)
    draft_full = rng.standard_normal((T, V), dtype=np.float32) * np.float32(draft_std)
    target = draft_full + rng.standard_normal((T, V), dtype=np.float32) * np.float32(sigma)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int64)
    keep = np.ones(T, dtype=bool)
    keep[cu[1:] - 1] = False
    draft = np.ascontiguousarray(draft_full[keep])
    # Gumbel-max: argmax(logit + G) is a draw from softmax(logit)
    tokens = np.empty(T - B, dtype=np.int32)
    for r in range(T - B):
        g = rng.gumbel(size=V)
        tokens[r] = int(np.argmax(draft[r].astype(np.float64) + g))
    return np.ascontiguousarray(target), draft, tokens


def make_paged_kv(rng: np.random.Generator, kv_len: np.ndarray, Hkv: int, d: int, dtype: str,
                  shuffle: bool, spare_frac: float = 0.25, block_size: int = BLOCK_SIZE):
    """N(0,1) K and V for every visible token, scattered into a page pool through a
    (shuffled) block table; tails and spare pages hold FILLER."""
    B = len(kv_len)
    nblk = (kv_len.astype(np.int64) + block_size - 1) // block_size
    need = int(nblk.sum())
    num_blocks = need + int(np.ceil(need * spare_frac)) if shuffle else need
    num_blocks = max(num_blocks, 1)
    max_blocks = int(nblk.max()) if B else 1
    order = rng.permutation(num_blocks)[:need] if shuffle else np.arange(need)
    block_table = np.zeros((B, max_blocks), dtype=np.int32)
    off = 0
    for b in range(B):
        block_table[b, : nblk[b]] = order[off: off + nblk[b]]
        off += int(nblk[b])

    def pool():
        data = rng.standard_normal((need, Hkv, block_size, d), dtype=np.float32)
        # overwrite the invisible tail of each request's last page
        o = 0
        for b in range(B):
            tail = int(kv_len[b]) % block_size
            if tail:
                data[o + int(nblk[b]) - 1, :, tail:, :] = FILLER
            o += int(nblk[b])
        if dtype == "bf16":
            full = np.full((num_blocks, Hkv, block_size, d), f32_to_bf16_bits(np.float32(FILLER)), dtype=np.uint16)
            full[order] = f32_to_bf16_bits(data)
        else:
            full = np.full((num_blocks, Hkv, block_size, d), FILLER, dtype=np.float32)
            full[order] = data
        return full

    k_pages = pool()
    v_pages = pool()
    return k_pages, v_pages, block_table


def make_workload(name: str, *, B: int, Hq: int, Hkv: int, d: int, V: int, dtype: str,
                  kv_len: Sequence[int], k: Sequence[int], draft_std: float, sigma: float,
                  data_seed: int, philox_seed: int, philox_step: int = 0, shuffle: bool = True,
                  with_kv: bool = True, with_logits: bool = True) -> VerifyWorkload:
    rng = np.random.default_rng(data_seed)
    kv_len = np.asarray(kv_len, dtype=np.int32)
    q_len = np.asarray(k, dtype=np.int32) + 1
    assert kv_len.shape == (B,) and q_len.shape == (B,)
    assert np.all(kv_len >= q_len) and np.all(q_len >= 1)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    T = int(cu[-1])
    if with_kv:
        qf = rng.standard_normal((T, Hq, d), dtype=np.float32)
        q = f32_to_bf16_bits(qf) if dtype == "bf16" else qf
        k_pages, v_pages, block_table = make_paged_kv(rng, kv_len, Hkv, d, dtype, shuffle)
    else:
        et = np.uint16 if dtype == "bf16" else np.float32
        q = np.zeros((T, Hq, d), dtype=et)
        k_pages = v_pages = np.zeros((1, Hkv, BLOCK_SIZE, d), dtype=et)
        block_table = np.zeros((B, 1), dtype=np.int32)
    # logits come from their own generator so they do not depend on the KV shape
    lrng = np.random.default_rng([data_seed, 7919])
    if with_logits:
        target, draft, tokens = make_logits(lrng, q_len, V, draft_std, sigma)
    else:
        target = np.zeros((T, 1), dtype=np.float32)
        draft = np.zeros((T - B, 1), dtype=np.float32)
        tokens = np.zeros(T - B, dtype=np.int32)
    return VerifyWorkload(name=name, B=B, Hq=Hq, Hkv=Hkv, d=d, V=V, dtype=dtype, block_size=BLOCK_SIZE,
                          kv_len=kv_len, q_len=q_len, cu_q_len=cu, block_table=block_table, q=q,
                          k_pages=k_pages, v_pages=v_pages, target_logits=target, draft_logits=draft,
                          draft_tokens=tokens, philox_seed=philox_seed, philox_step=philox_step, sigma=sigma)


def _sigma(V: int, draft_std: float, alpha: float) -> float:
    return SIGMA_FOR_ALPHA[(V, draft_std)][alpha]


def config(name: str, *, k: Optional[int] = None, alpha: Optional[float] = None,
           B: Optional[int] = None, L_scale: float = 1.0, V: Optional[int] = None,
           with_kv: bool = True, with_logits: bool = True) -> VerifyWorkload:
    """The five named workloads ("c1".."c5").  ``B``, ``L_scale`` and ``V`` shrink a
    workload for tests that need the CPU oracle to finish quickly; ``k`` and ``alpha``
    select the point of the c3 sweep (``k`` also overrides c4's draft length of 2)."""
    name = name.lower()
    if name == "c1":
        # tiny fp32: one request, 128 tokens as 8 consecutive pages with the identity table
        return make_workload("c1", B=1, Hq=8, Hkv=8, d=64, V=V or 1024, dtype="f32", kv_len=[128], k=[4],
                             draft_std=2.0, sigma=1.0, data_seed=1, philox_seed=0, shuffle=False,
                             with_kv=with_kv, with_logits=with_logits)
    if name == "c2":
        b = B or 8
        L = max(int(2048 * L_scale), 8)
        return make_workload("c2", B=b, Hq=32, Hkv=32, d=128, V=V or 32000, dtype="bf16", kv_len=[L] * b,
                             k=[4] * b, draft_std=3.0, sigma=_sigma(32000, 3.0, 0.7), data_seed=2,
                             philox_seed=2, with_kv=with_kv, with_logits=with_logits)
    if name == "c3":
        b = B or 32
        kk = 4 if k is None else k
        a = 0.7 if alpha is None else alpha
        L = max(int(1024 * L_scale), 16)
        run = kk * 3 + {0.5: 0, 0.7: 1, 0.9: 2}[a]
        w = make_workload("c3", B=b, Hq=32, Hkv=32, d=128, V=V or 32000, dtype="bf16", kv_len=[L] * b,
                          k=[kk] * b, draft_std=3.0, sigma=_sigma(32000, 3.0, a), data_seed=3,
                          philox_seed=3, philox_step=run, with_kv=with_kv, with_logits=with_logits)
        w.meta.update(k=kk, alpha=a)
        return w
    if name == "c4":
        b = B or 256
        rng = np.random.default_rng(40)
        lens = rng.integers(int(256 * L_scale), int(1024 * L_scale) + 1, size=b)
        return make_workload("c4", B=b, Hq=64, Hkv=8, d=128, V=V or 32000, dtype="bf16",
                             kv_len=np.maximum(lens, 9), k=[2 if k is None else k] * b, draft_std=3.0,
                             sigma=_sigma(32000, 3.0, 0.6), data_seed=4, philox_seed=4,
                             with_kv=with_kv, with_logits=with_logits)
    if name == "c5":
        b = B or 4
        rng = np.random.default_rng(50)
        lens = rng.integers(int(1024 * L_scale), int(32768 * L_scale) + 1, size=b)
        ks = rng.integers(1, 9, size=b)
        return make_workload("c5", B=b, Hq=32, Hkv=8, d=128, V=V or 128256, dtype="bf16",
                             kv_len=np.maximum(lens, 9), k=ks, draft_std=3.0,
                             sigma=_sigma(128256, 3.0, 0.75), data_seed=5, philox_seed=5,
                             with_kv=with_kv, with_logits=with_logits)
    raise KeyError(name)
