"""Seeded synthetic inputs for the verify+draft hot path.

This module only *draws inputs*: shapes, lengths, page tables, Gaussian tensors,
uniforms and token ids.  It contains none of the method's arithmetic (no
softmax, no arg-max, no masking, no acceptance rule), so that the HIP library
and the CPU oracle can both be fed from it without sharing anything that could
hide a common mistake.  Where an input has to depend on a function of another
input (a draft token that agrees with the target's arg-max, a draft token drawn
from the drafter's distribution), the caller computes that function and passes
it in.

The five workloads are the benchmark configurations of this build; they stand in
for Qwen3-8B decoding steps (32 query heads, 8 KV heads, head size 128, vocabulary
151936) with the lengths and block sizes the paper's decoding modes produce:
a parallel-mode step carries k verify rows plus a block of m mask tokens per
sequence (Sec. 4.1 "Inference"), a sequential-mode verify step carries only a
confidence-pruned number of verify rows (Sec. 4.3).

bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even of the
float32 draw) so that every consumer sees byte-identical values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 20022
VOCAB_QWEN3 = 151936


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _gauss(rng: np.random.Generator, shape, std: float, dtype: str) -> np.ndarray:
    """N(0, std) tensor; bf16 as uint16 bits.  Drawn in slabs to bound host memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    step = 1 << 25
    for s in range(0, n, step):
        e = min(n, s + step)
        blk = rng.standard_normal(e - s, dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        out[s:e] = f32_to_bf16_bits(blk) if dtype == "bf16" else blk
    return out.reshape(shape)


@dataclass
class AttnWorkload:
    name: str
    dtype: str                      # "bf16" | "f32"
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    kv_len_range: tuple             # inclusive (lo, hi); lo == hi for fixed length
    verify_len_range: tuple         # inclusive (lo, hi) for k_i
    mask_len: int                   # m: length of one mask block (same for every sequence)
    std: float                      # standard deviation of Q, K, V entries
    shuffled_pages: bool = True
    spare_page_frac: float = 0.03   # unused physical pages left in the pool
    seed: int = BASE_SEED
    mask_blocks: int = 1            # 0: one block per verify row (full parallel mode), else that many blocks

    def scaled(self, **kw) -> "AttnWorkload":
        d = dict(self.__dict__); d.update(kw)
        return AttnWorkload(**d)


@dataclass
class AcceptWorkload:
    name: str
    dtype: str                      # logits dtype
    vocab: int
    mode: str                       # "greedy" | "sample"
    target_std: float
    draft_noise_std: float = 0.0    # sampling: draft = target + N(0, this)
    p_agree: float = 0.0            # greedy: chance a draft equals the caller-supplied token
    temperature: float = 1.0
    seed: int = BASE_SEED


_INV_SQRT_128 = float(1.0 / np.sqrt(128.0))

# name -> (attention workload, acceptance workload or None)
CONFIGS = {
    # tiny fp32 case: parity to 1e-5, greedy acceptance on a 1000-token vocabulary
    "cfg1": (AttnWorkload("cfg1", "f32", 1, 4, 1, 64, 16, (64, 64), (4, 4), 4, 1.0,
                          shuffled_pages=False, spare_page_frac=0.0, seed=BASE_SEED + 0),
             AcceptWorkload("cfg1", "f32", 1000, "greedy", 1.0, seed=BASE_SEED + 0)),
    # one sequence, contiguous cache, parallel mode with 1 bonus row + 15 mask tokens
    "cfg2": (AttnWorkload("cfg2", "bf16", 1, 32, 8, 128, 16, (2048, 2048), (1, 1), 15, _INV_SQRT_128,
                          shuffled_pages=False, spare_page_frac=0.0, seed=BASE_SEED + 1),
             None),
    # ragged batch, shuffled page table, 8 verify rows + 8 mask tokens, greedy acceptance
    "cfg3": (AttnWorkload("cfg3", "bf16", 16, 32, 8, 128, 16, (512, 4096), (8, 8), 8, _INV_SQRT_128,
                          seed=BASE_SEED + 2),
             AcceptWorkload("cfg3", "bf16", VOCAB_QWEN3, "greedy", 3.0, p_agree=0.7, seed=BASE_SEED + 2)),
    # large-batch sequential mode: no mask tokens, confidence-pruned verify length
    "cfg4": (AttnWorkload("cfg4", "bf16", 128, 32, 8, 128, 16, (1024, 8192), (1, 16), 0, _INV_SQRT_128,
                          seed=BASE_SEED + 3),
             None),
    # long context, 16 verify rows + 16 mask tokens, rejection-sampling acceptance
    "cfg5": (AttnWorkload("cfg5", "bf16", 4, 32, 8, 128, 16, (32768, 32768), (16, 16), 16, _INV_SQRT_128,
                          seed=BASE_SEED + 4),
             AcceptWorkload("cfg5", "bf16", VOCAB_QWEN3, "sample", 2.0, draft_noise_std=0.5,
                            temperature=1.0, seed=BASE_SEED + 4)),
    # beyond the five benchmark configurations: full parallel mode, one candidate block of 8 mask
    # tokens per hypothetical number of accepted drafts (4 verify rows -> 4 blocks, 36 new rows)
    "par4": (AttnWorkload("par4", "bf16", 8, 32, 8, 128, 16, (2048, 8192), (4, 4), 8, _INV_SQRT_128,
                          seed=BASE_SEED + 5, mask_blocks=0),
             None),
}
# Decoupled execution (Sec. 4.3): the draft step of the large-batch mode runs the mask tokens alone
# over the cache target verification left behind -- cfg4's batch and prefix lengths (same seed, and
# the lengths are the first thing drawn), no verify rows, one block of 16 mask tokens.
CONFIGS["seq_draft"] = (AttnWorkload("seq_draft", "bf16", 128, 32, 8, 128, 16, (1024, 8192), (0, 0), 16, _INV_SQRT_128,
                                     seed=BASE_SEED + 3), None)
# Full parallel mode at the batch sizes it is used at (Sec. 4.3: batch <= 2): the anchor and 15 drafts
# are verified while one block of 16 mask tokens is drafted per hypothetical number of accepted drafts
# (Sec. 3: k + 1 hypotheses for k drafts) -- 16 + 16 x 16 = 272 new rows per sequence.
for _name, _b in (("par_b1", 1), ("par_b2", 2)):
    CONFIGS[_name] = (AttnWorkload(_name, "bf16", _b, 32, 8, 128, 16, (2048, 8192), (16, 16), 16, _INV_SQRT_128,
                                   seed=BASE_SEED + 6, mask_blocks=0), None)
# The other sizes of the model family the paper decodes with (Sec. 5, models table): cfg3's batch,
# lengths and paging with the attention shapes of the public Qwen3 configurations.  All of them keep
# D = 128 and 8 KV heads; what changes is the number of query heads per KV head.
for _name, _hq in (("q3_1p7b", 16), ("q3_14b", 40), ("q3_32b", 64)):     # 4B shares the 8B shape (32 / 8)
    CONFIGS[_name] = (AttnWorkload(_name, "bf16", 16, _hq, 8, 128, 16, (512, 4096), (8, 8), 8, _INV_SQRT_128,
                                   seed=BASE_SEED + 2), None)

# A head dim of 64 (the other size the matrix-core kernel takes; 32 / 8 heads with D = 64 is the attention
# shape of small Llama-3.2-class decoders): cfg3's batch, lengths and paging, entries scaled for D = 64.
CONFIGS["d64"] = (AttnWorkload("d64", "bf16", 16, 32, 8, 64, 16, (512, 4096), (8, 8), 8, 0.125, seed=BASE_SEED + 2), None)


def make_lengths(w: AttnWorkload):
    """Per-sequence lengths and the page table (no tensors).  Deterministic in w.seed."""
    rng = np.random.default_rng(np.random.PCG64(w.seed))
    B, ps = w.batch, w.page_size
    lo, hi = w.kv_len_range
    kv_len = rng.integers(lo, hi + 1, size=B, dtype=np.int64).astype(np.int32)
    klo, khi = w.verify_len_range
    verify_len = rng.integers(klo, khi + 1, size=B, dtype=np.int64).astype(np.int32)
    blocks = verify_len.copy() if w.mask_blocks == 0 else np.full(B, w.mask_blocks, dtype=np.int32)
    rows = verify_len + blocks * np.int32(w.mask_len)
    row_indptr = np.zeros(B + 1, dtype=np.int32)
    row_indptr[1:] = np.cumsum(rows)
    pages_per_seq = (kv_len.astype(np.int64) + ps - 1) // ps
    page_indptr = np.zeros(B + 1, dtype=np.int32)
    page_indptr[1:] = np.cumsum(pages_per_seq)
    used = int(page_indptr[-1])
    num_pages = max(1, used + int(np.ceil(used * w.spare_page_frac)))
    if w.shuffled_pages:
        page_indices = rng.permutation(num_pages)[:used].astype(np.int32)
    else:
        page_indices = np.arange(used, dtype=np.int32)
    return dict(kv_len=kv_len, verify_len=verify_len, row_indptr=row_indptr,
                page_indptr=page_indptr, page_indices=page_indices, num_pages=num_pages,
                mask_blocks=(None if w.mask_blocks == 1 else blocks.astype(np.int32)))


def make_attention_inputs(w: AttnWorkload, *, std: Optional[float] = None):
    """All inputs of one attention call as host arrays.

    Cache layout [num_pages, Hkv, page_size, D]; every slot of every page holds a
    Gaussian draw, including the slots past a sequence's length and the spare
    pages, so that a missing length mask or a wrong page lookup changes the result.
    `std` overrides the workload's scale (the "sharp" twin uses std = 1).
    """
    s = w.std if std is None else std
    lens = make_lengths(w)
    rng = np.random.default_rng(np.random.PCG64(w.seed + 1000))
    R = int(lens["row_indptr"][-1])
    Hq, Hkv, D, ps = w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size
    out = dict(lens)
    out["q"] = _gauss(rng, (R, Hq, D), s, w.dtype)
    out["k_new"] = _gauss(rng, (R, Hkv, D), s, w.dtype)
    out["v_new"] = _gauss(rng, (R, Hkv, D), s, w.dtype)
    out["k_cache"] = _gauss(rng, (lens["num_pages"], Hkv, ps, D), s, w.dtype)
    out["v_cache"] = _gauss(rng, (lens["num_pages"], Hkv, ps, D), s, w.dtype)
    out["workload"] = w
    return out


def kv_bytes(w: AttnWorkload, kv_len: np.ndarray) -> int:
    """Algorithmic cache bytes of one call: every cached token's K and V read once."""
    elt = 2 if w.dtype == "bf16" else 4
    return int(kv_len.astype(np.int64).sum()) * w.num_kv_heads * w.head_dim * 2 * elt


def attention_flops(w: AttnWorkload, kv_len: np.ndarray, row_indptr: np.ndarray) -> int:
    """2 contractions x 2 flops x rows x heads x D per cached token."""
    rows = np.diff(row_indptr).astype(np.int64)
    return int((rows * kv_len.astype(np.int64)).sum()) * w.num_q_heads * w.head_dim * 4


def make_logits(a: AcceptWorkload, num_rows: int):
    """Target logits (and, in sampling mode, draft logits = target + noise)."""
    rng = np.random.default_rng(np.random.PCG64(a.seed + 2000))
    out = {}
    t32 = rng.standard_normal((num_rows, a.vocab), dtype=np.float32) * np.float32(a.target_std)
    if a.dtype == "bf16":
        out["target_logits"] = f32_to_bf16_bits(t32)
        t32 = bf16_bits_to_f32(out["target_logits"])
    else:
        out["target_logits"] = t32
    if a.mode == "sample":
        d32 = t32 + rng.standard_normal((num_rows, a.vocab), dtype=np.float32) * np.float32(a.draft_noise_std)
        out["draft_logits"] = f32_to_bf16_bits(d32) if a.dtype == "bf16" else d32
        out["u_accept"] = rng.random(num_rows, dtype=np.float32)
        out["u_resample"] = rng.random(num_rows, dtype=np.float32)
    return out


def make_peaked_logits(vocab: int, num_rows: int, seed: int, dtype: str = "bf16", peak_lo: float = 6.0,
                       peak_hi: float = 16.0):
    """Drafter logits of a mask block: unit-normal background plus one raised entry per row, the
    raise drawn uniformly from [peak_lo, peak_hi] so that the rows' top probabilities spread from
    a few percent to nearly one (what the confidence threshold of selective verification sees)."""
    rng = np.random.default_rng(np.random.PCG64(seed + 4000))
    x = rng.standard_normal((num_rows, vocab), dtype=np.float32)
    if num_rows:
        top = rng.integers(0, vocab, size=num_rows)
        x[np.arange(num_rows), top] += rng.uniform(peak_lo, peak_hi, size=num_rows).astype(np.float32)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def make_draft_tokens_agreeing(a: AcceptWorkload, row_indptr: np.ndarray, agree_tokens: np.ndarray):
    """Tokens fed at the verify rows for a greedy workload.

    Row 0 of each sequence is the anchor (any token).  The token fed at row j+1
    equals agree_tokens[j] -- which the caller computed from row j's logits --
    with probability a.p_agree, otherwise a uniformly drawn *different* token.
    """
    rng = np.random.default_rng(np.random.PCG64(a.seed + 3000))
    Rv = int(row_indptr[-1])
    toks = rng.integers(0, a.vocab, size=Rv, dtype=np.int64)
    coin = rng.random(Rv)
    other = rng.integers(1, a.vocab, size=Rv, dtype=np.int64)
    for i in range(len(row_indptr) - 1):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        for j in range(r0, r1 - 1):
            want = int(agree_tokens[j])
            toks[j + 1] = want if coin[j] < a.p_agree else (want + int(other[j])) % a.vocab
    return toks.astype(np.int32)


def make_draft_tokens_from_probs(a: AcceptWorkload, row_indptr: np.ndarray, draft_probs):
    """Tokens fed at the verify rows for a sampling workload: the token at row j+1
    is drawn from the categorical distribution draft_probs(j) the caller supplies
    (a callable row -> probability vector, so that full rows are made one at a time)."""
    rng = np.random.default_rng(np.random.PCG64(a.seed + 3000))
    Rv = int(row_indptr[-1])
    toks = rng.integers(0, a.vocab, size=Rv, dtype=np.int64)
    for i in range(len(row_indptr) - 1):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        for j in range(r0, r1 - 1):
            pr = np.asarray(draft_probs(j), dtype=np.float64)
            toks[j + 1] = int(rng.choice(a.vocab, p=pr / pr.sum()))
    return toks.astype(np.int32)


def verify_row_indptr(lens: dict) -> np.ndarray:
    """Packed verify-row offsets (mask rows dropped): the acceptance step's row layout."""
    out = np.zeros(len(lens["verify_len"]) + 1, dtype=np.int32)
    out[1:] = np.cumsum(lens["verify_len"])
    return out


def subset_inputs(inp: dict, ids) -> dict:
    """The same problem restricted to sequences `ids` (caches and page ids untouched)."""
    ids = list(ids)
    rows = [np.arange(inp["row_indptr"][i], inp["row_indptr"][i + 1]) for i in ids]
    keep = np.concatenate(rows) if rows else np.zeros(0, dtype=np.int64)
    sub = dict(inp)
    for k in ("q", "k_new", "v_new"):
        sub[k] = inp[k][keep]
    sub["kv_len"] = inp["kv_len"][ids]
    sub["verify_len"] = inp["verify_len"][ids]
    if inp.get("mask_blocks") is not None:
        sub["mask_blocks"] = np.asarray(inp["mask_blocks"])[ids]
    sub["row_indptr"] = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    pages = [inp["page_indices"][inp["page_indptr"][i]:inp["page_indptr"][i + 1]] for i in ids]
    sub["page_indices"] = np.concatenate(pages).astype(np.int32) if pages else np.zeros(0, dtype=np.int32)
    sub["page_indptr"] = np.concatenate([[0], np.cumsum([len(p) for p in pages])]).astype(np.int32)
    sub["_rows"] = keep
    return sub
