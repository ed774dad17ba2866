"""Seeded synthetic inputs for the FlashMask hot path.

This module builds *inputs only*: bf16-rounded Q/K/V/dO tensors and the four
int32 column-bound vectors (LTS, LTE, UTS, UTE) that describe a mask family
(Section 2.1 mask types; Section 4.1 representation).  It holds none of the
method's arithmetic -- no attention, no softmax, no tile tables -- so that the
CPU oracle and the HIP path can both be fed from it without sharing code.

Conventions (0-based, half-open): query row i may NOT attend to key column j
iff LTS[j] <= i < LTE[j] or UTS[j] <= i < UTE[j].  "No interval" is written
(N, N) for the lower pair and (0, 0) for the upper pair.

The document / shared-question samplers follow the shapes of the paper's own
synthetic kernel-benchmark data (Appendix "Data Construction Method": sample a
document count, then lengths summing to N; shared-question documents are one
question plus several answers).  The paper's samples are unpublished, so these
are stand-ins drawn from a seeded generator.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20241002


# --------------------------------------------------------------------------
# bf16 tensors
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_tensors(seed: int, B: int, H: int, N: int, d: int, names=("q", "k", "v", "dout")):
    """~N(0,1) tensors [B,H,N,d], drawn in the order q, k, v, dout and rounded
    to bf16.  Returns {name: uint16 bit patterns}."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = {}
    for name in ("q", "k", "v", "dout"):
        x = rng.standard_normal((B, H, N, d), dtype=np.float32)
        if name in names:
            out[name] = to_bf16_bits(x)
        del x
    return out


# --------------------------------------------------------------------------
# Mask vectors from task structure
# --------------------------------------------------------------------------
def _empty(N):
    lts = np.full(N, N, dtype=np.int32)
    lte = np.full(N, N, dtype=np.int32)
    uts = np.zeros(N, dtype=np.int32)
    ute = np.zeros(N, dtype=np.int32)
    return lts, lte, uts, ute


def full_mask(N):
    return _empty(N)


def causal_mask(N):
    lts, lte, uts, ute = _empty(N)
    ute[:] = np.arange(N)                      # rows [0, j) cannot see column j
    return lts, lte, uts, ute


def sliding_window_mask(N, w):
    """Causal window: row i sees columns j with 0 <= i - j < w."""
    lts, lte, uts, ute = causal_mask(N)
    lts[:] = np.minimum(np.arange(N) + w, N)
    return lts, lte, uts, ute


def document_mask(N, spans):
    """Bidirectional attention inside each document [s, e)."""
    lts, lte, uts, ute = _empty(N)
    for s, e in spans:
        lts[s:e] = e
        ute[s:e] = s
    return lts, lte, uts, ute


def causal_document_mask(N, spans):
    lts, lte, uts, ute = causal_mask(N)
    for s, e in spans:
        lts[s:e] = e
    return lts, lte, uts, ute


def shared_question_mask(N, samples):
    """samples: list of (s, [a_1, ..., a_k], e): question [s, a_1), answers
    [a_m, a_{m+1}) with a_{k+1} = e.  Answers see the question and themselves,
    causally, but not sibling answers.  A sample with no answers is a plain
    causal document."""
    lts, lte, uts, ute = causal_mask(N)
    for s, starts, e in samples:
        if not starts:
            lts[s:e] = e
            continue
        lts[s:starts[0]] = e                    # question columns: visible to the whole sample
        bounds = list(starts) + [e]
        for a0, a1 in zip(bounds[:-1], bounds[1:]):
            lts[a0:a1] = a1                     # answer columns: visible inside that answer only
    return lts, lte, uts, ute


def prefix_lm_mask(N, p):
    """Columns of the prefix [0, p) are visible to every row; the rest causal."""
    lts, lte, uts, ute = causal_mask(N)
    ute[:p] = 0
    return lts, lte, uts, ute


def prefix_document_mask(N, docs):
    """docs: list of (s, p, e): inside document [s, e) the prefix columns
    [s, p) are visible to every row of the document, the rest causally."""
    lts, lte, uts, ute = _empty(N)
    for s, p, e in docs:
        lts[s:e] = e
        ute[s:p] = s
        ute[p:e] = np.arange(p, e)
    return lts, lte, uts, ute


def global_sliding_window_mask(N, g, w):
    """Bidirectional window |i - j| < w, plus g global tokens at the front:
    global columns are visible to everyone and global rows see everything."""
    lts, lte, uts, ute = _empty(N)
    j = np.arange(N)
    lts[:] = np.minimum(j + w, N)
    ute[:] = np.maximum(j - w + 1, 0)
    uts[:] = np.minimum(g, ute)                 # rows [0, g) are never masked
    lts[:g] = N
    ute[:g] = 0
    uts[:g] = 0
    return lts, lte, uts, ute


def causal_blockwise_mask(N, block, n_test):
    """In-context-learning layout: demonstrations in blocks of `block` tokens
    attend causally inside their own and the previous block; the last n_test
    rows (the test example) attend causally to everything."""
    lts, lte, uts, ute = causal_mask(N)
    t0 = N - n_test
    for j in range(t0):
        blk = j // block
        lts[j] = min((blk + 2) * block, t0)     # masked from two blocks on ...
        lte[j] = t0                             # ... until the test rows begin
    return lts, lte, uts, ute


def random_eviction_mask(N, evict_at):
    """Causal; key j is evicted from the cache at row evict_at[j] > j."""
    lts, lte, uts, ute = causal_mask(N)
    lts[:] = np.minimum(np.maximum(np.asarray(evict_at, dtype=np.int64), np.arange(N) + 1), N)
    return lts, lte, uts, ute


def qk_sparse_mask(N, dropped_keys, q_block):
    """Causal attention in which some keys and one block of queries take no part: key column j is
    dropped if dropped_keys[j], query rows [a, b) = q_block see nothing.  (A column carries one
    lower-triangle interval, so the dropped queries must be one contiguous block; the dropped keys may
    be any set.)"""
    lts, lte, uts, ute = causal_mask(N)
    a, b = q_block
    j = np.arange(N)
    first = np.maximum(a, j)                   # first dropped row at or below the diagonal
    has = first < b
    lts[:] = np.where(has, first, N)
    lte[:] = np.where(has, b, N)
    dk = np.asarray(dropped_keys, dtype=bool)
    lts[dk] = j[dk]                            # a dropped key: every row from the diagonal down
    lte[dk] = N
    return lts, lte, uts, ute


# --------------------------------------------------------------------------
# Span samplers
# --------------------------------------------------------------------------
def spans_from_lengths(lengths):
    spans, s = [], 0
    for n in lengths:
        spans.append((s, s + int(n)))
        s += int(n)
    return spans


def sample_partition(rng, N, n_docs, min_len):
    """Uniform composition of N into n_docs parts, each >= min_len."""
    slack = N - n_docs * min_len
    assert slack >= 0
    cuts = np.sort(rng.integers(0, slack + 1, size=n_docs - 1))
    edges = np.concatenate(([0], cuts, [slack]))
    return [int(min_len + g) for g in np.diff(edges)]


def sample_log_uniform_lengths(rng, N, n_docs, min_len):
    raw = np.exp(rng.uniform(math.log(min_len), math.log(N), size=n_docs))
    lens = np.maximum(np.floor(raw * (N / raw.sum())).astype(np.int64), min_len)
    # put the remainder (positive or negative) on the largest document
    lens[int(np.argmax(lens))] += N - int(lens.sum())
    assert lens.min() >= min_len and int(lens.sum()) == N
    return [int(x) for x in lens]


def sample_shared_question(rng, N, q_range=(512, 2048), a_range=(256, 1024), k_range=(2, 4)):
    """Pack question+answers samples until the next one no longer fits; the
    remainder becomes one causal padding document."""
    samples, s = [], 0
    while True:
        q = int(rng.integers(q_range[0], q_range[1] + 1))
        k = int(rng.integers(k_range[0], k_range[1] + 1))
        answers = [int(rng.integers(a_range[0], a_range[1] + 1)) for _ in range(k)]
        total = q + sum(answers)
        if s + total > N:
            break
        starts, a = [], s + q
        for n in answers:
            starts.append(a)
            a += n
        samples.append((s, starts, s + total))
        s += total
    if s < N:
        samples.append((s, [], N))
    return samples


# --------------------------------------------------------------------------
# The five benchmark configurations
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    seed: int
    mask_kind: str
    vectors: list = field(default_factory=list)     # per batch row: (lts, lte, uts, ute)
    structure: list = field(default_factory=list)   # per batch row: spans / samples / params

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.d)

    def stacked_vectors(self):
        """Four int32 arrays of shape [B, N]."""
        return tuple(np.stack([v[a] for v in self.vectors]).astype(np.int32) for a in range(4))

    def tensors(self, names=("q", "k", "v", "dout")):
        return make_tensors(self.seed, self.B, self.H, self.N, self.d, names)


def _mask_rng(seed):
    return np.random.Generator(np.random.PCG64(seed + 7))


def config(name: str) -> Workload:
    """name in {"1", "2", "3", "4a", "4b", "5"}."""
    if name == "1":
        w = Workload("1", 1, 2, 512, 64, BASE_SEED + 100, "causal_document")
        spans = spans_from_lengths([200, 180, 132])
        w.structure = [spans]
        w.vectors = [causal_document_mask(w.N, spans)]
    elif name == "2":
        w = Workload("2", 2, 32, 8192, 128, BASE_SEED + 200, "causal_document")
        rng = _mask_rng(w.seed)
        for _ in range(w.B):
            n_docs = int(rng.integers(2, 21))
            spans = spans_from_lengths(sample_partition(rng, w.N, n_docs, 128))
            w.structure.append(spans)
            w.vectors.append(causal_document_mask(w.N, spans))
    elif name == "3":
        w = Workload("3", 1, 32, 16384, 128, BASE_SEED + 300, "shared_question")
        rng = _mask_rng(w.seed)
        samples = sample_shared_question(rng, w.N)
        w.structure = [samples]
        w.vectors = [shared_question_mask(w.N, samples)]
    elif name == "4a":
        w = Workload("4a", 1, 16, 32768, 128, BASE_SEED + 400, "sliding_window")
        w.structure = [{"window": 1024}]
        w.vectors = [sliding_window_mask(w.N, 1024)]
    elif name == "4b":
        w = Workload("4b", 1, 16, 32768, 128, BASE_SEED + 401, "prefix_lm")
        w.structure = [{"prefix": 4096}]
        w.vectors = [prefix_lm_mask(w.N, 4096)]
    elif name == "4b-d64":
        # not one of the five configurations: run (b) of configuration 4 at head dimension 64 with twice the
        # heads (same hidden size, same FLOPs), the shape of the paper's d = 64 kernel tables
        w = Workload("4b-d64", 1, 32, 32768, 64, BASE_SEED + 402, "prefix_lm")
        w.structure = [{"prefix": 4096}]
        w.vectors = [prefix_lm_mask(w.N, 4096)]
    elif name == "5":
        w = Workload("5", 1, 8, 131072, 128, BASE_SEED + 500, "causal_document")
        rng = _mask_rng(w.seed)
        n_docs = int(rng.integers(4, 65))
        spans = spans_from_lengths(sample_log_uniform_lengths(rng, w.N, n_docs, 512))
        w.structure = [spans]
        w.vectors = [causal_document_mask(w.N, spans)]
    else:
        raise ValueError(f"unknown config {name!r}")
    return w


CONFIG_NAMES = ("1", "2", "3", "4a", "4b", "5")


def sweep_workloads(n_random: int = 20):
    """Workloads of the block-sparsity sweep: the shape of config 4 (B=1, H=16, N=32768, d=128)
    with causal-document masks of 1, 2, 4, ..., 128 equal documents and `n_random` seeded random
    partitions (2..64 documents, uniform composition with floor 128), then bidirectional document
    masks (the same equal partitions and n_random / 2 random ones) and n_random / 2 shared-question
    masks of growing sample size."""
    out = []
    N = 32768
    for k, n_docs in enumerate((1, 2, 4, 8, 16, 32, 64, 128)):
        w = Workload(f"sweep-eq{n_docs}", 1, 16, N, 128, BASE_SEED + 600 + k, "causal_document")
        spans = spans_from_lengths([N // n_docs] * n_docs)
        w.structure = [spans]
        w.vectors = [causal_document_mask(N, spans)]
        out.append(w)
    for k in range(n_random):
        w = Workload(f"sweep-rand{k}", 1, 16, N, 128, BASE_SEED + 650 + k, "causal_document")
        rng = _mask_rng(w.seed)
        n_docs = int(rng.integers(2, 65))
        spans = spans_from_lengths(sample_partition(rng, N, n_docs, 128))
        w.structure = [spans]
        w.vectors = [causal_document_mask(N, spans)]
        out.append(w)
    # the other two masks of the paper's sparsity experiment: bidirectional documents and shared questions
    for k, n_docs in enumerate((1, 2, 4, 8, 16, 32, 64, 128)):
        w = Workload(f"sweep-doc-eq{n_docs}", 1, 16, N, 128, BASE_SEED + 700 + k, "document")
        spans = spans_from_lengths([N // n_docs] * n_docs)
        w.structure = [spans]
        w.vectors = [document_mask(N, spans)]
        out.append(w)
    for k in range(n_random // 2):
        w = Workload(f"sweep-doc-rand{k}", 1, 16, N, 128, BASE_SEED + 720 + k, "document")
        rng = _mask_rng(w.seed)
        spans = spans_from_lengths(sample_partition(rng, N, int(rng.integers(2, 65)), 128))
        w.structure = [spans]
        w.vectors = [document_mask(N, spans)]
        out.append(w)
    for k in range(n_random // 2):
        w = Workload(f"sweep-sq{k}", 1, 16, N, 128, BASE_SEED + 740 + k, "shared_question")
        rng = _mask_rng(w.seed)
        f = 2 ** (k % 5)                       # sample sizes from the config-3 recipe up to 16 times that
        samples = sample_shared_question(rng, N, (512 * f, 2048 * f), (256 * f, 1024 * f), (2, 4))
        w.structure = [samples]
        w.vectors = [shared_question_mask(N, samples)]
        out.append(w)
    return out


def paper_table_workloads():
    """The deterministic rows of the paper's kernel-speed tables for head dim 128 (appendix on kernel
    performance): 128K tokens in total, 32 heads, sequence length 8K / 32K / 128K (batch 16 / 4 / 1),
    masks Full, Causal, Sliding window and Prefix-LM.  The paper states neither the window width nor the
    prefix length; its printed FLOPs fit window = N/16 and prefix = N/2 on 128 x 128 accounting tiles."""
    out = []
    for k, N in enumerate((8192, 32768, 131072)):
        B = 131072 // N
        for m, kind in enumerate(("full", "causal", "sliding_window", "prefix_lm")):
            w = Workload(f"table-{kind}-{N // 1024}K", B, 32, N, 128, BASE_SEED + 700 + 10 * k + m, kind)
            if kind == "full":
                st, vec = {}, full_mask(N)
            elif kind == "causal":
                st, vec = {}, causal_mask(N)
            elif kind == "sliding_window":
                st, vec = {"window": N // 16}, sliding_window_mask(N, N // 16)
            else:
                st, vec = {"prefix": N // 2}, prefix_lm_mask(N, N // 2)
            w.structure = [st] * B
            w.vectors = [vec] * B
            out.append(w)
    return out


def small_workload(mask_kind: str, N: int, seed: int, B: int = 1, H: int = 1, d: int = 64) -> Workload:
    """Small seeded case of any mask family, for parity tests."""
    w = Workload(f"small-{mask_kind}-{N}", B, H, N, d, seed, mask_kind)
    rng = _mask_rng(seed)
    for _ in range(B):
        if mask_kind == "full":
            st, vec = {}, full_mask(N)
        elif mask_kind == "causal":
            st, vec = {}, causal_mask(N)
        elif mask_kind == "sliding_window":
            wdt = int(rng.integers(1, max(2, N // 2)))
            st, vec = {"window": wdt}, sliding_window_mask(N, wdt)
        elif mask_kind in ("document", "causal_document"):
            n_docs = int(rng.integers(1, max(1, min(8, N // 8)) + 1))
            spans = spans_from_lengths(sample_partition(rng, N, n_docs, 1))
            st = spans
            vec = document_mask(N, spans) if mask_kind == "document" else causal_document_mask(N, spans)
        elif mask_kind == "shared_question":
            unit = max(N // 16, 2)
            samples = sample_shared_question(rng, N, (unit, 3 * unit), (unit // 2, 2 * unit), (2, 4))
            st, vec = samples, shared_question_mask(N, samples)
        elif mask_kind == "prefix_lm":
            p = int(rng.integers(1, N))
            st, vec = {"prefix": p}, prefix_lm_mask(N, p)
        elif mask_kind == "prefix_document":
            n_docs = int(rng.integers(1, max(1, min(6, N // 8)) + 1))
            docs = []
            for s, e in spans_from_lengths(sample_partition(rng, N, n_docs, 2)):
                docs.append((s, int(rng.integers(s + 1, e + 1)), e))
            st, vec = docs, prefix_document_mask(N, docs)
        elif mask_kind == "global_sliding_window":
            g = int(rng.integers(1, max(2, N // 8)))
            wdt = int(rng.integers(1, max(2, N // 4)))
            st, vec = {"global": g, "window": wdt}, global_sliding_window_mask(N, g, wdt)
        elif mask_kind == "causal_blockwise":
            block = int(rng.integers(2, max(3, N // 6)))
            n_test = int(rng.integers(1, max(2, N // 4)))
            st, vec = {"block": block, "n_test": n_test}, causal_blockwise_mask(N, block, n_test)
        elif mask_kind == "random_eviction":
            evict = np.arange(N) + 1 + rng.integers(0, N, size=N)
            keep = rng.random(N) < 0.5
            evict = np.where(keep, N, evict)
            st, vec = {"evict_at": evict}, random_eviction_mask(N, evict)
        elif mask_kind == "qk_sparse":
            dropped = rng.random(N) < 0.3
            a0 = int(rng.integers(0, N))
            b0 = int(rng.integers(a0, N + 1))
            st = {"dropped_keys": dropped, "q_block": (a0, b0)}
            vec = qk_sparse_mask(N, dropped, (a0, b0))
        elif mask_kind == "random_intervals":
            # arbitrary int32 pairs, including inverted, overlapping and out-of-range ones
            vec = tuple(rng.integers(-N // 4, N + N // 4 + 1, size=N).astype(np.int32) for _ in range(4))
            st = {}
        else:
            raise ValueError(mask_kind)
        w.structure.append(st)
        w.vectors.append(tuple(np.asarray(a, dtype=np.int32) for a in vec))
    return w
