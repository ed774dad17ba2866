"""Defining predicates of the mask families (Section 2.1 prose), written
directly as allowed(i, j) on the task structure.  Independent of the vector
builders in workloads.py and of the oracle: the tests expand the vectors with
the oracle and compare against these by brute force."""


def _doc_of(spans, x):
    for s, e in spans:
        if s <= x < e:
            return (s, e)
    raise AssertionError("token outside every span")


def full(i, j, st):
    return True


def causal(i, j, st):
    return j <= i


def sliding_window(i, j, st):
    return 0 <= i - j < st["window"]


def document(i, j, st):
    return _doc_of(st, i) == _doc_of(st, j)


def causal_document(i, j, st):
    return j <= i and _doc_of(st, i) == _doc_of(st, j)


def shared_question(i, j, st):
    def locate(x):
        for s, starts, e in st:
            if s <= x < e:
                if not starts or x < starts[0]:
                    return (s, e), -1           # question (or plain document)
                part = max(m for m, a in enumerate(starts) if a <= x)
                return (s, e), part
        raise AssertionError
    (si, pi), (sj, pj) = locate(i), locate(j)
    if si != sj or j > i:
        return False
    return pj == -1 or pi == pj


def prefix_lm(i, j, st):
    return j <= i or j < st["prefix"]


def prefix_document(i, j, st):
    for s, p, e in st:
        if s <= i < e:
            return s <= j < e and (j <= i or j < p)
    raise AssertionError


def global_sliding_window(i, j, st):
    g, w = st["global"], st["window"]
    return abs(i - j) < w or i < g or j < g


def causal_blockwise(i, j, st):
    block, n_test = st["block"], st["n_test"]
    if j > i:
        return False
    return True if i >= st["N"] - n_test else (i // block - j // block) <= 1


def random_eviction(i, j, st):
    return j <= i and i < max(int(st["evict_at"][j]), j + 1)


def qk_sparse(i, j, st):
    a, b = st["q_block"]
    return j <= i and not st["dropped_keys"][j] and not (a <= i < b)


PREDICATES = {
    "full": full, "causal": causal, "sliding_window": sliding_window,
    "document": document, "causal_document": causal_document,
    "shared_question": shared_question, "prefix_lm": prefix_lm,
    "prefix_document": prefix_document, "global_sliding_window": global_sliding_window,
    "causal_blockwise": causal_blockwise, "random_eviction": random_eviction, "qk_sparse": qk_sparse,
}
