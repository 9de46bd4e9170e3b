"""CPU oracle for the example-based drafter (paper Sec. 4.3): per-query n-gram lookup table,
draft generation, selective fallback, and the decode loop around greedy verification.
TEST INFRASTRUCTURE ONLY - never imported by the product path.

What the paper fixes: a window of n consecutive tokens slides over one token stream (few-shot
examples followed by the user query), one token at a time; each window records (first n-1
tokens -> n-th token); the table maps a key to the next token that occurs most often with it.
A draft is the table's answer to the n-1 most recent tokens, repeated (each draft becomes part
of the context) up to the draft length.  If the FIRST lookup of a round misses, selective
decoding skips speculation and decodes one token normally; after a first hit the remaining
drafts of the group are produced regardless of later misses, a miss yielding a "random" token.

Readings where the paper is silent: ties between equally frequent next tokens go to the one
recorded first; the "random" token is splitmix64(seed + index of the token in the generated
stream) mod vocab (any value works: it is only ever a wrong guess, verification decides).
"""
from __future__ import annotations

from . import decoder as O

MASK = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """The splitmix64 output function of counter x (public-domain generator by S. Vigna)."""
    z = (x + 0x9E3779B97F4A7C15) & MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def build_lut(stream, n: int) -> dict:
    """{tuple of n-1 tokens: most frequent next token (earliest recorded on ties)}."""
    assert n >= 1
    counts: dict = {}
    for i in range(len(stream) - n + 1):
        key = tuple(int(t) for t in stream[i:i + n - 1])
        nxt = int(stream[i + n - 1])
        c = counts.setdefault(key, {})            # dict keeps first-seen order
        c[nxt] = c.get(nxt, 0) + 1
    lut = {}
    for key, c in counts.items():
        best, best_n = None, 0
        for tok, cnt in c.items():                # first-seen order: strict > keeps the earliest
            if cnt > best_n:
                best, best_n = tok, cnt
        lut[key] = best
    return lut


def draft(lut: dict, n: int, context, k: int, selective: bool, vocab: int, seed: int, stream_pos: int):
    """Up to k drafts after `context` (most recent token last).  Returns (drafts, n_hits).
    Selective mode returns no drafts when the first lookup misses."""
    ctx = [int(t) for t in context]
    out, hits = [], 0
    for i in range(k):
        key = tuple(ctx[len(ctx) - (n - 1):]) if n > 1 else ()
        tok = lut.get(key) if len(ctx) >= n - 1 else None
        if tok is None:
            if i == 0 and selective:
                return [], 0
            tok = splitmix64((seed + stream_pos + i) & MASK) % vocab
        else:
            hits += 1
        out.append(tok)
        ctx.append(tok)
    return out, hits


def draft_accuracy(stats: dict) -> float:
    """Draft-token accuracy as the paper's Table 3 tabulates it: accepted drafts over generated
    drafts (0 when nothing was drafted)."""
    return stats["accepted"] / stats["drafted"] if stats["drafted"] else 0.0


def generate(shape, weights, kv, lut: dict, n: int, history, pending: int, max_new: int, k: int,
             selective: bool, seed: int = 0):
    """ExSpec decode loop: draft from the table, verify with the target model, roll back.

    `history`: tokens before `pending` that the drafter may use as context (the prompt tail).
    Emits max_new tokens after `pending`.  Returns (tokens, stats) with stats = dict(rounds,
    fallbacks, drafted, accepted): fallbacks counts rounds decoded without speculation,
    accuracy = accepted / drafted as in the paper's Table 3.
    """
    ctx = [int(t) for t in history] + [int(pending)]
    out = []
    st = dict(rounds=0, fallbacks=0, drafted=0, accepted=0)
    while len(out) < max_new:
        kk = min(k, max_new - len(out) - 1)        # never draft past the requested length
        d, _ = draft(lut, n, ctx, kk, selective, shape.vocab, seed, len(out)) if kk > 0 else ([], 0)
        if not d:
            st["fallbacks"] += 1
        a, nxt, _ = O.verify(shape, weights, kv, pending, d)
        st["rounds"] += 1
        st["drafted"] += len(d)
        st["accepted"] += a
        new = d[:a] + [nxt]
        out += new
        ctx += new
        pending = nxt
    return out, st
