"""Seeded synthetic text for the tokenization pipeline: JSONL documents and a byte-pair merge table.

Stands in for the web-text corpus and the third-party tokenizer tables the paper measures with
(neither is available here).  What is kept of them: documents as one JSON object per line with the
text under one key next to other fields; word frequencies that follow a Zipf law; document lengths
that are log-normal with a long tail (a few words to tens of thousands); mostly ASCII with some
multi-byte UTF-8; punctuation, digits, line breaks, runs of spaces; characters that JSON must escape;
and a merge table learnt from the same word distribution, so that common words become one or two tokens
and rare ones several, as with a trained tokenizer.

This module holds no part of the tokenizer itself (no pre-tokenization, no encoding): it only makes
inputs, for the oracle and the pipeline alike.
"""
from __future__ import annotations

import json
from collections import defaultdict

import numpy as np

_ONSETS = ["", "b", "c", "d", "f", "g", "h", "j", "k", "l", "m", "n", "p", "r", "s", "t", "v", "w", "st", "tr", "ch", "sh", "th", "pl"]
_NUCLEI = ["a", "e", "i", "o", "u", "ai", "ea", "ou", "io", "é", "ü", "ø"]
_CODAS = ["", "", "", "n", "r", "s", "t", "l", "ng", "nd", "st"]
_RARE = ["日本", "данные", "naïve", "😀", "ß", "Ω"]


def make_words(rng: np.random.Generator, n_words: int):
    words, seen = [], set()
    while len(words) < n_words:
        syl = int(rng.integers(1, 5))
        w = "".join(_ONSETS[int(rng.integers(len(_ONSETS)))] + _NUCLEI[int(min(rng.integers(0, 14), len(_NUCLEI) - 1)) if rng.random() < 0.15
                                                                       else int(rng.integers(0, 5))] + _CODAS[int(rng.integers(len(_CODAS)))]
                    for _ in range(syl))
        if rng.random() < 0.01:
            w += _RARE[int(rng.integers(len(_RARE)))]
        if w and w not in seen:
            seen.add(w)
            words.append(w)
    return words


def zipf_probabilities(n: int, exponent: float = 1.1) -> np.ndarray:
    p = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** exponent
    return p / p.sum()


def make_document(rng: np.random.Generator, words, probs, n_words: int) -> str:
    ids = rng.choice(len(words), size=n_words, p=probs)
    out = []
    sentence_left = 0
    for k, wi in enumerate(ids):
        w = words[int(wi)]
        if sentence_left == 0:
            w = w[:1].upper() + w[1:]
            sentence_left = int(rng.integers(4, 25))
        r = rng.random()
        if r < 0.03:
            w = str(int(rng.integers(0, 100000)))
        elif r < 0.04:
            w = '"' + w + '"'
        elif r < 0.045:
            w = w + "\\" + words[int(ids[k - 1])]
        sentence_left -= 1
        sep = " "
        if sentence_left == 0:
            w += ".!?"[int(rng.integers(3))]
            q = rng.random()
            sep = "\n\n" if q < 0.15 else "\n" if q < 0.25 else "  " if q < 0.30 else "\t" if q < 0.32 else " "
        elif rng.random() < 0.08:
            w += ",;:"[int(rng.integers(3))]
        out.append(w)
        out.append(sep)
    return "".join(out[:-1]) if out else ""


def make_jsonl(seed: int, n_docs: int, n_words: int = 5000, median_doc_words: float = 300.0, sigma: float = 1.0,
               max_doc_words: int = 20000) -> bytes:
    """n_docs documents as JSONL bytes (plus a few blank lines and one CRLF line end)."""
    rng = np.random.default_rng(seed)
    words = make_words(rng, n_words)
    probs = zipf_probabilities(n_words)
    lines = []
    for d in range(n_docs):
        nw = 0 if d % 97 == 41 else int(min(max_doc_words, max(1, round(float(rng.lognormal(np.log(median_doc_words), sigma))))))
        text = make_document(rng, words, probs, nw)
        obj = {"id": d, "text": text, "meta": {"text": "not this one", "n": [1, 2.5, None], "ok": True}}
        if d % 5 == 3:
            obj = {"meta": obj["meta"], "url": "http://x/%d" % d, "text": text}
        line = json.dumps(obj, ensure_ascii=(d % 2 == 0), separators=(",", ":") if d % 3 else (", ", ": "))
        lines.append(line.encode("utf-8"))
        if d % 50 == 7:
            lines.append(b"")
        if d % 61 == 9:
            lines.append(b"   ")
    data = b"\n".join(lines) + (b"\n" if n_docs % 2 else b"")
    first = data.find(b"\n")
    if first > 0:
        data = data[:first] + b"\r" + data[first:]      # one CRLF line end
    return data


def train_merges(seed: int, n_merges: int, n_words: int = 2000):
    """Byte-pair training (Sennrich et al. 2016) on the synthetic word distribution: [(left id, right id)]
    with ids 0..255 = bytes and 256 + r = the symbol of merge r.  Words are taken with their leading space."""
    rng = np.random.default_rng(seed)
    words = make_words(rng, n_words)
    freq = np.maximum(1, np.round(zipf_probabilities(n_words) * 1e6)).astype(np.int64)
    syms = [list((" " + w).encode("utf-8")) for w in words]
    counts = defaultdict(int)
    where = defaultdict(set)
    for wi, s in enumerate(syms):
        for a, b in zip(s, s[1:]):
            counts[(a, b)] += int(freq[wi])
            where[(a, b)].add(wi)
    merges = []
    for r in range(n_merges):
        if not counts:
            break
        best = max(counts.items(), key=lambda kv: (kv[1], -kv[0][0], -kv[0][1]))[0]
        if counts[best] <= 0:
            break
        merges.append(best)
        new = 256 + r
        for wi in list(where[best]):
            s = syms[wi]
            f = int(freq[wi])
            for a, b in zip(s, s[1:]):
                counts[(a, b)] -= f
                where[(a, b)].discard(wi)
            t, i = [], 0
            while i < len(s):
                if i + 1 < len(s) and (s[i], s[i + 1]) == best:
                    t.append(new)
                    i += 2
                else:
                    t.append(s[i])
                    i += 1
            syms[wi] = t
            for a, b in zip(t, t[1:]):
                counts[(a, b)] += f
                where[(a, b)].add(wi)
        counts = defaultdict(int, {k: v for k, v in counts.items() if v > 0})
    return merges
