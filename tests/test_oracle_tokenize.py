"""Pins of the tokenization oracle (oracle/tokenize.py) to things other than itself: a hand-worked
example, closed forms, invariants, brute force on tiny inputs and an independent library's byte-pair
model.  CPU only."""
import itertools
import json
import os
import struct

import numpy as np
import pytest

from oracle import tokenize as ot
from synth import text as st

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bpe_hand_worked.txt")


def _golden():
    f = {}
    for line in open(GOLDEN, encoding="utf-8"):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":", 1)
        f[k.strip()] = v.strip("\n")[1:] if v.startswith(" ") else v.strip("\n")
    merges = [tuple(int(x) for x in pair.split()) for pair in f["merges"].split("|")]
    return merges, f["text"].encode(), [int(x) for x in f["tokens"].split()]


def test_hand_worked_example():
    merges, text, tokens = _golden()
    ot.check_merges(merges)
    assert ot.encode(text, merges) == tokens


def test_pretokenization_on_written_out_cases():
    cases = {
        b"Hello  world\n\nfoo, bar42": [b"Hello", b" ", b" world", b"\n\n", b"foo", b",", b" bar", b"42"],
        b" a": [b" a"],
        b"a ": [b"a", b" "],
        b"a   ": [b"a", b"   "],
        b"\t x": [b"\t", b" x"],
        b"x \ny": [b"x", b" \n", b"y"],
        b"3.14 kg": [b"3", b".", b"14", b" kg"],
        b"caf\xc3\xa9!": [b"caf\xc3\xa9", b"!"],
        b" ...": [b" ..."],
        b"": [],
    }
    for text, want in cases.items():
        assert ot.pretokenize(text) == want, text


def test_pieces_partition_the_text_and_long_runs_are_cut():
    rng = np.random.default_rng(3)
    for _ in range(200):
        text = bytes(rng.choice(np.frombuffer(b"ab1 .\n\t\xc3\xa9", np.uint8), size=int(rng.integers(0, 60))).tolist())
        pieces = ot.pretokenize(text)
        assert b"".join(pieces) == text and all(pieces)
    long = b"x" * (2 * ot.MAX_PIECE + 5)
    assert [len(p) for p in ot.pretokenize(b"a " + long)] == [1, ot.MAX_PIECE, ot.MAX_PIECE, 6]   # " x..." is the cut piece


def test_without_merges_the_tokens_are_the_bytes():
    text = "naïve  text\n😀".encode()
    assert ot.encode(text, []) == list(text)


def test_round_trip_and_no_mergeable_pair_is_left():
    merges = st.train_merges(5, 200, 600)
    ranks = {p: r for r, p in enumerate(merges)}
    rng = np.random.default_rng(11)
    data = st.make_jsonl(2, 12, n_words=600, median_doc_words=60)
    texts = [ot.extract_text(data[o:o + n], "text") for o, n in ot.index_jsonl(data)]
    texts.append(bytes(rng.integers(0, 256, 500, dtype=np.uint8).tolist()))       # not even UTF-8
    for text in texts:
        toks = ot.encode(text, merges)
        assert ot.decode(toks, merges) == text
        at = 0
        for piece in ot.pretokenize(text):
            sym = ot.bpe(piece, ranks)
            assert all((a, b) not in ranks for a, b in zip(sym, sym[1:]))
            assert toks[at:at + len(sym)] == sym
            at += len(sym)


def test_bpe_against_brute_force_on_tiny_pieces():
    """On short pieces, the greedy rule's result is re-derived by a search that applies, at every step,
    every occurrence choice of the lowest-rank pair (the rule fixes the pair; leftmost-first and any other
    order must agree when merges are well formed)."""
    merges = [(97, 97), (256, 97), (98, 97), (256, 256), (97, 98)]
    ot.check_merges(merges)
    ranks = {p: r for r, p in enumerate(merges)}

    def all_results(sym):
        pairs = [ranks[(a, b)] for a, b in zip(sym, sym[1:]) if (a, b) in ranks]
        if not pairs:
            return {tuple(sym)}
        best = min(pairs)
        out = set()
        for i, (a, b) in enumerate(zip(sym, sym[1:])):
            if ranks.get((a, b)) == best:
                out |= all_results(sym[:i] + [256 + best] + sym[i + 2:])
        return out

    for n in range(1, 7):
        for piece in itertools.product(b"ab", repeat=n):
            got = tuple(ot.bpe(bytes(piece), ranks))
            res = all_results(list(piece))
            # overlapping occurrences ("aaa") make the order matter; the rule says leftmost
            left = list(piece)
            while True:
                c = [(ranks[(a, b)], i) for i, (a, b) in enumerate(zip(left, left[1:])) if (a, b) in ranks]
                if not c:
                    break
                r, i = min(c)
                left[i:i + 2] = [256 + r]
            assert got == tuple(left) and got in res


def test_bpe_agrees_with_an_independent_library():
    tokenizers = pytest.importorskip("tokenizers")
    merges = st.train_merges(9, 300, 800)
    ch = lambda b: chr(0x100 + b)      # one character per byte value
    table = [ch(b) for b in range(256)]
    for a, b in merges:
        table.append(table[a] + table[b])
    tk = tokenizers.Tokenizer(tokenizers.models.BPE(vocab={s: i for i, s in enumerate(table)},
                                                    merges=[(table[a], table[b]) for a, b in merges]))
    ranks = {p: r for r, p in enumerate(merges)}
    data = st.make_jsonl(4, 6, n_words=800, median_doc_words=80)
    n = 0
    for o, ln in ot.index_jsonl(data):
        for piece in ot.pretokenize(ot.extract_text(data[o:o + ln], "text")):
            assert tk.encode("".join(ch(b) for b in piece)).ids == ot.bpe(piece, ranks), piece
            n += 1
    assert n > 300


def test_json_text_extraction_on_written_out_lines():
    line = r'{"id": 3, "text": "a\"b\\c\n\u00e9\ud83d\ude00é/\/", "meta": {"text": "no"}}'.encode()
    assert ot.extract_text(line, "text") == b'a"b\\c\n\xc3\xa9\xf0\x9f\x98\x80\xc3\xa9//'
    assert ot.extract_text(rb'{"text": "first", "x": 1, "text": "last"}', "text") == b"last"
    assert ot.extract_text(rb'{"text": "\ud800x"}', "text") == b"\xed\xa0\x80x"          # lone surrogate keeps three bytes
    assert ot.extract_text('{"text": "raw é"}'.encode(), "text") == "raw é".encode()
    with pytest.raises(ValueError):
        ot.extract_text(rb'{"text": 5}', "text")
    with pytest.raises(ValueError):
        ot.extract_text(rb'{"body": "x"}', "text")


def test_indexation_finds_the_documents():
    data = b'{"text":"a"}\r\n\n   \n{"text":"b"}\n{"text":"c"}'
    idx = ot.index_jsonl(data)
    assert [data[o:o + n] for o, n in idx] == [b'{"text":"a"}', b'{"text":"b"}', b'{"text":"c"}']
    assert ot.index_jsonl(b"") == [] and ot.index_jsonl(b"\n\n") == []
    raw = ot.jsonl_index_bytes(idx)
    assert raw[:8] == b"MJLINDEX" and struct.unpack("<Q", raw[8:16])[0] == 3
    assert np.frombuffer(raw, "<u8", offset=16).reshape(-1, 2).tolist() == [list(p) for p in idx]


def test_token_file_gives_every_document_back_in_one_step():
    merges = st.train_merges(5, 150, 500)
    data = st.make_jsonl(6, 60, n_words=500, median_doc_words=30)
    docs = ot.tokenize_jsonl(data, merges, "text", eod=256 + len(merges))
    raw = ot.token_file_bytes(docs, 256 + len(merges) + 1)
    tb, index, tokens = ot.read_token_file(raw)
    assert tb == 2 and len(index) == len(docs) + 1 and index[0] == 0 and index[-1] == len(tokens)
    lines = ot.index_jsonl(data)
    for i in (0, 7, 41, 59, 20):
        one = ot.encode(ot.extract_text(data[lines[i][0]:lines[i][0] + lines[i][1]], "text"), merges) + [256 + len(merges)]
        assert tokens[int(index[i]):int(index[i + 1])].tolist() == one
    assert any(len(d) == 1 for d in docs)                 # the generator's empty documents hold only the end id
    wide = ot.token_file_bytes([[70000, 1]], 70001)
    assert ot.read_token_file(wide)[0] == 4 and ot.read_token_file(wide)[2].tolist() == [70000, 1]
    assert len(ot.token_file_bytes([], 10)) == 64 + 8


def test_planted_mistakes_are_caught():
    """A wrong rank order, a right-to-left merge and a dropped leading-space rule each change a pinned result."""
    merges, text, tokens = _golden()
    ranks = {p: r for r, p in enumerate(merges)}
    swapped = {p: (3 if r == 2 else 2 if r == 3 else r) for p, r in ranks.items()}     # " low" before "er"
    assert [t for p in ot.pretokenize(text) for t in ot.bpe(p, swapped)] != tokens
    assert ot.pretokenize(b"a b") == [b"a", b" b"] != [b"a", b" ", b"b"]
