"""Parity of the tokenization pipeline (C ABI of include/tokpipe.h, a CPU library) with the sequential
oracle: byte-identical index and token files on seeded synthetic JSONL, whatever the thread counts,
batch sizes and queue depths; O(1) document access through the memory map; error paths."""
import os
import re

import numpy as np
import pytest

from oracle import tokenize as ot
from paper_2602_08387_amd import tokpipe as tp
from synth import text as st

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "tokpipe.h")


def test_header_symbols_are_exported_and_bound():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    declared = set(re.findall(r"\b(tok(?:pipe|file)_\w+)\s*\(", text))
    assert declared == set(tp.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(tp.lib, name), name


def _run(tmp_path, data, merges, eod, **kw):
    src, idx, out = tmp_path / "in.jsonl", tmp_path / "in.idx", tmp_path / "out.tok"
    src.write_bytes(data)
    n = tp.index_jsonl(src, idx, kw.pop("index_threads", 1))
    stats = tp.tokenize(src, idx, out, merges, "text", eod, **kw)
    return n, idx.read_bytes(), out.read_bytes(), stats, out


@pytest.mark.parametrize("seed,n_docs,n_merges,eod", [(0, 120, 400, 656), (1, 37, 0, -1), (2, 64, 150, 0)])
def test_files_match_the_oracle_byte_for_byte(tmp_path, seed, n_docs, n_merges, eod):
    data = st.make_jsonl(seed, n_docs, n_words=1500, median_doc_words=120)
    merges = st.train_merges(seed, n_merges, 1200) if n_merges else []
    docs = ot.tokenize_jsonl(data, merges, "text", eod)
    want_idx = ot.jsonl_index_bytes(ot.index_jsonl(data))
    want_tok = ot.token_file_bytes(docs, max(256 + len(merges), eod + 1))
    results = set()
    for kw in (dict(n_workers=1, batch_docs=1, queue_depth=1), dict(n_workers=4, batch_docs=7, queue_depth=3, index_threads=3),
               dict(n_workers=8, batch_docs=1000, queue_depth=2), dict(n_workers=3, batch_docs=2, queue_depth=64, index_threads=8)):
        n, idx, tok, stats, _ = _run(tmp_path, data, merges, eod, **kw)
        assert n == len(docs) == stats.n_docs and stats.n_tokens == sum(map(len, docs))
        assert idx == want_idx
        assert tok == want_tok
        results.add(tok)
    assert len(results) == 1


def test_wide_tokens_and_document_access(tmp_path):
    data = st.make_jsonl(5, 80, n_words=800, median_doc_words=40)
    merges = st.train_merges(5, 100, 600)
    eod = 70000                                     # forces 4-byte tokens
    docs = ot.tokenize_jsonl(data, merges, "text", eod)
    _, _, tok, _, path = _run(tmp_path, data, merges, eod, n_workers=2, batch_docs=5)
    assert tok == ot.token_file_bytes(docs, eod + 1)
    with tp.TokenFile(path) as f:
        assert (f.num_docs, f.num_tokens, f.token_bytes) == (len(docs), sum(map(len, docs)), 4)
        for i in (79, 0, 41, 13):
            assert f.doc(i).tolist() == docs[i]
        with pytest.raises(tp.TokPipeError):
            f.doc(80)


def test_multithreaded_indexation_of_a_file_with_awkward_line_ends(tmp_path):
    rng = np.random.default_rng(0)
    lines = []
    for i in range(3000):
        lines.append(b'{"text":"%s"}' % (b"x" * int(rng.integers(0, 40))))
        if i % 7 == 0:
            lines.append(b"" if i % 2 else b" \t ")
    data = b"\r\n".join(lines)
    src, idx = tmp_path / "a.jsonl", tmp_path / "a.idx"
    src.write_bytes(data)
    want = ot.jsonl_index_bytes(ot.index_jsonl(data))
    for threads in (1, 2, 5, 16):
        assert tp.index_jsonl(src, idx, threads) == 3000
        assert idx.read_bytes() == want
    src.write_bytes(b"")
    assert tp.index_jsonl(src, idx, 4) == 0 and idx.read_bytes() == ot.jsonl_index_bytes([])
    out = tmp_path / "e.tok"
    tp.tokenize(src, idx, out, [], "text", -1, 2, 4, 2)
    assert out.read_bytes() == ot.token_file_bytes([], 256)


def test_json_corner_cases_against_the_oracle(tmp_path):
    lines = [
        r'{"id": 3, "text": "a\"b\\c\né😀é/\/\b\f\r\t", "meta": {"text": "no", "a": [1, {"text": "x"}]}}',
        r'{"text": "first", "x": [1, 2, {"y": "}"}], "text": "last one"}',
        r'{"text": "\ud800 lone and \udc00\ud83d pair-less"}',
        r'{ "a" : null , "b" : -1.5e3 , "c" : true , "text" : "spaced   out" }',
        r'{"text": ""}',
        '{"text": "' + "long" * 5000 + " x" * 3000 + '"}',
    ]
    data = "\n".join(lines).encode()
    merges = st.train_merges(3, 80, 400)
    docs = ot.tokenize_jsonl(data, merges, "text", 999)
    _, _, tok, _, _ = _run(tmp_path, data, merges, 999, n_workers=2, batch_docs=2)
    assert tok == ot.token_file_bytes(docs, 1000)


def test_errors_name_the_document_and_leave_no_hang(tmp_path):
    good = b'{"text": "ok"}'
    for bad, what in ((b'{"text": 5}', "no string member"), (b'{"body": "x"}', "no string member"), (b'["text"]', "not a JSON object"),
                      (b'{"text": "unterminated}', "not a JSON object")):
        data = b"\n".join([good] * 40 + [bad] + [good] * 40)
        src, idx, out = tmp_path / "b.jsonl", tmp_path / "b.idx", tmp_path / "b.tok"
        src.write_bytes(data)
        tp.index_jsonl(src, idx, 2)
        with pytest.raises(tp.TokPipeError, match=f"document 40.*{what}|{what}.*document 40|document 40"):
            tp.tokenize(src, idx, out, [], "text", -1, 4, 3, 2)
    with pytest.raises(tp.TokPipeError):
        tp.tokenize(tmp_path / "missing.jsonl", tmp_path / "b.idx", tmp_path / "o", [], "text")
    with pytest.raises(tp.TokPipeError):
        tp.tokenize(tmp_path / "b.jsonl", tmp_path / "b.jsonl", tmp_path / "o", [], "text")      # not an index file
    with pytest.raises(tp.TokPipeError):
        tp.tokenize(tmp_path / "b.jsonl", tmp_path / "b.idx", tmp_path / "o", [(300, 1)], "text")   # symbol 300 does not exist yet
    with pytest.raises(tp.TokPipeError):
        tp.tokenize(tmp_path / "b.jsonl", tmp_path / "b.idx", tmp_path / "o", [(1, 2), (1, 2)], "text")
    with pytest.raises(tp.TokPipeError):
        tp.tokenize(tmp_path / "b.jsonl", tmp_path / "b.idx", tmp_path / "o", [], "text", n_workers=0)
    with pytest.raises(tp.TokPipeError):
        tp.TokenFile(tmp_path / "b.jsonl")


def test_corrupt_index_and_token_files_are_rejected(tmp_path):
    """Counts and offsets in a file header are untrusted: values chosen so that count * size wraps around
    64 bits, or so that a range ends past the file, must give an error, never a crash or a huge allocation."""
    import struct
    src, idx, out = tmp_path / "c.jsonl", tmp_path / "c.idx", tmp_path / "c.tok"
    src.write_bytes(b'{"text": "one two"}\n{"text": "three"}\n')
    tp.index_jsonl(src, idx, 1)
    tp.tokenize(src, idx, out, [], "text", -1)
    good_idx, good_tok = idx.read_bytes(), out.read_bytes()
    # index: a document count whose byte size wraps to the true payload size; an entry past the end of the file;
    # an offset + length that wraps; entries out of order
    n = struct.unpack("<Q", good_idx[8:16])[0]
    cases = [
        good_idx[:8] + struct.pack("<Q", n + (1 << 60)) + good_idx[16:],
        good_idx[:16] + struct.pack("<QQ", 0, 1 << 40) + good_idx[32:],
        good_idx[:16] + struct.pack("<QQ", (1 << 64) - 4, 8) + good_idx[32:],
        good_idx[:16] + good_idx[32:48] + good_idx[16:32],
    ]
    for raw in cases:
        bad = tmp_path / "bad.idx"
        bad.write_bytes(raw)
        with pytest.raises(tp.TokPipeError):
            tp.tokenize(src, bad, tmp_path / "o.tok", [], "text", -1)
    # token file: header fields 16 (documents), 24 (tokens), 32 (index offset)
    def patched(at, value):
        return good_tok[:at] + struct.pack("<Q", value) + good_tok[at + 8:]
    for raw in (patched(16, (1 << 61) - 1), patched(16, 3), patched(24, 1 << 63), patched(24, 1 << 40),
                patched(32, 8), patched(32, len(good_tok) + 8), patched(32, 1 << 62), good_tok[:40]):
        bad = tmp_path / "bad.tok"
        bad.write_bytes(raw)
        with pytest.raises(tp.TokPipeError):
            tp.TokenFile(bad)
    with tp.TokenFile(out) as f:                       # the untouched file still opens
        assert f.num_docs == 2
