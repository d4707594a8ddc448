"""Plain CPU oracle for the data pipeline's tokenization stage: JSONL documents -> token file with a
document index (the paper's Data Pipeline paragraph: indexation finds the document boundaries of a
JSONL file, tokenization turns every document into token ids, and the result is one memory-mappable
file whose index gives O(1) access to any tokenized document).

TEST INFRASTRUCTURE ONLY (see oracle/decoder_layer.py for the rules): nothing under the product
package may import this module.  Everything here is sequential, one document at a time, with no
queues, threads, batching or caches: what the producer-consumer pipeline must reproduce byte for
byte.

The paper names its tokenizer (a byte-pair-encoding one shipped by a third party) but not its tables,
and they are not available here.  The reading taken: byte-level byte-pair encoding (Sennrich et al.
2016 over bytes, as in Radford et al. 2019) with a merge table that is an INPUT, and a
pre-tokenization rule stated below in full.

  document text   the string value of one top-level key of the line's JSON object (the last one if the
                  key repeats, as json.loads has it), as UTF-8 bytes; a lone surrogate escape keeps its
                  three-byte form.
  pieces          the text is cut into pieces; byte classes: letter (A-Z, a-z, any byte >= 0x80),
                  digit, space (0x20), other whitespace (\\t \\n \\v \\f \\r), other.  From position i:
                    * a space directly followed by a letter, digit or "other" byte opens a piece made of
                      the space and the maximal run of that following class;
                    * a letter, digit or "other" byte opens the maximal run of its class;
                    * whitespace opens the maximal run of whitespace (both whitespace classes); if that
                      run is longer than one byte, ends in a space and is followed by a
                      non-whitespace byte, the last space is left for the next piece.
                  A piece longer than MAX_PIECE bytes is cut into consecutive chunks of MAX_PIECE.
  byte-pair encoding of a piece: the symbols start as the piece's bytes (ids 0..255); as long as some
                  adjacent pair of symbols is in the merge table, the leftmost occurrence of the pair
                  with the lowest rank is replaced by the symbol 256 + rank.  Merge r may only combine
                  symbols below 256 + r (every table produced by byte-pair training has this form).
  document        the concatenation of its pieces' symbols, followed by the end-of-document id if one
                  is given.

Token file (little endian):
  0   8 bytes  b"MTOKFILE"
  8   u32      version (1)
  12  u32      bytes per token: 2 if every id fits 16 bits, else 4
  16  u64      number of documents n
  24  u64      number of tokens t
  32  u64      byte offset of the index
  40  24 bytes zero
  64  t tokens
  index (at the next multiple of 8): n + 1 u64, index[i] = number of tokens before document i
JSONL index file: b"MJLINDEX", u64 n, then n pairs (u64 byte offset of the line, u64 length without
its line end).  Lines that are empty or hold only whitespace are not documents.
"""
from __future__ import annotations

import json
import struct

import numpy as np

MAX_PIECE = 128
TOKFILE_MAGIC = b"MTOKFILE"
INDEX_MAGIC = b"MJLINDEX"
HEADER_BYTES = 64

_LETTER, _DIGIT, _SPACE, _WS, _OTHER = range(5)


def _cls(b: int) -> int:
    if b >= 0x80 or 0x41 <= b <= 0x5A or 0x61 <= b <= 0x7A:
        return _LETTER
    if 0x30 <= b <= 0x39:
        return _DIGIT
    if b == 0x20:
        return _SPACE
    if 0x09 <= b <= 0x0D:
        return _WS
    return _OTHER


def index_jsonl(data: bytes):
    """[(offset, length)] of the documents (non-blank lines) of a JSONL file's bytes."""
    docs = []
    pos, n = 0, len(data)
    while pos < n:
        end = data.find(b"\n", pos)
        if end < 0:
            end = n
        length = end - pos
        if length and data[end - 1:end] == b"\r":
            length -= 1
        if data[pos:pos + length].strip(b" \t\r\n\v\f"):
            docs.append((pos, length))
        pos = end + 1
    return docs


def extract_text(line: bytes, key: str) -> bytes:
    obj = json.loads(line)
    if not isinstance(obj, dict) or not isinstance(obj.get(key), str):
        raise ValueError(f"no string value under key {key!r}")
    return obj[key].encode("utf-8", "surrogatepass")


def pretokenize(text: bytes):
    pieces = []
    i, n = 0, len(text)
    while i < n:
        c = _cls(text[i])
        if c == _SPACE and i + 1 < n and _cls(text[i + 1]) in (_LETTER, _DIGIT, _OTHER):
            run = _cls(text[i + 1])
            j = i + 1
            while j < n and _cls(text[j]) == run:
                j += 1
        elif c in (_LETTER, _DIGIT, _OTHER):
            j = i
            while j < n and _cls(text[j]) == c:
                j += 1
        else:
            j = i
            while j < n and _cls(text[j]) in (_SPACE, _WS):
                j += 1
            if j - i > 1 and j < n and text[j - 1] == 0x20:
                j -= 1
        for k in range(i, j, MAX_PIECE):
            pieces.append(text[k:min(j, k + MAX_PIECE)])
        i = j
    return pieces


def check_merges(merges) -> None:
    seen = set()
    for r, (a, b) in enumerate(merges):
        if not (0 <= a < 256 + r and 0 <= b < 256 + r):
            raise ValueError(f"merge {r} combines a symbol that does not exist yet")
        if (a, b) in seen:
            raise ValueError(f"merge {r} repeats an earlier pair")
        seen.add((a, b))


def bpe(piece: bytes, ranks) -> list:
    """ranks: {(left id, right id): rank}."""
    sym = list(piece)
    while len(sym) > 1:
        best, at = None, -1
        for i in range(len(sym) - 1):
            r = ranks.get((sym[i], sym[i + 1]))
            if r is not None and (best is None or r < best):
                best, at = r, i
        if best is None:
            break
        sym[at:at + 2] = [256 + best]
    return sym


def encode(text: bytes, merges) -> list:
    ranks = {(int(a), int(b)): r for r, (a, b) in enumerate(merges)}
    out = []
    for piece in pretokenize(text):
        out.extend(bpe(piece, ranks))
    return out


def tokenize_jsonl(data: bytes, merges, key: str = "text", eod: int = -1):
    """Token lists of all documents of a JSONL file's bytes, in file order."""
    check_merges(merges)
    docs = []
    for off, length in index_jsonl(data):
        toks = encode(extract_text(data[off:off + length], key), merges)
        if eod >= 0:
            toks.append(eod)
        docs.append(toks)
    return docs


def token_file_bytes(docs, vocab_size: int) -> bytes:
    """The token file of a list of token lists; vocab_size = largest id + 1 that may occur."""
    tb = 2 if vocab_size <= 65536 else 4
    flat = np.concatenate([np.asarray(d, np.int64) for d in docs]) if docs else np.zeros(0, np.int64)
    index = np.zeros(len(docs) + 1, np.uint64)
    index[1:] = np.cumsum([len(d) for d in docs], dtype=np.uint64) if docs else []
    tokens = flat.astype("<u2" if tb == 2 else "<u4").tobytes()
    index_off = (HEADER_BYTES + len(tokens) + 7) // 8 * 8
    head = TOKFILE_MAGIC + struct.pack("<IIQQQ", 1, tb, len(docs), int(flat.size), index_off) + bytes(24)
    return head + tokens + bytes(index_off - HEADER_BYTES - len(tokens)) + index.astype("<u8").tobytes()


def jsonl_index_bytes(docs) -> bytes:
    flat = np.asarray(docs, np.uint64).reshape(-1)
    return INDEX_MAGIC + struct.pack("<Q", len(docs)) + flat.astype("<u8").tobytes()


def read_token_file(raw: bytes):
    """(bytes per token, index array, tokens array) of a token file's bytes."""
    assert raw[:8] == TOKFILE_MAGIC, "not a token file"
    version, tb, n, t, index_off = struct.unpack("<IIQQQ", raw[8:40])
    assert version == 1 and tb in (2, 4)
    tokens = np.frombuffer(raw, "<u2" if tb == 2 else "<u4", count=t, offset=HEADER_BYTES)
    index = np.frombuffer(raw, "<u8", count=n + 1, offset=index_off)
    return tb, index, tokens


def decode(tokens, merges) -> bytes:
    """Bytes a token sequence stands for (end-of-document ids must be removed by the caller)."""
    table = [bytes([b]) for b in range(256)]
    for a, b in merges:
        table.append(table[a] + table[b])
    return b"".join(table[int(t)] for t in tokens)
