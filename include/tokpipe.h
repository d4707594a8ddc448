/* C ABI of the tokenization stage of the data pipeline (host code only, no GPU involved).
 *
 * What it computes is fixed by the paper's Data Pipeline paragraph: a JSONL file is indexed (the byte
 * range of every document = line), every document's text is tokenized, and the result is ONE file
 * that can be memory-mapped and whose document index gives any tokenized document in O(1).
 * Tokenization runs as a producer-consumer pipeline: a single reader that reads runs of consecutive
 * documents with one read each, bounded queues that carry batches of documents, a configurable number
 * of tokenizer workers, and a single writer that appends the batches in document order.
 *
 * The tokenizer (the paper's is a third party's byte-pair encoder whose tables are not part of the
 * paper) is byte-level byte-pair encoding with the merge table as an argument:
 *   text     the string value of the LAST top-level member named `key` of the line's JSON object, as
 *            UTF-8 (escapes decoded, surrogate pairs combined, a lone surrogate escape as its
 *            three-byte form); it is an error if that member is missing or not a string.
 *   pieces   byte classes: letter (A-Z, a-z, bytes >= 0x80), digit, space (0x20), other whitespace
 *            (0x09..0x0d), other.  From position i: a space directly followed by a letter, digit or
 *            "other" byte opens a piece of the space plus the maximal run of that class; a letter, digit
 *            or "other" byte opens the maximal run of its class; whitespace opens the maximal whitespace
 *            run, whose last byte is left to the next piece if the run is longer than one byte, ends in
 *            a space and a non-whitespace byte follows.  Pieces longer than 128 bytes are cut into
 *            consecutive chunks of 128.
 *   merging  symbols start as the piece's bytes (ids 0..255); while some adjacent pair is in the merge
 *            table, the leftmost occurrence of the pair of lowest rank r becomes the symbol 256 + r.
 *   document = its pieces' symbols in order, then `eod_token` if that is >= 0.
 *
 * Token file, little endian: bytes 0..7 "MTOKFILE"; u32 version = 1; u32 bytes per token (2 if
 * max(256 + n_merges, eod_token + 1) <= 65536, else 4); u64 documents n; u64 tokens t; u64 byte offset
 * of the index; 24 zero bytes; at 64 the t tokens; at the next multiple of 8 the index: n + 1 u64,
 * index[i] = tokens before document i.
 * JSONL index file: bytes 0..7 "MJLINDEX"; u64 n; n pairs (u64 byte offset of the line, u64 length
 * without its line end).  Lines that are empty or all whitespace are not documents.
 *
 * All functions return 0 on success and a negative value on error (tokpipe_last_error() then
 * describes it; the string belongs to the library and is per thread).  Paths are NUL-terminated; output
 * files are created or overwritten; nothing is kept open or allocated after a call returns.
 */
#ifndef TOKPIPE_H
#define TOKPIPE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

const char* tokpipe_last_error(void);

/* Indexation: finds the documents of `jsonl_path` with n_threads threads, each scanning one contiguous
 * part of the file, and writes the JSONL index file.  *n_docs (may be NULL) receives their number.  */
int tokpipe_index_jsonl(const char* jsonl_path, const char* index_path, int n_threads, uint64_t* n_docs);

typedef struct {
  uint64_t n_docs;         /* documents written */
  uint64_t n_tokens;       /* tokens written, end-of-document ids included */
  uint64_t bytes_read;     /* bytes of JSONL read by the reader */
  double seconds;          /* wall-clock time of the call */
  uint64_t cache_hits;     /* pieces served from the workers' piece caches ... */
  uint64_t cache_misses;   /* ... and pieces merged from scratch */
} tokpipe_stats;

/* Tokenization of the documents listed in `index_path` (as written by tokpipe_index_jsonl for
 * `jsonl_path`) into the token file `out_path`.
 *   merges      host array [n_merges][2] of symbol ids; merge r may only name symbols < 256 + r and no
 *               pair may repeat (checked)
 *   key         name of the JSON member holding the text
 *   eod_token   id appended to every document, or < 0 for none
 *   n_workers   tokenizer threads (>= 1); batch_docs: documents per queue entry (>= 1);
 *   queue_depth entries the reader may be ahead of the workers (>= 1); batches in flight, and with
 *               them memory, are bounded by queue_depth + n_workers
 * The result does not depend on n_workers, batch_docs or queue_depth.  stats may be NULL.
 * On error (unreadable file, a line that is not a JSON object with a string under `key` - the message
 * names the document) the output file is left incomplete and must not be used.                     */
int tokpipe_tokenize(const char* jsonl_path, const char* index_path, const char* out_path,
                     const uint32_t* merges, uint32_t n_merges, const char* key, int64_t eod_token,
                     int n_workers, int batch_docs, int queue_depth, tokpipe_stats* stats);

/* Read access to a token file through a memory map.  tokfile_open returns NULL on error.  The pointer
 * tokfile_doc hands out points into the map (tokfile_token_bytes() bytes per token, little endian) and
 * is valid until tokfile_close.                                                                     */
typedef struct tokfile tokfile;
tokfile* tokfile_open(const char* path);
void tokfile_close(tokfile* f);
uint64_t tokfile_num_docs(const tokfile* f);
uint64_t tokfile_num_tokens(const tokfile* f);
uint32_t tokfile_token_bytes(const tokfile* f);
int tokfile_doc(const tokfile* f, uint64_t i, const void** tokens, uint64_t* n_tokens);

#ifdef __cplusplus
}
#endif
#endif /* TOKPIPE_H */
