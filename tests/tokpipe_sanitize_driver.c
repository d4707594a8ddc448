/* Driver for the sanitizer builds of the tokenization pipeline: runs indexation and tokenization of the
 * JSONL file named on the command line with several pipeline shapes, checks that all runs produce the same
 * token file, reads documents back through the memory map, and exercises the error paths.  Built with
 * -fsanitize=address,undefined and, separately, -fsanitize=thread by tests/test_tokpipe_sanitizers.py. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "../include/tokpipe.h"

static long file_sum(const char* path, long* size) {
  FILE* f = fopen(path, "rb");
  long s = 0, n = 0;
  int c;
  if (!f) return -1;
  while ((c = fgetc(f)) != EOF) { s = (s * 131 + c) % 1000000007L; ++n; }
  fclose(f);
  *size = n;
  return s;
}

int main(int argc, char** argv) {
  if (argc < 3) { fprintf(stderr, "usage: driver corpus.jsonl workdir\n"); return 2; }
  char idx[1024], out[1024];
  snprintf(idx, sizeof idx, "%s/c.idx", argv[2]);
  snprintf(out, sizeof out, "%s/c.tok", argv[2]);
  /* merges: "lo", "low", "er", " low", " lower" */
  const uint32_t merges[10] = {108, 111, 256, 119, 101, 114, 32, 257, 259, 258};
  const int shapes[4][4] = {{1, 1, 1, 1}, {3, 4, 7, 2}, {8, 6, 1, 64}, {2, 2, 1000, 1}};   /* index threads, workers, batch, depth */
  long first = -1, first_size = 0;
  for (int s = 0; s < 4; ++s) {
    uint64_t n = 0;
    tokpipe_stats st;
    if (tokpipe_index_jsonl(argv[1], idx, shapes[s][0], &n)) { fprintf(stderr, "index: %s\n", tokpipe_last_error()); return 1; }
    if (tokpipe_tokenize(argv[1], idx, out, merges, 5, "text", 261, shapes[s][1], shapes[s][2], shapes[s][3], &st)) {
      fprintf(stderr, "tokenize: %s\n", tokpipe_last_error());
      return 1;
    }
    long size = 0, sum = file_sum(out, &size);
    if (first < 0) { first = sum; first_size = size; }
    if (sum != first || size != first_size || st.n_docs != n) { fprintf(stderr, "shape %d gave another file\n", s); return 1; }
  }
  tokfile* f = tokfile_open(out);
  if (!f) { fprintf(stderr, "open: %s\n", tokpipe_last_error()); return 1; }
  uint64_t total = 0;
  for (uint64_t i = 0; i < tokfile_num_docs(f); ++i) {
    const void* p;
    uint64_t n;
    if (tokfile_doc(f, i, &p, &n)) return 1;
    if (n == 0 || ((const uint16_t*)p)[n - 1] != 261) { fprintf(stderr, "document %llu does not end in the end id\n", (unsigned long long)i); return 1; }
    total += n;
  }
  if (total != tokfile_num_tokens(f) || tokfile_token_bytes(f) != 2) return 1;
  {
    const void* p;
    uint64_t n;
    if (tokfile_doc(f, tokfile_num_docs(f), &p, &n) == 0) return 1;
  }
  tokfile_close(f);
  /* error paths */
  if (tokpipe_tokenize(argv[1], argv[1], out, merges, 5, "text", -1, 2, 2, 2, NULL) == 0) return 1;      /* not an index file */
  if (tokpipe_tokenize(argv[1], idx, out, merges, 5, "no such key", -1, 4, 3, 2, NULL) == 0) return 1;  /* every document fails */
  if (tokpipe_tokenize("/nonexistent", idx, out, merges, 5, "text", -1, 2, 2, 2, NULL) == 0) return 1;
  if (tokpipe_index_jsonl("/nonexistent", idx, 2, NULL) == 0) return 1;
  if (tokfile_open(argv[1]) != NULL) return 1;
  printf("tokpipe driver: all runs agree, %llu tokens\n", (unsigned long long)total);
  return 0;
}
