// Tokenization stage of the data pipeline (Data Pipeline paragraph of the paper): JSONL indexation and
// a producer-consumer tokenizer that writes one memory-mappable token file with a document index.
// Host code only.  Formats and the tokenizer's rules are stated in include/tokpipe.h.
//
// Threads of tokpipe_tokenize:
//   reader   walks the index in batches of consecutive documents, one pread per batch (the documents
//            of a batch are contiguous in the file), and queues the batches
//   workers  take a batch, decode each line's text, cut it into pieces, merge byte pairs (through a
//            per-worker cache of pieces already seen: natural text repeats its words) and hand the
//            batch's tokens and document lengths to the writer
//   writer   reorders finished batches by their number and appends them to the file; it also returns
//            the tickets that bound the batches in flight
#include "../../include/tokpipe.h"

#include <fcntl.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

namespace {

thread_local char g_err[512] = "";

int fail(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return -1;
}

constexpr char kTokMagic[9] = "MTOKFILE";
constexpr char kIdxMagic[9] = "MJLINDEX";
constexpr size_t kHeader = 64;
constexpr int kMaxPiece = 128;

struct Span { uint64_t off, len; };

// ------------------------------------------------------------------------------------------ files
struct Mapped {
  const unsigned char* p = nullptr;
  size_t n = 0;
  int fd = -1;
  bool open(const char* path) {
    fd = ::open(path, O_RDONLY);
    if (fd < 0) return false;
    struct stat st;
    if (fstat(fd, &st) != 0) return false;
    n = (size_t)st.st_size;
    if (n == 0) return true;
    void* m = mmap(nullptr, n, PROT_READ, MAP_PRIVATE, fd, 0);
    if (m == MAP_FAILED) return false;
    p = (const unsigned char*)m;
    return true;
  }
  ~Mapped() {
    if (p) munmap((void*)p, n);
    if (fd >= 0) ::close(fd);
  }
};

bool write_all(int fd, const void* data, size_t n) {
  const char* c = (const char*)data;
  while (n) {
    const ssize_t w = ::write(fd, c, n);
    if (w < 0) return false;
    c += w;
    n -= (size_t)w;
  }
  return true;
}

inline bool is_ws(unsigned char b) { return b == 0x20 || (b >= 0x09 && b <= 0x0d); }

// documents (non-blank lines) that START in [lo, hi)
void scan_lines(const unsigned char* p, size_t n, size_t lo, size_t hi, std::vector<Span>& out) {
  size_t pos = lo;
  if (lo > 0) {
    const void* nl = memchr(p + lo - 1, '\n', n - (lo - 1));
    if (!nl) return;
    pos = (size_t)((const unsigned char*)nl - p) + 1;
  }
  while (pos < hi && pos < n) {
    const void* nl = memchr(p + pos, '\n', n - pos);
    const size_t end = nl ? (size_t)((const unsigned char*)nl - p) : n;
    size_t len = end - pos;
    if (len && p[end - 1] == '\r') --len;
    bool blank = true;
    for (size_t i = 0; i < len && blank; ++i) blank = is_ws(p[pos + i]);
    if (!blank) out.push_back({pos, len});
    pos = end + 1;
  }
}

bool load_index(const char* path, std::vector<Span>& docs) {
  Mapped m;
  if (!m.open(path) || m.n < 16 || memcmp(m.p, kIdxMagic, 8) != 0) return false;
  uint64_t n;
  memcpy(&n, m.p + 8, 8);
  if (n > (m.n - 16) / 16 || m.n != 16 + n * 16) return false;   // the first test keeps n * 16 from wrapping
  docs.resize(n);
  if (n) memcpy(docs.data(), m.p + 16, n * 16);
  return true;
}

// ------------------------------------------------------------------------------------------ JSON
struct JsonLine {
  const unsigned char* p;
  size_t n, i = 0;
  void ws() { while (i < n && (p[i] == ' ' || p[i] == '\t' || p[i] == '\n' || p[i] == '\r')) ++i; }
  static int hex4(const unsigned char* q) {
    int v = 0;
    for (int k = 0; k < 4; ++k) {
      const unsigned char c = q[k];
      int d = c >= '0' && c <= '9' ? c - '0' : c >= 'a' && c <= 'f' ? c - 'a' + 10 : c >= 'A' && c <= 'F' ? c - 'A' + 10 : -1;
      if (d < 0) return -1;
      v = v * 16 + d;
    }
    return v;
  }
  static void utf8(uint32_t c, std::string& out) {
    if (c < 0x80) out.push_back((char)c);
    else if (c < 0x800) { out.push_back((char)(0xC0 | (c >> 6))); out.push_back((char)(0x80 | (c & 63))); }
    else if (c < 0x10000) { out.push_back((char)(0xE0 | (c >> 12))); out.push_back((char)(0x80 | ((c >> 6) & 63))); out.push_back((char)(0x80 | (c & 63))); }
    else { out.push_back((char)(0xF0 | (c >> 18))); out.push_back((char)(0x80 | ((c >> 12) & 63))); out.push_back((char)(0x80 | ((c >> 6) & 63))); out.push_back((char)(0x80 | (c & 63))); }
  }
  // at an opening quote: decodes (out != nullptr) or skips the string; false on malformed input
  bool string(std::string* out) {
    if (i >= n || p[i] != '"') return false;
    ++i;
    if (out) out->clear();
    while (i < n) {
      // plain run
      size_t j = i;
      while (j < n && p[j] != '"' && p[j] != '\\') ++j;
      if (out && j > i) out->append((const char*)p + i, j - i);
      i = j;
      if (i >= n) return false;
      if (p[i] == '"') { ++i; return true; }
      if (++i >= n) return false;     // backslash
      const unsigned char e = p[i++];
      char c;
      switch (e) {
        case '"': c = '"'; break;
        case '\\': c = '\\'; break;
        case '/': c = '/'; break;
        case 'b': c = '\b'; break;
        case 'f': c = '\f'; break;
        case 'n': c = '\n'; break;
        case 'r': c = '\r'; break;
        case 't': c = '\t'; break;
        case 'u': {
          if (i + 4 > n) return false;
          int u = hex4(p + i);
          if (u < 0) return false;
          i += 4;
          uint32_t cp = (uint32_t)u;
          if (u >= 0xD800 && u <= 0xDBFF && i + 6 <= n && p[i] == '\\' && p[i + 1] == 'u') {
            const int lo = hex4(p + i + 2);
            if (lo >= 0xDC00 && lo <= 0xDFFF) {
              cp = 0x10000 + (((uint32_t)u - 0xD800) << 10) + ((uint32_t)lo - 0xDC00);
              i += 6;
            }
          }
          if (out) utf8(cp, *out);
          continue;
        }
        default: return false;
      }
      if (out) out->push_back(c);
    }
    return false;
  }
  bool skip_value() {
    ws();
    if (i >= n) return false;
    if (p[i] == '"') return string(nullptr);
    if (p[i] == '{' || p[i] == '[') {
      int depth = 0;
      while (i < n) {
        const unsigned char c = p[i];
        if (c == '"') { if (!string(nullptr)) return false; continue; }
        if (c == '{' || c == '[') ++depth;
        else if (c == '}' || c == ']') { if (--depth == 0) { ++i; return true; } }
        ++i;
      }
      return false;
    }
    const size_t start = i;
    while (i < n && p[i] != ',' && p[i] != '}' && p[i] != ']' && !is_ws(p[i])) ++i;
    return i > start;
  }
};

// text of the last top-level member `key`; 0 ok, 1 malformed line, 2 member missing or not a string
int extract_text(const unsigned char* line, size_t n, const std::string& key, std::string& name, std::string& text) {
  JsonLine j{line, n};
  j.ws();
  if (j.i >= n || line[j.i] != '{') return 1;
  ++j.i;
  int state = 2;
  j.ws();
  if (j.i < n && line[j.i] == '}') { ++j.i; }
  else {
    for (;;) {
      j.ws();
      if (!j.string(&name)) return 1;
      j.ws();
      if (j.i >= n || line[j.i] != ':') return 1;
      ++j.i;
      j.ws();
      if (name == key) {
        if (j.i < n && line[j.i] == '"') {
          if (!j.string(&text)) return 1;
          state = 0;
        } else {
          if (!j.skip_value()) return 1;
          state = 2;
        }
      } else if (!j.skip_value()) return 1;
      j.ws();
      if (j.i < n && line[j.i] == ',') { ++j.i; continue; }
      if (j.i < n && line[j.i] == '}') { ++j.i; break; }
      return 1;
    }
  }
  j.ws();
  if (j.i != n) return 1;
  return state;
}

// ------------------------------------------------------------------------------------------ tokenizer
enum { LETTER, DIGIT, SPACE, WS, OTHER };
inline int cls(unsigned char b) {
  if (b >= 0x80 || (b >= 'A' && b <= 'Z') || (b >= 'a' && b <= 'z')) return LETTER;
  if (b >= '0' && b <= '9') return DIGIT;
  if (b == 0x20) return SPACE;
  if (b >= 0x09 && b <= 0x0d) return WS;
  return OTHER;
}

// pair (a, b) -> rank, open addressing
struct MergeTable {
  std::vector<uint64_t> keys;
  std::vector<uint32_t> vals;
  uint64_t mask = 0;
  static uint64_t mix(uint64_t k) { k *= 0x9E3779B97F4A7C15ull; return k ^ (k >> 29); }
  void build(const uint32_t* merges, uint32_t n) {
    uint64_t cap = 64;
    while (cap < 4ull * (n + 1)) cap <<= 1;
    keys.assign(cap, ~0ull);
    vals.assign(cap, 0);
    mask = cap - 1;
    for (uint32_t r = 0; r < n; ++r) {
      const uint64_t k = ((uint64_t)merges[2 * r] << 32) | merges[2 * r + 1];
      uint64_t h = mix(k) & mask;
      while (keys[h] != ~0ull) h = (h + 1) & mask;
      keys[h] = k;
      vals[h] = r;
    }
  }
  // rank of (a, b) or UINT32_MAX
  uint32_t rank(uint32_t a, uint32_t b) const {
    const uint64_t k = ((uint64_t)a << 32) | b;
    uint64_t h = mix(k) & mask;
    while (keys[h] != ~0ull) { if (keys[h] == k) return vals[h]; h = (h + 1) & mask; }
    return UINT32_MAX;
  }
};

// Cache of pieces already merged: open addressing over one arena that holds, per entry, the piece's
// bytes followed by its tokens.  Natural text repeats its words, so most pieces are found here and cost
// one hash and one comparison instead of the merge loop.
struct PieceCache {
  struct Slot { uint64_t hash; uint32_t at; uint16_t len, ntok; };   // at: offset of the entry in `arena`
  std::vector<Slot> slots;
  std::vector<unsigned char> arena;
  uint64_t mask = 0;
  size_t used = 0;
  static constexpr size_t kArenaLimit = 64u << 20;   // per worker; beyond it the cache starts over
  PieceCache() { reset(); }
  void reset() {
    slots.assign(1u << 16, Slot{0, UINT32_MAX, 0, 0});
    mask = slots.size() - 1;
    used = 0;
    arena.clear();
    arena.reserve(1u << 20);
  }
  static uint64_t hash(const unsigned char* p, int n) {
    uint64_t h = 0x9E3779B97F4A7C15ull ^ (uint64_t)n;
    int i = 0;
    for (; i + 8 <= n; i += 8) {
      uint64_t w;
      memcpy(&w, p + i, 8);
      h = (h ^ w) * 0xFF51AFD7ED558CCDull;
      h ^= h >> 32;
    }
    uint64_t w = 0;
    if (i < n) memcpy(&w, p + i, (size_t)(n - i));
    h = (h ^ w) * 0xC4CEB9FE1A85EC53ull;
    return h ^ (h >> 29);
  }
  // tokens of the piece or nullptr; *slot_out is where insert() must put it
  const uint32_t* find(const unsigned char* p, int n, uint64_t h, int* ntok, size_t* slot_out) const {
    size_t i = h & mask;
    for (;; i = (i + 1) & mask) {
      const Slot& s = slots[i];
      if (s.at == UINT32_MAX) { *slot_out = i; return nullptr; }
      if (s.hash == h && s.len == n && memcmp(arena.data() + s.at, p, (size_t)n) == 0) {
        *ntok = s.ntok;
        return reinterpret_cast<const uint32_t*>(arena.data() + s.at + ((n + 3) & ~3));
      }
    }
  }
  void insert(size_t slot, const unsigned char* p, int n, uint64_t h, const uint32_t* tok, int ntok) {
    const size_t need = (size_t)((n + 3) & ~3) + (size_t)ntok * 4;
    if (arena.size() + need > kArenaLimit || (used + 1) * 2 > slots.size()) {
      if (arena.size() + need > kArenaLimit) { reset(); slot = h & mask; }
      else { grow(); int d; if (find(p, n, h, &d, &slot)) return; }
    }
    const size_t at = (arena.size() + 3) & ~(size_t)3;
    arena.resize(at + need);
    memcpy(arena.data() + at, p, (size_t)n);
    memcpy(arena.data() + at + ((n + 3) & ~3), tok, (size_t)ntok * 4);
    slots[slot] = Slot{h, (uint32_t)at, (uint16_t)n, (uint16_t)ntok};
    ++used;
  }
  void grow() {
    std::vector<Slot> old;
    old.swap(slots);
    slots.assign(old.size() * 2, Slot{0, UINT32_MAX, 0, 0});
    mask = slots.size() - 1;
    for (const Slot& s : old)
      if (s.at != UINT32_MAX) {
        size_t i = s.hash & mask;
        while (slots[i].at != UINT32_MAX) i = (i + 1) & mask;
        slots[i] = s;
      }
  }
};

struct Encoder {
  const MergeTable& table;
  PieceCache cache;
  uint64_t hits = 0, misses = 0;
  explicit Encoder(const MergeTable& t) : table(t) {}

  // symbols of the piece after all merges, into sym[]; returns their number
  int merge_piece(const unsigned char* p, int n, uint32_t* sym) {
    for (int i = 0; i < n; ++i) sym[i] = p[i];
    while (n > 1) {
      uint32_t best = UINT32_MAX;
      int at = -1;
      for (int i = 0; i + 1 < n; ++i) {
        const uint32_t r = table.rank(sym[i], sym[i + 1]);
        if (r < best) { best = r; at = i; }
      }
      if (at < 0) break;
      sym[at] = 256 + best;
      memmove(sym + at + 1, sym + at + 2, (size_t)(n - at - 2) * sizeof(uint32_t));
      --n;
    }
    return n;
  }

  void piece(const unsigned char* p, int n, std::vector<uint32_t>& out) {
    if (n == 1) { out.push_back(p[0]); return; }
    const uint64_t h = PieceCache::hash(p, n);
    int ntok = 0;
    size_t slot = 0;
    if (const uint32_t* tok = cache.find(p, n, h, &ntok, &slot)) {
      ++hits;
      out.insert(out.end(), tok, tok + ntok);
      return;
    }
    ++misses;
    uint32_t sym[kMaxPiece];
    ntok = merge_piece(p, n, sym);
    out.insert(out.end(), sym, sym + ntok);
    cache.insert(slot, p, n, h, sym, ntok);
  }

  void encode(const unsigned char* t, size_t n, std::vector<uint32_t>& out) {
    size_t i = 0;
    while (i < n) {
      const int c = cls(t[i]);
      size_t j;
      if (c == SPACE && i + 1 < n && (cls(t[i + 1]) == LETTER || cls(t[i + 1]) == DIGIT || cls(t[i + 1]) == OTHER)) {
        const int run = cls(t[i + 1]);
        j = i + 1;
        while (j < n && cls(t[j]) == run) ++j;
      } else if (c == LETTER || c == DIGIT || c == OTHER) {
        j = i;
        while (j < n && cls(t[j]) == c) ++j;
      } else {
        j = i;
        while (j < n && (cls(t[j]) == SPACE || cls(t[j]) == WS)) ++j;
        if (j - i > 1 && j < n && t[j - 1] == 0x20) --j;
      }
      for (size_t k = i; k < j; k += kMaxPiece) piece(t + k, (int)((j - k) < (size_t)kMaxPiece ? (j - k) : (size_t)kMaxPiece), out);
      i = j;
    }
  }
};

// ------------------------------------------------------------------------------------------ pipeline
struct Batch {
  uint64_t id = 0, first_doc = 0;
  std::vector<Span> docs;            // offsets relative to `raw`
  std::vector<unsigned char> raw;    // the batch's bytes of the JSONL file
  std::vector<uint32_t> tokens;      // filled by a worker
  std::vector<uint64_t> lengths;
};

template <typename T>
class Queue {
 public:
  void push(T v) {
    { std::lock_guard<std::mutex> g(m_); q_.push_back(std::move(v)); }
    cv_.notify_one();
  }
  // false once closed and empty
  bool pop(T& v) {
    std::unique_lock<std::mutex> g(m_);
    cv_.wait(g, [&] { return !q_.empty() || closed_; });
    if (q_.empty()) return false;
    v = std::move(q_.front());
    q_.pop_front();
    return true;
  }
  void close() {
    { std::lock_guard<std::mutex> g(m_); closed_ = true; }
    cv_.notify_all();
  }
 private:
  std::mutex m_;
  std::condition_variable cv_;
  std::deque<T> q_;
  bool closed_ = false;
};

class Tickets {
 public:
  explicit Tickets(int n) : n_(n) {}
  // false if the pipeline was stopped
  bool take() {
    std::unique_lock<std::mutex> g(m_);
    cv_.wait(g, [&] { return n_ > 0 || stop_; });
    if (stop_) return false;
    --n_;
    return true;
  }
  void give() {
    { std::lock_guard<std::mutex> g(m_); ++n_; }
    cv_.notify_one();
  }
  void stop() {
    { std::lock_guard<std::mutex> g(m_); stop_ = true; }
    cv_.notify_all();
  }
 private:
  std::mutex m_;
  std::condition_variable cv_;
  int n_;
  bool stop_ = false;
};

struct Shared {
  std::atomic<bool> failed{false};
  std::mutex err_m;
  std::string err;
  void set_error(const std::string& e) {
    std::lock_guard<std::mutex> g(err_m);
    if (!failed.exchange(true)) err = e;
  }
};

}  // namespace

struct tokfile {
  Mapped map;
  uint32_t token_bytes = 0;
  uint64_t n_docs = 0, n_tokens = 0;
  const unsigned char* tokens = nullptr;
  const unsigned char* index = nullptr;
};

extern "C" {

const char* tokpipe_last_error(void) { return g_err; }

int tokpipe_index_jsonl(const char* jsonl_path, const char* index_path, int n_threads, uint64_t* n_docs) {
  if (!jsonl_path || !index_path) return fail("tokpipe_index_jsonl: null path");
  if (n_threads < 1 || n_threads > 1024) return fail("tokpipe_index_jsonl: n_threads %d outside 1..1024", n_threads);
  Mapped m;
  if (!m.open(jsonl_path)) return fail("tokpipe_index_jsonl: cannot read %s", jsonl_path);
  const size_t n = m.n;
  if (n < (size_t)n_threads * 4096) n_threads = 1;
  std::vector<std::vector<Span>> parts((size_t)n_threads);
  std::vector<std::thread> th;
  for (int t = 0; t < n_threads; ++t) {
    const size_t lo = n * (size_t)t / (size_t)n_threads, hi = n * (size_t)(t + 1) / (size_t)n_threads;
    th.emplace_back([&, t, lo, hi] { scan_lines(m.p, n, lo, hi, parts[(size_t)t]); });
  }
  for (auto& x : th) x.join();
  uint64_t total = 0;
  for (auto& v : parts) total += v.size();
  const int fd = ::open(index_path, O_WRONLY | O_CREAT | O_TRUNC, 0644);
  if (fd < 0) return fail("tokpipe_index_jsonl: cannot write %s", index_path);
  bool ok = write_all(fd, kIdxMagic, 8) && write_all(fd, &total, 8);
  for (auto& v : parts) ok = ok && (v.empty() || write_all(fd, v.data(), v.size() * sizeof(Span)));
  ok = (::close(fd) == 0) && ok;
  if (!ok) return fail("tokpipe_index_jsonl: write to %s failed", index_path);
  if (n_docs) *n_docs = total;
  return 0;
}

int tokpipe_tokenize(const char* jsonl_path, const char* index_path, const char* out_path, const uint32_t* merges,
                     uint32_t n_merges, const char* key, int64_t eod_token, int n_workers, int batch_docs,
                     int queue_depth, tokpipe_stats* stats) {
  const auto t0 = std::chrono::steady_clock::now();
  if (!jsonl_path || !index_path || !out_path || !key) return fail("tokpipe_tokenize: null path or key");
  if (n_merges && !merges) return fail("tokpipe_tokenize: merges is null");
  if (n_workers < 1 || n_workers > 1024 || batch_docs < 1 || queue_depth < 1 || queue_depth > (1 << 20))
    return fail("tokpipe_tokenize: need 1 <= n_workers <= 1024, batch_docs >= 1, 1 <= queue_depth <= 2^20");
  if (n_merges > (1u << 30) || eod_token >= ((int64_t)1 << 32)) return fail("tokpipe_tokenize: ids must fit 32 bits");
  MergeTable table;
  for (uint32_t r = 0; r < n_merges; ++r)
    if (merges[2 * r] >= 256 + r || merges[2 * r + 1] >= 256 + r)
      return fail("tokpipe_tokenize: merge %u combines a symbol that does not exist yet", r);
  {
    std::vector<uint64_t> seen;
    seen.reserve(n_merges);
    for (uint32_t r = 0; r < n_merges; ++r) seen.push_back(((uint64_t)merges[2 * r] << 32) | merges[2 * r + 1]);
    std::sort(seen.begin(), seen.end());
    for (uint32_t r = 1; r < n_merges; ++r)
      if (seen[r] == seen[r - 1]) return fail("tokpipe_tokenize: the pair (%u, %u) is merged twice", (unsigned)(seen[r] >> 32), (unsigned)seen[r]);
  }
  table.build(merges, n_merges);
  std::vector<Span> docs;
  if (!load_index(index_path, docs)) return fail("tokpipe_tokenize: %s is not a JSONL index file", index_path);
  const int in_fd = ::open(jsonl_path, O_RDONLY);
  if (in_fd < 0) return fail("tokpipe_tokenize: cannot read %s", jsonl_path);
  struct stat st;
  if (fstat(in_fd, &st) != 0) { ::close(in_fd); return fail("tokpipe_tokenize: cannot stat %s", jsonl_path); }
  for (size_t d = 0; d < docs.size(); ++d)
    if (docs[d].len > (uint64_t)st.st_size || docs[d].off > (uint64_t)st.st_size - docs[d].len ||
        (d && docs[d].off < docs[d - 1].off + docs[d - 1].len)) {
      ::close(in_fd);
      return fail("tokpipe_tokenize: index entry %zu does not fit %s", d, jsonl_path);
    }
  const int out_fd = ::open(out_path, O_WRONLY | O_CREAT | O_TRUNC, 0644);
  if (out_fd < 0) { ::close(in_fd); return fail("tokpipe_tokenize: cannot write %s", out_path); }

  const uint64_t vocab = std::max<uint64_t>(256ull + n_merges, eod_token >= 0 ? (uint64_t)eod_token + 1 : 0);
  const uint32_t token_bytes = vocab <= 65536 ? 2 : 4;
  const std::string key_s(key);
  const uint64_t n_docs = docs.size(), n_batches = (n_docs + (uint64_t)batch_docs - 1) / (uint64_t)batch_docs;

  Shared sh;
  Queue<std::unique_ptr<Batch>> to_workers, to_writer;
  Tickets tickets(queue_depth + n_workers);
  std::atomic<uint64_t> bytes_read{0}, hits{0}, misses{0};
  uint64_t n_tokens = 0;
  std::vector<uint64_t> index;
  index.reserve(n_docs + 1);
  index.push_back(0);

  std::thread reader([&] {
    for (uint64_t b = 0; b < n_batches && !sh.failed.load(); ++b) {
      if (!tickets.take()) break;
      auto batch = std::make_unique<Batch>();
      batch->id = b;
      batch->first_doc = b * (uint64_t)batch_docs;
      const uint64_t last = std::min(n_docs, batch->first_doc + (uint64_t)batch_docs);
      const uint64_t lo = docs[batch->first_doc].off, hi = docs[last - 1].off + docs[last - 1].len;
      batch->raw.resize(hi - lo);
      size_t got = 0;
      while (got < batch->raw.size()) {
        const ssize_t r = pread(in_fd, batch->raw.data() + got, batch->raw.size() - got, (off_t)(lo + got));
        if (r <= 0) { sh.set_error("read of the JSONL file failed"); break; }
        got += (size_t)r;
      }
      if (sh.failed.load()) break;
      bytes_read += batch->raw.size();
      batch->docs.reserve(last - batch->first_doc);
      for (uint64_t d = batch->first_doc; d < last; ++d) batch->docs.push_back({docs[d].off - lo, docs[d].len});
      to_workers.push(std::move(batch));
    }
    to_workers.close();
  });

  std::vector<std::thread> workers;
  std::atomic<int> workers_left{n_workers};
  for (int w = 0; w < n_workers; ++w)
    workers.emplace_back([&] {
      Encoder enc(table);
      std::string name, text;
      std::unique_ptr<Batch> batch;
      while (to_workers.pop(batch)) {
        if (!sh.failed.load()) {
          batch->lengths.reserve(batch->docs.size());
          batch->tokens.reserve(batch->raw.size() / 3);
          for (size_t d = 0; d < batch->docs.size(); ++d) {
            const int rc = extract_text(batch->raw.data() + batch->docs[d].off, batch->docs[d].len, key_s, name, text);
            if (rc) {
              char msg[256];
              snprintf(msg, sizeof msg, rc == 1 ? "document %llu is not a JSON object" : "document %llu has no string member \"%s\"",
                       (unsigned long long)(batch->first_doc + d), key);
              sh.set_error(msg);
              break;
            }
            const size_t before = batch->tokens.size();
            enc.encode((const unsigned char*)text.data(), text.size(), batch->tokens);
            if (eod_token >= 0) batch->tokens.push_back((uint32_t)eod_token);
            batch->lengths.push_back(batch->tokens.size() - before);
          }
          std::vector<unsigned char>().swap(batch->raw);
        }
        to_writer.push(std::move(batch));
      }
      hits += enc.hits;
      misses += enc.misses;
      if (--workers_left == 0) to_writer.close();
    });

  std::thread writer([&] {
    std::map<uint64_t, std::unique_ptr<Batch>> waiting;
    std::vector<uint16_t> narrow;
    uint64_t next = 0;
    bool ok = true;
    {
      unsigned char head[kHeader] = {0};   // patched when the totals are known
      ok = write_all(out_fd, head, kHeader);
    }
    std::unique_ptr<Batch> batch;
    while (to_writer.pop(batch)) {
      waiting.emplace(batch->id, std::move(batch));
      while (!waiting.empty() && waiting.begin()->first == next) {
        Batch& b = *waiting.begin()->second;
        if (ok && !sh.failed.load()) {
          if (token_bytes == 2) {
            narrow.resize(b.tokens.size());
            for (size_t i = 0; i < b.tokens.size(); ++i) narrow[i] = (uint16_t)b.tokens[i];
            ok = write_all(out_fd, narrow.data(), narrow.size() * 2);
          } else {
            ok = write_all(out_fd, b.tokens.data(), b.tokens.size() * 4);
          }
          for (uint64_t l : b.lengths) { n_tokens += l; index.push_back(n_tokens); }
          if (!ok) sh.set_error("write to the token file failed");
        }
        waiting.erase(waiting.begin());
        ++next;
        tickets.give();
      }
      if (sh.failed.load()) tickets.stop();
    }
  });

  reader.join();
  for (auto& w : workers) w.join();
  writer.join();
  ::close(in_fd);
  bool ok = !sh.failed.load();
  if (ok && index.size() != n_docs + 1) { ok = false; sh.set_error("internal: document count mismatch"); }
  if (ok) {
    const uint64_t data_end = kHeader + n_tokens * token_bytes, index_off = (data_end + 7) / 8 * 8;
    const unsigned char pad[8] = {0};
    ok = write_all(out_fd, pad, index_off - data_end) && write_all(out_fd, index.data(), index.size() * 8);
    unsigned char head[kHeader] = {0};
    memcpy(head, kTokMagic, 8);
    const uint32_t version = 1;
    memcpy(head + 8, &version, 4);
    memcpy(head + 12, &token_bytes, 4);
    memcpy(head + 16, &n_docs, 8);
    memcpy(head + 24, &n_tokens, 8);
    memcpy(head + 32, &index_off, 8);
    ok = ok && pwrite(out_fd, head, kHeader, 0) == (ssize_t)kHeader;
    if (!ok) sh.set_error("write to the token file failed");
  }
  ok = (::close(out_fd) == 0) && ok;
  if (!ok) return fail("tokpipe_tokenize: %s", sh.err.empty() ? "write to the token file failed" : sh.err.c_str());
  if (stats) {
    stats->n_docs = n_docs;
    stats->n_tokens = n_tokens;
    stats->bytes_read = bytes_read.load();
    stats->seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    stats->cache_hits = hits.load();
    stats->cache_misses = misses.load();
  }
  return 0;
}

tokfile* tokfile_open(const char* path) {
  if (!path) { fail("tokfile_open: null path"); return nullptr; }
  auto f = std::make_unique<tokfile>();
  if (!f->map.open(path) || f->map.n < kHeader || memcmp(f->map.p, kTokMagic, 8) != 0) {
    fail("tokfile_open: %s is not a token file", path);
    return nullptr;
  }
  uint32_t version;
  uint64_t index_off;
  memcpy(&version, f->map.p + 8, 4);
  memcpy(&f->token_bytes, f->map.p + 12, 4);
  memcpy(&f->n_docs, f->map.p + 16, 8);
  memcpy(&f->n_tokens, f->map.p + 24, 8);
  memcpy(&index_off, f->map.p + 32, 8);
  // sizes are compared by division so that a corrupt header cannot wrap a product
  if (version != 1 || (f->token_bytes != 2 && f->token_bytes != 4) || index_off % 8 || index_off < kHeader || index_off > f->map.n ||
      f->n_tokens > (index_off - kHeader) / f->token_bytes || f->n_docs >= (f->map.n - index_off) / 8) {
    fail("tokfile_open: %s has an inconsistent header", path);
    return nullptr;
  }
  f->tokens = f->map.p + kHeader;
  f->index = f->map.p + index_off;
  return f.release();
}

void tokfile_close(tokfile* f) { delete f; }
uint64_t tokfile_num_docs(const tokfile* f) { return f ? f->n_docs : 0; }
uint64_t tokfile_num_tokens(const tokfile* f) { return f ? f->n_tokens : 0; }
uint32_t tokfile_token_bytes(const tokfile* f) { return f ? f->token_bytes : 0; }

int tokfile_doc(const tokfile* f, uint64_t i, const void** tokens, uint64_t* n_tokens) {
  if (!f || !tokens || !n_tokens) return fail("tokfile_doc: null argument");
  if (i >= f->n_docs) return fail("tokfile_doc: document %llu of %llu", (unsigned long long)i, (unsigned long long)f->n_docs);
  uint64_t a, b;
  memcpy(&a, f->index + i * 8, 8);
  memcpy(&b, f->index + (i + 1) * 8, 8);
  if (a > b || b > f->n_tokens) return fail("tokfile_doc: corrupt index at document %llu", (unsigned long long)i);
  *tokens = f->tokens + a * f->token_bytes;
  *n_tokens = b - a;
  return 0;
}

}  // extern "C"
