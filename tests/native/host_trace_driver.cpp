// Replays a trace of allocator calls against the host half of libodma (compiled into this program together with
// odma_host.cpp, by g++ alone, under a sanitizer) and compares every result with the values the trace carries,
// which the test wrote from the allocator oracle.  Second mode: the background recalibrator under threads.
//
// Trace format, one call per line, integers separated by blanks ("-" = argument absent):
//   C main safety large_cap align max_requests window n_buckets b...            create the pool
//   A n | ids | preds | u bits or - | prompts or - | boundaries or - || buckets | offsets | caps | status
//   V n | ids | n_new or - || overflow | status
//   M id || rc offset cap
//   R n | ids || status
//   K n | lengths || boundaries
//   S || n_live then rows id arena offset cap len ; free extents of both arenas
// Exit status 0: everything matched.  1: mismatch (printed).  Sanitizer reports end the program on their own.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <iostream>
#include <sstream>
#include <string>
#include <thread>
#include <vector>
#include <atomic>

#include "odma.h"

static std::vector<std::string> split(const std::string& s, char sep) {
  std::vector<std::string> out;
  std::stringstream ss(s);
  std::string item;
  while (std::getline(ss, item, sep)) out.push_back(item);
  return out;
}
static std::vector<long long> ints(const std::string& s) {
  std::vector<long long> v;
  std::stringstream ss(s);
  long long x;
  while (ss >> x) v.push_back(x);
  return v;
}
static bool absent(const std::string& s) { return s.find('-') != std::string::npos && ints(s).empty(); }
template <class T>
static std::vector<T> cast(const std::vector<long long>& v) { return std::vector<T>(v.begin(), v.end()); }

static int fail(int line, const char* what) {
  std::printf("line %d: %s differs from the oracle\n", line, what);
  return 1;
}

static int replay(const char* path) {
  std::ifstream in(path);
  if (!in) {
    std::printf("cannot open %s\n", path);
    return 2;
  }
  odma_pool_t* pool = nullptr;
  int n_buckets = 0;
  std::string line;
  int ln = 0, calls = 0;
  while (std::getline(in, line)) {
    ++ln;
    if (line.empty()) continue;
    const char op = line[0];
    const auto halves = split(line.substr(1), '#');
    const auto args = split(halves[0], '|');
    const auto want = halves.size() > 1 ? split(halves[1], '|') : std::vector<std::string>();
    ++calls;
    if (op == 'C') {
      const auto a = ints(args[0]);
      odma_pool_config_t cfg;
      std::memset(&cfg, 0, sizeof cfg);
      cfg.n_layers = 1; cfg.n_q_heads = 4; cfg.n_kv_heads = 2; cfg.head_dim = 64;
      cfg.kv_dtype = ODMA_BF16; cfg.out_dtype = ODMA_BF16;
      cfg.main_tokens = a[0]; cfg.safety_tokens = a[1]; cfg.large_cap = (int32_t)a[2]; cfg.align_tokens = (int32_t)a[3];
      cfg.max_requests = (int32_t)a[4]; cfg.window = (int32_t)a[5]; cfg.n_buckets = n_buckets = (int32_t)a[6];
      std::vector<int32_t> b(a.begin() + 7, a.begin() + 7 + n_buckets);
      cfg.boundaries = b.data();
      cfg.gamma = 0.2; cfg.tau = 0.8;
      if (pool) odma_pool_destroy(pool);
      if (odma_pool_create(&cfg, &pool) != ODMA_OK) {
        std::printf("line %d: odma_pool_create failed: %s\n", ln, odma_last_error());
        return 1;
      }
    } else if (op == 'A') {
      const int n = (int)ints(args[0])[0];
      auto ids = cast<int32_t>(ints(args[1])), pred = cast<int32_t>(ints(args[2]));
      std::vector<float> u;
      if (!absent(args[3])) for (long long bits : ints(args[3])) { uint32_t x = (uint32_t)bits; float f; std::memcpy(&f, &x, 4); u.push_back(f); }
      auto prompt = absent(args[4]) ? std::vector<int32_t>() : cast<int32_t>(ints(args[4]));
      auto bnd = absent(args[5]) ? std::vector<int32_t>() : cast<int32_t>(ints(args[5]));
      std::vector<int32_t> bucket(n), cap(n), status(n);
      std::vector<int64_t> off(n);
      odma_assign(pool, n, ids.data(), pred.data(), u.empty() ? nullptr : u.data(), prompt.empty() ? nullptr : prompt.data(),
                  bnd.empty() ? nullptr : bnd.data(), (int32_t)bnd.size(), bucket.data(), off.data(), cap.data(), status.data());
      if (cast<long long>(ints(want[0])) != std::vector<long long>(bucket.begin(), bucket.end())) return fail(ln, "assign: bucket");
      if (ints(want[1]) != std::vector<long long>(off.begin(), off.end())) return fail(ln, "assign: offset");
      if (ints(want[2]) != std::vector<long long>(cap.begin(), cap.end())) return fail(ln, "assign: cap");
      if (ints(want[3]) != std::vector<long long>(status.begin(), status.end())) return fail(ln, "assign: status");
    } else if (op == 'V') {
      const int n = (int)ints(args[0])[0];
      auto ids = cast<int32_t>(ints(args[1]));
      auto nn = absent(args[2]) ? std::vector<int32_t>() : cast<int32_t>(ints(args[2]));
      std::vector<int32_t> ov(n), st(n);
      odma_advance(pool, n, ids.data(), nn.empty() ? nullptr : nn.data(), ov.data(), st.data());
      if (ints(want[0]) != std::vector<long long>(ov.begin(), ov.end())) return fail(ln, "advance: overflow");
      if (ints(want[1]) != std::vector<long long>(st.begin(), st.end())) return fail(ln, "advance: status");
    } else if (op == 'M') {
      int64_t off = -1;
      int32_t cap = 0;
      const int rc = odma_migrate(pool, (int32_t)ints(args[0])[0], nullptr, &off, &cap);
      const auto w = ints(want[0]);
      if (w[0] != rc || w[1] != off || w[2] != cap) return fail(ln, "migrate");
    } else if (op == 'R') {
      const int n = (int)ints(args[0])[0];
      auto ids = cast<int32_t>(ints(args[1]));
      std::vector<int32_t> st(n);
      odma_release(pool, n, ids.data(), st.data());
      if (ints(want[0]) != std::vector<long long>(st.begin(), st.end())) return fail(ln, "release: status");
    } else if (op == 'K') {
      const int n = (int)ints(args[0])[0];
      auto lens = cast<int32_t>(ints(args[1]));
      std::vector<int32_t> b(n_buckets);
      odma_recalibrate(pool, n, lens.data(), b.data());
      if (ints(want[0]) != std::vector<long long>(b.begin(), b.end())) return fail(ln, "recalibrate: boundaries");
    } else if (op == 'S') {
      int32_t n_live = 0;
      odma_pool_snapshot(pool, 0, &n_live, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
      std::vector<int32_t> id(n_live), arena(n_live), cap(n_live), len(n_live);
      std::vector<int64_t> off(n_live);
      odma_pool_snapshot(pool, n_live, &n_live, id.data(), arena.data(), off.data(), cap.data(), len.data(), nullptr);
      std::vector<long long> got{n_live};
      for (int i = 0; i < n_live; ++i) { got.push_back(id[i]); got.push_back(arena[i]); got.push_back(off[i]); got.push_back(cap[i]); got.push_back(len[i]); }
      if (ints(want[0]) != got) return fail(ln, "snapshot");
      std::vector<long long> ext;
      for (int arena_id = 0; arena_id < 2; ++arena_id) {
        int32_t ne = 0;
        odma_pool_free_extents(pool, arena_id, 0, &ne, nullptr, nullptr);
        std::vector<int64_t> s(ne), z(ne);
        odma_pool_free_extents(pool, arena_id, ne, &ne, s.data(), z.data());
        ext.push_back(ne);
        for (int i = 0; i < ne; ++i) { ext.push_back(s[i]); ext.push_back(z[i]); }
      }
      if (ints(want[1]) != ext) return fail(ln, "free extents");
    } else {
      std::printf("line %d: unknown call '%c'\n", ln, op);
      return 2;
    }
  }
  if (pool) odma_pool_destroy(pool);
  std::printf("replayed %d calls: all equal\n", calls);
  return 0;
}

// Background recalibrator under threads: one thread admits, advances and releases requests (the pool's single
// driver), two others report completions and ask for drains, as the ABI allows.  Prints the final epoch and the
// boundaries; the test compares them with the oracle's set for that epoch.
static int threads(int rounds) {
  const int32_t bounds[4] = {512, 1024, 2048, 4096};
  odma_pool_config_t cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 1; cfg.n_q_heads = 4; cfg.n_kv_heads = 2; cfg.head_dim = 64; cfg.kv_dtype = ODMA_BF16; cfg.out_dtype = ODMA_BF16;
  cfg.main_tokens = 1 << 18; cfg.safety_tokens = 4 * 65536; cfg.large_cap = 65536; cfg.align_tokens = 16;
  cfg.max_requests = 64; cfg.window = 256; cfg.n_buckets = 4; cfg.boundaries = bounds; cfg.gamma = 0.2; cfg.tau = 0.8;
  odma_pool_t* pool = nullptr;
  if (odma_pool_create(&cfg, &pool) != ODMA_OK) return 1;
  if (odma_recalibrator_start(pool, 50) != ODMA_OK) return 1;
  std::atomic<int> bad{0};
  auto reporter = [&](int which) {
    for (int i = 0; i < rounds; ++i) {
      std::vector<int32_t> lens;
      for (int j = 0; j < 25; ++j) lens.push_back(100 + ((i * 131 + j * 17 + which * 7) % 3000));   // same multiset from either thread order
      if (odma_report_completions(pool, (int32_t)lens.size(), lens.data()) != ODMA_OK) ++bad;
      if (i % 8 == 0) {
        int64_t epoch = 0;
        if (odma_recalibrator_drain(pool, &epoch) != ODMA_OK) ++bad;
      }
    }
  };
  std::thread t1(reporter, 0), t2(reporter, 1);
  for (int i = 0; i < rounds * 4; ++i) {                   // the pool's driver thread
    int32_t ids[4], pred[4], bucket[4], cap[4], status[4], ov[4];
    int64_t off[4];
    for (int j = 0; j < 4; ++j) { ids[j] = (i * 4 + j) % 64; pred[j] = 50 + (i * 37 + j * 101) % 3000; }
    odma_release(pool, 4, ids, status);
    const int rc = odma_assign(pool, 4, ids, pred, nullptr, nullptr, nullptr, 0, bucket, off, cap, status);
    if (rc != ODMA_OK && rc != ODMA_NOMEM) ++bad;          // the Large Bucket has four slabs: NOMEM is a valid answer
    odma_advance(pool, 4, ids, nullptr, ov, status);
  }
  t1.join();
  t2.join();
  // a last batch from this thread, longer than the window: what the window holds in the end does not depend on how
  // the two reporters interleaved
  std::vector<int32_t> last;
  for (int j = 0; j < 300; ++j) last.push_back(64 + (j * 37) % 5000);
  if (odma_report_completions(pool, (int32_t)last.size(), last.data()) != ODMA_OK) ++bad;
  int64_t epoch = 0;
  odma_recalibrator_drain(pool, &epoch);
  odma_recalibrator_stop(pool);
  int32_t b[4];
  odma_pool_snapshot(pool, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, b);
  std::printf("epoch %lld boundaries %d %d %d %d bad %d\n", (long long)epoch, b[0], b[1], b[2], b[3], bad.load());
  odma_pool_destroy(pool);
  return bad.load() ? 1 : 0;
}

int main(int argc, char** argv) {
  if (argc == 3 && std::string(argv[1]) == "replay") return replay(argv[2]);
  if (argc == 3 && std::string(argv[1]) == "threads") return threads(std::atoi(argv[2]));
  std::printf("usage: %s replay <trace> | threads <rounds>\n", argv[0]);
  return 2;
}
