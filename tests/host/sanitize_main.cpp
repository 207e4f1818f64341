// Host-only driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the runtime's host logic: the
// schedule generators (Section 3.3), the partitioner's dynamic program (Section 3.2), the arena planner behind
// pd_stage_query_bytes (Section 3.5), replica routing and checkpoint-file validation (Section 4).  It touches no GPU.
// Every call's result is checked against what the call's contract in include/pd.h promises; the sanitizers watch
// the memory accesses and the integer arithmetic on the way.  Exit code 0 = all checks passed.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/pd.h"
#include "../../include/pd_debug.h"

static int g_fail = 0;
#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::fprintf(stderr, "CHECK failed, line %d: %s (last error: %s)\n", __LINE__, #cond, pd_last_error()); \
      ++g_fail;                                                                  \
    }                                                                            \
  } while (0)

static uint64_t rng_state = 0x1806033770ull;
static uint64_t rnd() {  // splitmix64
  uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  return z ^ (z >> 31);
}
static double unif() { return (double)(rnd() >> 11) / 9007199254740992.0; }

static void schedules() {
  for (int S = 1; S <= 6; ++S)
    for (int noam = 1; noam <= S + 1; ++noam)
      for (int M : {0, 1, 2, 3, 7, 64, 1000})
        for (int s = 0; s < S; ++s) {
          size_t n = 0;
          // capacity query first: too small must report the count and write nothing past `cap`
          std::vector<pd_op> ops(M ? 3 * (size_t)M : 1);
          const int rc0 = pd_schedule_1f1b(S, noam, M, s, ops.data(), M ? 1 : 0, &n);
          CHECK(n == 3 * (size_t)M);
          CHECK(rc0 == (M ? PD_ENOMEM : PD_OK));
          CHECK(pd_schedule_1f1b(S, noam, M, s, ops.data(), ops.size(), &n) == PD_OK);
          const int depth = noam - s < 1 ? 1 : noam - s;
          int in_flight = 0, latest = 0, nf = 0, nb = 0;
          for (size_t k = 0; k < n; ++k) {
            const pd_op& o = ops[k];
            if (o.kind == PD_OP_F) { CHECK(o.mb_id == nf++ && o.version == latest); ++in_flight; }
            if (o.kind == PD_OP_B) { CHECK(o.mb_id == nb++); --in_flight; }
            if (o.kind == PD_OP_U) { CHECK(o.version == ++latest); }
            CHECK(o.slot == o.version % depth && in_flight <= depth && in_flight >= 0);
          }
          CHECK(nf == M && nb == M && latest == M);
          std::vector<pd_op> vs(ops.size());
          CHECK(pd_schedule_1f1b_vertical_sync(S, noam, M, s, vs.data(), vs.size(), &n) == PD_OK);
          for (size_t k = 0; k < n; ++k) CHECK(vs[k].kind == ops[k].kind && vs[k].mb_id == ops[k].mb_id && vs[k].slot == vs[k].version % noam);
        }
  size_t n = 0;
  CHECK(pd_schedule_1f1b(0, 1, 1, 0, nullptr, 0, &n) == PD_EINVAL);
  CHECK(pd_schedule_1f1b(2, 2, 4, 2, nullptr, 0, &n) == PD_EINVAL);
  CHECK(pd_schedule_1f1b(2, 2, 4, 0, nullptr, 100, &n) == PD_EINVAL);  // room but no array
  CHECK(pd_schedule_1f1b_depth(0, 4, nullptr, 0, &n) == PD_EINVAL);
  std::vector<pd_op> ops(12);
  CHECK(pd_schedule_1f1b_depth(3, 4, ops.data(), ops.size(), nullptr) == PD_OK);
  int32_t q = -1, k = -1;
  CHECK(pd_replica_route(11, 3, &q, &k) == PD_OK && q == 2 && k == 3);
  CHECK(pd_replica_route(-1, 3, &q, &k) == PD_EINVAL && pd_replica_route(1, 0, &q, &k) == PD_EINVAL);
}

static void partitions() {
  for (int trial = 0; trial < 200; ++trial) {
    const int N = 1 + (int)(rnd() % 24), M = 1 + (int)(rnd() % 16);
    std::vector<double> T(N), a(N), w(N);
    for (int l = 0; l < N; ++l) { T[l] = unif() * 10; a[l] = unif() * 1e6; w[l] = unif() * 1e7; }
    const double bw = 1e3 + unif() * 1e6;
    double best = -1;
    size_t ns = 0;
    int32_t noam = 0;
    std::vector<pd_stage_assign> st(N);
    const int rc = pd_partition(N, M, T.data(), a.data(), w.data(), bw, &best, st.data(), st.size(), &ns, &noam);
    CHECK(rc == PD_OK && ns >= 1 && ns <= (size_t)N && best > 0);
    int next = 0, workers = 0;
    double slowest = 0;
    for (size_t k = 0; k < ns && rc == PD_OK; ++k) {  // a feasible partition that reaches the reported optimum
      CHECK(st[k].first_layer == next && st[k].last_layer >= next && st[k].replicas >= 1);
      double t = 0, ws = 0;
      for (int l = st[k].first_layer; l <= st[k].last_layer && l < N; ++l) { t += T[l]; ws += w[l]; }
      const int m = st[k].replicas;
      const double sync = 4.0 * (m - 1) * ws / (m * bw);
      slowest = std::fmax(slowest, std::fmax(t, sync) / m);
      if (st[k].last_layer < N - 1) slowest = std::fmax(slowest, 2 * a[st[k].last_layer] / bw);
      next = st[k].last_layer + 1;
      workers += m;
    }
    CHECK(next == N && workers == M && std::fabs(slowest - best) <= 1e-9 * best);
    CHECK(noam == (M + st[0].replicas - 1) / st[0].replicas);
    if (ns > 1) {
      size_t ns2 = 0;
      CHECK(pd_partition(N, M, T.data(), a.data(), w.data(), bw, nullptr, st.data(), ns - 1, &ns2, nullptr) == PD_ENOMEM && ns2 == ns);
    }
  }
  double one = 1.0, neg = -1.0;
  CHECK(pd_partition(0, 1, &one, &one, &one, 1.0, nullptr, nullptr, 0, nullptr, nullptr) == PD_EINVAL);
  CHECK(pd_partition(1, 1, &neg, &one, &one, 1.0, nullptr, nullptr, 0, nullptr, nullptr) == PD_EINVAL);
  CHECK(pd_partition(1, 1, &one, &one, &one, 0.0, nullptr, nullptr, 0, nullptr, nullptr) == PD_EINVAL);
}

static pd_layer_desc layer(int kind, std::initializer_list<int> p) {
  pd_layer_desc d;
  std::memset(&d, 0, sizeof d);
  d.kind = kind;
  int k = 0;
  for (int v : p) d.p[k++] = v;
  return d;
}

static void arena_plans() {
  auto query = [](std::vector<pd_layer_desc> layers, int precision, int minibatch, int depth, size_t* bytes, int replicas = 0,
                  int vsync = 0) {
    pd_stage_config c;
    std::memset(&c, 0, sizeof c);
    c.stage_index = 0; c.num_stages = 1; c.noam = 1; c.in_flight_override = depth; c.minibatch = minibatch;
    c.precision = precision; c.lr = 0.01f; c.momentum = 0.9f; c.n_layers = (int)layers.size(); c.layers = layers.data();
    c.replicas = replicas; c.vertical_sync = vsync;
    return pd_stage_query_bytes(&c, bytes);
  };
  size_t b1 = 0, b2 = 0;
  // the VGG16 classifier stage: the ring alone is depth x parameters x 2 bytes
  std::vector<pd_layer_desc> fc = {layer(PD_LINEAR, {25088, 4096, 1}), layer(PD_LINEAR, {4096, 4096, 1}),
                                   layer(PD_LINEAR, {4096, 1000, 0}), layer(PD_SOFTMAX_XENT, {1000})};
  CHECK(query(fc, PD_BF16_F32ACC, 64, 4, &b1) == PD_OK && b1 > (size_t)4 * 123642856 * 2 && b1 < (size_t)4 << 30);
  CHECK(query(fc, PD_BF16_F32ACC, 64, 2, &b2) == PD_OK && b2 < b1);
  CHECK(query(fc, PD_F32, 64, 4, &b2) == PD_OK);
  // convolution stage, branched block, LSTM stage
  std::vector<pd_layer_desc> conv = {layer(PD_CONV2D, {3, 64, 3, 3, 1, 1, 1, 1, 224, 224}), layer(PD_CONV2D, {64, 64, 3, 3, 1, 1, 1, 1, 224, 224}),
                                     layer(PD_MAXPOOL2D, {2, 2, 64, 224, 224}), layer(PD_CONV2D, {64, 128, 3, 3, 1, 1, 1, 1, 112, 112})};
  CHECK(query(conv, PD_BF16_F32ACC, 64, 4, &b1) == PD_OK && b1 > 0);
  CHECK(query(conv, PD_BF16_F32ACC, 64, 4, &b2, 2) == PD_OK && b2 > b1);   // a replicated stage adds a gradient buffer
  CHECK(query(conv, PD_BF16_F32ACC, 64, 4, &b2, 2, 1) == PD_EINVAL);        // not with vertical sync
  CHECK(query(conv, PD_F32, 64, 4, &b2) == PD_EINVAL);                      // convolutions are bf16 only
  std::vector<pd_layer_desc> blk = {layer(PD_CONV2D, {8, 16, 3, 3, 1, 1, 1, 1, 9, 9}), layer(PD_CONCAT_BEGIN, {}), layer(PD_BRANCH, {}),
                                    layer(PD_CONV2D, {16, 16, 1, 1, 1, 0, 0, 1, 9, 9}), layer(PD_BRANCH, {}),
                                    layer(PD_AVGPOOL2D, {3, 1, 1, 16, 9, 9}), layer(PD_CONV2D, {16, 8, 1, 1, 1, 0, 0, 1, 9, 9}),
                                    layer(PD_CONCAT_END, {})};
  CHECK(query(blk, PD_BF16_F32ACC, 3, 2, &b1) == PD_OK);
  blk.pop_back();
  CHECK(query(blk, PD_BF16_F32ACC, 3, 2, &b1) == PD_EINVAL);                // block not closed
  std::vector<pd_layer_desc> lstm = {layer(PD_LSTM, {4096, 1000, 80})};
  CHECK(query(lstm, PD_BF16_F32ACC, 64, 2, &b1) == PD_OK && b1 > (size_t)2 * 20388000 * 2);
  // malformed descriptions come back as PD_EINVAL, never as a crash
  for (int trial = 0; trial < 2000; ++trial) {
    std::vector<pd_layer_desc> junk(1 + rnd() % 5);
    for (pd_layer_desc& d : junk) {
      d.kind = (int)(rnd() % 11) - 1;
      for (int& v : d.p) v = (int)(rnd() % 7 == 0 ? -(int)(rnd() % 4) : rnd() % 40);
    }
    size_t b = 0;
    const int rc = query(junk, (int)(rnd() % 2), 1 + (int)(rnd() % 8), (int)(rnd() % 4), &b);
    CHECK(rc == PD_OK || rc == PD_EINVAL);
  }
  pd_stage* st = nullptr;
  pd_stage_config c;
  std::memset(&c, 0, sizeof c);
  CHECK(pd_stage_create(&c, nullptr, 0, &st) == PD_EINVAL && st == nullptr);
  CHECK(pd_stage_create(nullptr, nullptr, 0, &st) == PD_EINVAL);
  CHECK(pd_stage_query_bytes(nullptr, &b1) == PD_EINVAL);
  CHECK(pd_stage_destroy(nullptr) == PD_OK);
  CHECK(pd_update(nullptr) == PD_EINVAL && pd_forward(nullptr, 0, nullptr, nullptr, nullptr, nullptr) == PD_EINVAL);
  CHECK(pd_stage_set_trace_limit(nullptr, 1) == PD_EINVAL);
}

static void put(std::string& s, const void* p, size_t n) { s.append(static_cast<const char*>(p), n); }

static void checkpoints(const char* dir) {
  // a file in the documented layout, written here byte by byte
  const uint64_t n = 5;
  const float w[5] = {1.f, -2.f, 3.5f, 0.f, 1e-3f}, m[5] = {0.f, 0.25f, -0.5f, 7.f, -1e3f};
  auto hash = [](uint64_t h, const float* p, size_t cnt) {
    for (size_t i = 0; i < cnt; i += 2) {
      uint32_t lo, hi = 0;
      std::memcpy(&lo, p + i, 4);
      if (i + 1 < cnt) std::memcpy(&hi, p + i + 1, 4);
      h = (h ^ ((uint64_t)hi << 32 | lo)) * 0x100000001b3ull;
    }
    return h;
  };
  const uint64_t sum = hash(hash(0xcbf29ce484222325ull, w, n), m, n);
  const uint32_t prec = 1, zero = 0;
  const int64_t version = 42;
  std::string good;
  put(good, "PDCKPT1\0", 8); put(good, &prec, 4); put(good, &zero, 4); put(good, &n, 8); put(good, &version, 8);
  put(good, &sum, 8); put(good, w, sizeof w); put(good, m, sizeof m);
  auto write = [&](const std::string& name, const std::string& data) {
    const std::string path = std::string(dir) + "/" + name;
    FILE* f = std::fopen(path.c_str(), "wb");
    if (!f) { CHECK(!"cannot write into the scratch directory"); return path; }
    std::fwrite(data.data(), 1, data.size(), f);
    std::fclose(f);
    return path;
  };
  size_t np = 0;
  int32_t latest = 0, precision = -1;
  CHECK(pd_checkpoint_info(write("good.ckpt", good).c_str(), &np, &latest, &precision) == PD_OK && np == 5 && latest == 42 && precision == 1);
  std::string bad = good;
  bad[45] ^= 4;
  CHECK(pd_checkpoint_info(write("flip.ckpt", bad).c_str(), &np, &latest, &precision) == PD_EINVAL);
  for (size_t cut : {(size_t)0, (size_t)7, (size_t)39, (size_t)41, good.size() - 1})
    CHECK(pd_checkpoint_info(write("cut.ckpt", good.substr(0, cut)).c_str(), &np, &latest, &precision) == PD_EINVAL);
  CHECK(pd_checkpoint_info(write("long.ckpt", good + "x").c_str(), &np, &latest, &precision) == PD_EINVAL);
  bad = good;
  const uint64_t huge = ~0ull / 3;  // a parameter count that would overflow any size computation
  std::memcpy(&bad[16], &huge, 8);
  CHECK(pd_checkpoint_info(write("huge.ckpt", bad).c_str(), &np, &latest, &precision) == PD_EINVAL);
  CHECK(pd_checkpoint_info((std::string(dir) + "/missing.ckpt").c_str(), &np, &latest, &precision) == PD_EINVAL);
  CHECK(pd_checkpoint_info(nullptr, &np, &latest, &precision) == PD_EINVAL);
  CHECK(pd_stage_checkpoint_save(nullptr, "x") == PD_EINVAL && pd_stage_checkpoint_load(nullptr, "x") == PD_EINVAL);
}

int main(int argc, char** argv) {
  if (argc < 2) {
    std::fprintf(stderr, "usage: %s <scratch directory>\n", argv[0]);
    return 2;
  }
  schedules();
  partitions();
  arena_plans();
  checkpoints(argv[1]);
  if (g_fail) {
    std::fprintf(stderr, "%d checks failed\n", g_fail);
    return 1;
  }
  std::puts("host logic: all checks passed under AddressSanitizer + UndefinedBehaviorSanitizer");
  return 0;
}
