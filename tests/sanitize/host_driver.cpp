// Exercises the host-only logic of libpbkd's runtime (descriptor validation, workspace layout and sizing, FLOP counts,
// the block scheduler, argument checks that return before any device work) under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Needs no GPU.  Built and run by tests/test_sanitizers.py; prints "ok" on success.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/pbkd.h"

#define CHECK(cond)                                                    \
  do {                                                                 \
    if (!(cond)) {                                                     \
      std::fprintf(stderr, "check failed at line %d: %s (last error: %s)\n", __LINE__, #cond, pbkd_last_error()); \
      return 1;                                                        \
    }                                                                  \
  } while (0)

static pbkd_arch_desc arch(int n, int c, int h, int w, const std::vector<pbkd_layer_desc> &layers, int shortcut, int sstride, int pool) {
  pbkd_arch_desc a{};
  a.n = n; a.c = c; a.h = h; a.w = w;
  a.n_layers = (int)layers.size();
  a.layers = layers.data();
  a.shortcut = shortcut; a.shortcut_stride = sstride; a.pool = pool; a.bn_eps = 1e-5f;
  return a;
}

int main() {
  // ---- descriptors: valid pairs of several shapes, and every class of rejection
  const int shapes[][4] = {{4, 16, 16, 16}, {128, 64, 16, 16}, {32, 3, 224, 224}, {3, 5, 9, 11}, {2, 7, 1, 1}, {5, 4, 2, 1}, {128, 512, 2, 2}};
  for (const auto &sh : shapes) {
    for (int stride0 = 1; stride0 <= 2; ++stride0) {
      for (int pool = 0; pool <= 2; pool += 2) {
        std::vector<pbkd_layer_desc> tl = {{PBKD_CONV3X3, sh[1], 24, stride0, 0}, {PBKD_CONV3X3, 24, 40, 1, 0}};
        std::vector<pbkd_layer_desc> sl = {{PBKD_DWSEP3X3, sh[1], 24, stride0, 1}, {PBKD_DWSEP3X3, 24, 40, 1, 1}};
        for (int shortcut = 0; shortcut <= 1; ++shortcut) {
          pbkd_arch_desc t = arch(sh[0], sh[1], sh[2], sh[3], tl, shortcut, stride0, pool);
          pbkd_arch_desc s = arch(sh[0], sh[1], sh[2], sh[3], sl, shortcut, stride0, pool);
          const pbkd_status st = pbkd_arch_validate(&t, &s);
          const int ho = (sh[2] - 1) / stride0 + 1, wo = (sh[3] - 1) / stride0 + 1;
          const bool pool_ok = pool == 0 || (ho >= 2 && wo >= 2);
          CHECK((st == PBKD_OK) == pool_ok);
          const size_t ws = pbkd_block_workspace_bytes(&t, &s);
          CHECK((ws > 0) == pool_ok);
          if (pool_ok) {
            CHECK(ws % 256 == 0);
            CHECK(pbkd_arch_flops(&t, 0) > 0 && pbkd_arch_flops(&s, 1) > pbkd_arch_flops(&s, 0));
          }
        }
      }
    }
  }
  {
    std::vector<pbkd_layer_desc> tl = {{PBKD_CONV3X3, 8, 8, 1, 0}}, sl = {{PBKD_DWSEP3X3, 8, 8, 1, 1}};
    pbkd_arch_desc t = arch(2, 8, 6, 6, tl, 0, 1, 0), s = arch(2, 8, 6, 6, sl, 0, 1, 0);
    CHECK(pbkd_arch_validate(nullptr, &s) == PBKD_EINVAL);
    pbkd_arch_desc bad = s;
    bad.n_layers = 0;
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_EINVAL);
    bad = s; bad.pool = 3;
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_EINVAL);
    bad = s; bad.h = 7;
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_ESHAPE);
    std::vector<pbkd_layer_desc> wrong = {{PBKD_DWSEP3X3, 9, 8, 1, 1}};
    bad = arch(2, 8, 6, 6, wrong, 0, 1, 0);
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_ESHAPE);
    std::vector<pbkd_layer_desc> two = {{PBKD_DWSEP3X3, 8, 8, 1, 1}, {PBKD_CONV3X3, 8, 8, 1, 1}};
    bad = arch(2, 8, 6, 6, two, 0, 1, 0);
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_EUNSUPPORTED);
    bad = s; bad.shortcut = 2;                       // identity skip with equal shapes is fine
    CHECK(pbkd_arch_validate(&t, &bad) == PBKD_OK);
    std::vector<pbkd_layer_desc> grow = {{PBKD_DWSEP3X3, 8, 12, 1, 1}}, tgrow = {{PBKD_CONV3X3, 8, 12, 1, 0}};
    pbkd_arch_desc tg = arch(2, 8, 6, 6, tgrow, 0, 1, 0), sg = arch(2, 8, 6, 6, grow, 2, 1, 0);
    CHECK(pbkd_arch_validate(&tg, &sg) == PBKD_ESHAPE);
    bad = arch(65536, 8, 300, 300, sl, 0, 1, 0);     // beyond 2^31 elements
    CHECK(pbkd_arch_validate(&bad, &bad) == PBKD_EUNSUPPORTED);
    CHECK(pbkd_block_workspace_bytes(&t, &bad) == 0);
    // create: refused before any device call
    pbkd_block_t *blk = reinterpret_cast<pbkd_block_t *>(1);
    pbkd_train_desc tr{0.9f, 0, 0.99f};
    const float *none[8] = {};
    CHECK(pbkd_block_create(&t, none, &s, none, &tr, nullptr, 0, nullptr, &blk) == PBKD_EINVAL && blk == nullptr);
    CHECK(pbkd_block_create(&t, none, &s, none, &tr, nullptr, 0, nullptr, nullptr) == PBKD_EINVAL);
    CHECK(pbkd_block_destroy(nullptr) == PBKD_OK);
    CHECK(pbkd_block_flops(nullptr, 0) == 0);
    float loss;
    CHECK(pbkd_block_last_loss(nullptr, &loss) == PBKD_EINVAL);
    double mse;
    CHECK(pbkd_feature_mse_noalloc(nullptr, nullptr, 4, &mse, nullptr) == PBKD_EINVAL);
    CHECK(pbkd_block_set_graph_mode(nullptr, 1) == PBKD_EINVAL);
    CHECK(pbkd_kernel_kinds() > 0 && pbkd_kernel_kind_name(0)[0] != 0 && pbkd_kernel_kind_name(-1)[0] == 0 &&
          pbkd_kernel_kind_name(pbkd_kernel_kinds())[0] == 0);
  }
  // ---- scheduler: exact-size output arrays, both policies, more workers than tasks, zero tasks
  {
    unsigned state = 7;
    for (int n = 0; n <= 13; ++n)
      for (int m = 1; m <= 6; ++m)
        for (int policy = 0; policy <= 1; ++policy) {
          std::vector<unsigned long long> w(n);
          unsigned long long total = 0;
          for (auto &v : w) { state = state * 1664525u + 1013904223u; v = 1 + (state >> 20); total += v; }
          std::vector<int> sob(n), order(n);
          std::vector<unsigned long long> load(m);
          CHECK(pbkd_schedule_blocks(n, w.data(), nullptr, m, policy, sob.data(), order.data(), load.data()) == PBKD_OK);
          unsigned long long sum = 0;
          for (auto v : load) sum += v;
          CHECK(sum == total);
          std::vector<int> count(m, 0);
          for (int i = 0; i < n; ++i) { CHECK(sob[i] >= 0 && sob[i] < m); ++count[sob[i]]; }
          for (int i = 0; i < n; ++i) CHECK(order[i] >= 0 && order[i] < count[sob[i]]);
        }
    int one[1], ord[1];
    unsigned long long w1[1] = {5};
    CHECK(pbkd_schedule_blocks(1, w1, nullptr, 0, 0, one, ord, nullptr) == PBKD_EINVAL);
    CHECK(pbkd_schedule_blocks(1, w1, nullptr, 2, 7, one, ord, nullptr) == PBKD_EINVAL);
    CHECK(pbkd_schedule_blocks(1, nullptr, nullptr, 2, 0, one, ord, nullptr) == PBKD_EINVAL);
    CHECK(pbkd_schedule_blocks(1, w1, nullptr, 2, 0, nullptr, ord, nullptr) == PBKD_EINVAL);
  }
  std::printf("ok\n");
  return 0;
}
