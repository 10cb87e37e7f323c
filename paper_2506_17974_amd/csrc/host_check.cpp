// Host-only exercise of the planner and of the C ABI's argument checking, built with
// -fsanitize=address,undefined (python -m paper_2506_17974_amd.build --sanitize) and run on a machine
// without a GPU: every call below must return the documented status, and the sanitizers must stay
// silent.  Nothing here computes anything of the method.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <vector>

#include "lqsgd.h"

static int failures = 0;
#define EXPECT(cond)                                                         \
  do {                                                                       \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

static lqsgd_config cfg(int rank, int bp, int bq, int W, float alpha = 255.0f, uint32_t flags = 0) {
  lqsgd_config c;
  c.rank = rank; c.bits_p = bp; c.bits_q = bq; c.workers = W; c.alpha = alpha; c.flags = flags;
  return c;
}

// Every work item of every sweep lies inside its layer, and the items of a sweep cover each
// (layer, worker) exactly once.
static void check_tiles(const lqsgd_config& c, const std::vector<lqsgd_layer>& layers) {
  for (int sweep = 0; sweep < 4; ++sweep) {
    const int64_t n = lqsgd_plan_tiles(&c, layers.data(), (int32_t)layers.size(), sweep, nullptr, 0);
    EXPECT(n >= 0);
    if (n < 0) return;
    std::vector<int32_t> t((size_t)n * 6 + 6, -7);
    EXPECT(lqsgd_plan_tiles(&c, layers.data(), (int32_t)layers.size(), sweep, t.data(), n) == n);
    std::vector<int64_t> covered(layers.size() * (size_t)c.workers, 0);
    for (int64_t i = 0; i < n; ++i) {
      const int32_t* o = &t[(size_t)i * 6];
      EXPECT(o[0] >= 0 && o[0] < (int32_t)layers.size());
      if (o[0] < 0 || o[0] >= (int32_t)layers.size()) continue;
      const lqsgd_layer& l = layers[(size_t)o[0]];
      EXPECT(!(l.flags & LQSGD_LAYER_VECTOR));
      EXPECT(o[1] >= 0 && o[1] < c.workers);
      EXPECT(o[2] >= 0 && o[3] > 0 && o[2] + o[3] <= l.rows);
      EXPECT(o[4] >= 0 && o[5] > 0 && o[4] + o[5] <= l.cols);
      if (o[1] >= 0 && o[1] < c.workers) covered[(size_t)o[0] * c.workers + o[1]] += (int64_t)o[3] * o[5];
    }
    EXPECT(t[(size_t)n * 6] == -7);                  // nothing written past the items asked for
    for (size_t li = 0; li < layers.size(); ++li) {
      if (layers[li].flags & LQSGD_LAYER_VECTOR) continue;
      const int wmax = sweep == 3 ? 1 : c.workers;  // the G-hat pass lists worker 0's items only
      for (int w = 0; w < wmax; ++w)
        EXPECT(covered[li * c.workers + w] == (int64_t)layers[li].rows * layers[li].cols);
    }
  }
}

int main() {
  lqsgd_plan_info info;
  std::vector<lqsgd_layer> resnet = {{64, 27, 0}, {64, 576, 0}, {128, 1152, 0}, {512, 4608, 0}, {10, 512, 0},
                                     {64, 1, LQSGD_LAYER_VECTOR}, {10, 1, LQSGD_LAYER_VECTOR}};
  // ---- valid plans over ranks, flags and shapes, with the work lists checked --------------------
  for (int rank : {1, 2, 3, 4, 7, 8, 12, 16, 20, 32, 50, 64})
    for (uint32_t flags : {0u, (uint32_t)LQSGD_FLAG_EAGER_RESIDUAL, (uint32_t)LQSGD_FLAG_AGGREGATE_FIRST,
                           (uint32_t)(LQSGD_FLAG_BF16_GRADIENTS | LQSGD_FLAG_AGGREGATE_FIRST)}) {
      const lqsgd_config c = cfg(rank, 8, 4, 3, 255.0f, flags);
      std::memset(&info, 0, sizeof info);
      EXPECT(lqsgd_plan_query(&c, resnet.data(), (int32_t)resnet.size(), &info) == LQSGD_OK);
      EXPECT(info.n_matrix == 5 && info.n_vector == 2 && info.rank_pad >= rank && info.device_bytes > 0);
      EXPECT(info.residual_stride >= 64 * 27 + 64 * 576 + 128 * 1152 + 512 * 4608 + 10 * 512);
      check_tiles(c, resnet);
    }
  std::mt19937 rng(20250617);
  for (int trial = 0; trial < 60; ++trial) {
    std::vector<lqsgd_layer> ls;
    const int n = 1 + (int)(rng() % 6);
    for (int i = 0; i < n; ++i) {
      lqsgd_layer l;
      const bool vec = rng() % 5 == 0;
      l.rows = 1 + (int32_t)(rng() % (trial % 7 == 0 ? 20000 : 700));
      l.cols = vec ? 1 : 1 + (int32_t)(rng() % (trial % 5 == 0 ? 9000 : 900));
      l.flags = vec ? LQSGD_LAYER_VECTOR : LQSGD_LAYER_MATRIX;
      ls.push_back(l);
    }
    const lqsgd_config c = cfg(1 + (int)(rng() % 64), (int)(rng() % 9), (int)(rng() % 9), 1 + (int)(rng() % 64), 0.5f + (float)(rng() % 1000));
    EXPECT(lqsgd_plan_query(&c, ls.data(), n, &info) == LQSGD_OK);
    check_tiles(c, ls);
  }
  // ---- rejected configurations ---------------------------------------------------------------
  {
    lqsgd_layer one = {256, 128, 0};
    lqsgd_config c = cfg(2, 8, 8, 2);
    EXPECT(lqsgd_plan_query(nullptr, &one, 1, &info) == LQSGD_EINVAL);
    EXPECT(lqsgd_plan_query(&c, nullptr, 1, &info) == LQSGD_EINVAL);
    EXPECT(lqsgd_plan_query(&c, &one, 1, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_plan_query(&c, &one, 0, &info) == LQSGD_EINVAL);
    EXPECT(std::strlen(lqsgd_last_error(nullptr)) > 0);
    c = cfg(0, 8, 8, 2);  EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(65, 8, 8, 2); EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EUNSUPPORTED);
    c = cfg(2, 9, 8, 2);  EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, -1, 2); EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 0);  EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 65); EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 2, 0.0f);  EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 2, -3.0f); EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 2, 255.0f, 1u << 9); EXPECT(lqsgd_plan_query(&c, &one, 1, &info) == LQSGD_EINVAL);
    c = cfg(2, 8, 8, 2);
    lqsgd_layer bad = {0, 128, 0};            EXPECT(lqsgd_plan_query(&c, &bad, 1, &info) == LQSGD_ESHAPE);
    bad = {256, -1, 0};                       EXPECT(lqsgd_plan_query(&c, &bad, 1, &info) == LQSGD_ESHAPE);
    bad = {65536, 32768, 0};                  EXPECT(lqsgd_plan_query(&c, &bad, 1, &info) == LQSGD_ESHAPE);
    bad = {16, 2, LQSGD_LAYER_VECTOR};        EXPECT(lqsgd_plan_query(&c, &bad, 1, &info) == LQSGD_ESHAPE);
    bad = {16, 16, 8};                        EXPECT(lqsgd_plan_query(&c, &bad, 1, &info) == LQSGD_EINVAL);
    EXPECT(lqsgd_plan_tiles(&c, &one, 1, 4, nullptr, 0) == LQSGD_EINVAL);
    EXPECT(lqsgd_plan_tiles(&c, &one, 1, -1, nullptr, 0) == LQSGD_EINVAL);
  }
  // ---- the ABI on NULL handles and, with no GPU in this machine, a create that must fail cleanly --
  {
    EXPECT(lqsgd_destroy(nullptr) == LQSGD_OK);
    EXPECT(lqsgd_synchronize(nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_step(nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_step_update(nullptr, nullptr, nullptr, 0.1f) == LQSGD_EINVAL);
    EXPECT(lqsgd_compress(nullptr, LQSGD_PHASE_P, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_decompress(nullptr, LQSGD_PHASE_Q) == LQSGD_EINVAL);
    EXPECT(lqsgd_set_q(nullptr, 0, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_get_state(nullptr, 0, 0, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_set_state(nullptr, 0, 0, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_get_packet(nullptr, 0, 0, 0, nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_set_packet(nullptr, 0, 0, 0, nullptr, nullptr, 1.0f) == LQSGD_EINVAL);
    EXPECT(lqsgd_get_packet_raw(nullptr, 0, 0, 0, nullptr, nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_packet_device(nullptr, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_get_factor(nullptr, 0, 0, 0, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_set_factor(nullptr, 0, 0, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_timing_enable(nullptr, 1) == LQSGD_EINVAL);
    EXPECT(lqsgd_timing_read(nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_wire_bytes(nullptr) == LQSGD_EINVAL);
    EXPECT(std::strcmp(lqsgd_launched_kernel(nullptr, 0), "") == 0);
    EXPECT(std::strlen(lqsgd_kernel_name(LQSGD_KERNEL_ORTH)) > 0 && std::strcmp(lqsgd_kernel_name(77), "") == 0);
    lqsgd_ctx* ctx = reinterpret_cast<lqsgd_ctx*>(0x1);
    const lqsgd_config c = cfg(4, 8, 8, 2);
    EXPECT(lqsgd_create(&c, resnet.data(), (int32_t)resnet.size(), nullptr, nullptr) == LQSGD_EINVAL);
    const int rc = lqsgd_create(&c, resnet.data(), (int32_t)resnet.size(), nullptr, &ctx);
    if (rc == LQSGD_OK) {                       // a GPU is present after all: the context works and goes away again
      EXPECT(ctx != nullptr);
      EXPECT(lqsgd_wire_bytes(ctx) > 0);
      EXPECT(lqsgd_destroy(ctx) == LQSGD_OK);
    } else {
      EXPECT(ctx == nullptr);
      EXPECT(rc == LQSGD_EHIP || rc == LQSGD_ENOMEM);
      EXPECT(std::strlen(lqsgd_last_error(nullptr)) > 0);
    }
    lqsgd_config badc = cfg(4, 8, 8, 0);
    EXPECT(lqsgd_create(&badc, resnet.data(), (int32_t)resnet.size(), nullptr, &ctx) == LQSGD_EINVAL && ctx == nullptr);
    const float* grads[4] = {nullptr, nullptr, nullptr, nullptr};
    EXPECT(lqsgd_step_static(nullptr, resnet.data(), 1, nullptr, grads, nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_step_static(&c, resnet.data(), 1, nullptr, nullptr, nullptr, nullptr, nullptr) == LQSGD_EINVAL);
    EXPECT(lqsgd_step_static(&c, resnet.data(), 1, nullptr, grads, nullptr, nullptr, nullptr) != LQSGD_OK);
  }
  if (failures) {
    std::printf("host_check: %d check(s) failed\n", failures);
    return 1;
  }
  std::printf("host_check: all checks passed\n");
  return 0;
}
