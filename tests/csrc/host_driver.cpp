// Host-only driver for sanitizer runs: exercises the library's control plane (RUDRA_FLAG_CONTROL_ONLY: no device
// work) through the C ABI: rejections, ring eviction, histogram growth, clocks, statistics, many threads.
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/rudra_ps.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      std::printf("CHECK failed line %d: %s\n", __LINE__, #cond); \
      return 1;                                                  \
    }                                                            \
  } while (0)

int main() {
  rudra_ps_config_t cfg;
  std::memset(&cfg, 0, sizeof(cfg));
  cfg.n_params = 1000;
  cfg.n_learners = 7;
  cfg.n_split = 2;  // c = 3
  cfg.protocol = RUDRA_SOFTSYNC;
  cfg.lr_mode = RUDRA_LR_AVG_STALENESS;
  cfg.alpha0 = 0.01f;
  cfg.lr_scale = 1.0f;
  cfg.flags = RUDRA_FLAG_CONTROL_ONLY;
  cfg.clock_ring = 5;
  rudra_ps_t* ps = nullptr;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_OK);
  rudra_push_result_t r;
  uint64_t ts = 0;
  for (int i = 0; i < 300; ++i) {
    const uint64_t stamp = (i % 11 == 0) ? 0 : ts;  // occasionally very stale: the histogram has to grow
    CHECK(rudra_ps_push_gradient(ps, nullptr, stamp, i % 7, &r) == RUDRA_OK);
    CHECK(r.staleness == ts - stamp);
    ts = r.ts_after;
  }
  CHECK(ts == 100);
  CHECK(rudra_ps_push_gradient(ps, nullptr, ts + 1, 0, &r) == RUDRA_EFUTURE_TS);
  CHECK(rudra_ps_push_gradient(ps, nullptr, ts, 7, &r) == RUDRA_EINVAL);
  CHECK(rudra_ps_push_gradient(ps, nullptr, ts, -2, nullptr) == RUDRA_EINVAL);
  uint64_t clock[3];
  uint32_t n = 0;
  double avg = 0;
  float lr = 0;
  CHECK(rudra_ps_vector_clock(ps, 99, clock, 3, &n, &avg, &lr) == RUDRA_OK && n == 3);
  CHECK(rudra_ps_vector_clock(ps, 95, clock, 3, &n, nullptr, nullptr) == RUDRA_OK);
  CHECK(rudra_ps_vector_clock(ps, 94, clock, 3, &n, nullptr, nullptr) == RUDRA_ERANGE);   // left the ring of 5
  CHECK(rudra_ps_vector_clock(ps, 100, clock, 3, &n, nullptr, nullptr) == RUDRA_ERANGE);  // not yet
  CHECK(rudra_ps_vector_clock(ps, 99, clock, 2, &n, nullptr, nullptr) == RUDRA_ERANGE);   // buffer too small
  rudra_ps_stats_t st;
  CHECK(rudra_ps_stats(ps, &st) == RUDRA_OK);
  CHECK(st.n_pushes == 300 && st.n_updates == 100 && st.n_rejected == 3 && st.pending == 0 && st.c == 3);
  std::vector<uint64_t> hist(st.hist_len);
  uint64_t hn = 0;
  CHECK(rudra_ps_staleness_hist(ps, hist.data(), 1, &hn) == RUDRA_ERANGE && hn == st.hist_len);
  CHECK(rudra_ps_staleness_hist(ps, hist.data(), hist.size(), &hn) == RUDRA_OK);
  uint64_t total = 0, weighted = 0;
  for (size_t s = 0; s < hist.size(); ++s) { total += hist[s]; weighted += s * hist[s]; }
  CHECK(total == 300 && weighted == st.sigma_sum && st.sigma_max + 1 == st.hist_len);
  float dummy;
  CHECK(rudra_ps_pull_weights(ps, &dummy, &ts) == RUDRA_ESTATE);
  CHECK(rudra_ps_pull_weights(ps, nullptr, &ts) == RUDRA_OK && ts == 100);
  const float* view = nullptr;
  CHECK(rudra_ps_weights_view(ps, &view, nullptr) == RUDRA_ESTATE);
  CHECK(rudra_ps_set_lr(ps, 0.001f) == RUDRA_OK && rudra_ps_sync(ps) == RUDRA_OK);
  // many threads at once: the mutex serialises them
  std::vector<std::thread> th;
  for (int t = 0; t < 6; ++t)
    th.emplace_back([ps, t] { for (int i = 0; i < 3000; ++i) rudra_ps_push_gradient(ps, nullptr, 0, t, nullptr); });
  for (auto& x : th) x.join();
  CHECK(rudra_ps_stats(ps, &st) == RUDRA_OK);
  CHECK(st.n_pushes == 300 + 18000 && st.n_updates == 100 + 6000);
  // runs of messages in one call, from several threads; a run that holds a message from the future stops there
  {
    std::vector<uint64_t> stamps(50, 0);
    std::vector<int32_t> who(50);
    for (int i = 0; i < 50; ++i) who[i] = i % 7;
    std::vector<rudra_push_result_t> res(50);
    uint32_t handled = 0;
    CHECK(rudra_ps_push_batch(ps, nullptr, stamps.data(), who.data(), 50, res.data(), &handled) == RUDRA_OK && handled == 50);
    CHECK(res[49].ts_after == 6100 + 16 && res[49].pending == 2);
    stamps[20] = ~0ull;
    CHECK(rudra_ps_push_batch(ps, nullptr, stamps.data(), nullptr, 50, nullptr, &handled) == RUDRA_EFUTURE_TS && handled == 20);
    CHECK(rudra_ps_push_batch(ps, nullptr, nullptr, nullptr, 0, nullptr, nullptr) == RUDRA_OK);
    CHECK(rudra_ps_push_batch(ps, nullptr, nullptr, nullptr, 3, nullptr, nullptr) == RUDRA_EINVAL);
    stamps[20] = 0;
    std::vector<std::thread> tb;
    for (int t = 0; t < 4; ++t)
      tb.emplace_back([ps, &stamps] { for (int i = 0; i < 200; ++i) rudra_ps_push_batch(ps, nullptr, stamps.data(), nullptr, 50, nullptr, nullptr); });
    for (auto& x : tb) x.join();
    CHECK(rudra_ps_stats(ps, &st) == RUDRA_OK);
    CHECK(st.n_pushes == 18300 + 50 + 20 + 4 * 200 * 50 && st.n_rejected == 3 + 1);
  }
  CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  // hardsync: duplicates and stale gradients
  cfg.protocol = RUDRA_HARDSYNC;
  cfg.lr_mode = RUDRA_LR_CONST;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_OK);
  for (int l = 0; l < 6; ++l) CHECK(rudra_ps_push_gradient(ps, nullptr, 0, l, &r) == RUDRA_OK && !r.applied);
  CHECK(rudra_ps_push_gradient(ps, nullptr, 0, 3, &r) == RUDRA_EHARDSYNC_DUP);
  CHECK(rudra_ps_push_gradient(ps, nullptr, 0, 6, &r) == RUDRA_OK && r.applied && r.ts_after == 1);
  CHECK(rudra_ps_push_gradient(ps, nullptr, 0, 0, &r) == RUDRA_EHARDSYNC_STALE);
  CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  // relayed averages (server tree): several timestamps per message, overshoot of c under softsync, none under hardsync
  cfg.max_aggregate = 3;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_OK);  // hardsync, lambda = 7
  {
    const uint64_t zeros[4] = {0, 0, 0, 0};
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 3, &r) == RUDRA_OK && r.pending == 3);
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 3, &r) == RUDRA_OK && r.pending == 6);
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 2, &r) == RUDRA_EHARDSYNC_DUP);  // 8 > lambda
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 4, &r) == RUDRA_EINVAL);         // more than max_aggregate
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 1, &r) == RUDRA_OK && r.applied && r.ts_after == 1);
    uint64_t clk[9]; uint32_t cn = 0;
    CHECK(rudra_ps_vector_clock(ps, 0, clk, 9, &cn, nullptr, nullptr) == RUDRA_OK && cn == 7);
  }
  CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  cfg.protocol = RUDRA_SOFTSYNC;  // c = 3, messages of up to 3: an update can collect 5
  cfg.lr_mode = RUDRA_LR_AVG_STALENESS;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_OK);
  {
    const uint64_t zeros[3] = {0, 0, 0};
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 2, &r) == RUDRA_OK && !r.applied);
    CHECK(rudra_ps_push_aggregate(ps, nullptr, zeros, 3, &r) == RUDRA_OK && r.applied && r.pending == 0);
    uint64_t clk[5]; uint32_t cn = 0;
    CHECK(rudra_ps_vector_clock(ps, 0, clk, 5, &cn, nullptr, nullptr) == RUDRA_OK && cn == 5);
    const uint64_t future[1] = {9};
    CHECK(rudra_ps_push_aggregate(ps, nullptr, future, 1, &r) == RUDRA_EFUTURE_TS);
    // what needs device memory says so in control-only mode
    const float* p = nullptr; uint64_t ticket = 0;
    CHECK(rudra_ps_weights_acquire(ps, nullptr, &p, nullptr, &ticket) == RUDRA_ESTATE);
    CHECK(rudra_ps_weights_release(ps, 0, nullptr) == RUDRA_ESTATE);
    float target[4];
    CHECK(rudra_ps_pull_weights_on(ps, target, nullptr, nullptr) == RUDRA_ESTATE);
    CHECK(rudra_ps_pull_weights_on(ps, nullptr, nullptr, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_pull_weights_on(nullptr, target, nullptr, nullptr) == RUDRA_EINVAL);
    alignas(16) float aligned[4];
    float* const dsts[1] = {aligned};
    float* const odd[1] = {aligned + 1};
    CHECK(rudra_ps_broadcast_weights(ps, dsts, 1, nullptr, nullptr) == RUDRA_ESTATE);
    CHECK(rudra_ps_broadcast_weights(ps, odd, 1, nullptr, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_broadcast_weights(ps, dsts, 0, nullptr, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_broadcast_weights(ps, nullptr, 1, nullptr, nullptr) == RUDRA_EINVAL);
    float f;
    CHECK(rudra_ps_pull_velocity(ps, &f) == RUDRA_ESTATE);
    uint32_t grid = 0, block = 0, lds = 0; uint64_t tiles = 0;
    CHECK(rudra_ps_launch_shape(ps, 0, &grid, &block, &tiles, &lds) == RUDRA_OK && block == 64 && tiles == 4 && grid == 4);   // 250 float4 in tiles of 64
    CHECK(rudra_ps_launch_shape(ps, 1, &grid, nullptr, nullptr, nullptr) == RUDRA_OK && grid == 4);
  }
  CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  cfg.max_aggregate = 0;
  // configurations that are refused
  cfg.n_split = 9;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL && ps == nullptr);
  cfg.n_split = 2;
  cfg.lr_scale = 0.0f;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL);
  cfg.lr_scale = 1.0f;
  cfg.launch_state_loads = 4;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL);
  cfg.launch_state_loads = 0;
  cfg.launch_phased = 3;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL);
  cfg.launch_phased = 0;
  cfg.n_learners = 1u << 25;  // a vector clock of 2^25 entries
  cfg.n_split = 1;
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL);
  cfg.n_learners = 4; cfg.c_override = 0xFFFFFFFFu; cfg.max_aggregate = 4096;   // c + max_aggregate - 1 would wrap in 32 bits
  CHECK(rudra_ps_create(&cfg, nullptr, &ps) == RUDRA_EINVAL);
  // the entry point that allocates nothing rejects bad arguments before it touches a device
  {
    float x[4] = {0, 0, 0, 0}; double nrm[4];
    const float* one[1] = {x};
    CHECK(rudra_ps_apply_update_noalloc(nullptr, 1, 4, x, x, 0.1f, 0.f, 0.f, RUDRA_OPT_SGD, 0.f, nrm, 0, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_apply_update_noalloc(one, 65, 4, x, x, 0.1f, 0.f, 0.f, RUDRA_OPT_SGD, 0.f, nrm, 0, nullptr) == RUDRA_ERANGE);
    CHECK(rudra_ps_apply_update_noalloc(one, 1, (1ull << 27) + 1, x, x, 0.1f, 0.f, 0.f, RUDRA_OPT_SGD, 0.f, nrm, 0, nullptr) == RUDRA_ERANGE);
    CHECK(rudra_ps_apply_update_noalloc(one, 1, 4, x, nullptr, 0.1f, 0.9f, 0.f, RUDRA_OPT_SGD, 0.f, nrm, 0, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_apply_update_noalloc(one, 1, 4, x, x, 0.1f, 0.9f, 0.f, RUDRA_OPT_ADAGRAD, 0.f, nrm, 0, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_apply_update_noalloc(one, 1, 4, x, x, 0.1f, 0.f, 0.f, 7, 0.f, nrm, 0, nullptr) == RUDRA_EINVAL);
    CHECK(rudra_ps_apply_update_noalloc(one, 1, 4, x, x, 0.1f, 0.f, 0.f, RUDRA_OPT_SGD, 0.f, nrm, -1, nullptr) == RUDRA_EINVAL);
  }
  std::printf("host driver ok\n");
  return 0;
}
