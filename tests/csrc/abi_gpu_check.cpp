// A plain C++ consumer of the C ABI on the GPU: no Python, no torch, no oracle.  Device memory comes from hipMalloc,
// every input is a constant vector of dyadic numbers, and every expected value is a closed form that binary32 holds
// exactly (Eq. 1c / Eq. 5 on constant gradients; geometric series of the momentum rule; (1 - alpha*wd)^u of the
// weight penalty; alpha0 / sigma of Eq. 6).  Exit status 0 and "abi gpu check ok" on success.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/rudra_ps.h"

#define CHECK(cond)                                                       \
  do {                                                                    \
    if (!(cond)) {                                                        \
      std::printf("CHECK failed line %d: %s\n", __LINE__, #cond);         \
      std::fflush(stdout);                                                \
      return 1;                                                           \
    }                                                                     \
  } while (0)

namespace {

const uint64_t P = 100003;  // several tiles and a ragged tail (P % 4 = 3)

float* device_constant(float value) {
  std::vector<float> h(P, value);
  float* d = nullptr;
  if (hipMalloc((void**)&d, P * sizeof(float)) != hipSuccess) return nullptr;
  if (hipMemcpy(d, h.data(), P * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
  return d;
}

// every element of the server's weights (or velocity) equals `want`
bool all_equal(rudra_ps_t* ps, float* scratch, float want, bool velocity = false) {
  if ((velocity ? rudra_ps_pull_velocity(ps, scratch) : rudra_ps_pull_weights(ps, scratch, nullptr)) != RUDRA_OK) return false;
  if (rudra_ps_sync(ps) != RUDRA_OK) return false;
  std::vector<float> h(P);
  if (hipMemcpy(h.data(), scratch, P * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return false;
  for (uint64_t k = 0; k < P; ++k)
    if (h[k] != want) {
      std::printf("element %llu: got %.9g want %.9g\n", (unsigned long long)k, h[k], want);
      return false;
    }
  return true;
}

rudra_ps_config_t base_config() {
  rudra_ps_config_t c;
  std::memset(&c, 0, sizeof(c));
  c.n_params = P;
  c.lr_scale = 1.0f;
  c.protocol = RUDRA_SOFTSYNC;
  c.lr_mode = RUDRA_LR_CONST;
  c.n_split = 1;
  return c;
}

}  // namespace

int main() {
  int n_dev = 0;
  CHECK(hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0);
  float* one = device_constant(1.0f);
  float* three = device_constant(3.0f);
  float* zero = device_constant(0.0f);
  float* scratch = device_constant(0.0f);
  CHECK(one && three && zero && scratch);
  rudra_push_result_t r;

  // --- Eq. 5 + Eq. 1c: lambda = 4, 1-softsync (c = 4), gradients 1,3,1,3 -> mean 2; alpha0 = 2^-4: theta_u = 1 - u/8
  {
    rudra_ps_config_t c = base_config();
    c.n_learners = 4;
    c.alpha0 = 0.0625f;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    for (int u = 0; u < 5; ++u)
      for (int l = 0; l < 4; ++l) {
        CHECK(rudra_ps_push_gradient(ps, (l & 1) ? three : one, (uint64_t)u, l, &r) == RUDRA_OK);
        CHECK(r.applied == (l == 3) && r.staleness == 0);
      }
    CHECK(all_equal(ps, scratch, 1.0f - 5 * 0.125f));
    uint64_t ts = 0;
    CHECK(rudra_ps_pull_weights(ps, nullptr, &ts) == RUDRA_OK && ts == 5);
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  }

  // --- momentum (rate inside the velocity), hardsync lambda = 2, g = 1, alpha = 1/4, m = 1/2:
  //     v_u = -alpha (1 - m^u) / (1 - m) = -(1 - 2^-u) / 2 ; theta_u = 1 + sum_{i<=u} v_i = 1 - u/2 + (1 - 2^-u)/2
  {
    rudra_ps_config_t c = base_config();
    c.n_learners = 2;
    c.protocol = RUDRA_HARDSYNC;
    c.alpha0 = 0.25f;
    c.momentum = 0.5f;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    const int U = 10;
    for (int u = 0; u < U; ++u)
      for (int l = 0; l < 2; ++l) CHECK(rudra_ps_push_gradient(ps, one, (uint64_t)u, l, &r) == RUDRA_OK);
    const float pw = std::ldexp(1.0f, -U);
    CHECK(all_equal(ps, scratch, -(1.0f - pw) / 2, /*velocity=*/true));
    CHECK(all_equal(ps, scratch, 1.0f - U / 2.0f + (1.0f - pw) / 2));
    CHECK(rudra_ps_push_gradient(ps, one, U - 1, 0, &r) == RUDRA_EHARDSYNC_STALE);  // staleness must be zero
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  }

  // --- weight penalty alone: zero gradients, alpha = 1/2, wd = 1/2: theta_u = (1 - alpha wd)^u = (3/4)^u
  {
    rudra_ps_config_t c = base_config();
    c.n_learners = 1;
    c.alpha0 = 0.5f;
    c.weight_decay = 0.5f;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    float want = 1.0f;
    for (int u = 0; u < 9; ++u) {  // 3^9 < 2^24: every power is exact in binary32
      CHECK(rudra_ps_push_gradient(ps, zero, (uint64_t)u, 0, &r) == RUDRA_OK && r.applied);
      want *= 0.75f;
    }
    CHECK(all_equal(ps, scratch, want));
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  }

  // --- Eq. 6, lambda-softsync (c = 1), lambda = 3: gradients stamped 0 arriving at timestamps 0,1,2,3,4 have
  //     sigma = 0,1,2,3,4 and rates alpha0 / max(1, sigma): theta = 1 - alpha0 (1 + 1 + 1/2 + 1/4) after four of them
  //     (sigma = 3 is left out: 1/3 is not dyadic), pushed both one by one and as one run
  for (int batched = 0; batched < 2; ++batched) {
    rudra_ps_config_t c = base_config();
    c.n_learners = 3;
    c.n_split = 3;
    c.lr_mode = RUDRA_LR_AVG_STALENESS;
    c.alpha0 = 0.125f;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    const uint64_t stamps[5] = {0, 0, 0, 3, 0};  // the fourth message is fresh (sigma 0, full rate, gradient zero)
    const float* grads[5] = {one, one, one, zero, one};
    const uint64_t sigma[5] = {0, 1, 2, 0, 4};
    rudra_push_result_t res[5];
    if (batched) {
      uint32_t handled = 0;
      CHECK(rudra_ps_push_batch(ps, grads, stamps, nullptr, 5, res, &handled) == RUDRA_OK && handled == 5);
    } else {
      for (int i = 0; i < 5; ++i) CHECK(rudra_ps_push_gradient(ps, grads[i], stamps[i], -1, &res[i]) == RUDRA_OK);
    }
    for (int i = 0; i < 5; ++i) {
      CHECK(res[i].staleness == sigma[i] && res[i].applied == 1 && res[i].ts_after == (uint64_t)i + 1);
      CHECK(res[i].lr_used == 0.125f / (sigma[i] > 1 ? (float)sigma[i] : 1.0f));
    }
    CHECK(all_equal(ps, scratch, 1.0f - 0.125f * (1.0f + 1.0f + 0.5f + 0.25f)));
    rudra_ps_stats_t st;
    CHECK(rudra_ps_stats(ps, &st) == RUDRA_OK);
    CHECK(st.n_updates == 5 && st.sigma_sum == 7 && st.sigma_max == 4 && st.n_apply_launches == (batched ? 1u : 5u));
    CHECK(rudra_ps_push_gradient(ps, one, 6, 0, &r) == RUDRA_EFUTURE_TS);
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
  }

  // --- tree node: (1 + 3 + 1 + 3) * (1/4) = 2, relayed as four gradients stamped 0 to a root with c = 4
  {
    const float* group[4] = {one, three, one, three};
    CHECK(rudra_ps_leaf_mean(group, 4, P, scratch, 0, nullptr) == RUDRA_OK);
    rudra_ps_config_t c = base_config();
    c.n_learners = 4;
    c.alpha0 = 0.25f;
    c.max_aggregate = 4;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    const uint64_t stamps[4] = {0, 0, 0, 0};
    CHECK(rudra_ps_push_aggregate(ps, scratch, stamps, 4, &r) == RUDRA_OK && r.applied == 1);
    float* out = device_constant(0.0f);
    CHECK(out && all_equal(ps, out, 1.0f - 0.25f * 2.0f));   // sum 4 * 2, mean 2
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
    (void)hipFree(out);
  }

  // --- the entry point that allocates nothing: one update of c = 2 gradients (1 and 3: mean 2) on the caller's own theta = 1
  //     and v = 0 with alpha = 1/4, m = 1/2: v = -1/2, theta = 1/2; norms: sum gbar^2 = 4P, sum theta^2 = P/4, sum v^2 = P/4,
  //     max |theta| = 1/2 (all exact in binary64); then a second call on the same state: v = -1/4 - 1/2 = -3/4, theta = -1/4
  {
    float* theta = device_constant(1.0f);
    float* vel = device_constant(0.0f);
    double* norms = nullptr;
    CHECK(theta && vel && hipMalloc((void**)&norms, 4 * sizeof(double)) == hipSuccess);
    const float* pair[2] = {one, three};
    double h[4];
    CHECK(rudra_ps_apply_update_noalloc(pair, 2, P, theta, vel, 0.25f, 0.5f, 0.0f, RUDRA_OPT_SGD, 0.0f, norms, 0, nullptr) == RUDRA_OK);
    CHECK(hipMemcpy(h, norms, sizeof(h), hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(h[0] == 4.0 * P && h[1] == 0.25 * P && h[2] == 0.25 * P && h[3] == 0.5);
    CHECK(rudra_ps_apply_update_noalloc(pair, 2, P, theta, vel, 0.25f, 0.5f, 0.0f, RUDRA_OPT_SGD, 0.0f, norms, 0, nullptr) == RUDRA_OK);
    CHECK(hipMemcpy(h, norms, sizeof(h), hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(h[0] == 4.0 * P && h[1] == 0.0625 * P && h[2] == 0.5625 * P && h[3] == 0.25);
    std::vector<float> ht(P), hv(P);
    CHECK(hipMemcpy(ht.data(), theta, P * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(hipMemcpy(hv.data(), vel, P * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    for (uint64_t k = 0; k < P; ++k) CHECK(ht[k] == -0.25f && hv[k] == -0.75f);
    (void)hipFree(theta); (void)hipFree(vel); (void)hipFree(norms);
  }

  // --- a reader on its own stream (Sec. 3.3: communication buffer): with two weight buffers it takes the weights of
  //     timestamp 1 (theta = 1 - 1/4 = 3/4 after one update with g = 1, alpha = 1/4), two more updates are enqueued (the
  //     second overwrites that buffer and must wait for the reader), and its copy still holds 3/4 everywhere
  {
    rudra_ps_config_t c = base_config();
    c.n_learners = 1;
    c.alpha0 = 0.25f;
    c.flags = RUDRA_FLAG_DOUBLE_BUFFER;
    hipStream_t server, reader;
    CHECK(hipStreamCreate(&server) == hipSuccess && hipStreamCreate(&reader) == hipSuccess);
    c.stream = server;
    rudra_ps_t* ps = nullptr;
    CHECK(rudra_ps_create(&c, one, &ps) == RUDRA_OK);
    CHECK(rudra_ps_push_gradient(ps, one, 0, 0, &r) == RUDRA_OK && r.applied);
    const float* view = nullptr;
    uint64_t ts = 0, ticket = 0;
    CHECK(rudra_ps_weights_acquire(ps, reader, &view, &ts, &ticket) == RUDRA_OK && ts == 1 && view);
    float* copy = device_constant(0.0f);
    CHECK(copy && hipMemcpyAsync(copy, view, P * sizeof(float), hipMemcpyDeviceToDevice, reader) == hipSuccess);
    CHECK(rudra_ps_weights_release(ps, ticket, reader) == RUDRA_OK);
    CHECK(rudra_ps_push_gradient(ps, one, 1, 0, &r) == RUDRA_OK && r.applied);
    CHECK(rudra_ps_push_gradient(ps, one, 2, 0, &r) == RUDRA_OK && r.applied);
    CHECK(rudra_ps_weights_release(ps, ticket, reader) == RUDRA_ESTATE);   // the overwriting launch is enqueued: too late now
    // the same in one call: the weights of timestamp 3 (1/4) pulled on the reader's stream, then two more updates
    float* pulled = device_constant(0.0f);
    CHECK(pulled && rudra_ps_pull_weights_on(ps, pulled, reader, &ts) == RUDRA_OK && ts == 3);
    CHECK(rudra_ps_push_gradient(ps, one, 3, 0, &r) == RUDRA_OK && r.applied);
    CHECK(rudra_ps_push_gradient(ps, one, 4, 0, &r) == RUDRA_OK && r.applied);
    CHECK(hipStreamSynchronize(reader) == hipSuccess && rudra_ps_sync(ps) == RUDRA_OK);
    std::vector<float> hc(P);
    CHECK(hipMemcpy(hc.data(), copy, P * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    for (uint64_t k = 0; k < P; ++k) CHECK(hc[k] == 0.75f);
    CHECK(hipMemcpy(hc.data(), pulled, P * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
    for (uint64_t k = 0; k < P; ++k) CHECK(hc[k] == 0.25f);
    CHECK(all_equal(ps, scratch, -0.25f));
    rudra_ps_stats_t st;
    CHECK(rudra_ps_stats(ps, &st) == RUDRA_OK && st.n_weight_acquires == 1 && st.n_reader_waits == 2);
    (void)hipFree(pulled);
    CHECK(rudra_ps_destroy(ps) == RUDRA_OK);
    (void)hipFree(copy);
    (void)hipStreamDestroy(server); (void)hipStreamDestroy(reader);
  }

  (void)hipFree(one); (void)hipFree(three); (void)hipFree(zero); (void)hipFree(scratch);
  std::printf("abi gpu check ok\n");
  return 0;
}
