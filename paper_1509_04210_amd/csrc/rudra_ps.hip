// Host control plane and C ABI of the Rudra parameter-server update path (see include/rudra_ps.h).
//
// Everything per message is O(1) integer work on the host (timestamps, staleness, vector
// clock, trigger: Sec. 3.1; learning rate: Sec. 3.2 / Sec. 5.1 Eq. 6); the only device work is
// the fused kernel launch on the c-th gradient.  No data crosses the host-device boundary on
// the push path and push never waits for the GPU.
#include "../../include/rudra_ps.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <exception>
#include <new>
#include <vector>

#include "apply_update.hip.h"

using rudra::BatchPlan;
using rudra::GradSet;
using rudra::kMaxBatchUpdates;
using rudra::kMaxFused;
using rudra::kNumNorms;
using rudra::UpdateArgs;

// Scratch of rudra_ps_apply_update_noalloc (see there).  Every GPU the library runs on holds its own copy at its own
// address; host code reaches it only through the address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) double g_noalloc_scratch[131072 * rudra::kNumNorms];

namespace {

constexpr uint32_t kDefaultBlock = 64;   // one wavefront per workgroup: finest dispatch granularity, measured fastest
constexpr uint32_t kDefaultUnroll = 4;
constexpr uint32_t kDefaultVec = 1;
constexpr uint32_t kInFlightKiBPerCu = 48;  // measured optimum of outstanding load bytes per compute unit
// Below this many parameters a launch is only a few generations of resident waves: capping the occupancy then mostly
// idles the chip during ramp-up and tail (c = 18: 2M parameters 6040 vs 5280 GB/s uncapped vs 26 waves, 4M 6250 vs 6070;
// from 8M on the cap wins, 6620 vs 6380).
constexpr uint64_t kSmallVector = 6000000;
constexpr uint32_t kDefaultClockRing = 1024;
constexpr uint64_t kMaxClockEntries = 1ull << 24;  // gradients one update may collect (c + max_aggregate - 1)
constexpr uint64_t kMaxRingEntries = 1ull << 27;   // timestamps the ring of closed clocks may hold (1 GiB of host memory)
constexpr uint32_t kTimerRing = 256;  // event pairs in flight in TIME_KERNELS mode
// Batched launches (measured at 72M parameters, c = 1, 4 to 64 messages per launch, and at 1.0M and 131k parameters):
// 26 resident waves are best or equal everywhere (16: -3 to -12 %, 32: -1 to -3 %): between two loads a wave does a
// whole update's arithmetic, so it takes more waves than the single-update kernel to keep the memory system busy.
constexpr uint32_t kBatchWavesPerCu = 26;

// Makes `device` current for the calling thread and puts the previous one back on scope exit: a library call must
// not leave the caller's thread on another device.
class DeviceGuard {
 public:
  explicit DeviceGuard(int device) {  // device < 0: no device work in this call, touch nothing
    if (device < 0) return;
    err_ = hipGetDevice(&prev_);
    if (err_ == hipSuccess && prev_ != device) {
      err_ = hipSetDevice(device);
      changed_ = err_ == hipSuccess;
    }
  }
  ~DeviceGuard() {
    if (changed_) (void)hipSetDevice(prev_);
  }
  DeviceGuard(const DeviceGuard&) = delete;
  DeviceGuard& operator=(const DeviceGuard&) = delete;
  hipError_t error() const { return err_; }

 private:
  int prev_ = 0;
  bool changed_ = false;
  hipError_t err_ = hipSuccess;
};

// rudra_ps_apply_update_noalloc: norm slots of its launch live in a file-scope device array instead of hipMalloc'ed
// memory: one slot (kNumNorms doubles) per tile of kNoAllocBlock float4 positions.
constexpr uint32_t kNoAllocBlock = 256;
constexpr uint32_t kNoAllocSlots = 131072;  // 4 MiB of slots per GPU, held until the process ends
constexpr uint64_t kNoAllocMaxParams = (uint64_t)kNoAllocSlots * kNoAllocBlock * 4;  // 134 217 728 parameters
constexpr int kNoAllocMaxDevices = 64;

static_assert(sizeof(g_noalloc_scratch) == (size_t)kNoAllocSlots * kNumNorms * sizeof(double), "scratch array and slot count disagree");
std::mutex g_noalloc_mu;
double* g_noalloc_slots[kNoAllocMaxDevices] = {};  // per device: address of its copy of g_noalloc_scratch
uint32_t g_noalloc_cus[kNoAllocMaxDevices] = {};   // per device: its compute units (looked up with the address)

struct Pending {
  const float* ptr;
  float weight;
};

struct DeferredUpdate {
  uint32_t n_grads;  // entries of deferred_grads it consumes
  uint32_t count;    // learner gradients it stands for (the divisor of the mean; > n_grads with relayed averages)
  float lr;
  bool weighted;
};

}  // namespace

struct rudra_ps {
  rudra_ps_config_t cfg;
  std::mutex mu;
  hipStream_t stream = nullptr;
  uint32_t c = 0;
  bool control_only = false, accumulate = false, want_norms = false, time_kernels = false, check_pointers = false;
  bool failed = false;
  int last_hip_error = 0;

  // device state (owned)
  float* theta2[2] = {nullptr, nullptr};  // [1] only with DOUBLE_BUFFER
  uint32_t cur = 0;                        // which of them holds the weights of ts_cur
  bool double_buffer = false;
  float* vel = nullptr;
  float* acc = nullptr;        // running sum: PUSH_ACCUMULATE, or folding more than kMaxFused gradients
  double* partials = nullptr;  // kNumNorms doubles per workgroup of the apply launch
  uint32_t partials_blocks = 0;

  // launch shape
  uint32_t block = kDefaultBlock, unroll = kDefaultUnroll, vec = kDefaultVec, grid_cap = 0, waves_per_cu = 0;
  bool alternate = true;
  uint32_t n_cus = 256;             // compute units of the device (the phase-aligned kernel launches as many waves as are resident at once)
  uint64_t n_phased_launches = 0;

  // protocol state
  uint64_t ts_cur = 0;
  uint32_t count = 0;
  uint64_t sigma_sum_open = 0;
  std::vector<uint64_t> open_clock;  // clock_cap entries
  uint32_t clock_cap = 0;            // c + max_aggregate - 1
  bool open_weighted = false;        // some pending message has a weight other than 1
  std::vector<Pending> open_grads;
  std::vector<uint8_t> seen;

  // closed clocks (ring over update index)
  uint32_t ring = kDefaultClockRing;
  std::vector<uint64_t> ring_ts;
  std::vector<uint32_t> ring_count;
  std::vector<double> ring_avg;
  std::vector<float> ring_lr;

  // statistics
  std::vector<uint64_t> hist;
  uint64_t n_pushes = 0, n_updates = 0, n_rejected = 0, sigma_sum = 0, sigma_max = 0;
  uint64_t n_weight_copies = 0, n_ts_inquiries = 0, n_weight_views = 0;
  double last_avg = 0.0;
  float last_lr = 0.f;
  uint32_t last_apply_blocks = 0;
  uint64_t n_apply_launches = 0;  // decides the direction of the next launch's walk over the vector
  uint64_t n_batched_launches = 0, n_batched_updates = 0;

  // rudra_ps_push_batch: updates that have fired but are not enqueued yet (flushed before the call returns)
  bool deferring = false;
  std::vector<Pending> deferred_grads;
  std::vector<DeferredUpdate> deferred;

  // readers of a weight buffer on other streams (rudra_ps_weights_acquire / _release)
  std::vector<hipEvent_t> free_events;         // created on demand, reused
  std::vector<hipEvent_t> reader_done[2];      // per weight buffer: reads the next launch that writes it must wait for
  size_t n_reader_events = 0;                  // events in existence (in one of the three lists, or in a caller's hand)
  uint64_t n_weight_acquires = 0, n_reader_waits = 0;

  // kernel timing
  std::vector<hipEvent_t> ev_start, ev_stop;
  uint64_t timed_launches = 0, timed_resolved = 0;
  double kernel_ms = 0.0;
};

namespace {

int hip_fail(rudra_ps* ps, hipError_t e) {
  ps->last_hip_error = (int)e;
  ps->failed = true;
  return RUDRA_EHIP;
}

#define RUDRA_HIP(ps, call)                       \
  do {                                            \
    hipError_t e_ = (call);                       \
    if (e_ != hipSuccess) return hip_fail(ps, e_); \
  } while (0)

int kernel_optimizer(const rudra_ps_config_t& cfg) {
  if (cfg.optimizer == RUDRA_OPT_ADAGRAD) return rudra::kOptAdagrad;
  return cfg.momentum != 0.0f ? rudra::kOptMomentum : rudra::kOptSgd;
}

uint32_t gradients_per_update(const rudra_ps_config_t& cfg) {
  if (cfg.c_override) return cfg.c_override;
  if (cfg.protocol == RUDRA_HARDSYNC) return cfg.n_learners;
  return cfg.n_learners / cfg.n_split;
}

struct LaunchShape {
  uint32_t grid, block;
  uint64_t ntiles;
  uint32_t lds_bytes;  // unused dynamic LDS reserved per workgroup: the occupancy cap
};

constexpr uint32_t kLdsPerCu = 160u * 1024u;  // gfx950
constexpr uint32_t kMaxDynamicLds = 64u * 1024u;

// LDS to reserve per workgroup so that at most `waves_per_cu` wavefronts are resident on a CU.
uint32_t lds_for_occupancy(uint32_t waves_per_cu, uint32_t block) {
  if (waves_per_cu == 0 || waves_per_cu >= 32) return 0;
  const uint32_t waves_per_wg = block / 64;
  uint32_t wgs = waves_per_cu / waves_per_wg;
  if (wgs == 0) wgs = 1;
  uint32_t bytes = (kLdsPerCu / wgs) & ~1023u;  // at most `wgs` such workgroups fit
  return bytes > kMaxDynamicLds ? kMaxDynamicLds : bytes;
}

// Workgroups for `tiles` tiles: one per tile, at least one (the scalar tail needs workgroup 0), at most `cap` when
// the caller set one, and never so many that grid * block reaches 2^32 (HIP rejects such a launch); the kernels walk
// the remaining tiles with a grid-stride loop.
uint32_t grid_for(uint64_t tiles, uint32_t block, uint32_t cap) {
  uint64_t grid = tiles ? tiles : 1;
  if (cap && grid > cap) grid = cap;
  const uint64_t most = 0xFFFFFFFFull / block;
  if (grid > most) grid = most;
  return (uint32_t)grid;
}

// Gradient loads a wave issues per round when the caller names no unroll.  Up to kDefaultUnroll gradients: all at once.
// More: one at a time (see default_waves_per_cu), except on short vectors.  A vector of fewer wavefront tiles than the
// chip holds resident wavefronts (32 per CU) is a single generation of waves: nothing queues behind them, the launch
// lasts about c / U memory round trips, and deeper rounds pay.  Measured in one process, c = 7 / 15 / 30, microseconds
// per update: 131k parameters 4.9 / 8.1 / 14.1 at U = 1 -> 3.7 / 4.6 / 6.6 at U = 8; 400k: 6.5 / 10.4 / 17.6 -> 5.6 / 7.7 /
// 11.5 at U = 4; 1.0M: 10.0 / 15.8 / 25.1 -> 10.4 / 14.9 / 23.1 at U = 2 (hence not for c <= 8); from 1.25M on U = 1 wins.
uint32_t default_unroll(uint32_t c, uint64_t n_params, uint32_t n_cus, uint32_t vec) {
  if (c <= kDefaultUnroll) return kDefaultUnroll;
  const uint64_t waves = ((n_params >> 2) + 63) / 64;
  const uint64_t resident = (uint64_t)n_cus * 32u;
  uint32_t u = 1;
  while (u < 8 && waves * (2u * u) <= resident) u *= 2;
  if (u == 2 && c <= 8) u = 1;
  while (u > 1 && u * vec > 8) u /= 2;
  return u;
}

// Resident wavefronts per CU for the single-update kernel when the caller names none.
// Measured at 72M parameters (GB/s of algorithmic bytes, medians): what counts is how many loads are in flight per
// CU, about kInFlightKiBPerCu KiB at 1 KiB per wave-load, and, at equal volume, that few tiles are open at once.
//   c <= unroll (4): a wave issues theta, the second state vector and all its gradients in one round; 48/(loads per
//           wave) resident waves, at least 16 (with the velocity loaded non-temporally, 8 / 10 / 12 / 16 / 20 waves:
//           c = 2 6.36 / 6.44 / 6.80 / 7.22 / 7.15 TB/s, c = 3 6.45 / 6.70 / 7.05 / 7.14 / 7.12, c = 4 6.21 / 6.54 / 6.96 /
//           7.16 / 7.15; c = 1: 12 / 16 / 20 / 26 waves 6.69 / 7.16 / 7.16 / 7.06).
//   c > 4 with the default unroll of 1: after the first round a wave has one gradient load outstanding, and 26
//           resident waves are best (c = 7: 6.78, c = 18: 6.41, c = 30: 6.13, c = 54: 6.22; 20 or 32 waves lose
//           2-4 %; 4 loads at a time with 8 waves is 1-2 % behind); small vectors run uncapped (kSmallVector).
//   an explicit unroll > 1 with c above it: 48/(unroll + state vectors) waves.
uint32_t default_waves_per_cu(uint32_t c, uint32_t unroll, int optimizer, uint64_t n_params, uint32_t block) {
  const uint32_t per_wave = std::min(c, unroll) + 1u + (optimizer != rudra::kOptSgd ? 1u : 0u);
  const uint32_t waves_per_wg = block / 64;
  uint32_t w = (kInFlightKiBPerCu + per_wave / 2) / per_wave;
  if (c <= unroll) w = std::max(w, 16u);
  else if (n_params < kSmallVector) w = 32;
  else if (unroll == 1) w = 26;
  w = std::max(w, std::max(4u, waves_per_wg));
  return std::min(w, 32u);
}

void choose_unroll_and_waves(rudra_ps* ps) {
  const rudra_ps_config_t& cfg = ps->cfg;
  ps->unroll = cfg.launch_unroll ? cfg.launch_unroll : default_unroll(ps->c, cfg.n_params, ps->n_cus, ps->vec);
  ps->waves_per_cu = cfg.launch_waves_per_cu ? cfg.launch_waves_per_cu
                                             : default_waves_per_cu(ps->c, ps->unroll, kernel_optimizer(cfg), cfg.n_params, ps->block);
}

LaunchShape shape_for(const rudra_ps* ps) {
  const uint64_t n4 = ps->cfg.n_params >> 2;
  const uint64_t tile = (uint64_t)ps->block * ps->vec;
  const uint64_t tiles = (n4 + tile - 1) / tile;
  return {grid_for(tiles, ps->block, ps->grid_cap), ps->block, tiles, lds_for_occupancy(ps->waves_per_cu, ps->block)};
}

// ---- kernel dispatch: runtime (optimizer, decay, weighted, stats, unroll, vec) -> template instance ----
template <int OPT, bool WD, bool W, bool ST, int U>
void launch_apply_v(int ntld, uint32_t vec, LaunchShape s, hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  // the state-load policies other than "both cached" exist for the default shapes only (one float4 per lane, 1 or 4 loads at a time)
  if (vec == 1 && (U == 1 || U == 4) && ntld != rudra::kStateLoadsCached) {
    if (ntld == rudra::kStateLoadsVelNt && OPT != rudra::kOptSgd) {
      hipLaunchKernelGGL((rudra::apply_update_kernel<OPT, WD, W, ST, (U == 1 || U == 4) ? U : 1, 1, rudra::kStateLoadsVelNt>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
      return;
    }
    if (ntld == rudra::kStateLoadsThetaNt) {
      hipLaunchKernelGGL((rudra::apply_update_kernel<OPT, WD, W, ST, (U == 1 || U == 4) ? U : 1, 1, rudra::kStateLoadsThetaNt>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
      return;
    }
  }
  switch (vec) {
    case 1: hipLaunchKernelGGL((rudra::apply_update_kernel<OPT, WD, W, ST, U, 1>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a); break;
    case 2: hipLaunchKernelGGL((rudra::apply_update_kernel<OPT, WD, W, ST, U, 2>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a); break;
    default: hipLaunchKernelGGL((rudra::apply_update_kernel<OPT, WD, W, ST, U, 4>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a); break;
  }
}
template <int OPT, bool WD, bool W, bool ST>
void launch_apply_u(int ntld, uint32_t unroll, uint32_t vec, LaunchShape s, hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  switch (unroll) {
    case 1: launch_apply_v<OPT, WD, W, ST, 1>(ntld, vec, s, st, gs, a); break;
    case 2: launch_apply_v<OPT, WD, W, ST, 2>(ntld, vec, s, st, gs, a); break;
    case 4: launch_apply_v<OPT, WD, W, ST, 4>(ntld, vec, s, st, gs, a); break;
    default: launch_apply_v<OPT, WD, W, ST, 8>(ntld, vec, s, st, gs, a); break;
  }
}
template <int OPT, bool WD>
void launch_apply_ws(bool weighted, bool stats, int ntld, uint32_t unroll, uint32_t vec, LaunchShape s, hipStream_t st,
                     const GradSet& gs, const UpdateArgs& a) {
  if (weighted) {
    if (stats) launch_apply_u<OPT, WD, true, true>(ntld, unroll, vec, s, st, gs, a);
    else launch_apply_u<OPT, WD, true, false>(ntld, unroll, vec, s, st, gs, a);
  } else {
    if (stats) launch_apply_u<OPT, WD, false, true>(ntld, unroll, vec, s, st, gs, a);
    else launch_apply_u<OPT, WD, false, false>(ntld, unroll, vec, s, st, gs, a);
  }
}
template <int OPT>
void launch_apply_d(bool decay, bool weighted, bool stats, int ntld, uint32_t unroll, uint32_t vec, LaunchShape s, hipStream_t st,
                    const GradSet& gs, const UpdateArgs& a) {
  if (decay) launch_apply_ws<OPT, true>(weighted, stats, ntld, unroll, vec, s, st, gs, a);
  else launch_apply_ws<OPT, false>(weighted, stats, ntld, unroll, vec, s, st, gs, a);
}
// ntld: which state vector is loaded non-temporally (rudra::kStateLoads...)
void launch_apply(int opt, bool decay, bool weighted, bool stats, int ntld, uint32_t unroll, uint32_t vec, LaunchShape s,
                  hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  switch (opt) {
    case rudra::kOptMomentum: launch_apply_d<rudra::kOptMomentum>(decay, weighted, stats, ntld, unroll, vec, s, st, gs, a); break;
    case rudra::kOptAdagrad: launch_apply_d<rudra::kOptAdagrad>(decay, weighted, stats, ntld, unroll, vec, s, st, gs, a); break;
    default: launch_apply_d<rudra::kOptSgd>(decay, weighted, stats, ntld, unroll, vec, s, st, gs, a); break;
  }
}

// Which state vector the update kernels load non-temporally (the caller's launch_state_loads wins).  Measured at 72M
// parameters with momentum or AdaGrad, all variants in one process on the same buffers, two machines (fraction of 8 TB/s,
// neither / velocity / weights non-temporal):
//   two weight buffers: the weights, always (the buffer read is dead once the update has run): c = 1 0.86 / 0.77-0.80 /
//     0.89, c = 18 0.80 / 0.78 / 0.82: the double buffer then costs nothing against updating in place.
//   in place, one update per launch: c = 1 0.887 / 0.905 / 0.903; c = 3 ... 14 +1.5 to +3.5 % for either (c = 5: 0.854 /
//     0.887 / 0.886; c = 12: 0.826 / 0.839 / 0.839); c = 2 looked like an exception at 12 resident waves (0.875 / 0.850)
//     but not at the 16 it runs with now (0.891 / 0.902); c >= 16 within 1 % either way (c = 18: 0.812 / 0.816 / 0.817;
//     c = 30: 0.78 / 0.76-0.78 / 0.78).  The velocity is taken, up to 14 gradients.
//   plain SGD (no second state vector): ordinary loads (c = 1: 0.881 vs 0.864; c = 18: 0.821 vs 0.809).
//   several updates per launch: up to about 40 gradients per launch the weights non-temporal is +1 to +6 % (varies
//     with the machine, never below -1 %), beyond that ordinary loads are equal or 1 % better.
int state_load_policy(const rudra_ps* ps, uint32_t n_grads) {
  if (ps->cfg.launch_state_loads) return (int)ps->cfg.launch_state_loads - 1;
  if (ps->double_buffer) return rudra::kStateLoadsThetaNt;
  if (kernel_optimizer(ps->cfg) == rudra::kOptSgd) return rudra::kStateLoadsCached;
  if (n_grads <= 14) return rudra::kStateLoadsVelNt;
  return rudra::kStateLoadsCached;
}
int batch_state_load_policy(const rudra_ps* ps, uint32_t n_grads) {
  if (ps->cfg.launch_state_loads) return (int)ps->cfg.launch_state_loads - 1;
  if (ps->double_buffer) return rudra::kStateLoadsThetaNt;
  if (kernel_optimizer(ps->cfg) == rudra::kOptSgd) return rudra::kStateLoadsCached;
  return n_grads <= 40 ? rudra::kStateLoadsThetaNt : rudra::kStateLoadsCached;
}

void launch_sum(bool weighted, LaunchShape s, uint32_t vec, hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  // the fold/accumulate path is not the measured one: a single shape (4 loads in flight)
  if (weighted) {
    if (vec == 1) hipLaunchKernelGGL((rudra::sum_gradients_kernel<true, false, 4, 1>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
    else if (vec == 2) hipLaunchKernelGGL((rudra::sum_gradients_kernel<true, false, 4, 2>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
    else hipLaunchKernelGGL((rudra::sum_gradients_kernel<true, false, 4, 4>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
  } else {
    if (vec == 1) hipLaunchKernelGGL((rudra::sum_gradients_kernel<false, false, 4, 1>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
    else if (vec == 2) hipLaunchKernelGGL((rudra::sum_gradients_kernel<false, false, 4, 2>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
    else hipLaunchKernelGGL((rudra::sum_gradients_kernel<false, false, 4, 4>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, a);
  }
}

UpdateArgs base_args(const rudra_ps* ps) {
  UpdateArgs a;
  std::memset(&a, 0, sizeof(a));
  a.theta = ps->theta2[ps->cur];
  a.theta_out = ps->theta2[ps->double_buffer ? (ps->cur ^ 1u) : ps->cur];  // = write_buffer(ps)
  a.vel = ps->vel;
  a.sum_out = ps->acc;
  a.partials = ps->partials;
  a.n_params = ps->cfg.n_params;
  a.momentum = ps->cfg.momentum;
  a.weight_decay = ps->cfg.weight_decay;
  a.adagrad_eps = ps->cfg.adagrad_eps;
  return a;
}

// The accumulator is allocated by rudra_ps_create whenever an update can hold more than kMaxFused messages, so
// that no push ever allocates.
int ensure_acc(rudra_ps* ps) { return ps->acc ? RUDRA_OK : RUDRA_ESTATE; }

// acc <- sum of `n` entries of `g` (which may start with acc itself), arrival order kept.
int enqueue_sum(rudra_ps* ps, const Pending* g, uint32_t n, bool weighted) {
  GradSet gs;
  std::memset(&gs, 0, sizeof(gs));
  for (uint32_t j = 0; j < n; ++j) { gs.p[j] = g[j].ptr; gs.w[j] = g[j].weight; }
  UpdateArgs a = base_args(ps);
  a.c = n;
  const LaunchShape s = shape_for(ps);
  a.ntiles = s.ntiles;
  launch_sum(weighted, s, ps->vec, ps->stream, gs, a);
  RUDRA_HIP(ps, hipGetLastError());
  return RUDRA_OK;
}

int resolve_timer(rudra_ps* ps, uint64_t launch_idx) {
  const uint32_t slot = (uint32_t)(launch_idx % kTimerRing);
  RUDRA_HIP(ps, hipEventSynchronize(ps->ev_stop[slot]));
  float ms = 0.f;
  RUDRA_HIP(ps, hipEventElapsedTime(&ms, ps->ev_start[slot], ps->ev_stop[slot]));
  ps->kernel_ms += (double)ms;
  ps->timed_resolved = launch_idx + 1;
  return RUDRA_OK;
}

// HIP events around one applyUpdate launch (TIME_KERNELS): begin_timed before the launch, end_timed after it.
int begin_timed(rudra_ps* ps, uint32_t* slot) {
  *slot = 0;
  if (!ps->time_kernels) return RUDRA_OK;
  if (ps->timed_launches - ps->timed_resolved >= kTimerRing) {
    int rc = resolve_timer(ps, ps->timed_resolved);
    if (rc != RUDRA_OK) return rc;
  }
  *slot = (uint32_t)(ps->timed_launches % kTimerRing);
  RUDRA_HIP(ps, hipEventRecord(ps->ev_start[*slot], ps->stream));
  return RUDRA_OK;
}
int end_timed(rudra_ps* ps, uint32_t slot) {
  if (!ps->time_kernels) return RUDRA_OK;
  RUDRA_HIP(ps, hipEventRecord(ps->ev_stop[slot], ps->stream));
  ps->timed_launches += 1;
  return RUDRA_OK;
}

// An event for ordering against a reader's stream: from the free list, or a new one (no timing data kept).
int take_event(rudra_ps* ps, hipEvent_t* ev) {
  if (!ps->free_events.empty()) {
    *ev = ps->free_events.back();
    ps->free_events.pop_back();
    return RUDRA_OK;
  }
  // Room for every event that exists is reserved in all three lists before the event is made, so that handing an
  // event from one list to another never allocates (and so never throws).
  try {
    const size_t n = ps->n_reader_events + 1;
    ps->free_events.reserve(n);
    ps->reader_done[0].reserve(n);
    ps->reader_done[1].reserve(n);
  } catch (const std::exception&) {
    return RUDRA_ENOMEM;
  }
  RUDRA_HIP(ps, hipEventCreateWithFlags(ev, hipEventDisableTiming));
  ps->n_reader_events += 1;
  return RUDRA_OK;
}

// The launch about to be enqueued writes weight buffer `buf`: it must not start before the reads that
// rudra_ps_weights_release has announced for that buffer are done.  The wait is on the device (the server's stream
// waits for the readers' events); the host does not block.
int wait_for_readers(rudra_ps* ps, uint32_t buf) {
  std::vector<hipEvent_t>& done = ps->reader_done[buf];
  for (hipEvent_t ev : done) {
    RUDRA_HIP(ps, hipStreamWaitEvent(ps->stream, ev, 0));
    ps->n_reader_waits += 1;
  }
  // an event may be recorded again once the wait on it has been enqueued: the wait refers to the record before it
  ps->free_events.insert(ps->free_events.end(), done.begin(), done.end());
  done.clear();
  return RUDRA_OK;
}

uint32_t write_buffer(const rudra_ps* ps) { return ps->double_buffer ? (ps->cur ^ 1u) : ps->cur; }

// Bookkeeping common to every applyUpdate launch: walk direction, double-buffer pointer swap.
void after_apply_launch(rudra_ps* ps, uint32_t grid) {
  ps->last_apply_blocks = grid;
  ps->n_apply_launches += 1;
  if (ps->double_buffer) ps->cur ^= 1u;  // the pointer swap: the buffer just written now holds the current weights
}

// ---- phase-aligned launch for updates of many gradients (apply_update_phased_kernel) ----
struct PhasedPlan {
  uint32_t n_waves, n_passes;
  uint64_t body_params;  // parameters the phased launch covers: n_waves * kPhasedTiles * n_passes tiles of 256
};

// The largest prefix of the vector that is a whole number of passes of n_waves * T tiles, with n_waves at most what is
// resident at once; {0, 0, 0} when the vector has fewer than T tiles.
PhasedPlan phased_plan(uint64_t n_params, uint32_t n_cus) {
  const uint64_t tiles = n_params / 256;  // whole tiles of 64 float4
  const uint64_t T = (uint64_t)rudra::kPhasedTiles;
  const uint64_t cap = (uint64_t)n_cus * 4u * (uint64_t)rudra::kPhasedWavesPerSimd;
  if (tiles < T) return {0, 0, 0};
  const uint64_t passes = (tiles + cap * T - 1) / (cap * T);
  const uint64_t waves = tiles / (T * passes);  // <= cap
  if (waves == 0 || passes > 0xFFFFFFFFull) return {0, 0, 0};
  return {(uint32_t)waves, (uint32_t)passes, waves * T * passes * 256};
}

template <int OPT>
void launch_phased_o(bool decay, bool weighted, const PhasedPlan& pl, hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  const dim3 g(pl.n_waves), b(64);
  if (decay) {
    if (weighted) hipLaunchKernelGGL((rudra::apply_update_phased_kernel<OPT, true, true>), g, b, 0, st, gs, a, pl.n_passes);
    else hipLaunchKernelGGL((rudra::apply_update_phased_kernel<OPT, true, false>), g, b, 0, st, gs, a, pl.n_passes);
  } else {
    if (weighted) hipLaunchKernelGGL((rudra::apply_update_phased_kernel<OPT, false, true>), g, b, 0, st, gs, a, pl.n_passes);
    else hipLaunchKernelGGL((rudra::apply_update_phased_kernel<OPT, false, false>), g, b, 0, st, gs, a, pl.n_passes);
  }
}
void launch_phased(int opt, bool decay, bool weighted, const PhasedPlan& pl, hipStream_t st, const GradSet& gs, const UpdateArgs& a) {
  switch (opt) {
    case rudra::kOptMomentum: launch_phased_o<rudra::kOptMomentum>(decay, weighted, pl, st, gs, a); break;
    case rudra::kOptAdagrad: launch_phased_o<rudra::kOptAdagrad>(decay, weighted, pl, st, gs, a); break;
    default: launch_phased_o<rudra::kOptSgd>(decay, weighted, pl, st, gs, a); break;
  }
}

// Whether this update goes through the phase-aligned kernel: only on the caller's request (launch_phased = 2; it is not
// a robust win, see the kernel's header) and never with fused norms (it has no reduction epilogue).
bool use_phased(const rudra_ps* ps) { return ps->cfg.launch_phased == 2 && !ps->want_norms; }

// sumGradients + applyUpdate for the `n` pending messages in `g` standing for `count` learner gradients (Eq. 3 /
// Eq. 5), one fused launch when n <= kMaxFused.
int enqueue_update(rudra_ps* ps, const Pending* g, size_t n_msgs, uint32_t count, float lr, bool weighted) {
  size_t first = 0;
  Pending head = {nullptr, 1.0f};
  bool have_head = false;
  // fold leading groups into acc until what is left fits one launch
  while ((n_msgs - first) + (have_head ? 1 : 0) > (size_t)kMaxFused) {
    int rc = ensure_acc(ps);
    if (rc != RUDRA_OK) return rc;
    Pending group[kMaxFused];
    uint32_t n = 0;
    if (have_head) group[n++] = head;
    while (n < (uint32_t)kMaxFused) group[n++] = g[first++];
    rc = enqueue_sum(ps, group, n, weighted);
    if (rc != RUDRA_OK) return rc;
    head = {ps->acc, 1.0f};
    have_head = true;
  }
  GradSet gs;
  std::memset(&gs, 0, sizeof(gs));
  uint32_t n = 0;
  if (have_head) { gs.p[n] = head.ptr; gs.w[n] = head.weight; ++n; }
  for (; first < n_msgs; ++first, ++n) { gs.p[n] = g[first].ptr; gs.w[n] = g[first].weight; }

  UpdateArgs a = base_args(ps);
  a.c = n;
  a.inv_c = 1.0f / (float)count;  // Eq. 5: the mean is over all gradients of the update (c of them, unless a
                                  // relayed average made the count overshoot)
  a.lr = lr;
  a.reverse = (ps->alternate && (ps->n_apply_launches & 1)) ? 1u : 0u;
  const LaunchShape s = shape_for(ps);
  a.ntiles = s.ntiles;
  uint32_t slot = 0;
  int rc = wait_for_readers(ps, write_buffer(ps));
  if (rc != RUDRA_OK) return rc;
  rc = begin_timed(ps, &slot);
  if (rc != RUDRA_OK) return rc;
  PhasedPlan pl = {0, 0, 0};
  if (use_phased(ps)) pl = phased_plan(ps->cfg.n_params, ps->n_cus);
  if (pl.body_params) {
    // the phase-aligned kernel on the prefix it tiles exactly, the ordinary kernel on what is left (same arithmetic)
    launch_phased(kernel_optimizer(ps->cfg), ps->cfg.weight_decay != 0.0f, weighted, pl, ps->stream, gs, a);
    RUDRA_HIP(ps, hipGetLastError());
    ps->n_phased_launches += 1;
    const uint64_t rest = ps->cfg.n_params - pl.body_params;
    if (rest) {
      GradSet gr = gs;
      for (uint32_t j = 0; j < n; ++j) gr.p[j] = gs.p[j] + pl.body_params;
      UpdateArgs ar = a;
      ar.theta = a.theta + pl.body_params;
      ar.theta_out = a.theta_out + pl.body_params;
      if (a.vel) ar.vel = a.vel + pl.body_params;
      ar.n_params = rest;
      const uint64_t tile = (uint64_t)ps->block * ps->vec;
      ar.ntiles = ((rest >> 2) + tile - 1) / tile;
      const LaunchShape sr = {grid_for(ar.ntiles, ps->block, ps->grid_cap), ps->block, ar.ntiles, 0};
      launch_apply(kernel_optimizer(ps->cfg), ps->cfg.weight_decay != 0.0f, weighted, false, rudra::kStateLoadsCached, ps->unroll, ps->vec, sr, ps->stream, gr, ar);
    }
  } else {
    launch_apply(kernel_optimizer(ps->cfg), ps->cfg.weight_decay != 0.0f, weighted, ps->want_norms, state_load_policy(ps, n), ps->unroll, ps->vec, s, ps->stream, gs, a);
  }
  RUDRA_HIP(ps, hipGetLastError());
  rc = end_timed(ps, slot);
  if (rc != RUDRA_OK) return rc;
  after_apply_launch(ps, s.grid);
  return RUDRA_OK;
}

// ---- batched launches: several consecutive updates applied in registers (rudra_ps_push_batch) ----
template <int OPT, bool WD, bool W, bool ST>
void launch_batch_d(int ntld, uint32_t rounds, LaunchShape s, hipStream_t st, const GradSet& gs, const BatchPlan& plan, const UpdateArgs& a) {
  if (rounds == 8)  // short vectors are cache-resident: no state-load policy there
    hipLaunchKernelGGL((rudra::apply_update_batch_kernel<OPT, WD, W, ST, rudra::kStateLoadsCached, 8>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, plan, a);
  else if (rounds == 4)
    hipLaunchKernelGGL((rudra::apply_update_batch_kernel<OPT, WD, W, ST, rudra::kStateLoadsCached, 4>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, plan, a);
  else if (ntld == rudra::kStateLoadsThetaNt)
    hipLaunchKernelGGL((rudra::apply_update_batch_kernel<OPT, WD, W, ST, rudra::kStateLoadsThetaNt>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, plan, a);
  else if (ntld == rudra::kStateLoadsVelNt && OPT != rudra::kOptSgd)
    hipLaunchKernelGGL((rudra::apply_update_batch_kernel<OPT, WD, W, ST, rudra::kStateLoadsVelNt>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, plan, a);
  else
    hipLaunchKernelGGL((rudra::apply_update_batch_kernel<OPT, WD, W, ST>), dim3(s.grid), dim3(s.block), s.lds_bytes, st, gs, plan, a);
}
template <int OPT, bool WD>
void launch_batch_ws(bool weighted, bool stats, int ntld, uint32_t rounds, LaunchShape s, hipStream_t st, const GradSet& gs,
                     const BatchPlan& plan, const UpdateArgs& a) {
  if (weighted) {
    if (stats) launch_batch_d<OPT, WD, true, true>(ntld, rounds, s, st, gs, plan, a);
    else launch_batch_d<OPT, WD, true, false>(ntld, rounds, s, st, gs, plan, a);
  } else {
    if (stats) launch_batch_d<OPT, WD, false, true>(ntld, rounds, s, st, gs, plan, a);
    else launch_batch_d<OPT, WD, false, false>(ntld, rounds, s, st, gs, plan, a);
  }
}
void launch_batch(int opt, bool decay, bool weighted, bool stats, int ntld, uint32_t rounds, LaunchShape s, hipStream_t st,
                  const GradSet& gs, const BatchPlan& plan, const UpdateArgs& a) {
  switch (opt) {
    case rudra::kOptMomentum:
      if (decay) launch_batch_ws<rudra::kOptMomentum, true>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      else launch_batch_ws<rudra::kOptMomentum, false>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      break;
    case rudra::kOptAdagrad:
      if (decay) launch_batch_ws<rudra::kOptAdagrad, true>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      else launch_batch_ws<rudra::kOptAdagrad, false>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      break;
    default:
      if (decay) launch_batch_ws<rudra::kOptSgd, true>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      else launch_batch_ws<rudra::kOptSgd, false>(weighted, stats, ntld, rounds, s, st, gs, plan, a);
      break;
  }
}

// Gradient loads per round in a batched launch: 1 = the rolling scheme (gradient j consumed while j + 1 is in flight), which
// is what long vectors want; short vectors (see default_unroll) take 8 or 4 at a time.  An explicit launch_unroll of 4
// or 8 selects that; 1 or 2 the rolling scheme.
uint32_t batch_rounds(const rudra_ps* ps) {
  if (ps->cfg.launch_unroll) return ps->cfg.launch_unroll >= 4 ? ps->cfg.launch_unroll : 1u;
  const uint64_t waves = ((ps->cfg.n_params >> 2) + 63) / 64;
  const uint64_t resident = (uint64_t)ps->n_cus * 32u;
  return waves * 8u <= resident ? 8u : waves * 4u <= resident ? 4u : 1u;
}

// Launch shape of a batched launch: one float4 per lane per tile whatever launch_vec says (theta and v stay in
// registers across the updates of the plan).
LaunchShape batch_shape_for(const rudra_ps* ps) {
  const uint64_t npos = ps->cfg.n_params >> 2;
  const uint64_t tiles = (npos + ps->block - 1) / ps->block;
  const uint32_t waves = ps->cfg.launch_waves_per_cu ? ps->cfg.launch_waves_per_cu : std::max(kBatchWavesPerCu, ps->block / 64);
  return {grid_for(tiles, ps->block, ps->grid_cap), ps->block, tiles, lds_for_occupancy(waves, ps->block)};
}

// Enqueue the updates `d[0..n_upd)` (consuming consecutive entries of `g`) as ONE batched launch.  Caller guarantees
// 2 <= n_upd <= kMaxBatchUpdates and at most kMaxFused messages in total.
int enqueue_batch(rudra_ps* ps, const Pending* g, const DeferredUpdate* d, uint32_t n_upd) {
  GradSet gs;
  BatchPlan plan;
  std::memset(&gs, 0, sizeof(gs));
  std::memset(&plan, 0, sizeof(plan));
  uint32_t n = 0;
  bool weighted = false;
  plan.n_updates = n_upd;
  for (uint32_t u = 0; u < n_upd; ++u) {
    plan.e[u].count = d[u].n_grads;
    plan.e[u].lr = d[u].lr;
    plan.e[u].inv_c = 1.0f / (float)d[u].count;
    weighted = weighted || d[u].weighted;
    for (uint32_t j = 0; j < d[u].n_grads; ++j, ++n) { gs.p[n] = g[n].ptr; gs.w[n] = g[n].weight; }
  }
  UpdateArgs a = base_args(ps);
  a.c = n;
  a.reverse = (ps->alternate && (ps->n_apply_launches & 1)) ? 1u : 0u;
  const LaunchShape s = batch_shape_for(ps);
  a.ntiles = s.ntiles;
  uint32_t slot = 0;
  int rc = wait_for_readers(ps, write_buffer(ps));
  if (rc != RUDRA_OK) return rc;
  rc = begin_timed(ps, &slot);
  if (rc != RUDRA_OK) return rc;
  launch_batch(kernel_optimizer(ps->cfg), ps->cfg.weight_decay != 0.0f, weighted, ps->want_norms, batch_state_load_policy(ps, n), batch_rounds(ps), s, ps->stream, gs, plan, a);
  RUDRA_HIP(ps, hipGetLastError());
  rc = end_timed(ps, slot);
  if (rc != RUDRA_OK) return rc;
  after_apply_launch(ps, s.grid);
  ps->n_batched_launches += 1;
  ps->n_batched_updates += n_upd;
  return RUDRA_OK;
}

// Enqueue everything rudra_ps_push_batch has deferred: runs of consecutive updates that fit one launch go out as
// one batched launch, a lone update (or one too large to batch) through the single-update path.
int flush_deferred(rudra_ps* ps) {
  const std::vector<DeferredUpdate>& d = ps->deferred;
  const Pending* g = ps->deferred_grads.data();
  size_t i = 0, g0 = 0;
  int rc = RUDRA_OK;
  while (i < d.size() && rc == RUDRA_OK) {
    size_t k = i, msgs = 0;
    while (k < d.size() && k - i < (size_t)kMaxBatchUpdates && d[k].n_grads <= (uint32_t)kMaxFused &&
           msgs + d[k].n_grads <= (size_t)kMaxFused) {
      msgs += d[k].n_grads;
      ++k;
    }
    if (k - i >= 2) {
      rc = enqueue_batch(ps, g + g0, &d[i], (uint32_t)(k - i));
      g0 += msgs;
      i = k;
    } else {
      rc = enqueue_update(ps, g + g0, d[i].n_grads, d[i].count, d[i].lr, d[i].weighted);
      g0 += d[i].n_grads;
      i += 1;
    }
  }
  ps->deferred.clear();
  ps->deferred_grads.clear();
  return rc;
}

// true if [p, p + bytes) is device memory of `device` according to the HIP runtime
bool is_device_range(const void* p, size_t bytes, int device) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();  // the query of a non-HIP pointer leaves an error behind: clear it
    return false;
  }
  if (attr.type != hipMemoryTypeDevice || attr.device != device) return false;
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  const char* lo = static_cast<const char*>(base);
  const char* q = static_cast<const char*>(p);
  return q >= lo && bytes <= size && (size_t)(q - lo) <= size - bytes;
}

void count_staleness(rudra_ps* ps, uint64_t sigma) {  // the caller has made the histogram long enough
  ps->hist[sigma] += 1;
  ps->sigma_sum += sigma;
  ps->sigma_max = std::max(ps->sigma_max, sigma);
}

int validate_config(const rudra_ps_config_t* c) {
  if (c->n_params == 0 || c->n_learners == 0) return RUDRA_EINVAL;
  if (c->protocol != RUDRA_HARDSYNC && c->protocol != RUDRA_SOFTSYNC) return RUDRA_EINVAL;
  if (c->lr_mode < RUDRA_LR_CONST || c->lr_mode > RUDRA_LR_PER_GRADIENT) return RUDRA_EINVAL;
  if (c->protocol == RUDRA_SOFTSYNC && (c->n_split < 1 || c->n_split > c->n_learners)) return RUDRA_EINVAL;
  if (c->lr_mode == RUDRA_LR_STATIC_N && c->n_split < 1) return RUDRA_EINVAL;  // alpha0/n needs n >= 1 under hardsync too
  if (c->lr_scale == 0.0f) return RUDRA_EINVAL;  // a zeroed config would freeze the weights silently: 1 means "no factor"
  if (gradients_per_update(*c) == 0) return RUDRA_EINVAL;
  {
    // an update collects at most c + max_aggregate - 1 timestamps; the ring keeps that many per closed clock
    const uint64_t cap = (uint64_t)gradients_per_update(*c) + (c->max_aggregate > 1 ? c->max_aggregate - 1 : 0);
    const uint64_t ring = c->clock_ring ? c->clock_ring : kDefaultClockRing;
    if (cap > kMaxClockEntries || ring > kMaxRingEntries / cap) return RUDRA_EINVAL;
  }
  if (c->optimizer != RUDRA_OPT_SGD && c->optimizer != RUDRA_OPT_ADAGRAD) return RUDRA_EINVAL;
  if (c->optimizer == RUDRA_OPT_ADAGRAD && (c->momentum != 0.0f || !(c->adagrad_eps >= 0.0f))) return RUDRA_EINVAL;
  if (c->launch_block && (c->launch_block < 64 || c->launch_block > 1024 || c->launch_block % 64)) return RUDRA_EINVAL;
  if (c->launch_unroll && c->launch_unroll != 1 && c->launch_unroll != 2 && c->launch_unroll != 4 && c->launch_unroll != 8)
    return RUDRA_EINVAL;
  if (c->launch_vec && c->launch_vec != 1 && c->launch_vec != 2 && c->launch_vec != 4) return RUDRA_EINVAL;
  if (c->launch_alternate > 2 || c->launch_state_loads > 3 || c->launch_phased > 2) return RUDRA_EINVAL;
  if (c->max_aggregate > 1 && c->lr_mode == RUDRA_LR_PER_GRADIENT) return RUDRA_EINVAL;  // a relayed average cannot be re-weighted
  if (c->max_aggregate > 4096) return RUDRA_EINVAL;
  if (c->launch_waves_per_cu && (c->launch_waves_per_cu < 2 || c->launch_waves_per_cu > 32)) return RUDRA_EINVAL;
  if ((c->launch_unroll ? c->launch_unroll : kDefaultUnroll) * (c->launch_vec ? c->launch_vec : kDefaultVec) > 8)
    return RUDRA_EINVAL;  // more 16-byte loads per lane than the register file holds without spilling
  if (c->flags & ~(uint32_t)(RUDRA_FLAG_STATS_NORMS | RUDRA_FLAG_PUSH_ACCUMULATE | RUDRA_FLAG_CONTROL_ONLY | RUDRA_FLAG_TIME_KERNELS |
                              RUDRA_FLAG_DOUBLE_BUFFER | RUDRA_FLAG_CHECK_POINTERS))
    return RUDRA_EINVAL;
  if (!(c->alpha0 == c->alpha0) || !(c->lr_scale == c->lr_scale) || !(c->momentum == c->momentum) ||
      !(c->weight_decay == c->weight_decay))
    return RUDRA_EINVAL;  // NaN
  return RUDRA_OK;
}

void release(rudra_ps* ps) {
  if (!ps->control_only) {
    DeviceGuard guard(ps->cfg.device);
    (void)hipStreamSynchronize(ps->stream);
    for (hipEvent_t e : ps->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : ps->ev_stop) (void)hipEventDestroy(e);
    for (hipEvent_t e : ps->free_events) (void)hipEventDestroy(e);
    for (int b = 0; b < 2; ++b)
      for (hipEvent_t e : ps->reader_done[b]) (void)hipEventDestroy(e);
    if (ps->theta2[0]) (void)hipFree(ps->theta2[0]);
    if (ps->theta2[1]) (void)hipFree(ps->theta2[1]);
    if (ps->vel) (void)hipFree(ps->vel);
    if (ps->acc) (void)hipFree(ps->acc);
    if (ps->partials) (void)hipFree(ps->partials);
  }
  delete ps;
}

}  // namespace

extern "C" {

int rudra_ps_create(const rudra_ps_config_t* config, const float* init_weights, rudra_ps_t** out) {
  if (!config || !out) return RUDRA_EINVAL;
  *out = nullptr;
  int rc = validate_config(config);
  if (rc != RUDRA_OK) return rc;
  const bool control_only = (config->flags & RUDRA_FLAG_CONTROL_ONLY) != 0;
  if (!control_only && !init_weights) return RUDRA_EINVAL;
  if (!control_only && (reinterpret_cast<uintptr_t>(init_weights) & 3u)) return RUDRA_EINVAL;

  rudra_ps* ps = new (std::nothrow) rudra_ps();
  if (!ps) return RUDRA_ENOMEM;
  ps->cfg = *config;
  ps->control_only = control_only;
  ps->accumulate = (config->flags & RUDRA_FLAG_PUSH_ACCUMULATE) != 0;
  ps->want_norms = (config->flags & RUDRA_FLAG_STATS_NORMS) != 0 && !control_only;
  ps->time_kernels = (config->flags & RUDRA_FLAG_TIME_KERNELS) != 0 && !control_only;
  ps->double_buffer = (config->flags & RUDRA_FLAG_DOUBLE_BUFFER) != 0 && !control_only;
  ps->check_pointers = (config->flags & RUDRA_FLAG_CHECK_POINTERS) != 0 && !control_only;
  ps->stream = (hipStream_t)config->stream;
  ps->c = gradients_per_update(*config);
  if (config->launch_block) ps->block = config->launch_block;
  if (config->launch_vec) ps->vec = config->launch_vec;
  ps->grid_cap = config->launch_grid;
  ps->alternate = config->launch_alternate != 2;
  choose_unroll_and_waves(ps);  // with the default CU count; again below once the device has been asked
  ps->ring = config->clock_ring ? config->clock_ring : kDefaultClockRing;
  try {
    ps->clock_cap = ps->c + (config->max_aggregate > 1 ? config->max_aggregate - 1 : 0);  // bounded by validate_config
    ps->open_clock.assign(ps->clock_cap, 0);
    ps->open_grads.reserve(ps->clock_cap);  // a message stands for at least one gradient: never more than this many
    ps->seen.assign(config->n_learners, 0);
    ps->ring_ts.assign((size_t)ps->ring * ps->clock_cap, 0);
    ps->ring_count.assign(ps->ring, 0);
    ps->ring_avg.assign(ps->ring, 0.0);
    ps->ring_lr.assign(ps->ring, 0.f);
    ps->hist.reserve(64);
  } catch (const std::exception&) {  // bad_alloc, length_error
    delete ps;
    return RUDRA_ENOMEM;
  }
  if (!control_only) {
    const size_t bytes = config->n_params * sizeof(float);
    DeviceGuard guard(config->device);
    hipError_t e = guard.error();
    if (e == hipSuccess && !is_device_range(init_weights, bytes, config->device)) {
      delete ps;
      return RUDRA_EINVAL;  // not P floats of this device's memory
    }
    if (e == hipSuccess) {
      int cus = 0;
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, config->device) == hipSuccess && cus > 0) ps->n_cus = (uint32_t)cus;
      else (void)hipGetLastError();
      choose_unroll_and_waves(ps);
    }
    if (e == hipSuccess) e = hipMalloc((void**)&ps->theta2[0], bytes);
    if (e == hipSuccess && ps->double_buffer) e = hipMalloc((void**)&ps->theta2[1], bytes);
    // the second state vector (velocity, or AdaGrad's h) exists only when the rule has one; the accumulator only
    // when gradients are summed at arrival or an update can hold more messages than one launch takes
    const bool second_state = kernel_optimizer(*config) != rudra::kOptSgd;
    if (e == hipSuccess && second_state) e = hipMalloc((void**)&ps->vel, bytes);
    if (e == hipSuccess && (ps->accumulate || ps->clock_cap > (uint32_t)kMaxFused)) e = hipMalloc((void**)&ps->acc, bytes);
    if (e == hipSuccess) e = hipMemcpyAsync(ps->theta2[0], init_weights, bytes, hipMemcpyDeviceToDevice, ps->stream);
    if (e == hipSuccess && second_state) e = hipMemsetAsync(ps->vel, 0, bytes, ps->stream);
    if (e == hipSuccess && ps->want_norms) {
      ps->partials_blocks = std::max(shape_for(ps).grid, batch_shape_for(ps).grid);
      e = hipMalloc((void**)&ps->partials, (size_t)ps->partials_blocks * kNumNorms * sizeof(double));
    }
    if (e == hipSuccess && ps->time_kernels) {
      ps->ev_start.resize(kTimerRing);
      ps->ev_stop.resize(kTimerRing);
      for (uint32_t i = 0; i < kTimerRing && e == hipSuccess; ++i) {
        e = hipEventCreate(&ps->ev_start[i]);
        if (e == hipSuccess) e = hipEventCreate(&ps->ev_stop[i]);
      }
    }
    if (e != hipSuccess) {
      release(ps);
      return e == hipErrorOutOfMemory ? RUDRA_ENOMEM : RUDRA_EHIP;
    }
  }
  *out = ps;
  return RUDRA_OK;
}

int rudra_ps_destroy(rudra_ps_t* ps) {
  if (!ps) return RUDRA_OK;
  release(ps);
  return RUDRA_OK;
}

// A message (one gradient, or a relayed average standing for m of them) that has passed validation: sumGradients
// bookkeeping, vector clock, and applyUpdate once at least c gradients are in.  Caller holds the mutex.
static int absorb(rudra_ps* ps, const float* grad, const uint64_t* ts, uint32_t m, int32_t learner, float weight,
                  rudra_push_result_t* out) {
  const rudra_ps_config_t& cfg = ps->cfg;
  // Whatever can fail for lack of host memory happens before any state changes: the histogram grows to the largest
  // staleness of this message (a gradient stamped long ago makes it long), the deferral lists get their room.
  try {
    uint64_t worst = 0;
    for (uint32_t j = 0; j < m; ++j) worst = std::max(worst, ps->ts_cur - ts[j]);
    if (worst >= ps->hist.size()) ps->hist.resize(worst + 1, 0);
    if (ps->deferring) {
      ps->deferred_grads.reserve(ps->deferred_grads.size() + ps->open_grads.size() + 1);
      ps->deferred.reserve(ps->deferred.size() + 1);
    }
  } catch (const std::exception&) {  // bad_alloc, or length_error for an absurd staleness
    ps->n_rejected++;
    return RUDRA_ENOMEM;
  }
  if (!ps->control_only) {
    if (ps->accumulate) {  // sumGradients at arrival: acc = w*g, or acc = acc + w*g
      const bool weighted = weight != 1.0f || ps->open_weighted;
      Pending two[2] = {{ps->acc, 1.0f}, {grad, weight}};
      int rc = (ps->count == 0) ? enqueue_sum(ps, two + 1, 1, weighted) : enqueue_sum(ps, two, 2, weighted);
      if (rc != RUDRA_OK) return rc;
    }
  }
  uint64_t worst = 0;
  for (uint32_t j = 0; j < m; ++j) {  // staleness and vector clock (Sec. 3.1), one entry per learner gradient
    const uint64_t sigma = ps->ts_cur - ts[j];
    worst = std::max(worst, sigma);
    count_staleness(ps, sigma);
    ps->open_clock[ps->count++] = ts[j];
    ps->sigma_sum_open += sigma;
  }
  ps->n_pushes += m;
  if (weight != 1.0f) ps->open_weighted = true;
  if (!ps->accumulate) ps->open_grads.push_back({grad, weight});
  if (learner >= 0 && cfg.protocol == RUDRA_HARDSYNC) ps->seen[learner] = 1;

  int applied = 0;
  float lr_used = 0.f;
  if (ps->count >= ps->c) {  // c or more gradients are in: exactly c unless a relayed average overshoots
    // <sigma> of this update: mean over its clock of (ts_cur - ts_k) = (i-1) - mean(i_k), Eq. 2
    const double avg_sigma = (double)ps->sigma_sum_open / (double)ps->count;
    double lr = (double)cfg.alpha0 * (double)cfg.lr_scale;
    if (cfg.lr_mode == RUDRA_LR_STATIC_N) lr = lr / (double)cfg.n_split;
    else if (cfg.lr_mode == RUDRA_LR_AVG_STALENESS) lr = lr / (avg_sigma > 1.0 ? avg_sigma : 1.0);
    lr_used = (float)lr;
    if (!ps->control_only) {
      if (ps->accumulate) {
        ps->open_grads.clear();
        ps->open_grads.push_back({ps->acc, 1.0f});
      }
      if (ps->deferring) {  // rudra_ps_push_batch enqueues it, fused with its neighbours, before it returns
        ps->deferred_grads.insert(ps->deferred_grads.end(), ps->open_grads.begin(), ps->open_grads.end());
        ps->deferred.push_back({(uint32_t)ps->open_grads.size(), ps->count, lr_used, ps->open_weighted});
      } else {
        int rc = enqueue_update(ps, ps->open_grads.data(), ps->open_grads.size(), ps->count, lr_used, ps->open_weighted);
        if (rc != RUDRA_OK) { ps->failed = true; return rc; }
      }
    }
    const size_t slot = (size_t)(ps->n_updates % ps->ring);
    std::copy(ps->open_clock.begin(), ps->open_clock.begin() + ps->count, ps->ring_ts.begin() + slot * ps->clock_cap);
    ps->ring_count[slot] = ps->count;
    ps->ring_avg[slot] = avg_sigma;
    ps->ring_lr[slot] = lr_used;
    ps->last_avg = avg_sigma;
    ps->last_lr = lr_used;
    ps->n_updates += 1;
    ps->ts_cur += 1;  // the timestamp counts the weight updates (Sec. 3.1)
    ps->count = 0;
    ps->sigma_sum_open = 0;
    ps->open_weighted = false;
    ps->open_grads.clear();
    std::fill(ps->seen.begin(), ps->seen.end(), 0);
    applied = 1;
  }
  if (out) {
    out->staleness = worst;
    out->ts_after = ps->ts_cur;
    out->pending = ps->count;
    out->applied = applied;
    out->lr_used = lr_used;
  }
  return RUDRA_OK;
}

// null / alignment / (optionally) runtime check of a pushed device pointer
static int check_pushed_pointer(rudra_ps* ps, const float* grad) {
  if (ps->control_only) return RUDRA_OK;
  if (!grad || (reinterpret_cast<uintptr_t>(grad) & 15u)) return RUDRA_EINVAL;
  if (ps->check_pointers) {
    if (!is_device_range(grad, ps->cfg.n_params * sizeof(float), ps->cfg.device)) return RUDRA_EINVAL;
  }
  return RUDRA_OK;
}

// One pushGradient message: validation (a rejected message changes nothing but the rejection counter), then absorb.
// Caller holds the mutex and has made the device current.
static int push_one(rudra_ps* ps, const float* grad, uint64_t ts, int32_t learner, rudra_push_result_t* out) {
  const rudra_ps_config_t& cfg = ps->cfg;
  int rc = check_pushed_pointer(ps, grad);
  if (rc == RUDRA_EHIP) return rc;
  if (rc != RUDRA_OK) { ps->n_rejected++; return rc; }
  if (learner < -1 || learner >= (int32_t)cfg.n_learners) { ps->n_rejected++; return RUDRA_EINVAL; }
  if (ts > ps->ts_cur) { ps->n_rejected++; return RUDRA_EFUTURE_TS; }
  if (cfg.protocol == RUDRA_HARDSYNC) {
    if (ts != ps->ts_cur) { ps->n_rejected++; return RUDRA_EHARDSYNC_STALE; }
    if (learner >= 0 && ps->seen[learner]) { ps->n_rejected++; return RUDRA_EHARDSYNC_DUP; }
  }
  const uint64_t sigma = ps->ts_cur - ts;
  float weight = 1.0f;
  if (cfg.lr_mode == RUDRA_LR_PER_GRADIENT) {  // Sec. 5.1 footnote: a staler gradient gets a smaller rate
    weight = (float)(1.0 / (sigma > 1 ? (double)sigma : 1.0));
    ps->open_weighted = true;  // every update of this mode runs the weighted kernel
  }
  return absorb(ps, grad, &ts, 1, learner, weight, out);
}

int rudra_ps_push_gradient(rudra_ps_t* ps, const float* grad, uint64_t ts, int32_t learner, rudra_push_result_t* out) {
  if (!ps) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->control_only ? -1 : ps->cfg.device);
  if (guard.error() != hipSuccess) return hip_fail(ps, guard.error());
  return push_one(ps, grad, ts, learner, out);
}

int rudra_ps_push_batch(rudra_ps_t* ps, const float* const* grads, const uint64_t* ts, const int32_t* learners, uint32_t n,
                        rudra_push_result_t* out, uint32_t* n_handled) {
  if (n_handled) *n_handled = 0;
  if (!ps || (n && !ts) || (n && !grads && !(ps->cfg.flags & RUDRA_FLAG_CONTROL_ONLY))) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->control_only ? -1 : ps->cfg.device);
  if (guard.error() != hipSuccess) return hip_fail(ps, guard.error());
  // accumulate-at-push reuses one accumulator from update to update, so its updates cannot wait for each other
  ps->deferring = !ps->control_only && !ps->accumulate;
  int rc = RUDRA_OK;
  uint32_t i = 0;
  try {
    for (; i < n; ++i) {
      rc = push_one(ps, grads ? grads[i] : nullptr, ts[i], learners ? learners[i] : -1, out ? out + i : nullptr);
      if (rc != RUDRA_OK) break;  // the messages before it stay handled; this one and the rest are not
    }
  } catch (const std::exception&) {  // cannot happen: absorb reserves before it changes anything
    rc = RUDRA_ENOMEM;
    ps->failed = true;  // the protocol state is ahead of the device state: nothing more can be trusted
  }
  ps->deferring = false;
  if (n_handled) *n_handled = i;
  if (!ps->failed) {
    const int frc = flush_deferred(ps);
    if (frc != RUDRA_OK) { ps->failed = true; return frc; }
  }
  return rc;
}

int rudra_ps_push_aggregate(rudra_ps_t* ps, const float* avg, const uint64_t* ts, uint32_t m, rudra_push_result_t* out) {
  if (!ps || !ts || m == 0) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->failed) return RUDRA_EHIP;
  const rudra_ps_config_t& cfg = ps->cfg;
  DeviceGuard guard(ps->control_only ? -1 : cfg.device);
  if (guard.error() != hipSuccess) return hip_fail(ps, guard.error());
  int rc = check_pushed_pointer(ps, avg);
  if (rc == RUDRA_EHIP) return rc;
  if (rc != RUDRA_OK) { ps->n_rejected++; return rc; }
  const uint32_t max_m = cfg.max_aggregate > 1 ? cfg.max_aggregate : 1;
  if (m > max_m || cfg.lr_mode == RUDRA_LR_PER_GRADIENT) { ps->n_rejected++; return RUDRA_EINVAL; }
  // hardsync averages exactly one gradient from each of the lambda learners (Eq. 3): a relayed average may complete
  // the step but not overshoot it (the "c or more" trigger belongs to n-softsync, Eq. 5)
  if (cfg.protocol == RUDRA_HARDSYNC && (uint64_t)ps->count + m > ps->c) { ps->n_rejected++; return RUDRA_EHARDSYNC_DUP; }
  for (uint32_t j = 0; j < m; ++j) {
    if (ts[j] > ps->ts_cur) { ps->n_rejected++; return RUDRA_EFUTURE_TS; }
    if (cfg.protocol == RUDRA_HARDSYNC && ts[j] != ps->ts_cur) { ps->n_rejected++; return RUDRA_EHARDSYNC_STALE; }
  }
  // the message stands for m learner gradients: the running sum takes m * avg
  return absorb(ps, avg, ts, m, -1, (float)m, out);
}

int rudra_ps_leaf_mean(const float* const* grads, uint32_t k, uint64_t n_params, float* out, int32_t device, void* stream) {
  if (!grads || !out || k == 0 || n_params == 0 || (reinterpret_cast<uintptr_t>(out) & 15u)) return RUDRA_EINVAL;
  for (uint32_t j = 0; j < k; ++j)
    if (!grads[j] || (reinterpret_cast<uintptr_t>(grads[j]) & 15u)) return RUDRA_EINVAL;
  DeviceGuard guard(device);
  if (guard.error() != hipSuccess) { (void)hipGetLastError(); return RUDRA_EHIP; }
  const uint64_t n4 = n_params >> 2;
  const uint32_t block = kDefaultBlock;
  const uint64_t tiles = (n4 + block - 1) / block;
  const uint32_t grid = grid_for(tiles, block, 0);
  // resident waves per CU (measured at 72M parameters, 4 loads at a time per lane): k = 2 uncapped 6.62 TB/s; k = 3: 16 waves
  // 6.57 (uncapped 6.40); k = 6: 12 waves 6.65 (6.25); k = 18: 8 waves 6.52 (5.92)
  const uint32_t waves = (k <= 2 || n_params < kSmallVector) ? 32u : k == 3 ? 16u : k <= 8 ? 12u : 8u;
  const LaunchShape shape = {grid, block, tiles, lds_for_occupancy(waves, block)};
  UpdateArgs a;
  std::memset(&a, 0, sizeof(a));
  a.sum_out = out;
  a.n_params = n_params;
  a.ntiles = tiles;
  uint32_t first = 0;
  bool have_head = false;
  while (first < k) {  // groups of at most kMaxFused pointers; the running sum continues through `out`
    GradSet gs;
    std::memset(&gs, 0, sizeof(gs));
    uint32_t n = 0;
    if (have_head) { gs.p[n] = out; gs.w[n] = 1.0f; ++n; }
    while (n < (uint32_t)kMaxFused && first < k) { gs.p[n] = grads[first++]; gs.w[n] = 1.0f; ++n; }
    a.c = n;
    a.inv_c = (first == k) ? 1.0f / (float)k : 1.0f;  // (g_1 + ... + g_k) * (1/k): scaled once, at the end
    if (first == k) hipLaunchKernelGGL((rudra::sum_gradients_kernel<false, true, 4, 1>), dim3(shape.grid), dim3(shape.block), shape.lds_bytes, (hipStream_t)stream, gs, a);
    else hipLaunchKernelGGL((rudra::sum_gradients_kernel<false, false, 4, 1>), dim3(shape.grid), dim3(shape.block), shape.lds_bytes, (hipStream_t)stream, gs, a);
    if (hipGetLastError() != hipSuccess) return RUDRA_EHIP;
    have_head = true;
  }
  return RUDRA_OK;
}

int rudra_ps_apply_update_noalloc(const float* const* grads, uint32_t c, uint64_t n_params, float* theta, float* state,
                                  float lr, float momentum, float weight_decay, int32_t optimizer, float adagrad_eps,
                                  double* norms_out, int32_t device, void* stream) {
  if (!grads || !theta || !norms_out || c == 0 || n_params == 0) return RUDRA_EINVAL;
  if (c > (uint32_t)kMaxFused || n_params > kNoAllocMaxParams) return RUDRA_ERANGE;  // beyond what the fixed scratch serves
  if (optimizer != RUDRA_OPT_SGD && optimizer != RUDRA_OPT_ADAGRAD) return RUDRA_EINVAL;
  if (optimizer == RUDRA_OPT_ADAGRAD && (momentum != 0.0f || !(adagrad_eps >= 0.0f))) return RUDRA_EINVAL;
  if (!(lr == lr) || !(momentum == momentum) || !(weight_decay == weight_decay)) return RUDRA_EINVAL;
  const int opt = optimizer == RUDRA_OPT_ADAGRAD ? rudra::kOptAdagrad : momentum != 0.0f ? rudra::kOptMomentum : rudra::kOptSgd;
  if (opt != rudra::kOptSgd && !state) return RUDRA_EINVAL;
  if ((reinterpret_cast<uintptr_t>(theta) & 15u) || (reinterpret_cast<uintptr_t>(state) & 15u) ||
      (reinterpret_cast<uintptr_t>(norms_out) & 7u))
    return RUDRA_EINVAL;
  for (uint32_t j = 0; j < c; ++j)
    if (!grads[j] || (reinterpret_cast<uintptr_t>(grads[j]) & 15u)) return RUDRA_EINVAL;
  if (device < 0 || device >= kNoAllocMaxDevices) return RUDRA_EINVAL;
  DeviceGuard guard(device);
  if (guard.error() != hipSuccess) { (void)hipGetLastError(); return RUDRA_EHIP; }

  // The device address of this GPU's copy of the scratch array, looked up once per device with that device current.
  // In host code the array's name is only a handle for this lookup: kernels and copies take `slots`, never the name.
  double* slots = nullptr;
  uint32_t n_cus = 256;
  {
    std::lock_guard<std::mutex> lock(g_noalloc_mu);
    if (!g_noalloc_slots[device]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return RUDRA_EHIP; }
      int cus = 0;
      if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0) { (void)hipGetLastError(); cus = 256; }
      g_noalloc_cus[device] = (uint32_t)cus;
      g_noalloc_slots[device] = static_cast<double*>(p);
    }
    slots = g_noalloc_slots[device];
    n_cus = g_noalloc_cus[device];
  }

  // one norm slot per tile of kNoAllocBlock float4 positions: no grid-stride, so the slot count is the tile count
  const uint64_t n4 = n_params >> 2;
  const uint64_t tiles = (n4 + kNoAllocBlock - 1) / kNoAllocBlock;
  const uint32_t grid = (uint32_t)(tiles ? tiles : 1);  // <= kNoAllocSlots by the size check above
  const uint32_t unroll = default_unroll(c, n_params, n_cus, 1);
  const LaunchShape shape = {grid, kNoAllocBlock, tiles,
                             lds_for_occupancy(default_waves_per_cu(c, unroll, opt, n_params, kNoAllocBlock), kNoAllocBlock)};
  GradSet gs;
  std::memset(&gs, 0, sizeof(gs));
  for (uint32_t j = 0; j < c; ++j) { gs.p[j] = grads[j]; gs.w[j] = 1.0f; }
  UpdateArgs a;
  std::memset(&a, 0, sizeof(a));
  a.theta = theta;
  a.theta_out = theta;
  a.vel = state;
  a.partials = slots;
  a.n_params = n_params;
  a.ntiles = tiles;
  a.c = c;
  a.inv_c = 1.0f / (float)c;  // Eq. 5
  a.lr = lr;
  a.momentum = momentum;
  a.weight_decay = weight_decay;
  a.adagrad_eps = adagrad_eps;
  launch_apply(opt, weight_decay != 0.0f, false, true, rudra::kStateLoadsCached, unroll, 1, shape, (hipStream_t)stream, gs, a);
  if (hipGetLastError() != hipSuccess) return RUDRA_EHIP;
  hipLaunchKernelGGL(rudra::reduce_norm_slots_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, slots, grid, norms_out);
  if (hipGetLastError() != hipSuccess) return RUDRA_EHIP;
  return RUDRA_OK;
}

namespace {
// dst = src (n floats) on `st`: the library's copy kernel when dst allows 128-bit stores (src is a hipMalloc'ed vector of
// the server: always aligned), else the runtime's copy.
hipError_t copy_vector(const float* src, float* dst, uint64_t n, hipStream_t st) {
  if (reinterpret_cast<uintptr_t>(dst) & 15u) return hipMemcpyAsync(dst, src, n * sizeof(float), hipMemcpyDeviceToDevice, st);
  const uint64_t n4 = n >> 2;
  const uint64_t tiles = std::max<uint64_t>(1, (n4 + kDefaultBlock - 1) / kDefaultBlock);
  hipLaunchKernelGGL(rudra::copy_vector_kernel, dim3(grid_for(tiles, kDefaultBlock, 0)), dim3(kDefaultBlock), 0, st, src, dst, n, tiles);
  return hipGetLastError();
}
}  // namespace

int rudra_ps_pull_weights(rudra_ps_t* ps, float* dst, uint64_t* ts_out) {
  if (!ps) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (dst) {
    if (ps->control_only) return RUDRA_ESTATE;
    if (ps->failed) return RUDRA_EHIP;
    DeviceGuard guard(ps->cfg.device);
    RUDRA_HIP(ps, guard.error());
    RUDRA_HIP(ps, copy_vector(ps->theta2[ps->cur], dst, ps->cfg.n_params, ps->stream));
    ps->n_weight_copies += 1;
  } else {
    ps->n_ts_inquiries += 1;
  }
  if (ts_out) *ts_out = ps->ts_cur;
  return RUDRA_OK;
}

int rudra_ps_weights_view(rudra_ps_t* ps, const float** theta_out, uint64_t* ts_out) {
  if (!ps || !theta_out) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_ESTATE;
  if (ps->failed) return RUDRA_EHIP;
  *theta_out = ps->theta2[ps->cur];
  if (ts_out) *ts_out = ps->ts_cur;
  ps->n_weight_views += 1;
  return RUDRA_OK;
}

int rudra_ps_weights_acquire(rudra_ps_t* ps, void* reader_stream, const float** theta_out, uint64_t* ts_out, uint64_t* ticket_out) {
  if (!ps || !theta_out || !ticket_out) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_ESTATE;
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  if ((hipStream_t)reader_stream != ps->stream) {
    // the weights of ts_cur are produced by work already on the server's stream: the reader's stream waits for it
    hipEvent_t ready;
    int rc = take_event(ps, &ready);
    if (rc != RUDRA_OK) return rc;
    hipError_t e = hipEventRecord(ready, ps->stream);
    if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)reader_stream, ready, 0);
    ps->free_events.push_back(ready);
    RUDRA_HIP(ps, e);
  }
  *theta_out = ps->theta2[ps->cur];
  if (ts_out) *ts_out = ps->ts_cur;
  // the ticket names the buffer and the launch count at which it was handed out
  *ticket_out = (ps->n_apply_launches << 1) | ps->cur;
  ps->n_weight_acquires += 1;
  return RUDRA_OK;
}

int rudra_ps_weights_release(rudra_ps_t* ps, uint64_t ticket, void* reader_stream) {
  if (!ps) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_ESTATE;
  if (ps->failed) return RUDRA_EHIP;
  const uint64_t seq = ticket >> 1;
  const uint32_t buf = (uint32_t)(ticket & 1u);
  if (seq > ps->n_apply_launches || (buf == 1 && !ps->double_buffer)) return RUDRA_EINVAL;
  // the launch that overwrites the buffer is the first one after the acquire (one buffer) or the second (two)
  const uint64_t lifetime = ps->double_buffer ? 2 : 1;
  if (ps->n_apply_launches - seq >= lifetime) return RUDRA_ESTATE;  // too late: that launch is already enqueued
  if ((hipStream_t)reader_stream == ps->stream) return RUDRA_OK;    // stream order already protects the reads
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  hipEvent_t done;
  int rc = take_event(ps, &done);
  if (rc != RUDRA_OK) return rc;
  hipError_t e = hipEventRecord(done, (hipStream_t)reader_stream);
  if (e != hipSuccess) {
    ps->free_events.push_back(done);
    return hip_fail(ps, e);
  }
  ps->reader_done[buf].push_back(done);  // room was reserved when the event was created
  return RUDRA_OK;
}

extern "C++" {
namespace {
// Work that reads the current weights, enqueued on the reader's stream `rs` and ordered against the server's launches:
// rs waits for the work that produces the weights, `enqueue(buffer, rs)` puts the reads there, and the applyUpdate launch
// that next writes that buffer waits for them on the device.  On the server's own stream plain stream order does it.
// Caller holds the mutex and has made the device current.
template <typename Enqueue>
int read_weights_on(rudra_ps* ps, hipStream_t rs, Enqueue enqueue) {
  const uint32_t buf = ps->cur;
  if (rs == ps->stream) {
    RUDRA_HIP(ps, enqueue(ps->theta2[buf], rs));
    return RUDRA_OK;
  }
  hipEvent_t ready, done;
  int rc = take_event(ps, &ready);
  if (rc != RUDRA_OK) return rc;
  hipError_t e = hipEventRecord(ready, ps->stream);
  if (e == hipSuccess) e = hipStreamWaitEvent(rs, ready, 0);
  ps->free_events.push_back(ready);
  RUDRA_HIP(ps, e);
  rc = take_event(ps, &done);
  if (rc != RUDRA_OK) return rc;
  e = enqueue(ps->theta2[buf], rs);
  if (e == hipSuccess) e = hipEventRecord(done, rs);
  if (e != hipSuccess) {
    ps->free_events.push_back(done);
    return hip_fail(ps, e);
  }
  ps->reader_done[buf].push_back(done);  // room was reserved when the event was created
  return RUDRA_OK;
}
}  // namespace
}  // extern "C++"

int rudra_ps_pull_weights_on(rudra_ps_t* ps, float* dst, void* reader_stream, uint64_t* ts_out) {
  if (!ps || !dst) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_ESTATE;
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  const uint64_t n = ps->cfg.n_params;
  int rc = read_weights_on(ps, (hipStream_t)reader_stream, [&](const float* theta, hipStream_t st) { return copy_vector(theta, dst, n, st); });
  if (rc != RUDRA_OK) return rc;
  ps->n_weight_copies += 1;
  if (ts_out) *ts_out = ps->ts_cur;
  return RUDRA_OK;
}

int rudra_ps_broadcast_weights(rudra_ps_t* ps, float* const* dsts, uint32_t k, void* reader_stream, uint64_t* ts_out) {
  if (!ps || !dsts || k == 0) return RUDRA_EINVAL;
  for (uint32_t j = 0; j < k; ++j)
    if (!dsts[j] || (reinterpret_cast<uintptr_t>(dsts[j]) & 15u)) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_ESTATE;
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  const uint64_t n = ps->cfg.n_params;
  const uint64_t tiles = std::max<uint64_t>(1, ((n >> 2) + kDefaultBlock - 1) / kDefaultBlock);
  const uint32_t grid = grid_for(tiles, kDefaultBlock, 0);
  int rc = read_weights_on(ps, (hipStream_t)reader_stream, [&](const float* theta, hipStream_t st) {
    for (uint32_t first = 0; first < k; first += (uint32_t)kMaxFused) {  // at most kMaxFused destinations per launch
      const uint32_t m = std::min<uint32_t>(k - first, (uint32_t)kMaxFused);
      GradSet set;
      std::memset(&set, 0, sizeof(set));
      for (uint32_t j = 0; j < m; ++j) set.p[j] = dsts[first + j];
      hipLaunchKernelGGL(rudra::broadcast_vector_kernel, dim3(grid), dim3(kDefaultBlock), 0, st, theta, set, m, n, tiles);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  });
  if (rc != RUDRA_OK) return rc;
  ps->n_weight_copies += k;
  if (ts_out) *ts_out = ps->ts_cur;
  return RUDRA_OK;
}

int rudra_ps_launch_shape(rudra_ps_t* ps, int32_t batched, uint32_t* grid_out, uint32_t* block_out, uint64_t* ntiles_out,
                          uint32_t* lds_bytes_out) {
  if (!ps) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  const LaunchShape s = batched ? batch_shape_for(ps) : shape_for(ps);
  if (grid_out) *grid_out = s.grid;
  if (block_out) *block_out = s.block;
  if (ntiles_out) *ntiles_out = s.ntiles;
  if (lds_bytes_out) *lds_bytes_out = s.lds_bytes;
  return RUDRA_OK;
}

int rudra_ps_pull_velocity(rudra_ps_t* ps, float* dst) {
  if (!ps || !dst) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only || !ps->vel) return RUDRA_ESTATE;  // plain SGD keeps no second state vector
  if (ps->failed) return RUDRA_EHIP;
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  RUDRA_HIP(ps, copy_vector(ps->vel, dst, ps->cfg.n_params, ps->stream));
  return RUDRA_OK;
}

int rudra_ps_stats(rudra_ps_t* ps, rudra_ps_stats_t* out) {
  if (!ps || !out) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  std::memset(out, 0, sizeof(*out));
  out->ts_cur = ps->ts_cur;
  out->n_pushes = ps->n_pushes;
  out->n_updates = ps->n_updates;
  out->n_rejected = ps->n_rejected;
  out->sigma_sum = ps->sigma_sum;
  out->sigma_max = ps->sigma_max;
  out->hist_len = ps->hist.size();
  out->bytes_absorbed = ps->n_pushes * 4ull * ps->cfg.n_params;
  out->sigma_mean = ps->n_pushes ? (double)ps->sigma_sum / (double)ps->n_pushes : 0.0;
  out->last_avg_staleness = ps->last_avg;
  out->pending = ps->count;
  out->c = ps->c;
  out->last_lr = ps->last_lr;
  out->last_hip_error = ps->last_hip_error;
  out->n_weight_copies = ps->n_weight_copies;
  out->n_ts_inquiries = ps->n_ts_inquiries;
  out->n_weight_views = ps->n_weight_views;
  out->n_apply_launches = ps->n_apply_launches;
  out->n_batched_updates = ps->n_batched_updates;
  out->n_weight_acquires = ps->n_weight_acquires;
  out->n_reader_waits = ps->n_reader_waits;
  out->n_phased_launches = ps->n_phased_launches;
  if (ps->failed) return RUDRA_EHIP;
  if (ps->time_kernels) {
    DeviceGuard guard(ps->cfg.device);
    RUDRA_HIP(ps, guard.error());
    while (ps->timed_resolved < ps->timed_launches) {
      int rc = resolve_timer(ps, ps->timed_resolved);
      if (rc != RUDRA_OK) return rc;
    }
    out->kernel_ms = ps->kernel_ms;
    out->kernel_launches = ps->timed_resolved;
  }
  if (ps->want_norms && ps->n_updates > 0 && ps->partials) {
    DeviceGuard guard(ps->cfg.device);
    RUDRA_HIP(ps, guard.error());
    std::vector<double> host((size_t)ps->last_apply_blocks * kNumNorms);
    RUDRA_HIP(ps, hipMemcpyAsync(host.data(), ps->partials, host.size() * sizeof(double), hipMemcpyDeviceToHost, ps->stream));
    RUDRA_HIP(ps, hipStreamSynchronize(ps->stream));
    double g = 0.0, t = 0.0, v = 0.0, m = 0.0;
    for (uint32_t b = 0; b < ps->last_apply_blocks; ++b) {  // workgroup order: reproducible
      g += host[(size_t)b * kNumNorms + 0];
      t += host[(size_t)b * kNumNorms + 1];
      v += host[(size_t)b * kNumNorms + 2];
      m = std::max(m, host[(size_t)b * kNumNorms + 3]);
    }
    out->gbar_sq = g; out->theta_sq = t; out->v_sq = v; out->theta_inf = m;
    out->norms_valid = 1;
  }
  return RUDRA_OK;
}

int rudra_ps_staleness_hist(rudra_ps_t* ps, uint64_t* out, uint64_t cap, uint64_t* n_out) {
  if (!ps || (!out && cap)) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  const uint64_t n = ps->hist.size();
  if (n_out) *n_out = n;
  const uint64_t k = std::min(n, cap);
  if (k) std::memcpy(out, ps->hist.data(), k * sizeof(uint64_t));
  return cap < n ? RUDRA_ERANGE : RUDRA_OK;
}

int rudra_ps_vector_clock(rudra_ps_t* ps, uint64_t update_idx, uint64_t* ts_out, uint32_t cap, uint32_t* n_out,
                          double* avg_sigma_out, float* lr_out) {
  if (!ps || !ts_out) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (n_out) *n_out = ps->c;
  if (update_idx >= ps->n_updates || ps->n_updates - update_idx > ps->ring) return RUDRA_ERANGE;
  const size_t slot = (size_t)(update_idx % ps->ring);
  const uint32_t n = ps->ring_count[slot];
  if (n_out) *n_out = n;
  if (cap < n) return RUDRA_ERANGE;
  std::memcpy(ts_out, ps->ring_ts.data() + slot * ps->clock_cap, n * sizeof(uint64_t));
  if (avg_sigma_out) *avg_sigma_out = ps->ring_avg[slot];
  if (lr_out) *lr_out = ps->ring_lr[slot];
  return RUDRA_OK;
}

int rudra_ps_set_lr(rudra_ps_t* ps, float alpha0) {
  if (!ps || !(alpha0 == alpha0)) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  ps->cfg.alpha0 = alpha0;
  return RUDRA_OK;
}

int rudra_ps_sync(rudra_ps_t* ps) {
  if (!ps) return RUDRA_EINVAL;
  std::lock_guard<std::mutex> lock(ps->mu);
  if (ps->control_only) return RUDRA_OK;
  DeviceGuard guard(ps->cfg.device);
  RUDRA_HIP(ps, guard.error());
  RUDRA_HIP(ps, hipStreamSynchronize(ps->stream));
  return RUDRA_OK;
}

const char* rudra_ps_strerror(int status) {
  switch (status) {
    case RUDRA_OK: return "ok";
    case RUDRA_EINVAL: return "invalid argument";
    case RUDRA_EFUTURE_TS: return "gradient timestamp is newer than the weight timestamp";
    case RUDRA_EHARDSYNC_STALE: return "hardsync gradient was not computed from the current weights";
    case RUDRA_EHARDSYNC_DUP: return "hardsync: learner already contributed to this step";
    case RUDRA_ENOMEM: return "out of memory";
    case RUDRA_EHIP: return "HIP call failed";
    case RUDRA_ERANGE: return "index out of range or buffer too small";
    case RUDRA_ESTATE: return "call not available in this mode";
    default: return "unknown status";
  }
}

}  // extern "C"
