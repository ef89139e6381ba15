// Fused sumGradients + applyUpdate kernels of the Rudra parameter server (gfx950 / CDNA4).
//
// One launch reads each of the c pushed gradients once, reads and writes theta (and the
// momentum velocity v) once, and does all of Eq. 5 (average of c gradients) and Eq. 1c
// (theta <- theta - alpha * gbar), plus the momentum and weight-penalty terms of Sec. 4.2, in
// registers.  The path is a pure HBM stream: (c+5) flops per (4c+16) bytes, so there is no
// MFMA and no LDS staging here; what matters is 128-bit coalesced access, the cache policy of
// each stream, and how many tiles are in flight at once (see "Cache policy" below).
//
// Arithmetic contract (must stay bit-compatible with a sequential binary32 evaluation):
//   s    = w_1*g_1[k]; s = s + w_l*g_l[k]  for l = 2..c, in arrival order   (w_l only in the
//          per-gradient-staleness mode, Sec. 5.1 footnote; otherwise no multiply at all)
//   gbar = s * inv_c;            if wd != 0: gbar = gbar + wd*theta[k]
//   momentum:  v[k] = m*v[k] - lr*gbar ; theta[k] = theta[k] + v[k]
//   AdaGrad:   h[k] = h[k] + gbar*gbar ; theta[k] = theta[k] - (lr*gbar) / (sqrt(h[k]) + eps)
//              (h shares the second state vector with v; sqrt and divide correctly rounded)
//   otherwise: theta[k] = theta[k] - lr*gbar
// every operation rounded on its own: this file is compiled with -ffp-contract=off and the
// pragma below, so no multiply-add is ever fused.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace rudra {

constexpr int kMaxFused = 64;  // gradient pointers one launch can take (kernarg: 64*8 + 64*4 bytes)
constexpr int kNumNorms = 4;   // gbar^2, theta^2, v^2, max|theta|
constexpr int kMaxBatchUpdates = 64;  // consecutive updates one batched launch can apply

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct GradSet {
  const float* p[kMaxFused];
  float w[kMaxFused];
};

struct UpdateArgs {
  const float* theta;  // weights before the update ...
  float* theta_out;    // ... and where the updated weights go: the same buffer, or the other half of a double buffer
  float* vel;
  float* sum_out;    // sum kernel only: where the running sum goes (may alias p[0])
  double* partials;  // STATS: kNumNorms doubles per workgroup
  uint64_t n_params;
  uint64_t ntiles;   // ceil((n_params/4) / (blockDim*V)), computed on the host
  uint32_t c;        // gradients in this launch, 1..kMaxFused
  uint32_t reverse;  // 1: walk the tiles from the last to the first
  float inv_c, lr, momentum, weight_decay, adagrad_eps;
};

// The consecutive updates that one batched launch applies, in order: update u consumes the next count[u] gradients of
// the GradSet (their counts sum to at most kMaxFused) with its own rate and its own 1/c.
struct BatchPlan {
  uint32_t n_updates;
  uint8_t count[kMaxBatchUpdates];
  float lr[kMaxBatchUpdates];
  float inv_c[kMaxBatchUpdates];
};

enum : int { kOptSgd = 0, kOptMomentum = 1, kOptAdagrad = 2 };  // which second state vector, if any

// Cache policy (measured on MI355X at 72M parameters, c = 18 and c = 1):
//   gradients   read once, never again: non-temporal loads (+4 %).
//   theta, v    written with non-temporal stores (+8 %: the two write streams, not the c read streams, are what
//               costs bandwidth in this access mix) but read with ordinary loads, because successive updates walk
//               the vector in opposite directions (UpdateArgs::reverse): the lines written last by update i are the
//               first read by update i+1 and part of them is still in the memory-side cache (+5 % at c = 18,
//               +9 % at c = 1).
//   scope bits (sc0/sc1) make no difference (all 512 load/load/store policy combinations were tried).
// Launch shape: one 64-lane wavefront per workgroup (6-8 % faster than 256-thread workgroups), and the host caps the
// resident waves per CU by reserving unused LDS: what counts is the volume of loads in flight per CU and, at equal
// volume, that few tiles are open at once (more concurrently open tiles keep more DRAM pages open and lose 3-6 %).
// Measured optimum: c <= 4: all loads of a wave in one round, 12-16 waves; c > 4: ONE gradient load at a time per wave
// (U = 1) and 26 waves.  Keeping 2-4 gradient loads rolling per wave, lanes that own 2-4 tiles (adjacent or strided),
// per-XCD contiguous regions and grid-stride persistence were all measured and are slower or equal.
__device__ __forceinline__ floatx4 load_grad4(const float* p, uint64_t iv) {
  return __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p) + iv);
}
__device__ __forceinline__ float load_grad1(const float* p, uint64_t k) { return __builtin_nontemporal_load(p + k); }
__device__ __forceinline__ floatx4 load_state4(const floatx4* p, uint64_t iv) { return p[iv]; }
__device__ __forceinline__ void store_state4(floatx4* p, uint64_t iv, floatx4 x) { __builtin_nontemporal_store(x, p + iv); }

// Sum of the c gradients at V vector positions, in arrival order.  Loads are issued U
// gradients x V positions at a time before the first add that needs them, so each lane keeps
// up to U*V independent 16-byte loads in flight (the host picks U; see "Launch shape" above).
template <bool WEIGHTED, int N, int V>
__device__ __forceinline__ void add_n(const GradSet& gs, uint32_t j, const uint64_t (&iv)[V], floatx4 (&s)[V]) {
  floatx4 t[N][V];
#pragma unroll
  for (int u = 0; u < N; ++u)
#pragma unroll
    for (int v = 0; v < V; ++v) t[u][v] = load_grad4(gs.p[j + u], iv[v]);
#pragma unroll
  for (int u = 0; u < N; ++u)
#pragma unroll
    for (int v = 0; v < V; ++v) {
      if (WEIGHTED) t[u][v] = t[u][v] * gs.w[j + u];
      s[v] = s[v] + t[u][v];
    }
}

template <bool WEIGHTED, int U, int V>
__device__ __forceinline__ void sum_gradients(const GradSet& gs, uint32_t c, const uint64_t (&iv)[V],
                                              floatx4 (&s)[V]) {
#pragma unroll
  for (int v = 0; v < V; ++v) {
    s[v] = load_grad4(gs.p[0], iv[v]);
    if (WEIGHTED) s[v] = s[v] * gs.w[0];
  }
  uint32_t j = 1;
  for (; j + U <= c; j += U) add_n<WEIGHTED, U, V>(gs, j, iv, s);
  if (U > 4 && (c - j) & 4u) { add_n<WEIGHTED, 4, V>(gs, j, iv, s); j += 4; }
  if (U > 2 && (c - j) & 2u) { add_n<WEIGHTED, 2, V>(gs, j, iv, s); j += 2; }
  if (U > 1 && (c - j) & 1u) { add_n<WEIGHTED, 1, V>(gs, j, iv, s); j += 1; }
}

template <bool WEIGHTED>
__device__ __forceinline__ float sum_gradients_scalar(const GradSet& gs, uint32_t c, uint64_t k) {
  float s = load_grad1(gs.p[0], k);
  if (WEIGHTED) s = s * gs.w[0];
  for (uint32_t j = 1; j < c; ++j) {
    float t = load_grad1(gs.p[j], k);
    if (WEIGHTED) t = t * gs.w[j];
    s = s + t;
  }
  return s;
}

struct Norms {
  float gbar_sq, theta_sq, v_sq, theta_inf;
};

// applyUpdate on one element.  The single place where the update rule is written.
template <int OPT, bool DECAY, bool STATS>
__device__ __forceinline__ void update_element(float s, float& th, float& v, const UpdateArgs& a, Norms& n) {
  float gbar = s * a.inv_c;
  if (DECAY) {
    float penalty = a.weight_decay * th;
    gbar = gbar + penalty;
  }
  if (OPT == kOptMomentum) {
    float keep = a.momentum * v;
    float step = a.lr * gbar;
    v = keep - step;
    th = th + v;
  } else if (OPT == kOptAdagrad) {
    float sq = gbar * gbar;
    v = v + sq;
    // __builtin_sqrtf and '/' compile to the correctly rounded sequences (v_sqrt_f32 plus the +-1 ulp fix-up;
    // v_div_scale/fmas/fixup); the __fsqrt_rn device function does not (bare v_sqrt_f32, 1 ulp)
    float denom = __builtin_sqrtf(v) + a.adagrad_eps;
    float step = a.lr * gbar;
    float scaled = step / denom;
    th = th - scaled;
  } else {
    float step = a.lr * gbar;
    th = th - step;
  }
  if (STATS) {
    n.gbar_sq += gbar * gbar;
    n.theta_sq += th * th;
    if (OPT != kOptSgd) n.v_sq += v * v;
    n.theta_inf = fmaxf(n.theta_inf, fabsf(th));
  }
}

template <int OPT, bool DECAY, bool STATS>
__device__ __forceinline__ void update_vec4(const floatx4& s, floatx4& th, floatx4& ve, const UpdateArgs& a, Norms& n) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float t = th[i], v = (OPT != kOptSgd) ? ve[i] : 0.f;
    update_element<OPT, DECAY, STATS>(s[i], t, v, a, n);
    th[i] = t;
    if (OPT != kOptSgd) ve[i] = v;
  }
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_down(x, off, 64));
  return x;
}

// Norm partials: each lane's fp32 partial -> wavefront reduction (cross-lane shuffles) -> the
// workgroup's waves combined in wave order by lane 0 in fp64 -> one slot per workgroup.  No
// atomics: the host adds the slots in workgroup order, so the result is reproducible for a
// given launch shape.
__device__ __forceinline__ void block_reduce_norms(const Norms& n, double* partials) {
  __shared__ float lds[16][kNumNorms];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
  float g = wave_sum(n.gbar_sq), t = wave_sum(n.theta_sq), v = wave_sum(n.v_sq), m = wave_max(n.theta_inf);
  if (lane == 0) {
    lds[wave][0] = g; lds[wave][1] = t; lds[wave][2] = v; lds[wave][3] = m;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double dg = 0.0, dt = 0.0, dv = 0.0, dm = 0.0;
    for (int w = 0; w < nwaves; ++w) {
      dg += (double)lds[w][0]; dt += (double)lds[w][1]; dv += (double)lds[w][2];
      dm = fmax(dm, (double)lds[w][3]);
    }
    double* out = partials + (uint64_t)blockIdx.x * kNumNorms;
    out[0] = dg; out[1] = dt; out[2] = dv; out[3] = dm;
  }
}

// Tiling: the vector of n4 = P/4 float4 positions is cut into tiles of blockDim*V positions;
// within a tile lane t handles positions t, t+blockDim, ... so every load instruction of a
// wave covers 1 KiB contiguous and a workgroup walks blockDim*V*16 contiguous bytes of each of
// the c+2 streams.  Workgroups take tiles blockIdx, blockIdx+gridDim, ... (grid-stride); the
// host normally launches one workgroup per tile.  The last P%4 elements are done by the first
// lanes of workgroup 0 with scalar accesses.
template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int U, int V>
__global__ void apply_update_kernel(const GradSet gs, const UpdateArgs a) {
  const uint64_t n4 = a.n_params >> 2;
  const uint64_t tile = (uint64_t)blockDim.x * V;
  const uint64_t ntiles = a.ntiles;
  const floatx4* theta4 = reinterpret_cast<const floatx4*>(a.theta);  // may alias theta_out4: each position is
  floatx4* theta_out4 = reinterpret_cast<floatx4*>(a.theta_out);     // read, then written, by one lane
  floatx4* vel4 = reinterpret_cast<floatx4*>(a.vel);
  Norms n = {0.f, 0.f, 0.f, 0.f};

  for (uint64_t t0 = blockIdx.x; t0 < ntiles; t0 += gridDim.x) {
    const uint64_t t = a.reverse ? ntiles - 1 - t0 : t0;
    const uint64_t base = t * tile + threadIdx.x;
    if (base + (uint64_t)(V - 1) * blockDim.x < n4) {  // all V positions of this lane in range
      uint64_t iv[V];
      floatx4 th[V], ve[V] = {}, s[V];
#pragma unroll
      for (int v = 0; v < V; ++v) iv[v] = base + (uint64_t)v * blockDim.x;
#pragma unroll
      for (int v = 0; v < V; ++v) {
        th[v] = load_state4(theta4, iv[v]);
        if (OPT != kOptSgd) ve[v] = load_state4(vel4, iv[v]);
      }
      sum_gradients<WEIGHTED, U, V>(gs, a.c, iv, s);
#pragma unroll
      for (int v = 0; v < V; ++v) {
        update_vec4<OPT, DECAY, STATS>(s[v], th[v], ve[v], a, n);
        store_state4(theta_out4, iv[v], th[v]);
        if (OPT != kOptSgd) store_state4(vel4, iv[v], ve[v]);
      }
    } else {
      for (int v = 0; v < V; ++v) {
        const uint64_t i1[1] = {base + (uint64_t)v * blockDim.x};
        if (i1[0] >= n4) break;
        floatx4 th = load_state4(theta4, i1[0]), ve = {0.f, 0.f, 0.f, 0.f}, s[1];
        if (OPT != kOptSgd) ve = load_state4(vel4, i1[0]);
        sum_gradients<WEIGHTED, U, 1>(gs, a.c, i1, s);
        update_vec4<OPT, DECAY, STATS>(s[0], th, ve, a, n);
        store_state4(theta_out4, i1[0], th);
        if (OPT != kOptSgd) store_state4(vel4, i1[0], ve);
      }
    }
  }
  if (blockIdx.x == 0) {
    const uint64_t k = (n4 << 2) + threadIdx.x;
    if (k < a.n_params) {
      float s = sum_gradients_scalar<WEIGHTED>(gs, a.c, k);
      float th = a.theta[k], ve = (OPT != kOptSgd) ? a.vel[k] : 0.f;
      update_element<OPT, DECAY, STATS>(s, th, ve, a, n);
      a.theta_out[k] = th;
      if (OPT != kOptSgd) a.vel[k] = ve;
    }
  }
  if (STATS) block_reduce_norms(n, a.partials);
}

// Several consecutive applyUpdates in one launch (a run of pushGradient messages that was handed over in one call):
// theta and v are read once, carried in registers through the updates of the plan, and written once, so u updates
// of c gradients move P*(4*u*c + 16) bytes instead of u*P*(4c + 16).  Every update is the same sequence of individually
// rounded operations as in apply_update_kernel, applied in the same order, so the final state has the same bits; the
// weights of the timestamps in between are never stored (nobody can ask for them inside one call).  D gradient
// loads are kept in flight per lane across update boundaries.  Norms (STATS) are those of the last update of the plan.
template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int D>
__device__ __forceinline__ void batch_updates_vec4(const GradSet& gs, const BatchPlan& plan, const UpdateArgs& a,
                                                   uint64_t iv, floatx4& th, floatx4& ve, Norms& n) {
  // The gradients of all updates form one list gs.p[0 .. a.c); D of them are kept in flight per lane (slot d holds
  // gradient j0 + d and is refilled with gradient j0 + d + D as soon as it has been taken), while a small state machine
  // (pos, cnt, u: all wave-uniform) walks the plan and applies an update whenever its last gradient has been added.
  const uint32_t total = a.c;
  Norms unused = {0.f, 0.f, 0.f, 0.f};
  UpdateArgs au = a;
  floatx4 q[D];
#pragma unroll
  for (int d = 0; d < D; ++d)
    if ((uint32_t)d < total) q[d] = load_grad4(gs.p[d], iv);
  uint32_t u = 0, pos = 0, cnt = plan.count[0];
  au.lr = plan.lr[0];
  au.inv_c = plan.inv_c[0];
  floatx4 s = {0.f, 0.f, 0.f, 0.f};
  for (uint32_t j0 = 0; j0 < total; j0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const uint32_t j = j0 + d;
      if (j < total) {
        floatx4 g = q[d];
        if (j + D < total) q[d] = load_grad4(gs.p[j + D], iv);
        if (WEIGHTED) g = g * gs.w[j];
        if (pos == 0) s = g;
        else s = s + g;
        if (++pos == cnt) {
          const bool last = u + 1 == plan.n_updates;
          if (STATS && last) update_vec4<OPT, DECAY, true>(s, th, ve, au, n);
          else update_vec4<OPT, DECAY, false>(s, th, ve, au, unused);
          pos = 0;
          if (!last) {
            ++u;
            cnt = plan.count[u];
            au.lr = plan.lr[u];
            au.inv_c = plan.inv_c[u];
          }
        }
      }
    }
  }
}

template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int D>
__global__ void apply_update_batch_kernel(const GradSet gs, const BatchPlan plan, const UpdateArgs a) {
  const uint64_t n4 = a.n_params >> 2;
  const uint64_t ntiles = a.ntiles;  // tiles of blockDim float4 positions
  const floatx4* theta4 = reinterpret_cast<const floatx4*>(a.theta);
  floatx4* theta_out4 = reinterpret_cast<floatx4*>(a.theta_out);
  floatx4* vel4 = reinterpret_cast<floatx4*>(a.vel);
  Norms n = {0.f, 0.f, 0.f, 0.f};
  for (uint64_t t0 = blockIdx.x; t0 < ntiles; t0 += gridDim.x) {
    const uint64_t t = a.reverse ? ntiles - 1 - t0 : t0;
    const uint64_t iv = t * blockDim.x + threadIdx.x;
    if (iv >= n4) continue;
    floatx4 th = load_state4(theta4, iv), ve = {0.f, 0.f, 0.f, 0.f};
    if (OPT != kOptSgd) ve = load_state4(vel4, iv);
    batch_updates_vec4<OPT, DECAY, WEIGHTED, STATS, D>(gs, plan, a, iv, th, ve, n);
    store_state4(theta_out4, iv, th);
    if (OPT != kOptSgd) store_state4(vel4, iv, ve);
  }
  if (blockIdx.x == 0) {
    const uint64_t k = (n4 << 2) + threadIdx.x;
    if (k < a.n_params) {
      float th = a.theta[k], ve = (OPT != kOptSgd) ? a.vel[k] : 0.f;
      Norms unused = {0.f, 0.f, 0.f, 0.f};
      UpdateArgs au = a;
      uint32_t j = 0;
      for (uint32_t u = 0; u < plan.n_updates; ++u) {
        const uint32_t cnt = plan.count[u];
        float s = load_grad1(gs.p[j], k);
        if (WEIGHTED) s = s * gs.w[j];
        for (uint32_t l = 1; l < cnt; ++l) {
          float g = load_grad1(gs.p[j + l], k);
          if (WEIGHTED) g = g * gs.w[j + l];
          s = s + g;
        }
        j += cnt;
        au.lr = plan.lr[u];
        au.inv_c = plan.inv_c[u];
        if (STATS && u + 1 == plan.n_updates) update_element<OPT, DECAY, true>(s, th, ve, au, n);
        else update_element<OPT, DECAY, false>(s, th, ve, au, unused);
      }
      a.theta_out[k] = th;
      if (OPT != kOptSgd) a.vel[k] = ve;
    }
  }
  if (STATS) block_reduce_norms(n, a.partials);
}

// sumGradients alone: sum_out[k] = w_1*g_1[k] + ... in arrival order.  Used when a gradient is
// accumulated at push time and to fold sets of more than kMaxFused gradients; sum_out may be
// the same buffer as gs.p[0] (each position is read, then written, by one lane).
// With SCALE the sum is multiplied by a.inv_c before it is stored: the average a node of the server tree relays
// to its parent (Sec. 3.3).
template <bool WEIGHTED, bool SCALE, int U, int V>
__global__ void sum_gradients_kernel(const GradSet gs, const UpdateArgs a) {
  const uint64_t n4 = a.n_params >> 2;
  const uint64_t tile = (uint64_t)blockDim.x * V;
  const uint64_t ntiles = a.ntiles;
  floatx4* out4 = reinterpret_cast<floatx4*>(a.sum_out);
  for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const uint64_t base = t * tile + threadIdx.x;
    for (int v = 0; v < V; ++v) {
      const uint64_t i1[1] = {base + (uint64_t)v * blockDim.x};
      if (i1[0] >= n4) break;
      floatx4 s[1];
      sum_gradients<WEIGHTED, U, 1>(gs, a.c, i1, s);
      if (SCALE) s[0] = s[0] * a.inv_c;
      store_state4(out4, i1[0], s[0]);
    }
  }
  if (blockIdx.x == 0) {
    const uint64_t k = (n4 << 2) + threadIdx.x;
    if (k < a.n_params) {
      float s = sum_gradients_scalar<WEIGHTED>(gs, a.c, k);
      if (SCALE) s = s * a.inv_c;
      a.sum_out[k] = s;
    }
  }
}

}  // namespace rudra
