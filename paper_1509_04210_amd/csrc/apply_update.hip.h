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
  struct Entry {     // 16 bytes: one scalar load fetches a whole entry
    uint32_t count;  // gradients of this update
    float lr, inv_c;
    uint32_t pad;
  };
  uint32_t n_updates;
  uint32_t pad[3];
  Entry e[kMaxBatchUpdates];
};

enum : int { kOptSgd = 0, kOptMomentum = 1, kOptAdagrad = 2 };  // which second state vector, if any
// which state vector is read with non-temporal loads (the other with ordinary ones); see "Cache policy" below
enum : int { kStateLoadsCached = 0, kStateLoadsVelNt = 1, kStateLoadsThetaNt = 2 };

// Cache policy (measured on MI355X at 72M parameters, c = 18 and c = 1):
//   gradients   read once, never again: non-temporal loads (+4 %).
//   theta, v    written with non-temporal stores (+8 %: the two write streams, not the c read streams, are what
//               costs bandwidth in this access mix) but read with ordinary loads, because successive updates walk
//               the vector in opposite directions (UpdateArgs::reverse): the lines written last by update i are the
//               first read by update i+1 and part of them is still in the memory-side cache (+5 % at c = 18,
//               +9 % at c = 1).
//               One of the two state loads can be made non-temporal as well (template parameter NTLD; the host picks
//               it by c and by whether there are two weight buffers, with the measurements, in state_load_policy).  With
//               all 32 combinations of ordinary / non-temporal theta load, theta store, v load, v store and gradient load
//               measured in one process on the same buffers, non-temporal stores and gradient loads always win and BOTH
//               state loads non-temporal always lose (c = 1: 0.82 against 0.88-0.90 of 8 TB/s).  Marking only a region of
//               theta / v as cacheable changes nothing (0 to 100 % of the vector tried): the reuse across updates happens in
//               the memory-side cache, which does not see these hints.
//   scope bits (sc0/sc1) make no difference (all 512 load/load/store policy combinations were tried).
// Launch shape: one 64-lane wavefront per workgroup (6-8 % faster than 256-thread workgroups), and the host caps the
// resident waves per CU by reserving unused LDS: what counts is the volume of loads in flight per CU and, at equal
// volume, that few tiles are open at once (more concurrently open tiles keep more DRAM pages open and lose 3-6 %).
// Measured optimum: c <= 4: all loads of a wave in one round, 16 waves; c > 4: ONE gradient load at a time per wave
// (U = 1) and 26 waves.  Keeping 2-4 gradient loads rolling per wave, lanes that own 2-4 tiles (adjacent or strided),
// per-XCD contiguous regions and grid-stride persistence were all measured and are slower or equal.  Short vectors are
// the exception: fewer tiles than the chip holds resident waves means one generation of waves and a launch that lasts
// c / U memory round trips, so the host picks U = 2, 4 or 8 there (default_unroll in the host code, with the figures).
__device__ __forceinline__ floatx4 load_grad4(const float* p, uint64_t iv) {
  return __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p) + iv);
}
// the same load of a float4 or a float from an address held as an integer (an address that has passed through an
// asm statement is no longer known to be global: the address space is stated explicitly)
template <typename T>
__device__ __forceinline__ T load_grad_global(uint64_t p, uint64_t i) {
  typedef const __attribute__((address_space(1))) T* global_ptr;
  return __builtin_nontemporal_load(reinterpret_cast<global_ptr>(p) + i);
}
__device__ __forceinline__ float load_grad1(const float* p, uint64_t k) { return __builtin_nontemporal_load(p + k); }
template <bool NT>
__device__ __forceinline__ floatx4 load_state4(const floatx4* p, uint64_t iv) {
  if (NT) return __builtin_nontemporal_load(p + iv);
  else return p[iv];
}
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
  if (U == 1) {
    // One gradient at a time: the pointer (and weight) of the next gradient is fetched from the kernarg while the
    // current gradient is in flight, so the scalar load's latency is off the wave's load-wait-add chain.
    uint64_t p_cur = reinterpret_cast<uint64_t>(gs.p[1]);
    float w_cur = gs.w[1];
    for (; j < c; ++j) {
      floatx4 t[V];
#pragma unroll
      for (int v = 0; v < V; ++v) t[v] = load_grad_global<floatx4>(p_cur, iv[v]);
      const uint32_t jn = j + 1 < (uint32_t)kMaxFused ? j + 1 : j;
      uint64_t p_next = reinterpret_cast<uint64_t>(gs.p[jn]);
      float w_next = gs.w[jn];
#pragma unroll
      for (int v = 0; v < V; ++v) {
        if (WEIGHTED) t[v] = t[v] * w_cur;
        s[v] = s[v] + t[v];
      }
      // the next pointer has to be in its registers here, after the wait for the gradient: without this the
      // compiler moves the scalar load to the top of the next iteration, back in front of the vector load
      if (WEIGHTED) asm volatile("" : "+s"(p_next), "+s"(w_next));
      else asm volatile("" : "+s"(p_next));
      p_cur = p_next;
      w_cur = w_next;
    }
    return;
  }
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

// Combines the per-workgroup norm slots of one launch on the device: lane t adds the slots t, t + blockDim, ... in
// that order, then the lanes' sums are added in lane order by lane 0 (fp64 throughout; the maximum likewise).  One
// workgroup; the order is fixed by n_slots and blockDim alone, so the result is reproducible.  out[0..3] =
// sum gbar^2, sum theta^2, sum v^2, max |theta|.
__global__ void reduce_norm_slots_kernel(const double* slots, uint32_t n_slots, double* out) {
  __shared__ double lds[256][kNumNorms];
  double g = 0.0, t = 0.0, v = 0.0, m = 0.0;
  for (uint32_t b = threadIdx.x; b < n_slots; b += blockDim.x) {
    const double* s = slots + (uint64_t)b * kNumNorms;
    g += s[0]; t += s[1]; v += s[2]; m = fmax(m, s[3]);
  }
  lds[threadIdx.x][0] = g; lds[threadIdx.x][1] = t; lds[threadIdx.x][2] = v; lds[threadIdx.x][3] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    double dg = 0.0, dt = 0.0, dv = 0.0, dm = 0.0;
    for (uint32_t l = 0; l < blockDim.x; ++l) {
      dg += lds[l][0]; dt += lds[l][1]; dv += lds[l][2]; dm = fmax(dm, lds[l][3]);
    }
    out[0] = dg; out[1] = dt; out[2] = dv; out[3] = dm;
  }
}

// Tiling: the vector of n4 = P/4 float4 positions is cut into tiles of blockDim*V positions;
// within a tile lane t handles positions t, t+blockDim, ... so every load instruction of a
// wave covers 1 KiB contiguous and a workgroup walks blockDim*V*16 contiguous bytes of each of
// the c+2 streams.  Workgroups take tiles blockIdx, blockIdx+gridDim, ... (grid-stride); the
// host normally launches one workgroup per tile.  The last P%4 elements are done by the first
// lanes of workgroup 0 with scalar accesses.
template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int U, int V, int NTLD = kStateLoadsCached>
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
        th[v] = load_state4<NTLD == kStateLoadsThetaNt>(theta4, iv[v]);
        if (OPT != kOptSgd) ve[v] = load_state4<NTLD == kStateLoadsVelNt>(vel4, iv[v]);
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
        floatx4 th = load_state4<NTLD == kStateLoadsThetaNt>(theta4, i1[0]), ve = {0.f, 0.f, 0.f, 0.f}, s[1];
        if (OPT != kOptSgd) ve = load_state4<NTLD == kStateLoadsVelNt>(vel4, i1[0]);
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
// weights of the timestamps in between are never stored (nobody can ask for them inside one call).  Norms (STATS)
// are those of the last update of the plan.
//
// A lane owns one position of type T: a float4, or, for the P % 4 tail done by workgroup 0, a single float.
template <int OPT, bool DECAY, bool STATS>
__device__ __forceinline__ void update_lane(const floatx4& s, floatx4& th, floatx4& ve, const UpdateArgs& a, Norms& n) {
  update_vec4<OPT, DECAY, STATS>(s, th, ve, a, n);
}
template <int OPT, bool DECAY, bool STATS>
__device__ __forceinline__ void update_lane(const float& s, float& th, float& ve, const UpdateArgs& a, Norms& n) {
  update_element<OPT, DECAY, STATS>(s, th, ve, a, n);
}

template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, typename T>
__device__ __forceinline__ void batch_updates(const GradSet& gs, const BatchPlan& plan, const UpdateArgs& a, uint64_t i,
                                              T& th, T& ve, Norms& n) {
  // The gradients of all updates form one list gs.p[0 .. a.c).  Gradient j is consumed (added and, if it completes an
  // update, that update applied) while the load of gradient j+1 is in flight; right behind that load the pointer (and
  // weight) of gradient j+2 and the plan entry of the next update are fetched from the kernarg.  pos, u, the pointers
  // and the plan entries are wave-uniform (scalar registers).  The empty asm pins the prefetched scalars into their
  // registers there: without it the compiler moves the scalar loads down to their first use, i.e. in front of the
  // next vector load, where their latency adds to the wave's load-wait-compute chain.  The last gradient is
  // consumed after the loop, so every iteration issues exactly one load and the wait counts stay exact.
  const uint32_t total = a.c;
  Norms unused = {0.f, 0.f, 0.f, 0.f};
  UpdateArgs au = a;
  uint32_t u = 0, pos = 0;
  BatchPlan::Entry cur = plan.e[0], nxt = plan.e[1];
  T s{};
  // gradient g with weight w joins the running sum; if it is the last one of update u, that update is applied
  auto consume = [&](T g, float w) {
    if (WEIGHTED) g = g * w;
    if (pos == 0) s = g;
    else s = s + g;
    if (++pos == cur.count) {
      au.lr = cur.lr;
      au.inv_c = cur.inv_c;
      if (STATS && u + 1 == plan.n_updates) update_lane<OPT, DECAY, true>(s, th, ve, au, n);
      else update_lane<OPT, DECAY, false>(s, th, ve, au, unused);
      pos = 0;
      ++u;
      cur = nxt;
    }
  };
  T g = load_grad_global<T>(reinterpret_cast<uint64_t>(gs.p[0]), i);
  uint64_t p_next = reinterpret_cast<uint64_t>(gs.p[1]);
  float w_cur = gs.w[0], w_next = gs.w[1];
  for (uint32_t j = 0; j + 1 < total; ++j) {  // gradient j is consumed while gradient j+1 is in flight
    T g_next = load_grad_global<T>(p_next, i);
    const uint32_t jn = j + 2 < (uint32_t)kMaxFused ? j + 2 : (uint32_t)kMaxFused - 1;
    const uint32_t un = u + 1 < (uint32_t)kMaxBatchUpdates ? u + 1 : u;
    uint64_t p_after = reinterpret_cast<uint64_t>(gs.p[jn]);
    float w_after = gs.w[jn];
    nxt = plan.e[un];
    if (WEIGHTED) asm volatile("" : "+s"(p_after), "+s"(w_after), "+s"(nxt.count), "+s"(nxt.lr), "+s"(nxt.inv_c));
    else asm volatile("" : "+s"(p_after), "+s"(nxt.count), "+s"(nxt.lr), "+s"(nxt.inv_c));
    consume(g, w_cur);
    g = g_next;
    p_next = p_after;
    w_cur = w_next;
    w_next = w_after;
  }
  consume(g, w_cur);
}

// The same walk for SHORT vectors (a single generation of waves, so a launch lasts as many memory round trips as a wave
// makes): R gradient loads per round, consumed in list order; the plan entry of the next update is fetched when an
// update completes.  Same operations in the same order per element as batch_updates.
template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int R, typename T>
__device__ __forceinline__ void batch_updates_rounds(const GradSet& gs, const BatchPlan& plan, const UpdateArgs& a, uint64_t i,
                                                     T& th, T& ve, Norms& n) {
  const uint32_t total = a.c;
  Norms unused = {0.f, 0.f, 0.f, 0.f};
  UpdateArgs au = a;
  uint32_t u = 0, pos = 0;
  BatchPlan::Entry cur = plan.e[0];
  T s{};
  auto consume = [&](T g, float w) {
    if (WEIGHTED) g = g * w;
    if (pos == 0) s = g;
    else s = s + g;
    if (++pos == cur.count) {
      au.lr = cur.lr;
      au.inv_c = cur.inv_c;
      if (STATS && u + 1 == plan.n_updates) update_lane<OPT, DECAY, true>(s, th, ve, au, n);
      else update_lane<OPT, DECAY, false>(s, th, ve, au, unused);
      pos = 0;
      ++u;
      cur = plan.e[u < (uint32_t)kMaxBatchUpdates ? u : (uint32_t)kMaxBatchUpdates - 1];
    }
  };
  uint32_t j = 0;
  for (; j + R <= total; j += R) {
    T g[R];
#pragma unroll
    for (int k = 0; k < R; ++k) g[k] = load_grad_global<T>(reinterpret_cast<uint64_t>(gs.p[j + k]), i);
#pragma unroll
    for (int k = 0; k < R; ++k) consume(g[k], gs.w[j + k]);
  }
  for (; j < total; ++j) consume(load_grad_global<T>(reinterpret_cast<uint64_t>(gs.p[j]), i), gs.w[j]);
}

template <int OPT, bool DECAY, bool WEIGHTED, bool STATS, int NTLD = kStateLoadsCached, int R = 1>
__global__ void apply_update_batch_kernel(const GradSet gs, const BatchPlan plan, const UpdateArgs a) {
  typedef floatx4 T;
  const uint64_t npos = a.n_params >> 2;
  const uint64_t ntiles = a.ntiles;  // tiles of blockDim positions
  const T* theta = reinterpret_cast<const T*>(a.theta);  // may alias theta_out: each position is read, then
  T* theta_out = reinterpret_cast<T*>(a.theta_out);      // written, by one lane
  T* vel = reinterpret_cast<T*>(a.vel);
  Norms n = {0.f, 0.f, 0.f, 0.f};
  for (uint64_t t0 = blockIdx.x; t0 < ntiles; t0 += gridDim.x) {
    const uint64_t t = a.reverse ? ntiles - 1 - t0 : t0;
    const uint64_t i = t * blockDim.x + threadIdx.x;
    if (i >= npos) continue;
    T th = load_state4<NTLD == kStateLoadsThetaNt>(theta, i), ve{};
    if (OPT != kOptSgd) ve = load_state4<NTLD == kStateLoadsVelNt>(vel, i);
    if (R > 1) batch_updates_rounds<OPT, DECAY, WEIGHTED, STATS, R, T>(gs, plan, a, i, th, ve, n);
    else batch_updates<OPT, DECAY, WEIGHTED, STATS, T>(gs, plan, a, i, th, ve, n);
    __builtin_nontemporal_store(th, theta_out + i);
    if (OPT != kOptSgd) __builtin_nontemporal_store(ve, vel + i);
  }
  if (blockIdx.x == 0) {  // the P % 4 elements behind the last float4
    const uint64_t k = (npos << 2) + threadIdx.x;
    if (k < a.n_params) {
      float th = a.theta[k], ve = (OPT != kOptSgd) ? a.vel[k] : 0.f;
      batch_updates<OPT, DECAY, WEIGHTED, STATS, float>(gs, plan, a, k, th, ve, n);
      a.theta_out[k] = th;
      if (OPT != kOptSgd) a.vel[k] = ve;
    }
  }
  if (STATS) block_reduce_norms(n, a.partials);
}


// ---------------------------------------------------------------------------------------------------------------------
// Phase-aligned variant for updates of MANY gradients.  Opt-in (launch_phased = 2): measured, and not a robust win.
//
// The kernels above let every wave walk the c gradients of its own tile, so at any moment the resident waves are spread
// over all c + 2 streams; DRAM then serves c + 2 concurrently open streams, and the rate falls with c (read-only probes:
// 3 streams 88 % of 8 TB/s, 20 streams 83 %; this path: c = 18 81 %, c = 54 78 %).  Here few persistent waves (as many as
// are resident at once: 4 per SIMD) each own T tiles per pass, keep the T running sums in registers and walk the
// gradients in the OUTER loop: the whole chip streams through gradient j, then through gradient j + 1, ... and only at
// the end of the pass through theta and v.  D loads are kept in flight per wave across tiles and across gradients (the
// first D tiles of the next gradient are requested while the last tiles of the current one are summed).  The vector is
// covered in n_passes passes of gridDim.x * T tiles of 64 float4 positions: in pass p, wave w owns the tiles
// (p * gridDim.x * T) + t * gridDim.x + w, t = 0..T-1, so that the waves sweep each stream front to back together.
// The host launches it on the largest prefix of the vector that is a whole number of such passes and runs the ordinary
// kernel on the rest (less than T * n_passes tiles).  Per element the operations and their order are those of
// apply_update_kernel: same bits.
// Measured against apply_update_kernel in one process (T = 25, D = 5): 72M parameters c = 40 / 48 / 54 / 64: 0 / +1 / +1 to
// +5 / +4 to +6 %; 144M: -0.5 / +2 / +2.6 / +4 %; 100M: -3.4 / -0.6 / -1.4 / +1.4 %; 36M: -2 to -6 %; c = 30 -3 %, c = 18 -8 %
// (the pass epilogue over theta and v runs with few requests in flight; it is 18 % of the bytes at c = 18, 7 % at c = 54).
// Other (T, D) that fit the registers are 3 to 8 % SLOWER than apply_update_kernel (24/4, 20/4, 16/4 at 4 waves per SIMD,
// 32/4 and 28/4 at 3, 40/4 and 48/4 at 2): the gain is small, confined to the largest c and vectors, and sensitive to the
// tiling, hence not the default.
#ifndef RUDRA_PHASED_T   // (overridable at build time for tuning runs)
#define RUDRA_PHASED_T 25
#define RUDRA_PHASED_D 5
#define RUDRA_PHASED_WPS 4
#endif
constexpr int kPhasedTiles = RUDRA_PHASED_T;          // T: 4T registers of running sums per lane
constexpr int kPhasedDepth = RUDRA_PHASED_D;          // D: gradient loads in flight per lane; must divide T (ring slots are reused in order)
constexpr int kPhasedWavesPerSimd = RUDRA_PHASED_WPS;  // 512 / this many registers per lane
static_assert(kPhasedTiles % kPhasedDepth == 0 && kPhasedDepth >= 2, "ring slots are reused in tile order");

// One gradient's phase for one wave: add its T tiles into s, keeping D requests in flight; the last D requests go to the
// next gradient's first tiles (MORE) so the queue never drains between gradients.  The empty asm keeps the compiler from
// hoisting later requests above earlier sums (it would need registers for all of them at once).
template <int T, int D, bool FIRST, bool MORE, bool WEIGHTED>
__device__ __forceinline__ void phased_accumulate(floatx4 (&s)[T], floatx4 (&ring)[D], const floatx4* q, const floatx4* qn,
                                                  uint64_t step, float w) {
#pragma unroll
  for (int t = 0; t < T - D; ++t) {
    floatx4 g = ring[t % D];
    if (WEIGHTED) g = g * w;
    if (FIRST) s[t] = g; else s[t] = s[t] + g;
    ring[t % D] = __builtin_nontemporal_load(q);
    q += step;
    asm volatile("" ::: "memory");
  }
#pragma unroll
  for (int t = T - D; t < T; ++t) {
    floatx4 g = ring[t % D];
    if (WEIGHTED) g = g * w;
    if (FIRST) s[t] = g; else s[t] = s[t] + g;
    if (MORE) { ring[t % D] = __builtin_nontemporal_load(qn); qn += step; }
    asm volatile("" ::: "memory");
  }
}

template <int OPT, bool DECAY, bool WEIGHTED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(kPhasedWavesPerSimd, kPhasedWavesPerSimd)))
void apply_update_phased_kernel(const GradSet gs, const UpdateArgs a, uint32_t n_passes) {
  constexpr int T = kPhasedTiles, D = kPhasedDepth, H = D / 2;
  const uint64_t nw = gridDim.x, w = blockIdx.x;
  const uint64_t step = nw * 64;  // float4 positions from one tile of this wave to its next
  const uint32_t c = a.c;
  Norms unused = {0.f, 0.f, 0.f, 0.f};
  for (uint32_t pass0 = 0; pass0 < n_passes; ++pass0) {
    const uint32_t pass = a.reverse ? n_passes - 1 - pass0 : pass0;
    const uint64_t first = ((uint64_t)pass * nw * T + w) * 64 + threadIdx.x;  // this lane's position in its wave's tile 0
    floatx4 s[T], ring[D];
    const floatx4* gcur = reinterpret_cast<const floatx4*>(gs.p[0]) + first;
    {
      const floatx4* q = gcur;
#pragma unroll
      for (int t = 0; t < D; ++t) { ring[t] = __builtin_nontemporal_load(q); q += step; }
      asm volatile("" ::: "memory");
    }
    if (c == 1) {
      phased_accumulate<T, D, true, false, WEIGHTED>(s, ring, gcur + (uint64_t)D * step, gcur, step, gs.w[0]);
    } else {
      const floatx4* gnext = reinterpret_cast<const floatx4*>(gs.p[1]) + first;
      phased_accumulate<T, D, true, true, WEIGHTED>(s, ring, gcur + (uint64_t)D * step, gnext, step, gs.w[0]);
      gcur = gnext;
      for (uint32_t j = 1; j + 1 < c; ++j) {
        gnext = reinterpret_cast<const floatx4*>(gs.p[j + 1]) + first;
        phased_accumulate<T, D, false, true, WEIGHTED>(s, ring, gcur + (uint64_t)D * step, gnext, step, gs.w[j]);
        gcur = gnext;
      }
      phased_accumulate<T, D, false, false, WEIGHTED>(s, ring, gcur + (uint64_t)D * step, gcur, step, gs.w[c - 1]);
    }
    // the pass's applyUpdate: theta and v of the T tiles, H tiles requested ahead (the ring's registers are free now)
    const floatx4* tq = reinterpret_cast<const floatx4*>(a.theta) + first;
    const floatx4* vq = reinterpret_cast<const floatx4*>(a.vel) + first;
    floatx4* to = reinterpret_cast<floatx4*>(a.theta_out) + first;
    floatx4* vo = reinterpret_cast<floatx4*>(a.vel) + first;
#pragma unroll
    for (int t = 0; t < H; ++t) {
      ring[t] = *tq; tq += step;
      if (OPT != kOptSgd) { ring[H + t] = *vq; vq += step; }
    }
    asm volatile("" ::: "memory");
#pragma unroll
    for (int t = 0; t < T; ++t) {
      floatx4 th = ring[t % H], ve = {0.f, 0.f, 0.f, 0.f};
      if (OPT != kOptSgd) ve = ring[H + t % H];
      if (t + H < T) {
        ring[t % H] = *tq; tq += step;
        if (OPT != kOptSgd) { ring[H + t % H] = *vq; vq += step; }
      }
      update_vec4<OPT, DECAY, false>(s[t], th, ve, a, unused);
      __builtin_nontemporal_store(th, to); to += step;
      if (OPT != kOptSgd) { __builtin_nontemporal_store(ve, vo); vo += step; }
      asm volatile("" ::: "memory");
    }
  }
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

// pullWeights (Sec. 2, Sec. 3.2): dst = src, P floats; 8 bytes per parameter, HBM-bound.  One float4 per lane, one
// wavefront per workgroup as in the update kernels; the source with ordinary loads (every learner pulls the same
// weights, and the update that follows reads them again), the destination (read by nobody on this side) with
// non-temporal stores.  Measured at 72M parameters against the runtime's device-to-device copy in one process: 83 us
// (6.9 TB/s read + written) vs 107 us (5.4 TB/s); non-temporal loads 86 us, ordinary stores 92 us, 256-thread
// workgroups 88 us.  The P % 4 tail by the first lanes of workgroup 0.  Both pointers 16-byte aligned.
__global__ void copy_vector_kernel(const float* __restrict__ src, float* __restrict__ dst, uint64_t n_params, uint64_t ntiles) {
  const uint64_t n4 = n_params >> 2;
  const floatx4* s4 = reinterpret_cast<const floatx4*>(src);
  floatx4* d4 = reinterpret_cast<floatx4*>(dst);
  for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const uint64_t i = t * blockDim.x + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(s4[i], d4 + i);
  }
  if (blockIdx.x == 0) {
    const uint64_t k = (n4 << 2) + threadIdx.x;
    if (k < n_params) dst[k] = src[k];
  }
}

// pullWeights for k learners at once (the broadcast of new weights that ends a hardsync step, Sec. 3.1; the weight
// broadcast of Rudra-adv*, Sec. 3.3): every lane reads its float4 of the weights ONCE and writes it to the k
// destinations, P * (4 + 4k) bytes instead of the P * 8k of k copies.  Destination pointers come by value in the
// kernarg (GradSet reused as a plain pointer list; the weights w[] are not read).  Same tiling and tail as
// copy_vector_kernel; all pointers 16-byte aligned.
__global__ void broadcast_vector_kernel(const float* __restrict__ src, const GradSet dsts, uint32_t k, uint64_t n_params, uint64_t ntiles) {
  const uint64_t n4 = n_params >> 2;
  const floatx4* s4 = reinterpret_cast<const floatx4*>(src);
  for (uint64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const uint64_t i = t * blockDim.x + threadIdx.x;
    if (i >= n4) continue;
    const floatx4 x = s4[i];
    for (uint32_t j = 0; j < k; ++j)
      __builtin_nontemporal_store(x, reinterpret_cast<floatx4*>(const_cast<float*>(dsts.p[j])) + i);
  }
  if (blockIdx.x == 0) {
    const uint64_t e = (n4 << 2) + threadIdx.x;
    if (e < n_params) {
      const float x = src[e];
      for (uint32_t j = 0; j < k; ++j) const_cast<float*>(dsts.p[j])[e] = x;
    }
  }
}

}  // namespace rudra
