// Bandwidth probes for the benchmark harness (gfx950): what plain streaming kernels reach on the same device memory the
// parameter server's update kernel walks.  NOT part of the parameter server and none of its arithmetic: a K-stream
// read-only kernel (every lane sums one float4 of each stream; nothing is written) and a copy kernel (one float4 per lane,
// read and written), both with non-temporal accesses and one 64-lane wavefront per workgroup, the access shape of the
// update kernel.  Each entry point launches its kernel `reps` times on `stream` between two HIP events and returns the
// average duration of one launch in milliseconds through `ms_out` (HOST pointer).  Returns 0 or a hipError_t.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kMaxStreams = 32;

struct Streams {
  const float* p[kMaxStreams];
};

template <int K>
__global__ void stream_read_kernel(const Streams s, float* sink, uint64_t n4) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int k = 0; k < K; ++k) acc += __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(s.p[k]) + i);
  // never true for finite inputs of this magnitude, but the compiler cannot know: the loads stay
  if (acc.x + acc.y + acc.z + acc.w == 1.2345e30f) sink[i & 1023] = acc.x;
}

__global__ void stream_copy_kernel(const float* src, float* dst, uint64_t n4) {
  const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const floatx4*>(src) + i), reinterpret_cast<floatx4*>(dst) + i);
}

template <int K>
void launch_read(const Streams& s, float* sink, uint64_t n4, unsigned grid, hipStream_t st) {
  hipLaunchKernelGGL((stream_read_kernel<K>), dim3(grid), dim3(64), 0, st, s, sink, n4);
}

int timed(hipStream_t st, uint32_t reps, float* ms_out, void (*launch)(void*), void* ctx) {
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return (int)e; }
  launch(ctx);  // one untimed launch
  e = hipEventRecord(e0, st);
  for (uint32_t r = 0; r < reps && e == hipSuccess; ++r) { launch(ctx); e = hipGetLastError(); }
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e == hipSuccess && ms_out) *ms_out = ms / (float)reps;
  return (int)e;
}

struct ReadCtx { Streams s; float* sink; uint64_t n4; unsigned grid; hipStream_t st; uint32_t k; };
struct CopyCtx { const float* src; float* dst; uint64_t n4; unsigned grid; hipStream_t st; };

void do_read(void* p) {
  ReadCtx* c = static_cast<ReadCtx*>(p);
  switch (c->k) {
    case 1: launch_read<1>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 2: launch_read<2>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 3: launch_read<3>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 4: launch_read<4>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 8: launch_read<8>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 16: launch_read<16>(c->s, c->sink, c->n4, c->grid, c->st); break;
    case 20: launch_read<20>(c->s, c->sink, c->n4, c->grid, c->st); break;
    default: launch_read<32>(c->s, c->sink, c->n4, c->grid, c->st); break;
  }
}
void do_copy(void* p) {
  CopyCtx* c = static_cast<CopyCtx*>(p);
  hipLaunchKernelGGL(stream_copy_kernel, dim3(c->grid), dim3(64), 0, c->st, c->src, c->dst, c->n4);
}

}  // namespace

extern "C" {

// streams: HOST array of k DEVICE pointers (n floats each, 16-byte aligned), k in {1, 2, 3, 4, 8, 16, 20, 32};
// sink: DEVICE pointer to at least 1024 floats (never written in practice).  n must be a multiple of 4, below 2^34.
int synth_stream_read(const float* const* streams, uint32_t k, uint64_t n, float* sink, uint32_t reps, void* stream, float* ms_out) {
  if (!streams || !sink || !reps || (n & 3u) || n == 0 || (n >> 2) > 0xFFFFFFFFull / 64 * 64) return (int)hipErrorInvalidValue;
  if (!(k == 1 || k == 2 || k == 3 || k == 4 || k == 8 || k == 16 || k == 20 || k == 32)) return (int)hipErrorInvalidValue;
  ReadCtx c;
  for (uint32_t j = 0; j < k; ++j) {
    if (!streams[j] || (reinterpret_cast<uintptr_t>(streams[j]) & 15u)) return (int)hipErrorInvalidValue;
    c.s.p[j] = streams[j];
  }
  c.sink = sink; c.n4 = n >> 2; c.grid = (unsigned)((c.n4 + 63) / 64); c.st = (hipStream_t)stream; c.k = k;
  return timed(c.st, reps, ms_out, do_read, &c);
}

// src, dst: DEVICE pointers, n floats each, 16-byte aligned, not overlapping.
int synth_stream_copy(const float* src, float* dst, uint64_t n, uint32_t reps, void* stream, float* ms_out) {
  if (!src || !dst || !reps || (n & 3u) || n == 0 || (n >> 2) > 0xFFFFFFFFull / 64 * 64) return (int)hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return (int)hipErrorInvalidValue;
  CopyCtx c = {src, dst, n >> 2, (unsigned)(((n >> 2) + 63) / 64), (hipStream_t)stream};
  return timed(c.st, reps, ms_out, do_copy, &c);
}

}  // extern "C"
