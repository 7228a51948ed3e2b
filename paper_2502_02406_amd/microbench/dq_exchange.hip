// Microbenchmark behind the design of the fused backward kernel: what does it cost to accumulate
// 32 x 128 float32 tiles of dQ from the 32 workgroups that share a K/V head (256 workgroups, one
// per compute unit, 256 tiles per head, every workgroup adds to every tile of its head once per
// "generation") while each workgroup also issues a step's worth of matrix instructions?
//   float atomics                          one atomicAdd per element
//   read-add-write, racy                   no lock: the bare traffic, with three cache policies
//                                          (plain, sc1 = agent scope, sc0 sc1 = system scope)
//   lock only                              an exchange-based lock per (tile, wave), no data
//   lock + read-add-write, synchronous     take, load, add, store, wait, release
//   lock + read-add-write, pipelined       the release waits one step
// "wrong" counts the elements that do not hold 32 x generations at the end: plain accesses under a
// lock LOSE updates when the workgroups of a head sit on different XCDs (spread 1) because the L2
// caches of the XCDs are not coherent with each other; agent-scope (sc1) accesses do not.
// Every spin is bounded (a wave that gives up counts a lock timeout and goes on).
// Build and run: python -m paper_2502_02406_amd.microbench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

constexpr int NSTEP = 256;          // tiles (steps) per head
constexpr int TILE_F = 32 * 128;    // floats per tile
constexpr int SPIN_LIMIT = 1 << 16;

__device__ __forceinline__ bool lock_acquire(int* lk, int lane, int* err) {
  int ok = 1;
  if (lane == 0) {
    int spins = 0;
    while (atomicCAS(lk, 0, 1) != 0) {
      if (++spins > SPIN_LIMIT || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { ok = 0; atomicAdd(err, 1); break; }
      __builtin_amdgcn_s_sleep(2);
    }
  }
  ok = __builtin_amdgcn_readfirstlane(ok);
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  return ok != 0;
}
__device__ __forceinline__ void lock_release(int* lk, int lane) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  if (lane == 0) __hip_atomic_store(lk, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int POL> __device__ __forceinline__ f32x4 ld4(const float* p) {
  f32x4 r;
  if (POL == 1) asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(r) : "v"(p) : "memory");
  else if (POL == 2) asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(r) : "v"(p) : "memory");
  else asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
template <int POL> __device__ __forceinline__ void st4(float* p, f32x4 v) {
  if (POL == 1) asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(p), "v"(v) : "memory");
  else if (POL == 2) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" :: "v"(p), "v"(v) : "memory");
  else asm volatile("global_store_dwordx4 %0, %1, off" :: "v"(p), "v"(v) : "memory");
}
// lock without fences: the data path carries its own cache policy
__device__ __forceinline__ void lock_acquire_nf(int* lk, int lane, int* err) {
  if (lane == 0) {
    int spins = 0;
    while (__hip_atomic_exchange(lk, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
      if (++spins > SPIN_LIMIT || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { atomicAdd(err, 1); break; }
      __builtin_amdgcn_s_sleep(2);
    }
  }
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void lock_release_nf(int* lk, int lane) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (lane == 0) __hip_atomic_store(lk, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// MODE2: 0 racy RMW, 1 lock synchronous, 2 lock with unlock one step later, 3 lock only (no data)
template <int MODE2, int POL>
__global__ void __launch_bounds__(256) k2(float* dq, int* locks, int* err, float* out, int gens, int nmfma, int spread) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int w = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = spread ? w / 32 : w % 8, slot = spread ? w % 32 : w / 8;
  float* const base = dq + (long)head * NSTEP * TILE_F;
  int* const lbase = locks + head * NSTEP * 4;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)0.0f; b[e] = (__bf16)1.0f; }
  f32x16 acc[8];
  for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  int* prev_lock = nullptr;
  for (int gen = 0; gen < gens; ++gen) {
    for (int s = 0; s < NSTEP; ++s) {
      const int t = (s + slot * 8) % NSTEP;
      float* const tp = base + (long)t * TILE_F + wave * 1024 + lane * 4;
      int* const lk = lbase + t * 4 + wave;
      f32x4 o4[4];
      if (MODE2 >= 1) lock_acquire_nf(lk, lane, err);
      if (MODE2 != 3) {
#pragma unroll
        for (int q = 0; q < 4; ++q) o4[q] = ld4<POL>(tp + q * 256);
      }
      for (int m = 0; m < nmfma; m += 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        if (MODE2 == 2 && m == 32 && prev_lock) { lock_release_nf(prev_lock, lane); prev_lock = nullptr; }
      }
      f32x16 r;
      if (MODE2 != 3) {
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(o4[0]), "+v"(o4[1]), "+v"(o4[2]), "+v"(o4[3]) :: "memory");
        for (int q = 0; q < 4; ++q) for (int e = 0; e < 4; ++e) r[4 * q + e] = o4[q][e];
      } else { for (int v = 0; v < 16; ++v) r[v] = 0.f; }
#pragma unroll
      for (int i = 0; i < 4; ++i) r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, r, 0, 0, 0);
      for (int v = 0; v < 16; ++v) r[v] += 1.0f;
      if (MODE2 != 3) {
#pragma unroll
        for (int q = 0; q < 4; ++q) { f32x4 y = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]}; st4<POL>(tp + q * 256, y); }
      } else { acc[0][0] += r[3]; }
      if (MODE2 == 1 || MODE2 == 3) lock_release_nf(lk, lane);
      if (MODE2 == 2) prev_lock = lk;
    }
  }
  if (MODE2 == 2 && prev_lock) lock_release_nf(prev_lock, lane);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  float sum = 0;
  for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) sum += acc[i][v];
  out[w * 256 + tid] = sum + smem[tid];
}

template <int MODE>
__global__ void __launch_bounds__(256) k(float* dq, int* locks, int* err, float* out, int gens, int nmfma, int spread) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int w = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int head = spread ? w / 32 : w % 8, slot = spread ? w % 32 : w / 8;
  float* const base = dq + (long)head * NSTEP * TILE_F;
  int* const lbase = locks + head * NSTEP * 4;
  bf16x8 a, b;
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)0.0f; b[e] = (__bf16)1.0f; }
  f32x16 acc[8];
  for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  int* prev_lock = nullptr;
  for (int gen = 0; gen < gens; ++gen) {
    for (int s = 0; s < NSTEP; ++s) {
      const int t = (s + slot * 8) % NSTEP;
      float* const tp = base + (long)t * TILE_F + wave * 1024 + lane * 4;     // fragment order: 4 x 1 KB per wave
      int* const lk = lbase + t * 4 + wave;
      f32x16 old;
      for (int v = 0; v < 16; ++v) old[v] = 0.f;
      if (MODE == 3 || MODE == 4) lock_acquire(lk, lane, err);
      if (MODE >= 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 x = *(const f32x4*)(tp + q * 256);
          for (int e = 0; e < 4; ++e) old[4 * q + e] = x[e];
        }
      }
      // the step's other matrix work
      for (int m = 0; m < nmfma; m += 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        if (MODE == 4 && m == 32 && prev_lock) { lock_release(prev_lock, lane); prev_lock = nullptr; }
      }
      // the dQ product starts from the old values (a = 0: adds nothing) ...
      f32x16 r = old;
#pragma unroll
      for (int i = 0; i < 4; ++i) r = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, r, 0, 0, 0);
      for (int v = 0; v < 16; ++v) r[v] += 1.0f;     // ... and this step's contribution is 1
      if (MODE == 1) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          for (int e = 0; e < 4; ++e) atomicAdd(tp + q * 256 + e, r[4 * q + e]);
      } else if (MODE >= 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 y = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]};
          *(f32x4*)(tp + q * 256) = y;
        }
      }
      if (MODE == 3) lock_release(lk, lane);
      if (MODE == 4) prev_lock = lk;
    }
  }
  if (MODE == 4 && prev_lock) lock_release(prev_lock, lane);
  float sum = 0;
  for (int i = 0; i < 8; ++i) for (int v = 0; v < 16; ++v) sum += acc[i][v];
  out[w * 256 + tid] = sum + smem[tid];
}

int main(int argc, char** argv) {
  const int gens = argc > 1 ? atoi(argv[1]) : 4, nmfma = argc > 2 ? atoi(argv[2]) : 64;
  hipDeviceProp_t prop; CK(hipGetDeviceProperties(&prop, 0));
  printf("CUs %d, gens %d, other mfma per step %d\n", prop.multiProcessorCount, gens, nmfma);
  float *dq, *out; int *locks, *err;
  const size_t nf = (size_t)8 * NSTEP * TILE_F;
  CK(hipMalloc(&dq, nf * 4)); CK(hipMalloc(&out, 256 * 256 * 4)); CK(hipMalloc(&locks, 8 * NSTEP * 4 * 4)); CK(hipMalloc(&err, 4));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  std::vector<float> h(nf);
  auto run = [&](auto kern, const char* name, int spread, bool check) {
    CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 100 * 1024));
    float best = 1e9;
    for (int rep = 0; rep < 3; ++rep) {
      CK(hipMemset(dq, 0, nf * 4)); CK(hipMemset(locks, 0, 8 * NSTEP * 16)); CK(hipMemset(err, 0, 4));
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      kern<<<256, 256, 100 * 1024>>>(dq, locks, err, out, gens, nmfma, spread);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      if (ms < best) best = ms;
    }
    int herr = 0; CK(hipMemcpy(&herr, err, 4, hipMemcpyDeviceToHost));
    long bad = 0;
    if (check) {
      CK(hipMemcpy(h.data(), dq, nf * 4, hipMemcpyDeviceToHost));
      const float want = 32.0f * gens;
      for (size_t i = 0; i < nf; ++i) bad += h[i] != want;
    }
    const double steps = (double)gens * NSTEP;
    printf("%-34s spread %d: %8.3f ms  %6.3f us/step  elements/s %.3e  lock timeouts %d  wrong %ld%s\n", name, spread, best,
           best * 1e3 / steps, 256.0 * steps * TILE_F / (best * 1e-3), herr, bad, check ? "" : " (not checked)");
    fflush(stdout);
  };
  for (int spread = 0; spread < 2; ++spread) {
    run(k<0>, "compute only", spread, false);
    run(k<1>, "float atomics", spread, true);
    run(k2<0, 0>, "rmw plain, racy", spread, false);
    run(k2<0, 1>, "rmw sc1, racy", spread, false);
    run(k2<0, 2>, "rmw sc0 sc1, racy", spread, false);
    run(k2<3, 0>, "lock only (xchg, no fence)", spread, false);
    run(k2<1, 0>, "lock sync, plain data", spread, true);
    run(k2<1, 1>, "lock sync, sc1 data", spread, true);
    run(k2<1, 2>, "lock sync, sc0 sc1 data", spread, true);
    run(k2<2, 0>, "lock pipelined, plain data", spread, true);
    run(k2<2, 1>, "lock pipelined, sc1 data", spread, true);
    run(k2<2, 2>, "lock pipelined, sc0 sc1 data", spread, true);
  }
  return 0;
}
