// Microbenchmark: do vector-memory stores and loads of one wave retire in issue order (one vmcnt
// counter), and how long is a store outstanding?  One wave issues a store of a fresh kilobyte
// (plain or agent-scope, sc1) and a load of a line that is already in its L1, in either order, and
// times s_waitcnt vmcnt(1) and vmcnt(0).  If the counter retired out of order, "store, then load"
// would pass vmcnt(1) after the load's ~130 clk; it takes as long as the store alone: whatever is
// issued behind a store waits for the store's acknowledgement.
// Build and run: python -m paper_2502_02406_amd.microbench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(4))) float f32x4;
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
__device__ __forceinline__ unsigned long long now() { return __builtin_readcyclecounter(); }
// mode 0: store sc1 then load; 1: load then store sc1; 2: store sc1 only; 3: load only; 4: plain store then load; 5: plain store only
template <int MODE>
__global__ void k(float* buf, float* warm, unsigned long long* out, int reps) {
  const int lane = threadIdx.x;
  float* sp = buf + ((size_t)blockIdx.x * 64 + 0) * 256 + lane * 4;
  const float* lp = warm + lane * 4;
  f32x4 v = {1.f, 2.f, 3.f, (float)lane};
  f32x4 r = *(const f32x4*)lp;     // warm the line
  unsigned long long acc1 = 0, acc0 = 0;
  for (int i = 0; i < reps; ++i) {
    sp += 256;   // a fresh kilobyte every time
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    const unsigned long long t0 = now();
    if (MODE == 0) {
      asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(sp), "v"(v) : "memory");
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(lp) : "memory");
    } else if (MODE == 1) {
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(lp) : "memory");
      asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(sp), "v"(v) : "memory");
    } else if (MODE == 2) {
      asm volatile("global_store_dwordx4 %0, %1, off sc1" :: "v"(sp), "v"(v) : "memory");
    } else if (MODE == 3) {
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(lp) : "memory");
    } else if (MODE == 4) {
      asm volatile("global_store_dwordx4 %0, %1, off" :: "v"(sp), "v"(v) : "memory");
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(lp) : "memory");
    } else {
      asm volatile("global_store_dwordx4 %0, %1, off" :: "v"(sp), "v"(v) : "memory");
    }
    asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
    const unsigned long long t1 = now();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const unsigned long long t2 = now();
    acc1 += t1 - t0; acc0 += t2 - t0;
  }
  if (lane == 0) { out[blockIdx.x * 2] = acc1 / reps; out[blockIdx.x * 2 + 1] = acc0 / reps; }
  if (r[0] == 12345.f) buf[0] = r[1];
}
int main() {
  float *buf, *warm; unsigned long long* out;
  const int nb = 256, reps = 50;
  CK(hipMalloc(&buf, (size_t)nb * 64 * 1024 + (size_t)reps * 1024 * 2)); CK(hipMalloc(&warm, 4096)); CK(hipMalloc(&out, nb * 16));
  CK(hipMemset(buf, 0, (size_t)nb * 64 * 1024)); CK(hipMemset(warm, 0, 4096));
  unsigned long long h[512];
  const char* names[] = {"sc1 store, then load", "load, then sc1 store", "sc1 store only", "load only", "plain store, then load", "plain store only"};
  for (int grid : {1, 256}) {
    for (int mode = 0; mode < 6; ++mode) {
      switch (mode) {
        case 0: k<0><<<grid, 64>>>(buf, warm, out, reps); break;
        case 1: k<1><<<grid, 64>>>(buf, warm, out, reps); break;
        case 2: k<2><<<grid, 64>>>(buf, warm, out, reps); break;
        case 3: k<3><<<grid, 64>>>(buf, warm, out, reps); break;
        case 4: k<4><<<grid, 64>>>(buf, warm, out, reps); break;
        case 5: k<5><<<grid, 64>>>(buf, warm, out, reps); break;
      }
      CK(hipDeviceSynchronize());
      CK(hipMemcpy(h, out, grid * 16, hipMemcpyDeviceToHost));
      double a1 = 0, a0 = 0; for (int i = 0; i < grid; ++i) { a1 += h[2 * i]; a0 += h[2 * i + 1]; }
      printf("grid %3d  %-24s: until vmcnt(1) %6.0f clk   until vmcnt(0) %6.0f clk\n", grid, names[mode], a1 / grid, a0 / grid);
    }
  }
  return 0;
}
