// Machine floors for the decode step on one MI355X: what the GPU charges for the things the step
// cannot avoid, measured with kernels that do nothing else.  Stand-alone program (no library code):
//
//     paper_2602_03152_amd/fasa_floors            prints one table; built by paper_2602_03152_amd/build.py
//
//   launch      an empty kernel, back to back on one stream (eager and as one captured graph)
//   read        plain streaming reads of 16 MiB and 128 MiB (16-byte loads, 16 per thread in flight)
//   read+write  1 MiB read, 64 KiB written (the traffic shape of a selection pass)
//   gather      8 MiB of 256-byte rows at random positions of a 128 MiB cache (K and V of one step of the
//               Llama-3-8B-shaped workload), and 97 MiB out of 512 MiB (the long-CoT workload: 32 rows x
//               6193 of 32768 tokens), ascending within a row as the selection leaves them
//   hand-off    inside one launch: store -> acknowledgement -> ticket atomic -> the last workgroup
//               reads what the others published (the cost of every "last workgroup merges" phase)
// Every timed buffer rotates over a pool larger than the last-level cache, so reads come from HBM.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); std::exit(1); } } while (0)

__global__ void empty_kernel(int* p) { if (p == reinterpret_cast<int*>(1)) *p = 0; }

// every thread reads 16 x 16 bytes, all in flight at once; a workgroup covers 64 KB: 16 chunks of 4 KB,
// `chunk16` uint4 apart (256 = one contiguous 64 KB block per workgroup; the scoring kernel's planes
// are n_cap * 4 bytes apart instead)
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t chunk16, size_t wg16,
                                                  uint32_t* __restrict__ sink) {
  const size_t i = (size_t)blockIdx.x * wg16 + threadIdx.x;
  uint4 v[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) v[u] = src[i + u * chunk16];
  uint32_t x = 0;
#pragma unroll
  for (int u = 0; u < 16; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  if (x == 0x12345678u) sink[0] = x;
}

// 4096 floats per workgroup read, 256 written
__global__ __launch_bounds__(256) void read_write_kernel(const float4* __restrict__ src,
                                                         float* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) { const float4 v = src[i + u * 256]; s += v.x + v.y + v.z + v.w; }
  dst[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// 16 lanes fetch one 256-byte row of K and one of V; 64 rows per workgroup
__global__ __launch_bounds__(256) void gather_kernel(const uint4* __restrict__ K, const uint4* __restrict__ V,
                                                     const int32_t* __restrict__ idx,
                                                     uint32_t* __restrict__ sink) {
  const int t = threadIdx.x, c = t & 15;
  uint32_t x = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int row = idx[(size_t)blockIdx.x * 64 + u * 16 + (t >> 4)];
    const uint4 a = K[(size_t)row * 16 + c], b = V[(size_t)row * 16 + c];
    x ^= a.x ^ a.w ^ b.y ^ b.z;
  }
  if (x == 0x12345678u) sink[0] = x;
}

// hand-off inside one launch: every workgroup publishes 2 KB with agent-scope stores, waits for the
// acknowledgement, takes a ticket; the last one reads all of it back with agent-scope loads.
// tm[0..3] of the last workgroup: ticks (10 ns) at start, after the acknowledgement, after the ticket,
// after the read-back.
__global__ __launch_bounds__(256) void handoff_kernel(unsigned long long* buf, unsigned* ticket,
                                                      unsigned long long* tm, unsigned* sink) {
  __shared__ unsigned tk;
  const int t = threadIdx.x;
  const unsigned long long t0 = wall_clock64();
  __hip_atomic_store(&buf[(size_t)blockIdx.x * 256 + t], (unsigned long long)t, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  const unsigned long long t1 = wall_clock64();
  if (t == 0) tk = atomicAdd(ticket, 1u);
  __syncthreads();
  const unsigned long long t2 = wall_clock64();
  if (tk != gridDim.x - 1) return;
  if (t == 0) *ticket = 0;
  unsigned long long acc = 0;
  for (unsigned b = 0; b < gridDim.x; b += 8) {
    unsigned long long v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = __hip_atomic_load(&buf[(size_t)min(b + u, gridDim.x - 1) * 256 + t], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  const unsigned long long t3 = wall_clock64();
  if (acc == 0x12345678ull) sink[0] = 1;
  if (t == 0) { tm[0] = t0; tm[1] = t1; tm[2] = t2; tm[3] = t3; }
}

template <typename F>
static double time_us(hipStream_t st, int reps, F&& launch_all) {
  hipEvent_t a, b;
  CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  launch_all();                                  // warm-up
  CK(hipStreamSynchronize(st));
  CK(hipEventRecord(a, st));
  for (int r = 0; r < reps; ++r) launch_all();
  CK(hipEventRecord(b, st));
  CK(hipStreamSynchronize(st));
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, a, b));
  CK(hipEventDestroy(a)); CK(hipEventDestroy(b));
  return (double)ms * 1000.0 / reps;
}

int main() {
  hipStream_t st;
  CK(hipStreamCreate(&st));
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  std::printf("device: %s, %d CUs, L2 %d KiB\n", prop.name, prop.multiProcessorCount, prop.l2CacheSize >> 10);
  uint32_t* sink; CK(hipMalloc(&sink, 256));

  // ---- launch ----
  const int chain = 64;
  for (int wgs : {1, 256, 2048}) {
    const double eager = time_us(st, 20, [&] {
      for (int i = 0; i < chain; ++i) hipLaunchKernelGGL(empty_kernel, dim3(wgs), dim3(256), 0, st, nullptr);
    }) / chain;
    hipGraph_t g; hipGraphExec_t ge;
    CK(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));
    for (int i = 0; i < chain; ++i) hipLaunchKernelGGL(empty_kernel, dim3(wgs), dim3(256), 0, st, nullptr);
    CK(hipStreamEndCapture(st, &g));
    CK(hipGraphInstantiate(&ge, g, nullptr, nullptr, 0));
    const double graph = time_us(st, 20, [&] { CK(hipGraphLaunch(ge, st)); }) / chain;
    std::printf("launch      empty kernel, %4d workgroups: %6.2f us each in a stream, %6.2f us each in a graph of %d\n",
                wgs, eager, graph, chain);
    CK(hipGraphExecDestroy(ge)); CK(hipGraphDestroy(g));
  }

  // ---- plain reads ----
  const size_t pool_bytes = (size_t)2 << 30;     // 2 GiB pool, rotated
  uint4* pool; CK(hipMalloc(&pool, pool_bytes));
  CK(hipMemset(pool, 1, pool_bytes));
  for (size_t mib : {(size_t)16, (size_t)128}) {
    const size_t bytes = mib << 20, n16 = bytes / 16;
    const int nbuf = (int)(pool_bytes / bytes);
    for (int planes = 0; planes < 2; ++planes) {
      // one contiguous 64 KB block per workgroup, or 16 planes of a [16][bytes / 16] array
      const size_t wgs = n16 / 4096;
      const size_t chunk16 = planes ? wgs * 256 : 256, wg16 = planes ? 256 : 4096;
      int k = 0;
      const double us = time_us(st, 4, [&] {
        for (int i = 0; i < nbuf; ++i, ++k)
          hipLaunchKernelGGL(read_kernel, dim3((unsigned)wgs), dim3(256), 0, st, pool + (size_t)(k % nbuf) * n16,
                             chunk16, wg16, sink);
      }) / nbuf;
      std::printf("read        %4zu MiB plain read, %-10s : %6.2f us  (%.2f TB/s)\n", mib,
                  planes ? "16 planes" : "contiguous", us, bytes / us * 1e-6);
    }
  }
  {
    const size_t bytes = (size_t)1 << 20;
    float* dst; CK(hipMalloc(&dst, (size_t)64 << 10));
    const int nbuf = 512; int k = 0;
    const double us = time_us(st, 2, [&] {
      for (int i = 0; i < nbuf; ++i, ++k)
        hipLaunchKernelGGL(read_write_kernel, dim3(64), dim3(256), 0, st,
                           reinterpret_cast<const float4*>(pool) + (size_t)(k % 1024) * (bytes / 16), dst);
    }) / nbuf;
    std::printf("read+write  1 MiB read, 64 KiB written    : %6.2f us\n", us);
    CK(hipFree(dst));
  }
  // ---- gather: rows x B entries of K and of V out of rows x 32768 cached rows ----
  for (int big = 0; big < 2; ++big) {
    const int rows = big ? 32 : 8, N = 32768, B = big ? 6193 : 2048, nsets = 4;
    const int Bp = (B + 63) / 64 * 64;                     // list padded to whole workgroups (repeats the last entry)
    const size_t cache16 = (size_t)rows * N * 16;          // uint4 per cache (64 MiB, or 256 MiB)
    std::vector<int32_t> h((size_t)nsets * rows * Bp);
    uint64_t s = 88172645463325252ull;
    for (int k = 0; k < nsets; ++k)
      for (int r = 0; r < rows; ++r) {
        std::vector<int32_t> pick(N);
        for (int j = 0; j < N; ++j) pick[j] = j;
        for (int j = 0; j < B; ++j) {                      // B distinct tokens, then ascending
          s ^= s << 13; s ^= s >> 7; s ^= s << 17;
          std::swap(pick[j], pick[j + (int)(s % (uint64_t)(N - j))]);
        }
        std::sort(pick.begin(), pick.begin() + B);
        for (int j = 0; j < Bp; ++j) h[((size_t)k * rows + r) * Bp + j] = r * N + pick[std::min(j, B - 1)];
      }
    int32_t* idx; CK(hipMalloc(&idx, h.size() * 4));
    CK(hipMemcpy(idx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    int k = 0;
    const double us = time_us(st, big ? 20 : 50, [&] {
      for (int i = 0; i < nsets; ++i, ++k) {
        const int set = k % nsets;
        hipLaunchKernelGGL(gather_kernel, dim3(rows * Bp / 64), dim3(256), 0, st, pool + (size_t)(2 * set) * cache16,
                           pool + (size_t)(2 * set + 1) * cache16, idx + (size_t)set * rows * Bp, sink);
      }
    }) / nsets;
    std::printf("gather      %5.1f MiB of 256-byte rows (K+V) : %6.2f us  (%.2f TB/s)\n", (double)rows * B * 512 / 1048576.0, us,
                (double)rows * B * 512 / us * 1e-6);
    CK(hipFree(idx));
  }
  // ---- hand-off ----
  {
    unsigned long long* buf; CK(hipMalloc(&buf, (size_t)256 * 256 * 8));
    unsigned* ticket; CK(hipMalloc(&ticket, 4)); CK(hipMemset(ticket, 0, 4));
    unsigned long long* tm; CK(hipMalloc(&tm, 32));
    for (int wgs : {32, 256}) {
      double acc[3] = {0, 0, 0};
      const int reps = 200;
      for (int r = 0; r < reps + 10; ++r) {
        hipLaunchKernelGGL(handoff_kernel, dim3(wgs), dim3(256), 0, st, buf, ticket, tm, sink);
        CK(hipStreamSynchronize(st));
        unsigned long long h[4];
        CK(hipMemcpy(h, tm, 32, hipMemcpyDeviceToHost));
        if (r >= 10) for (int i = 0; i < 3; ++i) acc[i] += (double)(h[i + 1] - h[i]) * 0.01;
      }
      std::printf("hand-off    %3d workgroups x 2 KB: store+acknowledge %5.2f us, ticket %5.2f us, last workgroup reads %3d KB back %5.2f us\n",
                  wgs, acc[0] / reps, acc[1] / reps, wgs * 2, acc[2] / reps);
    }
  }
  std::printf("done\n");
  return 0;
}
