// Measurement helpers: LDS gather micro-benchmark and a plain copy kernel.  They are not
// part of the layer path; they measure the denominators its throughput is compared with
// (LDS lookup rate with and without bank conflicts, HBM stream bandwidth).
#include <random>
#include <vector>

#include "ax_internal.h"
#include "axconv_probe.h"

namespace ax {

constexpr int kProbeSets = 8;  // independent addresses per lane, cycled through

// The reads of one iteration are issued back to back, then waited for together, so that
// each wave keeps kProbeSets gathers in flight.
template <int WIDTH>
__global__ __launch_bounds__(1024) void probe_lds_kernel(const uint32_t* __restrict__ offs, int iters,
                                                          int table_bytes, uint32_t* __restrict__ sink,
                                                          unsigned long long* __restrict__ cycles) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int tid = threadIdx.x, nt = blockDim.x;
  for (int i = tid * 4; i < table_bytes; i += nt * 4) *(uint32_t*)(lds + i) = (uint32_t)i * 2654435761u;
  __syncthreads();
  const uint32_t base = (uint32_t)(uintptr_t)lds;
  uint32_t a[kProbeSets];
#pragma unroll
  for (int j = 0; j < kProbeSets; ++j) a[j] = base + offs[(size_t)(blockIdx.x * nt + tid) * kProbeSets + j];
  uint32_t fold = 0;
  __syncthreads();
  const unsigned long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    if constexpr (WIDTH == 2 || WIDTH == 4) {
      uint32_t v[kProbeSets];
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) {
        if constexpr (WIDTH == 2)
          asm volatile("ds_read_u16 %0, %1" : "=v"(v[j]) : "v"(a[j]));
        else
          asm volatile("ds_read_b32 %0, %1" : "=v"(v[j]) : "v"(a[j]));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) fold += v[j];
    } else if constexpr (WIDTH == 8) {
      uint2 v[kProbeSets];
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) asm volatile("ds_read_b64 %0, %1" : "=v"(v[j]) : "v"(a[j]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) fold += v[j].x ^ v[j].y;
    } else {
      uint4 v[kProbeSets];
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) asm volatile("ds_read_b128 %0, %1" : "=v"(v[j]) : "v"(a[j]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int j = 0; j < kProbeSets; ++j) fold += (v[j].x ^ v[j].y) + (v[j].z ^ v[j].w);
    }
  }
  const unsigned long long t1 = clock64();
  sink[blockIdx.x * nt + tid] = fold;
  if (tid == 0) cycles[blockIdx.x] = t1 - t0;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src,
                                                          size_t n16) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n16; i += stride) dst[i] = src[i];
}

// Inner loop of the table-tile kernels in isolation: per tap one 16-byte gather per table
// group and eight adds per gather, no table building and no barrier.  It bounds what that
// instruction mix can reach when LDS gathers and integer adds overlap perfectly.
template <int THREADS, int P, int NG>
__global__ __launch_bounds__(THREADS) void probe_mac_kernel(const uint4* __restrict__ codes, int iters,
                                                             uint32_t* __restrict__ sink) {
  __shared__ uint4 tab[NG][256];
  const int tid = threadIdx.x;
  for (int i = tid; i < NG * 256; i += THREADS) {
    const uint32_t v = (uint32_t)i * 2654435761u;
    (&tab[0][0])[i] = make_uint4(v, v ^ 0x9e3779b9u, v * 3u, v * 7u);
  }
  __syncthreads();
  uint4 x[P];
#pragma unroll
  for (int p = 0; p < P; ++p) x[p] = codes[(size_t)(blockIdx.x * P + p) * THREADS + tid];
  uint32_t acc[P][NG * 8];
#pragma unroll
  for (int p = 0; p < P; ++p)
#pragma unroll
    for (int j = 0; j < NG * 8; ++j) acc[p][j] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const uint32_t w = (kk < 4) ? x[p].x : (kk < 8) ? x[p].y : (kk < 12) ? x[p].z : x[p].w;
        const uint32_t v = (w >> (8 * (kk & 3))) & 0xffu;
        const uint4* tp = &tab[0][v];
        uint4 e[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) e[g] = tp[g * 256];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          acc[p][g * 8 + 0] += e[g].x & 0xffffu;
          acc[p][g * 8 + 1] += e[g].x >> 16;
          acc[p][g * 8 + 2] += e[g].y & 0xffffu;
          acc[p][g * 8 + 3] += e[g].y >> 16;
          acc[p][g * 8 + 4] += e[g].z & 0xffffu;
          acc[p][g * 8 + 5] += e[g].z >> 16;
          acc[p][g * 8 + 6] += e[g].w & 0xffffu;
          acc[p][g * 8 + 7] += e[g].w >> 16;
        }
      }
    }
    // keep the loop from being collapsed: the codes change a little every iteration
#pragma unroll
    for (int p = 0; p < P; ++p) {
      x[p].x = x[p].x * 1664525u + 1013904223u;
      x[p].y = x[p].y * 1664525u + 1013904223u;
      x[p].z = x[p].z * 1664525u + 1013904223u;
      x[p].w = x[p].w * 1664525u + 1013904223u;
    }
  }
  uint32_t f = 0;
#pragma unroll
  for (int p = 0; p < P; ++p)
#pragma unroll
    for (int j = 0; j < NG * 8; ++j) f ^= acc[p][j];
  sink[(size_t)blockIdx.x * THREADS + tid] = f;
}

// Integer-add throughput: independent accumulators, no memory traffic in the loop.
__global__ __launch_bounds__(1024) void probe_valu_kernel(int iters, uint32_t* __restrict__ sink) {
  uint32_t a[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) a[j] = threadIdx.x + j;
  uint32_t s = blockIdx.x + 1;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int j = 0; j < 32; ++j) a[j] += (j & 1) ? (s >> 16) : (s & 0xffffu);
    s = s * 1664525u + a[0];
  }
  uint32_t f = 0;
#pragma unroll
  for (int j = 0; j < 32; ++j) f ^= a[j];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = f;
}

}  // namespace ax

extern "C" int ax_probe_lds_gather(int width_bytes, int pattern, int table_bytes, int threads, int iters,
                                   double* wave_reads, double* cycles, double* seconds, int* workgroups,
                                   void* hip_stream) {
  using namespace ax;
  if (!wave_reads || !cycles || !seconds || !workgroups) return AX_ERR_NULL;
  if (width_bytes != 2 && width_bytes != 4 && width_bytes != 8 && width_bytes != 16) return AX_ERR_OPTION;
  if (pattern < 0 || pattern > 6 || iters < 1 || iters > (1 << 20)) return AX_ERR_OPTION;
  if (pattern >= 3 && (width_bytes != 16 || table_bytes < 4096)) return AX_ERR_OPTION;
  if (threads < 64 || threads > 1024 || threads % 64) return AX_ERR_OPTION;
  if (table_bytes < 1024 || table_bytes > 160 * 1024 || table_bytes % 1024) return AX_ERR_OPTION;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return AX_ERR_HIP;
  const int wgs = prop.multiProcessorCount;
  const size_t nthreads = (size_t)wgs * threads;
  const uint32_t elems = (uint32_t)(table_bytes / width_bytes);

  std::vector<uint32_t> h(nthreads * kProbeSets);
  std::mt19937 rng(12345u + 7u * (uint32_t)pattern + (uint32_t)width_bytes);
  for (size_t t = 0; t < nthreads; ++t) {
    const uint32_t lane = (uint32_t)(t % (size_t)threads);
    for (int j = 0; j < kProbeSets; ++j) {
      uint32_t e;
      if (pattern == 0) {
        e = (lane + 64u * (uint32_t)j) % elems;
      } else if (pattern >= 3) {
        // sixteen tables interleaved entry by entry: element index = 16 * v + slot, v random; the
        // slot is a function of the lane only, so 16 lanes with distinct slots never share a bank
        const uint32_t slot = pattern == 3   ? (lane & 15u)
                              : pattern == 4 ? ((lane >> 2) & 15u)
                              : pattern == 5 ? ((lane & 7u) | ((lane >> 2) & 8u))
                                             : ((lane & 3u) | ((lane >> 2) & 12u));
        e = (rng() % (elems / 16u)) * 16u + slot;
      } else {
        e = rng() % elems;
        if (pattern == 2 && (rng() & 1u)) e = 0;
      }
      h[t * kProbeSets + j] = e * (uint32_t)width_bytes;
    }
  }
  uint32_t *d_offs = nullptr, *d_sink = nullptr;
  unsigned long long* d_cyc = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = AX_ERR_HIP;
  std::vector<unsigned long long> hc(wgs);
  float ms = 0.f;
  double csum = 0;
  do {
    if (hipMalloc(&d_offs, h.size() * 4) != hipSuccess) break;
    if (hipMalloc(&d_sink, nthreads * 4) != hipSuccess) break;
    if (hipMalloc(&d_cyc, (size_t)wgs * 8) != hipSuccess) break;
    if (hipMemcpyAsync(d_offs, h.data(), h.size() * 4, hipMemcpyHostToDevice, s) != hipSuccess) break;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
    void (*kern)(const uint32_t*, int, int, uint32_t*, unsigned long long*) =
        width_bytes == 2   ? probe_lds_kernel<2>
        : width_bytes == 4 ? probe_lds_kernel<4>
        : width_bytes == 8 ? probe_lds_kernel<8>
                           : probe_lds_kernel<16>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, table_bytes) != hipSuccess)
      break;
    // one untimed launch (code load, clocks), then the timed one
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(threads), table_bytes, s, d_offs, 4, table_bytes, d_sink, d_cyc);
    if (hipEventRecord(e0, s) != hipSuccess) break;
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(threads), table_bytes, s, d_offs, iters, table_bytes, d_sink, d_cyc);
    if (hipGetLastError() != hipSuccess) break;
    if (hipEventRecord(e1, s) != hipSuccess) break;
    if (hipMemcpyAsync(hc.data(), d_cyc, (size_t)wgs * 8, hipMemcpyDeviceToHost, s) != hipSuccess) break;
    if (hipStreamSynchronize(s) != hipSuccess) break;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) break;
    for (int i = 0; i < wgs; ++i) csum += (double)hc[i];
    rc = AX_OK;
  } while (0);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (d_offs) (void)hipFree(d_offs);
  if (d_sink) (void)hipFree(d_sink);
  if (d_cyc) (void)hipFree(d_cyc);
  if (rc != AX_OK) return rc;
  *wave_reads = (double)iters * kProbeSets * (threads / 64);
  *cycles = csum / wgs;
  *seconds = ms * 1e-3;
  *workgroups = wgs;
  return AX_OK;
}

extern "C" int ax_probe_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src) return AX_ERR_NULL;
  if (bytes == 0 || bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return AX_ERR_ALIGN;
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(ax::probe_copy_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     (uint4*)dst, (const uint4*)src, n16);
  return hipGetLastError() == hipSuccess ? AX_OK : AX_ERR_HIP;
}

// mode 0: probe_valu (128 adds per lane and iteration); mode 1..4: probe_mac with
// (threads, lane elements, groups) = (512,2,8), (1024,1,8), (512,4,4), (1024,2,4).
// pattern as in ax_probe_lds_gather (1 = uniform random codes, 2 = half of them zero).
extern "C" int ax_probe_mac(int mode, int pattern, int iters, int wgs_per_cu, double* ops, double* seconds,
                            void* hip_stream) {
  using namespace ax;
  if (!ops || !seconds) return AX_ERR_NULL;
  if (mode < 0 || mode > 4 || pattern < 1 || pattern > 2 || iters < 1 || iters > (1 << 20) || wgs_per_cu < 1 ||
      wgs_per_cu > 8)
    return AX_ERR_OPTION;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return AX_ERR_HIP;
  const int wgs = prop.multiProcessorCount * wgs_per_cu;
  const int threads = (mode == 0 || mode == 2 || mode == 4) ? 1024 : 512;
  const int P = (mode == 1 || mode == 4) ? 2 : (mode == 3 ? 4 : 1);
  const size_t lanes = (size_t)wgs * threads * P;
  std::vector<uint4> h(lanes);
  std::mt19937 rng(999u + (uint32_t)pattern);
  for (size_t i = 0; i < lanes; ++i) {
    uint32_t w[4];
    for (int c = 0; c < 4; ++c) {
      w[c] = rng();
      if (pattern == 2) {
        const uint32_t m = rng();
        for (int b = 0; b < 4; ++b)
          if ((m >> b) & 1u) w[c] &= ~(0xffu << (8 * b));
      }
    }
    h[i] = make_uint4(w[0], w[1], w[2], w[3]);
  }
  uint4* d_codes = nullptr;
  uint32_t* d_sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = AX_ERR_HIP;
  float ms = 0.f;
  do {
    if (hipMalloc(&d_codes, lanes * 16) != hipSuccess) break;
    if (hipMalloc(&d_sink, (size_t)wgs * threads * 4) != hipSuccess) break;
    if (hipMemcpyAsync(d_codes, h.data(), lanes * 16, hipMemcpyHostToDevice, s) != hipSuccess) break;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
    for (int rep = 0; rep < 2; ++rep) {
      const int n = rep == 0 ? 2 : iters;
      if (rep == 1 && hipEventRecord(e0, s) != hipSuccess) break;
      switch (mode) {
        case 0: hipLaunchKernelGGL(probe_valu_kernel, dim3(wgs), dim3(1024), 0, s, n, d_sink); break;
        case 1: hipLaunchKernelGGL((probe_mac_kernel<512, 2, 8>), dim3(wgs), dim3(512), 0, s, d_codes, n, d_sink); break;
        case 2: hipLaunchKernelGGL((probe_mac_kernel<1024, 1, 8>), dim3(wgs), dim3(1024), 0, s, d_codes, n, d_sink); break;
        case 3: hipLaunchKernelGGL((probe_mac_kernel<512, 4, 4>), dim3(wgs), dim3(512), 0, s, d_codes, n, d_sink); break;
        default: hipLaunchKernelGGL((probe_mac_kernel<1024, 2, 4>), dim3(wgs), dim3(1024), 0, s, d_codes, n, d_sink); break;
      }
    }
    if (hipGetLastError() != hipSuccess) break;
    if (hipEventRecord(e1, s) != hipSuccess) break;
    if (hipStreamSynchronize(s) != hipSuccess) break;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) break;
    rc = AX_OK;
  } while (0);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (d_codes) (void)hipFree(d_codes);
  if (d_sink) (void)hipFree(d_sink);
  if (rc != AX_OK) return rc;
  const int NG = (mode == 1 || mode == 2) ? 8 : 4;
  *ops = mode == 0 ? (double)wgs * 1024 * 128.0 * iters : (double)lanes * 16.0 * NG * 8 * iters;
  *seconds = ms * 1e-3;
  return AX_OK;
}

// Events are created and destroyed here, outside the layer path, and the stream is waited for.
extern "C" int ax_probe_layer_kernel_ms(const ax_layer_t* layer, const void* x, int32_t* acc_out, float* y_out,
                                        void* workspace, size_t workspace_bytes, int reps, float* ms,
                                        void* hip_stream) {
  using namespace ax;
  if (!ms) return AX_ERR_NULL;
  if (reps < 1 || reps > 64) return AX_ERR_OPTION;
  hipStream_t s = (hipStream_t)hip_stream;
  int rc = run_prepared(layer, x, acc_out, y_out, workspace, workspace_bytes, kPhCall, 1, s);
  if (rc) return rc;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  rc = AX_ERR_HIP;
  do {
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
    if (hipEventRecord(e0, s) != hipSuccess) break;
    rc = run_prepared(layer, x, acc_out, y_out, workspace, workspace_bytes, kPhMain, reps, s);
    if (rc) break;
    rc = AX_ERR_HIP;
    if (hipEventRecord(e1, s) != hipSuccess) break;
    rc = run_prepared(layer, x, acc_out, y_out, workspace, workspace_bytes, kPhFixup, 1, s);
    if (rc) break;
    rc = AX_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) break;
    float t = 0.f;
    if (hipEventElapsedTime(&t, e0, e1) != hipSuccess) break;
    *ms = t / (float)reps;
    rc = AX_OK;
  } while (0);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  return rc;
}
