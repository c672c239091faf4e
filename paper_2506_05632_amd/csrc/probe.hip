// Machine probes for the benchmark (not part of the sampler): what this GPU sustains on the
// instruction kinds the scan kernel is made of, on a plain streaming read and copy, and at which
// clock it runs the former.  Built into its own library (libllc_probe.so); `bench.py --workload peaks`
// prints the figures that the roofline discussion quotes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/llc_probe.h"

namespace {

constexpr int kIter = 4096;

// each kernel: 8 independent dependency chains per lane, kIter steps, 256 threads per workgroup

__global__ void __launch_bounds__(256) k_fma(float *out, float a0, long long *cyc) {
  const long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = a0 + threadIdx.x * 8 + j;
  for (int it = 0; it < kIter; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = fmaf(v[j], 1.0000001f, 0.5f);
  }
  float s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) s += v[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = __builtin_readcyclecounter() - c0; cyc[1] = wall_clock64() - w0; }
}

// one 32x32->64 product and one xor per step (the pair a Philox round is made of)
__global__ void __launch_bounds__(256) k_mad_xor(uint32_t *out, uint32_t a0, long long *cyc) {
  const long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  uint32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = a0 + threadIdx.x * 8 + j;
  for (int it = 0; it < kIter; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint64_t p = (uint64_t)v[j] * 0xD2511F53ull;
      v[j] = (uint32_t)(p >> 32) ^ (uint32_t)p;
    }
  }
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) s ^= v[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = __builtin_readcyclecounter() - c0; cyc[1] = wall_clock64() - w0; }
}

// three-input xor (one v_bitop3_b32 per step)
__global__ void __launch_bounds__(256) k_xor3(uint32_t *out, uint32_t a0, long long *cyc) {
  const long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  uint32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = a0 + threadIdx.x * 8 + j;
  for (int it = 0; it < kIter; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = __builtin_amdgcn_bitop3_b32(v[j], v[(j + 3) & 7], a0, 0x96);
  }
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) s ^= v[j];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = __builtin_readcyclecounter() - c0; cyc[1] = wall_clock64() - w0; }
}

// full Philox4x32-10 blocks, every counter word different per lane (20 products per block)
__global__ void __launch_bounds__(256) k_philox(uint32_t *out, uint32_t seed, int n, long long *cyc) {
  const long long t0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  uint32_t acc = 0;
  for (int it = 0; it < n; ++it) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      uint32_t c0 = it * 256 + threadIdx.x, c1 = m, c2 = blockIdx.x, c3 = threadIdx.x ^ 0x5555u;
      uint32_t k0 = seed, k1 = ~seed;
#pragma unroll
      for (int r = 0; r < 10; ++r) {
        const uint64_t pa = (uint64_t)c0 * 0xD2511F53ull, pb = (uint64_t)c2 * 0xCD9E8D57ull;
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96);
        c1 = (uint32_t)pb; c3 = (uint32_t)pa; c0 = n0; c2 = n2;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
      }
      acc ^= c0 ^ c1 ^ c2 ^ c3;
    }
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = __builtin_readcyclecounter() - t0; cyc[1] = wall_clock64() - w0; }
}

// streaming read: every workgroup walks its share with 128-bit loads
__global__ void __launch_bounds__(256) k_read(const float4 *src, long long n4, float *out) {
  float4 acc = make_float4(0, 0, 0, 0);
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 v = src[i];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if (acc.x + acc.y + acc.z + acc.w == 12345.678f) out[0] = 1.0f;  // (keeps the loads alive)
}

// streaming read with one full Philox4x32-10 block per 8 bytes read (the ratio of the shared-proposal
// scan with eight drafts on fp32 inputs), the words folded into the data: generator and memory together
__global__ void __launch_bounds__(256) k_philox_read(const float4 *src, long long n4, uint32_t seed, uint32_t *out, long long *cyc) {
  const long long t0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  uint32_t acc = 0;
  // a workgroup takes 1024 consecutive 16-byte words per step: four loads per lane in flight while
  // the blocks of the step before are generated (n4 is a multiple of 1024)
  const long long steps = n4 >> 10;
  long long st = blockIdx.x;
  float4 v[4];
  if (st < steps) {
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = src[(st << 10) + u * 256 + threadIdx.x];
  }
  for (; st < steps; st += gridDim.x) {
    float4 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = v[u];
    const long long nx = st + gridDim.x;
    if (nx < steps) {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = src[(nx << 10) + u * 256 + threadIdx.x];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      acc ^= __float_as_uint(w[u].x) ^ __float_as_uint(w[u].y) ^ __float_as_uint(w[u].z) ^ __float_as_uint(w[u].w);
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        uint32_t c0 = (uint32_t)st, c1 = u * 2 + m, c2 = (uint32_t)(st >> 32) + threadIdx.x, c3 = threadIdx.x ^ 0x5555u;
        uint32_t k0 = seed, k1 = ~seed;
#pragma unroll
        for (int r = 0; r < 10; ++r) {
          const uint64_t pa = (uint64_t)c0 * 0xD2511F53ull, pb = (uint64_t)c2 * 0xCD9E8D57ull;
          const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), c1, k0, 0x96);
          const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), c3, k1, 0x96);
          c1 = (uint32_t)pb; c3 = (uint32_t)pa; c0 = n0; c2 = n2;
          k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
        }
        acc ^= c0 ^ c1 ^ c2 ^ c3;
      }
    }
  }
  if (acc == 0x12345678u) out[0] = acc;  // (keeps the work alive)
  if (threadIdx.x == 0 && blockIdx.x == 0) { cyc[0] = __builtin_readcyclecounter() - t0; cyc[1] = wall_clock64() - w0; }
}

__global__ void __launch_bounds__(256) k_copy(const float4 *src, float4 *dst, long long n4) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

}  // namespace

#define CK(x) do { if ((x) != hipSuccess) { rc = -1; goto done; } } while (0)

extern "C" int llc_probe_run(int which, int reps, double *result, double *clock_ghz) {
  int rc = 0;
  hipEvent_t a = nullptr, b = nullptr;
  void *buf = nullptr, *buf2 = nullptr;
  long long *cyc = nullptr;
  float ms = 0.0f;
  const unsigned grid = 256 * 4;  // four workgroups of four wavefronts per compute unit: one round, all resident
  const size_t bytes = (size_t)4 << 30;
  *result = 0.0;
  if (clock_ghz) *clock_ghz = 0.0;
  if (reps < 1) return -1;
  CK(hipEventCreate(&a));
  CK(hipEventCreate(&b));
  CK(hipMalloc(&cyc, 64));
  if (which == LLC_PROBE_READ || which == LLC_PROBE_COPY || which == LLC_PROBE_PHILOX_READ) {
    CK(hipMalloc(&buf, bytes));
    CK(hipMemset(buf, 0, bytes));
    if (which == LLC_PROBE_COPY) CK(hipMalloc(&buf2, bytes));
  } else {
    CK(hipMalloc(&buf, (size_t)grid * 256 * 4));
  }
  for (int pass = 0; pass < 2; ++pass) {  // the first pass warms up
    CK(hipEventRecord(a, nullptr));
    for (int r = 0; r < reps; ++r) {
      switch (which) {
        case LLC_PROBE_FMA: hipLaunchKernelGGL(k_fma, dim3(grid), dim3(256), 0, nullptr, (float *)buf, 1.0f, cyc); break;
        case LLC_PROBE_MAD_XOR: hipLaunchKernelGGL(k_mad_xor, dim3(grid), dim3(256), 0, nullptr, (uint32_t *)buf, 7u, cyc); break;
        case LLC_PROBE_XOR3: hipLaunchKernelGGL(k_xor3, dim3(grid), dim3(256), 0, nullptr, (uint32_t *)buf, 7u, cyc); break;
        case LLC_PROBE_PHILOX: hipLaunchKernelGGL(k_philox, dim3(grid), dim3(256), 0, nullptr, (uint32_t *)buf, 7u, 256, cyc); break;
        case LLC_PROBE_READ: hipLaunchKernelGGL(k_read, dim3(1024), dim3(256), 0, nullptr, (const float4 *)buf, (long long)(bytes / 16), (float *)cyc); break;
        case LLC_PROBE_COPY: hipLaunchKernelGGL(k_copy, dim3(4096), dim3(256), 0, nullptr, (const float4 *)buf, (float4 *)buf2, (long long)(bytes / 16)); break;
        case LLC_PROBE_PHILOX_READ: hipLaunchKernelGGL(k_philox_read, dim3(2048), dim3(256), 0, nullptr, (const float4 *)buf, (long long)(bytes / 16), 7u, (uint32_t *)(cyc + 4), cyc); break;
        default: rc = -1; goto done;
      }
    }
    CK(hipEventRecord(b, nullptr));
    CK(hipEventSynchronize(b));
    CK(hipEventElapsedTime(&ms, a, b));
  }
  {
    const double s = (double)ms * 1e-3 / reps;
    const double lanes = (double)grid * 256;
    switch (which) {
      case LLC_PROBE_FMA: case LLC_PROBE_XOR3: *result = lanes * kIter * 8 / s; break;      // operations per second
      case LLC_PROBE_MAD_XOR: *result = lanes * kIter * 8 / s; break;                          // pairs per second
      case LLC_PROBE_PHILOX: *result = lanes * 256 * 4 * 4 / s; break;                         // 32-bit words per second
      case LLC_PROBE_READ: case LLC_PROBE_PHILOX_READ: *result = (double)bytes / s; break;     // bytes per second
      case LLC_PROBE_COPY: *result = 2.0 * (double)bytes / s; break;                           // bytes read + written per second
    }
    if (clock_ghz && which != LLC_PROBE_READ && which != LLC_PROBE_COPY) {
      long long c[2] = {0, 0};
      CK(hipMemcpy(c, cyc, sizeof(c), hipMemcpyDeviceToHost));
      // the first wavefront's shader-clock cycles over the same span on the constant 100 MHz counter
      // (the last launch's; the oldest wavefront of a unit issues first, so its span is shorter than
      // the launch, which is why both counters are read at the same two points)
      if (c[1] > 0) *clock_ghz = (double)c[0] / ((double)c[1] * 10.0);
    }
  }
done:
  if (buf) (void)hipFree(buf);
  if (buf2) (void)hipFree(buf2);
  if (cyc) (void)hipFree(cyc);
  if (a) (void)hipEventDestroy(a);
  if (b) (void)hipEventDestroy(b);
  return rc;
}
