// Machine-peak probes for MI355X (gfx950): a bench-only library (libprism_peaks.so), not part
// of libprism's ABI.  Each probe is a loop of nothing but the resource it measures, sized like
// the attention kernel uses that resource (32x32x16 bf16 MFMAs, 16-byte LDS operand reads with the
// tile swizzle, 16-byte streaming loads), so that "achievable" can be set beside the published
// peak: the chip is power-limited and does not hold its 2.4 GHz peak clock under matrix load.
//
//   int prism_peaks_count(void);
//   const char* prism_peaks_name(int probe);
//   int prism_peaks_measure(int probe, int arg, double out[4]);
//       out[0] = milliseconds of one timed launch (HIP events on the null stream)
//       out[1] = work of that launch (flop for the MFMA probes, bytes for the LDS / stream probes,
//                instructions for the VALU probes)
//       out[2] = shader clock in MHz seen by workgroup 0 (cycle counter / 100 MHz wall counter)
//       out[3] = cycles per MFMA (or per LDS read / VALU instruction) of one wave of workgroup 0
//     arg: workgroups per CU (1 or 2) for the on-chip probes, footprint in MiB for the stream probe.
//   Returns 0, or -1 on a HIP error / bad argument.  Allocates its own buffers and synchronises.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum Probe {
  kMfmaOnly = 0,        // 4 independent accumulators, operands in registers
  kMfmaLds1to1,         // one 16-byte LDS operand read per MFMA (a wave of 32 queries)
  kMfmaLds1to2,         // one LDS operand read per two MFMAs (a wave of 64 queries)
  kLdsReadOnly,         // the operand reads alone
  kValuFma,             // dependent-free v_fma_f32 stream
  kValuExp,             // v_exp_f32 stream
  kMfmaValuSameWave,    // per MFMA: 4 v_fma_f32 + 1 v_exp_f32 of the same wave in its shadow
  kStreamRead,          // 16-byte loads over a footprint of `arg` MiB, read again and again
  kProbeCount
};

const char* const kNames[kProbeCount] = {
    "mfma_32x32x16_bf16_only", "mfma_plus_lds_read_1_to_1", "mfma_plus_lds_read_1_to_2",
    "lds_read_b128_only", "valu_fma_f32", "valu_exp_f32", "mfma_plus_4fma_1exp_same_wave",
    "stream_read_16B"};

constexpr int kItersPerLaunch = 4000;      // outer iterations of the on-chip probes
constexpr int kSlots = 32;                 // MFMA slots per outer iteration

// One workgroup = 4 waves.  LDS holds two 32 KB tiles laid out like the attention kernel's K tile
// (rows of 256 bytes, 16-byte pieces XOR-swizzled by row), so the reads are conflict-free.
template <int PROBE>
__global__ __launch_bounds__(256) void onchip_kernel(float* out, long long* clk, int iters) {
  __shared__ __attribute__((aligned(16))) char lds[65536];
  for (int i = threadIdx.x; i < 65536 / 2; i += 256)
    reinterpret_cast<__bf16*>(lds)[i] = (__bf16)(0.01f * ((i * 7) % 13 - 6));
  __syncthreads();
  const int lane = threadIdx.x & 63, l32 = lane & 31, hf = lane >> 5;
  int off[8];
#pragma unroll
  for (int st = 0; st < 8; ++st) off[st] = l32 * 256 + (((2 * st + hf) ^ (l32 & 15)) << 4);
  bf16x8 q[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) q[i][j] = (__bf16)(0.02f * ((lane + i + j) % 5));
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  float x[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) x[j] = 0.001f * lane + 0.1f * j;

  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
    const char* base = lds + (it & 1) * 32768;
    if (PROBE == kMfmaOnly) {
#pragma unroll
      for (int i = 0; i < kSlots; ++i)
        acc[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[i % 8], q[(i + 3) % 8], acc[i % 4], 0, 0, 0);
    } else if (PROBE == kMfmaLds1to1 || PROBE == kMfmaLds1to2 || PROBE == kLdsReadOnly) {
      constexpr int kPer = PROBE == kMfmaLds1to2 ? 2 : 1;      // MFMAs fed by one read
      constexpr int kReads = kSlots / kPer;
      constexpr int kDepth = 8;                                  // reads in flight
      bf16x8 fr[kDepth];
#pragma unroll
      for (int i = 0; i < kDepth; ++i)
        fr[i] = *reinterpret_cast<const bf16x8*>(base + (i % 4) * 8192 + off[(i / 4) % 8]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < kReads; ++i) {
        if (PROBE != kLdsReadOnly) {
#pragma unroll
          for (int m = 0; m < kPer; ++m)
            acc[(i * kPer + m) % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                fr[i % kDepth], q[(i + m) % 8], acc[(i * kPer + m) % 4], 0, 0, 0);
        } else {
          x[i % 16] += (float)fr[i % kDepth][0];
        }
        if (i + kDepth < kReads) {
          const int j = i + kDepth;
          fr[i % kDepth] = *reinterpret_cast<const bf16x8*>(base + (j % 4) * 8192 + off[(j / 4) % 8]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (PROBE == kValuFma) {
#pragma unroll
      for (int i = 0; i < kSlots * 4; ++i) x[i % 16] = fmaf(x[i % 16], 1.0001f, 0.5f);
    } else if (PROBE == kValuExp) {
#pragma unroll
      for (int i = 0; i < kSlots * 4; ++i) x[i % 16] = __builtin_amdgcn_exp2f(x[i % 16]);
    } else if (PROBE == kMfmaValuSameWave) {
#pragma unroll
      for (int i = 0; i < kSlots; ++i) {
        acc[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q[i % 8], q[(i + 3) % 8], acc[i % 4], 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) x[(i * 5 + j) % 16] = fmaf(x[(i * 5 + j) % 16], 1.0001f, 0.5f);
        x[(i * 5 + 4) % 16] = __builtin_amdgcn_exp2f(x[(i * 5 + 4) % 16]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  if (threadIdx.x == 0) {
    clk[blockIdx.x * 2] = c1 - c0;
    clk[blockIdx.x * 2 + 1] = w1 - w0;
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
#pragma unroll
  for (int j = 0; j < 16; ++j) s += x[j];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Every workgroup walks the footprint in 16-byte pieces, 8 loads in flight per thread, starting at
// a different place, `passes` times.
__global__ __launch_bounds__(256) void stream_kernel(const u32x4* __restrict__ src, size_t pieces,
                                                     int passes, unsigned* out) {
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4 a = {0u, 0u, 0u, 0u};
  for (int p = 0; p < passes; ++p) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < pieces; i += 8 * stride) {
      u32x4 v[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = src[i + k * stride];
#pragma unroll
      for (int k = 0; k < 8; ++k) a ^= v[k];
    }
    for (; i < pieces; i += stride) a ^= src[i];
  }
  if ((a[0] ^ a[1] ^ a[2] ^ a[3]) == 0x12345u) out[0] = 1u;    // keeps the loads alive
}

template <int PROBE>
int run_onchip(int wgs_per_cu, int cus, double* res) {
  const int grid = cus * wgs_per_cu;
  float* out = nullptr;
  long long* clk = nullptr;
  if (hipMalloc(&out, (size_t)grid * 256 * sizeof(float)) != hipSuccess) return -1;
  if (hipMalloc(&clk, (size_t)grid * 2 * sizeof(long long)) != hipSuccess) return -1;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  hipLaunchKernelGGL(onchip_kernel<PROBE>, dim3(grid), dim3(256), 0, 0, out, clk, kItersPerLaunch / 8);   // warm-up
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(onchip_kernel<PROBE>, dim3(grid), dim3(256), 0, 0, out, clk, kItersPerLaunch);
  (void)hipEventRecord(e1, 0);
  int rc = hipEventSynchronize(e1) == hipSuccess && hipGetLastError() == hipSuccess ? 0 : -1;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  long long h[2] = {0, 1};
  (void)hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost);
  const double waves = (double)grid * 4, slots = (double)kItersPerLaunch * kSlots;
  double work = 0.0, per_wave = slots;
  if (PROBE == kMfmaOnly || PROBE == kMfmaLds1to1 || PROBE == kMfmaLds1to2 || PROBE == kMfmaValuSameWave)
    work = waves * slots * 2.0 * 32 * 32 * 16;
  else if (PROBE == kLdsReadOnly) work = waves * slots * 1024.0;
  else { work = waves * slots * 4; per_wave = slots * 4; }
  res[0] = ms;
  res[1] = work;
  res[2] = (double)h[0] / (double)h[1] * 100.0;
  res[3] = (double)h[0] / per_wave;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(out);
  (void)hipFree(clk);
  return rc;
}

int run_stream(int footprint_mib, int cus, double* res) {
  if (footprint_mib < 1 || footprint_mib > 16384) return -1;
  const size_t bytes = (size_t)footprint_mib << 20, pieces = bytes / 16;
  u32x4* src = nullptr;
  unsigned* out = nullptr;
  if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&out, 256) != hipSuccess) return -1;
  (void)hipMemset(src, 1, bytes);
  const double target = 16.0 * (1ull << 30);                     // bytes moved per timed launch
  int passes = (int)(target / (double)bytes);
  passes = passes < 1 ? 1 : passes;
  const int grid = cus * 8;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  hipLaunchKernelGGL(stream_kernel, dim3(grid), dim3(256), 0, 0, src, pieces, 1, out);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(stream_kernel, dim3(grid), dim3(256), 0, 0, src, pieces, passes, out);
  (void)hipEventRecord(e1, 0);
  int rc = hipEventSynchronize(e1) == hipSuccess && hipGetLastError() == hipSuccess ? 0 : -1;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  res[0] = ms;
  res[1] = (double)bytes * passes;
  res[2] = 0.0;
  res[3] = 0.0;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(src);
  (void)hipFree(out);
  return rc;
}

}  // namespace

extern "C" int prism_peaks_count(void) { return kProbeCount; }

extern "C" const char* prism_peaks_name(int probe) {
  return probe >= 0 && probe < kProbeCount ? kNames[probe] : "";
}

extern "C" int prism_peaks_measure(int probe, int arg, double* out) {
  if (out == nullptr) return -1;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
  const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (probe == kStreamRead) return run_stream(arg, cus, out);
  if (arg != 1 && arg != 2) return -1;
  switch (probe) {
    case kMfmaOnly: return run_onchip<kMfmaOnly>(arg, cus, out);
    case kMfmaLds1to1: return run_onchip<kMfmaLds1to1>(arg, cus, out);
    case kMfmaLds1to2: return run_onchip<kMfmaLds1to2>(arg, cus, out);
    case kLdsReadOnly: return run_onchip<kLdsReadOnly>(arg, cus, out);
    case kValuFma: return run_onchip<kValuFma>(arg, cus, out);
    case kValuExp: return run_onchip<kValuExp>(arg, cus, out);
    case kMfmaValuSameWave: return run_onchip<kMfmaValuSameWave>(arg, cus, out);
    default: return -1;
  }
}
