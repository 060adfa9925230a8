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
//     arg: workgroups per CU (1 or 2) for the on-chip probes, footprint in MiB for the stream probe,
//          pattern index for issue_pattern (prism_peaks_issue_patterns / _issue_pattern_name list them;
//          out[1] = pattern repetitions, out[3] = cycles per repetition for one wave per SIMD).
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
  kIssuePattern,        // `arg` = index of an instruction pattern: cycles one wave per SIMD needs per pattern
  kProbeCount
};

const char* const kNames[kProbeCount] = {
    "mfma_32x32x16_bf16_only", "mfma_plus_lds_read_1_to_1", "mfma_plus_lds_read_1_to_2",
    "lds_read_b128_only", "valu_fma_f32", "valu_exp_f32", "mfma_plus_4fma_1exp_same_wave",
    "stream_read_16B", "issue_pattern"};

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

// ---- instruction-issue patterns ------------------------------------------------------------------
// What a single wave per SIMD (the 64-queries-per-wave attention kernel's occupancy) can issue: each
// pattern is a short fixed instruction sequence on independent registers, repeated 64 times per loop
// trip in inline asm (so the order is the one written here), one workgroup of four waves per CU.
// The result is cycles per repetition of the pattern.
#define PRISM_FMA(d) "v_fma_f32 v" #d ", v120, v121, v" #d "\n"
#define PRISM_EXP(d) "v_exp_f32 v" #d ", v122\n"
#define PRISM_SALU "s_add_u32 s41, s41, 1\n"
#define PRISM_LDS(d) "ds_read_b128 v[" #d ":" #d "+3], v123\n"
#define PRISM_MFMA(a) "v_mfma_f32_32x32x16_bf16 a[" #a ":" #a "+15], v[124:127], v[124:127], a[" #a ":" #a "+15]\n"
#define PRISM_G6(a) PRISM_MFMA(a) PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103) PRISM_FMA(108) PRISM_FMA(109) PRISM_FMA(110)
#define PRISM_G7(a) PRISM_MFMA(a) PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_EXP(111) PRISM_FMA(103) PRISM_FMA(108)
#define PRISM_G8(a) PRISM_MFMA(a) PRISM_FMA(100) PRISM_FMA(101) PRISM_EXP(111) PRISM_SALU PRISM_FMA(102) PRISM_FMA(103)
#define PRISM_G9(a) PRISM_MFMA(a) PRISM_EXP(111) PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103) PRISM_FMA(108)
#define PRISM_DOT2(d) "v_dot2_f32_f16 v" #d ", v120, v121, v" #d "\n"
#define PRISM_G12(a) PRISM_MFMA(a) PRISM_FMA(100) PRISM_FMA(101) PRISM_DOT2(109) PRISM_EXP(111) PRISM_FMA(103) PRISM_FMA(108)
constexpr int kIssuePatterns = 20;
const char* const kIssueNames[kIssuePatterns] = {
    "2 x v_fma_f32",
    "v_exp_f32 + v_fma_f32",
    "v_exp_f32 + s_add_u32",
    "v_fma_f32 + s_add_u32",
    "v_exp_f32 + ds_read_b128",
    "v_fma_f32 + ds_read_b128",
    "2 x (v_mfma_32x32x16 + 7 v_fma_f32)",
    "2 x (v_mfma_32x32x16 + 5 v_fma_f32 + v_exp_f32)",
    "2 x (v_mfma_32x32x16 + 4 v_fma_f32 + v_exp_f32 + s_add_u32 right behind the exp)",
    "2 x (v_mfma_32x32x16 + v_exp_f32 right behind it + 5 v_fma_f32)",
    "2 x (v_exp_f32 + s_add_u32) + 2 v_fma_f32",
    "2 x v_exp_f32",
    "2 x (v_mfma_32x32x16 + 4 v_fma_f32 + v_dot2_f32_f16 + v_exp_f32)",
    "4 x v_fma_f32 on four registers",
    "4 x v_dot2_f32_f16 on four registers",
    "4 x v_max3_f32 on four registers",
    "4 x v_cvt_pk_f16_f32 on four registers",
    "4 x v_fma_f32 + s_waitcnt lgkmcnt(0)",
    "4 x v_fma_f32 + s_nop 0",
    "4 x v_fma_f32 + v_permlane32_swap_b32",
};

template <int PATTERN>
__global__ __launch_bounds__(256) void issue_kernel(float* out, long long* clk, int iters) {
  __shared__ __attribute__((aligned(16))) char lds[4096];
  lds[threadIdx.x * 16] = (char)threadIdx.x;
  __syncthreads();
  const int lds_off = (int)(size_t)lds + (threadIdx.x & 63) * 16;
  const long long c0 = clock64(), w0 = wall_clock64();
  asm volatile(
      "v_mov_b32 v120, 1.0\n v_mov_b32 v121, 0.5\n v_mov_b32 v122, 0.5\n v_mov_b32 v123, %1\n"
      "v_mov_b32 v124, 0\n v_mov_b32 v125, 0\n v_mov_b32 v126, 0\n v_mov_b32 v127, 0\n"
      "s_mov_b32 s40, %0\n s_mov_b32 s41, 0\n"
      "1:\n"
      ".rept 64\n"
      // the patterns; the assembler keeps only the one whose number matches
      ".if %c2 == 0\n" PRISM_FMA(100) PRISM_FMA(101) ".endif\n"
      ".if %c2 == 1\n" PRISM_EXP(100) PRISM_FMA(101) ".endif\n"
      ".if %c2 == 2\n" PRISM_EXP(100) PRISM_SALU ".endif\n"
      ".if %c2 == 3\n" PRISM_FMA(100) PRISM_SALU ".endif\n"
      ".if %c2 == 4\n" PRISM_EXP(100) PRISM_LDS(104) ".endif\n"
      ".if %c2 == 5\n" PRISM_FMA(100) PRISM_LDS(104) ".endif\n"
      // MFMA groups come in pairs on two accumulators, so consecutive MFMAs are independent
      ".if %c2 == 6\n" PRISM_G6(0) PRISM_G6(16) ".endif\n"
      ".if %c2 == 7\n" PRISM_G7(0) PRISM_G7(16) ".endif\n"
      ".if %c2 == 8\n" PRISM_G8(0) PRISM_G8(16) ".endif\n"
      ".if %c2 == 9\n" PRISM_G9(0) PRISM_G9(16) ".endif\n"
      ".if %c2 == 10\n" PRISM_EXP(100) PRISM_SALU PRISM_EXP(101) PRISM_SALU PRISM_FMA(102) PRISM_FMA(103) ".endif\n"
      ".if %c2 == 11\n" PRISM_EXP(100) PRISM_EXP(101) ".endif\n"
      ".if %c2 == 12\n" PRISM_G12(0) PRISM_G12(16) ".endif\n"
      ".if %c2 == 13\n" PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103) ".endif\n"
      ".if %c2 == 14\n" PRISM_DOT2(100) PRISM_DOT2(101) PRISM_DOT2(102) PRISM_DOT2(103) ".endif\n"
      ".if %c2 == 15\n v_max3_f32 v100, v120, v121, v100\n v_max3_f32 v101, v120, v121, v101\n"
      "v_max3_f32 v102, v120, v121, v102\n v_max3_f32 v103, v120, v121, v103\n .endif\n"
      ".if %c2 == 16\n v_cvt_pk_f16_f32 v100, v120, v121\n v_cvt_pk_f16_f32 v101, v120, v121\n"
      "v_cvt_pk_f16_f32 v102, v120, v121\n v_cvt_pk_f16_f32 v103, v120, v121\n .endif\n"
      ".if %c2 == 17\n" PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103) "s_waitcnt lgkmcnt(0)\n .endif\n"
      ".if %c2 == 18\n" PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103) "s_nop 0\n .endif\n"
      ".if %c2 == 19\n" PRISM_FMA(100) PRISM_FMA(101) PRISM_FMA(102) PRISM_FMA(103)
      "v_permlane32_swap_b32 v108, v109\n .endif\n"
      ".endr\n"
      "s_waitcnt lgkmcnt(0)\n"
      "s_sub_u32 s40, s40, 1\n s_cmp_lg_u32 s40, 0\n s_cbranch_scc1 1b\n"
      "s_nop 7\n s_nop 7\n s_nop 7\n"
      :
      : "s"(iters), "v"(lds_off), "n"(PATTERN)
      : "memory", "scc", "s40", "s41", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108",
        "v109", "v110", "v111", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "a0", "a1", "a2",
        "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", "a17", "a18", "a19",
        "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31");
  const long long c1 = clock64(), w1 = wall_clock64();
  if (threadIdx.x == 0) {
    clk[blockIdx.x * 2] = c1 - c0;
    clk[blockIdx.x * 2 + 1] = w1 - w0;
  }
  out[blockIdx.x * 256 + threadIdx.x] = 0.f;
}
#undef PRISM_FMA
#undef PRISM_EXP
#undef PRISM_SALU
#undef PRISM_LDS
#undef PRISM_MFMA
#undef PRISM_G6
#undef PRISM_G7
#undef PRISM_G8
#undef PRISM_G9
#undef PRISM_G12
#undef PRISM_DOT2

template <int PATTERN>
int run_issue(int cus, double* res) {
  constexpr int kTrips = 2000;
  float* out = nullptr;
  long long* clk = nullptr;
  if (hipMalloc(&out, (size_t)cus * 256 * sizeof(float)) != hipSuccess) return -1;
  if (hipMalloc(&clk, (size_t)cus * 2 * sizeof(long long)) != hipSuccess) return -1;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  hipLaunchKernelGGL(issue_kernel<PATTERN>, dim3(cus), dim3(256), 0, 0, out, clk, kTrips / 8);   // warm-up
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0, 0);
  hipLaunchKernelGGL(issue_kernel<PATTERN>, dim3(cus), dim3(256), 0, 0, out, clk, kTrips);
  (void)hipEventRecord(e1, 0);
  int rc = hipEventSynchronize(e1) == hipSuccess && hipGetLastError() == hipSuccess ? 0 : -1;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  long long h[2] = {0, 1};
  (void)hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost);
  res[0] = ms;
  res[1] = (double)cus * 4 * kTrips * 64;                 // pattern repetitions of the launch
  res[2] = (double)h[0] / (double)h[1] * 100.0;
  res[3] = (double)h[0] / ((double)kTrips * 64);          // cycles per repetition
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(out);
  (void)hipFree(clk);
  return rc;
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

extern "C" int prism_peaks_issue_patterns(void) { return kIssuePatterns; }

extern "C" const char* prism_peaks_issue_pattern_name(int pattern) {
  return pattern >= 0 && pattern < kIssuePatterns ? kIssueNames[pattern] : "";
}

extern "C" int prism_peaks_measure(int probe, int arg, double* out) {
  if (out == nullptr) return -1;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
  const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (probe == kStreamRead) return run_stream(arg, cus, out);
  if (probe == kIssuePattern) {
    switch (arg) {
      case 0: return run_issue<0>(cus, out);
      case 1: return run_issue<1>(cus, out);
      case 2: return run_issue<2>(cus, out);
      case 3: return run_issue<3>(cus, out);
      case 4: return run_issue<4>(cus, out);
      case 5: return run_issue<5>(cus, out);
      case 6: return run_issue<6>(cus, out);
      case 7: return run_issue<7>(cus, out);
      case 8: return run_issue<8>(cus, out);
      case 9: return run_issue<9>(cus, out);
      case 10: return run_issue<10>(cus, out);
      case 11: return run_issue<11>(cus, out);
      case 12: return run_issue<12>(cus, out);
      case 13: return run_issue<13>(cus, out);
      case 14: return run_issue<14>(cus, out);
      case 15: return run_issue<15>(cus, out);
      case 16: return run_issue<16>(cus, out);
      case 17: return run_issue<17>(cus, out);
      case 18: return run_issue<18>(cus, out);
      case 19: return run_issue<19>(cus, out);
      default: return -1;
    }
  }
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
