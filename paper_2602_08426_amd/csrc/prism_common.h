// Internal helpers shared by the libprism translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "prism.h"

namespace prism {

constexpr int kHeadDim = 128;           // the head dim of the 64-queries-per-wave attention kernel
constexpr int kMaxHeadDim = 256;        // head_dim is 64, 128 or 256
constexpr int kMaxBlocks = 2048;       // N <= 2048  (128K tokens at B = 64)
constexpr int kWave = 64;
constexpr int kMaxDevices = 64;         // GPUs of one process for which per-device host state is kept

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Validation shared by every entry point.  Returns PRISM_OK or an error code.
inline int check_params(const prism_params* p) {
  if (p == nullptr) return PRISM_ERR_INVALID_ARG;
  if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->seq_len <= 0) return PRISM_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return PRISM_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128 && p->head_dim != 256) return PRISM_ERR_UNSUPPORTED;
  if (p->block != 64 && p->block != 128) return PRISM_ERR_UNSUPPORTED;
  const int64_t n = ((int64_t)p->seq_len + p->block - 1) / p->block;   // a ragged last block is allowed
  if (n > kMaxBlocks) return PRISM_ERR_UNSUPPORTED;
  // CSR offsets are int32
  const int64_t pairs = (p->flags & PRISM_FLAG_BIDIRECTIONAL) ? (int64_t)p->n_q_heads * n * n
                                                               : (int64_t)p->n_q_heads * n * (n + 1) / 2;
  if (pairs >= (int64_t)1 << 31) return PRISM_ERR_UNSUPPORTED;
  if ((int64_t)p->n_q_heads * n + 1 >= (int64_t)1 << 31) return PRISM_ERR_UNSUPPORTED;
  return PRISM_OK;
}

// N = ceil(L / B) (Sec. 3.1, Eq. "mean-pooling": the last block holds the remaining tokens)
inline int n_blocks(const prism_params* p) { return (p->seq_len + p->block - 1) / p->block; }

inline int check_bands(const prism_params* p) {
  if (p->d_high < 0 || p->d_low < 0 || p->d_high > p->head_dim || p->d_low > p->head_dim)
    return PRISM_ERR_INVALID_ARG;
  if (p->d_high == 0 && p->d_low == 0) return PRISM_ERR_INVALID_ARG;
  if (!(p->top_p > 0.0f) || !(p->top_p <= 1.0f)) return PRISM_ERR_INVALID_ARG;   // also rejects NaN
  return PRISM_OK;
}

// Element strides between consecutive heads of the caller's tensors.  One sequence per call has
// contiguous heads (L * d); a sequence of a packed variable-length batch [heads, T, d] is addressed
// through pointers moved to its first token and the strides of the whole batch (T * d, T).
struct HeadStrides {
  size_t q;      // Q and O
  size_t kv;     // K and V
  size_t lse;    // the log-sum-exp output
};
inline HeadStrides contiguous_heads(const prism_params* p) {
  const size_t s = (size_t)p->seq_len * p->head_dim;
  return HeadStrides{s, s, (size_t)p->seq_len};
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int launch_status() {
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_ERR_HIP;
}

// ---- device helpers -------------------------------------------------------------
// Wave-wide reductions on the DPP cross-lane paths (no LDS round trips): two quad
// permutes, half-row and row mirrors, then the row broadcasts; lane 63 ends up with the
// result, which is returned to every lane through a scalar register.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f32(float old, float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old),
                                                               __builtin_bit_cast(int, x), CTRL,
                                                               ROW_MASK, 0xF, false));
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;
constexpr int kDppRowBcast15 = 0x142;
constexpr int kDppRowBcast31 = 0x143;

__device__ __forceinline__ float wave_sum(float x) {
  x += dpp_f32<kDppQuadSwap1>(0.f, x);
  x += dpp_f32<kDppQuadSwap2>(0.f, x);
  x += dpp_f32<kDppRowHalfMirror>(0.f, x);
  x += dpp_f32<kDppRowMirror>(0.f, x);
  x += dpp_f32<kDppRowBcast15, 0xA>(0.f, x);
  x += dpp_f32<kDppRowBcast31, 0xC>(0.f, x);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
__device__ __forceinline__ float wave_max(float x) {
  x = fmaxf(x, dpp_f32<kDppQuadSwap1>(x, x));
  x = fmaxf(x, dpp_f32<kDppQuadSwap2>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowHalfMirror>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowMirror>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowBcast15, 0xA>(x, x));
  x = fmaxf(x, dpp_f32<kDppRowBcast31, 0xC>(x, x));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ int dpp_i32(int old, int x) {
  return __builtin_amdgcn_update_dpp(old, x, CTRL, ROW_MASK, 0xF, false);
}
// inclusive prefix sum over the 64 lanes on the DPP paths: shifts by 1, 2, 3 inside a row of 16 lanes
// (a window of four), then by 4 and 8 for the banks they reach, then the row broadcasts
__device__ __forceinline__ int wave_scan_inclusive(int x) {
  int s = x;
  s += dpp_i32<0x111>(0, x);                         // row_shr:1
  s += dpp_i32<0x112>(0, x);                         // row_shr:2
  s += dpp_i32<0x113>(0, x);                         // row_shr:3
  s += __builtin_amdgcn_update_dpp(0, s, 0x114, 0xF, 0xE, false);   // row_shr:4, banks 1-3
  s += __builtin_amdgcn_update_dpp(0, s, 0x118, 0xF, 0xC, false);   // row_shr:8, banks 2-3
  s += dpp_i32<kDppRowBcast15, 0xA>(0, s);
  s += dpp_i32<kDppRowBcast31, 0xC>(0, s);
  return s;
}
__device__ __forceinline__ int wave_sum(int x) {
  x += dpp_i32<kDppQuadSwap1>(0, x);
  x += dpp_i32<kDppQuadSwap2>(0, x);
  x += dpp_i32<kDppRowHalfMirror>(0, x);
  x += dpp_i32<kDppRowMirror>(0, x);
  x += dpp_i32<kDppRowBcast15, 0xA>(0, x);
  x += dpp_i32<kDppRowBcast31, 0xC>(0, x);
  return __builtin_amdgcn_readlane(x, 63);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

}  // namespace prism
