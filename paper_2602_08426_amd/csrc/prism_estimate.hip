// Block-importance estimation kernels of libprism (gfx950).
//
// Pipeline (Sec. 3.4 "Prism: Spectral-Aware Block Selection", App. C "Top-P Block Selection"):
//   pool_energy_kernel : mean pooling of Q and K blocks + per-block band energies   (HBM-bound)
//   scale_kernel       : RMS energies -> tau_z -> 1 / (sqrt(d_z) tau_z) per q-head
//   select_kernel      : dual-band block logits on bf16 MFMA (pooled vectors split into
//                        three bf16 terms), row softmax, top-p, union, bit rows
//   scan/fill kernels  : bit rows -> CSR index lists
#include "prism_common.h"

#include <mutex>
#include <type_traits>
#include <utility>

namespace prism {

// The two bands as maps from head dims to band positions.  A band is a list of slices of
// the head dim (Sec. 3.4: first d_high / last d_low dims; App. "HunyuanVideo Spectral
// Configuration": first / last dims of every axis subspace); its vector is the
// concatenation of the slices, zero-padded to a multiple of 32 for the MFMA k-steps.
struct BandMap {
  int16_t pos[2][kMaxHeadDim];   // position of dim c inside band z (0 = high, 1 = low), -1: not a member
  int32_t dz[2];             // dims in the band, 0 = band disabled
  int32_t dpad[2];           // dz rounded up to a multiple of 32
};

// Band vectors of all heads and blocks: [z][term], term = hi, mid, lo, each bf16.
//   q-heads (read once per strip of 16 q-blocks): [h][N][bs], plain rows of bs = max(128, d)
//   elements (band_stride below);
//   kv heads (read by every strip of the g q-heads): behind them, in the order the score GEMM
//   reads them: per head ceil(N/16) tiles of 16 blocks; per tile bs/32 k-steps of 32 band dims; per
//   (tile, k-step) the 64 lanes' 16-byte MFMA operand pieces back to back (lane =
//   16 * (dim / 8 % 4) + block % 16).  One operand fetch of a wave is then one contiguous KB
//   instead of 16 rows of 64 bytes (a fetch of 16 rows costs the address path four times as
//   long).  Blocks N .. 16*ceil(N/16)-1 of a head's last tile are zero.
struct BandVectors {
  uint16_t* v[2][3];
};
// elements per band vector: room for the widest band a head dim allows, at least four k-steps
__host__ __device__ inline int band_stride(int head_dim) { return head_dim > 128 ? head_dim : 128; }

// element offset of (kv head, block, band position) behind the q-heads' h*N*bs elements; one tile
// of 16 blocks holds 16*bs elements
__device__ __forceinline__ size_t kv_band_offset(int h, int N, int bs, int kvh, int blk, int pz) {
  const int n_tiles = (N + 15) >> 4;
  const int tile = blk >> 4, r = blk & 15, ks = pz >> 5, piece = (pz >> 3) & 3, j = pz & 7;
  return (size_t)h * N * bs + ((size_t)kvh * n_tiles + tile) * 16 * bs + ks * 512 +
         (piece * 16 + r) * 8 + j;
}

// =====================================================================================
// Mean pooling (Eq. "mean-pooling") and band energies (Sec. 3.4, RMS definition).
// One workgroup per (block, head); 256 threads read B x d bf16 = 2*B*d contiguous bytes
// as 16-byte pieces: with d/8 pieces per row, thread t owns dims 8*(t % (d/8))..+7 of rows
// t / (d/8), that + 2048/d, ...
// Outputs per (head, block): the two band vectors, each as three bf16 terms hi + mid + lo
// (together they carry the full fp32 mantissa), an optional fp32 copy of the pooled vector,
// and the three sums of squares (all dims, high band, low band) in
// energy[(head*N + block)*4 + {0,1,2}].  Heads 0..h-1 are Q heads, h..h+h_kv-1 are K heads.
// =====================================================================================
// With kRope the kernel is also the producer of the post-RoPE tensors: q / k hold the vectors
// BEFORE the rotation, every feature pair (2j, 2j+1) of token n is rotated by the angle
// (position_offset + n) * theta_j (Sec. 3.1 "Spectral Structure of RoPE"), rounded to bf16, written
// to q_out / k_out, and the rounded values are what is pooled, so the statistics are bit for bit
// those of pooling the written tensors; the separate 2*(h + h_kv)*L*d bytes read of the pooling
// pass is saved.
struct RopeArgs {
  double ln_base;           // theta_j = exp(-(2j/d) ln b)
  double yarn_scale;        // s of the NTK-by-parts map (App. "Compatibility with YaRN"); <= 0: plain RoPE
  double yarn_alpha, yarn_beta;
  double yarn_native_len;   // L of r_j = L theta_j / (2 pi)
  int position_offset;
};

// theta'_j of feature pair j: plain RoPE, or (1 - gamma_j) theta_j / s + gamma_j theta_j with
// gamma_j = clamp((r_j - alpha) / (beta - alpha), 0, 1), r_j = L theta_j / (2 pi).
__device__ __forceinline__ double rope_theta(const RopeArgs& r, int j, int d) {
  const double theta = exp(-(2.0 * j / d) * r.ln_base);
  if (!(r.yarn_scale > 0.0)) return theta;
  const double rj = r.yarn_native_len * theta * 0.15915494309189535;          // / (2 pi)
  double gamma = (rj - r.yarn_alpha) / (r.yarn_beta - r.yarn_alpha);
  gamma = gamma < 0.0 ? 0.0 : (gamma > 1.0 ? 1.0 : gamma);
  return (1.0 - gamma) * theta / r.yarn_scale + gamma * theta;
}

// cos and sin of position * theta: the product and its reduction to [-pi, pi] in fp64 (the angle
// reaches 1e5 rad at 128K tokens, far beyond what fp32 resolves), the functions in fp32.
__device__ __forceinline__ void rope_cos_sin(double angle, float* c, float* s) {
  const double n = rint(angle * 0.15915494309189535);
  const double a = fma(-n, 6.283185307179586, angle) - n * 2.4492935982947064e-16;   // 2 pi = hi + lo
  sincosf((float)a, s, c);
}

template <int BLK, bool kRope, int D>
__global__ __launch_bounds__(256) void pool_energy_kernel(
    const uint16_t* q, const uint16_t* k, int h, int L, int N, size_t q_head_stride, size_t kv_head_stride,
    BandMap map, BandVectors bv, float* __restrict__ energy,
    float* __restrict__ pooled_q_f32, float* __restrict__ pooled_k_f32,
    RopeArgs rope, uint16_t* q_out, uint16_t* k_out) {      // q_out / k_out may alias q / k
  constexpr int CPR = D / 8;                 // 16-byte pieces per token row
  constexpr int RG = 256 / CPR;              // row groups: rows rg, rg + RG, ... belong to one thread
  constexpr int ROWS = BLK / RG;             // rows per thread
  constexpr int BS = D > 128 ? D : 128;      // band_stride(D)
  __shared__ float part[RG][D + 4];
  __shared__ float esum[4][4];
  const int blk = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
  const size_t head_off = (head < h) ? (size_t)head * q_head_stride : (size_t)(head - h) * kv_head_stride;
  const uint16_t* src = ((head < h) ? q : k) + head_off + (size_t)blk * BLK * D;
  const int c = t % CPR, rg = t / CPR;

  const int cnt = min(BLK, L - blk * BLK);          // tokens in this block (ragged last block)
  uint4 v[ROWS];
#pragma unroll
  for (int it = 0; it < ROWS; ++it) {
    const int row = rg + it * RG;
    // streaming read (non-temporal): every token row is read once per call
    if (row < cnt) {
      const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (size_t)row * D + c * 8));
      v[it] = make_uint4(x[0], x[1], x[2], x[3]);
    } else {
      v[it] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
  if (kRope) {
    // This thread holds feature pairs 4c .. 4c+3 of tokens rg, rg + RG, ...: one accurate
    // cos / sin per pair for its first token, then a rotation by RG theta per further token (the
    // fp32 recurrence runs over ROWS - 1 <= 15 steps).
    uint16_t* dst = ((head < h) ? q_out : k_out) + head_off + (size_t)blk * BLK * D;
    const int pos0 = rope.position_offset + blk * BLK + rg;
    float cs[4], sn[4], dc[4], ds[4];
#pragma unroll
    for (int pj = 0; pj < 4; ++pj) {
      const double theta = rope_theta(rope, 4 * c + pj, D);
      rope_cos_sin((double)pos0 * theta, &cs[pj], &sn[pj]);
      rope_cos_sin((double)RG * theta, &dc[pj], &ds[pj]);
    }
#pragma unroll
    for (int it = 0; it < ROWS; ++it) {
      const int row = rg + it * RG;
      uint32_t w[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
#pragma unroll
      for (int pj = 0; pj < 4; ++pj) {
        const float x = __uint_as_float(w[pj] << 16), y = __uint_as_float(w[pj] & 0xFFFF0000u);
        const float xr = x * cs[pj] - y * sn[pj];
        const float yr = x * sn[pj] + y * cs[pj];
        w[pj] = float_to_bf16_bits(xr) | (float_to_bf16_bits(yr) << 16);
        const float cn = cs[pj] * dc[pj] - sn[pj] * ds[pj];
        sn[pj] = sn[pj] * dc[pj] + cs[pj] * ds[pj];
        cs[pj] = cn;
      }
      v[it] = make_uint4(w[0], w[1], w[2], w[3]);
      if (row < cnt) *reinterpret_cast<uint4*>(dst + (size_t)row * D + c * 8) = v[it];
    }
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int it = 0; it < ROWS; ++it) {
    acc[0] += __uint_as_float(v[it].x << 16);
    acc[1] += __uint_as_float(v[it].x & 0xFFFF0000u);
    acc[2] += __uint_as_float(v[it].y << 16);
    acc[3] += __uint_as_float(v[it].y & 0xFFFF0000u);
    acc[4] += __uint_as_float(v[it].z << 16);
    acc[5] += __uint_as_float(v[it].z & 0xFFFF0000u);
    acc[6] += __uint_as_float(v[it].w << 16);
    acc[7] += __uint_as_float(v[it].w & 0xFFFF0000u);
  }
  *reinterpret_cast<float4*>(&part[rg][c * 8]) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  *reinterpret_cast<float4*>(&part[rg][c * 8 + 4]) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  __syncthreads();

  if (t < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RG; ++r) s += part[r][t];
    const float mean = s / (float)cnt;
    // mean = hi + mid + lo exactly up to 2^-26 relative (three bf16 terms of 8 bits each)
    const uint32_t hi = float_to_bf16_bits(mean);
    const float rem1 = mean - bf16_bits_to_float(hi);
    const uint32_t mid = float_to_bf16_bits(rem1);
    const float rem2 = rem1 - bf16_bits_to_float(mid);
    const uint32_t lo = float_to_bf16_bits(rem2);
    const size_t o = ((size_t)head * N + blk) * D + t;
    if (head < h) {
      const size_t vec = ((size_t)head * N + blk) * BS;
#pragma unroll
      for (int z = 0; z < 2; ++z) {
        const int pz = map.pos[z][t];
        if (pz >= 0) {
          bv.v[z][0][vec + pz] = (uint16_t)hi;
          bv.v[z][1][vec + pz] = (uint16_t)mid;
          bv.v[z][2][vec + pz] = (uint16_t)lo;
        }
        if (t >= map.dz[z] && t < map.dpad[z]) {           // zero padding of the last k-step
          bv.v[z][0][vec + t] = 0;
          bv.v[z][1][vec + t] = 0;
          bv.v[z][2][vec + t] = 0;
        }
      }
    } else {
      // the workgroup of a head's last block also clears the blocks that pad the last tile
      const int blk_end = blk == N - 1 ? ((N + 15) >> 4) * 16 : blk + 1;
#pragma unroll
      for (int z = 0; z < 2; ++z) {
        const int pz = map.pos[z][t];
        if (pz >= 0) {
          const size_t e = kv_band_offset(h, N, BS, head - h, blk, pz);
          bv.v[z][0][e] = (uint16_t)hi;
          bv.v[z][1][e] = (uint16_t)mid;
          bv.v[z][2][e] = (uint16_t)lo;
        }
        for (int b = blk; b < blk_end; ++b) {
          // zero padding of the last k-step (dims dz .. dpad-1), and whole padding blocks
          if (t < map.dpad[z] && (b > blk || t >= map.dz[z])) {
            const size_t e = kv_band_offset(h, N, BS, head - h, b, t);
            bv.v[z][0][e] = 0;
            bv.v[z][1][e] = 0;
            bv.v[z][2][e] = 0;
          }
        }
      }
    }
    if (head < h) {
      if (pooled_q_f32) pooled_q_f32[o] = mean;
    } else if (pooled_k_f32) {
      pooled_k_f32[((size_t)(head - h) * N + blk) * D + t] = mean;
    }
    const float sq = mean * mean;
    const float e_full = wave_sum(sq);
    const float e_high = wave_sum(map.pos[0][t] >= 0 ? sq : 0.f);
    const float e_low = wave_sum(map.pos[1][t] >= 0 ? sq : 0.f);
    if ((t & 63) == 0) {
      esum[t >> 6][0] = e_full;
      esum[t >> 6][1] = e_high;
      esum[t >> 6][2] = e_low;
    }
  }
  __syncthreads();
  if (t < 3) {
    float e = 0.f;
#pragma unroll
    for (int wv = 0; wv < D / 64; ++wv) e += esum[wv][t];      // fixed order: deterministic
    energy[((size_t)head * N + blk) * 4 + t] = e;
  }
}

// =====================================================================================
// Energy-based temperature calibration (Sec. 3.4): per q-head
//   tau_z = sqrt(d_z/d) * RMS(Qbar_z)/RMS(Qbar) * RMS(Kbar_z)/RMS(Kbar),  scale_z = sqrt(d_z) tau_z.
// One wave per q-head sums the per-block energies in a fixed order (fp64).
// inv_scale[hq*2 + z] = 1/scale_z, or 0 when the band is disabled or has no energy.
// =====================================================================================
__global__ __launch_bounds__(64) void scale_kernel(const float* __restrict__ energy, int h, int h_kv,
                                                   int N, int head_dim, int d_high, int d_low, int calibrate,
                                                   float* __restrict__ inv_scale,
                                                   float* __restrict__ scales_out) {
  const int hq = blockIdx.x, lane = threadIdx.x;
  const int kvh = h + hq / (h / h_kv);
  double eq[3] = {0, 0, 0}, ek[3] = {0, 0, 0};
  // one 16-byte load per (head, block); several blocks in flight (the sums keep their order)
#pragma unroll 4
  for (int i = lane; i < N; i += 64) {
    const float4 a = *reinterpret_cast<const float4*>(energy + ((size_t)hq * N + i) * 4);
    const float4 b = *reinterpret_cast<const float4*>(energy + ((size_t)kvh * N + i) * 4);
    eq[0] += (double)a.x;
    eq[1] += (double)a.y;
    eq[2] += (double)a.z;
    ek[0] += (double)b.x;
    ek[1] += (double)b.y;
    ek[2] += (double)b.z;
  }
#pragma unroll
  for (int z = 0; z < 3; ++z) {
    eq[z] = wave_sum(eq[z]);
    ek[z] = wave_sum(ek[z]);
  }
  if (lane == 0) {
    const double d = head_dim;
    const double rq = sqrt(eq[0] / (N * d)), rk = sqrt(ek[0] / (N * d));
    for (int z = 0; z < 2; ++z) {
      const int dz = z == 0 ? d_high : d_low;
      double scale = 0.0;
      if (dz > 0) {
        if (calibrate) {
          const double rqz = sqrt(eq[z + 1] / (N * (double)dz));
          const double rkz = sqrt(ek[z + 1] / (N * (double)dz));
          const double tau = sqrt(dz / d) * (rqz / rq) * (rkz / rk);
          scale = sqrt((double)dz) * tau;
        } else {
          scale = sqrt((double)dz);
        }
      }
      const bool ok = isfinite(scale) && scale > 0.0;
      inv_scale[hq * 2 + z] = ok ? (float)(1.0 / scale) : 0.f;
      if (scales_out) scales_out[hq * 2 + z] = ok ? (float)scale : 0.f;
    }
  }
}

// =====================================================================================
// Dual-band scoring, softmax, top-p, union (Sec. 3.4 steps 4-5, App. C).
//
// One workgroup (4 waves) per (strip of 16 q-blocks, q-head).  Per band:
//   phase A: logits[16][v <= u_max] = Qbar_z Kbar_z^T * inv_scale on
//            v_mfma_f32_16x16x32_bf16, with x = hi + mid + lo (three bf16 terms) and the
//            six products of weight >= 2^-16 (fp32 accumulate), written to LDS;
//   phase B: one wave per row: lanes hold the row (column i*64 + lane in register i),
//            softmax numerators e = exp(l - max), then the selection threshold is found
//            by bisection on the bit pattern of e: the smallest key T* whose strictly
//            larger elements carry mass < p * sum(e).  Elements above T* are selected;
//            elements equal to T* are taken in ascending block order while the mass before
//            them stays < p * sum(e)  (== minimal descending prefix with exclusive
//            cumulative mass < p, stable order).
// Bits of both bands are OR-ed in registers (lane i keeps word i of the row).
// DUMP = true writes the logits to global memory instead of selecting.
// =====================================================================================
constexpr int kStripRows = 16;

// Top-p selection of the four consecutive rows of one band that a wave owns.  Row k has
// n0 + k*nstep logits (nstep = 1: block-causal rows, 0: every row sees all N blocks); each row lives in registers: column
// 64*i + lane in e[k][i].  The four rows are advanced together so that their wave reductions
// (dependent DPP chains) overlap.  Selected bits are OR-ed into the rows' LDS bit words.
// rows per wave: 4 (workgroup of 4 waves) or 2 (8 waves: twice the waves in flight for the same LDS strip)

// lane I of (lo, hi) := the wave-uniform 64-bit word w.  Two lane writes with the lane number as an
// immediate: no per-lane predicate has to be formed or kept.  The s_nop gives the compare that wrote w
// its two wait states before a vector instruction reads the mask as a scalar source.
template <int I>
__device__ __forceinline__ void put_word(uint64_t w, int& lo, int& hi) {
  const int wl = (int)(uint32_t)w, wh = (int)(uint32_t)(w >> 32);
  asm("s_nop 1\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
      : "+v"(lo), "+v"(hi)
      : "s"(wl), "s"(wh), "n"(I));
}

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int NCH, int kRowsPerWave>
__device__ __forceinline__ void select_rows(const float* __restrict__ logits, int ld, int n0, int nstep,
                                            int nrows, float top_p, int lane,
                                            uint64_t* __restrict__ bits, int bits_ld) {
  float e[kRowsPerWave][NCH];
  float total[kRowsPerWave], target[kRowsPerWave];
#pragma unroll
  for (int k = 0; k < kRowsPerWave; ++k) {
    const int n = k < nrows ? n0 + k * nstep : 0;
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int idx = i * 64 + lane;
      e[k][i] = idx < n ? logits[k * ld + idx] : -INFINITY;
      mx = fmaxf(mx, e[k][i]);
    }
    mx = wave_max(mx);
    mx = mx == -INFINITY ? 0.f : mx;                 // a row without columns
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      e[k][i] = __expf(e[k][i] - mx);                // softmax numerators, max one = 1; columns past the end: exp(-inf) = 0
      part += e[k][i];
    }
    total[k] = wave_sum(part);
    target[k] = top_p * total[k];
  }
  const bool all = top_p >= 1.0f;

  uint32_t tstar[kRowsPerWave];                      // T* (rows with equal elements at the cut), else T
  float gstar[kRowsPerWave];
  bool one_tie[kRowsPerWave];                        // exactly one element has the key T*
#pragma unroll
  for (int k = 0; k < kRowsPerWave; ++k) {
    tstar[k] = 0;
    gstar[k] = 0.f;
    one_tie[k] = false;
  }
  if (!all) {
    // per row: largest key T with mass{key > T} >= target; T* = T + 1 is then the smallest key
    // whose strictly-larger mass is < target (and T* is some element's key).  Keys are bit
    // patterns of values in [0, 1], i.e. <= 0x3F800000: bit 30 is never set.
    // The search is a bisection on the key bits.  Beside the mass above a candidate it counts
    // the elements above it, which tells how many elements are left between the bounds: at
    // bit b the answer lies in [T, T + 2^(b+1) - 1], n_lo elements are above T and n_hi above
    // T + 2^(b+1).  When n_lo - n_hi = 1 the one element in between is T* and the search of
    // that row stops (typically after 12-16 of the 30 bits; rows whose cut falls among equal
    // elements run to the last bit).
    uint32_t T[kRowsPerWave];
    int n_lo[kRowsPerWave], n_hi[kRowsPerWave];
    float g_hi[kRowsPerWave];
    bool open[kRowsPerWave];
#pragma unroll
    for (int k = 0; k < kRowsPerWave; ++k) {
      T[k] = 0;
      n_hi[k] = 0;
      g_hi[k] = 0.f;
      // Elements above key 0: the row's length when it is 0 or 1 (its one element is exp(0) = 1).  Longer
      // rows get their count from the fixed-key passes below, or are counted when those do not settle it.
      n_lo[k] = k < nrows ? n0 + k * nstep : 0;
      open[k] = n_lo[k] > 1;
    }
    // The cut of a row lies within a few octaves of its largest element (= 1): two passes at fixed
    // keys stand for the first four or five of the search.  The mass above a key does not grow with
    // the key, so a row that passes at 0x3C000000 (2^-7) has passed at 0x20000000, 0x30000000 and
    // 0x38000000 as well, and its state is the one after bits 29..26; a row that fails there but
    // passes at 0x38000000 (2^-15) is in the state after bits 29..27 set and bit 26 refused.  Both go
    // on at bit 25.  If some row of the wave fails at 2^-15 too, the search starts at bit 29 as usual.
    int first_bit = 29;
    {
      constexpr uint32_t kKeyA = 0x3C000000u, kKeyB = 0x38000000u;
      float gA[kRowsPerWave], gB[kRowsPerWave];
      int nA[kRowsPerWave], nB[kRowsPerWave];
      bool passA[kRowsPerWave];
      bool anyB = false;
#pragma unroll
      for (int k = 0; k < kRowsPerWave; ++k) {
        float gp = 0.f;
        nA[k] = 0;
        if (open[k]) {
#pragma unroll
          for (int i = 0; i < NCH; ++i) {
            const bool above = __float_as_uint(e[k][i]) > kKeyA;
            gp += above ? e[k][i] : 0.f;
            nA[k] += __popcll(__builtin_amdgcn_ballot_w64(above));
          }
        }
        gA[k] = gp;
      }
#pragma unroll
      for (int k = 0; k < kRowsPerWave; ++k) {
        passA[k] = true;
        if (open[k]) {
          gA[k] = wave_sum(gA[k]);
          passA[k] = !(gA[k] < target[k]);
          anyB = anyB || !passA[k];
        }
      }
      bool all_ok = true;
      if (anyB) {                                     // uniform
#pragma unroll
        for (int k = 0; k < kRowsPerWave; ++k) {
          float gp = 0.f;
          nB[k] = 0;
          if (open[k] && !passA[k]) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
              const bool above = __float_as_uint(e[k][i]) > kKeyB;
              gp += above ? e[k][i] : 0.f;
              nB[k] += __popcll(__builtin_amdgcn_ballot_w64(above));
            }
          }
          gB[k] = gp;
        }
#pragma unroll
        for (int k = 0; k < kRowsPerWave; ++k)
          if (open[k] && !passA[k]) all_ok = all_ok && !(wave_sum(gB[k]) < target[k]);
      }
      if (all_ok) {
#pragma unroll
        for (int k = 0; k < kRowsPerWave; ++k) {
          if (open[k]) {
            if (passA[k]) {
              T[k] = kKeyA;
              n_lo[k] = nA[k];
            } else {
              T[k] = kKeyB;
              n_lo[k] = nB[k];
              n_hi[k] = nA[k];
              g_hi[k] = gA[k];
            }
            open[k] = n_lo[k] - n_hi[k] > 1;
          }
        }
        first_bit = 25;
      } else {
#pragma unroll
        for (int k = 0; k < kRowsPerWave; ++k) {
          if (open[k]) {
            int n = 0;
#pragma unroll
            for (int i = 0; i < NCH; ++i) n += __popcll(__builtin_amdgcn_ballot_w64(__float_as_uint(e[k][i]) > 0u));
            n_lo[k] = n;
            open[k] = n > 1;
          }
        }
      }
    }
    for (int bit = first_bit; bit >= 0; --bit) {
      bool any_open = false;
#pragma unroll
      for (int k = 0; k < kRowsPerWave; ++k) any_open |= open[k];
      if (!any_open) break;
      float gp[kRowsPerWave];
      int np[kRowsPerWave];
#pragma unroll
      for (int k = 0; k < kRowsPerWave; ++k) {
        gp[k] = 0.f;
        np[k] = 0;
        if (open[k]) {
          const uint32_t cand = T[k] | (1u << bit);
#pragma unroll
          for (int i = 0; i < NCH; ++i) {
            const bool above = __float_as_uint(e[k][i]) > cand;
            gp[k] += above ? e[k][i] : 0.f;
            np[k] += __popcll(__builtin_amdgcn_ballot_w64(above));
          }
        }
      }
#pragma unroll
      for (int k = 0; k < kRowsPerWave; ++k) {
        if (open[k]) {
          const float g = wave_sum(gp[k]);
          if (!(g < target[k])) {
            T[k] |= (1u << bit);
            n_lo[k] = np[k];
          } else {
            n_hi[k] = np[k];
            g_hi[k] = g;
          }
          open[k] = n_lo[k] - n_hi[k] > 1;
        }
      }
    }
#pragma unroll
    for (int k = 0; k < kRowsPerWave; ++k) {
      if (n_lo[k] - n_hi[k] == 1) {
        // One element lies above T and not above the upper bound: it is T*, the mass above it (g_hi) is
        // below the target, so it is selected, and with it exactly the elements above T.
        tstar[k] = T[k];
        one_tie[k] = true;
      } else {
        // the search ran to the last bit (equal elements at the cut), or the row is empty
        tstar[k] = T[k] + 1;
        float gp = 0.f;
#pragma unroll
        for (int i = 0; i < NCH; ++i) gp += (__float_as_uint(e[k][i]) > tstar[k]) ? e[k][i] : 0.f;
        gstar[k] = wave_sum(gp);
      }
    }
  }
  // elements above T* are selected; elements equal to T* in ascending block order while the
  // mass before them stays < target (stable descending order, exclusive cumulative mass < p).
  // Lane i collects word i of the row's bits (columns 64*i .. 64*i + 63) and ORs it into LDS.
#pragma unroll
  for (int k = 0; k < kRowsPerWave; ++k) {
    if (k >= nrows) break;
    const int n = n0 + k * nstep;
    int word_lo = 0, word_hi = 0;
    if (all) {
      static_for<NCH>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const uint64_t bal = __builtin_amdgcn_ballot_w64(i * 64 + lane < n);
        put_word<i>(bal, word_lo, word_hi);
      });
    } else if (one_tie[k]) {
      // everything above T (columns past the row's end hold 0)
      static_for<NCH>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const uint64_t bal = __builtin_amdgcn_ballot_w64(__float_as_uint(e[k][i]) > tstar[k]);
        put_word<i>(bal, word_lo, word_hi);
      });
    } else {
      const float tie_val = __uint_as_float(tstar[k]);
      int tie_base = 0;
      static_for<NCH>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        const uint32_t key = __float_as_uint(e[k][i]);
        const bool tie = key == tstar[k];
        const uint64_t tb = __builtin_amdgcn_ballot_w64(tie);
        const int rank = tie_base + __popcll(tb & ((1ull << lane) - 1ull));
        const bool sel = (key > tstar[k]) || (tie && (gstar[k] + (float)rank * tie_val < target[k]));
        tie_base += __popcll(tb);
        const uint64_t bal = __builtin_amdgcn_ballot_w64(sel);
        put_word<i>(bal, word_lo, word_hi);
      });
    }
    if (lane < NCH)
      bits[k * bits_ld + lane] |= ((uint64_t)(uint32_t)word_hi << 32) | (uint64_t)(uint32_t)word_lo;
  }
}

// Measurement builds only (python -m paper_2602_08426_amd.build --ablation "select_..." out.so): parts of
// select_kernel left out to see what they cost.  Grid, LDS and control flow stay as they are, the masks
// are wrong by construction.  The conditions are written against a run-time value (top_p is at most 1)
// so that the code around the part left out is not optimised away with it.
#ifndef PRISM_SELECT_ABLATION
#define PRISM_SELECT_ABLATION 0
#endif
constexpr bool kAblNoScores = (PRISM_SELECT_ABLATION & 1) != 0;      // no score MFMAs, no LDS strip
constexpr bool kAblNoSearch = (PRISM_SELECT_ABLATION & 2) != 0;      // no softmax / top-p search
constexpr bool kAblNoRefetch = (PRISM_SELECT_ABLATION & 4) != 0;     // pooled-K fragments fetched for a wave's first tile only

// select_flags
constexpr int kSelCausal = 1;          // key blocks v > u are excluded (block-causal estimation)
constexpr int kSelForceDiagonal = 2;   // block u of every row is switched on after the union
constexpr int kSelForceSink = 4;       // block 0 of every row is switched on after the union

template <int MAXCH, bool DUMP, int kRowsPerWave>
__global__ __launch_bounds__(kStripRows / kRowsPerWave * 64) void select_kernel(
    BandVectors bv, const float* __restrict__ inv_scale, int h, int h_kv,
    int N, int bs, int dpad_high, int dpad_low, float top_p, int select_flags,
    uint64_t* __restrict__ mask_bits, int32_t* __restrict__ row_ptr,
    float* __restrict__ logits_high, float* __restrict__ logits_low) {
  constexpr int kWaves = kStripRows / kRowsPerWave, kThreads = kWaves * 64;
  extern __shared__ float lds_logits[];
  __shared__ uint64_t lds_bits[kStripRows][kMaxBlocks / 64];
  // heavy strips (large u) first
  const int strip = gridDim.x - 1 - blockIdx.x, hq = blockIdx.y;
  const int kvh = h + hq / (h / h_kv);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: scalar branches below
  const int u0 = strip * kStripRows;
  const bool causal = (select_flags & kSelCausal) != 0;
  const int ncols = causal ? min(N, u0 + kStripRows) : N;
  const int ntiles = (ncols + 15) >> 4;
  const int ld = ntiles * 16 + 4;
  const int W = (N + 63) >> 6;

  if (!DUMP) {
    for (int i = threadIdx.x; i < kStripRows * (kMaxBlocks / 64); i += kThreads)
      (&lds_bits[0][0])[i] = 0ull;
  }

#pragma unroll 1
  for (int z = 0; z < 2; ++z) {
    const int dz = z == 0 ? dpad_high : dpad_low;
    if (dz == 0) continue;                         // uniform: same for the whole grid
    const int ksteps = dz >> 5;
    const float inv = inv_scale[hq * 2 + z];
    const uint16_t* __restrict__ pooled_hi = bv.v[z][0];
    const uint16_t* __restrict__ pooled_mid = bv.v[z][1];
    const uint16_t* __restrict__ pooled_lo = bv.v[z][2];

    // ---------------- phase A: logits of the strip into LDS ----------------
    // Four k-steps (128 band dims) per pass; a wider band (head dim 256) takes a second pass that
    // adds to the logits of the first.  A wave meets the same tiles, and a lane the same LDS
    // words, in every pass, so the passes need no barrier between them.
#pragma unroll 1
    for (int k0 = 0; k0 < ksteps; k0 += 4) {
      const int kn = min(4, ksteps - k0);
      const bool first = k0 == 0, last = k0 + 4 >= ksteps;
      const int arow = min(u0 + (lane & 15), N - 1);
      const size_t aoff = ((size_t)hq * N + arow) * bs + k0 * 32 + (lane >> 4) * 8;
      const size_t tile0 = kv_band_offset(h, N, bs, kvh - h, 0, 0) + k0 * 512 + lane * 8;   // this lane's piece of tile 0
      const size_t tile_stride = (size_t)16 * bs;
      // The pass with the number of k-steps and "first pass" as compile-time facts: a fixed number of
      // loads per tile lets the compiler wait for exactly the fragments of the tile whose MFMAs come next
      // while those of the tile after it stay in flight.  The B fragments alternate between two register
      // sets; past the wave's last tile the last tile is fetched once more and not used.
      auto score_pass = [&](auto kn_tag, auto first_tag) __attribute__((always_inline)) {
        constexpr int KN = decltype(kn_tag)::value;
        constexpr bool FIRST = decltype(first_tag)::value;
        struct Frag {
          bf16x8 h[KN], m[KN], l[KN];
        };
        Frag a;
#pragma unroll
        for (int ks = 0; ks < KN; ++ks) {
          a.h[ks] = *reinterpret_cast<const bf16x8*>(pooled_hi + aoff + ks * 32);
          a.m[ks] = *reinterpret_cast<const bf16x8*>(pooled_mid + aoff + ks * 32);
          a.l[ks] = *reinterpret_cast<const bf16x8*>(pooled_lo + aoff + ks * 32);
        }
        auto load_b = [&](Frag& f, int ct) __attribute__((always_inline)) {
          const size_t boff = tile0 + (size_t)min(ct, ntiles - 1) * tile_stride;
#pragma unroll
          for (int ks = 0; ks < KN; ++ks) {
            f.h[ks] = *reinterpret_cast<const bf16x8*>(pooled_hi + boff + ks * 512);
            f.m[ks] = *reinterpret_cast<const bf16x8*>(pooled_mid + boff + ks * 512);
            f.l[ks] = *reinterpret_cast<const bf16x8*>(pooled_lo + boff + ks * 512);
          }
        };
        auto tile = [&](const Frag& c, int ct) __attribute__((always_inline)) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KN; ++ks) {
            // all cross terms down to 2^-24 relative, smallest first
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.l[ks], c.h[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.h[ks], c.l[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.m[ks], c.m[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.m[ks], c.h[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.h[ks], c.m[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.h[ks], c.h[ks], acc, 0, 0, 0);
          }
          const int col = ct * 16 + (lane & 15);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = (lane >> 4) * 4 + r;
            float lg = acc[r] * inv;
            if (!FIRST) lg += lds_logits[row * ld + col];
            lds_logits[row * ld + col] = lg;
            if (DUMP && last) {
              const int u = u0 + row;
              float* dst = z == 0 ? logits_high : logits_low;
              if (dst != nullptr && u < N && col < N && (col <= u || !causal))
                dst[((size_t)hq * N + u) * N + col] = lg;
            }
          }
        };
        const bool refetch = !kAblNoRefetch || top_p > 5.f;
        Frag b0, b1;
        load_b(b0, wave);
        if (!refetch) load_b(b1, wave);
        // (the scheduling barriers keep the fetches of the next tile in front of the MFMAs of this one;
        // left to itself the scheduler sinks them to their first use to save registers)
        for (int ct = wave; ct < ntiles; ct += 2 * kWaves) {
          if (refetch) load_b(b1, ct + kWaves);
          __builtin_amdgcn_sched_barrier(0);
          tile(b0, ct);
          __builtin_amdgcn_sched_barrier(0);
          if (ct + kWaves < ntiles) {
            if (refetch) load_b(b0, ct + 2 * kWaves);
            __builtin_amdgcn_sched_barrier(0);
            tile(b1, ct + kWaves);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      };
      if (wave < ntiles && (!kAblNoScores || top_p > 5.f)) {
        auto pass = [&](auto kn_tag) __attribute__((always_inline)) {
          if (first) score_pass(kn_tag, std::true_type{});
          else score_pass(kn_tag, std::false_type{});
        };
        switch (kn) {                                  // uniform
          case 1: pass(std::integral_constant<int, 1>{}); break;
          case 2: pass(std::integral_constant<int, 2>{}); break;
          case 3: pass(std::integral_constant<int, 3>{}); break;
          default: pass(std::integral_constant<int, 4>{}); break;
        }
      }
    }
    __syncthreads();

    // ---------------- phase B: each wave selects its four rows ----------------
    if (!DUMP) {
      const int r0 = wave * kRowsPerWave;
      const int nrows = min(kRowsPerWave, N - (u0 + r0));          // uniform per wave, may be <= 0
      if (nrows > 0 && (!kAblNoSearch || top_p > 5.f)) {
        int n0 = causal ? u0 + r0 + 1 : N;                         // columns of the first row
        // opaque to the optimiser: the per-column "inside the row" predicates are then formed where they
        // are used, in each band, instead of being kept as 64 lane masks across both bands
        asm volatile("" : "+s"(n0));
        const int nstep = causal ? 1 : 0;
        const int nmax = n0 + (nrows - 1) * nstep;
        const float* lg = lds_logits + r0 * ld;
        uint64_t* bits = &lds_bits[r0][0];
        constexpr int bld = kMaxBlocks / 64;
        if (nmax <= 128) select_rows<2, kRowsPerWave>(lg, ld, n0, nstep, nrows, top_p, lane, bits, bld);
        else if (nmax <= 256) select_rows<4, kRowsPerWave>(lg, ld, n0, nstep, nrows, top_p, lane, bits, bld);
        else if (nmax <= 512) select_rows<8, kRowsPerWave>(lg, ld, n0, nstep, nrows, top_p, lane, bits, bld);
        else if (MAXCH <= 16 || nmax <= 1024) select_rows<16, kRowsPerWave>(lg, ld, n0, nstep, nrows, top_p, lane, bits, bld);
        else select_rows<MAXCH, kRowsPerWave>(lg, ld, n0, nstep, nrows, top_p, lane, bits, bld);
      }
      __syncthreads();                             // LDS logits are reused by the next band
    }
  }

  if (!DUMP) {
#pragma unroll 1
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
      const int r = wave * kRowsPerWave + rr;
      const int u = u0 + r;
      if (u >= N) break;
      const size_t row = (size_t)hq * N + u;
      uint64_t word = lane < W ? lds_bits[r][lane] : 0ull;
      if ((select_flags & kSelForceDiagonal) && lane == (u >> 6)) word |= 1ull << (u & 63);
      if ((select_flags & kSelForceSink) && lane == 0) word |= 1ull;
      const int cnt = wave_sum((int)__popcll(word));
      if (lane < W) mask_bits[row * W + lane] = word;
      if (lane == 0) row_ptr[row + 1] = cnt;
    }
  }
}

// =====================================================================================
// Bit rows -> CSR
// =====================================================================================
__global__ __launch_bounds__(256) void row_count_kernel(const uint64_t* __restrict__ mask_bits,
                                                        int R, int W, int32_t* __restrict__ row_ptr) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= R) return;
  int c = 0;
  for (int i = 0; i < W; ++i) c += __popcll(mask_bits[(size_t)r * W + i]);
  row_ptr[r + 1] = c;
}

// In-place: row_ptr[r+1] holds the count of row r on entry, the inclusive prefix sum on
// exit; row_ptr[0] = 0.  Single workgroup of 1024 threads; a chunk is 4096 counts, 4 consecutive ones
// per thread, so loads and stores are coalesced.
// Up to 16 chunks (65536 rows): every count is requested at once and held in registers, each wave scans
// its part of every chunk, wave 0 scans the 16 x NC wave totals, and every thread adds the base of its
// (chunk, wave): two barriers and one memory round trip in all.
template <int NC>
__device__ __forceinline__ void scan_resident(int32_t* __restrict__ row_ptr, int R, int64_t capacity,
                                              int32_t* __restrict__ info, int* tot, int* base) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int v[NC][4], inc[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = c * 4096 + t * 4 + k;
      v[c][k] = i < R ? row_ptr[1 + i] : 0;
    }
  }
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    v[c][1] += v[c][0];
    v[c][2] += v[c][1];
    v[c][3] += v[c][2];
    inc[c] = wave_scan_inclusive(v[c][3]);
    if (lane == 63) tot[c * 16 + wave] = inc[c];
  }
  __syncthreads();
  if (wave == 0) {
    // lane l owns the totals 4l .. 4l + 3 of the (chunk, wave) order
    int a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = lane * 4 + j < NC * 16 ? tot[lane * 4 + j] : 0;
    a[1] += a[0];
    a[2] += a[1];
    a[3] += a[2];
    const int incl = wave_scan_inclusive(a[3]);
    const int before = incl - a[3];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane * 4 + j < NC * 16) base[lane * 4 + j] = before + (j > 0 ? a[j - 1] : 0);
    if (lane == 63) {
      row_ptr[0] = 0;
      info[0] = incl;
      info[1] = ((int64_t)incl > capacity) ? 1 : 0;
      info[2] = 0;
      info[3] = 0;
    }
  }
  __syncthreads();
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int before = base[c * 16 + wave] + inc[c] - v[c][3];   // everything ahead of this thread's 4 counts
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = c * 4096 + t * 4 + k;
      if (i < R) row_ptr[1 + i] = before + v[c][k];
    }
  }
}

__global__ __launch_bounds__(1024) void scan_kernel(int32_t* __restrict__ row_ptr, int R,
                                                    int64_t capacity, int32_t* __restrict__ info) {
  __shared__ int wave_tot[2][16 * 16];
  const int chunks = (R + 4095) / 4096;              // uniform
  if (chunks <= 16) {
    if (chunks <= 1) scan_resident<1>(row_ptr, R, capacity, info, wave_tot[0], wave_tot[1]);
    else if (chunks <= 2) scan_resident<2>(row_ptr, R, capacity, info, wave_tot[0], wave_tot[1]);
    else if (chunks <= 4) scan_resident<4>(row_ptr, R, capacity, info, wave_tot[0], wave_tot[1]);
    else if (chunks <= 8) scan_resident<8>(row_ptr, R, capacity, info, wave_tot[0], wave_tot[1]);
    else scan_resident<16>(row_ptr, R, capacity, info, wave_tot[0], wave_tot[1]);
    return;
  }
  // more rows than that: sweep chunk by chunk
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int carry = 0;
  // the counts of the next chunk are requested before the current one is scanned, so a chunk costs
  // one scan and not one memory round trip
  int nxt[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) nxt[k] = (t * 4 + k < R) ? row_ptr[1 + t * 4 + k] : 0;
  int buf = 0;
  for (int base = 0; base < R; base += 4096, buf ^= 1) {
    const int i0 = base + t * 4;
    int v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = nxt[k];
    if (base + 4096 < R) {
#pragma unroll
      for (int k = 0; k < 4; ++k) nxt[k] = (i0 + 4096 + k < R) ? row_ptr[1 + i0 + 4096 + k] : 0;
    }
    v[1] += v[0];
    v[2] += v[1];
    v[3] += v[2];
    const int inc = wave_scan_inclusive(v[3]);
    if (lane == 63) wave_tot[buf][wave] = inc;
    __syncthreads();                               // the other buffer is free: its readers passed this barrier a chunk ago
    int before = carry + inc - v[3];               // everything ahead of this thread's 4 counts
    int chunk_total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int wt = wave_tot[buf][w];
      if (w < wave) before += wt;
      chunk_total += wt;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (i0 + k < R) row_ptr[1 + i0 + k] = before + v[k];
    carry += chunk_total;
  }
  if (t == 0) {
    row_ptr[0] = 0;
    info[0] = carry;
    info[1] = ((int64_t)carry > capacity) ? 1 : 0;
    info[2] = 0;
    info[3] = 0;
  }
}

// One wave per row: ascending columns of the set bits.  Lane i fetches word i of the row (one
// request for the whole row; W <= 32), the words are then taken from registers.
__global__ __launch_bounds__(256) void fill_kernel(const uint64_t* __restrict__ mask_bits, int R,
                                                   int W, const int32_t* __restrict__ row_ptr,
                                                   int32_t* __restrict__ col_idx, int64_t capacity) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (r >= R) return;
  int64_t base = row_ptr[r];
  const uint64_t mine = lane < W ? mask_bits[(size_t)r * W + lane] : 0ull;
  const int lo = (int)(uint32_t)mine, hi = (int)(uint32_t)(mine >> 32);
  for (int i = 0; i < W; ++i) {
    const uint64_t word = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(hi, i) << 32) |
                          (uint64_t)(uint32_t)__builtin_amdgcn_readlane(lo, i);
    if (word == 0ull) continue;                      // uniform
    const int rank = __popcll(word & ((1ull << lane) - 1ull));
    if (((word >> lane) & 1ull) && base + rank < capacity) col_idx[base + rank] = i * 64 + lane;
    base += __popcll(word);
  }
}

// Index lists of the all-ones mask: row (head,u) = {0..u} (causal) or {0..N-1}.
__global__ __launch_bounds__(256) void dense_csr_kernel(int h, int N, int causal,
                                                        int32_t* __restrict__ row_ptr,
                                                        int32_t* __restrict__ col_idx) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int R = h * N;
  if (r > R) return;
  const int64_t per_head = causal ? (int64_t)N * (N + 1) / 2 : (int64_t)N * N;
  if (r == R) {
    if (lane == 0) row_ptr[R] = (int32_t)(h * per_head);
    return;
  }
  const int hq = r / N, u = r % N;
  const int64_t base = hq * per_head + (causal ? (int64_t)u * (u + 1) / 2 : (int64_t)u * N);
  const int len = causal ? u + 1 : N;
  if (lane == 0) row_ptr[r] = (int32_t)base;
  for (int v = lane; v < len; v += 64) col_idx[base + v] = v;
}

// ---- band descriptors (host) -------------------------------------------------------
// Contiguous bands of Sec. 3.4: first d_high dims, last d_low dims.
static prism_bands default_bands(const prism_params* p) {
  prism_bands b = {};
  if (p->d_high > 0) {
    b.high.n_segments = 1;
    b.high.start[0] = 0;
    b.high.width[0] = p->d_high;
  }
  if (p->d_low > 0) {
    b.low.n_segments = 1;
    b.low.start[0] = p->head_dim - p->d_low;
    b.low.width[0] = p->d_low;
  }
  return b;
}

// Validates the descriptors and builds the dim -> band position maps.
static int make_band_map(const prism_params* p, const prism_bands* bands, BandMap* map) {
  if (bands == nullptr) return PRISM_ERR_INVALID_ARG;
  if (!(p->top_p > 0.0f) || !(p->top_p <= 1.0f)) return PRISM_ERR_INVALID_ARG;   // also rejects NaN
  const prism_band* zb[2] = {&bands->high, &bands->low};
  for (int z = 0; z < 2; ++z) {
    for (int c = 0; c < kMaxHeadDim; ++c) map->pos[z][c] = -1;
    if (zb[z]->n_segments < 0 || zb[z]->n_segments > PRISM_MAX_SEGMENTS) return PRISM_ERR_INVALID_ARG;
    int n = 0;
    for (int i = 0; i < zb[z]->n_segments; ++i) {
      const int64_t start = zb[z]->start[i], width = zb[z]->width[i];
      if (start < 0 || width <= 0 || start + width > p->head_dim) return PRISM_ERR_INVALID_ARG;
      for (int c = (int)start; c < (int)(start + width); ++c) {
        if (map->pos[z][c] >= 0) return PRISM_ERR_INVALID_ARG;          // slices of one band overlap
        map->pos[z][c] = (int16_t)n++;
      }
    }
    map->dz[z] = n;
    map->dpad[z] = (n + 31) / 32 * 32;
  }
  if (map->dz[0] == 0 && map->dz[1] == 0) return PRISM_ERR_INVALID_ARG;
  return PRISM_OK;
}

// ---- workspace layout ------------------------------------------------------------
struct EstimateWs {
  size_t band[2][3], energy, inv_scale, total;
};
static EstimateWs estimate_ws(const prism_params* p) {
  const size_t N = n_blocks(p);
  const size_t heads = (size_t)p->n_q_heads + p->n_kv_heads;
  EstimateWs w;
  size_t off = 0;
  for (int z = 0; z < 2; ++z)
    for (int term = 0; term < 3; ++term) {
      w.band[z][term] = off;
      // q-heads: N rows each; kv heads: whole tiles of 16 blocks
      off = align_up(off + ((size_t)p->n_q_heads * N + (size_t)p->n_kv_heads * ((N + 15) / 16 * 16)) *
                               band_stride(p->head_dim) * 2, 256);
    }
  w.energy = off;    off = align_up(off + heads * N * 4 * sizeof(float), 256);
  w.inv_scale = off; off = align_up(off + (size_t)p->n_q_heads * 2 * sizeof(float), 256);
  w.total = off;
  return w;
}

static BandVectors band_vectors(char* ws, const EstimateWs& L) {
  BandVectors bv;
  for (int z = 0; z < 2; ++z)
    for (int term = 0; term < 3; ++term) bv.v[z][term] = reinterpret_cast<uint16_t*>(ws + L.band[z][term]);
  return bv;
}

template <int BLK, bool kRope, int D>
static void launch_pool(const prism_params* p, const HeadStrides& hs, const BandMap& map, const BandVectors& bv,
                        const uint16_t* q, const uint16_t* k, float* energy, float* pooled_q, float* pooled_k,
                        const RopeArgs& rope, uint16_t* q_out, uint16_t* k_out, hipStream_t st) {
  const int N = n_blocks(p);
  hipLaunchKernelGGL((pool_energy_kernel<BLK, kRope, D>), dim3(N, p->n_q_heads + p->n_kv_heads), dim3(256), 0,
                     st, q, k, p->n_q_heads, p->seq_len, N, hs.q, hs.kv, map, bv, energy, pooled_q, pooled_k,
                     rope, q_out, k_out);
}

static int run_pool_and_scale(const prism_params* p, const HeadStrides& hs, const BandMap& map, const void* q,
                              const void* k, char* ws, const EstimateWs& L, float* pooled_q, float* pooled_k,
                              float* scales, hipStream_t st, const RopeArgs* rope = nullptr,
                              void* q_out = nullptr, void* k_out = nullptr) {
  const int N = n_blocks(p);
  const BandVectors bv = band_vectors(ws, L);
  float* energy = reinterpret_cast<float*>(ws + L.energy);
  float* inv = reinterpret_cast<float*>(ws + L.inv_scale);
  const uint16_t* qp = (const uint16_t*)q;
  const uint16_t* kp = (const uint16_t*)k;
  const RopeArgs ra = rope != nullptr ? *rope : RopeArgs{};
  uint16_t* qo = (uint16_t*)q_out;
  uint16_t* ko = (uint16_t*)k_out;
#define PRISM_POOL(BLK, D)                                                                              \
  do {                                                                                                  \
    if (rope == nullptr)                                                                                \
      launch_pool<BLK, false, D>(p, hs, map, bv, qp, kp, energy, pooled_q, pooled_k, ra, nullptr, nullptr, st); \
    else                                                                                                \
      launch_pool<BLK, true, D>(p, hs, map, bv, qp, kp, energy, pooled_q, pooled_k, ra, qo, ko, st);    \
  } while (0)
  if (p->block == 128) {
    if (p->head_dim == 64) PRISM_POOL(128, 64);
    else if (p->head_dim == 128) PRISM_POOL(128, 128);
    else PRISM_POOL(128, 256);
  } else {
    if (p->head_dim == 64) PRISM_POOL(64, 64);
    else if (p->head_dim == 128) PRISM_POOL(64, 128);
    else PRISM_POOL(64, 256);
  }
#undef PRISM_POOL
  hipLaunchKernelGGL(scale_kernel, dim3(p->n_q_heads), dim3(64), 0, st, energy, p->n_q_heads,
                     p->n_kv_heads, N, p->head_dim, map.dz[0], map.dz[1],
                     (p->flags & PRISM_FLAG_NO_CALIBRATION) ? 0 : 1, inv, scales);
  return launch_status();
}

template <int MAXCH, bool DUMP, int kRowsPerWave = 4>
static int launch_select(const prism_params* p, const BandMap& map, char* ws, const EstimateWs& L,
                         uint64_t* mask_bits, int32_t* row_ptr, float* lh, float* ll, hipStream_t st) {
  const int N = n_blocks(p);
  const int strips = (N + kStripRows - 1) / kStripRows;
  const size_t lds = (size_t)kStripRows * (((N + 15) / 16) * 16 + 4) * sizeof(float);
  auto kern = select_kernel<MAXCH, DUMP, kRowsPerWave>;
  if (lds > 64 * 1024) {
    // more than 64 KB of dynamic LDS has to be allowed once per kernel and device: what the
    // largest N needs is asked for on the first such call of this instantiation on a device
    static std::mutex mu;
    static bool raised[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PRISM_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!raised[dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(kStripRows * (kMaxBlocks + 4) * sizeof(float))) != hipSuccess)
        return PRISM_ERR_HIP;
      raised[dev] = true;
    }
  }
  int select_flags = 0;
  if (!(p->flags & PRISM_FLAG_BIDIRECTIONAL)) select_flags |= kSelCausal;
  if (p->flags & PRISM_FLAG_FORCE_DIAGONAL) select_flags |= kSelForceDiagonal;
  if (p->flags & PRISM_FLAG_FORCE_SINK) select_flags |= kSelForceSink;
  hipLaunchKernelGGL(kern, dim3(strips, p->n_q_heads), dim3(kStripRows / kRowsPerWave * 64), lds, st,
                     band_vectors(ws, L),
                     reinterpret_cast<const float*>(ws + L.inv_scale), p->n_q_heads, p->n_kv_heads, N,
                     band_stride(p->head_dim), map.dpad[0], map.dpad[1], p->top_p, select_flags, mask_bits, row_ptr, lh, ll);
  return launch_status();
}

static int run_compaction(const prism_params* p, const uint64_t* mask_bits, int32_t* row_ptr,
                          int32_t* col_idx, int64_t capacity, int32_t* info, bool count_rows,
                          hipStream_t st) {
  const int N = n_blocks(p);
  const int R = p->n_q_heads * N;
  const int W = (N + 63) / 64;
  if (count_rows)
    hipLaunchKernelGGL(row_count_kernel, dim3((R + 255) / 256), dim3(256), 0, st, mask_bits, R, W,
                       row_ptr);
  hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, row_ptr, R, capacity, info);
  hipLaunchKernelGGL(fill_kernel, dim3((R + 3) / 4), dim3(256), 0, st, mask_bits, R, W, row_ptr,
                     col_idx, capacity);
  return launch_status();
}

static int check_ws(const void* ws, size_t have, size_t need) {
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || have < need)
    return PRISM_ERR_WORKSPACE;
  return PRISM_OK;
}

}  // namespace prism

using namespace prism;

extern "C" int prism_version(void) { return 100; }

extern "C" const char* prism_status_string(int status) {
  switch (status) {
    case PRISM_OK: return "ok";
    case PRISM_ERR_INVALID_ARG: return "invalid argument";
    case PRISM_ERR_UNSUPPORTED: return "unsupported configuration";
    case PRISM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PRISM_ERR_HIP: return "HIP runtime error";
    case PRISM_ERR_TOO_LARGE: return "problem exceeds the library's static scratch (prism_estimate_static)";
    default: return "unknown status";
  }
}

extern "C" int prism_estimate_workspace_bytes(const prism_params* params, size_t* bytes) {
  if (bytes == nullptr) return PRISM_ERR_INVALID_ARG;
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  *bytes = estimate_ws(params).total;
  return PRISM_OK;
}

// The whole estimate of one sequence (arguments already validated): pooling (+ RoPE when `rope`
// is given), calibration, selection, compaction.
static int estimate_core(const prism_params* params, const HeadStrides& hs, const BandMap& map,
                         const void* q, const void* k, uint64_t* mask_bits, int32_t* row_ptr,
                         int32_t* col_idx, int64_t col_capacity, int32_t* info, char* ws,
                         hipStream_t st, const RopeArgs* rope = nullptr, void* q_out = nullptr,
                         void* k_out = nullptr) {
  const EstimateWs L = estimate_ws(params);
  int rc = run_pool_and_scale(params, hs, map, q, k, ws, L, nullptr, nullptr, nullptr, st, rope, q_out, k_out);
  if (rc != PRISM_OK) return rc;
  const int N = n_blocks(params);
  // up to 1024 blocks: 4 waves of 4 rows, two workgroups per CU; beyond (a 131 KB logit strip, one
  // workgroup per CU, rows of 32 registers): 8 waves of 2 rows (measured 1.89 -> 1.25 ms at N = 2048,
  // while at N = 1024 the 4-wave form is 2 % faster)
  rc = (N <= 1024)
           ? launch_select<16, false, 4>(params, map, ws, L, mask_bits, row_ptr, nullptr, nullptr, st)
           : launch_select<32, false, 2>(params, map, ws, L, mask_bits, row_ptr, nullptr, nullptr, st);
  if (rc != PRISM_OK) return rc;
  return run_compaction(params, mask_bits, row_ptr, col_idx, col_capacity, info, false, st);
}

extern "C" int prism_estimate_bands(const prism_params* params, const prism_bands* bands,
                                    const void* q_bf16, const void* k_bf16, uint64_t* mask_bits,
                                    int32_t* row_ptr, int32_t* col_idx, int64_t col_capacity,
                                    int32_t* info, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  BandMap map;
  rc = make_band_map(params, bands, &map);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16 || !mask_bits || !row_ptr || !col_idx || !info || col_capacity < 0)
    return PRISM_ERR_INVALID_ARG;
  rc = check_ws(workspace, workspace_bytes, estimate_ws(params).total);
  if (rc != PRISM_OK) return rc;
  return estimate_core(params, contiguous_heads(params), map, q_bf16, k_bf16, mask_bits, row_ptr, col_idx,
                       col_capacity, info, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

// ---- packed variable-length batches ---------------------------------------------------
// parameters of sequence s of the batch
static prism_params sequence_params(const prism_params* params, const int32_t* cu_seqlens, int s) {
  prism_params ps = *params;
  ps.seq_len = cu_seqlens[s + 1] - cu_seqlens[s];
  return ps;
}

extern "C" int prism_varlen_layout(const prism_params* params, const int32_t* cu_seqlens, int n_seqs,
                                   int64_t* mask_offsets, int64_t* row_offsets, int64_t* col_offsets) {
  // a batch may hold more tokens than one sequence may: only the per-sequence limits apply
  prism_params one = {};
  if (params != nullptr) {
    one = *params;
    one.seq_len = 1;
  }
  int rc = check_params(params != nullptr ? &one : nullptr);
  if (rc != PRISM_OK) return rc;
  if (cu_seqlens == nullptr || n_seqs <= 0 || cu_seqlens[0] != 0 || cu_seqlens[n_seqs] != params->seq_len)
    return PRISM_ERR_INVALID_ARG;
  int64_t mo = 0, ro = 0, co = 0;
  for (int s = 0; s < n_seqs; ++s) {
    if (cu_seqlens[s + 1] <= cu_seqlens[s]) return PRISM_ERR_INVALID_ARG;
    const prism_params ps = sequence_params(params, cu_seqlens, s);
    rc = check_params(&ps);
    if (rc != PRISM_OK) return rc;
    const int64_t N = n_blocks(&ps), h = ps.n_q_heads;
    if (mask_offsets) mask_offsets[s] = mo;
    if (row_offsets) row_offsets[s] = ro;
    if (col_offsets) col_offsets[s] = co;
    mo += h * N * ((N + 63) / 64);
    ro += h * N + 1;
    co += (ps.flags & PRISM_FLAG_BIDIRECTIONAL) ? h * N * N : h * N * (N + 1) / 2;
  }
  if (mask_offsets) mask_offsets[n_seqs] = mo;
  if (row_offsets) row_offsets[n_seqs] = ro;
  if (col_offsets) col_offsets[n_seqs] = co;
  return PRISM_OK;
}

extern "C" int prism_estimate_varlen_workspace_bytes(const prism_params* params, const int32_t* cu_seqlens,
                                                     int n_seqs, size_t* bytes) {
  if (bytes == nullptr) return PRISM_ERR_INVALID_ARG;
  int rc = prism_varlen_layout(params, cu_seqlens, n_seqs, nullptr, nullptr, nullptr);
  if (rc != PRISM_OK) return rc;
  size_t need = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const prism_params ps = sequence_params(params, cu_seqlens, s);
    const size_t b = estimate_ws(&ps).total;
    need = b > need ? b : need;
  }
  *bytes = need;
  return PRISM_OK;
}

extern "C" int prism_estimate_varlen(const prism_params* params, const int32_t* cu_seqlens, int n_seqs,
                                     const void* q_bf16, const void* k_bf16, uint64_t* mask_bits,
                                     int32_t* row_ptr, int32_t* col_idx, int32_t* info, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  size_t need = 0;
  int rc = prism_estimate_varlen_workspace_bytes(params, cu_seqlens, n_seqs, &need);
  if (rc != PRISM_OK) return rc;
  rc = check_bands(params);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16 || !mask_bits || !row_ptr || !col_idx || !info) return PRISM_ERR_INVALID_ARG;
  rc = check_ws(workspace, workspace_bytes, need);
  if (rc != PRISM_OK) return rc;
  const prism_bands bands = default_bands(params);
  BandMap map;
  rc = make_band_map(params, &bands, &map);
  if (rc != PRISM_OK) return rc;
  const size_t d = params->head_dim, T = params->seq_len;
  const HeadStrides hs{T * d, T * d, T};
  int64_t mo = 0, ro = 0, co = 0;
  for (int s = 0; s < n_seqs; ++s) {
    const prism_params ps = sequence_params(params, cu_seqlens, s);
    const int64_t N = n_blocks(&ps), h = ps.n_q_heads;
    const int64_t cap = (ps.flags & PRISM_FLAG_BIDIRECTIONAL) ? h * N * N : h * N * (N + 1) / 2;
    const size_t tok = (size_t)cu_seqlens[s] * d;
    // the sequences share the workspace: they run one after the other on the stream
    rc = estimate_core(&ps, hs, map, (const uint16_t*)q_bf16 + tok, (const uint16_t*)k_bf16 + tok, mask_bits + mo,
                       row_ptr + ro, col_idx + co, cap, info + 4 * s, static_cast<char*>(workspace),
                       static_cast<hipStream_t>(stream));
    if (rc != PRISM_OK) return rc;
    mo += h * N * ((N + 63) / 64);
    ro += h * N + 1;
    co += cap;
  }
  return PRISM_OK;
}

extern "C" int prism_estimate(const prism_params* params, const void* q_bf16, const void* k_bf16,
                              uint64_t* mask_bits, int32_t* row_ptr, int32_t* col_idx,
                              int64_t col_capacity, int32_t* info, void* workspace,
                              size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  rc = check_bands(params);
  if (rc != PRISM_OK) return rc;
  const prism_bands bands = default_bands(params);
  return prism_estimate_bands(params, &bands, q_bf16, k_bf16, mask_bits, row_ptr, col_idx,
                              col_capacity, info, workspace, workspace_bytes, stream);
}

// ---- the estimate for callers that cannot allocate -----------------------------------
// The scratch of prism_estimate lives in one file-scope device array instead of a caller
// workspace.  `scratch` below is only the host-side handle of that array: the address of the
// copy a given GPU holds is asked from the runtime once per device and kept; kernels and
// everything else on the host side use that address.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PRISM_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return PRISM_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PRISM_OK;
}

extern "C" int prism_estimate_static(const prism_params* params, const void* q_bf16,
                                     const void* k_bf16, uint64_t* mask_bits, int32_t* row_ptr,
                                     int32_t* col_idx, int64_t col_capacity, int32_t* info,
                                     void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  rc = check_bands(params);
  if (rc != PRISM_OK) return rc;
  if (estimate_ws(params).total > kStaticScratchBytes) return PRISM_ERR_TOO_LARGE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != PRISM_OK) return rc;
  // every part of the scratch that a kernel reads is written earlier in the same call, so the
  // previous call's contents need no clearing
  return prism_estimate(params, q_bf16, k_bf16, mask_bits, row_ptr, col_idx, col_capacity, info, ws,
                        kStaticScratchBytes, stream);
}

extern "C" int prism_rope_estimate(const prism_params* params, const prism_rope* rope,
                                   const prism_bands* bands, const void* q_in_bf16,
                                   const void* k_in_bf16, void* q_out_bf16, void* k_out_bf16,
                                   uint64_t* mask_bits, int32_t* row_ptr, int32_t* col_idx,
                                   int64_t col_capacity, int32_t* info, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  prism_bands def;
  if (bands == nullptr) {
    rc = check_bands(params);
    if (rc != PRISM_OK) return rc;
    def = default_bands(params);
    bands = &def;
  }
  BandMap map;
  rc = make_band_map(params, bands, &map);
  if (rc != PRISM_OK) return rc;
  if (!rope || !q_in_bf16 || !k_in_bf16 || !q_out_bf16 || !k_out_bf16 || !mask_bits || !row_ptr ||
      !col_idx || !info || col_capacity < 0)
    return PRISM_ERR_INVALID_ARG;
  if (!(rope->base > 1.0) || rope->position_offset < 0 ||
      (int64_t)rope->position_offset + params->seq_len > ((int64_t)1 << 30))
    return PRISM_ERR_INVALID_ARG;
  RopeArgs ra;
  ra.ln_base = log(rope->base);
  ra.position_offset = rope->position_offset;
  ra.yarn_scale = 0.0;
  ra.yarn_alpha = ra.yarn_beta = ra.yarn_native_len = 0.0;
  if (rope->yarn_native_len != 0) {
    if (rope->yarn_native_len < 0 || !(rope->yarn_scale >= 1.0) || !(rope->yarn_alpha >= 0.0) ||
        !(rope->yarn_beta > rope->yarn_alpha))
      return PRISM_ERR_INVALID_ARG;
    ra.yarn_scale = rope->yarn_scale;
    ra.yarn_alpha = rope->yarn_alpha;
    ra.yarn_beta = rope->yarn_beta;
    ra.yarn_native_len = (double)rope->yarn_native_len;
  }
  rc = check_ws(workspace, workspace_bytes, estimate_ws(params).total);
  if (rc != PRISM_OK) return rc;
  return estimate_core(params, contiguous_heads(params), map, q_in_bf16, k_in_bf16, mask_bits, row_ptr, col_idx,
                       col_capacity, info, static_cast<char*>(workspace), static_cast<hipStream_t>(stream),
                       &ra, q_out_bf16, k_out_bf16);
}

extern "C" int prism_block_scores_bands(const prism_params* params, const prism_bands* bands,
                                        const void* q_bf16, const void* k_bf16, float* pooled_q,
                                        float* pooled_k, float* scales, float* logits_high,
                                        float* logits_low, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  BandMap map;
  rc = make_band_map(params, bands, &map);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16) return PRISM_ERR_INVALID_ARG;
  const EstimateWs L = estimate_ws(params);
  rc = check_ws(workspace, workspace_bytes, L.total);
  if (rc != PRISM_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  rc = run_pool_and_scale(params, contiguous_heads(params), map, q_bf16, k_bf16, ws, L, pooled_q, pooled_k,
                          scales, st);
  if (rc != PRISM_OK) return rc;
  if (logits_high == nullptr && logits_low == nullptr) return PRISM_OK;
  return launch_select<16, true>(params, map, ws, L, nullptr, nullptr, logits_high, logits_low, st);
}

extern "C" int prism_block_scores(const prism_params* params, const void* q_bf16,
                                  const void* k_bf16, float* pooled_q, float* pooled_k, float* scales,
                                  float* logits_high, float* logits_low, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  rc = check_bands(params);
  if (rc != PRISM_OK) return rc;
  const prism_bands bands = default_bands(params);
  return prism_block_scores_bands(params, &bands, q_bf16, k_bf16, pooled_q, pooled_k, scales,
                                  logits_high, logits_low, workspace, workspace_bytes, stream);
}

extern "C" int prism_mask_to_csr(const prism_params* params, const uint64_t* mask_bits,
                                 int32_t* row_ptr, int32_t* col_idx, int64_t col_capacity,
                                 int32_t* info, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  if (!mask_bits || !row_ptr || !col_idx || !info || col_capacity < 0) return PRISM_ERR_INVALID_ARG;
  return run_compaction(params, mask_bits, row_ptr, col_idx, col_capacity, info, true,
                        static_cast<hipStream_t>(stream));
}

static int dense_csr(const prism_params* params, bool causal, int32_t* row_ptr, int32_t* col_idx,
                     int64_t col_capacity, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  if (!row_ptr || !col_idx) return PRISM_ERR_INVALID_ARG;
  const int64_t N = n_blocks(params);
  const int64_t need = (int64_t)params->n_q_heads * (causal ? N * (N + 1) / 2 : N * N);
  if (col_capacity < need) return PRISM_ERR_INVALID_ARG;
  const int R = params->n_q_heads * (int)N;
  hipLaunchKernelGGL(dense_csr_kernel, dim3((R + 1 + 3) / 4), dim3(256), 0,
                     static_cast<hipStream_t>(stream), params->n_q_heads, (int)N, causal ? 1 : 0,
                     row_ptr, col_idx);
  return launch_status();
}

extern "C" int prism_causal_csr(const prism_params* params, int32_t* row_ptr, int32_t* col_idx,
                                int64_t col_capacity, void* stream) {
  return dense_csr(params, true, row_ptr, col_idx, col_capacity, stream);
}

extern "C" int prism_dense_csr(const prism_params* params, int32_t* row_ptr, int32_t* col_idx,
                               int64_t col_capacity, void* stream) {
  const bool causal = params == nullptr || !(params->flags & PRISM_FLAG_BIDIRECTIONAL);
  return dense_csr(params, causal, row_ptr, col_idx, col_capacity, stream);
}
