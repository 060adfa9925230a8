// Block-sparse causal flash attention of libprism (gfx950, bf16 MFMA, fp32 online softmax).
//
// Sec. 2 "Block-Sparse Attention": dense QK^T / softmax / PV with online accumulation,
// restricted to the (q-block, kv-block) pairs listed in a CSR index list.
//
// Formulation.  Each wave owns 32 query rows and works on the TRANSPOSED problem so that
// every per-query quantity (running max, running sum, output scale) lives in one lane:
//     S^T = K Q^T      (v_mfma_f32_32x32x16_bf16: A = K tile rows, B = Q rows)
//     O^T += V^T P^T   (A = V^T rows, B = P^T, which is exactly the accumulator layout of S^T
//                       after bf16 conversion, so P never leaves registers)
// In the 32x32 accumulator layout lane l holds query column l%32 and, per 32-key tile,
// keys 8*(r/4) + 4*(l/32) + r%4 for r = 0..15.  One MFMA K-step of PV therefore consumes
// keys {16s + 8g + 4*(l/32) + i}; the V^T operand must present the same keys in the same
// slots, which is achieved by a one-off re-layout of V in HBM (vt_image_kernel): per kv
// block a [d][B] image whose key positions inside every group of 16 are permuted to
// pos = 8*hf + 4*g + i  for key = 8*g + 4*hf + i.  A 16-byte LDS read then yields one
// A operand.
#include "prism_common.h"

#include <mutex>
#include <type_traits>

namespace prism {

// =====================================================================================
// V re-layout: V [h_kv, L, d]  ->  image [h_kv, N, d, B] with permuted key positions; keys
// past the end of a ragged last block are written as zeros.
// =====================================================================================
// With vt16 != nullptr a second image with the same layout holds the values as fp16 (the
// 64-queries-per-wave kernel forms its P V product in fp16: 11 significant bits for P instead of 8).
// Every bf16 value of magnitude in [2^-17, 65504] (and zero) is an fp16 value, so the conversion is
// exact there; smaller magnitudes lose at most 2^-25 absolute.  A block holding a finite value beyond
// the fp16 range sets range_flags[kv head * N + block] = 1 (else 0): such inputs go through the
// general kernel and the bf16 image.
template <int BLK, int D>
__global__ __launch_bounds__(256) void vt_image_kernel(const uint16_t* __restrict__ v,
                                                       uint16_t* __restrict__ vt, int L, int N,
                                                       size_t kv_head_stride,
                                                       uint16_t* __restrict__ vt16,
                                                       int32_t* __restrict__ range_flags) {
  __shared__ uint16_t tile[BLK][D + 2];
  __shared__ int s_over;
  const int blk = blockIdx.x, kvh = blockIdx.y, t = threadIdx.x;
  const uint16_t* src = v + (size_t)kvh * kv_head_stride + (size_t)blk * BLK * D;
  const int cnt = min(BLK, L - blk * BLK);
  if (t == 0) s_over = 0;
  constexpr int RCH = D / 8;                         // 16-byte chunks per token row
  for (int idx = t; idx < BLK * RCH; idx += 256) {
    const int row = idx / RCH, c = idx % RCH;
    u32x4 x = {0u, 0u, 0u, 0u};                       // V is read once: streaming (non-temporal) loads
    if (row < cnt) x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (size_t)row * D + c * 8));
    uint32_t* dst = reinterpret_cast<uint32_t*>(&tile[row][c * 8]);   // 4-byte aligned: row stride 2*D + 4 B
    dst[0] = x[0]; dst[1] = x[1]; dst[2] = x[2]; dst[3] = x[3];
  }
  __syncthreads();
  constexpr int CPR = BLK / 8;                       // 16-byte chunks per image row
  uint16_t* dstb = vt + ((size_t)kvh * N + blk) * (size_t)D * BLK;
  bool over = false;
  for (int idx = t; idx < D * CPR; idx += 256) {
    const int d = idx / CPR, c = idx % CPR;
    uint32_t w[4], w16[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      // position p = c*8 + e inside the row; group a = p/16, hf = (p/8)&1, g = (p/4)&1, i = p&3
      const int p0 = c * 8 + e, p1 = p0 + 1;
      const int k0 = (p0 & ~15) + 8 * ((p0 >> 2) & 1) + 4 * ((p0 >> 3) & 1) + (p0 & 3);
      const int k1 = (p1 & ~15) + 8 * ((p1 >> 2) & 1) + 4 * ((p1 >> 3) & 1) + (p1 & 3);
      const uint32_t a = tile[k0][d], b = tile[k1][d];
      w[e >> 1] = a | (b << 16);
      if (vt16 != nullptr) {
        const float fa = bf16_bits_to_float(a), fb = bf16_bits_to_float(b);
        over |= (fabsf(fa) > 65504.f && fabsf(fa) < INFINITY) || (fabsf(fb) > 65504.f && fabsf(fb) < INFINITY);
        const _Float16 ha = (_Float16)fa, hb = (_Float16)fb;
        w16[e >> 1] = (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
      }
    }
    *reinterpret_cast<uint4*>(dstb + (size_t)d * BLK + c * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    if (vt16 != nullptr)
      *reinterpret_cast<uint4*>(vt16 + ((size_t)kvh * N + blk) * (size_t)D * BLK + (size_t)d * BLK + c * 8) =
          make_uint4(w16[0], w16[1], w16[2], w16[3]);
  }
  if (vt16 != nullptr) {
    if (over) s_over = 1;                            // benign race: every writer stores 1
    __syncthreads();
    if (t == 0) range_flags[kvh * N + blk] = s_over;
  }
}

// =====================================================================================
// Sparse attention kernel.  One workgroup works on one (q-head, q-block) row at a time;
// BLK/32 waves of 32 queries.
// LDS: K tile [BLK][d] bf16 and V^T tile [d][BLK] bf16 (d = 64, 128, 256), 16-byte chunks XOR-swizzled by
// row so that the 16-lane column reads are conflict-free.  Tiles are copied global -> LDS
// asynchronously, without passing through registers.
// Step per listed kv block (each tile buffer is refilled as soon as its last reader is done):
//     K(j) in LDS | start V(j) copy | S^T = K Q^T | barrier | start K(j+1) copy
//     online softmax | wait V(j) | barrier | O^T += V^T P^T | wait K(j+1) | barrier
// The workgroups are persistent: a workgroup pulls its next row from its XCD's queue at the top
// of the last step of the current row and reads that row's queue entry during the last PV, so
// a row switch exposes only the load of the Q rows and of the first K tile.
// =====================================================================================
// PAIR: a workgroup serves two neighbouring q-blocks of one q-head (twice the waves) and walks the
// union of their two lists, so a tile that both list is copied once.
template <int BLK, int D, bool PAIR = false>
struct AttnCfg {
  static constexpr int kRowWaves = BLK / 32;                // waves of one q-block
  static constexpr int kWaves = kRowWaves * (PAIR ? 2 : 1);
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kTileBytes = BLK * D * 2;
  static constexpr int kChunks = kTileBytes / 16;          // 16-byte pieces per tile
  static constexpr int kPerThread = kChunks / kThreads;    // = D / 16 (D / 32 with PAIR)
  static constexpr int kKCpr = D / 8;                      // chunks per K row
  static constexpr int kVtCpr = BLK / 8;                   // chunks per V^T row
  static constexpr int kDTiles = D / 32;                   // 32-dim tiles of the output
  static constexpr int kKSteps = D / 16;                   // MFMA k-steps of S^T = K Q^T
  static constexpr int kWavesPerSimd = D > 128 ? 1 : 2;    // register budget: 512 or 256 per lane
};

// Asynchronous global -> LDS tile copies (buffer_load_dwordx4 ... lds: every lane fetches 16
// bytes at rsrc.base + voffset + soffset and the wave's 64 pieces land contiguously in LDS
// at M0-base + 16*lane).  LDS slot p (16-byte units) of a tile belongs to (row, c') with c'
// the swizzled chunk position; the lane that fills it reads global chunk
// c = c' ^ swizzle(row), i.e. the swizzle is applied on the global side.
// Buffer (not flat/global) addressing is used on purpose: LDS reads issued while such
// copies are in flight then keep exact lgkmcnt tracking in the compiler.
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  // raw buffer, 32-bit data format, no swizzle, no TID addition
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// XOR applied to the chunk index of K-tile row `row` so that 16 consecutive rows put the same
// chunk on 16 different LDS bank groups: rows of 128 bytes (d = 64) come two to a 256-byte line,
// rows of 512 bytes (d = 256) wrap the banks twice.
template <int D>
__device__ __forceinline__ int k_row_swizzle(int row) {
  return D == 64 ? ((row >> 1) & 7) : (row & 15);
}

// byte offset inside a tile of the 16-byte piece that LDS slot p holds
template <int BLK, int D>
__device__ __forceinline__ int k_piece_offset(int p) {
  using C = AttnCfg<BLK, D>;
  const int row = p / C::kKCpr;
  return row * (D * 2) + (((p % C::kKCpr) ^ k_row_swizzle<D>(row)) << 4);
}
template <int BLK, int D>
__device__ __forceinline__ int vt_piece_offset(int p) {
  using C = AttnCfg<BLK, D>;
  const int row = p / C::kVtCpr;
  return row * (BLK * 2) + (((p % C::kVtCpr) ^ (row & (C::kVtCpr - 1))) << 4);
}

template <int BLK, int D, bool PAIR>
__device__ __forceinline__ void async_load_k_tile(__amdgpu_buffer_rsrc_t rs, int tile_off, char* lds,
                                                  int t) {
  using C = AttnCfg<BLK, D, PAIR>;
  // wave-uniform LDS base, re-materialised here so that the per-piece M0 values are formed
  // with scalar adds instead of being kept live (and spilled) across the whole loop
  int wave_base = __builtin_amdgcn_readfirstlane(t & ~63);
  asm volatile("" : "+s"(wave_base));
#pragma unroll
  for (int i = 0; i < C::kPerThread; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lptr_t)(lds + (i * C::kThreads + wave_base) * 16), 16,
                                             k_piece_offset<BLK, D>(i * C::kThreads + t), tile_off, 0, 0);
}

template <int BLK, int D, bool PAIR>
__device__ __forceinline__ void async_load_vt_tile(__amdgpu_buffer_rsrc_t rs, int tile_off, char* lds,
                                                   int t) {
  using C = AttnCfg<BLK, D, PAIR>;
  int wave_base = __builtin_amdgcn_readfirstlane(t & ~63);
  asm volatile("" : "+s"(wave_base));
#pragma unroll
  for (int i = 0; i < C::kPerThread; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lptr_t)(lds + (i * C::kThreads + wave_base) * 16), 16,
                                             vt_piece_offset<BLK, D>(i * C::kThreads + t), tile_off, 0, 0);
}

// Waits on the vector-memory counter, written with the builtin (immediate: vmcnt in bits 3:0,
// expcnt = 7 and lgkmcnt = 15 meaning "no wait") rather than inline asm, so that the compiler's
// own wait-count bookkeeping sees them: it then knows which tile copies have landed and adds no
// conservative vmcnt(0) of its own in front of the LDS reads of a finished tile.
__device__ __forceinline__ void wait_async_loads() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  asm volatile("" ::: "memory");
}
// all but the youngest tile copy (kPerThread = d/16 vector-memory operations per thread) are complete
template <int kPerThread>
__device__ __forceinline__ void wait_async_loads_but_last_tile() {
  static_assert(kPerThread <= 16, "vmcnt immediate");
  asm volatile("" ::: "memory");
  // vmcnt(kPerThread): low four bits in 3:0, the two high bits in 15:14
  __builtin_amdgcn_s_waitcnt(0x0F70 | (kPerThread & 15) | ((kPerThread >> 4) << 14));
  asm volatile("" ::: "memory");
}

// max / sum of a value with the lane 32 away (the two lanes that share a query), on the
// v_permlane32_swap cross-lane path: an LDS shuffle here would queue behind the tile traffic
// on the critical path of every step.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float other_half_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float other_half_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Workgroup barrier of the tile loop: this wave's LDS accesses are complete, then s_barrier.
// Unlike __syncthreads() it carries no memory fence, so the compiler adds no wait for the global
// loads, stores and atomics in flight (the next tile copies, the previous row's output, the
// queue pull); the tile copies are waited for explicitly with vmcnt where their data is needed.
__device__ __forceinline__ void tile_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Queue entry of one row, written by queue_fill_kernel:
//   x = q-head, y = q-block u | (first valid key block << 16), z = index of that entry in
//   col_idx, w = end of the row's list (z == w: the row has no valid entry).
// Every queue (one per XCD) owns a contiguous segment of the table: `plan` = { start[8], len[8],
// pull counters[8] }; a workgroup's pulls p = 0, 1, 2, ... from queue x are the entries
// start[x] + p while p < len[x].
enum { kItemEnd = 0, kItemRow = 2 };
// MI355X: 8 accelerator dies (XCDs), each with its own L2; workgroups are dealt to them round-robin,
// so the attention kernels keep one work queue per XCD (the plan below has room for exactly kXcds).
constexpr int kXcds = 8;
constexpr int kPlanStart = 0, kPlanLen = 8, kPlanCounter = 16, kPlanFlags = 24, kPlanInts = 32;
// plan[kPlanFlags]: bit 0 = some list holds an entry that must be skipped (negative, beyond the
// row's last admissible block): such lists go through the general kernel, clean lists through the
// 64-queries-per-wave kernel; each of the two kernels returns at once when it is not its turn.
constexpr int kFlagDirtyLists = 1;

__device__ __forceinline__ int item_kind(int pulled, int seg_start, int seg_len, int* entry) {
  if (pulled >= seg_len) return kItemEnd;
  *entry = seg_start + pulled;
  return kItemRow;
}

// kStreamOnly (PRISM_FLAG_STREAM_ONLY): the same tile copies, waits, barriers and queue traffic
// with the arithmetic left out; it measures how long the memory side of a call takes alone.
// kPair (B = 64, an even number of blocks, every list ascending and clean): items and plan describe PAIR
// rows (q-blocks 2u' and 2u' + 1 of a head, whose two lists lie one behind the other in col_idx); the
// workgroup walks the union of the two lists in ascending order, copies every tile of the union once,
// and the waves of a q-block compute only in the steps whose block their own list names.  `dirty_flag`
// is the flag word the list check wrote: the pair kernel returns at once when it is set, the plain
// kernel launched behind it (only_dirty) returns at once when it is not.
template <int BLK, bool kStreamOnly, int D, bool kPair>
__global__ __launch_bounds__((AttnCfg<BLK, D, kPair>::kThreads), (AttnCfg<BLK, D, kPair>::kWavesPerSimd)) void sparse_attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt,
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, const int4* __restrict__ items,
    int32_t* __restrict__ plan, const int32_t* __restrict__ dirty_flag,
    uint16_t* __restrict__ out, float* __restrict__ lse, int h, int h_kv, int L, int N,
    HeadStrides hs, int causal, int only_dirty) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the kernel's signature
  using C = AttnCfg<BLK, D, kPair>;
  constexpr int KS = C::kKSteps, DT = C::kDTiles;
  if (kPair) {
    if ((dirty_flag[0] & kFlagDirtyLists) != 0) return;     // the plain kernel takes this call
  } else if (only_dirty && (dirty_flag[0] & kFlagDirtyLists) == 0) {
    return;                                                 // the kernel launched in front of this one took it
  }
  constexpr int KT = BLK / 32;                       // 32-key tiles per kv block
  __shared__ __attribute__((aligned(16))) char lds_k[C::kTileBytes];
  __shared__ __attribute__((aligned(16))) char lds_v[C::kTileBytes];
  __shared__ int next_item, next_queue;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int g = h / h_kv;
  // which of the two q-blocks of a pair row this wave belongs to (wave-uniform)
  const int sub = kPair ? __builtin_amdgcn_readfirstlane(wave / C::kRowWaves) : 0;
  // log2(e) / sqrt(d)
  const float sm_scale = 1.4426950408889634f * (D == 64 ? 0.125f : (D == 128 ? 0.08838834764831845f : 0.0625f));

  // LDS read offsets of this lane inside a 32-row slab: row l32, swizzled chunk
  // (2*step + hf) ^ swizzle(row).  The K tile has d/8 chunks per row; the V^T tile has BLK/8
  // (for BLK = 128 and d = 128 the two tables coincide).
  constexpr int kDepth = 8;                                // LDS reads kept in flight
  int koff[KS], voff[KT * 2];
#pragma unroll
  for (int st = 0; st < KS; ++st) koff[st] = l32 * (D * 2) + (((2 * st + hf) ^ k_row_swizzle<D>(l32)) << 4);
#pragma unroll
  for (int st = 0; st < KT * 2; ++st)
    voff[st] = l32 * (BLK * 2) + (((2 * st + hf) ^ (l32 & (C::kVtCpr - 1))) << 4);

  // Persistent workgroups pull rows from per-XCD queues (workgroups are dealt round-robin to the
  // 8 XCDs, and each XCD has its own L2).  A queue runs through neighbouring q-blocks of one
  // q-head at a time, so the 64 workgroups of an XCD work on neighbouring rows of one head: such
  // rows list many of the same key blocks (stripes, sinks, local windows; all of them for dense
  // lists) at about the same position of their lists, and the tile one of them fetches is still
  // in the XCD's L2 when the others ask for it.
  // A workgroup whose queue is exhausted goes on with rows of another XCD's queue, so the XCDs
  // finish together although the lists of one may take longer per block than those of another;
  // it leaves the loop once it has seen every queue exhausted.
  const int n_queues = gridDim.x < kXcds ? 1 : kXcds;
  int my_queue = blockIdx.x % n_queues;
  int seg_start = plan[kPlanStart + my_queue];
  int seg_len = plan[kPlanLen + my_queue];
  int32_t* counter = plan + kPlanCounter;
  const int vmax_nc = N - 1;
  const int tail = L - (N - 1) * BLK;              // tokens in the last block (BLK unless ragged)
  const uint32_t head_bytes = (uint32_t)L * D * 2;
  const uint32_t image_head_bytes = (uint32_t)N * C::kTileBytes;

  // The queue is pulled when a workgroup is about to become free (at the top of the last
  // step of its row), so neighbouring rows of the queue start close together; the pull and the
  // read of the next row's queue entry are hidden behind that last step.
  int lane_zero;                                     // 0, but opaque to the compiler
  asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
  if (t == 0) next_item = atomicAdd(counter + my_queue, 1);
  __syncthreads();
  int cur_x = 0, cur_y = 0, cur_z = 0, cur_w = 0;     // the current row's queue entry, wave-uniform
  int kind_cur;
  {
    int e = 0;
    kind_cur = item_kind(__builtin_amdgcn_readfirstlane(next_item), seg_start, seg_len, &e);
    if (kind_cur == kItemRow) {
      const int4 it0 = items[e];
      cur_x = it0.x; cur_y = it0.y; cur_z = it0.z; cur_w = it0.w;
    }
  }
  __syncthreads();
  // requests of the last step of a row (not re-initialised per row: overwriting a register that a
  // load in flight will write would force a wait for every older memory operation)
  int4 item_nxt = make_int4(0, 0, 0, 0);
  int pulled_reg = 0;

  for (;;) {
    if (kind_cur == kItemEnd) {
      // Own queue exhausted: look (one coherent read of the 8 pull counters, no atomic) for a
      // queue that still has rows, nearest first round the ring, and pull from it.  A counter
      // only grows, so a queue seen exhausted stays so; the atomic pull decides who gets a row.
      if (wave == 0) {
        int pulls = 0x7fffffff, len = 0;
        if (lane < n_queues) {
          pulls = __hip_atomic_load(counter + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          len = plan[kPlanLen + lane];
        }
        const unsigned long long open = __ballot(pulls < len);
        int pick = -1;
        for (int s = 1; s < n_queues && pick < 0; ++s) {
          const int x = my_queue + s < n_queues ? my_queue + s : my_queue + s - n_queues;
          if ((open >> x) & 1ull) pick = x;
        }
        if (lane == 0) {
          next_queue = pick;
          if (pick >= 0) next_item = atomicAdd(counter + pick, 1);
        }
      }
      __syncthreads();
      const int pick = __builtin_amdgcn_readfirstlane(next_queue);
      if (pick < 0) break;
      my_queue = pick;
      seg_start = plan[kPlanStart + my_queue];
      seg_len = plan[kPlanLen + my_queue];
      int e = 0;
      kind_cur = item_kind(__builtin_amdgcn_readfirstlane(next_item), seg_start, seg_len, &e);
      if (kind_cur == kItemRow) {
        const int4 it0 = items[e];
        cur_x = it0.x; cur_y = it0.y; cur_z = it0.z; cur_w = it0.w;
      }
      __syncthreads();
      continue;
    }
    const int hq = cur_x;
    const int u = cur_y & 0xffff;
    int v = (cur_y >> 16) & 0xffff;
    int it = cur_z;
    const int end = cur_w;
    const bool has_work = kind_cur == kItemRow && it < end;
    const int kvh = hq / g;
    // `u` is the index of the row among the head's rows: a q-block, or a pair of them
    const int qrow = u * (C::kWaves * 32) + wave * 32 + l32;   // >= L for the padding rows of a ragged last block
    const int u_own = kPair ? 2 * u + sub : u;                 // the q-block this wave's queries belong to
    int kind_nxt = kItemEnd;

    if (!has_work) {
      // a row without a valid entry (o = 0, lse = -inf): no tile work; pull the next row right away
      if (kind_cur == kItemRow && qrow < L) {
        uint16_t* op = out + (size_t)hq * hs.q + (size_t)qrow * D + hf * (D / 2);
#pragma unroll
        for (int c = 0; c < D / 16; ++c) *reinterpret_cast<uint4*>(op + c * 8) = make_uint4(0u, 0u, 0u, 0u);
        if (lse != nullptr && hf == 0) lse[(size_t)hq * hs.lse + qrow] = -INFINITY;
      }
      if (t == 0) next_item = atomicAdd(counter + my_queue, 1);
      __syncthreads();
      int e = 0;
      kind_cur = item_kind(__builtin_amdgcn_readfirstlane(next_item), seg_start, seg_len, &e);
      if (kind_cur == kItemRow) {
        const int4 it0 = items[e];
        cur_x = it0.x; cur_y = it0.y; cur_z = it0.z; cur_w = it0.w;
      }
      __syncthreads();
      continue;
    }

    // K and V^T of this kv head as buffer resources (tile v starts at byte v * kTileBytes).
    // K is the caller's tensor: rows past L in a ragged last block are outside the resource and
    // read as zeros.  The V^T image is padded to whole blocks.
    const __amdgpu_buffer_rsrc_t krs = make_rsrc(k + (size_t)kvh * hs.kv, head_bytes);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(vt + (size_t)kvh * N * BLK * D, image_head_bytes);
    const int vmax = causal ? u_own : vmax_nc;

    // Pair rows: the two lists [it, mid) and [mid, end) are walked together, smallest block first;
    // `act` says whose list names the block (bit 0: q-block 2u, bit 1: q-block 2u + 1).  The heads of
    // both lists are fetched one step before they are looked at.
    constexpr int kNoEntry = 0x7fffffff;
    int mid = 0, ia = 0, ib = 0, act = 0, act_next = 0;
    int ca_raw = 0, cb_raw = 0;                       // heads of the two lists as loaded (looked at a step later)
    bool active = true;                               // this wave computes in the current step
    auto pair_advance = [&](int* vout, int* actout) __attribute__((always_inline)) {
      // precondition: ia < mid or ib < end
      const int ca = ia < mid ? __builtin_amdgcn_readfirstlane(ca_raw) : kNoEntry;
      const int cb = ib < end ? __builtin_amdgcn_readfirstlane(cb_raw) : kNoEntry;
      const int vv = ca < cb ? ca : cb;
      const int aa = (ca == vv ? 1 : 0) | (cb == vv ? 2 : 0);
      if (aa & 1) {
        ++ia;
        if (ia < mid) ca_raw = col_idx[ia];
      }
      if (aa & 2) {
        ++ib;
        if (ib < end) cb_raw = col_idx[ib];
      }
      *vout = vv;
      *actout = aa;
    };
    if (kPair) {
      mid = __builtin_amdgcn_readfirstlane(row_ptr[(size_t)hq * N + 2 * u + 1]);
      mid = mid < it ? it : (mid > end ? end : mid);
      ia = it;
      ib = mid;
      if (ia < mid) ca_raw = col_idx[ia];
      if (ib < end) cb_raw = col_idx[ib];
      pair_advance(&v, &act);                          // has_work: at least one entry
      active = ((act >> sub) & 1) != 0;
    }

    // Q fragments (B operand of S^T = K Q^T): query row 32*wave + l32, dims 16*ks + 8*hf ..+7
    bf16x8 qf[KS];
    {
      const uint16_t* qp = q + (size_t)hq * hs.q + (size_t)min(qrow, L - 1) * D + hf * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    }
    async_load_k_tile<BLK, D, kPair>(krs, v * C::kTileBytes, lds_k, t);
    wait_async_loads();
    tile_barrier();

    f32x16 oacc[DT];
#pragma unroll
    for (int i = 0; i < DT; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY;          // running max, in units of log2: s * sm_scale
    float l_run = 0.f;                // this lane's share of the running sum
    int v_next = 0;

    // One step = one listed kv block.  kLast distinguishes the last step of the row: an ordinary
    // step starts the copy of the next K tile after its S^T phase, the last one pulls the queue.
    auto step = [&](auto last_tag) __attribute__((always_inline)) {
      constexpr bool kLast = decltype(last_tag)::value;
      if (kLast && t == 0) pulled_reg = atomicAdd(counter + my_queue, 1);

      // ---- V(j) -> LDS, in flight during S^T and the softmax ----
      async_load_vt_tile<BLK, D, kPair>(vrs, v * C::kTileBytes, lds_v, t);

      f32x16 sacc[KT];
      if (!kStreamOnly && active) {
      // ---- S^T = K Q^T ----
      // Flat software pipeline over the KT*KS (tile, k-step) pairs: the LDS read of step
      // i + kDepth is issued right after the MFMA of step i, in source order.
      const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      {
        constexpr int kSteps = KT * KS;
        constexpr int kSlab = 32 * D * 2;              // bytes of 32 key rows
        static_assert(kSteps >= kDepth, "pipeline deeper than the phase");
        bf16x8 fr[kDepth];
#pragma unroll
        for (int i = 0; i < kDepth; ++i)
          fr[i] = *reinterpret_cast<const bf16x8*>(lds_k + (i % KT) * kSlab + koff[i / KT]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
          const int kt = i % KT, ks = i / KT;          // consecutive MFMAs: independent accumulators
          sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kDepth], qf[ks], ks == 0 ? zero16 : sacc[kt], 0, 0, 0);
          if (i + kDepth < kSteps) {
            const int j = i + kDepth;
            fr[i % kDepth] = *reinterpret_cast<const bf16x8*>(lds_k + (j % KT) * kSlab + koff[j / KT]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }

      }

      // every wave is done reading K(j): K(j+1) can start now and land during softmax + PV
      tile_barrier();
      if (!kLast) async_load_k_tile<BLK, D, kPair>(krs, v_next * C::kTileBytes, lds_k, t);

      bf16x8 pf[KT][2];
      if (!kStreamOnly && active) {
      // ---- causal mask inside the diagonal block ----
      if (causal && v == u_own) {
        const int qloc = (wave % C::kRowWaves) * 32 + l32;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kloc = kt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (kloc > qloc) sacc[kt][r] = -INFINITY;
          }
      }

      // ---- keys past the end of the sequence (ragged last block) ----
      if (v == N - 1 && tail < BLK) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kloc = kt * 32 + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (kloc >= tail) sacc[kt][r] = -INFINITY;
          }
      }

      // ---- online softmax (per query = per lane pair l, l^32) ----
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kt][r]);
      mx = other_half_max(mx);
      const float m_new = fmaxf(m_run, mx * sm_scale);       // finite: every query sees a key
      if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) { // some query's max moved: rescale
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < DT; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
        m_run = m_new;
      }
      // p = 2^(s*scale - m) as bf16 pairs (the PV operand); the row sum adds the fp32 values with
      // plain adds: the dot-product instructions that would add the rounded pairs run on the
      // matrix pipe and stall behind the other workgroup's MFMAs (measured: 2.2x slower there).
      float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
          for (int j = 0; j < 8; j += 2) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[kt][8 * s + j], sm_scale, -m_new));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[kt][8 * s + j + 1], sm_scale, -m_new));
            const f32x2 pp = {p0, p1};
            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
            pf[kt][s][j] = pb[0];
            pf[kt][s][j + 1] = pb[1];
            psum0 += p0;
            psum1 += p1;
          }
        }
      }
      l_run += psum0 + psum1;

      }

      if (kLast) {
        if (t == 0) next_item = pulled_reg;         // the queue position pulled at the top of the step
        wait_async_loads();                          // this wave's share of V(j) has landed
      } else {
        wait_async_loads_but_last_tile<C::kPerThread>();   // ... while the younger loads of K(j+1) may still be in flight
      }
      tile_barrier();                                // V(j) complete

      if (kLast) {
        // the next row's queue entry, read through a per-lane (vector) address so that it arrives
        // on the vector-memory counter and is waited for after the PV phase; a scalar load would be
        // waited for by the very next LDS read
        int e_nxt = 0;
        kind_nxt = item_kind(__builtin_amdgcn_readfirstlane(next_item), seg_start, seg_len, &e_nxt);
        if (kind_nxt == kItemRow) item_nxt = items[e_nxt + lane_zero];
      }

      if (!kStreamOnly && active) {
      // ---- O^T += V^T P^T ----  (same flat pipeline over the DT*KT*2 (d-tile, k-step) pairs)
      {
        constexpr int kPer = KT * 2;                   // k-steps per d-tile
        constexpr int kSteps = DT * kPer;
        static_assert(kSteps >= kDepth, "pipeline deeper than the phase");
        bf16x8 fr[kDepth];
#pragma unroll
        for (int i = 0; i < kDepth; ++i)
          fr[i] = *reinterpret_cast<const bf16x8*>(lds_v + (i % DT) * (32 * BLK * 2) + voff[i / DT]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
          const int dt = i % DT, st = i / DT;          // consecutive MFMAs: independent accumulators
          oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kDepth], pf[st >> 1][st & 1], oacc[dt], 0, 0, 0);
          if (i + kDepth < kSteps) {
            const int j = i + kDepth;
            fr[i % kDepth] = *reinterpret_cast<const bf16x8*>(lds_v + (j % DT) * (32 * BLK * 2) + voff[j / DT]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }

      }

      wait_async_loads();              // this wave's share of K(j+1) (or the next row's entry) has landed
      tile_barrier();                  // K(j+1) complete; everyone is done reading V(j)
    };

    // The list is walked one entry ahead of its use: col_idx[it + 1] is requested here and
    // before the MFMA phases of every block, and read only after the waits that end the block,
    // so the latency of the index load is never on the critical path of a block.
    if (kPair) {
      for (;;) {
        if (ia >= mid && ib >= end) break;
        pair_advance(&v_next, &act_next);
        step(std::false_type{});
        v = v_next;
        act = act_next;
        active = ((act >> sub) & 1) != 0;
      }
      step(std::true_type{});
    } else {
    int ahead = it + 1 < end ? col_idx[it + 1] : -1;
    for (;;) {
      // next valid entry (v_next <= vmax): normally the entry fetched one block ago; entries
      // that must be skipped (negative or beyond vmax) take the slow path
      int nx = it + 1;
      v_next = __builtin_amdgcn_readfirstlane(ahead);
      if (nx < end && !(v_next >= 0 && v_next <= vmax)) {
        ++nx;
        while (nx < end) {
          v_next = __builtin_amdgcn_readfirstlane(col_idx[nx]);
          if (v_next >= 0 && v_next <= vmax) break;
          ++nx;
        }
      }
      if (nx >= end) break;
      ahead = nx + 1 < end ? col_idx[nx + 1] : -1;
      step(std::false_type{});
      it = nx;
      v = v_next;
    }
    step(std::true_type{});
    }

    // ---- epilogue: O = O^T / l, bf16, [q][d] ----
    const float l_tot = other_half_sum(l_run);
    const float inv_l = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    uint16_t* op = out + (size_t)hq * hs.q + (size_t)qrow * D;
    if (qrow < L) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int d0 = dt * 32 + gq * 8 + hf * 4;
          const f32x2 a = {oacc[dt][gq * 4 + 0] * inv_l, oacc[dt][gq * 4 + 1] * inv_l};
          const f32x2 b = {oacc[dt][gq * 4 + 2] * inv_l, oacc[dt][gq * 4 + 3] * inv_l};
          const bf16x2 ab = __builtin_convertvector(a, bf16x2);
          const bf16x2 bb = __builtin_convertvector(b, bf16x2);
          uint2 w;
          w.x = *reinterpret_cast<const uint32_t*>(&ab);
          w.y = *reinterpret_cast<const uint32_t*>(&bb);
          *reinterpret_cast<uint2*>(op + d0) = w;
        }
    }
    if (lse != nullptr && hf == 0 && qrow < L)
      lse[(size_t)hq * hs.lse + qrow] =
          l_tot > 0.f ? (m_run + log2f(l_tot)) * 0.6931471805599453f : -INFINITY;

    // ---- the row pulled in the last step becomes the current one ----
    kind_cur = kind_nxt;
    cur_x = __builtin_amdgcn_readfirstlane(item_nxt.x);
    cur_y = __builtin_amdgcn_readfirstlane(item_nxt.y);
    cur_z = __builtin_amdgcn_readfirstlane(item_nxt.z);
    cur_w = __builtin_amdgcn_readfirstlane(item_nxt.w);
  }
#endif
}

// =====================================================================================
// The same computation with 64 queries per wave (B = 128, whole blocks, clean lists): workgroup =
// 2 waves = one (q-head, q-block) row, one wave per SIMD, two workgroups per CU.  Every K / V^T
// fragment read from LDS feeds two MFMAs, K and V^T travel as 64-key half tiles through two LDS
// buffers each, and the row loop (software-pipelined over half-steps, softmax in the shadow of the
// neighbouring half-steps' MFMAs, accumulators and Q fragments in AGPRs) is a generated,
// hand-scheduled instruction sequence: prism_attn_w64_body.inc, written by gen_attn_w64.py, which
// also documents the register map and the pipeline.  This function supplies the persistent-workgroup
// loop around it: the same per-XCD queues as the general kernel.
// =====================================================================================
__global__ __launch_bounds__(128) void sparse_attn_w64_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt,
    const int32_t* __restrict__ col_idx, const int4* __restrict__ items, int32_t* __restrict__ plan,
    uint16_t* __restrict__ out, float* __restrict__ lse, int h, int h_kv, int L, int N, HeadStrides hs,
    int causal) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ __attribute__((aligned(1024))) char lds_tiles[65536];
  __shared__ int s_pulled, s_queue;
  if ((plan[kPlanFlags] & kFlagDirtyLists) != 0) return;    // the general kernel takes this call

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int g = h / h_kv;
  const int n_queues = gridDim.x < kXcds ? 1 : kXcds;
  int my_queue = blockIdx.x % n_queues;
  int seg_start = plan[kPlanStart + my_queue];
  int seg_len = plan[kPlanLen + my_queue];
  int32_t* counter = plan + kPlanCounter;
  const uint32_t lds_base = (uint32_t)(size_t)lds_tiles;
  const uint32_t k_bytes = (uint32_t)L * kHeadDim * 2;
  const uint32_t vt_bytes = (uint32_t)N * 128u * kHeadDim * 2;

  int pulled = 0;
  if (t == 0) pulled = atomicAdd(counter + my_queue, 1);
  for (;;) {
    // hand the pulled queue position to both waves
    __syncthreads();
    if (t == 0) s_pulled = pulled;
    __syncthreads();
    int pos = __builtin_amdgcn_readfirstlane(s_pulled);
    if (pos >= seg_len) {
      // Own queue exhausted: go on with rows of the nearest queue that still has some.  A pull
      // counter only grows, so a queue seen exhausted stays so; the atomic decides who gets a row.
      __syncthreads();
      if (wave == 0) {
        int found_pos = -1, found_queue = -1;
        for (;;) {
          int pulls = 0x7fffffff, len = 0;
          if (lane < n_queues) {
            pulls = __hip_atomic_load(counter + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            len = plan[kPlanLen + lane];
          }
          const unsigned long long open = __ballot(pulls < len);
          if (open == 0ull) break;
          int pick = -1;
          for (int s = 1; s <= n_queues && pick < 0; ++s) {
            const int x = (my_queue + s) % n_queues;
            if ((open >> x) & 1ull) pick = x;
          }
          int got = 0;
          if (lane == 0) got = atomicAdd(counter + pick, 1);
          got = __builtin_amdgcn_readfirstlane(got);
          if (got < plan[kPlanLen + pick]) {
            found_pos = got;
            found_queue = pick;
            break;
          }
        }
        if (lane == 0) {
          s_pulled = found_pos;
          s_queue = found_queue;
        }
      }
      __syncthreads();
      pos = __builtin_amdgcn_readfirstlane(s_pulled);
      const int nq = __builtin_amdgcn_readfirstlane(s_queue);
      if (nq < 0) break;                                    // every queue is exhausted
      my_queue = nq;
      seg_start = plan[kPlanStart + my_queue];
      seg_len = plan[kPlanLen + my_queue];
    }
    const int4 it0 = items[seg_start + pos];
    const int hq = __builtin_amdgcn_readfirstlane(it0.x);
    const int u = __builtin_amdgcn_readfirstlane(it0.y) & 0xffff;
    const int c_first = (__builtin_amdgcn_readfirstlane(it0.y) >> 16) & 0xffff;   // first listed block
    const int it = __builtin_amdgcn_readfirstlane(it0.z);
    const int end = __builtin_amdgcn_readfirstlane(it0.w);
    // The next row's queue position is pulled when this row is almost done (inside the row loop, at
    // the start of its last PV phase) and looked at after it: pulling at the start of a row would
    // reserve a row that its neighbours in the queue have long passed by the time it is started.

    const size_t tok0 = (size_t)u * 128 + (size_t)wave * 64;                    // this wave's first query
    const size_t row0 = (size_t)hq * hs.q + tok0 * kHeadDim;                     // its element offset in Q / O
    if (it >= end) {
      // a row without entries: o = 0, lse = -inf
      const int r = lane;                                   // 64 rows per wave, one per lane
      uint16_t* op = out + row0 + (size_t)r * kHeadDim;
#pragma unroll
      for (int c = 0; c < 16; ++c) *reinterpret_cast<uint4*>(op + c * 8) = make_uint4(0u, 0u, 0u, 0u);
      if (lse != nullptr) lse[(size_t)hq * hs.lse + tok0 + r] = -INFINITY;
      if (t == 0) pulled = atomicAdd(counter + my_queue, 1);
      continue;
    }
    const uint16_t* q_row = q + row0;
    uint16_t* o_row = out + row0;
    float* lse_row = lse != nullptr ? lse + (size_t)hq * hs.lse + tok0 : nullptr;
    const int kvh = hq / g;
    const uint16_t* k_head = k + (size_t)kvh * hs.kv;
    const uint16_t* vt_head = vt + (size_t)kvh * N * 128 * kHeadDim;
    const int32_t* col_row = col_idx + it;
    const int n_entries = end - it;
    int32_t* pull_counter = counter + my_queue;
    int pulled_next;
#include "prism_attn_w64_body.inc"
    if (t == 0) pulled = pulled_next;
  }
#endif
}

// One wave per row: does the row's list hold an entry the attention kernels must skip?
// With need_sorted (the pair kernel merges two lists) a list that is not strictly ascending counts too.
__global__ __launch_bounds__(256) void queue_validate_kernel(const int32_t* __restrict__ row_ptr,
                                                             const int32_t* __restrict__ col_idx, int h,
                                                             int N, int cap, int causal, int need_sorted,
                                                             const int32_t* __restrict__ range_flags,
                                                             int n_range_flags, int32_t* __restrict__ plan) {
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // values of V beyond the fp16 range (flagged per block by vt_image_kernel) also need the general kernel
  const int fi = blockIdx.x * 256 + threadIdx.x;
  if (fi < n_range_flags && range_flags[fi] != 0) atomicOr(plan + kPlanFlags, kFlagDirtyLists);
  if (r >= h * N) return;
  int b = row_ptr[r], e = row_ptr[r + 1];
  const bool clamped = b < 0 || b > cap || e < b || e > cap;
  b = b < 0 ? 0 : (b > cap ? cap : b);
  e = e < b ? b : (e > cap ? cap : e);
  const int vmax = causal ? r % N : N - 1;
  bool bad = clamped;
  for (int i = b + lane; i < e; i += 64) {
    const int v = col_idx[i];
    bad |= v < 0 || v > vmax;
    if (need_sorted && i + 1 < e) bad |= col_idx[i + 1] <= v;
  }
  if (__ballot(bad) != 0ull && lane == 0) atomicOr(plan + kPlanFlags, kFlagDirtyLists);
}

// =====================================================================================
// Work queues.  The rows (q-head, q-block) are put in the order
//     (phase, length class, q-head, q-block descending)
// and every (phase, class) group of that order is cut into one contiguous part per queue, the
// parts of a group holding equal work (listed blocks + one per row).  A queue is the sequence of
// its parts.  So each XCD walks neighbouring q-blocks of one q-head at a time, all XCDs go
// through the long rows of a phase first and its short rows last (no long row is started at the
// end of the call), and the queues hold equal work.
//   phase = kv head / heads_per_phase: the kv heads are taken a few at a time so that the K and
//       V^T of the heads in flight fit the 256 MB memory-side cache (at 128K tokens a kv head is
//       67 MB of K + V^T and all eight do not fit).
//   class: list length in (512, ..], (256, 512], (128, 256], ... (1, 2], [0, 1].
//   queue_count_kernel  (one workgroup per q-head): rows and work of the head per class.
//   queue_rank_kernel   (one workgroup per q-head): every row's rank in its group and its part,
//       and the number of rows of every (group, part).
//   queue_fill_kernel   (one thread per row): the row's position in its queue and its entry.
// =====================================================================================
// N = rows per head: q-blocks, or pairs of q-blocks (stride = 2: row r of the plan covers the two
// consecutive lists of q-blocks 2r and 2r + 1 of the index lists).
struct PlanCfg {
  int h, g, N, heads_per_phase, n_phases, n_queues, cap, causal, stride;
};
constexpr int kClasses = 11;
constexpr int kMaxGroups = 512;           // (phase, class) groups held in LDS by queue_fill_kernel

// class 0: more than 512 listed blocks, class c = 1 .. 9: (2^(9-c), 2^(10-c)], class 10: 0 or 1
__device__ __forceinline__ int length_class(int len) {
  if (len <= 1) return kClasses - 1;
  const int k = 31 - __builtin_clz(len - 1);           // len in (2^k, 2^(k+1)]
  return k > 9 ? 0 : 9 - k;
}

// list bounds of row r clamped to [0, cap] (and end >= begin)
__device__ __forceinline__ void row_bounds(const int32_t* __restrict__ row_ptr, int r, int cap, int stride,
                                           int* beg, int* end) {
  int b = row_ptr[(size_t)r * stride], e = row_ptr[(size_t)r * stride + stride];
  b = b < 0 ? 0 : (b > cap ? cap : b);
  e = e < b ? b : (e > cap ? cap : e);
  *beg = b;
  *end = e;
}

// bins = { rows[h][kClasses], work[h][kClasses] }; parts[n_phases][kClasses][8] is cleared here.
__global__ __launch_bounds__(256) void queue_count_kernel(const int32_t* __restrict__ row_ptr, PlanCfg c,
                                                          int32_t* __restrict__ bins,
                                                          int32_t* __restrict__ parts,
                                                          int32_t* __restrict__ plan) {
  __shared__ int s_rows[kClasses], s_work[kClasses];
  const int t = threadIdx.x, hq = blockIdx.x;
  if (t < kClasses) {
    s_rows[t] = 0;
    s_work[t] = 0;
  }
  for (int i = hq * 256 + t; i < c.n_phases * kClasses * 8; i += c.h * 256) parts[i] = 0;
  if (hq == 0 && t < kPlanInts - kPlanFlags) plan[kPlanFlags + t] = 0;
  __syncthreads();
  for (int u = t; u < c.N; u += 256) {
    int beg, end;
    row_bounds(row_ptr, hq * c.N + u, c.cap, c.stride, &beg, &end);
    const int cls = length_class(end - beg);
    atomicAdd(&s_rows[cls], 1);
    atomicAdd(&s_work[cls], end - beg + 1);
  }
  __syncthreads();
  if (t < kClasses) {
    bins[hq * kClasses + t] = s_rows[t];
    bins[(c.h + hq) * kClasses + t] = s_work[t];
  }
}

// row_rank[r] = rank of row r inside its (phase, class) group; row_part[r] = group * 8 + part.
__global__ __launch_bounds__(256) void queue_rank_kernel(const int32_t* __restrict__ row_ptr, PlanCfg c,
                                                         const int32_t* __restrict__ bins,
                                                         int32_t* __restrict__ parts,
                                                         int32_t* __restrict__ row_rank,
                                                         int32_t* __restrict__ row_part) {
  __shared__ int s_rows_before[kClasses];            // rows of the group in earlier heads
  __shared__ long long s_work_before[kClasses], s_work_total[kClasses];
  __shared__ int s_parts[kClasses * 8];
  __shared__ long long s_wave_total[kClasses][4];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, hq = blockIdx.x;
  const int phase = (hq / c.g) / c.heads_per_phase;
  if (t < kClasses) {
    s_rows_before[t] = 0;
    s_work_before[t] = 0;
    s_work_total[t] = 0;
  }
  __syncthreads();
  {
    const int h0 = phase * c.heads_per_phase * c.g;
    const int h1 = min(c.h, h0 + c.heads_per_phase * c.g);
    for (int i = t; i < (h1 - h0) * kClasses; i += 256) {
      const int hh = h0 + i / kClasses, k = i % kClasses;
      const int w = bins[(c.h + hh) * kClasses + k];
      if (hh < hq) {
        atomicAdd(&s_rows_before[k], bins[hh * kClasses + k]);
        atomicAdd(reinterpret_cast<unsigned long long*>(&s_work_before[k]), (unsigned long long)w);
      }
      atomicAdd(reinterpret_cast<unsigned long long*>(&s_work_total[k]), (unsigned long long)w);
    }
  }
  for (int i = t; i < kClasses * 8; i += 256) s_parts[i] = 0;

  // Thread t owns the rows i = t*per .. t*per + per - 1 of the head's order (q-block N-1-i).
  // Per class, rows and work of a thread travel through the scan as one number: work * 2^16 + rows
  // (a head has at most 2048 rows).
  const int per = (c.N + 255) / 256;
  long long mine[kClasses];
#pragma unroll
  for (int k = 0; k < kClasses; ++k) mine[k] = 0;
  for (int j = 0; j < per; ++j) {
    const int i = t * per + j;
    if (i >= c.N) break;
    int beg, end;
    row_bounds(row_ptr, hq * c.N + (c.N - 1 - i), c.cap, c.stride, &beg, &end);
    const int cls = length_class(end - beg);
    const long long add = ((long long)(end - beg + 1) << 16) + 1;
#pragma unroll
    for (int k = 0; k < kClasses; ++k) mine[k] += k == cls ? add : 0;
  }
  long long before[kClasses];                        // exclusive prefix over the threads
#pragma unroll
  for (int k = 0; k < kClasses; ++k) {
    long long incl = mine[k];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const long long y = __shfl_up(incl, off, 64);
      if (lane >= off) incl += y;
    }
    if (lane == 63) s_wave_total[k][wave] = incl;
    before[k] = incl - mine[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kClasses; ++k)
    for (int w = 0; w < wave; ++w) before[k] += s_wave_total[k][w];

  for (int j = 0; j < per; ++j) {
    const int i = t * per + j;
    if (i >= c.N) break;
    const int r = hq * c.N + (c.N - 1 - i);
    int beg, end;
    row_bounds(row_ptr, r, c.cap, c.stride, &beg, &end);
    const int cls = length_class(end - beg);
    const long long add = ((long long)(end - beg + 1) << 16) + 1;
    long long upto = 0;                              // this row included
#pragma unroll
    for (int k = 0; k < kClasses; ++k)
      if (k == cls) {
        before[k] += add;
        upto = before[k];
      }
    const int rank = (int)(upto & 0xffff) - 1;
    const long long w_incl = (upto >> 16) + s_work_before[cls];
    int x = 0;
    if (c.n_queues > 1) {
      x = (int)(((w_incl - 1) * c.n_queues) / s_work_total[cls]);
      x = x < 0 ? 0 : (x > c.n_queues - 1 ? c.n_queues - 1 : x);
    }
    row_rank[r] = s_rows_before[cls] + rank;
    row_part[r] = (phase * kClasses + cls) * 8 + x;
    atomicAdd(&s_parts[cls * 8 + x], 1);
  }
  __syncthreads();
  for (int i = t; i < kClasses * 8; i += 256)
    if (s_parts[i] > 0) atomicAdd(&parts[phase * kClasses * 8 + i], s_parts[i]);
}

// The thread of a row writes the row's queue entry: list bounds clamped to [0, cap], and the
// first entry that names a valid key block (0 <= v <= u for causal attention, 0 <= v < N
// otherwise).  Queue x holds, group after group, the rows of its part of the group; workgroup 0
// also writes the plan (segment starts and lengths, cleared pull counters).
__global__ __launch_bounds__(256) void queue_fill_kernel(const int32_t* __restrict__ row_ptr,
                                                         const int32_t* __restrict__ col_idx, PlanCfg c,
                                                         const int32_t* __restrict__ parts,
                                                         const int32_t* __restrict__ row_rank,
                                                         const int32_t* __restrict__ row_part,
                                                         int32_t* __restrict__ plan,
                                                         int4* __restrict__ items) {
  __shared__ int s_parts[kMaxGroups * 8];            // rows of (group, part)
  __shared__ int s_before[kMaxGroups * 8];           // rows of the same part in earlier groups
  __shared__ int s_start[8];
  const int t = threadIdx.x;
  const int n_groups = c.n_phases * kClasses;
  for (int i = t; i < n_groups * 8; i += 256) s_parts[i] = parts[i];
  __syncthreads();
  if (t < 8) {
    int run = 0;
    for (int gq = 0; gq < n_groups; ++gq) {
      s_before[gq * 8 + t] = run;
      run += s_parts[gq * 8 + t];
    }
    s_start[t] = run;                                // length of queue t, turned into its start below
  }
  __syncthreads();
  if (t == 0) {
    int start = 0;
    for (int x = 0; x < 8; ++x) {
      const int len = s_start[x];
      s_start[x] = start;
      if (blockIdx.x == 0) {
        plan[kPlanStart + x] = start;
        plan[kPlanLen + x] = len;
        plan[kPlanCounter + x] = 0;
      }
      start += len;
    }
  }
  __syncthreads();

  const int r = blockIdx.x * 256 + t;
  if (r >= c.h * c.N) return;
  const int hq = r / c.N, u = r - hq * c.N;
  const int gp = row_part[r], x = gp & 7;
  int in_earlier_parts = 0;
  for (int y = 0; y < x; ++y) in_earlier_parts += s_parts[(gp & ~7) + y];
  const int entry = s_start[x] + s_before[gp] + row_rank[r] - in_earlier_parts;
  int beg, end;
  row_bounds(row_ptr, r, c.cap, c.stride, &beg, &end);
  const int vmax = c.causal ? u : c.N - 1;
  int it = beg, v = 0;
  if (c.stride == 1) {
    while (it < end) {
      v = col_idx[it];
      if (v >= 0 && v <= vmax) break;
      ++it;
    }
    if (it >= end) v = 0;
  }                                                  // pair rows: clean lists, the kernel finds its first block
  if (entry >= 0 && entry < c.h * c.N) items[entry] = make_int4(hq, u | (v << 16), it, end);
}

}  // namespace prism

using namespace prism;

// ---- workspace layout: [ V image | items[h*N] (queue entries) | row_rank[h*N] | row_part[h*N] |
//                            bins[2*h*kClasses] | parts[h_kv*kClasses*8] | plan[24] ] ----
struct AttnWs {
  size_t image, items, row_rank, row_part, bins, parts, plan, image16, range_flags, pair_items, pair_plan, total;
};
// the fp16 image exists where the 64-queries-per-wave kernel can take the call
static bool w64_shape(const prism_params* p) {
  return p->block == 128 && p->head_dim == kHeadDim && p->seq_len % 128 == 0;
}

// B = 64 with an even number of blocks: a second plan over pairs of q-blocks for the pair kernel
static bool pair_shape(const prism_params* p) { return p->block == 64 && n_blocks(p) % 2 == 0; }

static AttnWs attn_ws(const prism_params* p) {
  const size_t N = n_blocks(p);
  const size_t rows = (size_t)p->n_q_heads * N;
  const size_t image_bytes = (size_t)p->n_kv_heads * N * p->block * p->head_dim * 2;
  AttnWs w;
  size_t off = 0;
  w.image = off;    off = align_up(off + image_bytes, 256);
  w.items = off;    off = align_up(off + rows * sizeof(int4), 256);
  w.row_rank = off; off = align_up(off + rows * sizeof(int32_t), 256);
  w.row_part = off; off = align_up(off + rows * sizeof(int32_t), 256);
  w.bins = off;     off = align_up(off + (size_t)2 * p->n_q_heads * kClasses * sizeof(int32_t), 256);
  w.parts = off;    off = align_up(off + (size_t)p->n_kv_heads * kClasses * 8 * sizeof(int32_t), 256);
  w.plan = off;     off = align_up(off + kPlanInts * sizeof(int32_t), 256);
  w.image16 = off;
  w.range_flags = off;
  if (w64_shape(p)) {
    off = align_up(off + image_bytes, 256);
    w.range_flags = off;
    off = align_up(off + (size_t)p->n_kv_heads * N * sizeof(int32_t), 256);
  }
  w.pair_items = off;
  w.pair_plan = off;
  if (pair_shape(p)) {
    off = align_up(off + rows / 2 * sizeof(int4), 256);
    w.pair_plan = off;
    off = align_up(off + kPlanInts * sizeof(int32_t), 256);
  }
  w.total = off;
  return w;
}

static int check_image(const prism_params* params, const void* img, size_t bytes) {
  if (img == nullptr || (reinterpret_cast<uintptr_t>(img) & 255u) != 0 ||
      bytes < attn_ws(params).total)
    return PRISM_ERR_WORKSPACE;
  return PRISM_OK;
}

// Facts about the device the calls run on, asked from the runtime once per device.
struct DeviceFacts {
  int cus;          // compute units
};
static int device_facts(DeviceFacts* out) {
  static std::mutex mu;
  static DeviceFacts facts[kMaxDevices];
  static bool known[kMaxDevices];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PRISM_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!known[dev]) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return PRISM_ERR_HIP;
    facts[dev].cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    known[dev] = true;
  }
  *out = facts[dev];
  return PRISM_OK;
}

// The memory-side cache holds 256 MB; the K and V^T of the kv heads that are in flight together are
// kept to kCacheBudgetBytes of it.
constexpr size_t kCacheBudgetBytes = (size_t)160 << 20;

static int persistent_grid(int rows, int wgs_per_cu) {
  DeviceFacts f;
  if (device_facts(&f) != PRISM_OK) return -1;
  const int resident = f.cus * wgs_per_cu;
  return rows < resident ? rows : resident;
}

extern "C" int prism_sparse_attn_workspace_bytes(const prism_params* params, size_t* bytes) {
  if (bytes == nullptr) return PRISM_ERR_INVALID_ARG;
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  *bytes = attn_ws(params).total;
  return PRISM_OK;
}

template <int BLK, int D>
static void launch_vt_image(const prism_params* p, const HeadStrides& hs, const uint16_t* v, uint16_t* vt,
                            uint16_t* vt16, int32_t* range_flags, hipStream_t st) {
  const int N = n_blocks(p);
  hipLaunchKernelGGL((vt_image_kernel<BLK, D>), dim3(N, p->n_kv_heads), dim3(256), 0, st, v, vt, p->seq_len, N,
                     hs.kv, vt16, range_flags);
}

static int v_image_core(const prism_params* params, const HeadStrides& hs, const void* v_bf16, char* ws,
                        hipStream_t st) {
  const AttnWs W = attn_ws(params);
  uint16_t* vt16 = w64_shape(params) ? reinterpret_cast<uint16_t*>(ws + W.image16) : nullptr;
  int32_t* range_flags = w64_shape(params) ? reinterpret_cast<int32_t*>(ws + W.range_flags) : nullptr;
  const uint16_t* v = (const uint16_t*)v_bf16;
  uint16_t* vt = reinterpret_cast<uint16_t*>(ws + W.image);
  if (params->block == 128) {
    if (params->head_dim == 64) launch_vt_image<128, 64>(params, hs, v, vt, vt16, range_flags, st);
    else if (params->head_dim == 128) launch_vt_image<128, 128>(params, hs, v, vt, vt16, range_flags, st);
    else launch_vt_image<128, 256>(params, hs, v, vt, vt16, range_flags, st);
  } else {
    if (params->head_dim == 64) launch_vt_image<64, 64>(params, hs, v, vt, vt16, range_flags, st);
    else if (params->head_dim == 128) launch_vt_image<64, 128>(params, hs, v, vt, vt16, range_flags, st);
    else launch_vt_image<64, 256>(params, hs, v, vt, vt16, range_flags, st);
  }
  return launch_status();
}

extern "C" int prism_v_image(const prism_params* params, const void* v_bf16, void* v_image,
                             size_t v_image_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  if (!v_bf16) return PRISM_ERR_INVALID_ARG;
  rc = check_image(params, v_image, v_image_bytes);
  if (rc != PRISM_OK) return rc;
  return v_image_core(params, contiguous_heads(params), v_bf16, static_cast<char*>(v_image),
                      static_cast<hipStream_t>(stream));
}

template <int BLK, bool kStreamOnly, int D, bool kPair = false>
static void launch_attn(int grid, hipStream_t st, const uint16_t* q, const uint16_t* k, const uint16_t* vt,
                        const int32_t* row_ptr, const int32_t* col_idx, const int4* items, int32_t* plan,
                        const int32_t* dirty_flag, uint16_t* out, float* lse, int h, int h_kv, int L, int N,
                        const HeadStrides& hs, int causal, int only_dirty) {
  hipLaunchKernelGGL((sparse_attn_kernel<BLK, kStreamOnly, D, kPair>), dim3(grid),
                     dim3(AttnCfg<BLK, D, kPair>::kThreads), 0, st, q, k, vt, row_ptr, col_idx, items, plan,
                     dirty_flag, out, lse, h, h_kv, L, N, hs, causal, only_dirty);
}

// the three kernels that turn index lists into the queue plan of `pc`
static void build_plan(const PlanCfg& pc, const int32_t* row_ptr, const int32_t* col_idx, int32_t* bins,
                       int32_t* parts, int32_t* row_rank, int32_t* row_part, int32_t* plan, int4* items,
                       hipStream_t st) {
  const int R = pc.h * pc.N;
  hipLaunchKernelGGL(queue_count_kernel, dim3(pc.h), dim3(256), 0, st, row_ptr, pc, bins, parts, plan);
  hipLaunchKernelGGL(queue_rank_kernel, dim3(pc.h), dim3(256), 0, st, row_ptr, pc, bins, parts, row_rank,
                     row_part);
  hipLaunchKernelGGL(queue_fill_kernel, dim3((R + 255) / 256), dim3(256), 0, st, row_ptr, col_idx, pc,
                     parts, row_rank, row_part, plan, items);
}

// Queue build + attention kernels of one sequence (arguments already validated).
static int attn_core(const prism_params* params, const HeadStrides& hs, const void* q_bf16, const void* k_bf16,
                     char* ws, const int32_t* row_ptr, const int32_t* col_idx, int64_t col_count,
                     void* out_bf16, float* lse, hipStream_t st) {
  const int N = n_blocks(params);
  const int h = params->n_q_heads, h_kv = params->n_kv_heads, L = params->seq_len, d = params->head_dim;
  const int R = h * N;
  const AttnWs W = attn_ws(params);
  int4* items = reinterpret_cast<int4*>(ws + W.items);
  int32_t* row_rank = reinterpret_cast<int32_t*>(ws + W.row_rank);
  int32_t* row_part = reinterpret_cast<int32_t*>(ws + W.row_part);
  int32_t* bins = reinterpret_cast<int32_t*>(ws + W.bins);
  int32_t* parts = reinterpret_cast<int32_t*>(ws + W.parts);
  int32_t* plan = reinterpret_cast<int32_t*>(ws + W.plan);
  // resident workgroups per CU, by the LDS the two tiles of a workgroup take (2 * B * d * 2 bytes of the
  // CU's 160 KB) and its waves: 2 at B = 128, d = 128 (64 KB, 4 waves); one when d = 256
  const int tile_pair = 2 * params->block * d * 2;
  int per_cu = (160 * 1024) / tile_pair;
  per_cu = per_cu > 4 ? 4 : per_cu;
  if (d > 128) per_cu = 1;
  else if (params->block == 128 && per_cu > 2) per_cu = 2;
  const int grid = persistent_grid(R, per_cu);
  if (grid <= 0) return PRISM_ERR_HIP;

  // queue plan: kv heads in phases that fit the memory-side cache
  PlanCfg pc;
  pc.h = h;
  pc.g = h / h_kv;
  pc.N = N;
  pc.n_queues = grid < kXcds ? 1 : kXcds;
  const size_t head_bytes = (size_t)L * d * 2 * 2;                        // K + V^T of one kv head
  pc.heads_per_phase = (int)(kCacheBudgetBytes / head_bytes) < 1 ? 1 : (int)(kCacheBudgetBytes / head_bytes);
  pc.n_phases = (h_kv + pc.heads_per_phase - 1) / pc.heads_per_phase;
  if (pc.n_phases * kClasses > kMaxGroups) {                               // very many kv heads: larger phases
    pc.n_phases = kMaxGroups / kClasses;
    pc.heads_per_phase = (h_kv + pc.n_phases - 1) / pc.n_phases;
    pc.n_phases = (h_kv + pc.heads_per_phase - 1) / pc.heads_per_phase;
  }
  pc.cap = col_count > 0x7fffffff ? 0x7fffffff : (int)col_count;     // CSR offsets are int32
  pc.causal = (params->flags & PRISM_FLAG_BIDIRECTIONAL) ? 0 : 1;
  pc.stride = 1;
  build_plan(pc, row_ptr, col_idx, bins, parts, row_rank, row_part, plan, items, st);
  const int causal = pc.causal;
  const bool stream_only = (params->flags & PRISM_FLAG_STREAM_ONLY) != 0;
  const uint16_t* qp = (const uint16_t*)q_bf16;
  const uint16_t* kp = (const uint16_t*)k_bf16;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(ws + W.image);
  uint16_t* op = (uint16_t*)out_bf16;
  // Whole blocks of 128 tokens go through the 64-queries-per-wave kernel when every list is clean
  // (decided on the device, so the general kernel is queued behind it and returns at once unless
  // the lists turn out to need it).
  const bool w64 = w64_shape(params) && !stream_only &&
                   !(params->flags & PRISM_FLAG_GENERAL_KERNEL);
  // B = 64 with an even number of blocks: the pair kernel (two q-blocks per workgroup sharing the tiles of
  // the union of their lists) takes the call when every list is ascending and clean; decided on the
  // device in the same way.
  // Below kPairMinRows rows the call is short and launch-bound, and the second plan and the list check
  // (four more launches) cost more than the shared tiles save (measured: 25 -> 42 us at 32 rows).
  // At d = 64 a tile is 8 KB and the plain kernel is not bound by its copies: the pair form is 5 % slower
  // even on all-ones lists, where the two lists of a pair coincide (750 -> 712 TFLOP/s at 16K tokens;
  // d = 128: 948 -> 993, d = 256: 438 -> 753).
  constexpr int kPairMinRows = 4096;
  const bool pair = pair_shape(params) && !stream_only && !(params->flags & PRISM_FLAG_GENERAL_KERNEL) &&
                    ((R >= kPairMinRows && d >= 128) || (params->flags & PRISM_FLAG_PAIR_KERNEL));
  const int only_dirty = (w64 || pair) ? 1 : 0;
  const int32_t* dirty_flag = plan + kPlanFlags;
  if (pair) {
    PlanCfg pp = pc;
    pp.N = N / 2;
    pp.stride = 2;
    const int pair_grid = persistent_grid(h * pp.N, d > 128 ? 1 : 2);       // 4 waves and 2 * 64 * d * 2 bytes of LDS each
    if (pair_grid <= 0) return PRISM_ERR_HIP;
    pp.n_queues = pair_grid < kXcds ? 1 : kXcds;
    int4* pair_items = reinterpret_cast<int4*>(ws + W.pair_items);
    int32_t* pair_plan = reinterpret_cast<int32_t*>(ws + W.pair_plan);
    build_plan(pp, row_ptr, col_idx, bins, parts, row_rank, row_part, pair_plan, pair_items, st);
    hipLaunchKernelGGL(queue_validate_kernel, dim3((R + 3) / 4), dim3(256), 0, st, row_ptr, col_idx, h, N,
                       pc.cap, causal, 1, static_cast<const int32_t*>(nullptr), 0, plan);
#define PRISM_PAIR(D)                                                                                        \
  launch_attn<64, false, D, true>(pair_grid, st, qp, kp, vp, row_ptr, col_idx, pair_items, pair_plan, dirty_flag, \
                                  op, lse, h, h_kv, L, N, hs, causal, 0)
    if (d == 64) PRISM_PAIR(64);
    else if (d == 128) PRISM_PAIR(128);
    else PRISM_PAIR(256);
#undef PRISM_PAIR
  }
  if (w64) {
    const int n_range_flags = h_kv * N;
    const int vgrid = ((R + 3) / 4) > ((n_range_flags + 255) / 256) ? (R + 3) / 4 : (n_range_flags + 255) / 256;
    hipLaunchKernelGGL(queue_validate_kernel, dim3(vgrid), dim3(256), 0, st, row_ptr, col_idx, h, N,
                       pc.cap, causal, 0, reinterpret_cast<const int32_t*>(ws + W.range_flags), n_range_flags, plan);
    hipLaunchKernelGGL(sparse_attn_w64_kernel, dim3(grid), dim3(128), 0, st, qp, kp,
                       reinterpret_cast<const uint16_t*>(ws + W.image16), col_idx, items, plan, op, lse, h, h_kv,
                       L, N, hs, causal);
  }
#define PRISM_ATTN(BLK, SO, D)                                                                                \
  launch_attn<BLK, SO, D>(grid, st, qp, kp, vp, row_ptr, col_idx, items, plan, dirty_flag, op, lse, h, h_kv, L, N, \
                          hs, causal, only_dirty)
  if (stream_only) {
    // measurement aid of the d = 128 kernels only
    if (d != 128) return PRISM_ERR_UNSUPPORTED;
    if (params->block == 128) PRISM_ATTN(128, true, 128);
    else PRISM_ATTN(64, true, 128);
  } else if (params->block == 128) {
    if (d == 64) PRISM_ATTN(128, false, 64);
    else if (d == 128) PRISM_ATTN(128, false, 128);
    else PRISM_ATTN(128, false, 256);
  } else {
    if (d == 64) PRISM_ATTN(64, false, 64);
    else if (d == 128) PRISM_ATTN(64, false, 128);
    else PRISM_ATTN(64, false, 256);
  }
#undef PRISM_ATTN
  return launch_status();
}

extern "C" int prism_sparse_attn_pre(const prism_params* params, const void* q_bf16,
                                     const void* k_bf16, void* v_image, size_t v_image_bytes,
                                     const int32_t* row_ptr, const int32_t* col_idx,
                                     int64_t col_count, void* out_bf16, float* lse, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16 || !row_ptr || !col_idx || !out_bf16 || col_count < 0)
    return PRISM_ERR_INVALID_ARG;
  rc = check_image(params, v_image, v_image_bytes);
  if (rc != PRISM_OK) return rc;
  return attn_core(params, contiguous_heads(params), q_bf16, k_bf16, static_cast<char*>(v_image), row_ptr,
                   col_idx, col_count, out_bf16, lse, static_cast<hipStream_t>(stream));
}

extern "C" int prism_sparse_attn(const prism_params* params, const void* q_bf16, const void* k_bf16,
                                 const void* v_bf16, const int32_t* row_ptr, const int32_t* col_idx,
                                 int64_t col_count, void* out_bf16, float* lse, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  int rc = check_params(params);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16 || !v_bf16 || !row_ptr || !col_idx || !out_bf16 || col_count < 0)
    return PRISM_ERR_INVALID_ARG;
  rc = check_image(params, workspace, workspace_bytes);
  if (rc != PRISM_OK) return rc;
  rc = prism_v_image(params, v_bf16, workspace, workspace_bytes, stream);
  if (rc != PRISM_OK) return rc;
  return prism_sparse_attn_pre(params, q_bf16, k_bf16, workspace, workspace_bytes, row_ptr, col_idx,
                               col_count, out_bf16, lse, stream);
}

// ---- packed variable-length batches: one sequence after the other on the stream ---------
extern "C" int prism_sparse_attn_varlen_workspace_bytes(const prism_params* params, const int32_t* cu_seqlens,
                                                        int n_seqs, size_t* bytes) {
  if (bytes == nullptr) return PRISM_ERR_INVALID_ARG;
  int rc = prism_varlen_layout(params, cu_seqlens, n_seqs, nullptr, nullptr, nullptr);
  if (rc != PRISM_OK) return rc;
  size_t need = 0;
  for (int s = 0; s < n_seqs; ++s) {
    prism_params ps = *params;
    ps.seq_len = cu_seqlens[s + 1] - cu_seqlens[s];
    const size_t b = attn_ws(&ps).total;
    need = b > need ? b : need;
  }
  *bytes = need;
  return PRISM_OK;
}

extern "C" int prism_sparse_attn_varlen(const prism_params* params, const int32_t* cu_seqlens, int n_seqs,
                                        const void* q_bf16, const void* k_bf16, const void* v_bf16,
                                        const int32_t* row_ptr, const int32_t* col_idx, void* out_bf16,
                                        float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  size_t need = 0;
  int rc = prism_sparse_attn_varlen_workspace_bytes(params, cu_seqlens, n_seqs, &need);
  if (rc != PRISM_OK) return rc;
  if (!q_bf16 || !k_bf16 || !v_bf16 || !row_ptr || !col_idx || !out_bf16) return PRISM_ERR_INVALID_ARG;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return PRISM_ERR_WORKSPACE;
  const size_t d = params->head_dim, T = params->seq_len;
  const HeadStrides hs{T * d, T * d, T};
  hipStream_t st = static_cast<hipStream_t>(stream);
  int64_t ro = 0, co = 0;
  for (int s = 0; s < n_seqs; ++s) {
    prism_params ps = *params;
    ps.seq_len = cu_seqlens[s + 1] - cu_seqlens[s];
    const int64_t N = n_blocks(&ps), h = ps.n_q_heads;
    const int64_t cap = (ps.flags & PRISM_FLAG_BIDIRECTIONAL) ? h * N * N : h * N * (N + 1) / 2;
    const size_t tok = (size_t)cu_seqlens[s];
    rc = v_image_core(&ps, hs, (const uint16_t*)v_bf16 + tok * d, static_cast<char*>(workspace), st);
    if (rc != PRISM_OK) return rc;
    rc = attn_core(&ps, hs, (const uint16_t*)q_bf16 + tok * d, (const uint16_t*)k_bf16 + tok * d,
                   static_cast<char*>(workspace), row_ptr + ro, col_idx + co, cap, (uint16_t*)out_bf16 + tok * d,
                   lse != nullptr ? lse + tok : nullptr, st);
    if (rc != PRISM_OK) return rc;
    ro += h * N + 1;
    co += cap;
  }
  return PRISM_OK;
}
