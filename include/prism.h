/*
 * prism.h — C ABI of libprism: Prism block-importance estimation and block-sparse
 * causal prefill attention for AMD MI355X (gfx950).
 *
 * Section / equation names refer to "Prism: Spectral-Aware Block-Sparse Attention"
 * (arXiv 2602.08426).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HBM) owned by the caller, unless a
 *     parameter is explicitly marked "host".  The library never frees or keeps them.
 *   - Tensors are dense and contiguous:
 *        Q, O      : [n_q_heads , seq_len, head_dim]  bf16
 *        K, V      : [n_kv_heads, seq_len, head_dim]  bf16
 *     A batch is expressed by folding it into the head counts
 *     (n_q_heads = batch*h, n_kv_heads = batch*h_kv); q-head i reads kv-head
 *     i / (n_q_heads / n_kv_heads), which keeps the grouping inside each batch item.
 *   - RoPE has already been applied to Q and K; feature pair j is dims (2j, 2j+1)
 *     (Sec. 3.1 "Spectral Structure of RoPE"), so the high-frequency band is the
 *     FIRST d_high dims and the low-frequency band the LAST d_low dims (Sec. 3.4).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *     enqueue work; they return before it has run.  Outputs are valid after the
 *     stream has been synchronised.
 *   - Return value: PRISM_OK or a negative prism_status.  Arguments are validated on
 *     the host before anything is launched; on error nothing has been enqueued.
 *   - No entry point allocates device memory; scratch comes in through `workspace`
 *     (256-byte aligned) whose size the *_workspace_bytes calls report.
 */
#ifndef PRISM_H_
#define PRISM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum prism_status {
  PRISM_OK = 0,
  PRISM_ERR_INVALID_ARG = -1,     /* null pointer, inconsistent sizes, p outside (0,1], ... */
  PRISM_ERR_UNSUPPORTED = -2,     /* head_dim not in {64,128,256}, block not in {64,128}, more than 2048 blocks, ... */
  PRISM_ERR_WORKSPACE = -3,       /* workspace missing, misaligned or too small */
  PRISM_ERR_HIP = -4,             /* a HIP runtime call failed (launch error) */
  PRISM_ERR_TOO_LARGE = -5        /* prism_estimate_static: the problem needs more scratch than the
                                     library's static array holds */
} prism_status;

/* flags */
#define PRISM_FLAG_NO_CALIBRATION 1u   /* tau_high = tau_low = 1 (ablation of Sec. 4.4) */
#define PRISM_FLAG_BIDIRECTIONAL  2u   /* no causal restriction (the video-generation setting of
                                          Sec. 4.2 "Main Results"): every row may select any of
                                          the N key blocks and attends to every token of a
                                          listed block */
#define PRISM_FLAG_FORCE_DIAGONAL 4u   /* extra, not in the paper: block u of row u is always selected */
#define PRISM_FLAG_FORCE_SINK     8u   /* extra, not in the paper: block 0 is always selected */
#define PRISM_FLAG_GENERAL_KERNEL 0x20000000u /* measurement aid for prism_sparse_attn(_pre): always
                                          use the general attention kernel (32 queries per wave, one
                                          q-block per workgroup), also where the 64-queries-per-wave
                                          kernel (B = 128) or the pair kernel (B = 64) would take the call */
#define PRISM_FLAG_PAIR_KERNEL 0x10000000u /* measurement and test aid for prism_sparse_attn(_pre) at B = 64:
                                          use the pair kernel wherever the shape allows it (an even number
                                          of blocks), also for problems too small for it to pay */
#define PRISM_FLAG_STREAM_ONLY 0x40000000u /* measurement aid for prism_sparse_attn(_pre): run the
                                          kernel's K / V^T tile copies, waits and scheduling without
                                          its arithmetic; the outputs are then meaningless.  Shows how
                                          long the memory side of a call takes on its own.  Head dim
                                          128 only (PRISM_ERR_UNSUPPORTED otherwise). */

/* Problem description shared by all calls (plain data, host memory). */
typedef struct prism_params {
  int32_t n_q_heads;    /* h   (batch folded in)                                   */
  int32_t n_kv_heads;   /* h_kv, must divide n_q_heads                             */
  int32_t seq_len;      /* L; the last block may be ragged (holds L mod B tokens)   */
  int32_t head_dim;     /* d: 64, 128 or 256                                        */
  int32_t block;        /* B, 64 or 128; N = ceil(L / B) blocks, N <= 2048          */
  int32_t d_high;       /* width of the high-frequency band, 0..d (0 = band off)    */
  int32_t d_low;        /* width of the low-frequency band,  0..d (0 = band off)    */
  float   top_p;        /* p in (0,1]; p >= 1 selects every admissible block        */
  uint32_t flags;       /* PRISM_FLAG_*                                              */
} prism_params;

/* A band as up to PRISM_MAX_SEGMENTS slices [start, start+width) of the head dim; the band
 * vector is their concatenation and d_z their total width.  One slice per band gives the
 * contiguous bands of Sec. 3.4; several give the axis-wise bands of App. "HunyuanVideo
 * Spectral Configuration" (first d_high^a / last d_low^a dims of each axis subspace), or the
 * bands of RoPE stored as pairs (j, j + d/2): high = [0, d_high/2) + [d/2, d/2 + d_high/2).
 * Slices of one band must not overlap; the two bands may.  n_segments = 0 switches a band off. */
#define PRISM_MAX_SEGMENTS 8
typedef struct prism_band {
  int32_t n_segments;
  int32_t start[PRISM_MAX_SEGMENTS];
  int32_t width[PRISM_MAX_SEGMENTS];
} prism_band;
typedef struct prism_bands {
  prism_band high, low;
} prism_bands;

/* Library version as major*10000 + minor*100 + patch. */
int prism_version(void);

/* Static, human-readable text for a status code (host pointer, never NULL). */
const char* prism_status_string(int status);

/* ------------------------------------------------------------------------------------
 * Block importance estimation — Sec. 3.4 "Prism: Spectral-Aware Block Selection" and
 * App. C "Top-P Block Selection".
 *
 * Computes, per q-head:  mean-pooled Qbar, Kbar (Eq. "mean-pooling"; a ragged last block is
 * averaged over the tokens it holds);  RMS energies of
 * the full / high / low slices;  tau_z = sqrt(d_z/d) (RMS(Qbar_z)/RMS(Qbar))
 * (RMS(Kbar_z)/RMS(Kbar));  logits_z = Qbar_z Kbar_z^T / (tau_z sqrt(d_z)) for key
 * blocks v <= u (block-causal; every v with PRISM_FLAG_BIDIRECTIONAL);  row softmax;
 * top-p (smallest set of highest-probability blocks whose mass reaches p; equal
 * probabilities are taken in ascending block order);
 * M = M_high | M_low;  and the compacted per-(head, q-block) index lists of M.
 * A band with d_z == 0 is skipped.  Zero band energy gives flat logits.
 *
 * Outputs
 *   mask_bits : [n_q_heads, N, W] uint64, W = ceil(N/64); bit (v % 64) of word v / 64 of
 *               row (head, u) is M[u, v].  Fully overwritten.
 *   row_ptr   : [n_q_heads*N + 1] int32, CSR row offsets, row index = head*N + u.
 *   col_idx   : [col_capacity] int32, selected key blocks of each row in ascending order.
 *               n_q_heads*N*(N+1)/2 entries always suffice (n_q_heads*N*N when bidirectional).
 *   info      : [4] int32: info[0] = number of selected (head,u,v) triples,
 *               info[1] = 1 if that number exceeds col_capacity (col_idx then holds only
 *               the entries that fit and must not be used), info[2..3] reserved (0).
 * workspace: prism_estimate_workspace_bytes() bytes.
 * ---------------------------------------------------------------------------------- */
int prism_estimate_workspace_bytes(const prism_params* params, size_t* bytes /* host, out */);

int prism_estimate(const prism_params* params,
                   const void* q_bf16, const void* k_bf16,
                   uint64_t* mask_bits, int32_t* row_ptr,
                   int32_t* col_idx, int64_t col_capacity,
                   int32_t* info,
                   void* workspace, size_t workspace_bytes, void* stream);

/* prism_estimate with the bands given as slice lists (host memory); d_high and d_low of
 * `params` are ignored.  prism_estimate(params, ...) is this call with
 * high = {[0, d_high)}, low = {[d - d_low, d)}. */
int prism_estimate_bands(const prism_params* params, const prism_bands* bands /* host */,
                         const void* q_bf16, const void* k_bf16,
                         uint64_t* mask_bits, int32_t* row_ptr,
                         int32_t* col_idx, int64_t col_capacity,
                         int32_t* info,
                         void* workspace, size_t workspace_bytes, void* stream);

/* prism_estimate for callers that cannot allocate device memory or pass a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, outputs and results as prism_estimate, bit for bit, but the scratch is a
 * 16 MiB device array inside the library (one copy per GPU, held until the process ends;
 * its address is looked up on the first call on each device, which allocates nothing).
 * Returns PRISM_ERR_TOO_LARGE, with nothing enqueued, when
 * prism_estimate_workspace_bytes(params) exceeds 16 MiB (16 777 216 bytes; the Llama-shaped
 * layer fits up to 32K tokens at B = 128).  The call allocates nothing.  All calls on one GPU
 * share that GPU's array: calls that overlap there (different streams or threads) race and
 * must be serialised by the caller; calls in a row on one stream are fine, nothing needs
 * clearing between them. */
int prism_estimate_static(const prism_params* params,
                          const void* q_bf16, const void* k_bf16,
                          uint64_t* mask_bits, int32_t* row_ptr,
                          int32_t* col_idx, int64_t col_capacity,
                          int32_t* info, void* stream);

/* ------------------------------------------------------------------------------------
 * Estimation fused with the producer of the post-RoPE tensors.
 *
 * q_in / k_in hold the vectors BEFORE the rotary embedding.  Feature pair j = dims (2j, 2j+1)
 * of token n is rotated by the angle (position_offset + n) * theta_j, theta_j = base^(-2j/d)
 * (Sec. 3.1 "Spectral Structure of RoPE"):
 *      x' = x cos(a) - y sin(a),   y' = x sin(a) + y cos(a),
 * rounded to bf16 and written to q_out / k_out (same layouts; q_out may be q_in and k_out may be
 * k_in: the rotation is then done in place).  The same pass pools the rounded values, so the
 * masks and lists are exactly those prism_estimate_bands(q_out, k_out) would give, without
 * reading the tensors a second time.  With yarn_native_len != 0 the frequencies follow the
 * NTK-by-parts map of App. "Compatibility with YaRN":
 *      theta'_j = (1 - gamma_j) theta_j / yarn_scale + gamma_j theta_j,
 *      gamma_j = clamp((r_j - yarn_alpha) / (yarn_beta - yarn_alpha), 0, 1),
 *      r_j = yarn_native_len * theta_j / (2 pi).
 * The angle is formed and reduced in double precision; cos and sin are evaluated in fp32.
 * `bands` may be NULL (the bands of params->d_high / d_low).  Outputs, workspace and errors as
 * for prism_estimate; additionally PRISM_ERR_INVALID_ARG for base <= 1, a negative position
 * offset, yarn_scale < 1 or yarn_beta <= yarn_alpha.
 * ---------------------------------------------------------------------------------- */
typedef struct prism_rope {
  double  base;              /* b                                                        */
  int32_t position_offset;   /* position of token 0                                      */
  int32_t yarn_native_len;   /* L of r_j; 0 = plain RoPE (the yarn_* fields are ignored) */
  double  yarn_scale;        /* s >= 1                                                   */
  double  yarn_alpha;        /* 1 in the paper                                           */
  double  yarn_beta;         /* 32 in the paper                                          */
} prism_rope;

int prism_rope_estimate(const prism_params* params, const prism_rope* rope /* host */,
                        const prism_bands* bands /* host, may be NULL */,
                        const void* q_in_bf16, const void* k_in_bf16,
                        void* q_out_bf16, void* k_out_bf16,
                        uint64_t* mask_bits, int32_t* row_ptr,
                        int32_t* col_idx, int64_t col_capacity,
                        int32_t* info,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Same computation as prism_estimate up to the block scores, for inspection at small
 * sizes: writes the pooled vectors, the two scales sqrt(d_z)*tau_z and the dual-band
 * logits (Sec. 3.4, step "Dual-Band Scoring").  Any output pointer may be NULL.
 *   pooled_q : [n_q_heads , N, d] float      pooled_k : [n_kv_heads, N, d] float
 *   scales   : [n_q_heads, 2] float (high, low); 0 when the band is disabled
 *   logits_high, logits_low : [n_q_heads, N, N] float; entries with v > u are not written
 *                             (all N*N are written with PRISM_FLAG_BIDIRECTIONAL)
 * Uses the same workspace size as prism_estimate. */
int prism_block_scores(const prism_params* params,
                       const void* q_bf16, const void* k_bf16,
                       float* pooled_q, float* pooled_k, float* scales,
                       float* logits_high, float* logits_low,
                       void* workspace, size_t workspace_bytes, void* stream);

/* prism_block_scores with the bands given as slice lists (see prism_estimate_bands). */
int prism_block_scores_bands(const prism_params* params, const prism_bands* bands /* host */,
                             const void* q_bf16, const void* k_bf16,
                             float* pooled_q, float* pooled_k, float* scales,
                             float* logits_high, float* logits_low,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Compaction of a caller-supplied block mask (same layouts and `info` semantics as
 * prism_estimate; the mask -> index-list step that block-sparse kernels need,
 * Sec. 3.1 "Coarse-grained Attention": the mask decides which pairs (u,v) are computed).
 * Bits with v >= N must be 0.  Needs no workspace. */
int prism_mask_to_csr(const prism_params* params, const uint64_t* mask_bits,
                      int32_t* row_ptr, int32_t* col_idx, int64_t col_capacity,
                      int32_t* info, void* stream);

/* Index lists of the all-ones causal mask (dense attention as the special case M = 1):
 * row (head,u) = {0..u}.  col_capacity must be >= n_q_heads*N*(N+1)/2. */
int prism_causal_csr(const prism_params* params, int32_t* row_ptr, int32_t* col_idx,
                     int64_t col_capacity, void* stream);

/* Index lists of the all-ones mask under params->flags: as prism_causal_csr, or every row =
 * {0..N-1} with PRISM_FLAG_BIDIRECTIONAL (col_capacity >= n_q_heads*N*N). */
int prism_dense_csr(const prism_params* params, int32_t* row_ptr, int32_t* col_idx,
                    int64_t col_capacity, void* stream);

/* ------------------------------------------------------------------------------------
 * Block-sparse causal attention — Sec. 2 "Block-Sparse Attention": the dense
 * computation and online accumulation restricted to the selected block pairs.
 *
 * For token i of q-block u = i / B of head hq:
 *    J(i) = { j <= i : block j / B is listed in row (hq,u) },
 *    o_i  = sum_{j in J} softmax_J( q_i . k_j / sqrt(d) )_j  v_j       (bf16 in, fp32 accumulate)
 * Listed blocks v > u are ignored; a row with an empty list gives o = 0, lse = -inf.
 * With PRISM_FLAG_BIDIRECTIONAL the condition j <= i is dropped: J(i) is every token of every
 * listed block v < N.
 *
 *   row_ptr, col_idx : CSR as produced above; col_count = number of valid entries in
 *                      col_idx (row_ptr values are clamped to it).
 *   out_bf16         : [n_q_heads, L, d] bf16, fully overwritten.
 *   lse              : [n_q_heads, L] float natural-log sum-exp of the scaled scores, or NULL.
 * workspace: prism_sparse_attn_workspace_bytes() bytes (a transposed copy of V plus the
 *            kernel's work queues: one entry per row, ordered by list-length class and
 *            q-head and dealt to the eight XCDs in parts of equal work).
 * top_p, d_high, d_low and the other flags of `params` are ignored here.
 * ---------------------------------------------------------------------------------- */
int prism_sparse_attn_workspace_bytes(const prism_params* params, size_t* bytes /* host, out */);

int prism_sparse_attn(const prism_params* params,
                      const void* q_bf16, const void* k_bf16, const void* v_bf16,
                      const int32_t* row_ptr, const int32_t* col_idx, int64_t col_count,
                      void* out_bf16, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream);

/* The two halves of prism_sparse_attn, for callers that reuse one V image for several
 * attention calls (or time the attention kernel alone):
 *   prism_v_image          : writes the transposed, block-tiled copy of V that the attention
 *                            kernel reads into `v_image` (prism_sparse_attn_workspace_bytes()
 *                            bytes, 256-byte aligned).
 *   prism_sparse_attn_pre  : same computation and arguments as prism_sparse_attn, with the
 *                            image in place of V.  The tail of the same buffer (beyond the
 *                            image) is scratch for the kernel's work queue and is rewritten
 *                            by every call, so calls sharing one image must not overlap.
 * prism_sparse_attn(...) == prism_v_image(..., workspace) ; prism_sparse_attn_pre(..., workspace). */
int prism_v_image(const prism_params* params, const void* v_bf16, void* v_image,
                  size_t v_image_bytes, void* stream);

int prism_sparse_attn_pre(const prism_params* params,
                          const void* q_bf16, const void* k_bf16,
                          void* v_image, size_t v_image_bytes,
                          const int32_t* row_ptr, const int32_t* col_idx, int64_t col_count,
                          void* out_bf16, float* lse, void* stream);

/* ------------------------------------------------------------------------------------
 * Packed variable-length batches — the batch axis of Sec. 3.4 (Fig. "PyTorch-style
 * implementation of Prism" carries a leading batch dimension) for sequences of unequal length.
 *
 * The batch is stored without padding: Q, O are [n_q_heads, T, d], K, V are [n_kv_heads, T, d],
 * lse is [n_q_heads, T]; sequence s owns tokens cu_seqlens[s] .. cu_seqlens[s+1]-1 of the T
 * axis.  params->seq_len = T = cu_seqlens[n_seqs]; cu_seqlens is a HOST array of n_seqs + 1
 * strictly increasing offsets starting at 0.  Every sequence is a problem of its own, exactly
 * as if prism_estimate / prism_sparse_attn were called on its slice: own blocks (the first
 * block of a sequence starts at its first token, N_s = ceil(L_s / B) <= 2048), own RMS
 * statistics, own causal structure, own index lists.  The limits on N apply per sequence, not
 * to T.
 *
 * Outputs of the sequences lie one behind the other; prism_varlen_layout gives the start of
 * each (arrays of n_seqs + 1 int64 on the HOST, last entry = total; any may be NULL):
 *   mask_offsets : in uint64 words; sequence s holds [n_q_heads, N_s, ceil(N_s/64)] words
 *   row_offsets  : in int32;        sequence s holds n_q_heads*N_s + 1 row offsets, which start
 *                                   at 0 and index the sequence's own part of col_idx
 *   col_offsets  : in int32;        sequence s holds room for all its admissible pairs
 *                                   (n_q_heads*N_s*(N_s+1)/2, or n_q_heads*N_s*N_s when bidirectional)
 *   info         : [4 * n_seqs] int32, four per sequence as in prism_estimate (never overflows)
 * The sequences are processed one after the other on `stream` and share the workspace
 * (prism_*_varlen_workspace_bytes: the largest single sequence's need), so a batch of many
 * short sequences costs one set of kernel launches per sequence.
 * Errors: PRISM_ERR_INVALID_ARG for malformed offsets, PRISM_ERR_UNSUPPORTED if a sequence
 * exceeds the per-sequence limits; nothing is launched in either case.
 * ---------------------------------------------------------------------------------- */
int prism_varlen_layout(const prism_params* params, const int32_t* cu_seqlens /* host */, int n_seqs,
                        int64_t* mask_offsets, int64_t* row_offsets, int64_t* col_offsets /* host, out */);

int prism_estimate_varlen_workspace_bytes(const prism_params* params, const int32_t* cu_seqlens /* host */,
                                          int n_seqs, size_t* bytes /* host, out */);

int prism_estimate_varlen(const prism_params* params, const int32_t* cu_seqlens /* host */, int n_seqs,
                          const void* q_bf16, const void* k_bf16,
                          uint64_t* mask_bits, int32_t* row_ptr, int32_t* col_idx, int32_t* info,
                          void* workspace, size_t workspace_bytes, void* stream);

int prism_sparse_attn_varlen_workspace_bytes(const prism_params* params, const int32_t* cu_seqlens /* host */,
                                             int n_seqs, size_t* bytes /* host, out */);

int prism_sparse_attn_varlen(const prism_params* params, const int32_t* cu_seqlens /* host */, int n_seqs,
                             const void* q_bf16, const void* k_bf16, const void* v_bf16,
                             const int32_t* row_ptr, const int32_t* col_idx,
                             void* out_bf16, float* lse,
                             void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H_ */
