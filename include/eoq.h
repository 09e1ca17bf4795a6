/*
 * eoq.h -- C ABI of the eOptShrinkQ KV-cache block compression library for
 * AMD MI355X (gfx950).
 *
 * One "block" is n consecutive key (or value) vectors of one attention head,
 * a row-major n x d matrix (paper Sec. 2.3 last paragraph: the cache is cut
 * into blocks of n tokens, each processed independently; Alg. 3 takes one
 * block).  A batch is B blocks stored back to back, [B][n][d].
 *
 * Every pointer argument is documented as HOST or DEVICE.  Device buffers are
 * owned by the caller (e.g. torch tensors); the library allocates device
 * memory only in eoq_create (rotation and codebook tables) and frees it in
 * eoq_destroy.  The hot calls (eoq_compress*, eoq_expand_factors, eoq_qjl_encode,
 * eoq_decompress, eoq_scores*, eoq_softmax, eoq_attend*) launch kernels on the
 * given HIP stream and return without synchronising; they never allocate and can
 * be captured into a HIP graph (with the profiling of eoq_profile off).
 * All device pointers must be 16-byte aligned.  Functions return EOQ_OK or an
 * error code; they never abort.  A human-readable reason for the last failure
 * is kept per context (eoq_last_error).
 */
#ifndef EOQ_H_
#define EOQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eoq_ctx eoq_ctx;

typedef enum {
  EOQ_OK = 0,
  EOQ_ERR_ARG = 1,          /* null / misaligned pointer, negative size */
  EOQ_ERR_UNSUPPORTED = 2,  /* (n, d, bits, r_max, head grouping) outside the supported set */
  EOQ_ERR_WORKSPACE = 3,    /* workspace smaller than eoq_workspace_bytes() */
  EOQ_ERR_HIP = 4           /* a HIP runtime call failed */
} eoq_status;

typedef enum { EOQ_F16 = 0, EOQ_F32 = 1 } eoq_dtype;

/* Loss whose optimal shrinker Alg. 2 Step 3 evaluates (Eq. (shrinkers)); the paper's experiments use the first. */
typedef enum { EOQ_LOSS_FROBENIUS = 0, EOQ_LOSS_OPERATOR = 1, EOQ_LOSS_NUCLEAR = 2 } eoq_loss;

/* Flag bits of eoq_packed.flags[b]. */
#define EOQ_FLAG_RANK_CLAMPED 1u /* estimated rank exceeded r_max and was cut to r_max */
#define EOQ_FLAG_SHRINK_GUARD 2u /* a D-transform estimate was degenerate; that component got phi = 0 */
#define EOQ_FLAG_NO_CONVERGE  4u /* the eigensolver hit its sweep limit or produced a non-finite vector */
#define EOQ_FLAG_NONFINITE    16u /* the block holds an Inf or NaN entry: it is stored with rank 0, its other outputs are meaningless */
#define EOQ_FLAG_SWEEPS_SHIFT 8  /* bits 8..15: Jacobi sweeps run on this block (0: tridiagonal solver) (diagnostic) */

/*
 * The compressed record of a batch (Alg. 3, "Store": shrunken SVD factors of
 * the r^+ retained components, TQ indices and norms of the residual).  All
 * members are DEVICE pointers, caller-owned.
 *
 *   codes [B][n][bits*d/8]  per token `bits` bit-planes of d/8 bytes; plane p
 *                           holds bit p of the d code indices, coordinate j in
 *                           bit (j mod 8) of byte j/8.  Index 0 is the most
 *                           negative centroid (Alg. 1 line 5).
 *   norms [B][n]            binary16 bit patterns of the residual row norms
 *                           (Alg. 1 line 3; Remark 3.1: one FP16 norm per row).
 *   rank  [B]               r^+ of Alg. 2 Step 1, clamped to r_max.
 *   phi   [B][r_max]        shrunk singular values (Alg. 2 Step 3), first r^+ valid.
 *   sigma [B][r_max]        observed singular values of the same components.
 *   lfac  [B][r_max][n]     binary16 U diag(phi), one row per component
 *                           (Alg. 2 Return); only the first r^+ rows are written.
 *   rfac  [B][r_max][d]     binary16 right singular vectors, same convention.
 *   flags [B]               EOQ_FLAG_* bits.
 */
typedef struct {
  uint8_t*  codes;
  uint16_t* norms;
  int32_t*  rank;
  float*    phi;
  float*    sigma;
  uint16_t* lfac;
  uint16_t* rfac;
  uint32_t* flags;
} eoq_packed;

/*
 * SVD factors at 4 bits (Alg. 3 line 3 with b_s = 4; Sec. 3.1: data-adaptive Lloyd-Max codebooks, shrunk
 * singular values in binary16).  All members are DEVICE pointers, caller-owned.  Per block and factor matrix
 * the codebook is {+-m_0 .. +-m_7} (eight binary16 magnitudes fitted to the |entries| of that matrix); a code
 * is 3 bits of magnitude index plus the sign in bit 3 (set for x >= 0); two codes per byte, entry e in the low
 * (e even) or high nibble of byte e/2.
 *
 *   lcodes [B][r_max][n/2]  codes of the left singular vectors U (unit columns), one row per component.
 *   rcodes [B][r_max][d/2]  codes of the right singular vectors V.
 *   fbook  [B][2][8]        binary16 magnitudes: [0] for U, [1] for V.
 *   phi16  [B][r_max]       binary16 shrunk singular values.
 * Only the first r^+ rows of a block are written.  The record's lfac / rfac then hold what these codes expand
 * to, binary16(U_hat phi16) and V_hat: a cache that eoq_expand_factors rebuilds from the codes.
 */
typedef struct {
  uint8_t*  lcodes;
  uint8_t*  rcodes;
  uint16_t* fbook;
  uint16_t* phi16;
} eoq_factor_codes;

/*
 * TQ_prod side information of B blocks (Alg. 1 lines "TQ_prod": the norm of the quantisation residual and the signs
 * of its Gaussian projection).  DEVICE pointers, caller-owned, 16-byte aligned.
 *   signs [B][n][d/8]  bit (j mod 8) of byte j/8 of a token's row is set when (Phi r_x)_j >= 0 (sign(0) = +1);
 *   norms [B][n]       binary16 |r_x|.
 * One more bit per entry and 16/d for the norm (Alg. 1 last line counts b + 1 + 16/d).
 */
typedef struct {
  uint8_t*  signs;
  uint16_t* norms;
} eoq_qjl;

/*
 * Create a context for blocks of n x d, `bits` residual bits per entry (Alg. 3
 * REQUIRE), a Haar rotation drawn from `rot_seed` (Alg. 1 REQUIRE: one rotation
 * shared by all vectors) and at most r_max stored components per block.
 * Builds on the host, in double precision, the rotation (QR of a seeded
 * Gaussian matrix, R's diagonal made positive) and the Lloyd-Max codebook of
 * N(0,1) (Sec. 2.2 item 3; used scaled by 1/sqrt(d)), and uploads both to the
 * current HIP device.
 * Supported: d = 128; n a multiple of 128 with 128 <= n <= 4096; bits in 1..4;
 * 1 <= r_max <= 32.  On failure *out is NULL.  When the process sees no HIP
 * device the context is created host-only: eoq_rotation / eoq_codebook work,
 * the three hot calls return EOQ_ERR_HIP.
 */
eoq_status eoq_create(eoq_ctx** out, int n, int d, int bits, uint64_t rot_seed, int r_max);
void       eoq_destroy(eoq_ctx* ctx);

/* Pilot parameter k = floor(d^c), c = min(1/2.01, 1/log log d) of Alg. 2 (11 at d = 128). */
int        eoq_pilot_k(int d);

/* Bytes of DEVICE scratch eoq_compress needs for B blocks. */
size_t     eoq_workspace_bytes(const eoq_ctx* ctx, int64_t B);

/* Copy the rotation Pi (row-major [d][d], z = Pi u) into HOST memory, as the float32 table the kernels use. */
eoq_status eoq_rotation(const eoq_ctx* ctx, float* host_out);

/* Copy the Gaussian projection Phi of TQ_prod (Alg. 1 REQUIRE; iid N(0,1) drawn from rot_seed + 1 and rounded to
 * binary16, row-major [d][d], w = Phi r) into HOST memory, as float32 values of the binary16 table the kernels use. */
eoq_status eoq_projection(const eoq_ctx* ctx, float* host_out);

/* Copy the N(0,1) codebook into HOST memory: 2^bits ascending centroids and 2^bits-1 midpoints (float32). */
eoq_status eoq_codebook(const eoq_ctx* ctx, float* host_centroids, float* host_bounds);

/*
 * Alg. 3 on B blocks: eOptShrink (Alg. 2: eigen-decomposition of the d x d Gram
 * matrix, bulk edge and rank, imputed noise spectrum, D-transform shrinker),
 * residual against the stored binary16 factors (the whole block when r^+ = 0),
 * then TQ_MSE per residual row (Alg. 1 lines 3-5) and bit-packing.
 *   blocks     DEVICE, [B][n][d] of `dtype` (binary16 or float32), read only.
 *   out        DEVICE buffers as described at eoq_packed; fully overwritten
 *              except lfac/rfac rows >= rank[b].
 *   workspace  DEVICE, >= eoq_workspace_bytes(ctx, B) bytes.  After the call
 *              completes its first B*d doubles hold every block's Gram
 *              eigenvalues sigma_i^2 in descending order (diagnostic: the
 *              retained ones and the next are resolved to rounding level,
 *              the others to within 1e-9 of the largest).
 *   hip_stream hipStream_t (NULL = default stream).
 */
eoq_status eoq_compress(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B,
                        eoq_packed out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * eoq_compress for callers that cannot allocate device memory or hand in a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation): the same kernels on the same arguments, with the workspace
 * in a 16 MiB array that is part of the library's device image (one copy per GPU, held until the process ends).
 * The call allocates nothing, frees nothing and does not synchronise.
 *   B          at most eoq_static_max_blocks(ctx) (861 blocks at r_max = 32, 2339 at r_max = 8); more blocks:
 *              EOQ_ERR_WORKSPACE, nothing is launched.
 *   blocks, dtype, out, hip_stream   as eoq_compress; the record is bit-identical to eoq_compress's.
 * The diagnostic eigenvalues of eoq_compress stay inside the library.  Every call on a GPU, from any context, uses
 * that GPU's one array and leaves its contents behind (the call clears what must start at zero itself): two calls
 * that overlap in time on one GPU (different streams, or replays of graphs that contain them) race; calls on one
 * stream, or ordered by events, are safe.
 */
int64_t    eoq_static_max_blocks(const eoq_ctx* ctx);
eoq_status eoq_compress_static(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_packed out,
                               void* hip_stream);

/*
 * eoq_compress with the SVD factors stored at 4 bits (see eoq_factor_codes): the residual is taken against
 * the expanded 4-bit factors (closed loop), which are also left in out.lfac / out.rfac.  binary16 blocks only
 * (dtype must be EOQ_F16) and n * r_max <= 32768 (the left vectors of a block are fitted in LDS), otherwise
 * EOQ_ERR_UNSUPPORTED.  Everything else as eoq_compress.
 */
eoq_status eoq_compress_q4(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_packed out,
                           eoq_factor_codes fq, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Placement of a batch that is not stored block after block: chunk-at-a-time compression while a cache is being
 * filled (Sec. 3.1: blocks of 128 tokens compressed as soon as they are complete; Sec. 5: chunked prefill), with
 * the keys or values in the layout the model produced them in, written into a record store that is laid out for
 * scoring ([tensor][block]).  Strides are in ELEMENTS of the input dtype.
 *   input block b starts at  (b / in_group_size) * in_group_stride + (b % in_group_size) * in_block_stride,
 *   its token t at           + t * in_token_stride            (d contiguous entries per token),
 *   its record goes to slot  out_first + b * out_stride       of every array of the eoq_packed / eoq_factor_codes.
 * Example: a chunk of n tokens of L tensors [L][n][H][d] (token-major, H heads interleaved), records
 * [L*H][blocks_per_tensor], chunk number c:  {n*H*d, H, d, H*d, c, blocks_per_tensor}.
 * Input strides must be multiples of 8, in_token_stride >= d, in_group_size >= 1, out_first >= 0, out_stride >= 1.
 */
typedef struct {
  int64_t in_group_stride;
  int32_t in_group_size;
  int64_t in_block_stride;
  int64_t in_token_stride;
  int64_t out_first;
  int64_t out_stride;
} eoq_chunk_layout;

/*
 * eoq_compress (fq == NULL) or eoq_compress_q4 (fq != NULL) on B blocks placed by `lay`.  `out` and `fq` hold the
 * BASE pointers of the whole record store; only the slots `lay` names are written, and the caller guarantees that
 * they exist and are distinct.  The workspace is indexed by b (eoq_workspace_bytes(ctx, B) bytes), its first B*d
 * doubles hold the eigenvalues of input block b.  Results are bit-identical to the dense calls on the same blocks.
 */
eoq_status eoq_compress_chunk(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_chunk_layout lay,
                              eoq_packed out, const eoq_factor_codes* fq, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/*
 * Rebuild rec.lfac / rec.rfac (rows below rec.rank[b]) from the 4-bit codes, codebooks and phi16 of `fq`, e.g.
 * after loading a record that was stored without them.  Reads rec.rank, writes rec.lfac and rec.rfac.
 */
eoq_status eoq_expand_factors(eoq_ctx* ctx, eoq_packed rec, eoq_factor_codes fq, int64_t B, void* hip_stream);

/*
 * Inverse of eoq_compress: x_hat_t = rho_t Pi^T z_hat_t + (U diag(phi) V^T)[t,:]
 * (Alg. 1 line 6 plus the low-rank part), rounded to binary16.
 *   in        DEVICE record of B blocks, read only.
 *   out_fp16  DEVICE, [B][n][d] binary16, overwritten.
 */
eoq_status eoq_decompress(eoq_ctx* ctx, eoq_packed in, int64_t B, void* out_fp16, void* hip_stream);

/*
 * Attention logits on compressed keys without materialising them (Sec. 2.1,
 * Remark 6.5): scores[s][h][t] = <q[s][h], x_hat_t> / sqrt(d), split into the
 * low-rank term and rho_t <Pi q, z_hat_t>.
 *   keys             DEVICE record of n_seq*n_kv_heads*blocks_per_head blocks;
 *                    block j of KV head g of sequence s is at index
 *                    (s*n_kv_heads + g)*blocks_per_head + j.
 *   q_fp16           DEVICE, [n_seq][n_q_heads][d] binary16.  Query head h
 *                    reads KV head h / (n_q_heads / n_kv_heads).
 *   scores           DEVICE, [n_seq][n_q_heads][blocks_per_head*n] float32, overwritten.
 * Supported: n_q_heads a multiple of n_kv_heads with group size 1..8.
 */
eoq_status eoq_scores(eoq_ctx* ctx, eoq_packed keys, int64_t n_seq, int n_kv_heads,
                      int64_t blocks_per_head, const void* q_fp16, int n_q_heads,
                      float* scores, void* hip_stream);

/*
 * eoq_scores over a cache that is still being filled (Sec. 3.1 / Sec. 7: blocks are compressed as they complete, the
 * newest fewer-than-n tokens of every head wait uncompressed in binary16): the record store has room for
 * block_capacity blocks per (sequence, KV head), of which the first blocks_filled are valid, and the tail buffer
 * holds tail_len valid tokens per head.
 *   keys       DEVICE record store, block j of KV head g of sequence s at slot (s*n_kv_heads + g)*block_capacity + j.
 *   tail_fp16  DEVICE, [n_seq][n_kv_heads][tail_capacity][d] binary16; may be NULL when tail_len = 0.
 *   scores     DEVICE, [n_seq][n_q_heads][score_stride] float32: entries 0 .. blocks_filled*n - 1 of a row are the
 *              blocks' tokens, the next tail_len entries <q, tail token>/sqrt(d); the rest of the row is untouched.
 * blocks_filled <= block_capacity, tail_len <= tail_capacity, tail_len < n, score_stride >= blocks_filled*n + tail_len.
 * Everything else as eoq_scores.
 */
eoq_status eoq_scores_stream(eoq_ctx* ctx, eoq_packed keys, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                             int64_t blocks_filled, const void* tail_fp16, int64_t tail_capacity, int64_t tail_len,
                             const void* q_fp16, int n_q_heads, float* scores, int64_t score_stride,
                             void* hip_stream);

/*
 * TQ_prod for stored records (Alg. 1 lines "TQ_prod" where Alg. 3 applies TurboQuant, i.e. on the residual rows):
 * r_x = S_t - x_hat_t with x_hat the reconstruction of `rec` (what eoq_decompress returns before its rounding),
 * out.norms = binary16(|r_x|), out.signs = sign(Phi r_x).  Call after eoq_compress* on the same blocks.
 *   blocks_fp16  DEVICE, [B][n][d] binary16, the blocks `rec` was made from.  rec is read only.
 */
eoq_status eoq_qjl_encode(eoq_ctx* ctx, const void* blocks_fp16, int64_t B, eoq_packed rec, eoq_qjl out,
                          void* hip_stream);

/*
 * eoq_scores with the unbiased inner-product estimator of Eq. (qjl): every logit gets
 * |r_x| sqrt(pi/2)/d <Phi q, sign(Phi r_x)> / sqrt(d) added.  `qjl` holds the side information of the same blocks, in
 * the same order as `keys`.  Everything else as eoq_scores.
 */
eoq_status eoq_scores_prod(eoq_ctx* ctx, eoq_packed keys, eoq_qjl qjl, int64_t n_seq, int n_kv_heads,
                           int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores,
                           void* hip_stream);

/*
 * Attention weights: softmax over each of `rows` rows of `len` float32 logits, in place (Sec. 2.1, the softmax of
 * Attention(Q, K, V); the row maximum is subtracted first).  scores is DEVICE memory, row r at scores + r*row_stride,
 * row_stride >= len.
 */
eoq_status eoq_softmax(eoq_ctx* ctx, float* scores, int64_t rows, int64_t len, int64_t row_stride, void* hip_stream);

/*
 * Attention output on compressed values without materialising them (Sec. 2.1 with V replaced by its
 * reconstruction; the split of Remark 6.5 applied to the values): out[s][h] = sum_t weights[s][h][t] x_hat_t over
 * the tokens of the first blocks_filled blocks of KV head h / (n_q_heads / n_kv_heads) of sequence s.
 *   values         DEVICE record store, block j of KV head g of sequence s at slot (s*n_kv_heads + g)*block_capacity + j.
 *   weights        DEVICE, [n_seq][n_q_heads][weight_stride] float32 (e.g. eoq_softmax of eoq_scores' output); entry
 *                  j*n + t of a row weighs token t of block j.  weight_stride >= blocks_filled*n.
 *   out            DEVICE, [n_seq][n_q_heads][d] float32, overwritten.
 *   workspace      DEVICE, >= eoq_attend_workspace_bytes(ctx, n_seq, n_kv_heads, blocks_filled) bytes (partial sums;
 *                  they are added in a fixed order: the result does not depend on scheduling).
 * Supported group sizes as eoq_scores.  blocks_filled = 0 writes zeros.
 */
size_t     eoq_attend_workspace_bytes(const eoq_ctx* ctx, int64_t n_seq, int n_kv_heads, int64_t blocks_per_head);
eoq_status eoq_attend(eoq_ctx* ctx, eoq_packed values, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                      int64_t blocks_filled, const float* weights, int64_t weight_stride, int n_q_heads, float* out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * eoq_attend over a cache that is still being filled (see eoq_scores_stream): the uncompressed binary16 tail values
 * [n_seq][n_kv_heads][tail_capacity][d] contribute sum_t weights[s][h][blocks_filled*n + t] tail[s][g][t] for
 * t < tail_len, so a weight row covers the blocks' tokens and then the tail, exactly as eoq_scores_stream lays the
 * logits out.  tail_len < n, tail_len <= tail_capacity, weight_stride >= blocks_filled*n + tail_len; tail_fp16 may
 * be NULL when tail_len = 0.  Everything else as eoq_attend.
 */
eoq_status eoq_attend_stream(eoq_ctx* ctx, eoq_packed values, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                             int64_t blocks_filled, const void* tail_fp16, int64_t tail_capacity, int64_t tail_len,
                             const float* weights, int64_t weight_stride, int n_q_heads, float* out, void* workspace,
                             size_t workspace_bytes, void* hip_stream);

/*
 * Eigensolver used by eoq_compress for the d x d Gram matrix (the paper only asks for the SVD of the
 * block, Alg. 2 REQUIRE).  0 (default): Householder tridiagonalisation + Sturm multisection + twisted
 * factorisation, with blocks whose retained eigenvalues are numerically repeated handed to the Jacobi
 * solver; 1: LDS-resident one-sided Jacobi for every block.  Both give the same record up to rounding.
 */
eoq_status eoq_set_solver(eoq_ctx* ctx, int solver);

/*
 * Loss function L of Alg. 2 (REQUIRE, Step 3): which case of Eq. (shrinkers) turns the D-transform estimates d, a_1,
 * a_2 of a retained component into its shrunk singular value: Frobenius d sqrt(a_1 a_2) (default; Remark 3.1),
 * operator norm d sqrt(min(a_1, a_2) / max(a_1, a_2)), nuclear norm d (sqrt(a_1 a_2) - sqrt((1 - a_1)(1 - a_2))).
 * For the last two the overlap estimates are clipped to [0, 1] first; every result is clipped to [0, sigma_i], so a
 * component whose nuclear-norm value would be negative is stored with phi = 0.  Rank, eigenvalues and vectors do not
 * depend on the loss.  Applies to the eoq_compress* calls that follow.  Other values: EOQ_ERR_UNSUPPORTED.
 */
eoq_status eoq_set_loss(eoq_ctx* ctx, eoq_loss loss);

/*
 * Per-kernel timing for benchmarks (not part of the paper's method).  With profiling enabled every
 * hot call records HIP events on its stream around each kernel it launches; eoq_stage_ms waits for
 * those events and returns the duration, in milliseconds, of the kernels of the most recent
 * eoq_compress* (out[0] spectral, out[1] encode, with the factor fit of eoq_compress_q4), eoq_decompress (out[2]),
 * eoq_scores* (out[3]), eoq_attend (out[4]) and eoq_softmax (out[5]); a stage that has not run since profiling was
 * enabled reports -1.  `out` is HOST memory, 6 floats.
 * Events are created by eoq_profile, never inside a hot call.
 */
eoq_status eoq_profile(eoq_ctx* ctx, int enable);
eoq_status eoq_stage_ms(eoq_ctx* ctx, float* out);

/*
 * Measured ceilings of the device, for benchmark reports (not part of the paper's method): runs one micro-benchmark
 * and waits for it.  kind 0: plain copy of the first half of `device_buf` onto its second half (16-byte accesses;
 * the memory streams of kinds 0, 6 and 7 walk whole chunks of 32 KB per workgroup and leave a shorter rest alone);
 * 1: independent double-precision FMA chains on the vector ALUs; 2 / 3 / 4: chains of the matrix instructions the
 * kernels use (f16 32x32x16, i8 16x16x64, f64 16x16x4); 5: 32-bit vector instructions; 6 / 7: read-only / write-only
 * stream over `device_buf`; 10..15: two of these streams
 * side by side on the two waves of every SIMD (10: f64 matrix + f64 FMA, 11: i8 matrix + 32-bit vector, 12: f64 matrix
 * + 32-bit vector, 13: f64 FMA + 32-bit vector, 14: f16 matrix + f64 FMA, 15: i8 matrix + f64 FMA); 21 / 23 / 24 / 25:
 * stream 1 / 3 / 4 / 5 on one wave per SIMD only; 31..34 / 41..44: the f64 FMA / 32-bit vector stream on 1..4 waves
 * per SIMD (the first wave's work in out[1], the others' in out[2]).  `iters` is the loop count per wave (kinds >= 1).
 *   device_buf  DEVICE scratch, 16-byte aligned, buf_bytes >= 64 KB (kind 0 moves buf_bytes/2 in each direction).
 *   out         HOST, 4 doubles: milliseconds of one launch; work of the first stream (bytes moved for kind 0, flops
 *               or integer operations, wave instructions for the 32-bit vector stream); work of the second stream;
 *               compute units of the device.
 * Allocates two events, runs on the default stream and synchronises: not a hot call.
 */
eoq_status eoq_ceiling(eoq_ctx* ctx, int kind, void* device_buf, size_t buf_bytes, int iters, double* out);

/* Reason for the last error on this context (HOST string owned by the context); "" if none. */
const char* eoq_last_error(const eoq_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* EOQ_H_ */
