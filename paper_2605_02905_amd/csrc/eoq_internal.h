// Internal declarations shared by the host part (eoq_host.hip) and the kernel files (eoq_spectral.hip: Gram,
// eigensolvers, rank and shrinkage; eoq_mfma.hip: matrix-core encoder, decoder, TQ_prod; eoq_scores.hip: decode scoring; eoq_codec.hip:
// float32 encoder; eoq_factors.hip: 4-bit factors; eoq_attend.hip: softmax and attention output) of the
// eOptShrinkQ library.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "eoq.h"

constexpr int EOQ_D = 128;        // head dimension handled by the kernels
constexpr int EOQ_RMAX_CAP = 32;  // upper limit of r_max

struct eoq_ctx {
  int n = 0, d = 0, bits = 0, r_max = 0;
  int k = 0;              // pilot parameter of Alg. 2
  double rank_thr = 0.0;  // d^{-1/3}
  uint64_t seed = 0;
  int device = 0;
  std::vector<float> pi_host;    // [d][d], z = Pi u
  std::vector<float> cent_host;  // 2^bits centroids of N(0,1)
  std::vector<float> bnd_host;   // 2^bits - 1 midpoints
  float* d_pi = nullptr;         // device Pi   [c][j]
  float* d_pit = nullptr;        // device Pi^T [j][c]
  float* d_tab = nullptr;        // device: 16 centroids then 16 bounds (padded)
  uint16_t* d_pih = nullptr;     // device binary16: Pi hi [c][j], Pi lo [c][j], Pi^T hi [j][c], Pi^T lo [j][c]
  std::vector<float> phi_host;   // [d][d] Gaussian projection Phi of TQ_prod (Alg. 1 REQUIRE), float32
  float* d_phit = nullptr;       // device Phi^T [j][i]
  uint16_t* d_phih = nullptr;    // device binary16: Phi hi [i][j], Phi lo [i][j]
  std::string err;
  double gauss16[8] = {};  // Lloyd-Max magnitudes of N(0,1) at 16 levels: start of the per-block factor codebooks
  int loss = 0;    // eoq_loss: which case of Eq. (shrinkers) Alg. 2 Step 3 evaluates
  int solver = 0;  // 0: tridiagonal eigensolver with Jacobi for repeated eigenvalues, 1: Jacobi for every block
  // optional per-kernel timing: events [2*i], [2*i+1] bracket stage i (spectral, encode, decode, scores, attend,
  // softmax)
  bool profile = false;
  hipEvent_t ev[12] = {};
  bool ev_valid[6] = {false, false, false, false, false, false};
};

// Where the blocks of a batch sit in memory and which record slots they fill.  Input block b starts at element
// (b / group_size) * group_stride + (b % group_size) * block_stride, its token t at + t * token_stride; its
// record goes to slot out_first + b * out_stride.  Workspace arrays are always indexed by b.
struct EoqBlockMap {
  int64_t group_stride, block_stride, token_stride, out_first, out_stride;
  int32_t group_size;
  __host__ __device__ size_t in_base(size_t b) const {
    const unsigned g = (unsigned)b / (unsigned)group_size;
    return (size_t)g * (size_t)group_stride + (size_t)((unsigned)b - g * (unsigned)group_size) * (size_t)block_stride;
  }
  __host__ __device__ size_t slot(size_t b) const { return (size_t)out_first + b * (size_t)out_stride; }
};
inline EoqBlockMap eoq_dense_map(int n) { return EoqBlockMap{(int64_t)n * 128, 0, 128, 0, 1, 1}; }

// Device-side view of everything a launch needs.
struct EoqLaunch {
  EoqBlockMap map;
  int n, bits, r_max, k;
  double rank_thr;
  const float* pi;
  const float* pit;
  const float* tab;
  const uint16_t* pih;
  const float* phit;
  const uint16_t* phih;
  hipStream_t stream;
  const hipEvent_t* ev;  // null unless profiling
  int solver;
  int loss;
};

// Workspace layout for B blocks: lam[B][128] f64, then wfac[B][r_max][128] f32 (right singular vectors
// scaled by phi/sigma, the projection operand), then a counter (16 bytes) and a list of B block numbers
// (the blocks handed from the tridiagonal eigensolver to the Jacobi one), then, from the next 64-byte boundary,
// tri[B][128] pairs of doubles (the scaled tridiagonal matrix of every block, which the eigenvalue search reads
// back through the scalar cache: a block's 2 KB must not share a cache line with its neighbours').
inline size_t eoq_ws_lam_bytes(int64_t B) { return (size_t)B * EOQ_D * sizeof(double); }
inline size_t eoq_ws_wfac_bytes(int64_t B, int r_max) { return (size_t)B * r_max * EOQ_D * sizeof(float); }
inline size_t eoq_ws_list_bytes(int64_t B) { return 16 + (((size_t)B * sizeof(int) + 15) & ~(size_t)15); }
inline size_t eoq_ws_tri_bytes(int64_t B) { return B > 0 ? 64 + (size_t)B * EOQ_D * 2 * sizeof(double) : 0; }

hipError_t eoq_launch_spectral(const EoqLaunch& L, const void* blocks, int dtype, int64_t B, double* lam,
                               float* wfac, int* fb_count, int* fb_list, double* tri, eoq_packed out);
hipError_t eoq_launch_encode(const EoqLaunch& L, const void* blocks, int dtype, int64_t B, const float* wfac,
                             eoq_packed out);
hipError_t eoq_launch_encode_f16(const EoqLaunch& L, const void* blocks, int64_t B, const float* wfac,
                                 eoq_packed out, bool stored_factors = false);
hipError_t eoq_launch_factor_quant(const EoqLaunch& L, const void* blocks_fp16, int64_t B, const float* wfac,
                                   eoq_packed out, eoq_factor_codes fq, const double* gauss_levels);
hipError_t eoq_factor_quant_prepare();   // function attributes (dynamic LDS limits), once per device
hipError_t eoq_launch_factor_expand(const EoqLaunch& L, eoq_packed rec, eoq_factor_codes fq, int64_t B);
hipError_t eoq_launch_decode(const EoqLaunch& L, eoq_packed in, int64_t B, void* out_fp16);
// block_capacity / score_stride <= 0: the dense case (blocks_per_head slots per head, rows of blocks_per_head * n);
// tail_len > 0 adds the scores of the binary16 tail behind the blocks' scores
hipError_t eoq_launch_scores(const EoqLaunch& L, eoq_packed keys, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores,
                             int64_t block_capacity = 0, int64_t score_stride = 0, const void* tail_fp16 = nullptr,
                             int64_t tail_capacity = 0, int tail_len = 0);

// attention output on compressed values: number of partial-sum runs per (sequence, KV head) and the launches
int64_t eoq_attend_runs(int64_t sg_total, int64_t blocks_per_head, int* run_out);
hipError_t eoq_launch_attend(const EoqLaunch& L, eoq_packed values, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, int64_t block_capacity, const float* weights,
                             int64_t weight_stride, int n_q_heads, float* out, float* partial,
                             const void* tail_fp16 = nullptr, int64_t tail_capacity = 0, int tail_len = 0);
hipError_t eoq_launch_softmax(const EoqLaunch& L, float* x, int64_t rows, int64_t len, int64_t stride);

// TQ_prod side information of stored records and scores with the correction of Eq. (qjl)
hipError_t eoq_launch_qjl(const EoqLaunch& L, const void* blocks_fp16, int64_t B, eoq_packed rec, eoq_qjl out);
hipError_t eoq_launch_scores_prod(const EoqLaunch& L, eoq_packed keys, eoq_qjl qjl, int64_t n_seq, int n_kv_heads,
                                  int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores);
