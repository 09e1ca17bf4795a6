// Spectral stage of eOptShrinkQ (Alg. 2) on gfx950, one workgroup of 256 lanes per block, double precision:
// Gram matrix G = S^T S, its eigenvalues (= squared singular values of the block, Sec. 2.3), bulk edge and
// rank (Step 1), imputed noise spectrum (Step 2), D-transform shrinker (Step 3) and the right singular
// vectors of the retained components.
//
// Two eigensolvers produce the same outputs:
//   tridiagonal : Householder reduction of G with the matrix held in registers, all eigenvalues by
//                 Sturm-sequence multisection, the few retained eigenvectors by twisted factorisation of
//                 the tridiagonal matrix and back-transformation through the stored reflectors.
//   jacobi      : one-sided Jacobi on the columns of G, resident in LDS.  It takes the blocks whose retained
//                 eigenvalues are (numerically) repeated, where single-vector iterations do not give an
//                 orthogonal basis, and can be selected for every block.
#include <type_traits>

#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;

// ---------------------------------------------------------------------------------------------
// Gram matrix of one block into a per-lane 8x8 tile: lane (ty, tx) = (tid/16, tid%16) accumulates
// G[ty*8+i][tx*8+j] in acc[i*8+j].  `stage` holds 32 rows of the block as float.
// ---------------------------------------------------------------------------------------------
constexpr int STAGE_ROWS = 32;

__device__ __forceinline__ void gram_tile(const void* __restrict__ blocks, int dtype, size_t base_elem, size_t tok, int n,
                                          float* stage, int tid, double (&acc)[64]) {
  const int ty = tid >> 4, tx = tid & 15;
  EOQ_SFOR(i, 64, acc[i] = 0.0;);
  for (int t0 = 0; t0 < n; t0 += STAGE_ROWS) {
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int e = (g * THREADS + tid) * 8;
      float v[8];
      load8(blocks, dtype, base_elem + (size_t)(t0 + (e >> 7)) * tok + (e & (D - 1)), v);
#pragma unroll
      for (int i = 0; i < 8; ++i) stage[e + i] = v[i];
    }
    __syncthreads();
    for (int t = 0; t < STAGE_ROWS; ++t) {
      double a[8], b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[i] = (double)stage[t * D + ty * 8 + i];
        b[i] = (double)stage[t * D + tx * 8 + i];
      }
      EOQ_SFOR(e, 64, acc[e] = fma(a[e >> 3], b[e & 7], acc[e]););
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Alg. 2 Steps 1-3 from the eigenvalues lam_s[0..127] (descending, in LDS, visible to all lanes).
// Writes lam_out / phi / sigma for the block, fills atoms[] and scale_s[] (phi_i / sigma_i), sets flag
// bits, returns the (clamped) rank to every lane.  Must be called by all 256 lanes.
// ---------------------------------------------------------------------------------------------
__device__ int rank_and_shrink(const double* lam_s, double* atoms, double* scale_s, unsigned* flag_s, int n, int k,
                               double rank_thr, int r_max, int loss, size_t blk, size_t slot, double* __restrict__ lam_out,
                               float* __restrict__ phi_out, float* __restrict__ sigma_out) {
  const int tid = threadIdx.x;
  if (tid < D) lam_out[blk * D + tid] = lam_s[tid];

  // Step 1: lambda_+ = lam_{k+1} + (lam_{k+1} - lam_{2k+1}) / (2^{2/3} - 1);  r = #{ lam_i / lambda_+ - 1 > d^{-1/3} }
  const double edge_coef = 1.0 / (cbrt(4.0) - 1.0);
  const double lam_k1 = lam_s[k], lam_2k1 = lam_s[2 * k];
  const double lam_plus = lam_k1 + edge_coef * (lam_k1 - lam_2k1);
  const int above = (tid < D) ? ((lam_s[tid] / lam_plus - 1.0 > rank_thr) ? 1 : 0) : 0;
  int r = __syncthreads_count(above);
  if (*flag_s & EOQ_FLAG_NONFINITE) r = 0;   // Inf or NaN in the block (set by the Gram stage, before several barriers)
  if (r > r_max) {
    r = r_max;
    if (tid == 0) atomicOr(flag_s, EOQ_FLAG_RANK_CLAMPED);
  }

  // Step 2: the r outliers are dropped, the next k eigenvalues are re-drawn from the square-root edge law
  const int M = D - r;
  if (tid < M) {
    double v;
    if (tid < k) {
      const double a = lam_s[k + r], b = lam_s[2 * k + r];
      const double j = (double)(tid + 1);
      v = a + (1.0 - pow(j / (double)k, 2.0 / 3.0)) * edge_coef * (a - b);
    } else {
      v = lam_s[r + tid];
    }
    atoms[tid] = v;
  }
  __syncthreads();

  // Step 3: Stieltjes transforms of the noise measure at each outlier, D-transform, shrinker of the chosen loss
  {
    const int wave = tid >> 6, lane = tid & 63;
    const double beta = (n >= D) ? (double)D / (double)n : (double)n / (double)D;
    for (int i = wave; i < r; i += THREADS / 64) {
      const double z = lam_s[i];
      double s1 = 0.0, s2 = 0.0;
      for (int j = lane; j < M; j += 64) {
        const double inv = 1.0 / (atoms[j] - z);
        s1 += inv;
        s2 = fma(inv, inv, s2);
      }
      s1 = wave_sum_shfl(s1);
      s2 = wave_sum_shfl(s2);
      if (lane == 0) {
        // m_s: transform of the d x d Gram side; m_l: the n x n side, which has n - d more zero eigenvalues
        const double m_s = s1 / (double)M, dm_s = s2 / (double)M;
        const double m_l = beta * m_s - (1.0 - beta) / z;
        const double dm_l = beta * dm_s + (1.0 - beta) / (z * z);
        const double T = z * m_s * m_l;
        const double dT = m_s * m_l + z * dm_s * m_l + z * m_s * dm_l;
        const double sig = sqrt(fmax(z, 0.0));
        double phi = 0.0;
        bool ok = isfinite(T) && isfinite(dT) && T > 0.0 && dT < 0.0;
        if (ok) {
          // d = T^{-1/2}, a_x = m_x / (d^2 T'); Eq. (shrinkers): Frobenius d sqrt(a_1 a_2), operator
          // d sqrt(min(a)/max(a)), nuclear d (sqrt(a_1 a_2) - sqrt((1 - a_1)(1 - a_2))), the overlaps clipped to [0, 1]
          // before the last two take their roots
          const double dh = 1.0 / sqrt(T);
          const double a1 = m_l / (dh * dh * dT), a2 = m_s / (dh * dh * dT);
          if (loss == EOQ_LOSS_FROBENIUS) {
            phi = dh * sqrt(a1 * a2);
          } else {
            ok = isfinite(a1) && isfinite(a2);
            const double c1 = fmin(fmax(a1, 0.0), 1.0), c2 = fmin(fmax(a2, 0.0), 1.0);
            if (loss == EOQ_LOSS_OPERATOR) {
              const double hi = fmax(c1, c2);
              phi = (hi > 0.0) ? dh * sqrt(fmin(c1, c2) / hi) : 0.0;
            } else {
              phi = dh * (sqrt(c1 * c2) - sqrt((1.0 - c1) * (1.0 - c2)));
            }
          }
          ok = ok && isfinite(phi);
          if (ok) phi = fmin(fmax(phi, 0.0), sig);
        }
        if (!ok) {
          phi = 0.0;
          atomicOr(flag_s, EOQ_FLAG_SHRINK_GUARD);
        }
        phi_out[slot * r_max + i] = (float)phi;
        sigma_out[slot * r_max + i] = (float)sig;
        scale_s[i] = (sig > 0.0) ? phi / sig : 0.0;
      }
    }
    for (int i = r + tid; i < r_max; i += THREADS) {
      phi_out[slot * r_max + i] = 0.0f;
      sigma_out[slot * r_max + i] = 0.0f;
    }
  }
  __syncthreads();
  return r;
}

// =============================================================================================
// Jacobi solver
// =============================================================================================
constexpr int LDA = D + 1;  // padded column stride of the LDS-resident matrix
constexpr int MAX_SWEEPS = 30;
constexpr double JACOBI_TOL = 5e-14;  // a pair is orthogonal when |<a_p,a_q>| <= tol |a_p||a_q|

// With `list` non-null the workgroups walk the block numbers list[0 .. *count) (grid-stride); otherwise
// workgroup b handles block b.
__global__ __launch_bounds__(THREADS) void eoq_spectral_jacobi_kernel(
    const void* __restrict__ blocks, EoqBlockMap map, int dtype, int n, int k, double rank_thr, int r_max, int loss, int64_t B,
    const int* __restrict__ list, const int* __restrict__ count, double* __restrict__ lam_out,
    float* __restrict__ wfac, int32_t* __restrict__ rank_out, float* __restrict__ phi_out,
    float* __restrict__ sigma_out, uint16_t* __restrict__ rfac, uint32_t* __restrict__ flags_out) {
  __shared__ double A[D * LDA];            // column s of the working matrix at A[s*LDA ...]
  __shared__ float stage[STAGE_ROWS * D];
  __shared__ double lam_s[D];
  __shared__ double atoms[D];
  __shared__ double colnorm[D];
  __shared__ int slot_of[D];
  __shared__ double scale_s[EOQ_RMAX_CAP];
  __shared__ unsigned flag_s;

  const int tid = threadIdx.x;
  const int64_t total = list ? (int64_t)*count : B;
  for (int64_t item = blockIdx.x; item < total; item += gridDim.x) {
    const size_t blk = list ? (size_t)list[item] : (size_t)item;
    const size_t slot = map.slot(blk);
    __syncthreads();
    if (tid == 0) flag_s = 0u;

    {
      double acc[64];
      gram_tile(blocks, dtype, map.in_base(blk), (size_t)map.token_stride, n, stage, tid, acc);
      bool bad = false;
      EOQ_SFOR(e, 64, bad |= !(fabs(acc[e]) < INFINITY););
      if (bad) atomicOr(&flag_s, EOQ_FLAG_NONFINITE);
      const int ty = tid >> 4, tx = tid & 15;
      EOQ_SFOR(e, 64, A[(tx * 8 + (e & 7)) * LDA + ty * 8 + (e >> 3)] = acc[e];);
    }
    __syncthreads();

    // One-sided Jacobi on the columns of A = G: A V -> V Lambda.  64 pairs per step, one per group of 4
    // lanes; pair p works on slots 2p, 2p+1 and writes its rotated columns to the slots the round-robin
    // schedule pairs next.
    const int pr = tid >> 2, ql = tid & 3;
    const int m_pairs = D / 2;
    const int dst_top = (pr == 0) ? 0 : (pr == m_pairs - 1 ? 2 * (m_pairs - 1) + 1 : 2 * (pr + 1));
    const int dst_bot = (pr == 0) ? 2 : 2 * (pr - 1) + 1;
    int sweeps = 0;
    bool converged = false;
    for (; sweeps < MAX_SWEEPS && !converged; ++sweeps) {
      int sweep_rot = 0;
      for (int step = 0; step < D - 1; ++step) {
        double xp[D / 4], xq[D / 4];
        double alpha = 0.0, beta = 0.0, gamma = 0.0;
#pragma unroll
        for (int m = 0; m < D / 4; ++m) {
          xp[m] = A[(2 * pr) * LDA + ql + 4 * m];
          xq[m] = A[(2 * pr + 1) * LDA + ql + 4 * m];
          alpha = fma(xp[m], xp[m], alpha);
          beta = fma(xq[m], xq[m], beta);
          gamma = fma(xp[m], xq[m], gamma);
        }
        alpha = quad_sum(alpha);
        beta = quad_sum(beta);
        gamma = quad_sum(gamma);
        const bool rot = fabs(gamma) > JACOBI_TOL * sqrt(alpha * beta);
        double c = 1.0, s = 0.0;
        if (rot) {
          const double zeta = (beta - alpha) / (2.0 * gamma);
          const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
          c = 1.0 / sqrt(1.0 + t * t);
          s = c * t;
        }
        __syncthreads();  // every lane holds its operands; slots may now be overwritten
#pragma unroll
        for (int m = 0; m < D / 4; ++m) {
          A[dst_top * LDA + ql + 4 * m] = c * xp[m] - s * xq[m];
          A[dst_bot * LDA + ql + 4 * m] = s * xp[m] + c * xq[m];
        }
        sweep_rot |= __syncthreads_or(rot ? 1 : 0);
      }
      converged = (sweep_rot == 0);
    }
    if (!converged && tid == 0) flag_s |= EOQ_FLAG_NO_CONVERGE;

    // eigenvalues = column norms; order them
    {
      double alpha = 0.0;
#pragma unroll
      for (int m = 0; m < D / 4; ++m) {
        const double x = A[(tid >> 1) * LDA + (tid & 1) * 64 + m * 2 + 0];
        const double y = A[(tid >> 1) * LDA + (tid & 1) * 64 + m * 2 + 1];
        alpha = fma(x, x, alpha);
        alpha = fma(y, y, alpha);
      }
      alpha = pair_sum(alpha);
      if ((tid & 1) == 0) colnorm[tid >> 1] = sqrt(alpha);
    }
    __syncthreads();
    if (tid < D) {
      const double mine = colnorm[tid];
      int pos = 0;
      for (int t = 0; t < D; ++t) {
        const double o = colnorm[t];
        pos += (o > mine || (o == mine && t < tid)) ? 1 : 0;
      }
      lam_s[pos] = mine;
      slot_of[pos] = tid;
    }
    __syncthreads();

    const int r = rank_and_shrink(lam_s, atoms, scale_s, &flag_s, n, k, rank_thr, r_max, loss, blk, slot, lam_out, phi_out,
                                  sigma_out);

    // right singular vectors v_i = a_slot / lambda_i of the retained components
    for (int e = tid; e < r * D; e += THREADS) {
      const int i = e >> 7, j = e & (D - 1);
      const double li = lam_s[i];
      const double v = (li > 0.0) ? A[slot_of[i] * LDA + j] / li : 0.0;
      rfac[(slot * r_max + i) * D + j] = double_to_half_bits(v);
      wfac[(blk * r_max + i) * D + j] = (float)(v * scale_s[i]);
    }
    if (tid == 0) {
      rank_out[slot] = r;
      flags_out[slot] = flag_s | ((unsigned)sweeps << EOQ_FLAG_SWEEPS_SHIFT);
    }
  }
}

// =============================================================================================
// Tridiagonal solver
// =============================================================================================
// Cyclic layout of the working matrix: lane (ty, tx) = (tid / 16, tid % 16) owns the 8 x 8 entries
// A[a * 8 + b] = G[ty + 16 a][tx + 16 b].  Rows and columns are dealt round-robin, so the trailing submatrix
// of the reduction stays spread over all lanes while it shrinks: during steps 16 s .. 16 s + 15 every lane's
// live part is the sub-tile a, b >= s.  The 16 lanes of one DPP row share ty.
constexpr int GRAM_STRIP = 32;  // block rows staged per pass
// Position of column j in a staged row: the 8 columns {c + 16 m} that one lane needs are split into two groups
// of four consecutive floats, the groups of the 16 lanes side by side (16-byte reads without bank conflicts).
__device__ __forceinline__ int stage_pos(int j) { return ((j >> 6) << 6) | ((j & 15) << 2) | ((j >> 4) & 3); }
constexpr int XPAD = 17;  // row stride of a 16 x 16 exchange plane: transposed reads hit distinct banks
// the 28 sub-tiles above the diagonal, in the order they are mirrored
constexpr int PAIR_A[28] = {0, 0, 0, 0, 0, 0, 0, 1, 1, 1, 1, 1, 1, 2, 2, 2, 2, 2, 3, 3, 3, 3, 4, 4, 4, 5, 5, 6};
constexpr int PAIR_B[28] = {1, 2, 3, 4, 5, 6, 7, 2, 3, 4, 5, 6, 7, 3, 4, 5, 6, 7, 4, 5, 6, 7, 5, 6, 7, 6, 7, 7};

// packed reflector storage: reflector k has entries i = k+1 .. 127
__device__ __forceinline__ int refl_off(int k) { return k * (D - 1) - (k * (k - 1)) / 2; }
constexpr int REFL_LEN = (D - 1) * D / 2;  // 8128
constexpr int GRID_POINTS = 256;           // first localisation: one Sturm count per lane on a grid (cubically spaced)
constexpr int MULTISECT_ITERS = 17;        // then two lanes per eigenvalue down to the width of 17 trisections of a uniform
                                           // grid cell, 3^-17 / 257 < 2^-34.9 (plain trisection would take 18 rounds at most)
constexpr int REFINE_COUNT = 32;           // at most this many eigenvalues go on to full precision (the reduction
                                           // itself is good to ~2^-48), with 256 / 32 = 8 lanes each or more
constexpr int REFINE_KEEP = 48;            // brackets of the largest eigenvalues kept for that second phase
static_assert(REFINE_COUNT * 8 == THREADS && REFINE_COUNT >= EOQ_RMAX_CAP && 2 * REFINE_KEEP <= D, "second phase layout");
constexpr int EV_BATCH = 8;                // eigenvectors per twisted-factorisation pass
// Twisted-factorisation scratch: per eigenvector of a batch two arrays of D pairs, F then Bk.  The arrays are D + 1
// pairs apart: lanes that walk different arrays in step (one per array, same row) then fall into different banks;
// at a stride of D pairs = 2048 bytes all sixteen would hit the same ones.
constexpr int TW_STRIDE = D + 1;
constexpr int U1_BYTES = EV_BATCH * 2 * TW_STRIDE * 16;  // 33 KB; also the Gram strip (16 KB)
constexpr double CLUSTER_TOL = 1e-10;      // relative gap below which retained eigenvalues count as repeated
constexpr int REFL_SLACK = 16;             // floats in front of the reflectors (masked reads may reach them)
constexpr int REFL_BYTES = (REFL_LEN + REFL_SLACK) * 4;   // 32576 (a multiple of 16)
constexpr int POOL_BYTES = REFL_BYTES + U1_BYTES;

// G = S^T S in the cyclic layout.  Only the sub-tiles a <= b are accumulated (36 of 64 products per block row);
// the others are mirrored from the lane that holds the transposed position, through LDS.
__device__ __forceinline__ void gram_cyclic(const void* __restrict__ blocks, int dtype, size_t base_elem, size_t tok, int n,
                                            float* stage, int tid, double (&A)[64], unsigned* flag_s) {
  const int ty = tid >> 4, tx = tid & 15;
  EOQ_SFOR(i, 64, A[i] = 0.0;);
  float nxt[2][8];
  const int wrow = tid >> 4, wcol = (tid & 15) * 8;
  load8(blocks, dtype, base_elem + (size_t)wrow * tok + wcol, nxt[0]);
  load8(blocks, dtype, base_elem + (size_t)(16 + wrow) * tok + wcol, nxt[1]);
#pragma unroll 1
  for (int t0 = 0; t0 < n; t0 += GRAM_STRIP) {
    __syncthreads();  // the previous strip has been consumed
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int i = 0; i < 8; ++i) stage[(g * 16 + wrow) * D + stage_pos(wcol + i)] = nxt[g][i];
    __syncthreads();
    if (t0 + GRAM_STRIP < n) {  // next strip on its way while this one is multiplied
      const size_t e = base_elem + (size_t)(t0 + GRAM_STRIP + wrow) * tok + wcol;
      load8(blocks, dtype, e, nxt[0]);
      load8(blocks, dtype, e + 16 * tok, nxt[1]);
    }
#pragma unroll 2
    for (int t = 0; t < GRAM_STRIP; ++t) {
      const float4 a0 = *reinterpret_cast<const float4*>(stage + t * D + ty * 4);
      const float4 a1 = *reinterpret_cast<const float4*>(stage + t * D + 64 + ty * 4);
      const float4 b0 = *reinterpret_cast<const float4*>(stage + t * D + tx * 4);
      const float4 b1 = *reinterpret_cast<const float4*>(stage + t * D + 64 + tx * 4);
      const double a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
      const double b[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
      EOQ_SFOR(e, 64, if constexpr ((e >> 3) <= (e & 7)) A[e] = fma(a[e >> 3], b[e & 7], A[e]););
    }
  }
  {
    bool bad = false;   // an Inf or NaN entry of the block reaches the diagonal of G
    EOQ_SFOR(i, 8, bad |= !(fabs(A[i * 9]) < INFINITY););
    if (bad) atomicOr(flag_s, EOQ_FLAG_NONFINITE);
  }
  // mirror: G[ty+16b][tx+16a] (a < b) is what lane (tx, ty) accumulated as its sub-tile (a, b)
  double* X = reinterpret_cast<double*>(stage);
  EOQ_SFOR(round, 4,
    __syncthreads();
    EOQ_SFOR(q, 7, X[q * 16 * XPAD + ty * XPAD + tx] = A[PAIR_A[round * 7 + q] * 8 + PAIR_B[round * 7 + q]];);
    __syncthreads();
    EOQ_SFOR(q, 7, A[PAIR_B[round * 7 + q] * 8 + PAIR_A[round * 7 + q]] = X[q * 16 * XPAD + tx * XPAD + ty];);
  );
}

// ---------------------------------------------------------------------------------------------
// Gram matrix of a binary16 block by exact integer arithmetic on the matrix cores.
//
// Per group of 128 tokens every column j gets the exponent E_j of its largest entry and its entries become
// integers I = trunc(x 2^(29 - E_j)), |I| < 2^30: exact for every entry within a factor 2^19 of the column
// maximum (binary16 carries 11 significant bits), truncated below 2^(E_j - 29) otherwise.  I is split into four
// signed bytes, I = s0 + 2^8 s1 + 2^16 s2 + 2^24 s3, and the byte planes are multiplied with
// v_mfma_i32_16x16x64_i8, two instructions deep per plane pair (exact int32 sums over the 128 tokens); the sixteen
// plane pairs go to seven accumulators, one per weight 2^(8 (p + q)).  The group result, scaled by
// 2^(E_i + E_j - 58), is added to a double-precision accumulator: one conversion per 128 tokens.  Only the 36
// tiles of 16 x 16 on and above the diagonal are computed, nine per wave.  Element (ty, tx) of tile (a, b) is entry
// A[a * 8 + b] of lane (ty, tx) in the cyclic layout, so at the end the tiles only change lanes (through LDS), the
// mirrored ones read transposed.
// ---------------------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

constexpr int GI_TOK = 128;                      // tokens per group = two matrix instructions deep
constexpr int GI_ROW = GI_TOK;                   // bytes per (plane, column): eight chunks of 16 tokens
constexpr int GI_PLANE = D * GI_ROW;             // 16384
constexpr int GI_NPLANE = 4;
constexpr int GI_BYTES = GI_NPLANE * GI_PLANE;   // 64 KB: the four planes fill the pool
static_assert(GI_BYTES <= POOL_BYTES && GI_PLANE % 16 == 0, "Gram planes inside the pool");
// A row is exactly as wide as the banks, so the chunks of a row are stored permuted: chunk c of column col sits at
// position c ^ col ^ (col >> 3) (low three bits).  The sixteen lanes that read chunk c of sixteen consecutive
// columns (operand loads) and the sixteen loaders that write chunk c of columns 8 m + const both touch every
// position twice, which is what a 16-byte access of sixteen lanes needs anyway.
__device__ __forceinline__ int gi_chunk_off(int col, int c) { return ((c ^ col ^ (col >> 3)) & 7) << 4; }
constexpr int GI_TILES = 36;                     // upper tiles, row-major: (0,0) .. (0,7), (1,1) .. (7,7)
constexpr int UT_I[GI_TILES] = {0, 0, 0, 0, 0, 0, 0, 0, 1, 1, 1, 1, 1, 1, 1, 2, 2, 2, 2, 2, 2, 3, 3, 3, 3, 3, 4, 4, 4, 4, 5, 5, 5, 6, 6, 7};
constexpr int UT_J[GI_TILES] = {0, 1, 2, 3, 4, 5, 6, 7, 1, 2, 3, 4, 5, 6, 7, 2, 3, 4, 5, 6, 7, 3, 4, 5, 6, 7, 4, 5, 6, 7, 5, 6, 7, 6, 7, 7};
__device__ const int ut_i_dev[GI_TILES] = {0, 0, 0, 0, 0, 0, 0, 0, 1, 1, 1, 1, 1, 1, 1, 2, 2, 2, 2, 2, 2, 3, 3, 3, 3, 3, 4, 4, 4, 4, 5, 5, 5, 6, 6, 7};
__device__ const int ut_j_dev[GI_TILES] = {0, 1, 2, 3, 4, 5, 6, 7, 1, 2, 3, 4, 5, 6, 7, 2, 3, 4, 5, 6, 7, 3, 4, 5, 6, 7, 4, 5, 6, 7, 5, 6, 7, 6, 7, 7};

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  const ushort2v r = __builtin_elementwise_max(*reinterpret_cast<ushort2v*>(&a), *reinterpret_cast<ushort2v*>(&b));
  return *reinterpret_cast<const uint32_t*>(&r);
}
// cmax: 4 x 64 words (the waves' column maxima), cexp: 128 ints (exponent of the integer unit of each column); both
// outside the pool, which the planes fill.  n is a multiple of 128.
__device__ __forceinline__ void gram_int8(const uint16_t* __restrict__ src, size_t tok, int n, unsigned char* pool,
                                          uint32_t* cmax, int* cexp, int tid, double (&A)[64], unsigned* flag_s) {
  const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = tid & 15, q = tid >> 4;  // loader: columns 8m .. 8m+7, tokens 64 h + 4q .. 64 h + 4q + 3 of the group
  double Gacc[9][4];  // tile number wave + 4 s, rows 4 kg + v, column l16
  EOQ_SFOR(s, 9, EOQ_SFOR(v, 4, Gacc[s][v] = 0.0;););

  uint32_t top = 0u;  // largest |binary16 pattern| this lane has seen in its columns: 0x7C00 and above is Inf / NaN
  uint4 raw[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    raw[i] = *reinterpret_cast<const uint4*>(src + (size_t)(64 * (i >> 2) + 4 * q + (i & 3)) * tok + 8 * m);

#pragma unroll 1
  for (int t0 = 0; t0 < n; t0 += GI_TOK) {
    // ---- column maxima of the group: over the lane's eight tokens, the wave's four loader rows, the four waves ----
    uint32_t mx[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mx[0] = pk_max_u16(mx[0], raw[i].x & 0x7FFF7FFFu);
      mx[1] = pk_max_u16(mx[1], raw[i].y & 0x7FFF7FFFu);
      mx[2] = pk_max_u16(mx[2], raw[i].z & 0x7FFF7FFFu);
      mx[3] = pk_max_u16(mx[3], raw[i].w & 0x7FFF7FFFu);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      mx[i] = pk_max_u16(mx[i], (uint32_t)__shfl_xor((int)mx[i], 16, 64));
      mx[i] = pk_max_u16(mx[i], (uint32_t)__shfl_xor((int)mx[i], 32, 64));
    }
    __syncthreads();  // the previous group no longer reads planes, maxima or exponents
    if (kg == 0) *reinterpret_cast<uint4*>(cmax + wave * 64 + m * 4) = make_uint4(mx[0], mx[1], mx[2], mx[3]);
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint4 o = *reinterpret_cast<const uint4*>(cmax + w * 64 + m * 4);
      mx[0] = pk_max_u16(mx[0], o.x);
      mx[1] = pk_max_u16(mx[1], o.y);
      mx[2] = pk_max_u16(mx[2], o.z);
      mx[3] = pk_max_u16(mx[3], o.w);
    }
    top = pk_max_u16(top, pk_max_u16(pk_max_u16(mx[0], mx[1]), pk_max_u16(mx[2], mx[3])));
    // ---- integers, byte planes ----
    EOQ_SFOR(c, 8,
      const uint32_t hmax = (mx[c >> 1] >> (16 * (c & 1))) & 0xFFFFu;
      const int ef = max((int)(hmax >> 10), 1);               // biased exponent of the column maximum (subnormals: 1)
      const float scale = __int_as_float((171 - ef) << 23);   // 2^(29 - (ef - 15))
      if (q == 0) cexp[8 * m + c] = ef - 44;                  // one integer unit = 2^(ef - 15 - 29)
      // I = sum_k d_k 256^k with balanced digits d_k in [-128, 127]: adding 128 to every digit place makes them the
      // plain bytes of I + 0x80808080 (|I| < 2^30: no carry out of the top), and flipping the top bit of each byte
      // takes the 128 off again, as a two's-complement byte.  The four planes are those bytes.
      EOQ_SFOR(h, 2,
        uint32_t dg[4];
        EOQ_SFOR(it, 4,
          const uint4 rw = raw[4 * h + it];
          const uint32_t w = (c >> 1) == 0 ? rw.x : ((c >> 1) == 1 ? rw.y : ((c >> 1) == 2 ? rw.z : rw.w));
          const uint16_t hb = (uint16_t)(w >> (16 * (c & 1)));
          const int I = (int)(half_bits_to_float(hb) * scale);   // truncation towards zero
          dg[it] = ((uint32_t)I + 0x80808080u) ^ 0x80808080u;
        );
        uint32_t pl[4];
        transpose_bytes(dg[0], dg[1], dg[2], dg[3], pl);
        unsigned char* dst = pool + (8 * m + c) * GI_ROW + gi_chunk_off(8 * m + c, 4 * h + (q >> 2)) + 4 * (q & 3);
        *reinterpret_cast<uint32_t*>(dst) = pl[0];
        *reinterpret_cast<uint32_t*>(dst + GI_PLANE) = pl[1];
        *reinterpret_cast<uint32_t*>(dst + 2 * GI_PLANE) = pl[2];
        *reinterpret_cast<uint32_t*>(dst + 3 * GI_PLANE) = pl[3];
      );
    );
    if (t0 + GI_TOK < n) {  // next group on its way during the products
#pragma unroll
      for (int i = 0; i < 8; ++i)
        raw[i] = *reinterpret_cast<const uint4*>(src + (size_t)(t0 + GI_TOK + 64 * (i >> 2) + 4 * q + (i & 3)) * tok + 8 * m);
    }
    __syncthreads();
    // ---- products, one tile at a time: lane supplies row / column l16 of the tile, tokens 64 h + 16 kg .. + 15 ----
    EOQ_SFOR(s, 9,
      const int tile = wave + 4 * s;
      const int tI = ut_i_dev[tile]; const int tJ = ut_j_dev[tile];
      v4i acc[7];  // acc[c]: plane pairs (p, q) with p + q = c, weight 2^(8 c)
      EOQ_SFOR(cc, 7, EOQ_SFOR(v, 4, acc[cc][v] = 0;););
      const int ca = 16 * tI + l16, cb = 16 * tJ + l16;
      EOQ_SFOR(h, 2,
        const unsigned char* pa = pool + ca * GI_ROW + gi_chunk_off(ca, 4 * h + kg);
        const unsigned char* pb = pool + cb * GI_ROW + gi_chunk_off(cb, 4 * h + kg);
        v4i a[4]; v4i b[4];
        EOQ_SFOR(pl, 4,
          a[pl] = *reinterpret_cast<const v4i*>(pa + pl * GI_PLANE);
          b[pl] = *reinterpret_cast<const v4i*>(pb + pl * GI_PLANE);
        );
        // order: consecutive instructions hit different accumulators
        EOQ_SFOR(rot, 4,
          EOQ_SFOR(pl, 4,
            constexpr int ql = (pl + rot) & 3;
            acc[pl + ql] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[pl], b[ql], acc[pl + ql], 0, 0, 0);
          );
        );
      );
      // into double precision with the exponents of rows 4 kg + v (tile I) and column l16 (tile J)
      const int ej = cexp[16 * tJ + l16];
      const int4 ei = *reinterpret_cast<const int4*>(cexp + 16 * tI + 4 * kg);
      const int eiv[4] = {ei.x, ei.y, ei.z, ei.w};
      // Neighbouring weights are merged in int32 first, then four conversions and a Horner pass in double.  A digit
      // is at most 128 in magnitude and the top digit at most 64 (|I| < 2^30), so over 128 tokens the classes are
      // bounded by |c_0| <= 2^21, |c_1| <= 2^22, |c_2| <= 3 2^21, |c_3| <= 128 (2^15 + 2^14) = 3 2^21, |c_4| <=
      // 128 (2^14 + 2^14) = 2^22, |c_5| <= 2^21, and every c_even + 2^8 c_odd stays below 2^31 (the largest,
      // c_2 + 2^8 c_3, below 1.62e9).
      EOQ_SFOR(v, 4,
        const int m01 = acc[0][v] + (acc[1][v] << 8), m23 = acc[2][v] + (acc[3][v] << 8), m45 = acc[4][v] + (acc[5][v] << 8);
        const double val = fma(fma(fma((double)acc[6][v], 65536.0, (double)m45), 65536.0, (double)m23), 65536.0, (double)m01);
        Gacc[s][v] += ldexp(val, eiv[v] + ej);
      );
    );
  }
  // a column maximum with all exponent bits set: the integer conversion of that pass saturated, G is meaningless
  if (q == 0 && (((top & 0xFFFFu) >= 0x7C00u) || ((top >> 16) >= 0x7C00u))) atomicOr(flag_s, EOQ_FLAG_NONFINITE);
  // ---- tiles change lanes: three rounds of twelve tiles through LDS; lane (ty, tx) takes element (ty, tx) of tile
  // (a, b) as A[a * 8 + b] and, for a < b, element (tx, ty) as A[b * 8 + a] ----
  double* Tl = reinterpret_cast<double*>(pool);
  const int ty = tid >> 4, tx = tid & 15;
  EOQ_SFOR(rd, 3,
    __syncthreads();
    EOQ_SFOR(s3, 3,
      constexpr int s = 3 * rd + s3;
      double* dst = Tl + (wave + 4 * s3) * 16 * XPAD;
      EOQ_SFOR(v, 4, dst[(4 * kg + v) * XPAD + l16] = Gacc[s][v];);
    );
    __syncthreads();
    EOQ_SFOR(pp, 12,
      constexpr int tile = 12 * rd + pp;
      constexpr int a = UT_I[tile]; constexpr int b = UT_J[tile];
      A[a * 8 + b] = Tl[pp * 16 * XPAD + ty * XPAD + tx];
      if constexpr (a != b) A[b * 8 + a] = Tl[pp * 16 * XPAD + tx * XPAD + ty];
    );
  );
}

// Sum over the 16 lanes of a DPP row of the values p[S .. 7] of every lane (the values below S are dead),
// transposing as it folds: on return lane tx holds the row total of value number fold_index<S>(tx), and the lanes
// with fold_writer<S>(tx) hold each live total exactly once.  Partners: 15 - tx, tx ^ 7, tx ^ 2, tx ^ 1; at a
// transposing fold a lane keeps the half of its values selected by one bit of tx and hands the other half to its
// partner; once only half of the values are live that fold is a plain sum.
template <int S>
__device__ __forceinline__ int fold_index(int tx) {
  if constexpr (S < 4) return tx >> 1;
  else if constexpr (S < 6) return 4 + ((tx >> 1) & 3);
  else if constexpr (S == 6) return 6 + ((tx >> 1) & 1);
  else return 7;
}
template <int S>
__device__ __forceinline__ bool fold_writer(int tx) {
  if constexpr (S < 4) return (tx & 1) == 0;
  else if constexpr (S < 6) return (tx & 9) == 0;
  else if constexpr (S == 6) return (tx & 13) == 0;
  else return tx == 0;
}
template <int S>
__device__ __forceinline__ double row16_fold(const double (&p)[8], int tx) {
  const bool b3 = (tx & 8) != 0, b2 = (tx & 4) != 0, b1 = (tx & 2) != 0;
  double r1[4], r2[2], r3;
  if constexpr (S < 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double send = b3 ? p[i] : p[4 + i];
      const double keep = b3 ? p[4 + i] : p[i];
      r1[i] = keep + dpp_mov<0x140>(send);  // row_mirror
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) r1[i] = (4 + i >= S) ? p[4 + i] + dpp_mov<0x140>(p[4 + i]) : 0.0;
  }
  if constexpr (S < 6) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const double send = b2 ? r1[i] : r1[2 + i];
      const double keep = b2 ? r1[2 + i] : r1[i];
      r2[i] = keep + dpp_mov<0x141>(send);  // row_half_mirror
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i) r2[i] = (6 + i >= S) ? r1[2 + i] + dpp_mov<0x141>(r1[2 + i]) : 0.0;
  }
  if constexpr (S < 7) {
    const double send = b1 ? r2[0] : r2[1];
    const double keep = b1 ? r2[1] : r2[0];
    r3 = keep + dpp_mov<0x4E>(send);
  } else {
    r3 = r2[1] + dpp_mov<0x4E>(r2[1]);
  }
  return r3 + dpp_mov<0xB1>(r3);
}

// Square root and reciprocal by Newton steps from the hardware estimates (good to a few ulp: the reduction only
// needs alpha^2 = x^T x and beta = 2 / v^T v to hold to rounding level).
__device__ __forceinline__ double newton_sqrt(double s) {
  const double y = __builtin_amdgcn_rsq(s);
  double g = s * y, h = 0.5 * y;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const double r = fma(-h, g, 0.5);
    g = fma(g, r, g);
    h = fma(h, r, h);
  }
  return fma(fma(-g, g, s), h, g);
}
__device__ __forceinline__ double newton_rcp(double s) {
  double y = __builtin_amdgcn_rcp(s);
#pragma unroll
  for (int it = 0; it < 2; ++it) y = fma(fma(-s, y, 1.0), y, y);
  return y;
}

// Steps k = 16 S .. 16 S + 15 of the Householder reduction G = Q T Q^T, Q = H_0 H_1 ... H_125,
// H_k = I - beta_k v_k v_k^T.  Per step: the 16 lanes that own row k form v and beta (the other lanes wait),
// all lanes multiply p = beta A v over their live sub-tile (partial sums folded across the DPP row), then apply
// A <- A - v w^T - w v^T with w = p - (beta/2)(v^T p) v.
// A wave by itself issues a double-precision instruction in about seven cycles and a 32-bit or scalar one in four to
// five, however independent they are (two waves per SIMD, which is what the registers allow: four to five cycles per
// double-precision instruction between them), so what a step costs is the number of instructions of the wave the
// others wait for, while the SIMDs of the waiting waves serve the other workgroup of the compute unit.  The wave
// that forms the reflector therefore does nothing that another wave can do: the row goes to LDS as it is (one entry less alpha), and the
// float copy of the reflector for the back-transformation is made one step later by the next wave, which would wait
// otherwise.
// p = beta A v in LDS: entry i = l + 16 g at pbuf[l + PB_LD g].  Its writers are four consecutive rows l of up to eight
// groups g per wave; at a pitch of 20 doubles the groups start in eight different sets of eight banks.
constexpr int PB_LD = 20;
// float copy of reflector k (entries k + 1 .. 127 of v, in LDS as doubles) into the packed store, by one wave
__device__ __forceinline__ void stash_reflector(const double* v, int k, int lane, float* refl) {
  float* dst = refl + refl_off(k) - (k + 1);   // entry j at dst[j]
  if (lane > k) dst[lane] = (float)v[lane];
  if (lane + 64 > k) dst[lane + 64] = (float)v[lane + 64];
}
template <int S>
__device__ __forceinline__ void householder_stage(double (&A)[64], int tid, double (*vbuf)[D], double* pbuf,
                                                  float* refl, double* dT, double* eT, double* betaT) {
  const int lane = tid & 63, ty = tid >> 4, tx = tid & 15;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int KK_END = (S == 7) ? 14 : 16;
#pragma unroll 1
  for (int kk = 0; kk < KK_END; ++kk) {
    const int k = 16 * S + kk;
    double* vb = vbuf[kk & 1];
    if (wave == (kk >> 2)) {
      // every 16-lane row of this wave runs the arithmetic on its own matrix row; only the row k stores
      const bool owner = ((lane >> 4) == (kk & 3));
      const double xs = (tx > kk) ? A[S * 8 + S] : 0.0;  // columns j = tx + 16 b > k only
      double s0 = xs * xs, s1 = 0.0;
      EOQ_SFOR(b, 8,
        if constexpr (b > S) {
          if constexpr (((b - S) & 1) == 0) s0 = fma(A[S * 8 + b], A[S * 8 + b], s0);
          else s1 = fma(A[S * 8 + b], A[S * 8 + b], s1);
        });
      const double ss = row16_sum_uniform(s0 + s1);   // the same bits in the sixteen lanes of a row
      double xsel = xs;
      if constexpr (S < 7) xsel = (kk == 15) ? A[S * 8 + S + 1] : xsel;
      const double x0 = readlane_f64(xsel, 16 * (kk & 3) + ((kk + 1) & 15));  // x_{k+1} of row k
      double alpha = 0.0, beta = 0.0;
      if (ss > 0x1.0p-960) {
        const double sigma = newton_sqrt(ss);
        alpha = (x0 >= 0.0) ? -sigma : sigma;                 // H_k x = alpha e_1
        beta = newton_rcp(fma(sigma, fabs(x0), ss));          // 2 / (v^T v), v = x - alpha e_1
      }
      if (owner) {
        // v = x - alpha e_{k+1}: entry k + 1 sits in sub-tile S of lane kk + 1, or, at the last step of a stage, in
        // sub-tile S + 1 of lane 0
        const double fix = (tx == ((kk + 1) & 15)) ? alpha : 0.0;
        vb[tx + 16 * S] = xs - ((kk < 15) ? fix : 0.0);
        EOQ_SFOR(b, 8,
          if constexpr (b > S) vb[tx + 16 * b] = (b == S + 1) ? A[S * 8 + b] - ((kk == 15) ? fix : 0.0) : A[S * 8 + b];);
        if (tx == kk) {
          dT[k] = A[S * 8 + S];
          eT[k] = alpha;
          betaT[k] = beta;
        }
      }
    } else if (wave == (((kk >> 2) + 1) & 3) && k > 0) {
      stash_reflector(vbuf[(kk + 1) & 1], k - 1, lane, refl);   // the reflector of the step before, complete since that step's first barrier
    }
    __syncthreads();
    const double beta = betaT[k];
    double vj[8];
    EOQ_SFOR(b, 8, vj[b] = (b >= S) ? vb[tx + 16 * b] : 0.0;);
    {
      double part[8];
      EOQ_SFOR(a, 8,
        if constexpr (a >= S) {
          // one chain per row: the chains of the live rows interleave, which is independent work enough
          double s0 = 0.0;
          EOQ_SFOR(b, 8, if constexpr (b >= S) s0 = fma(A[a * 8 + b], vj[b], s0););
          part[a] = s0;
        } else {
          part[a] = 0.0;
        });
      const double tot = row16_fold<S>(part, tx);
      if (fold_writer<S>(tx)) pbuf[ty + PB_LD * fold_index<S>(tx)] = beta * tot;
    }
    __syncthreads();
    // v^T p from the column entries this lane holds anyway, summed over its DPP row (every row of 16 lanes covers
    // all 128 columns and gets the same bits)
    double wj[8], vi[8], wi[8];
    EOQ_SFOR(b, 8, wj[b] = (b >= S) ? pbuf[tx + PB_LD * b] : 0.0;);
    double dl0 = 0.0, dl1 = 0.0;
    EOQ_SFOR(b, 8,
      if constexpr (b >= S) {
        if constexpr ((b & 1) == 0) dl0 = fma(vj[b], wj[b], dl0);
        else dl1 = fma(vj[b], wj[b], dl1);
      });
    // v w^T + w v^T with w = p - K v is v p^T + q v^T with q = p - 2 K v: the correction is needed in the row view
    // only, the column view of p goes into the update as it was read
    const double K2 = beta * row16_sum_uniform(dl0 + dl1);
    EOQ_SFOR(a, 8, vi[a] = (a >= S) ? vb[ty + 16 * a] : 0.0;);
    EOQ_SFOR(a, 8, wi[a] = (a >= S) ? fma(-K2, vi[a], pbuf[ty + PB_LD * a]) : 0.0;);
    EOQ_SFOR(e, 64,
      if constexpr ((e >> 3) >= S && (e & 7) >= S)
        A[e] = fma(-vi[e >> 3], wj[e & 7], fma(-wi[e >> 3], vj[e & 7], A[e])););
  }
}

// Sum over eight consecutive lanes (an aligned group of a DPP row): butterfly of commutative pair sums
// (lane^1, lane^2, 7-lane), bit-identical in the eight lanes.
__device__ __forceinline__ double oct_sum_uniform(double v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  return v;
}

// The last 30 steps of the reduction (k = 96 .. 125) on the trailing 32 x 32 matrix, by ONE wave: lane (ly, lx) =
// (lane / 8, lane % 8) holds T[a][b] = M[ly + 8 a][lx + 8 b], a, b < 4 (rows and columns counted from 96).  With
// the four waves on it a step of this size costs as many instructions per wave as a step on the full matrix
// (reductions, exchanges and two barriers); here the other three waves issue nothing, the exchanges go through
// LDS without a barrier (operations of one wave complete in order) and the sums run over eight lanes.
// Steps 8 AO .. 8 AO + 7 (the last stage stops after local row 29): rows and columns below 8 AO are dead.
template <int AO>
__device__ __forceinline__ void tail32_stage(double (&T)[16], int lane, double* vring, double* pb, double* dT,
                                             double* eT, double* betaT) {
  const int ly = lane >> 3, lx = lane & 7;
  constexpr int KEND = (AO == 3) ? 6 : 8;
#pragma unroll 1
  for (int kk = 0; kk < KEND; ++kk) {
    const int kq = 8 * AO + kk, k = 96 + kq;
    // ---- v, beta from row kq: every group of eight lanes runs the arithmetic on its own row, the owner stores ----
    // (the reflector stays in LDS as doubles, every step in a slot of its own: `vring`; the float copy for the
    // back-transformation is made afterwards by all four waves)
    double* vb = vring + 32 * kq;
    const bool owner = (ly == kk);
    const double xs = (lx > kk) ? T[AO * 4 + AO] : 0.0;   // columns lx + 8 b > kq only
    double ss = xs * xs;
    EOQ_SFOR(b, 4, if constexpr (b > AO) ss = fma(T[AO * 4 + b], T[AO * 4 + b], ss););
    ss = oct_sum_uniform(ss);
    double xsel = xs;
    if constexpr (AO < 3) xsel = (kk == 7) ? T[AO * 4 + AO + 1] : xsel;
    const double x0 = readlane_f64(xsel, 8 * kk + ((kk + 1) & 7));   // M[kq][kq + 1]
    double alpha = 0.0, beta = 0.0;
    if (ss > 0x1.0p-960) {
      const double sigma = newton_sqrt(ss);
      alpha = (x0 >= 0.0) ? -sigma : sigma;
      beta = newton_rcp(fma(sigma, fabs(x0), ss));
    }
    if (owner) {
      // v = x - alpha e_{kq+1}: that entry sits in sub-tile AO of lane kk + 1, or, at the last step of a stage, in
      // sub-tile AO + 1 of lane 0
      const double fix = (lx == ((kk + 1) & 7)) ? alpha : 0.0;
      vb[lx + 8 * AO] = xs - ((kk < 7) ? fix : 0.0);
      EOQ_SFOR(b, 4,
        if constexpr (b > AO) vb[lx + 8 * b] = (b == AO + 1) ? T[AO * 4 + b] - ((kk == 7) ? fix : 0.0) : T[AO * 4 + b];);
      if (lx == kk) {
        dT[k] = T[AO * 4 + AO];
        eT[k] = alpha;
        betaT[k] = beta;
      }
    }
    __builtin_amdgcn_wave_barrier();   // one wave: its LDS operations complete in order
    const double bq = readlane_f64(beta, 8 * kk);
    double vc[4], vr[4];
    EOQ_SFOR(b, 4, vc[b] = (b >= AO) ? vb[lx + 8 * b] : 0.0;);
    EOQ_SFOR(a, 4, vr[a] = (a >= AO) ? vb[ly + 8 * a] : 0.0;);
    // ---- p = beta M v: row sums over the eight lanes of a group; the column view goes through LDS ----
    double pr[4];
    EOQ_SFOR(a, 4,
      if constexpr (a >= AO) {
        double acc = 0.0;
        EOQ_SFOR(b, 4, if constexpr (b >= AO) acc = fma(T[a * 4 + b], vc[b], acc););
        pr[a] = bq * oct_sum_uniform(acc);
      } else {
        pr[a] = 0.0;
      });
    if (lx == 0) { EOQ_SFOR(a, 4, if constexpr (a >= AO) pb[ly + 8 * a] = pr[a];); }
    __builtin_amdgcn_wave_barrier();
    double pc[4];
    EOQ_SFOR(b, 4, pc[b] = (b >= AO) ? pb[lx + 8 * b] : 0.0;);
    double dl = 0.0;
    EOQ_SFOR(b, 4, if constexpr (b >= AO) dl = fma(vc[b], pc[b], dl););
    const double K2 = bq * oct_sum_uniform(dl);
    // ---- M <- M - v p^T - q v^T, q = p - 2 K v (= M - v w^T - w v^T with w = p - K v) ----
    double wr[4];
    EOQ_SFOR(a, 4, wr[a] = (a >= AO) ? fma(-K2, vr[a], pr[a]) : 0.0;);
    EOQ_SFOR(e, 16,
      if constexpr ((e >> 2) >= AO && (e & 3) >= AO)
        T[e] = fma(-vr[e >> 2], pc[e & 3], fma(-wr[e >> 2], vc[e & 3], T[e])););
    __builtin_amdgcn_wave_barrier();   // pb is rewritten by the next step
  }
}

// Number of eigenvalues of the (scaled) tridiagonal matrix below x: sign changes of the leading principal minors
// p_i(x) = (d_i - x) p_{i-1} - e_{i-1}^2 p_{i-2}.  de[2 i] = d_i, de[2 i + 1] = e_{i-1}^2 (e_{-1} = 0), read from
// global memory with wave-uniform addresses (scalar loads: the operands cost no vector or LDS bandwidth).
// The signs are shifted into a mask, 32 per word, and the changes counted per word.
typedef __attribute__((address_space(4))) const double sc_double;
// four steps of the recurrence with the operands t[2 s] = d, t[2 s + 1] = e^2; SIGNS: the signs go into the mask
template <bool SIGNS>
__device__ __forceinline__ void sturm_steps4(const double (&t)[8], double x, double& pm, double& p, unsigned& m) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const double pn = fma(t[2 * s] - x, p, -(t[2 * s + 1] * pm));
    if constexpr (SIGNS) m = __builtin_amdgcn_alignbit(m, (unsigned)__double2hiint(pn), 31);  // m = (m << 1) | sign(pn)
    pm = p;
    p = pn;
  }
}
__device__ __forceinline__ int sturm_renorm(double& pm, double& p) {  // |p| into [1/2, 1), same factor on both
  const int e = __builtin_amdgcn_frexp_exp(p);
  p = ldexp(p, -e);
  pm = ldexp(pm, -e);
  return e;
}
// The count, and the value of the last minor p_{D-1}(x) = det(T - x I) as val * 2^vexp (|val| in [1/2, 1) or zero).
// SIGNS = false: the value alone (three instructions per step instead of four), the return value is meaningless.
template <bool SIGNS = true>
__device__ __forceinline__ int sturm_count(sc_double* de, double x, double* val = nullptr, int* vexp = nullptr) {
  double pm = 0.0, p = 1.0;  // p_{-2}, p_{-1}
  unsigned m = 0u;           // sign history, newest in bit 0; p_{-1} > 0
  int cnt = 0, esum = 0;
  // operands in groups of four steps (64 bytes), requested two groups ahead: three buffers in rotation
  double t0[8], t1[8], t2[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    t0[q] = de[q];
    t1[q] = de[8 + q];
  }
#pragma unroll 1
  for (int c = 0; c < 10; ++c) {  // groups 3c, 3c+1, 3c+2
    sc_double* g = de + 24 * c;
#pragma unroll
    for (int q = 0; q < 8; ++q) t2[q] = g[16 + q];
    sturm_steps4<SIGNS>(t0, x, pm, p, m);
#pragma unroll
    for (int q = 0; q < 8; ++q) t0[q] = g[24 + q];
    sturm_steps4<SIGNS>(t1, x, pm, p, m);
#pragma unroll
    for (int q = 0; q < 8; ++q) t1[q] = g[32 + q];
    sturm_steps4<SIGNS>(t2, x, pm, p, m);
    esum += sturm_renorm(pm, p);
    if constexpr (SIGNS) cnt += __popc((m ^ (m >> 1)) & 0xFFFu);  // bit 12 is the sign that preceded these twelve
  }
  sturm_steps4<SIGNS>(t0, x, pm, p, m);  // groups 30 and 31
  sturm_steps4<SIGNS>(t1, x, pm, p, m);
  if constexpr (SIGNS) cnt += __popc((m ^ (m >> 1)) & 0xFFu);
  if (val) {
    esum += sturm_renorm(pm, p);
    *val = p;
    *vexp = esum;
  }
  return cnt;
}

// Back-transformation through the reflectors 16 SG .. 16 SG + 15, four at a time, of the vector whose entries
// i = l + 16 m this lane holds in y[m].  All sixteen reflectors vanish on the entries m < SG, are full on m > SG, and
// reflector k starts inside m = SG (entries l > k % 16); so only that one entry needs a mask and the dead ones are
// skipped.  `refl` has 16 floats of slack in front, which the masked reads of the first reflectors may touch.
template <int SG>
__device__ __forceinline__ void backtransform_stage(double (&y)[8], const float* refl, const double* betaT,
                                                    const double* cW, int l) {
#pragma unroll 1
  for (int bl = 3; bl >= 0; --bl) {
    const int bb = 4 * SG + bl;
    double u[4][8], dt[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int k = 4 * bb + 3 - a;                           // k / 16 == SG
      const float* rp = refl + refl_off(k) - (k + 1) + l;     // entry i at rp[i - l]
      const bool head = (l > (k & 15)) && (SG < 7 || k < D - 2);  // reflectors 126, 127 do not exist
      double acc = 0.0;
#pragma unroll
      for (int m = SG; m < 8; ++m) {
        const float raw = rp[16 * m];
        u[a][m] = (m == SG) ? (head ? (double)raw : 0.0) : (double)raw;
        acc = fma(u[a][m], y[m], acc);
      }
      dt[a] = acc;
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) dt[a] = row16_sum_uniform(dt[a]);
    const double* c = cW + bb * 6;
    const double f1 = betaT[4 * bb + 3] * dt[0];
    const double f2 = betaT[4 * bb + 2] * fma(-c[0], f1, dt[1]);
    const double f3 = betaT[4 * bb + 1] * fma(-c[2], f2, fma(-c[1], f1, dt[2]));
    const double f4 = betaT[4 * bb] * fma(-c[5], f3, fma(-c[4], f2, fma(-c[3], f1, dt[3])));
#pragma unroll
    for (int m = SG; m < 8; ++m)
      y[m] = fma(-f4, u[3][m], fma(-f3, u[2][m], fma(-f2, u[1][m], fma(-f1, u[0][m], y[m]))));
  }
}

// Minors of T - mu I by the three-term recurrence, from the top (UP = false: p_i, stored with p_{i-1}) or from the
// bottom (UP = true: q_i, stored with q_{i+1}); de[i] = (d_i, e_{i-1}^2), de[D] = 0.  Eight steps per group, then
// both running values are rescaled by a power of two (the ratios of consecutive minors are what is used).
template <bool UP>
__device__ __forceinline__ void minors_sweep(const double2* de, double mu, double2* out) {
  double pm = 0.0, p = 1.0;
#pragma unroll 2
  for (int s0 = 0; s0 < D; s0 += 8) {
    double dmu[8], e2[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int i = UP ? D - 1 - (s0 + s) : s0 + s;
      dmu[s] = de[i].x - mu;
      e2[s] = de[i + (UP ? 1 : 0)].y;  // e_{i-1}^2 going down, e_i^2 going up
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int i = UP ? D - 1 - (s0 + s) : s0 + s;
      const double pn = fma(dmu[s], p, -(e2[s] * pm));
      out[i] = make_double2(pn, p);
      pm = p;
      p = pn;
    }
    const int e = __builtin_amdgcn_frexp_exp(p);
    p = ldexp(p, -e);
    pm = ldexp(pm, -e);
  }
}

// Entries of the twisted-factorisation vector on one side of the twist index rt (z_rt = 1): z_i = -mult_i z_{i+1}
// for i < rt (UP = false, multipliers e_i / D+_i in M[i].x) or z_i = -mult_i z_{i-1} for i > rt (UP = true,
// e_{i-1} / D-_i); z_i goes to F[i].y, the sum of their squares to *ssq_out.  Whole groups of eight rows first
// (constant offsets from one moving base, nothing conditional), then the rest row by row.
template <bool UP>
__device__ __forceinline__ void twisted_chain(double2* F, const double2* M, int rt, double* ssq_out) {
  const int count = UP ? D - 1 - rt : rt;
  double z = 1.0, ssq = 0.0;
  if (!UP) F[rt].y = 1.0;
  int s0 = 0;
#pragma unroll 1
  for (; s0 + 8 <= count; s0 += 8) {
    const int i0 = UP ? rt + s0 + 1 : rt - s0 - 8;   // lowest row of the group
    double mlt[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) mlt[s] = M[i0 + (UP ? s : 7 - s)].x;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      z = -mlt[s] * z;
      F[i0 + (UP ? s : 7 - s)].y = z;
      ssq = fma(z, z, ssq);
    }
  }
#pragma unroll 1
  for (; s0 < count; ++s0) {
    const int i = UP ? rt + s0 + 1 : rt - s0 - 1;
    z = -M[i].x * z;
    F[i].y = z;
    ssq = fma(z, z, ssq);
  }
  *ssq_out = ssq;
}

// Inner product number q of the reflectors of group q / 6 = {4b, .., 4b+3}, in the order the back-transformation applies
// them (u_1 = v_{4b+3} .. u_4 = v_{4b}): c21 c31 c32 c41 c42 c43; one product per lane, over the rows where both
// reflectors live (i > kb; what lies outside a reflector is arbitrary)
__device__ __forceinline__ void reflector_product(int q, const float* refl, double* cW) {
  const int bb = q / 6, pr = q - 6 * bb;
  const int a = (pr == 0) ? 2 : ((pr < 3) ? 3 : 4), b2 = (pr == 0) ? 1 : ((pr < 3) ? pr : pr - 2);
  const int ka = 4 * bb + 4 - a, kb = 4 * bb + 4 - b2;  // ka < kb
  const float* pa = refl + refl_off(ka) - (ka + 1);      // entry i of reflector ka at pa[i]
  const float* pb = refl + refl_off(kb) - (kb + 1);
  double acc = 0.0;
  if (kb < D - 2) {
#pragma unroll 4
    for (int i = kb + 1; i < D; ++i) acc = fma((double)pa[i], (double)pb[i], acc);
  }
  cW[q] = acc;
}

__global__ __launch_bounds__(THREADS, 2) void eoq_spectral_tridiag_kernel(
    const void* __restrict__ blocks, EoqBlockMap map, int dtype, int n, int k_pilot, double rank_thr, int r_max, int loss,
    int* __restrict__ fb_list, int* __restrict__ fb_count, double* __restrict__ lam_out, float* __restrict__ wfac,
    double* __restrict__ tri, int32_t* __restrict__ rank_out, float* __restrict__ phi_out, float* __restrict__ sigma_out,
    uint16_t* __restrict__ rfac, uint32_t* __restrict__ flags_out) {
  // one pool, used in turn by the Gram stage (byte planes / float strip), the reduction (reflectors) and the
  // eigenvector stage (u1)
  __shared__ __align__(16) unsigned char pool[POOL_BYTES];
  float* refl = reinterpret_cast<float*>(pool) + REFL_SLACK;
  unsigned char* u1 = pool + REFL_BYTES;
  __shared__ __align__(16) double vbuf[2][D];
  __shared__ __align__(16) double pbuf[8 * PB_LD];
  __shared__ __align__(16) double2 de[D + 1];  // (d_i, e_{i-1}^2) of the scaled tridiagonal matrix; de[D] = 0
  __shared__ double dT[D], eT[D], betaT[D];
  __shared__ double cW[(D / 4) * 6];  // inner products of the reflectors inside each group of four
  __shared__ double norm_s[EV_BATCH];
  __shared__ double chain_s[EV_BATCH][2];  // sums of squares of the two halves of each vector
  __shared__ int twist_s[EV_BATCH];
  __shared__ double lam_s[D], atoms[D];
  __shared__ double scale_s[EOQ_RMAX_CAP];
  __shared__ double tscale_s;
  __shared__ unsigned flag_s;

  const int tid = threadIdx.x;
  const size_t blk = blockIdx.x;
  const size_t slot = map.slot(blk);
  const int lane = tid & 63, wave = tid >> 6;
  if (tid == 0) {
    flag_s = 0u;
    betaT[D - 2] = betaT[D - 1] = 0.0;  // reflectors 126, 127 do not exist
    de[D] = make_double2(0.0, 0.0);
  }

  {
    double A[64];
    if (dtype == EOQ_F16)
      gram_int8(static_cast<const uint16_t*>(blocks) + map.in_base(blk), (size_t)map.token_stride, n, pool,
                reinterpret_cast<uint32_t*>(lam_s), reinterpret_cast<int*>(atoms), tid, A, &flag_s);
    else
      gram_cyclic(blocks, dtype, map.in_base(blk), (size_t)map.token_stride, n, reinterpret_cast<float*>(u1), tid, A, &flag_s);
    __syncthreads();  // the pool changes hands
    EOQ_SFOR(s, 6, householder_stage<s>(A, tid, vbuf, pbuf, refl, dT, eT, betaT););
    if (wave == 1) stash_reflector(vbuf[1], 95, lane, refl);   // reflector 95: the stages stash one step behind
    // the trailing 32 x 32 matrix (rows and columns 96 .. 127: sub-tiles a, b = 6, 7 of every lane) changes hands:
    // through LDS into the 64 lanes of wave 0, which finishes the reduction alone
    double* Ms = reinterpret_cast<double*>(u1);   // [32][33]
    double* vring = Ms + 32 * 33;                 // [30][32]: the reflectors of the last 30 steps as doubles
    {
      const int ty = tid >> 4, tx = tid & 15;
      EOQ_SFOR(a, 2, EOQ_SFOR(b, 2, Ms[(ty + 16 * a) * 33 + tx + 16 * b] = A[(6 + a) * 8 + 6 + b];););
    }
    __syncthreads();
    if (wave == 0) {
      const int ly = lane >> 3, lx = lane & 7;
      double T[16];
      EOQ_SFOR(e, 16, T[e] = Ms[(ly + 8 * (e >> 2)) * 33 + lx + 8 * (e & 3)];);
      EOQ_SFOR(ao, 4, tail32_stage<ao>(T, lane, vring, pbuf, dT, eT, betaT););
      // the last 2x2 block of T: rows and columns 126, 127 = local 30, 31 = (ly, lx) in {6, 7}, a = b = 3
      if (ly == 6 && lx == 6) dT[D - 2] = T[15];
      if (ly == 7 && lx == 6) eT[D - 2] = T[15];
      if (ly == 7 && lx == 7) dT[D - 1] = T[15];
    } else if (tid - 64 < 144) {
      // meanwhile the other waves form the inner products of the reflectors 0 .. 95 (groups 0 .. 23), whose float
      // copies are complete
      reflector_product(tid - 64, refl, cW);
    }
    __syncthreads();
    // float copies of the last 30 reflectors (local entries c > kq of step kq), by everybody
#pragma unroll
    for (int e = tid; e < 30 * 32; e += THREADS) {
      const int kq = e >> 5, c = e & 31;
      if (c > kq) refl[refl_off(96 + kq) + c - kq - 1] = (float)vring[e];
    }
  }
  __syncthreads();
  // the inner products of the reflectors 96 .. 127 (the others were formed beside the one-wave tail): by the last wave,
  // while the first scales the tridiagonal matrix
  if (tid >= THREADS - 48) reflector_product(144 + tid - (THREADS - 48), refl, cW);

  // ---- eigenvalues of T by Sturm-count multisection: lane pair j brackets the j-th smallest ----
  {
    // power-of-two scaling (exact) so that every |d_i| + |e_{i-1}| + |e_i| <= 1
    if (wave == 0) {
      double b0 = fabs(dT[lane]) + ((lane > 0) ? fabs(eT[lane - 1]) : 0.0) + fabs(eT[lane]);
      const int l2 = lane + 64;
      double b1 = fabs(dT[l2]) + fabs(eT[l2 - 1]) + ((l2 < D - 1) ? fabs(eT[l2]) : 0.0);
      double b = fmax(b0, b1);
#pragma unroll
      for (int m = 32; m >= 1; m >>= 1) b = fmax(b, __shfl_xor(b, m, 64));
      if (lane == 0) tscale_s = (b > 0.0) ? ldexp(1.0, -(ilogb(b) + 1)) : 1.0;
    }
    __syncthreads();
    const double sc = tscale_s;
    double2* tri_blk = reinterpret_cast<double2*>(tri) + blk * D;
    if (tid < D) {
      const double e = (tid > 0) ? eT[tid - 1] * sc : 0.0;
      const double2 t = make_double2(dT[tid] * sc, e * e);
      de[tid] = t;
      tri_blk[tid] = t;
    }
    __threadfence();
    __syncthreads();
    // the copy in global memory, addressed through the scalar unit; the address passes through an opaque
    // register move placed after the barrier so that none of these loads can be scheduled before the stores
    unsigned long long tri_addr = reinterpret_cast<unsigned long long>(tri_blk);
    asm volatile("" : "+s"(tri_addr) : : "memory");
    sc_double* sde = reinterpret_cast<sc_double*>(tri_addr);
    const int j = tid >> 1, sub = tid & 1;
    double lo = -0x1.0p-40, hi = 1.0 + 0x1.0p-40;   // G is positive semi-definite; Gershgorin bounds the top by 1
    // What is known about the two ends: the count there (c_lo <= j < c_hi always: every update below follows the
    // counts, so the bracket holds eigenvalue j whatever else happens) and, once an end is a point that was evaluated,
    // the value of det(T - x I) there as f * 2^e, f in float32 (its sign and a few digits are all that is used).
    // One word per end: e << 8 | count; f = 0 stands for "no value".
    int ce_lo = 0, ce_hi = D;
    float f_lo = 0.0f, f_hi = 0.0f;
    {
      // every lane counts at one point of a uniform grid; each eigenvalue then starts from its grid cell
      int* ce_s = reinterpret_cast<int*>(atoms);
      float* gval_s = reinterpret_cast<float*>(&vbuf[0][0]);   // the reduction's buffers are free by now
      // grid point g at ((g + 1) / 257)^3: most eigenvalues of a block are noise eigenvalues far below the largest
      // one, so the points crowd towards zero (a cell near the top is 3 / 257 wide, a cell at 0.03 is 0.001 wide)
      const double step = 1.0 / (GRID_POINTS + 1);
      auto grid_x = [&](int g) __attribute__((always_inline)) {
        const double t = (g + 1) * step;
        return t * t * t;
      };
      double gv;
      int ge;
      const int gc = sturm_count(sde, grid_x(tid), &gv, &ge);
      ce_s[tid] = (ge << 8) | gc;
      gval_s[tid] = (float)gv;
      __syncthreads();
      int gl = -1, gh = GRID_POINTS;  // counts at these grid points: <= j and > j
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        const int mid = (gl + gh) >> 1;
        if ((ce_s[mid] & 0xFF) > j) gh = mid; else gl = mid;
      }
      if (gl >= 0) {
        lo = grid_x(gl);
        ce_lo = ce_s[gl];
        f_lo = gval_s[gl];
      }
      if (gh < GRID_POINTS) {
        hi = grid_x(gh);
        ce_hi = ce_s[gh];
        f_hi = gval_s[gh];
      }
    }
    // Rounds of two points per eigenvalue (one per lane of the pair) until every bracket of the wave is at most
    // 3^-17 / 257 wide (what 17 trisections of a uniform grid cell give; the second phase counts on it).  A bracket
    // that holds exactly one eigenvalue and has values of det(T - x I) of opposite signs at its ends puts the two points
    // at t -+ delta around the secant point t (t kept 2 delta away from the ends).  delta starts at 1/6 -- thirds
    // centred on the secant point -- and a hit, which leaves 2 delta of the width, shrinks it fourfold for the next
    // round (the secant point of a smooth function with one root in the bracket is off by a fraction of the width that
    // is itself proportional to the width); a miss puts it back to 1/6, where either outcome leaves at most half.
    // Brackets with several eigenvalues are cut in thirds.  The loop bound is never reached: from the third round
    // after a miss at the latest every round halves the bracket.
    constexpr double WIDTH_TARGET = 1.0 / (129140163.0 * 257.0);
    float delta = 1.0f / 6.0f;
#pragma unroll 1
    for (int it = 0; it < 80; ++it) {
      const double w = hi - lo;
      if (__ballot(w > WIDTH_TARGET) == 0ull) break;   // wave-uniform
      // f_lo / (f_lo - f_hi) with the two values brought to one exponent
      const int ediff = min(max((ce_hi >> 8) - (ce_lo >> 8), -100), 100);
      const float fh = ldexpf(f_hi, ediff);
      const float ratio = f_lo * __builtin_amdgcn_rcpf(f_lo - fh);
      const bool secant = ((ce_hi - ce_lo) & 0xFF) == 1 && f_lo * fh < 0.0f && ratio > 0.0f && ratio < 1.0f;
      const float tc = fminf(fmaxf(ratio, 2.0f * delta), 1.0f - 2.0f * delta);
      const float tsel = secant ? (sub ? tc + delta : tc - delta) : (sub ? (2.0f / 3.0f) : (1.0f / 3.0f));
      const float toth = secant ? (sub ? tc - delta : tc + delta) : (sub ? (1.0f / 3.0f) : (2.0f / 3.0f));
      const double xm = fma((double)tsel, w, lo), xo = fma((double)toth, w, lo);   // this lane's point, the partner's
      double fv;
      int fe;
      int mine;
      // Once every bracket of the wave holds one eigenvalue and has a value at either end, the sign of det(T - x I)
      // alone says on which side of the point the eigenvalue lies (it changes sign once in the bracket): the count is
      // the lower end's, plus one where the sign differs from the one there.
      const bool by_sign = __ballot(((ce_hi - ce_lo) & 0xFF) != 1 || f_lo == 0.0f || f_hi == 0.0f) == 0ull;   // wave-uniform
      if (by_sign) {
        (void)sturm_count<false>(sde, xm, &fv, &fe);
        mine = (ce_lo & 0xFF) + (((__double2hiint(fv) ^ __float_as_int(f_lo)) < 0) ? 1 : 0);
      } else {
        mine = sturm_count(sde, xm, &fv, &fe);
      }
      const int cem = (fe << 8) | mine;
      const float fm = (float)fv;
      const int ceo = dpp_mov<0xB1>(cem);
      const float fo = dpp_mov<0xB1>(fm);
      const double x1 = sub ? xo : xm, x2 = sub ? xm : xo;
      const int ce1 = sub ? ceo : cem, ce2 = sub ? cem : ceo;
      const float f1 = sub ? fo : fm, f2 = sub ? fm : fo;
      const bool a1 = (ce1 & 0xFF) > j, a2 = (ce2 & 0xFF) > j;   // the eigenvalue lies below x1 / below x2
      // below x1: [lo, x1]; between: [x1, x2]; above x2: [x2, hi]
      hi = a1 ? x1 : (a2 ? x2 : hi);
      ce_hi = a1 ? ce1 : (a2 ? ce2 : ce_hi);
      f_hi = a1 ? f1 : (a2 ? f2 : f_hi);
      lo = a1 ? lo : (a2 ? x1 : x2);
      ce_lo = a1 ? ce_lo : (a2 ? ce1 : ce2);
      f_lo = a1 ? f_lo : (a2 ? f1 : f2);
      const bool hit = a2 && !a1;
      delta = !secant ? delta : (hit ? fmaxf(0.25f * delta, 0x1.0p-12f) : 1.0f / 6.0f);
    }
    if (sub == 0) lam_s[D - 1 - j] = fmax(0.5 * (lo + hi), 0.0) / sc;   // descending order, unscaled
    // Most eigenvalues stay at that width (3e-11 of the largest): they only enter sums.  Full precision is for those
    // that feed the twisted factorisations, the shrinker and the rank rule: with the rank rt that the eigenvalues
    // at hand give, the rt + 1 largest (the retained ones and the first one below them) and the two of the bulk-edge
    // estimate (Alg. 2 step 1: numbers k + 1 and 2k + 1).  They share the 256 lanes, G = 8 .. 64 lanes each: the
    // interval is cut in G + 1 at the points x_s = lo + (s + 1) w and the new bounds are recomputed by every lane
    // of a group from the same expression, so the lanes of a group stay identical.
    __syncthreads();   // the grid counts in `atoms` are no longer read; every lam_s is written
    {
      const int i_desc = D - 1 - j;
      if (sub == 0 && i_desc < REFINE_KEEP) {
        atoms[2 * i_desc] = lo;
        atoms[2 * i_desc + 1] = hi;
      }
    }
    int rt;
    {
      const double edge_coef = 1.0 / (cbrt(4.0) - 1.0);
      const double lam_k1 = lam_s[k_pilot], lam_2k1 = lam_s[2 * k_pilot];
      const double lam_plus = lam_k1 + edge_coef * (lam_k1 - lam_2k1);
      rt = __syncthreads_count((tid < D && lam_s[tid] / lam_plus - 1.0 > rank_thr) ? 1 : 0);   // also orders `atoms`
    }
    {
      // rt + 3 eigenvalues when they fit 32 groups, else the 32 largest (all that can be retained)
      const bool wide = rt + 3 <= REFINE_COUNT && 2 * k_pilot < REFINE_KEEP;
      const int count = wide ? rt + 3 : REFINE_COUNT;
      const int lg = !wide ? 3 : (count > 16 ? 3 : (count > 8 ? 4 : (count > 4 ? 5 : 6)));   // log2 of the group size
      const int G = 1 << lg;
      const int iters = (lg == 3) ? 5 : ((lg == 4) ? 4 : 3);   // (G + 1)^iters * 3^17 * 257 > 2^49
      const double inv = (lg == 3) ? 1.0 / 9.0 : ((lg == 4) ? 1.0 / 17.0 : ((lg == 5) ? 1.0 / 33.0 : 1.0 / 65.0));
      const int jj = tid >> lg, sg = tid & (G - 1);
      const bool act = jj < count;
      // descending index of this group's eigenvalue
      const int i_desc = !act ? 0 : (!wide ? jj : (jj <= rt ? jj : (jj == rt + 1 ? k_pilot : 2 * k_pilot)));
      const int jr = D - 1 - i_desc;
      double rlo = atoms[2 * i_desc], rhi = atoms[2 * i_desc + 1];
      const int shift = (tid & 63) & ~(G - 1);
      const unsigned long long gmask = (lg == 6) ? ~0ull : ((1ull << G) - 1ull);
#pragma unroll 1
      for (int it = 0; it < iters; ++it) {
        const double w = (rhi - rlo) * inv;
        const int c = sturm_count(sde, fma((double)(sg + 1), w, rlo));
        const unsigned long long below = __ballot(c <= jr);   // points not above the eigenvalue: a prefix of the group
        const int mcount = __popcll((below >> shift) & gmask);
        rhi = (mcount == G) ? rhi : fma((double)(mcount + 1), w, rlo);
        rlo = fma((double)mcount, w, rlo);
      }
      if (act && sg == 0) lam_s[i_desc] = fmax(0.5 * (rlo + rhi), 0.0) / sc;
    }
  }
  __syncthreads();

  const int r = rank_and_shrink(lam_s, atoms, scale_s, &flag_s, n, k_pilot, rank_thr, r_max, loss, blk, slot, lam_out,
                                phi_out, sigma_out);

  // repeated retained eigenvalues: leave the block to the Jacobi solver
  bool repeated = false;
  for (int i = 0; i < r; ++i)
    if (lam_s[i] - lam_s[i + 1] <= CLUSTER_TOL * lam_s[0]) repeated = true;
  if (repeated) {
    if (tid == 0) {
      const int fb_slot = atomicAdd(fb_count, 1);
      fb_list[fb_slot] = (int)blk;
      rank_out[slot] = r;
      flags_out[slot] = flag_s;
    }
    return;
  }

  // ---- eigenvectors of the retained components ----
  // For a retained eigenvalue mu the vector comes from the twisted factorisation of T - mu I.  Its pivots are
  // ratios of consecutive minors, D+_i = p_i / p_{i-1} (leading minors, from the top) and D-_i = q_i / q_{i+1}
  // (trailing minors, from the bottom), so the two sequential sweeps are division-free three-term recurrences and
  // every division happens afterwards, all rows in parallel.  The twist index minimises
  // |gamma_i| = |D+_i + D-_i - (d_i - mu)|; z_twist = 1, z_i = -(e_i / D+_i) z_{i+1} above it and
  // z_i = -(e_{i-1} / D-_i) z_{i-1} below it.
  double2* tw = reinterpret_cast<double2*>(u1);  // per eigenvector of a batch: F[128] (top-down) then Bk[128] (bottom-up)
  const double sc = tscale_s;
#pragma unroll 1
  for (int b0 = 0; b0 < r; b0 += EV_BATCH) {
    __syncthreads();
    // (1) minors: wave 0 runs the top-down recurrences, wave 1 the bottom-up ones, one lane per eigenvector (the
    // direction is then the same for a whole wave: constant offsets, no selects); F[i] = (p_i, p_{i-1}),
    // Bk[i] = (q_i, q_{i+1})
    if (wave < 2 && lane < EV_BATCH && b0 + lane < r) {
      const double mu = lam_s[b0 + lane] * sc;
      if (wave == 0) minors_sweep<false>(de, mu, tw + (lane * 2) * TW_STRIDE);
      else minors_sweep<true>(de, mu, tw + (lane * 2 + 1) * TW_STRIDE);
    }
    __syncthreads();
    // (2) pivots, multipliers and twist index: rows i = l + LG m of eigenvector tid / LG, with LG = 64 lanes per
    // eigenvector while a batch has at most four of them (the usual case: all four waves share the divisions, two
    // rows each) and 16 lanes otherwise
    {
      auto pivots = [&](auto lg_ic) __attribute__((always_inline)) {
        constexpr int LG = decltype(lg_ic)::value;
        const int ev = tid / LG, l = tid % LG;
        if (ev < EV_BATCH && b0 + ev < r) {
          const double mu = lam_s[b0 + ev] * sc;
          double2* F = tw + ev * 2 * TW_STRIDE;
          double2* Bk = F + TW_STRIDE;
          const double piv = 0x1.0p-100;  // smallest pivot magnitude (the matrix is scaled to norm <= 1)
          double best = INFINITY;
#pragma unroll
          for (int m = 0; m < D / LG; ++m) {
            const int i = l + LG * m;
            const double2 f = F[i], bq = Bk[i];
            const double fn = (fabs(f.x) < piv * fabs(f.y)) ? copysign(piv * fabs(f.y), f.x) : f.x;
            const double bn = (fabs(bq.x) < piv * fabs(bq.y)) ? copysign(piv * fabs(bq.y), bq.x) : bq.x;
            double g = fabs(fma(fn, newton_rcp(f.y), fma(bn, newton_rcp(bq.y), -(de[i].x - mu))));
            if (!(g == g)) g = INFINITY;
            double lmul = (i < D - 1) ? eT[i] * sc * f.y * newton_rcp(fn) : 0.0;   // e_i / D+_i
            double umul = (i > 0) ? eT[i - 1] * sc * bq.y * newton_rcp(bn) : 0.0;  // e_{i-1} / D-_i
            if (!isfinite(lmul)) lmul = 0.0;
            if (!isfinite(umul)) umul = 0.0;
            F[i].x = lmul;
            Bk[i].x = umul;
            // the row index rides in the low mantissa bits: the minimum of the keys carries its own position
            const double key = __hiloint2double(__double2hiint(g), (__double2loint(g) & ~127) | i);
            best = fmin(best, key);
          }
          best = fmin(best, dpp_mov<0xB1>(best));
          best = fmin(best, dpp_mov<0x4E>(best));
          best = fmin(best, dpp_mov<0x141>(best));
          best = fmin(best, dpp_mov<0x140>(best));
          if constexpr (LG == 64) {
            best = fmin(best, __shfl_xor(best, 16, 64));
            best = fmin(best, __shfl_xor(best, 32, 64));
          }
          if (l == 0) twist_s[ev] = __double2loint(best) & 127;
        }
      };
      if (r - b0 <= 4) pivots(std::integral_constant<int, 64>{});
      else pivots(std::integral_constant<int, 16>{});
    }
    __syncthreads();
    // (3) the vector itself, upwards (wave 0) and downwards (wave 1) from the twist index; z_i goes to F[i].y
    if (wave < 2 && lane < EV_BATCH && b0 + lane < r) {
      double2* F = tw + lane * 2 * TW_STRIDE;
      const int rt = twist_s[lane];
      if (wave == 0) twisted_chain<false>(F, F, rt, &chain_s[lane][0]);
      else twisted_chain<true>(F, F + TW_STRIDE, rt, &chain_s[lane][1]);
    }
    __syncthreads();
    if (tid < EV_BATCH && b0 + tid < r) {
      const double ssq = 1.0 + chain_s[tid][0] + chain_s[tid][1];
      norm_s[tid] = ssq;
      if (!(ssq > 0.0) || !isfinite(ssq)) atomicOr(&flag_s, EOQ_FLAG_NO_CONVERGE);
    }
    __syncthreads();
    // (4) back-transformation v = H_0 H_1 ... H_125 z, four reflectors at a time: 16 lanes per eigenvector, 8
    // entries (i = l + 16 m) each.  With u_1 .. u_4 = v_{4b+3} .. v_{4b} (order of application), d_a = u_a^T y and
    // c_ab = u_a^T u_b (prepared once per block), the four coefficients follow from a triangular recurrence and
    // y <- y - sum_a f_a u_a.
    if (tid < 16 * EV_BATCH) {
      const int ev = tid >> 4, l = tid & 15;
      const bool live = (b0 + ev < r);
      const double2* F = tw + ev * 2 * TW_STRIDE;
      double y[8];
      {
        const double ssq = live ? norm_s[ev] : 1.0;
        const double inv = (ssq > 0.0 && isfinite(ssq)) ? 1.0 / sqrt(ssq) : 0.0;
#pragma unroll
        for (int m = 0; m < 8; ++m) y[m] = live ? F[l + 16 * m].y * inv : 0.0;
      }
      EOQ_SFOR(sgr, 8, backtransform_stage<7 - sgr>(y, refl, betaT, cW, l););
      if (live) {
        const double s = scale_s[b0 + ev];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const int i = l + 16 * m;
          rfac[(slot * r_max + b0 + ev) * D + i] = double_to_half_bits(y[m]);
          wfac[(blk * r_max + b0 + ev) * D + i] = (float)(y[m] * s);
        }
      }
    }
  }
  if (tid == 0) {
    rank_out[slot] = r;
    flags_out[slot] = flag_s;
  }
}

__global__ void eoq_zero_counter_kernel(int* counter) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *counter = 0;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------------------------
hipError_t eoq_launch_spectral(const EoqLaunch& L, const void* blocks, int dtype, int64_t B, double* lam,
                               float* wfac, int* fb_count, int* fb_list, double* tri, eoq_packed out) {
  if (L.ev) (void)hipEventRecord(L.ev[0], L.stream);
  if (L.solver == 1) {
    hipLaunchKernelGGL(eoq_spectral_jacobi_kernel, dim3((unsigned)B), dim3(THREADS), 0, L.stream, blocks, L.map, dtype, L.n,
                       L.k, L.rank_thr, L.r_max, L.loss, B, (const int*)nullptr, (const int*)nullptr, lam, wfac, out.rank,
                       out.phi, out.sigma, out.rfac, out.flags);
  } else {
    hipLaunchKernelGGL(eoq_zero_counter_kernel, dim3(1), dim3(64), 0, L.stream, fb_count);
    hipLaunchKernelGGL(eoq_spectral_tridiag_kernel, dim3((unsigned)B), dim3(THREADS), 0, L.stream, blocks, L.map, dtype, L.n,
                       L.k, L.rank_thr, L.r_max, L.loss, fb_list, fb_count, lam, wfac, tri, out.rank, out.phi, out.sigma, out.rfac,
                       out.flags);
    const unsigned grid = (unsigned)((B < 256) ? B : 256);
    hipLaunchKernelGGL(eoq_spectral_jacobi_kernel, dim3(grid), dim3(THREADS), 0, L.stream, blocks, L.map, dtype, L.n, L.k,
                       L.rank_thr, L.r_max, L.loss, B, (const int*)fb_list, (const int*)fb_count, lam, wfac, out.rank, out.phi,
                       out.sigma, out.rfac, out.flags);
  }
  if (L.ev) (void)hipEventRecord(L.ev[1], L.stream);
  return hipGetLastError();
}
