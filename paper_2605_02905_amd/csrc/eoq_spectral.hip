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

// Compile-time loop: every index into a per-lane register array must be a constant before the optimiser
// first looks at the array, otherwise the array is kept in (scratch) memory.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}
#define EOQ_SFOR(var, n, ...) static_for<0, n>([&](auto var##_ic) __attribute__((always_inline)) { \
  constexpr int var = decltype(var##_ic)::value; __VA_ARGS__ })

__device__ __forceinline__ void gram_tile(const void* __restrict__ blocks, int dtype, size_t base_elem, int n,
                                          float* stage, int tid, double (&acc)[64]) {
  const int ty = tid >> 4, tx = tid & 15;
  EOQ_SFOR(i, 64, acc[i] = 0.0;);
  for (int t0 = 0; t0 < n; t0 += STAGE_ROWS) {
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int e = (g * THREADS + tid) * 8;
      float v[8];
      load8(blocks, dtype, base_elem + (size_t)t0 * D + e, v);
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
                               double rank_thr, int r_max, size_t blk, double* __restrict__ lam_out,
                               float* __restrict__ phi_out, float* __restrict__ sigma_out) {
  const int tid = threadIdx.x;
  if (tid < D) lam_out[blk * D + tid] = lam_s[tid];

  // Step 1: lambda_+ = lam_{k+1} + (lam_{k+1} - lam_{2k+1}) / (2^{2/3} - 1);  r = #{ lam_i / lambda_+ - 1 > d^{-1/3} }
  const double edge_coef = 1.0 / (cbrt(4.0) - 1.0);
  const double lam_k1 = lam_s[k], lam_2k1 = lam_s[2 * k];
  const double lam_plus = lam_k1 + edge_coef * (lam_k1 - lam_2k1);
  const int above = (tid < D) ? ((lam_s[tid] / lam_plus - 1.0 > rank_thr) ? 1 : 0) : 0;
  int r = __syncthreads_count(above);
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

  // Step 3: Stieltjes transforms of the noise measure at each outlier, D-transform, Frobenius shrinker
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
          // phi = d sqrt(a_1 a_2) with d = T^{-1/2}, a_x = m_x / (d^2 T')
          const double dh = 1.0 / sqrt(T);
          const double a1 = m_l / (dh * dh * dT), a2 = m_s / (dh * dh * dT);
          phi = dh * sqrt(a1 * a2);
          ok = isfinite(phi);
          if (ok) phi = fmin(fmax(phi, 0.0), sig);
        }
        if (!ok) {
          phi = 0.0;
          atomicOr(flag_s, EOQ_FLAG_SHRINK_GUARD);
        }
        phi_out[blk * r_max + i] = (float)phi;
        sigma_out[blk * r_max + i] = (float)sig;
        scale_s[i] = (sig > 0.0) ? phi / sig : 0.0;
      }
    }
    for (int i = r + tid; i < r_max; i += THREADS) {
      phi_out[blk * r_max + i] = 0.0f;
      sigma_out[blk * r_max + i] = 0.0f;
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
    const void* __restrict__ blocks, int dtype, int n, int k, double rank_thr, int r_max, int64_t B,
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
    __syncthreads();
    if (tid == 0) flag_s = 0u;

    {
      double acc[64];
      gram_tile(blocks, dtype, blk * (size_t)n * D, n, stage, tid, acc);
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

    const int r = rank_and_shrink(lam_s, atoms, scale_s, &flag_s, n, k, rank_thr, r_max, blk, lam_out, phi_out,
                                  sigma_out);

    // right singular vectors v_i = a_slot / lambda_i of the retained components
    for (int e = tid; e < r * D; e += THREADS) {
      const int i = e >> 7, j = e & (D - 1);
      const double li = lam_s[i];
      const double v = (li > 0.0) ? A[slot_of[i] * LDA + j] / li : 0.0;
      rfac[(blk * r_max + i) * D + j] = double_to_half_bits(v);
      wfac[(blk * r_max + i) * D + j] = (float)(v * scale_s[i]);
    }
    if (tid == 0) {
      rank_out[blk] = r;
      flags_out[blk] = flag_s | ((unsigned)sweeps << EOQ_FLAG_SWEEPS_SHIFT);
    }
  }
}

// =============================================================================================
// Tridiagonal solver
// =============================================================================================
// Row layout of the working matrix: lane pair (2i, 2i+1) owns row i; lane parity h holds the columns
// j = 2c + h in A[c], c = 0..63.  Vectors that are read along columns live in LDS in "split" order:
// element j at position (j & 1) * 64 + (j >> 1), so a lane reads its 64 columns contiguously.
__device__ __forceinline__ int split_pos(int j) { return ((j & 1) << 6) | (j >> 1); }
// packed reflector storage: reflector k has entries i = k+1 .. 127
__device__ __forceinline__ int refl_off(int k) { return k * (D - 1) - (k * (k - 1)) / 2; }
constexpr int REFL_LEN = (D - 1) * D / 2;  // 8128
constexpr int TPAD = D + 2;                // row stride of the transposition buffer
constexpr int U1_BYTES = 4 * 8 * TPAD * 8; // 33280: also covers the Gram strip (16 KB) and the twisted scratch (32 KB)
constexpr int MULTISECT_ITERS = 34;        // 3^34 > 2^53
constexpr int EV_BATCH = 8;                // eigenvectors per twisted-factorisation pass
constexpr double CLUSTER_TOL = 1e-10;      // relative gap below which retained eigenvalues count as repeated

// A[c] with a wave-uniform run-time index c: a two-level switch over values that are already in registers
// (all other accesses to the array use compile-time indices, so it never exists in memory).
// Keeps a value in a register at this point: stops the optimiser from merging the per-case loads / stores of
// the switches below into one access through a selected address (which would force the array into memory).
__device__ __forceinline__ double pinned(double v) {
  asm volatile("" : "+v"(v));
  return v;
}
template <int G>
__device__ __forceinline__ double pick8(const double (&A)[64], int e) {
  switch (e) {
    case 0: return pinned(A[G * 8 + 0]);
    case 1: return pinned(A[G * 8 + 1]);
    case 2: return pinned(A[G * 8 + 2]);
    case 3: return pinned(A[G * 8 + 3]);
    case 4: return pinned(A[G * 8 + 4]);
    case 5: return pinned(A[G * 8 + 5]);
    case 6: return pinned(A[G * 8 + 6]);
    default: return pinned(A[G * 8 + 7]);
  }
}
__device__ __forceinline__ double pick(const double (&A)[64], int c) {
  const int e = c & 7;
  switch (c >> 3) {
    case 0: return pick8<0>(A, e);
    case 1: return pick8<1>(A, e);
    case 2: return pick8<2>(A, e);
    case 3: return pick8<3>(A, e);
    case 4: return pick8<4>(A, e);
    case 5: return pick8<5>(A, e);
    case 6: return pick8<6>(A, e);
    default: return pick8<7>(A, e);
  }
}
template <int G>
__device__ __forceinline__ void add8(double (&A)[64], int e, double delta) {
  switch (e) {
    case 0: A[G * 8 + 0] = pinned(A[G * 8 + 0] + delta); break;
    case 1: A[G * 8 + 1] = pinned(A[G * 8 + 1] + delta); break;
    case 2: A[G * 8 + 2] = pinned(A[G * 8 + 2] + delta); break;
    case 3: A[G * 8 + 3] = pinned(A[G * 8 + 3] + delta); break;
    case 4: A[G * 8 + 4] = pinned(A[G * 8 + 4] + delta); break;
    case 5: A[G * 8 + 5] = pinned(A[G * 8 + 5] + delta); break;
    case 6: A[G * 8 + 6] = pinned(A[G * 8 + 6] + delta); break;
    default: A[G * 8 + 7] = pinned(A[G * 8 + 7] + delta); break;
  }
}
__device__ __forceinline__ void add_at(double (&A)[64], int c, double delta) {
  const int e = c & 7;
  switch (c >> 3) {
    case 0: add8<0>(A, e, delta); break;
    case 1: add8<1>(A, e, delta); break;
    case 2: add8<2>(A, e, delta); break;
    case 3: add8<3>(A, e, delta); break;
    case 4: add8<4>(A, e, delta); break;
    case 5: add8<5>(A, e, delta); break;
    case 6: add8<6>(A, e, delta); break;
    default: add8<7>(A, e, delta); break;
  }
}

// Number of eigenvalues of the (scaled) tridiagonal matrix below x.  de[i] = (d_i, e_{i-1}^2), e_{-1} = 0.
// Sign changes of the leading principal minors p_i(x) = (d_i - x) p_{i-1} - e_{i-1}^2 p_{i-2}.
__device__ __forceinline__ int sturm_count(const double2* de, double x) {
  double pm = 1.0, p = de[0].x - x;
  int cnt = (int)((unsigned)__double2hiint(p) >> 31);
#pragma unroll 8
  for (int i = 1; i < D; ++i) {
    const double2 t = de[i];
    const double pn = fma(t.x - x, p, -(t.y * pm));
    cnt += (int)(((unsigned)(__double2hiint(pn) ^ __double2hiint(p))) >> 31);
    pm = p;
    p = pn;
    if ((i & 7) == 7) {  // keep the pair in range; the matrix is scaled so |d - x| <= 2, e^2 <= 1
      const double a = fabs(p);
      const double s = (a > 0x1.0p+200) ? 0x1.0p-200 : ((a < 0x1.0p-200) ? 0x1.0p+200 : 1.0);
      p *= s;
      pm *= s;
    }
  }
  return cnt;
}

__global__ __launch_bounds__(THREADS, 2) void eoq_spectral_tridiag_kernel(
    const void* __restrict__ blocks, int dtype, int n, int k_pilot, double rank_thr, int r_max,
    int* __restrict__ fb_list, int* __restrict__ fb_count, double* __restrict__ lam_out, float* __restrict__ wfac,
    int32_t* __restrict__ rank_out, float* __restrict__ phi_out, float* __restrict__ sigma_out,
    uint16_t* __restrict__ rfac, uint32_t* __restrict__ flags_out) {
  __shared__ __align__(16) unsigned char u1[U1_BYTES];
  __shared__ float refl[REFL_LEN];
  __shared__ __align__(16) double xbuf[2][D];
  __shared__ __align__(16) double pbuf[2][D];
  __shared__ __align__(16) double2 de[D];  // (d_i, e_{i-1}^2) of the scaled tridiagonal matrix
  __shared__ double dT[D], eT[D], betaT[D];
  __shared__ double lam_s[D], atoms[D];
  __shared__ double scale_s[EOQ_RMAX_CAP];
  __shared__ double tscale_s;
  __shared__ unsigned flag_s;

  const int tid = threadIdx.x;
  const size_t blk = blockIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  if (tid == 0) flag_s = 0u;

  double A[64];
  // ---- Gram matrix as 8x8 tiles, then into the row layout through LDS (8 rows per wave and round) ----
  gram_tile(blocks, dtype, blk * (size_t)n * D, n, reinterpret_cast<float*>(u1), tid, A);
  {
    double* tb = reinterpret_cast<double*>(u1) + wave * (8 * TPAD);
    const int sub = lane >> 4, tx = lane & 15;
#pragma unroll 1
    for (int s = 0; s < 4; ++s) {
      __syncthreads();
      if (sub == s) {
        EOQ_SFOR(e, 64, tb[(e >> 3) * TPAD + tx * 8 + (e & 7)] = A[e];);
      }
      __syncthreads();
      if (sub == s) {
        const int rho = tx >> 1, hh = tx & 1;
        EOQ_SFOR(c, 64, A[c] = tb[rho * TPAD + 2 * c + hh];);
      }
    }
  }
  const int row = tid >> 1, h = tid & 1;

  // ---- Householder reduction G = Q T Q^T, Q = H_0 H_1 ... H_125, H_k = I - beta_k v_k v_k^T ----
#pragma unroll 1
  for (int k = 0; k < D - 2; ++k) {
    const int par = k & 1;
    double* xb = xbuf[par];
    double* pb = pbuf[par];
    {
      // column k below the diagonal = A[i][k], held by the lanes of parity k&1 at c = k>>1
      const double xi = pick(A, k >> 1);
      if (h == par) {
        xb[split_pos(row)] = (row > k) ? xi : 0.0;
        if (row == k) dT[k] = xi;
      }
    }
    __syncthreads();
    const double ss = wave_sum_uniform(fma(xb[lane], xb[lane], xb[lane + 64] * xb[lane + 64]));
    const double x0 = xb[split_pos(k + 1)];
    double alpha = 0.0, beta = 0.0;
    if (ss > 0.0) {
      const double sigma = sqrt(ss);
      alpha = (x0 >= 0.0) ? -sigma : sigma;          // H_k x = alpha e_1
      beta = 1.0 / (ss + sigma * fabs(x0));          // 2 / (v^T v), v = x - alpha e_1
    }
    const double v_i = xb[split_pos(row)] - ((row == k + 1) ? alpha : 0.0);
    if (h == 1 && row > k) refl[refl_off(k) + row - k - 1] = (float)v_i;
    if (tid == 0) {
      eT[k] = alpha;
      betaT[k] = beta;
    }
    // p = beta A v over the trailing columns; the entry v_{k+1} = x_0 - alpha is applied as a correction
    const int g0 = (k + 1) >> 4;  // first chunk of 8 columns (per parity) that still has live entries
    const double* xh = xb + h * 64;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    EOQ_SFOR(g, 8,
      if (g >= g0) {
        a0 = fma(A[g * 8 + 0], xh[g * 8 + 0], a0);
        a1 = fma(A[g * 8 + 1], xh[g * 8 + 1], a1);
        a2 = fma(A[g * 8 + 2], xh[g * 8 + 2], a2);
        a3 = fma(A[g * 8 + 3], xh[g * 8 + 3], a3);
        a0 = fma(A[g * 8 + 4], xh[g * 8 + 4], a0);
        a1 = fma(A[g * 8 + 5], xh[g * 8 + 5], a1);
        a2 = fma(A[g * 8 + 6], xh[g * 8 + 6], a2);
        a3 = fma(A[g * 8 + 7], xh[g * 8 + 7], a3);
      });
    double acc = (a0 + a1) + (a2 + a3);
    const int c1 = (k + 1) >> 1, h1 = (k + 1) & 1;
    {
      const double ak1 = pick(A, c1);
      if (h == h1) acc = fma(-alpha, ak1, acc);
    }
    acc = pair_sum(acc);
    const double p_i = beta * acc;
    if (h == 0) pb[split_pos(row)] = p_i;
    __syncthreads();
    // K = (beta/2) v^T p ;  w = p - K v ;  A <- A - v w^T - w v^T
    const int pk1 = split_pos(k + 1);
    const double va = xb[lane] - ((lane == pk1) ? alpha : 0.0);
    const double vb = xb[lane + 64] - ((lane + 64 == pk1) ? alpha : 0.0);
    const double dot = wave_sum_uniform(fma(va, pb[lane], vb * pb[lane + 64]));
    const double K = 0.5 * beta * dot;
    const double w_i = fma(-K, v_i, p_i);
    const double* ph = pb + h * 64;
    EOQ_SFOR(g, 8,
      if (g >= g0) {
        EOQ_SFOR(e, 8,
          const double xj = xh[g * 8 + e];
          const double wj = fma(-K, xj, ph[g * 8 + e]);
          A[g * 8 + e] = fma(-w_i, xj, fma(-v_i, wj, A[g * 8 + e]));
        );
      });
    // the loop used v_{k+1} = x_0: add the part that belongs to -alpha
    if (h == h1) add_at(A, c1, alpha * fma(-K, v_i, w_i));
  }
  // the last 2x2 block of T
  if (row == D - 2 && h == 0) dT[D - 2] = A[63];
  if (row == D - 1 && h == 0) eT[D - 2] = A[63];
  if (row == D - 1 && h == 1) dT[D - 1] = A[63];
  __syncthreads();

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
    if (tid < D) {
      const double e = (tid > 0) ? eT[tid - 1] * sc : 0.0;
      de[tid] = make_double2(dT[tid] * sc, e * e);
    }
    __syncthreads();
    const int j = tid >> 1, sub = tid & 1;
    double lo = -0x1.0p-40, hi = 1.0 + 0x1.0p-40;   // G is positive semi-definite; Gershgorin bounds the top by 1
#pragma unroll 1
    for (int it = 0; it < MULTISECT_ITERS; ++it) {
      const double third = (hi - lo) * (1.0 / 3.0);
      const double x1 = lo + third, x2 = hi - third;
      const int mine = sturm_count(de, sub ? x2 : x1);
      const int other = dpp_mov<0xB1>(mine);
      const int c1 = sub ? other : mine, c2 = sub ? mine : other;
      if (c1 > j) {
        hi = x1;
      } else if (c2 > j) {
        lo = x1;
        hi = x2;
      } else {
        lo = x2;
      }
    }
    if (sub == 0) lam_s[D - 1 - j] = fmax(0.5 * (lo + hi), 0.0) / sc;   // descending order, unscaled
  }
  __syncthreads();

  const int r = rank_and_shrink(lam_s, atoms, scale_s, &flag_s, n, k_pilot, rank_thr, r_max, blk, lam_out, phi_out,
                                sigma_out);

  // repeated retained eigenvalues: leave the block to the Jacobi solver
  bool repeated = false;
  for (int i = 0; i < r; ++i)
    if (lam_s[i] - lam_s[i + 1] <= CLUSTER_TOL * lam_s[0]) repeated = true;
  if (repeated) {
    if (tid == 0) {
      const int slot = atomicAdd(fb_count, 1);
      fb_list[slot] = (int)blk;
      rank_out[blk] = r;
      flags_out[blk] = flag_s;
    }
    return;
  }

  // ---- eigenvectors of the retained components ----
  double* tw = reinterpret_cast<double*>(u1);  // per eigenvector of the batch: Dp[128] Lp[128] Dm[128] Um[128]
  const double sc = tscale_s;
#pragma unroll 1
  for (int b0 = 0; b0 < r; b0 += EV_BATCH) {
    __syncthreads();
    // twisted factorisation of T - mu I: lane pair (forward, backward) per eigenvector, first wave only
    if (tid < 2 * EV_BATCH && b0 + (tid >> 1) < r) {
      const int ev = tid >> 1, role = tid & 1;
      const double mu = lam_s[b0 + ev] * sc;
      double* Dp = tw + ev * 4 * D;
      double* Lp = Dp + D;
      double* Dm = Dp + 2 * D;
      double* Um = Dp + 3 * D;
      const double piv = 0x1.0p-100;
      if (role == 0) {
        double dcur = de[0].x - mu;
        for (int i = 0; i < D - 1; ++i) {
          if (fabs(dcur) < piv) dcur = (dcur < 0.0) ? -piv : piv;
          Dp[i] = dcur;
          const double e = eT[i] * sc;
          const double l = e / dcur;
          Lp[i] = l;
          dcur = (de[i + 1].x - mu) - l * e;
        }
        Dp[D - 1] = dcur;
      } else {
        double dcur = de[D - 1].x - mu;
        for (int i = D - 2; i >= 0; --i) {
          if (fabs(dcur) < piv) dcur = (dcur < 0.0) ? -piv : piv;
          Dm[i + 1] = dcur;
          const double e = eT[i] * sc;
          const double u = e / dcur;
          Um[i] = u;
          dcur = (de[i].x - mu) - u * e;
        }
        Dm[0] = dcur;
      }
    }
    __syncthreads();
    if (tid < 2 * EV_BATCH && b0 + (tid >> 1) < r) {
      const int ev = tid >> 1, role = tid & 1;
      const double mu = lam_s[b0 + ev] * sc;
      double* Dp = tw + ev * 4 * D;
      const double* Lp = Dp + D;
      const double* Dm = Dp + 2 * D;
      const double* Um = Dp + 3 * D;
      // twist index: smallest |gamma_i|, gamma_i = D+_i + D-_i - (d_i - mu)
      int rt = 0;
      double best = INFINITY;
      for (int i = 0; i < D; ++i) {
        const double g = fabs(Dp[i] + Dm[i] - (de[i].x - mu));
        if (g < best) {
          best = g;
          rt = i;
        }
      }
      // z_rt = 1, upwards with the forward multipliers, downwards with the backward ones; written over Dp,
      // which is dead once both lanes of the pair (they run in lockstep) have finished the scan above
      double ssq = 0.0;
      if (role == 0) {
        double z = 1.0;
        for (int i = rt - 1; i >= 0; --i) {
          z = -Lp[i] * z;
          Dp[i] = z;
          ssq = fma(z, z, ssq);
        }
      } else {
        double z = 1.0;
        Dp[rt] = 1.0;
        ssq = 1.0;
        for (int i = rt; i < D - 1; ++i) {
          z = -Um[i] * z;
          Dp[i + 1] = z;
          ssq = fma(z, z, ssq);
        }
      }
      ssq = pair_sum(ssq);
      if (role == 0) {
        Dp[D + 0] = ssq;   // first slot of Lp: squared norm (Lp is dead now)
        if (!(ssq > 0.0) || !isfinite(ssq)) atomicOr(&flag_s, EOQ_FLAG_NO_CONVERGE);
      }
    }
    __syncthreads();
    // back-transformation v = H_0 H_1 ... H_125 z: 16 lanes per eigenvector, 8 elements (i = l + 16 m) each
    if (tid < 16 * EV_BATCH) {
      const int ev = tid >> 4, l = tid & 15;
      const bool live = (b0 + ev < r);
      const double* Dp = tw + ev * 4 * D;
      double y[8];
      {
        const double ssq = live ? Dp[D] : 1.0;
        const double inv = (ssq > 0.0 && isfinite(ssq)) ? 1.0 / sqrt(ssq) : 0.0;
#pragma unroll
        for (int m = 0; m < 8; ++m) y[m] = live ? Dp[l + 16 * m] * inv : 0.0;
      }
#pragma unroll 1
      for (int k = D - 3; k >= 0; --k) {
        const int ro = refl_off(k) - (k + 1);
        double v[8];
        double dot = 0.0;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const int i = l + 16 * m;
          v[m] = (i > k) ? (double)refl[ro + i] : 0.0;
          dot = fma(v[m], y[m], dot);
        }
        dot = row16_sum(dot);
        const double f = betaT[k] * dot;
#pragma unroll
        for (int m = 0; m < 8; ++m) y[m] = fma(-f, v[m], y[m]);
      }
      if (live) {
        const double s = scale_s[b0 + ev];
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          const int i = l + 16 * m;
          rfac[(blk * r_max + b0 + ev) * D + i] = double_to_half_bits(y[m]);
          wfac[(blk * r_max + b0 + ev) * D + i] = (float)(y[m] * s);
        }
      }
    }
  }
  if (tid == 0) {
    rank_out[blk] = r;
    flags_out[blk] = flag_s;
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
                               float* wfac, int* fb_count, int* fb_list, eoq_packed out) {
  if (L.ev) (void)hipEventRecord(L.ev[0], L.stream);
  if (L.solver == 1) {
    hipLaunchKernelGGL(eoq_spectral_jacobi_kernel, dim3((unsigned)B), dim3(THREADS), 0, L.stream, blocks, dtype, L.n,
                       L.k, L.rank_thr, L.r_max, B, (const int*)nullptr, (const int*)nullptr, lam, wfac, out.rank,
                       out.phi, out.sigma, out.rfac, out.flags);
  } else {
    hipLaunchKernelGGL(eoq_zero_counter_kernel, dim3(1), dim3(64), 0, L.stream, fb_count);
    hipLaunchKernelGGL(eoq_spectral_tridiag_kernel, dim3((unsigned)B), dim3(THREADS), 0, L.stream, blocks, dtype, L.n,
                       L.k, L.rank_thr, L.r_max, fb_list, fb_count, lam, wfac, out.rank, out.phi, out.sigma, out.rfac,
                       out.flags);
    const unsigned grid = (unsigned)((B < 256) ? B : 256);
    hipLaunchKernelGGL(eoq_spectral_jacobi_kernel, dim3(grid), dim3(THREADS), 0, L.stream, blocks, dtype, L.n, L.k,
                       L.rank_thr, L.r_max, B, (const int*)fb_list, (const int*)fb_count, lam, wfac, out.rank, out.phi,
                       out.sigma, out.rfac, out.flags);
  }
  if (L.ev) (void)hipEventRecord(L.ev[1], L.stream);
  return hipGetLastError();
}
