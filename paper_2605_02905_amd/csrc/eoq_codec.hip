// HIP kernels (gfx950) of the residual coder of eOptShrinkQ and its inverse:
//   encode : projection C = S V diag(phi/sigma) = U diag(phi), residual against the stored binary16 factors
//            (Alg. 3), then per row norm, rotation, Lloyd-Max index and bit-plane packing (Alg. 1 lines 3-5).
//   scores : <q, x_hat>/sqrt(d) from the record without forming x_hat (Remark 6.5).
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;

// ---------------------------------------------------------------------------
// encode kernel: 64 rows of one block per workgroup.
// ---------------------------------------------------------------------------
constexpr int ENC_ROWS = 64;
constexpr int ENC_THREADS = 256;
constexpr int LDS_X = D + 1;

__global__ __launch_bounds__(ENC_THREADS) void eoq_encode_kernel(
    const void* __restrict__ blocks, int dtype, int n, int bits, int r_max, const float* __restrict__ pit,
    const float* __restrict__ tab, const float* __restrict__ wfac, const int32_t* __restrict__ rank_in,
    const uint16_t* __restrict__ rfac, uint16_t* __restrict__ lfac, uint16_t* __restrict__ norms,
    uint8_t* __restrict__ codes) {
  __shared__ float X[ENC_ROWS * LDS_X];            // rows of S, then R, then sqrt(d) u
  __shared__ float PT[D * D];                      // Pi^T: PT[j*D + c] = Pi[c][j]
  __shared__ float Wl[EOQ_RMAX_CAP * D];           // V diag(phi/sigma), later reused for the code bytes
  __shared__ float Vl[EOQ_RMAX_CAP * D];           // stored binary16 right factors as float
  __shared__ float Cl[ENC_ROWS * (EOQ_RMAX_CAP + 1)];
  __shared__ float rho_s[ENC_ROWS];

  const int tid = threadIdx.x;
  const size_t blk = blockIdx.y;
  const int row0 = blockIdx.x * ENC_ROWS;
  const int r = rank_in[blk];

  // stage the strip, the rotation and the factors
  for (int g = tid; g < ENC_ROWS * D / 8; g += ENC_THREADS) {
    const int e = g * 8;
    float v[8];
    load8(blocks, dtype, (blk * (size_t)n + row0) * D + e, v);
    const int t = e >> 7, j = e & (D - 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) X[t * LDS_X + j + i] = v[i];
  }
  for (int e = tid; e < D * D / 4; e += ENC_THREADS)
    reinterpret_cast<float4*>(PT)[e] = reinterpret_cast<const float4*>(pit)[e];
  for (int e = tid; e < r * D; e += ENC_THREADS) {
    Wl[e] = wfac[blk * r_max * D + e];
    Vl[e] = half_bits_to_float(rfac[blk * r_max * D + e]);
  }
  __syncthreads();

  // C = S W^T (= U diag(phi)), rounded to the stored binary16 (Alg. 2 Return, Alg. 3 Store)
  {
    const int t = tid & (ENC_ROWS - 1);
    for (int i = tid >> 6; i < r; i += ENC_THREADS / ENC_ROWS) {
      float acc = 0.0f;
      for (int j = 0; j < D; ++j) acc = fmaf(X[t * LDS_X + j], Wl[i * D + j], acc);
      const uint16_t hb = float_to_half_bits(acc);
      lfac[(blk * r_max + i) * (size_t)n + row0 + t] = hb;
      Cl[t * (EOQ_RMAX_CAP + 1) + i] = half_bits_to_float(hb);
    }
  }
  __syncthreads();

  const int tr = tid >> 5, tc = tid & 31;  // rows tr*8 .. tr*8+7, columns tc + 32*m
  // R = S - C V^T (Alg. 3; the whole block when r = 0)
  if (r > 0) {
    for (int a = 0; a < 8; ++a) {
      const int t = tr * 8 + a;
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      for (int i = 0; i < r; ++i) {
        const float c = Cl[t * (EOQ_RMAX_CAP + 1) + i];
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[m] = fmaf(c, Vl[i * D + tc + 32 * m], acc[m]);
      }
#pragma unroll
      for (int m = 0; m < 4; ++m) X[t * LDS_X + tc + 32 * m] -= acc[m];
    }
  }
  __syncthreads();

  // rho_t = |R_t|, u = R_t / rho_t (Alg. 1 line 3); rows are rescaled to sqrt(d) u
  {
    const int t = tid >> 2, q = tid & 3;
    float ss = 0.0f;
    for (int m = 0; m < D / 4; ++m) {
      const float x = X[t * LDS_X + q + 4 * m];
      ss = fmaf(x, x, ss);
    }
    ss = quad_sum(ss);
    const float rho = sqrtf(ss);
    const float sc = (rho > 0.0f) ? sqrtf((float)D) / rho : 0.0f;
    for (int m = 0; m < D / 4; ++m) X[t * LDS_X + q + 4 * m] *= sc;
    if (q == 0) norms[blk * (size_t)n + row0 + t] = float_to_half_bits(rho);
  }
  __syncthreads();

  // z = Pi u (Alg. 1 line 4) and index of the nearest centroid (line 5)
  uint8_t* code_s = reinterpret_cast<uint8_t*>(Wl);  // [64][128] bytes
  {
    float acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int m = 0; m < 4; ++m) acc[a][m] = 0.0f;
    for (int j = 0; j < D; ++j) {
      float p[4], u[8];
#pragma unroll
      for (int m = 0; m < 4; ++m) p[m] = PT[j * D + tc + 32 * m];
#pragma unroll
      for (int a = 0; a < 8; ++a) u[a] = X[(tr * 8 + a) * LDS_X + j];
#pragma unroll
      for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[a][m] = fmaf(u[a], p[m], acc[a][m]);
    }
    const int nb = (1 << bits) - 1;
    float bnd[15];
#pragma unroll
    for (int i = 0; i < 15; ++i) bnd[i] = tab[16 + i];  // +inf beyond the last boundary
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        int code = 0;
#pragma unroll
        for (int i = 0; i < 15; ++i) code += (i < nb && bnd[i] <= acc[a][m]) ? 1 : 0;
        code_s[(tr * 8 + a) * D + tc + 32 * m] = (uint8_t)code;
      }
  }
  __syncthreads();

  // bit-plane packing: lane handles 32 coordinates of one row
  {
    const int t = tid >> 2, q = tid & 3;
    uint32_t plane[4] = {0u, 0u, 0u, 0u};
    for (int j = 0; j < 32; ++j) {
      const uint32_t c = code_s[t * D + q * 32 + j];
#pragma unroll
      for (int p = 0; p < 4; ++p) plane[p] |= ((c >> p) & 1u) << j;
    }
    uint32_t* dst = reinterpret_cast<uint32_t*>(codes + (blk * (size_t)n + row0 + t) * (size_t)(bits * D / 8));
    for (int p = 0; p < bits; ++p) dst[p * 4 + q] = plane[p];
  }
}

// ---------------------------------------------------------------------------
// scores: one workgroup per (sequence, KV head, run of SC_CHUNK blocks).  The group's
// queries are rotated once (q' = Pi q), then every token of the run is scored from
// its codes, norm and low-rank coefficients.
// ---------------------------------------------------------------------------
constexpr int SC_THREADS = 256;
constexpr int SC_MAXG = 8;
constexpr int SC_CHUNK = 8;

__global__ __launch_bounds__(SC_THREADS) void eoq_scores_kernel(
    int n, int bits, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, const float* __restrict__ pit,
    const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const uint16_t* __restrict__ q, float* __restrict__ scores) {
  __shared__ float qr[SC_MAXG * D];               // rotated queries of the group
  __shared__ float qraw[SC_MAXG * D];
  __shared__ float w[SC_MAXG * EOQ_RMAX_CAP];     // <v_i, q_h> of the current block

  const int tid = threadIdx.x;
  const size_t sg = blockIdx.y;                   // s*n_kv_heads + g
  const size_t s = sg / n_kv_heads, g = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  const size_t q0 = (s * n_q_heads + g * group) * D;   // first query of the group
  const size_t T = (size_t)blocks_per_head * n;

  for (int e = tid; e < group * D; e += SC_THREADS) qraw[e] = half_bits_to_float(q[q0 + e]);
  __syncthreads();
  for (int e = tid; e < group * D; e += SC_THREADS) {
    const int h = e >> 7, c = e & (D - 1);
    float acc = 0.0f;
    for (int j = 0; j < D; ++j) acc = fmaf(pit[j * D + c], qraw[h * D + j], acc);
    qr[e] = acc;
  }

  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const int row_bytes = bits * D / 8;
  const int64_t j_end = min((int64_t)(blockIdx.x + 1) * SC_CHUNK, blocks_per_head);
  for (int64_t jblk = (int64_t)blockIdx.x * SC_CHUNK; jblk < j_end; ++jblk) {
    const size_t blk = sg * (size_t)blocks_per_head + jblk;
    const int r = rank_in[blk];
    __syncthreads();
    for (int e = tid; e < group * r; e += SC_THREADS) {
      const int h = e / r, i = e % r;
      float acc = 0.0f;
      for (int j = 0; j < D; ++j)
        acc = fmaf(half_bits_to_float(rfac[(blk * r_max + i) * D + j]), qraw[h * D + j], acc);
      w[h * EOQ_RMAX_CAP + i] = acc;
    }
    __syncthreads();
    for (int t = tid; t < n; t += SC_THREADS) {
      const uint32_t* src = reinterpret_cast<const uint32_t*>(codes + (blk * (size_t)n + t) * (size_t)row_bytes);
      float acc[SC_MAXG];
#pragma unroll
      for (int h = 0; h < SC_MAXG; ++h) acc[h] = 0.0f;
      for (int qd = 0; qd < 4; ++qd) {
        uint32_t plane[4] = {0u, 0u, 0u, 0u};
        for (int p = 0; p < bits; ++p) plane[p] = src[p * 4 + qd];
        for (int j = 0; j < 32; ++j) {
          int c = 0;
#pragma unroll
          for (int p = 0; p < 4; ++p) c |= ((plane[p] >> j) & 1u) << p;
          const float zc = tab[c];
#pragma unroll
          for (int h = 0; h < SC_MAXG; ++h)
            if (h < group) acc[h] = fmaf(zc, qr[h * D + qd * 32 + j], acc[h]);
        }
      }
      const float rho = half_bits_to_float(norms[blk * (size_t)n + t]);
      // rho <Pi q, z_hat> with z_hat = centroid / sqrt(d)
#pragma unroll
      for (int h = 0; h < SC_MAXG; ++h) acc[h] *= rho * inv_sqrt_d;
      for (int i = 0; i < r; ++i) {
        const float c = half_bits_to_float(lfac[(blk * r_max + i) * (size_t)n + t]);
#pragma unroll
        for (int h = 0; h < SC_MAXG; ++h)
          if (h < group) acc[h] = fmaf(c, w[h * EOQ_RMAX_CAP + i], acc[h]);
      }
#pragma unroll
      for (int h = 0; h < SC_MAXG; ++h)
        if (h < group) scores[((s * n_q_heads + g * group + h) * T) + jblk * n + t] = acc[h] * inv_sqrt_d;
    }
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
hipError_t eoq_launch_encode(const EoqLaunch& L, const void* blocks, int dtype, int64_t B, const float* wfac,
                             eoq_packed out) {
  // gridDim.y is limited to 65535: split long batches
  if (L.ev) (void)hipEventRecord(L.ev[2], L.stream);
  for (int64_t b0 = 0; b0 < B; b0 += 32768) {
    const int64_t nb = (B - b0 < 32768) ? B - b0 : 32768;
    const size_t esz = (dtype == EOQ_F16) ? 2 : 4;
    hipLaunchKernelGGL(eoq_encode_kernel, dim3(L.n / ENC_ROWS, (unsigned)nb), dim3(ENC_THREADS), 0, L.stream,
                       static_cast<const char*>(blocks) + (size_t)b0 * L.n * D * esz, dtype, L.n, L.bits, L.r_max,
                       L.pit, L.tab, wfac + (size_t)b0 * L.r_max * D, out.rank + b0, out.rfac + (size_t)b0 * L.r_max * D,
                       out.lfac + (size_t)b0 * L.r_max * L.n, out.norms + (size_t)b0 * L.n,
                       out.codes + (size_t)b0 * L.n * (L.bits * D / 8));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (L.ev) (void)hipEventRecord(L.ev[3], L.stream);
  return hipSuccess;
}

hipError_t eoq_launch_scores(const EoqLaunch& L, eoq_packed keys, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores) {
  const int64_t chunks = (blocks_per_head + SC_CHUNK - 1) / SC_CHUNK;
  const int64_t sg_total = n_seq * n_kv_heads;
  if (sg_total > 65535 || chunks > 0x7FFFFFFF) return hipErrorInvalidValue;
  if (L.ev) (void)hipEventRecord(L.ev[6], L.stream);
  hipLaunchKernelGGL(eoq_scores_kernel, dim3((unsigned)chunks, (unsigned)sg_total), dim3(SC_THREADS), 0, L.stream,
                     L.n, L.bits, L.r_max, n_kv_heads, n_q_heads / n_kv_heads, blocks_per_head, L.pit, L.tab,
                     keys.codes, keys.norms, keys.rank, keys.lfac, keys.rfac, static_cast<const uint16_t*>(q_fp16),
                     scores);
  if (L.ev) (void)hipEventRecord(L.ev[7], L.stream);
  return hipGetLastError();
}
