// HIP kernels (gfx950) of the residual coder of eOptShrinkQ and its inverse:
//   encode : projection C = S V diag(phi/sigma) = U diag(phi), residual against the stored binary16 factors
//            (Alg. 3), then per row norm, rotation, Lloyd-Max index and bit-plane packing (Alg. 1 lines 3-5).
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
    const void* __restrict__ blocks, EoqBlockMap map, int64_t b0, int dtype, int n, int bits, int r_max,
    const float* __restrict__ pit,
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
  const size_t blk = (size_t)b0 + blockIdx.y;
  const size_t slot = map.slot(blk);
  const int row0 = blockIdx.x * ENC_ROWS;
  const int r = rank_in[slot];

  // stage the strip, the rotation and the factors
  for (int g = tid; g < ENC_ROWS * D / 8; g += ENC_THREADS) {
    const int e = g * 8;
    float v[8];
    const int t = e >> 7, j = e & (D - 1);
    load8(blocks, dtype, map.in_base(blk) + (size_t)(row0 + t) * (size_t)map.token_stride + j, v);
#pragma unroll
    for (int i = 0; i < 8; ++i) X[t * LDS_X + j + i] = v[i];
  }
  for (int e = tid; e < D * D / 4; e += ENC_THREADS)
    reinterpret_cast<float4*>(PT)[e] = reinterpret_cast<const float4*>(pit)[e];
  for (int e = tid; e < r * D; e += ENC_THREADS) {
    Wl[e] = wfac[blk * r_max * D + e];
    Vl[e] = half_bits_to_float(rfac[slot * r_max * D + e]);
  }
  __syncthreads();

  // C = S W^T (= U diag(phi)), rounded to the stored binary16 (Alg. 2 Return, Alg. 3 Store)
  {
    const int t = tid & (ENC_ROWS - 1);
    for (int i = tid >> 6; i < r; i += ENC_THREADS / ENC_ROWS) {
      float acc = 0.0f;
      for (int j = 0; j < D; ++j) acc = fmaf(X[t * LDS_X + j], Wl[i * D + j], acc);
      const uint16_t hb = float_to_half_bits(acc);
      lfac[(slot * r_max + i) * (size_t)n + row0 + t] = hb;
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
    if (q == 0) norms[slot * (size_t)n + row0 + t] = float_to_half_bits(rho);
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
    uint32_t* dst = reinterpret_cast<uint32_t*>(codes + (slot * (size_t)n + row0 + t) * (size_t)(bits * D / 8));
    for (int p = 0; p < bits; ++p) dst[p * 4 + q] = plane[p];
  }
}

}  // namespace

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
hipError_t eoq_launch_encode(const EoqLaunch& L, const void* blocks, int dtype, int64_t B, const float* wfac,
                             eoq_packed out) {
  if (L.ev) (void)hipEventRecord(L.ev[2], L.stream);
  if (dtype == EOQ_F16) {  // binary16 blocks go to the matrix-core kernel
    const hipError_t e = eoq_launch_encode_f16(L, blocks, B, wfac, out);
    if (L.ev) (void)hipEventRecord(L.ev[3], L.stream);
    return e;
  }
  // gridDim.y is limited to 65535: split long batches
  for (int64_t b0 = 0; b0 < B; b0 += 32768) {
    const int64_t nb = (B - b0 < 32768) ? B - b0 : 32768;
    hipLaunchKernelGGL(eoq_encode_kernel, dim3(L.n / ENC_ROWS, (unsigned)nb), dim3(ENC_THREADS), 0, L.stream, blocks,
                       L.map, b0, dtype, L.n, L.bits, L.r_max, L.pit, L.tab, wfac, out.rank, out.rfac, out.lfac,
                       out.norms, out.codes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (L.ev) (void)hipEventRecord(L.ev[3], L.stream);
  return hipSuccess;
}

