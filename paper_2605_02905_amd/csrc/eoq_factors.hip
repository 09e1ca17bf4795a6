// SVD factors of the retained components at 4 bits per entry with per-block data-adaptive codebooks (Alg. 3
// line 3; Sec. 3.1: "SVD factors are quantized at 4 bits via data-adaptive Lloyd-Max codebooks", the shrunk singular
// values stay in binary16).
//
// Per block and factor matrix (U: n x r, V: d x r, both with orthonormal columns) the codebook is {+-m_0 .. +-m_7}:
// eight magnitudes fitted to |entries| by Lloyd's iteration from the Lloyd-Max levels of a Gaussian with the
// entries' root mean square, eight rounds, then rounded to binary16.  A code is 3 bits of magnitude index (nearest
// level, ties up) plus the sign bit (bit 3 set for x >= 0): symmetric, so the arbitrary sign of a singular vector
// only flips sign bits.  Besides the codes the kernel writes what they expand to, lfac = binary16(U_hat phi16) and
// rfac = V_hat, which is what the residual (closed loop), the decoder and the scores use.
#include "eoq_device.h"
#include "eoq_internal.h"

#include <algorithm>

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int LEVELS = 8;
constexpr int LLOYD_ITERS = 8;

struct GaussLevels {
  double c[LEVELS];  // Lloyd-Max magnitudes of N(0,1) at 16 levels
};

__device__ __forceinline__ int cell_of(double a, const double (&b)[LEVELS - 1]) {
  int k = 0;
#pragma unroll
  for (int q = 0; q < LEVELS - 1; ++q) k += (a >= b[q]) ? 1 : 0;  // a tie goes to the upper cell
  return k;
}

__device__ __forceinline__ int code_of(double x, const double (&b)[LEVELS - 1]) {
  return cell_of(fabs(x), b) | ((x >= 0.0) ? 8 : 0);
}

__device__ __forceinline__ double swizzle_xor(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  if (mask == 4) {
    lo = __builtin_amdgcn_ds_swizzle(lo, 0x101F);
    hi = __builtin_amdgcn_ds_swizzle(hi, 0x101F);
  } else if (mask == 8) {
    lo = __builtin_amdgcn_ds_swizzle(lo, 0x201F);
    hi = __builtin_amdgcn_ds_swizzle(hi, 0x201F);
  } else if (mask == 16) {
    lo = __builtin_amdgcn_ds_swizzle(lo, 0x401F);
    hi = __builtin_amdgcn_ds_swizzle(hi, 0x401F);
  } else {
    lo = __shfl_xor(lo, 32, 64);
    hi = __shfl_xor(hi, 32, 64);
  }
  return __hiloint2double(hi, lo);
}

// Eight per-lane values summed over the wave, the eight totals spread over the lanes: lane l returns the total of
// value number 4 (l & 1) + 2 ((l >> 1) & 1) + ((l >> 2) & 1).  Halving exchange: every step hands the partner lane
// the half of the values it keeps, so 4 + 2 + 1 + 3 exchanges instead of 8 x 6.
__device__ __forceinline__ double wave_reduce8(const double (&v)[8], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4;
  double w[4], x[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const double keep = b0 ? v[i + 4] : v[i], send = b0 ? v[i] : v[i + 4];
    w[i] = keep + dpp_mov<0xB1>(send);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const double keep = b1 ? w[i + 2] : w[i], send = b1 ? w[i] : w[i + 2];
    x[i] = keep + dpp_mov<0x4E>(send);
  }
  double y = (b2 ? x[1] : x[0]) + swizzle_xor(b2 ? x[0] : x[1], 4);
  y += swizzle_xor(y, 8);
  y += swizzle_xor(y, 16);
  y += swizzle_xor(y, 32);
  return y;
}
// number of the value wave_reduce8 leaves in lane l (l < 8)
__device__ __forceinline__ int reduce8_slot(int l) { return 4 * (l & 1) + 2 * ((l >> 1) & 1) + ((l >> 2) & 1); }

// Partial Lloyd statistics of |x[0 .. count)| for the boundaries b: sums of the entries at or above every boundary
// (st[0..6]) and of all entries (st[7]) per lane; the counts at or above every boundary per WAVE (cnt, uniform).
__device__ __forceinline__ void lloyd_scan(const float* x, int count, const double (&b)[LEVELS - 1], int tid,
                                           double (&st)[8], int (&cnt)[LEVELS - 1]) {
#pragma unroll
  for (int k = 0; k < 8; ++k) st[k] = 0.0;
#pragma unroll
  for (int k = 0; k < LEVELS - 1; ++k) cnt[k] = 0;
  for (int e0 = 0; e0 < count; e0 += THREADS) {   // uniform trip count: the ballots need every lane
    const int e = e0 + tid;
    const double a = (e < count) ? fabs((double)x[e]) : -1.0;
#pragma unroll
    for (int q = 0; q < LEVELS - 1; ++q) {
      const bool ge = a >= b[q];
      st[q] += ge ? a : 0.0;
      cnt[q] += __popcll(__ballot(ge));
    }
    st[7] += (e < count) ? a : 0.0;
  }
}

template <int RCAP>
__global__ __launch_bounds__(THREADS) void eoq_factor_quant_kernel(
    const uint16_t* __restrict__ blocks, EoqBlockMap map, int64_t B, int n, int r_max, GaussLevels g,
    const int32_t* __restrict__ rank_in,
    const float* __restrict__ phi, const float* __restrict__ sigma, const float* __restrict__ wfac,
    uint16_t* __restrict__ rfac, uint16_t* __restrict__ lfac, uint8_t* __restrict__ lcodes,
    uint8_t* __restrict__ rcodes, uint16_t* __restrict__ fbook, uint16_t* __restrict__ phi16) {
  extern __shared__ __align__(16) float dyn[];  // Vs[r][D] then Us[r][n]
  __shared__ __align__(16) double red[2][4][16];   // [parity][wave][U: 8 sums, V: 8 sums]
  __shared__ int redc[2][4][16];                   // [parity][wave][U: 7 counts, pad, V: 7 counts, pad]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // The workgroups walk the batch with the grid's stride.  The launch with the small table has one workgroup per block
  // and takes the blocks of rank 1 .. 8 (and clears the codebook of rank-0 blocks); the launch with the large table is
  // a few persistent workgroups that look for the rest (usually there are none: a grid of B would only spend its
  // time placing workgroups with a large LDS allocation that return at once).
  for (size_t wblk = blockIdx.x; wblk < (size_t)B; wblk += gridDim.x) {   // number in the batch: workspace and input
  __syncthreads();                           // LDS of the previous block has been consumed
  const size_t blk = map.slot(wblk);         // record slot: everything that is stored
  const int r = rank_in[blk];
  if (RCAP == 8) {
    if (r == 0 && tid < 2 * LEVELS) fbook[blk * 2 * LEVELS + tid] = 0;
    if (r == 0 || r > 8) continue;
  } else {
    if (r <= 8) continue;
  }
  float* Vs = dyn;
  float* Us = dyn + (size_t)r * D;
  // right vectors back from the projection operand W = V phi / sigma (float32); where phi = 0 (guarded
  // component) from the stored binary16 vector
  for (int e = tid; e < r * D; e += THREADS) {
    const int i = e >> 7;
    const float ph = phi[blk * r_max + i], sg = sigma[blk * r_max + i];
    Vs[e] = (ph > 0.0f) ? wfac[wblk * (size_t)r_max * D + e] * (sg / ph) : half_bits_to_float(rfac[blk * (size_t)r_max * D + e]);
  }
  __syncthreads();
  // left vectors U = S V / sigma, one token per lane and pass, four components at a time
  for (int t = tid; t < n; t += THREADS) {
    const uint16_t* row = blocks + map.in_base(wblk) + (size_t)t * (size_t)map.token_stride;
    for (int i0 = 0; i0 < r; i0 += 4) {
      const float* vrow[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) vrow[c] = Vs + min(i0 + c, r - 1) * D;
      double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
      for (int q = 0; q < 16; ++q) {
        const uint4 raw = *reinterpret_cast<const uint4*>(row + 8 * q);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        double sv[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) sv[h] = (double)half_bits_to_float((uint16_t)(w[h >> 1] >> (16 * (h & 1))));
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float4 va = *reinterpret_cast<const float4*>(vrow[c] + 8 * q);
          const float4 vb = *reinterpret_cast<const float4*>(vrow[c] + 8 * q + 4);
          acc[c] = fma(sv[0], (double)va.x, acc[c]);
          acc[c] = fma(sv[1], (double)va.y, acc[c]);
          acc[c] = fma(sv[2], (double)va.z, acc[c]);
          acc[c] = fma(sv[3], (double)va.w, acc[c]);
          acc[c] = fma(sv[4], (double)vb.x, acc[c]);
          acc[c] = fma(sv[5], (double)vb.y, acc[c]);
          acc[c] = fma(sv[6], (double)vb.z, acc[c]);
          acc[c] = fma(sv[7], (double)vb.w, acc[c]);
        }
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (i0 + c < r) {
          const float sg = sigma[blk * r_max + i0 + c];
          Us[(size_t)(i0 + c) * n + t] = (sg > 0.0f) ? (float)(acc[c] / (double)sg) : 0.0f;
        }
    }
  }
  __syncthreads();

  // ---- Lloyd fits of the two codebooks, side by side (one barrier per round) ----
  const int cu = r * n, cv = r * D;
  double mu[LEVELS], mv[LEVELS];
  int par = 0;
  {
    double st[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    for (int e = tid; e < cu; e += THREADS) {
      const double a = (double)Us[e];
      st[0] = fma(a, a, st[0]);
    }
    for (int e = tid; e < cv; e += THREADS) {
      const double a = (double)Vs[e];
      st[4] = fma(a, a, st[4]);   // value 4 ends in lane 1, value 0 in lane 0
    }
    const double y = wave_reduce8(st, lane);
    if (lane < 2) red[par][wave][lane] = y;
    __syncthreads();
    const double su = (red[par][0][0] + red[par][1][0]) + (red[par][2][0] + red[par][3][0]);
    const double sv = (red[par][0][1] + red[par][1][1]) + (red[par][2][1] + red[par][3][1]);
    const double rms_u = sqrt(su / (double)cu), rms_v = sqrt(sv / (double)cv);
#pragma unroll
    for (int k = 0; k < LEVELS; ++k) {
      mu[k] = g.c[k] * rms_u;
      mv[k] = g.c[k] * rms_v;
    }
    par ^= 1;
  }
#pragma unroll 1
  for (int it = 0; it < LLOYD_ITERS; ++it) {
    double b[LEVELS - 1], st[8];
    int cnt[LEVELS - 1];
#pragma unroll
    for (int k = 0; k < LEVELS - 1; ++k) b[k] = 0.5 * (mu[k] + mu[k + 1]);
    lloyd_scan(Us, cu, b, tid, st, cnt);
    double y = wave_reduce8(st, lane);
    if (lane < 8) red[par][wave][reduce8_slot(lane)] = y;
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < LEVELS - 1; ++k) redc[par][wave][k] = cnt[k];
    }
#pragma unroll
    for (int k = 0; k < LEVELS - 1; ++k) b[k] = 0.5 * (mv[k] + mv[k + 1]);
    lloyd_scan(Vs, cv, b, tid, st, cnt);
    y = wave_reduce8(st, lane);
    if (lane < 8) red[par][wave][8 + reduce8_slot(lane)] = y;
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < LEVELS - 1; ++k) redc[par][wave][8 + k] = cnt[k];
    }
    __syncthreads();
    // Lane l < 16 of every wave moves one level: matrix f = l / 8, level k = l % 8 (the waves repeat the work and agree
    // bit for bit, so no second barrier).  Cell sum = difference of two "at or above" sums, T[0] = all (value 7),
    // T[j] = value j - 1, T[8] = 0; counts likewise.
    {
      const int f = (lane >> 3) & 1, k = lane & 7;
      const int ia = 8 * f + ((k == 0) ? 7 : k - 1), ib = 8 * f + min(k, LEVELS - 2);
      const double sa = (red[par][0][ia] + red[par][1][ia]) + (red[par][2][ia] + red[par][3][ia]);
      double sb = (red[par][0][ib] + red[par][1][ib]) + (red[par][2][ib] + red[par][3][ib]);
      const int ja = 8 * f + max(k - 1, 0);
      int ca = (redc[par][0][ja] + redc[par][1][ja]) + (redc[par][2][ja] + redc[par][3][ja]);
      int cb = (redc[par][0][ib] + redc[par][1][ib]) + (redc[par][2][ib] + redc[par][3][ib]);
      if (k == 0) ca = f ? cv : cu;
      if (k == LEVELS - 1) {
        sb = 0.0;
        cb = 0;
      }
      const int ck = ca - cb;
      double mine = 0.0;   // this lane's level before the round
#pragma unroll
      for (int q = 0; q < LEVELS; ++q) mine = (k == q) ? (f ? mv[q] : mu[q]) : mine;
      const double moved = (ck > 0) ? (sa - sb) / (double)ck : mine;   // an empty cell keeps its level
#pragma unroll
      for (int q = 0; q < LEVELS; ++q) {
        mu[q] = readlane_f64(moved, q);
        mv[q] = readlane_f64(moved, LEVELS + q);
      }
    }
    par ^= 1;
  }

  double m16[LEVELS];
  uint16_t bits16[LEVELS];
  double b[LEVELS - 1];
  // ---- U ----
#pragma unroll
  for (int k = 0; k < LEVELS; ++k) {
    bits16[k] = double_to_half_bits(mu[k]);
    m16[k] = (double)half_bits_to_float(bits16[k]);
  }
  if (tid < LEVELS) {
    uint16_t mine = 0;
#pragma unroll
    for (int k = 0; k < LEVELS; ++k) mine = (tid == k) ? bits16[k] : mine;
    fbook[blk * 2 * LEVELS + tid] = mine;
  }
#pragma unroll
  for (int k = 0; k < LEVELS - 1; ++k) b[k] = 0.5 * (m16[k] + m16[k + 1]);
  for (int e = tid; e < r * (n / 2); e += THREADS) {  // two tokens per byte
    const int i = e / (n / 2), t = 2 * (e - i * (n / 2));
    const uint16_t ph16 = float_to_half_bits(phi[blk * r_max + i]);
    const double p16 = (double)half_bits_to_float(ph16);
    int code[2];
    uint16_t outv[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const double x = (double)Us[(size_t)i * n + t + u];
      code[u] = code_of(x, b);
      double lev = 0.0;
#pragma unroll
      for (int k = 0; k < LEVELS; ++k) lev = ((code[u] & 7) == k) ? m16[k] : lev;
      outv[u] = double_to_half_bits(((code[u] & 8) ? lev : -lev) * p16);
    }
    *reinterpret_cast<uint32_t*>(lfac + (blk * r_max + i) * (size_t)n + t) = (uint32_t)outv[0] | ((uint32_t)outv[1] << 16);
    lcodes[(blk * r_max + i) * (size_t)(n / 2) + (t >> 1)] = (uint8_t)(code[0] | (code[1] << 4));
    if (t == 0) phi16[blk * r_max + i] = ph16;
  }
  // ---- V ----
#pragma unroll
  for (int k = 0; k < LEVELS; ++k) {
    bits16[k] = double_to_half_bits(mv[k]);
    m16[k] = (double)half_bits_to_float(bits16[k]);
  }
  if (tid < LEVELS) {
    uint16_t mine = 0;
#pragma unroll
    for (int k = 0; k < LEVELS; ++k) mine = (tid == k) ? bits16[k] : mine;
    fbook[blk * 2 * LEVELS + LEVELS + tid] = mine;
  }
#pragma unroll
  for (int k = 0; k < LEVELS - 1; ++k) b[k] = 0.5 * (m16[k] + m16[k + 1]);
  for (int e = tid; e < r * (D / 2); e += THREADS) {
    const int i = e / (D / 2), j = 2 * (e - i * (D / 2));
    int code[2];
    uint16_t outv[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const double x = (double)Vs[i * D + j + u];
      code[u] = code_of(x, b);
      uint16_t lev = 0;
#pragma unroll
      for (int k = 0; k < LEVELS; ++k) lev = ((code[u] & 7) == k) ? bits16[k] : lev;
      outv[u] = (code[u] & 8) ? lev : (uint16_t)(lev | 0x8000u);
    }
    *reinterpret_cast<uint32_t*>(rfac + (blk * r_max + i) * (size_t)D + j) = (uint32_t)outv[0] | ((uint32_t)outv[1] << 16);
    rcodes[(blk * r_max + i) * (size_t)(D / 2) + (j >> 1)] = (uint8_t)(code[0] | (code[1] << 4));
  }
  }  // blocks of this workgroup
}

// codes + codebooks + phi16 -> lfac = binary16(U_hat phi16), rfac = V_hat (rows below the rank)
__global__ __launch_bounds__(THREADS) void eoq_factor_expand_kernel(
    int n, int r_max, const int32_t* __restrict__ rank_in, const uint8_t* __restrict__ lcodes,
    const uint8_t* __restrict__ rcodes, const uint16_t* __restrict__ fbook, const uint16_t* __restrict__ phi16,
    uint16_t* __restrict__ lfac, uint16_t* __restrict__ rfac) {
  const int tid = threadIdx.x;
  const size_t blk = blockIdx.x;
  const int r = min(max(rank_in[blk], 0), r_max);   // a record read back from storage: never index past r_max rows
  __shared__ uint16_t book[2 * LEVELS];
  if (tid < 2 * LEVELS) book[tid] = fbook[blk * 2 * LEVELS + tid];
  __syncthreads();
  for (int e = tid; e < r * (n / 2); e += THREADS) {
    const int i = e / (n / 2), t = 2 * (e - i * (n / 2));
    const double p16 = (double)half_bits_to_float(phi16[blk * r_max + i]);
    const int byte = lcodes[(blk * r_max + i) * (size_t)(n / 2) + (t >> 1)];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int code = (byte >> (4 * u)) & 15;
      const double lev = (double)half_bits_to_float(book[code & 7]);
      lfac[(blk * r_max + i) * (size_t)n + t + u] = double_to_half_bits(((code & 8) ? lev : -lev) * p16);
    }
  }
  for (int e = tid; e < r * (D / 2); e += THREADS) {
    const int i = e / (D / 2), j = 2 * (e - i * (D / 2));
    const int byte = rcodes[(blk * r_max + i) * (size_t)(D / 2) + (j >> 1)];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int code = (byte >> (4 * u)) & 15;
      const uint16_t lev = book[LEVELS + (code & 7)];
      rfac[(blk * r_max + i) * (size_t)D + j + u] = (code & 8) ? lev : (uint16_t)(lev | 0x8000u);
    }
  }
}

}  // namespace

// Largest LDS tables the two variants are ever launched with (n * r_max <= 32768, n <= 4096): raised once per device
// at context creation, so that the hot call sets no function attribute.
hipError_t eoq_factor_quant_prepare() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(eoq_factor_quant_kernel<8>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 8 * (4096 + D) * (int)sizeof(float));
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(eoq_factor_quant_kernel<32>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (32768 + EOQ_RMAX_CAP * D) * (int)sizeof(float));
}

hipError_t eoq_launch_factor_quant(const EoqLaunch& L, const void* blocks_fp16, int64_t B, const float* wfac,
                                   eoq_packed out, eoq_factor_codes fq, const double* gauss_levels) {
  GaussLevels g;
  for (int k = 0; k < LEVELS; ++k) g.c[k] = gauss_levels[k];
  // two launches over all blocks, each taking the blocks of its rank class: the table of the factors in LDS is
  // sized for 8 components (most blocks: many workgroups per CU) or for r_max
  const size_t lds8 = (size_t)std::min(8, L.r_max) * (L.n + D) * sizeof(float);
  hipError_t e = hipSuccess;
  hipLaunchKernelGGL(eoq_factor_quant_kernel<8>, dim3((unsigned)B), dim3(THREADS), lds8, L.stream,
                     static_cast<const uint16_t*>(blocks_fp16), L.map, B, L.n, L.r_max, g, out.rank, out.phi, out.sigma, wfac,
                     out.rfac, out.lfac, fq.lcodes, fq.rcodes, fq.fbook, fq.phi16);
  e = hipGetLastError();
  if (e != hipSuccess || L.r_max <= 8) return e;
  const size_t lds = (size_t)L.r_max * (L.n + D) * sizeof(float);
  hipLaunchKernelGGL(eoq_factor_quant_kernel<32>, dim3((unsigned)(B < 512 ? B : 512)), dim3(THREADS), lds, L.stream,
                     static_cast<const uint16_t*>(blocks_fp16), L.map, B, L.n, L.r_max, g, out.rank, out.phi, out.sigma, wfac,
                     out.rfac, out.lfac, fq.lcodes, fq.rcodes, fq.fbook, fq.phi16);
  return hipGetLastError();
}

hipError_t eoq_launch_factor_expand(const EoqLaunch& L, eoq_packed rec, eoq_factor_codes fq, int64_t B) {
  hipLaunchKernelGGL(eoq_factor_expand_kernel, dim3((unsigned)B), dim3(THREADS), 0, L.stream, L.n, L.r_max, rec.rank,
                     fq.lcodes, fq.rcodes, fq.fbook, fq.phi16, rec.lfac, rec.rfac);
  return hipGetLastError();
}
