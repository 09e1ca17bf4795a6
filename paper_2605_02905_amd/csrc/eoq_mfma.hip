// Matrix-core (MFMA, gfx950) kernels of the residual coder for binary16 blocks:
//   decode : x_hat = (rho/sqrt(d)) z_hat Pi + C V^T  (Alg. 1 line 6 plus the stored low-rank part)
//   scores : <q, x_hat>/sqrt(d) from the record without forming x_hat (Sec. 2.1, Remark 6.5)
//
// Operand convention of v_mfma_f32_32x32x16_f16 (wave64): for D = A(32xK) * B(Kx32) + C, lane l supplies
// A[row = l%32][k = 8*(l/32) .. +7] and B[k = 8*(l/32) .. +7][col = l%32]; it receives
// D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator register v = 0..15.
//
// Layout of the work: the rotation is the stationary operand.  Wave w of a workgroup keeps the 32 columns
// j = 32w .. 32w+31 of Pi (as B operand, binary16 hi + lo parts) in registers for the whole block; the tokens
// stream through LDS in tiles of 32 (A operand), each tile prepared by one wave and consumed by all four.
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int CHUNK = 128;          // tokens per pass of a workgroup: one tile of 32 per wave
constexpr int ZLD = D + 8;          // row stride (halfs) of the token tiles in LDS: 272 B, conflict-free b128 reads
constexpr int CLD = EOQ_RMAX_CAP + 8;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

union H8 {
  half8 h;
  uint4 u;
  uint32_t w[4];
  uint16_t s[8];
};

__device__ __forceinline__ float16v mfma16(const H8& a, const H8& b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, c, 0, 0, 0);
}

// Mask table: entry m (a byte of one bit-plane) -> 8 halfwords, halfword e = 0xFFFF if bit e of m is set.
__device__ __forceinline__ void build_mask_table(uint4* tab, int tid) {
  if (tid < 256) {
    H8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x.s[e] = ((tid >> e) & 1) ? 0xFFFFu : 0u;
    tab[tid] = x.u;
  }
}

// Centroid magnitudes of the symmetric codebook as duplicated binary16 pairs: mag[m] = (h << 16) | h with
// h = binary16(centroid[L/2 + m]), m = 0 .. L/2-1.
template <int BITS>
struct Mags {
  uint32_t m[(1 << BITS) / 2];   // binary16(centroid), duplicated in both halves
  uint32_t lo[(1 << BITS) / 2];  // binary16(centroid - hi): the part the first rounding lost (signed)
  __device__ __forceinline__ void load(const float* __restrict__ tab) {
#pragma unroll
    for (int i = 0; i < (1 << BITS) / 2; ++i) {
      const float c = tab[(1 << BITS) / 2 + i];
      const uint32_t h = float_to_half_bits(c);
      m[i] = (h << 16) | h;
      const uint32_t l = float_to_half_bits(c - half_bits_to_float((uint16_t)h));
      lo[i] = (l << 16) | l;
    }
  }
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (mask & a) | (~mask & b); }

// 8 code indices (one byte of each bit-plane) -> 8 binary16 centroid values.
// Index = sum_p bit_p 2^p; the codebook is symmetric: the top bit is the sign (set = positive) and the lower
// bits count the magnitude outwards from zero (inverted for the negative half).
template <int BITS, bool WITH_LO = false>
__device__ __forceinline__ H8 centroids_of(const uint32_t (&byte)[BITS], const uint4* mask_tab, const Mags<BITS>& mg,
                                           H8* out_lo = nullptr) {
  H8 M[BITS];
#pragma unroll
  for (int p = 0; p < BITS; ++p) M[p].u = mask_tab[byte[p]];
  H8 out;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t top = M[BITS - 1].w[w];
    uint32_t mag, mlo = 0;
    if constexpr (BITS == 1) {
      mag = mg.m[0];
      if constexpr (WITH_LO) mlo = mg.lo[0];
    } else if constexpr (BITS == 2) {
      const uint32_t s0 = ~(M[0].w[w] ^ top);
      mag = bfi(s0, mg.m[1], mg.m[0]);
      if constexpr (WITH_LO) mlo = bfi(s0, mg.lo[1], mg.lo[0]);
    } else if constexpr (BITS == 3) {
      const uint32_t s0 = ~(M[0].w[w] ^ top), s1 = ~(M[1].w[w] ^ top);
      mag = bfi(s1, bfi(s0, mg.m[3], mg.m[2]), bfi(s0, mg.m[1], mg.m[0]));
      if constexpr (WITH_LO) mlo = bfi(s1, bfi(s0, mg.lo[3], mg.lo[2]), bfi(s0, mg.lo[1], mg.lo[0]));
    } else {
      const uint32_t s0 = ~(M[0].w[w] ^ top), s1 = ~(M[1].w[w] ^ top), s2 = ~(M[2].w[w] ^ top);
      const uint32_t lo = bfi(s1, bfi(s0, mg.m[3], mg.m[2]), bfi(s0, mg.m[1], mg.m[0]));
      const uint32_t hi = bfi(s1, bfi(s0, mg.m[7], mg.m[6]), bfi(s0, mg.m[5], mg.m[4]));
      mag = bfi(s2, hi, lo);
      if constexpr (WITH_LO) {
        const uint32_t llo = bfi(s1, bfi(s0, mg.lo[3], mg.lo[2]), bfi(s0, mg.lo[1], mg.lo[0]));
        const uint32_t lhi = bfi(s1, bfi(s0, mg.lo[7], mg.lo[6]), bfi(s0, mg.lo[5], mg.lo[4]));
        mlo = bfi(s2, lhi, llo);
      }
    }
    out.w[w] = bfi(0x7FFF7FFFu, mag, ~top);
    if constexpr (WITH_LO) out_lo->w[w] = mlo ^ (~top & 0x80008000u);   // negative centroid: flip the sign
  }
  return out;
}

// ---------------------------------------------------------------------------------------------
// decode: one workgroup per block
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(THREADS, 2) void eoq_decode_mfma_kernel(
    int n, int r_max, const uint16_t* __restrict__ pih, const float* __restrict__ tab,
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms, const int32_t* __restrict__ rank_in,
    const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac, uint16_t* __restrict__ out) {
  __shared__ __align__(16) uint16_t Z[CHUNK * ZLD];    // centroid values of the chunk, [token][coordinate]
  __shared__ __align__(16) uint16_t Ct[CHUNK * CLD];   // low-rank coefficients, [token][component]
  __shared__ __align__(16) float rho_s[CHUNK];         // rho / sqrt(d)
  __shared__ __align__(16) uint4 mask_tab[256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const size_t blk = blockIdx.x;
  const int r = rank_in[blk];
  const int jcol = 32 * wave + l32;  // output column of this lane

  build_mask_table(mask_tab, tid);
  Mags<BITS> mg;
  mg.load(tab);

  // stationary operands: Pi^T rows j (hi, lo) and the stored right factors V[i][j]
  const uint16_t* pit_hi = pih + 2 * D * D;
  const uint16_t* pit_lo = pih + 3 * D * D;
  H8 Bhi[8], Blo[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    Bhi[kk].u = *reinterpret_cast<const uint4*>(pit_hi + jcol * D + 16 * kk + 8 * hf);
    Blo[kk].u = *reinterpret_cast<const uint4*>(pit_lo + jcol * D + 16 * kk + 8 * hf);
  }
  H8 Bv[2];
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = 16 * k2 + 8 * hf + e;
      Bv[k2].s[e] = (i < r) ? rfac[(blk * r_max + i) * D + jcol] : (uint16_t)0;
    }
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  constexpr int ROWB = BITS * D / 8;

  for (int t0 = 0; t0 < n; t0 += CHUNK) {
    __syncthreads();  // previous chunk consumed; also orders the mask table before its first use
    // ---- phase 1: wave w prepares tile w (tokens t0 + 32w + l32) ----
    {
      const int tl = 32 * wave + l32;  // token within the chunk
      const size_t tok = blk * (size_t)n + t0 + tl;
      uint4 pl[BITS];
#pragma unroll
      for (int p = 0; p < BITS; ++p) pl[p] = *reinterpret_cast<const uint4*>(codes + tok * ROWB + p * 16);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        uint32_t byte[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) {
          const uint32_t wsel = (kk < 2) ? pl[p].x : (kk < 4) ? pl[p].y : (kk < 6) ? pl[p].z : pl[p].w;
          byte[p] = (wsel >> (16 * (kk & 1) + 8 * hf)) & 0xFFu;   // plane byte 2 kk + hf
        }
        const H8 c = centroids_of<BITS>(byte, mask_tab, mg);
        *reinterpret_cast<uint4*>(&Z[tl * ZLD + 16 * kk + 8 * hf]) = c.u;
      }
      if (hf == 0) rho_s[tl] = half_bits_to_float(norms[tok]) * inv_sqrt_d;
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) {
        H8 c;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int i = 16 * k2 + 8 * hf + e;
          c.s[e] = (i < r) ? lfac[(blk * r_max + i) * (size_t)n + t0 + tl] : (uint16_t)0;
        }
        *reinterpret_cast<uint4*>(&Ct[tl * CLD + 16 * k2 + 8 * hf]) = c.u;
      }
    }
    __syncthreads();
    // ---- phase 2: wave w produces columns 32w .. 32w+31 of every tile ----
#pragma unroll 1
    for (int tau = 0; tau < CHUNK / 32; ++tau) {
      float16v acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
      const int arow = 32 * tau + l32;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        H8 a;
        a.u = *reinterpret_cast<const uint4*>(&Z[arow * ZLD + 16 * kk + 8 * hf]);
        acc = mfma16(a, Bhi[kk], acc);
        acc = mfma16(a, Blo[kk], acc);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 s = *reinterpret_cast<const float4*>(&rho_s[32 * tau + 8 * q + 4 * hf]);
        acc[4 * q + 0] *= s.x;
        acc[4 * q + 1] *= s.y;
        acc[4 * q + 2] *= s.z;
        acc[4 * q + 3] *= s.w;
      }
      if (r > 0) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          if (16 * k2 < r) {
            H8 a;
            a.u = *reinterpret_cast<const uint4*>(&Ct[arow * CLD + 16 * k2 + 8 * hf]);
            acc = mfma16(a, Bv[k2], acc);
          }
        }
      }
      uint16_t* dst = out + (blk * (size_t)n + t0 + 32 * tau) * D + jcol;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v >> 2) + 4 * hf + (v & 3);
        dst[(size_t)row * D] = float_to_half_bits(acc[v]);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// scores: one workgroup per (sequence, KV head, run of blocks).  v_mfma_f32_16x16x32_f16: lane l supplies
// A[row = l%16][k = 8*(l/16) .. +7] and B[k = 8*(l/16) .. +7][col = l%16], receives D[row = 4*(l/16)+v][col = l%16].
// Rows are the query heads of the group (padded to 16), columns are 16 tokens; the 128 coordinates are
// visited in the order c = 32*(l/16) + 8*kk + e so that a lane needs exactly one 32-bit word of each bit-plane.
// ---------------------------------------------------------------------------------------------
typedef float float4v __attribute__((ext_vector_type(4)));
constexpr int SC_MAXG = 8;
constexpr int SC_RUN = 16;  // blocks per workgroup

__device__ __forceinline__ float4v mfma32(const H8& a, const H8& b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c, 0, 0, 0);
}
__device__ __forceinline__ void split_half(float v, uint16_t& hi, uint16_t& lo) {
  hi = float_to_half_bits(v);
  lo = float_to_half_bits(v - half_bits_to_float(hi));
}

template <int BITS>
__global__ __launch_bounds__(THREADS) void eoq_scores_mfma_kernel(
    int n, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, const float* __restrict__ pit,
    const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const uint16_t* __restrict__ q, float* __restrict__ scores) {
  __shared__ float qraw[SC_MAXG * D];
  __shared__ float qrot[SC_MAXG * D];
  __shared__ float wbuf[SC_MAXG * EOQ_RMAX_CAP];
  __shared__ __align__(16) uint4 mask_tab[256];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const size_t sg = blockIdx.y;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  const size_t q0 = (sq * n_q_heads + kv * group) * D;
  const size_t T = (size_t)blocks_per_head * n;
  constexpr int ROWB = BITS * D / 8;

  build_mask_table(mask_tab, tid);
  Mags<BITS> mg;
  mg.load(tab);
  for (int e = tid; e < group * D; e += THREADS) qraw[e] = half_bits_to_float(q[q0 + e]);
  __syncthreads();
  // q' = Pi q (the rotation moved to the query side: <q, Pi^T z> = <Pi q, z>)
  for (int e = tid; e < group * D; e += THREADS) {
    const int h = e >> 7, c = e & (D - 1);
    float acc = 0.0f;
    for (int j = 0; j < D; ++j) acc = fmaf(pit[j * D + c], qraw[h * D + j], acc);
    qrot[e] = acc;
  }
  __syncthreads();
  H8 Aq_hi[4], Aq_lo[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float v = (l16 < group) ? qrot[l16 * D + 32 * g + 8 * kk + e] : 0.0f;
      split_half(v, Aq_hi[kk].s[e], Aq_lo[kk].s[e]);
    }

  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  const int64_t j_end = min((int64_t)(blockIdx.x + 1) * SC_RUN, blocks_per_head);
  for (int64_t jb = (int64_t)blockIdx.x * SC_RUN; jb < j_end; ++jb) {
    const size_t blk = sg * (size_t)blocks_per_head + jb;
    const int r = rank_in[blk];
    __syncthreads();
    // w[h][i] = <v_i, q_h>: the low-rank term is <C_t, w_h>
    for (int e = tid; e < group * r; e += THREADS) {
      const int h = e / r, i = e % r;
      float acc = 0.0f;
      for (int j = 0; j < D; ++j)
        acc = fmaf(half_bits_to_float(rfac[(blk * r_max + i) * D + j]), qraw[h * D + j], acc);
      wbuf[h * EOQ_RMAX_CAP + i] = acc;
    }
    __syncthreads();
    H8 Aw_hi, Aw_lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = 8 * g + e;
      const float v = (l16 < group && i < r) ? wbuf[l16 * EOQ_RMAX_CAP + i] : 0.0f;
      split_half(v, Aw_hi.s[e], Aw_lo.s[e]);
    }
    for (int tile = wave; tile < n / 16; tile += THREADS / 64) {
      const int t = 16 * tile + l16;
      const size_t tok = blk * (size_t)n + t;
      uint32_t word[BITS];
#pragma unroll
      for (int p = 0; p < BITS; ++p) word[p] = *reinterpret_cast<const uint32_t*>(codes + tok * ROWB + p * 16 + 4 * g);
      float4v acc1 = {0.f, 0.f, 0.f, 0.f}, acc2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint32_t byte[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) byte[p] = (word[p] >> (8 * kk)) & 0xFFu;
        H8 blo;
        const H8 bhi = centroids_of<BITS, true>(byte, mask_tab, mg, &blo);
        acc1 = mfma32(Aq_hi[kk], bhi, acc1);
        acc1 = mfma32(Aq_lo[kk], bhi, acc1);
        acc1 = mfma32(Aq_hi[kk], blo, acc1);
      }
      if (r > 0) {
        H8 c;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int i = 8 * g + e;
          c.s[e] = (i < r) ? lfac[(blk * r_max + i) * (size_t)n + t] : (uint16_t)0;
        }
        acc2 = mfma32(Aw_hi, c, acc2);
        acc2 = mfma32(Aw_lo, c, acc2);
      }
      const float rho = half_bits_to_float(norms[tok]) * inv_sqrt_d;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int h = 4 * g + v;
        if (h < group)
          scores[(sq * n_q_heads + kv * group + h) * T + (size_t)jb * n + t] = fmaf(acc1[v], rho, acc2[v]) * inv_sqrt_d;
      }
    }
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
hipError_t eoq_launch_decode(const EoqLaunch& L, eoq_packed in, int64_t B, void* out_fp16) {
  if (L.ev) (void)hipEventRecord(L.ev[4], L.stream);
  const dim3 grid((unsigned)B), block(THREADS);
  uint16_t* out = static_cast<uint16_t*>(out_fp16);
#define EOQ_DECODE(BITS)                                                                                          \
  hipLaunchKernelGGL(eoq_decode_mfma_kernel<BITS>, grid, block, 0, L.stream, L.n, L.r_max, L.pih, L.tab, in.codes, \
                     in.norms, in.rank, in.lfac, in.rfac, out)
  switch (L.bits) {
    case 1: EOQ_DECODE(1); break;
    case 2: EOQ_DECODE(2); break;
    case 3: EOQ_DECODE(3); break;
    default: EOQ_DECODE(4); break;
  }
#undef EOQ_DECODE
  if (L.ev) (void)hipEventRecord(L.ev[5], L.stream);
  return hipGetLastError();
}

hipError_t eoq_launch_scores(const EoqLaunch& L, eoq_packed keys, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores) {
  const int64_t runs = (blocks_per_head + SC_RUN - 1) / SC_RUN;
  const int64_t sg_total = n_seq * n_kv_heads;
  if (sg_total > 65535 || runs > 0x7FFFFFFF) return hipErrorInvalidValue;
  if (L.ev) (void)hipEventRecord(L.ev[6], L.stream);
  const dim3 grid((unsigned)runs, (unsigned)sg_total), block(THREADS);
  const uint16_t* q = static_cast<const uint16_t*>(q_fp16);
#define EOQ_SCORES(BITS)                                                                                          \
  hipLaunchKernelGGL(eoq_scores_mfma_kernel<BITS>, grid, block, 0, L.stream, L.n, L.r_max, n_kv_heads,            \
                     n_q_heads / n_kv_heads, blocks_per_head, L.pit, L.tab, keys.codes, keys.norms, keys.rank,    \
                     keys.lfac, keys.rfac, q, scores)
  switch (L.bits) {
    case 1: EOQ_SCORES(1); break;
    case 2: EOQ_SCORES(2); break;
    case 3: EOQ_SCORES(3); break;
    default: EOQ_SCORES(4); break;
  }
#undef EOQ_SCORES
  if (L.ev) (void)hipEventRecord(L.ev[7], L.stream);
  return hipGetLastError();
}
