// Matrix-core (MFMA, gfx950) kernels of the residual coder for binary16 blocks:
//   decode : x_hat = (rho/sqrt(d)) z_hat Pi + C V^T  (Alg. 1 line 6 plus the stored low-rank part)
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
  uint32_t m[(1 << BITS) / 2];
  __device__ __forceinline__ void load(const float* __restrict__ tab) {
#pragma unroll
    for (int i = 0; i < (1 << BITS) / 2; ++i) {
      const uint32_t h = float_to_half_bits(tab[(1 << BITS) / 2 + i]);
      m[i] = (h << 16) | h;
    }
  }
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (mask & a) | (~mask & b); }

// 8 code indices (one byte of each bit-plane) -> 8 binary16 centroid values.
// Index = sum_p bit_p 2^p; the codebook is symmetric: the top bit is the sign (set = positive) and the lower
// bits count the magnitude outwards from zero (inverted for the negative half).
template <int BITS>
__device__ __forceinline__ H8 centroids_of(const uint32_t (&byte)[BITS], const uint4* mask_tab, const Mags<BITS>& mg) {
  H8 M[BITS];
#pragma unroll
  for (int p = 0; p < BITS; ++p) M[p].u = mask_tab[byte[p]];
  H8 out;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t top = M[BITS - 1].w[w];
    uint32_t mag;
    if constexpr (BITS == 1) {
      mag = mg.m[0];
    } else if constexpr (BITS == 2) {
      const uint32_t s0 = ~(M[0].w[w] ^ top);
      mag = bfi(s0, mg.m[1], mg.m[0]);
    } else if constexpr (BITS == 3) {
      const uint32_t s0 = ~(M[0].w[w] ^ top), s1 = ~(M[1].w[w] ^ top);
      mag = bfi(s1, bfi(s0, mg.m[3], mg.m[2]), bfi(s0, mg.m[1], mg.m[0]));
    } else {
      const uint32_t s0 = ~(M[0].w[w] ^ top), s1 = ~(M[1].w[w] ^ top), s2 = ~(M[2].w[w] ^ top);
      const uint32_t lo = bfi(s1, bfi(s0, mg.m[3], mg.m[2]), bfi(s0, mg.m[1], mg.m[0]));
      const uint32_t hi = bfi(s1, bfi(s0, mg.m[7], mg.m[6]), bfi(s0, mg.m[5], mg.m[4]));
      mag = bfi(s2, hi, lo);
    }
    out.w[w] = bfi(0x7FFF7FFFu, mag, ~top);
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
