// Matrix-core (MFMA, gfx950) kernels of the residual coder for binary16 blocks:
//   encode : projection, residual against the stored factors, norm, rotation, Lloyd-Max index, packing
//            (Alg. 3 with Alg. 1 lines 3-5)
//   decode : x_hat = (rho/sqrt(d)) z_hat Pi + C V^T  (Alg. 1 line 6 plus the stored low-rank part); the rotation enters
//            as its binary16 rounding (one matrix-core pass): |error| <= 2^-11 rho |z_hat| per entry, the size of the
//            binary16 rounding of the result itself
//   qjl    : TQ_prod side information of stored records (Alg. 1 optional lines)
//
// Operand convention of v_mfma_f32_32x32x16_f16 (wave64): for D = A(32xK) * B(Kx32) + C, lane l supplies
// A[row = l%32][k = 8*(l/32) .. +7] and B[k = 8*(l/32) .. +7][col = l%32]; it receives
// D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator register v = 0..15.
//
// Layout of the work: the rotation is the stationary operand.  In the encoder and the qjl kernel wave w of a workgroup
// keeps the 32 columns j = 32w .. 32w+31 of Pi (binary16 hi + lo parts, B operand) in registers for the whole block; the
// tokens stream through LDS in tiles of 32 (A operand), each tile prepared by one wave and consumed by all four.  In the
// decoder every wave keeps the whole of Pi^T (binary16 rounding, A operand) and works on tiles of its own.
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

// Buffer descriptor over `bytes` bytes at `base` (raw addressing: loads past the end return zero).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(bytes > 0x7FFFFFFFu ? 0x7FFFFFFFu : bytes),
                                           0x00020000);
}

__device__ __forceinline__ float16v mfma16(const H8& a, const H8& b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, c, 0, 0, 0);
}

__device__ __forceinline__ void split_half(float v, uint16_t& hi, uint16_t& lo) {
  hi = float_to_half_bits(v);
  lo = float_to_half_bits(v - half_bits_to_float(hi));
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

// Direct table for codes of 1 or 2 bits: entry (nibble of plane 0 | nibble of plane 1 << 4) -> the binary16 centroids of
// the four coordinates of that nibble (code of coordinate e = bit e of plane 0 + 2 * bit e of plane 1; index 0 is the most
// negative centroid of the ascending N(0,1) table).
template <int BITS>
__device__ __forceinline__ void build_centroid_table(uint2* tab4, const float* __restrict__ cent, int tid) {
  static_assert(BITS <= 2, "one nibble of two planes at most");
  if (tid < 256) {
    const int n0 = tid & 15, n1 = tid >> 4;
    uint16_t h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int code = ((n0 >> e) & 1) | ((BITS == 2) ? (((n1 >> e) & 1) << 1) : 0);
      h[e] = float_to_half_bits(cent[code]);
    }
    tab4[tid] = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
  }
}

// Tables for codes of 3 bits: entry (nibble of m_0 | nibble of m_1 << 4) -> the binary16 magnitudes of four coordinates
// (m_p = magnitude bit p of the code: plane p where the sign plane is set, its complement where it is clear; level
// m_0 + 2 m_1 is centroid L/2 + level of the ascending table), and behind them 16 entries (nibble of the sign plane) ->
// the sign bits of the four halfwords (set where the plane bit is clear: negative).
__device__ __forceinline__ void build_magnitude_table3(uint2* tab4, const float* __restrict__ cent, int tid) {
  if (tid < 256) {
    const int n0 = tid & 15, n1 = tid >> 4;
    uint16_t h[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) h[e] = float_to_half_bits(cent[4 + (((n0 >> e) & 1) | (((n1 >> e) & 1) << 1))]);
    tab4[tid] = make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
    if (tid < 16) {
      uint32_t lo = 0u, hi = 0u;
      if (!(tid & 1)) lo |= 0x8000u;
      if (!(tid & 2)) lo |= 0x80000000u;
      if (!(tid & 4)) hi |= 0x8000u;
      if (!(tid & 8)) hi |= 0x80000000u;
      tab4[256 + tid] = make_uint2(lo, hi);
    }
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
// Record fetches of the workgroup-per-block kernels (TQ_prod side information below).
// ---------------------------------------------------------------------------------------------
// What one thread requests of a chunk of 128 tokens: lane (l32, hf) of wave w unpacks half of token 32 w + l32;
// thread tid also carries 8 tokens of row (tid + 256 u) / 16 of the left factors, u = 0, 1.
template <int BITS>
struct DecodeFetch {
  uint4 pl[BITS];  // the token's bit-planes
  uint4 cf[2];     // left factors C[i][8 seg .. 8 seg + 7], (i, seg) = ((tid + 256 u) / 16, tid % 16), if i < r
  uint16_t rho;    // the token's stored norm
  int r;           // rank of the block the chunk belongs to
};
template <int BITS>
__device__ __forceinline__ void decode_fetch(DecodeFetch<BITS>& f, int64_t blk, int t0, int n, int r, int r_max, int tid, int tl,
                                             const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
                                             const uint16_t* __restrict__ lfac) {
  constexpr int ROWB = BITS * D / 8;
  const size_t tok = (size_t)blk * n + t0 + tl;
  f.r = r;
#pragma unroll
  for (int p = 0; p < BITS; ++p) f.pl[p] = *reinterpret_cast<const uint4*>(codes + tok * ROWB + p * 16);
  f.rho = norms[tok];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = (tid + THREADS * u) >> 4, seg = tid & 15;
    f.cf[u] = (i < r) ? *reinterpret_cast<const uint4*>(lfac + ((size_t)blk * r_max + i) * n + t0 + 8 * seg)
                      : make_uint4(0u, 0u, 0u, 0u);
  }
}
// right factors of a block as B operand of the low-rank product: V[i][jcol], i = 16 k2 + 8 hf + e.  The sixteen
// two-byte loads land in registers of their own and are packed by pack_v once they are needed, so that issuing
// them waits for nothing.
__device__ __forceinline__ void decode_fetch_v(uint32_t (&raw)[16], int64_t blk, int r, int r_max, int jcol, int hf,
                                               const uint16_t* __restrict__ rfac) {
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int i = 16 * (q >> 3) + 8 * hf + (q & 7);
    raw[q] = (i < r) ? (uint32_t)rfac[((size_t)blk * r_max + i) * D + jcol] : 0u;
  }
}
__device__ __forceinline__ void pack_v(H8 (&Bv)[2], const uint32_t (&raw)[16]) {
#pragma unroll
  for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
    for (int w = 0; w < 4; ++w) Bv[k2].w[w] = raw[8 * k2 + 2 * w] | (raw[8 * k2 + 2 * w + 1] << 16);
}
// Rank of block blk as a vector load (zero past the end of the array): a scalar load would share its counter with
// the LDS traffic and be waited for at the next LDS wait, a vector load is waited for where its value is read.
__device__ __forceinline__ int rank_request(__amdgpu_buffer_rsrc_t ranks, int64_t blk) {
  return __builtin_amdgcn_raw_buffer_load_b32(ranks, 0, (int)(blk * 4), 0);
}
__device__ __forceinline__ int rank_value(int raw, int r_max) {
  return min(max(__builtin_amdgcn_readfirstlane(raw), 0), r_max);   // records may come from storage
}

// ---------------------------------------------------------------------------------------------
// decode kernel proper: every wave is a worker of its own.  A unit of work is a run of consecutive 32-token tiles of
// one block (the whole block when the batch is large); wave g of the grid takes the units g, g + waves, ...  The whole
// of Pi^T (binary16) is stationary in the wave's registers as the A operand (4 column blocks x 8 instructions), the
// centroid values of a token go from the bit-planes straight into the B operand of the lane that owns the token, and
// the product comes out transposed: D[output column][token], so a lane holds 4 x 4 consecutive columns of ITS token
// per column block, scales them by its own rho, rounds them in pairs and hands them to a wave-private LDS tile from
// which the 32 rows leave as 16-byte stores, 1 KB contiguous per instruction.  No barrier after the set-up.
// The contraction index is permuted so that lane half hf owns coordinates 64 hf .. 64 hf + 63 (8 consecutive bytes
// of every bit-plane): slot e of instruction kk is coordinate 64 hf + 8 kk + e on both operands.
// ---------------------------------------------------------------------------------------------
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// What a lane requests of a tile: lane (l32, hf) owns token l32 of the tile.
template <int BITS>
struct TileFetch {
  u32x2 pl[BITS];   // bytes 8 hf .. 8 hf + 7 of every bit-plane of the token
  uint32_t rho;     // the token's stored norm (binary16 in the low half)
  u32x4 cf;         // lane L: stored coefficients C[tokens 8 (L % 4) .. + 7 of the tile][component L / 4]; zero at and above the rank
};
// Buffer descriptors of the block a tile belongs to (scalar registers).  Everything that must read as zero does so by
// the range check of the descriptor, which covers the per-lane offset: rows at and above the rank lie past the end of
// `lfac`, and a request behind the last tile goes through descriptors of size zero.
struct TileSource {
  __amdgpu_buffer_rsrc_t codes, norms, lfac;
};
constexpr int CTLD = 32 + 8;   // row stride (halfs) of a tile's coefficient rows in LDS, [component][token]

template <int BITS>
__global__ __launch_bounds__(THREADS, 2) void eoq_decode_mfma_kernel(
    int n, int r_max, int64_t B, int parts_log2, const uint16_t* __restrict__ pih, const float* __restrict__ tab,
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms, const int32_t* __restrict__ rank_in,
    const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac, uint16_t* __restrict__ out) {
  __shared__ __align__(16) uint4 mask_tab[256];            // BITS = 4: plane byte -> halfword masks; BITS <= 3: the nibble tables
  __shared__ __align__(16) uint16_t Ot[4 * 32 * ZLD];      // per wave: one output tile, [token][column]
  __shared__ __align__(16) uint16_t Cs[4 * 2 * 16 * CTLD]; // per wave: coefficient rows 0..15 and 16..31 of a tile
  __shared__ __align__(16) uint4 V2[4 * 4 * 64];           // per wave: operands of components 16..31 (blocks of rank > 16)
  uint2* cen_tab = reinterpret_cast<uint2*>(mask_tab);
  constexpr int ROWB = BITS * D / 8;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hf = lane >> 5;

  // binary16 results that overflow become the largest finite value instead of infinity (mode bit FP16_OVFL): the
  // output saturates like every other binary16 quantity of the record, without a clamp per element
  set_fp16_overflow_clamp();

  if constexpr (BITS <= 2) build_centroid_table<BITS>(cen_tab, tab, tid);
  else if constexpr (BITS == 3) build_magnitude_table3(cen_tab, tab, tid);
  else build_mask_table(mask_tab, tid);
  Mags<BITS> mg;
  if constexpr (BITS == 4) mg.load(tab);
  __syncthreads();   // the only one: from here on the waves do not meet again

  const int tiles_per_unit = (n / 32) >> parts_log2;
  const int part_mask = (1 << parts_log2) - 1;
  const int64_t U = B << parts_log2;
  const int64_t GW = (int64_t)gridDim.x * 4;
  int64_t u = (int64_t)blockIdx.x * 4 + wave;
  if (u >= U) return;

  // stationary operand: rows j = 32 cb + l32 of Pi^T rounded to binary16, contraction slots in the permuted order
  const uint16_t* pit_hi = pih + 2 * D * D;
  H8 Ap[4][8];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      Ap[cb][kk].u = *reinterpret_cast<const uint4*>(pit_hi + (32 * cb + l32) * D + 64 * hf + 8 * kk);
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);

  const __amdgpu_buffer_rsrc_t ranks = buffer_of(rank_in, (size_t)B * 4);
  // per-lane parts of the offsets (they never change)
  const uint32_t vo_code = (uint32_t)(l32 * ROWB + 8 * hf);
  const uint32_t vo_norm = (uint32_t)(2 * l32);
  const uint32_t vo_cf = (uint32_t)(((lane >> 2) * n + (lane & 3) * 8) * 2);   // row L / 4 of the coefficients: range-checked per row
  const uint32_t vo_row = (uint32_t)((lane >> 4) * (D * 2) + (lane & 15) * 16);   // 16-byte piece of row L / 16 of a [.][128] binary16 array
  uint16_t* ot = Ot + wave * (32 * ZLD);
  uint16_t* cs = Cs + wave * (2 * 16 * CTLD);
  uint4* v2 = V2 + wave * (4 * 64);

  auto source_of = [&](int64_t blk, int r, bool valid) __attribute__((always_inline)) {
    TileSource s;
    s.codes = buffer_of(codes + (size_t)blk * n * ROWB, valid ? (size_t)n * ROWB : 0);
    s.norms = buffer_of(norms + (size_t)blk * n, valid ? (size_t)n * 2 : 0);
    s.lfac = buffer_of(lfac + (size_t)blk * r_max * n, valid ? (size_t)r * n * 2 : 0);
    return s;
  };
  auto request = [&](TileFetch<BITS>& f, const TileSource& s, int t0) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < BITS; ++p) f.pl[p] = __builtin_amdgcn_raw_buffer_load_b64(s.codes, vo_code + 16 * p, t0 * ROWB, 0);
    f.rho = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(s.norms, vo_norm, t0 * 2, 0);
    f.cf = __builtin_amdgcn_raw_buffer_load_b128(s.lfac, vo_cf, t0 * 2, 0);
  };
  // V[8 hf + e + 16 k2][32 cb + l32], e = 0 .. 7, of the rows staged in the wave's LDS tile: an A operand of the low-rank product
  auto v_operand = [&](int cb) __attribute__((always_inline)) {
    H8 x;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t a = ot[(8 * hf + 2 * w) * ZLD + 32 * cb + l32], b = ot[(8 * hf + 2 * w + 1) * ZLD + 32 * cb + l32];
      x.w[w] = a | (b << 16);
    }
    return x;
  };
  // C[token l32][8 hf + e + 16 k2] of the rows staged in the wave's coefficient tile: the B operand of that product
  auto c_operand = [&](int k2) __attribute__((always_inline)) {
    H8 x;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t a = cs[(16 * k2 + 8 * hf + 2 * w) * CTLD + l32], b = cs[(16 * k2 + 8 * hf + 2 * w + 1) * CTLD + l32];
      x.w[w] = a | (b << 16);
    }
    return x;
  };

  // state of the unit being worked on and of the one after it
  int64_t blk = u >> parts_log2;
  int part = (int)u & part_mask;
  int r = rank_value(rank_request(ranks, blk), r_max);
  int rk_next = rank_request(ranks, min((u + GW) >> parts_log2, B - 1));   // behind the last unit: not used
  TileSource src = source_of(blk, r, true);
  TileFetch<BITS> cur, nxt;
  request(cur, src, 32 * part * tiles_per_unit);
  H8 Bv[4];   // right factors of the unit's block as A operand of the low-rank product: V[8 hf + e][32 cb + l32]
  __amdgpu_buffer_rsrc_t obuf = buffer_of(out, 0);
  int ti = 0;
  // nothing of the set-up is left in flight: inside the loop a wait then only ever covers what the loop itself
  // requested, and never the stores of the tile before
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  for (;;) {
    if (ti == 0) {
      // rows of the block's right factors travel as 16-byte pieces (rows at and above the rank read zero), change
      // lanes through the wave's LDS tile and are read back one binary16 at a time in operand order; rows 16 .. 31
      // (blocks of rank > 16, rare) are kept in LDS as finished operands
      const __amdgpu_buffer_rsrc_t vbuf = buffer_of(rfac + (size_t)blk * r_max * D, (size_t)r * D * 2);
      for (int k2 = (r > 16) ? 1 : 0; k2 >= 0; --k2) {   // uniform
        u32x4 vrow[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) vrow[k] = __builtin_amdgcn_raw_buffer_load_b128(vbuf, vo_row + (16 * k2 + 4 * k) * (D * 2), 0, 0);
#pragma unroll
        for (int k = 0; k < 4; ++k) *reinterpret_cast<u32x4*>(ot + (4 * k + (lane >> 4)) * ZLD + (lane & 15) * 8) = vrow[k];
        __builtin_amdgcn_wave_barrier();
        if (k2 == 1) {
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) v2[cb * 64 + lane] = v_operand(cb).u;
        } else {
#pragma unroll
          for (int cb = 0; cb < 4; ++cb) Bv[cb] = v_operand(cb);
        }
        __builtin_amdgcn_wave_barrier();
      }
      obuf = buffer_of(out + (size_t)blk * n * D, (size_t)n * D * 2);
    }
    const int t0 = 32 * (part * tiles_per_unit + ti);
    // ---- request the next tile: of this unit, or the first one of the wave's next unit ----
    const bool unit_ends = ti + 1 == tiles_per_unit;
    const int64_t un = u + GW;
    const bool more = un < U;
    int64_t blk_n = blk;
    int part_n = part, r_n = r, t_n = t0 + 32;
    if (unit_ends) {   // uniform
      blk_n = more ? (un >> parts_log2) : blk;
      part_n = (int)un & part_mask;
      r_n = rank_value(rk_next, r_max);
      rk_next = rank_request(ranks, min((un + GW) >> parts_log2, B - 1));
      src = source_of(blk_n, r_n, more);
      t_n = 32 * part_n * tiles_per_unit;
    }
    request(nxt, src, t_n);

    // ---- this tile ----
    const float rs = half_bits_to_float((uint16_t)cur.rho) * inv_sqrt_d;
    H8 Cop;   // C[token][8 hf + e], the B operand of the low-rank product
    if (r > 0) {   // uniform
      // lane L holds eight tokens of component L / 4: row L / 4 of the coefficient tile
      *reinterpret_cast<u32x4*>(cs + (lane >> 2) * CTLD + (lane & 3) * 8) = cur.cf;
      __builtin_amdgcn_wave_barrier();
      Cop = c_operand(0);
    }
    // nibble words of the lane's 64 coordinates (BITS <= 3): byte kk of word set [kk / 4] is instruction kk
    uint32_t even[2], odd[2], seven[2], sodd[2];
    if constexpr (BITS <= 3) {
#pragma unroll
      for (int wq = 0; wq < 2; ++wq) {
        uint32_t a, b;
        if constexpr (BITS == 1) {
          a = cur.pl[0][wq];
          b = 0u;
        } else if constexpr (BITS == 2) {
          a = cur.pl[0][wq];
          b = cur.pl[1][wq];
        } else {
          // magnitude bit p of a code: plane p where the sign plane is set, its complement where it is clear
          a = ~(cur.pl[0][wq] ^ cur.pl[2][wq]);
          b = ~(cur.pl[1][wq] ^ cur.pl[2][wq]);
          seven[wq] = cur.pl[2][wq] & 0x0F0F0F0Fu;
          sodd[wq] = (cur.pl[2][wq] >> 4) & 0x0F0F0F0Fu;
        }
        even[wq] = bfi(0x0F0F0F0Fu, a, b << 4);   // byte j: low nibbles of byte j of the two planes
        odd[wq] = bfi(0x0F0F0F0Fu, a >> 4, b);    // byte j: high nibbles
      }
    }
    auto operand = [&](auto kk_ic) __attribute__((always_inline)) {
      constexpr int kk = decltype(kk_ic)::value;
      H8 z;
      if constexpr (BITS <= 3) {
        const uint2 lo4 = cen_tab[(even[kk >> 2] >> (8 * (kk & 3))) & 0xFFu], hi4 = cen_tab[(odd[kk >> 2] >> (8 * (kk & 3))) & 0xFFu];
        z.u = make_uint4(lo4.x, lo4.y, hi4.x, hi4.y);
        if constexpr (BITS == 3) {
          const uint2 ls = cen_tab[256 + ((seven[kk >> 2] >> (8 * (kk & 3))) & 0xFFu)];
          const uint2 hs = cen_tab[256 + ((sodd[kk >> 2] >> (8 * (kk & 3))) & 0xFFu)];
          z.u = make_uint4(lo4.x | ls.x, lo4.y | ls.y, hi4.x | hs.x, hi4.y | hs.y);
        }
      } else {
        uint32_t byte[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) byte[p] = (cur.pl[p][kk >> 2] >> (8 * (kk & 3))) & 0xFFu;
        z = centroids_of<BITS>(byte, mask_tab, mg);
      }
      return z;
    };
    // all four column blocks at once (every unpacked operand feeds four matrix instructions); at 4 bits, where the
    // unpacking itself needs more registers, one at a time in four passes
    constexpr int NCB = (BITS == 4) ? 1 : 4;
#pragma unroll
    for (int pass = 0; pass < 4 / NCB; ++pass) {
      float16v acc[NCB];
#pragma unroll
      for (int c = 0; c < NCB; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
      EOQ_SFOR(kk, 8,
        const H8 z = operand(std::integral_constant<int, kk>{});
        EOQ_SFOR(c, NCB, acc[c] = mfma16(Ap[NCB * pass + c][kk], z, acc[c]););
      );
#pragma unroll
      for (int c = 0; c < NCB; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] *= rs;
      if (r > 0) {   // uniform
        EOQ_SFOR(c, NCB, acc[c] = mfma16(Bv[NCB * pass + c], Cop, acc[c]););
        if (r > 16) {
          // components 16 .. 31: their coefficient rows of this tile are fetched here, nothing of them is kept
          if (pass == 0) {
            const __amdgpu_buffer_rsrc_t lbuf = buffer_of(lfac + (size_t)blk * r_max * n, (size_t)r * n * 2);
            const u32x4 c2 = __builtin_amdgcn_raw_buffer_load_b128(lbuf, vo_cf + (uint32_t)(16 * n * 2), t0 * 2, 0);
            *reinterpret_cast<u32x4*>(cs + (16 + (lane >> 2)) * CTLD + (lane & 3) * 8) = c2;
            __builtin_amdgcn_wave_barrier();
          }
          const H8 c2op = c_operand(1);
          EOQ_SFOR(c, NCB,
            H8 va;
            va.u = v2[(NCB * pass + c) * 64 + lane];
            acc[c] = mfma16(va, c2op, acc[c]);
          );
        }
      }
      // register v of column block cb is column 32 cb + 8 (v / 4) + 4 hf + v % 4 of the lane's token
#pragma unroll
      for (int c = 0; c < NCB; ++c)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint2 pk = make_uint2(pack_half2(acc[c][4 * q], acc[c][4 * q + 1]), pack_half2(acc[c][4 * q + 2], acc[c][4 * q + 3]));
          *reinterpret_cast<uint2*>(ot + l32 * ZLD + 32 * (NCB * pass + c) + 8 * q + 4 * hf) = pk;
        }
    }
    // the tile leaves by rows: lane L stores 16 bytes of row 4 ps + L / 16 (one wave's LDS operations complete in order)
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int ps = 0; ps < 8; ++ps) {
      const uint4 val = *reinterpret_cast<const uint4*>(ot + (4 * ps + (lane >> 4)) * ZLD + (lane & 15) * 8);
      const u32x4 vv = {val.x, val.y, val.z, val.w};
      __builtin_amdgcn_raw_buffer_store_b128(vv, obuf, vo_row, (t0 + 4 * ps) * (D * 2), 0);
    }
    __builtin_amdgcn_wave_barrier();

    cur = nxt;
    if (unit_ends) {
      if (!more) break;
      u = un;
      blk = blk_n;
      part = part_n;
      r = r_n;
      ti = 0;
    } else {
      ++ti;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// TQ_prod side information (Alg. 1 lines "TQ_prod"): one workgroup per block.  The reconstruction of the record is
// formed as in the decoder, tile by tile in float32 accumulators (centroids and rotation as binary16 hi + lo here:
// the residual is a small difference), r_x = S - x_hat goes to LDS as binary16 hi + lo, its norm is taken there, and
// one more product with Phi (binary16 by definition, stationary in registers like the rotation) gives Phi r_x, of
// which only the signs are kept, packed like one more bit-plane.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(THREADS, 1) void eoq_qjl_kernel(
    const uint16_t* __restrict__ blocks, int n, int r_max, const uint16_t* __restrict__ pih,
    const uint16_t* __restrict__ phih, const float* __restrict__ tab, const uint8_t* __restrict__ codes,
    const uint16_t* __restrict__ norms, const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac,
    const uint16_t* __restrict__ rfac, uint8_t* __restrict__ qsigns, uint16_t* __restrict__ qnorms) {
  __shared__ __align__(16) uint16_t Z[CHUNK * ZLD];     // centroid values (hi) of the chunk, [token][coordinate]
  __shared__ __align__(16) uint16_t Zl[CHUNK * ZLD];    // their low parts
  __shared__ __align__(16) uint16_t Ct[CHUNK * CLD];    // low-rank coefficients, [token][component]
  __shared__ __align__(16) float rho_s[CHUNK];          // rho / sqrt(d)
  __shared__ __align__(16) uint4 mask_tab[256];
  // residual tiles of 64 tokens (two tiles of 32), hi and lo, double-buffered: while the products with Phi read one
  // pair the next two tiles are written into the other, so one barrier per 64 tokens is enough
  __shared__ __align__(16) uint16_t Eh[2][64 * ZLD];
  __shared__ __align__(16) uint16_t El[2][64 * ZLD];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const int jcol = 32 * wave + l32;
  const int tl = 32 * wave + l32;
  const size_t blk = blockIdx.x;

  build_mask_table(mask_tab, tid);
  for (int e = tid; e < CHUNK * CLD / 8; e += THREADS) *reinterpret_cast<uint4*>(&Ct[e * 8]) = make_uint4(0u, 0u, 0u, 0u);
  Mags<BITS> mg;
  mg.load(tab);
  const uint16_t* pit_hi = pih + 2 * D * D;
  const uint16_t* pit_lo = pih + 3 * D * D;
  // stationary operands: columns of Pi^T (hi + lo) and rows of Phi (binary16 as it is) of this lane
  H8 Bhi[8], Blo[8], Fhi[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    Bhi[kk].u = *reinterpret_cast<const uint4*>(pit_hi + jcol * D + 16 * kk + 8 * hf);
    Blo[kk].u = *reinterpret_cast<const uint4*>(pit_lo + jcol * D + 16 * kk + 8 * hf);
    Fhi[kk].u = *reinterpret_cast<const uint4*>(phih + jcol * D + 16 * kk + 8 * hf);
  }
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  DecodeFetch<BITS> cur;
  H8 Bv[2];
  const int r = min(max(rank_in[blk], 0), r_max);
  {
    uint32_t vraw[16];
    decode_fetch_v(vraw, blk, r, r_max, jcol, hf, rfac);
    pack_v(Bv, vraw);
  }
  int eb = 0;   // residual buffer of the current pair of tiles

  for (int t0 = 0; t0 < n; t0 += CHUNK) {
    decode_fetch<BITS>(cur, blk, t0, n, r, r_max, tid, tl, codes, norms, lfac);
    // the block's own entries S[row][jcol] of the first pair of tiles
    uint16_t sv[2][16];
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const uint16_t* srow = blocks + (blk * (size_t)n + t0 + 32 * h2) * D + jcol;
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[h2][v] = srow[(size_t)(8 * (v >> 2) + 4 * hf + (v & 3)) * D];
    }
    __syncthreads();  // previous chunk consumed; orders the mask table and the cleared Ct before first use
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      uint32_t byte[BITS];
#pragma unroll
      for (int p = 0; p < BITS; ++p) {
        const uint32_t wsel = (kk < 2) ? cur.pl[p].x : (kk < 4) ? cur.pl[p].y : (kk < 6) ? cur.pl[p].z : cur.pl[p].w;
        byte[p] = (wsel >> (16 * (kk & 1) + 8 * hf)) & 0xFFu;
      }
      H8 clo;
      const H8 c = centroids_of<BITS, true>(byte, mask_tab, mg, &clo);
      *reinterpret_cast<uint4*>(&Z[tl * ZLD + 16 * kk + 8 * hf]) = c.u;
      *reinterpret_cast<uint4*>(&Zl[tl * ZLD + 16 * kk + 8 * hf]) = clo.u;
    }
    if (hf == 0) rho_s[tl] = half_bits_to_float(cur.rho) * inv_sqrt_d;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int i = (tid + THREADS * u) >> 4, seg = tid & 15;
      if (i < r) {
        H8 c;
        c.u = cur.cf[u];
#pragma unroll
        for (int x = 0; x < 8; ++x) Ct[(8 * seg + x) * CLD + i] = c.s[x];
      }
    }
    __syncthreads();
#pragma unroll 1
    for (int tau = 0; tau < CHUNK / 32; tau += 2) {
      uint16_t svn[2][16];
      if (tau + 2 < CHUNK / 32) {   // the next pair's entries of S, requested before this pair's products
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const uint16_t* srow = blocks + (blk * (size_t)n + t0 + 32 * (tau + 2 + h2)) * D + jcol;
#pragma unroll
          for (int v = 0; v < 16; ++v) svn[h2][v] = srow[(size_t)(8 * (v >> 2) + 4 * hf + (v & 3)) * D];
        }
      }
      // ---- x_hat of tokens 32 tau .. 32 tau + 63, columns 32 wave .. 32 wave + 31: two independent chains ----
      float16v acc[2];
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[0][v] = acc[1][v] = 0.0f;
      const int arow = 32 * tau + l32;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        H8 a0, a1, b0, b1;
        a0.u = *reinterpret_cast<const uint4*>(&Z[arow * ZLD + 16 * kk + 8 * hf]);
        b0.u = *reinterpret_cast<const uint4*>(&Z[(arow + 32) * ZLD + 16 * kk + 8 * hf]);
        a1.u = *reinterpret_cast<const uint4*>(&Zl[arow * ZLD + 16 * kk + 8 * hf]);
        b1.u = *reinterpret_cast<const uint4*>(&Zl[(arow + 32) * ZLD + 16 * kk + 8 * hf]);
        acc[0] = mfma16(a0, Bhi[kk], acc[0]);
        acc[1] = mfma16(b0, Bhi[kk], acc[1]);
        acc[0] = mfma16(a0, Blo[kk], acc[0]);
        acc[1] = mfma16(b0, Blo[kk], acc[1]);
        acc[0] = mfma16(a1, Bhi[kk], acc[0]);
        acc[1] = mfma16(b1, Bhi[kk], acc[1]);
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 s = *reinterpret_cast<const float4*>(&rho_s[32 * (tau + h2) + 8 * q + 4 * hf]);
          acc[h2][4 * q + 0] *= s.x;
          acc[h2][4 * q + 1] *= s.y;
          acc[h2][4 * q + 2] *= s.z;
          acc[h2][4 * q + 3] *= s.w;
        }
      if (r > 0) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
          if (16 * k2 < r) {
            H8 a0, b0;
            a0.u = *reinterpret_cast<const uint4*>(&Ct[arow * CLD + 16 * k2 + 8 * hf]);
            b0.u = *reinterpret_cast<const uint4*>(&Ct[(arow + 32) * CLD + 16 * k2 + 8 * hf]);
            acc[0] = mfma16(a0, Bv[k2], acc[0]);
            acc[1] = mfma16(b0, Bv[k2], acc[1]);
          }
        }
      }
      // ---- r_x = S - x_hat into the pair's buffer, hi + lo ----
      uint16_t* eh = Eh[eb];
      uint16_t* el = El[eb];
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = 32 * h2 + 8 * (v >> 2) + 4 * hf + (v & 3);
          const float e = half_bits_to_float(sv[h2][v]) - acc[h2][v];
          uint16_t hi, lo;
          split_half(e, hi, lo);
          eh[row * ZLD + jcol] = hi;
          el[row * ZLD + jcol] = lo;
        }
      __syncthreads();  // the pair is complete; the other buffer was last read before the previous barrier
      // ---- norms: 4 lanes per token, 32 columns each ----
      {
        const int row = tid >> 2, seg = tid & 3;
        float ss = 0.0f;
#pragma unroll
        for (int h4 = 0; h4 < 4; ++h4) {
          H8 a, b;
          a.u = *reinterpret_cast<const uint4*>(&eh[row * ZLD + 32 * seg + 8 * h4]);
          b.u = *reinterpret_cast<const uint4*>(&el[row * ZLD + 32 * seg + 8 * h4]);
#pragma unroll
          for (int x = 0; x < 8; ++x) {
            const float e = half_bits_to_float(a.s[x]) + half_bits_to_float(b.s[x]);
            ss = fmaf(e, e, ss);
          }
        }
        ss += dpp_mov<0xB1>(ss);
        ss += dpp_mov<0x4E>(ss);
        if (seg == 0) qnorms[blk * (size_t)n + t0 + 32 * tau + row] = float_to_half_bits(sqrtf(ss));
      }
      // ---- Phi r_x for outputs i = 32 wave + l32 of both tiles, signs only ----
      float16v pr[2];
#pragma unroll
      for (int v = 0; v < 16; ++v) pr[0][v] = pr[1][v] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        H8 a0, a1, b0, b1;
        a0.u = *reinterpret_cast<const uint4*>(&eh[l32 * ZLD + 16 * kk + 8 * hf]);
        b0.u = *reinterpret_cast<const uint4*>(&eh[(l32 + 32) * ZLD + 16 * kk + 8 * hf]);
        a1.u = *reinterpret_cast<const uint4*>(&el[l32 * ZLD + 16 * kk + 8 * hf]);
        b1.u = *reinterpret_cast<const uint4*>(&el[(l32 + 32) * ZLD + 16 * kk + 8 * hf]);
        pr[0] = mfma16(a0, Fhi[kk], pr[0]);
        pr[1] = mfma16(b0, Fhi[kk], pr[1]);
        pr[0] = mfma16(a1, Fhi[kk], pr[0]);
        pr[1] = mfma16(b1, Fhi[kk], pr[1]);
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        uint32_t outw = 0u;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const unsigned long long m = __ballot(pr[h2][v] >= 0.0f);
          const int row_lo = 8 * (v >> 2) + (v & 3);   // token of the low word; the high word is row_lo + 4
          outw = (lane == row_lo) ? (uint32_t)m : ((lane == row_lo + 4) ? (uint32_t)(m >> 32) : outw);
        }
        if (lane < 32)
          *reinterpret_cast<uint32_t*>(qsigns + (blk * (size_t)n + t0 + 32 * (tau + h2) + lane) * (D / 8) + 4 * wave) = outw;
      }
      eb ^= 1;
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int v = 0; v < 16; ++v) sv[h2][v] = svn[h2][v];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// encode (binary16 blocks): one workgroup per block, 128 tokens per pass.
//   phase 1 (wave w, its own 32 tokens, v_mfma_f32_32x32x8_f16 so that every result feeds the next product
//            without leaving the registers):
//     C^T = W S^T          W = V diag(phi/sigma) as hi + lo binary16, S from the LDS tile
//     R^T = S^T - V16 C16^T  accumulator preloaded with S (the registers that were the B operand above)
//     rho_t = |R_t|, u = R sqrt(d)/rho as binary16 into the LDS tile (in place of S)
//   phase 2 (wave w = coordinates 32w .. 32w+31, rotation stationary in registers):
//     z = u Pi^T with Pi as hi + lo, Lloyd-Max index by binary search on the boundaries; the comparison
//     masks are the packed bit-planes (32 coordinates of two tokens per compare).
// ---------------------------------------------------------------------------------------------
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
union H4 {
  half4v h;
  uint2 u;
  uint16_t s[4];
};
__device__ __forceinline__ float16v mfma8(const H4& a, const H4& b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x8f16(a.h, b.h, c, 0, 0, 0);
}
constexpr int VLD = EOQ_RMAX_CAP + 8;  // row stride (halfs) of V^T in LDS

// FQ: the factors are already stored (4-bit codes expanded into lfac / rfac): the coefficients are read, not
// projected, and the residual is taken against them.
template <int BITS, bool FQ>
__global__ __launch_bounds__(THREADS, 2) void eoq_encode_mfma_kernel(
    const uint16_t* __restrict__ blocks, EoqBlockMap map, int n, int r_max, const uint16_t* __restrict__ pih,
    const float* __restrict__ tab, const float* __restrict__ wfac, const int32_t* __restrict__ rank_in,
    const uint16_t* __restrict__ rfac, uint16_t* lfac, uint16_t* __restrict__ norms,
    uint8_t* __restrict__ codes) {
  __shared__ __align__(16) uint16_t X[CHUNK * ZLD];                 // S tiles, then u tiles: [token][j]
  __shared__ __align__(16) uint16_t Wh[EOQ_RMAX_CAP * ZLD];         // W hi  [component][j]
  __shared__ __align__(16) uint16_t Wl[EOQ_RMAX_CAP * ZLD];         // W lo
  __shared__ __align__(16) uint16_t VT[D * VLD];                    // V16^T [j][component]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, hf = lane >> 5;
  const size_t blk = blockIdx.x;
  const size_t slot = map.slot(blk);
  const int r = rank_in[slot];
  constexpr int ROWB = BITS * D / 8;
  set_fp16_overflow_clamp();   // the stored coefficients saturate at the largest binary16 by the conversion itself
  // the 32 rows x 256 B of this wave's tokens, 16 B per lane and load (4 rows per instruction), are requested one
  // chunk ahead: the first chunk's here, before the tables
  const size_t tok = (size_t)map.token_stride;
  const uint16_t* src0 = blocks + map.in_base(blk) + (size_t)(32 * wave) * tok;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 pre[8];
  EOQ_SFOR(it, 8, pre[it] = *reinterpret_cast<const u32x4*>(src0 + (4 * it + (lane >> 4)) * tok + (lane & 15) * 8););

  // stationary rotation operand: rows c = 32w + l32 of Pi.  Up to 3 bits the binary16 rounding of Pi alone (one
  // matrix-core pass): it moves z sqrt(d) by a sum of 128 independent roundings, standard deviation 1.4e-4, the size of
  // what the binary16 rounding of u moves it by already; a coordinate that close to a cell boundary is reconstructed
  // equally well from either cell.  At 4 bits, where the cells are narrowest, the part that rounding lost goes through
  // a second pass.
  constexpr bool ROT_LO = BITS == 4;
  H8 Bhi[8], Blo[ROT_LO ? 8 : 1];
  {
    const int c = 32 * wave + l32;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Bhi[kk].u = *reinterpret_cast<const uint4*>(pih + c * D + 16 * kk + 8 * hf);
      if constexpr (ROT_LO) Blo[kk].u = *reinterpret_cast<const uint4*>(pih + D * D + c * D + 16 * kk + 8 * hf);
    }
  }
  // the decision boundaries as separate values, not an array or a vector: the compiler turns a select between two
  // elements into an element at a selected index (scratch memory for an array, a chain of sixteen selects for a
  // register vector)
#define EOQ_BND(i) const float bnd##i = ((i) < (1 << BITS) - 1) ? tab[16 + (i)] : 0.0f
  EOQ_BND(0); EOQ_BND(1); EOQ_BND(2); EOQ_BND(3); EOQ_BND(4); EOQ_BND(5); EOQ_BND(6); EOQ_BND(7);
  EOQ_BND(8); EOQ_BND(9); EOQ_BND(10); EOQ_BND(11); EOQ_BND(12); EOQ_BND(13); EOQ_BND(14);
#undef EOQ_BND

  // factors of the block: W = V diag(phi/sigma) split into hi + lo, and V16^T.  Only the rows below the rank
  // rounded up to a multiple of 8 are ever multiplied with something that is not forced to zero (see Cneg)
  const int r_up = (r + 7) & ~7;
  // thread (i0, j) = (tid / 128, tid % 128) takes the rows i0, i0 + 2, ...; four rows per round, their loads
  // issued together (rows at and above the rank read row r - 1 instead and store zeros)
  for (int i4 = 0; i4 < r_up; i4 += 8) {
    const int j = tid & (D - 1);
    float wv[4];
    uint16_t vv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ic = min(i4 + 2 * u + (tid >> 7), r - 1);
      if constexpr (!FQ) wv[u] = wfac[(blk * r_max + ic) * D + j];
      vv[u] = rfac[(slot * r_max + ic) * D + j];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = i4 + 2 * u + (tid >> 7);
      const bool live = i < r;
      if constexpr (!FQ) {
        uint16_t hi, lo;
        split_half(wv[u], hi, lo);
        Wh[i * ZLD + j] = live ? hi : (uint16_t)0;
        Wl[i * ZLD + j] = live ? lo : (uint16_t)0;
      }
      VT[j * VLD + i] = live ? vv[u] : (uint16_t)0;
    }
  }
  const float sqrt_d = sqrtf((float)D);
  const __amdgpu_buffer_rsrc_t lbuf = buffer_of(lfac + slot * r_max * (size_t)n, (size_t)r * n * 2);
  const __amdgpu_buffer_rsrc_t cbuf = buffer_of(codes + slot * (size_t)n * ROWB, (size_t)n * ROWB);

  for (int t0 = 0; t0 < n; t0 += CHUNK) {
    __syncthreads();  // previous chunk's tiles consumed (and the factor tables written)
    // ---- phase 1 ----
    {
      uint16_t* tile = X + 32 * wave * ZLD;
      EOQ_SFOR(it, 8, *reinterpret_cast<u32x4*>(tile + (4 * it + (lane >> 4)) * ZLD + (lane & 15) * 8) = pre[it];);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the tile is private to this wave, wait for its own LDS writes
      __builtin_amdgcn_wave_barrier();
      H4 Sreg[16];
#pragma unroll
      for (int kk = 0; kk < 16; ++kk) Sreg[kk].u = *reinterpret_cast<const uint2*>(tile + l32 * ZLD + 8 * kk + 4 * hf);
      float16v Racc[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) Racc[mt][v] = (float)Sreg[4 * mt + (v >> 2)].h[v & 3];
      if (r > 0) {
        H4 Cneg[4];
        // coefficient (i, token) of the block through a buffer descriptor that ends after row r - 1: the lane's part
        // of the offset in a register, the rest wave-uniform; loads from rows at and above the rank return zero and
        // stores to them are dropped
        const int cf_lane = (4 * hf * n + t0 + 32 * wave + l32) * 2;
        if constexpr (FQ) {
          // the stored coefficients of this token, negated: the next B operand
          EOQ_SFOR(v, 16,
            const int i = 8 * (v >> 2) + 4 * hf + (v & 3);
            const uint16_t c = __builtin_amdgcn_raw_buffer_load_b16(lbuf, cf_lane, (8 * (v >> 2) + (v & 3)) * n * 2, 0);
            Cneg[v >> 2].s[v & 3] = (i < r) ? (uint16_t)(c ^ 0x8000u) : (uint16_t)0;
          );
        } else {
          float16v Cacc;
#pragma unroll
          for (int v = 0; v < 16; ++v) Cacc[v] = 0.0f;
#pragma unroll
          for (int kk = 0; kk < 16; ++kk) {
            H4 ah, al;
            ah.u = *reinterpret_cast<const uint2*>(Wh + l32 * ZLD + 8 * kk + 4 * hf);
            al.u = *reinterpret_cast<const uint2*>(Wl + l32 * ZLD + 8 * kk + 4 * hf);
            Cacc = mfma8(ah, Sreg[kk], Cacc);
            Cacc = mfma8(al, Sreg[kk], Cacc);
          }
          // stored coefficients C16 = binary16(U diag(phi)); their negatives are the next B operand
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int i = 8 * (v >> 2) + 4 * hf + (v & 3);
            const uint16_t hb = float_to_half_bits_clamped_by_mode(Cacc[v]);
            __builtin_amdgcn_raw_buffer_store_b16(hb, lbuf, cf_lane, (8 * (v >> 2) + (v & 3)) * n * 2, 0);
            Cneg[v >> 2].s[v & 3] = (i < r) ? (uint16_t)(hb ^ 0x8000u) : (uint16_t)0;  // rows >= r of W are not initialised
          }
        }
#pragma unroll
        for (int k2 = 0; k2 < 4; ++k2) {
          if (8 * k2 < r) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
              H4 a;
              a.u = *reinterpret_cast<const uint2*>(VT + (32 * mt + l32) * VLD + 8 * k2 + 4 * hf);
              Racc[mt] = mfma8(a, Cneg[k2], Racc[mt]);
            }
          }
        }
      }
      // rho_t and u = sqrt(d) R_t / rho_t (Alg. 1 line 3); this lane holds 64 of the 128 entries of token l32
      float ss = 0.0f;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) ss = fmaf(Racc[mt][v], Racc[mt][v], ss);
      ss += __shfl_xor(ss, 32, 64);
      const float rho = sqrtf(ss);
      if (hf == 0) norms[slot * (size_t)n + t0 + 32 * wave + l32] = float_to_half_bits(rho);
      const float sc = (rho > 0.0f) ? sqrt_d / rho : 0.0f;
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          // |u_j| <= sqrt(d): no saturation to think of; two entries per conversion
          const uint2 u = make_uint2(pack_half2(Racc[mt][4 * q] * sc, Racc[mt][4 * q + 1] * sc),
                                     pack_half2(Racc[mt][4 * q + 2] * sc, Racc[mt][4 * q + 3] * sc));
          *reinterpret_cast<uint2*>(tile + l32 * ZLD + 32 * mt + 8 * q + 4 * hf) = u;
        }
    }
    // the next chunk's rows travel while this one is rotated and quantised (requested here and not earlier: phase 1
    // has no registers to spare)
    __builtin_amdgcn_sched_barrier(0);
    if (t0 + CHUNK < n) {
      const uint16_t* src = src0 + (size_t)(t0 + CHUNK) * tok;
      EOQ_SFOR(it, 8, pre[it] = *reinterpret_cast<const u32x4*>(src + (4 * it + (lane >> 4)) * tok + (lane & 15) * 8););
    }
    __syncthreads();
    // ---- phase 2 ---- (unrolled: a loop with stores in it would make the compiler wait for the rows requested above
    // before entering it)
#pragma unroll
    for (int tau = 0; tau < CHUNK / 32; ++tau) {
      float16v acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        H8 a;
        a.u = *reinterpret_cast<const uint4*>(X + (32 * tau + l32) * ZLD + 16 * kk + 8 * hf);
        acc = mfma16(a, Bhi[kk], acc);
        if constexpr (ROT_LO) acc = mfma16(a, Blo[kk], acc);
      }
      // index = number of boundaries <= z, found from the top bit down; every comparison mask holds one
      // bit-plane of coordinates 32w..32w+31 for the tokens 8q+e (low word) and 8q+4+e (high word)
      uint32_t outw[BITS];
#pragma unroll
      for (int p = 0; p < BITS; ++p) outw[p] = 0u;
      EOQ_SFOR(v, 16,
        const float z = acc[v];
        unsigned long long m[BITS];
        if constexpr (BITS == 1) {
          m[0] = __ballot(z >= bnd0);
        } else if constexpr (BITS == 2) {
          const bool b1 = z >= bnd1;
          m[1] = __ballot(b1);
          m[0] = __ballot(z >= (b1 ? bnd2 : bnd0));
        } else if constexpr (BITS == 3) {
          // the candidates of the later levels are selected by the earlier decisions as soon as those are known, so
          // the last comparison waits for one select only
          const bool b2 = z >= bnd3;
          m[2] = __ballot(b2);
          const float lo0 = b2 ? bnd4 : bnd0, lo1 = b2 ? bnd6 : bnd2;
          const bool b1 = z >= (b2 ? bnd5 : bnd1);
          m[1] = __ballot(b1);
          m[0] = __ballot(z >= (b1 ? lo1 : lo0));
        } else {
          const bool b3 = z >= bnd7;
          m[3] = __ballot(b3);
          const float q0 = b3 ? bnd8 : bnd0, q1 = b3 ? bnd10 : bnd2, q2 = b3 ? bnd12 : bnd4, q3 = b3 ? bnd14 : bnd6;
          const float h0 = b3 ? bnd9 : bnd1, h1 = b3 ? bnd13 : bnd5;
          const bool b2 = z >= (b3 ? bnd11 : bnd3);
          m[2] = __ballot(b2);
          const float lo0 = b2 ? q2 : q0, lo1 = b2 ? q3 : q1;
          const bool b1 = z >= (b2 ? h1 : h0);
          m[1] = __ballot(b1);
          m[0] = __ballot(z >= (b1 ? lo1 : lo0));
        }
        constexpr int row_lo = 8 * (v >> 2) + (v & 3);   // token of the low word; the high word is row_lo + 4
        EOQ_SFOR(p, BITS,
          outw[p] = write_lane<row_lo>(outw[p], (uint32_t)m[p]);
          outw[p] = write_lane<row_lo + 4>(outw[p], (uint32_t)(m[p] >> 32));
        );
      );
      // lane t < 32 stores the words of token t; the other lanes aim past the end of the descriptor and are dropped
      // (no branch: after a branch around the stores the compiler could not count them when it waits for the rows
      // requested above, and would wait for everything)
      {
        const int off = (lane < 32) ? (t0 + 32 * tau + lane) * ROWB + 4 * wave : 0x7FFFFFF0;
#pragma unroll
        for (int p = 0; p < BITS; ++p) __builtin_amdgcn_raw_buffer_store_b32(outw[p], cbuf, off, p * 16, 0);
      }
      __builtin_amdgcn_sched_barrier(0);   // one tile at a time: keeps the registers of the rows in flight free
    }
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
hipError_t eoq_launch_decode(const EoqLaunch& L, eoq_packed in, int64_t B, void* out_fp16) {
  if (L.ev) (void)hipEventRecord(L.ev[4], L.stream);
  if (B <= 0) {
    if (L.ev) (void)hipEventRecord(L.ev[5], L.stream);
    return hipGetLastError();
  }
  // Every wave is a worker; two workgroups of four per compute unit (2048 waves).  A unit of work is a whole block
  // when that leaves every wave at least two of them, otherwise a half or a quarter of a block's 32-token tiles.
  const int tiles = L.n / 32;
  int parts_log2 = 0;
  while (parts_log2 < 2 && (B << parts_log2) < 4096 && tiles % (2 << parts_log2) == 0) ++parts_log2;
  const int64_t units = B << parts_log2;
  const dim3 grid((unsigned)(units < 2048 ? (units + 3) / 4 : 512)), block(THREADS);
  uint16_t* out = static_cast<uint16_t*>(out_fp16);
#define EOQ_DECODE(BITS)                                                                                             \
  hipLaunchKernelGGL(eoq_decode_mfma_kernel<BITS>, grid, block, 0, L.stream, L.n, L.r_max, B, parts_log2, L.pih, L.tab,   \
                     in.codes, in.norms, in.rank, in.lfac, in.rfac, out)
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

hipError_t eoq_launch_qjl(const EoqLaunch& L, const void* blocks_fp16, int64_t B, eoq_packed rec, eoq_qjl out) {
  const dim3 grid((unsigned)B), block(THREADS);
  const uint16_t* src = static_cast<const uint16_t*>(blocks_fp16);
#define EOQ_QJL(BITS)                                                                                              \
  hipLaunchKernelGGL(eoq_qjl_kernel<BITS>, grid, block, 0, L.stream, src, L.n, L.r_max, L.pih, L.phih, L.tab,      \
                     rec.codes, rec.norms, rec.rank, rec.lfac, rec.rfac, out.signs, out.norms)
  switch (L.bits) {
    case 1: EOQ_QJL(1); break;
    case 2: EOQ_QJL(2); break;
    case 3: EOQ_QJL(3); break;
    default: EOQ_QJL(4); break;
  }
#undef EOQ_QJL
  return hipGetLastError();
}

hipError_t eoq_launch_encode_f16(const EoqLaunch& L, const void* blocks, int64_t B, const float* wfac,
                                 eoq_packed out, bool stored_factors) {
  const dim3 grid((unsigned)B), block(THREADS);
  const uint16_t* src = static_cast<const uint16_t*>(blocks);
#define EOQ_ENCODE(BITS)                                                                                            \
  do {                                                                                                              \
    if (stored_factors)                                                                                             \
      hipLaunchKernelGGL((eoq_encode_mfma_kernel<BITS, true>), grid, block, 0, L.stream, src, L.map, L.n, L.r_max,  \
                         L.pih, L.tab, wfac, out.rank, out.rfac, out.lfac, out.norms, out.codes);                   \
    else                                                                                                            \
      hipLaunchKernelGGL((eoq_encode_mfma_kernel<BITS, false>), grid, block, 0, L.stream, src, L.map, L.n, L.r_max, \
                         L.pih, L.tab, wfac, out.rank, out.rfac, out.lfac, out.norms, out.codes);                   \
  } while (0)
  switch (L.bits) {
    case 1: EOQ_ENCODE(1); break;
    case 2: EOQ_ENCODE(2); break;
    case 3: EOQ_ENCODE(3); break;
    default: EOQ_ENCODE(4); break;
  }
#undef EOQ_ENCODE
  return hipGetLastError();
}
