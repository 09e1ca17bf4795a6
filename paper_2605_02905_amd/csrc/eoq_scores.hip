// Decode scoring on compressed keys (Sec. 2.1 attention logits, Remark 6.5): scores[s][h][t] = <q_h, x_hat_t>/sqrt(d)
// from the record, without forming x_hat.  With x_hat_t = rho_t Pi^T z_hat_t + C_t V_r:
//     <q, x_hat_t> = rho_t <Pi q, z_hat_t> + <C_t, V_r^T q>.
//
// The first term runs on the integer matrix cores.  The codebook is symmetric, so a centroid is its sign times a
// magnitude that is a multilinear function of the magnitude bits m_p (index bit p of the code, inverted on the negative
// half):  z_hat_j = s_j sum_M coef[M] prod_{p in M} m_pj over the subsets M of the b-1 magnitude bits (b = 2: c_0 + (c_1 -
// c_0) m_0).  Every term is an inner product of q' = Pi q with a vector of entries in {-1, 0, +1}: exact in int8.  q' is
// held in 32-bit fixed point per head (a power-of-two unit, four balanced signed bytes), so the rows of the A operand of
// v_mfma_i32_16x16x64_i8 are the four byte planes of four query heads and all sixteen rows do work; the columns are sixteen
// tokens, the int32 sums are exact, and the four planes of a head meet again in float32 through two lane swaps.
// Operand convention of v_mfma_i32_16x16x64_i8 (wave64): lane l supplies A[row = l%16][k = 16*(l/16) .. +15] and
// B[k = 16*(l/16) .. +15][col = l%16] and receives D[row = 4*(l/16) + v][col = l%16] in accumulator register v.
// The {-1, 0, +1} operands come out of a 256-entry LDS table indexed by one nibble of the sign plane and one nibble of a
// magnitude plane: four coordinates of two operand kinds per 8-byte read, no select logic.
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int SC_MAXG = 8;      // most query heads per KV head
constexpr int SC_DEPTH = 2;     // passes of record bytes in flight per wave
constexpr int SC_RUN_MAX = 16;  // most blocks per workgroup (the run is shortened until the grid fills the chip)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
union H8 {
  half8 h;
  uint4 u;
  uint16_t s[8];
};

// Buffer descriptor over `bytes` bytes at `base` (raw addressing: loads past the end return zero).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, size_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(bytes > 0x7FFFFFFFu ? 0x7FFFFFFFu : bytes),
                                           0x00020000);
}
__device__ __forceinline__ float4v mfma32(const H8& a, const H8& b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, c, 0, 0, 0);
}
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (mask & a) | (~mask & b); }

// out[h][c] = sum_j table[c][j] q[h][j] for the heads of one group (rows above the group are zero), the table given as
// binary16 hi + lo parts [c][j]: the query side of the rotation (<q, Pi^T z> = <Pi q, z>) and of the projection Phi q.
// q is binary16, so every product is exact; v_mfma_f32_16x16x32_f16, 16 matrix instructions and 20 sixteen-byte loads
// per wave, all in flight together.  `out` is LDS, [SC_MAXG][D]; the caller synchronises.
__device__ __forceinline__ void rotate_query(const uint16_t* __restrict__ tab_hi, const uint16_t* __restrict__ tab_lo,
                                             const uint16_t* __restrict__ qg, int group, float* out, int wave, int l16,
                                             int g) {
  H8 a[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    a[ks].u = (l16 < group) ? *reinterpret_cast<const uint4*>(qg + l16 * D + 32 * ks + 8 * g) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int c = 16 * (2 * wave + tt) + l16;
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      H8 bh, bl;
      bh.u = *reinterpret_cast<const uint4*>(tab_hi + c * D + 32 * ks + 8 * g);
      acc = mfma32(a[ks], bh, acc);
      if (tab_lo) {   // uniform: a table that is binary16 to begin with has no low part
        bl.u = *reinterpret_cast<const uint4*>(tab_lo + c * D + 32 * ks + 8 * g);
        acc = mfma32(a[ks], bl, acc);
      }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (4 * g + v < SC_MAXG) out[(4 * g + v) * D + c] = acc[v];
  }
}

// Rows of `rows` ([SC_MAXG][D] float, LDS) to 32-bit fixed point: per row the unit is 2^(E - 29) with E the exponent
// of the row's largest magnitude, so |integer| <= 2^30; the integer is cut into four balanced signed bytes (the bytes of
// I + 0x80808080 with the top bit of each flipped) and byte plane p of row h goes to dig[(4 h + p) * D + coordinate].
// unit[h] = value of one integer unit (0 for a row that is zero, below 2^-87 or not finite).  All 256 lanes; barriers
// inside, the last one after the planes are written.
__device__ __forceinline__ void fixed_point_rows(const float* rows, unsigned char* dig, unsigned* max_s, float* unit, int tid) {
  if (tid < SC_MAXG) max_s[tid] = 0u;
  __syncthreads();
  const int h = tid >> 5, c0 = 4 * (tid & 31);
  float v[4];
  unsigned m = 0u;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[e] = rows[h * D + c0 + e];
    m = max(m, (unsigned)__float_as_uint(fabsf(v[e])));
  }
  atomicMax(&max_s[h], m);
  __syncthreads();
  const int eb = (int)(max_s[h] >> 23);   // biased exponent of the row maximum
  const bool live = eb >= 40 && eb < 255;
  const float up = live ? __uint_as_float((unsigned)(283 - eb) << 23) : 0.0f;   // 2^(29 - (eb - 127))
  uint32_t dg[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int I = live ? __float2int_rn(v[e] * up) : 0;
    dg[e] = ((uint32_t)I + 0x80808080u) ^ 0x80808080u;
  }
  uint32_t pl[4];
  transpose_bytes(dg[0], dg[1], dg[2], dg[3], pl);
#pragma unroll
  for (int p = 0; p < 4; ++p) *reinterpret_cast<uint32_t*>(dig + (4 * h + p) * D + c0) = pl[p];
  if ((tid & 31) == 0) unit[h] = live ? __uint_as_float((unsigned)(eb - 29) << 23) : 0.0f;
  __syncthreads();
}

// The {-1, 0, +1} operands of one token for this lane's 32 coordinates (bits 0..31 of the lane's word of every bit
// plane), as B operands of two matrix instructions (coordinates 0..15 and 16..31 of the word): B[slice][M] for the subset
// M of the magnitude bits; M = 0 is the sign alone.  Nibble k of the words (coordinates 4k .. 4k+3) is one table read:
// entry (sign nibble | magnitude nibble << 4) = (four sign bytes, the same bytes where the magnitude bit is set).
template <int BITS>
__device__ __forceinline__ void sign_operands(const uint32_t (&word)[BITS], const uint2* nib_tab, v4i (&B)[2][1 << (BITS - 1)]) {
  const uint32_t top = word[BITS - 1];
#pragma unroll
  for (int p = 0; p < (BITS > 1 ? BITS - 1 : 1); ++p) {
    // magnitude bit p of a code is plane p where the sign plane is set and its complement where it is clear
    const uint32_t x = (BITS > 1) ? ~(word[BITS > 1 ? p : 0] ^ top) : 0u;
    const uint32_t even = bfi(0x0F0F0F0Fu, top, x << 4);   // byte j: nibbles 2j of (top, x)
    const uint32_t odd = bfi(0x0F0F0F0Fu, top >> 4, x);    // byte j: nibbles 2j + 1
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t idx = (((k & 1) ? odd : even) >> (8 * (k >> 1))) & 0xFFu;
      if (p == 0) {
        const uint2 e = nib_tab[idx];
        B[k >> 2][0][k & 3] = (int)e.x;
        if constexpr (BITS > 1) B[k >> 2][1][k & 3] = (int)e.y;
      } else {
        B[k >> 2][1 << p][k & 3] = (int)nib_tab[idx].y;
      }
    }
  }
  // products of several magnitude bits: bytes are 0 or the sign byte, so the product is the bitwise AND
#pragma unroll
  for (int M = 3; M < (1 << (BITS - 1)); ++M) {
    if ((M & (M - 1)) != 0) {
      const int low = M & -M;
#pragma unroll
      for (int s = 0; s < 2; ++s) B[s][M] = B[s][low] & B[s][M ^ low];
    }
  }
}

// Sum of the four lanes l%16 + 16 g, g = 0..3, of value v[g'] for g' = 0..3, transposing: lane group g returns the total
// of v[g].  v_permlane32_swap exchanges the upper half of its first operand with the lower half of its second,
// v_permlane16_swap the odd 16-lane rows of the first with the even rows of the second.
__device__ __forceinline__ float fold_planes(float v0, float v1, float v2, float v3) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const u2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v0), __float_as_uint(v2), false, false);
  const u2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v1), __float_as_uint(v3), false, false);
  const float ra = __uint_as_float(a[0]) + __uint_as_float(a[1]);   // lower half: value 0, upper half: value 2
  const float rb = __uint_as_float(b[0]) + __uint_as_float(b[1]);   // lower half: value 1, upper half: value 3
  const u2 c = __builtin_amdgcn_permlane16_swap(__float_as_uint(ra), __float_as_uint(rb), false, false);
  return __uint_as_float(c[0]) + __uint_as_float(c[1]);
}

// What a lane requests of one pass (32 consecutive tokens per wave): lane (l16, g) works on tokens 2 l16 and 2 l16 + 1
// of the pass: word g of every bit plane of both, their two stored norms as one word (with QJL also the sign words and
// the residual norms).
template <int BITS, bool QJL>
struct ScoreFetch {
  uint32_t word[2][BITS];
  uint32_t rho2;
  uint32_t sword[2];
  uint32_t gam2;
};
// Buffer addressing: a resource descriptor in scalar registers (base of this workgroup's run of blocks, size of the
// run: reads past it return zero instead of faulting), a scalar byte offset that moves from pass to pass and a per-lane
// 32-bit offset that never changes -- no vector arithmetic per load.
struct ScoreBuffers {
  __amdgpu_buffer_rsrc_t codes, norms, lfac, qsigns, qnorms;
};
// `tokb` (first token of the pass, counted from the start of the run) is wave-uniform.
template <int BITS, bool QJL>
__device__ __forceinline__ void score_fetch(ScoreFetch<BITS, QJL>& f, const ScoreBuffers& sb, int tokb, uint32_t lane_c,
                                            uint32_t lane_s, uint32_t lane_n) {
  constexpr int ROWB = BITS * D / 8;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int p = 0; p < BITS; ++p)
      f.word[u][p] = __builtin_amdgcn_raw_buffer_load_b32(sb.codes, lane_c + u * ROWB + p * 16, tokb * ROWB, 0);
    if constexpr (QJL) f.sword[u] = __builtin_amdgcn_raw_buffer_load_b32(sb.qsigns, lane_s + u * (D / 8), tokb * (D / 8), 0);
  }
  f.rho2 = __builtin_amdgcn_raw_buffer_load_b32(sb.norms, lane_n, tokb * 2, 0);
  if constexpr (QJL) f.gam2 = __builtin_amdgcn_raw_buffer_load_b32(sb.qnorms, lane_n, tokb * 2, 0);
}

// One workgroup per (sequence, KV head, run of blocks).  NSETS = sets of four query heads (1 for groups up to 4).
// QJL: the logits get the correction of Eq. (qjl), |r_x| sqrt(pi/2)/d <Phi q, sign(Phi r_x)>, from one more bit plane
// (the signs) and the stored residual norm; Phi q goes through the same fixed-point form as Pi q.
template <int BITS, bool QJL, int NSETS>
__global__ __launch_bounds__(THREADS) void eoq_scores_i8_kernel(
    int n, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, int64_t block_capacity, int64_t score_stride,
    int run, const uint16_t* __restrict__ pih,
    const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const uint16_t* __restrict__ q, float* __restrict__ scores, const uint16_t* __restrict__ phih,
    const uint8_t* __restrict__ qsigns, const uint16_t* __restrict__ qnorms) {
  constexpr int TYPES = 1 << (BITS - 1);
  __shared__ float qraw[SC_MAXG * D];
  __shared__ float qrot[SC_MAXG * D];
  __shared__ __align__(16) float wbuf[SC_RUN_MAX * EOQ_RMAX_CAP * SC_MAXG];   // [block of the run][component][head]: <v_i, q_h>/sqrt(d)
  __shared__ int rank_s[SC_RUN_MAX];
  __shared__ __align__(16) uint2 nib_tab[256];
  __shared__ __align__(16) unsigned char qdig[SC_MAXG * 4 * D];               // byte planes of Pi q, [head][plane][coordinate]
  __shared__ __align__(16) unsigned char pdig[QJL ? SC_MAXG * 4 * D : 16];    // byte planes of Phi q
  __shared__ unsigned max_s[SC_MAXG];
  __shared__ float qunit[SC_MAXG], punit[SC_MAXG];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave: scalar
  const int l16 = lane & 15, g = lane >> 4;
  const size_t sg = blockIdx.y;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  const size_t q0 = (sq * n_q_heads + kv * group) * D;
  const size_t T = (size_t)score_stride;   // entries per score row (>= blocks_per_head * n)
  constexpr int ROWB = BITS * D / 8;
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);

  {
    const int tn = tid & 15, xn = tid >> 4;
    uint32_t sd = 0u, td = 0u;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t sb = ((tn >> e) & 1) ? 0x01u : 0xFFu;   // sign plane bit set: +1
      sd |= sb << (8 * e);
      if ((xn >> e) & 1) td |= sb << (8 * e);
    }
    nib_tab[tid] = make_uint2(sd, td);
  }
  for (int e = tid; e < SC_MAXG * D; e += THREADS) qraw[e] = (e < group * D) ? half_bits_to_float(q[q0 + e]) : 0.0f;
  __syncthreads();
  // q' = Pi q (the rotation moved to the query side: <q, Pi^T z> = <Pi q, z>), then its fixed-point byte planes
  rotate_query(pih, pih + D * D, q + q0, group, qrot, wave, l16, g);
  __syncthreads();
  fixed_point_rows(qrot, qdig, max_s, qunit, tid);
  if constexpr (QJL) {
    rotate_query(phih, nullptr, q + q0, group, qrot, wave, l16, g);
    __syncthreads();
    fixed_point_rows(qrot, pdig, max_s, punit, tid);
  }
  // A operands: row l16 = byte plane l16 / 4 of head 4 hs + l16 % 4; slice s covers the coordinates 32 g + 16 s .. + 15.
  // K[hs][v]: what one unit of accumulator register v (head 4 hs + v, plane g) is worth in the logit.
  v4i Aq[NSETS][2], Ap[QJL ? NSETS : 1][2];
  float Kq[NSETS][4], Kp[QJL ? NSETS : 1][4];
  const float qjl_scale = sqrtf(1.5707963267948966f) / (float)D;
  const float plane_w = (float)(1u << (8 * g));
#pragma unroll
  for (int hs = 0; hs < NSETS; ++hs) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int off = (4 * (4 * hs + (l16 & 3)) + (l16 >> 2)) * D + 32 * g + 16 * s;
      Aq[hs][s] = *reinterpret_cast<const v4i*>(qdig + off);
      if constexpr (QJL) Ap[hs][s] = *reinterpret_cast<const v4i*>(pdig + off);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      Kq[hs][v] = qunit[4 * hs + v] * plane_w * (1.0f / (float)D);   // z_hat = centroid / sqrt(d), logit = <q, x_hat> / sqrt(d)
      if constexpr (QJL) Kp[hs][v] = punit[4 * hs + v] * plane_w * (qjl_scale * inv_sqrt_d);
    }
  }
  // coefficients of the multilinear form of the magnitudes: level number sum_p m_p 2^p is centroid L/2 + level of the
  // ascending N(0,1) table; coef[M] = sum over subsets S of M of (-1)^(|M| - |S|) centroid[L/2 + S]
  float coef[TYPES];
#pragma unroll
  for (int M = 0; M < TYPES; ++M) {
    float c = 0.0f;
#pragma unroll
    for (int S = 0; S < TYPES; ++S)
      if ((S & M) == S) c += ((__builtin_popcount(M ^ S) & 1) ? -1.0f : 1.0f) * tab[TYPES + S];
    coef[M] = c;
  }

  // The work of this workgroup as a flat list of passes: pass p of a wave covers the 32 tokens from 32 (wave + 4 q) of
  // block jb0 + p / ppb, q = p % ppb.  The record bytes of a pass are requested SC_DEPTH passes ahead into a ring of
  // registers (the loop is unrolled over the ring, so nothing is copied and a pass only waits for its own bytes), the
  // stored coefficients one pass ahead.
  const int64_t jb0 = (int64_t)blockIdx.x * run;
  const int nblk = (int)(min(jb0 + run, blocks_per_head) - jb0);
  const int ppb = n / 128;
  const int P = nblk * ppb;
  const size_t blk0 = sg * (size_t)block_capacity + jb0;   // the store holds block_capacity slots per head

  // w[b][i][h] = <v_i, q_h>/sqrt(d) of every block of the run, up front (the low-rank term is <C_t, w_h>): all loads of
  // the set-up are in flight together and the pass loop below has no barrier.  16 lanes per (component, head): one
  // 16-byte load of eight entries of v_i each, then a sum over the DPP row.
  if (tid < nblk) rank_s[tid] = min(max(rank_in[blk0 + tid], 0), r_max);   // records may come from storage: never index past r_max rows
  __syncthreads();
  int rtop = 0;
  for (int b = 0; b < nblk; ++b) rtop = max(rtop, rank_s[b]);
  for (int e0 = 0; e0 < nblk * rtop * (SC_MAXG * 16); e0 += THREADS) {   // uniform trip count: whole rows reduce together
    const int e = e0 + tid;
    const int seg = e & 15, h = (e >> 4) & (SC_MAXG - 1);
    const int bi = e >> 7, b = bi / rtop, i = bi - b * rtop;
    const int rb = rank_s[min(b, nblk - 1)];
    float acc = 0.0f;
    if (b < nblk && i < rb) {
      float v[8];
      load8(rfac, EOQ_F16, ((blk0 + b) * r_max + i) * (size_t)D + 8 * seg, v);
#pragma unroll
      for (int x = 0; x < 8; ++x) acc = fmaf(v[x], qraw[h * D + 8 * seg + x], acc);
    }
    acc += dpp_mov<0xB1>(acc);
    acc += dpp_mov<0x4E>(acc);
    acc += dpp_mov<0x141>(acc);
    acc += dpp_mov<0x140>(acc);
    if (seg == 0 && b < nblk && i < rb) wbuf[(b * EOQ_RMAX_CAP + i) * SC_MAXG + h] = acc * inv_sqrt_d;
  }
  __syncthreads();

  const uint32_t lane_c = (uint32_t)(2 * l16 * ROWB + 4 * g);      // into the codes of a pass
  const uint32_t lane_s = (uint32_t)(2 * l16 * (D / 8) + 4 * g);   // into the sign planes of a pass
  const uint32_t lane_n = (uint32_t)(4 * l16);                     // into the norms / a coefficient row of a pass
  ScoreBuffers sb;
  sb.codes = buffer_of(codes + blk0 * (size_t)n * ROWB, (size_t)nblk * n * ROWB);
  sb.norms = buffer_of(norms + blk0 * (size_t)n, (size_t)nblk * n * 2);
  sb.lfac = buffer_of(lfac + blk0 * (size_t)r_max * n, (size_t)nblk * r_max * n * 2);
  if constexpr (QJL) {
    sb.qsigns = buffer_of(qsigns + blk0 * (size_t)n * (D / 8), (size_t)nblk * n * (D / 8));
    sb.qnorms = buffer_of(qnorms + blk0 * (size_t)n, (size_t)nblk * n * 2);
  }
  ScoreFetch<BITS, QJL> ring[SC_DEPTH];
  uint32_t cbr[2][4];      // [parity of the pass][component of the first four]: coefficients of the lane's two tokens
  int fb = 0, fq = 0;      // block and pass-in-block of the next pass to request
  auto request = [&](ScoreFetch<BITS, QJL>& f) __attribute__((always_inline)) {
    score_fetch<BITS, QJL>(f, sb, fb * n + 32 * (wave + 4 * fq), lane_c, lane_s, lane_n);
    if (++fq == ppb) {
      fq = 0;
      ++fb;
    }
  };
  // coefficients C[i][tokens] of the first four components of pass (cb_b, cb_q); row 0 is read when the rank is 0
  auto request_cb = [&](uint32_t (&cb)[4], int cb_b, int cb_q) __attribute__((always_inline)) {
    const int rr = __builtin_amdgcn_readfirstlane(max(rank_s[cb_b], 1));
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int row = (cb_b * r_max + min(a, rr - 1)) * n + 32 * (wave + 4 * cb_q);   // uniform, in entries
      cb[a] = __builtin_amdgcn_raw_buffer_load_b32(sb.lfac, lane_n, row * 2, 0);
    }
  };
  if (P > 0) request_cb(cbr[0], 0, 0);
#pragma unroll
  for (int dd = 0; dd < SC_DEPTH; ++dd)
    if (dd < P) request(ring[dd]);

  int cb_blk = 0, cq = 0;   // block and pass-in-block of the pass being worked on
  int r = 0;
  size_t blk = blk0;
  const float* wrow = wbuf;
  const bool even_stride = (T & 1) == 0;
  auto work = [&](ScoreFetch<BITS, QJL>& cur, uint32_t (&cb)[4], uint32_t (&cbn)[4], bool more) __attribute__((always_inline)) {
    if (cq == 0) {
      blk = blk0 + cb_blk;
      r = rank_s[cb_blk];
      wrow = wbuf + cb_blk * (EOQ_RMAX_CAP * SC_MAXG);
    }
    const int tok0 = 32 * (wave + 4 * cq);   // first token of the pass inside its block
    const int64_t jb = jb0 + cb_blk;
    // the coefficients of the next pass go out before this pass's matrix products
    {
      int nb = cb_blk, nq = cq + 1;
      if (nq == ppb) {
        nq = 0;
        ++nb;
      }
      if (more) request_cb(cbn, nb, nq);
    }
    float res[2][NSETS];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      v4i B[2][TYPES];
      sign_operands<BITS>(cur.word[u], nib_tab, B);
      const float rho = half_bits_to_float((uint16_t)(u ? (cur.rho2 >> 16) : (cur.rho2 & 0xFFFFu)));
#pragma unroll
      for (int hs = 0; hs < NSETS; ++hs) {
        v4i acc[TYPES];
#pragma unroll
        for (int M = 0; M < TYPES; ++M) {
          acc[M] = v4i{0, 0, 0, 0};
          acc[M] = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aq[hs][0], B[0][M], acc[M], 0, 0, 0);
          acc[M] = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aq[hs][1], B[1][M], acc[M], 0, 0, 0);
        }
        float val[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float s = coef[0] * (float)acc[0][v];
#pragma unroll
          for (int M = 1; M < TYPES; ++M) s = fmaf(coef[M], (float)acc[M][v], s);
          val[v] = s * Kq[hs][v];
        }
        res[u][hs] = fold_planes(val[0], val[1], val[2], val[3]) * rho;   // head 4 hs + g
      }
      if constexpr (QJL) {
        // sign(Phi r_x) is one more plane of +-1: the table's first entry kind with the magnitude nibble at zero
        const uint32_t sw = cur.sword[u];
        v4i Bs[2];
#pragma unroll
        for (int k = 0; k < 8; ++k) Bs[k >> 2][k & 3] = (int)nib_tab[(sw >> (4 * k)) & 0xFu].x;
        const float gam = half_bits_to_float((uint16_t)(u ? (cur.gam2 >> 16) : (cur.gam2 & 0xFFFFu)));
#pragma unroll
        for (int hs = 0; hs < NSETS; ++hs) {
          v4i acc = {0, 0, 0, 0};
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(Ap[hs][0], Bs[0], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(Ap[hs][1], Bs[1], acc, 0, 0, 0);
          const float t = fold_planes((float)acc[0] * Kp[hs][0], (float)acc[1] * Kp[hs][1], (float)acc[2] * Kp[hs][2],
                                      (float)acc[3] * Kp[hs][3]);
          res[u][hs] = fmaf(t, gam, res[u][hs]);
        }
      }
    }
    // low-rank term on the vector ALU: the lane has C[i][its two tokens] and reads w[i][head 4 hs + g]
    if (r > 0) {
      for (int i0 = 0; i0 < r; i0 += 4) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const int i = min(i0 + a, r - 1);
          const uint32_t cx = (i0 == 0) ? cb[a]
                                        : *reinterpret_cast<const uint32_t*>(lfac + (blk * r_max + i) * (size_t)n + tok0 + 2 * l16);
          const float c0 = half_bits_to_float((uint16_t)(cx & 0xFFFFu)), c1 = half_bits_to_float((uint16_t)(cx >> 16));
#pragma unroll
          for (int hs = 0; hs < NSETS; ++hs) {
            const float w = (i0 + a < r) ? wrow[i * SC_MAXG + 4 * hs + g] : 0.0f;
            res[0][hs] = fmaf(w, c0, res[0][hs]);
            res[1][hs] = fmaf(w, c1, res[1][hs]);
          }
        }
      }
    }
#pragma unroll
    for (int hs = 0; hs < NSETS; ++hs) {
      const int h = 4 * hs + g;
      if (h < group) {
        float* dst = scores + (sq * n_q_heads + kv * group + h) * T + (size_t)jb * n + tok0 + 2 * l16;
        if (even_stride) {
          *reinterpret_cast<float2*>(dst) = make_float2(res[0][hs], res[1][hs]);
        } else {
          dst[0] = res[0][hs];
          dst[1] = res[1][hs];
        }
      }
    }
    if (++cq == ppb) {
      cq = 0;
      ++cb_blk;
    }
  };

  // the ring has SC_DEPTH stages and the coefficient buffers two: the loop is unrolled over 2 passes
  static_assert(SC_DEPTH == 2, "the stages below are written out for a ring of two");
#define EOQ_SC_STAGE(dd)                                                                       \
  {                                                                                            \
    const int p = p0 + dd;                                                                     \
    if (p < P) {                                                                               \
      work(ring[dd % SC_DEPTH], cbr[dd & 1], cbr[(dd + 1) & 1], p + 1 < P);                    \
      if (p + SC_DEPTH < P) request(ring[dd % SC_DEPTH]);                                      \
    }                                                                                          \
  }
  for (int p0 = 0; p0 < P; p0 += SC_DEPTH) {
    EOQ_SC_STAGE(0)
    EOQ_SC_STAGE(1)
  }
#undef EOQ_SC_STAGE
}

// Scores of the uncompressed tail (the newest tokens of every head, binary16, not yet a full block):
// scores[s][h][offset + t] = <q[s][h], tail[s][g][t]> / sqrt(d).  One workgroup per (sequence, KV head); 16 lanes
// share a token (16 bytes each), float32 accumulation of exact binary16 products.
__global__ __launch_bounds__(THREADS) void eoq_scores_tail_kernel(
    int n_kv_heads, int group, int64_t tail_capacity, int tail_len, const uint16_t* __restrict__ tail,
    const uint16_t* __restrict__ q, float* __restrict__ scores, int64_t score_stride, int64_t offset) {
  __shared__ float qs[SC_MAXG * D];
  const int tid = threadIdx.x, l16 = tid & 15;
  const size_t sg = blockIdx.x;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  for (int e = tid; e < group * D; e += THREADS) qs[e] = half_bits_to_float(q[(sq * n_q_heads + kv * group) * D + e]);
  __syncthreads();
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  for (int t0 = 0; t0 < tail_len; t0 += THREADS / 16) {   // uniform trip count: the row sums need whole rows
    const int t = t0 + (tid >> 4);
    float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (t < tail_len) load8(tail, EOQ_F16, (sg * (size_t)tail_capacity + t) * D + 8 * l16, x);
    for (int h = 0; h < group; ++h) {
      float acc = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(x[e], qs[h * D + 8 * l16 + e], acc);
      acc += dpp_mov<0xB1>(acc);
      acc += dpp_mov<0x4E>(acc);
      acc += dpp_mov<0x141>(acc);
      acc += dpp_mov<0x140>(acc);
      if (l16 == 0 && t < tail_len) scores[(sq * n_q_heads + kv * group + h) * (size_t)score_stride + offset + t] = acc * inv_sqrt_d;
    }
  }
}

hipError_t launch_scores_impl(const EoqLaunch& L, eoq_packed keys, const eoq_qjl* qjl, int64_t n_seq, int n_kv_heads,
                              int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores,
                              int64_t block_capacity, int64_t score_stride, const void* tail_fp16,
                              int64_t tail_capacity, int tail_len) {
  const int64_t sg_total = n_seq * n_kv_heads;
  if (block_capacity <= 0) block_capacity = blocks_per_head;
  if (score_stride <= 0) score_stride = blocks_per_head * L.n;
  if (L.ev) (void)hipEventRecord(L.ev[6], L.stream);
  if (tail_len > 0)
    hipLaunchKernelGGL(eoq_scores_tail_kernel, dim3((unsigned)sg_total), dim3(THREADS), 0, L.stream, n_kv_heads,
                       n_q_heads / n_kv_heads, tail_capacity, tail_len, static_cast<const uint16_t*>(tail_fp16),
                       static_cast<const uint16_t*>(q_fp16), scores, score_stride, blocks_per_head * L.n);
  if (blocks_per_head == 0) {
    if (L.ev) (void)hipEventRecord(L.ev[7], L.stream);
    return hipGetLastError();
  }
  // blocks per workgroup: up to 16 (the query set-up is paid once per workgroup), shorter when that leaves fewer than ~16
  // workgroups per compute unit
  int64_t run = (sg_total * blocks_per_head) / 4096;
  run = run < 1 ? 1 : (run > SC_RUN_MAX ? SC_RUN_MAX : run);
  const int64_t runs = (blocks_per_head + run - 1) / run;
  if (sg_total > 65535 || runs > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)runs, (unsigned)sg_total), block(THREADS);
  const uint16_t* q = static_cast<const uint16_t*>(q_fp16);
  const int group = n_q_heads / n_kv_heads;
#define EOQ_SCORES_ARGS                                                                                              \
  grid, block, 0, L.stream, L.n, L.r_max, n_kv_heads, group, blocks_per_head, block_capacity, score_stride, (int)run, \
      L.pih, L.tab, keys.codes, keys.norms, keys.rank, keys.lfac, keys.rfac, q, scores
#define EOQ_SCORES(BITS, NSETS)                                                                                      \
  do {                                                                                                               \
    if (qjl)                                                                                                         \
      hipLaunchKernelGGL((eoq_scores_i8_kernel<BITS, true, NSETS>), EOQ_SCORES_ARGS, L.phih, qjl->signs, qjl->norms); \
    else                                                                                                             \
      hipLaunchKernelGGL((eoq_scores_i8_kernel<BITS, false, NSETS>), EOQ_SCORES_ARGS, (const uint16_t*)nullptr,      \
                         (const uint8_t*)nullptr, (const uint16_t*)nullptr);                                         \
  } while (0)
#define EOQ_SCORES_BITS(NSETS)              \
  switch (L.bits) {                         \
    case 1: EOQ_SCORES(1, NSETS); break;    \
    case 2: EOQ_SCORES(2, NSETS); break;    \
    case 3: EOQ_SCORES(3, NSETS); break;    \
    default: EOQ_SCORES(4, NSETS); break;   \
  }
  if (group <= 4) {
    EOQ_SCORES_BITS(1)
  } else {
    EOQ_SCORES_BITS(2)
  }
#undef EOQ_SCORES_BITS
#undef EOQ_SCORES
#undef EOQ_SCORES_ARGS
  if (L.ev) (void)hipEventRecord(L.ev[7], L.stream);
  return hipGetLastError();
}

}  // namespace

hipError_t eoq_launch_scores(const EoqLaunch& L, eoq_packed keys, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores,
                             int64_t block_capacity, int64_t score_stride, const void* tail_fp16,
                             int64_t tail_capacity, int tail_len) {
  return launch_scores_impl(L, keys, nullptr, n_seq, n_kv_heads, blocks_per_head, q_fp16, n_q_heads, scores,
                            block_capacity, score_stride, tail_fp16, tail_capacity, tail_len);
}

hipError_t eoq_launch_scores_prod(const EoqLaunch& L, eoq_packed keys, eoq_qjl qjl, int64_t n_seq, int n_kv_heads,
                                  int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores) {
  return launch_scores_impl(L, keys, &qjl, n_seq, n_kv_heads, blocks_per_head, q_fp16, n_q_heads, scores, 0, 0, nullptr,
                            0, 0);
}
