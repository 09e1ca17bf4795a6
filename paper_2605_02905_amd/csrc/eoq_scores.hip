// Decode scoring on compressed keys (Sec. 2.1 attention logits, Remark 6.5): scores[s][h][t] = <q_h, x_hat_t>/sqrt(d)
// from the record, without forming x_hat.  With x_hat_t = rho_t Pi^T z_hat_t + C_t V_r:
//     <q, x_hat_t> = rho_t <Pi q, z_hat_t> + <C_t, V_r^T q>.
//
// The first term runs on the integer matrix cores.  The codebook is symmetric, so a centroid is its sign times a
// magnitude that is a multilinear function of the magnitude bits m_p (index bit p of the code, inverted on the negative
// half):  z_hat_j = s_j sum_M coef[M] prod_{p in M} m_pj over the subsets M of the b-1 magnitude bits (b = 2: c_0 + (c_1 -
// c_0) m_0).  Every term is an inner product of q' = Pi q with a vector of entries in {-1, 0, +1}: exact in int8.  q' is
// multiplied by the coefficient of its term and held in 32-bit fixed point per head (a power-of-two unit, four balanced
// signed bytes), so the rows of the A operand of v_mfma_i32_16x16x64_i8 are the four byte planes of four query heads and
// all sixteen rows do work, the terms of a coordinate sit side by side along k (one int32 accumulator takes the whole
// sum, exactly), the columns are sixteen tokens, and the four planes of a head meet again through three lane swaps.
// Operand convention of v_mfma_i32_16x16x64_i8 (wave64): lane l supplies A[row = l%16][k = 16*(l/16) .. +15] and
// B[k = 16*(l/16) .. +15][col = l%16] and receives D[row = 4*(l/16) + v][col = l%16] in accumulator register v.
// The {-1, 0, +1} operands come out of a 256-entry LDS table indexed by one nibble of the sign plane and one nibble of a
// magnitude plane: four coordinates of two terms per 8-byte read, in the order the matrix instruction takes them.
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int SC_MAXG = 8;      // most query heads per KV head
constexpr int SC_DEPTH = 2;     // passes of record bytes in flight per wave
constexpr int SC_RUN_MAX = 16;  // most blocks per workgroup (the run is shortened until the grid fills the chip)
constexpr int SC_CBP = 8;       // stored coefficients of this many components are requested one pass ahead

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

// Rows of `rows` ([SC_MAXG][D] float, LDS), each multiplied by the NT coefficients coef[0 .. NT-1], to 32-bit fixed
// point: per row the unit is 2^(E - 29) with E the exponent of the largest |coef| |entry| of the row, so |integer| <=
// 2^30; the integer is cut into four balanced signed bytes (the bytes of I + 0x80808080 with the top bit of each flipped)
// and byte plane p of row h goes to dig[(4 h + p) * NT * D + ...] with the NT terms of four consecutive coordinates side
// by side: byte ((c / 4) * NT + term) * 4 + c % 4 -- the order of k in the matrix instructions.  unit[h] = value of one
// integer unit (0 for a row that is zero, below 2^-87 or not finite).  All 256 lanes; barriers inside, the last one
// after the planes are written.
template <int NT>
__device__ __forceinline__ void fixed_point_rows(const float* rows, const float (&coef)[NT], unsigned char* dig, unsigned* max_s,
                                                 float* unit, int tid) {
  if (tid < SC_MAXG) max_s[tid] = 0u;
  __syncthreads();
  const int h = tid >> 5, c0 = 4 * (tid & 31);
  float cmax = 0.0f;
#pragma unroll
  for (int t = 0; t < NT; ++t) cmax = fmaxf(cmax, fabsf(coef[t]));
  float v[4];
  unsigned m = 0u;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[e] = rows[h * D + c0 + e];
    m = max(m, (unsigned)__float_as_uint(fabsf(v[e]) * cmax));
  }
  atomicMax(&max_s[h], m);
  __syncthreads();
  const int eb = (int)(max_s[h] >> 23);   // biased exponent of the row maximum
  const bool live = eb >= 40 && eb < 255;
  const double up = live ? (double)__uint_as_float((unsigned)(283 - eb) << 23) : 0.0;   // 2^(29 - (eb - 127))
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    uint32_t dg[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int I = live ? __double2int_rn((double)v[e] * (double)coef[t] * up) : 0;   // one rounding, |I| <= 2^30
      dg[e] = ((uint32_t)I + 0x80808080u) ^ 0x80808080u;
    }
    uint32_t pl[4];
    transpose_bytes(dg[0], dg[1], dg[2], dg[3], pl);
#pragma unroll
    for (int p = 0; p < 4; ++p) *reinterpret_cast<uint32_t*>(dig + (size_t)(4 * h + p) * NT * D + ((c0 >> 2) * NT + t) * 4) = pl[p];
  }
  if ((tid & 31) == 0) unit[h] = live ? __uint_as_float((unsigned)(eb - 29) << 23) : 0.0f;
  __syncthreads();
}

// The {-1, 0, +1} operands of one token for this lane's 32 coordinates (bits 0..31 of the lane's word of every bit
// plane), in the order of k that fixed_point_rows gives the query side: for every nibble (four coordinates) the terms
// M = 0 .. TYPES-1 (M = subset of the magnitude bits, M = 0 the sign alone), four bytes each.  B[i] is the operand of
// matrix instruction i of the 2 TYPES that cover the word.  One table read per nibble and magnitude plane: entry (sign
// nibble | magnitude nibble << 4) = (the four sign bytes, the same bytes where the magnitude bit is set).
template <int BITS>
__device__ __forceinline__ void term_operands(const uint32_t (&word)[BITS], const uint2* nib_tab, v4i (&B)[2 << (BITS - 1)]) {
  constexpr int TYPES = 1 << (BITS - 1);
  const uint32_t top = word[BITS - 1];
  uint32_t term[8][TYPES];   // [nibble][term]
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
        if constexpr (BITS > 1) {
          const uint2 e = nib_tab[idx];
          term[k][0] = e.x;
          term[k][1] = e.y;
        } else {
          term[k][0] = nib_tab[idx].x;
        }
      } else {
        term[k][(1 << p) % TYPES] = nib_tab[idx].y;
      }
    }
  }
  // products of several magnitude bits: bytes are 0 or the sign byte, so the product is the bitwise AND
#pragma unroll
  for (int M = 3; M < TYPES; ++M) {
    if ((M & (M - 1)) != 0) {
      const int low = M & -M;
#pragma unroll
      for (int k = 0; k < 8; ++k) term[k][M] = term[k][low] & term[k][M ^ low];
    }
  }
#pragma unroll
  for (int i = 0; i < 2 * TYPES; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int flat = 4 * i + w;   // dword number along k: nibble flat / TYPES, term flat % TYPES
      B[i][w] = (int)term[flat / TYPES][flat % TYPES];
    }
}

// The four accumulator registers of a lane are four heads of byte plane g = lane / 16.  Joins the planes: lane group g
// returns sum_p 256^p (register g of plane p), the value of head g in integer units.  v_permlane16_swap exchanges the odd
// 16-lane rows of its first operand with the even rows of its second, v_permlane32_swap the upper half of the first with
// the lower half of the second; planes 2k and 2k + 1 are joined exactly in int32 (|register| < 2^18), the two halves in
// float32.
__device__ __forceinline__ float join_planes(const v4i& acc) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const u2 a = __builtin_amdgcn_permlane16_swap((unsigned)acc[0], (unsigned)acc[1], false, false);
  const u2 b = __builtin_amdgcn_permlane16_swap((unsigned)acc[2], (unsigned)acc[3], false, false);
  // even rows: (own plane, head r | plane + 1, head r), odd rows: (plane - 1, head r | own plane, head r); r = row parity
  const int ta = (int)a[0] + (int)a[1] * 256;   // head r,     planes 2k, 2k + 1
  const int tb = (int)b[0] + (int)b[1] * 256;   // head 2 + r, planes 2k, 2k + 1
  const u2 c = __builtin_amdgcn_permlane32_swap((unsigned)ta, (unsigned)tb, false, false);
  // lower half: (planes 0-1 of head r, planes 2-3 of head r); upper half: (planes 0-1 of head 2 + r, planes 2-3 of it)
  return fmaf((float)(int)c[1], 65536.0f, (float)(int)c[0]);
}

// 4 x 4 transpose across the four lane groups: on entry lane group g holds r0 .. r3, on return lane group s holds
// out[g] = (r_s of lane group g).
__device__ __forceinline__ void transpose_groups(float r0, float r1, float r2, float r3, float (&out)[4]) {
  typedef unsigned int u2 __attribute__((ext_vector_type(2)));
  const u2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(r0), __float_as_uint(r2), false, false);
  const u2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(r1), __float_as_uint(r3), false, false);
  const u2 c = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
  const u2 d = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
  out[0] = __uint_as_float(c[0]);
  out[1] = __uint_as_float(c[1]);
  out[2] = __uint_as_float(d[0]);
  out[3] = __uint_as_float(d[1]);
}

// What a lane requests of one chunk of 128 consecutive tokens (the unit of work of a wave): piece i of the chunk's codes
// (bytes 1024 i + 16 lane .. + 15: every load instruction covers 1 KB without gaps), the stored norms and the stored
// coefficients of ITS OWN two tokens 2 lane and 2 lane + 1 of the chunk (with QJL also the sign planes and residual norms).
template <int BITS, bool QJL>
struct ChunkFetch {
  uint4 code[2 * BITS];
  uint32_t rho2;
  uint32_t cf[SC_CBP];
  uint4 sign[QJL ? 2 : 1];
  uint32_t gam2;
};
// Buffer addressing: a resource descriptor in scalar registers (base of this workgroup's run of blocks, size of the
// run: reads past it return zero instead of faulting), a scalar byte offset that moves from chunk to chunk and a per-lane
// 32-bit offset that never changes -- no vector arithmetic per load.
struct ScoreBuffers {
  __amdgpu_buffer_rsrc_t codes, norms, lfac, qsigns, qnorms;
};
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_b128(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, int soffset) {
  const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voffset, soffset, 0);
  return make_uint4(v[0], v[1], v[2], v[3]);
}
// LDS staging of a chunk's codes: 16 bytes of padding after every 256, so that the sixteen token pairs a matrix
// instruction's lanes read side by side (64 BITS/2 bytes apart) fall into different banks while 16-byte pieces stay aligned.
__host__ __device__ constexpr int stage_pad(int a) { return a + ((a >> 8) << 4); }

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
  constexpr int WH = 4 * NSETS;   // heads the run's w table holds
  // One pool, used in turn: during the set-up the query (float), its rotation, and the byte planes of coef[M] Pi q
  // ([head][plane][k]) and of Phi q; in the chunk loop the four waves' staging buffers.  The barrier behind the w table
  // separates the two uses.
  constexpr int CODE_STAGE = stage_pad(128 * (BITS * D / 8)), SIGN_STAGE = QJL ? stage_pad(128 * (D / 8)) : 0;
  constexpr int SETUP_BYTES = 2 * SC_MAXG * D * 4 + SC_MAXG * 4 * TYPES * D + (QJL ? SC_MAXG * 4 * D : 0);
  constexpr int LOOP_BYTES = 4 * (CODE_STAGE + SIGN_STAGE);
  __shared__ __align__(16) unsigned char pool[SETUP_BYTES > LOOP_BYTES ? SETUP_BYTES : LOOP_BYTES];
  float* qraw = reinterpret_cast<float*>(pool);
  float* qrot = qraw + SC_MAXG * D;
  unsigned char* qdig = pool + 2 * SC_MAXG * D * 4;
  unsigned char* pdig = qdig + SC_MAXG * 4 * TYPES * D;
  __shared__ __align__(16) float wbuf[SC_RUN_MAX * EOQ_RMAX_CAP * WH];   // [block of the run][component][head]: <v_i, q_h>/sqrt(d)
  __shared__ int rank_s[SC_RUN_MAX];
  __shared__ __align__(16) uint2 nib_tab[256];
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
  // q' = Pi q (the rotation moved to the query side: <q, Pi^T z> = <Pi q, z>), then the byte planes of coef[M] q'
  rotate_query(pih, pih + D * D, q + q0, group, qrot, wave, l16, g);
  __syncthreads();
  fixed_point_rows<TYPES>(qrot, coef, qdig, max_s, qunit, tid);
  if constexpr (QJL) {
    rotate_query(phih, nullptr, q + q0, group, qrot, wave, l16, g);
    __syncthreads();
    const float one[1] = {1.0f};
    fixed_point_rows<1>(qrot, one, pdig, max_s, punit, tid);
  }
  // A operands: row l16 = byte plane l16 / 4 of head 4 hs + l16 % 4; instruction i of a token covers the 16 bytes of k
  // from 16 i of lane group g's 32 coordinates (32 TYPES bytes).  Kq / Kp: what one integer unit of head 4 hs + v is
  // worth in the logit.
  v4i Aq[NSETS][2 * TYPES], Ap[QJL ? NSETS : 1][2];
  float Kq[NSETS][4], Kp[QJL ? NSETS : 1][4];
  const float qjl_scale = sqrtf(1.5707963267948966f) / (float)D;
#pragma unroll
  for (int hs = 0; hs < NSETS; ++hs) {
    const int row = 4 * (4 * hs + (l16 & 3)) + (l16 >> 2);
#pragma unroll
    for (int i = 0; i < 2 * TYPES; ++i) Aq[hs][i] = *reinterpret_cast<const v4i*>(qdig + ((size_t)row * D + 32 * g) * TYPES + 16 * i);
#pragma unroll
    for (int v = 0; v < 4; ++v) Kq[hs][v] = qunit[4 * hs + v] * (1.0f / (float)D);   // z_hat = centroid / sqrt(d), logit = <q, x_hat> / sqrt(d)
    if constexpr (QJL) {
#pragma unroll
      for (int i = 0; i < 2; ++i) Ap[hs][i] = *reinterpret_cast<const v4i*>(pdig + row * D + 32 * g + 16 * i);
#pragma unroll
      for (int v = 0; v < 4; ++v) Kp[hs][v] = punit[4 * hs + v] * (qjl_scale * inv_sqrt_d);
    }
  }

  // The work of this workgroup as a flat list of chunks of 128 tokens: chunk u of the run is tokens 128 (u % cpb) ..
  // of block jb0 + u / cpb; wave w takes the chunks w, w + 4, ...  The record bytes of a chunk are requested one chunk
  // ahead into registers; the codes then pass through a wave-private LDS buffer, which hands every lane of a matrix
  // instruction the words of its token pair, in four sub-passes of 32 tokens (tile u of sub-pass s: tokens 32 s + 2 c + u
  // in column c).  After the four sub-passes a lane group holds one head of all four; a 4 x 4 transpose across the lane
  // groups gives lane L all heads of its own tokens 2 L and 2 L + 1, which it scales by its own stored norms, completes
  // with the low-rank term from its own stored coefficients and stores as 8 bytes per head: 512 contiguous bytes per wave
  // and score row.
  const int64_t jb0 = (int64_t)blockIdx.x * run;
  const int nblk = (int)(min(jb0 + run, blocks_per_head) - jb0);
  const int cpb = n / 128;
  const int NCH = nblk * cpb;
  const size_t blk0 = sg * (size_t)block_capacity + jb0;   // the store holds block_capacity slots per head

  // w[b][i][h] = <v_i, q_h>/sqrt(d) of every block of the run, up front (the low-rank term is <C_t, w_h>): all loads of
  // the set-up are in flight together and the chunk loop below has no barrier.  16 lanes per (component, head): one
  // 16-byte load of eight entries of v_i each, then a sum over the DPP row.
  if (tid < nblk) rank_s[tid] = min(max(rank_in[blk0 + tid], 0), r_max);   // records may come from storage: never index past r_max rows
  __syncthreads();
  int rtop = 0;
  for (int b = 0; b < nblk; ++b) rtop = max(rtop, rank_s[b]);
  for (int e0 = 0; e0 < nblk * rtop * (WH * 16); e0 += THREADS) {   // uniform trip count: whole rows reduce together
    const int e = e0 + tid;
    const int seg = e & 15, h = (e >> 4) & (WH - 1);
    const int bi = e / (WH * 16), b = bi / rtop, i = bi - b * rtop;
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
    if (seg == 0 && b < nblk && i < rb) wbuf[(b * EOQ_RMAX_CAP + i) * WH + h] = acc * inv_sqrt_d;
  }
  __syncthreads();

  ScoreBuffers sb;
  sb.codes = buffer_of(codes + blk0 * (size_t)n * ROWB, (size_t)nblk * n * ROWB);
  sb.norms = buffer_of(norms + blk0 * (size_t)n, (size_t)nblk * n * 2);
  sb.lfac = buffer_of(lfac + blk0 * (size_t)r_max * n, (size_t)nblk * r_max * n * 2);
  if constexpr (QJL) {
    sb.qsigns = buffer_of(qsigns + blk0 * (size_t)n * (D / 8), (size_t)nblk * n * (D / 8));
    sb.qnorms = buffer_of(qnorms + blk0 * (size_t)n, (size_t)nblk * n * 2);
  }
  // chunk u: block u / cpb of the run, tokens 128 (u % cpb) ..; rows at and above the rank are asked for at an offset
  // past the end of the buffer: those loads return zero without touching memory
  auto request = [&](ChunkFetch<BITS, QJL>& f, int u) __attribute__((always_inline)) {
    const int b = u / cpb, c = u - b * cpb;
    const int tokb = b * n + 128 * c;   // uniform: first token of the chunk, counted from the start of the run
#pragma unroll
    for (int i = 0; i < 2 * BITS; ++i) f.code[i] = load_b128(sb.codes, 16u * lane, tokb * ROWB + 1024 * i);
    f.rho2 = __builtin_amdgcn_raw_buffer_load_b32(sb.norms, 4u * lane, tokb * 2, 0);
    const int rr = __builtin_amdgcn_readfirstlane(rank_s[b]);
#pragma unroll
    for (int a = 0; a < SC_CBP; ++a) {
      const int row = (b * r_max + a) * n + 128 * c;   // uniform, in entries
      f.cf[a] = __builtin_amdgcn_raw_buffer_load_b32(sb.lfac, 4u * lane, (a < rr) ? row * 2 : 0x7FFFFF00, 0);
    }
    if constexpr (QJL) {
#pragma unroll
      for (int i = 0; i < 2; ++i) f.sign[i] = load_b128(sb.qsigns, 16u * lane, tokb * (D / 8) + 1024 * i);
      f.gam2 = __builtin_amdgcn_raw_buffer_load_b32(sb.qnorms, 4u * lane, tokb * 2, 0);
    }
  };

  // this wave's staging buffers and the lane's read addresses in them (sub-pass 0; sub-pass s is a constant further on)
  unsigned char* stage_c = pool + wave * (CODE_STAGE + SIGN_STAGE);
  unsigned char* stage_q = stage_c + CODE_STAGE;
  int rd_c[2][BITS], rd_q[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int p = 0; p < BITS; ++p) rd_c[u][p] = stage_pad((2 * l16 + u) * ROWB + 16 * p + 4 * g);
    rd_q[u] = stage_pad((2 * l16 + u) * (D / 8) + 4 * g);
  }
  constexpr int SUB_C = stage_pad(32 * ROWB), SUB_Q = stage_pad(32 * (D / 8));   // one sub-pass further (multiples of 256 before padding)
  const int wr = stage_pad(16 * lane);                                           // where the lane's piece of 1 KB number 0 goes

  const bool even_stride = (T & 1) == 0;
  auto work = [&](ChunkFetch<BITS, QJL>& cur, int u_chunk) __attribute__((always_inline)) {
    const int cb_blk = u_chunk / cpb, cq = u_chunk - cb_blk * cpb;
    const size_t blk = blk0 + cb_blk;
    const int r = rank_s[cb_blk];
    const float* wrow = wbuf + cb_blk * (EOQ_RMAX_CAP * WH);
    const int64_t jb = jb0 + cb_blk;
    // ---- the codes change lanes through LDS (the buffer is this wave's own: its LDS operations complete in order) ----
#pragma unroll
    for (int i = 0; i < 2 * BITS; ++i) *reinterpret_cast<uint4*>(stage_c + wr + stage_pad(1024) * i) = cur.code[i];
    if constexpr (QJL) {
#pragma unroll
      for (int i = 0; i < 2; ++i) *reinterpret_cast<uint4*>(stage_q + wr + stage_pad(1024) * i) = cur.sign[i];
    }
    __builtin_amdgcn_wave_barrier();
    float tq[4][2][NSETS], tp[QJL ? 4 : 1][2][NSETS];   // [sub-pass][tile][set]: head 4 hs + g in integer units
#pragma unroll
    for (int sp = 0; sp < 4; ++sp) {
      v4i B[2][2 * TYPES];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        uint32_t word[BITS];
#pragma unroll
        for (int p = 0; p < BITS; ++p) word[p] = *reinterpret_cast<const uint32_t*>(stage_c + rd_c[u][p] + SUB_C * sp);
        term_operands<BITS>(word, nib_tab, B[u]);
      }
#pragma unroll
      for (int hs = 0; hs < NSETS; ++hs) {
        v4i acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          acc[u] = v4i{0, 0, 0, 0};
#pragma unroll
          for (int i = 0; i < 2 * TYPES; ++i) acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(Aq[hs][i], B[u][i], acc[u], 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) tq[sp][u][hs] = join_planes(acc[u]);
      }
      if constexpr (QJL) {
        // sign(Phi r_x) is one more plane of +-1: the table's first entry kind with the magnitude nibble at zero
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const uint32_t sw = *reinterpret_cast<const uint32_t*>(stage_q + rd_q[u] + SUB_Q * sp);
          v4i Bs[2];
#pragma unroll
          for (int k = 0; k < 8; ++k) Bs[k >> 2][k & 3] = (int)nib_tab[(sw >> (4 * k)) & 0xFu].x;
#pragma unroll
          for (int hs = 0; hs < NSETS; ++hs) {
            v4i acc = {0, 0, 0, 0};
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(Ap[hs][0], Bs[0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(Ap[hs][1], Bs[1], acc, 0, 0, 0);
            tp[sp][u][hs] = join_planes(acc);
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();   // the staging buffer is rewritten by the next chunk
    // ---- to the lanes that own the tokens: lane group sp takes sub-pass sp, register index becomes the head ----
    const float rho[2] = {half_bits_to_float((uint16_t)(cur.rho2 & 0xFFFFu)), half_bits_to_float((uint16_t)(cur.rho2 >> 16))};
    float gam[2] = {0.0f, 0.0f};
    if constexpr (QJL) {
      gam[0] = half_bits_to_float((uint16_t)(cur.gam2 & 0xFFFFu));
      gam[1] = half_bits_to_float((uint16_t)(cur.gam2 >> 16));
    }
    float res[4][2][NSETS];   // [head of the set][token][set]
#pragma unroll
    for (int hs = 0; hs < NSETS; ++hs)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float h4[4];
        transpose_groups(tq[0][u][hs], tq[1][u][hs], tq[2][u][hs], tq[3][u][hs], h4);
#pragma unroll
        for (int v = 0; v < 4; ++v) res[v][u][hs] = h4[v] * (Kq[hs][v] * rho[u]);
        if constexpr (QJL) {
          transpose_groups(tp[0][u][hs], tp[1][u][hs], tp[2][u][hs], tp[3][u][hs], h4);
#pragma unroll
          for (int v = 0; v < 4; ++v) res[v][u][hs] = fmaf(h4[v], Kp[hs][v] * gam[u], res[v][u][hs]);
        }
      }
    // ---- low-rank term from the lane's own coefficients: sum_i C[i][token] w[i][head] ----
    if (r > 0) {
#pragma unroll
      for (int a = 0; a < SC_CBP; ++a) {
        if (a < r) {   // uniform
          const float c0 = half_bits_to_float((uint16_t)(cur.cf[a] & 0xFFFFu)), c1 = half_bits_to_float((uint16_t)(cur.cf[a] >> 16));
#pragma unroll
          for (int hs = 0; hs < NSETS; ++hs) {
            const float4 w = *reinterpret_cast<const float4*>(wrow + a * WH + 4 * hs);
            const float wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              res[v][0][hs] = fmaf(wv[v], c0, res[v][0][hs]);
              res[v][1][hs] = fmaf(wv[v], c1, res[v][1][hs]);
            }
          }
        }
      }
      for (int i = SC_CBP; i < r; ++i) {   // ranks above SC_CBP: read in place
        const uint32_t cx = *reinterpret_cast<const uint32_t*>(lfac + (blk * r_max + i) * (size_t)n + 128 * cq + 2 * lane);
        const float c0 = half_bits_to_float((uint16_t)(cx & 0xFFFFu)), c1 = half_bits_to_float((uint16_t)(cx >> 16));
#pragma unroll
        for (int hs = 0; hs < NSETS; ++hs) {
          const float4 w = *reinterpret_cast<const float4*>(wrow + i * WH + 4 * hs);
          const float wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            res[v][0][hs] = fmaf(wv[v], c0, res[v][0][hs]);
            res[v][1][hs] = fmaf(wv[v], c1, res[v][1][hs]);
          }
        }
      }
    }
#pragma unroll
    for (int hs = 0; hs < NSETS; ++hs)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int h = 4 * hs + v;
        if (h < group) {   // uniform
          float* dst = scores + (sq * n_q_heads + kv * group + h) * T + (size_t)jb * n + 128 * cq + 2 * lane;
          if (even_stride) {
            *reinterpret_cast<float2*>(dst) = make_float2(res[v][0][hs], res[v][1][hs]);
          } else {
            dst[0] = res[v][0][hs];
            dst[1] = res[v][1][hs];
          }
        }
      }
  };

  // two register sets in turn: the next chunk is requested before this one is worked on
  ChunkFetch<BITS, QJL> fa, fb;
  if (wave < NCH) request(fa, wave);
  for (int u0 = wave; u0 < NCH; u0 += 8) {
    if (u0 + 4 < NCH) request(fb, u0 + 4);
    work(fa, u0);
    if (u0 + 4 < NCH) {
      if (u0 + 8 < NCH) request(fa, u0 + 8);
      work(fb, u0 + 4);
    }
  }
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
  // blocks per workgroup: the query set-up is paid once per workgroup, so runs are as long as they can be (16) while the
  // grid still has a workgroup for each of the 4 x 256 places on the chip
  int64_t run = (sg_total * blocks_per_head + 1023) / 1024;
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
