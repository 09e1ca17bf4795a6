// Decode scoring on compressed keys (Sec. 2.1 attention logits, Remark 6.5): scores[s][h][t] = <q_h, x_hat_t>/sqrt(d)
// from the record, without forming x_hat.  With x_hat_t = rho_t Pi^T z_hat_t + C_t V_r:
//     <q, x_hat_t> = rho_t <Pi q, z_hat_t> + <C_t, V_r^T q>.
//
// The first term runs on the integer matrix cores.  The codebook is symmetric, so a centroid is its sign times a
// magnitude that is a multilinear function of the magnitude bits m_p (index bit p of the code, inverted on the negative
// half):  z_hat_j = s_j sum_M coef[M] prod_{p in M} m_pj over the subsets M of the b-1 magnitude bits (b = 2: c_0 + (c_1 -
// c_0) m_0).  Every term is an inner product of q' = Pi q with a vector of entries in {-1, 0, +1}: exact in int8.  q' is
// multiplied by the coefficient of its term and held in 32-bit fixed point per head (a power-of-two unit, four balanced
// signed bytes): the 32 rows of the A operand of v_mfma_i32_32x32x32_i8 are the four byte planes of eight query heads,
// the terms of a coordinate sit side by side along k (one int32 accumulator takes the whole sum, exactly) and the
// columns are 32 tokens.
// Operand convention of v_mfma_i32_32x32x32_i8 (wave64): lane l supplies A[row = l%32][k = 16*(l/32) .. +15] and
// B[k = 16*(l/32) .. +15][col = l%32] and receives D[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator
// register v.  Row 8 q + 4 f + e is byte plane e of head 2 q + f: lane (token, f) receives all four planes of the heads
// f, 2 + f, 4 + f, 6 + f of ITS token, joins them, scales by its own stored norm and stores -- nothing changes lanes.
// The low-rank term rides the f16 matrix cores the same way: rows e = 0 / 1 of head 2 q + f hold the binary16 hi / lo
// parts of w_h = V_r^T q_h / sqrt(d), the B operand the token's stored coefficients.
// The {-1, 0, +1} operands come out of a 256-entry LDS table indexed by one nibble of the sign plane and one nibble of a
// magnitude plane: four coordinates of two terms per 8-byte read, in the order the matrix instruction takes them; the
// lane that owns a token reads its 8 bytes of every bit-plane straight from the record (lane half f: coordinates 64 f ..
// 64 f + 63).
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int SC_MAXG = 8;      // most query heads per KV head
constexpr int SC_RUN_MAX = 16;  // most blocks per workgroup (the run is shortened until the grid fills the chip)

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
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

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float float16v __attribute__((ext_vector_type(16)));
constexpr int CTLD = 32 + 8;   // row stride (halfs) of a tile's coefficient rows in LDS, [component][token]

// What a lane requests of a tile of 32 consecutive tokens: lane (l32, hf) owns token l32.
template <int BITS, bool QJL>
struct TileFetch {
  u32x2 pl[BITS];            // bytes 8 hf .. 8 hf + 7 of every bit-plane of the token
  uint32_t rho;              // the token's stored norm (binary16 in the low half)
  u32x4 cf;                  // lane L: stored coefficients C[tokens 8 (L % 4) .. + 7][component L / 4]; zero at and above the rank
  u32x2 sg[QJL ? 1 : 0];     // the same bytes of sign(Phi r_x)
  uint32_t gam[QJL ? 1 : 0]; // the token's stored residual norm
};

// One workgroup per (sequence, KV head, run of blocks); every wave works on 32-token tiles of its own (tile u of the
// run: tokens 32 (u % tpb) .. of block u / tpb; wave w takes the tiles w, w + 4, ...), the record bytes of the next
// tile on their way while this one is worked on.  NQ = query heads a lane finishes per token (2 for groups up to 4).
// QJL: the logits get the correction of Eq. (qjl), |r_x| sqrt(pi/2)/d <Phi q, sign(Phi r_x)>, from one more bit plane
// (the signs) and the stored residual norm; Phi q goes through the same fixed-point form as Pi q.
template <int BITS, bool QJL, int NQ>
__global__ __launch_bounds__(THREADS, (BITS <= 2 && !QJL) ? 4 : 1) void eoq_scores_i8_kernel(
    int n, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, int64_t block_capacity, int64_t score_stride,
    int run, const uint16_t* __restrict__ pih,
    const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const uint16_t* __restrict__ q, float* __restrict__ scores, const uint16_t* __restrict__ phih,
    const uint8_t* __restrict__ qsigns, const uint16_t* __restrict__ qnorms) {
  constexpr int TYPES = 1 << (BITS - 1);
  constexpr int NMM = 4 * TYPES;   // matrix instructions per tile: 64 coordinates x TYPES bytes per lane, 16 at a time
  constexpr int WH = 2 * NQ;       // heads the run's w table holds
  // One pool, used in turn: during the set-up the query (float), its rotation, and the byte planes of coef[M] Pi q
  // ([head][plane][k]) and of Phi q; in the tile loop the four waves' coefficient tiles.  The barrier behind the w
  // table separates the two uses.
  constexpr int SETUP_BYTES = 2 * SC_MAXG * D * 4 + SC_MAXG * 4 * TYPES * D + (QJL ? SC_MAXG * 4 * D : 0);
  constexpr int CS_BYTES = 4 * 2 * 16 * CTLD * 2;            // the four waves' coefficient tiles
  constexpr int LOOP_BYTES = CS_BYTES + SC_RUN_MAX * 32 * 16;   // and the run's low-rank operands
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
  const int l32 = lane & 31, hf = lane >> 5;
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
  // A operands: row l32 = byte plane l32 % 4 of head 2 (l32 / 8) + (l32 / 4) % 2; instruction i covers the 16 bytes of k
  // from 16 i of lane half hf's 64 coordinates (64 TYPES bytes: per nibble of four coordinates the TYPES terms).  Kq / Kp:
  // what one integer unit of head 2 qq + hf is worth in the logit.
  const int arow = 4 * (2 * (l32 >> 3) + ((l32 >> 2) & 1)) + (l32 & 3);   // row of the byte planes: 4 head + plane
  v4i Aq[NMM], Ap[QJL ? 4 : 1];
  float Kq[NQ], Kp[QJL ? NQ : 1];
  const float qjl_scale = sqrtf(1.5707963267948966f) / (float)D;
#pragma unroll
  for (int i = 0; i < NMM; ++i) Aq[i] = *reinterpret_cast<const v4i*>(qdig + ((size_t)arow * D + 64 * hf) * TYPES + 16 * i);
#pragma unroll
  for (int qq = 0; qq < NQ; ++qq) Kq[qq] = qunit[2 * qq + hf] * (1.0f / (float)D);   // z_hat = centroid / sqrt(d), logit = <q, x_hat> / sqrt(d)
  if constexpr (QJL) {
#pragma unroll
    for (int i = 0; i < 4; ++i) Ap[i] = *reinterpret_cast<const v4i*>(pdig + arow * D + 64 * hf + 16 * i);
#pragma unroll
    for (int qq = 0; qq < NQ; ++qq) Kp[qq] = punit[2 * qq + hf] * (qjl_scale * inv_sqrt_d);
  }

  const int64_t jb0 = (int64_t)blockIdx.x * run;
  const int nblk = (int)(min(jb0 + run, blocks_per_head) - jb0);
  const int tpb = n / 32;
  const int NT = nblk * tpb;
  const size_t blk0 = sg * (size_t)block_capacity + jb0;   // the store holds block_capacity slots per head

  // w[b][i][h] = <v_i, q_h>/sqrt(d) of every block of the run, up front (the low-rank term is <C_t, w_h>): all loads of
  // the set-up are in flight together and the tile loop below has no barrier.  16 lanes per (component, head): one
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
  // A operands of the low-rank product, components 0 .. 15, for every block of the run: row 8 qq + 4 f of the matrix
  // instruction holds binary16(w) of head 2 qq + f, the row after it what that rounding lost, the other two rows are
  // zero and not stored.  Entry (b, ci): lane half ci / 16 (components 8 hf + e), row group (ci / 2) % 8, part ci % 2.
  uint4* wop = reinterpret_cast<uint4*>(pool + CS_BYTES);
  for (int e = tid; e < nblk * 32; e += THREADS) {
    const int b = e >> 5, ci = e & 31;
    const int ohf = ci >> 4, l4 = (ci >> 1) & 7, part = ci & 1;
    const int h = 2 * (l4 >> 1) + (l4 & 1), rb = rank_s[b];
    H8 x;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int i = 8 * ohf + k;
      const float w = (i < rb && h < WH) ? wbuf[(b * EOQ_RMAX_CAP + i) * WH + (h & (WH - 1))] : 0.0f;
      const uint16_t hi = float_to_half_bits(w);
      x.s[k] = part == 0 ? hi : float_to_half_bits(w - half_bits_to_float(hi));
    }
    wop[e] = x.u;
  }
  __syncthreads();
  if (wave >= NT) return;

  // Buffer addressing: a resource descriptor in scalar registers, a scalar byte offset that moves from tile to tile and
  // a per-lane 32-bit offset that never changes -- no vector arithmetic per load.  The coefficients get a descriptor per
  // block that ends behind row rank - 1, and the range check covers the per-lane part of the offset, which holds the
  // row: rows at and above the rank read zero.  A request or a store for a tile behind the wave's last one goes through
  // descriptors of size zero (nothing is read or written), so every pass of the loop below issues the same memory
  // instructions and a wait can name exactly the loads it needs.
  const uint8_t* codes0 = codes + blk0 * (size_t)n * ROWB;
  const uint16_t* norms0 = norms + blk0 * (size_t)n;
  const uint8_t* qsigns0 = QJL ? qsigns + blk0 * (size_t)n * (D / 8) : nullptr;
  const uint16_t* qnorms0 = QJL ? qnorms + blk0 * (size_t)n : nullptr;
  // score rows of this (sequence, KV head): row h at h T floats; lane (token, hf) stores head 2 qq + hf
  float* scores0 = scores + (sq * n_q_heads + kv * group) * T;
  const uint32_t vo_code = (uint32_t)(l32 * ROWB + 8 * hf);
  const uint32_t vo_sign = (uint32_t)(l32 * (D / 8) + 8 * hf);
  const uint32_t vo_norm = (uint32_t)(2 * l32);
  const uint32_t vo_cf = (uint32_t)(((lane >> 2) * n + (lane & 3) * 8) * 2);
  const uint32_t vo_out = (uint32_t)((hf * T + l32) * 4);
  uint16_t* cs = reinterpret_cast<uint16_t*>(pool) + wave * (2 * 16 * CTLD);

  // The scalar unit is shared by the whole compute unit, so what a tile costs in scalar instructions counts: the
  // descriptors of the run are built once, a tile is addressed by its first token counted from the start of the run
  // (the wave's tiles are 128 tokens apart, also across a block boundary), the ranks of the run's blocks sit in the
  // lanes of one register, and the descriptor of a block's coefficients is rebuilt only when the block changes.
  const __amdgpu_buffer_rsrc_t bcodes = buffer_of(codes0, (size_t)nblk * n * ROWB);
  const __amdgpu_buffer_rsrc_t bnorms = buffer_of(norms0, (size_t)nblk * n * 2);
  const __amdgpu_buffer_rsrc_t bsigns = buffer_of(qsigns0, QJL ? (size_t)nblk * n * (D / 8) : 0);
  const __amdgpu_buffer_rsrc_t bgam = buffer_of(qnorms0, QJL ? (size_t)nblk * n * 2 : 0);
  const __amdgpu_buffer_rsrc_t bout = buffer_of(scores0 + (size_t)jb0 * n, ((size_t)group * T - (size_t)jb0 * n) * 4);
  const __amdgpu_buffer_rsrc_t bnone = buffer_of(scores0, 0);
  const int rk_all = rank_s[min(lane, nblk - 1)];
  auto rank_of = [&](int b) __attribute__((always_inline)) { return __builtin_amdgcn_readlane(rk_all, b); };
  auto coef_buffer = [&](int b) __attribute__((always_inline)) {
    return buffer_of(lfac + (blk0 + b) * (size_t)r_max * n, (size_t)rank_of(b) * n * 2);
  };
  // the tile whose first token is number tok of the run, in block b (first token b n), coefficients through cfd
  auto request = [&](TileFetch<BITS, QJL>& f, int tok, int b, __amdgpu_buffer_rsrc_t cfd) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < BITS; ++p) f.pl[p] = __builtin_amdgcn_raw_buffer_load_b64(bcodes, vo_code + 16 * p, tok * ROWB, 0);
    f.rho = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(bnorms, vo_norm, tok * 2, 0);
    f.cf = __builtin_amdgcn_raw_buffer_load_b128(cfd, vo_cf, (tok - b * n) * 2, 0);
    if constexpr (QJL) {
      f.sg[0] = __builtin_amdgcn_raw_buffer_load_b64(bsigns, vo_sign, tok * (D / 8), 0);
      f.gam[0] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(bgam, vo_norm, tok * 2, 0);
    }
  };
  // A operand of the low-rank product for block b of the run, components 16 k2 + 8 hf + e: row 8 qq + 4 f of the matrix
  // instruction holds binary16(w) of head 2 qq + f, the row after it what that rounding lost, the other two rows zero
  auto w_operand = [&](int b, int k2) __attribute__((always_inline)) {
    const int h = 2 * (l32 >> 3) + ((l32 >> 2) & 1), part = l32 & 3;
    const int rb = rank_of(b);
    H8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = 16 * k2 + 8 * hf + e;
      const float w = (i < rb && h < WH && part < 2) ? wbuf[(b * EOQ_RMAX_CAP + i) * WH + (h & (WH - 1))] : 0.0f;
      const uint16_t hi = float_to_half_bits(w);
      x.s[e] = part == 0 ? hi : float_to_half_bits(w - half_bits_to_float(hi));
    }
    return x;
  };
  // C[token l32][16 k2 + 8 hf + e] of the rows staged in the wave's coefficient tile: the B operand of that product
  auto c_operand = [&](int k2) __attribute__((always_inline)) {
    H8 x;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t a = cs[(16 * k2 + 8 * hf + 2 * w) * CTLD + l32], b = cs[(16 * k2 + 8 * hf + 2 * w + 1) * CTLD + l32];
      x.w[w] = a | (b << 16);
    }
    return x;
  };

  int wb = -1;   // block of the run whose w operand the wave holds
  H8 Aw;
  Aw.u = make_uint4(0u, 0u, 0u, 0u);
  auto work = [&](TileFetch<BITS, QJL>& cur, int tok, int b, int r, bool valid) __attribute__((always_inline)) {
    if (b != wb) {   // uniform
      Aw.u = ((l32 & 3) < 2) ? wop[b * 32 + 16 * hf + 2 * (l32 >> 2) + (l32 & 1)] : make_uint4(0u, 0u, 0u, 0u);
      wb = b;
    }
    // ---- the integer term: the lane's 64 coordinates, byte kk of every plane at a time ----
    const uint32_t top0 = cur.pl[BITS - 1][0], top1 = cur.pl[BITS - 1][1];
    v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
    if constexpr (BITS <= 2) {
      // even / odd: byte j = (sign nibble | magnitude nibble << 4) of the low / high nibbles of byte j of the planes;
      // one table read gives the four sign bytes and the same bytes where the magnitude bit is set: 8 of the 16 bytes
      // of an instruction (BITS = 1: the sign bytes alone, 4 of 16)
      uint32_t even[2], odd[2];
#pragma unroll
      for (int wq = 0; wq < 2; ++wq) {
        const uint32_t t = wq ? top1 : top0;
        const uint32_t x = (BITS == 2) ? ~(cur.pl[0][wq] ^ t) : 0u;   // magnitude bit: plane 0 where the sign plane is set, its complement elsewhere
        even[wq] = bfi(0x0F0F0F0Fu, t, x << 4);
        odd[wq] = bfi(0x0F0F0F0Fu, t >> 4, x);
      }
      if constexpr (BITS == 2) {
        EOQ_SFOR(kk, 8,
          const uint2 lo = nib_tab[(even[kk >> 2] >> (8 * (kk & 3))) & 0xFFu], hi = nib_tab[(odd[kk >> 2] >> (8 * (kk & 3))) & 0xFFu];
          const v4i B = {(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(Aq[kk], B, acc, 0, 0, 0);
        );
      } else {
        EOQ_SFOR(i, 4,
          const v4i B = {(int)nib_tab[(even[i >> 1] >> (16 * (i & 1))) & 0xFFu].x, (int)nib_tab[(odd[i >> 1] >> (16 * (i & 1))) & 0xFFu].x,
                         (int)nib_tab[(even[i >> 1] >> (16 * (i & 1) + 8)) & 0xFFu].x, (int)nib_tab[(odd[i >> 1] >> (16 * (i & 1) + 8)) & 0xFFu].x};
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(Aq[i], B, acc, 0, 0, 0);
        );
      }
    } else {
      // per nibble of four coordinates the TYPES terms, four bytes each: term 0 the signs, term 2^p from the table read
      // of magnitude plane p, the other terms (products of magnitude bits) as bitwise ANDs of those
      EOQ_SFOR(nb, 16,
        constexpr int wq = nb >> 3, sh = 4 * (nb & 7);
        const uint32_t t = wq ? top1 : top0;
        uint32_t term[TYPES];
        EOQ_SFOR(p, BITS - 1,
          const uint32_t x = ~(cur.pl[p][wq] ^ t);
          const uint2 e = nib_tab[((t >> sh) & 0xFu) | (((x >> sh) & 0xFu) << 4)];
          term[0] = e.x;
          term[1 << p] = e.y;
        );
        EOQ_SFOR(M, TYPES,
          if constexpr ((M & (M - 1)) != 0) term[M] = term[M & -M] & term[M ^ (M & -M)];
        );
        EOQ_SFOR(i, TYPES / 4,
          const v4i B = {(int)term[4 * i], (int)term[4 * i + 1], (int)term[4 * i + 2], (int)term[4 * i + 3]};
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(Aq[nb * (TYPES / 4) + i], B, acc, 0, 0, 0);
        );
      );
    }
    // ---- the planes of a head meet in the lane: registers 4 qq .. 4 qq + 3 are head 2 qq + hf; planes 0-1 and 2-3
    // are joined exactly in int32 (|register| < 2^18), the halves in float32 ----
    const float rho = half_bits_to_float((uint16_t)cur.rho);
    float res[NQ];
#pragma unroll
    for (int qq = 0; qq < NQ; ++qq) {
      const int lo = acc[4 * qq] + (acc[4 * qq + 1] << 8), hi = acc[4 * qq + 2] + (acc[4 * qq + 3] << 8);
      res[qq] = fmaf((float)hi, 65536.0f, (float)lo) * (Kq[qq] * rho);
    }
    if constexpr (QJL) {
      // sign(Phi r_x) is one more plane of +-1: the table's first entry kind with the magnitude nibble at zero
      v16i ac2;
#pragma unroll
      for (int v = 0; v < 16; ++v) ac2[v] = 0;
      EOQ_SFOR(i, 4,
        const uint32_t sw = cur.sg[0][i >> 1] >> (16 * (i & 1));
        const v4i B = {(int)nib_tab[sw & 0xFu].x, (int)nib_tab[(sw >> 4) & 0xFu].x, (int)nib_tab[(sw >> 8) & 0xFu].x, (int)nib_tab[(sw >> 12) & 0xFu].x};
        ac2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(Ap[i], B, ac2, 0, 0, 0);
      );
      const float gam = half_bits_to_float((uint16_t)cur.gam[0]);
#pragma unroll
      for (int qq = 0; qq < NQ; ++qq) {
        const int lo = ac2[4 * qq] + (ac2[4 * qq + 1] << 8), hi = ac2[4 * qq + 2] + (ac2[4 * qq + 3] << 8);
        res[qq] = fmaf(fmaf((float)hi, 65536.0f, (float)lo), Kp[qq] * gam, res[qq]);
      }
    }
    // ---- low-rank term sum_i C[i][token] w[i][head] on the f16 matrix cores: the coefficients change lanes through the
    // wave's LDS tile (one wave's LDS operations complete in order) ----
    if (r > 0) {   // uniform
      *reinterpret_cast<u32x4*>(cs + (lane >> 2) * CTLD + (lane & 3) * 8) = cur.cf;
      __builtin_amdgcn_wave_barrier();
      float16v lr;
#pragma unroll
      for (int v = 0; v < 16; ++v) lr[v] = 0.0f;
      lr = __builtin_amdgcn_mfma_f32_32x32x16_f16(Aw.h, c_operand(0).h, lr, 0, 0, 0);
      if (r > 16) {
        // components 16 .. 31 (rare): fetched and prepared here, nothing of them is kept
        const u32x4 c2 = __builtin_amdgcn_raw_buffer_load_b128(coef_buffer(b), vo_cf + (uint32_t)(16 * n * 2), (tok - b * n) * 2, 0);
        *reinterpret_cast<u32x4*>(cs + (16 + (lane >> 2)) * CTLD + (lane & 3) * 8) = c2;
        __builtin_amdgcn_wave_barrier();
        lr = __builtin_amdgcn_mfma_f32_32x32x16_f16(w_operand(b, 1).h, c_operand(1).h, lr, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();   // the tile is rewritten by the next one
#pragma unroll
      for (int qq = 0; qq < NQ; ++qq) res[qq] += lr[4 * qq] + lr[4 * qq + 1];
    }
    // head 2 qq + hf of the group: lanes of a head that the group does not have aim behind the descriptor, and a pass
    // behind the wave's last tile stores through the empty descriptor
    const __amdgpu_buffer_rsrc_t bo = valid ? bout : bnone;
#pragma unroll
    for (int qq = 0; qq < NQ; ++qq) {
      const bool live = 2 * qq + hf < group;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(res[qq]), bo, live ? vo_out : 0xFFFFFFF0u,
                                            (int)((2 * qq * T + tok) * 4), 0);
    }
  };

  // Two register sets in turn: the next tile is on its way while this one is worked on.  The loop body has no branch
  // around a memory instruction (a wait can then name exactly the loads it needs): behind the wave's last tile a
  // request fetches that tile once more and a pass stores nothing.
  TileFetch<BITS, QJL> f0, f1;
  const int count = (NT - wave + 3) / 4;        // tiles of this wave: wave, wave + 4, ...
  const int tok_last = 32 * (wave + 4 * (count - 1));
  int tok_r = 32 * wave, b_r = 0, end_r = n;                  // next tile to request: first token, block, end of the block
  int tok_w = 32 * wave, b_w = 0, end_w = n, r_w = rank_of(0), nwk = 0;   // next tile to work on
  __amdgpu_buffer_rsrc_t cfd = coef_buffer(0);
#define EOQ_SC_REQUEST(F)                    \
  if (tok_r >= end_r) {                      \
    ++b_r;                                   \
    end_r += n;                              \
    cfd = coef_buffer(b_r);                  \
  }                                          \
  request(F, tok_r, b_r, cfd);               \
  tok_r = min(tok_r + 128, tok_last);
#define EOQ_SC_WORK(F)                       \
  if (tok_w >= end_w) {                      \
    ++b_w;                                   \
    end_w += n;                              \
    r_w = rank_of(b_w);                      \
  }                                          \
  work(F, tok_w, b_w, r_w, nwk < count);     \
  tok_w = min(tok_w + 128, tok_last);        \
  ++nwk;
  EOQ_SC_REQUEST(f0)
  for (int it = 0; it < (count + 1) / 2; ++it) {
    EOQ_SC_REQUEST(f1)
    EOQ_SC_WORK(f0)
    EOQ_SC_REQUEST(f0)
    EOQ_SC_WORK(f1)
  }
#undef EOQ_SC_REQUEST
#undef EOQ_SC_WORK
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
#define EOQ_SCORES(BITS, NQ)                                                                                         \
  do {                                                                                                               \
    if (qjl)                                                                                                         \
      hipLaunchKernelGGL((eoq_scores_i8_kernel<BITS, true, NQ>), EOQ_SCORES_ARGS, L.phih, qjl->signs, qjl->norms); \
    else                                                                                                             \
      hipLaunchKernelGGL((eoq_scores_i8_kernel<BITS, false, NQ>), EOQ_SCORES_ARGS, (const uint16_t*)nullptr,      \
                         (const uint8_t*)nullptr, (const uint16_t*)nullptr);                                         \
  } while (0)
#define EOQ_SCORES_BITS(NQ)                 \
  switch (L.bits) {                         \
    case 1: EOQ_SCORES(1, NQ); break;    \
    case 2: EOQ_SCORES(2, NQ); break;    \
    case 3: EOQ_SCORES(3, NQ); break;    \
    default: EOQ_SCORES(4, NQ); break;   \
  }
  if (group <= 4) {
    EOQ_SCORES_BITS(2)
  } else {
    EOQ_SCORES_BITS(4)
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
