// Attention weights and attention output on compressed values (Sec. 2.1: softmax(Q K^T / sqrt(d)) V with V
// replaced by its reconstruction x_hat_t = rho_t Pi^T z_hat_t + C_t V_r, Alg. 1 line 6 plus the low-rank part).
//
// out_h = sum_t w_ht x_hat_t is split the way the scores are (Remark 6.5): the rotation is linear and shared by all
// blocks, so the codebook term is summed in the rotated domain over ALL tokens of the head,
//     a_h[c] = sum_t (w_ht rho_t / sqrt(d)) centroid[code_tc],
// and rotated back once per head, and the low-rank term is (sum_t w_ht C_t) V_r per block.  Nothing of V is
// materialised.  Two kernels: partial sums per run of blocks (fixed order inside a run), then a finishing kernel that
// adds the runs in order and applies Pi^T: the result does not depend on scheduling.
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

using namespace eoqdev;

constexpr int D = EOQ_D;
constexpr int THREADS = 256;
constexpr int MAXG = 8;      // query heads per KV head
constexpr int CHUNK = 128;   // tokens staged per pass (n is a multiple of 128)

// One workgroup: blocks [blockIdx.x * run, ...) of (sequence, KV head) blockIdx.y.
// Codebook term: lane (cg, tg) = (tid % 32, tid / 32) owns the four coordinates 4 cg .. 4 cg + 3 and the tokens tg,
// tg + 8, ... of every chunk.  Per token it reads one byte of every bit-plane, and for codes of up to 2 bits one entry
// of a 256-entry table indexed by (nibble of plane 0 | nibble of plane 1 << 4) gives the four centroids at once; the
// weights of the token's heads are one or two 16-byte reads shared by the whole token group; 4 x GH multiply-adds.
// Low-rank term: lane (c, th) = (tid % 128, tid / 128) owns output coordinate c.
// GH: heads accumulated per lane (4 when the group has at most four query heads: half the multiply-adds and LDS reads).
template <int BITS, int GH>
__global__ __launch_bounds__(THREADS) void eoq_attend_partial_kernel(
    int n, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, int64_t block_capacity, int64_t weight_stride,
    int run, const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const float* __restrict__ weights, float* __restrict__ partial) {
  constexpr int ROWB = BITS * D / 8;
  // staging of a chunk; after the last chunk the same memory takes the four waves' sums of the codebook term
  constexpr int STAGE_BYTES = CHUNK * ROWB + 2 * CHUNK * MAXG * 4 + EOQ_RMAX_CAP * CHUNK * 2;
  constexpr int FOLD_BYTES = 4 * GH * D * 4;
  __shared__ __align__(16) uint8_t stage_s[STAGE_BYTES > FOLD_BYTES ? STAGE_BYTES : FOLD_BYTES];
  uint8_t* code_s = stage_s;
  float* wr_s = reinterpret_cast<float*>(stage_s + CHUNK * ROWB);                        // [t][h]: w_ht rho_t / sqrt(d)
  float* w_s = wr_s + CHUNK * MAXG;                                                      // [h][t]: w_ht
  uint16_t* cf_s = reinterpret_cast<uint16_t*>(w_s + MAXG * CHUNK);                      // [i][t]: stored coefficients C_ti of the chunk
  float* fold4_s = reinterpret_cast<float*>(stage_s);                                    // [wave][h][c]
  __shared__ __align__(16) float4 cen4_s[BITS <= 2 ? 256 : 1];
  __shared__ float cent_s[1 << BITS];
  __shared__ float bsum_s[4 * MAXG * EOQ_RMAX_CAP];      // [token segment][h][i]: sum_t w_ht C_ti of the current block
  __shared__ float fold_s[MAXG * D];

  const int tid = threadIdx.x;
  const int c = tid & (D - 1), th = tid >> 7;
  const int cg = tid & 31, tg = tid >> 5;
  const size_t sg = blockIdx.y;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  if (tid < (1 << BITS)) cent_s[tid] = tab[tid];
  if constexpr (BITS <= 2) {
    const int n0 = tid & 15, n1 = tid >> 4;
    float cv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) cv[e] = tab[((n0 >> e) & 1) | ((BITS == 2) ? (((n1 >> e) & 1) << 1) : 0)];
    cen4_s[tid] = make_float4(cv[0], cv[1], cv[2], cv[3]);
  }

  float rot[GH][4], lin[GH];
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    lin[h] = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) rot[h][e] = 0.0f;
  }

  // What a lane fetches of a chunk of 128 tokens; the next chunk's (of this block or the next) is requested before
  // this one is worked on, so the loads travel during the arithmetic instead of in front of a barrier.
  constexpr int NC = (CHUNK * ROWB / 16 + THREADS - 1) / THREADS;   // 16-byte pieces of the codes per lane
  struct Fetch {
    uint4 code[NC];
    float w[4];      // weights of heads th, 2 + th, 4 + th, 6 + th at token tid % 128
    uint16_t rho;    // stored norm of that token
    uint4 cf[2];     // stored coefficients: piece tid + 256 k of the chunk's [component][token] rows
  };
  __shared__ int rank_s[16];
  const int64_t j_begin = (int64_t)blockIdx.x * run;
  const int64_t j_end = min(j_begin + run, blocks_per_head);
  if (tid < (int)(j_end - j_begin)) rank_s[tid] = min(max(rank_in[sg * (size_t)block_capacity + j_begin + tid], 0), r_max);
  __syncthreads();
  auto fetch = [&](Fetch& f, int64_t jb, int t0) __attribute__((always_inline)) {
    const size_t blk = sg * (size_t)block_capacity + jb;
    const int r = rank_s[jb - j_begin];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
      const int e = tid + THREADS * k;
      f.code[k] = (e < CHUNK * ROWB / 16) ? reinterpret_cast<const uint4*>(codes + (blk * (size_t)n + t0) * ROWB)[e] : make_uint4(0u, 0u, 0u, 0u);
    }
    const int t = tid & (CHUNK - 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int h = 2 * k + th;
      f.w[k] = (h < group) ? weights[(sq * n_q_heads + kv * group + h) * (size_t)weight_stride + (size_t)jb * n + t0 + t] : 0.0f;
    }
    f.rho = norms[blk * (size_t)n + t0 + t];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int e = tid + THREADS * k, i = e >> 4;
      f.cf[k] = (i < r) ? *reinterpret_cast<const uint4*>(lfac + (blk * r_max + i) * (size_t)n + t0 + 8 * (e & 15)) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  Fetch cur, nxt;
  if (j_begin < j_end) fetch(cur, j_begin, 0);
  for (int64_t jb = j_begin; jb < j_end; ++jb) {
    const size_t blk = sg * (size_t)block_capacity + jb;
    const int r = rank_s[jb - j_begin];
    // low-rank weights of this block: lane (segment, i, h) = (tid / 64, (tid / 8) % 8, tid % 8) sums the 32 tokens
    // 32 segment .. of every chunk for the components i, i + 8, ... and head h
    const int bs = tid >> 6, bi = (tid >> 3) & 7, bh = tid & 7;
    float bacc[EOQ_RMAX_CAP / 8];
#pragma unroll
    for (int g = 0; g < EOQ_RMAX_CAP / 8; ++g) bacc[g] = 0.0f;
    for (int t0 = 0; t0 < n; t0 += CHUNK) {
      __syncthreads();  // the previous chunk has been consumed
      // stage the chunk: codes, weights, weights times norm, coefficients
#pragma unroll
      for (int k = 0; k < NC; ++k) {
        const int e = tid + THREADS * k;
        if (e < CHUNK * ROWB / 16) reinterpret_cast<uint4*>(code_s)[e] = cur.code[k];
      }
      {
        const int t = tid & (CHUNK - 1);
        const float rs = half_bits_to_float(cur.rho) * inv_sqrt_d;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int h = 2 * k + th;
          w_s[h * CHUNK + t] = cur.w[k];
          wr_s[t * MAXG + h] = cur.w[k] * rs;
        }
      }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int e = tid + THREADS * k;
        if ((e >> 4) < r) reinterpret_cast<uint4*>(cf_s)[e] = cur.cf[k];
      }
      // the next chunk's bytes are requested here
      {
        const bool last_chunk = t0 + CHUNK >= n;
        const int64_t jn = last_chunk ? jb + 1 : jb;
        if (jn < j_end) fetch(nxt, jn, last_chunk ? 0 : t0 + CHUNK);
      }
      __syncthreads();
      // codebook term: this lane's four coordinates, every eighth token of the chunk
      const int cbyte = cg >> 1, cshift = 4 * (cg & 1);
#pragma unroll 4
      for (int t = tg; t < CHUNK; t += 8) {
        float cv[4];
        if constexpr (BITS <= 2) {
          uint32_t idx = ((uint32_t)code_s[t * ROWB + cbyte] >> cshift) & 0xFu;
          if constexpr (BITS == 2) idx |= (((uint32_t)code_s[t * ROWB + 16 + cbyte] >> cshift) & 0xFu) << 4;
          const float4 c4 = cen4_s[idx];
          cv[0] = c4.x; cv[1] = c4.y; cv[2] = c4.z; cv[3] = c4.w;
        } else {
          uint32_t nib[BITS];
#pragma unroll
          for (int p = 0; p < BITS; ++p) nib[p] = ((uint32_t)code_s[t * ROWB + 16 * p + cbyte] >> cshift) & 0xFu;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            uint32_t idx = 0;
#pragma unroll
            for (int p = 0; p < BITS; ++p) idx |= ((nib[p] >> e) & 1u) << p;
            cv[e] = cent_s[idx];
          }
        }
        const float4 wa = *reinterpret_cast<const float4*>(wr_s + t * MAXG);
        const float wv[4] = {wa.x, wa.y, wa.z, wa.w};
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) rot[h][e] = fmaf(wv[h], cv[e], rot[h][e]);
        if constexpr (GH == 8) {
          const float4 wb = *reinterpret_cast<const float4*>(wr_s + t * MAXG + 4);
          const float wu[4] = {wb.x, wb.y, wb.z, wb.w};
#pragma unroll
          for (int h = 0; h < 4; ++h)
#pragma unroll
            for (int e = 0; e < 4; ++e) rot[4 + h][e] = fmaf(wu[h], cv[e], rot[4 + h][e]);
        }
      }
      // low-rank weights: components bi + 8 g, head bh, the segment's 32 tokens, 8 per load
#pragma unroll
      for (int g = 0; g < EOQ_RMAX_CAP / 8; ++g) {
        if (8 * g < r) {   // uniform
          const int i = bi + 8 * g;
          if (i < r) {
            const uint16_t* crow = cf_s + i * CHUNK;
#pragma unroll
            for (int t = 32 * bs; t < 32 * bs + 32; t += 8) {
              float cf[8];
              load8(crow, EOQ_F16, t, cf);
              const float4 wa = *reinterpret_cast<const float4*>(w_s + bh * CHUNK + t);
              const float4 wb = *reinterpret_cast<const float4*>(w_s + bh * CHUNK + t + 4);
              bacc[g] = fmaf(wa.x, cf[0], bacc[g]);
              bacc[g] = fmaf(wa.y, cf[1], bacc[g]);
              bacc[g] = fmaf(wa.z, cf[2], bacc[g]);
              bacc[g] = fmaf(wa.w, cf[3], bacc[g]);
              bacc[g] = fmaf(wb.x, cf[4], bacc[g]);
              bacc[g] = fmaf(wb.y, cf[5], bacc[g]);
              bacc[g] = fmaf(wb.z, cf[6], bacc[g]);
              bacc[g] = fmaf(wb.w, cf[7], bacc[g]);
            }
          }
        }
      }
      cur = nxt;
    }
    // low-rank term of the block: lin_h[c] += sum_i bsum[h][i] V[i][c]; the two lane halves take alternate components
    __syncthreads();
#pragma unroll
    for (int g = 0; g < EOQ_RMAX_CAP / 8; ++g) bsum_s[(bs * MAXG + bh) * EOQ_RMAX_CAP + bi + 8 * g] = bacc[g];
    __syncthreads();
    for (int i = th; i < r; i += 2) {
      const float v = half_bits_to_float(rfac[(blk * r_max + i) * D + c]);
#pragma unroll
      for (int h = 0; h < GH; ++h) {
        // the four token segments in order
        const float bsum = ((bsum_s[(0 * MAXG + h) * EOQ_RMAX_CAP + i] + bsum_s[(1 * MAXG + h) * EOQ_RMAX_CAP + i]) +
                            bsum_s[(2 * MAXG + h) * EOQ_RMAX_CAP + i]) + bsum_s[(3 * MAXG + h) * EOQ_RMAX_CAP + i];
        lin[h] = fmaf(bsum, v, lin[h]);
      }
    }
  }
  // The codebook term: the two token groups of a wave meet in registers (lane ^ 32: both get the same sum), the four
  // waves through LDS, added in wave order.  The low-rank term: the two lane halves through LDS.  Then the partial sums
  // of this run are written: [rot | lin][h][c].
  __syncthreads();   // the staging memory is free
#pragma unroll
  for (int h = 0; h < GH; ++h)
#pragma unroll
    for (int e = 0; e < 4; ++e) rot[h][e] += __shfl_xor(rot[h][e], 32, 64);
  if ((tid & 32) == 0) {
#pragma unroll
    for (int h = 0; h < GH; ++h)
      *reinterpret_cast<float4*>(fold4_s + ((tid >> 6) * GH + h) * D + 4 * cg) = make_float4(rot[h][0], rot[h][1], rot[h][2], rot[h][3]);
  }
  if (th == 1) {
#pragma unroll
    for (int h = 0; h < GH; ++h) fold_s[h * D + c] = lin[h];
  }
  __syncthreads();
  if (th == 0) {
    float* dst = partial + ((sg * gridDim.x + blockIdx.x) * 2 * MAXG) * D;
#pragma unroll
    for (int h = 0; h < MAXG; ++h) {   // heads past GH are written as zeros: the finishing kernel sums all eight
      float rsum = 0.0f, lsum = 0.0f;
      if (h < GH) {
        const int hh = h < GH ? h : 0;
        rsum = ((fold4_s[(0 * GH + hh) * D + c] + fold4_s[(1 * GH + hh) * D + c]) + fold4_s[(2 * GH + hh) * D + c]) + fold4_s[(3 * GH + hh) * D + c];
        lsum = lin[hh] + fold_s[hh * D + c];
      }
      dst[h * D + c] = rsum;
      dst[(MAXG + h) * D + c] = lsum;
    }
  }
}

// out[s][h][j] = sum_c Pi[c][j] a_h[c] + lin_h[j], the runs added in order.  One workgroup per (sequence, KV head,
// query head of the group): lane (j, half) sums the rotated-domain partials (half 0) or the low-rank partials (half 1)
// of the runs, one load per run with sixteen in flight; the rotation back and the tail are split between the halves
// (coordinates 64 half .. 64 half + 63, tail tokens of parity half) and met through LDS in a fixed order.
// With tail_len > 0 the uncompressed binary16 tail values are added: + sum_t weights[.., tail_offset + t] tail[t].
__global__ __launch_bounds__(THREADS) void eoq_attend_finish_kernel(int n_kv_heads, int group, int runs,
                                                                    const float* __restrict__ pi,
                                                                    const float* __restrict__ partial,
                                                                    float* __restrict__ out,
                                                                    const float* __restrict__ weights,
                                                                    int64_t weight_stride, int64_t tail_offset,
                                                                    const uint16_t* __restrict__ tail,
                                                                    int64_t tail_capacity, int tail_len) {
  __shared__ float a_s[D];
  __shared__ float meet_s[D];
  const int tid = threadIdx.x;
  const int j = tid & (D - 1), half = tid >> 7;
  const size_t sg = blockIdx.x;
  const int h = blockIdx.y;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  float sum = 0.0f;
  {
    const float* src = partial + (sg * runs * 2 * MAXG + (size_t)(half * MAXG + h)) * D + j;
#pragma unroll 16
    for (int rn = 0; rn < runs; ++rn) sum += src[(size_t)rn * 2 * MAXG * D];
  }
  if (half == 0) a_s[j] = sum;
  __syncthreads();
  float acc = (half == 1) ? sum : 0.0f;   // half 1 starts from the low-rank term
#pragma unroll 16
  for (int cc = 64 * half; cc < 64 * half + 64; ++cc) acc = fmaf(pi[cc * D + j], a_s[cc], acc);
  if (tail_len > 0) {
    const float* wrow = weights + (sq * n_q_heads + kv * group + h) * (size_t)weight_stride + tail_offset;
#pragma unroll 8
    for (int t = half; t < tail_len; t += 2)
      acc = fmaf(wrow[t], half_bits_to_float(tail[(sg * (size_t)tail_capacity + t) * D + j]), acc);
  }
  if (half == 1) meet_s[j] = acc;
  __syncthreads();
  if (half == 0) out[(sq * n_q_heads + kv * group + h) * D + j] = acc + meet_s[j];
}

// Row-wise softmax in place (the attention weights of Sec. 2.1): one workgroup per row, three passes; 16-byte
// accesses when the row allows them (VEC), several of them in flight per lane.
template <bool VEC>
__global__ __launch_bounds__(THREADS) void eoq_softmax_kernel(float* __restrict__ x, int64_t len, int64_t stride) {
  __shared__ float red[THREADS / 64];
  __shared__ float bcast;
  float* row = x + blockIdx.x * (size_t)stride;
  const int tid = threadIdx.x;
  constexpr int W = VEC ? 4 : 1;
  const int64_t items = len / W;   // VEC: len is a multiple of 4
  float m = -INFINITY;
#pragma unroll 4
  for (int64_t e = tid; e < items; e += THREADS) {
    if constexpr (VEC) {
      const float4 v = reinterpret_cast<const float4*>(row)[e];
      m = fmaxf(fmaxf(m, fmaxf(v.x, v.y)), fmaxf(v.z, v.w));
    } else {
      m = fmaxf(m, row[e]);
    }
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) m = fmaxf(m, __shfl_xor(m, s, 64));
  if ((tid & 63) == 0) red[tid >> 6] = m;
  __syncthreads();
  if (tid == 0) bcast = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  m = bcast;
  float sum = 0.0f;
#pragma unroll 4
  for (int64_t e = tid; e < items; e += THREADS) {
    if constexpr (VEC) {
      float4 v = reinterpret_cast<const float4*>(row)[e];
      v.x = expf(v.x - m);
      v.y = expf(v.y - m);
      v.z = expf(v.z - m);
      v.w = expf(v.w - m);
      reinterpret_cast<float4*>(row)[e] = v;
      sum += (v.x + v.y) + (v.z + v.w);
    } else {
      const float v = expf(row[e] - m);
      row[e] = v;
      sum += v;
    }
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) sum += __shfl_xor(sum, s, 64);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) bcast = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  const float inv = 1.0f / bcast;
#pragma unroll 4
  for (int64_t e = tid; e < items; e += THREADS) {
    if constexpr (VEC) {
      float4 v = reinterpret_cast<const float4*>(row)[e];
      v.x *= inv;
      v.y *= inv;
      v.z *= inv;
      v.w *= inv;
      reinterpret_cast<float4*>(row)[e] = v;
    } else {
      row[e] *= inv;
    }
  }
}

}  // namespace

int64_t eoq_attend_runs(int64_t sg_total, int64_t blocks_per_head, int* run_out) {
  // blocks per workgroup: up to 16, shorter when that leaves fewer than ~8 workgroups per compute unit
  int64_t run = (sg_total * blocks_per_head) / 2048;
  run = run < 1 ? 1 : (run > 16 ? 16 : run);
  *run_out = (int)run;
  return (blocks_per_head + run - 1) / run;
}

hipError_t eoq_launch_attend(const EoqLaunch& L, eoq_packed values, int64_t n_seq, int n_kv_heads,
                             int64_t blocks_per_head, int64_t block_capacity, const float* weights,
                             int64_t weight_stride, int n_q_heads, float* out, float* partial, const void* tail_fp16,
                             int64_t tail_capacity, int tail_len) {
  const uint16_t* tail = static_cast<const uint16_t*>(tail_fp16);
  const int64_t tail_offset = blocks_per_head * L.n;
  const int64_t sg_total = n_seq * n_kv_heads;
  const int group = n_q_heads / n_kv_heads;
  if (L.ev) (void)hipEventRecord(L.ev[8], L.stream);
  if (blocks_per_head == 0) {  // nothing stored yet: the finishing kernel with no runs writes zeros
    hipLaunchKernelGGL(eoq_attend_finish_kernel, dim3((unsigned)sg_total, (unsigned)group), dim3(THREADS), 0, L.stream, n_kv_heads, group, 0,
                       L.pi, partial, out, weights, weight_stride, tail_offset, tail, tail_capacity, tail_len);
    if (L.ev) (void)hipEventRecord(L.ev[9], L.stream);
    return hipGetLastError();
  }
  int run = 1;
  const int64_t runs = eoq_attend_runs(sg_total, blocks_per_head, &run);
  if (sg_total > 65535 || runs > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)runs, (unsigned)sg_total), block(THREADS);
#define EOQ_ATTEND(BITS)                                                                                              \
  do {                                                                                                                \
    if (group <= 4)                                                                                                   \
      hipLaunchKernelGGL((eoq_attend_partial_kernel<BITS, 4>), grid, block, 0, L.stream, L.n, L.r_max, n_kv_heads,    \
                         group, blocks_per_head, block_capacity, weight_stride, run, L.tab, values.codes,             \
                         values.norms, values.rank, values.lfac, values.rfac, weights, partial);                      \
    else                                                                                                              \
      hipLaunchKernelGGL((eoq_attend_partial_kernel<BITS, 8>), grid, block, 0, L.stream, L.n, L.r_max, n_kv_heads,    \
                         group, blocks_per_head, block_capacity, weight_stride, run, L.tab, values.codes,             \
                         values.norms, values.rank, values.lfac, values.rfac, weights, partial);                      \
  } while (0)
  switch (L.bits) {
    case 1: EOQ_ATTEND(1); break;
    case 2: EOQ_ATTEND(2); break;
    case 3: EOQ_ATTEND(3); break;
    default: EOQ_ATTEND(4); break;
  }
#undef EOQ_ATTEND
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(eoq_attend_finish_kernel, dim3((unsigned)sg_total, (unsigned)group), block, 0, L.stream, n_kv_heads, group,
                     (int)runs, L.pi, partial, out, weights, weight_stride, tail_offset, tail, tail_capacity, tail_len);
  if (L.ev) (void)hipEventRecord(L.ev[9], L.stream);
  return hipGetLastError();
}

hipError_t eoq_launch_softmax(const EoqLaunch& L, float* x, int64_t rows, int64_t len, int64_t stride) {
  if (L.ev) (void)hipEventRecord(L.ev[10], L.stream);
  if (((len | stride) & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0)
    hipLaunchKernelGGL(eoq_softmax_kernel<true>, dim3((unsigned)rows), dim3(THREADS), 0, L.stream, x, len, stride);
  else
    hipLaunchKernelGGL(eoq_softmax_kernel<false>, dim3((unsigned)rows), dim3(THREADS), 0, L.stream, x, len, stride);
  if (L.ev) (void)hipEventRecord(L.ev[11], L.stream);
  return hipGetLastError();
}
