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

// One workgroup: blocks [blockIdx.x * run, ...) of (sequence, KV head) blockIdx.y.  Lane (c, th) = (tid % 128,
// tid / 128) owns coordinate c and the tokens of parity-half th of every chunk.
// GH: heads accumulated per lane (4 when the group has at most four query heads: half the multiply-adds and LDS reads).
template <int BITS, int GH>
__global__ __launch_bounds__(THREADS) void eoq_attend_partial_kernel(
    int n, int r_max, int n_kv_heads, int group, int64_t blocks_per_head, int64_t block_capacity, int64_t weight_stride,
    int run, const float* __restrict__ tab, const uint8_t* __restrict__ codes, const uint16_t* __restrict__ norms,
    const int32_t* __restrict__ rank_in, const uint16_t* __restrict__ lfac, const uint16_t* __restrict__ rfac,
    const float* __restrict__ weights, float* __restrict__ partial) {
  constexpr int ROWB = BITS * D / 8;
  __shared__ __align__(16) uint8_t code_s[CHUNK * ROWB];
  __shared__ __align__(16) float wr_s[CHUNK * MAXG];     // [t][h]: w_ht rho_t / sqrt(d)
  __shared__ __align__(16) float w_s[MAXG * CHUNK];      // [h][t]: w_ht
  __shared__ __align__(16) uint16_t cf_s[EOQ_RMAX_CAP * CHUNK];   // [i][t]: stored coefficients C_ti of the chunk
  __shared__ float cent_s[1 << BITS];
  __shared__ float bsum_s[MAXG * EOQ_RMAX_CAP];          // [h][i]: sum_t w_ht C_ti of the current block
  __shared__ float fold_s[2 * MAXG * D];

  const int tid = threadIdx.x;
  const int c = tid & (D - 1), th = tid >> 7;
  const size_t sg = blockIdx.y;
  const size_t sq = sg / n_kv_heads, kv = sg % n_kv_heads;
  const int n_q_heads = n_kv_heads * group;
  const float inv_sqrt_d = 1.0f / sqrtf((float)D);
  if (tid < (1 << BITS)) cent_s[tid] = tab[tid];

  float rot[GH], lin[GH];
#pragma unroll
  for (int h = 0; h < GH; ++h) rot[h] = lin[h] = 0.0f;

  const int64_t j_end = min((int64_t)(blockIdx.x + 1) * run, blocks_per_head);
  for (int64_t jb = (int64_t)blockIdx.x * run; jb < j_end; ++jb) {
    const size_t blk = sg * (size_t)block_capacity + jb;
    const int r = min(max(rank_in[blk], 0), r_max);
    // low-rank weights of this block: lane (i, h) = (tid / 8, tid % 8)
    const int bi = tid >> 3, bh = tid & 7;
    float bacc = 0.0f;
    for (int t0 = 0; t0 < n; t0 += CHUNK) {
      __syncthreads();  // the previous chunk has been consumed
      // stage the chunk: codes, weights, weights times norm
      for (int e = tid; e < CHUNK * ROWB / 16; e += THREADS)
        reinterpret_cast<uint4*>(code_s)[e] = reinterpret_cast<const uint4*>(codes + (blk * (size_t)n + t0) * ROWB)[e];
      for (int e = tid; e < group * CHUNK; e += THREADS) {
        const int h = e / CHUNK, t = e - h * CHUNK;
        const float w = weights[(sq * n_q_heads + kv * group + h) * (size_t)weight_stride + (size_t)jb * n + t0 + t];
        const float rho = half_bits_to_float(norms[blk * (size_t)n + t0 + t]);
        w_s[h * CHUNK + t] = w;
        wr_s[t * MAXG + h] = w * rho * inv_sqrt_d;
      }
      for (int e = tid; e < r * (CHUNK / 8); e += THREADS) {
        const int i = e / (CHUNK / 8), seg = e - i * (CHUNK / 8);
        reinterpret_cast<uint4*>(cf_s)[e] = *reinterpret_cast<const uint4*>(lfac + (blk * r_max + i) * (size_t)n + t0 + 8 * seg);
      }
      if (group < MAXG)
        for (int e = tid; e < (MAXG - group) * CHUNK; e += THREADS) {
          const int h = group + e / CHUNK, t = e % CHUNK;
          w_s[h * CHUNK + t] = 0.0f;
          wr_s[t * MAXG + h] = 0.0f;
        }
      __syncthreads();
      // codebook term: this lane's coordinate, half of the chunk's tokens
      const int word = (c >> 5) * 4, bit = c & 31;
#pragma unroll 4
      for (int t = th * (CHUNK / 2); t < (th + 1) * (CHUNK / 2); ++t) {
        uint32_t idx = 0;
#pragma unroll
        for (int p = 0; p < BITS; ++p) {
          const uint32_t w32 = *reinterpret_cast<const uint32_t*>(code_s + t * ROWB + p * 16 + word);
          idx |= ((w32 >> bit) & 1u) << p;
        }
        const float cv = cent_s[idx];
        const float4 wa = *reinterpret_cast<const float4*>(wr_s + t * MAXG);
        rot[0] = fmaf(wa.x, cv, rot[0]);
        rot[1] = fmaf(wa.y, cv, rot[1]);
        rot[2] = fmaf(wa.z, cv, rot[2]);
        rot[3] = fmaf(wa.w, cv, rot[3]);
        if constexpr (GH == 8) {
          const float4 wb = *reinterpret_cast<const float4*>(wr_s + t * MAXG + 4);
          rot[4] = fmaf(wb.x, cv, rot[4]);
          rot[5] = fmaf(wb.y, cv, rot[5]);
          rot[6] = fmaf(wb.z, cv, rot[6]);
          rot[7] = fmaf(wb.w, cv, rot[7]);
        }
      }
      // low-rank weights: component bi, head bh, 8 tokens per load
      if (bi < r) {
        const uint16_t* crow = cf_s + bi * CHUNK;
#pragma unroll 4
        for (int t = 0; t < CHUNK; t += 8) {
          float cf[8];
          load8(crow, EOQ_F16, t, cf);
          const float4 wa = *reinterpret_cast<const float4*>(w_s + bh * CHUNK + t);
          const float4 wb = *reinterpret_cast<const float4*>(w_s + bh * CHUNK + t + 4);
          bacc = fmaf(wa.x, cf[0], bacc);
          bacc = fmaf(wa.y, cf[1], bacc);
          bacc = fmaf(wa.z, cf[2], bacc);
          bacc = fmaf(wa.w, cf[3], bacc);
          bacc = fmaf(wb.x, cf[4], bacc);
          bacc = fmaf(wb.y, cf[5], bacc);
          bacc = fmaf(wb.z, cf[6], bacc);
          bacc = fmaf(wb.w, cf[7], bacc);
        }
      }
    }
    // low-rank term of the block: lin_h[c] += sum_i bsum[h][i] V[i][c]; the two lane halves take alternate components
    __syncthreads();
    bsum_s[bh * EOQ_RMAX_CAP + bi] = bacc;
    __syncthreads();
    for (int i = th; i < r; i += 2) {
      const float v = half_bits_to_float(rfac[(blk * r_max + i) * D + c]);
#pragma unroll
      for (int h = 0; h < GH; ++h) lin[h] = fmaf(bsum_s[h * EOQ_RMAX_CAP + i], v, lin[h]);
    }
  }
  // fold the two lane halves and write the partial sums of this run: [rot | lin][h][c]
  __syncthreads();
  if (th == 1) {
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      fold_s[h * D + c] = rot[h];
      fold_s[(MAXG + h) * D + c] = lin[h];
    }
  }
  __syncthreads();
  if (th == 0) {
    float* dst = partial + ((sg * gridDim.x + blockIdx.x) * 2 * MAXG) * D;
#pragma unroll
    for (int h = 0; h < MAXG; ++h) {   // heads past GH are written as zeros: the finishing kernel sums all eight
      dst[h * D + c] = (h < GH) ? rot[h < GH ? h : 0] + fold_s[h * D + c] : 0.0f;
      dst[(MAXG + h) * D + c] = (h < GH) ? lin[h < GH ? h : 0] + fold_s[(MAXG + h) * D + c] : 0.0f;
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
