// Measured ceilings of the device the library runs on, to be quoted beside the datasheet peaks in benchmark
// reports: a plain device copy, a dependent-free fp64 FMA loop on the vector ALUs and loops of the matrix
// instructions the kernels use (f16 32x32x16, i8 16x16x64, f64 16x16x4).  Two instruction streams can also be run
// side by side, one on the first and one on the second wave of every SIMD, which shows whether the matrix pipeline
// runs in the shadow of vector work or takes turns with it.  Not part of the paper's method.
#include "eoq_device.h"
#include "eoq_internal.h"

namespace {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef double v4d __attribute__((ext_vector_type(4)));

enum Stream { S_NONE = 0, S_FMA64 = 1, S_MFMA_F16 = 2, S_MFMA_I8 = 3, S_MFMA_F64 = 4, S_VALU32 = 5 };

// work units of one iteration of a wave: flops (or integer operations) for the arithmetic streams, wave
// instructions for S_VALU32
__host__ __device__ constexpr double units_per_iter(int s) {
  return s == S_FMA64      ? 16.0 * 64 * 2
         : s == S_MFMA_F16 ? 4.0 * 32 * 32 * 16 * 2
         : s == S_MFMA_I8  ? 8.0 * 16 * 16 * 64 * 2
         : s == S_MFMA_F64 ? 8.0 * 16 * 16 * 4 * 2
         : s == S_VALU32   ? 16.0
                           : 0.0;
}

template <int S>
__device__ __forceinline__ void run_stream(int iters, int lane, double* sink) {
  if constexpr (S == S_FMA64) {
    double acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 1.0 + lane + i;
    const double m = 1.0 - 0x1.0p-30, a = 0x1.0p-40;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fma(acc[i], m, a);
    }
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i];
    if (s == 0.125) *sink = s;
  } else if constexpr (S == S_MFMA_F16) {
    v8h a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[i] = (_Float16)(0.001f * (lane + i));
      b[i] = (_Float16)(0.002f * (lane - i));
    }
    v16f acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[q][i] = 0.0f;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[q], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < 16; ++i) s += acc[q][i];
    if (s == 0.125f) *sink = s;
  } else if constexpr (S == S_MFMA_I8) {
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = 0x01020304 * (lane + i);
      b[i] = 0x04030201 * (lane - i);
    }
    v4i acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[q][i] = 0;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[q], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) s += acc[q][i];
    if (s == 0x7FFFFFF1) *sink = (double)s;
  } else if constexpr (S == S_MFMA_F64) {
    const double a = 1.0 + 0x1.0p-20 * lane, b = 1.0 - 0x1.0p-21 * lane;
    v4d acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[q][i] = 0.0;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[q], 0, 0, 0);
    }
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
      for (int i = 0; i < 4; ++i) s += acc[q][i];
    if (s == 0.125) *sink = s;
  } else if constexpr (S == S_VALU32) {
    uint32_t x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0x9E3779B9u * (lane + i + 1);
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = __builtin_amdgcn_alignbit(x[i], x[(i + 3) & 7], 7);
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) s ^= x[i];
    if (s == 0x12345u) *sink = (double)s;
  }
}

// 512 lanes: waves 0..3 (one per SIMD) run stream A, waves 4..7 (the second wave of every SIMD) stream B.  The launch
// asks for 96 KB of LDS per workgroup, so a compute unit holds one workgroup at a time: two waves per SIMD, no more.
constexpr int CEIL_LDS_BYTES = 96 * 1024;
template <int A, int B>
__global__ __launch_bounds__(1024) void eoq_ceiling_kernel(int iters, double* sink) {
  extern __shared__ char ceil_pad[];
  if (iters < 0) ceil_pad[threadIdx.x] = 0;   // never taken: keeps the allocation
  const int lane = threadIdx.x & 63;
  if (threadIdx.x < 256) run_stream<A>(iters, lane, sink);
  else run_stream<B>(iters, lane, sink);
}

// Memory streams.  Every workgroup walks contiguous chunks of 32 KB (chunk number += grid size), 16 bytes per lane
// and access, 4 KB per workgroup and step: on this device that order is 10-20 % faster than one grid-wide stride
// over the whole buffer (copy 5.4 against 4.8 TB/s, read 6.4 against 5.6, write 6.0 against 5.1), so it is the one
// quoted as the ceiling.  What lies beyond the last whole chunk is not touched (and not counted).
constexpr int STREAM_CHUNK_U4 = 2048;   // 32 KB
enum StreamMode { STREAM_READ = 0, STREAM_COPY = 1, STREAM_WRITE = 2 };
template <int MODE>
__global__ __launch_bounds__(256) void eoq_stream_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t chunks,
                                                         uint4* __restrict__ sink) {
  uint4 acc = make_uint4(threadIdx.x, blockIdx.x, 3u, 4u);
  for (size_t c = blockIdx.x; c < chunks; c += gridDim.x) {
#pragma unroll 4
    for (int t = 0; t < STREAM_CHUNK_U4 / 256; ++t) {
      const size_t i = c * STREAM_CHUNK_U4 + t * 256 + threadIdx.x;
      if constexpr (MODE == STREAM_WRITE) {
        dst[i] = acc;
      } else {
        const uint4 v = src[i];
        if constexpr (MODE == STREAM_COPY) {
          dst[i] = v;
        } else {   // the sum is kept so that the loads stay
          acc.x ^= v.x;
          acc.y ^= v.y;
          acc.z ^= v.z;
          acc.w ^= v.w;
        }
      }
    }
  }
  if (MODE == STREAM_READ && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u) sink[0] = acc;
}

template <int A, int B>
void launch_pair(int grid, int iters, double* sink, hipStream_t st, int waves_per_simd = 2) {
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&eoq_ceiling_kernel<A, B>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, CEIL_LDS_BYTES);
  hipLaunchKernelGGL((eoq_ceiling_kernel<A, B>), dim3(grid), dim3(256 * waves_per_simd), CEIL_LDS_BYTES, st, iters, sink);
}

}  // namespace

extern "C" eoq_status eoq_ceiling(eoq_ctx* ctx, int kind, void* device_buf, size_t buf_bytes, int iters, double* out) {
  if (!ctx || !out) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) {
    ctx->err = "context was created without a HIP device";
    return EOQ_ERR_HIP;
  }
  if (!device_buf || (reinterpret_cast<uintptr_t>(device_buf) & 15u) || buf_bytes < 65536 || iters < 1) {
    ctx->err = "eoq_ceiling: null or misaligned buffer, or no iterations";
    return EOQ_ERR_ARG;
  }
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, ctx->device) != hipSuccess) return EOQ_ERR_HIP;
  const int cus = prop.multiProcessorCount;
  const int grid = 4 * cus;   // four rounds of one workgroup per compute unit
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return EOQ_ERR_HIP;
  hipStream_t st = nullptr;
  double* sink = static_cast<double*>(device_buf);
  int sa = S_NONE, sb = S_NONE, waves = 2;
  const int reps = 3;
  double units_a = 0.0, units_b = 0.0;
  for (int rep = 0; rep < reps; ++rep) {   // the last repetition is the one timed
    if (rep == reps - 1) (void)hipEventRecord(e0, st);
    switch (kind) {
      case 0: {   // copy: first half of the buffer to the second
        const size_t chunks = buf_bytes / 2 / (STREAM_CHUNK_U4 * 16);
        const size_t half = chunks * STREAM_CHUNK_U4 * 16;
        hipLaunchKernelGGL(eoq_stream_kernel<STREAM_COPY>, dim3(cus * 8), dim3(256), 0, st, static_cast<const uint4*>(device_buf),
                           reinterpret_cast<uint4*>(static_cast<char*>(device_buf) + half), chunks, static_cast<uint4*>(nullptr));
        units_a = 2.0 * (double)half;
        break;
      }
      case 6: {   // read only (a match of the running sum, which does not occur, would write 16 bytes at the front)
        const size_t chunks = buf_bytes / (STREAM_CHUNK_U4 * 16);
        hipLaunchKernelGGL(eoq_stream_kernel<STREAM_READ>, dim3(cus * 8), dim3(256), 0, st, static_cast<const uint4*>(device_buf),
                           static_cast<uint4*>(nullptr), chunks, static_cast<uint4*>(device_buf));
        units_a = (double)chunks * STREAM_CHUNK_U4 * 16;
        break;
      }
      case 7: {   // write only
        const size_t chunks = buf_bytes / (STREAM_CHUNK_U4 * 16);
        hipLaunchKernelGGL(eoq_stream_kernel<STREAM_WRITE>, dim3(cus * 8), dim3(256), 0, st, static_cast<const uint4*>(nullptr),
                           static_cast<uint4*>(device_buf), chunks, static_cast<uint4*>(nullptr));
        units_a = (double)chunks * STREAM_CHUNK_U4 * 16;
        break;
      }
      case 1: sa = S_FMA64; launch_pair<S_FMA64, S_FMA64>(grid, iters, sink, st); sb = sa; break;
      case 2: sa = S_MFMA_F16; launch_pair<S_MFMA_F16, S_MFMA_F16>(grid, iters, sink, st); sb = sa; break;
      case 3: sa = S_MFMA_I8; launch_pair<S_MFMA_I8, S_MFMA_I8>(grid, iters, sink, st); sb = sa; break;
      case 4: sa = S_MFMA_F64; launch_pair<S_MFMA_F64, S_MFMA_F64>(grid, iters, sink, st); sb = sa; break;
      case 5: sa = S_VALU32; launch_pair<S_VALU32, S_VALU32>(grid, iters, sink, st); sb = sa; break;
      case 10: sa = S_MFMA_F64; sb = S_FMA64; launch_pair<S_MFMA_F64, S_FMA64>(grid, iters, sink, st); break;
      case 11: sa = S_MFMA_I8; sb = S_VALU32; launch_pair<S_MFMA_I8, S_VALU32>(grid, iters, sink, st); break;
      case 12: sa = S_MFMA_F64; sb = S_VALU32; launch_pair<S_MFMA_F64, S_VALU32>(grid, iters, sink, st); break;
      case 13: sa = S_FMA64; sb = S_VALU32; launch_pair<S_FMA64, S_VALU32>(grid, iters, sink, st); break;
      case 14: sa = S_MFMA_F16; sb = S_FMA64; launch_pair<S_MFMA_F16, S_FMA64>(grid, iters, sink, st); break;
      case 15: sa = S_MFMA_I8; sb = S_FMA64; launch_pair<S_MFMA_I8, S_FMA64>(grid, iters, sink, st); break;
      case 21: sa = S_FMA64; launch_pair<S_FMA64, S_NONE>(grid, iters, sink, st); break;
      case 24: sa = S_MFMA_F64; launch_pair<S_MFMA_F64, S_NONE>(grid, iters, sink, st); break;
      case 23: sa = S_MFMA_I8; launch_pair<S_MFMA_I8, S_NONE>(grid, iters, sink, st); break;
      case 25: sa = S_VALU32; launch_pair<S_VALU32, S_NONE>(grid, iters, sink, st); break;
      case 31: case 32: case 33: case 34:   // f64 FMA on 1 .. 4 waves per SIMD
        sa = S_FMA64; sb = S_FMA64; waves = kind - 30;
        launch_pair<S_FMA64, S_FMA64>(grid, iters, sink, st, waves);
        break;
      case 41: case 42: case 43: case 44:   // 32-bit vector instructions on 1 .. 4 waves per SIMD
        sa = S_VALU32; sb = S_VALU32; waves = kind - 40;
        launch_pair<S_VALU32, S_VALU32>(grid, iters, sink, st, waves);
        break;
      default:
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        ctx->err = "eoq_ceiling: unknown kind";
        return EOQ_ERR_UNSUPPORTED;
    }
  }
  (void)hipEventRecord(e1, st);
  hipError_t e = hipEventSynchronize(e1);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  if (kind != 0 && kind != 6 && kind != 7) {
    // per launch: `grid` workgroups, four waves per stream
    units_a = units_per_iter(sa) * 4.0 * grid * iters;
    units_b = units_per_iter(sb) * 4.0 * (waves - 1) * grid * iters;
  }
  out[0] = ms;
  out[1] = units_a;
  out[2] = units_b;
  out[3] = (double)cus;
  return EOQ_OK;
}
