// Host side of the eOptShrinkQ library: context, table construction, argument
// checks and the C ABI.  The kernels live in the other .hip files of this folder (see eoq_internal.h).
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "eoq_internal.h"

// ---------------------------------------------------------------------------
// Scratch of eoq_compress_static: the workspace of eoq_compress (eigenvalues, projection operands, hand-over list,
// tridiagonal matrices) for callers that cannot hand one in.  One copy per GPU, held until the process ends.  In host
// code the name below is only a stand-in for the symbol: the device address comes from hipGetSymbolAddress, once per
// device (eoq_create, with that device current), and only that pointer is ever passed to a kernel.
// ---------------------------------------------------------------------------
constexpr size_t EOQ_STATIC_SCRATCH_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[EOQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int EOQ_MAX_DEVICES = 64;
void* g_scratch_ptr[EOQ_MAX_DEVICES] = {};   // device address of `scratch` on each GPU this process has used

// ---------------------------------------------------------------------------
// Seeded Gaussian stream: SplitMix64 evaluated at a counter, Box-Muller cosine
// branch on the counter pair (2e, 2e+1) for draw number e.
// ---------------------------------------------------------------------------
inline uint64_t mix64(uint64_t seed, uint64_t counter) {
  uint64_t z = seed + (counter + 1ull) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

inline double unit_open(uint64_t bits) {  // (0,1), 53 bits
  return ((double)(bits >> 11) + 0.5) * 0x1.0p-53;
}

inline double gaussian_draw(uint64_t seed, uint64_t e) {
  const double u1 = unit_open(mix64(seed, 2 * e));
  const double u2 = unit_open(mix64(seed, 2 * e + 1));
  return std::sqrt(-2.0 * std::log(u1)) * std::cos(2.0 * M_PI * u2);
}

// ---------------------------------------------------------------------------
// Haar rotation (Alg. 1 REQUIRE; Sec. 2.2 item 2): Householder QR of a d x d
// Gaussian matrix filled row-major, Q's columns re-signed so that R's diagonal
// is positive.  Double precision; returned row-major as q[c*d + j].
// ---------------------------------------------------------------------------
std::vector<double> haar_rotation(int d, uint64_t seed) {
  std::vector<double> a((size_t)d * d), q((size_t)d * d, 0.0), v(d), rdiag(d);
  for (int i = 0; i < d * d; ++i) a[i] = gaussian_draw(seed, (uint64_t)i);
  for (int i = 0; i < d; ++i) q[(size_t)i * d + i] = 1.0;
  for (int j = 0; j < d; ++j) {
    double nrm = 0.0;
    for (int i = j; i < d; ++i) nrm += a[(size_t)i * d + j] * a[(size_t)i * d + j];
    nrm = std::sqrt(nrm);
    const double x0 = a[(size_t)j * d + j];
    const double alpha = (x0 >= 0.0) ? -nrm : nrm;  // R[j][j]
    rdiag[j] = alpha;
    double vn = 0.0;
    for (int i = j; i < d; ++i) {
      v[i] = a[(size_t)i * d + j] - (i == j ? alpha : 0.0);
      vn += v[i] * v[i];
    }
    if (vn == 0.0) continue;
    const double s = 2.0 / vn;
    // A <- (I - s v v^T) A on rows j.., columns j..
    for (int c = j; c < d; ++c) {
      double dot = 0.0;
      for (int i = j; i < d; ++i) dot += v[i] * a[(size_t)i * d + c];
      dot *= s;
      for (int i = j; i < d; ++i) a[(size_t)i * d + c] -= dot * v[i];
    }
    // Q <- Q (I - s v v^T)
    for (int r = 0; r < d; ++r) {
      double dot = 0.0;
      for (int i = j; i < d; ++i) dot += q[(size_t)r * d + i] * v[i];
      dot *= s;
      for (int i = j; i < d; ++i) q[(size_t)r * d + i] -= dot * v[i];
    }
  }
  for (int j = 0; j < d; ++j)
    if (rdiag[j] < 0.0)
      for (int r = 0; r < d; ++r) q[(size_t)r * d + j] = -q[(size_t)r * d + j];
  return q;
}

// ---------------------------------------------------------------------------
// Lloyd-Max quantizer of N(0,1) with 2^bits levels (Sec. 2.2 item 3).  The
// optimum is symmetric, so only the positive half is iterated: cells
// [t_0 = 0, t_1), ..., [t_{h-1}, inf) with centroids c_0 < ... < c_{h-1}.
// ---------------------------------------------------------------------------
inline double npdf(double x) { return std::exp(-0.5 * x * x) * 0.3989422804014326779; }
inline double ntail(double x) { return 0.5 * std::erfc(x * 0.7071067811865475244); }

void lloyd_max(int bits, std::vector<double>& cent, std::vector<double>& bnd) {
  const int L = 1 << bits, h = L / 2;
  std::vector<double> c(h), t(h + 1);
  for (int i = 0; i < h; ++i) c[i] = (i + 0.5) * 3.0 / h;
  for (int it = 0; it < 400000; ++it) {
    t[0] = 0.0;
    for (int i = 1; i < h; ++i) t[i] = 0.5 * (c[i - 1] + c[i]);
    double delta = 0.0;
    for (int i = 0; i < h; ++i) {
      const double lo = t[i];
      const double num = npdf(lo) - (i + 1 < h ? npdf(t[i + 1]) : 0.0);
      const double den = ntail(lo) - (i + 1 < h ? ntail(t[i + 1]) : 0.0);
      const double nc = num / den;
      delta = std::fmax(delta, std::fabs(nc - c[i]));
      c[i] = nc;
    }
    if (delta < 1e-16) break;
  }
  cent.assign(L, 0.0);
  bnd.assign(L - 1, 0.0);
  for (int i = 0; i < h; ++i) {
    cent[h + i] = c[i];
    cent[h - 1 - i] = -c[i];
  }
  for (int i = 0; i + 1 < L; ++i) bnd[i] = 0.5 * (cent[i] + cent[i + 1]);
  bnd[h - 1] = 0.0;
}

eoq_status fail(eoq_ctx* ctx, eoq_status st, const char* msg) {
  if (ctx) ctx->err = msg;
  return st;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

eoq_status check_packed(eoq_ctx* ctx, const eoq_packed& p) {
  const void* ptrs[] = {p.codes, p.norms, p.rank, p.phi, p.sigma, p.lfac, p.rfac, p.flags};
  for (const void* q : ptrs) {
    if (!q) return fail(ctx, EOQ_ERR_ARG, "eoq_packed has a null member");
    if (!aligned16(q)) return fail(ctx, EOQ_ERR_ARG, "eoq_packed member not 16-byte aligned");
  }
  return EOQ_OK;
}

EoqLaunch make_launch(const eoq_ctx* ctx, void* stream) {
  EoqLaunch L;
  L.n = ctx->n;
  L.bits = ctx->bits;
  L.r_max = ctx->r_max;
  L.k = ctx->k;
  L.rank_thr = ctx->rank_thr;
  L.pi = ctx->d_pi;
  L.pit = ctx->d_pit;
  L.tab = ctx->d_tab;
  L.pih = ctx->d_pih;
  L.phit = ctx->d_phit;
  L.phih = ctx->d_phih;
  L.stream = static_cast<hipStream_t>(stream);
  L.ev = ctx->profile ? ctx->ev : nullptr;
  L.solver = ctx->solver;
  L.loss = ctx->loss;
  L.map = eoq_dense_map(ctx->n);
  return L;
}

}  // namespace

extern "C" {

int eoq_pilot_k(int d) {
  if (d < 3) return 0;
  const double c = std::fmin(1.0 / 2.01, 1.0 / std::log(std::log((double)d)));
  return (int)std::floor(std::pow((double)d, c));
}

eoq_status eoq_create(eoq_ctx** out, int n, int d, int bits, uint64_t rot_seed, int r_max) {
  if (!out) return EOQ_ERR_ARG;
  *out = nullptr;
  if (d != EOQ_D || n < 128 || n > 4096 || (n % 128) != 0 || bits < 1 || bits > 4 || r_max < 1 ||
      r_max > EOQ_RMAX_CAP)
    return EOQ_ERR_UNSUPPORTED;
  eoq_ctx* ctx = new (std::nothrow) eoq_ctx;
  if (!ctx) return EOQ_ERR_ARG;
  ctx->n = n;
  ctx->d = d;
  ctx->bits = bits;
  ctx->r_max = r_max;
  ctx->seed = rot_seed;
  ctx->k = eoq_pilot_k(d);
  ctx->rank_thr = std::pow((double)d, -1.0 / 3.0);
  if (2 * ctx->k + r_max + 1 > d) {  // Alg. 2 Step 2 reads eigenvalue number 2k + r + 1
    delete ctx;
    return EOQ_ERR_UNSUPPORTED;
  }

  const std::vector<double> q = haar_rotation(d, rot_seed);
  ctx->pi_host.resize((size_t)d * d);
  std::vector<float> pit((size_t)d * d);
  for (int c = 0; c < d; ++c)
    for (int j = 0; j < d; ++j) {
      const float v = (float)q[(size_t)c * d + j];
      ctx->pi_host[(size_t)c * d + j] = v;
      pit[(size_t)j * d + c] = v;
    }
  // Phi of TQ_prod: iid N(0,1) from the same generator, seeded with rot_seed + 1, rounded to binary16: that is the
  // table (nothing in the estimator depends on more digits of a random Gaussian matrix, and one matrix-core pass
  // multiplies by it exactly)
  ctx->phi_host.resize((size_t)d * d);
  for (int i = 0; i < d * d; ++i) ctx->phi_host[i] = (float)(_Float16)gaussian_draw(rot_seed + 1, (uint64_t)i);
  std::vector<double> cent, bnd;
  lloyd_max(4, cent, bnd);
  for (int i = 0; i < 8; ++i) ctx->gauss16[i] = cent[8 + i];
  lloyd_max(bits, cent, bnd);
  ctx->cent_host.assign(cent.begin(), cent.end());
  ctx->bnd_host.assign(bnd.begin(), bnd.end());
  float tab[32];
  for (int i = 0; i < 16; ++i) tab[i] = (i < (1 << bits)) ? ctx->cent_host[i] : 0.0f;
  for (int i = 0; i < 16; ++i) tab[16 + i] = (i < (1 << bits) - 1) ? ctx->bnd_host[i] : INFINITY;

  // Without a HIP device the context is host-only: the tables can be read back, the hot calls fail.
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
    (void)hipGetLastError();
    ctx->device = -1;
    *out = ctx;
    return EOQ_OK;
  }
  hipError_t e = hipGetDevice(&ctx->device);
  if (e == hipSuccess && ctx->device >= 0 && ctx->device < EOQ_MAX_DEVICES && !g_scratch_ptr[ctx->device]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // this device's copy of the array
    if (e == hipSuccess) g_scratch_ptr[ctx->device] = p;
  }
  if (e == hipSuccess) e = eoq_factor_quant_prepare();
  const size_t mat_bytes = (size_t)d * d * sizeof(float);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_pi, mat_bytes);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_pit, mat_bytes);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_tab, sizeof(tab));
  // binary16 hi/lo split of the rotation for the matrix-core kernels: Pi = hi + lo to ~2^-24 absolute
  // (lo is subnormal for most entries; the matrix cores take subnormal operands)
  std::vector<uint16_t> split((size_t)4 * d * d);
  for (int c = 0; c < d; ++c)
    for (int j = 0; j < d; ++j) {
      const float v = ctx->pi_host[(size_t)c * d + j];
      const _Float16 hi = (_Float16)v;
      const _Float16 lo = (_Float16)(v - (float)hi);
      uint16_t hb, lb;
      std::memcpy(&hb, &hi, 2);
      std::memcpy(&lb, &lo, 2);
      split[(size_t)0 * d * d + (size_t)c * d + j] = hb;   // Pi hi   [c][j]
      split[(size_t)1 * d * d + (size_t)c * d + j] = lb;   // Pi lo   [c][j]
      split[(size_t)2 * d * d + (size_t)j * d + c] = hb;   // Pi^T hi [j][c]
      split[(size_t)3 * d * d + (size_t)j * d + c] = lb;   // Pi^T lo [j][c]
    }
  std::vector<float> phit((size_t)d * d);
  std::vector<uint16_t> psplit((size_t)2 * d * d);
  for (int i = 0; i < d; ++i)
    for (int j = 0; j < d; ++j) {
      const float v = ctx->phi_host[(size_t)i * d + j];
      phit[(size_t)j * d + i] = v;
      const _Float16 hi = (_Float16)v;
      const _Float16 lo = (_Float16)(v - (float)hi);
      std::memcpy(&psplit[(size_t)i * d + j], &hi, 2);
      std::memcpy(&psplit[(size_t)d * d + (size_t)i * d + j], &lo, 2);
    }
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_phit, mat_bytes);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_phih, psplit.size() * 2);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_phit, phit.data(), mat_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_phih, psplit.data(), psplit.size() * 2, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMalloc((void**)&ctx->d_pih, split.size() * 2);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_pih, split.data(), split.size() * 2, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_pi, ctx->pi_host.data(), mat_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_pit, pit.data(), mat_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_tab, tab, sizeof(tab), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    std::fprintf(stderr, "eoq_create: %s\n", hipGetErrorString(e));
    eoq_destroy(ctx);
    return EOQ_ERR_HIP;
  }
  *out = ctx;
  return EOQ_OK;
}

void eoq_destroy(eoq_ctx* ctx) {
  if (!ctx) return;
  if (ctx->d_pi) (void)hipFree(ctx->d_pi);
  if (ctx->d_pit) (void)hipFree(ctx->d_pit);
  if (ctx->d_tab) (void)hipFree(ctx->d_tab);
  if (ctx->d_pih) (void)hipFree(ctx->d_pih);
  if (ctx->d_phit) (void)hipFree(ctx->d_phit);
  if (ctx->d_phih) (void)hipFree(ctx->d_phih);
  if (ctx->profile)
    for (hipEvent_t& e : ctx->ev) (void)hipEventDestroy(e);
  delete ctx;
}

size_t eoq_workspace_bytes(const eoq_ctx* ctx, int64_t B) {
  if (!ctx || B < 0) return 0;
  return eoq_ws_lam_bytes(B) + eoq_ws_wfac_bytes(B, ctx->r_max) + eoq_ws_list_bytes(B) + eoq_ws_tri_bytes(B);
}

eoq_status eoq_rotation(const eoq_ctx* ctx, float* host_out) {
  if (!ctx || !host_out) return EOQ_ERR_ARG;
  std::memcpy(host_out, ctx->pi_host.data(), ctx->pi_host.size() * sizeof(float));
  return EOQ_OK;
}

eoq_status eoq_projection(const eoq_ctx* ctx, float* host_out) {
  if (!ctx || !host_out) return EOQ_ERR_ARG;
  std::memcpy(host_out, ctx->phi_host.data(), ctx->phi_host.size() * sizeof(float));
  return EOQ_OK;
}

eoq_status eoq_codebook(const eoq_ctx* ctx, float* host_centroids, float* host_bounds) {
  if (!ctx || !host_centroids || !host_bounds) return EOQ_ERR_ARG;
  std::memcpy(host_centroids, ctx->cent_host.data(), ctx->cent_host.size() * sizeof(float));
  std::memcpy(host_bounds, ctx->bnd_host.data(), ctx->bnd_host.size() * sizeof(float));
  return EOQ_OK;
}

}  // extern "C"

namespace {

// eoq_compress, eoq_compress_q4 and eoq_compress_chunk: `fq` null = binary16 factors
eoq_status compress_impl(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, const EoqBlockMap& map,
                         eoq_packed out, const eoq_factor_codes* fq, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (B < 0) return fail(ctx, EOQ_ERR_ARG, "negative block count");
  if (dtype != EOQ_F16 && dtype != EOQ_F32) return fail(ctx, EOQ_ERR_UNSUPPORTED, "dtype must be EOQ_F16 or EOQ_F32");
  if (fq) {
    if (dtype != EOQ_F16) return fail(ctx, EOQ_ERR_UNSUPPORTED, "4-bit factors: dtype must be EOQ_F16");
    if ((int64_t)ctx->n * ctx->r_max > 32768) return fail(ctx, EOQ_ERR_UNSUPPORTED, "4-bit factors: n * r_max exceeds 32768");
  }
  if (B == 0) return EOQ_OK;
  if (!blocks || !workspace) return fail(ctx, EOQ_ERR_ARG, "null blocks or workspace pointer");
  if (!aligned16(blocks) || !aligned16(workspace)) return fail(ctx, EOQ_ERR_ARG, "blocks/workspace not 16-byte aligned");
  if (eoq_status st = check_packed(ctx, out)) return st;
  if (fq && (!fq->lcodes || !fq->rcodes || !fq->fbook || !fq->phi16))
    return fail(ctx, EOQ_ERR_ARG, "eoq_factor_codes has a null member");
  if (fq && !(aligned16(fq->lcodes) && aligned16(fq->rcodes) && aligned16(fq->fbook) && aligned16(fq->phi16)))
    return fail(ctx, EOQ_ERR_ARG, "eoq_factor_codes member not 16-byte aligned");
  if (workspace_bytes < eoq_workspace_bytes(ctx, B)) return fail(ctx, EOQ_ERR_WORKSPACE, "workspace too small");
  if (B > (int64_t)1 << 24) return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");

  EoqLaunch L = make_launch(ctx, hip_stream);
  L.map = map;
  double* lam = static_cast<double*>(workspace);
  char* ws = static_cast<char*>(workspace);
  float* wfac = reinterpret_cast<float*>(ws + eoq_ws_lam_bytes(B));
  int* fb_count = reinterpret_cast<int*>(ws + eoq_ws_lam_bytes(B) + eoq_ws_wfac_bytes(B, ctx->r_max));
  int* fb_list = fb_count + 4;
  const uintptr_t tri_at = reinterpret_cast<uintptr_t>(reinterpret_cast<char*>(fb_count) + eoq_ws_list_bytes(B));
  double* tri = reinterpret_cast<double*>((tri_at + 63) & ~(uintptr_t)63);
  hipError_t e = eoq_launch_spectral(L, blocks, (int)dtype, B, lam, wfac, fb_count, fb_list, tri, out);
  if (fq) {
    if (L.ev && e == hipSuccess) (void)hipEventRecord(L.ev[2], L.stream);  // the factor stage counts as encode time
    if (e == hipSuccess) e = eoq_launch_factor_quant(L, blocks, B, wfac, out, *fq, ctx->gauss16);
    if (e == hipSuccess) e = eoq_launch_encode_f16(L, blocks, B, wfac, out, true);
    if (L.ev && e == hipSuccess) (void)hipEventRecord(L.ev[3], L.stream);
  } else if (e == hipSuccess) {
    e = eoq_launch_encode(L, blocks, (int)dtype, B, wfac, out);
  }
  if (ctx->profile) ctx->ev_valid[0] = ctx->ev_valid[1] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

}  // namespace

extern "C" {

eoq_status eoq_compress(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_packed out,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  return compress_impl(ctx, blocks, dtype, B, eoq_dense_map(ctx->n), out, nullptr, workspace, workspace_bytes,
                       hip_stream);
}

int64_t eoq_static_max_blocks(const eoq_ctx* ctx) {
  if (!ctx) return 0;
  int64_t lo = 0, hi = (int64_t)(EOQ_STATIC_SCRATCH_BYTES / (EOQ_D * sizeof(double))) + 1;   // eoq_workspace_bytes grows with B
  while (hi - lo > 1) {
    const int64_t mid = lo + (hi - lo) / 2;
    if (eoq_workspace_bytes(ctx, mid) <= EOQ_STATIC_SCRATCH_BYTES) lo = mid; else hi = mid;
  }
  return lo;
}

eoq_status eoq_compress_static(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_packed out,
                               void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (B > eoq_static_max_blocks(ctx))
    return fail(ctx, EOQ_ERR_WORKSPACE, "eoq_compress_static: more blocks than the built-in scratch holds (eoq_static_max_blocks)");
  void* ws = (ctx->device < EOQ_MAX_DEVICES) ? g_scratch_ptr[ctx->device] : nullptr;
  if (!ws) return fail(ctx, EOQ_ERR_HIP, "eoq_compress_static: no scratch address for this device");
  return compress_impl(ctx, blocks, dtype, B, eoq_dense_map(ctx->n), out, nullptr, ws, EOQ_STATIC_SCRATCH_BYTES, hip_stream);
}

eoq_status eoq_compress_q4(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_packed out,
                           eoq_factor_codes fq, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  return compress_impl(ctx, blocks, dtype, B, eoq_dense_map(ctx->n), out, &fq, workspace, workspace_bytes,
                       hip_stream);
}

eoq_status eoq_compress_chunk(eoq_ctx* ctx, const void* blocks, eoq_dtype dtype, int64_t B, eoq_chunk_layout lay,
                              eoq_packed out, const eoq_factor_codes* fq, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (lay.in_group_size < 1 || lay.in_token_stride < ctx->d || lay.in_group_stride < 0 || lay.in_block_stride < 0 ||
      lay.out_first < 0 || lay.out_stride < 1)
    return fail(ctx, EOQ_ERR_ARG, "chunk layout: sizes and strides out of range");
  if ((lay.in_token_stride | lay.in_group_stride | lay.in_block_stride) & 7)
    return fail(ctx, EOQ_ERR_ARG, "chunk layout: input strides must be multiples of 8 elements");
  const EoqBlockMap map{lay.in_group_stride, lay.in_block_stride, lay.in_token_stride, lay.out_first, lay.out_stride,
                        lay.in_group_size};
  return compress_impl(ctx, blocks, dtype, B, map, out, fq, workspace, workspace_bytes, hip_stream);
}

eoq_status eoq_expand_factors(eoq_ctx* ctx, eoq_packed rec, eoq_factor_codes fq, int64_t B, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (B < 0) return fail(ctx, EOQ_ERR_ARG, "negative block count");
  if (B == 0) return EOQ_OK;
  if (eoq_status st = check_packed(ctx, rec)) return st;
  if (!fq.lcodes || !fq.rcodes || !fq.fbook || !fq.phi16) return fail(ctx, EOQ_ERR_ARG, "eoq_factor_codes has a null member");
  if (!(aligned16(fq.lcodes) && aligned16(fq.rcodes) && aligned16(fq.fbook) && aligned16(fq.phi16)))
    return fail(ctx, EOQ_ERR_ARG, "eoq_factor_codes member not 16-byte aligned");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  const hipError_t e = eoq_launch_factor_expand(L, rec, fq, B);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_decompress(eoq_ctx* ctx, eoq_packed in, int64_t B, void* out_fp16, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (B < 0) return fail(ctx, EOQ_ERR_ARG, "negative block count");
  if (B == 0) return EOQ_OK;
  if (!out_fp16 || !aligned16(out_fp16)) return fail(ctx, EOQ_ERR_ARG, "null or misaligned output pointer");
  if (eoq_status st = check_packed(ctx, in)) return st;
  if (B > (int64_t)1 << 24) return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  hipError_t e = eoq_launch_decode(L, in, B, out_fp16);
  if (ctx->profile) ctx->ev_valid[2] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_scores(eoq_ctx* ctx, eoq_packed keys, int64_t n_seq, int n_kv_heads, int64_t blocks_per_head,
                      const void* q_fp16, int n_q_heads, float* scores, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (n_seq < 0 || blocks_per_head < 0 || n_kv_heads < 1 || n_q_heads < 1)
    return fail(ctx, EOQ_ERR_ARG, "negative or zero size");
  if (n_q_heads % n_kv_heads != 0 || n_q_heads / n_kv_heads > 8)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "query heads must be a multiple (1..8) of KV heads");
  if (n_seq == 0 || blocks_per_head == 0) return EOQ_OK;
  if (!q_fp16 || !scores || !aligned16(q_fp16) || !aligned16(scores))
    return fail(ctx, EOQ_ERR_ARG, "null or misaligned query/score pointer");
  if (eoq_status st = check_packed(ctx, keys)) return st;
  if (n_seq * n_kv_heads * blocks_per_head > (int64_t)1 << 24)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  if ((int64_t)(n_q_heads / n_kv_heads) * blocks_per_head * ctx->n * 4 > 0x7FFFFFFF)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "the score rows of one KV head exceed 2 GiB");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  hipError_t e = eoq_launch_scores(L, keys, n_seq, n_kv_heads, blocks_per_head, q_fp16, n_q_heads, scores);
  if (ctx->profile) ctx->ev_valid[3] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_scores_stream(eoq_ctx* ctx, eoq_packed keys, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                             int64_t blocks_filled, const void* tail_fp16, int64_t tail_capacity, int64_t tail_len,
                             const void* q_fp16, int n_q_heads, float* scores, int64_t score_stride,
                             void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (n_seq < 0 || blocks_filled < 0 || tail_len < 0 || n_kv_heads < 1 || n_q_heads < 1)
    return fail(ctx, EOQ_ERR_ARG, "negative or zero size");
  if (blocks_filled > block_capacity || tail_len > tail_capacity)
    return fail(ctx, EOQ_ERR_ARG, "more blocks or tail tokens than the stores hold");
  if (score_stride < blocks_filled * ctx->n + tail_len)
    return fail(ctx, EOQ_ERR_ARG, "score rows shorter than the blocks' tokens plus the tail");
  if (n_q_heads % n_kv_heads != 0 || n_q_heads / n_kv_heads > 8)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "query heads must be a multiple (1..8) of KV heads");
  if (tail_len >= ctx->n) return fail(ctx, EOQ_ERR_UNSUPPORTED, "the tail holds fewer than n tokens");
  if (n_seq == 0 || (blocks_filled == 0 && tail_len == 0)) return EOQ_OK;
  if (!q_fp16 || !scores || !aligned16(q_fp16) || !aligned16(scores))
    return fail(ctx, EOQ_ERR_ARG, "null or misaligned query/score pointer");
  if (tail_len > 0 && (!tail_fp16 || !aligned16(tail_fp16))) return fail(ctx, EOQ_ERR_ARG, "null or misaligned tail pointer");
  if (blocks_filled > 0)
    if (eoq_status st = check_packed(ctx, keys)) return st;
  if (n_seq * n_kv_heads * block_capacity > (int64_t)1 << 24)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  if ((int64_t)(n_q_heads / n_kv_heads) * score_stride * 4 > 0x7FFFFFFF)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "the score rows of one KV head exceed 2 GiB");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  hipError_t e = eoq_launch_scores(L, keys, n_seq, n_kv_heads, blocks_filled, q_fp16, n_q_heads, scores, block_capacity,
                                   score_stride, tail_fp16, tail_capacity, (int)tail_len);
  if (ctx->profile) ctx->ev_valid[3] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

size_t eoq_attend_workspace_bytes(const eoq_ctx* ctx, int64_t n_seq, int n_kv_heads, int64_t blocks_per_head) {
  if (!ctx || n_seq <= 0 || n_kv_heads <= 0 || blocks_per_head <= 0) return 0;
  int run = 1;
  const int64_t runs = eoq_attend_runs(n_seq * n_kv_heads, blocks_per_head, &run);
  return (size_t)(n_seq * n_kv_heads) * (size_t)runs * 16 * EOQ_D * sizeof(float);
}

eoq_status eoq_softmax(eoq_ctx* ctx, float* scores, int64_t rows, int64_t len, int64_t row_stride, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (rows < 0 || len < 0 || row_stride < len) return fail(ctx, EOQ_ERR_ARG, "negative size or rows that overlap");
  if (rows == 0 || len == 0) return EOQ_OK;
  if (!scores || !aligned16(scores)) return fail(ctx, EOQ_ERR_ARG, "null or misaligned score pointer");
  if (rows > 0x7FFFFFFF) return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^31 - 1 rows");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  const hipError_t e = eoq_launch_softmax(L, scores, rows, len, row_stride);
  if (ctx->profile) ctx->ev_valid[5] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

static eoq_status attend_impl(eoq_ctx* ctx, eoq_packed values, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                              int64_t blocks_filled, const void* tail_fp16, int64_t tail_capacity, int64_t tail_len,
                              const float* weights, int64_t weight_stride, int n_q_heads, float* out, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (n_seq < 0 || blocks_filled < 0 || n_kv_heads < 1 || n_q_heads < 1) return fail(ctx, EOQ_ERR_ARG, "negative or zero size");
  if (blocks_filled > block_capacity) return fail(ctx, EOQ_ERR_ARG, "more blocks than the store holds");
  if (tail_len < 0 || tail_len > tail_capacity) return fail(ctx, EOQ_ERR_ARG, "more tail tokens than the tail buffer holds");
  if (tail_len >= ctx->n) return fail(ctx, EOQ_ERR_UNSUPPORTED, "the tail holds fewer than n tokens");
  if (tail_len > 0 && (!tail_fp16 || !aligned16(tail_fp16))) return fail(ctx, EOQ_ERR_ARG, "null or misaligned tail pointer");
  if (weight_stride < blocks_filled * ctx->n + tail_len)
    return fail(ctx, EOQ_ERR_ARG, "weight rows shorter than the blocks' tokens plus the tail");
  if (n_q_heads % n_kv_heads != 0 || n_q_heads / n_kv_heads > 8)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "query heads must be a multiple (1..8) of KV heads");
  if (n_seq == 0) return EOQ_OK;
  if (!weights || !out || !aligned16(out) || !aligned16(weights))
    return fail(ctx, EOQ_ERR_ARG, "null or misaligned weight/output pointer");
  if (blocks_filled > 0) {
    if (eoq_status st = check_packed(ctx, values)) return st;
    if (!workspace || !aligned16(workspace)) return fail(ctx, EOQ_ERR_ARG, "null or misaligned workspace");
    if (workspace_bytes < eoq_attend_workspace_bytes(ctx, n_seq, n_kv_heads, blocks_filled))
      return fail(ctx, EOQ_ERR_WORKSPACE, "workspace too small");
  }
  if (n_seq * n_kv_heads * block_capacity > (int64_t)1 << 24)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  const hipError_t e = eoq_launch_attend(L, values, n_seq, n_kv_heads, blocks_filled, block_capacity, weights,
                                         weight_stride, n_q_heads, out, static_cast<float*>(workspace), tail_fp16,
                                         tail_capacity, (int)tail_len);
  if (ctx->profile) ctx->ev_valid[4] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_qjl_encode(eoq_ctx* ctx, const void* blocks_fp16, int64_t B, eoq_packed rec, eoq_qjl out,
                          void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (B < 0) return fail(ctx, EOQ_ERR_ARG, "negative block count");
  if (B == 0) return EOQ_OK;
  if (!blocks_fp16 || !aligned16(blocks_fp16)) return fail(ctx, EOQ_ERR_ARG, "null or misaligned blocks pointer");
  if (eoq_status st = check_packed(ctx, rec)) return st;
  if (!out.signs || !out.norms || !aligned16(out.signs) || !aligned16(out.norms))
    return fail(ctx, EOQ_ERR_ARG, "eoq_qjl has a null or misaligned member");
  if (B > (int64_t)1 << 24) return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  const hipError_t e = eoq_launch_qjl(L, blocks_fp16, B, rec, out);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_scores_prod(eoq_ctx* ctx, eoq_packed keys, eoq_qjl qjl, int64_t n_seq, int n_kv_heads,
                           int64_t blocks_per_head, const void* q_fp16, int n_q_heads, float* scores,
                           void* hip_stream) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (n_seq < 0 || blocks_per_head < 0 || n_kv_heads < 1 || n_q_heads < 1)
    return fail(ctx, EOQ_ERR_ARG, "negative or zero size");
  if (n_q_heads % n_kv_heads != 0 || n_q_heads / n_kv_heads > 8)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "query heads must be a multiple (1..8) of KV heads");
  if (n_seq == 0 || blocks_per_head == 0) return EOQ_OK;
  if (!q_fp16 || !scores || !aligned16(q_fp16) || !aligned16(scores))
    return fail(ctx, EOQ_ERR_ARG, "null or misaligned query/score pointer");
  if (eoq_status st = check_packed(ctx, keys)) return st;
  if (!qjl.signs || !qjl.norms || !aligned16(qjl.signs) || !aligned16(qjl.norms))
    return fail(ctx, EOQ_ERR_ARG, "eoq_qjl has a null or misaligned member");
  if (n_seq * n_kv_heads * blocks_per_head > (int64_t)1 << 24)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "more than 2^24 blocks in one call");
  if ((int64_t)(n_q_heads / n_kv_heads) * blocks_per_head * ctx->n * 4 > 0x7FFFFFFF)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "the score rows of one KV head exceed 2 GiB");
  const EoqLaunch L = make_launch(ctx, hip_stream);
  const hipError_t e = eoq_launch_scores_prod(L, keys, qjl, n_seq, n_kv_heads, blocks_per_head, q_fp16, n_q_heads, scores);
  if (ctx->profile) ctx->ev_valid[3] = (e == hipSuccess);
  if (e != hipSuccess) {
    ctx->err = std::string("HIP: ") + hipGetErrorString(e);
    return EOQ_ERR_HIP;
  }
  return EOQ_OK;
}

eoq_status eoq_attend(eoq_ctx* ctx, eoq_packed values, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                      int64_t blocks_filled, const float* weights, int64_t weight_stride, int n_q_heads, float* out,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return attend_impl(ctx, values, n_seq, n_kv_heads, block_capacity, blocks_filled, nullptr, 0, 0, weights, weight_stride,
                     n_q_heads, out, workspace, workspace_bytes, hip_stream);
}

eoq_status eoq_attend_stream(eoq_ctx* ctx, eoq_packed values, int64_t n_seq, int n_kv_heads, int64_t block_capacity,
                             int64_t blocks_filled, const void* tail_fp16, int64_t tail_capacity, int64_t tail_len,
                             const float* weights, int64_t weight_stride, int n_q_heads, float* out, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
  return attend_impl(ctx, values, n_seq, n_kv_heads, block_capacity, blocks_filled, tail_fp16, tail_capacity, tail_len,
                     weights, weight_stride, n_q_heads, out, workspace, workspace_bytes, hip_stream);
}

eoq_status eoq_set_solver(eoq_ctx* ctx, int solver) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (solver != 0 && solver != 1) return fail(ctx, EOQ_ERR_UNSUPPORTED, "solver must be 0 or 1");
  ctx->solver = solver;
  return EOQ_OK;
}

eoq_status eoq_set_loss(eoq_ctx* ctx, eoq_loss loss) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (loss != EOQ_LOSS_FROBENIUS && loss != EOQ_LOSS_OPERATOR && loss != EOQ_LOSS_NUCLEAR)
    return fail(ctx, EOQ_ERR_UNSUPPORTED, "loss must be EOQ_LOSS_FROBENIUS, EOQ_LOSS_OPERATOR or EOQ_LOSS_NUCLEAR");
  ctx->loss = (int)loss;
  return EOQ_OK;
}

eoq_status eoq_profile(eoq_ctx* ctx, int enable) {
  if (!ctx) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (ctx->device < 0) return fail(ctx, EOQ_ERR_HIP, "context was created without a HIP device");
  if (enable && !ctx->profile) {
    for (int i = 0; i < 12; ++i) {
      if (hipEventCreate(&ctx->ev[i]) != hipSuccess) {
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->ev[j]);
        return fail(ctx, EOQ_ERR_HIP, "hipEventCreate failed");
      }
    }
    ctx->profile = true;
  } else if (!enable && ctx->profile) {
    for (hipEvent_t& e : ctx->ev) (void)hipEventDestroy(e);
    ctx->profile = false;
  }
  for (bool& v : ctx->ev_valid) v = false;
  return EOQ_OK;
}

eoq_status eoq_stage_ms(eoq_ctx* ctx, float* out) {
  if (!ctx || !out) return EOQ_ERR_ARG;
  ctx->err.clear();
  if (!ctx->profile) return fail(ctx, EOQ_ERR_ARG, "profiling is not enabled");
  for (int i = 0; i < 6; ++i) {
    out[i] = -1.0f;
    if (!ctx->ev_valid[i]) continue;
    hipError_t e = hipEventSynchronize(ctx->ev[2 * i + 1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&out[i], ctx->ev[2 * i], ctx->ev[2 * i + 1]);
    if (e != hipSuccess) {
      ctx->err = std::string("HIP: ") + hipGetErrorString(e);
      return EOQ_ERR_HIP;
    }
  }
  return EOQ_OK;
}

const char* eoq_last_error(const eoq_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

}  // extern "C"
