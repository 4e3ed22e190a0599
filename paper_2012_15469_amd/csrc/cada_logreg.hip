// Dual minibatch gradient of the l2-regularised logistic loss for all workers, and the
// left-hand side of the communication rule (Section 2.2, conditions (workerrule1) and
// (workerrule2)); Algorithm 1, the workers' two gradient evaluations on the same samples.
//
// With z_b = x_b.theta, d = theta - theta_ref and dz_b = x_b.d (so x_b.theta_ref = z_b - dz_b),
//     r_b  = -y_b sigma(-y_b z_b)                         residual at theta
//     dr_b = r_b - r_ref,b = y_b sigma(a) sigma(-b') expm1(y_b dz_b),  a = -y_b z_b, b' = a + y_b dz_b
//     g      = X_B^T r / B + lambda theta                 fresh gradient
//     innov  = X_B^T dr / B + lambda d                    g(theta) - g(theta_ref), no cancellation
// The difference of the two gradients is formed from d and dr directly: subtracting two
// float32 gradients of nearby points would lose the digits the rule's comparison needs.
//
// Pass 1 (k_dots) streams the B gathered rows once for z and dz; pass 2 (k_grad) streams
// them again for g and innov, column-parallel, and reduces |innov|^2 (CADA2) or
// |innov - stored innovation|^2 (CADA1) per block in a fixed order.
#include "cada_internal.h"

namespace cada {

constexpr int kRowsPerBlock = 8;   // rows sharing one load of theta and d in pass 1

struct LogregArgs {
  DevState s;
  const int32_t *idx;    // [M][B]
  float *zpart;          // [M][B][nc][2]
  int nc;
  int64_t chunk_cols;
  int m0;                // first worker of this launch
};

template <int VEC> struct Vec;
template <> struct Vec<4> { using T = float4; };
template <> struct Vec<1> { using T = float; };

template <int VEC> __device__ __forceinline__ void load_vec(const float *p, float (&o)[VEC]) {
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4 *>(p);
    o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w;
  } else {
    o[0] = *p;
  }
}
template <int VEC> __device__ __forceinline__ void store_vec(float *p, const float (&o)[VEC]) {
  if constexpr (VEC == 4) {
    *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
  } else {
    *p = o[0];
  }
}

__device__ __forceinline__ int64_t clamp_row(const DevState &s, int m, int32_t local, bool *bad) {
  const int64_t n = s.row_off[m + 1] - s.row_off[m];
  int64_t r = local;
  if (r < 0) { r = 0; *bad = true; }
  if (r >= n) { r = n - 1; *bad = true; }
  return s.row_off[m] + r;
}

// grid (nc, ceil(B / kRowsPerBlock), M)
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_dots(const LogregArgs a) {
  const DevState &s = a.s;
  const int m = a.m0 + blockIdx.z;
  const int r0 = blockIdx.y * kRowsPerBlock;
  const int64_t k = s.k;
  const float *__restrict__ th = s.theta;
  const float *__restrict__ tl = s.theta_lo;
  const RefPtr ref = theta_ref(s, m, k);
  const int32_t *idx = a.idx + (int64_t)m * s.B;

  const float *xrow[kRowsPerBlock];
  bool bad = false;
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) {
    const int b = min(r0 + r, s.B - 1);
    xrow[r] = s.X + clamp_row(s, m, idx[b], &bad) * s.p;
  }
  if (bad && threadIdx.x == 0) atomicOr(s.err, 1u);

  float z[kRowsPerBlock], dz[kRowsPerBlock];
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) { z[r] = 0.f; dz[r] = 0.f; }

  const int64_t c0 = (int64_t)blockIdx.x * a.chunk_cols;
  const int64_t c1 = min(s.p, c0 + a.chunk_cols);
  for (int64_t j = c0 + (int64_t)threadIdx.x * VEC; j < c1; j += (int64_t)kBlock * VEC) {
    float t[VEC], d[VEC], lo[VEC], rlo[VEC];
    load_vec<VEC>(th + j, t);
    load_vec<VEC>(ref.hi + j, d);
    load_vec<VEC>(tl + j, lo);
    load_vec<VEC>(ref.lo + j, rlo);
#pragma unroll
    for (int v = 0; v < VEC; ++v) d[v] = (t[v] - d[v]) + (lo[v] - rlo[v]);
    float x[kRowsPerBlock][VEC];
#pragma unroll
    for (int r = 0; r < kRowsPerBlock; ++r) load_vec<VEC>(xrow[r] + j, x[r]);
#pragma unroll
    for (int r = 0; r < kRowsPerBlock; ++r) {
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        z[r] = fmaf(x[r][v], t[v], z[r]);
        dz[r] = fmaf(x[r][v], d[v], dz[r]);
      }
    }
  }

  __shared__ float red[4][2 * kRowsPerBlock];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int r = 0; r < kRowsPerBlock; ++r) {
    const float zs = wave_sum(z[r]);
    const float ds = wave_sum(dz[r]);
    if (lane == 0) { red[w][2 * r] = zs; red[w][2 * r + 1] = ds; }
  }
  __syncthreads();
  if (threadIdx.x < 2 * kRowsPerBlock) {
    const int r = threadIdx.x >> 1;
    if (r0 + r < s.B) {
      const float v = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
      a.zpart[(((int64_t)m * s.B + r0 + r) * a.nc + blockIdx.x) * 2 + (threadIdx.x & 1)] = v;
    }
  }
}

__device__ __forceinline__ float sigmoidf(float a) { return 1.0f / (1.0f + expf(-a)); }

// grid (ceil(p / (kBlock*VEC)), M); dynamic LDS: B * (2 floats + 1 int64)
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_grad(const LogregArgs a) {
  const DevState &s = a.s;
  extern __shared__ __align__(16) unsigned char smem[];
  int64_t *off_s = reinterpret_cast<int64_t *>(smem);
  float *r_s = reinterpret_cast<float *>(smem + sizeof(int64_t) * s.B);
  float *dr_s = r_s + s.B;
  __shared__ float red[4];

  const int m = a.m0 + blockIdx.y;
  const int64_t k = s.k;
  const int32_t *idx = a.idx + (int64_t)m * s.B;
  const float *yv = static_cast<const float *>(s.y);
  const float invB = 1.0f / (float)s.B;

  for (int b = threadIdx.x; b < s.B; b += kBlock) {
    bool bad = false;
    const int64_t row = clamp_row(s, m, idx[b], &bad);
    const float *zp = a.zpart + ((int64_t)m * s.B + b) * a.nc * 2;
    float z = 0.f, dz = 0.f;
    for (int c = 0; c < a.nc; ++c) { z += zp[2 * c]; dz += zp[2 * c + 1]; }
    const float y = yv[row];
    const float aa = -y * z;                 // -y x.theta
    const float bb = aa + y * dz;            // -y x.theta_ref
    const float sa = sigmoidf(aa);
    r_s[b] = -y * sa * invB;
    dr_s[b] = y * sa * sigmoidf(-bb) * expm1f(y * dz) * invB;
    off_s[b] = row * s.p;
  }
  __syncthreads();

  const int64_t j = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
  float sq = 0.f;
  if (j < s.p) {
    float g[VEC], iv[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { g[v] = 0.f; iv[v] = 0.f; }
    const float *__restrict__ X = s.X + j;
    int b = 0;
    for (; b + 8 <= s.B; b += 8) {
      float x[8][VEC];
#pragma unroll
      for (int u = 0; u < 8; ++u) load_vec<VEC>(X + off_s[b + u], x[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float r = r_s[b + u], dr = dr_s[b + u];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          g[v] = fmaf(r, x[u][v], g[v]);
          iv[v] = fmaf(dr, x[u][v], iv[v]);
        }
      }
    }
    for (; b < s.B; ++b) {
      float x[VEC];
      load_vec<VEC>(X + off_s[b], x);
      const float r = r_s[b], dr = dr_s[b];
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        g[v] = fmaf(r, x[v], g[v]);
        iv[v] = fmaf(dr, x[v], iv[v]);
      }
    }
    float t[VEC], d[VEC], lo[VEC], rlo[VEC];
    const RefPtr ref = theta_ref(s, m, k);
    load_vec<VEC>(s.theta + j, t);
    load_vec<VEC>(ref.hi + j, d);
    load_vec<VEC>(s.theta_lo + j, lo);
    load_vec<VEC>(ref.lo + j, rlo);
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      d[v] = (t[v] - d[v]) + (lo[v] - rlo[v]);
      g[v] = fmaf(s.lam, t[v], g[v]);
      iv[v] = fmaf(s.lam, d[v], iv[v]);
    }
    const int cur = s.sel[m];
    const int64_t mp = (int64_t)s.M * s.p;
    store_vec<VEC>(s.gbuf + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + j, g);
    if (s.rule == CADA_RULE_CADA1) {
      // left-hand side of (workerrule1): fresh innovation minus the stored one
      float st[VEC];
      load_vec<VEC>(s.dtl + (int64_t)cur * mp + (int64_t)m * s.p + j, st);
      store_vec<VEC>(s.dtl + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + j, iv);
#pragma unroll
      for (int v = 0; v < VEC; ++v) { const float e = iv[v] - st[v]; sq = fmaf(e, e, sq); }
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) sq = fmaf(iv[v], iv[v], sq);
    }
  }
  const float tot = block_sum(sq, red);
  if (threadIdx.x == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + blockIdx.x] = tot;
}

// The second pass keeps row offsets and residuals of the B rows in dynamic LDS: 16 bytes per row,
// 64 KB at the largest minibatch, which with the static part needs the allowance raised.
int logreg_init(Ctx *) {
  const int lds = CADA_MAX_B * (int)(sizeof(int64_t) + 2 * sizeof(float));
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_grad<4>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(k_grad<1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  if (e != hipSuccess) { set_error("hipFuncSetAttribute(LDS size) failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

int logreg_gradients(Ctx *c, const int32_t *idx) {
  LogregArgs a;
  a.s = c->s;
  a.s.k = c->k;
  a.idx = idx;
  a.zpart = c->zpart;
  a.nc = c->n_col_chunks;
  a.chunk_cols = c->chunk_cols;
  const DevState &s = c->s;
  const size_t lds = (size_t)s.B * (sizeof(int64_t) + 2 * sizeof(float));
  // Workers are processed in groups: the second pass over a group's rows follows its first
  // pass closely enough for the rows to still be in the memory-side cache.
  const int group = c->logreg_group > 0 ? c->logreg_group : s.M;
  prof_mark(c);
  for (int m0 = 0; m0 < s.M; m0 += group) {
    const int gm = min(group, s.M - m0);
    a.m0 = m0;
    const dim3 g1(c->n_col_chunks, (s.B + kRowsPerBlock - 1) / kRowsPerBlock, gm);
    const dim3 g2(s.n_lhs_part, gm);
    if (c->vec == 4) {
      hipLaunchKernelGGL(k_dots<4>, g1, dim3(kBlock), 0, c->stream, a);
      hipLaunchKernelGGL(k_grad<4>, g2, dim3(kBlock), lds, c->stream, a);
    } else {
      hipLaunchKernelGGL(k_dots<1>, g1, dim3(kBlock), 0, c->stream, a);
      hipLaunchKernelGGL(k_grad<1>, g2, dim3(kBlock), lds, c->stream, a);
    }
  }
  prof_mark(c);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("logistic gradient launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  return CADA_OK;
}


// ------------------------------------------------------------------------------------------
// Evaluation on all the data (not part of an iteration): logistic loss and accuracy per worker.
// grid (kEvalBlocks, M); a wavefront takes one row at a time, the block strides over the
// worker's rows; per-block sums in a fixed order, then one block per worker adds them up.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_eval_rows(const DevState s, double *part) {
  __shared__ double red[4][2];
  const int m = blockIdx.y, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t r0 = s.row_off[m], n = s.row_off[m + 1] - r0;
  double loss = 0.0, hits = 0.0;
  for (int64_t r = (int64_t)blockIdx.x * 4 + w; r < n; r += (int64_t)gridDim.x * 4) {
    const float *x = s.X + (r0 + r) * s.p;
    float z = 0.f;
    for (int64_t j = (int64_t)lane * VEC; j < s.p; j += (int64_t)kWave * VEC) {
      float xv[VEC], tv[VEC], tl[VEC];
      load_vec<VEC>(x + j, xv);
      load_vec<VEC>(s.theta + j, tv);
      load_vec<VEC>(s.theta_lo + j, tl);
#pragma unroll
      for (int v = 0; v < VEC; ++v) z = fmaf(xv[v], tv[v] + tl[v], z);
    }
    z = wave_sum(z);
    const float mg = static_cast<const float *>(s.y)[r0 + r] * z;       // margin y x.theta
    // log(1 + exp(-mg)) without overflow
    loss += (double)(fmaxf(-mg, 0.f) + log1pf(expf(-fabsf(mg))));
    hits += mg > 0.f ? 1.0 : 0.0;
  }
  if (lane == 0) { red[w][0] = loss; red[w][1] = hits; }
  __syncthreads();
  if (threadIdx.x < 2) {
    const int q = threadIdx.x;
    part[((int64_t)m * gridDim.x + blockIdx.x) * 2 + q] = (red[0][q] + red[1][q]) + (red[2][q] + red[3][q]);
  }
}

// acc[m] = (mean loss, mean accuracy) of worker m from its per-block sums.  grid M, one wavefront.
__global__ void k_eval_worker(const DevState s, const double *part, int nparts, double *acc) {
  const int m = blockIdx.x, lane = threadIdx.x;
  double a0 = 0.0, a1 = 0.0;
  for (int i = lane; i < nparts; i += kWave) { a0 += part[((int64_t)m * nparts + i) * 2]; a1 += part[((int64_t)m * nparts + i) * 2 + 1]; }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { a0 += __shfl_xor(a0, o, 64); a1 += __shfl_xor(a1, o, 64); }
  if (lane == 0) {
    const double n = (double)(s.row_off[m + 1] - s.row_off[m]);
    acc[2 * m] = a0 / n;
    acc[2 * m + 1] = a1 / n;
  }
}

// out = mean over the workers (+ the regulariser's (lambda/2)|theta|^2 when lam != 0).  One block.
__global__ __launch_bounds__(kBlock) void k_eval_finish(const DevState s, const double *acc, double *out, int with_reg) {
  __shared__ double red[kBlock];
  double sq = 0.0;
  if (with_reg)
    for (int64_t j = threadIdx.x; j < s.p; j += kBlock) {
      const double t = (double)s.theta[j] + (double)s.theta_lo[j];
      sq += t * t;
    }
  red[threadIdx.x] = sq;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double l = 0.0, a = 0.0;
    for (int m = 0; m < s.M; ++m) { l += acc[2 * m]; a += acc[2 * m + 1]; }
    out[0] = l / (double)s.M + (with_reg ? 0.5 * (double)s.lam * red[0] : 0.0);
    out[1] = a / (double)s.M;
  }
}

void eval_finish(Ctx *c, double *out, int with_reg) {
  hipLaunchKernelGGL(k_eval_finish, dim3(1), dim3(kBlock), 0, c->stream, c->s, c->eval_acc, out, with_reg);
}

// Evaluation for callers that cannot allocate: the per-block sums and the per-worker means live
// in this array instead of in a workspace.  One copy per GPU, held until the process ends and
// shared by every call on that GPU.  In host code the name is only a handle: the address on the
// current device comes from hipGetSymbolAddress, once per device.
constexpr size_t kEvalStaticDoubles = (size_t)CADA_EVAL_NOALLOC_MAX_M * (kEvalBlocks + 1) * 2;   // 2.1 MB
static __device__ __align__(256) double scratch[kEvalStaticDoubles];

constexpr int kMaxDevices = 64;
static double *g_scratch_ptr[kMaxDevices];      // address of `scratch` on each device, null until asked for

// Address of the array on the current device (asked for once per device), or null with the error text set.
static double *eval_scratch() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { set_error("hipGetDevice failed or device index beyond %d", kMaxDevices); return nullptr; }
  double *ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (ptr) return ptr;
  e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) { set_error("hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e)); return nullptr; }
  __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);
  return ptr;
}

int eval_scratch_init() { return eval_scratch() ? CADA_OK : CADA_EHIP; }

int logreg_eval_noalloc(Ctx *c, double *out) {
  const DevState &s = c->s;
  if (s.M > CADA_EVAL_NOALLOC_MAX_M) {
    set_error("cada_eval_noalloc serves at most %d workers (got %d): its fixed scratch array holds no more", CADA_EVAL_NOALLOC_MAX_M, s.M);
    return CADA_EINVAL;
  }
  double *ptr = eval_scratch();
  if (!ptr) return CADA_EHIP;
  // every element the later kernels read is written first by this call: nothing has to start at zero
  double *part = ptr, *acc = ptr + (size_t)s.M * kEvalBlocks * 2;
  const dim3 grid(kEvalBlocks, (unsigned)s.M);
  if (c->vec == 4) hipLaunchKernelGGL(k_eval_rows<4>, grid, dim3(kBlock), 0, c->stream, s, part);
  else hipLaunchKernelGGL(k_eval_rows<1>, grid, dim3(kBlock), 0, c->stream, s, part);
  hipLaunchKernelGGL(k_eval_worker, dim3((unsigned)s.M), dim3(kWave), 0, c->stream, s, part, kEvalBlocks, acc);
  hipLaunchKernelGGL(k_eval_finish, dim3(1), dim3(kBlock), 0, c->stream, s, acc, out, 1);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("evaluation launch failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

int logreg_eval(Ctx *c, double *out) {
  const DevState &s = c->s;
  const dim3 grid(kEvalBlocks, (unsigned)s.M);
  if (c->vec == 4) hipLaunchKernelGGL(k_eval_rows<4>, grid, dim3(kBlock), 0, c->stream, s, c->eval_part);
  else hipLaunchKernelGGL(k_eval_rows<1>, grid, dim3(kBlock), 0, c->stream, s, c->eval_part);
  hipLaunchKernelGGL(k_eval_worker, dim3((unsigned)s.M), dim3(kWave), 0, c->stream, s, c->eval_part, kEvalBlocks, c->eval_acc);
  eval_finish(c, out, 1);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("evaluation launch failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

}  // namespace cada
