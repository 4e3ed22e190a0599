// The communication rule's decision (Algorithm 1: upload iff the condition of Section 2.2
// is violated or tau_m^k >= D; tau bookkeeping) and the server side: stale-gradient
// aggregate nabla^k = (1/M) sum_m (stored gradient of m) and equations (CADA-1)-(CADA-3)
// of Section 1.2, fused with the squared step |theta^{k+1}-theta^k|^2 that the rules'
// right-hand side needs (identity in the proof of Lemma 4 of the supplement:
// |theta^{k+1}-theta^k|^2 = alpha^2 sum_i h_i^2 / (eps + vhat_i)).
#include "cada_internal.h"

namespace cada {

// Sum of the per-block partial sums of the squared step of iteration k-1 (the value of
// ring[(k-1) mod d_max]), in a fixed order; called by the whole block, valid in every thread.
__device__ float last_step_sq(const DevState &s, double *red /* [kBlock] LDS */) {
  // (sixteen loads in flight per thread; the additions keep their order, a missing term adds 0)
  double acc = 0.0;
  for (int i0 = threadIdx.x; i0 < s.n_ring_part; i0 += 16 * kBlock) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) { const int i = i0 + u * kBlock; v[u] = s.ring_part[min(i, s.n_ring_part - 1)]; if (i >= s.n_ring_part) v[u] = 0.f; }
#pragma unroll
    for (int u = 0; u < 16; ++u) acc += (double)v[u];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  const float r = (float)red[0];
  __syncthreads();
  return r;
}

// Left-hand side of condition (LAGrule), Section 2.1: |fresh gradient - stored gradient|^2 per
// worker (the stored one was taken at another iterate on other samples).  grid (blocks, M);
// block b of worker m writes lhs_part[m][b]; the remaining slots are cleared.
__global__ __launch_bounds__(kBlock) void k_lag_lhs(const DevState s) {
  __shared__ float red[4];
  const int m = blockIdx.y;
  const int64_t mp = (int64_t)s.M * s.ps;
  float sq = 0.f;
  if (s.gbuf16) {      // bf16 store (always-upload rule, which only records this value): the rows as they are kept
    const uint16_t *gs = s.gbuf16 + ((int64_t)s.sel[m] * s.M + m) * s.ps16;
    const uint16_t *gf = s.gbuf16 + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.ps16;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < s.p; i += (int64_t)gridDim.x * kBlock) {
      const float d = bf2f(gf[i]) - bf2f(gs[i]);
      sq = fmaf(d, d, sq);
    }
  } else {
    const float *gs = s.gbuf + (int64_t)s.sel[m] * mp + (int64_t)m * s.ps;
    const float *gf = s.gbuf + (int64_t)(1 - s.sel[m]) * mp + (int64_t)m * s.ps;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < s.p; i += (int64_t)gridDim.x * kBlock) {
      const float d = gf[i] - gs[i];
      sq = fmaf(d, d, sq);
    }
  }
  const float tot = block_sum(sq, red);
  float *lp = s.lhs_part + (int64_t)m * s.n_lhs_part;
  if (threadIdx.x == 0) lp[blockIdx.x] = tot;
  if (blockIdx.x == 0)
    for (int t = gridDim.x + threadIdx.x; t < s.n_lhs_part; t += kBlock) lp[t] = 0.f;
}

// S3 of the step: RHS, per-worker decision, tau, pointer swap, trace.  One wavefront per
// worker, four workers per block; every block forms the RHS itself (same operations, same
// value), block 0 records it.
__global__ __launch_bounds__(kBlock) void k_rule(const DevState s, const uint8_t *replay) {
  __shared__ double red[kBlock];
  __shared__ unsigned int cnt;
  const int64_t k = s.k;
  const int last = k > 0 ? (int)((k - 1) % s.d_max) : -1;
  const float newest = k > 0 ? last_step_sq(s, red) : 0.f;
  double sum = 0.0;
  for (int j = 0; j < s.d_max; ++j) sum += (double)(j == last ? newest : s.ring[j]);
  const double rhs = (s.c / (double)s.d_max) * sum;
  if (threadIdx.x == 0) cnt = 0;
  __syncthreads();
  const bool tr = k < s.trace_steps;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int m = blockIdx.x * (kBlock / kWave) + wv;
  if (m < s.M) {
    double lhs = 0.0;
    const float *lp = s.lhs_part + (int64_t)m * s.n_lhs_part;
    for (int t0 = lane; t0 < s.n_lhs_part; t0 += 16 * kWave) {       // sixteen loads in flight, additions in order
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) { const int t = t0 + u * kWave; v[u] = lp[min(t, s.n_lhs_part - 1)]; if (t >= s.n_lhs_part) v[u] = 0.f; }
#pragma unroll
      for (int u = 0; u < 16; ++u) lhs += (double)v[u];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lhs += __shfl_xor(lhs, o, 64);   // fixed tree order
    if (lane == 0) {
      const int32_t tau = s.tau[m];
      const bool own = (s.rule == CADA_RULE_ALWAYS) || (lhs > rhs) || (tau >= s.D);
      bool up = own;
      if (replay != nullptr && replay[m] != CADA_REPLAY_FREE) up = replay[m] != 0;
      if (tr) {
        const int64_t o = k * s.M + m;
        s.t_mask[o] = up ? 1 : 0;
        s.t_own[o] = own ? 1 : 0;
        s.t_lhs[o] = (float)lhs;
        s.t_tau[o] = tau;
      }
      s.lhs[m] = (float)lhs;
      s.mask[m] = up ? 1 : 0;
      if (up) {
        s.tau[m] = 1;
        s.sel[m] ^= 1;       // the fresh row becomes the stored one
        atomicAdd(&cnt, 1u);
      } else {
        s.tau[m] = tau + 1;
        // (only a replay mask can do this: the reference point theta^{k+1-(tau+1)} leaves the D+1 retained iterates)
        if (s.rule == CADA_RULE_CADA2 && tau >= s.D) atomicOr(s.err, 8u);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (cnt) {
      atomicAdd(reinterpret_cast<unsigned long long *>(s.uploads), (unsigned long long)cnt);
      atomicAdd(s.n_up + (k & 1), cnt);
    }
    if (blockIdx.x == 0) {
      if (last >= 0) s.ring[last] = newest;
      if (tr) s.t_rhs[k] = (float)rhs;
    }
  }
}

// One block; used when the state is read out after the last step.
__global__ __launch_bounds__(kBlock) void k_ring_finalize(const DevState s) {
  __shared__ double red[kBlock];
  if (s.k <= 0) return;
  const float newest = last_step_sq(s, red);
  if (threadIdx.x == 0) s.ring[(s.k - 1) % s.d_max] = newest;
}

// S5-S7.  A block owns 256 coordinates, four per lane: consecutive ones read as one 16-byte
// access when every row start is 16-byte aligned (VEC == 4), else the coordinates lane,
// lane + 64, lane + 128, lane + 192 of the block's range (VEC == 1, coalesced scalar accesses).
// Wavefront w sums the stored gradients of workers w, w+4, w+8, ... for them, the four sums
// are combined through LDS in a fixed order, and wavefront 0 applies the update.
// grid = n_ring_part = ceil(p / 256) blocks.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_server(const DevState s) {
  __shared__ float part[4][4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t base = (int64_t)blockIdx.x * 256;
  const int64_t mp = (int64_t)s.M * s.ps;
  // coordinate of this lane's v-th value, and whether it exists
  auto coord = [&](int v) -> int64_t { return VEC == 4 ? base + lane * 4 + v : base + lane + 64 * v; };
  auto get = [&](const float *x, float (&o)[4]) {
    if constexpr (VEC == 4) {
      if (coord(0) < s.p) {
        const float4 t = *reinterpret_cast<const float4 *>(x + coord(0));
        o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w;
      }
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (coord(v) < s.p) o[v] = x[coord(v)];
    }
  };
  auto put = [&](float *x, const float (&o)[4]) {
    if constexpr (VEC == 4) {
      if (coord(0) < s.p) *reinterpret_cast<float4 *>(x + coord(0)) = make_float4(o[0], o[1], o[2], o[3]);
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (coord(v) < s.p) x[coord(v)] = o[v];
    }
  };
  // Aggregate.  Plain form: the sum of all M stored gradients (eq. (CADA-1)).  Incremental form of
  // Section 1.2, nabla^k = nabla^{k-1} + (1/M) sum over the uploading workers of (fresh gradient - the
  // gradient it replaces): taken when it reads fewer rows (2 per upload + 1 against M); the plain
  // sum is formed whenever the host asks for it (every D iterations, and when the stored nabla is not that
  // of the step before), so rounding differences between the two forms cannot pile up.  The choice is
  // the same in every block: it depends on the iteration's upload count alone.
  const uint32_t n_up = s.n_up[s.k & 1];
  const bool incremental = !s.resum && 2 * (int64_t)n_up + 1 < (int64_t)s.M;
  if (blockIdx.x == 0 && threadIdx.x == 0) s.n_up[(s.k + 1) & 1] = 0u;      // (nobody reads that slot during this launch)
  float nab[4] = {0.f, 0.f, 0.f, 0.f};
  auto row_of = [&](int buf, int m) -> const float * { return s.gbuf + (int64_t)buf * mp + (int64_t)m * s.ps; };
  // bf16 store (rows of ps16 elements, 16-byte aligned; VEC == 4 on that path): four coordinates are 8 bytes
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  auto get16 = [&](int buf, int m, float (&o)[4]) {
    if (coord(0) < s.p) {
      const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(s.gbuf16 + ((int64_t)buf * s.M + m) * s.ps16 + coord(0)));
      o[0] = __uint_as_float(t.x << 16); o[1] = __uint_as_float(t.x & 0xffff0000u);
      o[2] = __uint_as_float(t.y << 16); o[3] = __uint_as_float(t.y & 0xffff0000u);
    }
  };
  if (incremental) {
    for (int m = w; m < s.M; m += 4) {
      if (!s.mask[m]) continue;                       // (uniform in the wavefront)
      const int cur = s.sel[m];                       // after the swap: cur holds the fresh gradient, 1 - cur the replaced one
      float a4[4] = {0.f, 0.f, 0.f, 0.f}, b4[4] = {0.f, 0.f, 0.f, 0.f};
      if (VEC == 4 && s.gbuf16) { get16(cur, m, a4); get16(1 - cur, m, b4); }
      else { get(row_of(cur, m), a4); get(row_of(1 - cur, m), b4); }
#pragma unroll
      for (int v = 0; v < 4; ++v) nab[v] += a4[v] - b4[v];
    }
  } else if (VEC == 4 && s.gbuf16) {
#pragma unroll 4
    for (int m = w; m < s.M; m += 4) {
      float t[4] = {0.f, 0.f, 0.f, 0.f};
      get16(s.sel[m], m, t);
#pragma unroll
      for (int v = 0; v < 4; ++v) nab[v] += t[v];
    }
  } else if constexpr (VEC == 4) {
    if (coord(0) < s.p) {
#pragma unroll 5
      for (int m = w; m < s.M; m += 4) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        // (the stored gradients are read once per step: non-temporal loads, which stream from HBM faster)
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(s.gbuf + (int64_t)s.sel[m] * mp + (int64_t)m * s.ps + coord(0)));
        nab[0] += t.x; nab[1] += t.y; nab[2] += t.z; nab[3] += t.w;
      }
    }
  } else {
#pragma unroll 4
    for (int m = w; m < s.M; m += 4) {
      float t[4] = {0.f, 0.f, 0.f, 0.f};
      const float *gm = s.gbuf + (int64_t)s.sel[m] * mp + (int64_t)m * s.ps;
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (coord(v) < s.p) t[v] = __builtin_nontemporal_load(gm + coord(v));
#pragma unroll
      for (int v = 0; v < 4; ++v) nab[v] += t[v];
    }
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) part[w][v][lane] = nab[v];
  __syncthreads();
  if (w != 0) return;
  float sq = 0.f;
  const float fM = (float)s.M;
  float th[4] = {0.f, 0.f, 0.f, 0.f}, tl[4] = {0.f, 0.f, 0.f, 0.f}, hh[4] = {0.f, 0.f, 0.f, 0.f};
  float vv[4], vh[4] = {0.f, 0.f, 0.f, 0.f};
  float prev[4] = {0.f, 0.f, 0.f, 0.f};
  get(s.h, hh); get(s.vhat, vh); get(s.theta, th); get(s.theta_lo, tl);
  if (incremental) get(s.nabla, prev);
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    nab[v] = prev[v] + ((part[0][v][lane] + part[1][v][lane]) + (part[2][v][lane] + part[3][v][lane])) / fM;
    // beta*x + (1-beta)*y written as x + (1-beta)*(y - x): float32(0.999) is off by 1.3e-8
    // relative, which compounds to 1e-5 over the ~1000-step memory of vhat, whereas
    // float32(1-beta) enters only linearly
    const float ho = hh[v];
    const float vo = vh[v];
    float step;
    if (s.server_sgd) {          // theta <- theta - alpha * nabla; h, v, vhat keep their zeros
      vv[v] = vo;
      step = s.alpha * nab[v];
    } else {
      hh[v] = fmaf(s.omb1, nab[v] - ho, ho);
      vv[v] = fmaf(s.omb2, nab[v] * nab[v] - vo, vo);
      vh[v] = fmaxf(vv[v], vo);
      step = s.alpha * hh[v] / sqrtf(s.eps + vh[v]);
    }
    if (VEC == 4 && coord(v) >= s.p) step = 0.f;   // (a coordinate of the 16-byte padding past p stays as it is, also with eps = 0)
    // (theta, theta_lo) - step in two-float arithmetic (TwoSum, then renormalise)
    const float a = th[v], ms = -step;
    const float sum = a + ms;
    const float bb = sum - a;
    const float err = (a - (sum - bb)) + (ms - bb);
    const float lo = tl[v] + err;
    th[v] = sum + lo;
    tl[v] = lo - (th[v] - sum);
    if (coord(v) < s.p) sq = fmaf(step, step, sq);
  }
  put(s.nabla, nab); put(s.h, hh); put(s.v, vv); put(s.vhat, vh); put(s.theta, th); put(s.theta_lo, tl);
  if (s.rule == CADA_RULE_CADA2) {
    put(s.hist + ((s.k + 1) % s.R) * s.ps, th);
    put(s.hist_lo + ((s.k + 1) % s.R) * s.ps, tl);
  } else if (s.rule == CADA_RULE_CADA1 && (s.k + 1) % s.D == 0) {
    put(s.snap, th);
    put(s.snap_lo, tl);
  }
  const float tot = wave_sum(sq);
  if (lane == 0) s.ring_part[blockIdx.x] = tot;
}

int rule_and_server(Ctx *c, const uint8_t *replay) {
  DevState s = c->s;
  s.k = c->k;
  s.alpha = stepsize(s, s.k);
  s.resum = (c->force_resum || s.k % s.D == 0) ? 1 : 0;
  if (s.rule == CADA_RULE_LAG || s.rule == CADA_RULE_ALWAYS) {   // (the always-upload rule only records it)
    const int nb = (int)min((int64_t)s.n_lhs_part, (s.p + 4 * kBlock - 1) / (4 * kBlock));
    hipLaunchKernelGGL(k_lag_lhs, dim3((unsigned)max(nb, 1), (unsigned)s.M), dim3(kBlock), 0, c->stream, s);
  }
  hipLaunchKernelGGL(k_rule, dim3((unsigned)((s.M + 3) / 4)), dim3(kBlock), 0, c->stream, s, replay);
  prof_mark(c);
  if (c->vec == 4)
    hipLaunchKernelGGL(k_server<4>, dim3(s.n_ring_part), dim3(kBlock), 0, c->stream, s);
  else
    hipLaunchKernelGGL(k_server<1>, dim3(s.n_ring_part), dim3(kBlock), 0, c->stream, s);
  prof_mark(c);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("rule/server launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  c->force_resum = 0;
  return CADA_OK;
}

int ring_finalize(Ctx *c) {
  DevState s = c->s;
  s.k = c->k;
  hipLaunchKernelGGL(k_ring_finalize, dim3(1), dim3(kBlock), 0, c->stream, s);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("ring finalize launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  return CADA_OK;
}

}  // namespace cada
