// The communication rule's decision (Algorithm 1: upload iff the condition of Section 2.2
// is violated or tau_m^k >= D; tau bookkeeping) and the server side: stale-gradient
// aggregate nabla^k = (1/M) sum_m (stored gradient of m) and equations (CADA-1)-(CADA-3)
// of Section 1.2, fused with the squared step |theta^{k+1}-theta^k|^2 that the rules'
// right-hand side needs (identity in the proof of Lemma 4 of the supplement:
// |theta^{k+1}-theta^k|^2 = alpha^2 sum_i h_i^2 / (eps + vhat_i)).
#include "cada_internal.h"

namespace cada {

// Folds the per-block partial sums of the squared step of iteration k-1 into
// ring[(k-1) mod d_max].  Called by the whole block; fixed summation order.
__device__ void finalize_ring(const DevState &s, int64_t k, double *red /* [kBlock] LDS */) {
  if (k <= 0) return;
  double acc = 0.0;
  for (int i = threadIdx.x; i < s.n_ring_part; i += kBlock) acc += (double)s.ring_part[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) s.ring[(k - 1) % s.d_max] = (float)red[0];
  __syncthreads();
}

// One block.  S3 of the step: RHS, per-worker decision, tau, pointer swap, trace.
__global__ __launch_bounds__(kBlock) void k_rule(const DevState s, const uint8_t *replay) {
  __shared__ double red[kBlock];
  __shared__ double rhs_s;
  __shared__ unsigned int cnt;
  const int64_t k = s.k;
  finalize_ring(s, k, red);
  if (threadIdx.x == 0) {
    double sum = 0.0;
    for (int j = 0; j < s.d_max; ++j) sum += (double)s.ring[j];
    rhs_s = (s.c / (double)s.d_max) * sum;
    cnt = 0;
  }
  __syncthreads();
  const double rhs = rhs_s;
  const bool tr = k < s.trace_steps;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  for (int m = wv; m < s.M; m += kBlock / kWave) {     // one wavefront per worker
    double lhs = 0.0;
    const float *lp = s.lhs_part + (int64_t)m * s.n_lhs_part;
    for (int t = lane; t < s.n_lhs_part; t += kWave) lhs += (double)lp[t];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lhs += __shfl_xor(lhs, o, 64);   // fixed tree order
    if (lane != 0) continue;
    const int32_t tau = s.tau[m];
    const bool own = (lhs > rhs) || (tau >= s.D);
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
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    *s.uploads += cnt;
    if (tr) s.t_rhs[k] = (float)rhs;
  }
}

// One block; used when the state is read out after the last step.
__global__ __launch_bounds__(kBlock) void k_ring_finalize(const DevState s) {
  __shared__ double red[kBlock];
  finalize_ring(s, s.k, red);
}

// S5-S7.  grid = n_ring_part blocks, one (VEC-wide) coordinate group per thread.
template <int VEC>
__global__ __launch_bounds__(kBlock) void k_server(const DevState s) {
  __shared__ float red[4];
  const int64_t j = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
  const int64_t mp = (int64_t)s.M * s.p;
  float sq = 0.f;
  if (j < s.p) {
    float nab[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) nab[v] = 0.f;
    for (int m = 0; m < s.M; ++m) {
      const float *row = s.gbuf + (int64_t)s.sel[m] * mp + (int64_t)m * s.p + j;
      if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(row);
        nab[0] += t.x; nab[1] += t.y; nab[2] += t.z; nab[3] += t.w;
      } else {
        nab[0] += *row;
      }
    }
    const float fM = (float)s.M;
    float th[VEC], tl[VEC], hh[VEC], vv[VEC], vh[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int64_t i = j + v;
      nab[v] = nab[v] / fM;
      // beta*x + (1-beta)*y written as x + (1-beta)*(y - x): float32(0.999) is off by 1.3e-8
      // relative, which compounds to 1e-5 over the ~1000-step memory of vhat, whereas
      // float32(1-beta) enters only linearly
      const float ho = s.h[i];
      hh[v] = fmaf(s.omb1, nab[v] - ho, ho);
      const float vo = s.vhat[i];
      vv[v] = fmaf(s.omb2, nab[v] * nab[v] - vo, vo);
      vh[v] = fmaxf(vv[v], vo);
      const float step = s.alpha * hh[v] / sqrtf(s.eps + vh[v]);
      // (theta, theta_lo) - step in two-float arithmetic (TwoSum, then renormalise)
      const float a = s.theta[i], ms = -step;
      const float sum = a + ms;
      const float bb = sum - a;
      const float err = (a - (sum - bb)) + (ms - bb);
      const float lo = s.theta_lo[i] + err;
      th[v] = sum + lo;
      tl[v] = lo - (th[v] - sum);
      sq = fmaf(step, step, sq);
    }
    const bool snap = (s.rule == CADA_RULE_CADA1) && ((s.k + 1) % s.D == 0);
    float *hs = (s.rule == CADA_RULE_CADA2) ? s.hist + ((s.k + 1) % s.R) * s.p : nullptr;
    float *hl = (s.rule == CADA_RULE_CADA2) ? s.hist_lo + ((s.k + 1) % s.R) * s.p : nullptr;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      const int64_t i = j + v;
      s.nabla[i] = nab[v];
      s.h[i] = hh[v];
      s.v[i] = vv[v];
      s.vhat[i] = vh[v];
      s.theta[i] = th[v];
      s.theta_lo[i] = tl[v];
      if (hs) { hs[i] = th[v]; hl[i] = tl[v]; }
      if (snap) { s.snap[i] = th[v]; s.snap_lo[i] = tl[v]; }
    }
  }
  const float tot = block_sum(sq, red);
  if (threadIdx.x == 0) s.ring_part[blockIdx.x] = tot;
}

int rule_and_server(Ctx *c, const uint8_t *replay) {
  DevState s = c->s;
  s.k = c->k;
  hipLaunchKernelGGL(k_rule, dim3(1), dim3(kBlock), 0, c->stream, s, replay);
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
