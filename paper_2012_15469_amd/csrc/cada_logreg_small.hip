// Whole iterations of Algorithm 1 in one kernel launch, for logistic workloads so small that a
// step is bound by launch and dependency latency rather than by memory (tens of workers, a few
// hundred coordinates): four dependent launches per step cost 35-40 us, the arithmetic well
// under one.  One workgroup per worker, launched cooperatively; n_steps iterations per launch
// with ONE grid-wide barrier each:
//   phase A (workgroup m = worker m): both minibatch gradients in the difference form of
//     cada_logreg.hip, the rule's left-hand side, the right-hand side from the ring, the
//     decision, tau, the stored/fresh pointer swap, the trace           [S1-S4 of the step]
//   -- barrier --
//   phase B (EVERY workgroup, all coordinates): aggregate of the stored gradients, the server
//     update, the squared step                                          [S5-S7]
// Every workgroup keeps the server's vectors (iterate, moments, snapshot) in its LDS and applies the same update
// to them, in the same order, so all copies stay bit for bit equal and the next phase A needs neither a second
// barrier nor the iterate from memory; workgroup (j / 256) mod M writes coordinate j's results to memory for
// the world outside and for the reference points theta^{k - tau}, tau >= 1, which are read a barrier later at
// the earliest.  What a fast workgroup writes in phase A of step k + 1 while a slow one is still in phase B of
// step k never is what the slow one reads: the fresh gradient goes to the row that is not the stored one, and
// the decisions of step k are published in slot k mod 2 of an array of their own.
// The barrier is that array: a workgroup's word carries the step's tag, its publication releases (writes back) and a
// workgroup that has seen every word of the step acquires (invalidates) the XCD-local caches.  Every wait is bounded:
// a wait that exceeds the bound sets bit 1 of the error flags and the workgroup stops waiting.
#include <cstring>
#include <new>
#include <type_traits>

#include "cada_internal.h"

namespace cada {

struct SmallArgs {
  DevState s;
  const int32_t *idx;        // [n_steps][M][B]
  const uint8_t *replay;     // [n_steps][M] or nullptr
  int64_t n_steps;
  uint32_t *bar;             // barrier words: [64 unused][2][M] {tag, selector} of the last two steps
  uint32_t bar_base;         // sequence number of this launch's first step (monotone over the life of the context)
  uint32_t spin_limit;
};
static_assert(sizeof(SmallArgs) <= kSmallArgsBytes, "room kept in the workspace for a replica launch");

// One launch serves one run (its arguments by value) or several independent runs (blockIdx.y
// picks the run).  A run's arguments that do not change from launch to launch (where its state
// lies) are kept in its own workspace, written once when the context is set up; what changes
// (schedules, iteration, barrier count) travels by value with the launch.
struct SmallVar {
  const int32_t *idx;
  const uint8_t *replay;
  int64_t k;
  uint32_t bar_base;
};
struct SmallLaunch {
  SmallArgs one;
  const SmallArgs *rep[CADA_MAX_REPLICAS];
  SmallVar var[CADA_MAX_REPLICAS];
  int64_t n_steps;
  int n_rep;                 // 0: `one`
};
static_assert(sizeof(SmallLaunch) <= 4096, "kernel arguments");

__device__ __forceinline__ float sigmoid_s(float a) { return 1.0f / (1.0f + expf(-a)); }

// The barrier of a step is also how the decisions travel.  Workgroup m publishes the word {tag of the step, its
// worker's buffer selector after the decision} with a release, in slot (step parity, m) of an array in the workspace; a
// workgroup has passed the barrier when the first wavefront, one lane per worker, has seen this step's tag in every
// word -- and then it holds every decision, which a counter plus a separate array cost a memory round trip more.
// (Two slots per worker: a workgroup can be one step ahead of another at most, so the word that a slow workgroup
// still waits for is not overwritten.  A tag is never 0, the value of a fresh workspace.)
// `while_waiting` runs between this workgroup's publication and its wait: loads issued there are under way while
// the others arrive.  dk_s[M] (LDS) receives the selectors; the function ends with a workgroup barrier.
template <typename F>
__device__ __forceinline__ void decision_barrier(const SmallArgs &a, uint32_t *words /* [M] of this parity */, int M, int m, uint32_t tag, int sel,
                                                 unsigned char *dk_s, bool &dead, F while_waiting) {
  __syncthreads();                      // every thread's stores have reached the L2 (the barrier waits for them) ...
  // ... and the publication releases at agent scope: it writes the L2's dirty lines back before the word changes
  if (threadIdx.x == 0) __hip_atomic_store(words + m, (tag << 1) | (uint32_t)sel, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
  while_waiting();
  if (threadIdx.x < kWave) {
    const int lane = threadIdx.x;
    for (int m0 = 0; m0 < M; m0 += kWave) {
      const int mm = m0 + lane;
      uint32_t v = 0, spins = 0;
      // (relaxed polls: the fence below is the acquire, once, instead of a cache invalidation per poll)
      for (;;) {
        if (mm < M) v = __hip_atomic_load(words + mm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ok = mm >= M || (v >> 1) == tag;
        if (dead || __all(ok)) break;
        if (++spins > a.spin_limit) { dead = true; if (lane == 0) atomicOr(a.s.err, 2u); break; }    // (the whole wavefront: spins is uniform)
        __builtin_amdgcn_s_sleep(2);
      }
      if (mm < M) dk_s[mm] = (unsigned char)(v & 1u);
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // acquire: drop stale cached lines
}

// grid = M workgroups of kBlock threads; dynamic LDS: the server's vectors and theta - theta_ref (7 p floats), r, dr,
// row offsets (B each) and the worker's whole minibatch (B p floats): the rows are fetched once, with every
// load independent of the others, and both passes over them run from LDS
__global__ __launch_bounds__(kBlock) void k_small(const SmallLaunch launch) {
  extern __shared__ __align__(16) unsigned char small_smem[];
  SmallArgs a = launch.n_rep ? *launch.rep[blockIdx.y] : launch.one;
  if (launch.n_rep) {
    const SmallVar &v = launch.var[blockIdx.y];
    a.idx = v.idx; a.replay = v.replay; a.s.k = v.k; a.bar_base = v.bar_base; a.n_steps = launch.n_steps;
  }
  DevState s = a.s;
  const int p = (int)s.p, B = s.B, M = s.M;
  float *th_s = reinterpret_cast<float *>(small_smem);     // [p] theta, [p] theta_lo, [p] h, [p] vhat: this workgroup's copies
  float *tl_s = th_s + p, *h_s = tl_s + p, *vh_s = h_s + p;
  float *sn_s = vh_s + p, *snl_s = sn_s + p;               // [p] each: CADA1's snapshot
  float *d_s = snl_s + p;                                  // [p] theta - theta_ref
  float *r_s = d_s + p;                                    // [B]
  float *dr_s = r_s + B;                                   // [B]
  long long *row_s = reinterpret_cast<long long *>(dr_s + B + ((7 * p + 2 * B) & 1));   // [B], 8-byte aligned
  long long *row_n = row_s + B;                            // [B] rows of the NEXT step's minibatch (row numbers)
  const size_t x_off = ((size_t)(reinterpret_cast<unsigned char *>(row_n + B) - small_smem) + 15) & ~(size_t)15;
  float *x_s = reinterpret_cast<float *>(small_smem + x_off);        // [B][p] the minibatch, 16-byte aligned
  // rows and columns are moved four floats at a time when every row starts on a 16-byte boundary
  const bool v4 = (p & 3) == 0 && (reinterpret_cast<uintptr_t>(s.X) & 15) == 0;
  __shared__ float red[4];
  __shared__ double redd[kBlock];
  __shared__ float bcast[2];
  __shared__ float ring_s[CADA_MAX_DMAX];      // the squared steps, kept up to date by every workgroup for itself
  __shared__ unsigned char dk_s[256];          // the workers' buffer selectors after this step's decisions (M <= CUs <= 256)

  const int m = blockIdx.x, nb = gridDim.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t mp = (int64_t)M * s.p;
  const float invB = 1.0f / (float)B;
  bool dead = false;
  // What only this workgroup changes during the launch -- its worker's delay and buffer selector -- and what every
  // workgroup can keep up to date by itself -- the ring of squared steps -- is read from memory once: a step is a
  // chain of dependent memory round trips, and each one taken off it is a microsecond.
  int32_t tau_m = s.tau[m];
  int cur = s.sel[m];
  const int64_t base = s.row_off[m], n_m = s.row_off[m + 1] - base;
  for (int j = tid; j < s.d_max; j += kBlock) ring_s[j] = s.ring[j];
  for (int j = tid; j < p; j += kBlock) {
    th_s[j] = s.theta[j]; tl_s[j] = s.theta_lo[j]; h_s[j] = s.h[j]; vh_s[j] = s.vhat[j];
    if (s.rule == CADA_RULE_CADA1) { sn_s[j] = s.snap[j]; snl_s[j] = s.snap_lo[j]; }
  }
  uint32_t *dec = a.bar + 64;                  // [2][M] {tag, selector after the decision} of step k in slot k mod 2
  // the squared step of the iteration before this launch: partial sums that the launch before (or cada_set_state) left
  float newest_c = 0.f;
  {
    double acc = 0.0;
    if (s.k > 0)
      for (int i = tid; i < s.n_ring_part; i += kBlock) acc += (double)s.ring_part[i];
    redd[tid] = acc;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) {
      if (tid < o) redd[tid] += redd[tid + o];
      __syncthreads();
    }
    newest_c = (float)redd[0];
  }

  // The next step's rows and labels are asked for while this workgroup waits at the barrier (LDS-direct loads: no
  // registers, and the buffers they land in are free by then), so only the first step of a launch fetches its own.
  bool have_rows = false;
  constexpr int NW = kBlock / kWave, RB = 8;
  for (int64_t step = 0; step < a.n_steps; ++step) {
    const int64_t k = s.k + step;
    const bool more = step + 1 < a.n_steps;
    // ------------------------------------------------------------ phase A
    if (s.rule == CADA_RULE_CADA2) {           // theta^{k - tau}: written a barrier ago at the latest (tau >= 1)
      const RefPtr ref = theta_ref_at(s, tau_m, k);
      for (int j = tid; j < p; j += kBlock) d_s[j] = (th_s[j] - ref.hi[j]) + (tl_s[j] - ref.lo[j]);
    } else if (s.rule == CADA_RULE_CADA1) {
      for (int j = tid; j < p; j += kBlock) d_s[j] = (th_s[j] - sn_s[j]) + (tl_s[j] - snl_s[j]);
    } else {
      for (int j = tid; j < p; j += kBlock) d_s[j] = 0.f;
    }
    const int32_t *idx = a.idx + (step * M + m) * (int64_t)B;
    for (int b = tid; b < B; b += kBlock) {
      if (!have_rows) {
        int64_t r = idx[b];
        if (r < 0 || r >= n_m) { atomicOr(s.err, 1u); r = r < 0 ? 0 : n_m - 1; }
        row_s[b] = (base + r) * s.p;
      }
      if (more) {
        int64_t r = idx[(int64_t)M * B + b];
        if (r < 0 || r >= n_m) { atomicOr(s.err, 1u); r = r < 0 ? 0 : n_m - 1; }
        row_n[b] = base + r;
      }
    }
    __syncthreads();
    // the rows: wavefront w fetches rows w, w+4, ..., eight rows at a time so that eight loads per
    // lane are in flight (no division per element; every load independent of the others)
    if (!have_rows) {
    for (int b0 = w; b0 < B; b0 += NW * RB) {
      const float *src[RB];
#pragma unroll
      for (int q = 0; q < RB; ++q) src[q] = s.X + row_s[min(b0 + NW * q, B - 1)];      // (a row past the end repeats the last one and is dropped)
      if (v4) {
#pragma unroll 2
        for (int j = lane * 4; j < p; j += 4 * kWave) {
          float4 v[RB];
#pragma unroll
          for (int q = 0; q < RB; ++q) v[q] = *reinterpret_cast<const float4 *>(src[q] + j);
#pragma unroll
          for (int q = 0; q < RB; ++q)
            if (b0 + NW * q < B) *reinterpret_cast<float4 *>(x_s + (b0 + NW * q) * p + j) = v[q];
        }
      } else {
#pragma unroll 2
        for (int j = lane; j < p; j += kWave) {
          float v[RB];
#pragma unroll
          for (int q = 0; q < RB; ++q) v[q] = src[q][j];
#pragma unroll
          for (int q = 0; q < RB; ++q)
            if (b0 + NW * q < B) x_s[(b0 + NW * q) * p + j] = v[q];
        }
      }
    }
    if (tid < B) r_s[tid] = static_cast<const float *>(s.y)[row_s[tid] / s.p];     // the labels, for now
    for (int b = kBlock + tid; b < B; b += kBlock) r_s[b] = static_cast<const float *>(s.y)[row_s[b] / s.p];
    }
    __syncthreads();
    // rows over the wavefronts, RP at a time per wavefront (their 2 RP reductions overlap; RP = 8 for more than 16
    // rows, so that 32 rows are one pass): z = x.theta, dz = x.d, then the residual and its difference
    auto products = [&](auto RPc) __attribute__((always_inline)) {
      constexpr int RP = decltype(RPc)::value;
      for (int b0 = w; b0 < B; b0 += RP * NW) {
        const float *x[RP];
        float z[RP], dz[RP];
#pragma unroll
        for (int q = 0; q < RP; ++q) { z[q] = 0.f; dz[q] = 0.f; x[q] = x_s + min(b0 + q * NW, B - 1) * p; }   // (a row past the end repeats the last one and is dropped)
        if (v4) {
          for (int j = lane * 4; j < p; j += 4 * kWave) {
            const float4 th = *reinterpret_cast<const float4 *>(th_s + j), dd = *reinterpret_cast<const float4 *>(d_s + j);
#pragma unroll
            for (int q = 0; q < RP; ++q) {
              const float4 xv = *reinterpret_cast<const float4 *>(x[q] + j);
              z[q] = fmaf(xv.x, th.x, z[q]); z[q] = fmaf(xv.y, th.y, z[q]); z[q] = fmaf(xv.z, th.z, z[q]); z[q] = fmaf(xv.w, th.w, z[q]);
              dz[q] = fmaf(xv.x, dd.x, dz[q]); dz[q] = fmaf(xv.y, dd.y, dz[q]); dz[q] = fmaf(xv.z, dd.z, dz[q]); dz[q] = fmaf(xv.w, dd.w, dz[q]);
            }
          }
        } else {
          for (int j = lane; j < p; j += kWave) {
            const float th = th_s[j], dd = d_s[j];
#pragma unroll
            for (int q = 0; q < RP; ++q) {
              const float xv = x[q][j];
              z[q] = fmaf(xv, th, z[q]);
              dz[q] = fmaf(xv, dd, dz[q]);
            }
          }
        }
#pragma unroll
        for (int q = 0; q < RP; ++q) { z[q] = wave_sum_dpp(z[q]); dz[q] = wave_sum_dpp(dz[q]); }
        {   // lane q takes row q of the RP (every lane holds all the sums): the exponentials of RP rows side by side
          float zq = z[0], dq = dz[0];
#pragma unroll
          for (int q = 1; q < RP; ++q) { zq = lane == q ? z[q] : zq; dq = lane == q ? dz[q] : dq; }
          const int b = b0 + lane * NW;
          if (lane < RP && b < B) {
            const float y = r_s[b];
            const float aa = -y * zq, bb = aa + y * dq;
            const float sa = sigmoid_s(aa);
            r_s[b] = -y * sa * invB;
            dr_s[b] = y * sa * sigmoid_s(-bb) * expm1f(y * dq) * invB;
          }
        }
      }
    };
    if (B > 16) products(std::integral_constant<int, 8>{}); else products(std::integral_constant<int, 4>{});
    __syncthreads();
    // columns over the threads: fresh gradient, innovation, the rule's left-hand side
    float *gf = s.gbuf + (int64_t)(1 - cur) * mp + (int64_t)m * s.p;
    const float *gs = s.gbuf + (int64_t)cur * mp + (int64_t)m * s.p;
    float sq = 0.f;
    if (v4) {
      for (int j = tid * 4; j < p; j += 4 * kBlock) {
        float g[4] = {0.f, 0.f, 0.f, 0.f}, iv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int b = 0; b < B; ++b) {
          const float4 xv = *reinterpret_cast<const float4 *>(x_s + b * p + j);
          const float rb = r_s[b], db = dr_s[b];
          g[0] = fmaf(rb, xv.x, g[0]); g[1] = fmaf(rb, xv.y, g[1]); g[2] = fmaf(rb, xv.z, g[2]); g[3] = fmaf(rb, xv.w, g[3]);
          iv[0] = fmaf(db, xv.x, iv[0]); iv[1] = fmaf(db, xv.y, iv[1]); iv[2] = fmaf(db, xv.z, iv[2]); iv[3] = fmaf(db, xv.w, iv[3]);
        }
        float st[4] = {0.f, 0.f, 0.f, 0.f};
        const int64_t o = (int64_t)m * s.p + j;
        if (s.rule == CADA_RULE_CADA1) {
          const float4 t = *reinterpret_cast<const float4 *>(s.dtl + (int64_t)cur * mp + o);
          st[0] = t.x; st[1] = t.y; st[2] = t.z; st[3] = t.w;
        } else if (s.rule != CADA_RULE_CADA2) {
          const float4 t = *reinterpret_cast<const float4 *>(gs + j);
          st[0] = t.x; st[1] = t.y; st[2] = t.z; st[3] = t.w;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          g[q] = fmaf(s.lam, th_s[j + q], g[q]);
          iv[q] = fmaf(s.lam, d_s[j + q], iv[q]);
          float lhs_term = iv[q];
          if (s.rule == CADA_RULE_CADA1) lhs_term = iv[q] - st[q];
          else if (s.rule != CADA_RULE_CADA2) lhs_term = g[q] - st[q];          // condition (LAGrule): against the stored gradient
          sq = fmaf(lhs_term, lhs_term, sq);
        }
        if (s.rule == CADA_RULE_CADA1) *reinterpret_cast<float4 *>(s.dtl + (int64_t)(1 - cur) * mp + o) = make_float4(iv[0], iv[1], iv[2], iv[3]);
        *reinterpret_cast<float4 *>(gf + j) = make_float4(g[0], g[1], g[2], g[3]);
      }
    } else
    for (int j = tid; j < p; j += kBlock) {
      float g = 0.f, iv = 0.f;
      for (int b = 0; b < B; ++b) {
        const float xv = x_s[b * p + j];
        g = fmaf(r_s[b], xv, g);
        iv = fmaf(dr_s[b], xv, iv);
      }
      g = fmaf(s.lam, th_s[j], g);
      iv = fmaf(s.lam, d_s[j], iv);
      float lhs_term = iv;
      if (s.rule == CADA_RULE_CADA1) {
        const int64_t o = (int64_t)m * s.p + j;
        s.dtl[(int64_t)(1 - cur) * mp + o] = iv;
        lhs_term = iv - s.dtl[(int64_t)cur * mp + o];
      } else if (s.rule != CADA_RULE_CADA2) {
        lhs_term = g - gs[j];                 // condition (LAGrule): against the stored gradient
      }
      gf[j] = g;
      sq = fmaf(lhs_term, lhs_term, sq);
    }
    const float lhs = block_sum_lds(sq, red);
    // right-hand side: the squared step of iteration k-1 is this workgroup's own sum of the step before
    if (tid == 0) {
      const int last = k > 0 ? (int)((k - 1) % s.d_max) : -1;
      const float newest = newest_c;
      double sum = 0.0;
      if (last >= 0) ring_s[last] = newest;
      for (int j = 0; j < s.d_max; ++j) sum += (double)ring_s[j];
      const double rhs = (s.c / (double)s.d_max) * sum;
      const int32_t tau = tau_m;
      const bool own = (s.rule == CADA_RULE_ALWAYS) || ((double)lhs > rhs) || (tau >= s.D);
      bool up = own;
      const uint8_t *replay = a.replay ? a.replay + step * M : nullptr;
      if (replay != nullptr && replay[m] != CADA_REPLAY_FREE) up = replay[m] != 0;
      if (k < s.trace_steps) {
        const int64_t o = k * M + m;
        s.t_mask[o] = up ? 1 : 0;
        s.t_own[o] = own ? 1 : 0;
        s.t_lhs[o] = lhs;
        s.t_tau[o] = tau;
        if (m == 0) s.t_rhs[k] = (float)rhs;
      }
      s.lhs[m] = lhs;
      s.mask[m] = up ? 1 : 0;
      if (up) {
        s.tau[m] = 1;
        s.sel[m] = cur ^ 1;
        atomicAdd(reinterpret_cast<unsigned long long *>(s.uploads), 1ull);
      } else {
        s.tau[m] = tau + 1;
        if (s.rule == CADA_RULE_CADA2 && tau >= s.D) atomicOr(s.err, 8u);   // (a replay mask outlasting the retained iterates)
      }
      bcast[0] = newest;
      bcast[1] = up ? 1.f : 0.f;
    }
    lds_sync();
    if (bcast[1] != 0.f) { tau_m = 1; cur ^= 1; } else tau_m += 1;
    const uint32_t tag = ((a.bar_base + (uint32_t)step) & 0x3fffffffu) + 1u;      // (bar_base advances by n_steps M >= n_steps per launch)
    decision_barrier(a, dec + (k & 1) * M, M, m, tag, cur, dk_s, dead, [&]() __attribute__((always_inline)) {
      if (!more) return;
      // (x_s and r_s were last read by the gradient pass, several workgroup barriers ago)
      for (int b = w; b < B; b += NW) {
        const float *src = s.X + row_n[b] * s.p;
        float *dst = x_s + (size_t)b * p;
        if (v4) {
          for (int j0 = 0; j0 < p; j0 += 4 * kWave)
            if (j0 + lane * 4 < p) __builtin_amdgcn_global_load_lds(src + j0 + lane * 4, (__attribute__((address_space(3))) void *)(dst + j0), 16, 0, 0);
        } else {
          for (int j0 = 0; j0 < p; j0 += kWave)
            if (j0 + lane < p) __builtin_amdgcn_global_load_lds(src + j0 + lane, (__attribute__((address_space(3))) void *)(dst + j0), 4, 0, 0);
        }
      }
      for (int b0 = w * kWave; b0 < B; b0 += NW * kWave)
        if (b0 + lane < B)
          __builtin_amdgcn_global_load_lds(static_cast<const float *>(s.y) + row_n[b0 + lane],
                                           (__attribute__((address_space(3))) void *)(r_s + b0), 4, 0, 0);
    });
    have_rows = more;
    // ------------------------------------------------------------ phase B
    if (m == 0 && tid == 0 && k > 0) s.ring[(k - 1) % s.d_max] = bcast[0];   // (for the world outside: every workgroup has its own copy)
    float sqs = 0.f;
    const float alpha = stepsize(s, k);
    const unsigned char *dk = dk_s;
    const bool snap_now = s.rule == CADA_RULE_CADA1 && (k + 1) % s.D == 0;
    // one coordinate: this workgroup's copies of the server's vectors, and its share of the results in memory
    auto update = [&](int j, float nab) __attribute__((always_inline)) {
      nab = nab / (float)M;
      float hh = h_s[j], vh = vh_s[j], vv = vh, stp;
      if (s.server_sgd) {
        stp = alpha * nab;
      } else {
        hh = fmaf(s.omb1, nab - hh, hh);
        vv = fmaf(s.omb2, nab * nab - vh, vh);
        vh = fmaxf(vv, vh);
        stp = alpha * hh / sqrtf(s.eps + vh);
      }
      // (theta, theta_lo) - step in two-float arithmetic (TwoSum, then renormalise)
      const float t0 = th_s[j], ms = -stp;
      const float sum = t0 + ms;
      const float bb = sum - t0;
      const float er = (t0 - (sum - bb)) + (ms - bb);
      const float lo = tl_s[j] + er;
      const float th = sum + lo, tl = lo - (th - sum);
      h_s[j] = hh; vh_s[j] = vh; th_s[j] = th; tl_s[j] = tl;
      if (snap_now) { sn_s[j] = th; snl_s[j] = tl; }
      if ((j / kBlock) % nb == m) {
        s.nabla[j] = nab; s.h[j] = hh; s.v[j] = vv; s.vhat[j] = vh; s.theta[j] = th; s.theta_lo[j] = tl;
        if (s.rule == CADA_RULE_CADA2) {
          s.hist[((k + 1) % s.R) * s.p + j] = th;
          s.hist_lo[((k + 1) % s.R) * s.p + j] = tl;
        } else if (snap_now) {
          s.snap[j] = th;
          s.snap_lo[j] = tl;
        }
      }
      sqs = fmaf(stp, stp, sqs);
    };
    // The aggregate: every load of a thread is independent of the others (the selectors are one cheap read for all),
    // four coordinates per 16-byte load where the rows allow it; the sum runs over the workers in their order.
    if (v4) {
      // (NG workers' rows asked for before the first is added: the sum is a chain of memory round trips otherwise;
      // 16 at a time, 32 when there are more workers than 16)
      auto aggregate = [&](auto NGc) __attribute__((always_inline)) {
        constexpr int NG = decltype(NGc)::value;
        for (int j = tid * 4; j < p; j += 4 * kBlock) {
          float4 nab = make_float4(0.f, 0.f, 0.f, 0.f);
          for (int m0 = 0; m0 < M; m0 += NG) {
            float4 g[NG];
#pragma unroll
            for (int q = 0; q < NG; ++q) {
              const int mm = min(m0 + q, M - 1);
              g[q] = *reinterpret_cast<const float4 *>(s.gbuf + (int64_t)dk[mm] * mp + (int64_t)mm * s.p + j);
            }
#pragma unroll
            for (int q = 0; q < NG; ++q)
              if (m0 + q < M) { nab.x += g[q].x; nab.y += g[q].y; nab.z += g[q].z; nab.w += g[q].w; }
          }
          update(j, nab.x); update(j + 1, nab.y); update(j + 2, nab.z); update(j + 3, nab.w);
        }
      };
      if (M > 16) aggregate(std::integral_constant<int, 32>{}); else aggregate(std::integral_constant<int, 16>{});
    } else {
      auto aggregate = [&](auto NGc) __attribute__((always_inline)) {
        constexpr int NG = decltype(NGc)::value;
        for (int j = tid; j < p; j += kBlock) {
          float nab = 0.f;
          for (int m0 = 0; m0 < M; m0 += NG) {
            float g[NG];
#pragma unroll
            for (int q = 0; q < NG; ++q) {
              const int mm = min(m0 + q, M - 1);
              g[q] = s.gbuf[(int64_t)dk[mm] * mp + (int64_t)mm * s.p + j];
            }
#pragma unroll
            for (int q = 0; q < NG; ++q)
              if (m0 + q < M) nab += g[q];
          }
          update(j, nab);
        }
      };
      if (M > 16) aggregate(std::integral_constant<int, 32>{}); else aggregate(std::integral_constant<int, 16>{});
    }
    newest_c = block_sum_lds(sqs, red);          // (ends with a workgroup barrier: the next phase A sees the new copies)
    if (tid == 0) s.ring_part[m] = m == 0 ? newest_c : 0.f;     // what a later launch, or reading the state out, adds up
  }
}

// Whether the multi-step kernel serves this configuration; sets the ring-partial count it uses.
bool small_plan(Ctx *c, const cada_config *cfg) {
  c->small = 0;
  const int64_t p = cfg->p;
  const int B = cfg->B, M = cfg->M;
  if (p >= 8192) return false;
  // Measured against the two-pass kernels (four launches, about 21 us at best): 9 us against 20 us for M = 10, B = 10,
  // p = 54; 18 against 21 us for M = 20, B = 32, p = 784; 23 against 26 us with M = 64; but 33 against 31 us with M = 128,
  // 58 against 37 us for M = 200 tiny workers (the server phase and the barrier grow with the workers) and 29 against
  // 28 us for B = 100 rows of p = 256: the path is taken by itself up to 64 workers of up to 64 rows.
  if (cfg->path != CADA_PATH_WHOLE_STEPS && (M > 64 || B > 64)) return false;
  int dev = 0, coop = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return false;
  if (M > cus) return false;
  c->small_lds = (size_t)(7 * p + 2 * B + 1) * sizeof(float) + (size_t)2 * B * sizeof(long long) + 16 + (size_t)B * p * sizeof(float);
  if (c->small_lds > 150 * 1024) return false;      // the minibatch of a worker and the server's vectors must fit in LDS
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(k_small), hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->small_lds) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  c->small = 1;
  c->small_plain_launch = cfg->plain_launch != 0 ? 1 : 0;
  return true;
}

constexpr uint32_t kSmallSpinLimit = 4000000u;

static SmallArgs small_args_of(Ctx *c, const int32_t *idx, const uint8_t *replay, int64_t n_steps) {
  SmallArgs a;
  a.s = c->s;
  a.s.k = c->k;
  a.idx = idx;
  a.replay = replay;
  a.n_steps = n_steps;
  a.bar = c->small_bar;
  a.bar_base = c->small_seq;
  a.spin_limit = kSmallSpinLimit;
  return a;
}

// Writes the launch-invariant arguments of this context into its workspace (for replica launches).
// The source is host memory that lives as long as the context.
int small_publish_args(Ctx *c) {
  if (!c->small) return CADA_OK;
  if (!c->small_args_host) {
    c->small_args_host = new (std::nothrow) unsigned char[sizeof(SmallArgs)];
    if (!c->small_args_host) { set_error("out of host memory"); return CADA_EINVAL; }
  }
  const SmallArgs a = small_args_of(c, nullptr, nullptr, 0);
  memcpy(c->small_args_host, &a, sizeof(a));
  const hipError_t e = hipMemcpyAsync(c->small_args, c->small_args_host, sizeof(SmallArgs), hipMemcpyHostToDevice, c->stream);
  if (e != hipSuccess) { set_error("copy of launch arguments failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

void small_free(Ctx *c) {
  delete[] static_cast<unsigned char *>(c->small_args_host);
  c->small_args_host = nullptr;
}

int small_steps_replicas(Ctx *const *cs, int n, const int32_t *const *idx, const uint8_t *const *replay, int64_t n_steps) {
  Ctx *c0 = cs[0];
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    set_error("cannot query the device");
    return CADA_EHIP;
  }
  if ((int64_t)n * c0->s.M > cus) { set_error("n_replicas x M = %lld workgroups exceed the %d CUs that must hold them at once", (long long)n * c0->s.M, cus); return CADA_EINVAL; }
  SmallLaunch l{};
  l.n_rep = n;
  l.n_steps = n_steps;
  for (int r = 0; r < n; ++r) {
    l.rep[r] = static_cast<const SmallArgs *>(cs[r]->small_args);
    l.var[r] = SmallVar{idx[r], replay ? replay[r] : nullptr, cs[r]->k, cs[r]->small_seq};
  }
  void *args[] = {&l};
  prof_mark(c0);
  const hipError_t e = hipLaunchCooperativeKernel(reinterpret_cast<const void *>(k_small), dim3((unsigned)c0->s.M, (unsigned)n), dim3(kBlock), args,
                                                  (unsigned)c0->small_lds, c0->stream);
  prof_mark(c0);
  if (e != hipSuccess) {
    set_error("replica launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  // (the barrier counters advance only with a launch that was accepted)
  for (int r = 0; r < n; ++r) cs[r]->small_seq += (uint32_t)(n_steps * cs[r]->s.M);
  return CADA_OK;
}

int small_steps(Ctx *c, const int32_t *idx, const uint8_t *replay, int64_t n_steps) {
  SmallLaunch l{};
  l.one = small_args_of(c, idx, replay, n_steps);
  void *args[] = {&l};
  prof_mark(c);
  hipError_t e;
  if (c->small_plain_launch) {      // (at most as many workgroups of 256 threads as CUs: all resident at once on an idle device)
    hipLaunchKernelGGL(k_small, dim3((unsigned)c->s.M), dim3(kBlock), c->small_lds, c->stream, l);
    e = hipGetLastError();
  } else {
    e = hipLaunchCooperativeKernel(reinterpret_cast<const void *>(k_small), dim3((unsigned)c->s.M), dim3(kBlock), args,
                                   (unsigned)c->small_lds, c->stream);
  }
  prof_mark(c);
  if (e != hipSuccess) {
    set_error("multi-step logistic launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  c->small_seq += (uint32_t)(n_steps * c->s.M);
  return CADA_OK;
}

}  // namespace cada
