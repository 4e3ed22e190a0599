// Single-pass dual minibatch gradient for the logistic model at large p (the HBM-bound
// workload): the B gathered rows of a worker cross HBM exactly once.
//
// Both passes of the gradient (z = X_B theta, then g = X_B^T r / B) need the same B x p
// rows, and a second pass over them costs as much as the first whether it is served by
// HBM or by the memory-side cache.  Here a cluster of Q workgroups owns one worker at a
// time; workgroup c of the cluster owns a fixed range of columns and streams the worker's
// rows through its registers in slabs of RS rows.  For every slab it
//   1. forms the partial dot products z_b, dz_b of its columns (from registers),
//   2. publishes them to the cluster as 8-byte words {value, sequence tag},
//   3. collects the Q partials of every row (polling the tags), sums them in a fixed tree
//      order, and turns z_b, dz_b into the residual r_b and the residual difference dr_b,
//   4. accumulates r_b x_b and dr_b x_b for its columns from the same registers.
// The next slab's loads are in flight during steps 1-4.  After the last slab the column
// range's gradient, innovation and squared-norm partial are written once.
//
// Notation and formulas as in cada_logreg.hip (Algorithm 1, the workers' two gradient
// evaluations on the same samples; conditions (workerrule1)/(workerrule2) for the norm).
//
// The cluster's workgroups wait for each other, so all of them must be resident: the
// kernel is launched cooperatively with a grid no larger than what fits the device, and
// every wait is bounded (a wait that exceeds the bound sets bit 1 of the error flags and
// the workgroup stops waiting for the rest of the launch, so every wave always exits).
#include "cada_internal.h"

namespace cada {

struct FusedArgs {
  DevState s;
  const int32_t *idx;            // [M][B]
  unsigned long long *zpost;     // [n_clusters][4][2*RS][Q] words {hi: tag, lo: float bits}
  int Q, n_clusters;
  int64_t cols_per_block;        // multiple of 4
  uint32_t seq_base;             // tags of this launch are seq_base+1, seq_base+2, ...
  uint32_t spin_limit;
};

template <int N> struct Log2 { static constexpr int v = 1 + Log2<N / 2>::v; };
template <> struct Log2<1> { static constexpr int v = 0; };

// Sums V per-lane values over the 64 lanes of a wave with V-1+log2(64/V) shuffles.
// Returns, in every lane, the wave-wide sum of value number bitreverse(lane mod V).
template <int V, int H>
__device__ __forceinline__ void reduce_scatter_step(float (&v)[V], const int lane) {
  if constexpr (H >= 1) {
    constexpr int o = V / (2 * H);      // exchange distance: 1, 2, 4, ...
    const bool up = (lane & o) != 0;
#pragma unroll
    for (int i = 0; i < H; ++i) {
      const float send = up ? v[i] : v[i + H];
      const float keep = up ? v[i + H] : v[i];
      v[i] = keep + __shfl_xor(send, o, 64);
    }
    reduce_scatter_step<V, H / 2>(v, lane);
  }
}

template <int V>
__device__ __forceinline__ float wave_reduce_scatter(float (&v)[V]) {
  reduce_scatter_step<V, V / 2>(v, threadIdx.x & 63);
  float r = v[0];
#pragma unroll
  for (int oo = V; oo < 64; oo <<= 1) r += __shfl_xor(r, oo, 64);
  return r;
}

__device__ __forceinline__ float sigmoid_f(float a) { return 1.0f / (1.0f + expf(-a)); }

template <int RS, int CPT4>
struct Slab {
  float4 x[RS][CPT4];
  float y;          // label of row (slab*RS + tid), threads tid < RS only
};

template <int RS, int CPT4>
__global__ __launch_bounds__(kBlock) void k_fused(const FusedArgs a) {
  constexpr int V = 2 * RS;
  constexpr int L = Log2<V>::v;
  static_assert(V >= 4 && V <= 64 && (V & (V - 1)) == 0, "2*RS must be a power of two in [4, 64]");
  const DevState &s = a.s;
  __shared__ float red[4][V];
  __shared__ float zs[V];
  __shared__ float r_s[RS], dr_s[RS];
  __shared__ float red4[4];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int Q = a.Q;
  const int cluster = blockIdx.x / Q, cb = blockIdx.x % Q;
  const int64_t colbase = (int64_t)cb * a.cols_per_block;
  const int64_t colend = min(s.p, colbase + a.cols_per_block);
  int64_t col[CPT4];
  bool cv[CPT4];
#pragma unroll
  for (int q = 0; q < CPT4; ++q) {
    col[q] = colbase + ((int64_t)q * kBlock + tid) * 4;
    cv[q] = col[q] < colend;
    if (!cv[q]) col[q] = 0;            // a valid address; the value is discarded
  }
  const float *yv = static_cast<const float *>(s.y);
  const float invB = 1.0f / (float)s.B;
  const int nslab = (s.B + RS - 1) / RS;
  const int64_t mp = (int64_t)s.M * s.p;
  unsigned long long *post_base = a.zpost + (int64_t)cluster * 4 * V * Q;
  uint32_t seq = a.seq_base;
  bool dead = false;
  // value index this lane holds after wave_reduce_scatter
  const int my_v = (int)(__brev((unsigned)lane) >> (32 - L)) & (V - 1);

  for (int m = cluster; m < s.M; m += a.n_clusters) {
    const int32_t *idx = a.idx + (int64_t)m * s.B;
    const int64_t n_m = s.row_off[m + 1] - s.row_off[m];
    const RefPtr ref = theta_ref(s, m, s.k);
    float4 th[CPT4], dd[CPT4], g[CPT4], iv[CPT4];
#pragma unroll
    for (int q = 0; q < CPT4; ++q) {
      const float4 t = *reinterpret_cast<const float4 *>(s.theta + col[q]);
      const float4 tl = *reinterpret_cast<const float4 *>(s.theta_lo + col[q]);
      const float4 rh = *reinterpret_cast<const float4 *>(ref.hi + col[q]);
      const float4 rl = *reinterpret_cast<const float4 *>(ref.lo + col[q]);
      th[q] = cv[q] ? t : make_float4(0.f, 0.f, 0.f, 0.f);
      dd[q] = cv[q] ? make_float4((t.x - rh.x) + (tl.x - rl.x), (t.y - rh.y) + (tl.y - rl.y),
                                  (t.z - rh.z) + (tl.z - rl.z), (t.w - rh.w) + (tl.w - rl.w))
                    : make_float4(0.f, 0.f, 0.f, 0.f);
      g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      iv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }

    // row of slab sl, slot r (clamped into the worker's range; slots past B reuse row B-1)
    auto row_of = [&](int sl, int r, bool *bad) -> int64_t {
      const int b = min(sl * RS + r, s.B - 1);
      int64_t loc = idx[b];
      if (loc < 0) { loc = 0; *bad = true; }
      if (loc >= n_m) { loc = n_m - 1; *bad = true; }
      return s.row_off[m] + loc;
    };
    auto load_slab = [&](Slab<RS, CPT4> &sb, int sl) {
      bool bad = false;
#pragma unroll
      for (int r = 0; r < RS; ++r) {
        const float *rowp = s.X + row_of(sl, r, &bad) * s.p;
#pragma unroll
        for (int q = 0; q < CPT4; ++q) sb.x[r][q] = *reinterpret_cast<const float4 *>(rowp + col[q]);
      }
      sb.y = (tid < RS) ? yv[row_of(sl, tid, &bad)] : 0.f;
      if (bad && tid == 0) atomicOr(s.err, 1u);
    };

    auto process = [&](const Slab<RS, CPT4> &sb, int sl) {
      seq += 1;
      // 1. partial dot products of this block's columns
      float pv[V];
#pragma unroll
      for (int r = 0; r < RS; ++r) {
        float z = 0.f, dz = 0.f;
#pragma unroll
        for (int q = 0; q < CPT4; ++q) {
          const float4 x = sb.x[r][q];
          z = fmaf(x.x, th[q].x, z); z = fmaf(x.y, th[q].y, z); z = fmaf(x.z, th[q].z, z); z = fmaf(x.w, th[q].w, z);
          dz = fmaf(x.x, dd[q].x, dz); dz = fmaf(x.y, dd[q].y, dz); dz = fmaf(x.z, dd[q].z, dz); dz = fmaf(x.w, dd[q].w, dz);
        }
        pv[2 * r] = z;
        pv[2 * r + 1] = dz;
      }
      const float mine = wave_reduce_scatter<V>(pv);
      if (lane < V) red[w][my_v] = mine;
      __syncthreads();
      // 2. publish {value, tag}
      unsigned long long *post = post_base + (int64_t)(seq & 3u) * V * Q;
      if (tid < V) {
        const float tot = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
        const unsigned long long word = ((unsigned long long)seq << 32) | (unsigned long long)__float_as_uint(tot);
        __hip_atomic_store(post + (int64_t)tid * Q + cb, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // 3. collect: wave w gathers values v = w, w+4, ...; lane j reads workgroup j's word
      constexpr int NV = V / 4;
      unsigned long long wd[NV];
      if (lane < Q) {
        uint32_t spins = 0;
        for (;;) {
          bool ok = true;
#pragma unroll
          for (int i = 0; i < NV; ++i) {
            wd[i] = __hip_atomic_load(post + (int64_t)(w + 4 * i) * Q + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = ok && ((uint32_t)(wd[i] >> 32) == seq);
          }
          if (ok || dead) break;
          if (++spins > a.spin_limit) {
            dead = true;
            atomicOr(s.err, 2u);
            break;
          }
          __builtin_amdgcn_s_sleep(2);
        }
      } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) wd[i] = 0ull;
      }
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const float tot = wave_sum(__uint_as_float((uint32_t)wd[i]));
        if (lane == 0) zs[w + 4 * i] = tot;
      }
      __syncthreads();
      if (tid < RS) {
        const int b = sl * RS + tid;
        float r = 0.f, dr = 0.f;
        if (b < s.B) {
          const float y = sb.y;
          const float z = zs[2 * tid], dz = zs[2 * tid + 1];
          const float aa = -y * z;
          const float bb = aa + y * dz;
          const float sa = sigmoid_f(aa);
          r = -y * sa * invB;
          dr = y * sa * sigmoid_f(-bb) * expm1f(y * dz) * invB;
        }
        r_s[tid] = r;
        dr_s[tid] = dr;
      }
      __syncthreads();
      // 4. accumulate the gradient and the innovation from the same registers
#pragma unroll
      for (int r = 0; r < RS; ++r) {
        const float rr = r_s[r], dr = dr_s[r];
#pragma unroll
        for (int q = 0; q < CPT4; ++q) {
          const float4 x = sb.x[r][q];
          g[q].x = fmaf(rr, x.x, g[q].x); g[q].y = fmaf(rr, x.y, g[q].y);
          g[q].z = fmaf(rr, x.z, g[q].z); g[q].w = fmaf(rr, x.w, g[q].w);
          iv[q].x = fmaf(dr, x.x, iv[q].x); iv[q].y = fmaf(dr, x.y, iv[q].y);
          iv[q].z = fmaf(dr, x.z, iv[q].z); iv[q].w = fmaf(dr, x.w, iv[q].w);
        }
      }
    };

    Slab<RS, CPT4> sa, sb;
    load_slab(sa, 0);
    for (int sl = 0; sl < nslab; sl += 2) {
      if (sl + 1 < nslab) load_slab(sb, sl + 1);
      process(sa, sl);
      if (sl + 1 < nslab) {
        if (sl + 2 < nslab) load_slab(sa, sl + 2);
        process(sb, sl + 1);
      }
    }

    // epilogue: regulariser, stores, squared norm of the rule's left-hand side
    const int cur = s.sel[m];
    float sq = 0.f;
#pragma unroll
    for (int q = 0; q < CPT4; ++q) {
      if (cv[q]) {
        float4 gg = g[q], ii = iv[q];
        gg.x = fmaf(s.lam, th[q].x, gg.x); gg.y = fmaf(s.lam, th[q].y, gg.y);
        gg.z = fmaf(s.lam, th[q].z, gg.z); gg.w = fmaf(s.lam, th[q].w, gg.w);
        ii.x = fmaf(s.lam, dd[q].x, ii.x); ii.y = fmaf(s.lam, dd[q].y, ii.y);
        ii.z = fmaf(s.lam, dd[q].z, ii.z); ii.w = fmaf(s.lam, dd[q].w, ii.w);
        *reinterpret_cast<float4 *>(s.gbuf + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + col[q]) = gg;
        if (s.rule == CADA_RULE_CADA1) {
          const float4 st = *reinterpret_cast<const float4 *>(s.dtl + (int64_t)cur * mp + (int64_t)m * s.p + col[q]);
          *reinterpret_cast<float4 *>(s.dtl + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + col[q]) = ii;
          ii.x -= st.x; ii.y -= st.y; ii.z -= st.z; ii.w -= st.w;
        }
        sq = fmaf(ii.x, ii.x, sq); sq = fmaf(ii.y, ii.y, sq); sq = fmaf(ii.z, ii.z, sq); sq = fmaf(ii.w, ii.w, sq);
      }
    }
    const float tot = block_sum(sq, red4);
    if (tid == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + cb] = tot;
  }
}

// Chooses the cluster geometry; returns false if the fused path does not apply.
bool fused_plan(Ctx *c, int64_t p, int B, int M) {
  c->fused = 0;
  // Off unless asked for: with one exchange per slab the workgroups spend longer waiting for
  // each other's partial sums (2 us idle, 4+ us under load per exchange) than the slab takes
  // to stream, so the two-pass path is faster.  Kept parity-tested as the basis of a deeper
  // pipeline that parks slabs in LDS while their exchange completes.
  const char *on = getenv("CADA_FUSED");
  if (!on || atoi(on) == 0) return false;
  if (c->vec != 4 || p < 8192) return false;
  int dev = 0, coop = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return false;
  // columns one workgroup can own: 256 threads x 4 columns x CPT4
  int cpt4 = 2;
  int64_t per_block = (int64_t)kBlock * 4 * cpt4;
  int Q = (int)((p + per_block - 1) / per_block);
  if (const char *e = getenv("CADA_FUSED_Q")) Q = max(Q, atoi(e));
  if (Q > 64) return false;
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_fused<8, 2>, kBlock, 0) != hipSuccess || per_cu < 1) return false;
  if (const char *e = getenv("CADA_FUSED_BLOCKS_PER_CU")) per_cu = min(per_cu, max(1, atoi(e)));
  else per_cu = 1;
  int ncl = (cus * per_cu) / Q;
  if (ncl < 1) return false;
  ncl = min(ncl, M);
  c->fused = 1;
  c->fused_Q = Q;
  c->fused_clusters = ncl;
  c->fused_cols = ((p + Q - 1) / Q + 3) / 4 * 4;
  c->fused_rs = 8;
  const int nslab = (B + 8 - 1) / 8;
  c->fused_seq_per_step = (uint32_t)(((M + ncl - 1) / ncl) * nslab);
  return true;
}

size_t fused_post_words(int Q, int n_clusters) { return (size_t)n_clusters * 4 * 16 * (size_t)Q; }

int logreg_gradients_fused(Ctx *c, const int32_t *idx) {
  FusedArgs a;
  a.s = c->s;
  a.s.k = c->k;
  a.idx = idx;
  a.zpost = c->fused_post;
  a.Q = c->fused_Q;
  a.n_clusters = c->fused_clusters;
  a.cols_per_block = c->fused_cols;
  a.seq_base = c->fused_seq;
  a.spin_limit = 4000000u;
  c->fused_seq += c->fused_seq_per_step;
  void *args[] = {&a};
  prof_mark(c);
  const hipError_t e = hipLaunchCooperativeKernel(reinterpret_cast<const void *>(k_fused<8, 2>),
                                                  dim3((unsigned)(a.Q * a.n_clusters)), dim3(kBlock), args, 0, c->stream);
  prof_mark(c);
  prof_mark(c);
  if (e != hipSuccess) {
    set_error("fused logistic gradient launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  return CADA_OK;
}

}  // namespace cada
