// Single-pass dual minibatch gradient for the logistic model at large p (the HBM-bound
// workload): the B gathered rows of a worker cross HBM exactly once.
//
// Both passes of the gradient (z = X_B theta, then g = X_B^T r / B) need the same B x p
// rows, and a second pass over them costs as much as the first whether it is served by
// HBM or by the memory-side cache (measured: re-reading a 64 MB window immediately runs at
// the same 6 TB/s as HBM).  Here a cluster of Q workgroups owns one worker at a time;
// workgroup c of the cluster owns a fixed set of 2048 columns (4 per streaming thread) and streams the
// worker's rows through its registers one row (slab) at a time.  For slab t it
//   1. forms the partial dot products z, dz of its columns (from registers) and publishes
//      them to the cluster as 8-byte words {value, sequence tag},
//   2. parks the slab in an LDS ring of NL = 16 slabs (each thread parks and later re-reads
//      only its own columns, so the ring itself needs no synchronisation),
//   3. LAG = 15 slabs later, when the Q partials of the row have long arrived, sums them in
//      a fixed tree order, turns z, dz into the residual r and the residual difference dr,
//      and accumulates r x and dr x for its columns from the ring.
// An exchange among workgroups takes 2 us idle and 3-4 us under load, far longer than a
// slab takes to stream (0.35 us), so everything hinges on the exchange being off the critical
// path: the 128 KB ring holds 5.5 us of stream per CU.
//
// Loads return in order within a wavefront, so waiting for a young load (a poll, an index,
// a label) means waiting for every older one: a wavefront that keeps 16 slabs of bulk loads
// in flight must issue no other load in its steady state.  The workgroup is therefore split
// into roles, ten wavefronts that meet at one LDS-only barrier per iteration (one or two slabs):
//   wavefronts 0-7  stream: bulk loads (PD = 16 slabs in flight), partial dot products,
//                   parking, accumulation; row addresses come from LDS;
//   wavefront 8     exchange: publishes the workgroup's partials, polls the cluster's
//                   (P polls in flight, first issued LAG-2-P slabs after publication),
//                   sums them;
//   wavefront 9     turns (z, dz, y) into (r, dr) one slab later, and every 64 slabs fetches
//                   the row indices and labels of 64 slabs to come into LDS, with the slot of
//                   the iterate history and the half of the gradient store of their worker.
// (Eight streaming wavefronts of four columns per thread need 150-160 registers; four of eight
// columns needed 256 and spilled.  The time is the same.)
// A change of worker costs a streaming wavefront no wait: theta stays in registers for the whole
// launch, and the next worker's reference point is asked for PDI iterations ahead, together with
// the bulk loads of that worker's first row, by loads that -- like the bulk loads -- the compiler
// does not see; a wait for every outstanding load, which a dependent load chain at the change
// used to need twice per worker, empties the 16-slab pipeline and costs its refill (2 % of a
// launch at 13 workers per cluster).  Minibatches of fewer than 32 rows, which the prefetch
// distance and the accumulation lag would overrun, compile to a variant that loads at the change
// and waits (DRAIN): a variant of its own so that in the other no second value ever shares, or is
// moved through, the registers with loads in flight.
// Every global memory operation of a steady-state iteration is executed by all lanes: the
// compiler counts outstanding operations per path, and one that a branch may skip does not
// count, which would turn every wait into a wait for the youngest load.
//
// Notation and formulas as in cada_logreg.hip (Algorithm 1, the workers' two gradient
// evaluations on the same samples; conditions (workerrule1)/(workerrule2) for the norm).
//
// The cluster's workgroups wait for each other, so all of them must be resident: the
// kernel is launched cooperatively, one workgroup per CU, and every wait is bounded (a wait
// that exceeds the bound sets bit 1 of the error flags and the workgroup stops waiting for
// the rest of the launch, so every wave always exits).
#include <cstdlib>
#include <type_traits>

#include "cada_internal.h"

namespace cada {

// R = rows (slabs) a workgroup takes per iteration, i.e. per barrier: 2 when the minibatch size is
// even (the per-iteration costs -- barrier, cursor updates, address and residual reads, branches --
// are paid once per two rows), else 1.
constexpr int F_PD = 16;             // slabs of loads in flight per thread
constexpr int F_NP = 32;             // publication buffers, in slabs
constexpr int F_V = 2;               // exchanged values per slab and workgroup: z and dz
constexpr int F_SW = kFusedWaves;    // streaming wavefronts
constexpr int F_STREAM = 64 * F_SW;  // streaming threads
constexpr int F_NQ = 2048 / (4 * F_STREAM);   // 16-byte pieces of a row per streaming thread (a workgroup owns 2048 columns)
constexpr int F_THREADS = F_STREAM + 128;   // + exchange wavefront + residual/feeder wavefront
static_assert(F_NQ >= 1 && F_NQ * 4 * F_STREAM == 2048 && (F_SW & (F_SW - 1)) == 0, "a workgroup owns 2048 columns");
constexpr int F_QMAX = 64;            // workgroups per cluster: 32 per poll word of an exchange lane, NJ = 1 or 2 words
constexpr int F_NE = 256;            // slabs whose row address and label are held in LDS (4 chunks of 64)
template <int R> struct FusedGeom {
  static constexpr int NL = 16 + 2 * (R - 1);     // one-row slabs parked in LDS (128 KB, 144 KB)
  static constexpr int LAGI = NL / R - 1;         // iterations between producing and consuming a slab
  static constexpr int PDI = F_PD / R;            // iterations of loads in flight = unroll factor of the loops
  static constexpr int P = 4 / R;                 // iterations of polls in flight in the exchange wavefront
  static constexpr int IPC = 64 / R;              // iterations per feeder chunk of 64 slabs
  static constexpr size_t lds = (size_t)NL * F_NQ * F_STREAM * sizeof(float4);   // dynamic part
  static_assert(PDI % P == 0 && F_NP >= (LAGI + 2) * R && F_NE % 64 == 0 && NL % R == 0, "pipeline constants");
};

struct FusedArgs {
  DevState s;
  const int32_t *idx;            // [M][B]
  unsigned long long *zpost;     // [n_clusters][F_NP][F_V][Q] words {hi: tag, lo: float bits}
  int Q, n_clusters;
  uint32_t seq_base;             // tag of slab t of this launch is seq_base + 1 + t
  uint32_t spin_limit;
  // Last round.  With M = full * n_clusters + rem workers, 0 < rem < n_clusters, the last round would keep only
  // rem clusters busy.  When tail_f = n_clusters / rem is a whole number >= 2 that divides the minibatch, the
  // rows of each of the rem last workers are split over tail_f clusters instead (tail_rows = B / tail_f each):
  // cluster c takes rows [(c % tail_f) tail_rows, +tail_rows) of worker full * n_clusters + c / tail_f and leaves
  // its part of the two sums (no regulariser) in tail_part[c % tail_f][c / tail_f][0|1][p]; k_fused_tail adds
  // the parts up in a fixed order.  tail_f = 0: no split.
  int tail_f, tail_rows, tail_rem;
  float *tail_part;
};

__device__ __forceinline__ float sigmoid_f(float a) { return 1.0f / (1.0f + expf(-a)); }

template <int I> using ic = std::integral_constant<int, I>;
template <bool B> using bc = std::integral_constant<bool, B>;

// f(ic<0>{}), f(ic<1>{}), ..., f(ic<N-1>{}) written out
template <class F, int... I>
__device__ __forceinline__ void unrolled(F &&f, std::integer_sequence<int, I...>) { (f(ic<I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void unrolled(F &&f) { unrolled(static_cast<F &&>(f), std::make_integer_sequence<int, N>{}); }

typedef float v4f __attribute__((ext_vector_type(4)));   // four consecutive registers

// The bulk loads of the steady state and the waits for them are written out: the compiler
// places a wait for a load from what it can prove about the loads issued since, and across
// the back edge of the unrolled loop (and past the rarely taken blocks inside it) it proves
// too little, so that it drains the whole prefetch pipeline once per trip.  A load issued here
// is invisible to the compiler's bookkeeping; wait_slab() is what orders its use.
// The rows are read once per step and never again soon: the loads carry the non-temporal hint.
// (Measured on a 2 GB stream over all CUs: 7.1 TB/s with it, 6.0 TB/s without.)
__device__ __forceinline__ void issue_slab(v4f (&x)[F_NQ], const float *row, const int64_t (&col)[F_NQ]) {
#pragma unroll
  for (int q = 0; q < F_NQ; ++q) asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(x[q]) : "v"(row + col[q]) : "memory");
}
// Workgroup barrier that orders LDS traffic only.  (__syncthreads() also fences global
// memory, which makes every wavefront wait for all its outstanding loads and would drain the
// prefetch pipeline each iteration; the wavefronts of a workgroup exchange data through LDS only.)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// x + (x of another lane), the other lane chosen by a data-parallel-primitive control word:
// quad_perm [1,0,3,2] = 0xB1 (lane ^ 1), quad_perm [2,3,0,1] = 0x4E (lane ^ 2),
// row_ror:4 = 0x124, row_ror:8 = 0x128 (rotation within a row of 16 lanes).
template <int CTRL>
__device__ __forceinline__ float dpp_get(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// Sum over the lanes of the same parity within each row of 16 lanes (every lane gets it).
__device__ __forceinline__ float row16_parity_sum(float v) {
  v += dpp_get<0x4E>(v);
  v += dpp_get<0x124>(v);
  v += dpp_get<0x128>(v);
  return v;
}

// Waits until at most N vector memory operations issued after the loads of x are outstanding.
template <int N, int R>
__device__ __forceinline__ void wait_rows(v4f (&x)[R][F_NQ]) {
  static_assert(R * F_NQ == 1 || R * F_NQ == 2 || R * F_NQ == 4, "registers named below");
  v4f *f = &x[0][0];
  if constexpr (R * F_NQ == 1) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(f[0]) : "n"(N));
  else if constexpr (R * F_NQ == 2) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(f[0]), "+v"(f[1]) : "n"(N));
  else asm volatile("s_waitcnt vmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N));
}

// The same wait, naming the registers of a reference point (see issue_ref in k_fused).
template <int N>
__device__ __forceinline__ void wait_ref(v4f (&x)[2][F_NQ]) {
  static_assert(F_NQ == 1 || F_NQ == 2, "registers named below");
  v4f *f = &x[0][0];
  if constexpr (F_NQ == 1) asm volatile("s_waitcnt vmcnt(%2)" : "+v"(f[0]), "+v"(f[1]) : "n"(N));
  else asm volatile("s_waitcnt vmcnt(%4)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "n"(N));
}

// NJ: poll words per lane of the exchange wavefront (a lane sums the partials of workgroups j, j + 32, ...):
// 1 for clusters of up to 32 workgroups (p <= 65536), 2 for up to 64 (p <= 131072).
// DRAIN: minibatches of fewer than 32 rows (see the worker changes of the streaming wavefronts).
template <int R, int NJ, bool DRAIN>
__global__ __launch_bounds__(F_THREADS) void k_fused(const FusedArgs a) {
  using G = FusedGeom<R>;
  constexpr int NL = G::NL, LAGI = G::LAGI, PDI = G::PDI, P = G::P, IPC = G::IPC;
  // iterations before the steady-state loop: it assumes that the previous iteration consumed rows
  constexpr int HEAD = (LAGI + 1 + PDI - 1) / PDI * PDI;
  const DevState &s = a.s;
  extern __shared__ __align__(16) unsigned char fused_smem[];
  v4f *ring = reinterpret_cast<v4f *>(fused_smem);            // [NL][F_NQ][F_STREAM]
  __shared__ __align__(16) float red[2][R][F_V][4 * F_SW];    // [iteration parity][row][z|dz][wavefront * 4 + row of 16 lanes]
  __shared__ float zz_s[2][R][F_V];                           // cluster sums z, dz
  __shared__ float r_s[2][R], dr_s[2][R];
  __shared__ __align__(16) long long off_s[F_NE];             // element offset of slab t's row in X, at t % NE
  __shared__ float y_s[F_NE];                                 // label of slab t
  __shared__ int ref_s[F_NE];                                 // slot of the iterate history that holds the reference point of slab t's worker
  __shared__ int sel_s[F_NE];                                 // which half of the gradient store holds that worker's stored gradient

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int Q = a.Q, ncl = a.n_clusters;
  const int cluster = blockIdx.x / Q, cb = blockIdx.x % Q;
  const int nslab = s.B;                                      // one row per slab; a multiple of R
  const bool split = a.tail_f > 0;
  // whole workers of this cluster, then (split) its share of one of the last workers
  const int rounds = split ? s.M / ncl : (s.M - cluster + ncl - 1) / ncl;
  const int m_end = cluster + rounds * ncl;                   // one past the last whole worker of this cluster
  const int mt = split ? (s.M / ncl) * ncl + cluster / a.tail_f : 0x40000000;     // the shared worker (none: never reached)
  const int ot = split ? (cluster % a.tail_f) * a.tail_rows : 0;                   // this cluster's first row of it
  const int S = rounds * nslab + (split ? a.tail_rows : 0);   // slabs of this cluster
  const int IS = S / R;                                       // iterations that produce
  const int total = IS + LAGI;                                // iterations (= barriers after the first) of every wavefront
  unsigned long long *post_base = a.zpost + (int64_t)cluster * F_NP * F_V * Q;
  // (worker, slab within worker) cursors advance one iteration (R slabs) at a time
  // (a cursor is (worker, slab, one past the worker's last slab for this cluster); the comparison of every
  // iteration is against a register, everything about the split worker sits in the rarely taken block)
  auto first_of = [&](int m) __attribute__((always_inline)) { return m == mt ? ot : 0; };
  auto end_of = [&](int m) __attribute__((always_inline)) { return m == mt ? ot + a.tail_rows : nslab; };
  auto advance = [&](int &m, int &loc, int &end, int &first) __attribute__((always_inline)) {
    loc += R;
    if (loc == end) {
      if (m + ncl < m_end) { m += ncl; loc = 0; }
      else { m = mt; loc = ot; end = ot + a.tail_rows; first = ot; }
    }
  };

  if (w == F_SW + 1) {
    // ================= residual / feeder wavefront =================
    const float invB = 1.0f / (float)s.B;
    // feeder registers (lane = slab 64 * chunk + lane): row index, first row and end of the
    // worker's row range, label.  Three stages several iterations apart, so that no stage
    // waits for a load it has just issued.
    int64_t f_base = 0, f_end = 0, f_r = 0;
    int f_tau = 0, f_sel = 0;
    float f_y = 0.f;
    auto feed_issue = [&](int chunk) __attribute__((always_inline)) {                 // stage 1: index and row range
      const int t = chunk * 64 + lane;
      const int tt = t < S ? t : S - 1;
      const bool whole = tt < rounds * nslab;
      const int m = whole ? cluster + (tt / nslab) * ncl : mt;
      const int row = whole ? tt % nslab : ot + (tt - rounds * nslab);
      f_base = s.row_off[m];
      f_end = s.row_off[m + 1];
      f_r = a.idx[(int64_t)m * s.B + row];
      f_tau = s.rule == CADA_RULE_CADA2 ? s.tau[m] : 0;
      f_sel = s.sel[m];
    };
    auto feed_label = [&]() __attribute__((always_inline)) {                          // stage 2: range check, label
      const int64_t n_m = f_end - f_base;
      if (f_r < 0 || f_r >= n_m) { atomicOr(s.err, 1u); f_r = f_r < 0 ? 0 : n_m - 1; }
      f_y = static_cast<const float *>(s.y)[f_base + f_r];
    };
    auto feed_write = [&](int chunk) __attribute__((always_inline)) {                 // stage 3
      const int e = (chunk * 64 + lane) % F_NE;
      off_s[e] = (f_base + f_r) * s.p;
      y_s[e] = f_y;
      int64_t slot = (s.k - (int64_t)min(f_tau, s.D)) % s.R;     // as theta_ref_at()
      if (slot < 0) slot += s.R;
      ref_s[e] = (int)slot;
      sel_s[e] = f_sel;
    };
    feed_issue(0); feed_label(); feed_write(0);
    lds_barrier();

    // lanes 2r, 2r+1 work on row r of the iteration: the even lane evaluates sigmoid(aa), the
    // odd lane sigmoid(-bb) (one evaluation for both)
    const int mr = (lane >> 1) & (R - 1);
    auto math_iter = [&](auto ST, const int it) __attribute__((always_inline)) {
      constexpr bool st = decltype(ST)::value;
      lds_barrier();
      const int c1 = it + 1 - LAGI;                    // summed by the exchange wavefront last iteration
      if (st || (c1 >= 0 && c1 < IS)) {
        const float z = zz_s[c1 & 1][mr][0], dz = zz_s[c1 & 1][mr][1];
        const float y = y_s[(c1 * R + mr) % F_NE];
        const float aa = -y * z;
        const float bb = aa + y * dz;
        const float sg = sigmoid_f((lane & 1) ? -bb : aa);
        const float sb = dpp_get<0xB1>(sg);            // the neighbour's value
        const float em = expm1f(y * dz);
        if ((lane & 1) == 0 && lane < 2 * R) {
          r_s[c1 & 1][mr] = -y * sg * invB;
          dr_s[c1 & 1][mr] = y * sg * sb * em * invB;
        }
      }
      // rows and labels of chunk it / IPC + 1, first needed PDI + 1 iterations before its first slab
      const int ph = it % IPC, chunk = it / IPC + 1;
      if (chunk * 64 < S) {
        if (ph == IPC / 4) feed_issue(chunk);
        else if (ph == IPC * 3 / 8) feed_label();
        else if (ph == IPC / 2) feed_write(chunk);
      }
    };
    // head, steady-state loop, tail: three loops of their own, so that the steady-state loop
    // has a single body and its loop-carried registers stay in place
    int s0 = 0;
    for (; s0 < HEAD && s0 < total; s0 += PDI)
      for (int i = 0; i < PDI; ++i)
        if (s0 + i < total) math_iter(bc<false>{}, s0 + i);
    for (; s0 + 2 * PDI < IS; s0 += PDI) {
#pragma unroll
      for (int i = 0; i < PDI; ++i) math_iter(bc<true>{}, s0 + i);
    }
    for (; s0 < total; s0 += PDI)
      for (int i = 0; i < PDI; ++i)
        if (s0 + i < total) math_iter(bc<false>{}, s0 + i);
    return;
  }

  if (w == F_SW) {
    // ================= exchange wavefront =================
    const int j = lane & 31, half = lane >> 5, par = lane & 1, pr = (lane >> 1) & (R - 1);
    bool jok[NJ];
    int jc[NJ];
#pragma unroll
    for (int q = 0; q < NJ; ++q) { jok[q] = j + 32 * q < Q; jc[q] = jok[q] ? j + 32 * q : Q - 1; }
    bool dead = false;
    unsigned long long pw[P][R][NJ];
#pragma unroll
    for (int i = 0; i < P; ++i)
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int q = 0; q < NJ; ++q) pw[i][r][q] = 0ull;
    lds_barrier();

    auto comm_iter = [&](auto PI, auto ST, const int it) __attribute__((always_inline)) {
      constexpr int pi = decltype(PI)::value;
      constexpr bool st = decltype(ST)::value;
      lds_barrier();
      // publish the rows of iteration it: lanes of equal (parity, row) compute and store the same word
      if (st || it < IS) {
        const float4 *rp = reinterpret_cast<const float4 *>(red[it & 1][pr][par]);
        float ws[F_SW];                                     // per streaming wavefront, then a fixed tree
#pragma unroll
        for (int i = 0; i < F_SW; ++i) { const float4 q = rp[i]; ws[i] = (q.x + q.y) + (q.z + q.w); }
#pragma unroll
        for (int st2 = 1; st2 < F_SW; st2 *= 2)
#pragma unroll
          for (int i = 0; i < F_SW; i += 2 * st2) ws[i] += ws[i + st2];
        const float tot = ws[0];
        const int t = it * R + pr;
        const uint32_t tag = a.seq_base + 1u + (uint32_t)t;
        const unsigned long long word = ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(tot);
        __hip_atomic_store(post_base + ((int64_t)(t % F_NP) * F_V + par) * Q + cb, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      // sum the cluster's partials of the rows of iteration c1 (first polled P iterations ago)
      const int c1 = it + 2 - LAGI;
      if (st || (c1 >= 0 && c1 < IS)) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const int t = c1 * R + r;
          const uint32_t tag = a.seq_base + 1u + (uint32_t)t;
          float v = 0.f;
#pragma unroll
          for (int q = 0; q < NJ; ++q) {
            if ((uint32_t)(pw[pi][r][q] >> 32) != tag) {      // not there yet: rare
              const unsigned long long *pp = post_base + ((int64_t)(t % F_NP) * F_V + half) * Q + jc[q];
              uint32_t spins = 0;
              while (!dead && (uint32_t)(pw[pi][r][q] >> 32) != tag) {
                if (++spins > a.spin_limit) { dead = true; atomicOr(s.err, 2u); break; }
                __builtin_amdgcn_s_sleep(1);
                pw[pi][r][q] = __hip_atomic_load(pp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              }
            }
            v += jok[q] ? __uint_as_float((uint32_t)pw[pi][r][q]) : 0.f;       // (NJ = 1: the value itself)
          }
          v += dpp_get<0xB1>(v);
          v = row16_parity_sum(v);                     // every lane: sum of its row of 16
          const float z0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
          const float z1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
          const float d0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
          const float d1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
          if (lane == 0) { zz_s[c1 & 1][r][0] = z0 + z1; zz_s[c1 & 1][r][1] = d0 + d1; }
        }
      }
      // first poll of the rows of iteration c2, summed P iterations from now
      const int c2 = it + 2 + P - LAGI;
      if (st || (c2 >= 0 && c2 < IS)) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int q = 0; q < NJ; ++q)
            pw[pi][r][q] = __hip_atomic_load(post_base + ((int64_t)((c2 * R + r) % F_NP) * F_V + half) * Q + jc[q], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
      }
    };

    int s0 = 0;
    for (; s0 < HEAD && s0 < total; s0 += PDI)
      unrolled<PDI>([&](auto I) __attribute__((always_inline)) {
        if (s0 + I.value < total) comm_iter(ic<I.value % P>{}, bc<false>{}, s0 + I.value);
      });
    for (; s0 + 2 * PDI < IS; s0 += PDI)
      unrolled<PDI>([&](auto I) __attribute__((always_inline)) { comm_iter(ic<I.value % P>{}, bc<true>{}, s0 + I.value); });
    for (; s0 < total; s0 += PDI)
      unrolled<PDI>([&](auto I) __attribute__((always_inline)) {
        if (s0 + I.value < total) comm_iter(ic<I.value % P>{}, bc<false>{}, s0 + I.value);
      });
    return;
  }

  // ================= streaming wavefronts =================
  // A row is cut into pieces of 256 columns (1 KB, one load of a wavefront); piece (q F_SW + w) Q + cb belongs to
  // streaming wavefront w of workgroup cb: the loads a workgroup issues together are 32 KB apart rather than 8 KB
  // in a row (measured: 1 % faster than eight consecutive pieces per workgroup).
  int64_t col[F_NQ];
  bool cv[F_NQ];
#pragma unroll
  for (int q = 0; q < F_NQ; ++q) {
    col[q] = (((int64_t)(q * F_SW + w) * Q + cb) * 64 + lane) * 4;
    cv[q] = col[q] < s.p;
    if (!cv[q]) col[q] = 0;            // a valid address; the value is discarded
  }
  const int64_t mp = (int64_t)s.M * s.p;
  // first element of a row from its LDS word (wavefront-uniform, from the feeder's table)
  auto to_row = [&](long long o) __attribute__((always_inline)) -> const float * {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)o);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((unsigned long long)o >> 32));
    return s.X + (int64_t)(((unsigned long long)hi << 32) | lo);
  };
  // th, tl: theta (two floats per value); dd: theta - reference point of the worker being produced (dd_m), ddc: of
  // the worker before it (ddc_m), whose last rows are accumulated LAGI iterations after its last dot products
  float4 th[F_NQ], tl[F_NQ], dd[F_NQ], ddc[F_NQ], g[F_NQ], iv[F_NQ];
  int dd_m = -1, ddc_m = -1;
#pragma unroll
  for (int q = 0; q < F_NQ; ++q) {
    th[q] = tl[q] = dd[q] = ddc[q] = g[q] = iv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (cv[q]) { th[q] = *reinterpret_cast<const float4 *>(s.theta + col[q]); tl[q] = *reinterpret_cast<const float4 *>(s.theta_lo + col[q]); }
  }

  // Worker changes without draining the load pipeline.  theta is the same for every worker and stays in
  // registers (th, tl); a worker's reference point differs.  Its columns are asked for (rq, loads the compiler does
  // not see, like the bulk loads) in the iteration that issues the bulk loads of the worker's first row, PDI
  // iterations before that row's dot products: they are older than that row's loads, so the wait for the row
  // covers them.  The worker's slot of the iterate history comes from the feeder's table.
  v4f rq[2][F_NQ];                      // reference point, high and low words
  auto ref_of = [&](int t) __attribute__((always_inline)) -> RefPtr {     // reference point of slab t's worker
    if (s.rule == CADA_RULE_CADA1) return RefPtr{s.snap, s.snap_lo};
    if (s.rule != CADA_RULE_CADA2) return RefPtr{s.theta, s.theta_lo};
    const int slot = __builtin_amdgcn_readfirstlane(ref_s[t % F_NE]);
    return RefPtr{s.hist + (int64_t)slot * s.ps, s.hist_lo + (int64_t)slot * s.ps};
  };
  auto issue_ref = [&](int t) __attribute__((always_inline)) {
    const RefPtr ref = ref_of(t);
#pragma unroll
    for (int q = 0; q < F_NQ; ++q) {
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rq[0][q]) : "v"(ref.hi + col[q]) : "memory");
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rq[1][q]) : "v"(ref.lo + col[q]) : "memory");
    }
  };
  // theta - reference point of slab t's worker at this thread's columns, loaded here and now (short minibatches)
  auto diff_now = [&](int t, float4 (&d)[F_NQ]) __attribute__((always_inline)) {
    const RefPtr ref = ref_of(t);
#pragma unroll
    for (int q = 0; q < F_NQ; ++q) {
      const float4 rh = *reinterpret_cast<const float4 *>(ref.hi + col[q]), rl = *reinterpret_cast<const float4 *>(ref.lo + col[q]);
      d[q] = cv[q] ? make_float4((th[q].x - rh.x) + (tl[q].x - rl.x), (th[q].y - rh.y) + (tl[q].y - rl.y),
                                 (th[q].z - rh.z) + (tl[q].z - rl.z), (th[q].w - rh.w) + (tl[q].w - rl.w))
                   : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): no load that the compiler tracks stays in flight
  };

  v4f xb[PDI][R][F_NQ];
  const int m_first = rounds > 0 ? cluster : mt;
  int pm = m_first, ploc = first_of(m_first), pend = end_of(m_first);   // first slab produced (dot products, parked) this iteration
  int cm = m_first, cloc = first_of(m_first), cend = end_of(m_first);   // first slab accumulated this iteration
  int pfirst = ploc, cfirst = cloc;                                     // first slab of the worker being produced / accumulated
  lds_barrier();                        // the feeder's first chunk is in LDS
  // Minibatches too short for that (a worker must outlast the prefetch, and the accumulation lag for ddc to hold)
  // load the reference point where it is used and wait for the pipeline.
  constexpr bool drain = DRAIN;
  if constexpr (!drain) issue_ref(0);
  int qloc = (PDI * R) % nslab;         // position within its worker of the first row whose loads an iteration issues
  int ct = 0;                           // first slab accumulated by the next accumulate()
  // prologue: loads of the first PDI iterations
#pragma unroll
  for (int i = 0; i < PDI; ++i)
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (i * R + r < S) {
        const float *rp = to_row(off_s[(i * R + r) % F_NE]);
#pragma unroll
        for (int q = 0; q < F_NQ; ++q) xb[i][r][q] = *reinterpret_cast<const v4f *>(rp + col[q]);
      }

  // Accumulation of the consumed rows, deferred by one iteration: their residuals are read from
  // LDS right after the barrier but first used here, after the next rows' dot products, so
  // that the wavefront never waits for that read.
  v4f xr[R][F_NQ];                      // the consumed rows' columns, from the ring
  float rr[R], dr[R];                   // their residuals and residual differences
#pragma unroll
  for (int r = 0; r < R; ++r) rr[r] = dr[r] = 0.f;
  bool pending = false;
  auto accumulate = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int q = 0; q < F_NQ; ++q) {
        const v4f x = xr[r][q];
        g[q].x = fmaf(rr[r], x.x, g[q].x); g[q].y = fmaf(rr[r], x.y, g[q].y);
        g[q].z = fmaf(rr[r], x.z, g[q].z); g[q].w = fmaf(rr[r], x.w, g[q].w);
        iv[q].x = fmaf(dr[r], x.x, iv[q].x); iv[q].y = fmaf(dr[r], x.y, iv[q].y);
        iv[q].z = fmaf(dr[r], x.z, iv[q].z); iv[q].w = fmaf(dr[r], x.w, iv[q].w);
      }
    if (cloc + R == cend && cm == mt) {
      // last rows of this cluster's share of a split worker: its part of the two sums, as they are
      float *pg = a.tail_part + (((int64_t)(cluster % a.tail_f) * a.tail_rem + cluster / a.tail_f) * 2) * s.p;
#pragma unroll
      for (int q = 0; q < F_NQ; ++q) {
        if (cv[q]) {
          *reinterpret_cast<float4 *>(pg + col[q]) = g[q];
          *reinterpret_cast<float4 *>(pg + s.p + col[q]) = iv[q];
        }
        g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        iv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    } else if (cloc + R == cend) {
      // last rows of worker cm: regulariser, stores, squared norm of the rule's left-hand side
      const int m = cm;
      const bool cur_worker = m == dd_m;          // (the last worker: nothing was produced after it)
      if constexpr (drain) diff_now(ct, ddc);     // (ddc has no other use with short minibatches)
      const int cur = __builtin_amdgcn_readfirstlane(sel_s[ct % F_NE]);
      float sq = 0.f;
#pragma unroll
      for (int q = 0; q < F_NQ; ++q) {
        if (cv[q]) {
          float4 gg = g[q], ii = iv[q];
          const float4 dm = (cur_worker && !drain) ? dd[q] : ddc[q];
          gg.x = fmaf(s.lam, th[q].x, gg.x); gg.y = fmaf(s.lam, th[q].y, gg.y);
          gg.z = fmaf(s.lam, th[q].z, gg.z); gg.w = fmaf(s.lam, th[q].w, gg.w);
          ii.x = fmaf(s.lam, dm.x, ii.x); ii.y = fmaf(s.lam, dm.y, ii.y);
          ii.z = fmaf(s.lam, dm.z, ii.z); ii.w = fmaf(s.lam, dm.w, ii.w);
          *reinterpret_cast<float4 *>(s.gbuf + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + col[q]) = gg;
          if (s.rule == CADA_RULE_CADA1) {
            // (the one load of a worker change: CADA1 waits for the pipeline here)
            const float4 stv = *reinterpret_cast<const float4 *>(s.dtl + (int64_t)cur * mp + (int64_t)m * s.p + col[q]);
            *reinterpret_cast<float4 *>(s.dtl + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + col[q]) = ii;
            ii.x -= stv.x; ii.y -= stv.y; ii.z -= stv.z; ii.w -= stv.w;
          }
          sq = fmaf(ii.x, ii.x, sq); sq = fmaf(ii.y, ii.y, sq); sq = fmaf(ii.z, ii.z, sq); sq = fmaf(ii.w, ii.w, sq);
        }
        g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        iv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
      const float tot = wave_sum(sq);
      if (lane == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + cb * F_SW + w] = tot;
      // a rarely taken block must leave no load the compiler still tracks in flight: a wait for it on the
      // main path would be a wait for nearly all the bulk loads issued since
      if (s.rule == CADA_RULE_CADA1) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    }
    ct += R;
    advance(cm, cloc, cend, cfirst);
  };

  // LDS words of the row addresses of iteration it + PDI, read one iteration before their use
  long long off_q[R];
#pragma unroll
  for (int r = 0; r < R; ++r) off_q[r] = (PDI < IS) ? off_s[(PDI * R + r) % F_NE] : 0;

  // One iteration.  The LDS reads whose results are needed later are issued first, and the
  // only LDS operation the barrier has to wait for (the partial sums) is followed by the
  // previous rows' accumulation, so that no LDS latency is exposed.
  auto stream_iter = [&](auto BI, auto ST, const int it) __attribute__((always_inline)) {
    constexpr int bi = decltype(BI)::value;
    constexpr bool st = decltype(ST)::value;
    const bool prod = st || it < IS;
    const bool more = st || it + PDI < IS;
    const float *rp[R];
#pragma unroll
    for (int r = 0; r < R; ++r) rp[r] = to_row(off_q[r]);
    if (st || it + PDI + 1 < IS) {
#pragma unroll
      for (int r = 0; r < R; ++r) off_q[r] = off_s[((it + PDI + 1) * R + r) % F_NE];
    }
    // 3a. ring entries of the rows of iteration c0 = it - LAGI, consumed after the barrier (this
    //     thread's own columns: no synchronisation needed)
    const bool cons = st || (it >= LAGI && it - LAGI < IS);
    const int c0 = it - LAGI;
    v4f xn[R][F_NQ];
    if (cons) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const v4f *slot = ring + (size_t)((c0 * R + r) % NL) * F_NQ * F_STREAM;
#pragma unroll
        for (int q = 0; q < F_NQ; ++q) xn[r][q] = slot[q * F_STREAM + tid];
      }
    }
    if (prod) {
      if constexpr (st) wait_rows<(PDI - 1) * F_NQ * R, R>(xb[bi]);
      if (ploc == pfirst) {
        // first rows of worker pm: its reference point was asked for before these rows (steady state: the wait
        // above covers it; elsewhere the compiler's own loads are in flight too: wait for everything)
        if constexpr (drain) {
          diff_now(it * R, dd);
        } else {
          if constexpr (st) wait_ref<(PDI - 1) * F_NQ * R>(rq); else wait_ref<0>(rq);
#pragma unroll
          for (int q = 0; q < F_NQ; ++q) {
            ddc[q] = dd[q];
            const v4f rh = rq[0][q], rl = rq[1][q];
            dd[q] = cv[q] ? make_float4((th[q].x - rh.x) + (tl[q].x - rl.x), (th[q].y - rh.y) + (tl[q].y - rl.y),
                                        (th[q].z - rh.z) + (tl[q].z - rl.z), (th[q].w - rh.w) + (tl[q].w - rl.w))
                          : make_float4(0.f, 0.f, 0.f, 0.f);
          }
          ddc_m = dd_m; dd_m = pm;
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        // 2. park the row
        v4f *slot = ring + (size_t)((it * R + r) % NL) * F_NQ * F_STREAM;
#pragma unroll
        for (int q = 0; q < F_NQ; ++q) slot[q * F_STREAM + tid] = xb[bi][r][q];
        // 1. partial dot products of this thread's columns
        float z = 0.f, dz = 0.f;
#pragma unroll
        for (int q = 0; q < F_NQ; ++q) {
          const v4f x = xb[bi][r][q];
          z = fmaf(x.x, th[q].x, z); z = fmaf(x.y, th[q].y, z); z = fmaf(x.z, th[q].z, z); z = fmaf(x.w, th[q].w, z);
          dz = fmaf(x.x, dd[q].x, dz); dz = fmaf(x.y, dd[q].y, dz); dz = fmaf(x.z, dd[q].z, dz); dz = fmaf(x.w, dd[q].w, dz);
        }
        // even lanes carry the sum of z, odd lanes of dz, over each row of 16 lanes (fixed tree)
        const bool up = (lane & 1) != 0;
        float v = (up ? dz : z) + dpp_get<0xB1>(up ? z : dz);
        v = row16_parity_sum(v);
        if ((lane & 15) < F_V) red[it & 1][r][lane & 1][w * 4 + (lane >> 4)] = v;
      }
      advance(pm, ploc, pend, pfirst);
      // the registers are free for the rows PDI iterations ahead
      if (more) {
        if constexpr (!drain) { if (qloc == 0) issue_ref((it + PDI) * R); }
        qloc += R;
        if (qloc == nslab) qloc = 0;
      }
      if constexpr (st) {
#pragma unroll
        for (int r = 0; r < R; ++r) issue_slab(xb[bi][r], rp[r], col);
      } else if (more) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int q = 0; q < F_NQ; ++q) xb[bi][r][q] = *reinterpret_cast<const v4f *>(rp[r] + col[q]);
      }
    }
    // 3b. accumulate the rows consumed in the previous iteration
    if (st || pending) accumulate();
    lds_barrier();
    pending = cons;
    if (cons) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        rr[r] = r_s[c0 & 1][r]; dr[r] = dr_s[c0 & 1][r];
#pragma unroll
        for (int q = 0; q < F_NQ; ++q) xr[r][q] = xn[r][q];
      }
    }
  };

  int s0 = 0;
  for (; s0 < HEAD && s0 < total; s0 += PDI)
    unrolled<PDI>([&](auto I) __attribute__((always_inline)) {
      if (s0 + I.value < total) stream_iter(I, bc<false>{}, s0 + I.value);
    });
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): nothing the compiler tracks is in flight from here on
  for (; s0 + 2 * PDI < IS; s0 += PDI)
    unrolled<PDI>([&](auto I) __attribute__((always_inline)) { stream_iter(I, bc<true>{}, s0 + I.value); });
  // the loads of the last trip are still in flight and unknown to the compiler
  unrolled<PDI>([&](auto I) __attribute__((always_inline)) { wait_rows<0, R>(xb[I.value]); });
  for (; s0 < total; s0 += PDI)
    unrolled<PDI>([&](auto I) __attribute__((always_inline)) {
      if (s0 + I.value < total) stream_iter(I, bc<false>{}, s0 + I.value);
    });
  if (pending) accumulate();
}

// Adds up the parts of the workers whose rows the last round split over several clusters (in the order
// of the row ranges), adds the regulariser's terms, stores the fresh gradient (CADA1: and the fresh
// innovation) and the partial sums of the rule's left-hand side.  grid (4 Q, rem), 128 threads, four columns
// each: block b owns columns [512 b, 512 b + 512), its two wavefronts slots 2 b and 2 b + 1 of the worker's
// partial sums (as many slots per 2048 columns as k_fused has streaming wavefronts).
__global__ __launch_bounds__(128) void k_fused_tail(const FusedArgs a) {
  static_assert(F_SW == 8, "two slots per 512 columns");
  const DevState &s = a.s;
  const int j = blockIdx.y, m = (s.M / a.n_clusters) * a.n_clusters + j;
  const int64_t c0 = ((int64_t)blockIdx.x * 128 + threadIdx.x) * 4;
  float sq = 0.f;
  if (c0 < s.p) {
    const RefPtr ref = theta_ref(s, m, s.k);
    const float4 tt = *reinterpret_cast<const float4 *>(s.theta + c0), tl = *reinterpret_cast<const float4 *>(s.theta_lo + c0);
    const float4 rh = *reinterpret_cast<const float4 *>(ref.hi + c0), rl = *reinterpret_cast<const float4 *>(ref.lo + c0);
    const float4 d = make_float4((tt.x - rh.x) + (tl.x - rl.x), (tt.y - rh.y) + (tl.y - rl.y), (tt.z - rh.z) + (tl.z - rl.z), (tt.w - rh.w) + (tl.w - rl.w));
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f), iv = g;
    for (int h = 0; h < a.tail_f; ++h) {
      const float *pg = a.tail_part + (((int64_t)h * a.tail_rem + j) * 2) * s.p;
      const float4 x = *reinterpret_cast<const float4 *>(pg + c0), y = *reinterpret_cast<const float4 *>(pg + s.p + c0);
      g.x += x.x; g.y += x.y; g.z += x.z; g.w += x.w;
      iv.x += y.x; iv.y += y.y; iv.z += y.z; iv.w += y.w;
    }
    g.x = fmaf(s.lam, tt.x, g.x); g.y = fmaf(s.lam, tt.y, g.y); g.z = fmaf(s.lam, tt.z, g.z); g.w = fmaf(s.lam, tt.w, g.w);
    iv.x = fmaf(s.lam, d.x, iv.x); iv.y = fmaf(s.lam, d.y, iv.y); iv.z = fmaf(s.lam, d.z, iv.z); iv.w = fmaf(s.lam, d.w, iv.w);
    const int cur = s.sel[m];
    const int64_t mp = (int64_t)s.M * s.p;
    *reinterpret_cast<float4 *>(s.gbuf + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + c0) = g;
    if (s.rule == CADA_RULE_CADA1) {
      const float4 stv = *reinterpret_cast<const float4 *>(s.dtl + (int64_t)cur * mp + (int64_t)m * s.p + c0);
      *reinterpret_cast<float4 *>(s.dtl + (int64_t)(1 - cur) * mp + (int64_t)m * s.p + c0) = iv;
      iv.x -= stv.x; iv.y -= stv.y; iv.z -= stv.z; iv.w -= stv.w;
    }
    sq = fmaf(iv.x, iv.x, sq); sq = fmaf(iv.y, iv.y, sq); sq = fmaf(iv.z, iv.z, sq); sq = fmaf(iv.w, iv.w, sq);
  }
  const float ws = wave_sum(sq);
  if ((threadIdx.x & 63) == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + blockIdx.x * 2 + (threadIdx.x >> 6)] = ws;
}

template <bool DRAIN>
static const void *fused_kernel_of(int R, int NJ) {
  if (R == 2) return NJ == 2 ? reinterpret_cast<const void *>(k_fused<2, 2, DRAIN>) : reinterpret_cast<const void *>(k_fused<2, 1, DRAIN>);
  return NJ == 2 ? reinterpret_cast<const void *>(k_fused<1, 2, DRAIN>) : reinterpret_cast<const void *>(k_fused<1, 1, DRAIN>);
}
static const void *fused_kernel(int R, int NJ, int B) { return B < 32 ? fused_kernel_of<true>(R, NJ) : fused_kernel_of<false>(R, NJ); }

// Chooses the cluster geometry; returns false if the single-pass path does not apply.
bool fused_plan(Ctx *c, const cada_config *cfg) {
  c->fused = 0;
  const int64_t p = cfg->p;
  const int B = cfg->B, M = cfg->M;
  if (c->vec != 4 || p < 8192) return false;
  int dev = 0, coop = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return false;
  const int64_t per_block = (int64_t)F_STREAM * 4 * F_NQ;        // 2048 columns per workgroup
  int Q = (int)((p + per_block - 1) / per_block);
  if (Q > F_QMAX || Q > cus) return false;
  int R = (B % 2 == 0) ? 2 : 1;                            // rows per iteration
  if (cfg->single_pass_rows == 1) R = 1;
  const int NJ = Q > 32 ? 2 : 1;
  const void *fn = fused_kernel(R, NJ, B);
  const size_t lds = R == 2 ? FusedGeom<2>::lds : FusedGeom<1>::lds;
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  int per_cu = 0;
  const hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, F_THREADS, lds);
  if (oe != hipSuccess || per_cu < 1) {
    (void)hipGetLastError();
    return false;
  }
  int ncl = cus / Q;                       // one workgroup per CU
  if (ncl < 1) return false;
  ncl = min(ncl, M);
  if (cfg->single_pass_clusters >= 1 && cfg->single_pass_clusters < ncl) ncl = cfg->single_pass_clusters;
  if ((size_t)ncl * F_NP * F_V * Q > kFusedPostWords) return false;
  c->fused = 1;
  c->fused_Q = Q;
  c->fused_clusters = ncl;
  c->fused_rs = R;
  c->fused_plain_launch = cfg->plain_launch != 0 ? 1 : 0;
  const int nslab = B;
  // last round: split the rows of the rem last workers over all clusters when that divides evenly
  const int rem = M % ncl;
  c->fused_tail_f = 0; c->fused_tail_rows = 0; c->fused_tail_rem = 0;
  if (rem > 0 && ncl % rem == 0 && nslab % (ncl / rem) == 0 && (nslab / (ncl / rem)) % R == 0 &&
      (size_t)ncl * 2 * (size_t)p <= kFusedTailFloatsPerP * (size_t)p) {
    c->fused_tail_f = ncl / rem; c->fused_tail_rows = nslab / (ncl / rem); c->fused_tail_rem = rem;
  }
  c->fused_seq_per_step = (uint32_t)(c->fused_tail_f ? (M / ncl) * nslab + c->fused_tail_rows : ((M + ncl - 1) / ncl) * nslab);
  return true;
}

int logreg_gradients_fused(Ctx *c, const int32_t *idx) {
  FusedArgs a;
  a.s = c->s;
  a.s.k = c->k;
  a.idx = idx;
  a.zpost = c->fused_post;
  a.Q = c->fused_Q;
  a.n_clusters = c->fused_clusters;
  a.seq_base = c->fused_seq;
  a.spin_limit = 2000000u;
  a.tail_f = c->fused_tail_f; a.tail_rows = c->fused_tail_rows; a.tail_rem = c->fused_tail_rem; a.tail_part = c->fused_tail;
  void *args[] = {&a};
  prof_mark(c);
  hipError_t e;
  const dim3 grid((unsigned)(a.Q * a.n_clusters)), block(F_THREADS);
  const bool two = c->fused_rs == 2;
  const size_t lds = two ? FusedGeom<2>::lds : FusedGeom<1>::lds;
  if (c->fused_plain_launch) {
    // Same grid without the cooperative-launch guarantee: one workgroup per CU is resident at once
    // on an otherwise idle device, and every wait in the kernel is bounded.  For profilers that
    // cannot trace cooperative dispatches.
    e = hipLaunchKernel(fused_kernel(c->fused_rs, a.Q > 32 ? 2 : 1, a.s.B), grid, block, args, lds, c->stream);
  } else {
    e = hipLaunchCooperativeKernel(fused_kernel(c->fused_rs, a.Q > 32 ? 2 : 1, a.s.B), grid, block, args, (unsigned)lds, c->stream);
  }
  if (a.tail_f > 0) prof_mark(c);          // (a phase of its own)
  if (e == hipSuccess && a.tail_f > 0) {
    hipLaunchKernelGGL(k_fused_tail, dim3((unsigned)(4 * a.Q), (unsigned)a.tail_rem), dim3(128), 0, c->stream, a);
    e = hipGetLastError();
  }
  prof_mark(c);
  if (e != hipSuccess) {
    set_error("fused logistic gradient launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  c->fused_seq += c->fused_seq_per_step;      // (the tags advance only with a launch that was accepted)
  return CADA_OK;
}

}  // namespace cada
