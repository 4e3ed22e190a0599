// Internal declarations shared by the HIP translation units of libcada.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "cada.h"

namespace cada {

constexpr int kBlock = 256;          // threads per workgroup = 4 wavefronts of 64
constexpr int kWave = 64;

// Everything the kernels need to find the state; passed by value.
struct DevState {
  // server vectors [p].  The iterate is kept as an unevaluated sum theta + theta_lo of two
  // floats (|theta_lo| <= ulp(theta)/2): theta - theta_ref, which the rules' left-hand side
  // is a function of, is then accurate to float32 relative precision of the DIFFERENCE even
  // when it is a single small step (rounding theta alone perturbs a one-step difference by
  // 1e-5..1e-4 relative, more than the rule comparison tolerates).
  float *theta, *theta_lo, *h, *v, *vhat, *nabla;
  // stored / fresh stochastic gradients: gbuf[s][m][p], s in {0,1}.  Worker m's stored
  // gradient is gbuf[sel[m]][m]; the fresh one of the current step is written to
  // gbuf[1-sel[m]][m] and an upload is sel[m] ^= 1 (no copy).
  float *gbuf;
  // CADA_STORE_BF16: the same two rows per worker as bf16, gbuf16[s][m][ps16] (gbuf is null).  Written rounded to
  // nearest even by the gradient kernels, summed as they are by the server.
  uint16_t *gbuf16;
  // CADA2: hist[R][p], slot j mod R holds theta^j, R = D+1.  theta^{k-tau_m} is read here.
  float *hist, *hist_lo;
  // CADA1: snapshot theta-tilde [p] and innovations dtl[s][m][p] indexed by sel like gbuf.
  float *snap, *snap_lo, *dtl;
  // MLP with CADA1: the stored innovations are kept as bf16, dtl16[s][m][ps16] (dtl is null).  They
  // enter only the rule's left-hand side |fresh - stored|^2, whose other operand comes from bf16
  // contractions anyway; the stored GRADIENTS, which the server sums, stay float32.
  uint16_t *dtl16;
  int64_t ps;               // floats from one row of gbuf / dtl / hist to the next: p, or p rounded up to a
                            // multiple of 4 (MLP) so that every row starts on a 16-byte boundary
  int64_t ps16;             // elements from one row of dtl16 / gbuf16 to the next (a multiple of 8)
  int32_t *tau, *sel;     // [M]
  float *lhs;             // [M]
  float *lhs_part;        // [M][n_lhs_part] partial sums of the left-hand side
  uint8_t *mask;          // [M]
  float *ring;            // [d_max]
  float *ring_part;       // [n_ring_part] per-block partial sums of the last squared step,
                          // folded into ring[(k-1) mod d_max] by the next rule kernel
  uint64_t *uploads;
  uint32_t *n_up;          // [2]: uploads of iteration k in slot k mod 2 (the server kernel clears the other slot)
  int32_t resum;           // this launch: form the aggregate as the plain sum over all workers (0: the kernel may
                           // take the incremental form of Section 1.2 when few workers uploaded)
  uint32_t *err;
  // trace
  uint8_t *t_mask, *t_own;
  float *t_lhs, *t_rhs;
  int32_t *t_tau;
  int64_t trace_steps;
  // problem
  const float *X;
  const void *y;
  const int64_t *row_off;   // device [M+1], prefix sums of N_m
  int32_t M, B, d_max, D, R, rule, server_sgd, n_lhs_part, n_ring_part;
  int64_t p;
  int64_t k;                // iteration of the launch this copy is passed to
  float alpha, beta1, beta2, omb1, omb2, eps, lam;   // omb = 1 - beta, rounded once from double
  double c;
  double alpha0;            // stepsize constant; alpha above is the stepsize of iteration k
  int64_t alpha_K0;         // 0: constant; else alpha_k = alpha0 K0 / (k + K0)
};

// Reference point of worker m at iteration k (Algorithm 1: theta-tilde for CADA1,
// theta^{k - tau_m^k} for CADA2).  The always-upload and the stochastic LAG rules evaluate no
// second gradient: their reference point is the iterate itself, so every difference the
// gradient kernels carry is exactly zero.
struct RefPtr { const float *hi, *lo; };
// (for a caller that already holds the worker's delay tau_m^k)
__device__ __forceinline__ RefPtr theta_ref_at(const DevState &s, int32_t tau_m, int64_t k) {
  if (s.rule == CADA_RULE_CADA1) return RefPtr{s.snap, s.snap_lo};
  if (s.rule != CADA_RULE_CADA2) return RefPtr{s.theta, s.theta_lo};
  int64_t j = k - (int64_t)min(tau_m, s.D);      // tau <= D unless a replay kept m silent longer
  int64_t slot = j % s.R;
  if (slot < 0) slot += s.R;
  return RefPtr{s.hist + slot * s.ps, s.hist_lo + slot * s.ps};
}
__device__ __forceinline__ RefPtr theta_ref(const DevState &s, int m, int64_t k) {
  return theta_ref_at(s, s.rule == CADA_RULE_CADA2 ? s.tau[m] : 0, k);
}

// Stepsize of iteration k (constant, or the decaying 2/(mu(k+K0)) of Theorem 2).
__host__ __device__ __forceinline__ float stepsize(const DevState &s, int64_t k) {
  return s.alpha_K0 <= 0 ? (float)s.alpha0 : (float)(s.alpha0 * (double)s.alpha_K0 / (double)(k + s.alpha_K0));
}

// bf16 storage: the hardware conversion (v_cvt_pk_bf16_f32: round to nearest even, NaN stays NaN),
// one value, or two packed into a register (first argument in the low half).
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t f2bf_pk(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// Sum over the 256 threads of a block in a fixed order; result valid in every thread.
__device__ __forceinline__ float block_sum(float x, float *red /* [4] LDS */) {
  x = wave_sum(x);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = x;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// Sum over the 64 lanes without the LDS permute path: four data-parallel-primitive steps inside each row of 16 lanes
// (quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_ror:4, row_ror:8), then the four rows' sums by lane reads.  Every
// lane gets the result; a __shfl_xor butterfly is six dependent LDS-path permutes.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = dpp_add<0xB1>(v); v = dpp_add<0x4E>(v); v = dpp_add<0x124>(v); v = dpp_add<0x128>(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}

// Workgroup barrier for data that is exchanged through LDS: it waits for this wavefront's LDS operations only, not, as
// __syncthreads() does, for the acknowledgement of every global store issued before it (a microsecond each time).
// Data that a thread loaded from memory and passes on through LDS is waited for where it is written to LDS.
__device__ __forceinline__ void lds_sync() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// block_sum with that barrier and the wavefront sums of wave_sum_dpp
__device__ __forceinline__ float block_sum_lds(float x, float *red /* [4] LDS */) {
  x = wave_sum_dpp(x);
  lds_sync();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  lds_sync();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

struct LogregLaunch;   // defined in cada_logreg.hip

// Host context.
struct Ctx {
  DevState s;
  hipStream_t stream;
  int64_t k;                 // steps enqueued
  int32_t model, gemm_dtype, n_layers;
  int32_t dims[CADA_MAX_LAYERS + 1];
  size_t ws_bytes;
  void *ws_base;             // the caller's workspace
  // logistic launch geometry
  int vec;                   // 4 if rows can be read as float4, else 1
  int n_col_chunks;          // column chunks of the dot-product kernel
  int64_t chunk_cols;
  float *zpart;              // [M][B][n_col_chunks][2]
  int n_server_blocks;
  int ring_cap;               // entries of ring_part in the workspace
  // single-pass (register-resident) logistic path, cada_logreg_fused.hip
  int fused, fused_Q, fused_clusters, fused_rs, fused_plain_launch;
  uint32_t fused_seq, fused_seq_per_step;
  unsigned long long *fused_post;
  int fused_tail_f, fused_tail_rows, fused_tail_rem;   // split of the last round's workers over the clusters (0: none)
  float *fused_tail;         // [clusters][2][p]: the clusters' parts of the split workers' sums
  // whole iterations in one launch for small logistic workloads, cada_logreg_small.hip
  int small;
  size_t small_lds;
  int small_plain_launch;    // launch it as an ordinary grid (profilers that cannot trace cooperative dispatches)
  uint32_t *small_bar;       // the whole-step kernel's barrier words in the workspace
  uint32_t small_seq;        // its value after everything enqueued so far
  void *small_args;          // room in the workspace for this context's launch-invariant arguments (replica launches)
  void *small_args_host;     // their host copy (owned by the context)
  // full-data evaluation scratch (cada_eval)
  double *eval_part;         // [M][kEvalBlocks][2] per-block sums of (loss, correct)
  double *eval_acc;          // [M][2]
  int32_t *eval_idx;         // [M][B] row ids of one evaluation chunk (MLP)
  int logreg_group;          // workers per launch pair of the logistic gradient kernels (0 = all)
  int force_resum;           // the stored aggregate does not belong to the state (first step, after cada_set_state)
  void *mlp;                 // MLP plan (cada_mlp.hip), or nullptr
  void *prof;                // profiling events (cada_api.hip), or nullptr
  int n_phases;              // phases per step = marks per step - 1
  const char *phase_names[16];
};

void set_error(const char *fmt, ...);
// Records the next profiling event on the stream when profiling is active (else no-op).
void prof_mark(Ctx *c);

// S1+S2 for the logistic model: fresh gradients into gbuf[1-sel], left-hand sides into lhs_part.
int logreg_gradients(Ctx *c, const int32_t *idx);
bool fused_plan(Ctx *c, const cada_config *cfg);
int logreg_gradients_fused(Ctx *c, const int32_t *idx);
int small_steps(Ctx *c, const int32_t *idx, const uint8_t *replay, int64_t n_steps);
int small_steps_replicas(Ctx *const *cs, int n, const int32_t *const *idx, const uint8_t *const *replay, int64_t n_steps);
constexpr size_t kSmallArgsBytes = 1024;    // >= sizeof(SmallArgs), checked where it is defined
bool small_plan(Ctx *c, const cada_config *cfg);
int small_publish_args(Ctx *c);             // after the state pointers are final, and after a checkpoint was loaded
void small_free(Ctx *c);
int logreg_init(Ctx *c);                    // LDS allowance of the two-pass kernels
constexpr int kFusedWaves = 8;                      // streaming wavefronts of a single-pass workgroup: one partial sum of the left-hand side each
constexpr size_t kFusedTailFloatsPerP = 2 * 32;     // room for the parts of 32 clusters (one per cluster, two sums)
constexpr size_t kFusedPostWords = 1024 * 4 * 16;   // upper bound: 1024 workgroups x 4 buffers x 16 values
// S1+S2 for the MLP.
int mlp_gradients(Ctx *c, const int32_t *idx);
int mlp_lhs_slots(const cada_config *cfg);
int mlp_eval(Ctx *c, double *out);
int logreg_eval(Ctx *c, double *out);
int logreg_eval_noalloc(Ctx *c, double *out);   // the same kernels with their scratch in a file-scope device array
int eval_scratch_init();                        // looks that array's address up on the current device
void eval_finish(Ctx *c, double *out, int with_reg);   // out = mean over the workers of eval_acc (+ regulariser)
constexpr int kEvalBlocks = 512;      // blocks per worker of the logistic evaluation kernel
size_t mlp_workspace_bytes(const cada_config *cfg, const int64_t total_rows);
int mlp_plan(Ctx *c, const cada_config *cfg, char *base, size_t *offset, int64_t total_rows);
int mlp_init_state(Ctx *c, const float *theta0);
void mlp_free(Ctx *c);
// S3: rule, mask, tau.  S5-S7: aggregate, AMSGrad, ring push.
int rule_and_server(Ctx *c, const uint8_t *replay);

}  // namespace cada
