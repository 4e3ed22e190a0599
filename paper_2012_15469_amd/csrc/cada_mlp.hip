// Dual minibatch gradient of a ReLU MLP with softmax cross-entropy for all workers, bf16
// MFMA contractions with float32 accumulation, and the left-hand side of the communication
// rule (Section 2.2, conditions (workerrule1)/(workerrule2); Algorithm 1, the two gradient
// evaluations on the same samples).
//
// The second gradient is never formed by itself.  With d = theta - theta_ref (float32, from
// the two-float iterate) every quantity of the reference evaluation is carried as a
// difference to the evaluation at theta, and the differences are propagated exactly:
//   forward   dZ_1 = A_0 dW_1 + db_1,           dZ_l = dA_{l-1} W_l + Aref_{l-1} dW_l + db_l
//             A_l = relu(Z_l), Aref_l = relu(Z_l - dZ_l), dA_l = A_l - Aref_l
//   loss      G_L = (softmax(Z_L) - onehot)/B,  dG_L = (softmax(Z_L) - softmax(Z_L - dZ_L))/B
//   backward  grad W_l = A_{l-1}^T G_l,         innov W_l = A_{l-1}^T dG_l + dA_{l-1}^T Gref_l
//             GA_{l-1} = G_l W_l^T,             dGA_{l-1} = dG_l W_l^T + Gref_l dW_l^T
//             G_{l-1} = GA_{l-1} [Z>0],         Gref_{l-1} = (GA - dGA)_{l-1} [Zref>0]
// (Gref = G - dG).  Rounding W and W_ref to bf16 separately would bury their difference (one
// Adam step is about one bf16 ulp of a weight); rounding d itself keeps 8 significant bits
// of the difference, which is what the rule's comparison needs.
//
// Precision.  The difference of two ReLU-network gradients at nearby points is dominated by
// the few units whose pre-activation changes sign between the two points, so the rule's
// left-hand side is only as good as the pre-activations Z_l are near zero: they must be
// resolved well below |dZ_l| ~ 1e-3 |Z_l|, which a single bf16 product (2^-9 per operand)
// cannot do.  The forward contractions Z_l = A_{l-1} W_l therefore use split operands
// x = hi + lo (two bf16 values, 16 significant bits) and three MFMA products
// hi*hi + hi*lo + lo*hi accumulated in float32.  The backward contractions of the gradient at
// theta (grad W_l, GA_l) are split the same way: the server's update divides by sqrt(vhat),
// so a coordinate whose gradient is smaller than its rounding error moves by a full
// +-alpha-sized step in a random direction, and with single bf16 products (0.2% gradient
// error) the iterate drifts from the fp64 trajectory by percents within tens of steps.
// Only the difference contractions (dZ, dGA, the innovation) are single bf16 products.
//
// One GEMM kernel serves every contraction: C = sum over up to four operand pairs of
// A_i B_i^T, 128x128 output tile per workgroup, 4 wavefronts of 64x64, K step 32,
// v_mfma_f32_32x32x16_bf16.  Either operand may be stored K-contiguous or M/N-contiguous
// (transposed while it is staged into LDS), rows may be gathered through an index array, and
// a batch index (the worker) offsets all three matrices.
#include <cstdlib>
#include <new>

#include "cada_internal.h"

namespace cada {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint16_t bf16_t;   // storage type

__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);                                          // round to nearest even
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }

inline int64_t P8(int64_t x) { return (x + 7) / 8 * 8; }

// ------------------------------------------------------------------------------------------
// GEMM
// ------------------------------------------------------------------------------------------
struct Operand {
  const bf16_t *ptr;
  int64_t ld;            // leading dimension of the row-major source (multiple of 8)
  int64_t batch_stride;  // elements added per batch index
  const int64_t *gather; // optional: source row r is read at row gather[batch*gather_stride + r]
  int64_t gather_stride;
  int kmajor;            // 1: source rows are the M (or N) index, K contiguous
                         // 0: source rows are the K index, M (or N) contiguous
};

struct GemmArgs {
  Operand A[4], B[4];
  int K[4];
  int npairs;
  int M, N;
  float *C;
  int64_t ldc, c_batch_stride;
  const int32_t *sel;      // optional: C += (1 - sel[batch]) * c_sel_stride  (fresh half of a double buffer)
  int64_t c_sel_stride;
};

constexpr int BM = 128, BN = 128, BK = 32, PITCH = BK + 8;

struct Chunk { uint4 v; };

// Loads the two 16-byte chunks this thread contributes to a 128 x 32 operand tile.
// rows0: first M/N index of the tile, k0: first K index, R: extent of the M/N index.
__device__ __forceinline__ void load_chunks(const Operand &op, const bf16_t *base, const int64_t *gat, int rows0, int R, int k0, int K,
                                            uint4 (&out)[2]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (op.kmajor) {
      const int row = rows0 + (t >> 2) + c * 64;       // 4 chunks of 8 k per row
      const int k = k0 + (t & 3) * 8;
      if (row < R && k < K) {
        const int64_t src = gat ? gat[row] : (int64_t)row;
        v = *reinterpret_cast<const uint4 *>(base + src * op.ld + k);
      }
    } else {
      const int k = k0 + (t >> 4) + c * 16;            // 16 chunks of 8 m per k-row
      const int row = rows0 + (t & 15) * 8;
      if (k < K && row < R) {
        const int64_t src = gat ? gat[k] : (int64_t)k;
        v = *reinterpret_cast<const uint4 *>(base + src * op.ld + row);
      }
    }
    out[c] = v;
  }
}

__device__ __forceinline__ void store_chunks(const Operand &op, bf16_t *lds, const uint4 (&in)[2]) {
  const int t = threadIdx.x;
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    if (op.kmajor) {
      const int row = (t >> 2) + c * 64, kc = (t & 3) * 8;
      *reinterpret_cast<uint4 *>(lds + row * PITCH + kc) = in[c];
    } else {
      const int k = (t >> 4) + c * 16, row = (t & 15) * 8;
      const uint32_t w[4] = {in[c].x, in[c].y, in[c].z, in[c].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) lds[(row + e) * PITCH + k] = (bf16_t)(w[e >> 1] >> ((e & 1) * 16));
    }
  }
}

// grid (ceil(N/128), ceil(M/128), batches)
__global__ __launch_bounds__(kBlock) void k_gemm(const GemmArgs g) {
  __shared__ __align__(16) bf16_t As[BM * PITCH];
  __shared__ __align__(16) bf16_t Bs[BN * PITCH];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wy = w >> 1, wx = w & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int64_t batch = blockIdx.z;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  for (int pr = 0; pr < g.npairs; ++pr) {
    const Operand &oa = g.A[pr], &ob = g.B[pr];
    const bf16_t *abase = oa.ptr + batch * oa.batch_stride;
    const bf16_t *bbase = ob.ptr + batch * ob.batch_stride;
    const int64_t *agat = oa.gather ? oa.gather + batch * oa.gather_stride : nullptr;
    const int64_t *bgat = ob.gather ? ob.gather + batch * ob.gather_stride : nullptr;
    const int K = g.K[pr];
    uint4 ra[2], rb[2];
    load_chunks(oa, abase, agat, m0, g.M, 0, K, ra);
    load_chunks(ob, bbase, bgat, n0, g.N, 0, K, rb);
    for (int k0 = 0; k0 < K; k0 += BK) {
      __syncthreads();                       // previous tile fully consumed
      store_chunks(oa, As, ra);
      store_chunks(ob, Bs, rb);
      __syncthreads();
      if (k0 + BK < K) {
        load_chunks(oa, abase, agat, m0, g.M, k0 + BK, K, ra);
        load_chunks(ob, bbase, bgat, n0, g.N, k0 + BK, K, rb);
      }
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        bf16x8 a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
          a[i] = *reinterpret_cast<const bf16x8 *>(As + (wy * 64 + i * 32 + (lane & 31)) * PITCH + ks + (lane >> 5) * 8);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          b[j] = *reinterpret_cast<const bf16x8 *>(Bs + (wx * 64 + j * 32 + (lane & 31)) * PITCH + ks + (lane >> 5) * 8);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
    }
  }

  float *C = g.C + batch * g.c_batch_stride;
  if (g.sel) C += (int64_t)(1 - g.sel[batch]) * g.c_sel_stride;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wx * 64 + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wy * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < g.M && col < g.N) C[(int64_t)row * g.ldc + col] = acc[i][j][r];
      }
    }
}

// ------------------------------------------------------------------------------------------
// plan
// ------------------------------------------------------------------------------------------
struct MlpPlan {
  int L, M, B, rule;
  int64_t R;                      // M * B rows per step
  int64_t total_rows;             // rows of X
  int d[CADA_MAX_LAYERS + 1];
  int64_t offW[CADA_MAX_LAYERS], offb[CADA_MAX_LAYERS];   // offsets into theta
  int64_t ldw[CADA_MAX_LAYERS];                           // P8(d_l): ld of the bf16 weights of layer l
  int64_t wb_off[CADA_MAX_LAYERS], wb_total;              // offsets into the bf16 weight copy
  int64_t lda[CADA_MAX_LAYERS + 1];                       // P8(d_l): ld of bf16 activations of width d_l
  int nW;                                                 // 1 (CADA1) or M (CADA2) delta-weight copies
  bf16_t *Xb, *Xl; int64_t ldx;          // features: hi and lo parts
  int64_t *grow;
  bf16_t *Wb, *Wl, *dWb;                 // weights hi, lo; delta weights
  float *Z[CADA_MAX_LAYERS], *dZ[CADA_MAX_LAYERS];         // [R][d_l], index l-1
  bf16_t *A[CADA_MAX_LAYERS], *Al[CADA_MAX_LAYERS], *dA[CADA_MAX_LAYERS], *Aref[CADA_MAX_LAYERS];   // hidden l = 1..L-1, index l
  bf16_t *G[CADA_MAX_LAYERS], *Gl[CADA_MAX_LAYERS], *dG[CADA_MAX_LAYERS], *Gref[CADA_MAX_LAYERS];   // index l-1; (G, Gl) = hi, lo
  float *GA[CADA_MAX_LAYERS], *dGA[CADA_MAX_LAYERS];       // [R][d_l], hidden l, index l
  float *innov;                                            // CADA2: [M][p]
};

namespace {
constexpr size_t kAlignB = 256;
struct Carve {
  char *base; size_t off;
  template <typename T> T *take(size_t n) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off = (off + n * sizeof(T) + kAlignB - 1) / kAlignB * kAlignB;
    return p;
  }
};

void layout(MlpPlan &P, const cada_config *cfg, int64_t total_rows, Carve &w) {
  P.L = cfg->n_layers; P.M = cfg->M; P.B = cfg->B; P.rule = cfg->rule;
  P.R = (int64_t)cfg->M * cfg->B;
  P.total_rows = total_rows;
  int64_t o = 0, wo = 0;
  for (int l = 0; l <= P.L; ++l) { P.d[l] = cfg->layer_dims[l]; P.lda[l] = P8(P.d[l]); }
  for (int l = 0; l < P.L; ++l) {
    P.offW[l] = o; o += (int64_t)P.d[l] * P.d[l + 1];
    P.offb[l] = o; o += P.d[l + 1];
    P.ldw[l] = P8(P.d[l + 1]);
    P.wb_off[l] = wo; wo += (int64_t)P.d[l] * P.ldw[l];
  }
  P.wb_total = wo;
  P.nW = (cfg->rule == CADA_RULE_CADA2) ? cfg->M : 1;
  P.ldx = P8(P.d[0]);
  P.Xb = w.take<bf16_t>((size_t)total_rows * P.ldx);
  P.Xl = w.take<bf16_t>((size_t)total_rows * P.ldx);
  P.grow = w.take<int64_t>((size_t)P.R);
  P.Wb = w.take<bf16_t>((size_t)P.wb_total);
  P.Wl = w.take<bf16_t>((size_t)P.wb_total);
  P.dWb = w.take<bf16_t>((size_t)P.wb_total * P.nW);
  for (int l = 1; l <= P.L; ++l) {
    P.Z[l - 1] = w.take<float>((size_t)P.R * P.d[l]);
    P.dZ[l - 1] = w.take<float>((size_t)P.R * P.d[l]);
    P.G[l - 1] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
    P.Gl[l - 1] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
    P.dG[l - 1] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
    P.Gref[l - 1] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
    if (l < P.L) {
      P.A[l] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
      P.Al[l] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
      P.dA[l] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
      P.Aref[l] = w.take<bf16_t>((size_t)P.R * P.lda[l]);
      P.GA[l] = w.take<float>((size_t)P.R * P.d[l]);
      P.dGA[l] = w.take<float>((size_t)P.R * P.d[l]);
    }
  }
  P.innov = (cfg->rule == CADA_RULE_CADA2) ? w.take<float>((size_t)cfg->M * (size_t)cfg->p) : nullptr;
}
}  // namespace

size_t mlp_workspace_bytes(const cada_config *cfg, const int64_t total_rows) {
  if (cfg->gemm_dtype != CADA_GEMM_BF16) { set_error("the MLP model computes its contractions in bf16 (gemm_dtype must be CADA_GEMM_BF16)"); return 0; }
  if (cfg->n_layers < 2) { set_error("the MLP model needs at least 2 layers"); return 0; }
  if (cfg->layer_dims[cfg->n_layers] > 32) { set_error("at most 32 classes"); return 0; }
  MlpPlan P;
  Carve w{nullptr, 0};
  layout(P, cfg, total_rows, w);
  return w.off + kAlignB;
}

int mlp_plan(Ctx *c, const cada_config *cfg, char *base, size_t *offset, int64_t total_rows) {
  if (mlp_workspace_bytes(cfg, total_rows) == 0) return CADA_EUNSUPPORTED;
  MlpPlan *P = new (std::nothrow) MlpPlan();
  if (!P) { set_error("out of host memory"); return CADA_EINVAL; }
  Carve w{base, (*offset + kAlignB - 1) / kAlignB * kAlignB};
  layout(*P, cfg, total_rows, w);
  *offset = w.off;
  c->mlp = P;
  c->n_phases = 4;
  c->phase_names[0] = "mlp_gradients"; c->phase_names[1] = "mlp_lhs";
  c->phase_names[2] = "rule"; c->phase_names[3] = "server_update";
  return CADA_OK;
}

void mlp_free(Ctx *c) {
  delete static_cast<MlpPlan *>(c->mlp);
  c->mlp = nullptr;
}

// ------------------------------------------------------------------------------------------
// elementwise kernels
// ------------------------------------------------------------------------------------------
// float32 features -> bf16 copy with padded leading dimension (once, at init)
__global__ void k_x_to_bf16(const float *X, bf16_t *Xb, bf16_t *Xl, int64_t rows, int d0, int64_t ldx) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * ldx) return;
  const int64_t r = i / ldx; const int c = (int)(i % ldx);
  const float x = c < d0 ? X[r * d0 + c] : 0.f;
  const bf16_t hi = f2bf(x);
  Xb[i] = hi;
  Xl[i] = f2bf(x - bf2f(hi));
}

// grow[m*B + b] = global row of worker m's b-th minibatch sample
__global__ void k_rows(const DevState s, const int32_t *idx, int64_t *grow) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)s.M * s.B) return;
  const int m = (int)(i / s.B);
  const int64_t n = s.row_off[m + 1] - s.row_off[m];
  int64_t r = idx[i];
  if (r < 0 || r >= n) { atomicOr(s.err, 1u); r = r < 0 ? 0 : n - 1; }
  grow[i] = s.row_off[m] + r;
}

struct PrepArgs {
  DevState s;
  bf16_t *Wb, *Wl, *dWb;
  int64_t offW, wb_off, wb_total;
  int din, dout;
  int64_t ldw;
  int nW;
};

// bf16 copies of one layer's weights and of its difference to each reference point.
// grid (ceil(din*dout/256), nW + 1): y = 0 -> W, y = 1 + m -> d_m = theta - theta_ref(m)
__global__ void k_prep_weights(const PrepArgs a) {
  const DevState &s = a.s;
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)a.din * a.dout) return;
  const int i = (int)(e / a.dout), o = (int)(e % a.dout);
  const int64_t src = a.offW + e, dst = a.wb_off + (int64_t)i * a.ldw + o;
  if (blockIdx.y == 0) {
    const float wv = s.theta[src];
    const bf16_t hi = f2bf(wv);
    a.Wb[dst] = hi;
    a.Wl[dst] = f2bf(wv - bf2f(hi));
  } else {
    const int m = blockIdx.y - 1;
    const RefPtr ref = theta_ref(s, m, s.k);
    const float d = (s.theta[src] - ref.hi[src]) + (s.theta_lo[src] - ref.lo[src]);
    a.dWb[(int64_t)m * a.wb_total + dst] = f2bf(d);
  }
}

struct FwdArgs {
  DevState s;
  const float *Z, *dZ;         // [R][d]
  bf16_t *A, *Al, *dA, *Aref;  // [R][lda]; (A, Al) = hi and lo parts of the activation
  int64_t offb;                // bias offset in theta
  int d; int64_t lda;
};

// hidden layer: bias, ReLU at theta and at the reference point, activation difference
__global__ void k_hidden_fwd(const FwdArgs a) {
  const DevState &s = a.s;
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t R = (int64_t)s.M * s.B;
  if (e >= R * a.d) return;
  const int64_t r = e / a.d; const int c = (int)(e % a.d);
  const int m = (int)(r / s.B);
  const RefPtr ref = theta_ref(s, m, s.k);
  const int64_t bi = a.offb + c;
  const float b = s.theta[bi];
  const float db = (b - ref.hi[bi]) + (s.theta_lo[bi] - ref.lo[bi]);
  const float z = a.Z[e] + b;
  const float dz = a.dZ[e] + db;
  const float act = fmaxf(z, 0.f), aref = fmaxf(z - dz, 0.f);
  const int64_t o = r * a.lda + c;
  const bf16_t hi = f2bf(act);
  a.A[o] = hi;
  a.Al[o] = f2bf(act - bf2f(hi));
  a.Aref[o] = f2bf(aref);
  a.dA[o] = f2bf(act - aref);
}

struct LossArgs {
  DevState s;
  const float *Z, *dZ;          // logits without bias [R][C]
  bf16_t *G, *Gl, *dG, *Gref;   // [R][ldg]; (G, Gl) = hi and lo parts
  const int64_t *grow;
  int64_t offb;
  int C; int64_t ldg;
  float *innov;                 // CADA2 scratch [M][p] or nullptr (CADA1 writes dtl)
};

__device__ __forceinline__ float *fresh_grad(const DevState &s, int m) {
  return s.gbuf + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.p;
}
__device__ __forceinline__ float *fresh_innov(const DevState &s, float *innov, int m) {
  if (s.rule == CADA_RULE_CADA1) return s.dtl + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.p;
  return innov + (int64_t)m * s.p;
}

// softmax cross-entropy: G = (P - onehot)/B, dG = (P - Pref)/B with
// P_i - Pref_i = P_i (sum_j P_j expm1(-dz_j) - expm1(-dz_i)) / (1 + sum_j P_j expm1(-dz_j)).
// One block per worker; also the bias gradient of the last layer and its innovation.
__global__ __launch_bounds__(kBlock) void k_loss(const LossArgs a) {
  const DevState &s = a.s;
  constexpr int MAXC = 32;
  __shared__ float red[kBlock];
  const int m = blockIdx.x;
  const RefPtr ref = theta_ref(s, m, s.k);
  const int32_t *yv = static_cast<const int32_t *>(s.y);
  const float invB = 1.0f / (float)s.B;
  float sumG[MAXC], sumD[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) { sumG[c] = 0.f; sumD[c] = 0.f; }
  for (int b = threadIdx.x; b < s.B; b += kBlock) {
    const int64_t r = (int64_t)m * s.B + b;
    float z[MAXC], dz[MAXC];
    float zmax = -INFINITY;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      if (c < a.C) {
        const int64_t bi = a.offb + c;
        const float bb = s.theta[bi];
        const float db = (bb - ref.hi[bi]) + (s.theta_lo[bi] - ref.lo[bi]);
        z[c] = a.Z[r * a.C + c] + bb;
        dz[c] = a.dZ[r * a.C + c] + db;
        zmax = fmaxf(zmax, z[c]);
      }
    }
    float den = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) if (c < a.C) { z[c] = expf(z[c] - zmax); den += z[c]; }
    float S = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) if (c < a.C) { z[c] = z[c] / den; dz[c] = expm1f(-dz[c]); S = fmaf(z[c], dz[c], S); }
    const int label = yv[a.grow[r]];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      if (c < a.C) {
        const float gl = (z[c] - (c == label ? 1.f : 0.f)) * invB;
        const float dg = z[c] * (S - dz[c]) / (1.0f + S) * invB;
        const int64_t o = r * a.ldg + c;
        const bf16_t hi = f2bf(gl);
        a.G[o] = hi;
        a.Gl[o] = f2bf(gl - bf2f(hi));
        a.dG[o] = f2bf(dg);
        a.Gref[o] = f2bf(gl - dg);
        sumG[c] += gl;
        sumD[c] += dg;
      }
    }
  }
  float *gf = fresh_grad(s, m) + a.offb;
  float *iv = fresh_innov(s, a.innov, m) + a.offb;
  for (int c = 0; c < a.C; ++c) {
    float vg = 0.f, vd = 0.f;
#pragma unroll
    for (int cc = 0; cc < MAXC; ++cc) if (cc == c) { vg = sumG[cc]; vd = sumD[cc]; }
    __syncthreads();
    red[threadIdx.x] = vg;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) { if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o]; __syncthreads(); }
    if (threadIdx.x == 0) gf[c] = red[0];
    __syncthreads();
    red[threadIdx.x] = vd;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) { if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o]; __syncthreads(); }
    if (threadIdx.x == 0) iv[c] = red[0];
  }
}

struct BwdArgs {
  DevState s;
  const float *GA, *dGA;         // [R][d]: gradient w.r.t. the activations and its difference
  const bf16_t *A, *Aref;        // [R][lda] activations (their sign is the ReLU mask)
  bf16_t *G, *Gl, *dG, *Gref;    // [R][lda]
  int64_t offb;
  int d; int64_t lda;
  float *innov;
};

// hidden layer backward through the two ReLUs; bias gradient and its innovation.
// grid (ceil(d/64), M), block 256 = 64 columns x 4 row lanes
__global__ __launch_bounds__(kBlock) void k_hidden_bwd(const BwdArgs a) {
  const DevState &s = a.s;
  __shared__ float redg[4][64], redd[4][64];
  const int m = blockIdx.y;
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  float sg = 0.f, sd = 0.f;
  if (c < a.d) {
    for (int b = rl; b < s.B; b += 4) {
      const int64_t r = (int64_t)m * s.B + b;
      const int64_t o = r * a.lda + c;
      const float ga = a.GA[r * a.d + c], dga = a.dGA[r * a.d + c];
      const bool on = bf2f(a.A[o]) > 0.f, onref = bf2f(a.Aref[o]) > 0.f;
      const float gl = on ? ga : 0.f;
      const float gref = onref ? (ga - dga) : 0.f;
      const float dg = gl - gref;
      const bf16_t hi = f2bf(gl);
      a.G[o] = hi;
      a.Gl[o] = f2bf(gl - bf2f(hi));
      a.Gref[o] = f2bf(gref);
      a.dG[o] = f2bf(dg);
      sg += gl;
      sd += dg;
    }
  }
  redg[rl][cl] = sg;
  redd[rl][cl] = sd;
  __syncthreads();
  if (rl == 0 && c < a.d) {
    fresh_grad(s, m)[a.offb + c] = (redg[0][cl] + redg[1][cl]) + (redg[2][cl] + redg[3][cl]);
    fresh_innov(s, a.innov, m)[a.offb + c] = (redd[0][cl] + redd[1][cl]) + (redd[2][cl] + redd[3][cl]);
  }
}

// Left-hand side partial sums: CADA2 |innov_m|^2, CADA1 |innov_m - stored innovation_m|^2.
// grid (n_lhs_part, M)
__global__ __launch_bounds__(kBlock) void k_mlp_lhs(const DevState s, const float *innov) {
  __shared__ float red[4];
  const int m = blockIdx.y;
  const int64_t per = (s.p + s.n_lhs_part - 1) / s.n_lhs_part;
  const int64_t e0 = (int64_t)blockIdx.x * per, e1 = min(s.p, e0 + per);
  float sq = 0.f;
  if (s.rule == CADA_RULE_CADA1) {
    const int cur = s.sel[m];
    const float *fr = s.dtl + ((int64_t)(1 - cur) * s.M + m) * s.p;
    const float *st = s.dtl + ((int64_t)cur * s.M + m) * s.p;
    for (int64_t e = e0 + threadIdx.x; e < e1; e += kBlock) { const float d = fr[e] - st[e]; sq = fmaf(d, d, sq); }
  } else {
    const float *fr = innov + (int64_t)m * s.p;
    for (int64_t e = e0 + threadIdx.x; e < e1; e += kBlock) { const float d = fr[e]; sq = fmaf(d, d, sq); }
  }
  const float tot = block_sum(sq, red);
  if (threadIdx.x == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + blockIdx.x] = tot;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
namespace {

Operand op(const bf16_t *p, int64_t ld, int64_t bstride, int kmajor, const int64_t *gather = nullptr, int64_t gstride = 0) {
  Operand o;
  o.ptr = p; o.ld = ld; o.batch_stride = bstride; o.gather = gather; o.gather_stride = gstride; o.kmajor = kmajor;
  return o;
}

void launch_gemm(Ctx *c, GemmArgs &g, int batches) {
  const dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, batches);
  hipLaunchKernelGGL(k_gemm, grid, dim3(kBlock), 0, c->stream, g);
}

}  // namespace

// One-time work at init: the bf16 copy of the features.
int mlp_init_state(Ctx *c, const float *) {
  MlpPlan &P = *static_cast<MlpPlan *>(c->mlp);
  const int64_t n = P.total_rows * P.ldx;
  hipLaunchKernelGGL(k_x_to_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->s.X, P.Xb, P.Xl, P.total_rows, P.d[0], P.ldx);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("feature conversion launch failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

int mlp_gradients(Ctx *c, const int32_t *idx) {
  MlpPlan &P = *static_cast<MlpPlan *>(c->mlp);
  DevState s = c->s;
  s.k = c->k;
  hipStream_t st = c->stream;
  const int L = P.L, M = P.M, B = P.B;
  const int64_t R = P.R;
  const bool per_worker = (P.rule == CADA_RULE_CADA2);
  const int64_t dw_stride = per_worker ? P.wb_total : 0;   // batch stride of the delta weights
  float *innov = P.innov;

  prof_mark(c);
  hipLaunchKernelGGL(k_rows, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, s, idx, P.grow);
  for (int l = 0; l < L; ++l) {
    PrepArgs pa;
    pa.s = s; pa.Wb = P.Wb; pa.Wl = P.Wl; pa.dWb = P.dWb; pa.offW = P.offW[l]; pa.wb_off = P.wb_off[l]; pa.wb_total = P.wb_total;
    pa.din = P.d[l]; pa.dout = P.d[l + 1]; pa.ldw = P.ldw[l]; pa.nW = P.nW;
    const int64_t n = (int64_t)pa.din * pa.dout;
    hipLaunchKernelGGL(k_prep_weights, dim3((unsigned)((n + 255) / 256), P.nW + 1), dim3(256), 0, st, pa);
  }

  // ---- forward.  All GEMMs are batched over the workers: rows [m*B, (m+1)*B).
  for (int l = 1; l <= L; ++l) {
    const int din = P.d[l - 1], dout = P.d[l];
    const bf16_t *W = P.Wb + P.wb_off[l - 1];
    const bf16_t *dW = P.dWb + P.wb_off[l - 1];
    GemmArgs g{};
    g.M = B; g.N = dout; g.ldc = dout; g.c_batch_stride = (int64_t)B * dout; g.sel = nullptr;
    // Z_l = A_{l-1} W_l with split operands: hi*hi + hi*lo + lo*hi
    const bf16_t *Wlo = P.Wl + P.wb_off[l - 1];
    g.npairs = 3; g.K[0] = g.K[1] = g.K[2] = din; g.C = P.Z[l - 1];
    const Operand ahi = (l == 1) ? op(P.Xb, P.ldx, 0, 1, P.grow, B) : op(P.A[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 1);
    const Operand alo = (l == 1) ? op(P.Xl, P.ldx, 0, 1, P.grow, B) : op(P.Al[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 1);
    g.A[0] = alo; g.B[0] = op(W, P.ldw[l - 1], 0, 0);          // small terms first
    g.A[1] = ahi; g.B[1] = op(Wlo, P.ldw[l - 1], 0, 0);
    g.A[2] = ahi; g.B[2] = op(W, P.ldw[l - 1], 0, 0);
    launch_gemm(c, g, M);
    // dZ_l = dA_{l-1} W_l + Aref_{l-1} dW_l   (layer 1: A_0 dW_1)
    g.C = P.dZ[l - 1];
    if (l == 1) {
      g.npairs = 1; g.K[0] = din;
      g.A[0] = op(P.Xb, P.ldx, 0, 1, P.grow, B);
      g.B[0] = op(dW, P.ldw[0], dw_stride, 0);
    } else {
      g.npairs = 2; g.K[0] = din; g.K[1] = din;
      g.A[0] = op(P.dA[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 1);
      g.B[0] = op(W, P.ldw[l - 1], 0, 0);
      g.A[1] = op(P.Aref[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 1);
      g.B[1] = op(dW, P.ldw[l - 1], dw_stride, 0);
    }
    launch_gemm(c, g, M);
    if (l < L) {
      FwdArgs fa;
      fa.s = s; fa.Z = P.Z[l - 1]; fa.dZ = P.dZ[l - 1]; fa.A = P.A[l]; fa.Al = P.Al[l]; fa.dA = P.dA[l]; fa.Aref = P.Aref[l];
      fa.offb = P.offb[l - 1]; fa.d = dout; fa.lda = P.lda[l];
      const int64_t n = R * dout;
      hipLaunchKernelGGL(k_hidden_fwd, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, fa);
    }
  }
  {
    LossArgs la;
    la.s = s; la.Z = P.Z[L - 1]; la.dZ = P.dZ[L - 1]; la.G = P.G[L - 1]; la.Gl = P.Gl[L - 1]; la.dG = P.dG[L - 1]; la.Gref = P.Gref[L - 1];
    la.grow = P.grow; la.offb = P.offb[L - 1]; la.C = P.d[L]; la.ldg = P.lda[L]; la.innov = innov;
    hipLaunchKernelGGL(k_loss, dim3(M), dim3(kBlock), 0, st, la);
  }

  // ---- backward
  const int64_t mp = (int64_t)s.M * s.p;
  for (int l = L; l >= 1; --l) {
    const int din = P.d[l - 1], dout = P.d[l];
    const bf16_t *W = P.Wb + P.wb_off[l - 1];
    const bf16_t *dW = P.dWb + P.wb_off[l - 1];
    const int64_t gstride = (int64_t)B * P.lda[l];
    // weight gradient of worker m: A_{l-1}[m]^T G_l[m] (split operands) -> fresh row of the gradient store
    GemmArgs g{};
    g.M = din; g.N = dout; g.ldc = dout; g.npairs = 3; g.K[0] = g.K[1] = g.K[2] = B;
    const Operand athi = (l == 1) ? op(P.Xb, P.ldx, 0, 0, P.grow, B) : op(P.A[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 0);
    const Operand atlo = (l == 1) ? op(P.Xl, P.ldx, 0, 0, P.grow, B) : op(P.Al[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 0);
    g.A[0] = atlo; g.B[0] = op(P.G[l - 1], P.lda[l], gstride, 0);
    g.A[1] = athi; g.B[1] = op(P.Gl[l - 1], P.lda[l], gstride, 0);
    g.A[2] = athi; g.B[2] = op(P.G[l - 1], P.lda[l], gstride, 0);
    g.C = s.gbuf + P.offW[l - 1]; g.c_batch_stride = s.p; g.sel = s.sel; g.c_sel_stride = mp;
    launch_gemm(c, g, M);
    // its innovation: A_{l-1}^T dG_l + dA_{l-1}^T Gref_l
    g.npairs = 1;
    g.A[0] = athi;
    g.B[0] = op(P.dG[l - 1], P.lda[l], gstride, 0);
    if (l > 1) {
      g.npairs = 2; g.K[1] = B;
      g.A[1] = op(P.dA[l - 1], P.lda[l - 1], (int64_t)B * P.lda[l - 1], 0);
      g.B[1] = op(P.Gref[l - 1], P.lda[l], gstride, 0);
    }
    if (P.rule == CADA_RULE_CADA1) { g.C = s.dtl + P.offW[l - 1]; g.sel = s.sel; g.c_sel_stride = mp; }
    else { g.C = innov + P.offW[l - 1]; g.sel = nullptr; g.c_sel_stride = 0; }
    launch_gemm(c, g, M);
    if (l > 1) {
      // gradient w.r.t. the activations of layer l-1 and its difference
      GemmArgs h{};
      h.M = B; h.N = din; h.ldc = din; h.c_batch_stride = (int64_t)B * din; h.sel = nullptr;
      const bf16_t *Wlo = P.Wl + P.wb_off[l - 1];
      h.npairs = 3; h.K[0] = h.K[1] = h.K[2] = dout; h.C = P.GA[l - 1];
      h.A[0] = op(P.Gl[l - 1], P.lda[l], gstride, 1); h.B[0] = op(W, P.ldw[l - 1], 0, 1);
      h.A[1] = op(P.G[l - 1], P.lda[l], gstride, 1);  h.B[1] = op(Wlo, P.ldw[l - 1], 0, 1);
      h.A[2] = op(P.G[l - 1], P.lda[l], gstride, 1);  h.B[2] = op(W, P.ldw[l - 1], 0, 1);
      launch_gemm(c, h, M);
      h.npairs = 2; h.K[1] = dout; h.C = P.dGA[l - 1];
      h.A[0] = op(P.dG[l - 1], P.lda[l], gstride, 1);
      h.B[0] = op(W, P.ldw[l - 1], 0, 1);
      h.A[1] = op(P.Gref[l - 1], P.lda[l], gstride, 1);
      h.B[1] = op(dW, P.ldw[l - 1], dw_stride, 1);
      launch_gemm(c, h, M);
      BwdArgs ba;
      ba.s = s; ba.GA = P.GA[l - 1]; ba.dGA = P.dGA[l - 1]; ba.A = P.A[l - 1]; ba.Aref = P.Aref[l - 1];
      ba.G = P.G[l - 2]; ba.Gl = P.Gl[l - 2]; ba.dG = P.dG[l - 2]; ba.Gref = P.Gref[l - 2];
      ba.offb = P.offb[l - 2]; ba.d = din; ba.lda = P.lda[l - 1]; ba.innov = innov;
      hipLaunchKernelGGL(k_hidden_bwd, dim3((unsigned)((din + 63) / 64), M), dim3(kBlock), 0, st, ba);
    }
  }
  prof_mark(c);
  hipLaunchKernelGGL(k_mlp_lhs, dim3(s.n_lhs_part, M), dim3(kBlock), 0, st, s, innov);
  prof_mark(c);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("MLP gradient launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  return CADA_OK;
}

}  // namespace cada
