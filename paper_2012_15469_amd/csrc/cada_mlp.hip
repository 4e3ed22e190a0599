// Dual minibatch gradient of a ReLU MLP with softmax cross-entropy for all workers, bf16
// MFMA contractions with float32 accumulation, and the left-hand side of the communication
// rule (Section 2.2, conditions (workerrule1)/(workerrule2); Algorithm 1, the two gradient
// evaluations on the same samples).
//
// The second gradient is never formed by itself.  With d = theta - theta_ref every quantity
// of the reference evaluation is carried as a difference to the evaluation at theta, and the
// differences are propagated exactly:
//   forward   dZ_1 = A_0 dW_1 + db_1,           dZ_l = dA_{l-1} W_l + Aref_{l-1} dW_l + db_l
//             A_l = relu(Z_l), Aref_l = relu(Z_l - dZ_l), dA_l = A_l - Aref_l
//   loss      G_L = (softmax(Z_L) - onehot)/B,  dG_L = (softmax(Z_L) - softmax(Z_L - dZ_L))/B
//   backward  grad W_l = A_{l-1}^T G_l,         innov W_l = A_{l-1}^T dG_l + dA_{l-1}^T Gref_l
//             GA_{l-1} = G_l W_l^T,             dGA_{l-1} = dG_l W_l^T + Gref_l dW_l^T
//             G_{l-1} = GA_{l-1} [Z>0],         Gref_{l-1} = (GA - dGA)_{l-1} [Zref>0]
// (Gref = G - dG).  Rounding W and W_ref to bf16 separately would bury their difference (one
// Adam step is about one bf16 ulp of a weight); rounding d itself keeps 8 significant bits
// of the difference.
//
// Precision.  The difference of two ReLU-network gradients at nearby points is dominated by
// the few units whose pre-activation changes sign between the two points, so the rule's
// left-hand side is only as good as the pre-activations Z_l are near zero: they must be
// resolved well below |dZ_l| ~ 1e-3 |Z_l|, which a single bf16 product (2^-9 per operand)
// cannot do.  Every contraction of the evaluation at theta (Z_l, grad W_l, GA_l) therefore
// uses split operands x = hi + lo (two bf16 values, 16 significant bits) and three MFMA
// products hi*hi + hi*lo + lo*hi accumulated in float32.  The backward ones need it because
// the server's update divides by sqrt(vhat): a coordinate whose gradient is smaller than its
// rounding error moves by a full alpha-sized step in a random direction, and with single
// bf16 products (0.2% gradient error) the iterate drifts from the fp64 trajectory by
// percents within tens of steps.  The difference contractions are single bf16 products.
//
// Every activation-side tensor (sampled rows, activations, back-propagated signals) exists in ONE
// orientation, (row, unit).  The weight-gradient contractions, which sum over the rows, read the
// same chunks and transpose on the way from LDS into the registers (ds_read_b64_tr_b16).
//
// One kernel, k_mm5, serves all three contraction shapes (forward, weight gradient,
// activation gradient).  For a 128 x 128 output tile of worker m it accumulates
//     C1 = Ah Bh^T + Ah Bl^T + Al Bh^T          (evaluation at theta, split operands)
//     C2 = Ad Bx^T + Ar Bd^T                    (difference to the reference evaluation)
// from up to four A-side and four B-side bf16 tensors, all stored in chunks of 128 rows x 32
// contraction indices, moved into LDS chunk by chunk, with v_mfma_f32_32x32x16_bf16 on four
// wavefronts of 64 x 64.  The epilogues apply bias/ReLU/masks, split results into hi/lo,
// write the tensors the later contractions need, reduce bias gradients
// and the squared norm of the innovation, so no float32 intermediate except the logits
// round-trips through HBM.  k_skinny computes the same products for outputs of at most 32
// columns (the last layer).
#include <cstdlib>
#include <new>

#include "cada_internal.h"

namespace cada {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint16_t bf16_t;   // storage type
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));   // four floats at any 4-byte aligned address
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes in flight (a native vector: stays in registers)
typedef uint32_t u32x2u __attribute__((ext_vector_type(2), aligned(4)));   // four bf16 values at any 4-byte aligned address

static inline int64_t P8(int64_t x) { return (x + 7) / 8 * 8; }

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int TILE = 128 * BK;                    // bf16 elements of one chunk (8 KB)
constexpr int kMaxSlots = 4;

// Operand layout.  Every bf16 tensor a contraction reads is stored in chunks of 128 rows x 32
// contraction indices, each chunk 8 KB of consecutive memory, the chunks of a 128-row tile one
// after the other: element (r, k) of a tensor with kt chunks per row tile lies at
//     ((r / 128) * kt + k / 32) * 4096 + (r % 128) * 32 + k % 32.
// A tile step of the contraction then reads whole 128-byte lines only.  With rows stored one
// after the other a step reads a 64-byte piece of each of 128 rows, and the vector L1, which
// works line by line, delivers those at half the rate (measured from L2: 27 against 51 B/clk
// per CU), which made the loads, not the MFMAs, the longest phase of a step.  Rows and indices
// beyond a tensor's extent, up to whole chunks, exist in memory and stay zero: nothing is
// clamped or masked on the way in.
__host__ __device__ __forceinline__ int64_t tm(int64_t r, int64_t k, int64_t kt) {
  return (((r >> 7) * kt + (k >> 5)) << 12) + ((r & 127) << 5) + (k & 31);
}
static inline int tiles128(int64_t x) { return (int)((x + 127) / 128); }
// chunks per 128-row tile of a tensor with x contraction indices: whole groups of four, so that a
// 128-unit tile of the weight-gradient contractions (which take units as output rows) finds all its
// four chunks; the padding stays zero
static inline int chunks32(int64_t x) { return 4 * (int)((x + 127) / 128); }

// In LDS a chunk keeps its 8 KB (row r at byte 64 r, no padding); the four 16-byte pieces of a row
// are stored in the order q ^ ((r >> 2) & 3).  A fragment read takes one piece of each of 32
// consecutive rows; rows 4 apart lie 256 bytes = one pass over the 64 banks apart, and with this
// order the same piece of 16 consecutive rows covers every bank once.
__device__ __forceinline__ int lds_piece(int piece) {   // piece = 4 row + q  ->  position (16-byte units)
  return piece ^ ((piece >> 4) & 3);
}

enum { EPI_FWD_HIDDEN = 0, EPI_STORE2 = 1, EPI_DW = 2, EPI_DA = 3, EPI_LOSS = 4 };

// LDS: a ring of 8 KB slots (one chunk each); behind it a buffer per multiplying wavefront for the
// way out: 32 rows x 64 floats for the weight gradients, 8 KB for the bf16 tensors of the forward
// and activation-gradient variants (the logits of the last layer are stored directly).  The pitch of
// 72 floats puts the two half-wavefronts of an accumulator store (rows 4 apart) into different
// halves of the banks.
constexpr int kDwPitch = 72;
constexpr int mm5_slots(int epi) { return epi == EPI_STORE2 ? 19 : 15; }
constexpr size_t mm5_lds_bytes(int epi) {
  return (size_t)mm5_slots(epi) * TILE * sizeof(bf16_t) +
         (epi == EPI_DW ? 4 * 32 * kDwPitch * sizeof(float) : epi == EPI_STORE2 ? 0 : 4 * 8192);
}

// Up to four tensors that share the row index of one side of the product.
struct Side {
  const bf16_t *ptr[kMaxSlots];
  int64_t kt[kMaxSlots];        // chunks per 128-row tile
  int64_t bstride[kMaxSlots];   // elements added per worker
  int n;
};

struct Mm5Args {
  DevState s;
  Side A, B;
  int a_h, a_l, a_d, a_r;       // role -> slot of A (-1: absent)
  int b_h, b_l, b_x, b_d;       // role -> slot of B
  int M, N, K;                  // extents of the tile index spaces and of the contraction
  int workers;
  const int32_t *rep;           // optional: the B side of worker m is read at worker rep[m]'s offset (shared reference points)
  int Bp;                       // padded rows per worker (multiple of 128)
  // EPI_FWD_HIDDEN / EPI_DA: bias offset, outputs
  int64_t offb;
  bf16_t *o_h, *o_l, *o_d, *o_r;        // (padded row, column), kto chunks per tile
  int64_t kto;
  uint64_t *maskbits;                   // ReLU mask bits [workers][row tiles][column tiles][256 lanes][2]: written by EPI_FWD_HIDDEN, read by EPI_DA
  float *dbpart, *ddbpart;              // EPI_DA: [M_workers][2 x row tiles][N], one partial sum per 64-row band
  // EPI_STORE2
  float *c1, *c2;                       // [Rp][N]
  // EPI_DW
  int64_t offW;
  int lhs_slot0;
  // EPI_LOSS (last layer's forward product with the loss in its epilogue; outputs o_h/o_l/o_d/o_r, bias at offb) and the
  // last layer's EPI_DW, which finishes that layer's bias gradient from the row blocks' sums
  const int64_t *grow;                  // global row of every padded minibatch row (its label)
  float *lastb;                         // [workers][nrb][32][2]: per block of 32 rows, sums over the rows of G and of dG
  int nrb;                              // blocks of 32 rows per worker
  int lhs_slot_b;                       // slot of the bias innovation's part of the left-hand side
};

__device__ __forceinline__ float delta_theta(const DevState &s, const RefPtr &ref, int64_t i) {
  return (s.theta[i] - ref.hi[i]) + (s.theta_lo[i] - ref.lo[i]);
}
__device__ __forceinline__ float *fresh_grad(const DevState &s, int m) {
  return s.gbuf + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.ps;
}
// (bf16 gradient store: the same row of gbuf16; exactly one of the two stores exists)
__device__ __forceinline__ uint16_t *fresh_grad16(const DevState &s, int m) {
  return s.gbuf16 + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.ps16;
}
// coordinate i of worker m's fresh gradient, into whichever store the context keeps
__device__ __forceinline__ void put_fresh_grad(const DevState &s, int m, int64_t i, float v) {
  if (s.gbuf16) fresh_grad16(s, m)[i] = f2bf(v);
  else fresh_grad(s, m)[i] = v;
}

// CADA1's stored innovations (bf16): the row this step writes and the row of the last upload.
__device__ __forceinline__ bf16_t *fresh_innov(const DevState &s, int m) {
  return s.dtl16 + ((int64_t)(1 - s.sel[m]) * s.M + m) * s.ps16;
}
__device__ __forceinline__ const bf16_t *stored_innov(const DevState &s, int m) {
  return s.dtl16 + ((int64_t)s.sel[m] * s.M + m) * s.ps16;
}

__device__ __forceinline__ u32x4 pack8(const bf16_t (&v)[8]) {
  u32x4 o;
  o.x = (uint32_t)v[0] | ((uint32_t)v[1] << 16); o.y = (uint32_t)v[2] | ((uint32_t)v[3] << 16);
  o.z = (uint32_t)v[4] | ((uint32_t)v[5] << 16); o.w = (uint32_t)v[6] | ((uint32_t)v[7] << 16);
  return o;
}

// NA, NB: tensors on the A and the B side (compile-time, so that the loads of a tile step are a
// fixed number of instructions and the waits can count them).  HAS_D: the product Ad Bx^T is present.
//
// A workgroup has eight wavefronts in two roles and works through several tiles.  Wavefronts 4-7
// move chunks from global memory straight into LDS (16-byte LDS-direct loads: no registers, no
// second pass through the LDS write port); wavefronts 0-3 read fragments, issue MFMAs and run the
// epilogue of each tile.  LDS is a ring of 8 KB slots, one chunk each, filled tensor by tensor in
// the order the tile steps read them, across tile boundaries: while the multipliers write one
// tile out, the first steps of the next are already landing.  One barrier per tile step: it
// tells the multipliers that the step has landed, and the movers that the slots of the step before
// are free (NS more loads may go out).  The epilogues use no workgroup barrier, so both roles
// execute the same number of them.  (With four wavefronts doing load, LDS write and multiply in
// turn, the three phases of a step, each near 1000 cycles, ran one after the other.)
//
// Weight gradient (EPI_DW): the product sums over a worker's rows, and both operands are (row, unit)
// tensors whose 128-row tiles hold the rows.  A tile step covers 32 rows; the operand of a side is the
// 32 rows x 128 units block of them, which lies in four chunks (one per 32 units) as 2 KB of
// consecutive memory each.  It is stored in its ring slot as [unit chunk][row][unit], and a fragment
// (8 consecutive rows of one unit per lane) is read with two transposing LDS loads.
typedef short i16x4 __attribute__((ext_vector_type(4)));

// Fragment of a transposed operand: 8 consecutive rows (k) of unit (lane % 32) from a [32 rows][32 units]
// block at `blk` (bf16), rows from `krow` on.  ds_read_b64_tr_b16 works on groups of 16 lanes: source lane s
// of a group passes the address of four consecutive units of row s / 4, and lane l receives, for
// e = 0..3, element l % 4 of source lane 4 e + l / 4: unit l of rows 0..3.  The four groups of a
// wavefront are (units 0-15 | 16-31) x (rows 0-7 | 8-15 of the half step, as the MFMA operand wants).
__device__ __forceinline__ bf16x8 tr_fragment(const bf16_t *blk, int lane_off) {
  const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(blk + lane_off));
  const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(blk + lane_off + 4 * 32));
  typedef short i16x8 __attribute__((ext_vector_type(8)));
  const i16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

template <int EPI, int NA, int NB, bool HAS_D>
__global__ __launch_bounds__(2 * kBlock, 1) void k_mm5(const Mm5Args g) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *lds = reinterpret_cast<bf16_t *>(smem_raw);
  constexpr int NS = NA + NB, NSLOT = mm5_slots(EPI);
  constexpr bool TR = EPI == EPI_DW;          // operands are (row, unit) tensors read across the rows
  static_assert(NSLOT >= 2 * NS, "the ring must hold two tile steps");
  const DevState &s = g.s;
  const bool mover = __builtin_amdgcn_readfirstlane((int)threadIdx.x) >= kBlock;   // uniform per wavefront
  const int t = threadIdx.x & (kBlock - 1), lane = t & 63, w = t >> 6;
  const int wy = w >> 1, wx = w & 1;
  // Tiles of this workgroup.  Workgroups are dealt to the 8 XCDs (each with an L2 of its own) in
  // turn; XCD x takes the x-th eighth of the tiles (columns fastest, then rows, then workers), its
  // workgroups every nbx-th of those: an XCD's L2 then sees whole workers, or a few row tiles of
  // one worker with all their column tiles, instead of every worker's operands.
  const int gx = (g.N + BN - 1) / BN, gy = (g.M + BM - 1) / BM;
  const int total = gx * gy * g.workers, per = (total + 7) / 8;
  const int nbx = gridDim.x >> 3;
  const int t_first = (blockIdx.x & 7) * per + (blockIdx.x >> 3), t_end = min(((int)(blockIdx.x & 7) + 1) * per, total);
  if (t_first >= t_end) return;
  const int nt = (t_end - t_first + nbx - 1) / nbx;
  const int nk = (g.K + BK - 1) / BK;
  const int nsteps = nt * nk;

  if (mover) {
    // Instruction c of wavefront w fills the 64 pieces from position 64 (2 w + c) on of a slot;
    // the lane at position P fetches the piece that the LDS order puts there.
    const int lw = __builtin_amdgcn_readfirstlane(w);
    int goff[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if constexpr (TR) goff[c] = (lw << 12) + (c << 9) + lane * 8;    // kilobyte 2 w + c of the step's operand: half c of unit chunk w
      else goff[c] = lds_piece((2 * lw + c) * 64 + lane) * 8;          // (the order is its own inverse)
    }
    // issue cursor: tile ordinal, step in the tile, first chunk of the tile's rows in every tensor, ring slot
    int ord = 0, h = 0, slot = 0;
    const bf16_t *pa[NA], *pb[NB];
    auto set_tile = [&](int o) __attribute__((always_inline)) {
      const int tix = t_first + o * nbx;
      const int bx = tix % gx, by = (tix / gx) % gy, bz = tix / (gx * gy);
      // (TR: the worker's first row tile, chunk 4 by / 4 bx of its units; else row tile by / bx, first chunk)
#pragma unroll
      for (int sl = 0; sl < NA; ++sl) pa[sl] = g.A.ptr[sl] + (int64_t)bz * g.A.bstride[sl] + (((int64_t)by * (TR ? 4 : g.A.kt[sl])) << 12);
      const int bzb = g.rep ? g.rep[bz] : bz;
#pragma unroll
      for (int sl = 0; sl < NB; ++sl) pb[sl] = g.B.ptr[sl] + (int64_t)bzb * g.B.bstride[sl] + (((int64_t)bx * (TR ? 4 : g.B.kt[sl])) << 12);
    };
    // next tile step; past the last one the cursor stays (those loads re-read the last chunk into slots nobody reads)
    auto next_step = [&]() __attribute__((always_inline)) {
      if (h + 1 < nk) ++h;
      else if (ord + 1 < nt) { ++ord; h = 0; set_tile(ord); }
    };
    auto load = [&](int sl) __attribute__((always_inline)) {
      const bf16_t *src = sl < NA ? pa[sl < NA ? sl : 0] : pb[sl < NA ? 0 : sl - NA];
      if constexpr (TR) {      // rows 32 h .. 32 h + 31 of the worker: row tile h / 4, 32 rows of 32 units from row 32 (h % 4) on
        const int64_t kt = sl < NA ? g.A.kt[sl < NA ? sl : 0] : g.B.kt[sl < NA ? 0 : sl - NA];
        src += (((int64_t)(h >> 2) * kt) << 12) + ((h & 3) << 10);
      } else {
        src += (int64_t)h << 12;
      }
      bf16_t *dst = lds + ((size_t)slot << 12) + (2 * lw << 9);
#pragma unroll
      for (int c = 0; c < 2; ++c)
        __builtin_amdgcn_global_load_lds(src + goff[c], (__attribute__((address_space(3))) void *)(dst + (c << 9)), 16, 0, 0);
      slot = slot + 1 == NSLOT ? 0 : slot + 1;
    };
    set_tile(0);
#pragma unroll
    for (int q = 0; q < NSLOT; ++q) {          // fill the ring
      if (q % NS == 0 && q > 0) next_step();
      load(q % NS);
    }
    // Barrier m: step m has landed when at most the NSLOT - 2 NS tensors issued after it are
    // outstanding (two instructions each); then the NS slots of step m - 1 are free.
    for (int m = 0; m < nsteps; ++m) {
      asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(2 * (NSLOT - 2 * NS)) : "memory");
      if (m > 0) {
#pragma unroll
        for (int i = 0; i < NS; ++i) {
          constexpr int r0 = NSLOT % NS;
          if ((r0 + i) % NS == 0) next_step();
          load((r0 + i) % NS);
        }
      }
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");     // nothing may land after the workgroup has gone
    return;
  }

  // fragment of this lane inside a 32-row band: row lane % 32, piece lane / 32 (+ 2 in the second half step)
  const int fro = lds_piece((lane & 31) * 4 + (lane >> 5)) * 8;
  // transposed operands: this lane's source address inside a [32 rows][32 units] block (see tr_fragment)
  const int fro_tr = (8 * (lane >> 5) + ((lane & 15) >> 2)) * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int sb = 0;                                  // ring slot of the current step's first tensor
  for (int ord = 0; ord < nt; ++ord) {
  const int tix = t_first + ord * nbx;
  const int bx = tix % gx, by = (tix / gx) % gy, wk = tix / (gx * gy);     // wk: worker
  const int m0 = by * BM, n0 = bx * BN;

  f32x16 acc1[2][2], acc2[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc1[i][j][r] = 0.f; acc2[i][j][r] = 0.f; }

  for (int h = 0; h < nk; ++h) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    auto slot_of = [&](int idx) __attribute__((always_inline)) { const int p = sb + idx; return lds + ((size_t)(p >= NSLOT ? p - NSLOT : p) << 12); };
    const bf16_t *tah = slot_of(g.a_h), *tal = slot_of(g.a_l), *tad = slot_of(HAS_D ? g.a_d : 0), *tar = slot_of(NA == 4 ? g.a_r : 0);
    const bf16_t *tbh = slot_of(NA + g.b_h), *tbl = slot_of(NA + g.b_l), *tbx = slot_of(NA + (HAS_D && NB == 4 ? g.b_x : 0)), *tbd = slot_of(NA + g.b_d);
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 ah[2], al[2], ad[2], ar[2], bh[2], bl[2], bx_[2], bd[2];
      // (TR: unit block 2 wy + i of the step's [4][32 rows][32 units], rows ks .. ks + 15)
      auto frag = [&](const bf16_t *slot, int half, int blk) __attribute__((always_inline)) -> bf16x8 {
        if constexpr (TR) return tr_fragment(slot + (half * 2 + blk) * 1024 + ks * 32, fro_tr);
        else return *reinterpret_cast<const bf16x8 *>(slot + (half * 64 + blk * 32) * BK + (fro ^ ks));
      };
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        ah[i] = frag(tah, wy, i);
        al[i] = frag(tal, wy, i);
        if constexpr (HAS_D) ad[i] = frag(tad, wy, i);
        // with fewer than four A tensors the reference operand is the hi part itself
        if constexpr (NA == 4) ar[i] = frag(tar, wy, i);
        else ar[i] = ah[i];
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        bh[j] = frag(tbh, wx, j);
        bl[j] = frag(tbl, wx, j);
        // with fewer than four B tensors the single-bf16 operand is the hi part itself
        if constexpr (HAS_D) {
          if constexpr (NB == 4) bx_[j] = frag(tbx, wx, j);
          else bx_[j] = bh[j];
        }
        bd[j] = frag(tbd, wx, j);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc1[i][j], 0, 0, 0);
          acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc1[i][j], 0, 0, 0);
          acc1[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc1[i][j], 0, 0, 0);
          if constexpr (HAS_D) acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad[i], bx_[j], acc2[i][j], 0, 0, 0);
          acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ar[i], bd[j], acc2[i][j], 0, 0, 0);
        }
    }
    sb = sb + NS >= NSLOT ? sb + NS - NSLOT : sb + NS;
  }

  // accumulator element (i, j, r) is output (row, col):
  //   row = m0 + wy*64 + i*32 + 8*(r>>2) + 4*(lane>>5) + (r&3),  col = n0 + wx*64 + j*32 + (lane&31)
  const int rbase = m0 + wy * 64 + 4 * (lane >> 5);
  const int cbase = n0 + wx * 64 + (lane & 31);
  const int64_t rp0 = (int64_t)wk * g.Bp;            // first padded row of this worker
  if constexpr (EPI == EPI_STORE2) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = cbase + j * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
          if (row < g.M && col < g.N) {
            g.c1[(rp0 + row) * g.N + col] = acc1[i][j][r];
            g.c2[(rp0 + row) * g.N + col] = acc2[i][j][r];
          }
        }
      }
  } else if constexpr (EPI == EPI_FWD_HIDDEN || EPI == EPI_DA) {
    // Forward: bias, ReLU of both evaluations.  Activation gradient: ReLU masks of the layer
    // below, bias-gradient partial sums.  Both: the result split into hi/lo, its difference and
    // its reference value, each written as a (row, column) tensor.
    // A lane's accumulators are one column and 16 rows of a 32 x 32 quarter: written from there
    // every store instruction would move 2 bytes per lane (some 300 instructions per wavefront and
    // tile; the CU's address unit then needs longer for them than the whole contraction took for
    // small K).  In the chunked layout a quarter is 2 KB of consecutive memory, so each wavefront puts
    // the quarter's values into an LDS buffer of its own in the layout of the destination and
    // copies it out 16 bytes per lane.  (LDS operations of one wavefront are carried out in
    // order, so the buffer needs no barrier.)
    bf16_t *sg = reinterpret_cast<bf16_t *>(smem_raw + (size_t)NSLOT * TILE * sizeof(bf16_t)) + w * 4096;   // 4 x 2 KB
    const int wr0 = m0 + wy * 64, wc0 = n0 + wx * 64;       // first row and column of this wavefront's 64 x 64 part
    bf16_t *const orow_t[4] = {g.o_h, g.o_l, g.o_d, g.o_r};
    auto copy_out = [&](bf16_t *const (&dst)[4], int64_t goff) __attribute__((always_inline)) {
      asm volatile("" ::: "memory");
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if (dst[b] != nullptr) {
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const int e8 = (hh * 64 + lane) * 8;
            *reinterpret_cast<u32x4 *>(dst[b] + goff + e8) = *reinterpret_cast<const u32x4 *>(sg + b * 1024 + e8);
          }
        }
      asm volatile("" ::: "memory");
    };

    // ReLU masks: one bit per accumulator element, set where the activation is positive (at theta,
    // at the reference point).  The forward contraction of a layer and the activation-gradient
    // contraction into it have the same tiles and the same element-to-lane map, so the forward
    // epilogue leaves each lane's 2 x 64 bits where the backward one finds them: 16 bytes per lane.
    uint64_t bit_on = 0, bit_ref = 0;
    uint64_t *mbits = g.maskbits + ((((int64_t)wk * gy + by) * gx + bx) * kBlock + t) * 2;
    if constexpr (EPI == EPI_DA) {
      const u32x4 mb = *reinterpret_cast<const u32x4 *>(mbits);
      bit_on = (uint64_t)mb.x | ((uint64_t)mb.y << 32);
      bit_ref = (uint64_t)mb.z | ((uint64_t)mb.w << 32);
    }

    // (both columns' biases are asked for before either is used: one memory latency, not two)
    float bias[2] = {0.f, 0.f}, dbias[2] = {0.f, 0.f};
    if constexpr (EPI == EPI_FWD_HIDDEN) {
      const RefPtr ref = theta_ref(s, wk, s.k);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = min(cbase + j * 32, g.N - 1);
        bias[j] = s.theta[g.offb + col];
        dbias[j] = delta_theta(s, ref, g.offb + col);
      }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = cbase + j * 32;
      const bool cok = col < g.N;
      const float b = bias[j], db = dbias[j];
      float sg_sum = 0.f, sd_sum = 0.f;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        // the quarter's four values per element, packed two rows to a register
        uint32_t ph[8], pl[8], pd[8], pr[8];
#pragma unroll
        for (int rp = 0; rp < 8; ++rp) {
          float x[2], xref[2];                      // value at theta, at the reference point; rows r, r + 1
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int r = 2 * rp + e;
            const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
            x[e] = 0.f; xref[e] = 0.f;
            if (cok && row < g.M) {
              if constexpr (EPI == EPI_FWD_HIDDEN) {
                const float z = acc1[i][j][r] + b, dz = acc2[i][j][r] + db;
                x[e] = fmaxf(z, 0.f); xref[e] = fmaxf(z - dz, 0.f);
              } else {
                const float ga = acc1[i][j][r], dga = acc2[i][j][r];
                x[e] = (bit_on >> ((i * 2 + j) * 16 + r)) & 1 ? ga : 0.f;
                xref[e] = (bit_ref >> ((i * 2 + j) * 16 + r)) & 1 ? (ga - dga) : 0.f;
              }
            }
            sg_sum += x[e]; sd_sum += x[e] - xref[e];
          }
          const uint32_t vh = f2bf_pk(x[0], x[1]), vr = f2bf_pk(xref[0], xref[1]);
          ph[rp] = vh; pr[rp] = vr;
          pl[rp] = f2bf_pk(x[0] - __uint_as_float(vh << 16), x[1] - __uint_as_float(vh & 0xffff0000u));
          pd[rp] = f2bf_pk(x[0] - xref[0], x[1] - xref[1]);
          if constexpr (EPI == EPI_FWD_HIDDEN) {      // (the sign of the stored, rounded value)
            const int sh = (i * 2 + j) * 16 + 2 * rp;
            bit_on |= (uint64_t)((__uint_as_float(vh << 16) > 0.f ? 1u : 0u) | (__uint_as_float(vh & 0xffff0000u) > 0.f ? 2u : 0u)) << sh;
            bit_ref |= (uint64_t)((__uint_as_float(vr << 16) > 0.f ? 1u : 0u) | (__uint_as_float(vr & 0xffff0000u) > 0.f ? 2u : 0u)) << sh;
          }
        }
        // (row, column) layout: element (rl, cl) of the quarter at 32 rl + cl
        if (g.o_h != nullptr && wc0 + j * 32 < (int)g.kto * 32) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int e = (8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * 32 + (lane & 31), sh = 16 * (r & 1);
            sg[e] = (bf16_t)(ph[r >> 1] >> sh); sg[1024 + e] = (bf16_t)(pl[r >> 1] >> sh);
            sg[2048 + e] = (bf16_t)(pd[r >> 1] >> sh); sg[3072 + e] = (bf16_t)(pr[r >> 1] >> sh);
          }
          copy_out(orow_t, tm(rp0 + wr0 + i * 32, wc0 + j * 32, g.kto));
        }
      }
      if constexpr (EPI == EPI_DA) {
        // the other half-wave holds the rows offset by 4: add it, then one value per column and
        // 64-row band (partial sum 2 by + wy of the column)
        sg_sum += __shfl_xor(sg_sum, 32, 64);
        sd_sum += __shfl_xor(sd_sum, 32, 64);
        if (lane < 32 && cok) {
          const int64_t o = ((int64_t)wk * (2 * gy) + 2 * by + wy) * g.N + col;
          g.dbpart[o] = sg_sum;
          g.ddbpart[o] = sd_sum;
        }
      }
    }
    if constexpr (EPI == EPI_FWD_HIDDEN) {
      u32x4 mb;
      mb.x = (uint32_t)bit_on; mb.y = (uint32_t)(bit_on >> 32); mb.z = (uint32_t)bit_ref; mb.w = (uint32_t)(bit_ref >> 32);
      *reinterpret_cast<u32x4 *>(mbits) = mb;
    }
  } else {   // EPI_DW
    // A lane's accumulators are one column and 16 rows of the tile: stored from there, an
    // instruction moves 4 bytes per lane, and the 192 such instructions of a wavefront kept the
    // CU's address unit busy for longer than the contraction took.  Each wavefront instead passes
    // its 64 x 64 part through an LDS buffer of its own, one 32-row band at a time, and writes it
    // out row by row, 16 bytes per lane, 256 bytes per row.  (LDS operations of one wavefront are
    // carried out in order, so the buffer needs no barrier.)
    constexpr int SP = kDwPitch;
    float *st = reinterpret_cast<float *>(smem_raw + (size_t)NSLOT * TILE * sizeof(bf16_t)) + w * (32 * SP);
    const bool g16 = s.gbuf16 != nullptr;
    float *gf = g16 ? nullptr : fresh_grad(s, wk) + g.offW;
    bf16_t *gf16 = g16 ? fresh_grad16(s, wk) + g.offW : nullptr;
    const bool cada1 = s.rule == CADA_RULE_CADA1;
    bf16_t *ivf = cada1 ? fresh_innov(s, wk) + g.offW : nullptr;
    const bf16_t *ivs = cada1 ? stored_innov(s, wk) + g.offW : nullptr;
    // row-wise pass: this lane has columns c4 .. c4+3 of the band's rows rr + 4 it, it = 0..7
    const int c4 = (lane & 15) * 4, rr = lane >> 4;
    const int colg = n0 + wx * 64 + c4;
    // every column of this wavefront's part exists: 16-byte accesses (4-byte aligned; with stored bf16
    // innovations or gradients their 8-byte accesses need an even offset and row length for that)
    const bool wide = n0 + wx * 64 + 64 <= g.N && (!(cada1 || g16) || ((g.offW | (int64_t)g.N) & 1) == 0);
    auto put_band = [&](const f32x16 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) st[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * SP + j * 32 + (lane & 31)] = acc[j][r];
      asm volatile("" ::: "memory");
    };
    // CADA1: the stored innovations of the part, all loads issued before anything waits for one
    // (rows clamped into the matrix so that no load sits under a branch).  Gradients and innovations
    // are written once and read once per step, megabytes apart in time: non-temporal accesses.
    u32x2u old[2][8];        // four bf16 values each
    if (cada1 && wide) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const int row = min(m0 + wy * 64 + i * 32 + rr + 4 * it, g.M - 1);
          old[i][it] = *reinterpret_cast<const u32x2u *>(ivs + (int64_t)row * g.N + colg);
        }
    }
    // The innovation first, the gradient last: the innovation's part waits for the loads of the stored
    // innovations (and a wait for a load also waits for every store issued before it), whereas nothing
    // in this tile waits behind the gradient's stores: they drain while the next tile's products run.
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rowb = m0 + wy * 64 + i * 32 + rr;
      if (!cada1) {       // nothing to store or to subtract: the squared norm needs no particular order of the elements
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = m0 + wy * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), col = n0 + wx * 64 + j * 32 + (lane & 31);
            const float v = (row < g.M && col < g.N) ? acc2[i][j][r] : 0.f;
            sq = fmaf(v, v, sq);
          }
        continue;
      }
      put_band(acc2[i]);
      if (wide) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          f32x4u v = *reinterpret_cast<const f32x4u *>(st + (rr + 4 * it) * SP + c4);
          if (rowb + 4 * it < g.M) {
            u32x2u nw;
            nw.x = f2bf_pk(v.x, v.y); nw.y = f2bf_pk(v.z, v.w);
            *reinterpret_cast<u32x2u *>(ivf + (int64_t)(rowb + 4 * it) * g.N + colg) = nw;
            const u32x2u o = old[i][it];
            v.x -= bf2f((bf16_t)o.x); v.y -= bf2f((bf16_t)(o.x >> 16)); v.z -= bf2f((bf16_t)o.y); v.w -= bf2f((bf16_t)(o.y >> 16));
            sq = fmaf(v.x, v.x, sq); sq = fmaf(v.y, v.y, sq); sq = fmaf(v.z, v.z, sq); sq = fmaf(v.w, v.w, sq);
          }
        }
      } else if (colg < g.N) {                 // a part that overhangs the matrix: element by element
        for (int it = 0; it < 8 && rowb + 4 * it < g.M; ++it)
          for (int e = 0; e < 4 && colg + e < g.N; ++e) {
            const int64_t o = (int64_t)(rowb + 4 * it) * g.N + colg + e;
            float iv = st[(rr + 4 * it) * SP + c4 + e];
            ivf[o] = f2bf(iv);
            iv -= bf2f(ivs[o]);
            sq = fmaf(iv, iv, sq);
          }
      }
      asm volatile("" ::: "memory");
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rowb = m0 + wy * 64 + i * 32 + rr;
      put_band(acc1[i]);
      if (wide) {
#pragma unroll
        for (int it = 0; it < 8; ++it) {
          const f32x4u v = *reinterpret_cast<const f32x4u *>(st + (rr + 4 * it) * SP + c4);
          if (rowb + 4 * it < g.M) {
            if (g16) {
              u32x2u nw;
              nw.x = f2bf_pk(v.x, v.y); nw.y = f2bf_pk(v.z, v.w);
              __builtin_nontemporal_store(nw, reinterpret_cast<u32x2u *>(gf16 + (int64_t)(rowb + 4 * it) * g.N + colg));
            } else {
              __builtin_nontemporal_store(v, reinterpret_cast<f32x4u *>(gf + (int64_t)(rowb + 4 * it) * g.N + colg));
            }
          }
        }
      } else if (colg < g.N) {
        for (int it = 0; it < 8 && rowb + 4 * it < g.M; ++it)
          for (int e = 0; e < 4 && colg + e < g.N; ++e) {
            const int64_t o = (int64_t)(rowb + 4 * it) * g.N + colg + e;
            const float v = st[(rr + 4 * it) * SP + c4 + e];
            if (g16) gf16[o] = f2bf(v); else gf[o] = v;
          }
      }
      asm volatile("" ::: "memory");
    }
    const float tot = wave_sum(sq);           // one partial sum of the left-hand side per wavefront and tile
    if (lane == 0) s.lhs_part[(int64_t)wk * s.n_lhs_part + g.lhs_slot0 + (by * gx + bx) * 4 + w] = tot;
  }
  }   // tiles
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // the movers' last barrier
}

__device__ __forceinline__ float group16_sum(float x) {
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// The same products for an output of at most 32 columns (the last layer: C <= 32 classes).  A
// 128 x 128 tile would leave nine tenths of its MFMAs and of its workgroups idle and the launch
// would run on a few CUs (32 tiles for the logits of 16 workers).  Here a workgroup computes
// 32 rows x 32 columns; its wavefronts (eight; fewer for the few steps of a weight gradient) split the
// tile steps (wavefront w takes steps w, w + nw, ...), read their fragments straight from the chunks in
// global memory (a fragment is 16 consecutive bytes of a chunk row) and add their partial accumulators up
// through LDS in a fixed order.  grid (ceil(M / 32), workers), 64 nw threads, 8 KB of dynamic LDS per
// wavefront (EPI_DW: 14 KB).
// EPI_STORE2: logits (evaluation); EPI_LOSS: the logits stay in the workgroup, whose epilogue is the loss (the signals
// the backward contractions read, and per-block sums for the bias gradient); EPI_DW: weight gradient, innovation, its
// squared norm (slot lhs_slot0 + row band), and (one more workgroup) the last layer's bias gradient from those sums.
// The weight gradient sums over the worker's rows: its operands are (row, unit) tensors, a step's part of
// one is a [32 rows][32 units] block (2 KB of consecutive memory), which the wavefront copies into an
// LDS area of its own and reads back transposed (tr_fragment).
template <int EPI, int NA, int NB, bool HAS_D>
__global__ __launch_bounds__(2 * kBlock) void k_skinny(const Mm5Args g) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  float *red = reinterpret_cast<float *>(smem_raw);                  // [8 wavefronts][2 accumulators][16][64]
  const DevState &s = g.s;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int nw = blockDim.x >> 6;          // wavefronts of this launch (1..8): fewer for short contractions, so that more workgroups fit a CU
  const int m0 = blockIdx.x * 32, wk = blockIdx.y;
  const int nk = (g.K + BK - 1) / BK;
  // this lane's fragment in a chunk: row lane % 32 of the band (A) or of the first 32 rows (B), piece lane / 32 (+ 2)
  const int64_t offa = (((int64_t)(m0 >> 7) * g.A.kt[0]) << 12) + (((m0 & 127) + (lane & 31)) << 5) + ((lane >> 5) << 3);
  const int64_t offb = ((lane & 31) << 5) + ((lane >> 5) << 3);
  if constexpr (EPI == EPI_DW) {
    // The last layer's launch has one workgroup more than tiles: it forms that layer's bias gradient, its innovation
    // and the innovation's part of the left-hand side from the sums that the forward launch left per block of 32 rows
    // (added up in the order of the rows).
    if (g.lastb != nullptr && (int)blockIdx.x == (g.M + 31) / 32) {
      if (w != 0) return;
      const bool cada1 = s.rule == CADA_RULE_CADA1;
      float sqb = 0.f;
      if (lane < g.N) {
        float gsum = 0.f, iv = 0.f;
        for (int rb = 0; rb < g.nrb; ++rb) {
          const float *q = g.lastb + ((((int64_t)wk * g.nrb + rb) * 32 + lane) << 1);
          gsum += q[0]; iv += q[1];
        }
        put_fresh_grad(s, wk, g.offb + lane, gsum);
        if (cada1) {
          fresh_innov(s, wk)[g.offb + lane] = f2bf(iv);
          iv -= bf2f(stored_innov(s, wk)[g.offb + lane]);
        }
        sqb = iv * iv;
      }
      const float totb = wave_sum(sqb);
      if (lane == 0) s.lhs_part[(int64_t)wk * s.n_lhs_part + g.lhs_slot_b] = totb;
      return;
    }
  }
  const bf16_t *pa[NA], *pb[NB];
  f32x16 acc1, acc2;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc1[r] = 0.f; acc2[r] = 0.f; }
  // EPI_LOSS: sixteen lanes share a row of the 32 x 32 result, each with two of the (at most 32) classes.  The
  // biases, their differences to the reference point and the row's label are asked for here, so that their
  // latency passes under the products.
  float bz[2] = {0.f, 0.f}, dbz[2] = {0.f, 0.f};
  int label = 0;
  if constexpr (EPI == EPI_LOSS) {
    const RefPtr ref = theta_ref(s, wk, s.k);
    const int c0 = 2 * (t & 15);
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (c0 + e < g.N) { bz[e] = s.theta[g.offb + c0 + e]; dbz[e] = delta_theta(s, ref, g.offb + c0 + e); }
    label = static_cast<const int32_t *>(s.y)[g.grow[(int64_t)wk * g.Bp + min(m0 + (t >> 4), g.M - 1)]];
  }
  if constexpr (EPI == EPI_DW) {
    // units m0 .. m0 + 31 of the A tensors are chunk m0 / 32 of every row tile, the (at most 32) output
    // columns chunk 0 of the B tensors; step kc covers the worker's rows 32 kc .. 32 kc + 31
#pragma unroll
    for (int sl = 0; sl < NA; ++sl) pa[sl] = g.A.ptr[sl] + (int64_t)wk * g.A.bstride[sl] + ((int64_t)(m0 >> 5) << 12);
#pragma unroll
    for (int sl = 0; sl < NB; ++sl) pb[sl] = g.B.ptr[sl] + (int64_t)wk * g.B.bstride[sl];
    bf16_t *area = reinterpret_cast<bf16_t *>(smem_raw) + w * (7 * 1024);       // room for seven blocks per wavefront
    const int fro_tr = (8 * (lane >> 5) + ((lane & 15) >> 2)) * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    for (int kc = w; kc < nk; kc += nw) {
      u32x4 v[NA + NB][2];
#pragma unroll
      for (int sl = 0; sl < NA + NB; ++sl) {
        const bf16_t *src = (sl < NA ? pa[sl < NA ? sl : 0] + (((int64_t)(kc >> 2) * g.A.kt[sl < NA ? sl : 0]) << 12)
                                     : pb[sl < NA ? 0 : sl - NA] + (((int64_t)(kc >> 2) * g.B.kt[sl < NA ? 0 : sl - NA]) << 12)) + ((kc & 3) << 10);
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) v[sl][hh] = *reinterpret_cast<const u32x4 *>(src + (hh * 64 + lane) * 8);
      }
#pragma unroll
      for (int sl = 0; sl < NA + NB; ++sl)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) *reinterpret_cast<u32x4 *>(area + sl * 1024 + (hh * 64 + lane) * 8) = v[sl][hh];
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // (one wavefront's LDS operations are carried out in order)
#pragma unroll
      for (int ks = 0; ks < BK; ks += 16) {
        auto fr = [&](int sl) __attribute__((always_inline)) { return tr_fragment(area + sl * 1024 + ks * 32, fro_tr); };
        // (roles as below: hi, lo, [difference] on the A side; hi, lo, [reference,] difference on the B side)
        const bf16x8 ah = fr(0), al = fr(1), bh = fr(NA), bl = fr(NA + 1), bd = fr(NA + NB - 1);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc1, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc1, 0, 0, 0);
        if constexpr (HAS_D) {
          const bf16x8 ad = fr(2), bx = NB == 4 ? fr(NA + 2) : bh;
          acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, bx, acc2, 0, 0, 0);
        }
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bd, acc2, 0, 0, 0);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the fragments are in registers before the area is written again
    }
    __syncthreads();                                         // the areas are done with: `red` lies over them
  } else {
#pragma unroll
  for (int sl = 0; sl < NA; ++sl) pa[sl] = g.A.ptr[sl] + (int64_t)wk * g.A.bstride[sl] + offa;
#pragma unroll
  for (int sl = 0; sl < NB; ++sl) pb[sl] = g.B.ptr[sl] + (int64_t)(g.rep ? g.rep[wk] : wk) * g.B.bstride[sl] + offb;
  for (int kc = w; kc < nk; kc += nw) {
    u32x4 fa[2][NA], fb[2][NB];          // (kept as integer vectors: arrays of them stay in registers)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int64_t o = ((int64_t)kc << 12) + half * 16;
#pragma unroll
      for (int sl = 0; sl < NA; ++sl) fa[half][sl] = *reinterpret_cast<const u32x4 *>(pa[sl] + o);
#pragma unroll
      for (int sl = 0; sl < NB; ++sl) fb[half][sl] = *reinterpret_cast<const u32x4 *>(pb[sl] + o);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // (the roles of the tensors follow from their number: hi, lo, [difference, [reference]] on the A
      // side, hi, lo, [reference,] difference on the B side; the host checks it)
      auto fr = [&](const u32x4 &v) __attribute__((always_inline)) { return __builtin_bit_cast(bf16x8, v); };
      const bf16x8 ah = fr(fa[half][0]), al = fr(fa[half][1]), bh = fr(fb[half][0]), bl = fr(fb[half][1]), bd = fr(fb[half][NB - 1]);
      const bf16x8 ar = NA == 4 ? fr(fa[half][NA - 1]) : ah;
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc1, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc1, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc1, 0, 0, 0);
      if constexpr (HAS_D) {
        const bf16x8 ad = fr(fa[half][2]), bx = NB == 4 ? fr(fb[half][2]) : bh;
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, bx, acc2, 0, 0, 0);
      }
      acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ar, bd, acc2, 0, 0, 0);
    }
  }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    red[((w * 2 + 0) * 16 + r) * 64 + lane] = acc1[r];
    red[((w * 2 + 1) * 16 + r) * 64 + lane] = acc2[r];
  }
  __syncthreads();
  if constexpr (EPI == EPI_LOSS) {
    // softmax cross-entropy on the tile's rows: G = (P - onehot)/B, dG = (P - Pref)/B.  With e_i = exp(-dz_i) and
    // T = sum_j P_j e_j the reference probabilities are Pref_i = P_i e_i / T, so
    //     P_i - Pref_i = P_i (S - expm1(-dz_i)) / (1 + S),  S = sum_j P_j expm1(-dz_j) = T - 1,
    // which keeps the digits of a small difference (no subtraction of nearly equal probabilities) and
    // is used while every |dz_j| of the row is below 1/2.  For larger differences (a reference point
    // many iterations old) 1 + S cancels instead (T can be far below float32's resolution of 1), so
    // there P_i - Pref_i is formed directly with Pref = softmax(z - dz), the exponents shifted by their
    // maximum; the difference is then no longer small against its operands.
    // Also the sums over the tile's rows of G and dG: the last layer's bias gradient and its innovation, which the
    // weight-gradient launch of that layer adds up over the row blocks.
    __shared__ float part[8][16][4];
    const int rl = t >> 4, cp = t & 15, c0 = 2 * cp;
    const bool on[2] = {c0 < g.N, c0 + 1 < g.N};
    const int row = m0 + rl;
    const bool live = row < g.M;                    // (rows past the minibatch are padding)
    // accumulator element (r, lane) is (row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32) of the tile
    const int ra = 4 * (rl >> 3) + (rl & 3), lb = 32 * ((rl >> 2) & 1);
    const float invB = 1.0f / (float)s.B;
    float z[2], x[2], ndz[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      float zs = 0.f, ds = 0.f;
      for (int ww = 0; ww < nw; ++ww) {
        zs += red[((ww * 2 + 0) * 16 + ra) * 64 + lb + c0 + e];
        ds += red[((ww * 2 + 1) * 16 + ra) * 64 + lb + c0 + e];
      }
      z[e] = on[e] ? zs + bz[e] : -INFINITY;
      ndz[e] = on[e] ? -(ds + dbz[e]) : 0.f;
      x[e] = expm1f(ndz[e]);
    }
    const float zr[2] = {z[0] + ndz[0], z[1] + ndz[1]};       // logits at the reference point (-inf for an absent class)
    float nabs = fmaxf(fabsf(ndz[0]), fabsf(ndz[1]));        // (an absent class contributes 0)
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) nabs = fmaxf(nabs, __shfl_xor(nabs, o, 64));
    const bool far = !(nabs < 0.5f);             // (also taken by a NaN, which then shows in the result)
    float zmax = fmaxf(z[0], z[1]);
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) zmax = fmaxf(zmax, __shfl_xor(zmax, o, 64));
#pragma unroll
    for (int e = 0; e < 2; ++e) z[e] = on[e] ? expf(z[e] - zmax) : 0.f;
    const float den = group16_sum(z[0] + z[1]);
    z[0] = z[0] / den; z[1] = z[1] / den;
    const float S = group16_sum(fmaf(z[0], x[0], z[1] * x[1]));
    // the direct form: Pref = softmax of the reference logits z - dz, shifted by their maximum
    float rmax = fmaxf(zr[0], zr[1]);
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) rmax = fmaxf(rmax, __shfl_xor(rmax, o, 64));
    const float er[2] = {on[0] ? expf(zr[0] - rmax) : 0.f, on[1] ? expf(zr[1] - rmax) : 0.f};
    const float rden = group16_sum(er[0] + er[1]);
    // (row, class) tensors: a row's classes are consecutive, written two at a time (an absent odd
    // class is a zero in the padding)
    uint32_t ph = 0, pl = 0, pd = 0, pr = 0;
    float sumG[2] = {0.f, 0.f}, sumD[2] = {0.f, 0.f};
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      if (on[e] && live) {
        const int c = c0 + e;
        const float gl = (z[e] - (c == label ? 1.f : 0.f)) * invB;
        const float dg = (far ? z[e] - er[e] / rden : z[e] * (S - x[e]) / (1.0f + S)) * invB;
        const bf16_t hi = f2bf(gl), lo = f2bf(gl - bf2f(hi)), bd = f2bf(dg), br = f2bf(gl - dg);
        ph |= (uint32_t)hi << (16 * e); pl |= (uint32_t)lo << (16 * e); pd |= (uint32_t)bd << (16 * e); pr |= (uint32_t)br << (16 * e);
        sumG[e] = gl;
        sumD[e] = dg;
      }
    }
    if (on[0] && live) {
      const int64_t o = tm((int64_t)wk * g.Bp + row, 0, g.kto) + c0;          // classes 0..31 lie in the row's first chunk
      *reinterpret_cast<uint32_t *>(g.o_h + o) = ph; *reinterpret_cast<uint32_t *>(g.o_l + o) = pl;
      *reinterpret_cast<uint32_t *>(g.o_d + o) = pd;
      if (g.o_r) *reinterpret_cast<uint32_t *>(g.o_r + o) = pr;
    }
    // sums over the tile's rows in a fixed order: the wavefront's four rows, then the wavefronts
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      sumG[e] += __shfl_xor(sumG[e], 16, 64); sumG[e] += __shfl_xor(sumG[e], 32, 64);
      sumD[e] += __shfl_xor(sumD[e], 16, 64); sumD[e] += __shfl_xor(sumD[e], 32, 64);
    }
    if (lane < 16) { part[w][cp][0] = sumG[0]; part[w][cp][1] = sumG[1]; part[w][cp][2] = sumD[0]; part[w][cp][3] = sumD[1]; }
    __syncthreads();
    if (w == 0 && lane < g.N) {
      const int c = lane;
      float gsum = 0.f, iv = 0.f;
      for (int ww = 0; ww < nw; ++ww) { gsum += part[ww][c >> 1][c & 1]; iv += part[ww][c >> 1][2 + (c & 1)]; }
      float *q = g.lastb + ((((int64_t)wk * g.nrb + blockIdx.x) * 32 + c) << 1);
      q[0] = gsum; q[1] = iv;
    }
    return;
  }
  // 2 x 16 x 64 values over the threads, each the sum of the wavefronts' partial results in wavefront order
  float *gf = nullptr;
  bf16_t *gf16 = nullptr;
  bf16_t *ivf = nullptr;
  const bf16_t *ivs = nullptr;
  const bool cada1 = s.rule == CADA_RULE_CADA1;
  if constexpr (EPI == EPI_DW) {
    if (s.gbuf16) gf16 = fresh_grad16(s, wk) + g.offW;
    else gf = fresh_grad(s, wk) + g.offW;
    if (cada1) {
      ivf = fresh_innov(s, wk) + g.offW;
      ivs = stored_innov(s, wk) + g.offW;
    }
  }
  float sq = 0.f;
  for (int e = t; e < 2 * 16 * 64; e += (int)blockDim.x) {       // (accumulator, r, lane)
    const int a = e >> 10, r = (e >> 6) & 15, ln = e & 63;
    float v = 0.f;
    for (int ww = 0; ww < nw; ++ww) v += red[((ww * 2 + a) * 16 + r) * 64 + ln];
    const int row = m0 + 8 * (r >> 2) + 4 * (ln >> 5) + (r & 3), col = ln & 31;
    if (row < g.M && col < g.N) {
      if constexpr (EPI == EPI_STORE2) {
        const int64_t o = ((int64_t)wk * g.Bp + row) * g.N + col;
        if (a == 0) g.c1[o] = v; else g.c2[o] = v;
      } else {
        const int64_t o = (int64_t)row * g.N + col;
        if (a == 0) {
          if (gf16) gf16[o] = f2bf(v); else gf[o] = v;
        } else {
          if (cada1) { ivf[o] = f2bf(v); v -= bf2f(ivs[o]); }
          sq = fmaf(v, v, sq);
        }
      }
    }
  }
  if constexpr (EPI == EPI_DW) {
    const float ws = wave_sum(sq);
    __syncthreads();
    if (lane == 0) red[w] = ws;
    __syncthreads();
    if (t == 0) {
      float tot = 0.f;
      for (int ww = 0; ww < nw; ++ww) tot += red[ww];
      s.lhs_part[(int64_t)wk * s.n_lhs_part + g.lhs_slot0 + blockIdx.x] = tot;
    }
  }
}

// ------------------------------------------------------------------------------------------
// plan
// ------------------------------------------------------------------------------------------
struct MlpPlan {
  int L, M, B, Bp, rule, RT;
  int64_t Rp;                     // M * Bp padded rows per step (Bp a multiple of 128: a worker's rows start a tile)
  int64_t total_rows;             // rows of X
  int64_t max_rows_per_worker;
  int d[CADA_MAX_LAYERS + 1];
  int64_t offW[CADA_MAX_LAYERS], offb[CADA_MAX_LAYERS];   // offsets into theta, index l-1
  int64_t kta[CADA_MAX_LAYERS + 1];                       // chunks32(d_l): chunks per tile of (row, d_l) tensors
  int64_t wt_off[CADA_MAX_LAYERS], wt_total;              // W_l^T (d_l, d_{l-1}), index l-1
  int64_t wn_off[CADA_MAX_LAYERS], wn_total;              // W_l   (d_{l-1}, d_l), l >= 2
  int lhs_w_slot[CADA_MAX_LAYERS], lhs_b_slot[CADA_MAX_LAYERS];
  int nW;                                                 // delta-weight copies: 1 (CADA1) or M (CADA2)
  bf16_t *Xh, *Xl; int64_t ldx;                           // all features, rows one after the other [total_rows][ldx]
  bf16_t *XGh, *XGl;                                      // gathered minibatch, (padded row, feature)
  int64_t *grow;
  bf16_t *WTh, *WTl, *dWT, *WNh, *WNl, *dWN;
  bf16_t *Ah[CADA_MAX_LAYERS], *Al[CADA_MAX_LAYERS], *dA[CADA_MAX_LAYERS], *Aref[CADA_MAX_LAYERS];   // hidden l, (row, unit)
  bf16_t *Gh[CADA_MAX_LAYERS + 1], *Gl[CADA_MAX_LAYERS + 1], *dG[CADA_MAX_LAYERS + 1], *Gref[CADA_MAX_LAYERS + 1];       // layer l >= 1, (row, unit)
  float *ZL, *dZL;                                        // logits [Rp][C]
  uint64_t *maskbits[CADA_MAX_LAYERS];                    // hidden l: ReLU mask bits per tile and lane
  int32_t *rep;                                           // CADA2: first worker with the same reference point [M]
  float *dbpart, *ddbpart;                                // [M][2 RT][max hidden width]
  float *lastb;                                           // [M][Bp / 32][32][2]: last layer, sums of G and dG per block of 32 rows
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

// elements of a chunked tensor of r rows and k contraction indices (whole chunks)
size_t tm_elems(int64_t r, int64_t k) { return (size_t)tiles128(r) * chunks32(k) * TILE; }

void layout(MlpPlan &P, const cada_config *cfg, int64_t total_rows, Carve &w) {
  P.L = cfg->n_layers; P.M = cfg->M; P.B = cfg->B; P.rule = cfg->rule;
  P.RT = tiles128(cfg->B);
  P.Bp = P.RT * 128;
  P.Rp = (int64_t)cfg->M * P.Bp;
  P.total_rows = total_rows;
  P.max_rows_per_worker = 0;
  for (int m = 0; m < cfg->M; ++m)
    if (cfg->n_samples[m] > P.max_rows_per_worker) P.max_rows_per_worker = cfg->n_samples[m];
  for (int l = 0; l <= P.L; ++l) { P.d[l] = cfg->layer_dims[l]; P.kta[l] = chunks32(P.d[l]); }
  int64_t o = 0, wt = 0, wn = 0;
  int slot = 0, maxh = 1;
  for (int l = 1; l <= P.L; ++l) {
    P.offW[l - 1] = o; o += (int64_t)P.d[l - 1] * P.d[l];
    P.offb[l - 1] = o; o += P.d[l];
    P.wt_off[l - 1] = wt; wt += (int64_t)tm_elems(P.d[l], P.d[l - 1]);
    P.wn_off[l - 1] = wn; if (l >= 2) wn += (int64_t)tm_elems(P.d[l - 1], P.d[l]);
    P.lhs_w_slot[l - 1] = slot; slot += 4 * tiles128(P.d[l - 1]) * tiles128(P.d[l]);
    P.lhs_b_slot[l - 1] = slot; slot += (P.d[l] + 255) / 256;
    if (l < P.L && P.d[l] > maxh) maxh = P.d[l];
  }
  P.wt_total = wt; P.wn_total = wn;
  P.nW = (cfg->rule == CADA_RULE_CADA2) ? cfg->M : 1;
  P.ldx = P8(P.d[0]);
  const size_t Rp = (size_t)P.Rp;
  P.Xh = w.take<bf16_t>((size_t)total_rows * P.ldx);
  P.Xl = w.take<bf16_t>((size_t)total_rows * P.ldx);
  P.XGh = w.take<bf16_t>(tm_elems(Rp, P.d[0]));
  P.XGl = w.take<bf16_t>(tm_elems(Rp, P.d[0]));
  P.grow = w.take<int64_t>(Rp);
  P.rep = w.take<int32_t>((size_t)cfg->M);
  P.WTh = w.take<bf16_t>((size_t)wt); P.WTl = w.take<bf16_t>((size_t)wt); P.dWT = w.take<bf16_t>((size_t)wt * P.nW);
  P.WNh = w.take<bf16_t>((size_t)wn + 8); P.WNl = w.take<bf16_t>((size_t)wn + 8); P.dWN = w.take<bf16_t>((size_t)wn * P.nW + 8);
  for (int l = 1; l < P.L; ++l) {
    const size_t n = tm_elems(Rp, P.d[l]);
    P.Ah[l] = w.take<bf16_t>(n); P.Al[l] = w.take<bf16_t>(n); P.dA[l] = w.take<bf16_t>(n); P.Aref[l] = w.take<bf16_t>(n);
    P.maskbits[l] = w.take<uint64_t>((size_t)cfg->M * P.RT * tiles128(P.d[l]) * kBlock * 2);
  }
  for (int l = 1; l <= P.L; ++l) {
    const size_t n = tm_elems(Rp, P.d[l]);
    P.Gh[l] = w.take<bf16_t>(n); P.Gl[l] = w.take<bf16_t>(n); P.dG[l] = w.take<bf16_t>(n);
    P.Gref[l] = l >= 2 ? w.take<bf16_t>(n) : nullptr;       // (the first layer has no propagated difference to pair it with)
  }
  P.ZL = w.take<float>(Rp * P.d[P.L]);
  P.dZL = w.take<float>(Rp * P.d[P.L]);
  P.dbpart = w.take<float>((size_t)cfg->M * 2 * P.RT * maxh);
  P.ddbpart = w.take<float>((size_t)cfg->M * 2 * P.RT * maxh);
  P.lastb = w.take<float>((size_t)cfg->M * (P.Bp / 32) * 32 * 2);
}
}  // namespace

// Number of partial sums of the left-hand side per worker (one per weight-gradient tile and
// per 256 biases).
int mlp_lhs_slots(const cada_config *cfg) {
  int slot = 0;
  for (int l = 1; l <= cfg->n_layers; ++l)
    slot += 4 * tiles128(cfg->layer_dims[l - 1]) * tiles128(cfg->layer_dims[l]) + (cfg->layer_dims[l] + 255) / 256;
  return slot;
}

size_t mlp_workspace_bytes(const cada_config *cfg, const int64_t total_rows) {
  if (cfg->gemm_dtype != CADA_GEMM_BF16) { set_error("the MLP model computes its contractions in bf16 (gemm_dtype must be CADA_GEMM_BF16)"); return 0; }
  if (cfg->layer_dims[cfg->n_layers] > 32) { set_error("at most 32 classes"); return 0; }
  for (int l = 0; l <= cfg->n_layers; ++l)    // the kernels index one worker's activations with 32 bits
    if (((int64_t)cfg->B + 128) * (cfg->layer_dims[l] + 32) >= (1ll << 31)) { set_error("B x layer width must stay below 2^31"); return 0; }
  {   // the staging launch numbers its 64 x 64 tiles of the minibatch and of every weight copy in one grid dimension
    const int64_t nz = (cfg->rule == CADA_RULE_CADA2) ? cfg->M + 1 : 2;
    int64_t nblk = ((int64_t)cfg->layer_dims[0] + 71) / 64 * ((cfg->B + 63) / 64) * cfg->M;
    for (int l = 1; l <= cfg->n_layers; ++l)
      nblk += ((int64_t)cfg->layer_dims[l] + 63) / 64 * ((cfg->layer_dims[l - 1] + 63) / 64) * nz;
    if (nblk >= (1ll << 31)) { set_error("too many operand tiles for one launch (M x layer sizes / 4096 must stay below 2^31)"); return 0; }
  }
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
  c->n_phases = 3;
  c->phase_names[0] = "mlp_gradients"; c->phase_names[1] = "rule"; c->phase_names[2] = "server_update";
  return CADA_OK;
}

void mlp_free(Ctx *c) {
  delete static_cast<MlpPlan *>(c->mlp);
  c->mlp = nullptr;
}

// ------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------
// float32 features -> bf16 hi/lo copies with padded leading dimension (once, at init)
__global__ void k_x_to_bf16(const float *X, bf16_t *Xh, bf16_t *Xl, int64_t rows, int d0, int64_t ldx) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * ldx) return;
  const int64_t r = i / ldx; const int c = (int)(i % ldx);
  const float x = c < d0 ? X[r * d0 + c] : 0.f;
  const bf16_t hi = f2bf(x);
  Xh[i] = hi;
  Xl[i] = f2bf(x - bf2f(hi));
}

// Per-step staging of the contractions' operands, one launch: the chunked copy of the gathered
// minibatch, and bf16 copies (in both orientations) of every layer's weights and of their
// differences to the reference points.  The blocks of the launch are numbered through the parts
// (minibatch tiles first, then the layers in order); the parts are independent of each other.
struct PrepLayer {
  bf16_t *WTh, *WTl, *dWT, *WNh, *WNl, *dWN;   // already offset to this layer
  int64_t offW;
  int din, dout;
  int64_t ktt, ktn;      // chunks32(din), chunks32(dout)
  int want_n;            // also write the [in][out] orientation (layers >= 2)
  int gx, gy;            // 64 x 64 tiles over (dout, din)
};

struct StageArgs {
  DevState s;
  // minibatch: XG(m*Bp + b, c) = X[grow[m*Bp + b]][c]
  const bf16_t *Xh, *Xl; int64_t ldx;
  const int32_t *idx;    // [M][B] sampled rows, local to each worker's shard
  int64_t *grow;         // out: grow[m*Bp + b] = global row of worker m's b-th sample (b < B)
  bf16_t *XGh, *XGl;
  int d0, B, Bp; int64_t ktx;
  int gx, gy;            // 64 x 64 tiles over (ldx, B)
  // weights
  PrepLayer layer[CADA_MAX_LAYERS];
  int n_layers, nz;      // nz = 1 + number of workers with a difference of their own
  int64_t wt_total, wn_total;
  // CADA2 only, else null: workers whose last upload happened at the same iteration share their
  // reference point theta^{k - tau}, hence the difference theta - theta_ref and its bf16 copies;
  // out: rep[m] = the first worker with worker m's (clamped) tau.  Only that worker's difference is computed.
  int32_t *rep;
  uint32_t first[CADA_MAX_LAYERS + 2];   // first block of the minibatch part (0), of each layer, and the total
};

// A 64 x 64 tile of the minibatch, moved 16 bytes (8 values) per lane: the sampled rows of X's bf16
// copies go to XG as they are.
__device__ __forceinline__ void stage_minibatch(const StageArgs &a, int bx, int by, int m) {
  const int c0 = bx * 64, b0 = by * 64;
  const int t = threadIdx.x;
  const int cg = (t & 7) * 8;                   // this thread's 8 columns
  const int64_t row0 = a.s.row_off[m], n_m = a.s.row_off[m + 1] - row0;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = (t >> 3) + 32 * pass, b = b0 + r, c = c0 + cg;
    if (b < a.B && c < a.ldx) {                 // (columns from d0 to ldx hold zeros in X's copies)
      int64_t row = a.idx[(int64_t)m * a.B + b];
      if (row < 0 || row >= n_m) {              // reported once per sample, by the tile that also records the row
        if (bx == 0 && cg == 0) atomicOr(a.s.err, 1u);
        row = row < 0 ? 0 : n_m - 1;
      }
      row += row0;
      if (bx == 0 && cg == 0) a.grow[(int64_t)m * a.Bp + b] = row;
      const int64_t src = row * a.ldx + c;
      const u32x4 vh = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.Xh + src));      // (a sampled row is not read again soon)
      const u32x4 vl = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.Xl + src));
      const int64_t dst = tm((int64_t)m * a.Bp + b, c, a.ktx);
      *reinterpret_cast<u32x4 *>(a.XGh + dst) = vh;
      *reinterpret_cast<u32x4 *>(a.XGl + dst) = vl;
    }
  }
}

// A 64 x 64 tile of one layer's weights (z = 0: hi and lo parts of W) or of their difference to
// worker z - 1's reference point, 8 values per lane: rows of W are read (4-byte aligned 16-byte
// loads) and written as they are, and turned through LDS for the other orientation.
__device__ __forceinline__ void stage_weights(const StageArgs &a, const PrepLayer &p, unsigned char *sm, int bx, int by, int z, bool first_tile) {
  const DevState &s = a.s;
  typedef float tile_t[64][65];
  tile_t &tile = *reinterpret_cast<tile_t *>(sm);
  const int o0 = bx * 64, i0 = by * 64;
  const int t = threadIdx.x;
  const bool is_w = z == 0;
  const int m = is_w ? 0 : z - 1;
  if (!is_w && a.rep) {
    const int tau_m = min(s.tau[m], s.D);
    int r = m;                                        // (every wavefront finds it for itself)
    for (int j0 = 0; j0 < m && r == m; j0 += kWave) {
      const int j = j0 + (t & 63);
      const unsigned long long same = __ballot(j < m && min(s.tau[j], s.D) == tau_m);
      if (same) r = j0 + __ffsll(same) - 1;
    }
    if (first_tile && t == 0) a.rep[m] = r;
    if (r != m) return;                               // another worker with the same reference point stands for this one
  }
  const RefPtr ref = theta_ref(s, m, s.k);
  const int og = (t & 7) * 8;
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = (t >> 3) + 32 * pass, i = i0 + r, o = o0 + og;
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (i < p.din && o < p.dout) {
      const int64_t src = p.offW + (int64_t)i * p.dout + o;
      if (o + 8 <= p.dout) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          f32x4u x = *reinterpret_cast<const f32x4u *>(s.theta + src + 4 * q);
          if (!is_w) {
            const f32x4u xl = *reinterpret_cast<const f32x4u *>(s.theta_lo + src + 4 * q);
            const f32x4u rh = *reinterpret_cast<const f32x4u *>(ref.hi + src + 4 * q);
            const f32x4u rl = *reinterpret_cast<const f32x4u *>(ref.lo + src + 4 * q);
            x = (x - rh) + (xl - rl);             // the same expression as delta_theta
          }
          v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
        }
      } else {
        for (int e = 0; e < 8 && o + e < p.dout; ++e) v[e] = is_w ? s.theta[src + e] : delta_theta(s, ref, src + e);
      }
      if (p.want_n) {                             // (values past dout are zeros, like the padding they land in)
        const int64_t dn = tm(i, o, p.ktn);
        bf16_t h8[8], l8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { h8[e] = f2bf(v[e]); l8[e] = f2bf(v[e] - bf2f(h8[e])); }
        if (is_w) { *reinterpret_cast<u32x4 *>(p.WNh + dn) = pack8(h8); *reinterpret_cast<u32x4 *>(p.WNl + dn) = pack8(l8); }
        else *reinterpret_cast<u32x4 *>(p.dWN + (int64_t)m * a.wn_total + dn) = pack8(h8);
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[r][og + e] = v[e];
  }
  __syncthreads();
  const int oo = t & 63;
  if (o0 + oo < p.dout) {
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int ig = ((t >> 6) + 4 * pass) * 8;
      if (i0 + ig < p.din) {                      // (rows past din are zeros in the tile)
        bf16_t h8[8], l8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float x = tile[ig + e][oo]; h8[e] = f2bf(x); l8[e] = f2bf(x - bf2f(h8[e])); }
        const int64_t dt = tm(o0 + oo, i0 + ig, p.ktt);
        if (is_w) { *reinterpret_cast<u32x4 *>(p.WTh + dt) = pack8(h8); *reinterpret_cast<u32x4 *>(p.WTl + dt) = pack8(l8); }
        else *reinterpret_cast<u32x4 *>(p.dWT + (int64_t)m * a.wt_total + dt) = pack8(h8);
      }
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_stage(const StageArgs a) {
  __shared__ __align__(16) unsigned char sm[64 * 65 * sizeof(float)];     // a weight tile on its way to the other orientation
  const uint32_t blk = blockIdx.x;
  if (blk < a.first[1]) {
    const uint32_t per = (uint32_t)a.gx * a.gy;
    const uint32_t m = blk / per, r = blk - m * per;
    stage_minibatch(a, (int)(r % a.gx), (int)(r / a.gx), (int)m);
    return;
  }
  int l = 0;
  while (blk >= a.first[l + 2]) ++l;             // (blk < first[n_layers + 1], the grid's size)
  const PrepLayer &p = a.layer[l];
  const uint32_t rel = blk - a.first[l + 1];
  const uint32_t per = (uint32_t)p.gx * p.gy;
  const uint32_t z = rel / per, r = rel - z * per;
  stage_weights(a, p, sm, (int)(r % p.gx), (int)(r / p.gx), (int)z, l == 0 && r == 0);
}

// Hidden-layer bias gradient and its innovation from the per-tile partial sums of k_mm5<EPI_DA>.
// grid (ceil(d/256), M)
__global__ __launch_bounds__(kBlock) void k_bias_finish(const DevState s, const float *dbpart, const float *ddbpart, int RT, int d,
                                                        int64_t offb, int lhs_slot) {
  __shared__ float red[4];
  const int m = blockIdx.y;
  const int c = blockIdx.x * kBlock + threadIdx.x;
  float sq = 0.f;
  if (c < d) {
    float gsum = 0.f, dsum = 0.f;
    for (int rt = 0; rt < RT; ++rt) {
      gsum += dbpart[((int64_t)m * RT + rt) * d + c];
      dsum += ddbpart[((int64_t)m * RT + rt) * d + c];
    }
    put_fresh_grad(s, m, offb + c, gsum);
    if (s.rule == CADA_RULE_CADA1) {
      fresh_innov(s, m)[offb + c] = f2bf(dsum);
      dsum -= bf2f(stored_innov(s, m)[offb + c]);
    }
    sq = dsum * dsum;
  }
  const float tot = block_sum(sq, red);
  if (threadIdx.x == 0) s.lhs_part[(int64_t)m * s.n_lhs_part + lhs_slot + blockIdx.x] = tot;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
namespace {

void side_add(Side &sd, const bf16_t *p, int64_t kt, int64_t bstride) {
  sd.ptr[sd.n] = p; sd.kt[sd.n] = kt; sd.bstride[sd.n] = bstride; sd.n += 1;
}

// The (tensor count, product set) combinations the layers use.
template <int EPI, int NA, int NB, bool HAS_D> hipError_t mm5_allow_lds() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(k_mm5<EPI, NA, NB, HAS_D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)mm5_lds_bytes(EPI));
}
template <int EPI, int NA, int NB, bool HAS_D> int launch_mm5_as(Ctx *c, const Mm5Args &g) {
  // one workgroup per CU at most (8 XCDs x 32 CUs), each XCD's tiles dealt over its workgroups
  const int total = ((g.N + BN - 1) / BN) * ((g.M + BM - 1) / BM) * g.workers, per = (total + 7) / 8;
  const dim3 grid(8 * (per < 32 ? per : 32));
  hipLaunchKernelGGL((k_mm5<EPI, NA, NB, HAS_D>), grid, dim3(2 * kBlock), mm5_lds_bytes(EPI), c->stream, g);
  return CADA_OK;
}
// first layer: two A tensors (hi, lo) and no propagated difference on the A side; deeper layers: all of them
// per wavefront: its partial results (8 KB); weight gradient: the seven blocks it stages (14 KB), over which the partial results are laid later
constexpr int skinny_lds_bytes(int epi, int nw = 8) { return nw * (epi == EPI_DW ? 7 * 1024 * (int)sizeof(bf16_t) : 8192); }
// Wavefronts of a launch: one per two tile steps, eight at most.  A weight gradient sums over a worker's few rows (4-8
// steps); with eight wavefronts half of them would idle while their LDS kept other workgroups off the CU.
static int skinny_waves(int epi, int K) {
  const int nk = (K + BK - 1) / BK;
  if (epi != EPI_DW) return 8;
  return nk >= 16 ? 8 : nk >= 2 ? nk / 2 : 1;
}
template <int EPI, int NA, int NB, bool HAS_D> hipError_t skinny_allow_lds() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(k_skinny<EPI, NA, NB, HAS_D>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             skinny_lds_bytes(EPI));
}
template <int EPI, int NA, int NB, bool HAS_D> int launch_skinny_as(Ctx *c, const Mm5Args &g) {
  const int nw = skinny_waves(EPI, g.K);
  const unsigned extra = (EPI == EPI_DW && g.lastb != nullptr) ? 1u : 0u;      // (the workgroup that finishes the last layer's bias gradient)
  hipLaunchKernelGGL((k_skinny<EPI, NA, NB, HAS_D>), dim3((unsigned)((g.M + 31) / 32) + extra, g.workers), dim3(64 * nw), skinny_lds_bytes(EPI, nw), c->stream, g);
  return CADA_OK;
}
// Returns CADA_OK after enqueueing the launch, CADA_EUNSUPPORTED (and launches nothing) when the
// operands do not fit a compiled variant.
template <int EPI> int launch_mm5(Ctx *c, Mm5Args &g, int workers) {
  g.workers = workers;
  const bool has_d = g.a_d >= 0;
  if constexpr (EPI == EPI_STORE2 || EPI == EPI_DW || EPI == EPI_LOSS) {
    if (g.N <= 32) {            // at most 32 output columns (the last layer)
      for (int i = 1; i < g.A.n; ++i)
        if (g.A.kt[i] != g.A.kt[0]) { set_error("internal: A tensors with different chunk counts"); return CADA_EUNSUPPORTED; }
      if (g.a_h != 0 || g.a_l != 1 || (has_d && g.a_d != 2) || g.a_r != (g.A.n == 4 ? 3 : 0) || g.b_h != 0 || g.b_l != 1 ||
          (has_d && g.b_x != (g.B.n == 4 ? 2 : 0)) || g.b_d != g.B.n - 1) {
        set_error("internal: unexpected tensor roles");
        return CADA_EUNSUPPORTED;
      }
      if (EPI == EPI_DW) {
        if (!has_d && g.A.n == 2 && g.B.n == 3) return launch_skinny_as<EPI, 2, 3, false>(c, g);
        if (has_d && g.A.n == 3 && g.B.n == 4) return launch_skinny_as<EPI, 3, 4, true>(c, g);
      } else {
        if (!has_d && g.A.n == 2 && g.B.n == 3) return launch_skinny_as<EPI, 2, 3, false>(c, g);
        if (has_d && g.A.n == 4 && g.B.n == 3) return launch_skinny_as<EPI, 4, 3, true>(c, g);
      }
    }
  }
  if constexpr (EPI == EPI_LOSS) {
    set_error("internal: the loss epilogue serves at most 32 classes");
    return CADA_EUNSUPPORTED;
  } else {
  // every tensor must hold the chunks the tile steps walk through: the contraction indices along a row
  // tile, or (weight gradient: units are output rows, the steps walk down the worker's rows) whole
  // 128-unit tiles and the worker's padded rows
  const int64_t needA = EPI == EPI_DW ? 4 * ((g.M + BM - 1) / BM) : (g.K + BK - 1) / BK;
  const int64_t needB = EPI == EPI_DW ? 4 * ((g.N + BN - 1) / BN) : (g.K + BK - 1) / BK;
  for (int i = 0; i < g.A.n; ++i)
    if (g.A.kt[i] < needA) { set_error("internal: A tensor with fewer chunks than the tiles walk through"); return CADA_EUNSUPPORTED; }
  for (int i = 0; i < g.B.n; ++i)
    if (g.B.kt[i] < needB) { set_error("internal: B tensor with fewer chunks than the tiles walk through"); return CADA_EUNSUPPORTED; }
  if (EPI == EPI_DW && (int64_t)((g.K + BK - 1) / BK) * BK > g.Bp) { set_error("internal: more rows than a worker's padded tile"); return CADA_EUNSUPPORTED; }
  if constexpr (EPI == EPI_DW) {
    if (!has_d && g.A.n == 2 && g.B.n == 3) return launch_mm5_as<EPI, 2, 3, false>(c, g);
    if (has_d && g.A.n == 3 && g.B.n == 4) return launch_mm5_as<EPI, 3, 4, true>(c, g);
  } else if constexpr (EPI == EPI_DA) {
    if (has_d && g.A.n == 4 && g.B.n == 3) return launch_mm5_as<EPI, 4, 3, true>(c, g);
  } else {
    if (!has_d && g.A.n == 2 && g.B.n == 3) return launch_mm5_as<EPI, 2, 3, false>(c, g);
    if (has_d && g.A.n == 4 && g.B.n == 3) return launch_mm5_as<EPI, 4, 3, true>(c, g);
  }
  set_error("internal: no MFMA kernel variant for %d + %d tensors", g.A.n, g.B.n);
  return CADA_EUNSUPPORTED;
  }
}

Mm5Args blank(const DevState &s, const MlpPlan &P) {
  Mm5Args g{};
  g.s = s; g.Bp = P.Bp;
  g.a_h = g.a_l = g.a_d = g.a_r = -1;
  g.b_h = g.b_l = g.b_x = g.b_d = -1;
  return g;
}

}  // namespace

// One-time work at init: the bf16 copies of the features and the kernels' LDS allowance.
int mlp_init_state(Ctx *c, const float *) {
  MlpPlan &P = *static_cast<MlpPlan *>(c->mlp);
  hipError_t e = hipSuccess;
  e = mm5_allow_lds<EPI_FWD_HIDDEN, 2, 3, false>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_FWD_HIDDEN, 4, 3, true>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_STORE2, 2, 3, false>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_STORE2, 4, 3, true>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_DW, 2, 3, false>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_DW, 3, 4, true>();
  if (e == hipSuccess) e = mm5_allow_lds<EPI_DA, 4, 3, true>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_STORE2, 2, 3, false>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_STORE2, 4, 3, true>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_LOSS, 2, 3, false>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_LOSS, 4, 3, true>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_DW, 2, 3, false>();
  if (e == hipSuccess) e = skinny_allow_lds<EPI_DW, 3, 4, true>();
  if (e != hipSuccess) { set_error("hipFuncSetAttribute(LDS size) failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  const int64_t n = P.total_rows * P.ldx;
  hipLaunchKernelGGL(k_x_to_bf16, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->s.X, P.Xh, P.Xl, P.total_rows, P.d[0], P.ldx);
  e = hipGetLastError();
  if (e != hipSuccess) { set_error("feature conversion launch failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

// Gathers the minibatch rows, prepares the bf16 weights and runs the forward contractions:
// leaves the activations of every layer and the logits (without bias) of the last one.
// with_loss: the last layer's launch also evaluates the loss (training step); else it leaves the logits (evaluation).
static int mlp_forward(Ctx *c, MlpPlan &P, const DevState &s, const int32_t *idx, bool with_loss) {
  hipStream_t st = c->stream;
  const int L = P.L, M = P.M, B = P.B, Bp = P.Bp;
  const bool per_worker = (P.rule == CADA_RULE_CADA2);
  const int64_t dwt_stride = per_worker ? P.wt_total : 0;
  int32_t *rep = per_worker ? P.rep : nullptr;
  {
    StageArgs sa;
    sa.s = s;
    sa.Xh = P.Xh; sa.Xl = P.Xl; sa.ldx = P.ldx; sa.idx = idx; sa.grow = P.grow;
    sa.XGh = P.XGh; sa.XGl = P.XGl;
    sa.d0 = P.d[0]; sa.B = B; sa.Bp = Bp; sa.ktx = P.kta[0];
    sa.gx = (int)((P.ldx + 63) / 64); sa.gy = (B + 63) / 64;
    sa.n_layers = L; sa.nz = P.nW + 1; sa.wt_total = P.wt_total; sa.wn_total = P.wn_total; sa.rep = rep;
    uint64_t nblk = (uint64_t)sa.gx * sa.gy * M;
    sa.first[0] = 0;
    for (int l = 1; l <= L; ++l) {
      PrepLayer &pl = sa.layer[l - 1];
      pl.WTh = P.WTh + P.wt_off[l - 1]; pl.WTl = P.WTl + P.wt_off[l - 1]; pl.dWT = P.dWT + P.wt_off[l - 1];
      pl.WNh = P.WNh + P.wn_off[l - 1]; pl.WNl = P.WNl + P.wn_off[l - 1]; pl.dWN = P.dWN + P.wn_off[l - 1];
      pl.offW = P.offW[l - 1];
      pl.din = P.d[l - 1]; pl.dout = P.d[l]; pl.ktt = P.kta[l - 1]; pl.ktn = P.kta[l]; pl.want_n = l >= 2;
      pl.gx = (pl.dout + 63) / 64; pl.gy = (pl.din + 63) / 64;
      sa.first[l] = (uint32_t)nblk;
      nblk += (uint64_t)pl.gx * pl.gy * sa.nz;
    }
    sa.first[L + 1] = (uint32_t)nblk;
    for (int l = L + 2; l < CADA_MAX_LAYERS + 2; ++l) sa.first[l] = (uint32_t)nblk;
    hipLaunchKernelGGL(k_stage, dim3((unsigned)nblk), dim3(kBlock), 0, st, sa);
  }

  // ---- forward: worker m owns padded rows [m*Bp, m*Bp + B)
  for (int l = 1; l <= L; ++l) {
    const int din = P.d[l - 1], dout = P.d[l];
    Mm5Args g = blank(s, P);
    g.M = B; g.N = dout; g.K = din;
    if (l == 1) {
      const int64_t bs0 = (int64_t)Bp * P.kta[0] * 32;     // a worker's Bp / 128 row tiles
      side_add(g.A, P.XGh, P.kta[0], bs0); side_add(g.A, P.XGl, P.kta[0], bs0);
      g.a_h = 0; g.a_l = 1; g.a_r = 0;                    // dZ_1 = A_0 dW_1
    } else {
      const int64_t bs = (int64_t)Bp * P.kta[l - 1] * 32;
      side_add(g.A, P.Ah[l - 1], P.kta[l - 1], bs); side_add(g.A, P.Al[l - 1], P.kta[l - 1], bs);
      side_add(g.A, P.dA[l - 1], P.kta[l - 1], bs); side_add(g.A, P.Aref[l - 1], P.kta[l - 1], bs);
      g.a_h = 0; g.a_l = 1; g.a_d = 2; g.a_r = 3;         // dZ_l = dA W + Aref dW
    }
    const int64_t ktt = P.kta[l - 1];
    side_add(g.B, P.WTh + P.wt_off[l - 1], ktt, 0); side_add(g.B, P.WTl + P.wt_off[l - 1], ktt, 0);
    side_add(g.B, P.dWT + P.wt_off[l - 1], ktt, dwt_stride);
    g.b_h = 0; g.b_l = 1; g.b_x = 0; g.b_d = 2;
    g.rep = rep;
    if (l < L) {
      g.offb = P.offb[l - 1]; g.kto = P.kta[l];
      g.o_h = P.Ah[l]; g.o_l = P.Al[l]; g.o_d = P.dA[l]; g.o_r = P.Aref[l];
      g.maskbits = P.maskbits[l];
      if (const int rc = launch_mm5<EPI_FWD_HIDDEN>(c, g, M)) return rc;
    } else if (with_loss) {
      g.offb = P.offb[L - 1]; g.kto = P.kta[L];
      g.o_h = P.Gh[L]; g.o_l = P.Gl[L]; g.o_d = P.dG[L]; g.o_r = P.Gref[L];     // (Gref: null for a single-layer network)
      g.grow = P.grow; g.lastb = P.lastb; g.nrb = Bp / 32;
      if (const int rc = launch_mm5<EPI_LOSS>(c, g, M)) return rc;
    } else {
      g.c1 = P.ZL; g.c2 = P.dZL;
      if (const int rc = launch_mm5<EPI_STORE2>(c, g, M)) return rc;
    }
  }
  return CADA_OK;
}

int mlp_gradients(Ctx *c, const int32_t *idx) {
  MlpPlan &P = *static_cast<MlpPlan *>(c->mlp);
  DevState s = c->s;
  s.k = c->k;
  hipStream_t st = c->stream;
  const int L = P.L, M = P.M, B = P.B, Bp = P.Bp;
  const bool per_worker = (P.rule == CADA_RULE_CADA2);
  const int64_t dwn_stride = per_worker ? P.wn_total : 0;

  prof_mark(c);
  if (const int rc = mlp_forward(c, P, s, idx, true)) return rc;

  // ---- backward
  for (int l = L; l >= 1; --l) {
    const int din = P.d[l - 1], dout = P.d[l];
    {   // weight gradient and its innovation: contraction over the worker's rows, both operands (row, unit) tensors
      Mm5Args g = blank(s, P);
      g.M = din; g.N = dout; g.K = B;
      const int64_t bsA = (int64_t)Bp * P.kta[l - 1] * 32, bsB = (int64_t)Bp * P.kta[l] * 32;     // a worker's Bp / 128 row tiles
      if (l == 1) {
        side_add(g.A, P.XGh, P.kta[0], bsA); side_add(g.A, P.XGl, P.kta[0], bsA);
        g.a_h = 0; g.a_l = 1; g.a_r = 0;
      } else {
        side_add(g.A, P.Ah[l - 1], P.kta[l - 1], bsA); side_add(g.A, P.Al[l - 1], P.kta[l - 1], bsA); side_add(g.A, P.dA[l - 1], P.kta[l - 1], bsA);
        g.a_h = 0; g.a_l = 1; g.a_d = 2; g.a_r = 0;       // innov = A^T dG + dA^T Gref
      }
      side_add(g.B, P.Gh[l], P.kta[l], bsB); side_add(g.B, P.Gl[l], P.kta[l], bsB);
      if (l == 1) {     // no dA^T Gref term in the first layer
        side_add(g.B, P.dG[l], P.kta[l], bsB);
        g.b_h = 0; g.b_l = 1; g.b_d = 2;
      } else {
        side_add(g.B, P.Gref[l], P.kta[l], bsB); side_add(g.B, P.dG[l], P.kta[l], bsB);
        g.b_h = 0; g.b_l = 1; g.b_x = 2; g.b_d = 3;
      }
      g.offW = P.offW[l - 1]; g.lhs_slot0 = P.lhs_w_slot[l - 1];
      if (l == L) {     // the last layer's launch also finishes its bias gradient from the forward launch's row-block sums
        g.lastb = P.lastb; g.nrb = Bp / 32; g.offb = P.offb[L - 1]; g.lhs_slot_b = P.lhs_b_slot[L - 1];
      }
      if (const int rc = launch_mm5<EPI_DW>(c, g, M)) return rc;
    }
    if (l >= 2) {   // gradient w.r.t. the activations of layer l-1, masks, bias partials
      Mm5Args g = blank(s, P);
      g.M = B; g.N = din; g.K = dout;
      const int64_t bs = (int64_t)Bp * P.kta[l] * 32;
      side_add(g.A, P.Gh[l], P.kta[l], bs); side_add(g.A, P.Gl[l], P.kta[l], bs);
      side_add(g.A, P.dG[l], P.kta[l], bs); side_add(g.A, P.Gref[l], P.kta[l], bs);
      g.a_h = 0; g.a_l = 1; g.a_d = 2; g.a_r = 3;         // dGA = dG W^T + Gref dW^T
      const int64_t ktn = P.kta[l];
      side_add(g.B, P.WNh + P.wn_off[l - 1], ktn, 0); side_add(g.B, P.WNl + P.wn_off[l - 1], ktn, 0);
      side_add(g.B, P.dWN + P.wn_off[l - 1], ktn, dwn_stride);
      g.b_h = 0; g.b_l = 1; g.b_x = 0; g.b_d = 2;
      g.rep = per_worker ? P.rep : nullptr;
      const int q = l - 1;
      g.offb = P.offb[q - 1]; g.kto = P.kta[q];
      g.o_h = P.Gh[q]; g.o_l = P.Gl[q]; g.o_d = P.dG[q]; g.o_r = P.Gref[q];     // (Gref: null for q = 1)
      g.maskbits = P.maskbits[q];
      g.dbpart = P.dbpart; g.ddbpart = P.ddbpart;
      if (const int rc = launch_mm5<EPI_DA>(c, g, M)) return rc;
      hipLaunchKernelGGL(k_bias_finish, dim3((din + 255) / 256, M), dim3(kBlock), 0, st, s, P.dbpart, P.ddbpart, 2 * P.RT, din,
                         P.offb[q - 1], P.lhs_b_slot[q - 1]);
    }
  }
  prof_mark(c);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("MLP gradient launch failed: %s", hipGetErrorString(e));
    return CADA_EHIP;
  }
  return CADA_OK;
}


// ------------------------------------------------------------------------------------------
// Evaluation on all the data (not part of an iteration).
// idx[m][b] = min(chunk*B + b, N_m - 1): the rows of one evaluation chunk (the tail repeats the
// last row; those copies are not counted)
__global__ void k_eval_idx(const DevState s, int32_t *idx, int chunk) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)s.M * s.B) return;
  const int m = (int)(i / s.B), b = (int)(i % s.B);
  const int64_t n = s.row_off[m + 1] - s.row_off[m];
  const int64_t r = (int64_t)chunk * s.B + b;
  idx[i] = (int32_t)(r < n ? r : n - 1);
}

// Softmax cross-entropy and top-1 hits of the chunk's valid rows, added to acc[m] (sums, not yet
// means).  One block per worker, so consecutive chunks add in a fixed order.
__global__ __launch_bounds__(kBlock) void k_eval_chunk(const DevState s, const float *Z, const int64_t *grow, int64_t offb, int C, int Bp,
                                                      int chunk, double *acc) {
  constexpr int MAXC = 32;
  __shared__ double red[kBlock][2];
  const int m = blockIdx.x;
  const int64_t n = s.row_off[m + 1] - s.row_off[m];
  const int64_t left = n - (int64_t)chunk * s.B;
  const int valid = (int)(left < 0 ? 0 : (left > s.B ? s.B : left));
  const int32_t *yv = static_cast<const int32_t *>(s.y);
  double loss = 0.0, hits = 0.0;
  for (int b = threadIdx.x; b < valid; b += kBlock) {
    const int64_t r = (int64_t)m * Bp + b;
    const int label = yv[grow[r]];
    float zmax = -INFINITY, zl = 0.f;
    int arg = 0;
    float z[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
      if (c < C) {
        z[c] = Z[r * C + c] + s.theta[offb + c];
        if (z[c] > zmax) { zmax = z[c]; arg = c; }
        if (c == label) zl = z[c];
      }
    float den = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) if (c < C) den += expf(z[c] - zmax);
    loss += (double)(zmax + logf(den) - zl);
    hits += arg == label ? 1.0 : 0.0;
  }
  red[threadIdx.x][0] = loss; red[threadIdx.x][1] = hits;
  __syncthreads();
  for (int o = kBlock / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { red[threadIdx.x][0] += red[threadIdx.x + o][0]; red[threadIdx.x][1] += red[threadIdx.x + o][1]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { acc[2 * m] += red[0][0]; acc[2 * m + 1] += red[0][1]; }
}

__global__ void k_eval_means(const DevState s, double *acc) {
  const int m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m >= s.M) return;
  const double n = (double)(s.row_off[m + 1] - s.row_off[m]);
  acc[2 * m] /= n;
  acc[2 * m + 1] /= n;
}

int mlp_eval(Ctx *c, double *out) {
  MlpPlan &P = *static_cast<MlpPlan *>(c->mlp);
  DevState s = c->s;
  s.k = c->k;
  hipStream_t st = c->stream;
  if (P.d[P.L] > 32) { set_error("evaluation supports at most 32 classes"); return CADA_EINVAL; }
  hipError_t e = hipMemsetAsync(c->eval_acc, 0, (size_t)P.M * 2 * sizeof(double), st);
  if (e != hipSuccess) { set_error("hipMemsetAsync failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  const int64_t nmax = P.max_rows_per_worker;
  const int chunks = (int)((nmax + P.B - 1) / P.B);
  const unsigned nb = (unsigned)(((int64_t)P.M * P.B + 255) / 256);
  for (int ch = 0; ch < chunks; ++ch) {
    hipLaunchKernelGGL(k_eval_idx, dim3(nb), dim3(256), 0, st, s, c->eval_idx, ch);
    if (const int rc = mlp_forward(c, P, s, c->eval_idx, false)) return rc;
    hipLaunchKernelGGL(k_eval_chunk, dim3((unsigned)P.M), dim3(kBlock), 0, st, s, P.ZL, P.grow, P.offb[P.L - 1], P.d[P.L], P.Bp, ch, c->eval_acc);
  }
  hipLaunchKernelGGL(k_eval_means, dim3((unsigned)((P.M + 63) / 64)), dim3(64), 0, st, s, c->eval_acc);
  eval_finish(c, out, 0);
  e = hipGetLastError();
  if (e != hipSuccess) { set_error("evaluation launch failed: %s", hipGetErrorString(e)); return CADA_EHIP; }
  return CADA_OK;
}

}  // namespace cada
