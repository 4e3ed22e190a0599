// Device-side generator of the counter-based synthetic rows ("counter_gauss" recipe):
// every feature is a pure function of (seed, worker, sample, column) through
// Philox4x32-10 (Salmon et al., SC'11), so the 107 GB dataset of the high-dimensional
// logistic workload is produced directly in HBM and any row can be regenerated on a CPU.
// This is input generation only; it shares nothing with libcada.
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

namespace {

constexpr uint32_t kM0 = 0xD2511F53u, kM1 = 0xCD9E8D57u, kW0 = 0x9E3779B9u, kW1 = 0xBB67AE85u;
constexpr uint32_t kKey1 = 0x43414441u;

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += kW0; k1 += kW1; }
    const uint32_t hi0 = __umulhi(kM0, c.x), lo0 = kM0 * c.x;
    const uint32_t hi1 = __umulhi(kM1, c.z), lo1 = kM1 * c.z;
    U4 n;
    n.x = hi1 ^ c.y ^ k0; n.y = lo1; n.z = hi0 ^ c.w ^ k1; n.w = lo0;
    c = n;
  }
  return c;
}

__device__ __forceinline__ int32_t irwin_hall(uint32_t a, uint32_t b) {
  return (int32_t)((a & 0xFFFFu) + (a >> 16) + (b & 0xFFFFu) + (b >> 16)) - 131070;
}

__global__ void k_teacher(uint32_t seed, int64_t p, int32_t *t) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= p) return;
  const U4 o = philox4x32_10(U4{(uint32_t)j, 0u, 0u, 1u}, seed, kKey1);
  t[j] = (int32_t)(o.x % 255u) - 127;
}

// grid = rows to fill; block = 256 threads, each producing 4 columns per iteration.
__global__ __launch_bounds__(256) void k_rows(uint32_t seed, int64_t N_m, int64_t p, int64_t row_begin, float scale,
                                              const float *__restrict__ shift, const int32_t *__restrict__ tdir,
                                              float *__restrict__ X, float *__restrict__ y) {
  const int64_t row = row_begin + blockIdx.x;
  const uint32_t m = (uint32_t)(row / N_m), n = (uint32_t)(row % N_m);
  const float *sh = shift + (int64_t)m * p;
  float *xr = X + row * p;
  long long score = 0;
  for (int64_t j = (int64_t)threadIdx.x * 4; j < p; j += 256 * 4) {
    const U4 a = philox4x32_10(U4{(uint32_t)(j >> 1), n, m, 0u}, seed, kKey1);
    const U4 b = philox4x32_10(U4{(uint32_t)(j >> 1) + 1u, n, m, 0u}, seed, kKey1);
    const int32_t ih0 = irwin_hall(a.x, a.y), ih1 = irwin_hall(a.z, a.w);
    const int32_t ih2 = irwin_hall(b.x, b.y), ih3 = irwin_hall(b.z, b.w);
    const float4 s4 = *reinterpret_cast<const float4 *>(sh + j);
    const int4 t4 = *reinterpret_cast<const int4 *>(tdir + j);
    float4 o;
    // product and sum are rounded separately (the definition has two roundings): this file
    // is compiled with -ffp-contract=off so that no fused multiply-add is formed
    o.x = (float)ih0 * scale + s4.x;
    o.y = (float)ih1 * scale + s4.y;
    o.z = (float)ih2 * scale + s4.z;
    o.w = (float)ih3 * scale + s4.w;
    *reinterpret_cast<float4 *>(xr + j) = o;
    score += (long long)ih0 * t4.x + (long long)ih1 * t4.y + (long long)ih2 * t4.z + (long long)ih3 * t4.w;
  }
  // exact integer reduction: order does not matter
  __shared__ long long red[256];
  red[threadIdx.x] = score;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) y[row] = red[0] >= 0 ? 1.0f : -1.0f;
}

}  // namespace

extern "C" {

// Fills X (DEVICE float32 [M*N_m, p]) and y (DEVICE float32 [M*N_m]) for rows
// [row_begin, row_begin + n_rows).  shift: DEVICE float32 [M, p]; tdir: DEVICE int32 [p]
// scratch that receives the planted integer direction.  p must be a multiple of 4.
// Returns 0 or a hipError_t value.  Asynchronous on `stream`.
int cada_synth_counter_rows(uint32_t seed, int64_t N_m, int64_t p, int64_t row_begin, int64_t n_rows, float scale,
                            const float *shift, int32_t *tdir, float *X, float *y, void *stream) {
  if (p % 4 != 0 || n_rows < 0 || n_rows > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(k_teacher, dim3((unsigned)((p + 255) / 256)), dim3(256), 0, st, seed, p, tdir);
  if (n_rows > 0)
    hipLaunchKernelGGL(k_rows, dim3((unsigned)n_rows), dim3(256), 0, st, seed, N_m, p, row_begin, scale, shift, tdir, X, y);
  return (int)hipGetLastError();
}

}  // extern "C"
