/* CPU generator of the counter-based synthetic rows ("counter_gauss" recipe), the same
 * published function (Philox4x32-10, Salmon et al., SC'11) as philox.py, in C so that the
 * rows a test touches can be regenerated quickly.  Input generation only. */
#include <stdint.h>
#include <stdlib.h>

#define M0 0xD2511F53u
#define M1 0xCD9E8D57u
#define W0 0x9E3779B9u
#define W1 0xBB67AE85u
#define KEY1 0x43414441u

static void philox(uint32_t c[4], uint32_t k0, uint32_t k1) {
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const uint64_t p0 = (uint64_t)M0 * c[0], p1 = (uint64_t)M1 * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1, n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
  }
}

static int32_t irwin_hall(uint32_t a, uint32_t b) {
  return (int32_t)((a & 0xFFFFu) + (a >> 16) + (b & 0xFFFFu) + (b >> 16)) - 131070;
}

/* X_out [n, p] float32, y_out [n] float32; rows = worker-local sample ids of worker m.
 * Returns 0, or -1 if memory for the planted direction could not be allocated. */
int cada_synth_rows_cpu(uint32_t seed, int32_t m, const int64_t *rows, int64_t n, int64_t p, float scale,
                        const float *shift_m, float *X_out, float *y_out) {
  int32_t *tdir = (int32_t *)malloc((size_t)p * sizeof(int32_t));
  if (!tdir) return -1;
  #pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < p; ++j) {
    uint32_t t[4] = {(uint32_t)j, 0u, 0u, 1u};
    philox(t, seed, KEY1);
    tdir[j] = (int32_t)(t[0] % 255u) - 127;
  }
  #pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < n; ++r) {
    long long score = 0;
    float *x = X_out + r * p;
    for (int64_t jp = 0; jp < p / 2; ++jp) {
      uint32_t c[4] = {(uint32_t)jp, (uint32_t)rows[r], (uint32_t)m, 0u};
      philox(c, seed, KEY1);
      const int32_t ih0 = irwin_hall(c[0], c[1]), ih1 = irwin_hall(c[2], c[3]);
      volatile float a = (float)ih0 * scale, b = (float)ih1 * scale;   /* round the product first */
      x[2 * jp] = a + shift_m[2 * jp];
      x[2 * jp + 1] = b + shift_m[2 * jp + 1];
      score += (long long)ih0 * tdir[2 * jp] + (long long)ih1 * tdir[2 * jp + 1];
    }
    y_out[r] = score >= 0 ? 1.0f : -1.0f;
  }
  free(tdir);
  return 0;
}
