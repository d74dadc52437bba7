/*
 * oracle_gemv.c -- plain C fp64 oracle for y = What x read from the packed buffers.
 *
 * TEST INFRASTRUCTURE ONLY: linked by tests/, __graft_entry__.smoke() and bench.py's
 * cpu_baseline leg, never by the product path.  Shares no code or headers with the HIP
 * library; the offsets below are written from the layout text of include/lutgemm.h.
 *
 * For every requested row it rebuilds the dequantised row of section 3.3 eq. 3,
 *     What[r][k] = sum_i alpha[i][r][k/g] * B_i[r][k] + z[r][k/g],
 * in fp64 and takes the plain dot product with x (section 3.2).  No table, no blocking,
 * no reordering: k runs upward, planes run upward.  Rows are independent, so OpenMP
 * splits them over the host cores; the arithmetic per row is unchanged by that.
 *
 * Pinned by the same tests as the numpy oracle (brute force, sum(+-x) identity, dense
 * sum-of-planes + numpy.dot).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int f = h & 0x3ff;
  double v;
  if (e == 0)
    v = ldexp((double)f, -24);
  else if (e == 31)
    v = f ? NAN : INFINITY;
  else
    v = ldexp((double)(f | 0x400), e - 25);
  return sign ? -v : v;
}

/* Byte offset of the key of (plane i, row r, chunk c). */
static int64_t key_offset(int64_t m, int64_t n, int q, int i, int64_t r, int64_t c) {
  int64_t RB = (m + 15) / 16;
  int64_t rb = r / 16, rho = r % 16;
  int64_t kt = c / 128;
  int64_t C = n / 8 - 128 * kt;
  if (C > 128) C = 128;
  int64_t T = C > 64 ? 2 : 1;
  int64_t L = (c - 128 * kt) / T, t = (c - 128 * kt) % T;
  int64_t j = L / 4, cq = L % 4, k = rho / 4; /* quad, slot in quad, owning lane of the quad */
  int64_t slab = kt * RB * q * 2048 + ((rb * q + i) * T + t) * 1024;
  return slab + (4 * j + k) * 16 + 4 * ((cq - k + 4) % 4) + rho % 4;
}

/*
 * y[b * nrows + a] = sum_k What[rows[a]][k] * x[b][k]   (fp64)
 * bits/alpha/z: packed layouts; z may be NULL; g == 0 means g = n.
 * rows == NULL means rows 0..nrows-1.  Returns the number of threads used, or -1.
 */
int oracle_gemv_packed(const uint8_t* bits, const uint16_t* alpha, const uint16_t* z,
                       const uint16_t* x, int64_t m, int64_t n, int q, int g, int batch,
                       const int64_t* rows, int64_t nrows, double* y, int nthreads) {
  if (!bits || !alpha || !x || !y || m < 1 || n < 8 || n % 8 || q < 1 || q > 8 || batch < 1 || batch > 32) return -1;
  int64_t gg = g == 0 ? n : g;
  if (gg % 8 || n % gg) return -1;
  int64_t NG = n / gg;
  int used = 1;
#ifdef _OPENMP
  if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel
  {
#pragma omp single
    used = omp_get_num_threads();
  }
#endif
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t a = 0; a < nrows; ++a) {
    int64_t r = rows ? rows[a] : a;
    int64_t rb = r / 16, rho = r % 16;
    double acc[32];
    for (int b = 0; b < batch; ++b) acc[b] = 0.0;
    for (int64_t k = 0; k < n; ++k) {
      int64_t G = k / gg;
      double w = 0.0;
      for (int i = 0; i < q; ++i) {
        uint8_t key = bits[key_offset(m, n, q, i, r, k / 8)];
        double bsign = ((key >> (k % 8)) & 1) ? 1.0 : -1.0;
        w += half_to_double(alpha[(((rb * NG + G) * 4 + rho / 4) * q + i) * 4 + rho % 4]) * bsign;
      }
      if (z) w += half_to_double(z[(rb * NG + G) * 16 + rho]);
      for (int b = 0; b < batch; ++b) acc[b] += w * half_to_double(x[(int64_t)b * n + k]);
    }
    for (int b = 0; b < batch; ++b) y[(int64_t)b * nrows + a] = acc[b];
  }
  return used;
}
