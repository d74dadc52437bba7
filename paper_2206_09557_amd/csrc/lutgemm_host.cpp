// Host side of the LUT-GEMM library: buffer sizes, the BCQ quantisers and the packing of
// planes / scales / offsets into the layouts that include/lutgemm.h specifies.
// Formats: paper section 2.3 (BCQ), section 3.3 eq. 3 (offset), appendix C (uniform to
// BCQ), section 3.4 eq. 4 (sizes).  Nothing here touches the GPU.
#include "lutgemm.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

namespace {

constexpr int kRowsPerBlock = 16;    // rows whose keys share one 16-byte lane word
constexpr int kChunksPerTile = 128;  // 1024 input columns per K tile
constexpr int kSlabBytes = 1024;     // 64 lanes x 16 rows, one plane, one sub-slab

struct Shape {
  int64_t m, n, RB, nchunks, NT, NG, g;
  int q;
};

bool make_shape(int64_t m, int64_t n, int q, int g, Shape* s) {
  if (m < 1 || n < 8 || n % 8 != 0 || q < 1 || q > 8 || g < 0) return false;
  int64_t gg = g == 0 ? n : g;
  if (gg % 8 != 0 || n % gg != 0) return false;
  s->m = m;
  s->n = n;
  s->q = q;
  s->g = gg;
  s->RB = (m + kRowsPerBlock - 1) / kRowsPerBlock;
  s->nchunks = n / 8;
  s->NT = (s->nchunks + kChunksPerTile - 1) / kChunksPerTile;
  s->NG = n / gg;
  return true;
}

inline int tile_T(const Shape& s, int64_t kt) {
  int64_t C = std::min<int64_t>(kChunksPerTile, s.nchunks - kt * kChunksPerTile);
  return C > 64 ? 2 : 1;
}

// Per-chunk part of the key offset: slab base of (tile, sub-slab), the quad and the slot
// inside the quad, and the tile's T.
struct ChunkSlot {
  int64_t base;  // kt*RB*q*2048 + t*1024
  int quad;      // j: lanes 4j..4j+3
  int cq;        // slot within the quad
  int T;
};

std::vector<ChunkSlot> chunk_slots(const Shape& s) {
  std::vector<ChunkSlot> v(s.nchunks);
  for (int64_t c = 0; c < s.nchunks; ++c) {
    int64_t kt = c / kChunksPerTile;
    int T = tile_T(s, kt);
    int64_t cc = c - kt * kChunksPerTile;
    int64_t L = cc / T, t = cc % T;
    v[c].base = kt * s.RB * s.q * 2 * kSlabBytes + t * kSlabBytes;
    v[c].quad = (int)(L / 4);
    v[c].cq = (int)(L % 4);
    v[c].T = T;
  }
  return v;
}

// The lane of the quad that owns row rho is k = rho / 4; it keeps the keys of slot cq in
// its dword (cq - k) mod 4, byte rho % 4.
inline int64_t key_offset(const Shape& s, const ChunkSlot& cs, int i, int64_t r) {
  int64_t rb = r / kRowsPerBlock, rho = r % kRowsPerBlock;
  int64_t k = rho / 4;
  return cs.base + (rb * s.q + i) * cs.T * kSlabBytes + (4 * cs.quad + k) * 16 + 4 * ((cs.cq - k + 4) % 4) + rho % 4;
}

size_t bits_bytes(const Shape& s) {
  return (size_t)s.RB * s.q * kSlabBytes * (2 * (s.NT - 1) + tile_T(s, s.NT - 1));
}

inline float half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  uint32_t e = (h >> 10) & 0x1f, f = h & 0x3ffu, bits;
  if (e == 0) {
    if (f == 0) {
      bits = sign;
    } else {  // subnormal: renormalise
      int sh = 0;
      while (!(f & 0x400u)) {
        f <<= 1;
        ++sh;
      }
      bits = sign | ((uint32_t)(113 - sh) << 23) | ((f & 0x3ffu) << 13);
    }
  } else if (e == 31) {
    bits = sign | 0x7f800000u | (f << 13);
  } else {
    bits = sign | ((e + 112) << 23) | (f << 13);
  }
  float out;
  std::memcpy(&out, &bits, 4);
  return out;
}

// double -> binary16, one rounding, nearest even (the default rounding mode is assumed).
inline uint16_t double_to_half(double d) {
  uint16_t sign = std::signbit(d) ? 0x8000u : 0;
  double x = std::fabs(d);
  if (std::isnan(x)) return sign | 0x7e00u;
  if (x >= 65520.0) return sign | 0x7c00u;
  if (x < 6.103515625e-05) {  // below the smallest normal: multiples of 2^-24
    return sign | (uint16_t)std::nearbyint(std::ldexp(x, 24));
  }
  int e;
  std::frexp(x, &e);                                       // x = f * 2^e, f in [0.5, 1)
  double mant = std::nearbyint(std::ldexp(x, 11 - e));     // in [1024, 2048]
  int be = e - 1 + 15;
  if (mant == 2048.0) {
    mant = 1024.0;
    ++be;
  }
  return sign | (uint16_t)((be << 10) | ((int)mant - 1024));
}

template <class F>
void parallel_blocks(int64_t nblocks, F&& fn) {
  unsigned hw = std::thread::hardware_concurrency();
  int64_t nt = std::max<int64_t>(1, std::min<int64_t>(hw ? hw : 1, std::min<int64_t>(nblocks, 64)));
  if (nt == 1) {
    fn(0, nblocks);
    return;
  }
  std::vector<std::thread> th;
  for (int64_t t = 0; t < nt; ++t) {
    int64_t b0 = nblocks * t / nt, b1 = nblocks * (t + 1) / nt;
    th.emplace_back([=, &fn] { fn(b0, b1); });
  }
  for (auto& t : th) t.join();
}

// fp64 sum in increasing index order.
inline double seq_sum_abs(const float* r, int64_t g) {
  double s = 0.0;
  for (int64_t k = 0; k < g; ++k) s += std::fabs((double)r[k]);
  return s;
}
inline double seq_sum(const float* r, int64_t g) {
  double s = 0.0;
  for (int64_t k = 0; k < g; ++k) s += (double)r[k];
  return s;
}

// ---- alternating BCQ (mode LUTGEMM_Q_ALTERNATING): fp64 throughout, every sum in index order ----

// G a = c by Gaussian elimination with partial pivoting; false if singular.
inline bool solve_in_order(int q, double (&A)[8][9], double (&a)[8]) {
  for (int col = 0; col < q; ++col) {
    int piv = col;
    for (int r = col + 1; r < q; ++r)
      if (std::fabs(A[r][col]) > std::fabs(A[piv][col])) piv = r;
    if (std::fabs(A[piv][col]) < 1e-9) return false;
    if (piv != col)
      for (int j = 0; j <= q; ++j) std::swap(A[col][j], A[piv][j]);
    for (int r = col + 1; r < q; ++r) {
      const double f = A[r][col] / A[col][col];
      for (int j = col; j <= q; ++j) A[r][j] = A[r][j] - f * A[col][j];
    }
  }
  for (int i = q - 1; i >= 0; --i) {
    double acc = A[i][q];
    for (int j = i + 1; j < q; ++j) acc = acc - A[i][j] * a[j];
    a[i] = acc / A[i][i];
  }
  return true;
}

// Nearest of the 2^q levels sum_i +-a_i for every weight; ties to the smallest code.
inline void assign_codes(const double* w, int64_t g, int q, const double (&a)[8], int* code) {
  double levels[256];
  for (int c = 0; c < (1 << q); ++c) {
    double v = 0.0;
    for (int i = 0; i < q; ++i) v = v + (((c >> i) & 1) ? a[i] : -a[i]);
    levels[c] = v;
  }
  for (int64_t k = 0; k < g; ++k) {
    int best = 0;
    double best_d = std::fabs(w[k] - levels[0]);
    for (int c = 1; c < (1 << q); ++c) {
      const double d = std::fabs(w[k] - levels[c]);
      if (d < best_d) {
        best = c;
        best_d = d;
      }
    }
    code[k] = best;
  }
}

// One group: greedy start, then { least-squares scales for the signs; planes with a negative
// scale negated; nearest level per weight } until the signs stop changing or kAltIters rounds;
// scales rounded to fp16, signs assigned once more for the stored scales.
constexpr int kAltIters = 15;
inline void alternating_group(const double* w, int64_t g, int q, std::vector<int>& code, std::vector<int>& code_new,
                              std::vector<double>& r, uint16_t (&a16)[8]) {
  double a[8];
  for (int64_t k = 0; k < g; ++k) {
    r[k] = w[k];
    code[k] = 0;
  }
  for (int i = 0; i < q; ++i) {
    double sum = 0.0;
    for (int64_t k = 0; k < g; ++k) {
      if (r[k] >= 0.0) code[k] |= 1 << i;
      sum = sum + std::fabs(r[k]);
    }
    a[i] = sum / (double)g;
    for (int64_t k = 0; k < g; ++k) r[k] = r[k] - a[i] * (((code[k] >> i) & 1) ? 1.0 : -1.0);
  }
  for (int it = 0; it < kAltIters; ++it) {
    double A[8][9];
    for (int i = 0; i < q; ++i) {
      for (int j = 0; j < q; ++j) {
        int64_t t = 0;
        for (int64_t k = 0; k < g; ++k) t += (((code[k] >> i) ^ (code[k] >> j)) & 1) ? -1 : 1;
        A[i][j] = (double)t;
      }
      double c = 0.0;
      for (int64_t k = 0; k < g; ++k) c = c + (((code[k] >> i) & 1) ? w[k] : -w[k]);
      A[i][q] = c;
    }
    double sol[8];
    if (!solve_in_order(q, A, sol)) break;
    int flip = 0;
    for (int i = 0; i < q; ++i) {
      a[i] = sol[i];
      if (a[i] < 0.0) {
        a[i] = -a[i];
        flip |= 1 << i;
      }
    }
    bool changed = false;
    assign_codes(w, g, q, a, code_new.data());
    for (int64_t k = 0; k < g; ++k) {
      if (code_new[k] != (code[k] ^ flip)) changed = true;
      code[k] = code_new[k];
    }
    if (!changed) break;
  }
  double stored[8];
  for (int i = 0; i < q; ++i) {
    a16[i] = double_to_half(a[i]);
    stored[i] = (double)half_to_float(a16[i]);
  }
  assign_codes(w, g, q, stored, code.data());
}

}  // namespace

extern "C" {

size_t lutgemm_bits_bytes(int64_t m, int64_t n, int q) {
  Shape s;
  if (!make_shape(m, n, q, 0, &s)) return 0;
  return bits_bytes(s);
}

size_t lutgemm_alpha_bytes(int64_t m, int64_t n, int q, int g) {
  Shape s;
  if (!make_shape(m, n, q, g, &s)) return 0;
  return (size_t)s.RB * s.NG * q * kRowsPerBlock * 2;
}

size_t lutgemm_z_bytes(int64_t m, int64_t n, int g) {
  Shape s;
  if (!make_shape(m, n, 1, g, &s)) return 0;
  return (size_t)s.RB * s.NG * kRowsPerBlock * 2;
}

size_t lutgemm_alpha_shared_bytes(int64_t m, int64_t n, int g) { return lutgemm_z_bytes(m, n, g); }

int lutgemm_share_scales(const uint16_t* alpha_packed, int64_t m, int64_t n, int q, int g,
                         uint16_t* alpha_shared_out) {
  Shape s;
  if (!alpha_packed || !alpha_shared_out || !make_shape(m, n, q, g, &s)) return LUTGEMM_EINVAL;
  for (int64_t rb = 0; rb < s.RB; ++rb)
    for (int64_t gi = 0; gi < s.NG; ++gi)
      for (int64_t rho = 0; rho < kRowsPerBlock; ++rho) {
        const uint16_t* a = alpha_packed + (((rb * s.NG + gi) * 4 + rho / 4) * q) * 4 + rho % 4;   // plane i at a[4 * i]
        const float a0 = half_to_float(a[0]);
        for (int i = 1; i < q; ++i)
          if (half_to_float(a[4 * i]) != std::ldexp(a0, i)) return LUTGEMM_EINVAL;
        alpha_shared_out[(rb * s.NG + gi) * kRowsPerBlock + rho] = a[0];
      }
  return LUTGEMM_OK;
}

size_t lutgemm_workspace_bytes(int64_t m, int64_t n, int q, int g, int mu, int batch) {
  Shape s;
  if (mu != 8 || batch < 1 || batch > 32 || !make_shape(m, n, q, g, &s)) return 0;
  // arrival counters (32 KB), then one fp32
  // partial per (K group, activation vector, row of an even number of row blocks); four
  // vectors at a time split K over quarter tiles, two over half tiles, so up to four (two)
  // times as many groups as tiles can occur
  const size_t groups = (size_t)s.NT * (batch >= 3 ? 4 : (batch >= 2 ? 2 : 1));
  const size_t rows = (size_t)(s.RB + (s.RB & 1)) * kRowsPerBlock;
  const size_t vectors = (size_t)batch + (batch % 4 == 3 ? 1 : 0);   // three left over run as four
  return (size_t)32768 + groups * vectors * rows * sizeof(float);
}

int lutgemm_pack_bcq(const uint16_t* W, int64_t m, int64_t n, int q, int g, int mu, int mode,
                     void* bits_out, uint16_t* alpha_out, uint16_t* z_out) {
  Shape s;
  if (!W || !bits_out || !alpha_out) return LUTGEMM_EINVAL;
  if (!make_shape(m, n, q, g, &s)) return LUTGEMM_EINVAL;
  if (mu != 8) return LUTGEMM_EUNSUPPORTED;
  if (mode != LUTGEMM_Q_GREEDY && mode != LUTGEMM_Q_GREEDY_MEAN_OFFSET && mode != LUTGEMM_Q_UNIFORM_RTN &&
      mode != LUTGEMM_Q_ALTERNATING)
    return LUTGEMM_EUNSUPPORTED;
  const bool has_offset = mode == LUTGEMM_Q_GREEDY_MEAN_OFFSET || mode == LUTGEMM_Q_UNIFORM_RTN;
  if (has_offset && !z_out) return LUTGEMM_EINVAL;

  uint8_t* bits = static_cast<uint8_t*>(bits_out);
  std::memset(bits, 0, bits_bytes(s));
  std::memset(alpha_out, 0, lutgemm_alpha_bytes(m, n, q, g));
  if (z_out) std::memset(z_out, 0, lutgemm_z_bytes(m, n, g));
  const std::vector<ChunkSlot> slots = chunk_slots(s);
  const int64_t G = s.g, cpg = G / 8;

  parallel_blocks(s.RB, [&](int64_t rb0, int64_t rb1) {
    std::vector<float> res(G);
    std::vector<int> code(G), code_new(G);
    std::vector<double> w64(G), r64(G);
    for (int64_t r = rb0 * kRowsPerBlock; r < std::min<int64_t>(m, rb1 * kRowsPerBlock); ++r) {
      const int64_t rb = r / kRowsPerBlock, rho = r % kRowsPerBlock;
      for (int64_t gi = 0; gi < s.NG; ++gi) {
        const uint16_t* w = W + r * n + gi * G;
        for (int64_t k = 0; k < G; ++k) res[k] = half_to_float(w[k]);
        // plane i of this (row, group) sits at a_dst[i * 4]: quarters of four rows, planes together
        uint16_t* a_dst = alpha_out + (((rb * s.NG + gi) * 4 + rho / 4) * q) * 4 + rho % 4;
        uint16_t* z_dst = z_out ? z_out + (rb * s.NG + gi) * kRowsPerBlock + rho : nullptr;

        if (mode == LUTGEMM_Q_UNIFORM_RTN) {
          float lo = res[0], hi = res[0];
          for (int64_t k = 1; k < G; ++k) {
            lo = std::min(lo, res[k]);
            hi = std::max(hi, res[k]);
          }
          const float levels = (float)((1 << q) - 1);
          const float range_step = (hi - lo) / levels;
          const uint16_t s16 = double_to_half((double)range_step);
          const float sf = half_to_float(s16);
          for (int64_t k = 0; k < G; ++k) {
            if (sf == 0.0f) {
              code[k] = (1 << q) - 1;
            } else {
              float u = std::nearbyint((res[k] - lo) / sf);
              u = std::min(std::max(u, 0.0f), levels);
              code[k] = (int)u;
            }
          }
          float zsum = 0.0f;
          for (int i = 0; i < q; ++i) {
            const uint16_t a16 = double_to_half((double)(std::ldexp(1.0f, i - 1) * sf));
            a_dst[i * 4] = a16;
            zsum = zsum + half_to_float(a16);
            for (int64_t c = 0; c < cpg; ++c) {
              unsigned key = 0;
              for (int j = 0; j < 8; ++j) key |= (unsigned)((code[c * 8 + j] >> i) & 1) << j;
              bits[key_offset(s, slots[gi * cpg + c], i, r)] = (uint8_t)key;
            }
          }
          *z_dst = double_to_half((double)(zsum + lo));
          continue;
        }

        if (mode == LUTGEMM_Q_ALTERNATING) {
          uint16_t a16[8];
          for (int64_t k = 0; k < G; ++k) w64[k] = (double)res[k];
          alternating_group(w64.data(), G, q, code, code_new, r64, a16);
          for (int i = 0; i < q; ++i) {
            a_dst[i * 4] = a16[i];
            for (int64_t c = 0; c < cpg; ++c) {
              unsigned key = 0;
              for (int j = 0; j < 8; ++j) key |= (unsigned)((code[c * 8 + j] >> i) & 1) << j;
              bits[key_offset(s, slots[gi * cpg + c], i, r)] = (uint8_t)key;
            }
          }
          continue;
        }

        if (mode == LUTGEMM_Q_GREEDY_MEAN_OFFSET) {
          const uint16_t z16 = double_to_half(seq_sum(res.data(), G) / (double)G);
          *z_dst = z16;
          const float zf = half_to_float(z16);
          for (int64_t k = 0; k < G; ++k) res[k] = res[k] - zf;
        }
        for (int i = 0; i < q; ++i) {
          const uint16_t a16 = double_to_half(seq_sum_abs(res.data(), G) / (double)G);
          a_dst[i * 4] = a16;
          const float af = half_to_float(a16);
          for (int64_t c = 0; c < cpg; ++c) {
            unsigned key = 0;
            for (int j = 0; j < 8; ++j) {
              float& rv = res[c * 8 + j];
              if (rv >= 0.0f) {  // sign(0) = +1
                key |= 1u << j;
                rv = rv - af;
              } else {
                rv = rv + af;
              }
            }
            bits[key_offset(s, slots[gi * cpg + c], i, r)] = (uint8_t)key;
          }
        }
      }
    }
  });
  return LUTGEMM_OK;
}

int lutgemm_unpack_bcq(const void* bits_in, int64_t m, int64_t n, int q, int mu, int8_t* B_pm1) {
  Shape s;
  if (!bits_in || !B_pm1 || !make_shape(m, n, q, 0, &s)) return LUTGEMM_EINVAL;
  if (mu != 8) return LUTGEMM_EUNSUPPORTED;
  const uint8_t* bits = static_cast<const uint8_t*>(bits_in);
  const std::vector<ChunkSlot> slots = chunk_slots(s);
  parallel_blocks(s.RB, [&](int64_t rb0, int64_t rb1) {
    for (int i = 0; i < q; ++i)
      for (int64_t r = rb0 * kRowsPerBlock; r < std::min<int64_t>(m, rb1 * kRowsPerBlock); ++r) {
        int8_t* dst = B_pm1 + ((int64_t)i * m + r) * n;
        for (int64_t c = 0; c < s.nchunks; ++c) {
          unsigned key = bits[key_offset(s, slots[c], i, r)];
          for (int j = 0; j < 8; ++j) dst[c * 8 + j] = ((key >> j) & 1) ? 1 : -1;
        }
      }
  });
  return LUTGEMM_OK;
}

int lutgemm_pack_planes(const int8_t* B_pm1, int64_t m, int64_t n, int q, int mu, void* bits_out) {
  Shape s;
  if (!bits_out || !B_pm1 || !make_shape(m, n, q, 0, &s)) return LUTGEMM_EINVAL;
  if (mu != 8) return LUTGEMM_EUNSUPPORTED;
  uint8_t* bits = static_cast<uint8_t*>(bits_out);
  std::memset(bits, 0, bits_bytes(s));
  const std::vector<ChunkSlot> slots = chunk_slots(s);
  parallel_blocks(s.RB, [&](int64_t rb0, int64_t rb1) {
    for (int i = 0; i < q; ++i)
      for (int64_t r = rb0 * kRowsPerBlock; r < std::min<int64_t>(m, rb1 * kRowsPerBlock); ++r) {
        const int8_t* src = B_pm1 + ((int64_t)i * m + r) * n;
        for (int64_t c = 0; c < s.nchunks; ++c) {
          unsigned key = 0;
          for (int j = 0; j < 8; ++j) key |= (unsigned)(src[c * 8 + j] > 0) << j;
          bits[key_offset(s, slots[c], i, r)] = (uint8_t)key;
        }
      }
  });
  return LUTGEMM_OK;
}

int lutgemm_pack_scales(const uint16_t* alpha, const uint16_t* z, int64_t m, int64_t n, int q, int g,
                        uint16_t* alpha_out, uint16_t* z_out) {
  Shape s;
  if (!alpha || !alpha_out || !make_shape(m, n, q, g, &s)) return LUTGEMM_EINVAL;
  if ((z == nullptr) != (z_out == nullptr)) return LUTGEMM_EINVAL;
  std::memset(alpha_out, 0, lutgemm_alpha_bytes(m, n, q, g));
  if (z_out) std::memset(z_out, 0, lutgemm_z_bytes(m, n, g));
  for (int64_t r = 0; r < m; ++r) {
    const int64_t rb = r / kRowsPerBlock, rho = r % kRowsPerBlock;
    for (int64_t gi = 0; gi < s.NG; ++gi) {
      for (int i = 0; i < q; ++i)
        alpha_out[(((rb * s.NG + gi) * 4 + rho / 4) * q + i) * 4 + rho % 4] = alpha[((int64_t)i * m + r) * s.NG + gi];
      if (z) z_out[(rb * s.NG + gi) * kRowsPerBlock + rho] = z[r * s.NG + gi];
    }
  }
  return LUTGEMM_OK;
}

const char* lutgemm_strerror(int code) {
  switch (code) {
    case LUTGEMM_OK: return "ok";
    case LUTGEMM_EINVAL: return "invalid argument";
    case LUTGEMM_EUNSUPPORTED: return "unsupported configuration";
    case LUTGEMM_EWORKSPACE: return "workspace too small";
    case LUTGEMM_EHIP: return "HIP call failed";
    default: return "unknown error";
  }
}

}  // extern "C"
