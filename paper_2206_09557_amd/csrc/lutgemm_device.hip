// Device side of the LUT-GEMM library for gfx950 (MI355X): the table build, the
// lookup/accumulate loop, the scale/offset epilogue and the cross-tile reduction
// (paper section 3.1, section 3.2, appendix B), behind lutgemm_gemv / lutgemm_gemm.
//
// Mapping (this library's own; the paper's thread-block design was made for another GPU):
//   * One workgroup of 16 wavefronts owns one K tile (1024 input columns = 128 tables
//     of 256 fp32 entries = 128 KB of LDS) for a contiguous range of row blocks, so a
//     table set is built once per workgroup and reused for thousands of rows.
//   * Table (t, L) lives at LDS byte address  t<<16 | key<<8 | L<<2 : every lane of a
//     wavefront reads its own table, whose 256 entries all sit in bank L, so a lookup
//     wave is bank-conflict free for any keys, and the address is one byte permute of
//     the packed key word.
//   * A lane therefore accumulates, for 16 rows, the contribution of its own 16 input
//     columns, already multiplied by the group's scales; a 64-lane transpose-reduce with
//     DPP row operations turns 16 per-lane sums into 16 row sums.
//   * The per-tile partial sums go to a workspace and a second small kernel adds the
//     tiles in a fixed order (deterministic, unlike the atomic accumulation of appendix B).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "lutgemm.h"

namespace {

constexpr int kWaves = 16;
constexpr int kThreads = kWaves * 64;
constexpr int kLutBytes = 2 * 256 * 64 * 4;  // two sub-slabs x 256 keys x 64 lanes x fp32

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemvParams {
  const __half* x;        // [n]
  const uint8_t* bits;    // packed
  const __half* alpha;    // packed
  const __half* z;        // packed or null
  float* partial;         // [NT][m_pad]
  int64_t m_pad;
  int RB;                 // row blocks
  int NT;                 // K tiles
  int NG;                 // groups per row
  int g;                  // group size (columns)
  int nchunks;            // n / 8
  int row_splits;         // workgroups per K tile
};

// DPP controls (GFX9 encoding)
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowMirror = 0x140;     // lane i <- lane 15-i within a row of 16
constexpr int kDppRowHalfMirror = 0x141; // lane i <- lane 7-i within 8

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ float lds_f32(uint32_t byte_addr) {
  // The table array is the only LDS object of the kernel and starts at LDS address 0.
  return *(const __attribute__((address_space(3))) float*)(uintptr_t)byte_addr;
}

__device__ __forceinline__ float half_lo(uint32_t packed) {
  return __half2float(__ushort_as_half((unsigned short)(packed & 0xffffu)));
}
__device__ __forceinline__ float half_hi(uint32_t packed) {
  return __half2float(__ushort_as_half((unsigned short)(packed >> 16)));
}

// Build the tables of sub-slab t for key range [kh*32, kh*32+32): lane L owns the table
// of slot (t, L).  xs = the 8 activations of the slot's chunk (zeros for an empty slot).
// Entry `key` = sum_j (bit j of key ? +x_j : -x_j)   (section 3.1).
__device__ __forceinline__ void build_tables(float* lut, int t, int kh, int lane, const float (&xs)[8]) {
  float base = -(xs[0] + xs[1] + xs[2] + xs[3] + xs[4]);
#pragma unroll
  for (int j = 5; j < 8; ++j) base += ((kh >> (j - 5)) & 1) ? xs[j] : -xs[j];
  float e[32];
  e[0] = base;
#pragma unroll
  for (int j = 0; j < 5; ++j) {
    const float two_x = 2.0f * xs[j];
#pragma unroll
    for (int k = 0; k < (1 << j); ++k) e[k + (1 << j)] = e[k] + two_x;
  }
#pragma unroll
  for (int k = 0; k < 32; ++k) lut[(t << 14) | ((kh * 32 + k) << 6) | lane] = e[k];
}

// 16 per-lane values -> lane (L % 16) of every row of 16 lanes holds the 64-lane sum of
// value number L % 16.  Halving exchange: at each step a lane keeps the half of its
// values selected by one bit of its id and receives that half from its partner.
__device__ __forceinline__ float transpose_reduce16(const float (&acc)[16], int lane) {
  const bool b3 = lane & 8, b2 = lane & 4, b1 = lane & 2, b0 = lane & 1;
  float s8[8], s4[4], s2[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float keep = b3 ? acc[8 + i] : acc[i];
    const float send = b3 ? acc[i] : acc[8 + i];
    s8[i] = keep + dpp_f32<kDppRowMirror>(send);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float keep = b2 ? s8[4 + i] : s8[i];
    const float send = b2 ? s8[i] : s8[4 + i];
    s4[i] = keep + dpp_f32<kDppRowHalfMirror>(send);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float keep = b1 ? s4[2 + i] : s4[i];
    const float send = b1 ? s4[i] : s4[2 + i];
    s2[i] = keep + dpp_f32<kDppQuadSwap2>(send);
  }
  const float keep = b0 ? s2[1] : s2[0];
  const float send = b0 ? s2[0] : s2[1];
  float s = keep + dpp_f32<kDppQuadSwap1>(send);
  s += __shfl_xor(s, 16);
  s += __shfl_xor(s, 32);
  return s;
}

// One workgroup: K tile kt, row blocks [rb0, rb1).  T = sub-slabs of the tile (1 or 2).
// SPLIT: the two chunks of a lane may lie in different groups (g % 16 != 0).
template <int Q, int T, bool HAS_Z, bool SPLIT>
__device__ __forceinline__ void tile_body(const GemvParams& p, float* lut, int kt, int rb0, int rb1) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);

  // ---- table build (section 3.1; appendix B: each block fills its tables first) ----
  for (int slot = wave; slot < T * 8; slot += kWaves) {
    const int t = slot >> 3, kh = slot & 7;
    const int cc = T * lane + t;
    float xs[8];
    if (cc < chunks_in_tile) {
      const u32x4 raw = *reinterpret_cast<const u32x4*>(p.x + (int64_t)(128 * kt + cc) * 8);
      xs[0] = half_lo(raw.x); xs[1] = half_hi(raw.x);
      xs[2] = half_lo(raw.y); xs[3] = half_hi(raw.y);
      xs[4] = half_lo(raw.z); xs[5] = half_hi(raw.z);
      xs[6] = half_lo(raw.w); xs[7] = half_hi(raw.w);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) xs[j] = 0.0f;
    }
    build_tables(lut, t, kh, lane, xs);
  }
  __syncthreads();

  // ---- per-lane constants ----
  uint32_t lane_base[T];
  int grp[T];
  float sum_x[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    lane_base[t] = ((uint32_t)t << 16) | ((uint32_t)lane << 2);
    const int cc = min(T * lane + t, chunks_in_tile - 1);
    grp[t] = ((128 * kt + cc) * 8) / p.g;
    sum_x[t] = HAS_Z ? lds_f32(lane_base[t] | (0xffu << 8)) : 0.0f;   // entry 0xFF = +x0..+x7
  }
  const float sum_x_pair = (T == 2) ? sum_x[0] + sum_x[T - 1] : sum_x[0];

  const int64_t tile_base = (int64_t)kt * p.RB * Q * 2048;
  float* partial = p.partial + (int64_t)kt * p.m_pad;

  // ---- lookup / accumulate over this workgroup's row blocks ----
  for (int rb = rb0 + wave; rb < rb1; rb += kWaves) {
    const u32x4* bp = reinterpret_cast<const u32x4*>(p.bits + tile_base + (int64_t)rb * Q * T * 1024) + lane;
    u32x4 w[Q][T];
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
      for (int t = 0; t < T; ++t) w[i][t] = __builtin_nontemporal_load(bp + (i * T + t) * 64);

    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;

    constexpr int NA = SPLIT ? T : 1;   // distinct scale groups per lane
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const u32x4* ap = reinterpret_cast<const u32x4*>(p.alpha + ((int64_t)rb * p.NG + grp[a]) * Q * 16);
      u32x4 al[Q][2];
#pragma unroll
      for (int i = 0; i < Q; ++i) {
        al[i][0] = ap[i * 2];
        al[i][1] = ap[i * 2 + 1];
      }
#pragma unroll
      for (int i = 0; i < Q; ++i) {
        const uint32_t aw[8] = {al[i][0].x, al[i][0].y, al[i][0].z, al[i][0].w,
                                al[i][1].x, al[i][1].y, al[i][1].z, al[i][1].w};
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const uint32_t sel = 0x0c020000u | ((4u + (r & 3)) << 8);   // {0, base.b2, key, base.b0}
          float v;
          if (SPLIT) {
            v = lds_f32(__builtin_amdgcn_perm(w[i][a][r >> 2], lane_base[a], sel));
          } else {
            v = lds_f32(__builtin_amdgcn_perm(w[i][0][r >> 2], lane_base[0], sel));
            if (T == 2) v += lds_f32(__builtin_amdgcn_perm(w[i][T - 1][r >> 2], lane_base[T - 1], sel));
          }
          const float a_r = (r & 1) ? half_hi(aw[r >> 1]) : half_lo(aw[r >> 1]);
          acc[r] = fmaf(a_r, v, acc[r]);   // scale applied once per (row, group, plane): section 3.2 rule 2
        }
      }
      if (HAS_Z) {  // offset term of eq. 3: z[r][G] * sum of the lane's activations
        const u32x4* zp = reinterpret_cast<const u32x4*>(p.z + ((int64_t)rb * p.NG + grp[a]) * 16);
        const u32x4 z0 = zp[0], z1 = zp[1];
        const uint32_t zw[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
        const float sx = SPLIT ? sum_x[a] : sum_x_pair;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float z_r = (r & 1) ? half_hi(zw[r >> 1]) : half_lo(zw[r >> 1]);
          acc[r] = fmaf(z_r, sx, acc[r]);
        }
      }
    }

    const float s = transpose_reduce16(acc, lane);
    if (lane < 16) partial[rb * 16 + lane] = s;
  }
}

template <int Q, bool HAS_Z, bool SPLIT>
__global__ __launch_bounds__(kThreads) void lutgemm_gemv_kernel(GemvParams p) {
  __shared__ float lut[kLutBytes / 4];
  // The lookup addresses are formed as if the tables start at LDS address 0.
  if ((uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)lut != 0u) return;
  const int kt = blockIdx.x % p.NT;
  const int rs = blockIdx.x / p.NT;
  const int rb0 = (int)((int64_t)p.RB * rs / p.row_splits);
  const int rb1 = (int)((int64_t)p.RB * (rs + 1) / p.row_splits);
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  if (chunks_in_tile > 64)
    tile_body<Q, 2, HAS_Z, SPLIT>(p, lut, kt, rb0, rb1);
  else
    tile_body<Q, 1, HAS_Z, false>(p, lut, kt, rb0, rb1);
}

// y[b][r] = sum over K tiles of partial[(kt * batch + b)][r], in tile order (appendix B's
// cross-block accumulation, made order-fixed), rounded to the output type.
template <bool F32OUT>
__global__ __launch_bounds__(256) void lutgemm_reduce_kernel(const float* __restrict__ partial, void* __restrict__ y,
                                                             int64_t m, int64_t m_pad, int NT, int batch) {
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int b = blockIdx.y;
  if (r >= m) return;
  float s = 0.0f;
  for (int kt = 0; kt < NT; ++kt) s += partial[((int64_t)kt * batch + b) * m_pad + r];
  if (F32OUT)
    static_cast<float*>(y)[(int64_t)b * m + r] = s;
  else
    static_cast<__half*>(y)[(int64_t)b * m + r] = __float2half_rn(s);
}

using GemvKernel = void (*)(GemvParams);

template <bool HAS_Z, bool SPLIT>
GemvKernel pick_q(int q) {
  switch (q) {
    case 1: return lutgemm_gemv_kernel<1, HAS_Z, SPLIT>;
    case 2: return lutgemm_gemv_kernel<2, HAS_Z, SPLIT>;
    case 3: return lutgemm_gemv_kernel<3, HAS_Z, SPLIT>;
    case 4: return lutgemm_gemv_kernel<4, HAS_Z, SPLIT>;
    case 5: return lutgemm_gemv_kernel<5, HAS_Z, SPLIT>;
    case 6: return lutgemm_gemv_kernel<6, HAS_Z, SPLIT>;
    case 7: return lutgemm_gemv_kernel<7, HAS_Z, SPLIT>;
    case 8: return lutgemm_gemv_kernel<8, HAS_Z, SPLIT>;
  }
  return nullptr;
}

GemvKernel pick_kernel(int q, bool has_z, bool split) {
  if (has_z) return split ? pick_q<true, true>(q) : pick_q<true, false>(q);
  return split ? pick_q<false, true>(q) : pick_q<false, false>(q);
}

int compute_units() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
  if (cached[dev] == 0) {
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) return -1;
    cached[dev] = cu;
  }
  return cached[dev];
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

int lutgemm_gemm(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !bits || !alpha || !y || !workspace) return LUTGEMM_EINVAL;
  if (m < 1 || n < 8 || n % 8 != 0 || q < 1 || q > 8 || g < 0 || batch < 1) return LUTGEMM_EINVAL;
  const int64_t gg = g == 0 ? n : g;
  if (gg % 8 != 0 || n % gg != 0) return LUTGEMM_EINVAL;
  if (!aligned16(x) || !aligned16(bits) || !aligned16(alpha) || !aligned16(z) || !aligned16(y) || !aligned16(workspace))
    return LUTGEMM_EINVAL;
  if (mu != 8 || batch > 32 || (flags & ~1u) != 0) return LUTGEMM_EUNSUPPORTED;
  if (m > (int64_t)1 << 30 || n > (int64_t)1 << 30) return LUTGEMM_EUNSUPPORTED;
  const size_t need = lutgemm_workspace_bytes(m, n, q, g, mu, batch);
  if (need == 0) return LUTGEMM_EINVAL;
  if (workspace_bytes < need) return LUTGEMM_EWORKSPACE;

  const int cus = compute_units();
  if (cus <= 0) return LUTGEMM_EHIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  GemvParams p;
  p.bits = static_cast<const uint8_t*>(bits);
  p.alpha = static_cast<const __half*>(alpha);
  p.z = static_cast<const __half*>(z);
  p.RB = (int)((m + 15) / 16);
  p.m_pad = (int64_t)p.RB * 16;
  p.nchunks = (int)(n / 8);
  p.NT = (p.nchunks + 127) / 128;
  p.NG = (int)(n / gg);
  p.g = (int)gg;
  // One workgroup per compute unit: split the rows of every K tile so that NT * splits
  // fills the chip, but keep at least one row block per wavefront.
  int splits = cus / p.NT;
  splits = splits < 1 ? 1 : splits;
  const int max_splits = (p.RB + kWaves - 1) / kWaves;
  p.row_splits = splits > max_splits ? max_splits : splits;

  const bool split_alpha = (gg % 16) != 0;
  GemvKernel kern = pick_kernel(q, z != nullptr, split_alpha);
  if (!kern) return LUTGEMM_EUNSUPPORTED;

  for (int b = 0; b < batch; ++b) {
    // partial index: (kt * batch + b) * m_pad  ->  base b * m_pad, tile stride batch * m_pad
    GemvParams pb = p;
    pb.x = static_cast<const __half*>(x) + (int64_t)b * n;
    pb.partial = static_cast<float*>(workspace) + (int64_t)b * p.m_pad;
    pb.m_pad = p.m_pad * batch;
    void* args[] = {&pb};
    if (hipLaunchKernel(reinterpret_cast<const void*>(kern), dim3(p.NT * p.row_splits), dim3(kThreads), args, 0,
                        stream) != hipSuccess)
      return LUTGEMM_EHIP;
  }
  const float* partial = static_cast<const float*>(workspace);
  int64_t m_arg = m, m_pad_arg = p.m_pad;
  int nt_arg = p.NT, batch_arg = batch;
  void* rargs[] = {&partial, &y, &m_arg, &m_pad_arg, &nt_arg, &batch_arg};
  const void* rkern = (flags & LUTGEMM_Y_F32) ? reinterpret_cast<const void*>(lutgemm_reduce_kernel<true>)
                                              : reinterpret_cast<const void*>(lutgemm_reduce_kernel<false>);
  if (hipLaunchKernel(rkern, dim3((unsigned)((m + 255) / 256), (unsigned)batch), dim3(256), rargs, 0, stream) !=
      hipSuccess)
    return LUTGEMM_EHIP;
  return LUTGEMM_OK;
}

int lutgemm_gemv(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  return lutgemm_gemm(x, bits, alpha, z, y, q, g, mu, m, n, 1, flags, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
