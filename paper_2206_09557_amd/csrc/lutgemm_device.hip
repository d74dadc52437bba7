// Device side of the LUT-GEMM library for gfx950 (MI355X): the table build, the
// lookup/accumulate loop, the scale/offset epilogue and the cross-tile reduction
// (paper section 3.1, section 3.2, appendix B), behind lutgemm_gemv / lutgemm_gemm.
//
// Mapping (this library's own; the paper's thread-block design was made for another GPU):
//   * One workgroup of 16 wavefronts owns a K group (one or a few consecutive K tiles; a
//     tile is 1024 input columns = 128 tables of 256 fp32 entries = 128 KB of LDS) for a
//     contiguous range of row blocks, so a table set is built once per workgroup and tile
//     and reused for hundreds to thousands of rows; with several tiles the row sums stay
//     in LDS from tile to tile.
//   * Table (t, L) lives at LDS byte address  t<<16 | key<<8 | L<<2 : its 256 entries all
//     sit in bank L, and the address of a lookup is one byte permute of the packed key word.
//   * Inside a quad of lanes the rows are dealt out (lane k owns rows 4k..4k+3 of the
//     16-row block) and the quad's four tables are visited in rotation (in its dword s lane
//     k finds the keys of table 4j + (s+k) mod 4).  At any instant the 64 lanes address 64
//     different tables, so a lookup wave is bank-conflict free for any keys, and a lane
//     ends up with just four row sums whose scales are its own: no scale is fetched twice
//     inside a quad, and the cross-lane reduction shrinks to four values over 16 quads.
//   * The per-K-group partial sums go to a workspace; the last workgroup to finish a row
//     range (an arrival counter per range) adds the groups in a fixed order and writes y,
//     so the result does not depend on arrival order (unlike the atomic accumulation of
//     appendix B) and no second kernel is needed.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <mutex>

#include "lutgemm.h"

namespace {

constexpr int kWaves = 16;     // wavefronts per workgroup (four per SIMD: 128 registers each)
constexpr int kThreads = kWaves * 64;
constexpr int kLutBytes = 2 * 256 * 64 * 4;  // two sub-slabs x 256 keys x 64 lanes x fp32
constexpr int kQueueWord = kLutBytes / 4;      // one extra LDS word after the tables: the workgroup's unit queue
// Behind the queue word: running row sums of a workgroup whose K group has several tiles (GEMV
// kernel): 16 floats per row block of its row range, carried in LDS from tile to tile instead
// of through memory.  The host never plans such a K group for a longer row range.
constexpr int kRunBlocks = 480;
constexpr int kRunWord = kQueueWord + 4;
constexpr int kGemvLdsFloats = kRunWord + kRunBlocks * 16;   // 161,808 bytes of the 160 KB

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemvParams {
  const __half* x;        // [n]
  const uint8_t* bits;    // packed
  const __half* alpha;    // packed
  const __half* z;        // packed or null
  float* partial;         // this activation vector's partials: [KG][kg_stride]
  uint32_t* counters;     // this activation vector's arrival counters: [row_splits]
  void* y;                // this activation vector's output, fp16 or fp32 [m]
  int64_t kg_stride;      // floats between the partials of consecutive K groups
  int m;                  // rows
  int RB;                 // row blocks
  int NT;                 // K tiles
  int NG;                 // groups per row
  int g;                  // group size (columns)
  int nchunks;            // n / 8
  int KG;                 // K groups (workgroups along K)
  int TPG;                // K tiles per K group
  int row_splits;         // workgroups along the rows (grid y; K groups are grid x)
  int range_base;         // row units (row blocks; pairs of them in the quad kernel) per row range ...
  int range_rem;          // ... plus one for the first range_rem ranges
  int y_f32;              // output type
  int g_shift;            // log2(g / 8) when g is a power of two, else -1
  // pair kernel only
  int n;                  // columns
  int64_t vec_stride;     // floats between the partials of the two vectors of a pair
  // matrix-core kernel: activation vectors; quad kernel: live vectors of this launch (3 or 4)
  int batch;
};

// Row range rs in row units: ranges differ by at most one unit.  (Grid x = K group, grid y =
// row range: no division anywhere in the preamble of the one-layer kernels.)
__device__ __forceinline__ void row_range(const GemvParams& p, int rs, int* u0, int* u1) {
  *u0 = rs * p.range_base + min(rs, p.range_rem);
  *u1 = *u0 + p.range_base + (rs < p.range_rem ? 1 : 0);
}

// Group of a chunk (8 columns): chunk / (g / 8), a shift for the usual power-of-two group sizes.
__device__ __forceinline__ int group_of_chunk(const GemvParams& p, int chunk) {
  return p.g_shift >= 0 ? (chunk >> p.g_shift) : (chunk * 8) / p.g;
}

// v under a DPP control (GFX9 encoding)
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Lane exchanges of the row reductions, in registers (no trip through the LDS crossbar,
// whose latency every unit of a wavefront would wait for three or four times in a row).
// The two halving steps of the row reductions.  The partner's value comes through DPP moves
// written into the banks of four lanes each is right for (the compiler folds them into the
// additions where it can, and it is the compiler that keeps the wait states a DPP read needs
// after the write of its source: hand-written DPP instructions in inline assembly would not get
// them and have returned stale values here):
//   lanes with bit 2 clear: a0[i] + a0[i + 4],  lanes with bit 2 set: a2[i] + a2[i - 4];
//   lanes with bit 3 clear: h0[i] + h0[i + 8],  lanes with bit 3 set: h1[i] + h1[i - 8].
__device__ __forceinline__ float halve_over_lane_bit2(float a0, float a2, bool bit2) {
  const unsigned x0 = __builtin_bit_cast(unsigned, a0), x2 = __builtin_bit_cast(unsigned, a2);
  unsigned t = __builtin_amdgcn_update_dpp(x2, x0, 0x104 /* row_shl:4 */, 0xf, 0x5, false);   // banks 0, 2: a0 of lane i + 4
  t = __builtin_amdgcn_update_dpp(t, x2, 0x114 /* row_shr:4 */, 0xf, 0xa, false);             // banks 1, 3: a2 of lane i - 4
  return (bit2 ? a2 : a0) + __builtin_bit_cast(float, t);
}
__device__ __forceinline__ float halve_over_lane_bit3(float h0, float h1, bool bit3) {
  const unsigned x0 = __builtin_bit_cast(unsigned, h0), x1 = __builtin_bit_cast(unsigned, h1);
  unsigned t = __builtin_amdgcn_update_dpp(x1, x0, 0x128 /* row_ror:8 */, 0xf, 0x3, false);   // lanes 0..7 of a row: h0 of lane i + 8
  t = __builtin_amdgcn_update_dpp(t, x1, 0x128, 0xf, 0xc, false);                              // lanes 8..15: h1 of lane i - 8
  return (bit3 ? h1 : h0) + __builtin_bit_cast(float, t);
}
// s + (s of lane i ^ 16), s + (s of lane i ^ 32): the swap instructions exchange the odd rows
// of 16 (the upper 32 lanes) of one operand with the even rows (the lower 32) of the other;
// with both operands s, the two results are s and its partner, in one order or the other.
__device__ __forceinline__ float sum_lane_xor16(float s) {
  const unsigned x = __builtin_bit_cast(unsigned, s);
  const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
__device__ __forceinline__ float sum_lane_xor32(float s) {
  const unsigned x = __builtin_bit_cast(unsigned, s);
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

__device__ __forceinline__ float lds_f32(uint32_t byte_addr) {
  // The table array is the only LDS object of the kernel and starts at LDS address 0.
  return *(const __attribute__((address_space(3))) float*)(uintptr_t)byte_addr;
}

// The split-K partials cross workgroups (and L2s) inside one kernel.  They are written and
// read with device-scope atomics only: such a store is written through to memory and stays
// in the wavefront's memory counter until that write is acknowledged, and such a load is
// served from the device's point of coherence, never from a stale cached copy.  What orders
// one workgroup's partials before another workgroup's reads is described at
// finish_row_range.
__device__ __forceinline__ void store_device_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_device_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
  // two batches of 16 entries (key bit 4 clear, then set) keep the register footprint small:
  // the first units of the row loop are already in flight while the tables are built
#pragma unroll
  for (int hi = 0; hi < 2; ++hi) {
    float e[16];
    e[0] = hi ? base + 2.0f * xs[4] : base;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float two_x = 2.0f * xs[j];
#pragma unroll
      for (int k = 0; k < (1 << j); ++k) e[k + (1 << j)] = e[k] + two_x;
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) lut[(t << 14) | ((kh * 32 + hi * 16 + k) << 6) | lane] = e[k];
  }
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kDppRowRor8 = 0x128;       // lane i <- lane (i + 8) mod 16 within a row of 16

// Four per-lane values (rows 4k..4k+3 of the block, k = lane % 4) -> every lane holds the
// 64-lane sum (over the 16 quads) of ONE of its rows, and returns which: row_in_block.
// Halving exchange over lane bits 2 and 3, then a plain sum over lane bits 4 and 5.
__device__ __forceinline__ float quad_rows_reduce(const float (&acc)[4], int lane, int* row_in_block) {
  const bool b2 = lane & 4, b3 = lane & 8;
  const float h0 = halve_over_lane_bit2(acc[0], acc[2], b2);   // rows 0 or 2 of the lane's four
  const float h1 = halve_over_lane_bit2(acc[1], acc[3], b2);   // rows 1 or 3
  float s = halve_over_lane_bit3(h0, h1, b3);
  s = sum_lane_xor16(s);
  s = sum_lane_xor32(s);
  *row_in_block = 4 * (lane & 3) + (b2 ? 2 : 0) + (b3 ? 1 : 0);
  return s;
}

// How a lane gets the scales of its four rows.
//   kAlphaQuad     the four slots of the quad lie in one group (g % (32 * T) == 0): one
//                  fetch of four rows x q planes serves all the lane's lookups.
//   kAlphaPerSlot  one fetch per dword (slot); the two chunks of a slot share a group
//                  (g % 16 == 0, or T == 1).
//   kAlphaPerChunk one fetch per (dword, sub-slab): g % 16 != 0 with T == 2.
//   kAlphaSlotPair one fetch per pair of slots (g % 32 == 0 with T == 2: slots 2P and 2P + 1
//                  are 32 columns of one group).  Which of a lane's dwords make a pair depends
//                  on the lane (its dword s holds slot (s + k) mod 4 of the quad): dwords
//                  (0, 1) and (2, 3) in the lanes with even k, (0, 3) and (1, 2) with odd k.
//                  So the odd lanes take their dwords in the order 0, 3, 2, 1 (dword_of):
//                  every per-lane constant is computed in that order, and the fetched key
//                  words have dwords 1 and 3 exchanged by two selects before the lookups.
// Added to any of them, kAlphaShared says that the scale buffer holds ONE value per (row,
// group), alpha_0, and that plane i has the scale 2^i * alpha_0 (appendix C: the scales of
// uniformly quantised weights): one fetch of four rows instead of four rows x q planes.
enum { kAlphaQuad = 0, kAlphaPerSlot = 1, kAlphaPerChunk = 2, kAlphaSlotPair = 3, kAlphaShared = 4 };

// The s-th dword a lane works on, as an index into its fetched key words.
template <int AMODE>
__device__ __forceinline__ int dword_of(int s, int lane) {
  return ((AMODE & 3) == kAlphaSlotPair && (lane & 1)) ? ((4 - s) & 3) : s;
}

// What one wavefront fetches for planes I0 .. I0+QP-1 of one (K tile, row block) unit of a
// Q-plane layer.  (The GEMV kernel fetches all planes of a unit at once, except one plane at
// a time where every chunk has a scale set of its own; the pair and quad kernels, whose
// lookups need more registers, fetch layers of more than four planes in two or three parts.)
template <int Q, int I0, int QP, int T, int AMODE, bool HAS_Z>
struct Unit {
  static constexpr int NS = ((AMODE & 3) == kAlphaQuad) ? 1 : ((AMODE & 3) == kAlphaSlotPair ? 2 : 4);   // scale sets along the dwords
  static constexpr int NC = ((AMODE & 3) == kAlphaPerChunk) ? T : 1;             // ... and along the sub-slabs
  u32x4 w[QP][T];           // key words: dword s = four rows of slot 4j + (s + k) mod 4
  u32x2 al[NS][NC][QP];     // fp16 scales of the lane's four rows
  u32x2 zz[NS][NC];         // fp16 offsets of the lane's four rows (used when I0 == 0)
  float prev;               // partial sum of the earlier tiles of this K group (used when I0 == 0)
};

// Group index of every (dword, sub-slab) of this lane in tile kt.
template <int T, bool SHIFT = true, int AMODE = kAlphaQuad>
__device__ __forceinline__ void lane_groups(const GemvParams& p, int kt, int lane, int chunks_in_tile, int (&grp)[4][T]) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int slot = (lane & ~3) | ((dword_of<AMODE>(s, lane) + lane) & 3);
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int cc = min(T * slot + t, chunks_in_tile - 1);
      grp[s][t] = SHIFT ? group_of_chunk(p, 128 * kt + cc) : ((128 * kt + cc) * 8) / p.g;
    }
  }
}

// All loads are unconditional (no branch between a fetch and the waits of the compute that
// follows it), so that the wait counters let later fetches stay in flight.
template <bool SUB = false, int Q, int I0, int QP, int T, int AMODE, bool HAS_Z>
__device__ __forceinline__ void load_unit(Unit<Q, I0, QP, T, AMODE, HAS_Z>& u, const GemvParams& p, int64_t tile_base,
                                          int rb, int lane, const int (&grp)[4][T], const float* partial, int out_row,
                                          bool add_prev, int sub_T = T, int sub_t0 = 0) {
  // SUB: the unit is ONE sub-slab (sub_t0) of a tile laid out with sub_T sub-slabs per plane
  // (the pair kernel); otherwise all T sub-slabs of the tile are fetched.
  using U = Unit<Q, I0, QP, T, AMODE, HAS_Z>;
  const int tile_T = SUB ? sub_T : T;
  const int t0 = SUB ? sub_t0 : 0;
  const u32x4* bp = reinterpret_cast<const u32x4*>(p.bits + tile_base + (int64_t)rb * Q * tile_T * 1024) + lane;
#pragma unroll
  for (int i = 0; i < QP; ++i)
#pragma unroll
    for (int t = 0; t < T; ++t) u.w[i][t] = __builtin_nontemporal_load(bp + ((I0 + i) * tile_T + t0 + t) * 64);
#pragma unroll
  for (int s = 0; s < U::NS; ++s)
#pragma unroll
    for (int c = 0; c < U::NC; ++c) {
      const int64_t blk = (int64_t)rb * p.NG + grp[s * (4 / U::NS) % 4][c];   // first dword of the set
      if ((AMODE & kAlphaShared) != 0) {   // one scale per (row, group), laid out like the offsets
        u.al[s][c][0] = *reinterpret_cast<const u32x2*>(p.alpha + blk * 16 + (lane & 3) * 4);
      } else {
        const u32x2* ap = reinterpret_cast<const u32x2*>(p.alpha + ((blk * 4 + (lane & 3)) * Q) * 4);
#pragma unroll
        for (int i = 0; i < QP; ++i) u.al[s][c][i] = ap[I0 + i];
      }
      if (HAS_Z && I0 == 0) u.zz[s][c] = *reinterpret_cast<const u32x2*>(p.z + blk * 16 + (lane & 3) * 4);
    }
  // first tile of the K group: nothing to add (the value read is never used)
  if (I0 == 0) u.prev = add_prev ? load_device_coherent(partial + rb * 16 + out_row) : 0.0f;
}

__device__ __forceinline__ float half_of(const u32x2& v, int j) {   // j-th of the 4 halves
  const uint32_t wrd = (j & 2) ? v.y : v.x;
  return (j & 1) ? half_hi(wrd) : half_lo(wrd);
}

// Scale of plane number `plane` (the i-th of the QP planes fetched together) for row rho of
// the lane's four.  Shared layout: al[0] holds alpha_0 and the plane's scale is 2^plane times
// it, an exact product, so the result equals that of the per-plane layout bit for bit.
template <int AMODE, int QP>
__device__ __forceinline__ float scale_of(const u32x2 (&al)[QP], int i, int plane, int rho) {
  if ((AMODE & kAlphaShared) != 0) return half_of(al[0], rho) * (float)(1 << plane);
  return half_of(al[i], rho);
}

// Lookup / accumulate / scale for the planes of u (section 3.1: partial sums are retrieved
// and added, then multiplied by the scale; section 3.2 rule 2: one scale per run of
// lookups), plus the offset term with the first planes.  acc[rho]: row 4k + rho of the block.
template <int Q, int I0, int QP, int T, int AMODE, bool HAS_Z>
__device__ __forceinline__ void accumulate_unit(const Unit<Q, I0, QP, T, AMODE, HAS_Z>& u,
                                                const uint32_t (&lane_base)[4], const float (&sum_x)[4][T],
                                                float (&acc)[4]) {
  using U = Unit<Q, I0, QP, T, AMODE, HAS_Z>;
  constexpr bool kPairs = (AMODE & 3) == kAlphaSlotPair;
  const bool odd = kPairs && ((lane_base[0] >> 2) & 1u) != 0;   // k of the lane: its first slot is 4j + k
#pragma unroll
  for (int i = 0; i < QP; ++i) {
    uint32_t kw[T][4];   // the key words in the lane's dword order
#pragma unroll
    for (int t = 0; t < T; ++t) {
      kw[t][0] = u.w[i][t][0];
      kw[t][1] = odd ? u.w[i][t][3] : u.w[i][t][1];
      kw[t][2] = u.w[i][t][2];
      kw[t][3] = odd ? u.w[i][t][1] : u.w[i][t][3];
    }
#pragma unroll
    for (int rho = 0; rho < 4; ++rho) {
      // address bytes {0, t, key byte rho, slot * 4}: byte 1 of lane_base is the constant 1
      const uint32_t sel_t[2] = {0x0c0c0000u | ((4u + rho) << 8), 0x0c010000u | ((4u + rho) << 8)};
      float run = 0.0f;        // lookups that share one scale
      bool run_open = false;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const float v = lds_f32(__builtin_amdgcn_perm(kw[t][s], lane_base[s], sel_t[t]));
          run = run_open ? run + v : v;
          run_open = true;
          const bool close = ((AMODE & 3) == kAlphaPerChunk) || ((AMODE & 3) == kAlphaPerSlot && t == T - 1) ||
                             (kPairs && (s & 1) && t == T - 1) || (s == 3 && t == T - 1);
          if (close) {
            const int ss = ((AMODE & 3) == kAlphaQuad) ? 0 : (kPairs ? s >> 1 : s);
            const int cc = ((AMODE & 3) == kAlphaPerChunk) ? t : 0;
            acc[rho] = fmaf(scale_of<AMODE>(u.al[ss][cc], i, I0 + i, rho), run, acc[rho]);
            run_open = false;
          }
        }
      }
    }
  }
  if (HAS_Z && I0 == 0) {   // offset term of eq. 3: z[r][G] * (sum of the activations of the columns it covers)
#pragma unroll
    for (int s = 0; s < U::NS; ++s)
#pragma unroll
      for (int c = 0; c < U::NC; ++c) {
        float sx;
        if ((AMODE & 3) == kAlphaQuad) {
          sx = 0.0f;
#pragma unroll
          for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
            for (int t = 0; t < T; ++t) sx += sum_x[s2][t];
        } else if ((AMODE & 3) == kAlphaPerSlot) {
          sx = (T == 2) ? sum_x[s][0] + sum_x[s][T - 1] : sum_x[s][0];
        } else if (kPairs) {
          sx = 0.0f;
#pragma unroll
          for (int s2 = 2 * s; s2 < 2 * s + 2; ++s2)
#pragma unroll
            for (int t = 0; t < T; ++t) sx += sum_x[s2][t];
        } else {
          sx = sum_x[s][c];
        }
#pragma unroll
        for (int rho = 0; rho < 4; ++rho) acc[rho] = fmaf(half_of(u.zz[s][c], rho), sx, acc[rho]);
      }
  }
}

// Planes I0, I0+PP, ... of one unit, PP at a time: fetch, then accumulate.
template <int Q, int I0, int PP, int T, int AMODE, bool HAS_Z>
__device__ __forceinline__ void plane_passes(const GemvParams& p, int64_t tile_base, int rb, int lane,
                                             const int (&grp)[4][T], const float* partial, int out_row, bool add_prev,
                                             const uint32_t (&lane_base)[4], const float (&sum_x)[4][T], float (&acc)[4],
                                             float* prev) {
  constexpr int QP = (Q - I0 < PP) ? Q - I0 : PP;
  Unit<Q, I0, QP, T, AMODE, HAS_Z> u;
  load_unit(u, p, tile_base, rb, lane, grp, partial, out_row, add_prev);
  accumulate_unit(u, lane_base, sum_x, acc);
  if constexpr (I0 == 0) *prev = u.prev;
  if constexpr (I0 + QP < Q)
    plane_passes<Q, I0 + QP, PP, T, AMODE, HAS_Z>(p, tile_base, rb, lane, grp, partial, out_row, add_prev, lane_base, sum_x,
                                                  acc, prev);
}

// Whole-unit compute for layers fetched in one piece.  Returns the 64-lane sum for the row
// quad_rows_reduce assigns to this lane.
template <int Q, int T, int AMODE, bool HAS_Z>
__device__ __forceinline__ float compute_unit(const Unit<Q, 0, Q, T, AMODE, HAS_Z>& u, int lane,
                                              const uint32_t (&lane_base)[4], const float (&sum_x)[4][T],
                                              int* row_in_block) {
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  accumulate_unit(u, lane_base, sum_x, acc);
  return quad_rows_reduce(acc, lane, row_in_block);
}

// Table build of one tile (section 3.1; appendix B: each block fills its tables first).  A
// table slot is (sub-slab t, key range [32 * kh, +32)) = slot 8 * t + kh, 16 slots at T = 2;
// lane L of the building wavefront owns the table of chunk T * L + t.  The activations of a
// slot are fetched first (fetch_slot_x) so that their latency overlaps whatever is issued in
// between; the caller ends the build with the workgroup barrier that publishes the tables.

template <int T>
__device__ __forceinline__ u32x4 fetch_slot_x(const GemvParams& p, int kt, int chunks_in_tile, int slot, int lane) {
  const int t = slot >> 3;
  const int cc = min(T * lane + t, chunks_in_tile - 1);   // clamped: unconditional load, value unused if out of range
  return *reinterpret_cast<const u32x4*>(p.x + (int64_t)(128 * kt + cc) * 8);
}

template <int T>
__device__ __forceinline__ void build_slot(float* lut, int chunks_in_tile, int slot, int lane, const u32x4& raw) {
  if (slot < T * 8) {
    const int t = slot >> 3, kh = slot & 7;
    const bool live = T * lane + t < chunks_in_tile;
    float xs[8];
    xs[0] = half_lo(raw.x); xs[1] = half_hi(raw.x);
    xs[2] = half_lo(raw.y); xs[3] = half_hi(raw.y);
    xs[4] = half_lo(raw.z); xs[5] = half_hi(raw.z);
    xs[6] = half_lo(raw.w); xs[7] = half_hi(raw.w);
#pragma unroll
    for (int j = 0; j < 8; ++j) xs[j] = live ? xs[j] : 0.0f;   // empty slot: an all-zero table
    build_tables(lut, t, kh, lane, xs);
  }
}

// Next unit of the workgroup's queue (wave-uniform).  Units are handed out in order, so the
// workgroup still walks its slice of the packed weights front to back, but a wavefront that
// runs ahead simply takes more of them: all wavefronts run dry within one unit of each other.
__device__ __forceinline__ int next_unit(float* lut, int lane) {
  int v = 0;
  if (lane == 0)
    v = __hip_atomic_fetch_add(reinterpret_cast<int*>(lut + kQueueWord), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  return __builtin_amdgcn_readfirstlane(v);
}

// Per-lane lookup constants: dword s of this lane looks into the table of slot
// 4j + (s + k) mod 4.  lane_base byte 0: slot * 4; byte 1: the constant 1 (source of the
// sub-slab address bit).  sum_x: entry 0xFF of each table = the sum of its 8 activations.
template <int T, bool HAS_Z, int AMODE = kAlphaQuad>
__device__ __forceinline__ void lane_tables(int lane, uint32_t (&lane_base)[4], float (&sum_x)[4][T]) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t slot = ((uint32_t)lane & ~3u) | ((uint32_t)(dword_of<AMODE>(s, lane) + lane) & 3u);
    lane_base[s] = (slot << 2) | 0x100u;
#pragma unroll
    for (int t = 0; t < T; ++t)
      sum_x[s][t] = HAS_Z ? lds_f32(((uint32_t)t << 16) | (0xffu << 8) | (slot << 2)) : 0.0f;
  }
}

// One workgroup, one K tile kt, row blocks [rb0, rb1).  T = sub-slabs of the tile (1 or 2).
// AMODE: how the lanes get their scales (see above).
// A row's sum over the tile leaves a wavefront in one of three ways:
//   * as a partial sum for the cross-group reduction (the usual case: one tile per K group);
//   * directly as y, when the launch has a single K group of a single tile (n <= 1024):
//     nothing is left to add, and the trip through the workspace and the arrival counter
//     would be most of the run time of so small a product;
//   * with several tiles per K group (`carry`), into the workgroup's running sums in LDS:
//     the first tile writes them, later tiles add to them, and when the last tile is done
//     the workgroup copies them to the workspace as its partial sums (flush_row_sums).  Any
//     wavefront may take any unit of any tile: the barrier between two tiles orders one
//     tile's LDS writes before the next tile's reads.  The lookup loop then needs neither
//     the output pointers nor a trip through memory per tile.
__device__ __forceinline__ void store_row_sum(const GemvParams& p, float* partial, bool direct, int row, float v) {
  if (direct) {
    if (row < p.m) {
      if (p.y_f32)
        static_cast<float*>(p.y)[row] = v;
      else   // fp16 output, nearest even (paper table 1)
        static_cast<__half*>(p.y)[row] = __float2half_rn(v);
    }
  } else {
    store_device_coherent(partial + row, v);
  }
}

// Running sums: add this tile's sum for (row block of the range, row of the block).
__device__ __forceinline__ void carry_row_sum(float* lut, int block_in_range, int row_in_block, float v, bool first_tile) {
  float* r = lut + kRunWord + block_in_range * 16 + row_in_block;
  *r = first_tile ? v : *r + v;
}

// After the last tile of a K group of several: the running sums become the partial sums.
__device__ __forceinline__ void flush_row_sums(const GemvParams& p, const float* lut, int rb0, int rb1, float* partial) {
  __syncthreads();
  const int rows = (rb1 - rb0) * 16;
  for (int i = threadIdx.x; i < rows; i += kThreads) store_device_coherent(partial + rb0 * 16 + i, lut[kRunWord + i]);
}

template <int Q, int T, int AMODE, bool HAS_Z>
__device__ __forceinline__ void tile_body(const GemvParams& p, float* lut, int kt, int rb0, int rb1, float* partial,
                                          bool carry, bool first_tile, bool direct) {
  using U = Unit<Q, 0, Q, T, AMODE, HAS_Z>;
  int lane = threadIdx.x & 63;
  // Everything derived from the lane id below belongs to this tile only: the empty asm
  // stops the optimiser from hoisting it out of the tile loop, where the values of the
  // two-sub-slab and the one-sub-slab paths would all be live at once (and spill).
  asm volatile("" : "+v"(lane));
  // wave-uniform by construction; saying so keeps row-block indices and base addresses in SGPRs
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  const int64_t tile_base = (int64_t)kt * p.RB * Q * 2048;

  int grp[4][T];
  // (the per-chunk scale mode has no registers to spare for the two code paths of the shift)
  lane_groups<T, (AMODE & 3) != kAlphaPerChunk, AMODE>(p, kt, lane, chunks_in_tile, grp);
  // the row of the 16-row block whose sum this lane ends up with (see quad_rows_reduce)
  const int out_row = 4 * (lane & 3) + ((lane & 4) ? 2 : 0) + ((lane & 8) ? 1 : 0);

  // Planes fetched together: all of them (up to 8 x 2 x 4 registers of key words: measured 2
  // to 15 % faster than two halves for five to eight planes); one at a time when every
  // (dword, sub-slab) has a scale set of its own.  Keeps a wavefront within its registers in
  // every variant.
  constexpr int PP = ((AMODE & 3) == kAlphaPerChunk) ? 1 : Q;
  if constexpr (PP < Q) {
    // ---- several fetches per unit, no fetch-ahead ----
    build_slot<T>(lut, chunks_in_tile, wave, lane, fetch_slot_x<T>(p, kt, chunks_in_tile, wave, lane));
    __syncthreads();
    uint32_t lane_base[4];
    float sum_x[4][T];
    lane_tables<T, HAS_Z, AMODE>(lane, lane_base, sum_x);
    for (int rb = rb0 + wave; rb < rb1; rb += kWaves) {
      float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      float prev = 0.0f;
      // (this register-bound variant has no running sums in LDS: the sum of the
      // K group's earlier tiles comes back from the workspace with the first fetch of a unit,
      // always in the wavefront that wrote it, and the new sum goes there again)
      plane_passes<Q, 0, PP, T, AMODE, HAS_Z>(p, tile_base, rb, lane, grp, partial, out_row, !first_tile, lane_base, sum_x,
                                              acc, &prev);
      int row_in_block;
      const float s = quad_rows_reduce(acc, lane, &row_in_block) + prev;
      store_row_sum(p, partial, direct, rb * 16 + row_in_block, s);
    }
  } else {
  // Units of the workgroup: u = 0 .. n_units-1 (row block rb0 + u).  A wavefront starts with
  // unit `wave` and takes every further one from the queue.  Nothing is fetched ahead of the
  // unit being computed: the other fifteen wavefronts cover a fetch.
  const int n_units = rb1 - rb0;
  const int u_clamp = n_units - 1;
  if (threadIdx.x == 0) reinterpret_cast<int*>(lut + kQueueWord)[0] = kWaves;   // units 0..kWaves-1 are taken
  U u;
  int cur = wave;                               // unit being computed (or about to be)
  // kEarly: the scale modes with one or two scale sets per lane, which have the registers for
  // the fetch code twice (all but eight planes with offsets and two scale sets).
  constexpr bool kEarly = (AMODE & 3) == kAlphaQuad || ((AMODE & 3) == kAlphaSlotPair && !(Q == 8 && HAS_Z));
  if (kEarly) {
    // Two roles at the start of a tile.  Wavefronts 8..15 build the tables, two slots each.
    // Wavefronts 0..7 ask for their first unit meanwhile, but not before the builders HAVE
    // their activations (the first barrier says so): asked for earlier, the weights would
    // fill the compute unit's memory pipeline and the activations, which every lookup waits
    // for, would queue behind them (measured).  The builders ask for their first unit once
    // the tables stand, so the first requests of a workgroup reach memory in two halves, a
    // table build apart (measured: 0.4 us per launch better than all sixteen wavefronts
    // fetching and building alike; a fetch is unconditional, a wavefront without a unit
    // re-reads the last one: no branch between a fetch and its use, so that the wait
    // counters stay exact).
    const bool builder = wave >= kWaves / 2;
    const int slot0 = 2 * (wave & 7);
    u32x4 xr0 = {0u, 0u, 0u, 0u}, xr1 = {0u, 0u, 0u, 0u};
    if (builder) {
      xr0 = fetch_slot_x<T>(p, kt, chunks_in_tile, slot0, lane);
      xr1 = fetch_slot_x<T>(p, kt, chunks_in_tile, slot0 + 1, lane);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    if (!builder) {
      load_unit(u, p, tile_base, rb0 + min(cur, u_clamp), lane, grp, partial, out_row, false);
    } else {
      build_slot<T>(lut, chunks_in_tile, slot0, lane, xr0);
      build_slot<T>(lut, chunks_in_tile, slot0 + 1, lane, xr1);
    }
    __syncthreads();
    if (builder) load_unit(u, p, tile_base, rb0 + min(cur, u_clamp), lane, grp, partial, out_row, false);
  } else {
    build_slot<T>(lut, chunks_in_tile, wave, lane, fetch_slot_x<T>(p, kt, chunks_in_tile, wave, lane));
    __syncthreads();
  }
  uint32_t lane_base[4];
  float sum_x[4][T];
  lane_tables<T, HAS_Z, AMODE>(lane, lane_base, sum_x);

  // ---- lookup / accumulate ----
  // Up to four results are parked in ONE register (the j-th of a trip in lanes 16j..16j+15)
  // and written by a single store.  A store shares the wave's memory counter with the
  // loads: an outstanding store issued BEFORE a load makes every wait for that load wait
  // for the store's round trip too, so stores are few and younger than the loads in flight.
  const int lane_row = lane >> 4;
  while (cur < n_units) {
    float parked = 0.0f;
    int parked_rb = 0, n_parked = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!kEarly) load_unit(u, p, tile_base, rb0 + cur, lane, grp, partial, out_row, false);
      int row_in_block;
      const float s = compute_unit(u, lane, lane_base, sum_x, &row_in_block);
      parked = (lane_row == j) ? s : parked;
      parked_rb = (lane_row == j) ? rb0 + cur : parked_rb;
      n_parked = j + 1;
      cur = next_unit(lut, lane);
      if (cur >= n_units) break;
      if (kEarly) load_unit(u, p, tile_base, rb0 + cur, lane, grp, partial, out_row, false);   // no fetch in flight at the exit above
    }
    if (lane_row < n_parked) {
      if (carry)
        carry_row_sum(lut, parked_rb - rb0, out_row, parked, first_tile);
      else
        store_row_sum(p, partial, direct, parked_rb * 16 + out_row, parked);
    }
  }
  }   // PP == Q
}

// Sum over the K groups and store for rows [rb0 * 16, row_end): RPP rows per thread per pass,
// KB K groups per row per batch, i.e. RPP * KB independent loads in flight per thread, because
// every one of them goes to memory (the partials were written through by other workgroups).
// Addresses are clamped, not predicated, so RPP and KB are chosen to fit the row range and
// the group count (a clamped load is a wasted load); the sum over the groups of a row always
// runs in ascending group order.
template <int RPP, int KB>
__device__ __forceinline__ void reduce_rows(const GemvParams& p, int rb0, int row_end) {
  for (int r0 = rb0 * 16 + (int)threadIdx.x; r0 < row_end; r0 += RPP * kThreads) {
    const float* src[RPP];
    float sum[RPP];
#pragma unroll
    for (int j = 0; j < RPP; ++j) {
      src[j] = p.partial + min(r0 + j * kThreads, row_end - 1);
      sum[j] = 0.0f;
    }
    for (int kb = 0; kb < p.KG; kb += KB) {
      float v[RPP][KB];
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const int64_t off = (int64_t)min(kb + u, p.KG - 1) * p.kg_stride;
#pragma unroll
        for (int j = 0; j < RPP; ++j) v[j][u] = load_device_coherent(src[j] + off);
      }
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const bool live = kb + u < p.KG;
#pragma unroll
        for (int j = 0; j < RPP; ++j) sum[j] += live ? v[j][u] : 0.0f;
      }
    }
#pragma unroll
    for (int j = 0; j < RPP; ++j) {
      const int r = r0 + j * kThreads;
      if (r < row_end) {
        if (p.y_f32)
          static_cast<float*>(p.y)[r] = sum[j];
        else   // fp16 output, nearest even (paper table 1)
          static_cast<__half*>(p.y)[r] = __float2half_rn(sum[j]);
      }
    }
  }
}

// The same for NVEC activation vectors (2 or 4; a quad launched for three vectors has nothing
// to write for the fourth).  The (vector, row) pairs of the range are dealt to the threads as
// ONE list, RPP of them per thread per pass, so that the passes of the workgroup, each a
// round trip to memory, are as few as the rows allow.
template <int NVEC, int RPP, int KB>
__device__ __forceinline__ void reduce_vector_rows(const GemvParams& p, int rb0, int row_end) {
  const int row0 = rb0 * 16;
  const int rows = row_end - row0;
  const int items = (NVEC == 4 ? min(p.batch, 4) : NVEC) * rows;
  for (int i0 = (int)threadIdx.x; i0 < items; i0 += RPP * kThreads) {
    const float* src[RPP];
    float sum[RPP];
#pragma unroll
    for (int j = 0; j < RPP; ++j) {
      const int i = min(i0 + j * kThreads, items - 1);
      const int vec = i / rows;
      src[j] = p.partial + (int64_t)vec * p.vec_stride + (row0 + i - vec * rows);
      sum[j] = 0.0f;
    }
    for (int kb = 0; kb < p.KG; kb += KB) {
      float v[RPP][KB];
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const int64_t off = (int64_t)min(kb + u, p.KG - 1) * p.kg_stride;
#pragma unroll
        for (int j = 0; j < RPP; ++j) v[j][u] = load_device_coherent(src[j] + off);
      }
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const bool live = kb + u < p.KG;
#pragma unroll
        for (int j = 0; j < RPP; ++j) sum[j] += live ? v[j][u] : 0.0f;
      }
    }
#pragma unroll
    for (int j = 0; j < RPP; ++j) {
      const int i = i0 + j * kThreads;
      if (i < items) {
        const int vec = i / rows;
        const int64_t dst = (int64_t)vec * p.m + (row0 + i - vec * rows);
        if (p.y_f32)
          static_cast<float*>(p.y)[dst] = sum[j];
        else
          static_cast<__half*>(p.y)[dst] = __float2half_rn(sum[j]);
      }
    }
  }
}

// FINE: also batches of 4, 6 and 8 groups (the kernels with registers and code space for them:
// on the tall OPT-175B layers, which run 6 K groups, a batch of 12 wastes half its loads).
template <int NVEC, int RPP, int KB>
__device__ __forceinline__ void reduce_rows_batched(const GemvParams& p, int rb0, int row_end) {
  if constexpr (NVEC == 1)
    reduce_rows<RPP, KB>(p, rb0, row_end);
  else
    reduce_vector_rows<NVEC, RPP, KB>(p, rb0, row_end);
}

template <int NVEC, int RPP, bool FINE>
__device__ __forceinline__ void reduce_rows_by_groups(const GemvParams& p, int rb0, int row_end) {
  if (FINE && p.KG <= 4)
    reduce_rows_batched<NVEC, RPP, 4>(p, rb0, row_end);
  else if (FINE && p.KG <= 6)
    reduce_rows_batched<NVEC, RPP, 6>(p, rb0, row_end);
  else if (FINE && p.KG <= 8)
    reduce_rows_batched<NVEC, RPP, 8>(p, rb0, row_end);
  else if (p.KG <= 12)
    reduce_rows_batched<NVEC, RPP, 12>(p, rb0, row_end);
  else
    reduce_rows_batched<NVEC, RPP, 16>(p, rb0, row_end);
}

// Cross-group reduction by the last workgroup to arrive for a row range, for NVEC activation
// vectors (appendix B accumulates the per-block partial outputs with atomics; here the
// groups are added in index order by whoever arrives last, so y is reproducible bit for bit).
template <int NVEC, bool FINE = false>
__device__ __forceinline__ void finish_row_range(const GemvParams& p, float* lut, int rs, int rb0, int rb1) {
  // Hand-off of the partials to whichever workgroup arrives last for this row range, ordered
  // by completion rather than by fences:
  //  1. every wavefront waits (s_waitcnt vmcnt(0)) until its own partial stores have been
  //     acknowledged; they are write-through device-scope stores, so they are in memory then;
  //  2. the workgroup barrier follows, so thread 0 issues the arrival increment only after
  //     every partial of the workgroup is in memory;
  //  3. the workgroup that reads KG - 1 from the counter knows that all other groups'
  //     partials were in memory before their increments, hence before its own; its loads of
  //     them are issued after a second barrier that follows the return of the increment, and
  //     they are device-scope loads.
  // The language's memory model would express 2 and 3 as a release / acquire pair on the
  // counter.  On this device either half writes back or invalidates a whole L2 and costs 6
  // to 14 microseconds per launch (measured), for stores that are already in memory and
  // loads that bypass the caches anyway; the explicit wait of step 1 is what the hardware
  // needs and what a barrier alone does not give (it does not wait for other wavefronts'
  // stores in flight).  The counter itself is a relaxed device-scope read-modify-write.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                 // every lookup is done as well: the table memory is free
  uint32_t* flag = reinterpret_cast<uint32_t*>(lut);
  if (threadIdx.x == 0) {
    const uint32_t arrived = __hip_atomic_fetch_add(p.counters + rs, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag[0] = (arrived == (uint32_t)(p.KG - 1)) ? 1u : 0u;
  }
  __syncthreads();
  if (flag[0] == 0u) return;
  const int row_end = min(rb1 * 16, p.m);
  const int rows = NVEC * (row_end - rb0 * 16);   // (vector, row) pairs to sum
  if (rows <= kThreads)
    reduce_rows_by_groups<NVEC, 1, FINE>(p, rb0, row_end);
  else if (rows <= 2 * kThreads)
    reduce_rows_by_groups<NVEC, 2, FINE>(p, rb0, row_end);
  else
    reduce_rows_by_groups<NVEC, 3, FINE>(p, rb0, row_end);
  if (threadIdx.x == 0)            // leave the counter at zero for the next call on this workspace
    __hip_atomic_store(p.counters + rs, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One workgroup of a GEMV: K group kg, row range rs of layer p.  The lookup addresses are formed
// as if `lut` started at LDS address 0: it is the only LDS object of the kernels that call
// this, which the host verifies before the first launch of each of them (lds_layout_ok).
// AM2 / AM1: scale modes of the two-sub-slab tiles and of a one-sub-slab last tile.
template <int Q, bool HAS_Z, int AM2, int AM1>
__device__ __forceinline__ void gemv_workgroup(const GemvParams& p, float* lut, int kg, int rs) {
  int rb0, rb1;
  row_range(p, rs, &rb0, &rb1);
  float* partial = p.partial + (int64_t)kg * p.kg_stride;
  const bool direct = p.NT == 1;   // one tile, hence one K group: the sums of the tile are y
  const int kt_end = min((kg + 1) * p.TPG, p.NT);
  // several tiles per K group: running sums in LDS (see carries_in_lds; a last K group with a
  // single tile takes the same path as the others)
  constexpr bool kCarry = (AM2 & 3) != kAlphaPerChunk;
  const bool carry = kCarry && p.TPG > 1;

  for (int kt = kg * p.TPG; kt < kt_end; ++kt) {
    const bool first_tile = kt == kg * p.TPG;
    if (!first_tile) {
      // every lookup of the previous tile is done before its tables are overwritten, every
      // running sum of it written before it is read (those that go through memory:
      // acknowledged, as in finish_row_range)
      if (!kCarry) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
    if (min(128, p.nchunks - 128 * kt) > 64)
      tile_body<Q, 2, AM2, HAS_Z>(p, lut, kt, rb0, rb1, partial, carry, first_tile, direct);
    else
      tile_body<Q, 1, AM1, HAS_Z>(p, lut, kt, rb0, rb1, partial, carry, first_tile, direct);
  }

  if (carry) flush_row_sums(p, lut, rb0, rb1, partial);
  if (!direct) finish_row_range<1, (Q <= 4)>(p, lut, rs, rb0, rb1);
}

template <int Q, bool HAS_Z, int AM2, int AM1>
__global__ __launch_bounds__(kThreads) void lutgemm_gemv_kernel(GemvParams p) {
  __shared__ float lut[kGemvLdsFloats];
  gemv_workgroup<Q, HAS_Z, AM2, AM1>(p, lut, blockIdx.x, blockIdx.y);
}

// Several independent GEMVs in one launch (lutgemm_gemv_group): a one-dimensional grid, the
// workgroups of layer 0 first, then those of layer 1, and so on, each layer with the grid it
// would have on its own.  Workgroups are handed to compute units in that order as earlier
// ones leave, so the last workgroups of a layer (stragglers, the last-arrival sums) share the
// device with the first of the next (activation fetch, table build, first weights): the
// start and the end of a launch, which a GEMV alone spends with the memory system half
// idle, overlap with streaming.
constexpr int kMaxGroup = 8;
struct GroupParams {
  GemvParams layer[kMaxGroup];
  int first_wg[kMaxGroup + 1];   // first_wg[i] .. first_wg[i + 1] - 1: workgroups of layer i
  int count;
};

template <int Q, bool HAS_Z, int AM2, int AM1>
__global__ __launch_bounds__(kThreads) void lutgemm_gemv_group_kernel(GroupParams gp) {
  __shared__ float lut[kGemvLdsFloats];
  int li = 0;
  for (int k = 1; k < gp.count; ++k)
    if ((int)blockIdx.x >= gp.first_wg[k]) li = k;
  const GemvParams& p = gp.layer[li];
  const int local = (int)blockIdx.x - gp.first_wg[li];
  const int rs = local / p.KG;
  gemv_workgroup<Q, HAS_Z, AM2, AM1>(p, lut, local - rs * p.KG, rs);
}

// ---------------------------------------------------------------------------------------
// Two activation vectors per pass (small batch, section 6).  The tables of BOTH vectors for
// one sub-slab (512 columns) fill the LDS, the two entries of a (slot, key) side by side:
// byte address  (L / 32) << 16 | key << 8 | (L % 32) << 3 | v << 2,  so that ONE 8-byte
// lookup returns the partial sums of both vectors (a wavefront's 64 lookups still fall in
// distinct banks: 32 lanes x 8 consecutive bytes per half).  The weights are streamed once
// per pair; lookups and table builds double per byte of weights, which is the limitation
// the paper states for growing batch.  K is split over "half tiles" (K tile, sub-slab);
// a unit is (half tile, row block).
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kPairDepth = 1;   // units fetched ahead in the pair kernel, where the registers allow

__device__ __forceinline__ f32x2 lds_f32x2(uint32_t byte_addr) {
  return *(const __attribute__((address_space(3))) f32x2*)(uintptr_t)byte_addr;
}

__device__ __forceinline__ void unpack_x(const u32x4& raw, bool live, float (&xs)[8]) {
  xs[0] = half_lo(raw.x); xs[1] = half_hi(raw.x);
  xs[2] = half_lo(raw.y); xs[3] = half_hi(raw.y);
  xs[4] = half_lo(raw.z); xs[5] = half_hi(raw.z);
  xs[6] = half_lo(raw.w); xs[7] = half_hi(raw.w);
#pragma unroll
  for (int j = 0; j < 8; ++j) xs[j] = live ? xs[j] : 0.0f;   // empty slot: an all-zero table
}

// Entries of keys [kh*32 + hi*16, +16) of one table (section 3.1), by doubling.
__device__ __forceinline__ void table_entries16(int kh, int hi, const float (&xs)[8], float (&e)[16]) {
  float base = -(xs[0] + xs[1] + xs[2] + xs[3]);
  base += hi ? xs[4] : -xs[4];
#pragma unroll
  for (int j = 5; j < 8; ++j) base += ((kh >> (j - 5)) & 1) ? xs[j] : -xs[j];
  e[0] = base;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float two_x = 2.0f * xs[j];
#pragma unroll
    for (int k = 0; k < (1 << j); ++k) e[k + (1 << j)] = e[k] + two_x;
  }
}

// The lookups of one (plane, row-of-four) step: the four dwords' key bytes, one 8-byte read each.
template <int Q, int I0, int QP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void pair_lookups(const Unit<Q, I0, QP, 1, AMODE, HAS_Z>& u, const uint32_t (&lane_base)[4],
                                             int step, f32x2 (&e)[4]) {
  const int i = step >> 2, rho = step & 3;
  // address bytes {0, L / 32, key byte rho, (L % 32) * 8}: lane_base holds bytes 0 and 2 (as its bytes 0 and 1)
  const uint32_t sel = 0x0c010000u | ((4u + rho) << 8);
#pragma unroll
  for (int s = 0; s < 4; ++s) e[s] = lds_f32x2(__builtin_amdgcn_perm(u.w[i][0][s], lane_base[s], sel));
}

// Software-pipelined by hand: the reads of step k + 1 are in flight while the additions of
// step k run (the scheduling barriers keep it so; left to itself the compiler waits for
// every read or two right after issuing them).
template <int Q, int I0, int QP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void accumulate_pair(const Unit<Q, I0, QP, 1, AMODE, HAS_Z>& u, const uint32_t (&lane_base)[4],
                                                const f32x2 (&sum_x)[4], float (&acc)[2][4]) {
  using U = Unit<Q, I0, QP, 1, AMODE, HAS_Z>;
  constexpr int kSteps = 4 * QP;
  // (with a scale set per dword the registers hold one step's reads only)
  constexpr int kAhead = (AMODE & 3) == kAlphaQuad ? 1 : 0;
  f32x2 e[kAhead + 1][4];
  if (kAhead) pair_lookups(u, lane_base, 0, e[0]);
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    if (step + kAhead < kSteps) pair_lookups(u, lane_base, step + kAhead, e[(step + kAhead) & kAhead]);
    __builtin_amdgcn_sched_barrier(0);
    const int i = step >> 2, rho = step & 3;
    const f32x2(&cur)[4] = e[step & kAhead];
    if ((AMODE & 3) == kAlphaQuad) {   // section 3.2 rule 2: one scale per run of lookups
      const f32x2 run = (cur[0] + cur[1]) + (cur[2] + cur[3]);
      const float a = scale_of<AMODE>(u.al[0][0], i, I0 + i, rho);
      acc[0][rho] = fmaf(a, run.x, acc[0][rho]);
      acc[1][rho] = fmaf(a, run.y, acc[1][rho]);
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float a = scale_of<AMODE>(u.al[s][0], i, I0 + i, rho);
        acc[0][rho] = fmaf(a, cur[s].x, acc[0][rho]);
        acc[1][rho] = fmaf(a, cur[s].y, acc[1][rho]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (HAS_Z && I0 == 0) {   // offset term of eq. 3
#pragma unroll
    for (int s = 0; s < U::NS; ++s) {
      f32x2 sx = sum_x[s];
      if ((AMODE & 3) == kAlphaQuad) sx = (sum_x[0] + sum_x[1]) + (sum_x[2] + sum_x[3]);
#pragma unroll
      for (int rho = 0; rho < 4; ++rho) {
        const float zf = half_of(u.zz[s][0], rho);
        acc[0][rho] = fmaf(zf, sx.x, acc[0][rho]);
        acc[1][rho] = fmaf(zf, sx.y, acc[1][rho]);
      }
    }
  }
}

template <int Q, int I0, int PP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void pair_passes(const GemvParams& p, int64_t tile_base, int rb, int lane, const int (&grp)[4][1],
                                            const float* partial, int out_row, int tile_T, int t0,
                                            const uint32_t (&lane_base)[4], const f32x2 (&sum_x)[4], float (&acc)[2][4]) {
  constexpr int QP = (Q - I0 < PP) ? Q - I0 : PP;
  Unit<Q, I0, QP, 1, AMODE, HAS_Z> u;
  load_unit<true>(u, p, tile_base, rb, lane, grp, partial, out_row, false, tile_T, t0);
  accumulate_pair(u, lane_base, sum_x, acc);
  if constexpr (I0 + QP < Q)
    pair_passes<Q, I0 + QP, PP, AMODE, HAS_Z>(p, tile_base, rb, lane, grp, partial, out_row, tile_T, t0, lane_base, sum_x, acc);
}

// The activations lane L needs for the table build of half tile h (sub-slab h % 2 of K
// tile h / 2): the 8 halfs of its slot's chunk, of vector v.
__device__ __forceinline__ u32x4 pair_fetch_x(const GemvParams& p, int h, int v, int lane) {
  const int kt = h >> 1, t0 = h & 1;
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  const int tile_T = chunks_in_tile > 64 ? 2 : 1;
  const int chunk = min(tile_T * lane + t0, chunks_in_tile - 1);   // clamped: value unused if out of range
  return *reinterpret_cast<const u32x4*>(p.x + (int64_t)(128 * kt + chunk) * 8 + (int64_t)v * p.n);
}

// One workgroup, one half tile (kt, t0), row blocks [rb0, rb1).  kDepth as in tile_body.
// xraw0, xraw1: what pair_fetch_x returned for this half tile and the two vectors.
template <int Q, int AMODE, bool HAS_Z, int kDepth>
__device__ __forceinline__ void pair_tile_body(const GemvParams& p, float* lut, int kt, int t0, int rb0, int rb1,
                                               bool first_tile, const u32x4& xraw0, const u32x4& xraw1) {
  using U = Unit<Q, 0, Q, 1, AMODE, HAS_Z>;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));   // see tile_body
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  const int tile_T = chunks_in_tile > 64 ? 2 : 1;
  const int64_t tile_base = (int64_t)kt * p.RB * Q * 2048;
  const int out_row = 4 * (lane & 3) + ((lane & 4) ? 2 : 0) + ((lane & 8) ? 1 : 0);
  int grp[4][1];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int slot = (lane & ~3) | ((s + lane) & 3);
    grp[s][0] = group_of_chunk(p, 128 * kt + min(tile_T * slot + t0, chunks_in_tile - 1));
  }

  const int my_chunk = tile_T * lane + t0;   // the chunk of the slot whose tables this lane builds

  // planes fetched together: all up to four; beyond that half of them, or three where every
  // dword has a scale set of its own (a set is 2 * planes registers per dword)
  constexpr int PP = Q > 4 ? ((AMODE & 3) == kAlphaQuad ? (Q + 1) / 2 : 3) : Q;
  // Units fetched ahead (D): as many as the registers of a wavefront hold, up to kDepth.  A
  // unit is the key words plus a scale set (and offsets) per dword when the scales are not
  // shared by the quad.  A unit is only 1 KB per plane, so it takes two of them in flight
  // per wavefront to cover the memory latency at full bandwidth.
  constexpr int kScaleRegs = (AMODE & kAlphaShared) ? 2 : 2 * Q;   // per scale set
  constexpr int kUnitRegs = 4 * Q + ((AMODE & 3) == kAlphaQuad ? kScaleRegs : 4 * kScaleRegs + (HAS_Z ? 8 : 0));
  constexpr int kFit = (PP < Q || kUnitRegs > 30) ? 0 : (kUnitRegs > 24 ? 1 : 2);
  constexpr int D = kFit < kDepth ? kFit : kDepth;
  const int n_units = rb1 - rb0;
  const int u_clamp = n_units - 1;
  // Ring of D + 1 units; uid[k]: the unit (row block rb0 + uid) in slot k.  A wavefront starts
  // with units wave, wave + kWaves, ... and takes every further one from the queue.
  U u[D + 1];
  int uid[D + 1];
  if (PP == Q && threadIdx.x == 0) reinterpret_cast<int*>(lut + kQueueWord)[0] = (D > 0 ? D : 1) * kWaves;
#pragma unroll
  for (int k = 0; k <= D; ++k) uid[k] = wave + k * kWaves;
  if (PP == Q) {
#pragma unroll
    for (int k = 0; k < D; ++k)
      load_unit<true>(u[k], p, tile_base, rb0 + min(uid[k], u_clamp), lane, grp, nullptr, out_row, false, tile_T, t0);
  }

  // ---- tables: build slot b (of 16) = 16 keys [32 * (b % 8) + 16 * (b / 8), +16) of both vectors ----
  {
    float xa[8], xb[8];
    unpack_x(xraw0, my_chunk < chunks_in_tile, xa);
    unpack_x(xraw1, my_chunk < chunks_in_tile, xb);
    f32x2* dst = reinterpret_cast<f32x2*>(lut) + ((lane >> 5) << 13) + (lane & 31);
    const int kh = wave & 7, hi = wave >> 3;   // 16 slots, 16 wavefronts
    float ea[16], eb[16];
    table_entries16(kh, hi, xa, ea);
    table_entries16(kh, hi, xb, eb);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      f32x2 e;
      e.x = ea[k];
      e.y = eb[k];
      dst[(kh * 32 + hi * 16 + k) << 5] = e;
    }
  }
  __syncthreads();

  uint32_t lane_base[4];
  f32x2 sum_x[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t slot = ((uint32_t)lane & ~3u) | ((uint32_t)(s + lane) & 3u);
    lane_base[s] = ((slot & 31u) << 3) | ((slot >> 5) << 8);
    f32x2 zero;
    zero.x = 0.0f;
    zero.y = 0.0f;
    sum_x[s] = HAS_Z ? lds_f32x2(((slot >> 5) << 16) | (0xffu << 8) | ((slot & 31u) << 3)) : zero;
  }

  // Each of a unit's two results (one per vector) is in all four 16-lane groups after the
  // reduction: lanes 0..15 add vector 0's, lanes 16..31 vector 1's to the running sums.
  const int run_vec = (lane >> 4) & 1;
  float* const run_lane = lut + kRunWord + run_vec * 16 + out_row;
  if constexpr (PP < Q) {
    for (int rb = rb0 + wave; rb < rb1; rb += kWaves) {
      float acc[2][4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
      pair_passes<Q, 0, PP, AMODE, HAS_Z>(p, tile_base, rb, lane, grp, nullptr, out_row, tile_T, t0, lane_base, sum_x, acc);
      int row_in_block;
      const float s0 = quad_rows_reduce(acc[0], lane, &row_in_block);
      const float s1 = quad_rows_reduce(acc[1], lane, &row_in_block);
      if (lane < 32) {
        float* r = run_lane + (rb - rb0) * 32;
        const float s = run_vec ? s1 : s0;
        *r = first_tile ? s : *r + s;
      }
    }
  } else {
    // Dynamic unit queue (see tile_body), D units fetched ahead, D + 1 units per pass of the
    // loop, ONE loop exit at the bottom: an exit in mid-loop would give the compiler a path
    // that carries an unused fetch back to the loop head, and with it a wait for all memory
    // traffic on every pass.  A wavefront that finds the queue empty part way through a pass
    // still fetches (the last unit, again) but skips the lookups.
    if (uid[0] >= n_units) return;
    do {
#pragma unroll
      for (int j = 0; j <= D; ++j) {
        constexpr int kRing = D + 1;
        const int fill = (j + D) % kRing;   // the slot consumed one pass of j ago (for D == 0: this one)
        if (D > 0) uid[fill] = next_unit(lut, lane);
        load_unit<true>(u[fill], p, tile_base, rb0 + min(uid[fill], u_clamp), lane, grp, nullptr, out_row, false, tile_T, t0);
        __builtin_amdgcn_sched_barrier(0);   // the fetch stays ahead of the lookups below
        if (uid[j] < n_units) {
          float acc[2][4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
          accumulate_pair(u[j], lane_base, sum_x, acc);
          int row_in_block;
          const float s0 = quad_rows_reduce(acc[0], lane, &row_in_block);
          const float s1 = quad_rows_reduce(acc[1], lane, &row_in_block);
          if (lane < 32) {
            float* r = run_lane + uid[j] * 32;
            const float s = run_vec ? s1 : s0;
            *r = first_tile ? s : *r + s;
          }
        }
        if (D == 0) uid[0] = next_unit(lut, lane);
      }
    } while (uid[0] < n_units);
  }
}

// The running sums of NVEC vectors for row blocks [rb0, rb1), [block][vector][16 rows] in
// LDS, become the workgroup's partial sums in the workspace.
template <int NVEC>
__device__ __forceinline__ void flush_vector_sums(const GemvParams& p, const float* lut, int rb0, int rb1, float* partial) {
  __syncthreads();
  const int rows = (rb1 - rb0) * 16;
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));   // the store addresses are formed here, not kept in registers from the kernel's start on
#pragma unroll
  for (int v = 0; v < NVEC; ++v) {
    if (NVEC == 4 && v >= p.batch) continue;   // a quad launched for three vectors
    for (int i = tid; i < rows; i += kThreads)
      store_device_coherent(partial + v * p.vec_stride + rb0 * 16 + i, lut[kRunWord + ((i >> 4) * NVEC + v) * 16 + (i & 15)]);
  }
}

// p.NT counts HALF tiles here; half tile h is sub-slab h % 2 of K tile h / 2 (a last tile
// with one sub-slab contributes one half tile).  AM2 / AM1 as in the GEMV kernel.

// A workgroup walks its row range in stretches of at most kRunBlocks / 2 row blocks (one
// stretch, but for layers of more than 60,000 rows or so): the half tiles of its K group for
// one stretch, whose sums over those half tiles stand in LDS all the while (no trip through
// memory per half tile), then the stretch's sums go to the workspace as partial sums.
template <int Q, bool HAS_Z, int AM2, int AM1>
__global__ __launch_bounds__(kThreads) void lutgemm_pair_kernel(GemvParams p) {
  __shared__ float lut[kGemvLdsFloats];   // (the kernel's only LDS object: see gemv_workgroup)
  const int kg = blockIdx.x;
  const int rs = blockIdx.y;
  int rb0, rb1;
  row_range(p, rs, &rb0, &rb1);
  float* partial = p.partial + (int64_t)kg * p.kg_stride;
  const int lane = threadIdx.x & 63;
  constexpr int kStretch = kRunBlocks / 2;
  for (int s0 = rb0; s0 < rb1; s0 += kStretch) {
    const int s1 = min(s0 + kStretch, rb1);
    // (with quad-shared scales, which leave the registers for it, the activations of the
    // next half tile are fetched before the lookups of this one start)
    constexpr bool kAheadX = (AM2 & 3) == kAlphaQuad && (AM1 & 3) == kAlphaQuad;
    const int h_end = min((kg + 1) * p.TPG, p.NT);
    u32x4 xraw0 = {0u, 0u, 0u, 0u}, xraw1 = {0u, 0u, 0u, 0u};
    if (kAheadX) {
      xraw0 = pair_fetch_x(p, kg * p.TPG, 0, lane);
      xraw1 = pair_fetch_x(p, kg * p.TPG, 1, lane);
    }
    for (int h = kg * p.TPG; h < h_end; ++h) {
      // every lookup of the half tile before is done before its tables are overwritten (and
      // the stretch before has been copied out before its sums are)
      if (h > kg * p.TPG || s0 > rb0) __syncthreads();
      if (!kAheadX) {
        xraw0 = pair_fetch_x(p, h, 0, lane);
        xraw1 = pair_fetch_x(p, h, 1, lane);
      }
      u32x4 xnext0 = xraw0, xnext1 = xraw1;
      if (kAheadX) {
        const int hn = min(h + 1, h_end - 1);
        xnext0 = pair_fetch_x(p, hn, 0, lane);
        xnext1 = pair_fetch_x(p, hn, 1, lane);
      }
      const int kt = h >> 1, t0 = h & 1;
      if (min(128, p.nchunks - 128 * kt) > 64)
        pair_tile_body<Q, AM2, HAS_Z, kPairDepth>(p, lut, kt, t0, s0, s1, h == kg * p.TPG, xraw0, xraw1);
      else
        pair_tile_body<Q, AM1, HAS_Z, kPairDepth>(p, lut, kt, t0, s0, s1, h == kg * p.TPG, xraw0, xraw1);
      xraw0 = xnext0;
      xraw1 = xnext1;
    }
    flush_vector_sums<2>(p, lut, s0, s1, partial);
  }
  finish_row_range<2, (Q <= 4)>(p, lut, rs, rb0, rb1);
}

#include "lutgemm_quad.h"
#include "lutgemm_planes_mfma.h"

#if !defined(LUT_PART) || LUT_PART == 0
// Zero the arrival counters of a fresh workspace.
__global__ __launch_bounds__(256) void lutgemm_zero_counters_kernel(uint32_t* counters, int count) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count) counters[i] = 0u;
}
#endif

// Kernel handles as hipLaunchKernel takes them.  The kernel families are instantiated in
// separate translation units of this one source (-DLUT_PART=k compiles family k only, see
// build.py), so that a build uses several cores; without LUT_PART everything is one unit.
using GemvKernel = const void*;
#ifdef LUT_PART
#define LUT_HAS_PART(k) (LUT_PART == (k))
#else
#define LUT_HAS_PART(k) 1
#endif
}  // namespace

namespace lutgemm_parts {
// family: 0 = no offsets, 1 = offsets, 2 = shared-scale layout (always with offsets)
const void* gemv_family0(int q, int64_t g);
const void* gemv_family1(int q, int64_t g);
const void* gemv_family2(int q, int64_t g);
const void* pair_family0(int q, int64_t g);
const void* pair_family1(int q, int64_t g);
const void* pair_family2(int q, int64_t g);
const void* quad_family0(int q, int64_t g);
const void* quad_family1(int q, int64_t g);
const void* quad_family2(int q, int64_t g);
const void* planes_family(int q, bool has_z, int batch);
const void* dequant_family(int q, bool has_z, int batch);
const void* group_family0(int q, int64_t g);
const void* group_family1(int q, int64_t g);
const void* group_family2(int q, int64_t g);
}  // namespace lutgemm_parts

namespace {

template <bool HAS_Z, int AM2, int AM1>
GemvKernel pick_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<1, HAS_Z, AM2, AM1>);
    case 2: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<2, HAS_Z, AM2, AM1>);
    case 3: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<3, HAS_Z, AM2, AM1>);
    case 4: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<4, HAS_Z, AM2, AM1>);
    case 5: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<5, HAS_Z, AM2, AM1>);
    case 6: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<6, HAS_Z, AM2, AM1>);
    case 7: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<7, HAS_Z, AM2, AM1>);
    case 8: return reinterpret_cast<const void*>(lutgemm_gemv_kernel<8, HAS_Z, AM2, AM1>);
  }
  return nullptr;
}

template <bool HAS_Z, int SH>
GemvKernel pick_mode(int q, int64_t g) {
  if (g % 64 == 0) return pick_q<HAS_Z, kAlphaQuad | SH, kAlphaQuad | SH>(q);
  if (g % 32 == 0) return pick_q<HAS_Z, kAlphaSlotPair | SH, kAlphaQuad | SH>(q);
  if (g % 16 == 0) return pick_q<HAS_Z, kAlphaPerSlot | SH, kAlphaPerSlot | SH>(q);
  return pick_q<HAS_Z, kAlphaPerChunk | SH, kAlphaPerSlot | SH>(q);
}

// shared: the scale buffer is in the shared-scale layout (offsets are then always present)
GemvKernel pick_kernel(int q, bool has_z, bool shared, int64_t g) {
  if (shared) return lutgemm_parts::gemv_family2(q, g);
  return has_z ? lutgemm_parts::gemv_family1(q, g) : lutgemm_parts::gemv_family0(q, g);
}

template <bool HAS_Z, int AM2, int AM1>
GemvKernel pick_group_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<1, HAS_Z, AM2, AM1>);
    case 2: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<2, HAS_Z, AM2, AM1>);
    case 3: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<3, HAS_Z, AM2, AM1>);
    case 4: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<4, HAS_Z, AM2, AM1>);
    case 5: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<5, HAS_Z, AM2, AM1>);
    case 6: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<6, HAS_Z, AM2, AM1>);
    case 7: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<7, HAS_Z, AM2, AM1>);
    case 8: return reinterpret_cast<const void*>(lutgemm_gemv_group_kernel<8, HAS_Z, AM2, AM1>);
  }
  return nullptr;
}

template <bool HAS_Z, int SH>
GemvKernel pick_group_mode(int q, int64_t g) {   // as pick_mode, without the register-bound scale set per chunk
  if (g % 64 == 0) return pick_group_q<HAS_Z, kAlphaQuad | SH, kAlphaQuad | SH>(q);
  if (g % 32 == 0) return pick_group_q<HAS_Z, kAlphaSlotPair | SH, kAlphaQuad | SH>(q);
  if (g % 16 == 0) return pick_group_q<HAS_Z, kAlphaPerSlot | SH, kAlphaPerSlot | SH>(q);
  return nullptr;
}

GemvKernel pick_group_kernel(int q, bool has_z, bool shared, int64_t g) {
  if (shared) return lutgemm_parts::group_family2(q, g);
  return has_z ? lutgemm_parts::group_family1(q, g) : lutgemm_parts::group_family0(q, g);
}

// Pair kernel: a lane's dword is one chunk, so the per-chunk scale mode does not occur.
template <bool HAS_Z, int AM2, int AM1>
GemvKernel pick_pair_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_pair_kernel<1, HAS_Z, AM2, AM1>);
    case 2: return reinterpret_cast<const void*>(lutgemm_pair_kernel<2, HAS_Z, AM2, AM1>);
    case 3: return reinterpret_cast<const void*>(lutgemm_pair_kernel<3, HAS_Z, AM2, AM1>);
    case 4: return reinterpret_cast<const void*>(lutgemm_pair_kernel<4, HAS_Z, AM2, AM1>);
    case 5: return reinterpret_cast<const void*>(lutgemm_pair_kernel<5, HAS_Z, AM2, AM1>);
    case 6: return reinterpret_cast<const void*>(lutgemm_pair_kernel<6, HAS_Z, AM2, AM1>);
    case 7: return reinterpret_cast<const void*>(lutgemm_pair_kernel<7, HAS_Z, AM2, AM1>);
    case 8: return reinterpret_cast<const void*>(lutgemm_pair_kernel<8, HAS_Z, AM2, AM1>);
  }
  return nullptr;
}

template <bool HAS_Z, int SH>
GemvKernel pick_pair_mode(int q, int64_t g) {
  // quad mode needs the quad's four chunks of one sub-slab in one group: they span 56 columns
  // of an aligned 64 in a two-sub-slab tile, 32 columns in a one-sub-slab tile
  if (g % 64 == 0) return pick_pair_q<HAS_Z, kAlphaQuad | SH, kAlphaQuad | SH>(q);
  if (g % 32 == 0) return pick_pair_q<HAS_Z, kAlphaPerSlot | SH, kAlphaQuad | SH>(q);
  return pick_pair_q<HAS_Z, kAlphaPerSlot | SH, kAlphaPerSlot | SH>(q);
}

GemvKernel pick_pair_kernel(int q, bool has_z, bool shared, int64_t g) {
  if (shared) return lutgemm_parts::pair_family2(q, g);
  return has_z ? lutgemm_parts::pair_family1(q, g) : lutgemm_parts::pair_family0(q, g);
}

template <bool HAS_Z, int AM2, int AM1>
GemvKernel pick_quad_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_quad_kernel<1, HAS_Z, AM2, AM1>);
    case 2: return reinterpret_cast<const void*>(lutgemm_quad_kernel<2, HAS_Z, AM2, AM1>);
    case 3: return reinterpret_cast<const void*>(lutgemm_quad_kernel<3, HAS_Z, AM2, AM1>);
    case 4: return reinterpret_cast<const void*>(lutgemm_quad_kernel<4, HAS_Z, AM2, AM1>);
    case 5: return reinterpret_cast<const void*>(lutgemm_quad_kernel<5, HAS_Z, AM2, AM1>);
    case 6: return reinterpret_cast<const void*>(lutgemm_quad_kernel<6, HAS_Z, AM2, AM1>);
    case 7: return reinterpret_cast<const void*>(lutgemm_quad_kernel<7, HAS_Z, AM2, AM1>);
    case 8: return reinterpret_cast<const void*>(lutgemm_quad_kernel<8, HAS_Z, AM2, AM1>);
  }
  return nullptr;
}

template <bool HAS_Z, int SH>
GemvKernel pick_quad_mode(int q, int64_t g) {   // a lane's dwords are chunks of one sub-slab, as in the pair kernel
  if (g % 64 == 0) return pick_quad_q<HAS_Z, kAlphaQuad | SH, kAlphaQuad | SH>(q);
  if (g % 32 == 0) return pick_quad_q<HAS_Z, kAlphaPerSlot | SH, kAlphaQuad | SH>(q);
  return pick_quad_q<HAS_Z, kAlphaPerSlot | SH, kAlphaPerSlot | SH>(q);
}

GemvKernel pick_quad_kernel(int q, bool has_z, bool shared, int64_t g) {
  if (shared) return lutgemm_parts::quad_family2(q, g);
  return has_z ? lutgemm_parts::quad_family1(q, g) : lutgemm_parts::quad_family0(q, g);
}

int compute_units_of_device() {
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

// Tuning overrides for sweeps (environment variables, read once per process; 0 = unset):
// LUTGEMM_TPG / LUTGEMM_RS, LUTGEMM_PAIR_TPG / _RS, LUTGEMM_QUAD_TPG / _RS (K tiles per group,
// row ranges of the three lookup kernels), LUTGEMM_MFMA_TPG.
struct Tuning {
  int tpg[3], rs[3];   // by kernel: GEMV, pair, quad
  int mfma_tpg;
};
const Tuning& tuning() {
  static const Tuning t = [] {
    auto env = [](const char* name) {
      const char* v = getenv(name);
      return v ? atoi(v) : 0;
    };
    Tuning r;
    r.tpg[0] = env("LUTGEMM_TPG");
    r.rs[0] = env("LUTGEMM_RS");
    r.tpg[1] = env("LUTGEMM_PAIR_TPG");
    r.rs[1] = env("LUTGEMM_PAIR_RS");
    r.tpg[2] = env("LUTGEMM_QUAD_TPG");
    r.rs[2] = env("LUTGEMM_QUAD_RS");
    r.mfma_tpg = env("LUTGEMM_MFMA_TPG");
    return r;
  }();
  return t;
}

// How the GEMV kernel of a (q, g) layer carries row sums from tile to tile of a K group: the
// variants that fetch a unit in one piece keep them in LDS, which bounds the row range of a
// workgroup; the register-bound one (a scale set per chunk: g % 16 != 0) sends them through
// the workspace.
bool carries_in_lds(int64_t g) { return g % 16 == 0; }

// Workgroup grid: KG groups of TPG consecutive K tiles times row_splits row ranges, one
// workgroup per compute unit.  Cost model in units of one round of units of a workgroup (16
// units, one per wavefront: about 4 us when the whole device streams), fitted to twelve layer
// shapes (OPT-13B, OPT-175B, LLaMA-65B) timed with weights that no cache holds:
//   * per tile, the rounds of units of a row range (the queue lets the wavefronts share a
//     partly filled round once there are several; one or two rounds cost whole rounds) plus
//     0.6 rounds for the activations, the table build and the first fetch;
//   * per K group, the partial sums it writes and the last-arrival sum reads back, which grow
//     with the rows (0.13 rounds per group at 49152 rows), and a small charge per workgroup
//     column.
// With the running sums of a K group in LDS, two tiles per group beat one on the tall layers
// with 12 tiles (36864 and 49152 rows x 12288: 6 groups instead of 12), three beat one on
// 12288 x 49152; the small layers keep one tile per group.
// Most row ranges the GEMV kernel is given: at least eight units per workgroup.  (Layers too
// small to give every compute unit sixteen run faster on twice the workgroups with half the
// wavefronts fetching, the builders of the tile start only building: 5120 x 5120 at q = 4
// 9.6 -> 8.8 us, 4096 x 4096 8.0 -> 7.1, 1024 x 1024 5.6 -> 5.0; four units per workgroup
// are faster still below 2048 x 2048 and slower above.)
inline int max_row_ranges(int RB) { return (RB + kWaves / 2 - 1) / (kWaves / 2); }

void choose_grid(int cus, int NT, int RB, bool lds_carry, int* KG, int* TPG, int* RS) {
  double best = 1e30;
  const int max_rs = max_row_ranges(RB);
  for (int tpg = 1; tpg <= NT && tpg <= 8; ++tpg) {
    const int kg = (NT + tpg - 1) / tpg;
    int rs = cus / kg;
    rs = rs < 1 ? 1 : (rs > max_rs ? max_rs : rs);
    const int blocks = (RB + rs - 1) / rs;
    const double rounds = blocks >= 3 * kWaves ? (double)blocks / kWaves : (double)((blocks + kWaves - 1) / kWaves);
    const int tiles = (NT + kg - 1) / kg;
    if (lds_carry && tpg > 1 && blocks > kRunBlocks) continue;   // the running sums of a row range live in LDS
    // (the variants that carry sums through memory pay a round trip per tile on top)
    const double cost = tiles * (rounds + 0.6) + 0.03 * kg + 0.13 * kg * (RB / 3072.0) + (lds_carry ? 0.0 : 0.3 * (tpg - 1));
    if (cost < best) {
      best = cost;
      *KG = kg;
      *TPG = tpg;
      *RS = rs;
    }
  }
}

// The same choice for the pair and quad kernels (NT counts half tiles or quarter ids, a
// row unit is a row block or a pair of them).  Their running sums stay in LDS for the whole
// K group, so a K group costs its partial sums once.  Cost in rounds of units of a workgroup,
// fitted to twelve layer shapes (OPT-13B, OPT-175B, LLaMA-65B) at batch 2 and 4, every tiles-
// per-group count from 1 to 8 (16) timed: per half tile or quarter the rounds of units (the
// queue shares a partly filled round out, but one round is the least) plus the table build;
// the last-arrival sum, which ONE workgroup per row range does, by the partial sums a thread
// of it loads; and a charge per K group beyond a few (more partial sums to write, more
// workgroup columns).  The choice is within 2 % (quad) and 6 % (pair) of the best measured
// on every one of the twelve shapes.
void choose_vector_grid(int vectors, int cus, int NT, int row_units, int* KG, int* TPG, int* RS) {
  const bool quad = vectors == 4;
  const double build = quad ? 0.6 : 0.4, per_load = quad ? 0.01 : 0.005, per_group = quad ? 0.1 : 0.05;
  const int free_groups = quad ? 8 : 12, rows_per_unit = quad ? 32 : 16;
  double best = 1e30;
  const int max_rs = (row_units + kWaves - 1) / kWaves;
  for (int tpg = 1; tpg <= NT && tpg <= (quad ? 16 : 8); ++tpg) {
    const int kg = (NT + tpg - 1) / tpg;
    int rs = cus / kg;
    rs = rs < 1 ? 1 : (rs > max_rs ? max_rs : rs);
    const int units = (row_units + rs - 1) / rs;
    const double rounds = units > kWaves ? (double)units / kWaves : 1.0;
    const int tiles = (NT + kg - 1) / kg;
    const int loads = kg * ((vectors * rows_per_unit * units + kThreads - 1) / kThreads);
    const double cost = tiles * (rounds + build) + per_load * loads + per_group * (kg > free_groups ? kg - free_groups : 0);
    if (cost < best) {
      best = cost;
      *KG = kg;
      *TPG = tpg;
      *RS = rs;
    }
  }
}

// choose_grid plus the tuning overrides.
// vectors: 1 (GEMV kernel), 2 (pair kernel), 4 (quad kernel)
void plan_grid(int cus, int vectors, int q, int64_t g, GemvParams* p) {
  const int wgs = cus > 256 ? 256 : cus;
  const bool lds_carry = carries_in_lds(g);
  if (vectors == 4)
    choose_vector_grid(4, wgs, p->NT, (p->RB + 1) / 2, &p->KG, &p->TPG, &p->row_splits);
  else if (vectors == 2)
    choose_vector_grid(2, wgs, p->NT, p->RB, &p->KG, &p->TPG, &p->row_splits);
  else
    choose_grid(wgs, p->NT, p->RB, lds_carry, &p->KG, &p->TPG, &p->row_splits);
  const int which = vectors == 4 ? 2 : (vectors == 2 ? 1 : 0);
  const int tpg = tuning().tpg[which], rs = tuning().rs[which];
  const int row_units = vectors == 4 ? (p->RB + 1) / 2 : p->RB;
  const int max_rs = vectors == 1 ? max_row_ranges(row_units) : (row_units + kWaves - 1) / kWaves;
  if (tpg > 0) {
    p->TPG = tpg > p->NT ? p->NT : tpg;
    p->KG = (p->NT + p->TPG - 1) / p->TPG;
    p->row_splits = wgs / p->KG;
    p->row_splits = p->row_splits < 1 ? 1 : (p->row_splits > max_rs ? max_rs : p->row_splits);
  }
  if (rs > 0) p->row_splits = rs > 256 ? 256 : (rs > row_units ? row_units : rs);
  if (vectors == 1 && lds_carry && p->TPG > 1 && (p->RB + p->row_splits - 1) / p->row_splits > kRunBlocks) {
    // an override that the running sums in LDS do not cover: back to the chooser's own grid
    choose_grid(wgs, p->NT, p->RB, lds_carry, &p->KG, &p->TPG, &p->row_splits);
  }
}

constexpr size_t kCounterBytes = 32768;   // 32 activation vectors x 256 row ranges


template <bool HAS_Z, int NB>
GemvKernel pick_dequant_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<1, HAS_Z, NB, true>);
    case 2: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<2, HAS_Z, NB, true>);
    case 3: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<3, HAS_Z, NB, true>);
    case 4: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<4, HAS_Z, NB, true>);
    case 5: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<5, HAS_Z, NB, true>);
    case 6: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<6, HAS_Z, NB, true>);
    case 7: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<7, HAS_Z, NB, true>);
    case 8: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<8, HAS_Z, NB, true>);
  }
  return nullptr;
}

template <bool HAS_Z, int NB>
GemvKernel pick_planes_q(int q) {
  switch (q) {
    case 1: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<1, HAS_Z, NB>);
    case 2: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<2, HAS_Z, NB>);
    case 3: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<3, HAS_Z, NB>);
    case 4: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<4, HAS_Z, NB>);
    case 5: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<5, HAS_Z, NB>);
    case 6: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<6, HAS_Z, NB>);
    case 7: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<7, HAS_Z, NB>);
    case 8: return reinterpret_cast<const void*>(lutgemm_planes_mfma_kernel<8, HAS_Z, NB>);
  }
  return nullptr;
}

GemvKernel pick_planes_kernel(int q, bool has_z, int batch) { return lutgemm_parts::planes_family(q, has_z, batch); }

// Grid of the matrix-core kernel: K groups x row ranges.  A wavefront keeps the outputs of at
// most kPlanesMaxUnits row blocks in registers, which bounds the row range; few K groups keep
// the split-K partials (batch x rows x 4 bytes per group, written and read back) small
// against the weights.  Costs in microseconds, from measurement on the OPT-175B shapes: 2.7 per
// unit, 1.5 per tile, 6 per pass of workgroups over the device (sign table, first X tile,
// start-up), 5 TB/s for the partials, 3 for the final reduction.
void plan_planes_grid(int cus, int waves, int batch, GemvParams* p) {
  const int slots = cus > 256 ? 256 : cus;
  const int min_rs = (p->RB + kPlanesMaxUnits * waves - 1) / (kPlanesMaxUnits * waves);
  double best = 1e30;
  for (int tpg = 1; tpg <= p->NT; ++tpg) {
    const int kg = (p->NT + tpg - 1) / tpg;
    if (kg > 256) continue;
    int rs = slots / kg;
    rs = rs < min_rs ? min_rs : rs;
    rs = rs > p->RB ? p->RB : rs;
    const int blocks = (p->RB + rs - 1) / rs;
    const int units = (blocks + waves - 1) / waves;
    const int rounds = (kg * rs + slots - 1) / slots;           // passes of workgroups over the device
    const double partial_mb = kg > 1 ? (double)kg * p->RB * 16 * batch * 8 / 1e6 : 0.0;
    const double cost = rounds * (tpg * (units * 2.7 + 1.5) + 6.0) + partial_mb / 5.0 + (kg > 1 ? 3.0 : 0.0);
    if (cost < best) {
      best = cost;
      p->KG = kg;
      p->TPG = tpg;
      p->row_splits = rs;
    }
  }
}

}  // namespace

namespace lutgemm_parts {
#if LUT_HAS_PART(0)
const void* gemv_family0(int q, int64_t g) { return pick_mode<false, 0>(q, g); }
#endif
#if LUT_HAS_PART(1)
const void* gemv_family1(int q, int64_t g) { return pick_mode<true, 0>(q, g); }
#endif
#if LUT_HAS_PART(2)
const void* gemv_family2(int q, int64_t g) { return pick_mode<true, kAlphaShared>(q, g); }
#endif
#if LUT_HAS_PART(3)
const void* pair_family0(int q, int64_t g) { return pick_pair_mode<false, 0>(q, g); }
#endif
#if LUT_HAS_PART(4)
const void* pair_family1(int q, int64_t g) { return pick_pair_mode<true, 0>(q, g); }
#endif
#if LUT_HAS_PART(5)
const void* pair_family2(int q, int64_t g) { return pick_pair_mode<true, kAlphaShared>(q, g); }
#endif
#if LUT_HAS_PART(6)
const void* quad_family0(int q, int64_t g) { return pick_quad_mode<false, 0>(q, g); }
#endif
#if LUT_HAS_PART(7)
const void* quad_family1(int q, int64_t g) { return pick_quad_mode<true, 0>(q, g); }
#endif
#if LUT_HAS_PART(8)
const void* quad_family2(int q, int64_t g) { return pick_quad_mode<true, kAlphaShared>(q, g); }
#endif
#if LUT_HAS_PART(10)
const void* group_family0(int q, int64_t g) { return pick_group_mode<false, 0>(q, g); }
#endif
#if LUT_HAS_PART(11)
const void* group_family1(int q, int64_t g) { return pick_group_mode<true, 0>(q, g); }
#endif
#if LUT_HAS_PART(12)
const void* group_family2(int q, int64_t g) { return pick_group_mode<true, kAlphaShared>(q, g); }
#endif
#if LUT_HAS_PART(13)
const void* dequant_family(int q, bool has_z, int batch) {
  if (batch <= 16) return has_z ? pick_dequant_q<true, 1>(q) : pick_dequant_q<false, 1>(q);
  return has_z ? pick_dequant_q<true, 2>(q) : pick_dequant_q<false, 2>(q);
}
#endif
#if LUT_HAS_PART(9)
const void* planes_family(int q, bool has_z, int batch) {
  if (batch <= 16) return has_z ? pick_planes_q<true, 1>(q) : pick_planes_q<false, 1>(q);
  return has_z ? pick_planes_q<true, 2>(q) : pick_planes_q<false, 2>(q);
}
#endif
}  // namespace lutgemm_parts

#if LUT_HAS_PART(0)   // the entry points and the two small kernels: once per library
// ---------------------------------------------------------------------------------------
// Measurement aid: a kernel that only reads.  Every workgroup walks one contiguous share of
// the buffer front to back, the way a GEMV workgroup walks its share of the packed weights
// (16 bytes per lane, consecutive lanes on consecutive addresses, several fetches in flight
// per lane, nothing kept in the caches), and keeps an XOR of everything it saw, so that its
// rate is what this device delivers to a pure stream of that shape: the yardstick next to
// the nominal HBM figure.  (Measured: contiguous shares beat a grid-stride walk by 6 %,
// non-temporal loads beat plain ones by 12 %.)
constexpr int kProbeGroups = 2048;   // eight 256-thread workgroups per compute unit
constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;      // independent 16-byte fetches per lane

__global__ __launch_bounds__(kProbeThreads) void lutgemm_stream_read_kernel(const u32x4* src, int64_t n16, uint32_t* sink) {
  const int64_t share = (n16 + gridDim.x - 1) / gridDim.x;
  const int64_t begin = min(share * blockIdx.x, n16), end = min(begin + share, n16);
  u32x4 acc = {0u, 0u, 0u, 0u};
  int64_t i = begin + threadIdx.x;
  for (; i + (kProbeUnroll - 1) * kProbeThreads < end; i += kProbeUnroll * kProbeThreads) {
    u32x4 v[kProbeUnroll];
#pragma unroll
    for (int j = 0; j < kProbeUnroll; ++j) v[j] = __builtin_nontemporal_load(src + i + j * kProbeThreads);
#pragma unroll
    for (int j = 0; j < kProbeUnroll; ++j) acc ^= v[j];
  }
  for (; i < end; i += kProbeThreads) acc ^= __builtin_nontemporal_load(src + i);
  uint32_t w = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) w ^= (uint32_t)__shfl_xor((int)w, d, 64);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * (kProbeThreads / 64) + (threadIdx.x >> 6)] = w;
}

// The lookup kernels form LDS addresses as if their table array started at LDS address 0, which
// holds when that array is the kernel's only LDS object.  Verified on the host before the first
// launch of every kernel: its static LDS size must be exactly the array's (anything else in
// LDS would make it larger), else the call fails with LUTGEMM_EHIP instead of computing
// nonsense.
bool lds_layout_ok(const void* kernel, size_t table_array_bytes) {
  static std::mutex lock;
  static const void* verified[1024];
  static int n_verified = 0;
  std::lock_guard<std::mutex> guard(lock);
  for (int i = 0; i < n_verified; ++i)
    if (verified[i] == kernel) return true;
  hipFuncAttributes attr;
  if (hipFuncGetAttributes(&attr, kernel) != hipSuccess) return false;
  if (attr.sharedSizeBytes != table_array_bytes) return false;
  if (n_verified < 1024) verified[n_verified++] = kernel;
  return true;
}

// Shape-derived fields of a launch.
void fill_shape(GemvParams* p, int64_t m, int64_t n, int64_t gg) {
  p->m = (int)m;
  p->n = (int)n;
  p->RB = (int)((m + 15) / 16);
  p->nchunks = (int)(n / 8);
  p->NT = (p->nchunks + 127) / 128;
  p->NG = (int)(n / gg);
  p->g = (int)gg;
  p->g_shift = -1;
  for (int sh = 0; sh < 31; ++sh)
    if ((gg >> 3) == ((int64_t)1 << sh)) p->g_shift = sh;
}

extern "C" {

int lutgemm_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || !aligned16(workspace)) return LUTGEMM_EINVAL;
  if (workspace_bytes < kCounterBytes) return LUTGEMM_EWORKSPACE;
  uint32_t* counters = static_cast<uint32_t*>(workspace);
  int count = (int)(kCounterBytes / 4);
  void* args[] = {&counters, &count};
  if (hipLaunchKernel(reinterpret_cast<const void*>(lutgemm_zero_counters_kernel), dim3(count / 256), dim3(256), args,
                      0, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return LUTGEMM_EHIP;
  return LUTGEMM_OK;
}

int lutgemm_gemm(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !bits || !alpha || !y || !workspace) return LUTGEMM_EINVAL;
  if (m < 1 || n < 8 || n % 8 != 0 || q < 1 || q > 8 || g < 0 || batch < 1) return LUTGEMM_EINVAL;
  const int64_t gg = g == 0 ? n : g;
  if (gg % 8 != 0 || n % gg != 0) return LUTGEMM_EINVAL;
  if (!aligned16(x) || !aligned16(bits) || !aligned16(alpha) || !aligned16(z) || !aligned16(y) || !aligned16(workspace))
    return LUTGEMM_EINVAL;
  if (mu != 8 || batch > 32 || (flags & ~7u) != 0) return LUTGEMM_EUNSUPPORTED;
  if (m > (int64_t)1 << 30 || n > (int64_t)1 << 30) return LUTGEMM_EUNSUPPORTED;
  const bool shared = (flags & LUTGEMM_ALPHA_SHARED) != 0;
  if (shared && !z) return LUTGEMM_EINVAL;   // the shared-scale form always comes with offsets
  // Measured on MI355X (q = 3, thirteen layer shapes from 4096^2 to 49152 x 12288): the
  // lookup path costs less than two GEMVs per four vectors, the matrix-core path the same
  // for any batch up to 16; the lookup path wins up to four vectors (two on layers of at most
  // 2^25 weights), the two tie at five and six on the layers of more than 2^28 weights, and
  // the matrix cores win beyond.
  if ((flags & LUTGEMM_PATH_AUTO) != 0 && !shared && gg % 64 == 0 &&
      (batch >= 6 || (batch == 5 && m * n < (int64_t)1 << 28) || (batch >= 3 && m * n <= (int64_t)1 << 25)))
    return lutgemm_gemm_mfma(x, bits, alpha, z, y, q, g, mu, m, n, batch, flags & LUTGEMM_Y_F32, workspace,
                             workspace_bytes, hip_stream);
  const size_t need = lutgemm_workspace_bytes(m, n, q, g, mu, batch);
  if (need == 0) return LUTGEMM_EINVAL;
  if (workspace_bytes < need) return LUTGEMM_EWORKSPACE;

  const int cus = compute_units_of_device();
  if (cus <= 0) return LUTGEMM_EHIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  GemvParams p;
  p.bits = static_cast<const uint8_t*>(bits);
  p.alpha = static_cast<const __half*>(alpha);
  p.z = static_cast<const __half*>(z);
  fill_shape(&p, m, n, gg);
  p.y_f32 = (flags & LUTGEMM_Y_F32) ? 1 : 0;
  plan_grid(cus, 1, q, gg, &p);
  const int64_t m_pad = (int64_t)(p.RB + (p.RB & 1)) * 16;   // an even number of row blocks (the quad kernel works on pairs)
  p.kg_stride = m_pad * (batch + (batch % 4 == 3 ? 1 : 0));   // room for the dropped fourth vector of a quad of three

  GemvKernel kern = pick_kernel(q, z != nullptr, shared, gg);
  if (!kern) return LUTGEMM_EUNSUPPORTED;
  if (p.TPG > 1 && carries_in_lds(gg) && (p.RB + p.row_splits - 1) / p.row_splits > kRunBlocks)
    return LUTGEMM_EUNSUPPORTED;   // (never planned: the kernel's running sums would not fit)

  uint32_t* counters = static_cast<uint32_t*>(workspace);
  float* partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterBytes);
  p.vec_stride = m_pad;
  const size_t y_elem = p.y_f32 ? sizeof(float) : sizeof(__half);

  // Activation vectors four at a time (one stream of the weights per four), then a pair or a
  // single one; three left over go through the quad kernel as well, the fourth table set
  // repeating the third vector and its results being dropped (cheaper than a pair plus one).
  GemvParams pq = p, pp = p;
  GemvKernel quad_kern = nullptr, pair_kern = nullptr;
  if (batch >= 3) {
    pq.NT = 4 * p.NT;   // quarter ids; those a ragged last tile does not have are skipped by the kernel
    plan_grid(cus, 4, q, gg, &pq);
    quad_kern = pick_quad_kernel(q, z != nullptr, shared, gg);
    if (!quad_kern) return LUTGEMM_EUNSUPPORTED;
  }
  if (batch % 4 == 2) {
    const int last_chunks = p.nchunks - 128 * (p.NT - 1);
    pp.NT = 2 * (p.NT - 1) + (last_chunks > 64 ? 2 : 1);   // half tiles
    plan_grid(cus, 2, q, gg, &pp);
    pair_kern = pick_pair_kernel(q, z != nullptr, shared, gg);
    if (!pair_kern) return LUTGEMM_EUNSUPPORTED;
  }
  for (int b = 0; b < batch;) {
    const int left = batch - b;
    const int take = left >= 3 ? 4 : left;          // kernel width: 4, 2 or 1
    const int live = left >= 4 ? 4 : left;          // vectors it really computes
    GemvParams pb = take == 4 ? pq : (take == 2 ? pp : p);
    GemvKernel kb = take == 4 ? quad_kern : (take == 2 ? pair_kern : kern);
    pb.x = static_cast<const __half*>(x) + (int64_t)b * n;
    pb.partial = partials + (int64_t)b * m_pad;
    pb.counters = counters + (int64_t)b * 256;
    pb.y = static_cast<char*>(y) + (int64_t)b * m * y_elem;
    pb.batch = live;
    const int row_units = take == 4 ? (pb.RB + 1) / 2 : pb.RB;
    pb.range_base = row_units / pb.row_splits;
    pb.range_rem = row_units % pb.row_splits;
    void* args[] = {&pb};
    if (!lds_layout_ok(kb, (size_t)kGemvLdsFloats * sizeof(float)))
      return LUTGEMM_EHIP;
    if (hipLaunchKernel(kb, dim3(pb.KG, pb.row_splits), dim3(kThreads), args, 0,
                        stream) != hipSuccess)
      return LUTGEMM_EHIP;
    b += live;
  }
  return LUTGEMM_OK;
}

static int gemm_matrix_cores(bool dequant, const void* x, const void* bits, const void* alpha, const void* z, void* y,
                             int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !bits || !alpha || !y || !workspace) return LUTGEMM_EINVAL;
  if (m < 1 || n < 8 || n % 8 != 0 || q < 1 || q > 8 || g < 0 || batch < 1) return LUTGEMM_EINVAL;
  const int64_t gg = g == 0 ? n : g;
  if (gg % 8 != 0 || n % gg != 0) return LUTGEMM_EINVAL;
  if (!aligned16(x) || !aligned16(bits) || !aligned16(alpha) || !aligned16(z) || !aligned16(y) || !aligned16(workspace))
    return LUTGEMM_EINVAL;
  if (mu != 8 || batch > 32 || (flags & ~1u) != 0) return LUTGEMM_EUNSUPPORTED;
  if (gg % 64 != 0) return LUTGEMM_EUNSUPPORTED;   // a matrix-core step covers 64 columns of one group
  if (m > (int64_t)1 << 30 || n > (int64_t)1 << 30) return LUTGEMM_EUNSUPPORTED;
  const size_t need = lutgemm_workspace_bytes(m, n, q, g, mu, batch);
  if (need == 0) return LUTGEMM_EINVAL;
  if (workspace_bytes < need) return LUTGEMM_EWORKSPACE;

  const int cus = compute_units_of_device();
  if (cus <= 0) return LUTGEMM_EHIP;
  GemvParams p;
  p.x = static_cast<const __half*>(x);
  p.bits = static_cast<const uint8_t*>(bits);
  p.alpha = static_cast<const __half*>(alpha);
  p.z = static_cast<const __half*>(z);
  p.y = y;
  fill_shape(&p, m, n, gg);
  p.batch = batch;
  p.y_f32 = (flags & LUTGEMM_Y_F32) ? 1 : 0;
  const int waves = q > 4 ? 4 : 8;
  plan_planes_grid(cus, waves, batch, &p);
  {
    const int tpg = tuning().mfma_tpg;
    if (tpg > 0) {
      const int min_rs = (p.RB + kPlanesMaxUnits * waves - 1) / (kPlanesMaxUnits * waves);
      p.TPG = tpg > p.NT ? p.NT : tpg;
      p.KG = (p.NT + p.TPG - 1) / p.TPG;
      int rs = (cus > 256 ? 256 : cus) / p.KG;
      rs = rs < min_rs ? min_rs : rs;
      p.row_splits = rs > p.RB ? p.RB : rs;
    }
  }
  if (p.row_splits > 256 && p.KG > 1) return LUTGEMM_EUNSUPPORTED;   // 256 arrival counters per call
  const int64_t m_pad = (int64_t)(p.RB + (p.RB & 1)) * 16;
  p.kg_stride = m_pad * batch;
  p.vec_stride = m_pad;
  p.counters = static_cast<uint32_t*>(workspace);
  p.partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterBytes);
  GemvKernel kern = dequant ? lutgemm_parts::dequant_family(q, z != nullptr, batch) : pick_planes_kernel(q, z != nullptr, batch);
  if (!kern) return LUTGEMM_EUNSUPPORTED;
  if (p.row_splits > 65535) return LUTGEMM_EUNSUPPORTED;   // grid y
  p.range_base = p.RB / p.row_splits;
  p.range_rem = p.RB % p.row_splits;
  void* args[] = {&p};
  if (hipLaunchKernel(kern, dim3(p.KG, p.row_splits), dim3(waves * 64), args, 0,
                      static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return LUTGEMM_EHIP;
  return LUTGEMM_OK;
}

int lutgemm_gemm_mfma(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                      int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return gemm_matrix_cores(false, x, bits, alpha, z, y, q, g, mu, m, n, batch, flags, workspace, workspace_bytes, hip_stream);
}

int lutgemm_gemm_dequant_mfma(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                              int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  return gemm_matrix_cores(true, x, bits, alpha, z, y, q, g, mu, m, n, batch, flags, workspace, workspace_bytes, hip_stream);
}

int lutgemm_plan_grid(int64_t m, int64_t n, int q, int g, int vectors, int compute_units, int* out) {
  if (!out || m < 1 || n < 8 || n % 8 != 0 || m > (int64_t)1 << 30 || n > (int64_t)1 << 30) return LUTGEMM_EINVAL;
  if (q < 1 || q > 8 || g < 0) return LUTGEMM_EINVAL;
  const int64_t gg = g == 0 ? n : g;
  if (gg % 8 != 0 || n % gg != 0) return LUTGEMM_EINVAL;
  if (vectors != 1 && vectors != 2 && vectors != 4) return LUTGEMM_EINVAL;
  const int cus = compute_units > 0 ? compute_units : compute_units_of_device();
  if (cus <= 0) return LUTGEMM_EHIP;
  GemvParams p;
  p.RB = (int)((m + 15) / 16);
  p.nchunks = (int)(n / 8);
  p.NT = (p.nchunks + 127) / 128;
  if (vectors == 2) {
    const int last_chunks = p.nchunks - 128 * (p.NT - 1);
    p.NT = 2 * (p.NT - 1) + (last_chunks > 64 ? 2 : 1);
  } else if (vectors == 4) {
    p.NT = 4 * p.NT;
  }
  plan_grid(cus, vectors, q, gg, &p);
  out[0] = p.KG;
  out[1] = p.TPG;
  out[2] = p.row_splits;
  return LUTGEMM_OK;
}

int lutgemm_stream_read(const void* src, size_t bytes, void* sink, size_t sink_bytes, void* hip_stream) {
  if (!src || !sink || bytes == 0 || bytes % 16 != 0) return LUTGEMM_EINVAL;
  if (((uintptr_t)src & 15) != 0 || ((uintptr_t)sink & 3) != 0) return LUTGEMM_EINVAL;
  if (sink_bytes < (size_t)kProbeGroups * (kProbeThreads / 64) * 4) return LUTGEMM_EWORKSPACE;
  const u32x4* s = static_cast<const u32x4*>(src);
  int64_t n16 = (int64_t)(bytes / 16);
  uint32_t* out = static_cast<uint32_t*>(sink);
  void* args[] = {&s, &n16, &out};
  if (hipLaunchKernel(reinterpret_cast<const void*>(lutgemm_stream_read_kernel), dim3(kProbeGroups), dim3(kProbeThreads),
                      args, 0, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return LUTGEMM_EHIP;
  return LUTGEMM_OK;
}

int lutgemm_gemv(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  return lutgemm_gemm(x, bits, alpha, z, y, q, g, mu, m, n, 1, flags, workspace, workspace_bytes, hip_stream);
}

size_t lutgemm_group_workspace_bytes(const int64_t* m, const int64_t* n, int count, int q, int g, int mu) {
  if (!m || !n || count < 1 || count > kMaxGroup) return 0;
  size_t total = kCounterBytes;
  for (int i = 0; i < count; ++i) {
    const size_t one = lutgemm_workspace_bytes(m[i], n[i], q, g, mu, 1);
    if (one == 0) return 0;
    total += (one - kCounterBytes + 255) / 256 * 256;   // the layer's partial sums
  }
  return total;
}

int lutgemm_gemv_group(const void* const* x, const void* const* bits, const void* const* alpha, const void* const* z,
                       void* const* y, const int64_t* m, const int64_t* n, int count, int q, int g, int mu,
                       unsigned flags, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!x || !bits || !alpha || !y || !m || !n || !workspace || !aligned16(workspace)) return LUTGEMM_EINVAL;
  if (count < 1 || q < 1 || q > 8 || g < 0) return LUTGEMM_EINVAL;
  if (mu != 8 || count > kMaxGroup || (flags & ~3u) != 0) return LUTGEMM_EUNSUPPORTED;
  const bool shared = (flags & LUTGEMM_ALPHA_SHARED) != 0;
  if (shared && !z) return LUTGEMM_EINVAL;
  const int cus = compute_units_of_device();
  if (cus <= 0) return LUTGEMM_EHIP;

  GroupParams gp;
  gp.count = count;
  gp.first_wg[0] = 0;
  uint32_t* counters = static_cast<uint32_t*>(workspace);
  float* partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kCounterBytes);
  size_t used = kCounterBytes;
  int64_t g_first = -1;
  for (int i = 0; i < count; ++i) {
    if (!x[i] || !bits[i] || !alpha[i] || !y[i] || (z && !z[i])) return LUTGEMM_EINVAL;
    if (m[i] < 1 || n[i] < 8 || n[i] % 8 != 0) return LUTGEMM_EINVAL;
    if (m[i] > (int64_t)1 << 30 || n[i] > (int64_t)1 << 30) return LUTGEMM_EUNSUPPORTED;
    const int64_t gg = g == 0 ? n[i] : g;
    if (gg % 8 != 0 || n[i] % gg != 0) return LUTGEMM_EINVAL;
    // one kernel serves the group, and the kernel is chosen by how the group size divides a
    // quad's 64 columns: row-wise scales (g == 0) must put every layer in the same class
    const int64_t cls = gg % 64 == 0 ? 64 : (gg % 32 == 0 ? 32 : (gg % 16 == 0 ? 16 : 8));
    if (g_first < 0) g_first = cls;
    if (cls != g_first) return LUTGEMM_EUNSUPPORTED;
    if (!aligned16(x[i]) || !aligned16(bits[i]) || !aligned16(alpha[i]) || !aligned16(y[i]) || (z && !aligned16(z[i])))
      return LUTGEMM_EINVAL;
    GemvParams& p = gp.layer[i];
    p = GemvParams();
    p.x = static_cast<const __half*>(x[i]);
    p.bits = static_cast<const uint8_t*>(bits[i]);
    p.alpha = static_cast<const __half*>(alpha[i]);
    p.z = z ? static_cast<const __half*>(z[i]) : nullptr;
    p.y = y[i];
    fill_shape(&p, m[i], n[i], gg);
    p.y_f32 = (flags & LUTGEMM_Y_F32) ? 1 : 0;
    p.batch = 1;
    plan_grid(cus, 1, q, gg, &p);
    if (p.TPG > 1 && carries_in_lds(gg) && (p.RB + p.row_splits - 1) / p.row_splits > kRunBlocks)
      return LUTGEMM_EUNSUPPORTED;   // (never planned)
    if (p.row_splits > 256) return LUTGEMM_EUNSUPPORTED;   // 256 arrival counters per layer
    const int64_t m_pad = (int64_t)(p.RB + (p.RB & 1)) * 16;
    p.kg_stride = m_pad;
    p.vec_stride = m_pad;
    p.range_base = p.RB / p.row_splits;
    p.range_rem = p.RB % p.row_splits;
    p.counters = counters + (size_t)i * 256;
    p.partial = partials;
      const size_t one = lutgemm_workspace_bytes(m[i], n[i], q, g, mu, 1);
    if (one == 0) return LUTGEMM_EINVAL;
    const size_t part_bytes = (one - kCounterBytes + 255) / 256 * 256;
    partials += part_bytes / sizeof(float);
    used += part_bytes;
    const int64_t wgs = (int64_t)p.KG * p.row_splits;
    if (gp.first_wg[i] + wgs > (int64_t)1 << 30) return LUTGEMM_EUNSUPPORTED;
    gp.first_wg[i + 1] = gp.first_wg[i] + (int)wgs;
  }
  for (int i = count; i < kMaxGroup; ++i) gp.first_wg[i + 1] = gp.first_wg[count];
  if (workspace_bytes < used) return LUTGEMM_EWORKSPACE;
  const int64_t gg0 = g == 0 ? n[0] : g;
  GemvKernel kern = pick_group_kernel(q, z != nullptr, shared, gg0);
  if (!kern) return LUTGEMM_EUNSUPPORTED;
  if (!lds_layout_ok(kern, (size_t)kGemvLdsFloats * sizeof(float))) return LUTGEMM_EHIP;
  void* args[] = {&gp};
  if (hipLaunchKernel(kern, dim3(gp.first_wg[count]), dim3(kThreads), args, 0, static_cast<hipStream_t>(hip_stream)) !=
      hipSuccess)
    return LUTGEMM_EHIP;
  return LUTGEMM_OK;
}

// ---------------------------------------------------------------------------------------
// lutgemm_gemv for callers that cannot allocate: the workspace is a device array of this
// library.  `static_scratch` below is a host-side stand-in for the device array, not a device
// address: the address every device keeps of its own copy comes from hipGetSymbolAddress, once
// per device, and only that address is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];

// Device address of this device's copy of the array (nullptr on error), looked up at the
// first call on the device; that call also enqueues the zeroing of the arrival counters.
static void* static_scratch_of_device(hipStream_t stream, int* rc) {
  static std::mutex lock;
  static void* address[64] = {nullptr};
  *rc = LUTGEMM_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    *rc = LUTGEMM_EHIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> guard(lock);
  if (!address[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)) != hipSuccess || !ptr) {
      *rc = LUTGEMM_EHIP;
      return nullptr;
    }
    // the counters start at zero (a small fill kernel, so that the call may be captured)
    const int init = lutgemm_workspace_init(ptr, kStaticScratchBytes, stream);
    if (init != LUTGEMM_OK) {
      *rc = init;
      return nullptr;
    }
    address[dev] = ptr;
  }
  return address[dev];
}

int lutgemm_gemv_static(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                        int q, int g, int mu, int64_t m, int64_t n, unsigned flags, void* hip_stream) {
  const size_t need = lutgemm_workspace_bytes(m, n, q, g, mu, 1);
  if (need == 0) return mu != 8 && m >= 1 && n >= 8 ? LUTGEMM_EUNSUPPORTED : LUTGEMM_EINVAL;
  if (need > kStaticScratchBytes) return LUTGEMM_EWORKSPACE;   // the layer needs more than the array holds
  int rc = LUTGEMM_OK;
  void* scratch = static_scratch_of_device(static_cast<hipStream_t>(hip_stream), &rc);
  if (!scratch) return rc;
  return lutgemm_gemm(x, bits, alpha, z, y, q, g, mu, m, n, 1, flags, scratch, kStaticScratchBytes, hip_stream);
}

size_t lutgemm_static_scratch_bytes(void) { return kStaticScratchBytes; }

}  // extern "C"
#endif   // LUT_HAS_PART(0)
