// Plane-wise matrix-core path for small batches — included inside the anonymous namespace of
// lutgemm_device.hip (it uses GemvParams and the helpers defined there).
//
// Same result as the lookup path, y = sum_i A_i o (B_i . X) (section 3.2, eq. 3), but the
// binary planes go through the matrix cores instead of through tables of partial sums: every
// key byte is expanded to eight fp16 values of +-1 (two reads of a 16-entry table in LDS),
// B_i . X is accumulated per group on v_mfma_f32_16x16x32_f16 (products +-x are exact, the
// accumulation is fp32), and the group's scale multiplies the accumulator once per group
// (section 3.2 rule 2).  This is the alternative the paper's discussion of batch points to
// (section 6: with growing batch the table lookups become the limit): its cost does not grow
// with batch up to 16 vectors, so it overtakes the lookup path at a batch of three to six
// (small layers earlier).
//
// Work split: a workgroup owns a row range and a K group (a run of K tiles) and keeps the
// outputs of its row blocks in registers across the tiles of the group; K groups are combined
// as in the GEMV kernel (partials, arrival counter, last workgroup sums in group order), or
// not at all when there is one K group.  Group size must be a multiple of 64 columns.

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int Q>
struct PlanesCfg {
  static constexpr int kWavesM = Q > 4 ? 4 : 8;         // wavefronts per workgroup
  static constexpr int kThreadsM = kWavesM * 64;
  static constexpr int kMaxSeg = 17;                    // group segments a tile can touch (g >= 64)
  static constexpr int kStageBytes = Q * 2048;          // per wavefront: Q planes x 2 sub-slabs, as fetched
  static constexpr int kAlphaBytes = kMaxSeg * Q * 32;  // per wavefront: scales of one unit
  static constexpr int kZBytes = kMaxSeg * 32;          // per wavefront: offsets of one unit
  static constexpr int kAlphaPasses = (kAlphaBytes + 1023) / 1024;
};
constexpr int kPlanesMaxUnits = 3;   // row blocks per wavefront (outputs held in registers)

// LDS map (bytes): sign table | block sums | X tile | per-wavefront key / scale / offset staging
constexpr int kSignOff = 0;          // 16 nibbles x 32 copies x 8 B
constexpr int kBlkSumOff = 4096;     // 16 blocks x 32 vectors fp32
constexpr int kXOff = 6144;          // 128 chunks x (NB * 16) vectors x 16 B

template <int Q, int NB>
constexpr int planes_lds_bytes() {
  using C = PlanesCfg<Q>;
  return kXOff + 32768 * NB + C::kWavesM * (C::kStageBytes + C::kAlphaBytes + C::kZBytes);
}

// Raw data of one unit (K tile x row block) as fetched from memory.
template <int Q, bool HAS_Z>
struct PlanesRaw {
  u32x4 w[Q][2];
  u32x4 al[PlanesCfg<Q>::kAlphaPasses];
  u32x4 zz;
};

struct PlanesTile {
  int kt, chunks, T, nblk, G0, nseg;
  int64_t base;
};

__device__ __forceinline__ PlanesTile planes_tile_info(const GemvParams& p, int kt, int Q) {
  PlanesTile t;
  t.kt = kt;
  t.chunks = min(128, p.nchunks - 128 * kt);
  t.T = t.chunks > 64 ? 2 : 1;
  t.nblk = t.chunks / (4 * t.T);                         // blocks of 4 slots (32 * T columns)
  t.G0 = (1024 * kt) / p.g;
  t.nseg = (1024 * kt + t.chunks * 8 - 1) / p.g - t.G0 + 1;
  t.base = (int64_t)kt * p.RB * Q * 2048;
  return t;
}

template <int Q, bool HAS_Z>
__device__ __forceinline__ void planes_fetch(PlanesRaw<Q, HAS_Z>& r, const GemvParams& p, const PlanesTile& t, int rb,
                                             int lane) {
  using C = PlanesCfg<Q>;
  const u32x4* bp = reinterpret_cast<const u32x4*>(p.bits + t.base + (int64_t)rb * Q * t.T * 1024) + lane;
#pragma unroll
  for (int i = 0; i < Q; ++i) {
    r.w[i][0] = __builtin_nontemporal_load(bp + (i * t.T) * 64);
    if (t.T == 2) r.w[i][1] = __builtin_nontemporal_load(bp + (i * 2 + 1) * 64);
  }
  // the unit's scales are one contiguous block: [segment][quarter][plane][4 rows] fp16
  const unsigned char* ap = reinterpret_cast<const unsigned char*>(p.alpha + ((int64_t)rb * p.NG + t.G0) * 16 * Q);
  const int abytes = t.nseg * Q * 32;
#pragma unroll
  for (int k = 0; k < C::kAlphaPasses; ++k) {
    const int off = (k * 64 + lane) * 16;
    if (off < abytes) r.al[k] = *reinterpret_cast<const u32x4*>(ap + off);
  }
  if (HAS_Z) {
    const unsigned char* zp = reinterpret_cast<const unsigned char*>(p.z + ((int64_t)rb * p.NG + t.G0) * 16);
    if (lane * 16 < t.nseg * 32) r.zz = *reinterpret_cast<const u32x4*>(zp + lane * 16);
  }
}

// Copy a fetched unit into this wavefront's LDS staging area.  The key slabs are stored as
// they lie in memory (slab (plane, sub-slab) at dword (plane * 2 + sub-slab) * 256, lane L's
// four dwords at 4 * L): one 16-byte store per slab and lane, free of bank conflicts.  The
// key of (row r, slot 4j + c) is then byte r % 4 of the dword at
// 16 * j + 4 * (r / 4) + (c - r / 4) mod 4 of the slab: a per-lane constant plus 16 * j.
template <int Q, bool HAS_Z>
__device__ __forceinline__ void planes_stage(const PlanesRaw<Q, HAS_Z>& r, const PlanesTile& t, int lane,
                                             uint32_t* stage, unsigned char* astage, unsigned char* zstage) {
  using C = PlanesCfg<Q>;
#pragma unroll
  for (int i = 0; i < Q; ++i)
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
      if (tt < t.T) *reinterpret_cast<u32x4*>(stage + (i * 2 + tt) * 256 + lane * 4) = r.w[i][tt];
  const int abytes = t.nseg * Q * 32;
#pragma unroll
  for (int kk = 0; kk < C::kAlphaPasses; ++kk) {
    const int off = (kk * 64 + lane) * 16;
    if (off < abytes) *reinterpret_cast<u32x4*>(astage + off) = r.al[kk];
  }
  if (HAS_Z && lane * 16 < t.nseg * 32) *reinterpret_cast<u32x4*>(zstage + lane * 16) = r.zz;
}

// One unit: all planes, all blocks of the tile; fin[nb][r] += contribution of this tile to
// row 4 * (lane / 16) + r of the block for activation vector nb * 16 + lane % 16.
// The key words of four blocks are read from the staging area in one go; then, block by
// block: key byte -> two sign-table reads -> matrix-core instructions, fully unrolled.  The
// scales of a group are read when the group starts and used when it ends.  (The path is
// bound by LDS bandwidth: 16 bytes of +-1 values per lane and matrix-core instruction.)
template <int Q, int NB, int T>
struct PlanesOperands {
  f16x8 a[T][Q];    // +-1 rows of the planes
  f16x8 b[T][NB];   // activations
};

template <int Q, int NB, int T>
__device__ __forceinline__ void planes_issue(PlanesOperands<Q, NB, T>& o, const uint32_t (&kd)[Q][T][4], int jj, int j,
                                             int key_shift, const u32x2* my_sign, const f16x8* my_x) {
  constexpr int NB16 = NB * 16;
#pragma unroll
  for (int tt = 0; tt < T; ++tt) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) o.b[tt][nb] = my_x[(T * 4 * j + tt) * NB16 + nb * 16];
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      // two 8-byte reads (low and high nibble of the key), each from this lane's own copy of
      // the 16-entry table: no two lanes of a pass share a bank
      const uint32_t key = kd[i][tt][jj] >> key_shift;
      const u32x2 lo = my_sign[(key & 15u) * 32];
      const u32x2 hi = my_sign[((key >> 4) & 15u) * 32];
      o.a[tt][i] = __builtin_bit_cast(f16x8, u32x4{lo.x, lo.y, hi.x, hi.y});
    }
  }
}

// The dequantising variant of planes_compute (DQ): the comparison kernel the small-batch
// workload names and the kind of kernel the paper's section 2.2 / section 4 discuss as
// dequantisation-based.  The +-1 operands of the planes are combined, in packed fp16
// arithmetic, into the fp16 weights  What = sum_i alpha_i b_i + z  of the lane's operand row
// (eq. 3), and ONE matrix-core instruction per 32 columns multiplies them with the
// activations, accumulating straight into the outputs.  The fp16 rounding of What costs about
// 3e-4 relative error in y, which the plane-wise form does not have.
template <int Q, bool HAS_Z, int NB, int T>
__device__ __forceinline__ void dequant_compute(const GemvParams& p, const PlanesTile& t, int lane, const u32x2* sign,
                                                const f16x8* Xs, const uint32_t* stage, const unsigned char* astage,
                                                const unsigned char* zstage, f32x4 (&fin)[NB]) {
  constexpr int NB16 = NB * 16;
  const int sub = lane >> 4;        // slot within the block
  const int col = lane & 15;        // row supplied to the A operand / activation vector of the outputs
  const int key_shift = 8 * (col & 3);
  const uint32_t* my_stage = stage + 4 * (col >> 2) + ((sub - (col >> 2)) & 3);
  const u32x2* my_sign = sign + (lane & 31);
  const f16x8* my_x = Xs + (T * sub) * NB16 + col;
  // scales and offset of the lane's OPERAND row (row `col` of the block) in group segment seg:
  // staging layout [segment][quarter of 4 rows][plane][4 rows] fp16, offsets [segment][16 rows]
  const unsigned char* my_alpha = astage + (col >> 2) * Q * 8 + (col & 3) * 2;
  const unsigned char* my_z = zstage + col * 2;
  f16x8 a8[Q], z8;
  auto load_scales = [&](int seg) {
#pragma unroll
    for (int i = 0; i < Q; ++i) {
      const _Float16 h = *reinterpret_cast<const _Float16*>(my_alpha + (seg * 4 * Q + i) * 8);
      a8[i] = f16x8{h, h, h, h, h, h, h, h};
    }
    const _Float16 zh = HAS_Z ? *reinterpret_cast<const _Float16*>(my_z + seg * 32) : (_Float16)0.0f;
    z8 = f16x8{zh, zh, zh, zh, zh, zh, zh, zh};
  };
  int seg = 0;
  const int seg_blocks = p.g / (32 * T);
  int left = (p.g - (1024 * t.kt) % p.g) / (32 * T);   // blocks until the first group ends
  load_scales(0);
#pragma unroll 1
  for (int j0 = 0; j0 < t.nblk; j0 += 4) {
    uint32_t kd[Q][T][4];
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
      for (int tt = 0; tt < T; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) kd[i][tt][jj] = my_stage[i * 512 + (tt * 16 + j0 + jj) * 16];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = j0 + jj;
      PlanesOperands<Q, NB, T> o;
      planes_issue<Q, NB, T>(o, kd, jj, j, key_shift, my_sign, my_x);
      if (j < t.nblk) {   // wave-uniform
#pragma unroll
        for (int tt = 0; tt < T; ++tt) {
          f16x8 w = z8;   // eq. 3 for eight columns of the operand row, rounded to fp16 at every step
#pragma unroll
          for (int i = 0; i < Q; ++i) w = o.a[tt][i] * a8[i] + w;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) fin[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(w, o.b[tt][nb], fin[nb], 0, 0, 0);
        }
        --left;
        if (left == 0 && j != t.nblk - 1) {   // wave-uniform: the next block starts a new group
          left = seg_blocks;
          seg = min(seg + 1, t.nseg - 1);
          load_scales(seg);
        }
      }
    }
  }
}

template <int Q, bool HAS_Z, int NB, int T>
__device__ __forceinline__ void planes_compute(const GemvParams& p, const PlanesTile& t, int lane, const u32x2* sign,
                                               const float* blksum, const f16x8* Xs, const uint32_t* stage,
                                               const unsigned char* astage, const unsigned char* zstage,
                                               f32x4 (&fin)[NB]) {
  constexpr int NB16 = NB * 16;
  const int sub = lane >> 4;        // slot within the block / quarter of the output rows
  const int col = lane & 15;        // row supplied to the A operand / activation vector of the outputs
  const int key_shift = 8 * (col & 3);
  f32x4 acc[Q][NB];
  float sx[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    sx[nb] = 0.0f;
#pragma unroll
    for (int i = 0; i < Q; ++i) acc[i][nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  }
  const uint32_t* my_stage = stage + 4 * (col >> 2) + ((sub - (col >> 2)) & 3);   // (row col, slot sub) of block 0
  const u32x2* my_sign = sign + (lane & 31);
  const f16x8* my_x = Xs + (T * sub) * NB16 + col;
  const unsigned char* my_alpha = astage + sub * Q * 8;
  const unsigned char* my_z = zstage + sub * 8;
  int seg = 0;                      // group segment of the current block, relative to t.G0
  // group ends are counted in blocks (no division in the loop): g is a multiple of the 64
  // columns of a block pair, and so is the distance from the tile's first column to a group end
  const int seg_blocks = p.g / (32 * T);
  int left = (p.g - (1024 * t.kt) % p.g) / (32 * T);   // blocks until the first group ends
  u32x2 a4[Q], z4;                  // scales / offsets of segment `seg` for this lane's four rows
#pragma unroll
  for (int i = 0; i < Q; ++i) a4[i] = *reinterpret_cast<const u32x2*>(my_alpha + i * 8);
  if (HAS_Z) z4 = *reinterpret_cast<const u32x2*>(my_z);

#pragma unroll 1
  for (int j0 = 0; j0 < t.nblk; j0 += 4) {
    uint32_t kd[Q][T][4];
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
      for (int tt = 0; tt < T; ++tt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) kd[i][tt][jj] = my_stage[i * 512 + (tt * 16 + j0 + jj) * 16];
    // Operands of the next block are read while the current block is on the matrix cores,
    // where two sets of operands fit the registers (few planes); otherwise block by block.
    constexpr bool kAhead = Q * NB <= 3;
    PlanesOperands<Q, NB, T> ops[kAhead ? 2 : 1];
    if (kAhead) planes_issue<Q, NB, T>(ops[0], kd, 0, j0, key_shift, my_sign, my_x);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = j0 + jj;
      // (blocks past the end of a ragged tile read stale but valid staging memory and are not used)
      if (kAhead) {
        if (jj < 3) planes_issue<Q, NB, T>(ops[(jj + 1) & 1], kd, jj + 1, j + 1, key_shift, my_sign, my_x);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        planes_issue<Q, NB, T>(ops[0], kd, jj, j, key_shift, my_sign, my_x);
      }
      if (j < t.nblk) {   // wave-uniform
        const PlanesOperands<Q, NB, T>& o = ops[kAhead ? (jj & 1) : 0];
#pragma unroll
        for (int tt = 0; tt < T; ++tt)
#pragma unroll
          for (int i = 0; i < Q; ++i)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[i][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(o.a[tt][i], o.b[tt][nb], acc[i][nb], 0, 0, 0);
        if (HAS_Z) {
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) sx[nb] += blksum[j * 32 + nb * 16 + col];
        }
        --left;
        if (j == t.nblk - 1 || left == 0) {   // wave-uniform: the group ends here (section 3.2 rule 2)
#pragma unroll
          for (int i = 0; i < Q; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float af = half_of(a4[i], r);
#pragma unroll
              for (int nb = 0; nb < NB; ++nb) fin[nb][r] = fmaf(af, acc[i][nb][r], fin[nb][r]);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
          }
          if (HAS_Z) {   // offset term of eq. 3
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float zf = half_of(z4, r);
#pragma unroll
              for (int nb = 0; nb < NB; ++nb) fin[nb][r] = fmaf(zf, sx[nb], fin[nb][r]);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) sx[nb] = 0.0f;
          }
          left = seg_blocks;
          seg = min(seg + 1, t.nseg - 1);   // the next group's scales, used when that group ends
#pragma unroll
          for (int i = 0; i < Q; ++i) a4[i] = *reinterpret_cast<const u32x2*>(my_alpha + (seg * 4 * Q + i) * 8);
          if (HAS_Z) z4 = *reinterpret_cast<const u32x2*>(my_z + seg * 32);
        }
      }
    }
  }
}

// Sum over the K groups and store for all (activation vector, row) pairs of a row range,
// spread evenly over the threads: E pairs per thread per pass, KB groups per pair per batch
// (E * KB independent loads in flight per thread; addresses clamped, not predicated, so KB
// follows the group count).  The sum over the groups always runs in ascending group order.
template <int THREADS, int E, int KB>
__device__ __forceinline__ void reduce_rows_batch(const GemvParams& p, int rb0, int row_end) {
  const int rows = row_end - rb0 * 16;
  const int total = rows * p.batch;
  for (int e0 = threadIdx.x; e0 < total; e0 += E * THREADS) {
    const float* src[E];
    int64_t dst[E];
    float sum[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const int e = min(e0 + j * THREADS, total - 1);
      const int vec = e / rows, r = rb0 * 16 + e % rows;
      src[j] = p.partial + (int64_t)vec * p.vec_stride + r;
      dst[j] = (int64_t)vec * p.m + r;
      sum[j] = 0.0f;
    }
    for (int kb = 0; kb < p.KG; kb += KB) {
      float v[E][KB];
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const int64_t off = (int64_t)min(kb + u, p.KG - 1) * p.kg_stride;
#pragma unroll
        for (int j = 0; j < E; ++j) v[j][u] = load_device_coherent(src[j] + off);
      }
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const bool live = kb + u < p.KG;
#pragma unroll
        for (int j = 0; j < E; ++j) sum[j] += live ? v[j][u] : 0.0f;
      }
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
      if (e0 + j * THREADS < total) {
        if (p.y_f32)
          static_cast<float*>(p.y)[dst[j]] = sum[j];
        else   // fp16 output, nearest even (paper table 1)
          static_cast<__half*>(p.y)[dst[j]] = __float2half_rn(sum[j]);
      }
    }
  }
}

// Cross-group reduction by the last workgroup to arrive for a row range (as in the GEMV
// kernel, with a run-time vector count and workgroup size).
template <int THREADS>
__device__ __forceinline__ void finish_rows_batch(const GemvParams& p, uint32_t* flag, int rs, int rb0, int rb1) {
  // the hand-off of finish_row_range: own stores acknowledged, barrier, arrival count
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t arrived = __hip_atomic_fetch_add(p.counters + rs, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag[0] = (arrived == (uint32_t)(p.KG - 1)) ? 1u : 0u;
  }
  __syncthreads();
  if (flag[0] == 0u) return;
  const int row_end = min(rb1 * 16, p.m);
  if (p.KG <= 2)
    reduce_rows_batch<THREADS, 8, 2>(p, rb0, row_end);
  else if (p.KG <= 4)
    reduce_rows_batch<THREADS, 4, 4>(p, rb0, row_end);
  else
    reduce_rows_batch<THREADS, 2, 8>(p, rb0, row_end);
  if (threadIdx.x == 0) __hip_atomic_store(p.counters + rs, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int Q, bool HAS_Z, int NB, bool DQ = false>
__global__ __launch_bounds__(PlanesCfg<Q>::kThreadsM) void lutgemm_planes_mfma_kernel(GemvParams p) {
  using C = PlanesCfg<Q>;
  constexpr int NB16 = NB * 16;
  constexpr int kThr = C::kThreadsM;
  __shared__ __attribute__((aligned(16))) unsigned char lds[planes_lds_bytes<Q, NB>()];
  u32x2* sign = reinterpret_cast<u32x2*>(lds + kSignOff);
  float* blksum = reinterpret_cast<float*>(lds + kBlkSumOff);
  u32x4* Xs = reinterpret_cast<u32x4*>(lds + kXOff);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char* wave_area = lds + kXOff + 32768 * NB + wave * (C::kStageBytes + C::kAlphaBytes + C::kZBytes);
  uint32_t* stage = reinterpret_cast<uint32_t*>(wave_area);
  unsigned char* astage = wave_area + C::kStageBytes;
  unsigned char* zstage = astage + C::kAlphaBytes;

  // nibble -> four fp16 values of +-1 (bit j set: +1), 32 copies side by side (one per lane of
  // an 8-byte read pass): entry (nibble, copy) at nibble * 256 + copy * 8 bytes
  for (int k = threadIdx.x; k < 512; k += kThr) {
    const int nib = k >> 5;
    const uint32_t one = 0x3C00u, minus_one = 0xBC00u;
    u32x2 e;
    e.x = ((nib & 1) ? one : minus_one) | (((nib & 2) ? one : minus_one) << 16);
    e.y = ((nib & 4) ? one : minus_one) | (((nib & 8) ? one : minus_one) << 16);
    sign[k] = e;
  }

  const int kg = blockIdx.x;
  const int rs = blockIdx.y;
  int rb0, rb1;
  row_range(p, rs, &rb0, &rb1);
  const int kt0 = kg * p.TPG;
  const int kt1 = min(kt0 + p.TPG, p.NT);

  // this wavefront's row blocks: rb0 + wave + u * waves, u < kPlanesMaxUnits (the host sizes
  // the row ranges accordingly)
  f32x4 fin[kPlanesMaxUnits][NB];
#pragma unroll
  for (int u = 0; u < kPlanesMaxUnits; ++u)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) fin[u][nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

  PlanesRaw<Q, HAS_Z> raw;
  if (kt0 < kt1 && rb0 + wave < rb1) {
    const PlanesTile t0 = planes_tile_info(p, kt0, Q);
    planes_fetch(raw, p, t0, rb0 + wave, lane);
  }
  // The X tile of the NEXT K tile is fetched into registers while the current tile is being
  // multiplied, so that a tile switch costs two barriers and an LDS write, not a trip to memory.
  constexpr int kXPerThread = 128 * NB16 / kThr;
  static_assert(128 * NB16 % kThr == 0, "X tile elements per thread");
  u32x4 xnext[kXPerThread];
  auto fetch_x_tile = [&](int kt) {
    const int chunks = min(128, p.nchunks - 128 * kt);
#pragma unroll
    for (int e = 0; e < kXPerThread; ++e) {
      const int idx = threadIdx.x + e * kThr;
      const int c = idx / NB16, n = idx % NB16;
      // clamped address, the load itself is unconditional; empty slots are zeroed when the
      // tile is written to LDS (no use of the value here: the fetch stays in flight)
      xnext[e] = *reinterpret_cast<const u32x4*>(p.x + (int64_t)min(n, p.batch - 1) * p.n +
                                                 (int64_t)(128 * kt + min(c, chunks - 1)) * 8);
    }
  };
  constexpr bool kAheadX = Q * NB <= 6;   // (more planes x vectors: no registers to hold the tile)
  if (kAheadX) fetch_x_tile(kt0);
  for (int kt = kt0; kt < kt1; ++kt) {
    const PlanesTile t = planes_tile_info(p, kt, Q);
    __syncthreads();   // the previous tile's X is no longer read (first pass: nothing to wait for)
    if (!kAheadX) fetch_x_tile(kt);
#pragma unroll
    for (int e = 0; e < kXPerThread; ++e) {
      const int idx = threadIdx.x + e * kThr;
      const int c = idx / NB16, n = idx % NB16;
      Xs[idx] = (c < t.chunks && n < p.batch) ? xnext[e] : u32x4{0u, 0u, 0u, 0u};
    }
    __syncthreads();
    if (kAheadX) fetch_x_tile(min(kt + 1, kt1 - 1));
    if (HAS_Z && !DQ) {   // sum of the activations of every block (the offset term needs it per group)
      for (int idx = threadIdx.x; idx < 16 * NB16; idx += kThr) {
        const int j = idx / NB16, n = idx % NB16;
        float s = 0.0f;
        for (int c = 4 * t.T * j; c < 4 * t.T * (j + 1); ++c) {
          const u32x4 v = Xs[c * NB16 + n];
          s += (half_lo(v.x) + half_hi(v.x)) + (half_lo(v.y) + half_hi(v.y)) + (half_lo(v.z) + half_hi(v.z)) +
               (half_lo(v.w) + half_hi(v.w));
        }
        blksum[j * 32 + n] = s;
      }
      __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < kPlanesMaxUnits; ++u) {
      const int rb = rb0 + wave + u * C::kWavesM;
      if (rb < rb1) {   // wave-uniform
        planes_stage(raw, t, lane, stage, astage, zstage);
        // fetch the next unit of this wavefront (same tile, else first row block of the next tile)
        const int rb_next = rb + C::kWavesM;
        if (u + 1 < kPlanesMaxUnits && rb_next < rb1) {
          planes_fetch(raw, p, t, rb_next, lane);
        } else if (kt + 1 < kt1) {
          const PlanesTile tn = planes_tile_info(p, kt + 1, Q);
          planes_fetch(raw, p, tn, rb0 + wave, lane);
        }
        if constexpr (DQ) {
          if (t.T == 2)
            dequant_compute<Q, HAS_Z, NB, 2>(p, t, lane, sign, reinterpret_cast<const f16x8*>(Xs), stage, astage, zstage,
                                             fin[u]);
          else
            dequant_compute<Q, HAS_Z, NB, 1>(p, t, lane, sign, reinterpret_cast<const f16x8*>(Xs), stage, astage, zstage,
                                             fin[u]);
        } else if (t.T == 2) {
          planes_compute<Q, HAS_Z, NB, 2>(p, t, lane, sign, blksum, reinterpret_cast<const f16x8*>(Xs), stage, astage,
                                          zstage, fin[u]);
        } else {
          planes_compute<Q, HAS_Z, NB, 1>(p, t, lane, sign, blksum, reinterpret_cast<const f16x8*>(Xs), stage, astage,
                                          zstage, fin[u]);
        }
      }
    }
  }

  // ---- outputs: row 4 * (lane / 16) + r of block rb, activation vector nb * 16 + lane % 16 ----
  const int sub = lane >> 4, col = lane & 15;
#pragma unroll
  for (int u = 0; u < kPlanesMaxUnits; ++u) {
    const int rb = rb0 + wave + u * C::kWavesM;
    if (rb < rb1) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int vec = nb * 16 + col;
        if (vec < p.batch) {
          const int row = rb * 16 + 4 * sub;
          if (p.KG == 1) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              if (row + r < p.m) {
                if (p.y_f32)
                  static_cast<float*>(p.y)[(int64_t)vec * p.m + row + r] = fin[u][nb][r];
                else   // fp16 output, nearest even (paper table 1)
                  static_cast<__half*>(p.y)[(int64_t)vec * p.m + row + r] = __float2half_rn(fin[u][nb][r]);
              }
            }
          } else {
            float* dst = p.partial + (int64_t)kg * p.kg_stride + (int64_t)vec * p.vec_stride + row;
#pragma unroll
            for (int r = 0; r < 4; ++r) store_device_coherent(dst + r, fin[u][nb][r]);
          }
        }
      }
    }
  }
  if (p.KG > 1) finish_rows_batch<kThr>(p, reinterpret_cast<uint32_t*>(lds), rs, rb0, rb1);
}
