// Four activation vectors per pass — included inside the anonymous namespace of
// lutgemm_device.hip (after the pair kernel, whose helpers it uses).
//
// Same method as the GEMV and pair kernels (section 3.1 tables, section 3.2 scale rule), for
// the small-batch case of section 6: the tables of FOUR vectors for one quarter of a K tile
// (32 slots = 256 columns of one sub-slab) fill the 128 KB of LDS, the four entries of a
// (slot, key) side by side at byte address  (L / 16) << 16 | key << 8 | (L % 16) << 4 | v << 2,
// so one 16-byte lookup returns the partial sums of all four vectors for a fetched key byte
// and one v_perm_b32 forms its address.  A 16-lane pass of such a lookup touches 16 distinct
// 16-byte columns: no bank conflicts for any keys.  The weights are streamed once per four
// vectors.
//
// A quarter uses 32 of the 64 lanes' worth of a 1 KB slab, so a wavefront works on TWO row
// blocks at once: lanes 0..31 on row block 2u, lanes 32..63 on row block 2u + 1, both on the
// same 32 slots.  A unit is (quarter, pair of row blocks).  K is split over quarters
// (id = 4 * tile + 2 * sub-slab + half); the sums over the quarters of a K group stand in
// LDS (as in the GEMV and pair kernels), split-K partials and the final reduction are those
// of the GEMV kernel, for four vectors.

typedef float f32x4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4v lds_f32x4(uint32_t byte_addr) {
  return *(const __attribute__((address_space(3))) f32x4v*)(uintptr_t)byte_addr;
}

// quad_rows_reduce for a 32-lane half: four per-lane values (rows 4k..4k+3, k = lane % 4) ->
// every lane holds the sum over the 8 quads of its half for ONE of its rows.
// IN_REGISTERS: the exchanges stay in registers (see halve_over_lane_bit2); the kernels that are short
// of registers (several fetches per unit) send them through the LDS crossbar instead.
template <bool IN_REGISTERS = true>
__device__ __forceinline__ float half_rows_reduce(const float (&acc)[4], int lane) {
  const bool b2 = lane & 4, b3 = lane & 8;
  if (IN_REGISTERS) {
    const float h0 = halve_over_lane_bit2(acc[0], acc[2], b2);
    const float h1 = halve_over_lane_bit2(acc[1], acc[3], b2);
    return sum_lane_xor16(halve_over_lane_bit3(h0, h1, b3));
  }
  const float keep0 = b2 ? acc[2] : acc[0], send0 = b2 ? acc[0] : acc[2];
  const float keep1 = b2 ? acc[3] : acc[1], send1 = b2 ? acc[1] : acc[3];
  const float h0 = keep0 + __shfl_xor(send0, 4);
  const float h1 = keep1 + __shfl_xor(send1, 4);
  const float keep = b3 ? h1 : h0, send = b3 ? h0 : h1;
  const float s = keep + dpp_f32<kDppRowRor8>(send);
  return s + __shfl_xor(s, 16);
}

// The lookups of one (plane, row-of-four) step: the four dwords' key bytes, one 16-byte read each.
template <int Q, int I0, int QP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void quad_lookups(const Unit<Q, I0, QP, 1, AMODE, HAS_Z>& u, const uint32_t (&lane_base)[4],
                                             int step, f32x4v (&e)[4]) {
  const int i = step >> 2, rho = step & 3;
  // address bytes {0, L / 16, key byte rho, (L % 16) * 16}: lane_base holds bytes 0 and 2 (as its bytes 0 and 1)
  const uint32_t sel = 0x0c010000u | ((4u + rho) << 8);
#pragma unroll
  for (int s = 0; s < 4; ++s) e[s] = lds_f32x4(__builtin_amdgcn_perm(u.w[i][0][s], lane_base[s], sel));
}

// The steps are software-pipelined by hand: the reads of step k + 1 are issued, then the
// additions of step k run while they are in flight (the scheduling barriers keep it so).
// Left to itself the compiler waits for every read or two right after issuing them, and the
// wavefronts of a compute unit then take turns at the LDS and at the vector ALU instead of
// using both at once.
template <int Q, int I0, int QP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void accumulate_quad(const Unit<Q, I0, QP, 1, AMODE, HAS_Z>& u, const uint32_t (&lane_base)[4],
                                                const f32x4v (&sum_x)[4], float (&acc)[4][4]) {
  using U = Unit<Q, I0, QP, 1, AMODE, HAS_Z>;
  constexpr int kSteps = 4 * QP;
  // (with a scale set per dword the registers hold one step's reads only)
  constexpr int kAhead = (AMODE & 3) == kAlphaQuad ? 1 : 0;
  f32x4v e[kAhead + 1][4];
  if (kAhead) quad_lookups(u, lane_base, 0, e[0]);
#pragma unroll
  for (int step = 0; step < kSteps; ++step) {
    if (step + kAhead < kSteps) quad_lookups(u, lane_base, step + kAhead, e[(step + kAhead) & kAhead]);
    __builtin_amdgcn_sched_barrier(0);
    const int i = step >> 2, rho = step & 3;
    const f32x4v(&cur)[4] = e[step & kAhead];
    if ((AMODE & 3) == kAlphaQuad) {   // section 3.2 rule 2: one scale per run of lookups
      const f32x4v run = (cur[0] + cur[1]) + (cur[2] + cur[3]);
      const float a = scale_of<AMODE>(u.al[0][0], i, I0 + i, rho);
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[v][rho] = fmaf(a, run[v], acc[v][rho]);
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float a = scale_of<AMODE>(u.al[s][0], i, I0 + i, rho);
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v][rho] = fmaf(a, cur[s][v], acc[v][rho]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (HAS_Z && I0 == 0) {   // offset term of eq. 3
#pragma unroll
    for (int s = 0; s < U::NS; ++s) {
      const f32x4v sx = sum_x[s];   // (quad-shared scales: the caller has put the sum over the four slots into sum_x[0])
#pragma unroll
      for (int rho = 0; rho < 4; ++rho) {
        const float zf = half_of(u.zz[s][0], rho);
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v][rho] = fmaf(zf, sx[v], acc[v][rho]);
      }
    }
  }
}

template <int Q, int I0, int PP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void quad_passes(const GemvParams& p, int64_t tile_base, int rb, int slab_lane,
                                            const int (&grp)[4][1], const float* partial, int out_row, int tile_T, int t0,
                                            const uint32_t (&lane_base)[4], const f32x4v (&sum_x)[4], float (&acc)[4][4]) {
  constexpr int QP = (Q - I0 < PP) ? Q - I0 : PP;
  Unit<Q, I0, QP, 1, AMODE, HAS_Z> u;
  load_unit<true>(u, p, tile_base, rb, slab_lane, grp, partial, out_row, false, tile_T, t0);
  accumulate_quad(u, lane_base, sum_x, acc);
  if constexpr (I0 + QP < Q)
    quad_passes<Q, I0 + QP, PP, AMODE, HAS_Z>(p, tile_base, rb, slab_lane, grp, partial, out_row, tile_T, t0, lane_base,
                                              sum_x, acc);
}

// Table build of a quarter: lane (sl = lane / 4, v = lane % 4) of wavefront b writes the keys
// [32 * (b / 2), +32) of vector v for slot 16 * (b % 2) + sl, i.e. the 64 lanes of a store
// write 64 consecutive floats (16 slots x 4 vectors of one key): no bank conflicts.  (A quad
// launched for three vectors builds the fourth table set from the third vector.)  The
// activations a lane needs for that: 8 halfs, fetched a quarter ahead.
__device__ __forceinline__ u32x4 quad_fetch_x(const GemvParams& p, int id, int wave, int lane) {
  const int kt = id >> 2, t0 = (id >> 1) & 1, h = id & 1;
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  const int tile_T = chunks_in_tile > 64 ? 2 : 1;
  const int chunk = tile_T * (32 * h + 16 * (wave & 1) + (lane >> 2)) + t0;
  const __half* xp = p.x + (int64_t)(128 * kt + min(chunk, chunks_in_tile - 1)) * 8;   // clamped: value unused if out of range
  return *reinterpret_cast<const u32x4*>(xp + (int64_t)min(lane & 3, p.batch - 1) * p.n);
}

// Does quarter `id` (4 * tile + 2 * sub-slab + half) exist?  Not in a ragged last tile
// whose sub-slab or half has no columns.
__device__ __forceinline__ bool quarter_exists(const GemvParams& p, int id) {
  const int kt = id >> 2, t0 = (id >> 1) & 1, h = id & 1;
  const int chunks = min(128, p.nchunks - 128 * kt);
  const int T = chunks > 64 ? 2 : 1;
  return t0 < T && 32 * h * T + t0 < chunks;
}

__device__ __forceinline__ int next_quarter(const GemvParams& p, int id, int id_end) {
  while (id < id_end && !quarter_exists(p, id)) ++id;
  return id;
}

// What a wavefront prepares for a quarter while the slower wavefronts of the workgroup are
// still busy with the quarter before (it would otherwise only wait for them at the barrier
// that frees the tables): the 32 table entries it will store, the groups of its dwords, and
// the fetch of its first unit.  After the barrier the entries are stored, a second barrier
// says that the tables stand, and the lookups start on a unit that has arrived meanwhile.
template <int Q, int AMODE, bool HAS_Z, bool AHEAD>
struct QuadQuarter {
  // planes fetched together: all up to four; beyond that half of them, or two where every
  // dword has a scale set of its own (16 accumulators leave fewer registers than in the
  // other kernels: three of eight planes even with quad-shared scales)
  static constexpr int PP = (AMODE & 3) == kAlphaQuad ? (Q > 4 ? (Q > 7 ? 3 : (Q + 1) / 2) : Q)
                                                      : ((Q > 4 || (Q >= 3 && HAS_Z)) ? 2 : Q);
  // AHEAD (the kernel's every tile has quad-shared scales): the first unit's fetch is part
  // of the preparation where a unit is fetched in one piece (a scale set per dword leaves no
  // registers for it)
  static constexpr bool kFirstUnit = AHEAD && PP == Q && (AMODE & 3) == kAlphaQuad;
  // ... and likewise the table entries and the next quarter's activations are only held
  // across the lookups and the barrier with quad-shared scales
  static constexpr bool kAheadTables = AHEAD && (AMODE & 3) == kAlphaQuad;
  int kt, t0, h, tile_T;
  int64_t tile_base;
  int grp[4][1];
  float entries[32];
  Unit<Q, 0, Q, 1, AMODE, HAS_Z> u;   // the wavefront's first unit (kFirstUnit)
};

template <int Q, int AMODE, bool HAS_Z, bool AHEAD>
__device__ __forceinline__ void quad_entries(QuadQuarter<Q, AMODE, HAS_Z, AHEAD>& qq, const GemvParams& p, int wave, int lane,
                                             const u32x4& xraw) {
  const int chunks_in_tile = min(128, p.nchunks - 128 * qq.kt);
  float xs[8];
  unpack_x(xraw, qq.tile_T * (32 * qq.h + 16 * (wave & 1) + (lane >> 2)) + qq.t0 < chunks_in_tile, xs);
#pragma unroll
  for (int hi = 0; hi < 2; ++hi) {
    float e[16];
    table_entries16(wave >> 1, hi, xs, e);
#pragma unroll
    for (int k = 0; k < 16; ++k) qq.entries[hi * 16 + k] = e[k];
  }
}

// rb0: first row block of the stretch (even), n_units: its pairs of row blocks.
template <int Q, int AMODE, bool HAS_Z, bool AHEAD>
__device__ __forceinline__ void quad_prepare(QuadQuarter<Q, AMODE, HAS_Z, AHEAD>& qq, const GemvParams& p, int id, int rb0,
                                             int n_units, int wave, int lane, const u32x4& xraw, bool with_entries) {
  qq.kt = id >> 2;
  qq.t0 = (id >> 1) & 1;
  qq.h = id & 1;
  const int chunks_in_tile = min(128, p.nchunks - 128 * qq.kt);
  qq.tile_T = chunks_in_tile > 64 ? 2 : 1;
  qq.tile_base = (int64_t)qq.kt * p.RB * Q * 2048;
  const int half = lane >> 5, lq = lane & 31;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int L = (lq & ~3) | ((s + lq) & 3);
    qq.grp[s][0] = group_of_chunk(p, 128 * qq.kt + min(qq.tile_T * (32 * qq.h + L) + qq.t0, chunks_in_tile - 1));
  }
  if constexpr (QuadQuarter<Q, AMODE, HAS_Z, AHEAD>::kFirstUnit) {
    // (unconditional: a wavefront without a unit fetches the last one and does not use it)
    const int rb = min(rb0 + 2 * min(wave, n_units - 1) + half, p.RB - 1);
    load_unit<true>(qq.u, p, qq.tile_base, rb, 32 * qq.h + lq, qq.grp, nullptr, 0, false, qq.tile_T, qq.t0);
  }
  if (with_entries) quad_entries(qq, p, wave, lane, xraw);
}

// One workgroup, the quarters [id, id_end) that exist (all of tiles with the same number of
// sub-slabs, hence one scale mode AMODE), row blocks [rb0, rb1) with rb0 even: a stretch of
// the workgroup's row range whose running sums fit LDS.  `first`: no quarter of the K group
// has been added to the running sums of this stretch yet (in and out); `fresh`: nothing in
// LDS is in use by other wavefronts when the call starts.
template <int Q, int AMODE, bool HAS_Z, bool AHEAD>
__device__ __forceinline__ void quad_quarters(const GemvParams& p, float* lut, int id, int id_end, int rb0, int rb1,
                                              bool& first, bool fresh) {
  using QQ = QuadQuarter<Q, AMODE, HAS_Z, AHEAD>;
  constexpr int PP = QQ::PP;
  id = next_quarter(p, id, id_end);
  if (id >= id_end) return;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_units = (rb1 - rb0 + 1) >> 1;   // pairs of row blocks
  const int rb_last = p.RB - 1;               // a pair's second block may lie past the end: fetch the last one instead

  QQ qq;
  quad_prepare(qq, p, id, rb0, n_units, wave, (int)(threadIdx.x & 63), quad_fetch_x(p, id, wave, threadIdx.x & 63),
               QQ::kAheadTables);
  for (;;) {
    const int next = next_quarter(p, id + 1, id_end);
    // Everything derived from the lane id below belongs to this quarter only: the empty asm
    // stops the optimiser from keeping it in registers from quarter to quarter.
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));
    const int half = lane >> 5;                 // which row block of the pair this lane works on
    const int lq = lane & 31;                   // position in the quarter
    const int out_row = 4 * (lane & 3) + ((lane & 4) ? 2 : 0) + ((lane & 8) ? 1 : 0);
    // Running sums in LDS, [row block of the stretch][vector][16 rows].  After the reduction
    // both 16-lane groups of a half hold the results of the half's row block for all four
    // vectors: group 0 adds vectors 0 and 2, group 1 vectors 1 and 3.  (A pair's second block
    // may be the padded one past the range: it has a place in LDS and is never copied out.)
    const int odd = (lane >> 4) & 1;
    float* const run_lane = lut + kRunWord + (half * 4 + odd) * 16 + out_row;
    // every lookup of the quarter before is done before its tables are overwritten (and the
    // stretch before has been copied out before its sums are)
    if (!first || !fresh) __syncthreads();
    if (!QQ::kAheadTables) quad_entries(qq, p, wave, lane, quad_fetch_x(p, id, wave, lane));
    {
      float* dst = lut + ((wave & 1) << 14) + lane;
#pragma unroll
      for (int k = 0; k < 32; ++k) dst[((wave >> 1) * 32 + k) << 6] = qq.entries[k];
    }
    if (PP == Q && threadIdx.x == 0) reinterpret_cast<int*>(lut + kQueueWord)[0] = kWaves;   // units 0..kWaves-1 are taken
    // the activations of the quarter after this one, on their way during the lookups
    u32x4 xnext = {0u, 0u, 0u, 0u};
    if (QQ::kAheadTables) xnext = quad_fetch_x(p, next < id_end ? next : id, wave, lane);
    __syncthreads();   // the tables stand

    uint32_t lane_base[4];
    f32x4v sum_x[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t L = ((uint32_t)lq & ~3u) | ((uint32_t)(s + lq) & 3u);
      lane_base[s] = ((L & 15u) << 4) | ((L >> 4) << 8);
      sum_x[s] = HAS_Z ? lds_f32x4(((L >> 4) << 16) | (0xffu << 8) | ((L & 15u) << 4)) : f32x4v{0.0f, 0.0f, 0.0f, 0.0f};
    }
    // one offset per quad of slots: only the sum over the four slots is needed
    if (HAS_Z && (AMODE & 3) == kAlphaQuad) sum_x[0] = (sum_x[0] + sum_x[1]) + (sum_x[2] + sum_x[3]);

    const int slab_lane = 32 * qq.h + lq;      // lane position inside the 1 KB slabs
    if constexpr (PP < Q) {
      for (int un = wave; un < n_units; un += kWaves) {
        const int rb = min(rb0 + 2 * un + half, rb_last);
        float acc[4][4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[v][r] = 0.0f;
        quad_passes<Q, 0, PP, AMODE, HAS_Z>(p, qq.tile_base, rb, slab_lane, qq.grp, nullptr, out_row, qq.tile_T, qq.t0,
                                            lane_base, sum_x, acc);
        float sv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) sv[v] = half_rows_reduce<false>(acc[v], lane);
        float* r = run_lane + un * 128;
        const float lo = odd ? sv[1] : sv[0], hi = odd ? sv[3] : sv[2];
        r[0] = first ? lo : r[0] + lo;
        r[32] = first ? hi : r[32] + hi;
      }
    } else {
      // Dynamic unit queue (see tile_body): a wavefront starts with unit `wave`, whose fetch
      // quad_prepare has issued, and takes every further one from the queue; nothing is
      // fetched ahead of the unit being computed.
      int cur = wave;
      if (cur < n_units) {
        for (;;) {
          if (!QQ::kFirstUnit)
            load_unit<true>(qq.u, p, qq.tile_base, min(rb0 + 2 * cur + half, rb_last), slab_lane, qq.grp, nullptr, 0, false,
                            qq.tile_T, qq.t0);
          float acc[4][4];
#pragma unroll
          for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[v][r] = 0.0f;
          accumulate_quad(qq.u, lane_base, sum_x, acc);
          float sv[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) sv[v] = half_rows_reduce(acc[v], lane);
          float* r = run_lane + cur * 128;
          const float lo = odd ? sv[1] : sv[0], hi = odd ? sv[3] : sv[2];
          r[0] = first ? lo : r[0] + lo;
          r[32] = first ? hi : r[32] + hi;
          cur = next_unit(lut, lane);
          if (cur >= n_units) break;
          if (QQ::kFirstUnit)
            load_unit<true>(qq.u, p, qq.tile_base, min(rb0 + 2 * cur + half, rb_last), slab_lane, qq.grp, nullptr, 0, false,
                            qq.tile_T, qq.t0);
        }
      }
    }
    first = false;
    if (next >= id_end) break;
    quad_prepare(qq, p, next, rb0, n_units, wave, lane, xnext, QQ::kAheadTables);   // in the shadow of the slower wavefronts
    id = next;
  }
}

// p.NT counts quarter ids here: id = 4 * tile + 2 * sub-slab + half; ids whose sub-slab or
// half does not exist in a ragged last tile are skipped.  Row ranges start at even row blocks.
// Stretches of at most kRunBlocks / 4 row blocks, as in the pair kernel.
template <int Q, bool HAS_Z, int AM2, int AM1>
__global__ __launch_bounds__(kThreads) void lutgemm_quad_kernel(GemvParams p) {
  __shared__ float lut[kGemvLdsFloats];   // (the kernel's only LDS object: see gemv_workgroup)
  const int kg = blockIdx.x;
  const int rs = blockIdx.y;
  int pair0, pair1;                 // row units are pairs of row blocks here
  row_range(p, rs, &pair0, &pair1);
  const int rb0 = 2 * pair0;
  const int rb1 = min(2 * pair1, p.RB);
  float* partial = p.partial + (int64_t)kg * p.kg_stride;
  // the K group's quarters: those of tiles with two sub-slabs, then those of a last tile with one
  const int id0 = kg * p.TPG, id1 = min(id0 + p.TPG, p.NT);
  const int last_tile = (p.nchunks - 1) >> 7;
  const int split = (p.nchunks - 128 * last_tile > 64) ? id1 : max(id0, min(id1, 4 * last_tile));
  constexpr int kStretch = kRunBlocks / 4;   // even
  // (the preparation ahead of the barrier needs registers that only the kernels have whose
  // scale mode is the quad-shared one for every tile)
  constexpr bool kAhead = (AM2 & 3) == kAlphaQuad && (AM1 & 3) == kAlphaQuad;
  for (int s0 = rb0; s0 < rb1; s0 += kStretch) {
    const int s1 = min(s0 + kStretch, rb1);
    bool first = true;
    quad_quarters<Q, AM2, HAS_Z, kAhead>(p, lut, id0, split, s0, s1, first, s0 == rb0);
    quad_quarters<Q, AM1, HAS_Z, kAhead>(p, lut, split, id1, s0, s1, first, s0 == rb0);
    if (first) {   // a K group made of non-existent quarters only: its sums are zeros
      if (s0 > rb0) __syncthreads();
      for (int i = threadIdx.x; i < (s1 - s0) * 64; i += kThreads) lut[kRunWord + i] = 0.0f;
    }
    flush_vector_sums<4>(p, lut, s0, s1, partial);
  }
  finish_row_range<4, (Q <= 4)>(p, lut, rs, rb0, rb1);
}
