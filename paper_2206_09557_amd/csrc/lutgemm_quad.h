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
// (id = 4 * tile + 2 * sub-slab + half); split-K partials and the final reduction are those
// of the GEMV kernel, for four vectors.

typedef float f32x4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4v lds_f32x4(uint32_t byte_addr) {
  return *(const __attribute__((address_space(3))) f32x4v*)(uintptr_t)byte_addr;
}

// quad_rows_reduce for a 32-lane half: four per-lane values (rows 4k..4k+3, k = lane % 4) ->
// every lane holds the sum over the 8 quads of its half for ONE of its rows.
__device__ __forceinline__ float half_rows_reduce(const float (&acc)[4], int lane) {
  const bool b2 = lane & 4, b3 = lane & 8;
  const float keep0 = b2 ? acc[2] : acc[0], send0 = b2 ? acc[0] : acc[2];
  const float keep1 = b2 ? acc[3] : acc[1], send1 = b2 ? acc[1] : acc[3];
  const float h0 = keep0 + __shfl_xor(send0, 4);
  const float h1 = keep1 + __shfl_xor(send1, 4);
  const float keep = b3 ? h1 : h0, send = b3 ? h0 : h1;
  float s = keep + dpp_f32<kDppRowRor8>(send);
  s += __shfl_xor(s, 16);
  return s;
}

template <int Q, int I0, int QP, int AMODE, bool HAS_Z>
__device__ __forceinline__ void accumulate_quad(const Unit<Q, I0, QP, 1, AMODE, HAS_Z>& u, const uint32_t (&lane_base)[4],
                                                const f32x4v (&sum_x)[4], float (&acc)[4][4]) {
  using U = Unit<Q, I0, QP, 1, AMODE, HAS_Z>;
#pragma unroll
  for (int i = 0; i < QP; ++i) {
#pragma unroll
    for (int rho = 0; rho < 4; ++rho) {
      // address bytes {0, L / 16, key byte rho, (L % 16) * 16}: lane_base holds bytes 0 and 2 (as its bytes 0 and 1)
      const uint32_t sel = 0x0c010000u | ((4u + rho) << 8);
      float run[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const f32x4v e = lds_f32x4(__builtin_amdgcn_perm(u.w[i][0][s], lane_base[s], sel));
        const bool first = ((AMODE & 3) == kAlphaQuad) ? (s == 0) : true;
#pragma unroll
        for (int v = 0; v < 4; ++v) run[v] = first ? e[v] : run[v] + e[v];
        if ((AMODE & 3) != kAlphaQuad || s == 3) {   // section 3.2 rule 2: one scale per run of lookups
          const float a = scale_of<AMODE>(u.al[((AMODE & 3) == kAlphaQuad) ? 0 : s][0], i, I0 + i, rho);
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[v][rho] = fmaf(a, run[v], acc[v][rho]);
        }
      }
    }
  }
  if (HAS_Z && I0 == 0) {   // offset term of eq. 3
#pragma unroll
    for (int s = 0; s < U::NS; ++s) {
      f32x4v sx = sum_x[s];
      if ((AMODE & 3) == kAlphaQuad) sx = (sum_x[0] + sum_x[1]) + (sum_x[2] + sum_x[3]);
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

// One workgroup, one quarter (kt, t0, h), row blocks [rb0, rb1) with rb0 even.
template <int Q, int AMODE, bool HAS_Z, int kDepth>
__device__ __forceinline__ void quad_tile_body(const GemvParams& p, float* lut, int kt, int t0, int h, int rb0, int rb1,
                                               float* partial, bool first_tile) {
  using U = Unit<Q, 0, Q, 1, AMODE, HAS_Z>;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));   // see tile_body
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int chunks_in_tile = min(128, p.nchunks - 128 * kt);
  const int tile_T = chunks_in_tile > 64 ? 2 : 1;
  const int64_t tile_base = (int64_t)kt * p.RB * Q * 2048;
  const int half = lane >> 5;                 // which row block of the pair this lane works on
  const int lq = lane & 31;                   // lane within the half = slot it builds / position in the quarter
  const int slab_lane = 32 * h + lq;          // lane position inside the 1 KB slabs
  const int out_row = 4 * (lane & 3) + ((lane & 4) ? 2 : 0) + ((lane & 8) ? 1 : 0);
  const int pair_row = half * 16 + out_row;   // row within the pair of row blocks

  int grp[4][1];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int L = (lq & ~3) | ((s + lq) & 3);
    grp[s][0] = group_of_chunk(p, 128 * kt + min(tile_T * (32 * h + L) + t0, chunks_in_tile - 1));
  }

  // ---- activations: wavefront id b (of 16) builds key range 32 * (b % 8) of vectors
  //      2 * (b / 8) + half for the slot lq ----
  const int my_chunk = tile_T * (32 * h + lq) + t0;
  const __half* xp = p.x + (int64_t)(128 * kt + min(my_chunk, chunks_in_tile - 1)) * 8;
  u32x4 xraw[kBuildPasses];
#pragma unroll
  for (int b = 0; b < kBuildPasses; ++b) {
    const int v = 2 * ((wave + b * kWaves) >> 3) + half;
    // (a quad launched for three vectors builds the fourth table set from the third vector)
    xraw[b] = *reinterpret_cast<const u32x4*>(xp + (int64_t)min(v, p.batch - 1) * p.n);
  }

  // planes fetched together: all up to four; beyond that half of them, or two where every
  // dword has a scale set of its own (16 accumulators leave fewer registers than in the
  // other kernels); a second unit in flight only with quad-shared scales
  constexpr int PP = Q > 4 ? ((AMODE & 3) == kAlphaQuad ? (Q + 1) / 2 : 2) : Q;
  constexpr int kScaleRegs = (AMODE & kAlphaShared) ? 2 : 2 * Q;
  constexpr int kFit = (PP < Q || (AMODE & 3) != kAlphaQuad || 4 * Q + kScaleRegs > 24) ? 0 : 1;
  constexpr int D = kFit < kDepth ? kFit : kDepth;
  const int n_units = (rb1 - rb0 + 1) >> 1;   // pairs of row blocks
  const int u_clamp = n_units - 1;
  const int rb_last = p.RB - 1;               // a pair's second block may lie past the end: fetch the last one instead
  U u[D + 1];
  float prev[D + 1][4];
  int uid[D + 1];
  if (PP == Q && threadIdx.x == 0) reinterpret_cast<int*>(lut + kQueueWord)[0] = (D > 0 ? D : 1) * kWaves;
#pragma unroll
  for (int k = 0; k <= D; ++k) uid[k] = wave + k * kWaves;
  if (PP == Q) {
#pragma unroll
    for (int k = 0; k < D; ++k) {
      const int rb = min(rb0 + 2 * min(uid[k], u_clamp) + half, rb_last);
      load_unit<true>(u[k], p, tile_base, rb, slab_lane, grp, partial, out_row, false, tile_T, t0);
#pragma unroll
      for (int v = 0; v < 4; ++v)
        prev[k][v] = !first_tile ? load_device_coherent(partial + v * p.vec_stride + rb * 16 + out_row) : 0.0f;
    }
  }

  // ---- tables ----
#pragma unroll
  for (int b = 0; b < kBuildPasses; ++b) {
    const int id = wave + b * kWaves;
    const int kh = id & 7;
    const int v = 2 * (id >> 3) + half;
    float xs[8];
    unpack_x(xraw[b], my_chunk < chunks_in_tile, xs);
    float* dst = lut + ((lq >> 4) << 14) + ((lq & 15) << 2) + v;
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      float e[16];
      table_entries16(kh, hi, xs, e);
#pragma unroll
      for (int k = 0; k < 16; ++k) dst[(kh * 32 + hi * 16 + k) << 6] = e[k];
    }
  }
  __syncthreads();

  uint32_t lane_base[4];
  f32x4v sum_x[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t L = ((uint32_t)lq & ~3u) | ((uint32_t)(s + lq) & 3u);
    lane_base[s] = ((L & 15u) << 4) | ((L >> 4) << 8);
    sum_x[s] = HAS_Z ? lds_f32x4(((L >> 4) << 16) | (0xffu << 8) | ((L & 15u) << 4)) : f32x4v{0.0f, 0.0f, 0.0f, 0.0f};
  }

  if constexpr (PP < Q) {
    for (int un = wave; un < n_units; un += kWaves) {
      const int rb_store = rb0 + 2 * un + half;           // may be the padded block past the end (never read back)
      const int rb = min(rb_store, rb_last);
      float acc[4][4];
      float pv[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        pv[v] = !first_tile ? load_device_coherent(partial + v * p.vec_stride + rb_store * 16 + out_row) : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[v][r] = 0.0f;
      }
      quad_passes<Q, 0, PP, AMODE, HAS_Z>(p, tile_base, rb, slab_lane, grp, partial, out_row, tile_T, t0, lane_base, sum_x,
                                          acc);
#pragma unroll
      for (int v = 0; v < 4; ++v)
        store_device_coherent(partial + v * p.vec_stride + rb_store * 16 + out_row, half_rows_reduce(acc[v], lane) + pv[v]);
    }
  } else {
    // The pair kernel's loop: dynamic unit queue, D units fetched ahead, one exit at the
    // bottom, results stored one unit later right after a fetch, surplus passes store to the
    // wavefront's spare 128 bytes (all four vectors onto the same 32 floats).
    if (uid[0] >= n_units) return;
    float* const spare0 = p.spare + (((blockIdx.y * gridDim.x + blockIdx.x) & 255) * 16 + wave) * 32;
    float held[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    float* held_to = spare0;       // wave-uniform; vector v goes v * held_step further
    int64_t held_step = 0;
    do {
#pragma unroll
      for (int j = 0; j <= D; ++j) {
        constexpr int kRing = D + 1;
        const int fill = (j + D) % kRing;
        if (D > 0) uid[fill] = next_unit(lut, lane);
        {
          const int rb = min(rb0 + 2 * min(uid[fill], u_clamp) + half, rb_last);
          load_unit<true>(u[fill], p, tile_base, rb, slab_lane, grp, partial, out_row, false, tile_T, t0);
#pragma unroll
          for (int v = 0; v < 4; ++v)
            prev[fill][v] = !first_tile ? load_device_coherent(partial + v * p.vec_stride + rb * 16 + out_row) : 0.0f;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) store_device_coherent(held_to + v * held_step + pair_row, held[v]);
        __builtin_amdgcn_sched_barrier(0);   // fetch and stores stay ahead of the lookups below
        const bool real = uid[j] < n_units;
        if (real) {
          float acc[4][4];
#pragma unroll
          for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[v][r] = 0.0f;
          accumulate_quad(u[j], lane_base, sum_x, acc);
#pragma unroll
          for (int v = 0; v < 4; ++v) held[v] = half_rows_reduce(acc[v], lane) + prev[j][v];
        }
        held_to = real ? partial + (rb0 + 2 * uid[j]) * 16 : spare0;
        held_step = real ? p.vec_stride : 0;
        if (D == 0) uid[0] = next_unit(lut, lane);
      }
    } while (uid[0] < n_units);
#pragma unroll
    for (int v = 0; v < 4; ++v) store_device_coherent(held_to + v * held_step + pair_row, held[v]);
  }
}

// p.NT counts quarter ids here: id = 4 * tile + 2 * sub-slab + half; ids whose sub-slab or
// half does not exist in a ragged last tile are skipped.  Row ranges start at even row blocks.
template <int Q, bool HAS_Z, int AM2, int AM1>
__global__ __launch_bounds__(kThreads) void lutgemm_quad_kernel(GemvParams p) {
  __shared__ float lut[kLutBytes / 4 + 4];   // (the kernel's only LDS object: see gemv_workgroup)
  const int kg = blockIdx.x;
  const int rs = blockIdx.y;
  int pair0, pair1;                 // row units are pairs of row blocks here
  row_range(p, rs, &pair0, &pair1);
  const int rb0 = 2 * pair0;
  const int rb1 = min(2 * pair1, p.RB);
  float* partial = p.partial + (int64_t)kg * p.kg_stride;
  bool first = true;
  for (int ti = 0; ti < p.TPG; ++ti) {
    const int id = kg * p.TPG + ti;
    if (id >= p.NT) break;
    const int kt = id >> 2, t0 = (id >> 1) & 1, h = id & 1;
    const int chunks = min(128, p.nchunks - 128 * kt);
    const int T = chunks > 64 ? 2 : 1;
    if (t0 >= T || 32 * h * T + t0 >= chunks) continue;   // no such quarter in this tile (wave-uniform)
    if (!first) {
      // every lookup of the previous quarter is done before its tables are overwritten, and
      // every partial sum of it is in memory before another wavefront reads it back
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
    if (T == 2)
      quad_tile_body<Q, AM2, HAS_Z, kPairDepth>(p, lut, kt, t0, h, rb0, rb1, partial, first);
    else
      quad_tile_body<Q, AM1, HAS_Z, kPairDepth>(p, lut, kt, t0, h, rb0, rb1, partial, first);
    first = false;
  }
  if (first) {   // a K group made of non-existent quarters only: its partials are zeros
    for (int v = 0; v < 4; ++v)
      for (int r = rb0 * 16 + (int)threadIdx.x; r < rb1 * 16; r += kThreads)
        store_device_coherent(partial + v * p.vec_stride + r, 0.0f);
  }
  finish_row_range<4>(p, lut, rs, rb0, rb1);
}
