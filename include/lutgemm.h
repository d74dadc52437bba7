/*
 * lutgemm.h -- C ABI of the MI355X (gfx950) LUT-GEMM library.
 *
 * The library computes the weight-only-quantised product
 *
 *      y[b][r] = sum_{k<n} What[r][k] * x[b][k]
 *      What[r][k] = sum_{i<q} alpha[i][r][G(k)] * B_i[r][k]  +  z[r][G(k)],   G(k) = k / g
 *
 * with B_i in {-1,+1} (binary-coding quantisation, paper section 2.3; bias-extended
 * form, section 3.3 eq. 3; one scale per group of g input columns, section 3.4).
 * The product is evaluated the way section 3.1 describes: every run of mu = 8
 * activations becomes a 2^mu-entry table of signed partial sums, and mu packed weight
 * bits, read as one byte, index that table. Nothing is dequantised.
 *
 * Conventions shared by every entry point
 *   - Return value: LUTGEMM_OK (0) or a negative LUTGEMM_E* code. Nothing throws,
 *     aborts, allocates device memory or synchronises a stream.
 *   - The caller owns every buffer, before and after the call.
 *   - "fp16" is IEEE binary16 carried as uint16_t.
 *   - g == 0 means row-wise quantisation (g = n).
 *   - Required: 1 <= q <= 8, mu == 8, m >= 1, n >= 8, n % 8 == 0, g % 8 == 0,
 *     n % g == 0. Anything else is LUTGEMM_EINVAL (malformed) or
 *     LUTGEMM_EUNSUPPORTED (well-formed, not implemented: mu != 8, batch > 32).
 *
 * ---------------------------------------------------------------------------------
 * Packed ("device") layouts.  These are a contract: lutgemm_pack_bcq writes them,
 * the kernels read them, and an independent decoder can be written from this text.
 *
 * Notation: chunk c = k / 8 (n/8 chunks per row); the key of (plane i, row r, chunk c)
 * is the byte whose bit j (LSB = bit 0) is 1 iff B_i[r][8c + j] = +1  (section 3.1:
 * a key is mu concatenated binary elements; polarity and bit order are this
 * library's choice).  Row block rb = r / 16, rho = r % 16, RB = ceil(m / 16).
 * K tile kt = c / 128, NT = ceil((n/8) / 128).  Tile kt holds
 * C = min(128, n/8 - 128*kt) chunks and has T = 2 sub-slabs if C > 64, else T = 1
 * (only the last tile can have C < 128).  Slot (t, L), t < T, L < 64, of tile kt
 * stands for chunk 128*kt + T*L + t.
 *
 *   bits   one byte per (plane, row, chunk), in slabs of 1024 bytes = 64 lanes x 16 bytes
 *          per (tile, row block, plane, sub-slab):
 *            slab offset = kt * RB * q * 2048 + ((rb * q + i) * T + t) * 1024
 *          Inside a slab the four lanes of a quad hold four rows each, and the four
 *          slots of the quad are rotated across them: with k = rho / 4 and the slot
 *          written L = 4*j + c (quad j, c < 4), the key sits in
 *            lane 4*j + k,  byte 4 * ((c - k) mod 4) + rho % 4,
 *          i.e. at  slab offset + (4*j + k) * 16 + 4 * ((c - k) mod 4) + rho % 4.
 *          (A lane thus owns rows 4k..4k+3; in its dword s it finds the keys of slot
 *          4*j + (s + k) mod 4, so the four lanes of a quad always address four
 *          different tables.)  Bytes of rows >= m and of slots whose chunk >= n/8 are 0.
 *          Size = RB * q * 1024 * (2 * (NT - 1) + T_last) bytes, which equals
 *          m*n*q/8 (the binary-weight term of section 3.4 eq. 4) when m % 16 == 0
 *          and n % 512 == 0.
 *   alpha  fp16, one per (plane, row, group), NG = n / g groups; the 16 rows of a block
 *          are kept as four quarters of four rows, the planes of a quarter together:
 *            index = (((rb * NG + G) * 4 + rho / 4) * q + i) * 4 + rho % 4
 *          Rows >= m hold 0.  Size = RB * NG * q * 32 bytes ( = 2*m*(n/g)*q, the
 *          scale term of eq. 4, when m % 16 == 0).
 *   z      fp16, one per (row, group):  index = (rb * NG + G) * 16 + rho.
 *          Rows >= m hold 0.  Size = RB * NG * 32 bytes.
 * ---------------------------------------------------------------------------------
 */
#ifndef LUTGEMM_H
#define LUTGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LUTGEMM_OK = 0,
  LUTGEMM_EINVAL = -1,       /* null pointer, size out of range, n % 8, n % g, g % 8, misaligned pointer */
  LUTGEMM_EUNSUPPORTED = -2, /* mu != 8, batch > 32, unknown mode or flag */
  LUTGEMM_EWORKSPACE = -3,   /* workspace_bytes < lutgemm_workspace_bytes(...) */
  LUTGEMM_EHIP = -4          /* a HIP runtime call (device query, kernel launch) returned an error */
};

/* Quantiser selected by lutgemm_pack_bcq's `mode`. */
enum {
  /* Symmetric greedy BCQ (section 2.3 format). Per (row, group), residual r0 = w (fp32):
     plane i: B_i = sign(r_i) with sign(0) = +1; alpha_i = fp16(mean_k |r_i[k]|), the mean
     being an fp64 sum in increasing k divided by g, rounded once to fp16 (nearest even);
     r_{i+1} = r_i - alpha_i * B_i in fp32 using the rounded alpha_i.  No offset.        */
  LUTGEMM_Q_GREEDY = 0,
  /* As above on w - z, with z = fp16(mean_k w[k]) (same fp64 sum, one rounding); the
     asymmetric format of section 3.3 eq. 3.                                              */
  LUTGEMM_Q_GREEDY_MEAN_OFFSET = 1,
  /* Asymmetric min/max round-to-nearest uniform quantisation converted to BCQ as in
     appendix C: zhat = min, s = fp16((max - min) / (2^q - 1)) (fp32 arithmetic, one
     rounding), u = clamp(rint((w - zhat) / s), 0, 2^q - 1) in fp32, plane i = bit i of u,
     alpha_i = fp16(2^(i-1) * s), z = fp16(zhat + sum_i alpha_i) (fp32 sum over the stored
     alpha_i, i ascending, then + zhat).  If s == 0 every bit is 1, alpha_i = 0, z = zhat. */
  LUTGEMM_Q_UNIFORM_RTN = 2,
  /* Alternating BCQ, no offset: the iterative solver the paper's appendix on compression
     ratios cites for obtaining BCQ weights.  Per (row, group), all in fp64 with every sum in
     index order: start from the greedy solution (unrounded scales); then up to 15 rounds of
     { scales = least-squares fit for the current signs (normal equations, Gaussian
     elimination with partial pivoting; stop if singular); a plane whose scale comes out
     negative is negated; every weight takes the nearest of the 2^q levels sum_i +-alpha_i
     (levels summed in plane order, ties to the smallest code, bit i of the code = plane i
     is +1) }, stopping early when no sign changes; finally the scales are rounded to fp16
     and the signs assigned once more for the stored scales.  Never worse than the greedy
     start before the rounding; cost grows with 2^q per weight and round.                 */
  LUTGEMM_Q_ALTERNATING = 3
};

/* `flags` of lutgemm_gemv / lutgemm_gemm. */
enum {
  LUTGEMM_Y_F16 = 0, /* y is fp16, rounded to nearest even from the fp32 sum (paper table 1: FP16 output) */
  LUTGEMM_Y_F32 = 1, /* y is fp32 */
  /* `alpha` is in the shared-scale layout: ONE fp16 per (row, group), alpha_0, and plane i
     has the scale 2^i * alpha_0, as appendix C gives for uniformly quantised weights
     (buffer of lutgemm_alpha_shared_bytes, written by lutgemm_share_scales).  Requires z.
     Results are bit-for-bit those of the per-plane layout holding the same scales.       */
  LUTGEMM_ALPHA_SHARED = 2,
  /* lutgemm_gemm only: let the library take the matrix-core path (lutgemm_gemm_mfma) where
     it measured faster on MI355X and is applicable (group size a multiple of 64, per-plane
     scales): from five activation vectors on, and from three on layers of at most 2^27
     weights.  Section 6 of the paper: the lookup path pays per vector, the matrix cores
     do not.  Either path meets the same tolerance; which one ran is decided by shape and
     batch only, so results stay reproducible.                                            */
  LUTGEMM_PATH_AUTO = 4
};

/* Buffer sizes in bytes of the packed layouts above (section 3.4 eq. 4, padded to the
   tile grid).  Return 0 for arguments that violate the requirements at the top.        */
size_t lutgemm_bits_bytes(int64_t m, int64_t n, int q);
size_t lutgemm_alpha_bytes(int64_t m, int64_t n, int q, int g);
size_t lutgemm_z_bytes(int64_t m, int64_t n, int g);

/* Bytes of the shared-scale layout: fp16 [row block][group][16 rows], index
   ((r / 16) * NG + G) * 16 + r % 16, the layout of z.                                   */
size_t lutgemm_alpha_shared_bytes(int64_t m, int64_t n, int g);

/* Device scratch a gemv/gemm call needs: 32 KB of arrival counters and the split-K partial
   sums (the per-block partial outputs that appendix B accumulates across thread blocks).
   0 on invalid arguments.                                                               */
size_t lutgemm_workspace_bytes(int64_t m, int64_t n, int q, int g, int mu, int batch);

/* DEVICE.  Enqueue the one-time preparation of a freshly allocated workspace (zeroes its
   arrival counters with a small kernel, so the call may be captured in a HIP graph).
   Needed once per workspace, before the first gemv/gemm that uses it; every gemv/gemm
   leaves the counters zero again when its kernel has finished.  A workspace whose first
   32 KB the caller has zero-filled by other means needs no call.                        */
int lutgemm_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/* HOST.  Quantise W (fp16, row-major m x n, host memory) to q planes with group size g
   using `mode`, and write the packed layouts into host buffers of the sizes above.
   z_out must be non-null for the two offset modes and may be null for LUTGEMM_Q_GREEDY
   (if non-null it is filled with zeros).  Deterministic: same input, same bytes.
   Format: section 2.3, section 3.3 eq. 3, appendix C.                                   */
int lutgemm_pack_bcq(const uint16_t* W, int64_t m, int64_t n, int q, int g, int mu, int mode,
                     void* bits_out, uint16_t* alpha_out, uint16_t* z_out);

/* HOST.  Decode packed bits back to the binary planes B_pm1[q][m][n] in {-1,+1} (int8, host
   memory): the b_i of section 2.3's  w ~ sum_i alpha_i b_i, bit j of the key of chunk c being
   column 8c + j (section 3.1's keys read back).  Inverse of lutgemm_pack_planes.       */
int lutgemm_unpack_bcq(const void* bits, int64_t m, int64_t n, int q, int mu, int8_t* B_pm1);

/* HOST.  Write already-known planes B_pm1[q][m][n] (entries -1/+1) in the packed bits
   layout; used when a quantiser outside this library produced the planes (appendix C:
   integer weights of any uniform quantiser turned into binary weights).                 */
int lutgemm_pack_planes(const int8_t* B_pm1, int64_t m, int64_t n, int q, int mu, void* bits_out);

/* HOST.  Reorder canonical scales alpha[q][m][NG] (and offsets z[m][NG], nullable pair)
   into the packed alpha / z layouts.                                                    */
int lutgemm_pack_scales(const uint16_t* alpha, const uint16_t* z, int64_t m, int64_t n, int q, int g,
                        uint16_t* alpha_out, uint16_t* z_out);

/* HOST.  Packed per-plane scales (as written by lutgemm_pack_bcq / lutgemm_pack_scales) ->
   shared-scale layout, for weights whose scales satisfy alpha_i = 2^i * alpha_0 exactly in
   every (row, group): the output of LUTGEMM_Q_UNIFORM_RTN (appendix C).  LUTGEMM_EINVAL if
   some scale is not of that form (nothing useful is written then).  The scale bytes shrink
   q-fold: section 3.4's footprint with one scale per group, which is what the compression
   ratios of table 5 count.                                                              */
int lutgemm_share_scales(const uint16_t* alpha_packed, int64_t m, int64_t n, int q, int g,
                         uint16_t* alpha_shared_out);

/* DEVICE pointers, all 16-byte aligned.  y = What * x for one activation vector
   (section 3.2: y = sum_i A_i o (B_i . x); offset term from eq. 3).
     x      fp16 [n]                       bits, alpha, z   packed layouts above (z nullable)
     y      fp16 [m] or fp32 [m] (flags); overwritten, never read
     workspace  at least lutgemm_workspace_bytes(m, n, q, g, mu, 1) bytes, prepared once
                by lutgemm_workspace_init; beyond the first 32 KB its contents need not be
                initialised and are undefined afterwards.  One workspace serves calls of
                any shape it is large enough for
     hip_stream a hipStream_t (NULL = the null stream); the work is enqueued and the call
                returns without waiting.  Calls that share a workspace must be ordered on
                one stream (two calls running at once need two workspaces).
   The result is bitwise reproducible from run to run.                                   */
int lutgemm_gemv(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* DEVICE pointers in host arrays.  `count` (1..8) independent products y[i] = What_i x[i] in
   ONE kernel launch, e.g. the four linear layers of a decoder block (appendix A: attention
   QKV and output projections, the two feed-forward layers) when their inputs are at hand,
   the separate Q / K / V or gate / up projections of one activation vector, or the experts
   of a mixture layer.  Arguments as lutgemm_gemv, per layer:
     x[i], bits[i], alpha[i], y[i]   device pointers of layer i, shape m[i] x n[i];
     z                               NULL (no layer has offsets) or an array of `count`
                                     offset buffers
   and q, g, mu, flags common to all layers (with g == 0 every layer's group size is its own
   n; the group sizes must then fall in the same class: all multiples of 64, or of 32, or of
   16, else LUTGEMM_EUNSUPPORTED, as are group sizes that are not multiples of 16).  Workspace of lutgemm_group_workspace_bytes(m, n, count, q,
   g, mu) bytes, prepared like any other (lutgemm_workspace_init once).
   Every layer runs on the grid it would have alone; the workgroups of layer i + 1 follow those
   of layer i onto the compute units as these become free, so the end of one product (its
   stragglers, its cross-tile sums) and the start of the next (activation fetch, table build)
   overlap with streaming instead of leaving the memory system half idle: on the OPT-175B
   layers the four products take less time than four launches.  The layers must not depend
   on one another: a layer's x must not be another layer's y.  For dependent layers, call
   lutgemm_gemv once per layer on one stream; they may share one workspace.
   Each y[i] is bit for bit what lutgemm_gemv gives for that layer.                      */
int lutgemm_gemv_group(const void* const* x, const void* const* bits, const void* const* alpha,
                       const void* const* z, void* const* y, const int64_t* m, const int64_t* n, int count,
                       int q, int g, int mu, unsigned flags, void* workspace, size_t workspace_bytes,
                       void* hip_stream);
size_t lutgemm_group_workspace_bytes(const int64_t* m, const int64_t* n, int count, int q, int g, int mu);

/* For callers that cannot allocate device memory or pass a workspace along: code that runs
   under HIP graph capture, tight serving loops, harnesses that forbid allocation.
   lutgemm_gemv with the same arguments minus the workspace: the scratch memory is an array
   of lutgemm_static_scratch_bytes() (8 MiB) inside the library's device image, one copy per
   GPU, held until the process ends.  The call allocates nothing and never synchronises; the
   first call on a device looks the array's address up and enqueues a small kernel that
   zeroes its arrival counters.  LUTGEMM_EWORKSPACE if the layer needs more scratch than
   the array holds (lutgemm_workspace_bytes(m, n, q, g, mu, 1) > 8 MiB: beyond about 2^21
   weights-rows x K-tiles; the OPT-175B layers need 0.6 to 2.3 MiB).  All calls on one GPU
   share that GPU's array, which keeps the last call's partial sums: calls must be ordered
   on one stream (or otherwise not overlap); two that overlap race.  Same result, bit for
   bit, as lutgemm_gemv.                                                                 */
int lutgemm_gemv_static(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                        int q, int g, int mu, int64_t m, int64_t n, unsigned flags, void* hip_stream);
size_t lutgemm_static_scratch_bytes(void);

/* As lutgemm_gemv for `batch` activation vectors (1 <= batch <= 32): x is fp16
   [batch][n], y is [batch][m], workspace sized for this batch.  The vectors are taken four
   at a time; two or one left over have kernels of their own, three left over run as four
   (the fourth table set repeats the third vector, its results are dropped).  One table set
   per activation vector, each fetched key looked up in all of them with one LDS read, so
   the weights are streamed once per four vectors (the small-batch case discussed in
   section 6).  A vector's result does not depend on the other vectors of the call, only on
   whether it is processed in a group of four, two or one; between those three it agrees
   to the documented tolerance, not bit for bit.  Bitwise reproducible from run to run.                                       */
int lutgemm_gemm(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                 int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same arguments, same result (to the same tolerance) as lutgemm_gemm, computed without
   tables of partial sums: every key byte is expanded to eight values of +-1 and each
   plane's B_i . X runs on the matrix cores, fp32 accumulation, one multiplication by the
   scale per group (section 3.2: y = sum_i A_i o (B_i . x); offset term of eq. 3).  Its
   time does not grow with batch up to 16 vectors, where the lookup path's does (the
   limitation discussed in section 6), so it is the faster of the two from a batch of
   three to six, depending on the layer (LUTGEMM_PATH_AUTO).  Requires a group size that is a multiple of 64 columns (g == 0, row-wise,
   included when n % 64 == 0): LUTGEMM_EUNSUPPORTED otherwise, as is
   LUTGEMM_ALPHA_SHARED or LUTGEMM_PATH_AUTO.  Bitwise reproducible.                     */
int lutgemm_gemm_mfma(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                      int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Same arguments as lutgemm_gemm_mfma; the comparison kernel of the small-batch workload:
   dequantise, then multiply on the matrix cores (the dequantisation-based kind of kernel the
   paper sets its method against in section 2.2 and section 4).  Every 8 weights of a row are
   rebuilt as fp16 values  What = sum_i alpha_i b_i + z  (eq. 3) in packed fp16 arithmetic and
   ONE matrix-core instruction per 32 columns multiplies them with the activations (fp32
   accumulation).  The fp16 rounding of What is part of the method: y agrees with the exact
   product to a relative L2 error of about 3e-4 (bound asked of it: 1e-3), not to the 1e-5
   of the other paths' fp32 outputs.  Same restrictions as lutgemm_gemm_mfma.  Bitwise
   reproducible.  Measured beside the plane-wise form on MI355X (49152 x 12288, q = 3): 157 us
   against 124 us up to 16 activation vectors, 185 against 183 at 32: rebuilding fp16
   weights buys nothing over multiplying the planes, and costs accuracy.                  */
int lutgemm_gemm_dequant_mfma(const void* x, const void* bits, const void* alpha, const void* z, void* y,
                              int q, int g, int mu, int64_t m, int64_t n, int batch, unsigned flags,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* HOST.  The workgroup grid the lookup kernels are launched with for an m x n layer of q
   planes and group size g, as chosen from these alone (appendix B: every block owns a tile
   of the weights and a set of tables; the partial outputs of the blocks along a row are
   then combined):
     vectors  activation vectors per pass: 1 (lutgemm_gemv), 2 or 4 (the kernels
              lutgemm_gemm uses for pairs and fours)
     compute_units  of the device to plan for; <= 0 asks the current device
     out[0]   K groups (workgroups along the columns),
     out[1]   K tiles of 1024 columns per K group (half tiles of 512 for vectors = 2,
              quarter tiles of 256 for vectors = 4),
     out[2]   row ranges (workgroups along the rows).
   Tests use it to show which code path a shape reaches; tuning scripts to explain a time.
   The choice can be overridden for sweeps by environment variables read once per process
   (LUTGEMM_TPG / LUTGEMM_RS for vectors = 1, LUTGEMM_PAIR_TPG / _RS, LUTGEMM_QUAD_TPG / _RS,
   LUTGEMM_MFMA_TPG: tiles per K group, row ranges); results do not depend on the grid
   beyond the order of the additions.
   LUTGEMM_EINVAL for malformed arguments, LUTGEMM_EHIP if the device cannot be asked.  */
int lutgemm_plan_grid(int64_t m, int64_t n, int q, int g, int vectors, int compute_units, int* out);

/* DEVICE pointers.  Measurement aid, no part of the product: reads `bytes` bytes at src
   (bytes % 16 == 0, src 16-byte aligned) exactly once, every workgroup a contiguous share
   front to back, in the access shape of the weight stream of section 3.4's memory-bound
   regime (16 bytes per lane, coalesced, non-temporal), and writes the XOR of all 32-bit words seen by each of its 8192 wavefronts to sink
   (uint32_t[8192]; the XOR of those is the XOR of the whole buffer).  Its rate is the
   read bandwidth this device sustains, which benchmarks report beside the nominal figure.
   sink_bytes < 32768 is LUTGEMM_EWORKSPACE.                                              */
int lutgemm_stream_read(const void* src, size_t bytes, void* sink, size_t sink_bytes, void* hip_stream);

/* Human-readable name of an error code (static storage).                                */
const char* lutgemm_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LUTGEMM_H */
