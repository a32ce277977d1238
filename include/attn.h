/* C ABI of the MI355X (gfx950) fused attention-forward library.
 *
 * The operation is the kernel the paper tunes: fused multi-head attention
 * forward ("flash-attention", Sec. 1 and Sec. 5 "Experiment setup"), on tensors
 * laid out [batch, heads, seq, head_dim] (Table 2 caption), in 16-bit floating
 * point.  The paper does not write the formula out; it is the textbook one:
 *
 *     for every (b, h) and query row i, over the visible keys j
 *     (all j when causal == 0, j <= i when causal != 0):
 *         x_j    = scale * sum_c Q[b,h,i,c] * K[b,h,j,c]
 *         lse    = ln sum_j exp(x_j)                       (natural logarithm)
 *         O[c]   = sum_j exp(x_j - lse) * V[b,h,j,c]
 *
 * computed in one pass over K/V tiles with an online softmax: both contractions
 * run on bf16/fp16 MFMA with fp32 accumulation, the probabilities are rounded to
 * the input type (nearest-even) before the second contraction, O is rounded once
 * at the end.
 *
 * The schedule-variant entry points are the analogue of the paper's search
 * space (Sec. 3.1): a variant is one compile-time instruction schedule of the
 * same kernel (tile shape, loop order, LDS prefetch distance, instruction-group
 * interleaving, position of the tile loads, wave priority placement, load path,
 * occupancy; attn_knob_name lists them).  All variants compute the same function.
 *
 * General rules
 *  - every pointer named "device" is a HIP device pointer owned by the caller;
 *    the library allocates no device memory and frees none.  Its only mutable state
 *    is process-wide and small: the compute-unit count of each device, read once,
 *    and the tables of loaded code objects and deployed schedules (attn_codeobj_*,
 *    attn_deploy_*), which are not synchronised;
 *  - calls are asynchronous: work is enqueued on `stream` (a hipStream_t passed
 *    as void*, NULL = the default stream) and the call returns without waiting;
 *  - the return value is ATTN_OK or a negative error code; on error nothing has
 *    been enqueued and no output byte is written;
 *  - no C++ exception crosses this boundary.
 */
#ifndef PAPER_2403_16863_AMD_ATTN_H
#define PAPER_2403_16863_AMD_ATTN_H

#ifdef __cplusplus
extern "C" {
#endif

enum { ATTN_F16 = 0, ATTN_BF16 = 1 };

enum {
    ATTN_OK = 0,
    ATTN_EINVAL = -1,       /* null pointer, non-positive size, misaligned or aliased buffer,
                               non-finite scale, unknown dtype, variant id out of range */
    ATTN_EUNSUPPORTED = -2, /* head_dim other than 64 or 128; B*H or N beyond the grid limits;
                               variant not built for this (d, dtype, causal) */
    ATTN_ELAUNCH = -3       /* the HIP runtime refused the launch */
};

/* Fused attention forward with the library's default schedule variant for the
 * shape (attn_default_variant).
 *
 *  q, k, v : device, [B,H,N,d] contiguous row-major, 16-bit elements of `dtype`,
 *            16-byte aligned.  Read only.
 *  out     : device, [B,H,N,d] contiguous, same dtype, 16-byte aligned; must not
 *            overlap q, k or v.  Every element is written.
 *  lse     : device, [B,H,N] fp32, 4-byte aligned: natural-log log-sum-exp of the
 *            scaled scores over the visible keys.  Every element is written.
 *  B,H,N   : >= 1, any N (ragged last tiles are masked).  Limits, reported as
 *            ATTN_EUNSUPPORTED: B*H*N*d <= 2^40 elements, and B*H*ceil(N/bm) <= 2^31-1
 *            work items (bm = the variant's query tile, 128 or 256 rows).
 *  d       : 64 or 128.
 *  causal  : 0 = every key visible, otherwise key j is visible to query i iff j <= i.
 *  scale   : finite; multiplies q.k before the softmax (callers pass 1/sqrt(d)).
 *
 * Accuracy (fp32 accumulation, P rounded to `dtype` before the second contraction, O rounded
 * once): with u = 2^-11 (binary16) or 2^-8 (bfloat16), the half-unit roundoff of `dtype`,
 *     |O[c] - exact| <= u * |O[c]|  +  u * sum_j p_j |V[j,c]|  +  small fp32 terms,
 * i.e. at most about 2 u max_j |V[j,c]|: 1e-3 * Vmax for binary16, 8e-3 * Vmax for bfloat16.
 * The absolute bounds 1e-2 / 3e-2 that the tests use therefore hold for |V| below about 10
 * (binary16) and 3.8 (bfloat16) in the worst case (a row that puts all its weight on large
 * values of one sign); for larger outputs the bound is the relative one.
 * lse is accurate to about 1e-6 relative (fp32 sums of unrounded probabilities).
 * Score magnitude: the scaled scores x_j are formed in fp32 (MFMA accumulation, then one fused
 * multiply-add against the reference maximum), so a probability carries a relative error of about
 * |x_j| * 2^-22 on top of the above: nothing up to |x| ~ 1e4, a per cent at |x| ~ 1e5.
 * Overflow: the exact O never exceeds max |V| (a convex combination), but the computed one may
 * by the error above; in binary16 a finite result beyond the largest finite value (65504) is
 * stored as +-65504, not as infinity (infinities and NaN that come from the inputs pass
 * unchanged).  bfloat16 outputs cannot get there within the V magnitude limit below.
 * V magnitude: the one-pass method keeps the un-normalised sum of p*v in fp32, with p up to
 * 2^8 before the reference maximum is raised, so |V| * N * 2^8 must stay below the fp32 range
 * (3.4e38): every finite binary16 V qualifies, bfloat16 V must stay below about 1e38 / (256 N).
 *  dtype   : ATTN_F16 or ATTN_BF16.
 *  stream  : hipStream_t as void*, NULL = default stream.
 */
int attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse,
             int B, int H, int N, int d, int causal, float scale, int dtype, void* stream);

/* Same operation with an explicit schedule variant (0 <= variant_id <
 * attn_num_variants()).  This is what the schedule search calls (Sec. 3, Alg. 1:
 * each visited schedule is executed on the device). */
int attn_fwd_variant(const void* q, const void* k, const void* v, void* out, float* lse,
                     int B, int H, int N, int d, int causal, float scale, int dtype,
                     void* stream, int variant_id);

/* Number of schedule variants compiled into the library (same table for every
 * shape; a variant that was not built for a given head_dim reports
 * ATTN_EUNSUPPORTED from attn_fwd_variant / attn_variant_supported). */
int attn_num_variants(void);

/* 1 if variant_id can run this (d, dtype, causal), 0 if not, ATTN_EINVAL if the id
 * is out of range. */
int attn_variant_supported(int variant_id, int d, int dtype, int causal);

/* Writes a NUL-terminated human-readable knob vector ("bm=128 bn=64 ...") into
 * buf (host memory, buflen bytes, truncated if needed).  Returns the untruncated
 * length, or ATTN_EINVAL. */
int attn_variant_desc(int variant_id, char* buf, int buflen);

/* The search space as a lattice (Sec. 3.1 / 3.2): every variant is a point with
 * attn_num_knobs() integer coordinates; a mutation moves one coordinate by one.
 * attn_variant_coords writes the coordinates of a variant into coords[nknobs];
 * attn_variant_from_coords returns the id at a lattice point or ATTN_EINVAL if no
 * variant is built there; attn_knob_name / attn_knob_size describe a coordinate. */
int attn_num_knobs(void);
const char* attn_knob_name(int knob);
int attn_knob_size(int knob);
int attn_variant_coords(int variant_id, int* coords);
int attn_variant_from_coords(const int* coords);

/* How work reaches the device (host logic, no device call).  A work item is one
 * query tile of one head (the outer, data-parallel loop of the tiled forward pass);
 * a launch uses a grid of persistent workgroups, each of which takes items round
 * after round from a fixed schedule: items sorted by weight (under a causal mask the
 * last query tiles see the most keys) are dealt to the workgroups in serpentine
 * order, inside each of the 8 XCDs over that XCD's own heads when the grid and the
 * number of heads are multiples of 8.
 * attn_schedule_grid returns the grid size a launch of this variant uses for the
 * shape on a device with `compute_units` CUs (ATTN_EINVAL / ATTN_EUNSUPPORTED on bad
 * or oversized arguments).
 * attn_schedule_item names the item of workgroup `workgroup` (0 <= workgroup < grid)
 * in round `round` for BH = B*H heads of nqt query tiles each: returns 1 and writes
 * *bh (0 .. BH-1) and *qt (0 .. nqt-1), 0 when that workgroup has no item in that
 * round (nor in any later one), ATTN_EINVAL on bad arguments.  Over all workgroups
 * and rounds every item is named exactly once. */
int attn_schedule_grid(int variant_id, int compute_units, int B, int H, int N);
int attn_schedule_item(int grid, int workgroup, int BH, int nqt, int round, int* bh, int* qt);

/* The variant attn_fwd uses for this shape: the best admitted variant of the stored searches
 * on MI355X (Sec. 4.1: candidates are ranked offline and the best one is deployed, at no
 * run-time cost).  The choice depends on d and N only; dtype and causal are accepted so that a
 * later ranking may use them, and are ignored today. */
int attn_default_variant(int N, int d, int dtype, int causal);

/* Feedback measurement of Sec. 3.3: `warmup` untimed launches, then `iters`
 * launches each bracketed by its own pair of HIP events on `stream`; the elapsed
 * milliseconds of launch i are written to ms[i] (host memory, iters floats).
 * Blocks the calling thread until the last launch has finished.  Same argument
 * rules as attn_fwd_variant; additionally iters >= 1 and warmup >= 0. */
int attn_time_variant(const void* q, const void* k, const void* v, void* out, float* lse,
                      int B, int H, int N, int d, int causal, float scale, int dtype,
                      void* stream, int variant_id, int warmup, int iters, float* ms);

/* Instruction-level schedule search (Sec. 3.1 to 3.3 applied to machine code): the
 * assembly of a variant's kernel, with the positions of some memory instructions changed,
 * is assembled into a code object outside this library and run through these calls.
 * attn_codeobj_load loads the code object file `path` (host string) and looks up
 * `kernel_name` in it; the kernel must be a re-scheduled copy of the kernel that
 * `variant_id` uses for (d, dtype, causal): same arguments, same block size, same LDS.
 * Returns a handle >= 0, or ATTN_EINVAL (bad argument), ATTN_EUNSUPPORTED (no such
 * variant kernel, or all 64 handles in use), ATTN_ELAUNCH (file or symbol not loadable).
 * attn_fwd_codeobj / attn_time_codeobj behave like attn_fwd_variant / attn_time_variant
 * with the loaded kernel in place of the variant's own; a shape that does not match what
 * the handle was loaded for gives ATTN_EUNSUPPORTED.  attn_codeobj_unload releases a
 * handle; the caller makes sure no launch of it is still in flight.  The handle table is
 * process-wide and not synchronised: use it from one thread. */
int attn_codeobj_load(const char* path, const char* kernel_name, int variant_id, int d, int dtype, int causal);
int attn_codeobj_unload(int handle);
int attn_fwd_codeobj(int handle, const void* q, const void* k, const void* v, void* out, float* lse,
                     int B, int H, int N, int d, int causal, float scale, int dtype, void* stream);
int attn_time_codeobj(int handle, const void* q, const void* k, const void* v, void* out, float* lse,
                      int B, int H, int N, int d, int causal, float scale, int dtype, void* stream,
                      int warmup, int iters, float* ms);

/* Deployment of a searched schedule (Sec. 4.1: the candidates of the offline searches are
 * ranked, and the best one that passed the tests is what the application runs, chosen once,
 * at no cost per call).  After attn_deploy_variant, attn_fwd launches `variant_id` for every
 * problem with this d, dtype and causal flag (0 / non-zero) and n_min <= N <= n_max, instead
 * of attn_default_variant's choice; attn_deploy_codeobj does the same for a loaded code object
 * (the instruction-level search's winner), for the d, dtype and causal flag it was loaded for.
 * The newest matching entry wins.  A deployed schedule that refuses a problem
 * (ATTN_EUNSUPPORTED, e.g. the interleaved order beyond 4 GiB per head) is replaced by the
 * library default for that call.  attn_deployed reports what attn_fwd would launch for a
 * shape: returns 1 and writes *variant_id (the schedule, or the schedule the code object was
 * derived from) and *handle (the code object, -1 if none) when an entry matches, 0 when the
 * default applies (*variant_id = the default, *handle = -1); either pointer may be NULL.
 * attn_deploy_clear removes every entry; attn_codeobj_unload removes the entries of its handle.
 * Up to 16 entries (ATTN_EUNSUPPORTED beyond, or if the variant was not built for the
 * shape); ATTN_EINVAL for bad ids, handles or an empty range.  Host logic only: no device
 * call, nothing is validated here (admission is the search's job, Sec. 4.2).  The table is
 * process-wide and not synchronised, like the handle table: set it up from one thread
 * before the launches that rely on it. */
int attn_deploy_variant(int variant_id, int d, int dtype, int causal, int n_min, int n_max);
int attn_deploy_codeobj(int handle, int n_min, int n_max);
int attn_deploy_clear(void);
int attn_deployed(int N, int d, int dtype, int causal, int* variant_id, int* handle);

/* Measurement aid for the roofline (not part of the attention path): runs a kernel
 * that does nothing but independent 32x32x16 bf16 MFMAs from registers on every SIMD
 * (`iters` rounds of four per wave, 8 waves per CU) and reports the rate it sustained
 * (*tflops, host) and the core clock during the run (*core_ghz, host; 0 if the clock
 * counters could not be read).  random_operands = 0 uses constant operands (the
 * clock-limited peak), 1 uses operands with random signs and mantissas: the device
 * then lowers its clock, and that rate bounds what a kernel fed real data can reach.
 * counters: device memory, 3 x 8 bytes, written by the kernel (caller-owned).
 * Blocks until the kernel has finished.  ATTN_EINVAL on bad arguments, ATTN_ELAUNCH
 * if a HIP call fails. */
int attn_mfma_ceiling(int random_operands, int iters, void* stream, unsigned long long* counters,
                      double* tflops, double* core_ghz);

/* Measurement aid: the ceiling of the tile loop's own instruction mix on this device (not part
 * of the attention path).  Per 32x32x16 MFMA the loop reads one 1 KB operand fragment from LDS and
 * issues one multiply-add, one exp2, one add and half a conversion to 16 bit per lane for the
 * softmax.  The kernel issues that and nothing else (random operands, fragments read four steps
 * ahead, two waves per SIMD, `iters` rounds of 16 MFMAs per wave; no tile loads, barriers, masks
 * or item boundaries; launched twice, the second launch is the one timed): mode 0 = MFMAs only,
 * 1 = MFMAs and LDS reads, 2 = the whole mix, every wave issuing all of it interleaved.  Modes 3
 * and 4 run the whole mix in the ping-pong form of the default kernels instead: per round a wave
 * runs one cluster of 32 MFMAs with their LDS reads and one cluster of the softmax's vector
 * instructions for 32 scores per lane, the two waves of a SIMD in opposite order, with two
 * workgroup barriers per round (mode 3) or one (mode 4); `iters` rounds of 32 MFMAs per wave.  The
 * device runs it at its power limit, as it runs the attention kernel, so *tflops (host) is what
 * the loop body can reach there; *core_ghz (host) is the clock during the run (0 if the clock
 * counters could not be read).  counters: device memory, 3 x 8 bytes, written by the kernel
 * (caller-owned).  Blocks until the kernel has finished.  ATTN_EINVAL on bad arguments,
 * ATTN_ELAUNCH if a HIP call fails. */
int attn_mix_ceiling(int mode, int iters, void* stream, unsigned long long* counters,
                     double* tflops, double* core_ghz);

/* Measurement aid for the second ceiling of the path, the vector ALU (not part of the
 * attention path).  Per score element the one-pass softmax issues one multiply-add, one exp2,
 * one add and half a conversion to 16 bit; the kernel issues exactly that mix on register data
 * (16 elements per round and lane, `iters` rounds) with `waves_per_simd` waves (1 to 4) on every
 * SIMD, and reports the elements per second it sustained (*elements_per_s, host) and the core
 * clock during the run (*core_ghz, host; 0 if the clock counters could not be read).  An
 * element stands for 4*d floating-point operations of the two contractions, so
 * 4 * d * elements_per_s is the rate the matrix cores would have to be fed at for the softmax
 * not to be the bound.  counters: device memory, 3 x 8 bytes, written by the kernel
 * (caller-owned).  Blocks until the kernel has finished.  ATTN_EINVAL on bad arguments,
 * ATTN_ELAUNCH if a HIP call fails. */
int attn_valu_ceiling(int waves_per_simd, int iters, void* stream, unsigned long long* counters,
                      double* elements_per_s, double* core_ghz);

/* Static text for an error code. */
const char* attn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
