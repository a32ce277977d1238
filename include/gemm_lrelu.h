/* C ABI of the second tuned workload: fused GEMM + LeakyReLU on gfx950 (MI355X).
 *
 *     C = leaky_relu(A B),   leaky_relu(x) = x for x >= 0, slope * x otherwise
 *
 * The operation is the second kernel the paper tunes (Sec. 5, "Fused GEMM LeakyReLU", Table 3:
 * M, N, K = 512, 512, 2048 in binary16).  The paper does not state the slope; it is an argument.
 *
 * Layout: A [M, K], B [K, N], C [M, N], all row-major, contiguous, 16-bit elements (binary16 or
 * bfloat16 bit patterns, the same type for all three), DEVICE pointers aligned to 16 bytes.
 * Products are accumulated in fp32 on the matrix cores; the activation is applied to the fp32
 * sum, and the result is rounded once, to nearest even, into C.  The library owns no buffers and
 * allocates nothing; every call is asynchronous on the given stream.
 *
 * C must not overlap A or B.
 *
 * Shapes: M >= 1; N and K positive multiples of 8 (rows start on 16-byte boundaries); N, K < 2^24.
 * Ragged tiles are handled inside the kernel (rows and columns past the end are never stored,
 * k past the end contributes exact zeros).
 *
 * Every function returns GEMM_OK (0) or a negative error; nothing is launched on error.
 */
#ifndef PAPER_2403_16863_GEMM_LRELU_H
#define PAPER_2403_16863_GEMM_LRELU_H

#ifdef __cplusplus
extern "C" {
#endif

#define GEMM_OK 0
#define GEMM_EINVAL (-1)        /* null, misaligned or overlapping pointer, bad shape, dtype or variant */
#define GEMM_ELAUNCH (-2)       /* the HIP runtime refused a launch, an event or a copy */

#define GEMM_F16 0
#define GEMM_BF16 1

/* C = leaky_relu(A B) with the library's default schedule for the shape. */
int gemm_lrelu(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype, void* stream);

/* The same with schedule variant `variant_id` in [0, gemm_lrelu_num_variants()): the variants
 * are the points the schedule search (Alg. 1) walks for this workload. */
int gemm_lrelu_variant(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype,
                       void* stream, int variant_id);

int gemm_lrelu_num_variants(void);
int gemm_lrelu_default_variant(int M, int N, int K);

/* Knobs of a variant, in this order: "wk" (waves per workgroup; they split K), "bkw" (k extent a
 * wave loads per pipeline stage), "stages" (stages of each wave's LDS ring), "rot" (1: the workgroups of an XCD start at
 * different k and wrap around, so that their L2 misses do not coincide).  knobs: host, 4 ints. */
int gemm_lrelu_variant_knobs(int variant_id, int* knobs);

/* Timing aid for the search and the benchmark: `warmup` untimed launches, then `iters` launches
 * back to back between one pair of events; *ms_total (host) receives the time of all `iters`. */
int gemm_lrelu_time(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype,
                    void* stream, int variant_id, int warmup, int iters, float* ms_total);

/* Kernels loaded from code objects: the instruction-level schedule search (Sec. 3.1 to 3.3) takes
 * the compiled kernel of a variant, moves memory instructions in its assembly, assembles the result
 * and runs it through these.  `path` names a gfx950 code object file (host string), `kernel_name`
 * the kernel symbol in it; the kernel must take the arguments, launch shape and LDS of variant
 * `variant_id` for element type `dtype`.  Returns a handle >= 0 (at most 64 are open at a time;
 * GEMM_EINVAL when the table is full), or a negative error.  Unload only after the work that
 * uses the handle has finished.  The table of handles is process-wide and unguarded: load and
 * unload from one thread at a time (launches may come from any thread). */
int gemm_lrelu_codeobj_load(const char* path, const char* kernel_name, int variant_id, int dtype);
int gemm_lrelu_codeobj_unload(int handle);
/* gemm_lrelu / gemm_lrelu_time with the loaded kernel in place of the built-in one. */
int gemm_lrelu_codeobj(int handle, const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype,
                       void* stream);
int gemm_lrelu_time_codeobj(int handle, const void* a, const void* b, void* c, int M, int N, int K, float slope,
                            int dtype, void* stream, int warmup, int iters, float* ms_total);

/* The tile of C that workgroup `block` of `nblocks` computes (host logic, no GPU needed): tiles
 * are 32 x 32; ntm = ceil(M / 32), ntn = ceil(N / 32), nblocks = ntm * ntn.  Workgroups are
 * placed round-robin on the 8 XCDs; the map gives each XCD a contiguous run of tiles, ordered in
 * panels of 8 tile columns, so that one XCD's L2 holds few row strips of A and column strips of B.
 * Returns GEMM_EINVAL unless 0 <= block < nblocks = ntm * ntn. */
int gemm_lrelu_tile_of_block(int block, int ntm, int ntn, int* tm, int* tn);

#ifdef __cplusplus
}
#endif
#endif
