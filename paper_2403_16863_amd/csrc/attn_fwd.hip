// C ABI of the fused attention-forward library: argument checking, the table of
// schedule variants (the search space of Sec. 3.1 as compile-time instantiations of
// one kernel) and the event-timed measurement used as search feedback (Sec. 3.3).
#include "attn_kernel.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include "../../include/attn.h"

namespace {

using attn::Params;

typedef void (*KernelFn)(const Params);

struct Variant {
    int bn, nw, qb, occ, ldp, pipe, pf, prio, ilv, ldpos;  // knob values
    int coords[10];                                     // lattice coordinates (indices into the knob value lists)
    // kernels indexed [d == 128][dtype][causal]; null = not built for that combination
    KernelFn fn[2][2][2];
};

// Knob value lists (lattice axes): bn {32,64,128}  nw {4,8}  qb {1,2}  ldp {0,1}
// pipe {0,1,2,3}  pf {2,4,6,8}  prio {0,1,2}  dense {0,1}  ilv {0,1,2}  ldpos {0,1,2}.  The occupancy
// target follows from nw and qb (two workgroups per CU when one holds four waves of one query block
// each); dense = 1 asks for one workgroup more than that (three waves per SIMD: their vector
// instructions fill the issue slots a single wave leaves empty; d = 64 only, where the registers
// allow it).  ilv = how MFMA, LDS-read, transcendental and other vector instructions are grouped
// in the interleaved order (sched_group_barrier patterns), and for the ping-pong order the order of
// the softmax's vector instructions (0: every exponential followed by a multiply-add, an addition
// and every other time a conversion, pinned; 1: multiply-adds and exponentials alternating, then the
// sums and the conversion, pinned; 2: the compiler's own order); ldpos = where in the interleaved order's stream a
// wave issues its tile loads (all after the barrier, after fixed MFMA slots, after slots that
// depend on the wave): the position of the memory instructions, which is what Sec. 3.1 perturbs.
// On the ping-pong order ldpos 1 moves the tile loads one tile further ahead, into a third pair of
// buffers, which leaves one workgroup barrier per tile instead of two.
const char* const kKnobNames[] = {"bn", "nw", "qb", "ldp", "pipe", "pf", "prio", "dense", "ilv", "ldpos"};
const int kKnobSizes[] = {3, 2, 2, 2, 4, 4, 3, 2, 3, 3};
constexpr int kNumKnobs = 10;

#define ATTN_KN(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, ILV, LDPOS) attn::Knobs<BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, ILV, LDPOS>
#define ATTN_KERNELS_FOR(D, ...)                                                        \
    {                                                                                   \
        {(KernelFn)attn::attn_fwd_kernel<attn::F16, D, false, ATTN_KN(__VA_ARGS__)>,      \
         (KernelFn)attn::attn_fwd_kernel<attn::F16, D, true, ATTN_KN(__VA_ARGS__)>},      \
        {(KernelFn)attn::attn_fwd_kernel<attn::BF16, D, false, ATTN_KN(__VA_ARGS__)>,     \
         (KernelFn)attn::attn_fwd_kernel<attn::BF16, D, true, ATTN_KN(__VA_ARGS__)>}      \
    }
#define ATTN_NO_KERNELS {{nullptr, nullptr}, {nullptr, nullptr}}

// index helpers for the coordinate lists above
#define IDX_BN(x) ((x) == 32 ? 0 : (x) == 64 ? 1 : 2)
#define IDX_NW(x) ((x) == 4 ? 0 : 1)
#define IDX_QB(x) ((x) == 1 ? 0 : 1)
#define IDX_PF(x) ((x) / 2 - 1)
#define IDX_DENSE(NW, QB, OCC) ((OCC) - (((NW) == 4 && (QB) == 1) ? 2 : 1))
#define VARIANT_HEAD(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, ILV, LDPOS)                              \
    BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, ILV, LDPOS,                                               \
    {IDX_BN(BN), IDX_NW(NW), IDX_QB(QB), LDP, PIPE, IDX_PF(PF), PRIO, IDX_DENSE(NW, QB, OCC), ILV, LDPOS}

// variants of the first three loop orders have no interleave pattern and no load position
#define VARIANT_BOTH(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO)                                          \
    {VARIANT_HEAD(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0),                                      \
     {ATTN_KERNELS_FOR(64, BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0),                             \
      ATTN_KERNELS_FOR(128, BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0)}}
#define VARIANT_D64(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO)                                           \
    {VARIANT_HEAD(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0),                                      \
     {ATTN_KERNELS_FOR(64, BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0), ATTN_NO_KERNELS}}
#define VARIANT_D128(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO)                                          \
    {VARIANT_HEAD(BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0),                                      \
     {ATTN_NO_KERNELS, ATTN_KERNELS_FOR(128, BN, NW, QB, OCC, LDP, PIPE, PF, PRIO, 0, 0)}}
// the interleaved order (pipe 3), d = 128: 256-row query tiles, 64-key tiles
#define VARIANT_ILV(LDP, PF, PRIO, ILV, LDPOS)                                                      \
    {VARIANT_HEAD(64, 8, 1, 1, LDP, 3, PF, PRIO, ILV, LDPOS),                                       \
     {ATTN_NO_KERNELS, ATTN_KERNELS_FOR(128, 64, 8, 1, 1, LDP, 3, PF, PRIO, ILV, LDPOS)}}

// the ping-pong order of variant 11 with another order of the V cluster's vector instructions (d = 128)
#define VARIANT_PP_ILV(ILV)                                                                         \
    {VARIANT_HEAD(64, 8, 1, 1, 1, 1, 4, 1, ILV, 0),                                                 \
     {ATTN_NO_KERNELS, ATTN_KERNELS_FOR(128, 64, 8, 1, 1, 1, 1, 4, 1, ILV, 0)}}

// the ping-pong order with three buffers and one barrier per tile (ldpos 1 on that order; d = 128)
#define VARIANT_PP_3BUF(PF)                                                                         \
    {VARIANT_HEAD(64, 8, 1, 1, 1, 1, PF, 1, 0, 1),                                                  \
     {ATTN_NO_KERNELS, ATTN_KERNELS_FOR(128, 64, 8, 1, 1, 1, 1, PF, 1, 0, 1)}}

const Variant kVariants[] = {
    VARIANT_BOTH(64, 4, 1, 2, 1, 0, 4, 0),   // 0: the hand-written default
    VARIANT_BOTH(64, 4, 1, 2, 1, 0, 2, 0),
    VARIANT_BOTH(64, 4, 1, 2, 1, 0, 6, 0),
    VARIANT_BOTH(64, 4, 1, 2, 1, 0, 4, 1),
    VARIANT_BOTH(64, 4, 1, 2, 0, 0, 4, 0),
    VARIANT_BOTH(32, 4, 1, 2, 1, 0, 4, 0),
    VARIANT_BOTH(32, 4, 1, 2, 1, 0, 2, 0),
    VARIANT_BOTH(64, 8, 1, 1, 1, 0, 4, 0),
    VARIANT_BOTH(64, 8, 1, 1, 1, 0, 6, 0),
    VARIANT_BOTH(64, 8, 1, 1, 1, 1, 2, 0),
    VARIANT_BOTH(64, 8, 1, 1, 1, 1, 4, 0),
    VARIANT_BOTH(64, 8, 1, 1, 1, 1, 4, 1),
    VARIANT_BOTH(64, 8, 1, 1, 0, 1, 4, 0),
    VARIANT_BOTH(64, 4, 2, 1, 1, 0, 4, 0),
    VARIANT_D64(128, 4, 1, 2, 1, 0, 4, 0),
    VARIANT_D128(64, 8, 1, 1, 1, 2, 2, 1),   // 15, 16: MFMA work in both ping-pong clusters
    VARIANT_D128(64, 8, 1, 1, 1, 2, 4, 1),
    VARIANT_D64(64, 4, 1, 3, 1, 0, 4, 0),    // 17 .. 19: three free-running workgroups per CU (d = 64)
    VARIANT_D64(64, 4, 1, 3, 1, 0, 4, 1),
    VARIANT_D64(64, 4, 1, 3, 1, 0, 2, 1),
    VARIANT_BOTH(64, 8, 1, 1, 1, 1, 4, 2),   // 20: ping-pong, priority raised while a wave issues tile loads
    VARIANT_ILV(0, 4, 0, 0, 0),              // 21 ..: the interleaved order, tiles through registers
    VARIANT_ILV(0, 4, 0, 0, 1),
    VARIANT_ILV(0, 4, 0, 0, 2),
    VARIANT_ILV(0, 2, 0, 0, 1),
    VARIANT_ILV(0, 8, 0, 0, 1),
    VARIANT_ILV(0, 4, 1, 0, 1),
    VARIANT_ILV(0, 4, 2, 0, 1),
    VARIANT_ILV(0, 4, 0, 1, 1),
    VARIANT_ILV(0, 4, 0, 2, 1),
    VARIANT_ILV(1, 4, 0, 0, 0),              // 30 .. 32: the interleaved order, tiles straight to LDS
    VARIANT_ILV(1, 4, 0, 0, 1),
    VARIANT_ILV(1, 4, 1, 0, 0),              // (one knob away from variant 16: the lattice stays connected)
    VARIANT_PP_ILV(1),                       // 33, 34: the default ping-pong kernel with the other orders of the softmax
    VARIANT_PP_ILV(2),                       //         instructions (a second pinned order; the compiler's own order)
    VARIANT_PP_3BUF(4),                      // 35, 36: ping-pong with three K/V buffers, loads one tile further ahead,
    VARIANT_PP_3BUF(2),                      //         one workgroup barrier per tile (pf 4 / 2)
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

// Compute units of the current device (queried once per device).
int cu_count() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

// Persistent workgroups: as many as the device keeps resident (occ per CU), a multiple of 8
// when every XCD can be given whole heads, never more than there are work items.
long long grid_size(int cus, int occ, int BH, long long nqt) {
    const long long total = (long long)BH * nqt, resident = (long long)cus * occ;
    if ((BH & 7) == 0 && (resident & 7) == 0) {
        const long long per_xcd_items = (long long)(BH >> 3) * nqt, per_xcd_wg = resident >> 3;
        return 8 * (per_xcd_items < per_xcd_wg ? per_xcd_items : per_xcd_wg);
    }
    return total < resident ? total : resident;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// Everything that can be rejected without touching the device.
int check_args(const void* q, const void* k, const void* v, void* out, float* lse, int B, int H,
               int N, int d, float scale, int dtype, int variant_id) {
    if (!q || !k || !v || !out || !lse) return ATTN_EINVAL;
    if (B < 1 || H < 1 || N < 1) return ATTN_EINVAL;
    if (dtype != ATTN_F16 && dtype != ATTN_BF16) return ATTN_EINVAL;
    if (!isfinite(scale)) return ATTN_EINVAL;
    if (variant_id < 0 || variant_id >= kNumVariants) return ATTN_EINVAL;
    if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16) || !aligned(lse, 4))
        return ATTN_EINVAL;
    if (d != 64 && d != 128) return ATTN_EUNSUPPORTED;
    const unsigned long long elems = (unsigned long long)B * H * N * d;
    if (elems > (1ull << 40)) return ATTN_EUNSUPPORTED;  // keeps every byte offset far inside 64 bits
    const size_t bytes = (size_t)elems * 2;
    if (overlaps(out, bytes, q, bytes) || overlaps(out, bytes, k, bytes) || overlaps(out, bytes, v, bytes))
        return ATTN_EINVAL;
    const size_t lse_bytes = (size_t)B * H * N * 4;
    if (overlaps(lse, lse_bytes, q, bytes) || overlaps(lse, lse_bytes, k, bytes) ||
        overlaps(lse, lse_bytes, v, bytes) || overlaps(lse, lse_bytes, out, bytes))
        return ATTN_EINVAL;
    return ATTN_OK;
}

// Launches the variant's own kernel, or, when `module_fn` is given, a kernel loaded from a
// code object that was derived from that variant's kernel (same arguments, same grid, same
// block, same LDS).
int launch(const void* q, const void* k, const void* v, void* out, float* lse, int B, int H, int N,
           int d, int causal, float scale, int dtype, void* stream, int variant_id,
           hipFunction_t module_fn = nullptr) {
    const int rc = check_args(q, k, v, out, lse, B, H, N, d, scale, dtype, variant_id);
    if (rc != ATTN_OK) return rc;
    const Variant& var = kVariants[variant_id];
    const KernelFn fn = var.fn[d == 128][dtype][causal ? 1 : 0];
    if (!fn) return ATTN_EUNSUPPORTED;
    const int bm = 32 * var.qb * var.nw;
    const long long nqt = ((long long)N + bm - 1) / bm;
    const long long total = nqt * B * H;
    if (total > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    // the interleaved order addresses K and V of a head through a buffer descriptor: 32-bit byte offsets
    if (var.pipe == 3 && (long long)N * d * 2 > 0xffffffffLL) return ATTN_EUNSUPPORTED;

    Params p;
    p.q = (const uint16_t*)q;
    p.k = (const uint16_t*)k;
    p.v = (const uint16_t*)v;
    p.out = (uint16_t*)out;
    p.lse = lse;
    p.H = H;
    p.N = N;
    p.nqt = (int)nqt;
    p.BH = B * H;
    // The kernel tracks the running maximum of the raw dot products, which needs a
    // positive multiplier: a negative scale is moved into the sign of Q, a zero scale
    // into Q = 0.
    p.qmode = scale > 0.f ? 0 : (scale < 0.f ? 1 : 2);
    p.scale = scale > 0.f ? scale : (scale < 0.f ? -scale : 1.0f);
    p.scale_l2 = p.scale * 1.44269504088896340736f;
    const long long grid = grid_size(cu_count(), var.occ, p.BH, nqt);
    // The launch's own return code is used (not hipGetLastError, which can report a
    // stale, unrelated status left behind by another library's earlier call).
    void* args[] = {&p};
    const hipError_t e =
        module_fn ? hipModuleLaunchKernel(module_fn, (unsigned)grid, 1, 1, var.nw * 64, 1, 1, 0, (hipStream_t)stream, args, nullptr)
                  : hipLaunchKernel((const void*)fn, dim3((unsigned)grid), dim3(var.nw * 64), args, 0, (hipStream_t)stream);
    if (e != hipSuccess) fprintf(stderr, "attn: kernel launch failed: %s (%d), grid=%lld block=%d\n", hipGetErrorString(e), (int)e, grid, var.nw * 64);
    return e == hipSuccess ? ATTN_OK : ATTN_ELAUNCH;
}

// ---- kernels loaded from code objects (instruction-level schedule search).  A small fixed
// table; a slot records what the kernel was derived from so that a launch can be refused
// when the shape does not match.
struct LoadedKernel {
    hipModule_t module = nullptr;
    hipFunction_t fn = nullptr;
    int variant_id = -1, d = 0, dtype = 0, causal = 0;
};
constexpr int kMaxLoaded = 64;
LoadedKernel g_loaded[kMaxLoaded];

const LoadedKernel* loaded_for(int handle, int d, int dtype, int causal, int* rc) {
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn) { *rc = ATTN_EINVAL; return nullptr; }
    const LoadedKernel& lk = g_loaded[handle];
    if (lk.d != d || lk.dtype != dtype || lk.causal != (causal ? 1 : 0)) { *rc = ATTN_EUNSUPPORTED; return nullptr; }
    *rc = ATTN_OK;
    return &lk;
}

// Shared by the two timing entry points: `warmup` untimed launches, then `iters` launches
// each bracketed by its own pair of events.
template <class LaunchFn>
int time_launches(LaunchFn&& do_launch, void* stream, int warmup, int iters, float* ms) {
    if (!ms || iters < 1 || warmup < 0) return ATTN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < warmup; ++i) {
        const int rc = do_launch();
        if (rc != ATTN_OK) return rc;
    }
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return ATTN_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return ATTN_ELAUNCH; }
    int rc = ATTN_OK;
    for (int i = 0; i < iters && rc == ATTN_OK; ++i) {
        if (hipEventRecord(e0, s) != hipSuccess) { rc = ATTN_ELAUNCH; break; }
        rc = do_launch();
        if (rc != ATTN_OK) break;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms[i], e0, e1) != hipSuccess)
            rc = ATTN_ELAUNCH;
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return rc;
}


// ---- measurement aid: what the MFMA pipe sustains on this device.  Every wave issues
// independent 32x32x16 bf16 MFMAs back to back (four accumulators, operands fixed in
// registers, no memory traffic), two waves per SIMD.  With constant operands this reaches
// the clock-limited peak; with random operands the switching activity makes the device
// lower its clock (power management), which bounds what any kernel fed real data can reach.
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(unsigned long long* counters, int iters, int random_operands) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    u32x4 a[4], b[4];
    unsigned st = (blockIdx.x * 256 + threadIdx.x) * 2654435761u + 12345u;
    for (int n = 0; n < 4; ++n)
        for (int j = 0; j < 4; ++j) {
            st = st * 1664525u + 1013904223u;
            unsigned ra = st;
            st = st * 1664525u + 1013904223u;
            unsigned rb = st;
            if (!random_operands) {
                ra = rb = 0x3f803f80u;  // 1.0, 1.0
            } else {  // random sign and mantissa, exponent 126 or 127: magnitudes in [0.5, 2)
                ra = (ra & 0x807f807fu) | 0x3f003f00u | ((ra >> 3) & 0x00800080u);
                rb = (rb & 0x807f807fu) | 0x3f003f00u | ((rb >> 5) & 0x00800080u);
            }
            a[n][j] = ra;
            b[n][j] = rb;
        }
    f32x16 acc[4];
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 4; ++n)
            acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[n]), __builtin_bit_cast(bf16x8, b[n]), acc[n], 0, 0, 0);
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    float sum = 0;
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) sum += acc[n][v];
    if (blockIdx.x == 7 && threadIdx.x == 0) {
        counters[0] = c1 - c0;  // core clock cycles
        counters[1] = r1 - r0;  // ticks of the constant 100 MHz clock
    }
    if (sum == 1.2345e-30f) counters[2] = 1;  // keeps the accumulators alive
}

// ---- measurement aid: what a kernel with this path's instruction mix sustains.  Per 32x32x16 MFMA
// the tile loop reads one 1 KB operand fragment from LDS and issues, for the softmax of the one
// score element a lane owns per MFMA (a wave's 32 x 64 scores take 32 MFMAs), one multiply-add,
// one exp2, one add and half a conversion.  This
// kernel issues exactly that per MFMA, with random operands, fragments read from LDS four steps
// ahead, two waves per SIMD, and nothing else: no tile loads, no barriers, no masks, no item
// boundaries.  The device runs it at its power limit like the attention kernel, so the rate is
// the ceiling of the loop body on this device; mode 0 leaves out the LDS reads and the vector
// work (the MFMA-only rate with two waves per SIMD), mode 1 adds the LDS reads, mode 2 adds both.
template <int MODE>
__global__ __launch_bounds__(512) void mix_ceiling_kernel(unsigned long long* counters, int iters) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    __shared__ u32x4 lds[4096];  // 64 KB of random 16-bit patterns
    unsigned st = (blockIdx.x * 512 + threadIdx.x) * 2654435761u + 12345u;
    auto rnd = [&]() {  // random sign and mantissa, exponent 126 or 127: magnitudes in [0.5, 2)
        st = st * 1664525u + 1013904223u;
        return (st & 0x807f807fu) | 0x3f003f00u | ((st >> 3) & 0x00800080u);
    };
    for (int i = threadIdx.x; i < 4096; i += 512) lds[i] = u32x4{rnd(), rnd(), rnd(), rnd()};
    __syncthreads();
    u32x4 a[4], b[4];
    for (int n = 0; n < 4; ++n) {
        a[n] = u32x4{rnd(), rnd(), rnd(), rnd()};
        b[n] = u32x4{rnd(), rnd(), rnd(), rnd()};
    }
    f32x16 acc[4];
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = -0.01f * (float)((st >> (i & 7)) & 255);
    float rs0 = 0.f, rs1 = 0.f;
    unsigned keep = 0;
    const char* lb = reinterpret_cast<const char*>(lds) + ((threadIdx.x * 16) & 0x3ff0);
    u32x4 ring[4];
    for (int n = 0; n < 4; ++n) ring[n] = *reinterpret_cast<const u32x4*>(lb + n * 16384);
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            u32x4 av = a[n & 3];
            if constexpr (MODE >= 1) av = ring[n & 3];
            acc[n & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, b[n & 3]), acc[n & 3], 0, 0, 0);
            if constexpr (MODE >= 1) ring[n & 3] = *reinterpret_cast<const u32x4*>(lb + (n & 3) * 16384);
            if constexpr (MODE >= 2) {
                const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x[n], 0.127517f, -0.25f));
                if (n & 1) {
                    rs1 += e;
                    unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{x[n - 1], e}, bf16x2));
                    asm volatile("" : "+v"(pk));
                    keep ^= pk;
                } else {
                    rs0 += e;
                }
                asm volatile("" : "+v"(x[n]));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    float sum = rs0 + rs1;
    for (int n = 0; n < 4; ++n)
        for (int v = 0; v < 16; ++v) sum += acc[n][v];
    if (blockIdx.x == 7 && threadIdx.x == 0) {
        counters[0] = c1 - c0;  // core clock cycles
        counters[1] = r1 - r0;  // ticks of the constant 100 MHz clock
    }
    if (sum == 1.2345e-30f || keep == 0x12345678u) counters[2] = 1;  // keeps the results alive
}

// ---- measurement aid: the same work in the ping-pong form and nothing else.  Eight waves per workgroup,
// two per SIMD; per "tile" a wave runs one MFMA cluster (32 MFMAs, each with one 1 KB fragment read
// from LDS two steps ahead, the first 16 on four accumulators, the other 16 on two, like PV and S) and
// one vector cluster (per lane 32 multiply-adds, 32 exp2, 32 additions, 16 conversions, in the pinned
// order of the attention kernel), the waves 4..7 in the opposite order, with BARRIERS workgroup
// barriers per tile (2: after every cluster; 1: after every tile).  No tile loads, masks, item
// boundaries or epilogues: what is left is the structure itself, one wave of a SIMD feeding the
// matrix pipe while the other one issues vector instructions.
template <int BARRIERS>
__global__ __launch_bounds__(512) void pingpong_ceiling_kernel(unsigned long long* counters, int iters) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    __shared__ u32x4 lds[4096];  // 64 KB of random 16-bit patterns
    unsigned st = (blockIdx.x * 512 + threadIdx.x) * 2654435761u + 12345u;
    auto rnd = [&]() {  // random sign and mantissa, exponent 126 or 127: magnitudes in [0.5, 2)
        st = st * 1664525u + 1013904223u;
        return (st & 0x807f807fu) | 0x3f003f00u | ((st >> 3) & 0x00800080u);
    };
    for (int i = threadIdx.x; i < 4096; i += 512) lds[i] = u32x4{rnd(), rnd(), rnd(), rnd()};
    __syncthreads();
    u32x4 b[4];
    for (int n = 0; n < 4; ++n) b[n] = u32x4{rnd(), rnd(), rnd(), rnd()};
    f32x16 acc[6];
    for (int n = 0; n < 6; ++n)
        for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
    float x[32];
    for (int i = 0; i < 32; ++i) x[i] = -0.01f * (float)((st >> (i & 7)) & 255);
    float rs0 = 0.f, rs1 = 0.f;
    unsigned keep = 0;
    const char* lb = reinterpret_cast<const char*>(lds) + ((threadIdx.x * 16) & 0x3ff0);
    const bool grp_b = threadIdx.x >= 256;
    auto cluster_m = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_setprio(2);
        u32x4 ring[2];
        ring[0] = *reinterpret_cast<const u32x4*>(lb);
        ring[1] = *reinterpret_cast<const u32x4*>(lb + 16384);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            const int a = n < 16 ? (n & 3) : 4 + (n & 1);
            acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ring[n & 1]), __builtin_bit_cast(bf16x8, b[n & 3]), acc[a], 0, 0, 0);
            if (n + 2 < 32) ring[n & 1] = *reinterpret_cast<const u32x4*>(lb + ((n + 2) & 3) * 16384);
            __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_s_setprio(0);
    };
    auto cluster_v = [&]() __attribute__((always_inline)) {
        float xa = 0.f, xb = 0.f, ea = 0.f, eb = 0.f;
#pragma unroll
        for (int i = 0; i < 18; ++i) {  // pair i enters, pair i-1 in exp2, pair i-2 leaves
            float na = 0.f, nb = 0.f, fa = 0.f, fb = 0.f;
            if (i >= 1 && i <= 16) { fa = __builtin_amdgcn_exp2f(xa); __builtin_amdgcn_sched_barrier(0); }
            if (i < 16) { na = __builtin_fmaf(x[2 * i], 0.127517f, -0.25f); __builtin_amdgcn_sched_barrier(0); }
            if (i >= 2) { rs0 += ea; __builtin_amdgcn_sched_barrier(0); }
            if (i >= 2) {
                unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{ea, eb}, bf16x2));
                asm volatile("" : "+v"(pk));
                keep ^= pk;
                __builtin_amdgcn_sched_barrier(0);
            }
            if (i >= 1 && i <= 16) { fb = __builtin_amdgcn_exp2f(xb); __builtin_amdgcn_sched_barrier(0); }
            if (i < 16) { nb = __builtin_fmaf(x[2 * i + 1], 0.127517f, -0.25f); __builtin_amdgcn_sched_barrier(0); }
            if (i >= 2) { rs1 += eb; __builtin_amdgcn_sched_barrier(0); }
            xa = na; xb = nb; ea = fa; eb = fb;
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) asm volatile("" : "+v"(x[i]));
    };
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    if (!grp_b) {
        for (int it = 0; it < iters; ++it) {
            cluster_m();
            if constexpr (BARRIERS == 2) __syncthreads();
            cluster_v();
            __syncthreads();
        }
    } else {
        for (int it = 0; it < iters; ++it) {
            cluster_v();
            if constexpr (BARRIERS == 2) __syncthreads();
            cluster_m();
            __syncthreads();
        }
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    float sum = rs0 + rs1;
    for (int n = 0; n < 6; ++n)
        for (int v = 0; v < 16; ++v) sum += acc[n][v];
    if (blockIdx.x == 7 && threadIdx.x == 0) {
        counters[0] = c1 - c0;  // core clock cycles
        counters[1] = r1 - r0;  // ticks of the constant 100 MHz clock
    }
    if (sum == 1.2345e-30f || keep == 0x12345678u) counters[2] = 1;  // keeps the results alive
}

// ---- measurement aid: what the vector ALU sustains on the softmax's own instruction mix.  Per
// score element the one-pass softmax issues one fma (scale and shift), one exp2, one add (row sum)
// and half a conversion (two probabilities per packed 16-bit pair); this kernel issues exactly
// that mix on independent data from registers, 16 elements per round like one 32-key half tile,
// with a chosen number of waves per SIMD.  Ordinary scalar float code: the build keeps the compiler
// from forming packed-fp32 instructions.
__global__ __launch_bounds__(256) void valu_ceiling_kernel(unsigned long long* counters, int iters, float scale, float shift) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = -0.01f * (float)((threadIdx.x * 16 + i) & 255);
    float rs0 = 0.f, rs1 = 0.f;
    unsigned keep = 0;
    const unsigned long long c0 = clock64(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], scale, shift));
            const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i + 1], scale, shift));
            rs0 += e0;
            rs1 += e1;
            unsigned pk = __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{e0, e1}, bf16x2));
            asm volatile("" : "+v"(pk));  // the conversion is part of the mix: keep it
            keep ^= pk;
        }
        asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]));
        asm volatile("" : "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14]), "+v"(x[15]));
    }
    const unsigned long long c1 = clock64(), r1 = wall_clock64();
    if (blockIdx.x == 7 && threadIdx.x == 0) {
        counters[0] = c1 - c0;  // core clock cycles
        counters[1] = r1 - r0;  // ticks of the constant 100 MHz clock
    }
    if (rs0 + rs1 == 1.2345e-30f || keep == 0x12345678u) counters[2] = 1;  // keeps the results alive
}

}  // namespace

extern "C" {

int attn_num_variants(void) { return kNumVariants; }

int attn_schedule_grid(int variant_id, int compute_units, int B, int H, int N) {
    if (variant_id < 0 || variant_id >= kNumVariants || compute_units < 1 || B < 1 || H < 1 || N < 1) return ATTN_EINVAL;
    const Variant& var = kVariants[variant_id];
    const int bm = 32 * var.qb * var.nw;
    const long long nqt = ((long long)N + bm - 1) / bm, g = grid_size(compute_units, var.occ, B * H, nqt);
    if ((long long)B * H > 0x7fffffffLL / nqt || g > 0x7fffffffLL) return ATTN_EUNSUPPORTED;
    return (int)g;
}

int attn_schedule_item(int grid, int workgroup, int BH, int nqt, int round, int* bh, int* qt) {
    if (grid < 1 || workgroup < 0 || workgroup >= grid || BH < 1 || nqt < 1 || round < 0 || !bh || !qt) return ATTN_EINVAL;
    int b = 0, q = 0;
    if (!attn::schedule_item(grid, workgroup, BH, nqt, round, b, q)) return 0;
    *bh = b;
    *qt = q;
    return 1;
}

int attn_variant_supported(int variant_id, int d, int dtype, int causal) {
    if (variant_id < 0 || variant_id >= kNumVariants) return ATTN_EINVAL;
    if ((d != 64 && d != 128) || (dtype != ATTN_F16 && dtype != ATTN_BF16)) return 0;
    return kVariants[variant_id].fn[d == 128][dtype][causal ? 1 : 0] != nullptr;
}

int attn_variant_desc(int variant_id, char* buf, int buflen) {
    if (variant_id < 0 || variant_id >= kNumVariants || !buf || buflen < 1) return ATTN_EINVAL;
    const Variant& v = kVariants[variant_id];
    return snprintf(buf, (size_t)buflen, "bm=%d bn=%d nw=%d qb=%d occ=%d ldp=%d pipe=%d pf=%d prio=%d ilv=%d ldpos=%d",
                    32 * v.qb * v.nw, v.bn, v.nw, v.qb, v.occ, v.ldp, v.pipe, v.pf, v.prio, v.ilv, v.ldpos);
}

int attn_num_knobs(void) { return kNumKnobs; }

const char* attn_knob_name(int knob) { return (knob < 0 || knob >= kNumKnobs) ? nullptr : kKnobNames[knob]; }

int attn_knob_size(int knob) { return (knob < 0 || knob >= kNumKnobs) ? ATTN_EINVAL : kKnobSizes[knob]; }

int attn_variant_coords(int variant_id, int* coords) {
    if (variant_id < 0 || variant_id >= kNumVariants || !coords) return ATTN_EINVAL;
    for (int i = 0; i < kNumKnobs; ++i) coords[i] = kVariants[variant_id].coords[i];
    return ATTN_OK;
}

int attn_variant_from_coords(const int* coords) {
    if (!coords) return ATTN_EINVAL;
    for (int id = 0; id < kNumVariants; ++id)
        if (memcmp(kVariants[id].coords, coords, sizeof(int) * kNumKnobs) == 0) return id;
    return ATTN_EINVAL;
}

// Defaults chosen from the measured search over the variant table on MI355X: the
// two-cluster ping-pong order (256-row query tiles) wins for head_dim 128, in its form with
// three buffers, one barrier per tile and an LDS prefetch distance of 2 (about 1 % ahead of the
// two-buffer form, variant 11, on both long workloads, every time the two were timed alternately);
// long sequences with head_dim 64 run three free-running workgroups per compute unit, short ones
// have too few 256-row tiles to go round and run the free-running order on 128-row tiles.
// (Ids index kVariants.)
constexpr int kDefaultD128 = 36;
constexpr int kDefaultD64Long = 18;
constexpr int kDefaultD64Short = 3;

int attn_default_variant(int N, int d, int dtype, int causal) {
    (void)dtype; (void)causal;
    if (d == 128) return kDefaultD128;
    return N >= 2048 ? kDefaultD64Long : kDefaultD64Short;
}

int attn_fwd_variant(const void* q, const void* k, const void* v, void* out, float* lse, int B, int H,
                     int N, int d, int causal, float scale, int dtype, void* stream, int variant_id) {
    return launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream, variant_id);
}

// ---- deployed schedules (Sec. 4.1): what attn_fwd launches instead of the default, by shape
// class.  A small fixed table searched newest first; handle >= 0 names a loaded code object.
struct Deployment {
    bool used = false;
    int variant_id = -1, handle = -1, d = 0, dtype = 0, causal = 0, n_min = 0, n_max = 0;
};
constexpr int kMaxDeployed = 16;
static Deployment g_deployed[kMaxDeployed];
static int g_num_deployed = 0;

static const Deployment* deployed_for(int N, int d, int dtype, int causal) {
    for (int i = g_num_deployed - 1; i >= 0; --i) {
        const Deployment& e = g_deployed[i];
        if (e.used && e.d == d && e.dtype == dtype && e.causal == (causal ? 1 : 0) && N >= e.n_min && N <= e.n_max) return &e;
    }
    return nullptr;
}

static int add_deployment(const Deployment& e) {
    if (g_num_deployed == kMaxDeployed) {  // reuse the room of removed entries, keeping the order
        int n = 0;
        for (int i = 0; i < kMaxDeployed; ++i)
            if (g_deployed[i].used) g_deployed[n++] = g_deployed[i];
        for (int i = n; i < kMaxDeployed; ++i) g_deployed[i] = Deployment();
        g_num_deployed = n;
        if (n == kMaxDeployed) return ATTN_EUNSUPPORTED;
    }
    g_deployed[g_num_deployed++] = e;
    return ATTN_OK;
}

int attn_fwd(const void* q, const void* k, const void* v, void* out, float* lse, int B, int H, int N,
             int d, int causal, float scale, int dtype, void* stream) {
    if (g_num_deployed > 0) {
        if (const Deployment* e = deployed_for(N, d, dtype, causal)) {
            const int rc = launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream, e->variant_id,
                                  e->handle >= 0 ? g_loaded[e->handle].fn : nullptr);
            if (rc != ATTN_EUNSUPPORTED) return rc;
        }
    }
    return launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream,
                  attn_default_variant(N, d, dtype, causal));
}

int attn_deploy_variant(int variant_id, int d, int dtype, int causal, int n_min, int n_max) {
    if (variant_id < 0 || variant_id >= kNumVariants || n_min < 1 || n_max < n_min) return ATTN_EINVAL;
    if ((d != 64 && d != 128) || (dtype != ATTN_F16 && dtype != ATTN_BF16)) return ATTN_EINVAL;
    if (!kVariants[variant_id].fn[d == 128][dtype][causal ? 1 : 0]) return ATTN_EUNSUPPORTED;
    Deployment e;
    e.used = true;
    e.variant_id = variant_id;
    e.d = d;
    e.dtype = dtype;
    e.causal = causal ? 1 : 0;
    e.n_min = n_min;
    e.n_max = n_max;
    return add_deployment(e);
}

int attn_deploy_codeobj(int handle, int n_min, int n_max) {
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn || n_min < 1 || n_max < n_min) return ATTN_EINVAL;
    const LoadedKernel& lk = g_loaded[handle];
    Deployment e;
    e.used = true;
    e.variant_id = lk.variant_id;
    e.handle = handle;
    e.d = lk.d;
    e.dtype = lk.dtype;
    e.causal = lk.causal;
    e.n_min = n_min;
    e.n_max = n_max;
    return add_deployment(e);
}

int attn_deploy_clear(void) {
    for (int i = 0; i < kMaxDeployed; ++i) g_deployed[i] = Deployment();
    g_num_deployed = 0;
    return ATTN_OK;
}

int attn_deployed(int N, int d, int dtype, int causal, int* variant_id, int* handle) {
    if (N < 1 || (d != 64 && d != 128) || (dtype != ATTN_F16 && dtype != ATTN_BF16)) return ATTN_EINVAL;
    const Deployment* e = deployed_for(N, d, dtype, causal);
    if (variant_id) *variant_id = e ? e->variant_id : attn_default_variant(N, d, dtype, causal);
    if (handle) *handle = e ? e->handle : -1;
    return e ? 1 : 0;
}

int attn_time_variant(const void* q, const void* k, const void* v, void* out, float* lse, int B, int H,
                      int N, int d, int causal, float scale, int dtype, void* stream, int variant_id,
                      int warmup, int iters, float* ms) {
    return time_launches([&] { return launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream, variant_id); },
                         stream, warmup, iters, ms);
}

int attn_codeobj_load(const char* path, const char* kernel_name, int variant_id, int d, int dtype, int causal) {
    if (!path || !kernel_name || variant_id < 0 || variant_id >= kNumVariants) return ATTN_EINVAL;
    if ((d != 64 && d != 128) || (dtype != ATTN_F16 && dtype != ATTN_BF16)) return ATTN_EINVAL;
    if (!kVariants[variant_id].fn[d == 128][dtype][causal ? 1 : 0]) return ATTN_EUNSUPPORTED;
    int slot = -1;
    for (int i = 0; i < kMaxLoaded; ++i)
        if (!g_loaded[i].fn) { slot = i; break; }
    if (slot < 0) return ATTN_EUNSUPPORTED;  // table full: unload something first
    // A failed runtime call leaves its status behind for whoever asks next (another library in
    // the process would report it as its own): look at the file first, and consume the status
    // of a load that fails anyway.
    if (FILE* f = fopen(path, "rb")) fclose(f);
    else return ATTN_ELAUNCH;
    LoadedKernel lk;
    if (hipModuleLoad(&lk.module, path) != hipSuccess) {
        (void)hipGetLastError();
        return ATTN_ELAUNCH;
    }
    if (hipModuleGetFunction(&lk.fn, lk.module, kernel_name) != hipSuccess) {
        (void)hipGetLastError();
        hipModuleUnload(lk.module);
        return ATTN_ELAUNCH;
    }
    lk.variant_id = variant_id;
    lk.d = d;
    lk.dtype = dtype;
    lk.causal = causal ? 1 : 0;
    g_loaded[slot] = lk;
    return slot;
}

int attn_codeobj_unload(int handle) {
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn) return ATTN_EINVAL;
    for (int i = 0; i < kMaxDeployed; ++i)  // attn_fwd must not launch a kernel that is gone
        if (g_deployed[i].used && g_deployed[i].handle == handle) g_deployed[i] = Deployment();
    const hipError_t e = hipModuleUnload(g_loaded[handle].module);
    g_loaded[handle] = LoadedKernel();
    return e == hipSuccess ? ATTN_OK : ATTN_ELAUNCH;
}

int attn_fwd_codeobj(int handle, const void* q, const void* k, const void* v, void* out, float* lse,
                     int B, int H, int N, int d, int causal, float scale, int dtype, void* stream) {
    int rc;
    const LoadedKernel* lk = loaded_for(handle, d, dtype, causal, &rc);
    if (!lk) return rc;
    return launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream, lk->variant_id, lk->fn);
}

int attn_time_codeobj(int handle, const void* q, const void* k, const void* v, void* out, float* lse,
                      int B, int H, int N, int d, int causal, float scale, int dtype, void* stream,
                      int warmup, int iters, float* ms) {
    int rc;
    const LoadedKernel* lk = loaded_for(handle, d, dtype, causal, &rc);
    if (!lk) return rc;
    return time_launches([&] { return launch(q, k, v, out, lse, B, H, N, d, causal, scale, dtype, stream, lk->variant_id, lk->fn); },
                         stream, warmup, iters, ms);
}

int attn_mfma_ceiling(int random_operands, int iters, void* stream, unsigned long long* counters,
                      double* tflops, double* core_ghz) {
    if (iters < 1 || !counters || !tflops || !core_ghz) return ATTN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int blocks = 2 * cu_count();  // 8 waves per CU
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return ATTN_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return ATTN_ELAUNCH; }
    int rc = ATTN_OK;
    float ms = 0.f;
    unsigned long long h[2] = {0, 0};
    void* args[] = {&counters, &iters, &random_operands};
    if (hipEventRecord(e0, s) != hipSuccess ||
        hipLaunchKernel((const void*)mfma_ceiling_kernel, dim3(blocks), dim3(256), args, 0, s) != hipSuccess ||
        hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(h, counters, sizeof h, hipMemcpyDeviceToHost) != hipSuccess)
        rc = ATTN_ELAUNCH;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != ATTN_OK) return rc;
    *tflops = (double)blocks * 4 * (double)iters * 4 * 32768.0 / ((double)ms * 1e-3) / 1e12;
    *core_ghz = h[1] ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;
    return ATTN_OK;
}

int attn_mix_ceiling(int mode, int iters, void* stream, unsigned long long* counters, double* tflops, double* core_ghz) {
    if (mode < 0 || mode > 4 || iters < 1 || !counters || !tflops || !core_ghz) return ATTN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int blocks = cu_count();  // one workgroup of 8 waves per CU: two waves per SIMD
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return ATTN_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return ATTN_ELAUNCH; }
    int rc = ATTN_OK;
    float ms = 0.f;
    unsigned long long h[2] = {0, 0};
    void* args[] = {&counters, &iters};
    const void* kernels[5] = {(const void*)mix_ceiling_kernel<0>, (const void*)mix_ceiling_kernel<1>, (const void*)mix_ceiling_kernel<2>,
                              (const void*)pingpong_ceiling_kernel<2>, (const void*)pingpong_ceiling_kernel<1>};
    // one untimed launch first: from idle the device takes tens of milliseconds to reach the clock it sustains
    if (hipLaunchKernel(kernels[mode], dim3(blocks), dim3(512), args, 0, s) != hipSuccess ||
        hipEventRecord(e0, s) != hipSuccess ||
        hipLaunchKernel(kernels[mode], dim3(blocks), dim3(512), args, 0, s) != hipSuccess ||
        hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(h, counters, sizeof h, hipMemcpyDeviceToHost) != hipSuccess)
        rc = ATTN_ELAUNCH;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != ATTN_OK) return rc;
    *tflops = (double)blocks * 8 * (double)iters * (mode >= 3 ? 32 : 16) * 32768.0 / ((double)ms * 1e-3) / 1e12;
    *core_ghz = h[1] ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;
    return ATTN_OK;
}

int attn_valu_ceiling(int waves_per_simd, int iters, void* stream, unsigned long long* counters,
                      double* elements_per_s, double* core_ghz) {
    if (waves_per_simd < 1 || waves_per_simd > 4 || iters < 1 || !counters || !elements_per_s || !core_ghz) return ATTN_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    const int blocks = waves_per_simd * cu_count();  // 256 threads: one wave on each SIMD of a CU
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return ATTN_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) { hipEventDestroy(e0); return ATTN_ELAUNCH; }
    int rc = ATTN_OK;
    float ms = 0.f, scale = 0.127517f, shift = -0.25f;
    unsigned long long h[2] = {0, 0};
    void* args[] = {&counters, &iters, &scale, &shift};
    if (hipEventRecord(e0, s) != hipSuccess ||
        hipLaunchKernel((const void*)valu_ceiling_kernel, dim3(blocks), dim3(256), args, 0, s) != hipSuccess ||
        hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(h, counters, sizeof h, hipMemcpyDeviceToHost) != hipSuccess)
        rc = ATTN_ELAUNCH;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (rc != ATTN_OK) return rc;
    *elements_per_s = (double)blocks * 256.0 * (double)iters * 16.0 / ((double)ms * 1e-3);
    *core_ghz = h[1] ? (double)h[0] / ((double)h[1] * 10.0) : 0.0;
    return ATTN_OK;
}

const char* attn_strerror(int code) {
    switch (code) {
        case ATTN_OK: return "ok";
        case ATTN_EINVAL: return "invalid argument";
        case ATTN_EUNSUPPORTED: return "unsupported shape or variant";
        case ATTN_ELAUNCH: return "HIP launch or event call failed";
        default: return "unknown error code";
    }
}

}  // extern "C"
