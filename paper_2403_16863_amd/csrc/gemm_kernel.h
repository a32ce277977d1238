// Fused GEMM + LeakyReLU for gfx950 (MI355X): C = leaky_relu(A B), 16-bit inputs, fp32
// accumulation on 32x32x16 MFMA, one rounding into the 16-bit output.
//
// The operation is the second kernel the paper tunes (Sec. 5, Table 3: M, N, K = 512, 512,
// 2048, binary16).  At that size the whole problem is 1 GFLOP over 4.5 MB: the time goes
// into memory latency, not arithmetic, and the design below is built around that; it is not
// the paper's (a Triton tutorial kernel for another machine).
//
//  * One workgroup per 32 x 32 tile of C: 256 tiles for the paper's shape, one per compute
//    unit.  Larger tiles would reuse operands better but leave most of the chip idle.
//  * The WK waves of a workgroup split K between them (wave w takes the k ranges
//    [(t*WK + w) * BKW, +BKW), t = 0, 1, ...) and each runs a pipeline of its own: a ring of S
//    stages in LDS that only this wave writes (direct global -> LDS loads) and reads, so the
//    main loop has no barrier at all, only counted waits (s_waitcnt vmcnt) on the wave's own
//    loads.  With S - 1 stages of every wave in flight a compute unit keeps about 100 KB of
//    loads outstanding, which is what it takes to cover the memory latency at full rate.
//  * Transposed product, as in the attention kernel: C^T += B^T A^T.  The A operand of the MFMA
//    (32 rows n, 8 consecutive k per lane) comes from the row-major B piece through the
//    transposing LDS read; the B operand (32 columns m, 8 consecutive k per lane) is a plain
//    16-byte read of a row of the A piece.  A lane of the accumulator then holds, for one row
//    m of C, runs of four consecutive n.
//  * The partial sums of the WK waves meet in LDS once, after the loop; every wave then
//    finishes 16 / WK of the accumulator registers: sum in wave order, activation in fp32,
//    rounding, store.
//  * Workgroups are placed round-robin on the 8 XCDs, each with its own L2: tile_of_block gives
//    every XCD a compact block of tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_kernel.h"

namespace gemm {

using attn::f32x16;
using attn::lds_address;
using attn::lds_s16x4_ptr;
using attn::load_to_lds_16;
using attn::u32x2;
using attn::u32x4;

struct Params {
    const char* a;
    const char* b;
    uint16_t* c;
    int M, N, K;
    int ntm, ntn;  // tiles of 32 rows / 32 columns
    float slope;
};

// Tile of workgroup b.  XCD x = b % 8 owns the tiles  [x*per + min(x, rem), ...)  of a linear
// order (per = nblocks / 8, rem = nblocks % 8) in which the tile columns are cut into panels of
// 8 and each panel runs row by row: 32 consecutive tiles are 4 rows x 8 columns.
__host__ __device__ inline void tile_of_block(int b, int ntm, int ntn, int& tm, int& tn) {
    const int nblocks = ntm * ntn;
    const int per = nblocks >> 3, rem = nblocks & 7, x = b & 7, i = b >> 3;
    const int L = x * per + (x < rem ? x : rem) + i;
    constexpr int GW = 8;
    const int panel = L / (ntm * GW), r = L - panel * ntm * GW;
    const int left = ntn - panel * GW, w = left < GW ? left : GW;
    tm = r / w;
    tn = panel * GW + r % w;
}

template <int WK_, int BKW_, int S_, int ROT_>
struct Knobs {
    static constexpr int WK = WK_;    // waves per workgroup, splitting K
    static constexpr int BKW = BKW_;  // k extent of one stage of one wave
    static constexpr int S = S_;      // stages in a wave's ring
    static constexpr int ROT = ROT_;  // 1: every workgroup of an XCD starts at another k (see the kernel)
};

// A piece in LDS: 32 rows of CPA 16-byte chunks, read row-wise (lane = row).  The LDS serves 16
// lanes x 16 bytes = 256 bytes per clock, i.e. 16 / CPA whole rows of bank groups: the chunk index
// is XOR-ed with (row / (16 / CPA)), so the 16 consecutive rows of one clock, all reading the
// same logical chunk, land on 16 different bank groups.  An involution: the same function maps
// both ways.
template <int CPA>
__device__ __forceinline__ int a_code(int row) {
    return CPA == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
// B piece in LDS: BKW rows (k) of 64 bytes (32 columns), read with the transposing load, which
// touches 4 consecutive rows x 32 bytes per 16 lanes, two such groups (the two halves of the
// rows) per clock: 256 contiguous bytes, conflict-free as they lie.  The halves of a row swap
// on rows 2, 3 (mod 4), which keeps that true and costs nothing.
__device__ __forceinline__ int b_code(int row) { return (row >> 1) & 1; }

template <class T, class KN>
__global__ __launch_bounds__(KN::WK * 64) void gemm_lrelu_kernel(Params p) {
    constexpr int WK = KN::WK, BKW = KN::BKW, S = KN::S, ROT = KN::ROT;
    constexpr int CPA = BKW / 8;    // chunks per row of the A piece
    constexpr int RBA = BKW * 2;    // bytes per row of the A piece
    constexpr int A_BYTES = 32 * RBA;
    constexpr int RBB = 64;         // bytes per row of the B piece
    constexpr int B_BYTES = BKW * RBB;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int LA = 32 * CPA / 64, LB = BKW * 4 / 64, LPS = LA + LB;  // loads per lane and stage
    constexpr int KPW = BKW / 16;   // MFMA steps per stage
    constexpr int RING = S * STAGE;
    static_assert(CPA == 4 || CPA == 8, "A swizzle is defined for 64- and 128-byte rows");
    static_assert(S >= 3 && (S - 2) * LPS <= 63, "the counted wait must fit s_waitcnt's field");
    static_assert(RING >= 4096, "a wave's ring also holds its 32 x 32 partial sums");
    static_assert(WK == 1 || WK == 2 || WK == 4 || WK == 8, "16 accumulator registers are dealt to WK waves");

    __shared__ __attribute__((aligned(256))) u32x4 smem[WK * RING / 16];
    char* const smem_b = reinterpret_cast<char*>(smem);

    const int lane = threadIdx.x & 63;
    const int wk = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 5, c = lane & 31;
    char* const ring = smem_b + wk * RING;

    int tm, tn;
    tile_of_block((int)blockIdx.x, p.ntm, p.ntn, tm, tn);
    const int m0 = tm * 32, n0 = tn * 32;
    const int M = p.M, N = p.N, K = p.K;

    // ---- what each lane loads.  Load i of a piece fills physical chunks i*64 .. i*64+63 of it
    // (that is where a direct load puts the 64 lanes' data); lane l fetches the logical chunk
    // that belongs there.  Rows of A past M and columns of B past N are redirected to the last
    // valid ones: they only feed rows / columns of C that are never stored.
    unsigned voffA[LA], voffB[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int pch = i * 64 + lane, row = pch / CPA, ch = (pch % CPA) ^ a_code<CPA>(row);
        const int rowc = min(m0 + row, M - 1) - m0;
        voffA[i] = (unsigned)rowc * (unsigned)(K * 2) + ch * 16;
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int pch = i * 64 + lane, row = pch >> 2, pc = pch & 3;
        const int lc = ((((pc >> 1) ^ b_code(row)) << 1) | (pc & 1));
        const int col = min(n0 + lc * 8, N - 8);
        voffB[i] = (unsigned)row * (unsigned)(N * 2) + col * 2;
    }
    const char* const pa = p.a + (size_t)m0 * K * 2;

    // this wave's k ranges: t = 0 .. nkt-1 with  k0 = (t*WK + wk) * BKW < K
    const int nkt = K > wk * BKW ? (K - wk * BKW + WK * BKW - 1) / (WK * BKW) : 0;

    // Rotation: the workgroups of one XCD share rows of A and columns of B through that XCD's L2.
    // Started together at k = 0 they all ask for the same lines at the same time, and the L2
    // has only as many distinct lines on order as ONE ring is deep.  With ROT the i-th workgroup
    // of an XCD walks its ranges from i/32 of the way through (and wraps around): a line is
    // still fetched into the L2 once, but the misses of 32 rings are in flight side by side.
    const int rot = ROT ? (int)(((blockIdx.x >> 3) & 31) * (unsigned)nkt) >> 5 : 0;

    auto issue = [&](int t, int stage) __attribute__((always_inline)) {
        t += rot;
        if (t >= nkt) t -= nkt;
        const int k0 = (t * WK + wk) * BKW;
        char* st = ring + stage * STAGE;
        const char* ab = pa + (size_t)k0 * 2;
        const char* bb = p.b + (size_t)k0 * N * 2;
        if (k0 + BKW <= K) {
#pragma unroll
            for (int i = 0; i < LA; ++i) load_to_lds_16(ab, voffA[i], lds_address(st + i * 1024));
#pragma unroll
            for (int i = 0; i < LB; ++i) load_to_lds_16(bb, voffB[i], lds_address(st + A_BYTES + i * 1024));
        } else {
            // The last, partial k range (K is a multiple of 8, so chunks are in or out as a
            // whole): through registers, with exact zeros past K on both sides.  Everything
            // issued before has landed first, so the counted waits below stay on the safe side.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const int pch = i * 64 + lane, row = pch / CPA, ch = (pch % CPA) ^ a_code<CPA>(row);
                u32x4 val = {0, 0, 0, 0};
                if (k0 + ch * 8 < K) val = *reinterpret_cast<const u32x4*>(ab + voffA[i]);
                *reinterpret_cast<u32x4*>(st + pch * 16) = val;
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const int pch = i * 64 + lane, row = pch >> 2;
                u32x4 val = {0, 0, 0, 0};
                if (k0 + row < K) val = *reinterpret_cast<const u32x4*>(bb + voffB[i]);
                *reinterpret_cast<u32x4*>(st + A_BYTES + pch * 16) = val;
            }
        }
    };

    // per-lane read offsets inside a stage
    int aoff[KPW];
#pragma unroll
    for (int j = 0; j < KPW; ++j) aoff[j] = (c * CPA + ((2 * j + g) ^ a_code<CPA>(c))) * 16;
    const int r4 = (lane & 15) >> 2;
    const int boff = A_BYTES + (8 * g + r4) * RBB + ((((lane >> 4) & 1) ^ b_code(r4)) * 32) + (lane & 3) * 8;

    f32x16 acc[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][v] = acc[1][v] = 0.f;

#pragma unroll
    for (int t = 0; t < S - 1; ++t)
        if (t < nkt) issue(t, t);

    // One iteration: stage `stage` (range number t of this wave) has landed; read its fragments,
    // refill the stage read one iteration ago, multiply.
    int stage = 0;  // t % S
    auto read_stage = [&](u32x4(&af)[KPW], u32x4(&bf)[KPW]) __attribute__((always_inline)) {
        const char* st = ring + stage * STAGE;
#pragma unroll
        for (int j = 0; j < KPW; ++j) {
            af[j] = *reinterpret_cast<const u32x4*>(st + aoff[j]);
            const char* bp = st + boff + j * 16 * RBB;
            const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp)));
            const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(bp + 4 * RBB)));
            bf[j] = u32x4{lo[0], lo[1], hi[0], hi[1]};
        }
        // The stage read one iteration ago is refilled next; its reads (and the ones above) have
        // returned once the LDS counter is zero.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    };
    auto multiply = [&](const u32x4(&af)[KPW], const u32x4(&bf)[KPW]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < KPW; ++j) acc[j & 1] = T::mfma(bf[j], af[j], acc[j & 1]);
        stage = stage == S - 1 ? 0 : stage + 1;
    };

    // Steady state, straight-line code: every range touched is a whole one (only this wave's
    // last range can cross K), so the wait is the counted one and the refill the direct one.
    // Loads return in order: once at most (S-2)*LPS are outstanding, stage t has landed.
    int t = 0;
    if constexpr (ROT == 0) {
        const int nwhole = (nkt > 0 && ((nkt - 1) * WK + wk) * BKW + BKW > K) ? nkt - 1 : nkt;
        const char* ab = pa + (size_t)((S - 1) * WK + wk) * BKW * 2;           // range t + S - 1
        const char* bb = p.b + (size_t)((S - 1) * WK + wk) * BKW * N * 2;
        const size_t bstep = (size_t)WK * BKW * N * 2;
        for (; t + S - 1 < nwhole; ++t) {
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LPS) : "memory");
            u32x4 af[KPW], bf[KPW];
            read_stage(af, bf);
            char* st = ring + (stage == 0 ? S - 1 : stage - 1) * STAGE;
#pragma unroll
            for (int i = 0; i < LA; ++i) load_to_lds_16(ab, voffA[i], lds_address(st + i * 1024));
#pragma unroll
            for (int i = 0; i < LB; ++i) load_to_lds_16(bb, voffB[i], lds_address(st + A_BYTES + i * 1024));
            ab += WK * BKW * 2;
            bb += bstep;
            multiply(af, bf);
        }
    }
    // The rest (all of it with a rotated start): the same steps with the decisions taken per range.
    for (; t < nkt; ++t) {
        // Near the end fewer stages follow; waiting for everything is then right and cheap.
        if (t + S - 2 < nkt) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((S - 2) * LPS) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        u32x4 af[KPW], bf[KPW];
        read_stage(af, bf);
        if (t + S - 1 < nkt) issue(t + S - 1, stage == 0 ? S - 1 : stage - 1);
        multiply(af, bf);
    }

    f32x16 sum;
#pragma unroll
    for (int v = 0; v < 16; ++v) sum[v] = acc[0][v] + acc[1][v];

    // ---- the waves' partial sums meet in LDS (each wave's ring is idle by now: its last wait
    // was for all of its loads); wave wk finishes registers wk*RPW .. +RPW-1.
    constexpr int RPW = 16 / WK;
    float r[RPW];
    if constexpr (WK > 1) {
        float* mine = reinterpret_cast<float*>(ring);
#pragma unroll
        for (int v = 0; v < 16; ++v) mine[v * 64 + lane] = sum[v];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < RPW; ++q) {
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < WK; ++w) tot += reinterpret_cast<const float*>(smem_b + w * RING)[(wk * RPW + q) * 64 + lane];
            r[q] = tot;
        }
    } else {
#pragma unroll
        for (int q = 0; q < RPW; ++q) r[q] = sum[q];
    }

    // C^T accumulator layout: lane = column m (c), register v = row n = 8*(v/4) + 4*g + v%4.
    const int m = m0 + c;
    const float slope = p.slope;
#pragma unroll
    for (int q = 0; q < RPW; q += 2) {
        const int v = wk * RPW + q;
        const int n = n0 + 8 * (v >> 2) + 4 * g + (v & 3);
        const float x0 = r[q] >= 0.f ? r[q] : slope * r[q];
        const float x1 = r[q + 1] >= 0.f ? r[q + 1] : slope * r[q + 1];
        if (m < M && n < N) *reinterpret_cast<unsigned*>(p.c + (size_t)m * N + n) = T::pack2(x0, x1);
    }
}

}  // namespace gemm
