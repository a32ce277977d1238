// Fused attention forward for gfx950 (MI355X): one pass over K/V tiles with an
// online softmax, both contractions on 32x32x16 MFMA, fp32 accumulation.
//
// The operation is the kernel the paper tunes (fused attention forward, Sec. 1
// and Sec. 5 "Experiment setup", tensors [batch, heads, seq, head_dim], Table 2
// caption).  The tiling below is designed for CDNA4 and is not the paper's.
//
// Formulation ("transposed"): a wave owns QB blocks of 32 query rows and computes
//     S^T = K_tile . Q^T        (A operand = K rows from LDS, B operand = Q, kept in registers)
//     O^T += V_tile^T . P^T     (A operand = V read from LDS with the transposing
//                                ds_read_b64_tr_b16, B operand = P straight from
//                                the S^T accumulator registers)
// In the 32x32 accumulator layout every lane then holds 16 scores of ONE query
// (column = lane % 32), so the softmax row statistics are lane-local except for
// one exchange between lane l and lane l^32 per tile, and the S^T accumulators
// are, after conversion to 16 bit, already laid out as the B operand of the
// second contraction (with the key order permuted identically on the V side).
//
// 32x32x16 MFMA register layout (checked on hardware):
//   A (32 x 16): lane l holds row l%32, k = 8*(l/32) .. +7
//   B (16 x 32): lane l holds col l%32, k = 8*(l/32) .. +7
//   C (32 x 32): lane l holds col l%32, register v holds row 8*(v/4) + 4*(l/32) + v%4
// ds_read_b64_tr_b16 (checked on hardware): within each group of 16 lanes the 16 x 4
// elements addressed by the lanes are taken as a row-major 4 x 16 block and lane i
// receives column i, i.e. four consecutive rows of one column.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace attn {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;
typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

struct Params {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* out;
    float* lse;
    int H, N;
    int nqt;          // query tiles per head
    int BH;           // B * H
    float scale;      // multiplies q'.k, always > 0 (see qmode)
    float scale_l2;   // scale * log2(e)
    int qmode;        // 0: q' = q;  1: q' = -q (caller's scale was negative);
                      // 2: q' = 0 (caller's scale was zero, kernel runs with scale 1)
};

struct F16 {
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float a, float b) {  // nearest-even
        return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{a, b}, f16x2));
    }
};
struct BF16 {
    static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ unsigned pack2(float a, float b) {  // nearest-even
        return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{a, b}, bf16x2));
    }
};

// Exchange between lane l and lane l^32 with v_permlane32_swap_b32, which swaps the
// upper 32 lanes of its first operand with the lower 32 lanes of its second.  Starting
// from two copies of x, the first then holds the lower half's values in both halves
// and the second the upper half's.  Written as inline asm with two read-write
// operands: the compiler folds the builtin away when both inputs are the same value.
__device__ __forceinline__ void swap_halves(float x, float& lo_vals, float& hi_vals) {
    float a = x, b = x;
    // the s_nop covers the VALU-write -> permlane-read hazard the compiler cannot see
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    lo_vals = a;
    hi_vals = b;
}
// Direct global -> LDS load of 16 bytes per lane: lane l reads  base + voff  and the
// data lands at LDS address  lds_base + 16*l.  base and lds_base are wave-uniform and
// travel in scalar registers, the per-lane part is one 32-bit VGPR that the caller
// keeps for the whole kernel.  Written out by hand so that consecutive loads share no
// address VGPR: with a freshly computed 64-bit VGPR address per load, the VALU write of
// the next address has to wait until the previous load has left the issue queue.
__device__ __forceinline__ void load_to_lds_16(const char* base, unsigned voff, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
    return (unsigned)(unsigned long)(const __attribute__((address_space(3))) char*)p;
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}
__device__ __forceinline__ float xhalf_sum(float x) {
    float a, b;
    swap_halves(x, a, b);
    return a + b;
}
__device__ __forceinline__ float xhalf_max(float x) {
    float a, b;
    swap_halves(x, a, b);
    return fmaxf(a, b);
}

// ---- LDS layouts ------------------------------------------------------------
// A K/V tile is BN rows of D 16-bit elements, addressed in 16-byte chunks.  Both
// swizzles below are involutions that keep a chunk inside its 256-byte line (K) or
// its row (V), so the same function maps logical -> physical and physical -> logical.
//
// K is read row-wise (ds_read_b128, lane = key row): the chunk index is XOR-ed with
// the 256-byte line index so 16 consecutive rows land on 16 distinct bank groups.
__device__ __forceinline__ int k_swz(int chunk) { return (chunk & ~15) | ((chunk ^ (chunk >> 4)) & 15); }
// V is read with the transposing load: a 16-lane group touches 4 consecutive key
// rows x 32 bytes, and the LDS serves two such groups (the two 16-column halves of a
// 32-column block: two neighbouring 32-byte slots) per clock, 256 bytes wide.  32-byte
// slots are XOR-ed with a code of (row & 3) chosen so that those 4 rows x 2 slots hit eight
// different 32-byte bank groups: with 256-byte rows (d = 128) every row covers all groups and
// the codes 0, 2, 5, 7 do it; with 128-byte rows (d = 64) rows r and r + 2 share their groups
// and the codes 0, 0, 2, 2 do.
template <int D>
__device__ __forceinline__ int v_swz_slot(int row, int slot) {
    const int r = row & 3;
    const int code = D == 128 ? (((r << 1) & 6) | (r >> 1)) : (r & 2);
    return slot ^ code;
}

// ---- work items and their schedule.  A work item is one query tile of one head; the grid
// holds G persistent workgroups (as many as the device keeps resident), and workgroup gidx
// takes, in round 0, 1, 2 ..., the item this function names, until it returns false.
// Items in head-major order, inside a head from the last query tile (the heaviest under a
// causal mask) to the first, are dealt to the workgroups in serpentine order (0..G-1,
// G-1..0, ...): a workgroup's items of two consecutive rounds then sit at mirrored
// positions of the weight sawtooth, so the sums come out even, and at any time the
// workgroups of a round work on few heads, whose K and V stay in L2.  Workgroups are placed
// round-robin on the 8 XCDs, each with its own L2: when G and the number of heads BH are
// multiples of 8, the deal runs inside each XCD over that XCD's heads (x, x+8, ...), so all
// query tiles of a head share one L2.  Every item is named exactly once over all (gidx, round).
__host__ __device__ inline bool schedule_item(int G, int gidx, int BH, int nqt, int round, int& bh, int& qt) {
    int r, nh, h0, hs;
    if ((G & 7) == 0 && (BH & 7) == 0) {
        const int C = G >> 3, cidx = gidx >> 3;
        r = round * C + ((round & 1) ? C - 1 - cidx : cidx);
        nh = BH >> 3, h0 = gidx & 7, hs = 8;
    } else {
        r = round * G + ((round & 1) ? G - 1 - gidx : gidx);
        nh = BH, h0 = 0, hs = 1;
    }
    if (r >= nh * nqt) return false;
    qt = nqt - 1 - r % nqt;
    bh = h0 + hs * (r / nqt);
    return true;
}

// Schedule / shape knobs of one variant (the lattice the search walks).
template <int BN_, int NW_, int QB_, int OCC_, int LDP_, int PIPE_, int PF_, int PRIO_, int ILV_ = 0, int LDPOS_ = 0>
struct Knobs {
    static constexpr int BN = BN_;      // keys per K/V tile
    static constexpr int NW = NW_;      // waves per workgroup
    static constexpr int QB = QB_;      // 32-row query blocks per wave
    static constexpr int OCC = OCC_;    // workgroups per CU the register budget aims for
    static constexpr int LDP = LDP_;    // K/V load path: 0 = through VGPRs, 1 = global -> LDS directly
    static constexpr int PIPE = PIPE_;  // 0 = per tile S, softmax, PV, waves run free;
                                        // 1 = two-cluster ping-pong between the two waves of a SIMD (MFMA | VALU),
                                        // 2 = ping-pong with MFMA work in both clusters, softmax inside the PV MFMAs,
                                        // 3 = one interleaved stream of MFMAs and softmax arithmetic per wave
    static constexpr int PF = PF_;      // LDS fragment prefetch distance of the MFMA streams, in MFMA steps
    static constexpr int PRIO = PRIO_;  // where the wave priority is raised (s_setprio): 0 = nowhere, 1 = while the wave runs an
                                        // MFMA stream, 2 = while it issues tile loads (PIPE 1) / in the second wave of every SIMD (PIPE 3)
    static constexpr int ILV = ILV_;    // PIPE 3: how MFMA, LDS-read and softmax instructions are grouped (see there)
    static constexpr int LDPOS = LDPOS_;  // PIPE 3: where a wave issues its four tile loads of an iteration: 0 = all after the
                                          // barrier, 1 = after MFMA slots 3, 11, 19, 27, 2 = after slots that depend on the wave
};

template <class T, int D, bool CAUSAL, class KN>
__global__ __launch_bounds__(KN::NW * 64, KN::OCC) void attn_fwd_kernel(const Params p) {
    constexpr int BN = KN::BN, NW = KN::NW, QB = KN::QB, LDP = KN::LDP, PIPE = KN::PIPE, PF = KN::PF, PRIO = KN::PRIO;
    constexpr int ILV = KN::ILV, LDPOS = KN::LDPOS;
    // Ping-pong order with LDPOS 1: three K and three V buffers, tile loads one tile further ahead,
    // ONE workgroup barrier per tile (see there).  Layout then K0 K1 K2 V0 V1 V2, so that the
    // immediate offsets of the K reads and of the V reads each stay inside their 64 KB.
    constexpr bool NB3 = PIPE == 1 && LDPOS == 1;
    constexpr int NB = NB3 ? 3 : 2;  // K buffers and V buffers in LDS
    constexpr int NT = NW * 64;
    constexpr int BM = 32 * QB * NW;
    constexpr int KS = D / 16;       // k-steps of the first contraction
    constexpr int DT = D / 32;       // 32-wide d tiles of O^T
    constexpr int KT = BN / 32;      // 32-key sub-tiles of one K/V tile
    constexpr int CPR = D / 8;       // 16-byte chunks per row
    constexpr int RB = D * 2;        // bytes per row
    constexpr int TILE_CHUNKS = BN * CPR;
    constexpr int LD_PER_THREAD = TILE_CHUNKS / NT;
    static_assert(TILE_CHUNKS % NT == 0, "tile must divide over the workgroup");
    constexpr int TILE_BYTES = TILE_CHUNKS * 16;
    constexpr int NVF = KT * 2 * DT;  // V fragments (MFMA steps of the second contraction) per tile
    constexpr int NKF = KS * KT;      // K fragments (MFMA steps of the first contraction) per tile

    // The ping-pong order with tiles straight to LDS also brings Q in through LDS: the B-operand
    // layout wants 32 bytes of each of 32 rows per load instruction, which the texture path
    // takes as 32 separate requests (a workgroup's 64 KB of Q then cost more than all its first
    // tiles together); whole rows, 1 KB per wave instruction, land in a staging area laid out
    // like a K tile of BM rows, and each wave reads its fragments from there.
    // (Also for the free-running order at d = 64, where the staging area fits next to the tiles
    // of three workgroups per compute unit; at d = 128 two such workgroups would need 192 KB.)
    constexpr bool QSTAGE = LDP == 1 && QB == 1 && (PIPE == 1 || (PIPE == 0 && D == 64));
    __shared__ __attribute__((aligned(256))) u32x4 smem[2 * NB * TILE_CHUNKS + (QSTAGE ? BM * CPR : 0)];  // K0 V0 K1 V1 (three buffers: K0 K1 K2 V0 V1 V2), then the Q staging area
    char* const smem_b = reinterpret_cast<char*>(smem);

    auto k_off = [](int b) { return NB3 ? b * TILE_BYTES : b * 2 * TILE_BYTES; };                       // K buffer b, bytes from the start of LDS
    auto v_off = [](int b) { return NB3 ? (NB + b) * TILE_BYTES : b * 2 * TILE_BYTES + TILE_BYTES; };  // V buffer b
    auto v_rel = [](int b) { return NB3 ? b * TILE_BYTES : b * 2 * TILE_BYTES + TILE_BYTES; };         // the same, from where voff[] counts

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 5;
    const int c = lane & 31;

    auto item_of_round = [&](int round, int& bh, int& qt) __attribute__((always_inline)) -> bool {
        return schedule_item((int)gridDim.x, (int)blockIdx.x, p.BH, p.nqt, round, bh, qt);
    };
    const int N = p.N;
    // binary16 only: a finite result above the largest finite binary16 value is stored as that
    // value, not as infinity (mode bit FP16_OVFL; true infinities and NaN pass unchanged).  The
    // exact O is a convex combination of V values, so it never exceeds max |V|; the computed one
    // can, by a rounding error: P is rounded to 16 bits before the second contraction while the
    // row sum keeps the unrounded values, and with V at the largest finite value a few
    // probabilities rounded upwards put O half a unit in the last place above it.
    if constexpr (std::is_same_v<T, F16>) asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 23, 1), 1");
    for (int round = 0;; ++round) {
        int bh, qt;
        if (!item_of_round(round, bh, qt)) break;
        if (round > 0) __syncthreads();  // every wave is done with the previous item's tiles in LDS
        const int q0 = qt * BM;
        // Row block of this wave inside the query tile.  Waves w and w + NW/2 share a SIMD; under a
        // causal mask the interleaved order (PIPE 3) gives them the blocks s and NW-1-s, so every SIMD
        // gets the same number of visible keys on the diagonal tiles.
        const int rblk = (PIPE == 3 && CAUSAL) ? (wave < NW / 2 ? wave : NW + NW / 2 - 1 - wave) : wave;
        const int qw0 = q0 + rblk * (32 * QB);  // first query row of this wave
        const int qw_last = qw0 + 32 * QB - 1;  // causal: tile j is active for this wave iff j*BN <= qw_last

        const size_t head_off = (size_t)bh * N * D;
        const uint16_t* __restrict__ Qh = p.q + head_off;
        const char* __restrict__ Kh = reinterpret_cast<const char*>(p.k + head_off);
        const char* __restrict__ Vh = reinterpret_cast<const char*>(p.v + head_off);

        // ---- Q as B operand, resident in registers.  Loaded after the first K/V tiles have
        // been issued, so that the wait for Q (which every item reads exactly once, from
        // HBM) does not delay them.
        u32x4 qreg[QB][KS];
        auto load_q = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const int row = qw0 + qb * 32 + c;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    u32x4 val = {0, 0, 0, 0};
                    if (row < N && p.qmode != 2)
                        val = *reinterpret_cast<const u32x4*>(Qh + (size_t)row * D + ks * 16 + g * 8);
                    if (p.qmode == 1) val ^= 0x80008000u;  // flip the sign of all eight elements
                    qreg[qb][ks] = val;
                }
            }
        };

        f32x16 o[QB][DT];
        float m_use[QB], l_run[QB];  // reference maximum in use (raw units), partial row sum
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            m_use[qb] = -INFINITY;
            l_run[qb] = 0.f;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[qb][dt][v] = 0.f;
        }

        // key tiles this workgroup visits
        const int kend = CAUSAL ? min(N, q0 + BM) : N;  // keys [0, kend)
        const int nkt = (kend + BN - 1) / BN;
        auto tile_active = [&](int j) __attribute__((always_inline)) { return j < nkt && (!CAUSAL || j * BN <= qw_last); };

        // ---- per-lane LDS read offsets (bytes inside one K or V tile), loop invariant.
        // K: lane reads row (kt*32 + c), logical chunk (2*ks + g); moving kt by one adds
        // 32 rows, which leaves the swizzle term unchanged, so kt is an immediate offset.
        int koff[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) koff[ks] = k_swz(c * CPR + 2 * ks + g) * 16;
        // V: lane (16-lane group gq = lane/16, i = lane%16) addresses row 4*g + i/4 (+ 16*t + 8*hi
        // + 32*kt, all multiples of 4, again immediates) and d column dt*32 + (gq&1)*16 + 4*(i%4).
        int voff[DT];
        {
            const int i16 = lane & 15;
            const int row = 4 * g + (i16 >> 2);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const int dcol = dt * 32 + ((lane >> 4) & 1) * 16 + 4 * (i16 & 3);
                voff[dt] = row * RB + v_swz_slot<D>(row, dcol >> 4) * 32 + (dcol & 15) * 2;
            }
            if constexpr (NB3) {  // the V buffers start NB tiles into LDS; opaque, or the compiler folds it into the immediates
                int shift = NB * TILE_BYTES;
                asm volatile("" : "+v"(shift));
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) voff[dt] += shift;
            }
        }

        // All helper lambdas below are force-inlined: they capture the register arrays (o, s,
        // pk, qreg ...) by reference, and a call that is not inlined would push those arrays
        // out of registers into scratch memory.

        // ---- K/V tile movement.  A tile is moved by LNT loader threads (the whole workgroup,
        // or one wave group of it): loader thread t moves chunks  i*LNT + t  (i < TILE_CHUNKS /
        // LNT) of the physical LDS tile.  LNT is a multiple of 256, so piece i advances by a
        // whole number of swizzle periods and the matching logical chunk in the row-major
        // global tile is   goff0 + i * (LNT / CPR) * RB   (goff0 per lane, the rest compile-time).
        auto goff_k = [&](int lt) __attribute__((always_inline)) {
            const int Lk = k_swz(lt);
            return (unsigned)((Lk / CPR) * RB + (Lk % CPR) * 16);
        };
        auto goff_v = [&](int lt) __attribute__((always_inline)) {
            const int rowv = lt / CPR, pc = lt % CPR;
            return (unsigned)(rowv * RB + ((v_swz_slot<D>(rowv, pc >> 1) << 1) | (pc & 1)) * 16);
        };
        const unsigned goffK0 = goff_k(tid), goffV0 = goff_v(tid);
        u32x4 kst[LDP == 0 ? LD_PER_THREAD : 1], vst[LDP == 0 ? LD_PER_THREAD : 1];

        // Piece i of the tile that starts at key row kt0: the source is a wave-uniform base
        // (tile start + i * LNT / CPR rows) plus the per-lane 32-bit offset.  `whole` says that
        // the tile lies inside the sequence; otherwise rows past the end are redirected to the
        // last row (their scores are masked, so only finiteness of what is loaded matters).
        auto issue_piece = [&](auto lnt_c, bool whole, const char* head, unsigned goff0, int lwave, int kt0, char* lds_tile,
                               int i, u32x4& stage) __attribute__((always_inline)) {
            constexpr int LNT = decltype(lnt_c)::value;
            static_assert(LNT % 256 == 0 && TILE_CHUNKS % LNT == 0, "load mapping assumes whole swizzle periods per piece");
            constexpr int ROWS_PER_PIECE = LNT / CPR;
            char* dst = lds_tile + (i * LNT + lwave * 64) * 16;
            if (whole) {
                const char* pb = head + (size_t)kt0 * RB + (size_t)(i * ROWS_PER_PIECE * RB);
                if constexpr (LDP == 1)
                    load_to_lds_16(pb, goff0, lds_address(dst));
                else
                    stage = *reinterpret_cast<const u32x4*>(pb + goff0);
            } else {
                const int r = min(kt0 + (int)(goff0 / RB) + i * ROWS_PER_PIECE, N - 1);
                const char* src = head + (size_t)r * RB + goff0 % RB;
                if constexpr (LDP == 1)
                    __builtin_amdgcn_global_load_lds((global_void_ptr)src, (lds_void_ptr)dst, 16, 0, 0);
                else
                    stage = *reinterpret_cast<const u32x4*>(src);
            }
        };
        // K tile jk into K buffer kbuf and / or V tile jv into V buffer vbuf (a negative index
        // skips that tile).  Tile indices are clamped to the last tile (a redundant reload into
        // a buffer nobody reads any more is cheaper than a branch in every iteration).  One
        // decision covers all pieces: the common case is straight-line code, a few scalar
        // operations and the loads, which also leaves their placement open to scheduling.
        auto issue_tiles = [&](int jk, int kbuf, int jv, int vbuf) __attribute__((always_inline)) {
            constexpr std::integral_constant<int, NT> nt_c{};
            const int ktk = min(jk, nkt - 1) * BN, ktv = min(jv, nkt - 1) * BN;
            const bool whole = max(ktk, ktv) + BN <= N;
            auto pieces = [&](auto whole_c) __attribute__((always_inline)) {
                constexpr bool W = decltype(whole_c)::value;
                if (jk >= 0) {
#pragma unroll
                    for (int i = 0; i < LD_PER_THREAD; ++i)
                        issue_piece(nt_c, W, Kh, goffK0, wave, ktk, smem_b + k_off(kbuf), i, kst[LDP == 0 ? i : 0]);
                }
                if (jv >= 0) {
#pragma unroll
                    for (int i = 0; i < LD_PER_THREAD; ++i)
                        issue_piece(nt_c, W, Vh, goffV0, wave, ktv, smem_b + v_off(vbuf), i, vst[LDP == 0 ? i : 0]);
                }
            };
            if (whole) pieces(std::true_type{});
            else pieces(std::false_type{});
        };
        // Q through LDS (QSTAGE): the BM rows of the query tile move like a K tile of BM rows
        // (piece i = rows i * NT / CPR onward, rows past the end of the sequence redirected to the
        // last row: those queries are never stored), and wave w finds row c, chunk 2 ks + g of its
        // 32 rows at the K read offset of the same (c, ks, g), 32 w rows further on.
        auto request_q = [&]() __attribute__((always_inline)) {
            constexpr std::integral_constant<int, NT> nt_c{};
            const bool whole = q0 + BM <= N;
            u32x4 unused;
            auto pieces = [&](auto whole_c) __attribute__((always_inline)) {
#pragma unroll
                for (int i = 0; i < BM * CPR / NT; ++i)
                    issue_piece(nt_c, decltype(whole_c)::value, reinterpret_cast<const char*>(Qh), goffK0, wave, q0,
                                smem_b + 2 * NB * TILE_BYTES, i, unused);
            };
            if (whole) pieces(std::true_type{});
            else pieces(std::false_type{});
        };
        auto read_q = [&]() __attribute__((always_inline)) {
            static_assert(QB == 1 || !QSTAGE, "one 32-row block per wave");
            // (the offset is made opaque here: otherwise the compiler forms the eight addresses
            // once, ahead of the item loop, and spills them)
            int mine = 2 * NB * TILE_BYTES + wave * (32 * RB);
            asm volatile("" : "+s"(mine));
            const unsigned flip = p.qmode == 1 ? 0x80008000u : 0u, keep = p.qmode == 2 ? 0u : 0xffffffffu;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const u32x4 val = *reinterpret_cast<const u32x4*>(smem_b + mine + koff[ks]);
                qreg[0][ks] = (val ^ flip) & keep;  // q' = -q flips the sign of all eight elements, q' = 0 clears them
            }
        };
        auto issue_k = [&](int j, int buf) __attribute__((always_inline)) { issue_tiles(j, buf, -1, 0); };
        auto issue_v = [&](int j, int buf) __attribute__((always_inline)) { issue_tiles(-1, 0, j, buf); };
        // make the tiles issued last visible in LDS to this thread (K into buffer kbuf, V into vbuf)
        auto land_loads = [&](int kbuf, int vbuf) __attribute__((always_inline)) {
            if constexpr (LDP == 1) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            } else {
                char* kb = smem_b + k_off(kbuf);
                char* vb = smem_b + v_off(vbuf);
#pragma unroll
                for (int i = 0; i < LD_PER_THREAD; ++i) {
                    *reinterpret_cast<u32x4*>(kb + (i * NT + tid) * 16) = kst[i];
                    *reinterpret_cast<u32x4*>(vb + (i * NT + tid) * 16) = vst[i];
                }
            }
        };

        // ---- MFMA work as a software-pipelined stream: NVF steps of O^T += V^T P^T (each needs
        // one V fragment = two transposing reads; k-slot s of step (kt, t) for lane group g is
        // key kt*32 + 16*t + 8*(s/4) + 4*g + s%4) and/or NKF steps of S^T = K Q^T (one 16-byte K
        // fragment each, alternating between the KT independent accumulators).  Fragments are
        // read PF steps ahead into a ring of registers, in source order pinned by scheduling
        // fences, so an MFMA never waits for an LDS read issued just before it.  Buffer indices
        // are compile-time constants so every LDS offset folds into the instruction.
        auto mfma_stream = [&](auto has_pv_c, auto has_qk_c, auto vbuf_c, auto kbuf_c,
                               const u32x4(&pk)[QB][KT][2], f32x16(&s)[QB][KT]) __attribute__((always_inline)) {
            constexpr bool HAS_PV = decltype(has_pv_c)::value, HAS_QK = decltype(has_qk_c)::value;
            constexpr int VB = decltype(vbuf_c)::value, KB = decltype(kbuf_c)::value;
            constexpr int N0 = HAS_PV ? NVF : 0, NS = N0 + (HAS_QK ? NKF : 0);
            const char* vb = smem_b + v_rel(VB);
            const char* kb = smem_b + k_off(KB);
            auto read_frag = [&](int i) __attribute__((always_inline)) -> u32x4 {
                if (i < N0) {  // V fragment i = (kt*2 + t)*DT + dt
                    const int dt = i % DT, t = (i / DT) & 1, kt = i / (2 * DT);
                    const char* base = vb + (kt * 32 + 16 * t) * RB + voff[dt];
                    const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base)));
                    const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + 8 * RB)));
                    return u32x4{lo[0], lo[1], hi[0], hi[1]};
                } else {       // K fragment f = ks*KT + kt
                    const int f = i - N0;
                    return *reinterpret_cast<const u32x4*>(kb + (f % KT) * 32 * RB + koff[f / KT]);
                }
            };
            if constexpr (HAS_QK) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) s[qb][kt][v] = 0.f;
            }
            if constexpr (PRIO == 1) __builtin_amdgcn_s_setprio(2);
            constexpr int NPRE = PF < NS ? PF : NS;
            u32x4 ring[PF];
#pragma unroll
            for (int i = 0; i < NPRE; ++i) ring[i] = read_frag(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                if (i < N0) {
                    const int dt = i % DT, t = (i / DT) & 1, kt = i / (2 * DT);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) o[qb][dt] = T::mfma(ring[i % PF], pk[qb][kt][t], o[qb][dt]);
                } else {
                    const int f = i - N0, ks = f / KT, kt = f % KT;
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) s[qb][kt] = T::mfma(ring[i % PF], qreg[qb][ks], s[qb][kt]);
                }
                if (i + PF < NS) ring[i % PF] = read_frag(i + PF);
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (PRIO == 1) __builtin_amdgcn_s_setprio(0);
        };

        // ---- softmax of one tile (per query = per lane column): S -> P^T packed as B operand.
        //
        // P = exp2(scale_l2 * (S - m_use)) with a reference maximum m_use that is NOT updated on
        // every tile: the probabilities are first formed against the current reference, and
        // only if a lane's partial row sum leaves [0, 2^8] (a score grew past the reference by a
        // lot, or this is the first tile, where m_use = -inf makes the sum inf or NaN) the wave
        // takes the slow path: raise the reference to the true running maximum, rescale l and
        // O, and form the probabilities again.  Values up to 2^8 lose nothing in fp32 sums or in
        // 16-bit P, and the final normalisation divides by the true sum, so the result is the
        // same function; the common tile needs neither a row maximum nor a rescale.
        auto mask = [&](f32x16(&s)[QB][KT], int k0) __attribute__((always_inline)) {  // keys past the end, and keys after the query
            const bool need_mask = (k0 + BN > N) || (CAUSAL && (k0 + BN - 1 > qw0));
            if (need_mask) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int qi = qw0 + qb * 32 + c;
                    const int lim = CAUSAL ? min(qi, N - 1) : N - 1;  // last visible key
                    // register v of sub-tile kt holds key k0 + kt*32 + 8*(v/4) + 4*g + v%4: compare
                    // the compile-time part with one per-lane value
                    const int rel = lim - k0 - 4 * g;
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            if (kt * 32 + 8 * (v >> 2) + (v & 3) > rel) s[qb][kt][v] = -INFINITY;
                }
            }
        };
        auto exp_pack = [&](const f32x16(&s)[QB][KT], u32x4(&pk)[QB][KT][2], float(&rs)[QB]) __attribute__((always_inline)) {
            static_for<QB>([&](auto qb_c) __attribute__((always_inline)) {
                constexpr int qb = decltype(qb_c)::value;
                const float mb = m_use[qb] * p.scale_l2;
                float rs0 = 0.f, rs1 = 0.f;  // row sum of the unrounded probabilities, fp32
                if constexpr (PIPE == 1 && ILV != 2) {
                    // The V cluster is one wave's vector instructions, back to back.  Left to the compiler
                    // their order comes out differently from one build to the next (an unrelated edit
                    // elsewhere in the kernel is enough), and the builds fall into two groups 5 to 7 % of
                    // the tile loop apart.  Pinned in the source, as a three-stage pipeline over the pairs
                    // (multiply-adds of pair i+1, exponentials of pair i, sums and conversion of pair
                    // i-1, the conversion kept next to its pair instead of sinking behind the slow-path
                    // test), every order tried lands in the fast group.  ILV 0: exponential, multiply-add,
                    // sum, conversion, exponential, multiply-add, sum; ILV 1: multiply-add, exponential,
                    // multiply-add, exponential, sum, conversion, sum; ILV 2 leaves the order to the
                    // compiler (a lattice point for the search to compare).
                    float xa = 0.f, xb = 0.f, ea = 0.f, eb = 0.f;
                    static_for<KT * 8 + 2>([&](auto i_c) __attribute__((always_inline)) {
                        constexpr int i = decltype(i_c)::value;  // step: pair i enters, pair i-1 in exp, pair i-2 leaves
                        constexpr bool IN = i < KT * 8, MID = i >= 1 && i <= KT * 8, OUT = i >= 2;
                        constexpr int kt = (IN ? i : 0) / 8, t = ((IN ? i : 0) / 4) % 2, h = (IN ? i : 0) % 4;
                        constexpr int j = OUT ? i - 2 : 0, jkt = j / 8, jt = (j / 4) % 2, jh = j % 4;
                        float na = 0.f, nb = 0.f, fa = 0.f, fb = 0.f;
                        auto exp_a = [&]() __attribute__((always_inline)) { if constexpr (MID) { fa = __builtin_amdgcn_exp2f(xa); __builtin_amdgcn_sched_barrier(0); } };
                        auto exp_b = [&]() __attribute__((always_inline)) { if constexpr (MID) { fb = __builtin_amdgcn_exp2f(xb); __builtin_amdgcn_sched_barrier(0); } };
                        auto fma_a = [&]() __attribute__((always_inline)) { if constexpr (IN) { na = __builtin_fmaf(s[qb][kt][8 * t + 2 * h], p.scale_l2, -mb); __builtin_amdgcn_sched_barrier(0); } };
                        auto fma_b = [&]() __attribute__((always_inline)) { if constexpr (IN) { nb = __builtin_fmaf(s[qb][kt][8 * t + 2 * h + 1], p.scale_l2, -mb); __builtin_amdgcn_sched_barrier(0); } };
                        auto add_a = [&]() __attribute__((always_inline)) { if constexpr (OUT) { rs0 += ea; __builtin_amdgcn_sched_barrier(0); } };
                        auto add_b = [&]() __attribute__((always_inline)) { if constexpr (OUT) { rs1 += eb; __builtin_amdgcn_sched_barrier(0); } };
                        auto cvt = [&]() __attribute__((always_inline)) {
                            if constexpr (OUT) {
                                unsigned packed = T::pack2(ea, eb);
                                asm volatile("" : "+v"(packed));
                                pk[qb][jkt][jt][jh] = packed;
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        };
                        if constexpr (ILV == 0) { exp_a(); fma_a(); add_a(); cvt(); exp_b(); fma_b(); add_b(); }
                        else { fma_a(); exp_a(); fma_b(); exp_b(); add_a(); cvt(); add_b(); }
                        xa = na; xb = nb; ea = fa; eb = fb;
                    });
                    rs[qb] = rs0 + rs1;
                    return;
                }
                static_for<KT * 2>([&](auto kk_c) __attribute__((always_inline)) {
                    constexpr int kt = decltype(kk_c)::value / 2, t = decltype(kk_c)::value % 2;
                    u32x4 w;
                    static_for<4>([&](auto h_c) __attribute__((always_inline)) {
                        constexpr int h = decltype(h_c)::value;
                        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][kt][8 * t + 2 * h], p.scale_l2, -mb));
                        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][kt][8 * t + 2 * h + 1], p.scale_l2, -mb));
                        w[h] = T::pack2(e0, e1);
                        rs0 += e0;
                        rs1 += e1;
                    });
                    pk[qb][kt][t] = w;
                });
                rs[qb] = rs0 + rs1;
            });
        };
        auto raise_reference = [&](const f32x16(&s)[QB][KT]) __attribute__((always_inline)) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = s[qb][0][0];
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[qb][kt][v]);
                const float m_new = fmaxf(m_use[qb], xhalf_max(mx));
                // m_new is finite: key 0 is visible to every query and lives in tile 0, the first
                // tile every wave processes.  There m_use = -inf and alpha = exp2(-inf) = 0.
                const float alpha = __builtin_amdgcn_exp2f((m_use[qb] - m_new) * p.scale_l2);
                m_use[qb] = m_new;
                l_run[qb] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[qb][dt][v] *= alpha;
            }
        };
        auto softmax_tile = [&](f32x16(&s)[QB][KT], u32x4(&pk)[QB][KT][2], int k0) __attribute__((always_inline)) {
            mask(s, k0);
            float rs[QB];
            exp_pack(s, pk, rs);
            bool ok = true;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) ok = ok && (rs[qb] <= 256.0f);  // false for inf and NaN too
            if (__builtin_amdgcn_ballot_w64(!ok) != 0) {                    // wave-uniform, rare
                raise_reference(s);
                exp_pack(s, pk, rs);
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) l_run[qb] += rs[qb];
        };

        // Tile 0 always takes the slow path (m_use = -inf): go there directly.
        auto softmax_first_tile = [&](f32x16(&s)[QB][KT], u32x4(&pk)[QB][KT][2]) __attribute__((always_inline)) {
            mask(s, 0);
            float rs[QB];
            raise_reference(s);
            exp_pack(s, pk, rs);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) l_run[qb] += rs[qb];
        };

        // ---- O^T += V^T P^T for tile j with the softmax of tile j+1 worked into it: after
        // each MFMA a few elements of S(j+1) go through scale, exp2, row sum and packing while
        // the MFMA is in the pipe (a wave's own VALU instructions issue behind its MFMA).
        // pk holds P(j) on entry and P(j+1) on exit: MFMA step i reads the vector pk[kt][t] with
        // (kt*2 + t) = i / DT, and the pairs formed during the DT steps that read one vector
        // make up exactly the new contents of that vector, which replace it after its last
        // read.  Same arithmetic, element by element, as softmax_tile.
        auto pv_softmax_stream = [&](auto vbuf_c, u32x4(&pk)[QB][KT][2], f32x16(&s)[QB][KT], int k0,
                                     bool next_active) __attribute__((always_inline)) {
            static_assert(QB == 1 && DT == 4, "pairing of MFMA steps and P vectors assumes one query block and d = 128");
            constexpr int VB = decltype(vbuf_c)::value;
            const char* vb = smem_b + VB * 2 * TILE_BYTES + TILE_BYTES;
            auto read_v = [&](int i) __attribute__((always_inline)) -> u32x4 {  // V fragment i = (kt*2 + t)*DT + dt
                const int dt = i % DT, t = (i / DT) & 1, kt = i / (2 * DT);
                const char* base = vb + (kt * 32 + 16 * t) * RB + voff[dt];
                const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base)));
                const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + 8 * RB)));
                return u32x4{lo[0], lo[1], hi[0], hi[1]};
            };
            mask(s, k0);
            float mb[QB], rs0[QB], rs1[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                mb[qb] = m_use[qb] * p.scale_l2;
                rs0[qb] = 0.f;
                rs1[qb] = 0.f;
            }
            if constexpr (PRIO == 1) __builtin_amdgcn_s_setprio(2);
            constexpr int NPRE = PF < NVF ? PF : NVF;
            u32x4 ring[PF];
#pragma unroll
            for (int i = 0; i < NPRE; ++i) ring[i] = read_v(i);
            __builtin_amdgcn_sched_barrier(0);
            // Two-stage software pipeline over the MFMA steps: step i forms the exponentials of
            // pair i+1 and packs / sums pair i, so the operations inside one step (which the
            // fences keep together) do not wait for each other.
            u32x4 w;
            auto exp_pair = [&](int i, float& e0, float& e1) __attribute__((always_inline)) {
                const int t = (i / DT) & 1, kt = i / (2 * DT), h = i % DT;
                e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][kt][8 * t + 2 * h], p.scale_l2, -mb[0]));
                e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][kt][8 * t + 2 * h + 1], p.scale_l2, -mb[0]));
            };
            float ea0, ea1, eb0, eb1;
            exp_pair(0, ea0, ea1);
#pragma unroll
            for (int i = 0; i < NVF; ++i) {
                const int dt = i % DT, t = (i / DT) & 1, kt = i / (2 * DT), h = i % DT;
                o[0][dt] = T::mfma(ring[i % PF], pk[0][kt][t], o[0][dt]);
                if (i + PF < NVF) ring[i % PF] = read_v(i + PF);
                if (i + 1 < NVF) exp_pair(i + 1, eb0, eb1);
                unsigned packed = T::pack2(ea0, ea1);
                // pinned here: the slow path below overwrites P, so the compiler would otherwise
                // sink the conversions into the fast path and keep every exponential alive
                asm volatile("" : "+v"(packed));
                w[h] = packed;
                rs0[0] += ea0;
                rs1[0] += ea1;
                ea0 = eb0;
                ea1 = eb1;
                if (h == DT - 1) pk[0][kt][t] = w;  // all reads of the old vector have been issued
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (PRIO == 1) __builtin_amdgcn_s_setprio(0);
            // On a wave's last active tile there is no S(j+1): the stream above still runs in
            // full (a second, PV-only code path would make the register allocator move the
            // O accumulators between the two), on stale scores whose results are dropped here.
            // The row sums are consumed unconditionally (select, not branch): otherwise the
            // compiler sinks the additions into the branch and keeps every exponential alive.
            float rs[QB];
            bool bad = false;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                rs[qb] = rs0[qb] + rs1[qb];
                bad = bad || !(rs[qb] <= 256.0f);  // true for inf and NaN too
            }
            if (__builtin_amdgcn_ballot_w64(bad && next_active) != 0) {  // wave-uniform, rare
                raise_reference(s);
                exp_pack(s, pk, rs);
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) l_run[qb] += next_active ? rs[qb] : 0.f;
        };

        constexpr std::integral_constant<int, 0> c0{};
        constexpr std::integral_constant<int, 1> c1{};
        constexpr std::true_type yes{};
        constexpr std::false_type no{};
        f32x16 s[QB][KT];
        u32x4 pk[QB][KT][2];

        if constexpr (PIPE == 0) {
            // Plain order: every tile is loaded one iteration ahead; per tile S, softmax, PV.
            // Overlap of MFMA and VALU work comes from the other waves resident on the SIMD.
            auto step = [&](auto buf_c, int j) __attribute__((always_inline)) {
                constexpr int BUF = decltype(buf_c)::value;
                issue_tiles(j + 1, BUF ^ 1, j + 1, BUF ^ 1);
                if (tile_active(j)) {
                    mfma_stream(no, yes, buf_c, buf_c, pk, s);
                    softmax_tile(s, pk, j * BN);
                    mfma_stream(yes, no, buf_c, buf_c, pk, s);
                }
                land_loads(BUF ^ 1, BUF ^ 1);
                __syncthreads();
            };
            issue_k(0, 0);
            issue_v(0, 0);
            if constexpr (QSTAGE) request_q();
            else load_q();
            land_loads(0, 0);
            __syncthreads();
            if constexpr (QSTAGE) read_q();
            for (int j = 0; j < nkt; j += 2) {
                step(c0, j);
                if (j + 1 < nkt) step(c1, j + 1);
            }
        } else if constexpr (PIPE == 3) {
            // Interleaved order: every wave runs ONE instruction stream in which the MFMAs of two
            // contractions and the softmax arithmetic of a third 32-key half tile alternate, so
            // both waves of a SIMD always have matrix and vector work to issue (a wave that
            // only issues MFMAs leaves about one pipe slot in six empty, a wave that only
            // issues vector instructions gets one every 7 clocks against the port's 4.6).
            // Work is cut into half tiles h = 0, 1, 2 ... of 32 keys:
            //     QK(h): S_h = K_h Q^T          8 MFMAs, one accumulator
            //     SM(h): P_h = exp2(..S_h..)     16 x (fma, exp2, add) + 8 conversions per lane
            //     PV(h): O^T += V_h^T P_h^T      8 MFMAs, four accumulators
            // and iteration j >= 1 of the tile loop (K tile j, V tile j-1 in LDS) runs
            //     step a:  QK(2j)   -> sA | PV(2j-2) with pA | SM(2j-1): sB -> pB
            //     step b:  QK(2j+1) -> sB | PV(2j-1) with pB | SM(2j):   sA -> pA
            // 32 slots of one MFMA, its share of LDS reads (PF slots ahead) and one element of
            // the softmax each.  Iteration 0 (S_0, S_1, P_0) is the prologue; a wave whose last
            // visible tile is jl runs iterations 1 .. jl+1, the last one with QK on a tile it does
            // not need (results dropped): one code path keeps the accumulators in place.  For the
            // same reason there is one copy of the iteration, and the LDS buffers rotate through
            // the per-lane read addresses (twelve additions per iteration) and the scalar load
            // targets instead of through unrolled code.
            // One workgroup barrier per tile: before it every wave has waited for its own share
            // of K(j), V(j-1); after it the loads of K(j+1), V(j) go out into the buffers that
            // were read in iteration j-1.
            static_assert(NW == 8 && QB == 1 && BN == 64 && D == 128, "the interleaved order is written for 8 waves of 32 query rows, 64-key tiles and d = 128");
            static_assert(32 % PF == 0, "the fragment ring must divide the 32 slots of an iteration");
            const int jl = CAUSAL ? min(nkt - 1, qw_last / BN) : nkt - 1;  // last tile with a key this wave sees
            f32x16 sA, sB;
            u32x4 pA[2], pB[2];
            const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

            auto mask_half = [&](f32x16& sh, int k0h) __attribute__((always_inline)) {
                const bool need_mask = (k0h + 32 > N) || (CAUSAL && (k0h + 31 > qw0));
                if (need_mask) {
                    const int qi = qw0 + c;
                    const int lim = CAUSAL ? min(qi, N - 1) : N - 1;  // last visible key
                    const int rel = lim - k0h - 4 * g;               // register v holds key k0h + 8*(v/4) + 4*g + v%4
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (8 * (v >> 2) + (v & 3) > rel) sh[v] = -INFINITY;
                }
            };
            auto exp_pack_half = [&](const f32x16& sh, u32x4(&ph)[2], float& rs) __attribute__((always_inline)) {
                const float mb = m_use[0] * p.scale_l2;
                float rs0 = 0.f, rs1 = 0.f;
                static_for<2>([&](auto t_c) __attribute__((always_inline)) {
                    constexpr int t = decltype(t_c)::value;
                    u32x4 w;
                    static_for<4>([&](auto h_c) __attribute__((always_inline)) {
                        constexpr int h = decltype(h_c)::value;
                        const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sh[8 * t + 2 * h], p.scale_l2, -mb));
                        const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sh[8 * t + 2 * h + 1], p.scale_l2, -mb));
                        w[h] = T::pack2(e0, e1);
                        rs0 += e0;
                        rs1 += e1;
                    });
                    ph[t] = w;
                });
                rs = rs0 + rs1;
            };
            auto raise_reference_half = [&](const f32x16& sh) __attribute__((always_inline)) {
                float mx = sh[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sh[v]);
                const float m_new = fmaxf(m_use[0], xhalf_max(mx));
                // finite from half tile 0 on: key 0 is visible to every query
                const float alpha = __builtin_amdgcn_exp2f((m_use[0] - m_new) * p.scale_l2);
                m_use[0] = m_new;
                l_run[0] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[0][dt][v] *= alpha;
            };

            // Tile movement of this order: buffer loads straight into LDS.  The buffer descriptor
            // covers the head's N rows, the tile and piece go into the scalar offset, the lane's
            // share (with the swizzle) is the one vector offset kept for the whole kernel.  Rows
            // past the end of the sequence, and whole tiles past it, arrive as zeros (the range
            // check of the buffer descriptor), so ragged tails need neither a branch nor a clamp;
            // their scores are masked.  which = 0: K, 1: V; piece = 0, 1 (NT chunks each).
            static_assert(LD_PER_THREAD == 2, "two pieces per tile and lane");
            // (descriptor: base, stride 0, number of bytes, and the flag word of an untyped 32-bit buffer)
            const int head_bytes = (int)((unsigned)N * (unsigned)RB);  // below 2^32: checked by the host before the launch
            const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Kh), 0, head_bytes, 0x00020000);
            const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(Vh), 0, head_bytes, 0x00020000);
            auto tile_load = [&](int which, int tile, int buf, int piece) __attribute__((always_inline)) {
                constexpr int ROWS_PER_PIECE = NT / CPR;
                char* dst = smem_b + buf * 2 * TILE_BYTES + which * TILE_BYTES + (piece * NT + wave * 64) * 16;
                const unsigned soff = (unsigned)tile * (BN * RB) + piece * (ROWS_PER_PIECE * RB);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(which ? v_rsrc : k_rsrc, (lds_void_ptr)dst, 16, which ? goffV0 : goffK0, soff, 0, 0);
            };
            // The same piece through registers (LDP = 0): a wave's LDS reads queue behind its own loads
            // to LDS that are still in flight, which stalls a stream that reads LDS all the time; a
            // load into registers does not, and the piece is written to LDS when the stream is over.
            auto tile_load_reg = [&](int which, int tile, int piece) __attribute__((always_inline)) -> u32x4 {
                constexpr int ROWS_PER_PIECE = NT / CPR;
                const unsigned soff = (unsigned)tile * (BN * RB) + piece * (ROWS_PER_PIECE * RB);
                return __builtin_amdgcn_raw_buffer_load_b128(which ? v_rsrc : k_rsrc, which ? goffV0 : goffK0, soff, 0);
            };
            auto tile_store_reg = [&](int which, int buf, int piece, u32x4 val) __attribute__((always_inline)) {
                *reinterpret_cast<u32x4*>(smem_b + buf * 2 * TILE_BYTES + which * TILE_BYTES + (piece * NT + tid) * 16) = val;
            };

            // Per-lane LDS read addresses of the tiles the current iteration reads (K tile j in
            // buffer j % NB, V tile j-1 in buffer (j-1) % NB), advanced once per iteration.
            int kaddr[KS], vaddr[DT];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kaddr[ks] = (int)lds_address(smem_b) + koff[ks];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vaddr[dt] = (int)lds_address(smem_b) + TILE_BYTES + voff[dt];
            // LDS fragment of slot i (0 .. 31) of an iteration: slots 0..15 are step a (first halves of
            // both tiles), 16..31 step b; inside a step even slots are QK k-steps, odd slots PV
            // steps (t, dt) = ((i/2)/4, (i/2)%4).
            auto read_frag = [&](int i) __attribute__((always_inline)) -> u32x4 {
                const int half = i >> 4, si = i & 15;
                if (si & 1) {
                    const int idx = si >> 1, t = idx >> 2, dt = idx & 3;
                    const unsigned a = (unsigned)vaddr[dt] + (half * 32 + 16 * t) * RB;
                    const u32x2 lo = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(unsigned long)a));
                    const u32x2 hi = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(unsigned long)(a + 8 * RB)));
                    return u32x4{lo[0], lo[1], hi[0], hi[1]};
                } else {
                    typedef const u32x4 __attribute__((address_space(3))) * lds_u32x4_ptr;
                    return *(lds_u32x4_ptr)(unsigned long)((unsigned)kaddr[si >> 1] + half * 32 * RB);
                }
            };
            // Fence between instruction groups.  ILV picks the group: 0 = one slot (an MFMA, then its
            // LDS reads, then the softmax element), 1 = two slots, 2 = four slots; inside a
            // group the order MFMA, LDS reads, transcendental, other vector work is requested
            // from the scheduler with sched_group_barrier.
            auto slot_fence = [&](int si) __attribute__((always_inline)) {
                constexpr int G = ILV == 0 ? 1 : (ILV == 1 ? 2 : 4);
                if ((si + 1) % G == 0) {
                    if constexpr (ILV != 0) {
#pragma unroll
                        for (int r = 0; r < G; ++r) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // LDS reads
                            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);  // transcendental
                            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);  // other vector instructions
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };

            u32x4 ring[PF];
            // One step of 16 slots: QK of a half tile into sN (overwritten), PV with pO, softmax of
            // sC into pN.  k0C = first key of the half tile sC belongs to; act = that half tile
            // exists for this wave (false only for the dropped work of the last iteration).
            auto half_step = [&](auto half_c, f32x16& sN, f32x16& sC, const u32x4(&pO)[2], u32x4(&pN)[2], int k0C, bool act,
                                 auto&& after_mfma) __attribute__((always_inline)) {
                constexpr int HALF = decltype(half_c)::value;
                mask_half(sC, k0C);
                const float mb = m_use[0] * p.scale_l2;
                float rs0 = 0.f, rs1 = 0.f;
                // two-stage software pipeline over the elements: slot si forms the exponential of
                // element si+1 and sums / converts element si
                float e_cur = __builtin_amdgcn_exp2f(__builtin_fmaf(sC[0], p.scale_l2, -mb));
                float e_prev = 0.f;
                u32x4 w;
                static_for<16>([&](auto si_c) __attribute__((always_inline)) {
                    constexpr int si = decltype(si_c)::value, i = HALF * 16 + si;
                    if constexpr ((si & 1) == 0) {
                        constexpr int ks = si >> 1;
                        if constexpr (ks == 0) sN = T::mfma(ring[i % PF], qreg[0][ks], zero16);
                        else sN = T::mfma(ring[i % PF], qreg[0][ks], sN);
                    } else {
                        constexpr int idx = si >> 1, t = idx >> 2, dt = idx & 3;
                        o[0][dt] = T::mfma(ring[i % PF], pO[t], o[0][dt]);
                    }
                    after_mfma(std::integral_constant<int, i>{});
                    if constexpr (i + PF < 32) ring[i % PF] = read_frag(i + PF);
                    float e_next = 0.f;
                    if constexpr (si + 1 < 16) e_next = __builtin_amdgcn_exp2f(__builtin_fmaf(sC[si + 1], p.scale_l2, -mb));
                    if constexpr (si & 1) {
                        rs1 += e_cur;
                        unsigned packed = T::pack2(e_prev, e_cur);
                        // pinned here: the slow path below overwrites P, so the compiler would otherwise
                        // sink the conversions into the fast path and keep every exponential alive
                        asm volatile("" : "+v"(packed));
                        w[(si & 7) >> 1] = packed;
                        if constexpr ((si & 7) == 7) pN[si >> 3] = w;
                    } else {
                        rs0 += e_cur;
                    }
                    e_prev = e_cur;
                    e_cur = e_next;
                    slot_fence(si);
                });
                // The row sum is consumed unconditionally (select, not branch): otherwise the
                // compiler sinks the additions into the branch and keeps every exponential alive.
                float rs = rs0 + rs1;
                const bool bad = !(rs <= 256.0f);                       // true for inf and NaN too
                if (__builtin_amdgcn_ballot_w64(bad && act) != 0) {  // wave-uniform, rare
                    raise_reference_half(sC);
                    exp_pack_half(sC, pN, rs);
                }
                l_run[0] += act ? rs : 0.f;
            };

            // ---- iteration 0: the first tiles, S_0 and S_1, P_0
#pragma unroll
            for (int piece = 0; piece < 2; ++piece) tile_load(0, 0, 0, piece);
#pragma unroll
            for (int piece = 0; piece < 2; ++piece) tile_load(1, 0, 0, piece);
#pragma unroll
            for (int piece = 0; piece < 2; ++piece) tile_load(0, 1, 1, piece);
            load_q();
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            {
                u32x4 kf[2];
                kf[0] = *reinterpret_cast<const u32x4*>(smem_b + koff[0]);
                kf[1] = *reinterpret_cast<const u32x4*>(smem_b + 32 * RB + koff[0]);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    u32x4 a0 = kf[0], a1 = kf[1];
                    if (ks + 1 < KS) {
                        kf[0] = *reinterpret_cast<const u32x4*>(smem_b + koff[ks + 1]);
                        kf[1] = *reinterpret_cast<const u32x4*>(smem_b + 32 * RB + koff[ks + 1]);
                    }
                    sA = T::mfma(a0, qreg[0][ks], ks == 0 ? zero16 : sA);
                    sB = T::mfma(a1, qreg[0][ks], ks == 0 ? zero16 : sB);
                }
                mask_half(sA, 0);
                raise_reference_half(sA);
                float rs;
                exp_pack_half(sA, pA, rs);
                l_run[0] += rs;
            }

            // ---- iterations 1 .. nkt.  kb / vb: buffers read in iteration j; kn: buffer K(j+1) goes to
            // (V(j) goes to the buffer with K(j)'s index).  A wave runs the stream in iterations
            // 1 .. jl+1 and only moves its share of the tiles in the others; these are two loops,
            // because a branch around the stream makes the register allocator copy all accumulators
            // on every trip.  Both loops together pass the same number of barriers in every wave.
            int kb = 1 % NB, vb = 0;
            u32x4 stg[LDP == 0 ? 4 : 1];
            // load l of iteration j: 0, 1 = the pieces of K(j+1) (into buffer kn), 2, 3 = the pieces of V(j)
            // (into the buffer with K(j)'s index)
            auto load_number = [&](int j, int l, int kn) __attribute__((always_inline)) {
                if constexpr (LDP == 1) {
                    if (l < 2) tile_load(0, j + 1, kn, l & 1);
                    else tile_load(1, j, kb, l & 1);
                } else {
                    stg[l] = tile_load_reg(l >> 1, l < 2 ? j + 1 : j, l & 1);
                }
            };
            auto land_staged = [&](int kn) __attribute__((always_inline)) {  // LDP = 0: registers -> LDS, before the next barrier
                if constexpr (LDP == 0) {
#pragma unroll
                    for (int l = 0; l < 4; ++l) tile_store_reg(l >> 1, l < 2 ? kn : kb, l & 1, stg[l]);
                }
            };
            const int jrun = jl + 1;
            for (int j = 1; j <= jrun; ++j) {
                const int kn = kb + 1 == NB ? 0 : kb + 1;
                // advance the read addresses: K from tile j-1's buffer to tile j's, V from tile j-2's to tile j-1's
                {
                    const int kstep = kb == 0 ? -(NB - 1) * 2 * TILE_BYTES : 2 * TILE_BYTES;
                    const int vstep = j == 1 ? 0 : (vb == 0 ? -(NB - 1) * 2 * TILE_BYTES : 2 * TILE_BYTES);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) kaddr[ks] += kstep;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) vaddr[dt] += vstep;
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of K(j), V(j-1) has landed
                __syncthreads();
                // This iteration's loads: K(j+1) and V(j), two 16-byte pieces per lane each, into
                // buffers nobody reads in this iteration.  LDPOS = 0: all four right after the
                // barrier.  LDPOS > 0: between the MFMAs of the stream (a load holds the issuing wave
                // until the texture path has taken it, and eight waves issuing four loads each right
                // after the barrier queue behind each other).
                if constexpr (LDPOS == 0) {
#pragma unroll
                    for (int l = 0; l < 4; ++l) load_number(j, l, kn);
                }
                auto stream_load = [&](auto i_c) __attribute__((always_inline)) {
                    constexpr int i = decltype(i_c)::value;
                    // load l goes out after slot 8*l + 3 (LDPOS 1) or 8*l + wave (LDPOS 2: one wave per slot)
                    if constexpr (LDPOS == 1) {
                        if constexpr ((i & 7) == 3) load_number(j, i >> 3, kn);
                    } else if constexpr (LDPOS == 2) {
                        if ((i & 7) == wave) load_number(j, i >> 3, kn);
                    }
                };
                if constexpr (PRIO == 1) __builtin_amdgcn_s_setprio(1);
                if constexpr (PRIO == 2) { if (wave >= NW / 2) __builtin_amdgcn_s_setprio(1); }
#pragma unroll
                for (int i = 0; i < PF; ++i) ring[i] = read_frag(i);
                __builtin_amdgcn_sched_barrier(0);
                half_step(c0, sA, sB, pA, pB, (2 * j - 1) * 32, true, stream_load);
                half_step(c1, sB, sA, pB, pA, 2 * j * 32, j <= jl, stream_load);
                if constexpr (PRIO != 0) __builtin_amdgcn_s_setprio(0);
                land_staged(kn);
                vb = kb;
                kb = kn;
            }
            for (int j = jrun + 1; j <= nkt; ++j) {
                const int kn = kb + 1 == NB ? 0 : kb + 1;
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
#pragma unroll
                for (int l = 0; l < 4; ++l) load_number(j, l, kn);
                land_staged(kn);
                vb = kb;
                kb = kn;
            }
        } else {
            // Ping-pong order for two waves per SIMD.  The tile loop is cut into two clusters:
            //     M_j : O += P(j) V(j)  and  S(j+1) = K(j+1) Q^T      (MFMA + LDS reads only)
            //     V_j : mask, softmax of S(j+1) -> P(j+1)              (VALU only)
            // and the workgroup into two groups of NW/2 waves (waves w and w + NW/2 share a
            // SIMD).  Group B runs one cluster behind group A, with a workgroup barrier between
            // clusters ("slots"), so in every slot one wave of each SIMD feeds the MFMA pipe
            // while the other one uses the VALU:
            //     slot   0    1    2    3   ...
            //     A      M_0  V_0  M_1  V_1
            //     B      -    M_0  V_0  M_1
            // S lives in registers from M to V, P from V to the next M; no second S buffer.
            // LDS: M_j reads K(j+1) from K buffer (j+1)&1 and V(j) from V buffer j&1.  The loads
            // of K(j+2) and V(j+1) may start in slot 2j (their targets were last read in slot
            // 2j-1) and must have landed when slot 2j+1 ends.  Every wave issues its share at
            // the start of one of its V clusters (group B in slot 2j, group A in slot 2j+1):
            // a wave that has LDS-direct loads in flight gets its own LDS reads queued behind
            // them, which would stall an MFMA cluster but costs a VALU cluster nothing.
            static_assert(NW == 8, "the ping-pong order needs two waves per SIMD in one workgroup");
            const bool grp_b = wave >= NW / 2;
            auto cluster_m = [&](auto par_c, int j) __attribute__((always_inline)) {  // par = j & 1
                constexpr int PAR = decltype(par_c)::value;
                constexpr std::integral_constant<int, PAR ^ 1> kbuf{};
                // On a wave's last active tile the S part runs on a K buffer nobody needs (its
                // result is dropped by cluster V): one code path instead of two keeps the
                // accumulators in place.
                if (tile_active(j)) mfma_stream(yes, yes, par_c, kbuf, pk, s);
            };

            issue_k(0, 0);
            issue_v(0, 0);
            if constexpr (QSTAGE) {
                issue_k(1, 1);  // all three first tiles in flight together, one wait
                request_q();
                land_loads(0, 0);
            } else if constexpr (LDP == 1) {
                issue_k(1, 1);  // all three first tiles in flight together, one wait
                load_q();
                land_loads(0, 0);
            } else {
                load_q();
                land_loads(0, 0);
                issue_k(1, 1);
                issue_v(1, 1);  // the staging path lands K and V together
                land_loads(1, 1);
            }
            __syncthreads();
            if constexpr (QSTAGE) read_q();
            mfma_stream(no, yes, c0, c0, pk, s);
            if constexpr (NB3) issue_tiles(2, 2, 1, 1);
            softmax_first_tile(s, pk);
            if constexpr (NB3) land_loads(0, 0);
            __syncthreads();  // every wave has read K(0) before K(2) overwrites it

            if constexpr (NB3) {
                // Three buffers: in period j (from one barrier to the next; group A runs M_j then V_j,
                // group B V_(j-1) then M_j) the M clusters read K(j+1) in K buffer (j+1)%3 and V(j) in V
                // buffer j%3, and the loads bring K(j+3) into K buffer j%3 and V(j+2) into V buffer
                // (j+2)%3, both last read in period j-1 and first read in period j+2.  The only thing
                // a barrier still has to separate is one period from the next: one barrier per tile
                // instead of two, and the two waves of a SIMD keep their alternation by themselves
                // (each does one M and one V cluster per period, in opposite order).  K(2) and V(1),
                // which periods 0 and 1 read, were requested behind the S(0) stream.
                static_assert(LDP == 1, "three buffers: tiles straight to LDS");
                auto period_loads = [&](int j) __attribute__((always_inline)) { issue_tiles(j + 3, j % 3, j + 2, (j + 2) % 3); };
                auto cluster_m3 = [&](auto r_c, int j) __attribute__((always_inline)) {  // r = j % 3
                    constexpr int R = decltype(r_c)::value;
                    constexpr std::integral_constant<int, (R + 1) % 3> kbuf{};
                    if (tile_active(j)) mfma_stream(yes, yes, r_c, kbuf, pk, s);
                };
                auto cluster_v = [&](int j) __attribute__((always_inline)) {
                    if (tile_active(j + 1)) softmax_tile(s, pk, (j + 1) * BN);
                };
                constexpr std::integral_constant<int, 2> c2{};
                // (one loop per group: a branch on the group inside one loop would give the accumulators
                // two code paths and the register allocator a reason to move them)
                if (!grp_b) {
                    auto period = [&](auto r_c, int j) __attribute__((always_inline)) {
                        cluster_m3(r_c, j);
                        period_loads(j);
                        cluster_v(j);
                        land_loads(0, 0);
                        __syncthreads();
                    };
                    for (int j = 0; j < nkt; j += 3) {
                        period(c0, j);
                        if (j + 1 >= nkt) break;
                        period(c1, j + 1);
                        if (j + 2 >= nkt) break;
                        period(c2, j + 2);
                    }
                } else {
                    auto period = [&](auto r_c, int j) __attribute__((always_inline)) {
                        period_loads(j);
                        if (j > 0) cluster_v(j - 1);
                        land_loads(0, 0);
                        cluster_m3(r_c, j);
                        __syncthreads();
                    };
                    for (int j = 0; j < nkt; j += 3) {
                        period(c0, j);
                        if (j + 1 >= nkt) break;
                        period(c1, j + 1);
                        if (j + 2 >= nkt) break;
                        period(c2, j + 2);
                    }
                }
            } else if constexpr (PIPE == 1) {
                // Every wave issues its share of a tile at the start of one of its V clusters
                // (group B in slot 2j, group A in slot 2j+1).
                auto slot_loads = [&](int j) __attribute__((always_inline)) {  // the loads of slot 2j; buffer indices are runtime here
                    if constexpr (PRIO == 2) __builtin_amdgcn_s_setprio(2);
                    issue_tiles(j + 2, j & 1, j + 1, (j + 1) & 1);
                    if constexpr (PRIO == 2) __builtin_amdgcn_s_setprio(0);
                };
                auto cluster_v = [&](int j) __attribute__((always_inline)) {
                    if (tile_active(j + 1)) softmax_tile(s, pk, (j + 1) * BN);
                };
                // lands what slot_loads(j) issued: K(j+2) -> K buffer j&1, V(j+1) -> V buffer (j+1)&1
                auto land_slot = [&](int j) __attribute__((always_inline)) { land_loads(j & 1, (j + 1) & 1); };
                if (!grp_b) {
                    for (int j = 0; j < nkt; j += 2) {
                        cluster_m(c0, j);
                        __syncthreads();
                        slot_loads(j);
                        cluster_v(j);
                        land_slot(j);
                        __syncthreads();
                        if (j + 1 < nkt) {
                            cluster_m(c1, j + 1);
                            __syncthreads();
                            slot_loads(j + 1);
                            cluster_v(j + 1);
                            land_slot(j + 1);
                            __syncthreads();
                        }
                    }
                } else {
                    slot_loads(0);
                    __syncthreads();
                    for (int j = 0; j < nkt; j += 2) {
                        cluster_m(c0, j);
                        land_slot(j);
                        __syncthreads();
                        if (j + 1 < nkt) slot_loads(j + 1);
                        cluster_v(j);
                        if (j + 1 < nkt) {
                            __syncthreads();
                            cluster_m(c1, j + 1);
                            land_slot(j + 1);
                            __syncthreads();
                            if (j + 2 < nkt) slot_loads(j + 2);
                            cluster_v(j + 1);
                            if (j + 2 < nkt) __syncthreads();
                        }
                    }
                }
            } else {
                // PIPE == 2: both clusters use the MFMA pipe.
                //     X_j : S(j+1) = K(j+1) Q^T                      (MFMA only; issues tile loads)
                //     Y_j : O += P(j) V(j), with the softmax of S(j+1) worked in between the
                //           MFMAs -> P(j+1)                          (MFMA + VALU)
                //     slot   0    1    2    3   ...
                //     A      X_0  Y_0  X_1  Y_1
                //     B      -    X_0  Y_0  X_1
                // Every slot then carries the MFMA work of half a tile from each wave of a SIMD
                // and the VALU work of one softmax, instead of all MFMA work on one wave and
                // all VALU work on the other.
                // LDS: K(j+1) is read in slots 2j, 2j+1 and V(j) in slots 2j+1, 2j+2.  Group A
                // moves the K tiles (K(j+2) issued at the start of X_j in slot 2j, landed when
                // its Y_j ends in slot 2j+1), group B the V tiles (V(j+1) issued at the start of
                // its X_j in slot 2j+1, landed when its Y_j ends in slot 2j+2): a wave in an X
                // cluster can afford the issue stalls, it mostly waits for the shared pipe.
                static_assert(LDP == 1, "tile loads of this order go straight to LDS");
                constexpr int LNT = NT / 2, LLD = TILE_CHUNKS / LNT;
                constexpr std::integral_constant<int, LNT> lnt_c{};
                const int lt = tid & (LNT - 1), lwave = wave & (NW / 2 - 1);
                const unsigned goff_grp = grp_b ? goff_v(lt) : goff_k(lt);
                u32x4 none;
                // group A: K(j+2) -> K buffer j&1;  group B: V(j+1) -> V buffer (j+1)&1
                auto group_loads = [&](int j) __attribute__((always_inline)) {
                    const int jt = grp_b ? j + 1 : j + 2;
                    if (jt < nkt) {
                        const int kt0 = jt * BN;
                        const bool whole = kt0 + BN <= N;
                        char* dst = grp_b ? smem_b + ((j + 1) & 1) * 2 * TILE_BYTES + TILE_BYTES : smem_b + (j & 1) * 2 * TILE_BYTES;
#pragma unroll
                        for (int q = 0; q < LLD; ++q) issue_piece(lnt_c, whole, grp_b ? Vh : Kh, goff_grp, lwave, kt0, dst, q, none);
                    }
                };
                auto cluster_x = [&](auto par_c, int j) __attribute__((always_inline)) {  // par = j & 1
                    constexpr int PAR = decltype(par_c)::value;
                    constexpr std::integral_constant<int, PAR ^ 1> kbuf{};
                    group_loads(j);
                    if (tile_active(j + 1)) mfma_stream(no, yes, par_c, kbuf, pk, s);
                };
                auto cluster_y = [&](auto par_c, int j) __attribute__((always_inline)) {
                    if (tile_active(j)) pv_softmax_stream(par_c, pk, s, (j + 1) * BN, tile_active(j + 1));
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this group's tile has landed
                };
                if (!grp_b) {
                    for (int j = 0; j < nkt; j += 2) {
                        cluster_x(c0, j);
                        __syncthreads();
                        cluster_y(c0, j);
                        __syncthreads();
                        if (j + 1 < nkt) {
                            cluster_x(c1, j + 1);
                            __syncthreads();
                            cluster_y(c1, j + 1);
                            __syncthreads();
                        }
                    }
                } else {
                    __syncthreads();
                    for (int j = 0; j < nkt; j += 2) {
                        cluster_x(c0, j);
                        __syncthreads();
                        cluster_y(c0, j);
                        if (j + 1 < nkt) {
                            __syncthreads();
                            cluster_x(c1, j + 1);
                            __syncthreads();
                            cluster_y(c1, j + 1);
                            if (j + 2 < nkt) __syncthreads();
                        }
                    }
                }
            }
        }

        // ---- epilogue: normalise, round once, store O and lse.  A lane holds 8-byte pieces
        // of one row of O; stored directly they would scatter over 32 rows per instruction.
        // Each wave transposes its 32*QB rows through its own part of LDS instead (the K/V
        // tiles are dead by now) and writes whole rows, 16 bytes per lane, 1 KB contiguous
        // per instruction.  Chunk k of row r sits at chunk k ^ (r mod CPR): conflict-free
        // row-wise reads, two-way conflicts on the column-wise writes.
        static_assert(BM * RB <= 4 * TILE_BYTES, "the O tile must fit into the K/V buffers");
        __syncthreads();  // every wave has finished reading the last K/V tiles
        {
            char* stage = smem_b + wave * (32 * QB * RB);
            // Per-lane addresses below are the same for every work item; an opaque copy of the
            // lane id keeps the compiler from computing them once, ahead of the item loop, and
            // holding (or spilling) them through the tile loops.
            int le = lane;
            asm volatile("" : "+v"(le));
            const int ce = le & 31, ge = le >> 5;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float l_tot = xhalf_sum(l_run[qb]);
                const float inv = 1.0f / l_tot;
                const int qi = qw0 + qb * 32 + ce;
                char* srow = stage + (qb * 32 + ce) * RB + ge * 8;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        u32x2 w;
                        w[0] = T::pack2(o[qb][dt][4 * v4 + 0] * inv, o[qb][dt][4 * v4 + 1] * inv);
                        w[1] = T::pack2(o[qb][dt][4 * v4 + 2] * inv, o[qb][dt][4 * v4 + 3] * inv);
                        *reinterpret_cast<u32x2*>(srow + (((dt * 4 + v4) ^ (ce & (CPR - 1))) * 16)) = w;
                    }
                if (ge == 0 && qi < N) p.lse[(size_t)bh * N + qi] = m_use[qb] * p.scale + __logf(l_tot);
            }
            asm volatile("" ::: "memory");  // same wave: LDS executes its writes and reads in order
            uint16_t* obase = p.out + head_off + (size_t)qw0 * D;
#pragma unroll
            for (int i = 0; i < 32 * QB * CPR / 64; ++i) {
                const int f = i * 64 + le, row = f / CPR, k = f % CPR;
                const u32x4 val = *reinterpret_cast<const u32x4*>(stage + row * RB + ((k ^ (row & (CPR - 1))) * 16));
                if (qw0 + row < N) *reinterpret_cast<u32x4*>(obase + (size_t)row * D + k * 8) = val;
            }
        }
    }
}

}  // namespace attn
