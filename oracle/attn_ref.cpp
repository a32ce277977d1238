// CPU oracle for scaled-dot-product attention forward (softmax(scale * Q K^T) V
// and the row log-sum-exp).  TEST INFRASTRUCTURE ONLY: plain, slow, fp64, two
// passes per row, no tiling, no online softmax.  It shares no code with the GPU
// library and must never be reached from the product path.
//
// What it follows: the paper only *names* the kernel it tunes (fused attention
// a.k.a. flash-attention, Sec. 1 and Sec. 5 "Experiment setup"), its tensor
// format [batch, heads, seq, head_dim] (Table 2 caption) and that a mutated
// kernel is compared with a reference output on random inputs (Sec. 4.2).  The
// fused kernel reaches exactly the textbook result, so the oracle is the
// textbook definition written out:
//
//   for every (b, h) and query row i:
//     J(i)  = {0..N-1}            (non-causal)   or   {0..i}   (causal)
//     x_j   = scale * sum_c Q[i,c] K[j,c]                       j in J(i)
//     M     = max_j x_j ;  L = sum_j exp(x_j - M)
//     lse_i = M + ln L
//     O[i,c]= sum_j (exp(x_j - M) / L) * V[j,c]
//
// Inputs are raw 16-bit patterns (IEEE binary16 or bfloat16); both embed exactly
// in fp64 and are decoded here by hand.  All arithmetic after decoding is fp64.
//
// Pins (see tests/test_oracle_*.py): brute force with a differently written
// long-double evaluation on tiny inputs, closed forms (N=1, N=2 -> logistic
// sigmoid, Q=0 -> uniform average), invariants (rows of P sum to 1, constant V,
// joint K/V permutation, causal prefix property, key-shift invariance) and a
// library composition (softmax/logsumexp in fp64).
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

double decode_f16(uint16_t h) {
    const int sign = (h >> 15) & 1;
    const int e = (h >> 10) & 0x1f;
    const int m = h & 0x3ff;
    double val;
    if (e == 0) {
        val = std::ldexp((double)m, -24);  // subnormal: m * 2^-10 * 2^-14
    } else if (e == 31) {
        val = m ? std::nan("") : INFINITY;
    } else {
        val = std::ldexp((double)(m | 0x400), e - 25);  // (1 + m/1024) * 2^(e-15)
    }
    return sign ? -val : val;
}

double decode_bf16(uint16_t h) {
    // bfloat16 is the upper half of an IEEE binary32.
    const uint32_t bits = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &bits, sizeof f);
    return (double)f;
}

double decode(uint16_t h, int dtype) { return dtype == 0 ? decode_f16(h) : decode_bf16(h); }

struct Problem {
    const uint16_t *q, *k, *v;
    int B, H, N, d, causal, dtype;
    double scale;
};

// K and V of one head decoded to fp64 once, so the row loops below read plain
// doubles.  (Decoding is exact; this only hoists it out of the inner loops.)
struct HeadCache {
    long long bh = -1;
    std::vector<double> K, V;
    void load(const Problem& p, long long want) {
        if (want == bh) return;
        const size_t n = (size_t)p.N * p.d;
        K.resize(n);
        V.resize(n);
        const uint16_t* k = p.k + (size_t)want * n;
        const uint16_t* v = p.v + (size_t)want * n;
        for (size_t e = 0; e < n; ++e) {
            K[e] = decode(k[e], p.dtype);
            V[e] = decode(v[e], p.dtype);
        }
        bh = want;
    }
};

// One query row of one head.  `x` is scratch of length N, `qd` of length d.  If
// `probs` is not null the normalised softmax row is written there (zeros for
// masked keys).
void one_row(const Problem& p, const HeadCache& hc, int i, double* x, double* qd, double* o_row,
             double* lse_out, double* probs) {
    const int N = p.N, d = p.d;
    const uint16_t* Q = p.q + ((size_t)hc.bh * N + i) * d;
    for (int c = 0; c < d; ++c) qd[c] = decode(Q[c], p.dtype);
    const double* K = hc.K.data();
    const double* V = hc.V.data();
    const int nvis = p.causal ? i + 1 : N;  // key j is visible iff j <= i

    double M = -INFINITY;
    for (int j = 0; j < nvis; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += qd[c] * K[(size_t)j * d + c];
        x[j] = p.scale * dot;
        if (x[j] > M) M = x[j];
    }
    double L = 0.0;
    for (int j = 0; j < nvis; ++j) L += std::exp(x[j] - M);
    *lse_out = M + std::log(L);

    for (int c = 0; c < d; ++c) o_row[c] = 0.0;
    for (int j = 0; j < nvis; ++j) {
        const double pj = std::exp(x[j] - M) / L;
        if (probs) probs[j] = pj;
        for (int c = 0; c < d; ++c) o_row[c] += pj * V[(size_t)j * d + c];
    }
    if (probs)
        for (int j = nvis; j < N; ++j) probs[j] = 0.0;
}

bool bad_args(const void* q, const void* k, const void* v, const void* out, const void* lse, int B,
              int H, int N, int d, int dtype) {
    return !q || !k || !v || !out || !lse || B < 1 || H < 1 || N < 1 || d < 1 ||
           (dtype != 0 && dtype != 1);
}

}  // namespace

extern "C" {

// Host buffers only.  q, k, v: [B,H,N,d] contiguous, raw 16-bit patterns
// (dtype 0 = binary16, 1 = bfloat16).  If rows == NULL every row is computed,
// out is [B,H,N,d] and lse is [B,H,N]; otherwise rows[r] is a flattened
// (b*H + h)*N + i index, out is [nrows,d] and lse is [nrows].  nthreads <= 0
// means std::thread::hardware_concurrency().  Returns 0, or -1 on bad arguments.
// *threads_used (may be NULL) receives the number of worker threads started.
int attn_ref_f64(const uint16_t* q, const uint16_t* k, const uint16_t* v, double* out, double* lse,
                 int B, int H, int N, int d, int causal, double scale, int dtype,
                 const long long* rows, long long nrows, int nthreads, int* threads_used) {
    if (bad_args(q, k, v, out, lse, B, H, N, d, dtype)) return -1;
    const long long total = rows ? nrows : (long long)B * H * N;
    if (rows) {
        if (nrows < 0) return -1;
        for (long long r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= (long long)B * H * N) return -1;
    }
    Problem p{q, k, v, B, H, N, d, causal ? 1 : 0, dtype, scale};

    int nt = nthreads > 0 ? nthreads : (int)std::thread::hardware_concurrency();
    if (nt < 1) nt = 1;
    if ((long long)nt > total) nt = (int)(total > 0 ? total : 1);
    if (threads_used) *threads_used = nt;

    auto work = [&](int t) {
        std::vector<double> x((size_t)N), qd((size_t)d);
        HeadCache hc;
        // interleaved assignment keeps the causal triangle balanced over threads
        for (long long r = t; r < total; r += nt) {
            const long long flat = rows ? rows[r] : r;
            hc.load(p, flat / N);
            one_row(p, hc, (int)(flat % N), x.data(), qd.data(), out + (size_t)r * d, lse + r,
                    nullptr);
        }
    };
    if (nt == 1) {
        work(0);
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < nt; ++t) pool.emplace_back(work, t);
        for (auto& th : pool) th.join();
    }
    return 0;
}

// Debug entry point: the normalised softmax row P[b,h,i,:] (length N, zeros at
// masked keys), for the "rows of P sum to one" pin.
int attn_ref_probs_f64(const uint16_t* q, const uint16_t* k, int B, int H, int N, int d, int causal,
                       double scale, int dtype, long long row, double* probs) {
    if (!q || !k || !probs || B < 1 || H < 1 || N < 1 || d < 1 || (dtype != 0 && dtype != 1))
        return -1;
    if (row < 0 || row >= (long long)B * H * N) return -1;
    // V is irrelevant for P: reuse K as a stand-in so one_row can run unchanged.
    Problem p{q, k, k, B, H, N, d, causal ? 1 : 0, dtype, scale};
    std::vector<double> x((size_t)N), qd((size_t)d), o((size_t)d);
    HeadCache hc;
    hc.load(p, row / N);
    double lse;
    one_row(p, hc, (int)(row % N), x.data(), qd.data(), o.data(), &lse, probs);
    return 0;
}

// Decoders exposed so the tests can pin them against numpy's own float16 /
// float32 conversions over all 65536 bit patterns.
double attn_ref_decode(uint16_t bits, int dtype) { return decode(bits, dtype); }

}  // extern "C"
