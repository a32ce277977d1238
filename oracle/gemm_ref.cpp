// CPU oracle of the second workload: C = leaky_relu(A B), the fused GEMM + LeakyReLU of the
// paper's Sec. 5 (Table 3: M, N, K = 512, 512, 2048, binary16 tensors).
//
// TEST INFRASTRUCTURE ONLY: used by tests/ and by the benchmark's cpu_baseline leg, never by
// the product path, and it shares no code with the HIP kernels.
//
// The definition written out, in double precision: inputs are decoded exactly from their
// 16-bit patterns, every product and the whole sum are formed in fp64 in index order, then
// leaky_relu(x) = x for x >= 0 and slope * x otherwise.  No blocking, no reordering.
// The paper names the operation but not the slope; it is an argument here.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

double decode16(uint16_t h, int dtype) {
    if (dtype == 1) {  // bfloat16: the upper half of a binary32
        uint32_t u = (uint32_t)h << 16;
        float f;
        std::memcpy(&f, &u, 4);
        return (double)f;
    }
    const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;  // binary16
    double v;
    if (e == 0) v = std::ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = std::ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

}  // namespace

extern "C" {

// a: [M, K], b: [K, N] row-major 16-bit patterns (host); out: [M, N] doubles (host).
// dtype 0 = binary16, 1 = bfloat16.  nthreads <= 0: all hardware threads; *threads_used
// (may be null) receives the number actually started.  Returns 0, or -1 on bad arguments.
int gemm_lrelu_ref_f64(const uint16_t* a, const uint16_t* b, double* out, int M, int N, int K,
                       double slope, int dtype, int nthreads, int* threads_used) {
    if (!a || !b || !out || M < 1 || N < 1 || K < 1 || (dtype != 0 && dtype != 1)) return -1;
    std::vector<double> bd((size_t)K * N);
    for (size_t i = 0; i < bd.size(); ++i) bd[i] = decode16(b[i], dtype);
    int nt = nthreads > 0 ? nthreads : (int)std::thread::hardware_concurrency();
    if (nt < 1) nt = 1;
    if (nt > M) nt = M;
    if (threads_used) *threads_used = nt;
    auto work = [&](int t) {
        std::vector<double> ar(K);
        for (int i = t; i < M; i += nt) {
            for (int k = 0; k < K; ++k) ar[k] = decode16(a[(size_t)i * K + k], dtype);
            for (int j = 0; j < N; ++j) {
                double s = 0.0;
                for (int k = 0; k < K; ++k) s += ar[k] * bd[(size_t)k * N + j];
                out[(size_t)i * N + j] = s >= 0.0 ? s : slope * s;
            }
        }
    };
    std::vector<std::thread> th;
    for (int t = 1; t < nt; ++t) th.emplace_back(work, t);
    work(0);
    for (auto& x : th) x.join();
    return 0;
}

}  // extern "C"
