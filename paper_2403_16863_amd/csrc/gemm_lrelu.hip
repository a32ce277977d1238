// Host side of the fused GEMM + LeakyReLU library entry points: variant table, argument checks,
// launches, timing, kernels loaded from code objects.  The kernel is in gemm_kernel.h.
#include "../../include/gemm_lrelu.h"

#include <stdio.h>

#include "gemm_kernel.h"

namespace gemm {

// ---- host side -----------------------------------------------------------------------------
typedef void (*KernelFn)(Params);
struct Variant {
    int wk, bkw, stages, rot;
    KernelFn fn[2];  // by dtype
};
#define GEMM_VARIANT(WK, BKW, S, ROT) \
    { WK, BKW, S, ROT, { gemm_lrelu_kernel<attn::F16, Knobs<WK, BKW, S, ROT>>, gemm_lrelu_kernel<attn::BF16, Knobs<WK, BKW, S, ROT>> } }
static const Variant kVariants[] = {
    GEMM_VARIANT(4, 32, 8, 0),   // 0
    GEMM_VARIANT(4, 32, 4, 0),   // 1
    GEMM_VARIANT(4, 32, 10, 0),  // 2
    GEMM_VARIANT(4, 64, 4, 0),   // 3
    GEMM_VARIANT(4, 64, 3, 0),   // 4
    GEMM_VARIANT(8, 32, 4, 0),   // 5
    GEMM_VARIANT(8, 32, 3, 0),   // 6
    GEMM_VARIANT(2, 64, 8, 0),   // 7
    GEMM_VARIANT(2, 64, 4, 0),   // 8
    GEMM_VARIANT(2, 32, 8, 0),   // 9
    GEMM_VARIANT(1, 64, 8, 0),   // 10
    GEMM_VARIANT(2, 32, 4, 0),   // 11
    GEMM_VARIANT(4, 32, 4, 1),   // 12
    GEMM_VARIANT(4, 32, 8, 1),   // 13
    GEMM_VARIANT(4, 64, 3, 1),   // 14
    GEMM_VARIANT(4, 64, 4, 1),   // 15
    GEMM_VARIANT(8, 32, 3, 1),   // 16
    GEMM_VARIANT(8, 32, 4, 1),   // 17
    GEMM_VARIANT(4, 32, 3, 0),   // 18
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr int kDefault = 1;

static int check_args(const void* a, const void* b, const void* c, int M, int N, int K, int dtype, int variant_id) {
    if (!a || !b || !c) return GEMM_EINVAL;
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 15) return GEMM_EINVAL;
    if (M < 1 || N < 8 || K < 8 || (N & 7) || (K & 7) || N >= (1 << 24) || K >= (1 << 24)) return GEMM_EINVAL;
    if ((long long)((M + 31) / 32) * ((N + 31) / 32) > 0x7fffffffLL) return GEMM_EINVAL;
    if (dtype != GEMM_F16 && dtype != GEMM_BF16) return GEMM_EINVAL;
    // C is written while other workgroups still read A and B: it must not overlap them
    const uintptr_t c0 = (uintptr_t)c, c1 = c0 + (size_t)M * N * 2;
    const uintptr_t a0 = (uintptr_t)a, a1 = a0 + (size_t)M * K * 2, b0 = (uintptr_t)b, b1 = b0 + (size_t)K * N * 2;
    if ((c0 < a1 && a0 < c1) || (c0 < b1 && b0 < c1)) return GEMM_EINVAL;
    if (variant_id < 0 || variant_id >= kNumVariants) return GEMM_EINVAL;
    return GEMM_OK;
}

static int launch(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype, void* stream,
                  int variant_id, hipFunction_t module_fn = nullptr) {
    const int rc = check_args(a, b, c, M, N, K, dtype, variant_id);
    if (rc != GEMM_OK) return rc;
    Params p;
    p.a = (const char*)a;
    p.b = (const char*)b;
    p.c = (uint16_t*)c;
    p.M = M, p.N = N, p.K = K;
    p.ntm = (M + 31) / 32, p.ntn = (N + 31) / 32;
    p.slope = slope;
    const Variant& v = kVariants[variant_id];
    void* args[] = {&p};
    const hipError_t e =
        module_fn ? hipModuleLaunchKernel(module_fn, (unsigned)(p.ntm * p.ntn), 1, 1, v.wk * 64, 1, 1, 0, (hipStream_t)stream, args, nullptr)
                  : hipLaunchKernel((const void*)v.fn[dtype], dim3(p.ntm * p.ntn), dim3(v.wk * 64), args, 0, (hipStream_t)stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ELAUNCH;
    }
    return GEMM_OK;
}

// ---- kernels loaded from code objects: the same kernel after its instructions were reordered
// outside the compiler.  A handle remembers which variant (launch shape) and type it replaces.
struct LoadedKernel {
    hipModule_t module = nullptr;
    hipFunction_t fn = nullptr;
    int variant_id = -1, dtype = 0;
};
constexpr int kMaxLoaded = 64;
static LoadedKernel g_loaded[kMaxLoaded];

template <class LaunchFn>
static int time_back_to_back(LaunchFn&& do_launch, void* stream, int warmup, int iters, float* ms_total) {
    if (!ms_total || iters < 1 || warmup < 0) return GEMM_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < warmup; ++i) {
        const int rc = do_launch();
        if (rc != GEMM_OK) return rc;
    }
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return GEMM_ELAUNCH;
    if (hipEventCreate(&e1) != hipSuccess) {
        hipEventDestroy(e0);
        return GEMM_ELAUNCH;
    }
    int rc = hipEventRecord(e0, s) == hipSuccess ? GEMM_OK : GEMM_ELAUNCH;
    for (int i = 0; i < iters && rc == GEMM_OK; ++i) rc = do_launch();
    if (rc == GEMM_OK &&
        (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
         hipEventElapsedTime(ms_total, e0, e1) != hipSuccess))
        rc = GEMM_ELAUNCH;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return rc;
}

}  // namespace gemm

extern "C" {

int gemm_lrelu_num_variants(void) { return gemm::kNumVariants; }
int gemm_lrelu_default_variant(int, int, int) { return gemm::kDefault; }

int gemm_lrelu_variant_knobs(int variant_id, int* knobs) {
    if (!knobs || variant_id < 0 || variant_id >= gemm::kNumVariants) return GEMM_EINVAL;
    knobs[0] = gemm::kVariants[variant_id].wk;
    knobs[1] = gemm::kVariants[variant_id].bkw;
    knobs[2] = gemm::kVariants[variant_id].stages;
    knobs[3] = gemm::kVariants[variant_id].rot;
    return GEMM_OK;
}

int gemm_lrelu_variant(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype, void* stream,
                       int variant_id) {
    return gemm::launch(a, b, c, M, N, K, slope, dtype, stream, variant_id);
}

int gemm_lrelu(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype, void* stream) {
    return gemm::launch(a, b, c, M, N, K, slope, dtype, stream, gemm_lrelu_default_variant(M, N, K));
}

int gemm_lrelu_time(const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype, void* stream,
                    int variant_id, int warmup, int iters, float* ms_total) {
    return gemm::time_back_to_back([&] { return gemm::launch(a, b, c, M, N, K, slope, dtype, stream, variant_id); }, stream,
                                   warmup, iters, ms_total);
}

int gemm_lrelu_codeobj_load(const char* path, const char* kernel_name, int variant_id, int dtype) {
    using namespace gemm;
    if (!path || !kernel_name || variant_id < 0 || variant_id >= kNumVariants) return GEMM_EINVAL;
    if (dtype != GEMM_F16 && dtype != GEMM_BF16) return GEMM_EINVAL;
    int slot = -1;
    for (int i = 0; i < kMaxLoaded; ++i)
        if (!g_loaded[i].fn) {
            slot = i;
            break;
        }
    if (slot < 0) return GEMM_EINVAL;  // table full: unload something first
    // A failed runtime call leaves its status behind for whoever asks next: look at the file
    // first, and consume the status of a load that fails anyway.
    if (FILE* f = fopen(path, "rb")) fclose(f);
    else return GEMM_ELAUNCH;
    LoadedKernel lk;
    if (hipModuleLoad(&lk.module, path) != hipSuccess) {
        (void)hipGetLastError();
        return GEMM_ELAUNCH;
    }
    if (hipModuleGetFunction(&lk.fn, lk.module, kernel_name) != hipSuccess) {
        (void)hipGetLastError();
        hipModuleUnload(lk.module);
        return GEMM_ELAUNCH;
    }
    lk.variant_id = variant_id;
    lk.dtype = dtype;
    g_loaded[slot] = lk;
    return slot;
}

int gemm_lrelu_codeobj_unload(int handle) {
    using namespace gemm;
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn) return GEMM_EINVAL;
    const hipError_t e = hipModuleUnload(g_loaded[handle].module);
    g_loaded[handle] = LoadedKernel();
    return e == hipSuccess ? GEMM_OK : GEMM_ELAUNCH;
}

int gemm_lrelu_codeobj(int handle, const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype,
                       void* stream) {
    using namespace gemm;
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn || g_loaded[handle].dtype != dtype) return GEMM_EINVAL;
    return launch(a, b, c, M, N, K, slope, dtype, stream, g_loaded[handle].variant_id, g_loaded[handle].fn);
}

int gemm_lrelu_time_codeobj(int handle, const void* a, const void* b, void* c, int M, int N, int K, float slope, int dtype,
                            void* stream, int warmup, int iters, float* ms_total) {
    using namespace gemm;
    if (handle < 0 || handle >= kMaxLoaded || !g_loaded[handle].fn || g_loaded[handle].dtype != dtype) return GEMM_EINVAL;
    const LoadedKernel lk = g_loaded[handle];
    return time_back_to_back([&] { return launch(a, b, c, M, N, K, slope, dtype, stream, lk.variant_id, lk.fn); }, stream,
                             warmup, iters, ms_total);
}

int gemm_lrelu_tile_of_block(int block, int ntm, int ntn, int* tm, int* tn) {
    if (!tm || !tn || ntm < 1 || ntn < 1 || (long long)ntm * ntn > 0x7fffffffLL) return GEMM_EINVAL;
    if (block < 0 || block >= ntm * ntn) return GEMM_EINVAL;
    gemm::tile_of_block(block, ntm, ntn, *tm, *tn);
    return GEMM_OK;
}

}  // extern "C"
