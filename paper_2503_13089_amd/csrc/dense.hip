// Dense product for the layer's forward pass at prefill-sized batches (layer listing, Appendix on inference):
// once M reaches the hundreds, the weight is cheaper to rebuild into memory once (cc::launch_layer_weight)
// and multiply with the vendor's tuned GEMM than to gather codebook rows again for every tile of x.
// The GEMM library (hipBLASLt) is opened at run time: a process that already holds a copy (PyTorch ships one)
// keeps using that copy, any other gets the ROCm installation's. Nothing here is needed by the clustering path.
#include <dlfcn.h>
#include <hipblaslt/hipblaslt.h>

#include <map>
#include <mutex>
#include <tuple>

#include "common.h"

namespace cc {
namespace {

struct Lt {
    bool ok = false;
    decltype(&hipblasLtCreate) Create = nullptr;
    decltype(&hipblasLtMatmulDescCreate) DescCreate = nullptr;
    decltype(&hipblasLtMatmulDescSetAttribute) DescSet = nullptr;
    decltype(&hipblasLtMatrixLayoutCreate) LayoutCreate = nullptr;
    decltype(&hipblasLtMatmulPreferenceCreate) PrefCreate = nullptr;
    decltype(&hipblasLtMatmulPreferenceSetAttribute) PrefSet = nullptr;
    decltype(&hipblasLtMatmulPreferenceDestroy) PrefDestroy = nullptr;
    decltype(&hipblasLtMatmulAlgoGetHeuristic) Heuristic = nullptr;
    decltype(&hipblasLtMatmul) Matmul = nullptr;
};

template <typename F>
bool bind(void* so, const char* name, F& fn)
{
    fn = reinterpret_cast<F>(dlsym(so, name));
    return fn != nullptr;
}

const Lt& lt()
{
    static Lt L;
    static std::once_flag once;
    std::call_once(once, [] {
        const char* soname = "libhipblaslt.so.1";
        void* so = dlopen(soname, RTLD_NOW | RTLD_NOLOAD);  // the copy this process already runs, if any
        if (!so) so = dlopen(soname, RTLD_NOW | RTLD_LOCAL);
        if (!so) return;
        L.ok = bind(so, "hipblasLtCreate", L.Create) && bind(so, "hipblasLtMatmulDescCreate", L.DescCreate) &&
               bind(so, "hipblasLtMatmulDescSetAttribute", L.DescSet) &&
               bind(so, "hipblasLtMatrixLayoutCreate", L.LayoutCreate) &&
               bind(so, "hipblasLtMatmulPreferenceCreate", L.PrefCreate) &&
               bind(so, "hipblasLtMatmulPreferenceSetAttribute", L.PrefSet) &&
               bind(so, "hipblasLtMatmulPreferenceDestroy", L.PrefDestroy) &&
               bind(so, "hipblasLtMatmulAlgoGetHeuristic", L.Heuristic) && bind(so, "hipblasLtMatmul", L.Matmul);
    });
    return L;
}

// One plan per (device, shape, dtype, bias): descriptors and the chosen algorithm are kept for the life of
// the process (a model has a handful of layer shapes).
struct Plan {
    bool valid = false;
    hipblasLtMatmulDesc_t desc = nullptr;
    hipblasLtMatrixLayout_t a = nullptr, b = nullptr, c = nullptr;
    hipblasLtMatmulAlgo_t algo;
    size_t scratch = 0;
    // every candidate of the library's heuristic that fits the scratch buffer, for tune_dense_forward
    static constexpr int kAsk = 16;
    hipblasLtMatmulHeuristicResult_t candidates[kAsk];
    int n_candidates = 0;
};

using Key = std::tuple<int, uint32_t, uint32_t, uint32_t, int, bool, bool>;
std::mutex g_mutex;
std::map<int, hipblasLtHandle_t> g_handles;
std::map<Key, Plan> g_plans;

Plan make_plan(const Lt& L, hipblasLtHandle_t h, uint32_t M, uint32_t in_features, uint32_t out_features, int dtype,
               bool with_bias, bool f32_out)
{
    Plan p;
    const hipDataType t = dtype == 1 ? HIP_R_16F : HIP_R_16BF;
    if (L.DescCreate(&p.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F) != HIPBLAS_STATUS_SUCCESS) return p;
    if (with_bias) {
        const uint32_t epilogue = HIPBLASLT_EPILOGUE_BIAS;
        const int32_t bias_type = int32_t(t);
        if (L.DescSet(p.desc, HIPBLASLT_MATMUL_DESC_EPILOGUE, &epilogue, sizeof(epilogue)) != HIPBLAS_STATUS_SUCCESS ||
            L.DescSet(p.desc, HIPBLASLT_MATMUL_DESC_BIAS_DATA_TYPE, &bias_type, sizeof(bias_type)) != HIPBLAS_STATUS_SUCCESS)
            return p;
    }
    // Row-major y [M][out] = x [M][in] . W [in][out] is, read column-major, y^T (out x M) = W^T (out x in) . x^T (in x M).
    if (L.LayoutCreate(&p.a, t, out_features, in_features, out_features) != HIPBLAS_STATUS_SUCCESS ||
        L.LayoutCreate(&p.b, t, in_features, M, in_features) != HIPBLAS_STATUS_SUCCESS ||
        L.LayoutCreate(&p.c, f32_out ? HIP_R_32F : t, out_features, M, out_features) != HIPBLAS_STATUS_SUCCESS)
        return p;
    hipblasLtMatmulPreference_t pref = nullptr;
    if (L.PrefCreate(&pref) != HIPBLAS_STATUS_SUCCESS) return p;
    const uint64_t max_scratch = kDenseScratchBytes;
    // the library's first choice may ask for more scratch than the preference allows: take the first that fits
    constexpr int kAsk = Plan::kAsk;
    hipblasLtMatmulHeuristicResult_t found[kAsk];
    int n_found = 0;
    if (L.PrefSet(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &max_scratch, sizeof(max_scratch)) == HIPBLAS_STATUS_SUCCESS &&
        L.Heuristic(h, p.desc, p.a, p.b, p.c, p.c, pref, kAsk, found, &n_found) == HIPBLAS_STATUS_SUCCESS) {
        for (int i = 0; i < n_found; ++i) {
            if (found[i].state != HIPBLAS_STATUS_SUCCESS || found[i].workspaceSize > kDenseScratchBytes) continue;
            p.candidates[p.n_candidates++] = found[i];
            if (p.valid) continue;
            p.algo = found[i].algo;
            p.scratch = found[i].workspaceSize;
            p.valid = true;
        }
    }
    L.PrefDestroy(pref);
    return p;
}

}  // namespace

bool dense_available() { return lt().ok; }

// y = x . W (+ bias) with W [in][out] already in memory in the same 16-bit dtype; with f32_out, y holds the fp32
// sums themselves (no bias then). Returns hipErrorNotSupported when the library has no algorithm for the shape
// (the caller then takes the fused kernel); `scratch` has kDenseScratchBytes bytes.
// (call with g_mutex held) the handle of the current device and the plan of this product; nullptr if there is none
static hipError_t find_plan(const Lt& L, uint32_t M, uint32_t in_features, uint32_t out_features, int dtype, bool with_bias,
                            bool f32_out, hipblasLtHandle_t& handle, Plan*& plan)
{
    int device = 0;
    if (hipError_t e = hipGetDevice(&device); e != hipSuccess) return e;
    hipblasLtHandle_t& h = g_handles[device];
    if (!h && L.Create(&h) != HIPBLAS_STATUS_SUCCESS) {
        h = nullptr;
        return hipErrorNotSupported;
    }
    const Key key{device, M, in_features, out_features, dtype, with_bias, f32_out};
    auto it = g_plans.find(key);
    if (it == g_plans.end()) it = g_plans.emplace(key, make_plan(L, h, M, in_features, out_features, dtype, with_bias, f32_out)).first;
    if (!it->second.valid) return hipErrorNotSupported;
    handle = h;
    plan = &it->second;
    return hipSuccess;
}

hipError_t launch_dense_forward(const void* x, uint32_t M, const void* weight, int dtype, uint32_t in_features,
                                uint32_t out_features, const void* bias, void* y, bool f32_out, void* scratch, hipStream_t s)
{
    if (f32_out && bias) return hipErrorInvalidValue;
    const Lt& L = lt();
    if (!L.ok) return hipErrorNotSupported;
    std::lock_guard<std::mutex> lock(g_mutex);
    hipblasLtHandle_t h = nullptr;
    Plan* p = nullptr;
    if (hipError_t e = find_plan(L, M, in_features, out_features, dtype, bias != nullptr, f32_out, h, p); e != hipSuccess) return e;
    if (bias && L.DescSet(p->desc, HIPBLASLT_MATMUL_DESC_BIAS_POINTER, &bias, sizeof(bias)) != HIPBLAS_STATUS_SUCCESS)
        return hipErrorNotSupported;
    const float one = 1.0f, zero = 0.0f;
    const hipblasStatus_t st = L.Matmul(h, p->desc, &one, weight, p->a, x, p->b, &zero, y, p->c, y, p->c, &p->algo, scratch,
                                        p->scratch, s);
    return st == HIPBLAS_STATUS_SUCCESS ? hipSuccess : hipErrorLaunchFailure;
}

namespace {
// finite, varied 16-bit floats in either format (0x3c00..0x3cff: around 1 in fp16, around 0.008 in bf16)
__global__ __launch_bounds__(256) void fill_operand_kernel(uint16_t* __restrict__ p, size_t n)
{
    for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += size_t(gridDim.x) * 256)
        p[i] = uint16_t(0x3c00u | ((uint32_t(i) * 2654435761u) >> 24));
}
}  // namespace

hipError_t launch_fill_operand(void* p, size_t n16, hipStream_t s)
{
    if (n16 == 0) return hipSuccess;
    const size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(fill_operand_kernel, dim3(uint32_t(blocks < 4096 ? blocks : 4096)), dim3(256), 0, s,
                       static_cast<uint16_t*>(p), n16);
    return hipGetLastError();
}

// Times every candidate algorithm of this product on the given (arbitrary) operands and keeps the fastest for later
// launch_dense_forward calls. Synchronises the stream several times. `kept_us` / `first_us`: the chosen
// algorithm's time and that of the library's own first choice.
hipError_t tune_dense_forward(const void* x, uint32_t M, const void* weight, int dtype, uint32_t in_features,
                              uint32_t out_features, const void* bias, void* y, bool f32_out, void* scratch, hipStream_t s,
                              float* kept_us, float* first_us)
{
    if (f32_out && bias) return hipErrorInvalidValue;
    const Lt& L = lt();
    if (!L.ok) return hipErrorNotSupported;
    std::lock_guard<std::mutex> lock(g_mutex);
    hipblasLtHandle_t h = nullptr;
    Plan* p = nullptr;
    if (hipError_t e = find_plan(L, M, in_features, out_features, dtype, bias != nullptr, f32_out, h, p); e != hipSuccess) return e;
    if (bias && L.DescSet(p->desc, HIPBLASLT_MATMUL_DESC_BIAS_POINTER, &bias, sizeof(bias)) != HIPBLAS_STATUS_SUCCESS)
        return hipErrorNotSupported;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    if (hipError_t e = hipEventCreate(&t0); e != hipSuccess) return e;
    if (hipError_t e = hipEventCreate(&t1); e != hipSuccess) {
        (void)hipEventDestroy(t0);
        return e;
    }
    const float one = 1.0f, zero = 0.0f;
    hipError_t err = hipSuccess;
    float best = 3.0e38f;
    int best_c = -1;
    for (int c = 0; c < p->n_candidates && err == hipSuccess; ++c) {
        const hipblasLtMatmulHeuristicResult_t& cand = p->candidates[c];
        float fastest = 3.0e38f;
        for (int rep = 0; rep < 4 && err == hipSuccess; ++rep) {  // the first run warms up
            if ((err = hipEventRecord(t0, s)) != hipSuccess) break;
            if (L.Matmul(h, p->desc, &one, weight, p->a, x, p->b, &zero, y, p->c, y, p->c, &cand.algo, scratch,
                         cand.workspaceSize, s) != HIPBLAS_STATUS_SUCCESS) {
                fastest = 3.0e38f;  // a candidate that does not run is simply not chosen
                break;
            }
            if ((err = hipEventRecord(t1, s)) != hipSuccess) break;
            if ((err = hipEventSynchronize(t1)) != hipSuccess) break;
            float ms = 0.0f;
            if ((err = hipEventElapsedTime(&ms, t0, t1)) != hipSuccess) break;
            if (rep > 0 && ms < fastest) fastest = ms;
        }
        if (c == 0 && first_us) *first_us = fastest * 1e3f;
        if (fastest < best) {
            best = fastest;
            best_c = c;
        }
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (err != hipSuccess) return err;
    if (best_c < 0) return hipErrorNotSupported;
    p->algo = p->candidates[best_c].algo;
    p->scratch = p->candidates[best_c].workspaceSize;
    if (kept_us) *kept_us = best * 1e3f;
    return hipSuccess;
}

}  // namespace cc
