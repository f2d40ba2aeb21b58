// C ABI of the conv1d library: argument validation, kernel-family dispatch, status strings.
// Every entry point only enqueues kernels on the caller's stream.
#include <atomic>
#include <mutex>
#include <unordered_map>

#include "conv1d_internal.h"

using namespace conv1d;

namespace conv1d {

hipError_t ensure_dynamic_lds(const void* kern, size_t bytes) {
    static std::mutex mutex;
    static std::unordered_map<uintptr_t, size_t> granted;  // key: kernel address mixed with the GPU's index
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uintptr_t key = reinterpret_cast<uintptr_t>(kern) ^ (static_cast<uintptr_t>(dev + 1) << 56);
    std::lock_guard<std::mutex> lock(mutex);
    auto it = granted.find(key);
    if (it != granted.end() && it->second >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
    if (e == hipSuccess) granted[key] = bytes;
    return e;
}

}  // namespace conv1d

// Partial sums of conv1d_bwd_weight_noalloc: one array per GPU the library runs on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[CONV1D_NOALLOC_SCRATCH_BYTES];

namespace {

std::atomic<int> g_variant{CONV1D_VARIANT_AUTO};

// device address of `scratch` on each GPU, looked up on the first call with that GPU current
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_for_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

struct Geom {
    int N, C, K, W, S, d, P, Q;
};

bool make_geom(int N, int C, int K, int W, int S, int d, int P, Geom* g) {
    if (N < 1 || C < 1 || K < 1 || W < 1 || S < 1 || d < 1 || P < 0) return false;
    const long Q = static_cast<long>(W) + 2L * P - static_cast<long>(S - 1) * d;
    if (Q < 1 || Q > 0x7fffffffL) return false;
    // every tensor must be addressable with the 32-bit row arithmetic of the tiled kernels' hosts
    // (element offsets themselves are 64-bit inside the kernels)
    *g = Geom{N, C, K, W, S, d, P, static_cast<int>(Q)};
    return true;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

CorrProblem fwd_problem(const Geom& g, const void* x, const void* w, float* y, int bf16) {
    CorrProblem p{};
    p.in = x; p.wt = w; p.out = y;
    p.N = g.N; p.R = g.C; p.M = g.K; p.Win = g.W; p.Wout = g.Q; p.S = g.S; p.d = g.d; p.P = g.P;
    p.w_sm = static_cast<long>(g.C) * g.S; p.w_sr = g.S; p.w_s0 = 0; p.w_ss = 1;
    p.bf16 = bf16;
    p.in_sn = static_cast<long>(p.R) * p.Win; p.out_sn = static_cast<long>(p.M) * p.Wout; p.accumulate = 0; p.w_contig = 1;
    return p;
}

// Section 3.2: the same contraction over dy with C and K swapped, taps reversed, P' = (S-1)d - P.
CorrProblem bwd_data_problem(const Geom& g, const void* dy, const void* w, float* dx, int bf16) {
    CorrProblem p{};
    p.in = dy; p.wt = w; p.out = dx;
    p.N = g.N; p.R = g.K; p.M = g.C; p.Win = g.Q; p.Wout = g.W; p.S = g.S; p.d = g.d;
    p.P = (g.S - 1) * g.d - g.P;
    p.w_sm = g.S; p.w_sr = static_cast<long>(g.C) * g.S; p.w_s0 = g.S - 1; p.w_ss = -1;
    p.bf16 = bf16;
    p.in_sn = static_cast<long>(p.R) * p.Win; p.out_sn = static_cast<long>(p.M) * p.Wout; p.accumulate = 0; p.w_contig = 1;
    return p;
}

WgradProblem wgrad_problem(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t wsb, int bf16) {
    WgradProblem p{};
    p.x = x; p.dy = dy; p.dw = dw; p.ws = ws; p.ws_bytes = wsb;
    p.N = g.N; p.C = g.C; p.K = g.K; p.W = g.W; p.Q = g.Q; p.S = g.S; p.d = g.d; p.P = g.P;
    p.bf16 = bf16;
    p.x_sn = static_cast<long>(g.C) * g.W; p.dy_sn = static_cast<long>(g.K) * g.Q;
    p.dw_sk = static_cast<long>(g.C) * g.S; p.dw_sc = g.S;
    return p;
}

// Which family runs a correlation problem under the current variant setting (-1: none).
int pick_corr(const CorrProblem& p) {
    const int v = g_variant.load(std::memory_order_relaxed);
    switch (v) {
        case CONV1D_VARIANT_GENERIC: return CONV1D_VARIANT_GENERIC;
        case CONV1D_VARIANT_SMALLC: return smallc_corr_supported(p) ? v : -1;
        case CONV1D_VARIANT_IGEMM: return igemm_corr_supported(p) ? v : -1;
        default: break;
    }
    if (smallc_corr_supported(p)) return CONV1D_VARIANT_SMALLC;
    if (igemm_corr_supported(p)) return CONV1D_VARIANT_IGEMM;
    return CONV1D_VARIANT_GENERIC;
}

int pick_wgrad(const WgradProblem& p) {
    const int v = g_variant.load(std::memory_order_relaxed);
    switch (v) {
        case CONV1D_VARIANT_GENERIC: return CONV1D_VARIANT_GENERIC;
        case CONV1D_VARIANT_SMALLC: return smallc_wgrad_supported(p) ? v : -1;
        case CONV1D_VARIANT_IGEMM: return igemm_wgrad_supported(p) ? v : -1;
        default: break;
    }
    if (smallc_wgrad_supported(p)) return CONV1D_VARIANT_SMALLC;
    if (igemm_wgrad_supported(p)) return CONV1D_VARIANT_IGEMM;
    return CONV1D_VARIANT_GENERIC;
}

int run_corr(const CorrProblem& p, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (pick_corr(p)) {
        case CONV1D_VARIANT_GENERIC: e = generic_corr_launch(p, st); break;
        case CONV1D_VARIANT_SMALLC: e = smallc_corr_launch(p, st); break;
        case CONV1D_VARIANT_IGEMM: e = igemm_corr_launch(p, st); break;
        default: return CONV1D_EUNSUPPORTED;
    }
    if (e == hipErrorInvalidValue) return CONV1D_EUNSUPPORTED;
    return e == hipSuccess ? CONV1D_OK : CONV1D_EHIP;
}

int run_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t wsb, int dtype, void* stream) {
    WgradProblem p = wgrad_problem(g, x, dy, dw, ws, wsb, dtype == CONV1D_BF16);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (pick_wgrad(p)) {
        case CONV1D_VARIANT_GENERIC: e = generic_wgrad_launch(p, st); break;
        case CONV1D_VARIANT_SMALLC: e = smallc_wgrad_launch(p, st); break;
        case CONV1D_VARIANT_IGEMM: e = igemm_wgrad_launch(p, st); break;
        default: return CONV1D_EUNSUPPORTED;
    }
    if (e == hipErrorInvalidValue) return CONV1D_EUNSUPPORTED;
    return e == hipSuccess ? CONV1D_OK : CONV1D_EHIP;
}

const char* family_name(int fam, int bf16, bool wgrad) {
    switch (fam) {
        case CONV1D_VARIANT_GENERIC: return bf16 ? (wgrad ? "generic_wgrad_bf16" : "generic_fma_bf16") : (wgrad ? "generic_wgrad_fp32" : "generic_fma_fp32");
        case CONV1D_VARIANT_SMALLC: return bf16 ? (wgrad ? "smallc_wgrad_mfma_bf16" : "smallc_mfma_bf16") : (wgrad ? "smallc_wgrad_mfma_fp32" : "smallc_mfma_fp32");
        case CONV1D_VARIANT_IGEMM: return bf16 ? (wgrad ? "igemm_wgrad_mfma_bf16" : "igemm_mfma_bf16") : (wgrad ? "igemm_wgrad_mfma_fp32" : "igemm_mfma_fp32");
        default: return "unsupported";
    }
}

}  // namespace

extern "C" {

int conv1d_out_width(int W, int S, int dilation, int padding) {
    Geom g;
    if (!make_geom(1, 1, 1, W, S, dilation, padding, &g)) {
        const long Q = static_cast<long>(W) + 2L * padding - static_cast<long>(S - 1) * dilation;
        return Q < 0 ? static_cast<int>(Q < -0x7fffffffL ? -0x7fffffffL : Q) : 0;
    }
    return g.Q;
}

int conv1d_fwd(const void* x, const void* w, float* y, int N, int C, int K, int W, int S, int dilation,
               int padding, int dtype, void* stream) {
    return conv1d_fwd_ex(x, w, nullptr, y, N, C, K, W, S, dilation, padding, dtype, 0, stream);
}

int conv1d_fwd_ex(const void* x, const void* w, const float* bias, void* y, int N, int C, int K, int W, int S,
                  int dilation, int padding, int dtype, int flags, void* stream) {
    Geom g;
    if (!x || !w || !y || (dtype != CONV1D_FP32 && dtype != CONV1D_BF16)) return CONV1D_EINVAL;
    if (flags & ~(CONV1D_EPI_RELU | CONV1D_EPI_OUT_BF16)) return CONV1D_EINVAL;
    const bool out_bf16 = flags & CONV1D_EPI_OUT_BF16;
    if (out_bf16 && dtype != CONV1D_BF16) return CONV1D_EINVAL;
    if (!make_geom(N, C, K, W, S, dilation, padding, &g)) return CONV1D_EINVAL;
    const size_t ea = dtype == CONV1D_BF16 ? 2 : 4;
    if (!aligned(x, ea) || !aligned(w, ea) || !aligned(y, out_bf16 ? 2 : 4) || !aligned(bias, 4)) return CONV1D_EINVAL;
    CorrProblem p = fwd_problem(g, x, w, static_cast<float*>(y), dtype == CONV1D_BF16);
    p.epi = Epilogue{bias, (flags & CONV1D_EPI_RELU) ? 1 : 0, out_bf16 ? 1 : 0};
    return run_corr(p, stream);
}

int conv1d_bwd_data(const void* dy, const void* w, float* dx, int N, int C, int K, int W, int S, int dilation,
                    int padding, int dtype, void* stream) {
    return conv1d_bwd_data_ex(dy, w, dx, N, C, K, W, S, dilation, padding, dtype, 0, stream);
}

int conv1d_bwd_data_ex(const void* dy, const void* w, void* dx, int N, int C, int K, int W, int S, int dilation,
                       int padding, int dtype, int flags, void* stream) {
    Geom g;
    if (!dy || !w || !dx || (dtype != CONV1D_FP32 && dtype != CONV1D_BF16)) return CONV1D_EINVAL;
    if (flags & ~CONV1D_EPI_OUT_BF16) return CONV1D_EINVAL;  // a gradient has no bias and no ReLU of its own
    const bool out_bf16 = flags & CONV1D_EPI_OUT_BF16;
    if (out_bf16 && dtype != CONV1D_BF16) return CONV1D_EINVAL;
    if (!make_geom(N, C, K, W, S, dilation, padding, &g)) return CONV1D_EINVAL;
    const size_t ea = dtype == CONV1D_BF16 ? 2 : 4;
    if (!aligned(dy, ea) || !aligned(w, ea) || !aligned(dx, out_bf16 ? 2 : 4)) return CONV1D_EINVAL;
    CorrProblem p = bwd_data_problem(g, dy, w, static_cast<float*>(dx), dtype == CONV1D_BF16);
    p.epi = Epilogue{nullptr, 0, out_bf16 ? 1 : 0};
    return run_corr(p, stream);
}

size_t conv1d_bwd_weight_workspace_bytes(int N, int C, int K, int W, int S, int dilation, int padding, int dtype) {
    Geom g;
    if ((dtype != CONV1D_FP32 && dtype != CONV1D_BF16) || !make_geom(N, C, K, W, S, dilation, padding, &g)) return 0;
    WgradProblem p = wgrad_problem(g, nullptr, nullptr, nullptr, nullptr, 0, dtype == CONV1D_BF16);
    size_t need = generic_wgrad_workspace(p);
    if (smallc_wgrad_supported(p)) { size_t b = smallc_wgrad_workspace(p); if (b > need) need = b; }
    if (igemm_wgrad_supported(p)) { size_t b = igemm_wgrad_workspace(p); if (b > need) need = b; }
    return (need + 255) & ~static_cast<size_t>(255);
}

int conv1d_bwd_weight(const void* x, const void* dy, float* dw, void* workspace, size_t workspace_bytes, int N,
                      int C, int K, int W, int S, int dilation, int padding, int dtype, void* stream) {
    Geom g;
    if (!x || !dy || !dw || (dtype != CONV1D_FP32 && dtype != CONV1D_BF16)) return CONV1D_EINVAL;
    if (!make_geom(N, C, K, W, S, dilation, padding, &g)) return CONV1D_EINVAL;
    const size_t ea = dtype == CONV1D_BF16 ? 2 : 4;
    if (!aligned(x, ea) || !aligned(dy, ea) || !aligned(dw, 4)) return CONV1D_EINVAL;
    const size_t need = conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype);
    if (!workspace || workspace_bytes < need) return CONV1D_EWORKSPACE;
    if (!aligned(workspace, 256)) return CONV1D_EINVAL;
    return run_wgrad(g, x, dy, dw, workspace, workspace_bytes, dtype, stream);
}

size_t conv1d_bwd_workspace_bytes(int N, int C, int K, int W, int S, int dilation, int padding, int dtype) {
    return conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype);
}

int conv1d_bwd(const void* x, const void* dy, const void* w, float* dx, float* dw, void* workspace,
               size_t workspace_bytes, int N, int C, int K, int W, int S, int dilation, int padding, int dtype,
               void* stream) {
    Geom g;
    if (!x || !dy || !w || !dx || !dw || (dtype != CONV1D_FP32 && dtype != CONV1D_BF16)) return CONV1D_EINVAL;
    if (!make_geom(N, C, K, W, S, dilation, padding, &g)) return CONV1D_EINVAL;
    const size_t ea = dtype == CONV1D_BF16 ? 2 : 4;
    if (!aligned(x, ea) || !aligned(dy, ea) || !aligned(w, ea) || !aligned(dx, 4) || !aligned(dw, 4)) return CONV1D_EINVAL;
    const size_t need = conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype);
    if (!workspace || workspace_bytes < need) return CONV1D_EWORKSPACE;
    if (!aligned(workspace, 256)) return CONV1D_EINVAL;
    const int bf16 = dtype == CONV1D_BF16;
    CorrProblem cp = bwd_data_problem(g, dy, w, dx, bf16);
    WgradProblem wp = wgrad_problem(g, x, dy, dw, workspace, workspace_bytes, bf16);
    const int corr_family = pick_corr(cp), wgrad_family = pick_wgrad(wp);
    if (corr_family < 0 || wgrad_family < 0) return CONV1D_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Small-channel bf16 layers: the first stage of the weight gradient runs first, and the backward-data kernel that
    // follows adds up its partial tiles while it waits for its own first inputs (no second-stage launch).
    if (bf16 && corr_family == CONV1D_VARIANT_SMALLC && wgrad_family == CONV1D_VARIANT_SMALLC &&
        smallc_bf16_corr_grid(cp) >= 4 * g.S) {
        int nwg = 0;
        hipError_t e = smallc_bf16_wgrad_stage1_launch(wp, st, &nwg);
        if (e == hipErrorInvalidValue) return CONV1D_EUNSUPPORTED;
        if (e != hipSuccess) return CONV1D_EHIP;
        cp.tail = WgradTail{static_cast<const float*>(workspace), dw, g.K, g.C, g.S, nwg, wp.dw_sk, wp.dw_sc};
        return run_corr(cp, stream);
    }
    const int r = run_wgrad(g, x, dy, dw, workspace, workspace_bytes, dtype, stream);
    if (r != CONV1D_OK) return r;
    return run_corr(cp, stream);
}

int conv1d_bwd_weight_noalloc(const void* x, const void* dy, float* dw, int N, int C, int K, int W, int S,
                              int dilation, int padding, int dtype, void* stream) {
    Geom g;
    if (!x || !dy || !dw || (dtype != CONV1D_FP32 && dtype != CONV1D_BF16)) return CONV1D_EINVAL;
    if (!make_geom(N, C, K, W, S, dilation, padding, &g)) return CONV1D_EINVAL;
    const size_t ea = dtype == CONV1D_BF16 ? 2 : 4;
    if (!aligned(x, ea) || !aligned(dy, ea) || !aligned(dw, 4)) return CONV1D_EINVAL;
    const size_t need = conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype);
    if (need > CONV1D_NOALLOC_SCRATCH_BYTES) return CONV1D_ESCRATCH;
    void* ws = nullptr;
    if (scratch_for_current_device(&ws) != hipSuccess) return CONV1D_EHIP;
    // nothing has to start at zero: every kernel family writes each partial sum before its second stage reads it
    return run_wgrad(g, x, dy, dw, ws, CONV1D_NOALLOC_SCRATCH_BYTES, dtype, stream);
}
int conv1d_set_variant(int variant) {
    if (variant < CONV1D_VARIANT_AUTO || variant > CONV1D_VARIANT_IGEMM) return CONV1D_EINVAL;
    g_variant.store(variant, std::memory_order_relaxed);
    return CONV1D_OK;
}

const char* conv1d_kernel_name(int pass, int N, int C, int K, int W, int S, int dilation, int padding, int dtype) {
    Geom g;
    if ((dtype != CONV1D_FP32 && dtype != CONV1D_BF16) || !make_geom(N, C, K, W, S, dilation, padding, &g)) return "invalid";
    const int bf16 = dtype == CONV1D_BF16;
    switch (pass) {
        case CONV1D_PASS_FWD: return family_name(pick_corr(fwd_problem(g, nullptr, nullptr, nullptr, bf16)), bf16, false);
        case CONV1D_PASS_BWD_DATA: return family_name(pick_corr(bwd_data_problem(g, nullptr, nullptr, nullptr, bf16)), bf16, false);
        case CONV1D_PASS_BWD_WEIGHT: return family_name(pick_wgrad(wgrad_problem(g, nullptr, nullptr, nullptr, nullptr, 0, bf16)), bf16, true);
        default: return "invalid";
    }
}

const char* conv1d_status_string(int status) {
    switch (status) {
        case CONV1D_OK: return "ok";
        case CONV1D_EINVAL: return "invalid argument (null or misaligned pointer, bad size, dilation, padding or dtype)";
        case CONV1D_EUNSUPPORTED: return "geometry not supported by the selected kernel variant";
        case CONV1D_EWORKSPACE: return "workspace missing or too small";
        case CONV1D_EHIP: return "HIP runtime error on launch";
        case CONV1D_ESCRATCH: return "geometry needs more scratch than the library's built-in buffer (CONV1D_NOALLOC_SCRATCH_BYTES): use conv1d_bwd_weight with a workspace";
        default: return "unknown status";
    }
}

}  // extern "C"
