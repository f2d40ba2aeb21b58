// Runtime of the host-side bounds model: runs the library's kernels (compiled as CPU code through hip_cpu_shim.h)
// workgroup by workgroup and thread by thread, with every tensor of a call placed against an inaccessible guard
// page, and reports the first access that leaves a tensor.  TEST INFRASTRUCTURE, never part of the product library.
#include "hip_cpu_shim.h"

#include <setjmp.h>
#include <signal.h>
#include <stdio.h>
#include <sys/mman.h>
#include <unistd.h>

#include <vector>

#include "../../include/conv1d.h"
#include "conv1d_internal.h"  // (this file is compiled from a copy that sits beside the kernels' sources)

namespace hostmodel {

thread_local Idx g_thread, g_block, g_grid, g_bdim;

namespace {
const size_t kPage = 4096;
// inaccessible address space on either side of every tensor: a wrong sample or row index lands megabytes away
const size_t kGuard = size_t(1) << 28;
struct Region {
    char* map = nullptr;
    size_t map_bytes = 0;
    char* data = nullptr;
    size_t bytes = 0;
    const char* name = "";
};
std::vector<Region> g_regions;
Region g_lds;
sigjmp_buf g_jump;
volatile sig_atomic_t g_armed = 0;
void* volatile g_fault_addr = nullptr;

// [guard zone][pages for `bytes`][guard zone]; the data ends at the trailing guard (end_aligned: up to 15 bytes of
// slack keep the 16-byte alignment the fast kernels ask for) or starts right behind the leading one
Region make_region(size_t bytes, bool end_aligned, const char* name) {
    Region r;
    r.name = name;
    r.bytes = bytes;
    const size_t body = (bytes + kPage - 1) / kPage * kPage + (bytes == 0 ? kPage : 0);
    r.map_bytes = body + 2 * kGuard;
    r.map = static_cast<char*>(mmap(nullptr, r.map_bytes, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0));
    if (r.map == MAP_FAILED) {
        r.map = nullptr;
        return r;
    }
    mprotect(r.map + kGuard, body, PROT_READ | PROT_WRITE);
    r.data = end_aligned ? r.map + kGuard + ((body - bytes) & ~static_cast<size_t>(15)) : r.map + kGuard;
    return r;
}
void free_region(Region& r) {
    if (r.map) munmap(r.map, r.map_bytes);
    r = Region{};
}

void on_fault(int, siginfo_t* info, void*) {
    if (!g_armed) _exit(139);
    g_fault_addr = info->si_addr;
    siglongjmp(g_jump, 1);
}
}  // namespace

void* dynamic_lds() { return g_lds.data; }

void run_grid(dim3 grid, dim3 block, size_t lds_bytes, const std::function<void()>& fn) {
    free_region(g_lds);
    g_lds = make_region(lds_bytes, true, "dynamic LDS");
    g_grid = Idx{grid.x, grid.y, grid.z};
    g_bdim = Idx{block.x, block.y, block.z};
    for (unsigned by = 0; by < grid.y; ++by)
        for (unsigned bx = 0; bx < grid.x; ++bx) {
            g_block = Idx{bx, by, 0};
            for (unsigned t = 0; t < block.x; ++t) {
                g_thread = Idx{t, 0, 0};
                fn();
            }
        }
}

}  // namespace hostmodel

using namespace hostmodel;

// pass: 0 conv1d_fwd, 1 conv1d_bwd_data, 2 conv1d_bwd_weight, 3 conv1d_bwd, 4 conv1d_fwd_ex (bias, ReLU, bfloat16 output
// when dtype is bfloat16), 5 conv1d_bwd_data_ex (bfloat16 output).  placement: 0 tensors end at a guard page, 1 tensors
// start behind one, 2 as 0 with every tensor shifted by one element (the element-aligned paths).
// Returns 0 (every access inside its tensor), 1 (an access left its tensor; msg says where), or 100 - status when the
// library refused the call.
extern "C" int hostmodel_run(int pass, int N, int C, int K, int W, int S, int d, int P, int dtype, int variant, int placement,
                             char* msg, int msglen) {
    const long Q = static_cast<long>(W) + 2L * P - static_cast<long>(S - 1) * d;
    if (Q < 1) return 100 - CONV1D_EINVAL;
    const size_t e = dtype == CONV1D_BF16 ? 2 : 4;
    const bool out16 = dtype == CONV1D_BF16 && (pass == 4 || pass == 5);
    const size_t shift = placement == 2 ? 1 : 0;
    const bool end_aligned = placement != 1;
    const size_t nx = static_cast<size_t>(N) * C * W, ny = static_cast<size_t>(N) * K * Q, nw = static_cast<size_t>(K) * C * S;
    for (auto& r : g_regions) free_region(r);
    g_regions.clear();
    auto tensor = [&](size_t elems, size_t esize, const char* name) -> char* {
        // a bfloat16 tensor may be read up to its next 4-byte boundary (include/conv1d.h)
        const size_t bytes = ((elems + shift) * esize + 3) & ~static_cast<size_t>(3);
        g_regions.push_back(make_region(bytes, end_aligned, name));
        return g_regions.back().data;
    };
    char* x = tensor(nx, e, "x");
    char* w = tensor(nw, e, "w");
    char* dy = tensor(ny, e, "dy");
    char* y = tensor(ny, out16 ? 2 : 4, "y");
    char* dx = tensor(nx, out16 ? 2 : 4, "dx");
    char* dw = tensor(nw, 4, "dw");
    char* bias = tensor(K, 4, "bias");
    const size_t wsb = conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, d, P, dtype);
    g_regions.push_back(make_region(wsb + 256, false, "workspace"));
    char* ws = g_regions.back().data;
    if (shift) {  // one element into each allocation: only element alignment is left
        x += e; w += e; dy += e; y += out16 ? 2 : 4; dx += out16 ? 2 : 4; dw += 4;
    }
    struct sigaction sa, old_segv, old_bus;
    memset(&sa, 0, sizeof(sa));
    sa.sa_sigaction = on_fault;
    sa.sa_flags = SA_SIGINFO | SA_NODEFER;
    sigaction(SIGSEGV, &sa, &old_segv);
    sigaction(SIGBUS, &sa, &old_bus);
    conv1d_set_variant(variant);
    int rc;
    if (sigsetjmp(g_jump, 1) == 0) {
        g_armed = 1;
        int st = CONV1D_OK;
        switch (pass) {
            case 0: st = conv1d_fwd(x, w, reinterpret_cast<float*>(y), N, C, K, W, S, d, P, dtype, nullptr); break;
            case 1: st = conv1d_bwd_data(dy, w, reinterpret_cast<float*>(dx), N, C, K, W, S, d, P, dtype, nullptr); break;
            case 2: st = conv1d_bwd_weight(x, dy, reinterpret_cast<float*>(dw), ws, wsb, N, C, K, W, S, d, P, dtype, nullptr); break;
            case 3: st = conv1d_bwd(x, dy, w, reinterpret_cast<float*>(dx), reinterpret_cast<float*>(dw), ws, wsb, N, C, K, W, S, d, P, dtype, nullptr); break;
            case 4: st = conv1d_fwd_ex(x, w, reinterpret_cast<float*>(bias), y, N, C, K, W, S, d, P, dtype,
                                       CONV1D_EPI_RELU | (out16 ? CONV1D_EPI_OUT_BF16 : 0), nullptr); break;
            case 5: st = conv1d_bwd_data_ex(dy, w, dx, N, C, K, W, S, d, P, dtype, out16 ? CONV1D_EPI_OUT_BF16 : 0, nullptr); break;
            default: st = CONV1D_EINVAL;
        }
        g_armed = 0;
        rc = st == CONV1D_OK ? 0 : 100 - st;
    } else {
        g_armed = 0;
        const char* fa = static_cast<const char*>(g_fault_addr);
        const char* where = "no tensor of this call";
        long off = 0;
        for (const auto& r : g_regions)
            if (fa >= r.map && fa < r.map + r.map_bytes) {
                where = r.name;
                off = fa - r.data;
            }
        if (g_lds.map && fa >= g_lds.map && fa < g_lds.map + g_lds.map_bytes) {
            where = g_lds.name;
            off = fa - g_lds.data;
        }
        if (msg && msglen > 0)
            snprintf(msg, msglen, "access outside %s (address %p, byte offset %ld from its start) by workgroup (%u,%u) thread %u of a kernel of pass %d",
                     where, static_cast<const void*>(fa), off, g_block.x, g_block.y, g_thread.x, pass);
        rc = 1;
    }
    conv1d_set_variant(0);
    sigaction(SIGSEGV, &old_segv, nullptr);
    sigaction(SIGBUS, &old_bus, nullptr);
    return rc;
}

extern "C" const char* hostmodel_kernel_name(int pass, int N, int C, int K, int W, int S, int d, int P, int dtype) {
    return conv1d_kernel_name(pass, N, C, K, W, S, d, P, dtype);
}

// The multiply-high division of the kernels against the plain one: the first n <= nmax whose quotient differs, -1 if
// none does, -2 if make_fastdiv refuses the pair (it must refuse every pair for which the quotient could be wrong).
extern "C" long hostmodel_fastdiv_mismatch(long d, long nmax) {
    conv1d::FastDiv f;
    if (!conv1d::make_fastdiv(f, d, nmax)) return -2;
    for (long n = 0; n <= nmax; ++n)
        if (conv1d::fast_div(static_cast<int>(n), f) != static_cast<int>(n / d)) return n;
    return -1;
}
