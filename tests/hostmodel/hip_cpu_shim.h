// A minimal stand-in for the HIP runtime and the gfx950 builtins, so that the library's kernels compile as plain
// host C++ and run one thread after the other on the CPU.  TEST INFRASTRUCTURE: it exists to check, without a GPU,
// that every global-memory address a kernel forms lies inside its tensor (the tensors of the model sit against
// inaccessible guard pages, see model.cpp).  Data values are not modelled faithfully: matrix instructions return
// their accumulator, barriers do nothing, so what a thread reads from LDS is whatever the threads before it left.
// That is enough because no kernel derives an address or a branch from data.
#pragma once
#define HIP_INCLUDE_HIP_HIP_RUNTIME_H  // keeps <hip/hip_runtime.h> out
#define HOSTMODEL 1

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <functional>

struct dim3 {
    unsigned x, y, z;
    constexpr dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
typedef void* hipStream_t;
typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorInvalidDevice = 101, hipErrorInvalidSymbol = 13 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __shared__ static
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x

namespace hostmodel {
struct Idx { unsigned x, y, z; };
extern thread_local Idx g_thread, g_block, g_grid, g_bdim;
// the dynamic LDS of the workgroup that is running (sized as the launch asked, against a guard page)
void* dynamic_lds();
// runs fn once per (block, thread) with the index variables set
void run_grid(dim3 grid, dim3 block, size_t lds_bytes, const std::function<void()>& fn);
}  // namespace hostmodel
#define threadIdx (hostmodel::g_thread)
#define blockIdx (hostmodel::g_block)
#define gridDim (hostmodel::g_grid)
#define blockDim (hostmodel::g_bdim)

inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
inline hipError_t hipGetSymbolAddress(void** p, const void* sym) { *p = const_cast<void*>(sym); return hipSuccess; }

inline void __syncthreads() {}
inline float __uint_as_float(unsigned u) { float f; std::memcpy(&f, &u, 4); return f; }
inline unsigned __float_as_uint(float f) { unsigned u; std::memcpy(&u, &f, 4); return u; }
inline float __shfl_down(float v, int, int) { return v; }
inline unsigned __umulhi(unsigned a, unsigned b) { return static_cast<unsigned>((static_cast<unsigned long long>(a) * b) >> 32); }
inline int min(int a, int b) { return a < b ? a : b; }
inline int max(int a, int b) { return a > b ? a : b; }
inline unsigned min(unsigned a, unsigned b) { return a < b ? a : b; }
inline unsigned max(unsigned a, unsigned b) { return a > b ? a : b; }
inline long min(long a, long b) { return a < b ? a : b; }
inline long max(long a, long b) { return a > b ? a : b; }

#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_sched_group_barrier(a, b, c) ((void)0)
#define __builtin_amdgcn_s_setprio(x) ((void)0)
#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, x, y, z) (c)
#define __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, x, y, z) (c)
inline unsigned hostmodel_perm(unsigned hi, unsigned lo, unsigned sel) {
    const uint64_t v = (static_cast<uint64_t>(hi) << 32) | lo;
    unsigned r = 0;
    for (int i = 0; i < 4; ++i) {
        const unsigned s = (sel >> (8 * i)) & 0xff;
        const unsigned byte = s < 8 ? static_cast<unsigned>((v >> (8 * s)) & 0xff) : 0u;
        r |= byte << (8 * i);
    }
    return r;
}
#define __builtin_amdgcn_perm(a, b, s) hostmodel_perm(a, b, s)
inline unsigned hostmodel_alignbit(unsigned hi, unsigned lo, unsigned sh) {
    return static_cast<unsigned>(((static_cast<uint64_t>(hi) << 32) | lo) >> (sh & 31));
}
#define __builtin_amdgcn_alignbit(a, b, s) hostmodel_alignbit(a, b, s)

// raw buffer loads: the descriptor is the base address, the load an ordinary (guard-checked) read
struct hostmodel_rsrc {
    const char* base;
};
#define __amdgpu_buffer_rsrc_t hostmodel_rsrc
inline hostmodel_rsrc hostmodel_make_rsrc(const void* p) { return hostmodel_rsrc{static_cast<const char*>(p)}; }
#define __builtin_amdgcn_make_buffer_rsrc(p, stride, num, flags) hostmodel_make_rsrc(p)
inline unsigned hostmodel_buffer_load_b32(hostmodel_rsrc r, int voff, int soff) {
    unsigned v;
    std::memcpy(&v, r.base + static_cast<long>(voff) + static_cast<long>(soff), 4);
    return v;
}
#define __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, aux) hostmodel_buffer_load_b32(r, voff, soff)
typedef __attribute__((ext_vector_type(4))) unsigned int hostmodel_u32x4;
inline hostmodel_u32x4 hostmodel_buffer_load_b128(hostmodel_rsrc r, int voff, int soff) {
    hostmodel_u32x4 v;
    std::memcpy(&v, r.base + static_cast<long>(static_cast<unsigned>(voff)) + static_cast<long>(soff), 16);
    return v;
}
#define __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, aux) hostmodel_buffer_load_b128(r, voff, soff)
inline unsigned short hostmodel_buffer_load_b16(hostmodel_rsrc r, int voff, int soff) {
    unsigned short v;
    std::memcpy(&v, r.base + static_cast<long>(static_cast<unsigned>(voff)) + static_cast<long>(soff), 2);
    return v;
}
#define __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, aux) hostmodel_buffer_load_b16(r, voff, soff)

// launch_kernel() in conv1d_internal.h calls this instead of hipLaunchKernel when HOSTMODEL is defined
template <typename... Params, typename... Args>
inline hipError_t hostmodel_launch(void (*kern)(Params...), dim3 grid, dim3 block, size_t lds_bytes, const Args&... args) {
    hostmodel::run_grid(grid, block, lds_bytes, [&] { kern(static_cast<Params>(args)...); });
    return hipSuccess;
}
