// Internal declarations shared by the HIP translation units of the conv1d library.
// Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "../../include/conv1d.h"

namespace conv1d {

// What happens to an output value between the accumulator and memory.  Section 3 leaves the bias to the framework
// and Section 4.4 follows the layer with a ReLU that stays in bfloat16; fused here, they cost no extra pass over the
// output: z = acc + bias[m]; z = max(z, 0) if relu; stored as float, or as bfloat16 (nearest, ties to even).
struct Epilogue {
    const float* bias;  // one value per output row m (filter); nullptr: none
    int relu;
    int out_bf16;       // the output tensor holds bfloat16 elements
};

// Second stage of a backward-weight pass whose first stage left one S x 16 x 16 partial tile per workgroup
// (ws[(g*S + s)*256 + k*16 + c]): dw[k][c][s] = sum over g, in a fixed order.  Either a kernel of its own, or a side
// job of the backward-data kernel that follows the first stage in a fused backward call (ws == nullptr: none).
struct WgradTail {
    const float* ws;
    float* dw;
    int K, C, S, nwg;
    long dw_sk, dw_sc;
};

// One "correlation problem": the forward pass and the backward-data pass are both
//   out[n][m][o] = sum_{r<R} sum_{s<S} in[n][r][o + s*d - P] * wt(m, r, s),   in = 0 outside [0, Win)
// The forward pass (Eq. 2) has in = x, R = C, M = K, P = padding and wt(m,r,s) = w[m][r][s].
// The backward-data pass (Section 3.2) is the same contraction over dy with the roles of C and K
// swapped, the taps reversed and P' = (S-1)*d - P:  wt(m,r,s) = w[r][m][S-1-s].
// Weight element (m, r, s) lives at wt[m*w_sm + r*w_sr + w_s0 + s*w_ss] (in elements).
struct CorrProblem {
    const void* in;
    const void* wt;
    float* out;
    int N, R, M, Win, Wout, S, d, P;  // P may be negative for bwd_data when padding > (S-1)*d
    long w_sm, w_sr;
    int w_s0, w_ss;
    int bf16;  // 0: float inputs, 1: bfloat16 inputs
    // A problem may be a channel block of a larger layer: rows r < R / m < M of samples that are in_sn / out_sn
    // elements apart (in_sn = R*Win, out_sn = M*Wout for a whole layer).  accumulate != 0 adds to `out`.
    long in_sn, out_sn;
    int accumulate;
    // != 0 when the M*R*S weights wt(m,r,s) are exactly the contiguous elements wt[0 .. M*R*S)
    int w_contig;
    // applied by the kernel that completes an output element; never combined with accumulate != 0
    Epilogue epi;
    // side job for the first 4*S workgroups of the small-channel bf16 kernel (fused backward); else ws == nullptr
    WgradTail tail;
};

// The backward-weight problem (Section 3.3):
//   dw[k][c][s] = sum_n sum_q x[n][c][q + s*d - P] * dy[n][k][q]
struct WgradProblem {
    const void* x;
    const void* dy;
    float* dw;
    void* ws;
    size_t ws_bytes;
    int N, C, K, W, Q, S, d, P;
    int bf16;
    // A problem may be a (filter block, channel block) of a larger layer: sample strides of x and dy in elements
    // (C*W and K*Q for a whole layer) and the strides of dw between filters and between channels (C*S and S).
    long x_sn, dy_sn, dw_sk, dw_sc;
};

// generic (plain FMA) family: any geometry
hipError_t generic_corr_launch(const CorrProblem& p, hipStream_t st);
// bias and ReLU of p.epi applied in place to a float output (after launches that accumulated into it)
hipError_t generic_epilogue_launch(const CorrProblem& p, hipStream_t st);
size_t generic_wgrad_workspace(const WgradProblem& p);
hipError_t generic_wgrad_launch(const WgradProblem& p, hipStream_t st);

// small-channel MFMA family: R, M <= 16 (C, K <= 16)
bool smallc_corr_supported(const CorrProblem& p);
hipError_t smallc_corr_launch(const CorrProblem& p, hipStream_t st);
bool smallc_wgrad_supported(const WgradProblem& p);
size_t smallc_wgrad_workspace(const WgradProblem& p);
hipError_t smallc_wgrad_launch(const WgradProblem& p, hipStream_t st);

// FP32 forward / backward-data with any R, M: filter blocks of 16 as rows of a single grid, channel blocks reduced
// inside the kernel (needs the weights of all channel blocks of a filter block in LDS)
bool smallc_corr_f32_blocks_supported(const CorrProblem& p);
hipError_t smallc_corr_f32_blocks_launch(const CorrProblem& p, hipStream_t st);

// FP32 backward-weight with any C, K: every 16 x 16 block pair as one row of a single grid, one second stage
size_t smallc_wgrad_f32_blocks_workspace(const WgradProblem& p);  // 0: not supported
hipError_t smallc_wgrad_f32_blocks_launch(const WgradProblem& p, hipStream_t st);

// bf16 members of the small-channel family (own translation unit)
bool smallc_bf16_corr_supported(const CorrProblem& p);
hipError_t smallc_bf16_corr_launch(const CorrProblem& p, hipStream_t st);
bool smallc_bf16_wgrad_supported(const WgradProblem& p);
size_t smallc_bf16_wgrad_workspace(const WgradProblem& p);
hipError_t smallc_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st);
// first stage only: *nwg receives the number of partial tiles it leaves in the workspace
hipError_t smallc_bf16_wgrad_stage1_launch(const WgradProblem& p, hipStream_t st, int* nwg);
// number of workgroups smallc_bf16_corr_launch would start for this problem (0: not supported)
int smallc_bf16_corr_grid(const CorrProblem& p);
// fixed-order sum of per-workgroup partial tiles ws[(wg*S + s)*256 + k*16 + c] into dw[k][c][s]
hipError_t smallc_wgrad_reduce_launch(const float* ws, float* dw, int K, int C, int S, long dw_sk, long dw_sc, int nwg,
                                      hipStream_t st);

// bf16 backward-weight for any dilation and channel count: (filter group x channel block x tap group) tiles, the
// positions cut into strips whose partial tensors a second kernel adds
bool blocked_bf16_wgrad_supported(const WgradProblem& p);
size_t blocked_bf16_wgrad_workspace(const WgradProblem& p);
hipError_t blocked_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st);

// bf16 backward-weight for dilations 1, 2, 4, 8, 16 and many taps: every consumer wave owns every fourth tap and
// keeps the x operands that neighbouring taps and k-steps share in a register ring
bool toeplitz_bf16_wgrad_supported(const WgradProblem& p);
size_t toeplitz_bf16_wgrad_workspace(const WgradProblem& p);
hipError_t toeplitz_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st);

// bf16 backward-weight for dilations 1, 2, 4 and few taps ((S - 1) d <= 16, 32 at even dilations): x is staged once and the tap shift is
// applied in registers
bool shift_bf16_wgrad_supported(const WgradProblem& p);
size_t shift_bf16_wgrad_workspace(const WgradProblem& p);
hipError_t shift_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st);

// bf16 forward / backward-data for many channels: implicit GEMM over (channel chunk, tap) with the weights
// gathered into LDS stage by stage
bool igemm_bf16_corr_supported(const CorrProblem& p);
hipError_t igemm_bf16_corr_launch(const CorrProblem& p, hipStream_t st);

// the same for dilations 1, 2, 4, 8, 16 and 14 to 52 taps, while the weights of a filter group fit in LDS: resident
// weight entries, input operands shared between taps and position blocks
bool igemm_ring_bf16_corr_supported(const CorrProblem& p);
hipError_t igemm_ring_bf16_corr_launch(const CorrProblem& p, hipStream_t st);

// the same dilations with 5 to 20 taps and weights too large for LDS: streamed weights, tiles of 32 filters x 1024
// columns, input operands shared between taps and position blocks
bool igemm_stream_bf16_corr_supported(const CorrProblem& p);
hipError_t igemm_stream_bf16_corr_launch(const CorrProblem& p, hipStream_t st);

// channel-blocked MFMA family
bool igemm_corr_supported(const CorrProblem& p);
hipError_t igemm_corr_launch(const CorrProblem& p, hipStream_t st);
bool igemm_wgrad_supported(const WgradProblem& p);
size_t igemm_wgrad_workspace(const WgradProblem& p);
hipError_t igemm_wgrad_launch(const WgradProblem& p, hipStream_t st);

// ---- device helpers -------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_float(unsigned short b) {
    return __uint_as_float(static_cast<unsigned int>(b) << 16);
}

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* base, long idx) {
    if constexpr (BF16) {
        return bf16_to_float(static_cast<const unsigned short*>(base)[idx]);
    } else {
        return static_cast<const float*>(base)[idx];
    }
}

typedef __attribute__((ext_vector_type(4))) float epi_f32x4;
typedef __attribute__((ext_vector_type(4))) __bf16 epi_bf16x4;

__device__ __forceinline__ float epi_bias(const Epilogue& e, int m) { return e.bias ? e.bias[m] : 0.f; }

// bias and ReLU (a comparison, not a max: NaN stays NaN)
__device__ __forceinline__ float epi_apply(const Epilogue& e, float v, float bias_m) {
    v += bias_m;
    return (e.relu && v < 0.f) ? 0.f : v;
}

__device__ __forceinline__ epi_f32x4 epi_apply4(const Epilogue& e, epi_f32x4 v, float bias_m) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = epi_apply(e, v[i], bias_m);
    return v;
}

// element `idx` of an output tensor whose element type the epilogue names (float -> bfloat16 is the hardware's
// nearest-even conversion)
__device__ __forceinline__ void epi_store(const Epilogue& e, float* out, long idx, float v) {
    if (e.out_bf16) {
        reinterpret_cast<__bf16*>(out)[idx] = static_cast<__bf16>(v);
    } else {
        out[idx] = v;
    }
}

// four adjacent elements from idx on; idx is a multiple of 4 and the tensor is 16-byte aligned
__device__ __forceinline__ void epi_store4(const Epilogue& e, float* out, long idx, epi_f32x4 v) {
    if (e.out_bf16) {
        *reinterpret_cast<epi_bf16x4*>(reinterpret_cast<__bf16*>(out) + idx) = __builtin_convertvector(v, epi_bf16x4);
    } else {
        *reinterpret_cast<epi_f32x4*>(out + idx) = v;
    }
}

// the same with non-temporal stores, for kernels whose output lines would only push their own input out of L2
__device__ __forceinline__ void epi_store4_nt(const Epilogue& e, float* out, long idx, epi_f32x4 v) {
    if (e.out_bf16) {
        __builtin_nontemporal_store(__builtin_convertvector(v, epi_bf16x4), reinterpret_cast<epi_bf16x4*>(reinterpret_cast<__bf16*>(out) + idx));
    } else {
        __builtin_nontemporal_store(v, reinterpret_cast<epi_f32x4*>(out + idx));
    }
}

// ---- staging helpers of the bf16 backward-weight kernels: 16-byte pieces of a row, clamped at its ends ----------
typedef __attribute__((ext_vector_type(4))) unsigned int stage_u32x4;

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// v holds the 8 elements of a row of `limit` >= 8 columns from column clamp(c, 0, limit - 8) on; returns the
// elements of columns c .. c+7, zero outside the row.
__device__ __forceinline__ stage_u32x4 fix128(stage_u32x4 v, int c, int limit) {
    const int sh = c - clampi(c, 0, limit - 8);
    if (sh == 0) return v;
    if (sh >= 8 || sh <= -8) return stage_u32x4{0u, 0u, 0u, 0u};
    unsigned long lo = v.x | (static_cast<unsigned long>(v.y) << 32), hi = v.z | (static_cast<unsigned long>(v.w) << 32);
    if (sh > 0) {  // the row ends inside the slot: drop the low elements, zeros come in at the top
        const int s = 16 * sh;
        if (s < 64) {
            lo = (lo >> s) | (hi << (64 - s));
            hi >>= s;
        } else {
            lo = hi >> (s - 64);
            hi = 0;
        }
    } else {  // the row starts inside the slot
        const int s = -16 * sh;
        if (s < 64) {
            hi = (hi << s) | (lo >> (64 - s));
            lo <<= s;
        } else {
            hi = lo << (s - 64);
            lo = 0;
        }
    }
    return stage_u32x4{static_cast<unsigned>(lo), static_cast<unsigned>(lo >> 32), static_cast<unsigned>(hi), static_cast<unsigned>(hi >> 32)};
}

// 16-byte load of the columns clamp(c, 0, limit - 8) .. + 7 of the row at `row` (c even, row 4-byte aligned)
__device__ __forceinline__ stage_u32x4 load128_clamped(const unsigned short* row, int c, int limit) {
    return *reinterpret_cast<const stage_u32x4*>(row + clampi(c, 0, limit - 8));
}
// the element pair at the even column c, zero outside the row (limit even)
__device__ __forceinline__ unsigned load_pair(const unsigned short* row, int c, int limit) {
    const unsigned v = *reinterpret_cast<const unsigned*>(row + clampi(c, 0, limit - 2));
    return (c >= 0 && c < limit) ? v : 0u;
}
__device__ __forceinline__ stage_u32x4 shift_one(stage_u32x4 v, unsigned next) {
    return stage_u32x4{__builtin_amdgcn_alignbit(v.y, v.x, 16), __builtin_amdgcn_alignbit(v.z, v.y, 16), __builtin_amdgcn_alignbit(v.w, v.z, 16),
                 __builtin_amdgcn_alignbit(next, v.w, 16)};
}


// ---- second stage of the small-channel backward-weight kernels ------------------------------------------------
// Work of "block" b (b < 4*S) of 512 threads on 64 consecutive elements of the S*256 partial tile: thread
// (grp = tid >> 4, el = tid & 15) adds the tiles of workgroup group grp (of 32 contiguous groups) left to right for
// the 4 elements 4 el .. 4 el + 3 (phase 1, result in part[grp][el]); after a workgroup barrier the threads of
// group 0 add the 32 group sums left to right and store (phase 2).  The order never depends on who runs it.
constexpr int kTailGroups = 32;
constexpr int kTailPartSlots = kTailGroups * 17;  // 16-byte LDS slots the two phases share

__device__ __forceinline__ void wgrad_tail_phase1(const WgradTail& t, int b, int tid, epi_f32x4* part) {
    const int el = tid & 15, grp = tid >> 4;
    const int e = b * 64 + 4 * el;
    const int total = t.S * 256;
    const int per = (t.nwg + kTailGroups - 1) / kTailGroups;
    const int g0 = grp * per, g1 = min(t.nwg, g0 + per);
    epi_f32x4 sum = epi_f32x4{0.f, 0.f, 0.f, 0.f};
    const float* src = t.ws + e;
#pragma unroll 8
    for (int g = g0; g < g1; ++g) sum += *reinterpret_cast<const epi_f32x4*>(src + static_cast<long>(g) * total);
    part[grp * 17 + el] = sum;
}

__device__ __forceinline__ void wgrad_tail_phase2(const WgradTail& t, int b, int tid, const epi_f32x4* part) {
    if (tid >= 16) return;
    const int el = tid;
    epi_f32x4 sum = part[el];
#pragma unroll
    for (int i = 1; i < kTailGroups; ++i) sum += part[i * 17 + el];
    const int e = b * 64 + 4 * el;
    const int s = e >> 8, k = (e >> 4) & 15, c0 = e & 15;  // the 4 elements are 4 adjacent channels
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (k < t.K && c0 + j < t.C) t.dw[k * t.dw_sk + (c0 + j) * t.dw_sc + s] = sum[j];
}

// Workgroups are dealt round-robin to the 8 XCDs (workgroup b runs on XCD b % 8).  The logical index numbers
// the workgroups XCD by XCD, so that consecutive logical indices share an XCD and its L2, for any grid size.
__device__ __forceinline__ int xcd_logical_id(int b, int grid) {
    const int x = b & 7, base = grid >> 3, rem = grid & 7;
    return x * base + (x < rem ? x : rem) + (b >> 3);
}

inline int cdiv(long a, long b) { return static_cast<int>((a + b - 1) / b); }

// Division of a small non-negative number by a divisor fixed for the launch: one multiply-high instead of the
// several dozen instructions of a 32-bit division.  With m = ceil(2^32 / d) the quotient umulhi(n, m) is exact
// while n * (m * d - 2^32) < 2^32; the host checks that for the largest n the kernel will divide.
struct FastDiv {
    unsigned d, m;
};
inline bool make_fastdiv(FastDiv& f, long d, long nmax) {
    if (d < 1 || d >= (1L << 31) || nmax < 0 || nmax >= (1L << 31)) return false;
    f.d = static_cast<unsigned>(d);
    if (d == 1) {
        f.m = 0;
        return true;
    }
    const unsigned long m = ((1UL << 32) + d - 1) / d;
    f.m = static_cast<unsigned>(m);
    return static_cast<unsigned long>(nmax) * (m * d - (1UL << 32)) < (1UL << 32);
}
__device__ __forceinline__ int fast_div(int n, const FastDiv& f) {
    return f.d == 1 ? n : static_cast<int>(__umulhi(static_cast<unsigned>(n), f.m));
}

// ---- host helpers: launches ---------------------------------------------------------------------
// Raise a kernel's dynamic LDS limit to `bytes` on the current GPU.  The runtime call costs microseconds, so the
// largest size granted so far is remembered per (kernel, GPU) and the call is made only when it has to grow.
hipError_t ensure_dynamic_lds(const void* kern, size_t bytes);

namespace detail {
template <typename Tuple, size_t... I>
inline void arg_pointers(Tuple& vals, void** ptrs, std::index_sequence<I...>) {
    ((ptrs[I] = static_cast<void*>(&std::get<I>(vals))), ...);
}
}  // namespace detail

// Launch `kern` and return the status of THIS launch (hipGetLastError would also report, and clear, an error that
// an unrelated earlier call of the host program left behind).
template <typename... Params, typename... Args>
inline hipError_t launch_kernel(void (*kern)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t st,
                                const Args&... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "kernel argument count");
#ifdef HOSTMODEL  // the host-side bounds model of the tests compiles the kernels as CPU code and runs them here
    (void)st;
    return hostmodel_launch(kern, grid, block, lds_bytes, args...);
#else
    std::tuple<Params...> vals(static_cast<Params>(args)...);
    void* ptrs[sizeof...(Params) > 0 ? sizeof...(Params) : 1];
    detail::arg_pointers(vals, ptrs, std::index_sequence_for<Params...>{});
    return hipLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, lds_bytes, st);
#endif
}

}  // namespace conv1d
