// Plain-FMA kernels for any geometry: the correctness floor of the library and the
// fallback when no MFMA family fits.  One thread per output element for the forward /
// backward-data contraction (Eq. 2; Section 3.2); one workgroup per weight-gradient
// element and sample chunk for the backward-weight pass (Section 3.3), finished by a
// fixed-order sum over the chunks.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxChunks = 16;

template <bool BF16>
__global__ __launch_bounds__(kThreads) void generic_corr_kernel(CorrProblem p, int otiles) {
    const long blk = blockIdx.x;
    const int ot = static_cast<int>(blk % otiles);
    const long nm = blk / otiles;
    const int m = static_cast<int>(nm % p.M);
    const int n = static_cast<int>(nm / p.M);
    const int o = ot * kThreads + threadIdx.x;
    if (o >= p.Wout) return;
    float acc = 0.f;
    for (int r = 0; r < p.R; ++r) {
        const long in_row = static_cast<long>(n) * p.in_sn + static_cast<long>(r) * p.Win;
        const long w_row = m * p.w_sm + r * p.w_sr + p.w_s0;
        for (int s = 0; s < p.S; ++s) {
            const int i = o + s * p.d - p.P;
            if (i >= 0 && i < p.Win) {
                acc = fmaf(load_elem<BF16>(p.in, in_row + i), load_elem<BF16>(p.wt, w_row + static_cast<long>(s) * p.w_ss), acc);
            }
        }
    }
    const long idx = static_cast<long>(n) * p.out_sn + static_cast<long>(m) * p.Wout + o;
    if (p.accumulate) {
        p.out[idx] += acc;
    } else {
        epi_store(p.epi, p.out, idx, epi_apply(p.epi, acc, epi_bias(p.epi, m)));
    }
}

// bias and ReLU in place on a float output whose sums were accumulated by several launches
__global__ __launch_bounds__(kThreads) void generic_epilogue_kernel(CorrProblem p, int otiles) {
    const long blk = blockIdx.x;
    const int ot = static_cast<int>(blk % otiles);
    const long nm = blk / otiles;
    const int m = static_cast<int>(nm % p.M);
    const int n = static_cast<int>(nm / p.M);
    const int o = ot * kThreads + threadIdx.x;
    if (o >= p.Wout) return;
    float* dst = p.out + static_cast<long>(n) * p.out_sn + static_cast<long>(m) * p.Wout + o;
    *dst = epi_apply(p.epi, *dst, epi_bias(p.epi, m));
}

// partial[chunk][k][c][s] = sum over the chunk's samples and all q.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void generic_wgrad_partial_kernel(WgradProblem p, int nchunks, int n_per_chunk) {
    __shared__ float red[kThreads / 64];
    const long kcs = static_cast<long>(p.K) * p.C * p.S;
    const long blk = blockIdx.x;
    const int chunk = static_cast<int>(blk / kcs);
    const long e = blk % kcs;
    const int s = static_cast<int>(e % p.S);
    const int c = static_cast<int>((e / p.S) % p.C);
    const int k = static_cast<int>(e / (static_cast<long>(p.S) * p.C));
    const int n0 = chunk * n_per_chunk;
    const int n1 = min(p.N, n0 + n_per_chunk);
    const int shift = s * p.d - p.P;
    // q range for which q + shift lies in [0, W)
    const int qlo = max(0, -shift);
    const int qhi = min(p.Q, p.W - shift);
    float acc = 0.f;
    for (int n = n0; n < n1; ++n) {
        const long xrow = (static_cast<long>(n) * p.C + c) * p.W + shift;
        const long grow = (static_cast<long>(n) * p.K + k) * p.Q;
        for (int q = qlo + threadIdx.x; q < qhi; q += kThreads) {
            acc = fmaf(load_elem<BF16>(p.x, xrow + q), load_elem<BF16>(p.dy, grow + q), acc);
        }
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = red[0];
        for (int i = 1; i < kThreads / 64; ++i) t += red[i];
        static_cast<float*>(p.ws)[chunk * kcs + e] = t;
    }
}

__global__ __launch_bounds__(kThreads) void generic_wgrad_reduce_kernel(const float* partial, float* dw, long kcs, int nchunks) {
    const long e = static_cast<long>(blockIdx.x) * kThreads + threadIdx.x;
    if (e >= kcs) return;
    float t = 0.f;
    for (int ch = 0; ch < nchunks; ++ch) t += partial[ch * kcs + e];
    dw[e] = t;
}

int wgrad_chunks(const WgradProblem& p) { return p.N < kMaxChunks ? p.N : kMaxChunks; }

}  // namespace

hipError_t generic_corr_launch(const CorrProblem& p, hipStream_t st) {
    const int otiles = cdiv(p.Wout, kThreads);
    const long blocks = static_cast<long>(p.N) * p.M * otiles;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    return launch_kernel(p.bf16 ? generic_corr_kernel<true> : generic_corr_kernel<false>, dim3(static_cast<unsigned>(blocks)),
                         dim3(kThreads), 0, st, p, otiles);
}

hipError_t generic_epilogue_launch(const CorrProblem& p, hipStream_t st) {
    if (p.epi.out_bf16) return hipErrorInvalidValue;
    const int otiles = cdiv(p.Wout, kThreads);
    const long blocks = static_cast<long>(p.N) * p.M * otiles;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    return launch_kernel(generic_epilogue_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, st, p, otiles);
}

size_t generic_wgrad_workspace(const WgradProblem& p) {
    return static_cast<size_t>(wgrad_chunks(p)) * p.K * p.C * p.S * sizeof(float);
}

hipError_t generic_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const int nchunks = wgrad_chunks(p);
    const int npc = cdiv(p.N, nchunks);
    const long kcs = static_cast<long>(p.K) * p.C * p.S;
    const long blocks = kcs * nchunks;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipError_t e = launch_kernel(p.bf16 ? generic_wgrad_partial_kernel<true> : generic_wgrad_partial_kernel<false>,
                                 dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0, st, p, nchunks, npc);
    if (e != hipSuccess) return e;
    return launch_kernel(generic_wgrad_reduce_kernel, dim3(cdiv(kcs, kThreads)), dim3(kThreads), 0, st,
                       static_cast<const float*>(p.ws), p.dw, kcs, nchunks);
}

}  // namespace conv1d
