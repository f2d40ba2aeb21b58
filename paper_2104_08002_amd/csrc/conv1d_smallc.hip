// Small-channel MFMA kernels (C, K <= 16): family dispatch and the FP32 members.
//
// The forward / backward-data contraction (Eq. 2; Section 3.2) for one sample is the product of a
// 16 x (taps*channels) weight matrix with a (taps*channels) x width matrix whose rows are shifted
// copies of the input (Algorithm 1 written as one GEMM).  Where the paper keeps a 64-wide block
// of the input in cache across the taps of a batch-reduce GEMM, here a workgroup keeps a window of
// the input (tile + halo of (S-1)*d columns) in LDS, and each wave walks the (tap, channel-chunk)
// reduction with v_mfma_f32_16x16x4_f32, reading the shifted windows straight out of LDS.
//
// The backward-weight pass (Section 3.3, Algorithm 4) contracts over positions: per tap a
// 16 x 16 (filters x channels) accumulator tile lives in registers while the workgroup streams
// through its share of the width axis; per-workgroup partial sums go to the workspace and a
// second kernel adds them in a fixed order.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;

// ------------------------------------------------------------------------------------------------
// FP32 forward / backward-data
// ------------------------------------------------------------------------------------------------
// Workgroup: WAVES waves; wave v owns T adjacent 16-column output tiles.  LDS holds
//   wfrag[S*RC][64]   weights in MFMA A-operand order: entry (step = s*RC + cc, lane = m + 16*kb)
//                     is wt(m, 4*cc + kb, s)  (zero outside M x R)
//   win[4*RC][LPS]    the input window, row r, column i <-> input position G0 + i
template <int RC, int T, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void smallc_corr_f32_kernel(CorrProblem p, int tiles_per_row, int ntiles, int LPS) {
    extern __shared__ float lds[];
    constexpr int TQ = WAVES * T * 16;
    const int nsteps = p.S * RC;
    float* wfrag = lds;
    float* win = lds + nsteps * 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 15;  // row of A / column of B and D
    const int kb = lane >> 4;  // k index of A/B; row block of D
    const float* __restrict__ in = static_cast<const float*>(p.in);
    const float* __restrict__ wt = static_cast<const float*>(p.wt);

    for (int e = tid; e < nsteps * 64; e += WAVES * 64) {
        const int step = e >> 6, l = e & 63;
        const int m = l & 15, r = 4 * (step % RC) + (l >> 4), s = step / RC;
        float v = 0.f;
        if (m < p.M && r < p.R) v = wt[m * p.w_sm + r * p.w_sr + p.w_s0 + s * p.w_ss];
        wfrag[e] = v;
    }

    const int halo = (p.S - 1) * p.d;
    const int LP = TQ + halo;
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int n = tile / tiles_per_row;
        const int O0 = (tile - n * tiles_per_row) * TQ;
        const int G0 = O0 - p.P;
        __syncthreads();  // previous tile's readers are done (and wfrag is written on the first pass)
        for (int r = 0; r < 4 * RC; ++r) {
            float* row = win + r * LPS;
            if (r < p.R) {
                const float* src = in + (static_cast<long>(n) * p.R + r) * p.Win;
                for (int i = tid; i < LP; i += WAVES * 64) {
                    const int g = G0 + i;
                    row[i] = (g >= 0 && g < p.Win) ? src[g] : 0.f;
                }
            } else {
                for (int i = tid; i < LP; i += WAVES * 64) row[i] = 0.f;
            }
        }
        __syncthreads();

        f32x4 acc[T];
#pragma unroll
        for (int j = 0; j < T; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int ob = wave * T * 16;
        const float* bptr = win + kb * LPS + ob + li;
        const float* aptr = wfrag + lane;
        // operands of tap s+1 are fetched from LDS while the MFMAs of tap s run
        float a_cur[RC], b_cur[RC][T];
#pragma unroll
        for (int cc = 0; cc < RC; ++cc) {
            a_cur[cc] = aptr[cc * 64];
#pragma unroll
            for (int j = 0; j < T; ++j) b_cur[cc][j] = bptr[cc * 4 * LPS + j * 16];
        }
        for (int s = 0; s < p.S; ++s) {
            const int sn = s + 1 < p.S ? s + 1 : s;
            const float* bs = bptr + sn * p.d;
            float a_nxt[RC], b_nxt[RC][T];
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) {
                a_nxt[cc] = aptr[(sn * RC + cc) * 64];
#pragma unroll
                for (int j = 0; j < T; ++j) b_nxt[cc][j] = bs[cc * 4 * LPS + j * 16];
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of the MFMA block
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) {
#pragma unroll
                for (int j = 0; j < T; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[cc], b_cur[cc][j], acc[j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) {
                a_cur[cc] = a_nxt[cc];
#pragma unroll
                for (int j = 0; j < T; ++j) b_cur[cc][j] = b_nxt[cc][j];
            }
        }
#pragma unroll
        for (int j = 0; j < T; ++j) {
            const int o = O0 + ob + j * 16 + li;
            if (o < p.Wout) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = 4 * kb + i;
                    if (m < p.M) p.out[(static_cast<long>(n) * p.M + m) * p.Wout + o] = acc[j][i];
                }
            }
        }
    }
}

struct CorrF32Plan {
    int RC, LPS, tiles_per_row, ntiles;
    size_t lds_bytes;
    bool ok;
};

constexpr int kCorrT = 4, kCorrWaves = 8;

CorrF32Plan corr_f32_plan(const CorrProblem& p) {
    CorrF32Plan pl{};
    pl.ok = false;
    if (p.R > 16 || p.M > 16) return pl;
    constexpr int TQ = kCorrWaves * kCorrT * 16;
    pl.RC = (p.R + 3) / 4;
    const long halo = static_cast<long>(p.S - 1) * p.d;
    const long LP = TQ + halo;
    // row stride == 16 (mod 32) words: the four k rows of a B fragment fall on disjoint bank halves
    long LPS = (LP + 31) / 32 * 32 + 16;
    const long bytes = (static_cast<long>(p.S) * pl.RC * 64 + 4L * pl.RC * LPS) * 4;
    if (bytes > kLdsBudget) return pl;
    pl.LPS = static_cast<int>(LPS);
    pl.tiles_per_row = cdiv(p.Wout, TQ);
    const long nt = static_cast<long>(p.N) * pl.tiles_per_row;
    if (nt > 0x7fffffffL) return pl;
    pl.ntiles = static_cast<int>(nt);
    pl.lds_bytes = static_cast<size_t>(bytes);
    pl.ok = true;
    return pl;
}

template <int RC>
hipError_t corr_f32_launch_rc(const CorrProblem& p, const CorrF32Plan& pl, hipStream_t st) {
    auto kern = smallc_corr_f32_kernel<RC, kCorrT, kCorrWaves>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    const int grid = pl.ntiles < kNumCU ? pl.ntiles : kNumCU;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kCorrWaves * 64), pl.lds_bytes, st, p, pl.tiles_per_row, pl.ntiles, pl.LPS);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// FP32 backward-weight
// ------------------------------------------------------------------------------------------------
// Workgroup of 4 waves; wave v owns taps s = v, v+4, v+8, ... (at most NT of them) and keeps one
// 16 x 16 accumulator tile per tap.  The workgroup walks chunks of QC output columns of one sample:
//   dyt[16][LQS]  rows = filters, column j <-> q = Qs + j
//   xt [16][LXS]  rows = channels, column i <-> input position Qs - P + i
// One MFMA k-step covers 4 positions: A = dy[m][q0 + kb], B = x[c][q0 + kb + s*d - P].
// Partial sums: ws[(wg * S + s) * 256 + m * 16 + c].
template <int NT>
__global__ __launch_bounds__(256) void smallc_wgrad_f32_kernel(WgradProblem p, int chunks_per_row, int nchunks, int QC, int LQS, int LXS) {
    extern __shared__ float lds[];
    float* dyt = lds;
    float* xt = lds + 16 * LQS;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15;
    const int kb = lane >> 4;
    const float* __restrict__ x = static_cast<const float*>(p.x);
    const float* __restrict__ dy = static_cast<const float*>(p.dy);
    const int LX = QC + (4 * NT - 1) * p.d;  // every tap slot a wave may read, valid tap or not
    const int nt = (p.S - wave + 3) / 4;     // real taps of this wave; slots beyond compute unused sums

    f32x4 acc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
        const int n = chunk / chunks_per_row;
        const int Qs = (chunk - n * chunks_per_row) * QC;
        const int G0 = Qs - p.P;
        __syncthreads();
        for (int r = 0; r < 16; ++r) {
            float* drow = dyt + r * LQS;
            float* xrow = xt + r * LXS;
            if (r < p.K) {
                const float* src = dy + (static_cast<long>(n) * p.K + r) * p.Q;
                for (int i = tid; i < QC; i += 256) drow[i] = (Qs + i < p.Q) ? src[Qs + i] : 0.f;
            } else {
                for (int i = tid; i < QC; i += 256) drow[i] = 0.f;
            }
            if (r < p.C) {
                const float* src = x + (static_cast<long>(n) * p.C + r) * p.W;
                for (int i = tid; i < LX; i += 256) {
                    const int g = G0 + i;
                    xrow[i] = (g >= 0 && g < p.W) ? src[g] : 0.f;
                }
            } else {
                for (int i = tid; i < LX; i += 256) xrow[i] = 0.f;
            }
        }
        __syncthreads();
        const float* ap = dyt + li * LQS + kb;
        const float* bp = xt + li * LXS + kb + wave * p.d;
        const int dstep = 4 * p.d;
        // operands of k-step t+4 are fetched from LDS while the MFMAs of k-step t run
        float a_cur = ap[0], b_cur[NT];
#pragma unroll
        for (int i = 0; i < NT; ++i) b_cur[i] = bp[i * dstep];
        for (int t = 0; t < QC; t += 4) {
            const int tn = t + 4 < QC ? t + 4 : t;
            const float a_nxt = ap[tn];
            float b_nxt[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) b_nxt[i] = bp[tn + i * dstep];
            __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of the MFMA block
#pragma unroll
            for (int i = 0; i < NT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur, b_cur[i], acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a_cur = a_nxt;
#pragma unroll
            for (int i = 0; i < NT; ++i) b_cur[i] = b_nxt[i];
        }
    }
    float* ws = static_cast<float*>(p.ws) + static_cast<long>(blockIdx.x) * p.S * 256;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        if (i < nt) {
            const int s = wave + 4 * i;
#pragma unroll
            for (int j = 0; j < 4; ++j) ws[s * 256 + (4 * kb + j) * 16 + li] = acc[i][j];
        }
    }
}

// dw[k][c][s] = sum over workgroups, in workgroup order, of ws[(wg*S + s)*256 + k*16 + c]
__global__ __launch_bounds__(256) void smallc_wgrad_reduce_kernel(const float* __restrict__ ws, float* __restrict__ dw, int K, int C, int S, int nwg) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= K * C * S) return;
    const int s = e % S;
    const int c = (e / S) % C;
    const int k = e / (S * C);
    const float* src = ws + s * 256 + k * 16 + c;
    float t = 0.f;
    for (int g = 0; g < nwg; ++g) t += src[static_cast<long>(g) * S * 256];
    dw[e] = t;
}

struct WgradF32Plan {
    int QC, LQS, LXS, chunks_per_row, nchunks, grid;
    size_t lds_bytes;
    bool ok;
};

constexpr int kWgradNT = 13;

WgradF32Plan wgrad_f32_plan(const WgradProblem& p) {
    WgradF32Plan pl{};
    pl.ok = false;
    if (p.C > 16 || p.K > 16 || p.S > 4 * kWgradNT) return pl;
    const long halo = static_cast<long>(4 * kWgradNT - 1) * p.d;
    int QC = 256;
    // row strides == 2 (mod 32) words: the 16 rows x 4 columns of an operand fragment hit distinct banks
    auto pad = [](long v) { return (v + 31) / 32 * 32 + 2; };
    long LQS = pad(QC), LXS = pad(QC + halo);
    long bytes = 16 * (LQS + LXS) * 4;
    if (bytes > kLdsBudget) return pl;
    pl.QC = QC;
    pl.LQS = static_cast<int>(LQS);
    pl.LXS = static_cast<int>(LXS);
    pl.chunks_per_row = cdiv(p.Q, QC);
    const long nc = static_cast<long>(p.N) * pl.chunks_per_row;
    if (nc > 0x7fffffffL) return pl;
    pl.nchunks = static_cast<int>(nc);
    pl.grid = pl.nchunks < 2 * kNumCU ? pl.nchunks : 2 * kNumCU;
    pl.lds_bytes = static_cast<size_t>(bytes);
    pl.ok = true;
    return pl;
}

}  // namespace

hipError_t smallc_wgrad_reduce_launch(const float* ws, float* dw, int K, int C, int S, int nwg, hipStream_t st) {
    const int kcs = K * C * S;
    hipLaunchKernelGGL(smallc_wgrad_reduce_kernel, dim3(cdiv(kcs, 256)), dim3(256), 0, st, ws, dw, K, C, S, nwg);
    return hipGetLastError();
}

bool smallc_corr_supported(const CorrProblem& p) {
    if (p.bf16) return smallc_bf16_corr_supported(p);
    return corr_f32_plan(p).ok;
}

hipError_t smallc_corr_launch(const CorrProblem& p, hipStream_t st) {
    if (p.bf16) return smallc_bf16_corr_launch(p, st);
    const CorrF32Plan pl = corr_f32_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    switch (pl.RC) {
        case 1: return corr_f32_launch_rc<1>(p, pl, st);
        case 2: return corr_f32_launch_rc<2>(p, pl, st);
        case 3: return corr_f32_launch_rc<3>(p, pl, st);
        default: return corr_f32_launch_rc<4>(p, pl, st);
    }
}

bool smallc_wgrad_supported(const WgradProblem& p) {
    if (p.bf16) return smallc_bf16_wgrad_supported(p);
    return wgrad_f32_plan(p).ok;
}

size_t smallc_wgrad_workspace(const WgradProblem& p) {
    if (p.bf16) return smallc_bf16_wgrad_workspace(p);
    const WgradF32Plan pl = wgrad_f32_plan(p);
    if (!pl.ok) return 0;
    return static_cast<size_t>(pl.grid) * p.S * 256 * sizeof(float);
}

hipError_t smallc_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    if (p.bf16) return smallc_bf16_wgrad_launch(p, st);
    const WgradF32Plan pl = wgrad_f32_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    auto kern = smallc_wgrad_f32_kernel<kWgradNT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(pl.grid), dim3(256), pl.lds_bytes, st, p, pl.chunks_per_row, pl.nchunks, pl.QC, pl.LQS, pl.LXS);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return smallc_wgrad_reduce_launch(static_cast<const float*>(p.ws), p.dw, p.K, p.C, p.S, pl.grid, st);
}

}  // namespace conv1d
