// Small-channel MFMA kernels (C, K <= 16), bfloat16 inputs, FP32 accumulation and output.
//
// Forward / backward-data (Eq. 2; Section 3.2).  One v_mfma_f32_16x16x32_bf16 multiplies a
// 16 x 32 slice of the weight matrix (16 filters x [2 taps x 16 channels]) with a 32 x 16 slice of
// the shifted-input matrix (the same [2 taps x 16 channels] x 16 adjacent output columns).  All
// weight slices of a layer (NP = ceil(S/2) of them: taps p and p+NP share a slice) stay in
// registers for the lifetime of a workgroup.  The input window (tile + halo) is transposed into
// LDS as [position][8 channels] 16-byte slots so that one lane's 8 k-values are one ds_read_b128.
// A batch-reduce GEMM over taps (Algorithm 2) would re-read the window once per tap; here the
// Toeplitz structure of the shifted-input matrix is used instead: when d divides 16, the operand
// for (tile j, tap p) is the operand for (tile j+1, tap p - 16/d), so a wave that owns T adjacent
// tiles loads each operand once and feeds up to T MFMAs from it.
//
// Backward-weight (Section 3.3, Algorithm 4) for d == 8.  The contraction runs over positions:
// A = dy (16 filters x 32 positions), B = x shifted by the tap (32 positions x 16 channels), one
// 16 x 16 accumulator per tap.  With d = 8 the B operand of (k-step t, tap s) equals that of
// (t+1, s-4); wave v of a workgroup owns the taps s = v (mod 4) and keeps their 13 operands in a
// register ring, loading one new operand per k-step.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kWaves = 4;
constexpr unsigned kPermLo = 0x05040100u;  // {b.lo16, a.lo16} -> a.lo | b.lo << 16
constexpr unsigned kPermHi = 0x07060302u;  // {b.hi16, a.hi16} -> a.hi | b.hi << 16

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ------------------------------------------------------------------------------------------------
// forward / backward-data
// ------------------------------------------------------------------------------------------------
// k-slot layout of one MFMA (lane = li + 16*kb, element j of the lane's 8):
//   channel r = 8*(kb & 1) + j,  tap s = p + NP*(kb >> 1)
// LDS: plane h = kb & 1 holds channels 8h..8h+7; slot (h*LPS + i) <-> input position G0 + i.
template <int NP, int G, int T>
__global__ __launch_bounds__(kWaves * 64, 2) void smallc_corr_bf16_kernel(CorrProblem p, int tiles_per_row, int ntiles, int LPS, int fast) {
    extern __shared__ u32x4 lds4[];
    constexpr int TQ = kWaves * T * 16;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 15;
    const int kb = lane >> 4;
    const unsigned short* __restrict__ in = static_cast<const unsigned short*>(p.in);
    const unsigned short* __restrict__ wt = static_cast<const unsigned short*>(p.wt);
    const int d = (G > 0) ? 16 / (G > 0 ? G : 1) : p.d;

    // weight slices in A-operand order, built once in LDS, then held in registers
    for (int e = tid; e < NP * 64; e += kWaves * 64) {
        const int pi = e >> 6, l = e & 63;
        const int m = l & 15, h = (l >> 4) & 1, s = pi + NP * (l >> 5);
        unsigned v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 8 * h + j;
            v[j] = (m < p.M && r < p.R && s < p.S) ? wt[m * p.w_sm + r * p.w_sr + p.w_s0 + s * p.w_ss] : 0u;
        }
        lds4[e] = u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
    }
    __syncthreads();
    bf16x8 wreg[NP];
#pragma unroll
    for (int pi = 0; pi < NP; ++pi) wreg[pi] = as_bf16x8(lds4[pi * 64 + lane]);

    const int LP = TQ + (2 * NP - 1) * d;
    const int LP2 = (LP + 1) >> 1;
    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int n = tile / tiles_per_row;
        const int O0 = (tile - n * tiles_per_row) * TQ;
        const int G0 = O0 - p.P;
        __syncthreads();
        // transpose the window into LDS: one task = 8 channels x 2 adjacent positions
        for (int task = tid; task < 2 * LP2; task += kWaves * 64) {
            const int h = task >= LP2 ? 1 : 0;
            const int pp = task - h * LP2;
            const int g = G0 + 2 * pp;
            unsigned v[8];
            if (fast && g >= 0 && g + 1 < p.Win) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = 8 * h + j;
                    v[j] = r < p.R ? *reinterpret_cast<const unsigned*>(in + (static_cast<long>(n) * p.R + r) * p.Win + g) : 0u;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = 8 * h + j;
                    unsigned lo = 0u, hi = 0u;
                    if (r < p.R) {
                        const unsigned short* row = in + (static_cast<long>(n) * p.R + r) * p.Win;
                        if (g >= 0 && g < p.Win) lo = row[g];
                        if (g + 1 >= 0 && g + 1 < p.Win) hi = row[g + 1];
                    }
                    v[j] = lo | (hi << 16);
                }
            }
            u32x4 ev, od;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                ev[q] = __builtin_amdgcn_perm(v[2 * q + 1], v[2 * q], kPermLo);
                od[q] = __builtin_amdgcn_perm(v[2 * q + 1], v[2 * q], kPermHi);
            }
            lds4[h * LPS + 2 * pp] = ev;
            lds4[h * LPS + 2 * pp + 1] = od;
        }
        __syncthreads();

        f32x4 acc[T];
#pragma unroll
        for (int j = 0; j < T; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        const int ob = wave * T * 16;
        const u32x4* bbase = lds4 + (kb & 1) * LPS + ob + li + (kb >> 1) * NP * d;
        // Operands are fetched PF steps ahead of the MFMAs that consume them; the scheduling
        // barriers keep the compiler from sinking the LDS reads back down to their first use.
        constexpr int PF = 4;
        if constexpr (G > 0) {
            constexpr int D = 16 / (G > 0 ? G : 1);
            constexpr int NF = G * (T - 1) + NP;
            bf16x8 fr[NF];
#pragma unroll
            for (int m = 0; m < PF && m < NF; ++m) fr[m] = as_bf16x8(bbase[m * D]);
#pragma unroll
            for (int m = 0; m < NF; ++m) {
                if (m + PF < NF) fr[m + PF] = as_bf16x8(bbase[(m + PF) * D]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < T; ++j) {
                    const int pi = m - G * j;
                    if (pi >= 0 && pi < NP) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[pi < 0 ? 0 : (pi >= NP ? 0 : pi)], fr[m], acc[j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            bf16x8 fr[NP][T];
#pragma unroll
            for (int j = 0; j < T; ++j) fr[0][j] = as_bf16x8(bbase[16 * j]);
#pragma unroll
            for (int pi = 0; pi < NP; ++pi) {
                if (pi + 1 < NP) {
#pragma unroll
                    for (int j = 0; j < T; ++j) fr[pi + 1][j] = as_bf16x8(bbase[16 * j + (pi + 1) * d]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < T; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wreg[pi], fr[pi][j], acc[j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
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

constexpr int kCorrT = 8;
constexpr int kNPBuckets[] = {3, 5, 9, 13, 17, 26};

struct CorrPlan {
    int NP, G, LPS, tiles_per_row, ntiles, fast;
    size_t lds_bytes;
    bool ok;
};

CorrPlan corr_plan(const CorrProblem& p) {
    CorrPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.R > 16 || p.M > 16) return pl;
    const int need = (p.S + 1) / 2;
    pl.NP = 0;
    for (int b : kNPBuckets) {
        if (b >= need) { pl.NP = b; break; }
    }
    if (pl.NP == 0) return pl;
    pl.G = (p.d <= 16 && 16 % p.d == 0) ? 16 / p.d : 0;
    constexpr int TQ = kWaves * kCorrT * 16;
    const long LP = TQ + static_cast<long>(2 * pl.NP - 1) * p.d;
    const long LPS = (LP + 2 + 7) / 8 * 8;
    long slots = 2 * LPS;
    if (slots < pl.NP * 64) slots = pl.NP * 64;
    if (slots * 16 > kLdsBudget / 2) return pl;  // two workgroups per CU
    pl.LPS = static_cast<int>(LPS);
    pl.tiles_per_row = cdiv(p.Wout, TQ);
    const long nt = static_cast<long>(p.N) * pl.tiles_per_row;
    if (nt > 0x7fffffffL) return pl;
    pl.ntiles = static_cast<int>(nt);
    pl.lds_bytes = static_cast<size_t>(slots) * 16;
    // dword loads of position pairs need even row starts and an even window origin
    pl.fast = (p.Win % 2 == 0) && (p.P % 2 == 0) && (reinterpret_cast<uintptr_t>(p.in) % 4 == 0);
    pl.ok = true;
    return pl;
}

template <int NP, int G>
hipError_t corr_launch_t(const CorrProblem& p, const CorrPlan& pl, hipStream_t st) {
    auto kern = smallc_corr_bf16_kernel<NP, G, kCorrT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    const int grid = pl.ntiles < 2 * kNumCU ? pl.ntiles : 2 * kNumCU;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kWaves * 64), pl.lds_bytes, st, p, pl.tiles_per_row, pl.ntiles, pl.LPS, pl.fast);
    return hipGetLastError();
}

template <int NP>
hipError_t corr_launch_np(const CorrProblem& p, const CorrPlan& pl, hipStream_t st) {
    switch (pl.G) {
        case 1: return corr_launch_t<NP, 1>(p, pl, st);
        case 2: return corr_launch_t<NP, 2>(p, pl, st);
        case 4: return corr_launch_t<NP, 4>(p, pl, st);
        case 8: return corr_launch_t<NP, 8>(p, pl, st);
        case 16: return corr_launch_t<NP, 16>(p, pl, st);
        default: return corr_launch_t<NP, 0>(p, pl, st);
    }
}

// ------------------------------------------------------------------------------------------------
// backward-weight, d == 8
// ------------------------------------------------------------------------------------------------
// LDS rows of 16-byte slots (8 positions each):
//   dyt[16][LQS]  row = filter,  slot i <-> q = Qs + 8i .. 8i+7
//   xt [16][LXS]  row = channel, slot i <-> input positions Qs - P + 8i .. +7
// k-step t covers q = Qs + 32t .. +31; lane (li, kb) holds positions 8*kb .. 8*kb+7 of it.
// Tap s = v + 4i of wave v reads x slot 4*(t+i) + v + kb: operand index f = t + i.
template <int NT>
__global__ __launch_bounds__(256, 2) void smallc_wgrad_bf16_d8_kernel(WgradProblem p, int chunks_per_row, int nchunks, int QC, int LQS, int LXS, int fast) {
    extern __shared__ u32x4 lds4[];
    u32x4* dyt = lds4;
    u32x4* xt = lds4 + 16 * LQS;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15;
    const int kb = lane >> 4;
    const unsigned short* __restrict__ x = static_cast<const unsigned short*>(p.x);
    const unsigned short* __restrict__ dy = static_cast<const unsigned short*>(p.dy);
    const int nt = (p.S - wave + 3) / 4;
    const int QS8 = QC / 8;       // dy slots per row
    const int XS8 = QS8 + 56;     // x slots per row that the ring may touch
    const int nsteps = QC / 32;   // multiple of NT

    f32x4 acc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int chunk = blockIdx.x; chunk < nchunks; chunk += gridDim.x) {
        const int n = chunk / chunks_per_row;
        const int Qs = (chunk - n * chunks_per_row) * QC;
        const int G0 = Qs - p.P;
        __syncthreads();
        for (int e = tid; e < 16 * (QS8 + XS8); e += 256) {
            const bool is_x = e >= 16 * QS8;
            const int e2 = is_x ? e - 16 * QS8 : e;
            const int per_row = is_x ? XS8 : QS8;
            const int r = e2 / per_row;
            const int i = e2 - r * per_row;
            const int rows = is_x ? p.C : p.K;
            const int width = is_x ? p.W : p.Q;
            const int g = (is_x ? G0 : Qs) + 8 * i;
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (r < rows && g + 8 > 0 && g < width) {
                const unsigned short* row = (is_x ? x : dy) + (static_cast<long>(n) * rows + r) * width;
                if (fast && g >= 0 && g + 8 <= width) {
                    v = *reinterpret_cast<const u32x4*>(row + g);
                } else {
                    unsigned t[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) t[j] = (g + j >= 0 && g + j < width) ? row[g + j] : 0u;
                    v = u32x4{t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16)};
                }
            }
            (is_x ? xt + r * LXS : dyt + r * LQS)[i] = v;
        }
        __syncthreads();

        const u32x4* ap = dyt + li * LQS + kb;
        const u32x4* xp = xt + li * LXS + wave + kb;
        bf16x8 ring[NT];
#pragma unroll
        for (int i = 0; i < NT; ++i) ring[i] = as_bf16x8(xp[4 * i]);
        bf16x8 a = as_bf16x8(ap[0]);
        for (int tb = 0; tb < nsteps; tb += NT) {
#pragma unroll
            for (int u = 0; u < NT; ++u) {
                const int t = tb + u;
                // slot u is dead once tap 0 has consumed it: refill it (and fetch the next dy operand)
                // right away so the other taps' MFMAs cover the LDS latency
                acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ring[u], acc[0], 0, 0, 0);
                const bf16x8 a_nxt = as_bf16x8(ap[4 * (t + 1 < nsteps ? t + 1 : t)]);
                ring[u] = as_bf16x8(xp[4 * (t + NT)]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 1; i < NT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ring[(u + i) % NT], acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                a = a_nxt;
            }
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

constexpr int kWgradNT = 13;

struct WgradPlan {
    int QC, LQS, LXS, chunks_per_row, nchunks, grid, fast;
    size_t lds_bytes;
    bool ok;
};

WgradPlan wgrad_plan(const WgradProblem& p) {
    WgradPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.C > 16 || p.K > 16 || p.d != 8 || p.S > 4 * kWgradNT) return pl;
    const int unit = 32 * kWgradNT;  // 416 columns: one turn of the operand ring
    // pick the chunk length (1..3 ring turns) that gives the shortest critical path over 2 WGs/CU
    auto lds_for = [](int qc, int* lqs, int* lxs) {
        const int QS8 = qc / 8, XS8 = QS8 + 56;
        *lqs = (QS8 + 7) / 8 * 8 + 1;  // row stride == 16 bytes (mod 128): 8 rows of one column hit 8 bank groups
        *lxs = (XS8 + 7) / 8 * 8 + 1;
        return 16L * (*lqs + *lxs) * 16;
    };
    int best_m = 0;
    long best_cost = -1;
    for (int m = 1; m <= 3; ++m) {
        int a, b;
        if (lds_for(unit * m, &a, &b) > kLdsBudget / 2) break;  // two workgroups per CU
        const long chunks = static_cast<long>(p.N) * cdiv(p.Q, unit * m);
        const long rounds = (chunks + 2 * kNumCU - 1) / (2 * kNumCU);
        const long cost = rounds * (unit * m + 450);  // columns computed + window re-staged per chunk
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_m = m; }
    }
    if (best_m == 0) return pl;
    pl.QC = unit * best_m;
    const long bytes = lds_for(pl.QC, &pl.LQS, &pl.LXS);
    pl.chunks_per_row = cdiv(p.Q, pl.QC);
    const long nc = static_cast<long>(p.N) * pl.chunks_per_row;
    if (nc > 0x7fffffffL) return pl;
    pl.nchunks = static_cast<int>(nc);
    pl.grid = pl.nchunks < 2 * kNumCU ? pl.nchunks : 2 * kNumCU;
    pl.lds_bytes = static_cast<size_t>(bytes);
    pl.fast = (p.W % 8 == 0) && (p.Q % 8 == 0) && (p.P % 8 == 0) && (reinterpret_cast<uintptr_t>(p.x) % 16 == 0) &&
              (reinterpret_cast<uintptr_t>(p.dy) % 16 == 0);
    pl.ok = true;
    return pl;
}

}  // namespace

bool smallc_bf16_corr_supported(const CorrProblem& p) { return corr_plan(p).ok; }

hipError_t smallc_bf16_corr_launch(const CorrProblem& p, hipStream_t st) {
    const CorrPlan pl = corr_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    switch (pl.NP) {
        case 3: return corr_launch_np<3>(p, pl, st);
        case 5: return corr_launch_np<5>(p, pl, st);
        case 9: return corr_launch_np<9>(p, pl, st);
        case 13: return corr_launch_np<13>(p, pl, st);
        case 17: return corr_launch_np<17>(p, pl, st);
        case 26: return corr_launch_np<26>(p, pl, st);
        default: return hipErrorInvalidValue;
    }
}

bool smallc_bf16_wgrad_supported(const WgradProblem& p) { return wgrad_plan(p).ok; }

size_t smallc_bf16_wgrad_workspace(const WgradProblem& p) {
    const WgradPlan pl = wgrad_plan(p);
    return pl.ok ? static_cast<size_t>(pl.grid) * p.S * 256 * sizeof(float) : 0;
}

hipError_t smallc_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const WgradPlan pl = wgrad_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    auto kern = smallc_wgrad_bf16_d8_kernel<kWgradNT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(pl.grid), dim3(256), pl.lds_bytes, st, p, pl.chunks_per_row, pl.nchunks, pl.QC, pl.LQS, pl.LXS,
                       pl.fast);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return smallc_wgrad_reduce_launch(static_cast<const float*>(p.ws), p.dw, p.K, p.C, p.S, pl.grid, st);
}

}  // namespace conv1d
