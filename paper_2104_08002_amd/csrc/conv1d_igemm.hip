// Channel-blocked MFMA family: layers with more than 16 channels or filters.
//
// Algorithms 1-4 of the paper block the channel and filter dimensions and run one small GEMM per
// (tap, block pair).  The same blocking is applied here one level up: C and K are cut into blocks of 16, the
// width of the MFMA tile the small-channel kernels are built around, and every (filter block, channel block)
// pair is one launch of those kernels on a strided view of the tensors.
//   fwd / bwd_data  out[:, mb, :] = sum over rb of corr(in[:, rb, :], wt[mb, rb, :])   one launch per filter block
//                   when the kernel can hold the weights of all channel blocks (it then reduces over them in
//                   its accumulators), else one launch per pair: the first channel block overwrites the output,
//                   the following ones accumulate
//   bwd_weight      dw[kb, cb, :]  = wgrad(x[:, cb, :], dy[:, kb, :])      each pair owns its block of dw
// All launches go to the caller's stream in a fixed order, so results are deterministic and the one
// workspace is reused by every pair.
#include "conv1d_internal.h"

namespace conv1d {
namespace {

constexpr int kBlock = 16;

inline const void* advance(const void* base, long elems, int bf16) {
    return static_cast<const char*>(base) + elems * (bf16 ? 2 : 4);
}

CorrProblem corr_block(const CorrProblem& p, int m0, int r0) {
    CorrProblem b = p;
    b.M = p.M - m0 < kBlock ? p.M - m0 : kBlock;
    b.R = p.R - r0 < kBlock ? p.R - r0 : kBlock;
    b.in = advance(p.in, static_cast<long>(r0) * p.Win, p.bf16);
    b.wt = advance(p.wt, m0 * p.w_sm + r0 * p.w_sr, p.bf16);
    b.out = reinterpret_cast<float*>(reinterpret_cast<char*>(p.out) + static_cast<long>(m0) * p.Wout * (p.epi.out_bf16 ? 2 : 4));
    if (p.epi.bias) b.epi.bias = p.epi.bias + m0;
    b.accumulate = p.accumulate || r0 > 0;
    b.w_contig = 0;
    return b;
}

WgradProblem wgrad_block(const WgradProblem& p, int k0, int c0) {
    WgradProblem b = p;
    b.K = p.K - k0 < kBlock ? p.K - k0 : kBlock;
    b.C = p.C - c0 < kBlock ? p.C - c0 : kBlock;
    b.x = advance(p.x, static_cast<long>(c0) * p.W, p.bf16);
    b.dy = advance(p.dy, static_cast<long>(k0) * p.Q, p.bf16);
    b.dw = p.dw + k0 * p.dw_sk + c0 * p.dw_sc;
    return b;
}

// FP32 backward-weight: all block pairs as one launch while their partial sums fit a moderate workspace
constexpr size_t kMaxPairsWorkspace = 512u << 20;
bool fp32_pairs_in_one_launch(const WgradProblem& p) {
    if (p.bf16 || p.dw_sc != p.S) return false;
    const size_t bytes = smallc_wgrad_f32_blocks_workspace(p);
    return bytes > 0 && bytes <= kMaxPairsWorkspace;
}

// How a layer with more than one block runs.
enum class CorrRoute {
    kNone,
    kRing, kStream, kStaged,   // bf16: one launch of a many-channel kernel
    kF32Whole,                 // fp32: one launch, channel blocks reduced in the accumulators
    kF32PerChannelBlock,       // fp32: one launch per channel block, accumulating into the output
    kRows,                     // one launch per filter block (each reduces its channel blocks itself)
    kPairs                     // some filter block needs one launch per channel block, accumulating into the output
};

CorrProblem without_epilogue(CorrProblem p) {
    p.epi = Epilogue{};
    return p;
}

CorrRoute corr_route(const CorrProblem& p) {
    if (p.bf16 && igemm_ring_bf16_corr_supported(p)) return CorrRoute::kRing;
    if (p.bf16 && igemm_stream_bf16_corr_supported(p)) return CorrRoute::kStream;
    if (p.bf16 && igemm_bf16_corr_supported(p)) return CorrRoute::kStaged;
    if (p.R <= kBlock && p.M <= kBlock) return CorrRoute::kNone;  // one block: that is the small-channel family itself
    if (!smallc_corr_supported(corr_block(p, 0, 0))) return CorrRoute::kNone;  // the first block pair is the largest one
    if (!p.bf16) {
        CorrProblem whole = p;
        whole.w_contig = 0;
        if (smallc_corr_f32_blocks_supported(whole)) return CorrRoute::kF32Whole;
        CorrProblem cols = corr_block(p, 0, 0);
        cols.M = p.M;
        if (smallc_corr_f32_blocks_supported(cols)) return CorrRoute::kF32PerChannelBlock;
    }
    for (int m0 = 0; m0 < p.M; m0 += kBlock) {
        CorrProblem rows = corr_block(p, m0, 0);
        rows.R = p.R;
        if (!smallc_corr_supported(rows)) return CorrRoute::kPairs;
    }
    return CorrRoute::kRows;
}

bool accumulates(CorrRoute r) { return r == CorrRoute::kF32PerChannelBlock || r == CorrRoute::kPairs; }

}  // namespace

bool igemm_corr_supported(const CorrProblem& p) {
    const CorrRoute r = corr_route(p);
    if (r == CorrRoute::kNone) return false;
    // partial sums that pass through the output tensor need it to hold floats
    return !(p.epi.out_bf16 && accumulates(r));
}

hipError_t igemm_corr_launch(const CorrProblem& p, hipStream_t st) {
    if (!igemm_corr_supported(p)) return hipErrorInvalidValue;
    const CorrRoute route = corr_route(p);
    switch (route) {
        case CorrRoute::kRing: return igemm_ring_bf16_corr_launch(p, st);
        case CorrRoute::kStream: return igemm_stream_bf16_corr_launch(p, st);
        case CorrRoute::kStaged: return igemm_bf16_corr_launch(p, st);
        case CorrRoute::kF32Whole: {
            // every filter block in one launch: the kernel holds the weights of all channel blocks of a block
            CorrProblem whole = p;
            whole.w_contig = 0;
            return smallc_corr_f32_blocks_launch(whole, st);
        }
        default: break;
    }
    // Launches that accumulate into the output leave the epilogue to one elementwise kernel at the end.
    const CorrProblem q = accumulates(route) ? without_epilogue(p) : p;
    if (route == CorrRoute::kF32PerChannelBlock) {
        // one launch per channel block (all filter blocks each)
        for (int r0 = 0; r0 < q.R; r0 += kBlock) {
            CorrProblem cols = corr_block(q, 0, r0);
            cols.M = q.M;
            const hipError_t e = smallc_corr_f32_blocks_launch(cols, st);
            if (e != hipSuccess) return e;
        }
    } else {
        for (int m0 = 0; m0 < q.M; m0 += kBlock) {
            // all channel blocks in one launch when the kernel can keep their weights in LDS ...
            CorrProblem rows = corr_block(q, m0, 0);
            rows.R = q.R;
            if (smallc_corr_supported(rows)) {
                const hipError_t e = smallc_corr_launch(rows, st);
                if (e != hipSuccess) return e;
                continue;
            }
            // ... else one launch per channel block, accumulating into the output
            for (int r0 = 0; r0 < q.R; r0 += kBlock) {
                const CorrProblem b = corr_block(q, m0, r0);
                const hipError_t e = smallc_corr_launch(b, st);
                if (e != hipSuccess) return e;
            }
        }
    }
    if (accumulates(route) && (p.epi.bias || p.epi.relu)) return generic_epilogue_launch(p, st);
    return hipSuccess;
}

// the register-shift kernel wherever it applies: the others stage several phase copies of x for these shapes (measured
// on C = K = 64: 23.4 against 24.7 us at S = 5, d = 4; 35.2 against 37.4 us at S = 17, d = 2; 24 against 50 us at S = 5, d = 1)
// Its four consumer waves take the four channel blocks of a group of 64 channels: with fewer than three of the four real
// (C = 16, 32, 80 ...) most of its MFMA waves idle and the phase-copy kernel is faster (batch 56, d = 4, S = 5,
// Q = 60000: 58 against 85 us at C = K = 16, 122 against 132 us at C = K = 32).
static bool prefer_shift_wgrad(const WgradProblem& p) {
    if (!p.bf16 || !shift_bf16_wgrad_supported(p)) return false;
    const int blocks = (p.C + 15) / 16, groups = (p.C + 63) / 64;
    return 4 * blocks >= 3 * 4 * groups || !toeplitz_bf16_wgrad_supported(p);
}

bool igemm_wgrad_supported(const WgradProblem& p) {
    if (p.bf16 && (shift_bf16_wgrad_supported(p) || toeplitz_bf16_wgrad_supported(p) || blocked_bf16_wgrad_supported(p))) return true;
    if (p.C <= kBlock && p.K <= kBlock) return false;
    return smallc_wgrad_supported(wgrad_block(p, 0, 0));
}

size_t igemm_wgrad_workspace(const WgradProblem& p) {
    if (!igemm_wgrad_supported(p)) return 0;
    if (prefer_shift_wgrad(p)) return shift_bf16_wgrad_workspace(p);
    if (p.bf16 && toeplitz_bf16_wgrad_supported(p)) return toeplitz_bf16_wgrad_workspace(p);
    if (p.bf16 && blocked_bf16_wgrad_supported(p)) return blocked_bf16_wgrad_workspace(p);
    if (fp32_pairs_in_one_launch(p)) return smallc_wgrad_f32_blocks_workspace(p);
    return smallc_wgrad_workspace(wgrad_block(p, 0, 0));
}

hipError_t igemm_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    if (!igemm_wgrad_supported(p)) return hipErrorInvalidValue;
    if (prefer_shift_wgrad(p)) return shift_bf16_wgrad_launch(p, st);
    if (p.bf16 && toeplitz_bf16_wgrad_supported(p)) return toeplitz_bf16_wgrad_launch(p, st);
    if (p.bf16 && blocked_bf16_wgrad_supported(p)) return blocked_bf16_wgrad_launch(p, st);
    if (fp32_pairs_in_one_launch(p)) return smallc_wgrad_f32_blocks_launch(p, st);
    for (int k0 = 0; k0 < p.K; k0 += kBlock) {
        for (int c0 = 0; c0 < p.C; c0 += kBlock) {
            const WgradProblem b = wgrad_block(p, k0, c0);
            const hipError_t e = smallc_wgrad_launch(b, st);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace conv1d
