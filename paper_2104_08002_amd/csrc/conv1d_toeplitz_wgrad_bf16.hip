// Backward-weight pass (Section 3.3, Algorithm 4), bfloat16, dilations 1, 2, 4, 8, 16: launch plan, second stage
// and dispatch of the register-ring kernels (the kernel template and its description are in the header; every
// dilation is instantiated in a translation unit of its own).
#include "conv1d_toeplitz_wgrad_bf16.h"

namespace conv1d {

namespace {

using tz::TzArgs;
using tz::TzPlan;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Adds the strips in a fixed order (16 interleaved running sums per element, then those 16 in order) and
// scatters the tiles into dw[k][c][s].  A block of 16 x 16 threads handles 64 consecutive tile elements: thread
// (g, el) adds the strips g, g + 16, ... of the 4 elements 4 el .. 4 el + 3 with 16-byte loads.  The tile size is
// a multiple of 256, so a block never straddles two combinations.
__global__ __launch_bounds__(256) void toeplitz_wgrad_reduce_kernel(const float* __restrict__ ws, float* __restrict__ dw, TzArgs a, int FB, int NTW) {
    __shared__ f32x4 part[16][17];
    const int el = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int tile = 4 * FB * NTW * 256;
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const long idx = static_cast<long>(blockIdx.x) * 64 + 4 * el;  // (combo, tile element)
    const int combo = static_cast<int>(idx / tile), e = static_cast<int>(idx - static_cast<long>(combo) * tile);
    f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
    if (combo < ncombos)
        for (int s = g; s < a.nstrips; s += 16) sum += *reinterpret_cast<const f32x4*>(ws + (static_cast<long>(s) * ncombos + combo) * tile + e);
    part[g][el] = sum;
    __syncthreads();
    if (g == 0 && combo < ncombos) {
        f32x4 t = part[0][el];
#pragma unroll
        for (int j = 1; j < 16; ++j) t += part[j][el];
        // the 4 elements are the filters 4 (l >> 4) .. + 3 of one (block, tap, channel)
        const int tg = combo % a.ntg, cbi = (combo / a.ntg) % a.ncb, fg = combo / (a.ntg * a.ncb);
        const int blk = e >> 8, l = (e & 255) >> 2;
        const int i = blk % NTW, fb = (blk / NTW) % FB, v = blk / (NTW * FB);
        const int k0 = (fg * FB + fb) * 16 + 4 * (l >> 4), c = cbi * 16 + (l & 15), s = tg * 4 * NTW + v + 4 * i;
        if (c < a.C && s < a.S) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (k0 + jj < a.K) dw[(static_cast<long>(k0 + jj) * a.C + c) * a.S + s] = t[jj];
        }
    }
}

template <int D, int NTW>
bool tz_geometry(const WgradProblem& p, int FB, TzPlan& pl) {
    using G = tz::Tz<D, NTW>;
    TzArgs& a = pl.a;
    a.ntg = cdiv(p.S, 4 * NTW);
    a.nfg = cdiv(cdiv(p.K, 16), FB);
    a.ncb = cdiv(p.C, 16);
    // phases in use: (E0 + v d + 4 q) & 7 over the waves, classes and tap groups
    a.phase_mask = 0;
    for (int tg = 0; tg < a.ntg; ++tg)
        for (int v = 0; v < 4; ++v)
            for (int q = 0; q < G::NQ; ++q) a.phase_mask |= 1u << ((static_cast<long>(tg * 4 * NTW + v) * D - p.P + 4 * q) & 7);
    const int ncopies = __builtin_popcount(a.phase_mask);
    a.gmask = 0;
    for (int g = 0; g < 4; ++g)
        if ((a.phase_mask >> (2 * g)) & 3u) a.gmask |= 1u << g;
    const int ng = __builtin_popcount(a.gmask);
    if (ng != G::NG) return false;
    if (cdiv(FB * 16 * 4 * G::LU, 256) > tz::kMaxY) return false;
    if (cdiv(16 * G::NXS, 256) * ng > tz::kMaxI) return false;
    a.RSY = 4 * G::LU + 1;
    a.RSX = G::NXS | 1;
    a.RSXP = G::NXP | 1;
    a.xcopy_slots = 16 * a.RSX;
    a.pcopy_slots = 16 * a.RSXP;
    a.ybuf_slots = FB * 16 * a.RSY;
    a.stage_slots = a.ybuf_slots + ncopies * a.xcopy_slots;
    if (ncopies * a.pcopy_slots > a.stage_slots) return false;  // the first fill borrows buffer 1
    // + slack for the reads that run ahead of the last k-step
    pl.lds_bytes = static_cast<size_t>(2 * a.stage_slots + 8) * 16;
    if (pl.lds_bytes > static_cast<size_t>(tz::kLdsBudget)) return false;
    const int QB = 32 * G::LU * G::NB;  // columns per body
    a.BPR = cdiv(p.Q, QB);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const long total_bodies = static_cast<long>(p.N) * a.BPR;
    long want = tz::kNumCU / ncombos;  // strips
    if (want < 1) want = 1;
    long bps = (total_bodies + want - 1) / want;
    if (bps < 1) bps = 1;
    if (bps > a.BPR) bps = a.BPR;
    a.BPS = static_cast<int>(bps);
    a.SPR = cdiv(a.BPR, a.BPS);
    const long nstrips = static_cast<long>(p.N) * a.SPR;
    const long grid = nstrips * ncombos;
    if (grid > 0x7fffffffL) return false;
    a.nstrips = static_cast<int>(nstrips);
    pl.grid = static_cast<int>(grid);
    pl.tile = 4 * FB * NTW * 256;
    return true;
}

template <int NTW>
bool tz_geometry_d(const WgradProblem& p, int FB, TzPlan& pl) {
    switch (p.d) {
        case 1: return tz_geometry<1, NTW>(p, FB, pl);
        case 2: return tz_geometry<2, NTW>(p, FB, pl);
        case 4: return tz_geometry<4, NTW>(p, FB, pl);
        case 8: return tz_geometry<8, NTW>(p, FB, pl);
        case 16: return tz_geometry<16, NTW>(p, FB, pl);
        default: return false;
    }
}

TzPlan tz_plan(const WgradProblem& p) {
    TzPlan pl{};
    pl.ok = false;
    if (!p.bf16) return pl;
    if (p.d != 1 && p.d != 2 && p.d != 4 && p.d != 8 && p.d != 16) return pl;
    if (p.dw_sc != p.S || p.dw_sk != static_cast<long>(p.C) * p.S) return pl;  // writes the whole dw tensor
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    if (static_cast<long>(p.K) * p.C * p.S >= (1L << 31)) return pl;
    // taps per wave: the fewest MFMA slots (a tap group is padded to 4 NTW taps); with too many of them
    // wasted the blocked kernel, whose tap groups are finer, is the better choice
    int best = 0, best_slots = 0;
    for (int ntw : tz::kNTWs) {
        const int slots = cdiv(p.S, 4 * ntw) * 4 * ntw;
        if (best == 0 || slots < best_slots) { best = ntw; best_slots = slots; }
    }
    // Few taps: small layers are bound by memory latency, not by MFMA slots, and this kernel's deeper request
    // queue wins; layers with many channel and filter blocks are bound by the bytes staged per MFMA, where the
    // blocked kernel's larger tiles win (measured on C = K = 256, S = 9: 623 us against 465 us).
    if (best == 0) return pl;
    if (20 * best_slots > 29 * p.S && (best_slots > 12 || cdiv(p.C, 16) * cdiv(p.K, 16) > 16)) return pl;
    if (best < 5 && cdiv(p.C, 16) * cdiv(p.K, 16) > 16) return pl;
    if (best == 2 && p.d == 1) return pl;  // 8 phase copies for 2 taps per wave: the blocked kernel is faster (53 us against 61 us)
    pl.D = p.d;
    pl.NTW = best;
    bool ok = false;
    auto geometry = [&](int FB) {
        pl.FB = FB;
        switch (best) {
            case 13: return tz_geometry_d<13>(p, FB, pl);
            case 9: return tz_geometry_d<9>(p, FB, pl);
            case 5: return tz_geometry_d<5>(p, FB, pl);
            case 3: return tz_geometry_d<3>(p, FB, pl);
            case 2: return tz_geometry_d<2>(p, FB, pl);
            default: return false;
        }
    };
    for (int FB = p.K > 16 ? 2 : 1; FB >= 1 && !ok; --FB) ok = geometry(FB);
    if (!ok) return pl;
    TzArgs& a = pl.a;
    a.x = static_cast<const unsigned short*>(p.x);
    a.dy = static_cast<const unsigned short*>(p.dy);
    a.ws = static_cast<float*>(p.ws);
    a.C = p.C; a.K = p.K; a.W = p.W; a.Q = p.Q; a.S = p.S; a.P = p.P;
    a.x_sn = p.x_sn; a.dy_sn = p.dy_sn;
    pl.fast = (p.W >= 8) && (p.Q >= 8) && (p.W % 2 == 0) && (p.Q % 2 == 0) && (p.x_sn % 2 == 0) && (p.dy_sn % 2 == 0) &&
              (reinterpret_cast<uintptr_t>(p.x) % 4 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 4 == 0);
    pl.ok = true;
    return pl;
}

}  // namespace

bool toeplitz_bf16_wgrad_supported(const WgradProblem& p) { return tz_plan(p).ok; }

size_t toeplitz_bf16_wgrad_workspace(const WgradProblem& p) {
    const TzPlan pl = tz_plan(p);
    return pl.ok ? static_cast<size_t>(pl.grid) * pl.tile * sizeof(float) : 0;
}

hipError_t toeplitz_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const TzPlan pl = tz_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e;
    switch (pl.D) {
        case 1: e = tz::launch_d1(pl, st); break;
        case 2: e = tz::launch_d2(pl, st); break;
        case 4: e = tz::launch_d4(pl, st); break;
        case 8: e = tz::launch_d8(pl, st); break;
        case 16: e = tz::launch_d16(pl, st); break;
        default: e = hipErrorInvalidValue; break;
    }
    if (e != hipSuccess) return e;
    const long nel = static_cast<long>(pl.grid / pl.a.nstrips) * pl.tile;
    return launch_kernel(toeplitz_wgrad_reduce_kernel, dim3(cdiv(nel, 64)), dim3(256), 0, st, static_cast<const float*>(p.ws), p.dw, pl.a, pl.FB,
                       pl.NTW);
}

}  // namespace conv1d
