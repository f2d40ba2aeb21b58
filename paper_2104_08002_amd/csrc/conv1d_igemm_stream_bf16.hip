// Forward / backward-data passes (Eq. 2; Section 3.2) for bfloat16 inputs, MANY channels with FEW taps (5 to 20)
// and dilations 1, 2, 4, 8, 16: implicit GEMM with streamed weights and shared input operands.
//
//   out[n][m][o] = sum_r sum_s in[n][r][o + s*d - P] * wt(m, r, s)
//
// Layers such as C = K = 256, S = 9 are bound by the bytes a workgroup has to have in flight (memory latency x
// bytes per MFMA), and their weights do not fit in LDS next to useful windows.  This kernel lowers the bytes per
// MFMA: a tile is 32 filters x 1024 output columns (a consumer wave owns 16 position blocks and both filter
// blocks: every window slot and every weight entry feeds twice as many MFMAs as in the staged kernel of
// conv1d_igemm_bf16.hip), which the register-frugal operand walk of conv1d_igemm_ring_bf16.h makes possible:
// k-block kb of a lane = tap 4 jj + kb of tap group jj; the input operand of (position block t, tap group jj) is
// operand number G = alpha t + beta jj, read from LDS once and used for all (t, jj) on its line.
//
// The weights are streamed as in the staged kernel: the entries of a stage (NG planes of 8 channels, all taps, both
// filter blocks) are gathered from raw runs of the [K][C][S] tensor that were parked in LDS one stage earlier.
// Windows and raw runs travel in TWO register sets each, so that every load has two stages to arrive.
// Workgroup = 8 waves: waves 0-3 consume, waves 4-7 produce; one workgroup barrier per stage.  Teams of filter-group
// workgroups share the windows of a strip of tiles through one XCD's L2.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kFB = 2;            // filter blocks of 16 per workgroup
constexpr int kT = 16;            // position blocks of 16 per consumer wave
constexpr int kTW = 4 * kT * 16;  // output columns per tile
constexpr int kMaxWT = 5;         // window tasks per producer thread
constexpr int kMaxWI = 3;         // weight entries per producer thread
constexpr int kMaxRP = 3;         // raw 16-byte pieces per producer thread
constexpr int kQS = 68;           // slots per (plane, tap group, filter block): 4 k-blocks x 17
constexpr int kXD = 5;            // input operands in flight in a consumer wave
constexpr unsigned kPermLo = 0x05040100u;  // {b.lo16, a.lo16} -> a.lo | b.lo << 16
constexpr unsigned kPermHi = 0x07060302u;  // {b.hi16, a.hi16} -> a.hi | b.hi << 16

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct SgArgs {
    const unsigned short* in;
    const unsigned short* wt;
    float* out;
    int N, R, M, Win, Wout, S, P;
    long w_sm, w_sr, in_sn, out_sn;
    int tiles_per_row, nfg, nct, nteams;  // column blocks per row, filter groups, N * tiles_per_row, teams of nfg workgroups
    int NG, ncc;       // planes of 8 channels per stage, stages per tile
    int LP, LPS;       // window positions staged (even), plane stride in slots
    int delta;         // (o0 - P) - window origin: 0 or 1
    int stage_slots;   // NG * LPS + NG * JT * kFB * kQS
    int fwd_mode;      // weights are [m][r][s] (forward) or [r][m][S-1-s] (backward-data)
    int NU, NPc;       // raw runs per stage, 16-byte pieces per run
    long su;           // elements between the starts of consecutive runs
    long wbytes;       // size of the weight tensor
    int raw_slots;     // NU * NPc
    int vec_out;       // output rows and the base pointer are 16-byte aligned
    Epilogue epi;
};

template <int D, int JT>
__global__ __launch_bounds__(512, 2) void igemm_stream_bf16_kernel(SgArgs a) {
    constexpr int U = D == 1 ? 4 : (D == 2 ? 8 : 16);  // positions between consecutive input operands
    constexpr int ALPHA = 16 / U, BETA = 4 * D / U;
    constexpr int GMAX = ALPHA * (kT - 1) + BETA * (JT - 1);
    extern __shared__ u32x4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;
    const int rtid = tid & 255;
    if (!consumer) __builtin_amdgcn_s_setprio(3);
    const int li = lane & 15;
    const int kb = lane >> 4;

    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int team = lid / a.nfg, fg = lid - team * a.nfg;
    const int t_begin = static_cast<int>(static_cast<long>(team) * a.nct / a.nteams);
    const int t_end = static_cast<int>(static_cast<long>(team + 1) * a.nct / a.nteams);
    const int nstages = (t_end - t_begin) * a.ncc;
    const int wbase = a.NG * a.LPS;                 // entries behind the window planes of a stage buffer
    const int nentries = a.NG * JT * kFB * kQS;
    if (nstages <= 0) return;  // the whole workgroup (the plan gives every team at least one tile)

    // zero both entry areas once: the entries of padded taps are never written again
    for (int b = 0; b < 2; ++b)
        for (int e = tid; e < nentries; e += 512) lds4[b * a.stage_slots + wbase + e] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        //   weight operand (plane g, tap group jj, filter block fb): slot wbase + ((g * JT + jj) * 2 + fb) * 68 + 17 kb + li
        //   input operand G of plane g:  slot g * LPS + 256 cw + li + kb d + delta + U G
        const unsigned wlane = 16u * static_cast<unsigned>(wbase + 17 * kb + li);
        const unsigned xlane = 16u * static_cast<unsigned>(cw * (kT * 16) + li + kb * D + a.delta);
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };
        f32x4 acc[kFB][kT];
#pragma unroll
        for (int fb = 0; fb < kFB; ++fb)
#pragma unroll
            for (int t = 0; t < kT; ++t) acc[fb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        // The bias of the lane's filters, loaded once: a load where a tile completes would wait, with the counter
        // the vector memory instructions share, for every output store still in flight.
        float bm[kFB];
#pragma unroll
        for (int fb = 0; fb < kFB; ++fb) {
            const int m = (fg * kFB + fb) * 16 + li;
            bm[fb] = m < a.M ? epi_bias(a.epi, m) : 0.f;
        }

        int tile = t_begin, cc = 0;
        __syncthreads();  // raw weights of stage 0 are in LDS
        __syncthreads();  // stage 0 is in LDS
        for (int st = 0; st < nstages; ++st) {
            const unsigned sb = 16u * static_cast<unsigned>((st & 1) * a.stage_slots);
            for (int g = 0; g < a.NG; ++g) {
                const unsigned xo = sb + xlane + 16u * static_cast<unsigned>(g * a.LPS);
                const unsigned wo = sb + wlane + 16u * static_cast<unsigned>(g * JT * kFB * kQS);
                bf16x8 W[kFB][JT], X[kXD];
#pragma unroll
                for (int jj = 0; jj < JT; ++jj)
#pragma unroll
                    for (int fb = 0; fb < kFB; ++fb) W[fb][jj] = ld(wo + 16u * static_cast<unsigned>((jj * kFB + fb) * kQS));
#pragma unroll
                for (int i = 0; i < kXD - 1; ++i)
                    if (i <= GMAX) X[i] = ld(xo + 16u * U * i);
#pragma unroll
                for (int G = 0; G <= GMAX; ++G) {
                    if (G + kXD - 1 <= GMAX) X[(G + kXD - 1) % kXD] = ld(xo + 16u * U * (G + kXD - 1));
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < kT; ++t) {
                        const int r = G - ALPHA * t;
                        if (r >= 0 && r % BETA == 0 && r / BETA < JT) {
#pragma unroll
                            for (int fb = 0; fb < kFB; ++fb)
                                acc[fb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(X[G % kXD], W[fb][r / BETA], acc[fb][t], 0, 0, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if (++cc == a.ncc) {
                // the tile is complete.  The MFMA operands are swapped (A = input slots, B = weights), so lane
                // (li, kb) holds filter li of each block at the 4 adjacent columns 4 kb .. 4 kb + 3 of each position block
                const int ct = tile;
                const int n = ct / a.tiles_per_row;
                const int o = (ct - n * a.tiles_per_row) * kTW + cw * (kT * 16) + 4 * kb;
                const long base = static_cast<long>(n) * a.out_sn;
#pragma unroll
                for (int fb = 0; fb < kFB; ++fb) {
                    const int m = (fg * kFB + fb) * 16 + li;
                    if (m < a.M) {
                        const long row = base + static_cast<long>(m) * a.Wout + o;
#pragma unroll
                        for (int t = 0; t < kT; ++t) {
                            const f32x4 v = epi_apply4(a.epi, acc[fb][t], bm[fb]);
                            if (a.vec_out && o + 16 * t + 3 < a.Wout) {
                                epi_store4(a.epi, a.out, row + 16 * t, v);
                            } else {
#pragma unroll
                                for (int i = 0; i < 4; ++i)
                                    if (o + 16 * t + i < a.Wout) epi_store(a.epi, a.out, row + 16 * t + i, v[i]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int fb = 0; fb < kFB; ++fb)
#pragma unroll
                    for (int t = 0; t < kT; ++t) acc[fb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
                cc = 0;
                ++tile;
            }
            __syncthreads();
        }
        if (nstages & 1) __syncthreads();  // the producers' loop takes the stages in pairs
    } else {
        // ---- producer side -----------------------------------------------------------------------
        // Window task (plane g, pair i): positions G0 + 2i, G0 + 2i + 1 of the 8 channels of plane g; 8 dword
        // loads (row starts, the window origin and Win are even) from clamped addresses, two slots out.
        // Weights: the runs of a stage are fetched as 16-byte pieces from 4-byte aligned addresses, written as they
        // are into a raw LDS area, and the entries (8 channels of one tap per lane) are gathered from there with
        // 2-byte LDS reads one stage later.
        const int LP2 = a.LP >> 1;
        const int NWT = a.NG * LP2;
        const int NWI = kFB * 16 * a.NG * a.S;
        const int NRP = a.NU * a.NPc;
        const int RSH = a.NPc * 8;  // halfwords per raw run
        const int cs = a.fwd_mode ? a.S : RSH;
        int wt_plane8[kMaxWT], wt_pair[kMaxWT], wt_dst[kMaxWT];
        unsigned wt_voff[kMaxWT];
#pragma unroll
        for (int k = 0; k < kMaxWT; ++k) {
            const int e = min(rtid + k * 256, NWT - 1);
            const int g = e / LP2;
            wt_plane8[k] = 8 * g;
            wt_pair[k] = e - g * LP2;
            wt_voff[k] = 2u * (static_cast<unsigned>(wt_plane8[k]) * static_cast<unsigned>(a.Win) + 2u * static_cast<unsigned>(wt_pair[k]));
            wt_dst[k] = g * a.LPS + 2 * wt_pair[k];
        }
        int rp_u[kMaxRP], rp_q[kMaxRP];
#pragma unroll
        for (int k = 0; k < kMaxRP; ++k) {
            const int e = min(rtid + k * 256, NRP - 1);
            rp_u[k] = e / a.NPc;
            rp_q[k] = e - rp_u[k] * a.NPc;
        }
        int wi_idx0[kMaxWI], wi_lds[kMaxWI], wi_g8[kMaxWI], wi_par[kMaxWI], wi_ml[kMaxWI];
#pragma unroll
        for (int k = 0; k < kMaxWI; ++k) {
            const int e = min(rtid + k * 256, NWI - 1);
            const int sx = e % a.S, mg = e / a.S;
            const int g = mg % a.NG, ml = mg / a.NG;
            if (a.fwd_mode) {
                wi_idx0[k] = ml * RSH + 8 * g * a.S + sx;
                const int pm = static_cast<int>((ml * a.w_sm) & 1);
                wi_par[k] = pm | (pm << 1);
            } else {
                wi_idx0[k] = 8 * g * RSH + ml * a.S + (a.S - 1 - sx);
                wi_par[k] = static_cast<int>(a.w_sr & 1) << 1;  // runs of odd channels start at the other parity
            }
            wi_lds[k] = ((g * JT + (sx >> 2)) * kFB + (ml >> 4)) * kQS + 17 * (sx & 3) + (ml & 15);
            wi_g8[k] = 8 * g;
            wi_ml[k] = ml;
        }
        const int m0 = fg * kFB * 16;
        struct Geo {
            int n, G0, r0;  // sample, window origin, first channel of the stage
        };
        // The geometry of stage st + k follows from that of stage st (sample n0, column block tc0, channel chunk cc0)
        // by counting: no integer divisions in the loop (the producers share their SIMDs' issue slots with the
        // MFMA waves, and a division is ~40 instructions).
        int n0 = t_begin / a.tiles_per_row, tc0 = t_begin - n0 * a.tiles_per_row, cc0 = 0, st0 = 0;
        auto geo = [&](int st) -> Geo {
            int cc = cc0 + (st - st0), tc = tc0, n = n0;
            while (cc >= a.ncc) {
                cc -= a.ncc;
                if (++tc == a.tiles_per_row) {
                    tc = 0;
                    ++n;
                }
            }
            // a stage behind the current one: with an odd number of stages the last pass asks for the (clamped) last
            // stage after the counters have moved on to the tile behind it, which may lie in a sample that does not exist
            while (cc < 0) {
                cc += a.ncc;
                if (tc-- == 0) {
                    tc = a.tiles_per_row - 1;
                    --n;
                }
            }
            Geo g;
            g.n = n;
            g.G0 = tc * kTW - a.P - a.delta;
            g.r0 = cc * a.NG * 8;
            return g;
        };
        auto advance = [&]() {  // st0 -> st0 + 1
            ++st0;
            if (++cc0 == a.ncc) {
                cc0 = 0;
                if (++tc0 == a.tiles_per_row) {
                    tc0 = 0;
                    ++n0;
                }
            }
        };
        auto interior = [&](const Geo& g) { return g.G0 >= 0 && g.G0 + a.LP <= a.Win && g.r0 + 8 * a.NG <= a.R; };
        unsigned wreg[2][kMaxWT][8];
        u32x4 rreg[2][kMaxRP];
        // Every path through the loop issues the same loads in the same order (stages past the end repeat the last
        // one, tasks past the end repeat the last task, addresses are clamped instead of branched around): only then
        // does the compiler count the loads that may still be in flight when a register set is used, instead of
        // waiting for all of them, and only then do two register sets buy two stages of latency.
        auto window_prefetch = [&](int st, unsigned (&wr)[kMaxWT][8]) {
            const Geo g = geo(min(st, nstages - 1));
            const char* ib = reinterpret_cast<const char*>(a.in + static_cast<long>(g.n) * a.in_sn);
            const unsigned rowb = static_cast<unsigned>(a.Win) * 2u;
#pragma unroll
            for (int k = 0; k < kMaxWT; ++k) {
                int pos = g.G0 + 2 * wt_pair[k];
                pos = pos < 0 ? 0 : (pos > a.Win - 2 ? a.Win - 2 : pos);
                const unsigned offmax = static_cast<unsigned>((a.R - 1) * a.Win + pos) * 2u;
                unsigned off = static_cast<unsigned>((g.r0 + wt_plane8[k]) * a.Win + pos) * 2u;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    wr[k][j] = *reinterpret_cast<const unsigned*>(ib + min(off, offmax));
                    off += rowb;
                }
            }
        };
        auto window_commit = [&](int st, unsigned (&wr)[kMaxWT][8]) {
            if (st >= nstages) return;
            const Geo g = geo(st);
            u32x4* win = lds4 + (st & 1) * a.stage_slots;
            const bool inner = interior(g);
#pragma unroll
            for (int k = 0; k < kMaxWT; ++k)
                if (rtid + k * 256 < NWT) {
                    const int pos = g.G0 + 2 * wt_pair[k];
                    const bool ok = inner || (pos >= 0 && pos < a.Win);  // a pair is inside or outside the row as a whole
                    u32x4 ev, od;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const unsigned lo = ok ? wr[k][2 * q] : 0u, hi = ok ? wr[k][2 * q + 1] : 0u;
                        ev[q] = __builtin_amdgcn_perm(hi, lo, kPermLo);
                        od[q] = __builtin_amdgcn_perm(hi, lo, kPermHi);
                    }
                    u32x4* dst = win + wt_dst[k];
                    dst[0] = ev;
                    dst[1] = od;
                }
        };
        // element offset of the stage's first run from the tensor base
        auto stage_base = [&](int r0) -> long { return static_cast<long>(m0) * a.w_sm + static_cast<long>(r0) * a.w_sr; };
        auto raw_prefetch = [&](int st, u32x4 (&rr)[kMaxRP]) {
            const int r0 = geo(min(st, nstages - 1)).r0;
            const unsigned eb = static_cast<unsigned>(stage_base(r0));  // the tensor has fewer than 2^31 elements
            const int umax = a.fwd_mode ? a.M - 1 - m0 : a.R - 1 - r0;
            const char* wb = reinterpret_cast<const char*>(a.wt);
            const unsigned su = static_cast<unsigned>(a.su);
            const unsigned last_dw = static_cast<unsigned>(a.wbytes - 2) & ~3u;  // the last dword that holds an element
#pragma unroll
            for (int k = 0; k < kMaxRP; ++k) {
                const unsigned eu = eb + static_cast<unsigned>(max(0, min(rp_u[k], umax))) * su;
                const unsigned B = ((eu * 2u) & ~3u) + 16u * static_cast<unsigned>(rp_q[k]);
#pragma unroll
                for (int i = 0; i < 4; ++i) rr[k][i] = *reinterpret_cast<const unsigned*>(wb + min(B + 4u * i, last_dw));
            }
        };
        // raw runs of stage st -> raw buffer st & 1
        auto raw_commit = [&](int st, const u32x4 (&rr)[kMaxRP]) {
            if (st >= nstages) return;
            u32x4* raw = lds4 + 2 * a.stage_slots + (st & 1) * a.raw_slots;
#pragma unroll
            for (int k = 0; k < kMaxRP; ++k)
                if (rtid + k * 256 < NRP) raw[rp_u[k] * a.NPc + rp_q[k]] = rr[k];
        };
        // entries of stage st: raw buffer st & 1 -> stage buffer st & 1
        auto gather = [&](int st) {
            if (st >= nstages) return;
            const unsigned short* raw = reinterpret_cast<const unsigned short*>(lds4 + 2 * a.stage_slots + (st & 1) * a.raw_slots);
            u32x4* wgt = lds4 + (st & 1) * a.stage_slots + wbase;
            const int r0 = geo(st).r0;
            const int pb = static_cast<int>(stage_base(r0) & 1);
            unsigned v[kMaxWI][8];
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (k * 256 < NWI) {
                    const int ie = wi_idx0[k] + (pb ^ (wi_par[k] & 1)), io = wi_idx0[k] + (pb ^ (wi_par[k] >> 1));
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[k][j] = raw[((j & 1) ? io : ie) + j * cs];
                }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (rtid + k * 256 < NWI) {
                    const int nv = m0 + wi_ml[k] < a.M ? a.R - r0 - wi_g8[k] : 0;  // channels that exist
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[k][j] = j < nv ? v[k][j] : 0u;
                    wgt[wi_lds[k]] = u32x4{v[k][0] | (v[k][1] << 16), v[k][2] | (v[k][3] << 16), v[k][4] | (v[k][5] << 16), v[k][6] | (v[k][7] << 16)};
                }
        };
        // Stage st: its window travels in window set st & 1, its raw runs in raw set st & 1.  While the consumers
        // work on stage st the producers write window st + 1 and request window st + 3, park the raw runs of stage
        // st + 2 and request those of stage st + 4, and gather the entries of stage st + 1.  Commits come before
        // requests, so that no wait for an old set can cover a request just made.
        // The loads before the loop end in the order in which a pass through the loop leaves them.
        window_prefetch(0, wreg[0]);
        raw_prefetch(0, rreg[0]);
        raw_prefetch(1, rreg[1]);
        raw_commit(0, rreg[0]);
        __syncthreads();
        gather(0);
        window_commit(0, wreg[0]);
        raw_prefetch(2, rreg[0]);
        window_prefetch(1, wreg[1]);
        raw_commit(1, rreg[1]);
        raw_prefetch(3, rreg[1]);
        window_prefetch(2, wreg[0]);
        __syncthreads();
        for (int st = 0; st < nstages; st += 2) {
            // consumers on stage st (even)
            window_commit(st + 1, wreg[1]);
            raw_commit(st + 2, rreg[0]);
            raw_prefetch(st + 4, rreg[0]);
            window_prefetch(st + 3, wreg[1]);
            gather(st + 1);
            advance();
            __syncthreads();
            // consumers on stage st + 1 (odd; with an odd number of stages they meet this barrier after their loop)
            window_commit(st + 2, wreg[0]);
            raw_commit(st + 3, rreg[1]);
            raw_prefetch(st + 5, rreg[1]);
            window_prefetch(st + 4, wreg[0]);
            gather(st + 2);
            advance();
            __syncthreads();
        }
    }
}

struct SgPlan {
    bool ok;
    int D, JT, grid;
    size_t lds_bytes;
    SgArgs a;
};

SgPlan sg_plan(const CorrProblem& p) {
    SgPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.accumulate) return pl;
    if (p.M <= 16 || p.R <= 16) return pl;
    if (p.d != 1 && p.d != 2 && p.d != 4 && p.d != 8 && p.d != 16) return pl;
    if (p.S < 5 || p.S > 20) return pl;
    if ((p.Win & 1) || (p.in_sn & 1) || (reinterpret_cast<uintptr_t>(p.in) & 3) || p.Win < 2) return pl;
    if (reinterpret_cast<uintptr_t>(p.wt) & 3) return pl;
    const bool fwd_mode = p.w_ss == 1 && p.w_sr == p.S && p.w_s0 == 0;
    const bool bwd_mode = p.w_ss == -1 && p.w_sm == p.S && p.w_s0 == p.S - 1;
    if (!fwd_mode && !bwd_mode) return pl;
    if (static_cast<long>(p.R) * p.Win >= (1L << 30)) return pl;
    if (static_cast<long>(p.M) * p.R * p.S >= (1L << 31) || p.M * p.w_sm >= (1L << 31) || p.R * p.w_sr >= (1L << 31)) return pl;
    const int JT = p.S <= 8 ? 2 : (p.S <= 12 ? 3 : 5);
    SgArgs& a = pl.a;
    a.in = static_cast<const unsigned short*>(p.in);
    a.wt = static_cast<const unsigned short*>(p.wt);
    a.out = p.out;
    a.epi = p.epi;
    a.N = p.N; a.R = p.R; a.M = p.M; a.Win = p.Win; a.Wout = p.Wout; a.S = p.S; a.P = p.P;
    a.w_sm = p.w_sm; a.w_sr = p.w_sr; a.in_sn = p.in_sn; a.out_sn = p.out_sn;
    a.delta = (p.P & 1) ? 1 : 0;
    const long halo = static_cast<long>(4 * JT - 1) * p.d;
    const long LP = (kTW + halo + a.delta + 1) / 2 * 2;
    const long LPS = LP + 8;
    const int planes = cdiv(p.R, 8);
    for (int NG = 4; NG >= 1; NG /= 2) {
        if (NG > 1 && NG / 2 >= planes) continue;
        if (cdiv(NG * (LP / 2), 256) > kMaxWT) continue;
        if (cdiv(static_cast<long>(kFB) * 16 * NG * p.S, 256) > kMaxWI) continue;
        const int NU = fwd_mode ? kFB * 16 : 8 * NG;
        const long L = fwd_mode ? 8L * NG * p.S : static_cast<long>(kFB) * 16 * p.S;
        const long NPc = (2 * L + 2 + 15) / 16;
        if (cdiv(NU * NPc, 256) > kMaxRP) continue;
        const long stage = NG * LPS + static_cast<long>(NG) * JT * kFB * kQS;
        const size_t bytes = static_cast<size_t>(2 * stage + 2 * NU * NPc) * 16;
        if (bytes > static_cast<size_t>(kLdsBudget)) continue;
        pl.D = p.d; pl.JT = JT;
        a.NG = NG;
        a.ncc = cdiv(planes, NG);
        a.LP = static_cast<int>(LP);
        a.LPS = static_cast<int>(LPS);
        a.stage_slots = static_cast<int>(stage);
        a.fwd_mode = fwd_mode;
        a.NU = NU;
        a.NPc = static_cast<int>(NPc);
        a.raw_slots = static_cast<int>(NU * NPc);
        a.su = fwd_mode ? p.w_sm : p.w_sr;
        a.wbytes = (fwd_mode ? static_cast<long>(p.M) * p.w_sm : static_cast<long>(p.R) * p.w_sr) * 2;
        a.vec_out = (p.Wout % 4 == 0) && (p.out_sn % 4 == 0) && (reinterpret_cast<uintptr_t>(p.out) % 16 == 0);
        a.tiles_per_row = cdiv(p.Wout, kTW);
        a.nfg = cdiv(p.M, kFB * 16);
        const long nct = static_cast<long>(p.N) * a.tiles_per_row;
        if (nct > 0x7fffffffL / 64 || a.nfg > 65535) return pl;
        a.nct = static_cast<int>(nct);
        // The staged kernel's tiles are half as wide, and it is the faster one while the tiles of this kernel would
        // leave half of the CUs idle (measured at C = K = 256: N = 8, W = 2048, S = 9: 54 us against 41 us; N = 4,
        // W = 8192, S = 9: 57 us against 72 us; N = 8, W = 4096, S = 17: 90 us against 118 us)
        if (nct * a.nfg <= kNumCU / 2) return pl;
        const int fit = kNumCU / a.nfg > 0 ? kNumCU / a.nfg : 1;  // teams that run at the same time
        a.nteams = a.nct < fit ? a.nct : fit;
        pl.grid = a.nteams * a.nfg;
        pl.lds_bytes = bytes;
        pl.ok = true;
        return pl;
    }
    return pl;
}

template <int D, int JT>
hipError_t sg_launch(const SgPlan& pl, hipStream_t st) {
    auto kern = igemm_stream_bf16_kernel<D, JT>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

template <int D>
hipError_t sg_launch_d(const SgPlan& pl, hipStream_t st) {
    switch (pl.JT) {
        case 2: return sg_launch<D, 2>(pl, st);
        case 3: return sg_launch<D, 3>(pl, st);
        case 5: return sg_launch<D, 5>(pl, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool igemm_stream_bf16_corr_supported(const CorrProblem& p) { return sg_plan(p).ok; }

hipError_t igemm_stream_bf16_corr_launch(const CorrProblem& p, hipStream_t st) {
    const SgPlan pl = sg_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    switch (pl.D) {
        case 1: return sg_launch_d<1>(pl, st);
        case 2: return sg_launch_d<2>(pl, st);
        case 8: return sg_launch_d<8>(pl, st);
        case 16: return sg_launch_d<16>(pl, st);
        case 4: return sg_launch_d<4>(pl, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace conv1d
