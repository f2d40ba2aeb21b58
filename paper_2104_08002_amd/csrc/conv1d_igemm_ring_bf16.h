// Forward / backward-data passes (Eq. 2; Section 3.2) for bfloat16 inputs, many channels (R or M > 16) and
// dilations 1, 2, 4, 8, 16: implicit GEMM with resident weights and shared input operands.
//
//   out[n][m][o] = sum_r sum_s in[n][r][o + s*d - P] * wt(m, r, s)
//
// One v_mfma_f32_16x16x32_bf16 contracts four k-blocks (8 channels of one tap each): lane (li, kb) holds filter li
// (A operand) or output column li (B operand) of k-block kb = tap 4 jj + kb of tap group jj, for one plane of 8
// channels.  Two things differ from the staged implicit GEMM of conv1d_igemm_bf16.hip:
//
// Resident weights.  A workgroup owns FB blocks of 16 filters and keeps their operand entries for ALL channels and
// taps in LDS for its whole life (entry (plane, tap group, filter block, lane) = 16 bytes); they are gathered
// once, in the prologue, from the [K][C][S] tensor as it is.  The producers then only stage input windows.
//
// Shared input operands.  The B operand of (position block t, tap group jj) starts at window position
// 16 t + 4 d jj (+ li + kb d): with u = gcd(16, 4 d), alpha = 16 / u and beta = 4 d / u it is operand number
// G = alpha t + beta jj.  A consumer wave owns 8 position blocks and walks G upwards: every operand is read from
// LDS once and feeds all (t, jj) on its line, acc[t] += W[jj] * X[G]; the weight operands of a plane sit in
// registers and are replaced by the next plane's as they fall out of use.  LDS operand reads per MFMA drop from
// 0.62 to 0.2 - 0.4.
//
// Tile = 16 FB filters x 64 KT output columns of one sample (KT = 8 or 5); consumer wave v takes KT position blocks.
// The reduction runs in stages of NG planes; the window of a stage is double-buffered as [plane][position] 16-byte
// slots (8 channels at one position).  Workgroup = 8 waves, persistent over a strip of tiles: waves 0-3 consume,
// waves 4-7 stage the windows of the next stages; one workgroup barrier per stage.  Workgroups of the filter
// groups of one strip form a team on one XCD (the window is fetched from HBM once).
// Taps beyond S (the last tap group) have zero weights.
#pragma once
#include <type_traits>

#include "conv1d_internal.h"

namespace conv1d {

namespace rg {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;

constexpr int kMaxWT = 5;         // window tasks per producer thread
constexpr int kMaxWI = 4;         // weight entries per thread and chunk (prologue, 512 threads)
constexpr int kMaxRP = 3;         // raw 16-byte pieces per thread and chunk
constexpr int kMaxDE = 8;         // weight entries per thread of the direct prologue
constexpr int kQS = 68;           // slots per (plane, tap group, filter block): 4 k-blocks x 17
constexpr int kBufferRsrcFlags = 0x00020000;  // fourth dword of a raw buffer descriptor (32-bit data format, no swizzle)
constexpr unsigned kPermLo = 0x05040100u;  // {b.lo16, a.lo16} -> a.lo | b.lo << 16
constexpr unsigned kPermHi = 0x07060302u;  // {b.hi16, a.hi16} -> a.hi | b.hi << 16

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct RgArgs {
    const unsigned short* in;
    const unsigned short* wt;
    float* out;
    int N, R, M, Win, Wout, S, P;
    long w_sm, w_sr, in_sn, out_sn;
    int tiles_per_row, nfg, nct, nteams;  // column blocks per row, filter groups, N * tiles_per_row, teams of nfg workgroups
    int NG, ncc;       // planes of 8 channels per stage, stages per tile
    int NGW;           // planes per chunk of the weight prologue (divides NG * ncc)
    int LP, LPS;       // window positions staged (even), plane stride in slots
    int delta;         // (o0 - P) - window origin: 0 or 1
    int win_slots;     // NG * LPS
    int wres_slots;    // ncc * NG * JT * FB * kQS: the resident weight entries
    int fwd_mode;      // weights are [m][r][s] (forward) or [r][m][S-1-s] (backward-data)
    int NU, NPc;       // raw runs per chunk, 16-byte pieces per run
    long su;           // elements between the starts of consecutive runs
    long wbytes;       // size of the weight tensor
    int raw_slots;     // NU * NPc
    int t_base, t_rem; // tiles per team: t_base, and one more for the first t_rem teams
    FastDiv dv_nfg, dv_tpr, dv_ncc, dv_lp2, dv_npc, dv_s, dv_ngw;  // nfg, tiles_per_row, ncc, LP / 2, NPc, S, NGW
    FastDiv dv_pl;     // ncc * NG
    int direct;        // few weights: every thread loads its entries straight from the tensor (no raw buffers)
    int vec_out;       // output rows and the base pointer are 16-byte aligned
    Epilogue epi;
};

// operand geometry of a dilation
template <int D>
struct Ring {
    static constexpr int U = D == 1 ? 4 : (D == 2 ? 8 : 16);  // positions between consecutive operands
    static constexpr int ALPHA = 16 / U;
    static constexpr int BETA = 4 * D / U;
    static constexpr int XD = 5;  // input operands in flight: the reads run 4 steps (8 - 32 MFMAs) ahead of their use
};

template <int D, int FB, int JT, int KT>
__global__ __launch_bounds__(512, 2) void igemm_ring_bf16_kernel(RgArgs a) {
    constexpr int kT = KT, kTW = 64 * KT;
    using G_ = Ring<D>;
    constexpr int ALPHA = G_::ALPHA, BETA = G_::BETA, XD = G_::XD;
    constexpr int GMAX = ALPHA * (kT - 1) + BETA * (JT - 1);
    extern __shared__ u32x4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;
    const int rtid = tid & 255;
    const int li = lane & 15;
    const int kb = lane >> 4;

    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int team = fast_div(lid, a.dv_nfg), fg = lid - team * a.nfg;
    const int t_begin = team * a.t_base + min(team, a.t_rem);
    const int t_end = t_begin + a.t_base + (team < a.t_rem ? 1 : 0);
    const int nstages = (t_end - t_begin) * a.ncc;
    if (nstages <= 0) return;  // the whole workgroup (the plan gives every team at least one tile)

    const int wbase = a.wres_slots;  // the two window buffers follow the resident weights

    // ---- window staging (producer waves): tables, and the first window requested before the prologue ----
    // Window task (plane g, pair i): positions G0 + 2i, G0 + 2i + 1 of the 8 channels of plane g; 8 dword
    // loads (row starts, the window origin and Win are even) from clamped addresses, two slots out.
    const int LP2 = a.LP >> 1;
    const int NWT = a.NG * LP2;
    int wt_plane8[kMaxWT], wt_pair[kMaxWT], wt_dst[kMaxWT];
    unsigned wt_off[kMaxWT];  // byte offset of the task's first load from that of (channel r0, position G0)
#pragma unroll
    for (int k = 0; k < kMaxWT; ++k) {
        const int e = min(rtid + k * 256, NWT - 1);
        const int g = fast_div(e, a.dv_lp2);
        wt_plane8[k] = 8 * g;
        wt_pair[k] = e - g * LP2;
        wt_dst[k] = g * a.LPS + 2 * wt_pair[k];
        wt_off[k] = static_cast<unsigned>(8 * g * a.Win + 2 * wt_pair[k]) * 2u;
    }
    struct Geo {
        int n, G0, r0;  // sample, window origin, first channel of the stage
    };
    auto geo = [&](int st) -> Geo {
        const int tq = fast_div(st, a.dv_ncc);
        const int ct = t_begin + tq, cc = st - tq * a.ncc;
        Geo g;
        g.n = fast_div(ct, a.dv_tpr);
        g.G0 = (ct - g.n * a.tiles_per_row) * kTW - a.P - a.delta;
        g.r0 = cc * a.NG * 8;
        return g;
    };
    auto interior = [&](const Geo& g) { return g.G0 >= 0 && g.G0 + a.LP <= a.Win && g.r0 + 8 * a.NG <= a.R; };
    unsigned wreg[2][kMaxWT][8];
    // The task count is a compile-time number and every path issues the same loads (tasks and stages past the end
    // repeat the last one, edge addresses are clamped instead of branched around): only then does the compiler
    // count the loads that may still be in flight when a register set is used, instead of waiting for all of
    // them, and only then do two register sets buy two stages of memory latency.
    auto window_prefetch = [&](auto nt_, const Geo& g, unsigned (&wr)[kMaxWT][8]) {
        constexpr int NT = decltype(nt_)::value;
        const char* ib = reinterpret_cast<const char*>(a.in + static_cast<long>(g.n) * a.in_sn);
        const unsigned rowb = static_cast<unsigned>(a.Win) * 2u;
        if (interior(g)) {
            // Nothing to clamp: buffer loads from the sample's [R][Win] block, whose address is a per-thread offset
            // that never changes plus a scalar offset (stage origin, row) - no vector instruction per load.  (The
            // range check of the descriptor is not relied upon: every address is inside the block.)
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(ib), 0, a.R * static_cast<int>(rowb), kBufferRsrcFlags);
            const int so = g.r0 * static_cast<int>(rowb) + 2 * g.G0;
#pragma unroll
            for (int k = 0; k < NT; ++k) {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    wr[k][j] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, static_cast<int>(wt_off[k]), so + j * static_cast<int>(rowb), 0);
            }
            return;
        }
#pragma unroll
        for (int k = 0; k < NT; ++k) {
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
    auto window_commit = [&](const Geo& g, int b, unsigned (&wr)[kMaxWT][8]) {
        u32x4* win = lds4 + wbase + b * a.win_slots;
        if (interior(g)) {  // nothing to mask
#pragma unroll
            for (int k = 0; k < kMaxWT; ++k)
                if (rtid + k * 256 < NWT) {
                    u32x4 ev, od;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        ev[q] = __builtin_amdgcn_perm(wr[k][2 * q + 1], wr[k][2 * q], kPermLo);
                        od[q] = __builtin_amdgcn_perm(wr[k][2 * q + 1], wr[k][2 * q], kPermHi);
                    }
                    u32x4* dst = win + wt_dst[k];
                    dst[0] = ev;
                    dst[1] = od;
                }
            return;
        }
#pragma unroll
        for (int k = 0; k < kMaxWT; ++k)
            if (rtid + k * 256 < NWT) {
                const int pos = g.G0 + 2 * wt_pair[k];
                const bool ok = pos >= 0 && pos < a.Win;  // a pair is inside or outside the row as a whole
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
    Geo g0 = geo(0), g1 = geo(1 < nstages ? 1 : 0), g2 = g1;
    // The only weight entries no gather writes are those of the taps S .. 4 JT - 1 that pad the last tap groups:
    // they must be zero (they multiply real input positions), everything else is written (masked where a channel or
    // a filter does not exist) before it is read.
    auto zero_padded_taps = [&]() {
        const int nrows = a.ncc * a.NG * FB * 16;  // (plane, filter block, filter)
        for (int t = a.S; t < 4 * JT; ++t)
            for (int idx = tid; idx < nrows; idx += 512) {
                const int fbg = idx >> 4, g = fbg / FB, fb = fbg - g * FB;
                lds4[((g * JT + (t >> 2)) * FB + fb) * kQS + 17 * (t & 3) + (idx & 15)] = u32x4{0u, 0u, 0u, 0u};
            }
    };

    // ---- prologue: the workgroup's weight entries, gathered chunk by chunk (every thread helps) --------------
    // The weights of a chunk (NGW planes of 8 channels) are NU contiguous runs of the [K][C][S] tensor (forward: one run of 8 NGW channels x
    // S taps per filter; backward-data: one run of 16 FB channels-of-dx x S taps per channel-of-dy).  The runs are
    // fetched as 16-byte pieces from 4-byte aligned addresses (two chunks ahead), parked raw in the LDS that
    // will later hold the windows, and the entries (8 channels of one tap per lane) are gathered with 2-byte LDS
    // reads.  Entries of padded taps, channels beyond R and filters beyond M stay zero.
    // The prologue runs on 8 waves that share 4 SIMDs and every vector instruction of it costs the workgroup about 8
    // cycles: whatever does not depend on the chunk is computed once, and the steps an aligned, complete tensor
    // does not need (masks, the shift of the last pieces) sit behind launch- or chunk-uniform branches.
    if (a.direct) {
        // Few weights (at most kMaxDE entries per thread): the 8 channels of an entry are 8 two-byte loads from the
        // tensor, all requested at once, before anything else; nothing passes through raw buffers, so the first
        // window can be written as soon as it arrives.  What the workgroup waits for is one memory round trip.
        const int PL = a.ncc * a.NG;
        const int NE = FB * 16 * PL * a.S;
        const int m0 = fg * FB * 16;
        unsigned dv[kMaxDE][8];
        int dslot[kMaxDE], dnv[kMaxDE];
        // channels beyond R or filters beyond M anywhere in the launch?  (else no entry needs a clamp or a mask)
        const bool wmask = PL * 8 != a.R || a.nfg * FB * 16 != a.M;
        // buffer loads: one byte offset per entry plus a scalar offset per channel (the range check of the descriptor
        // is not relied upon: every address is inside the tensor)
        const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned short*>(a.wt), 0, static_cast<int>(static_cast<unsigned>(a.wbytes)), kBufferRsrcFlags);
        const int sr2 = 2 * static_cast<int>(a.w_sr);
#pragma unroll
        for (int k = 0; k < kMaxDE; ++k)
            if (k * 512 < NE) {  // uniform
                const int e = min(tid + k * 512, NE - 1);
                const int mg = fast_div(e, a.dv_s), sx = e - mg * a.S;
                // neighbouring lanes take neighbouring addresses: after the taps, the planes of one filter
                // (forward, [m][r][s]) or the filters of one plane (backward-data, [r][m][s])
                int ml, g;
                if (a.fwd_mode) {
                    ml = fast_div(mg, a.dv_pl);
                    g = mg - ml * PL;
                } else {
                    g = mg / (FB * 16);
                    ml = mg - g * (FB * 16);
                }
                const unsigned base = static_cast<unsigned>(min(m0 + ml, a.M - 1)) * static_cast<unsigned>(a.w_sm) +
                                      static_cast<unsigned>(a.fwd_mode ? sx : a.S - 1 - sx);
                dslot[k] = ((g * JT + (sx >> 2)) * FB + (ml >> 4)) * kQS + 17 * (sx & 3) + (ml & 15);
                if (!wmask) {
                    const int vo = static_cast<int>((base + static_cast<unsigned>(8 * g) * static_cast<unsigned>(a.w_sr)) << 1);
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        dv[k][j] = static_cast<unsigned short>(__builtin_amdgcn_raw_buffer_load_b16(wrsrc, vo, j * sr2, 0));
                } else {
                    dnv[k] = m0 + ml < a.M ? a.R - 8 * g : 0;  // channels of the entry that exist
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        dv[k][j] = a.wt[base + static_cast<unsigned>(min(8 * g + j, a.R - 1)) * static_cast<unsigned>(a.w_sr)];
                }
            }
        if (!consumer) {
            __builtin_amdgcn_s_setprio(3);
            window_prefetch(std::integral_constant<int, kMaxWT>{}, g0, wreg[0]);
        }
        zero_padded_taps();
        // (no barrier: the slots just zeroed are no gathered entry's)
#pragma unroll
        for (int k = 0; k < kMaxDE; ++k)
            if (tid + k * 512 < NE) {
                if (wmask) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) dv[k][j] = j < dnv[k] ? dv[k][j] : 0u;
                }
                lds4[dslot[k]] = u32x4{dv[k][0] | (dv[k][1] << 16), dv[k][2] | (dv[k][3] << 16), dv[k][4] | (dv[k][5] << 16), dv[k][6] | (dv[k][7] << 16)};
            }
        // (no barrier here: the one that hands stage 0 to the consumers follows)
    } else {
        const int NWI = FB * 16 * a.NGW * a.S;  // entries of one chunk (NGW planes)
        const int nchunks = a.ncc * a.NG / a.NGW;
        const int NRP = a.NU * a.NPc;
        const int RSH = a.NPc * 8;  // halfwords per raw run
        const int cs2 = 2 * (a.fwd_mode ? a.S : RSH);  // bytes between the 8 channels of an entry in a raw buffer
        const int m0 = fg * FB * 16;
        // element offset of the first run of chunk cc (even: m0 is a multiple of 16 and the chunks start at multiples of 8 channels)
        auto chunk_base = [&](int cc) -> unsigned {  // the tensor has fewer than 2^31 elements
            return static_cast<unsigned>(static_cast<long>(m0) * a.w_sm + static_cast<long>(cc * a.NGW * 8) * a.w_sr);
        };
        // raw piece k of the thread: piece q of run u, parked at slot u * NPc + q = tid + 512 k of the raw buffer
        unsigned rp_run[kMaxRP], rp_q16[kMaxRP];
        int rp_u[kMaxRP];
#pragma unroll
        for (int k = 0; k < kMaxRP; ++k) {
            const int e = min(tid + k * 512, NRP - 1);
            const int u = fast_div(e, a.dv_npc);
            rp_u[k] = u;
            rp_q16[k] = 16u * static_cast<unsigned>(e - u * a.NPc);
            // forward: the runs are filters, the same in every chunk; filters beyond M repeat the last one
            rp_run[k] = static_cast<unsigned>(a.fwd_mode ? min(u, a.M - 1 - m0) : u) * static_cast<unsigned>(a.su);
        }
        constexpr int kDepth = 4;  // chunks whose raw pieces are in flight
        u32x4 rreg[kDepth][kMaxRP];
        // byte offset of piece k of chunk cc (4-byte aligned), and the last offset a 16-byte load may start at
        const unsigned last_dw = static_cast<unsigned>(a.wbytes - 2) & ~3u;  // the last dword that holds an element
        const unsigned last_piece = last_dw - 12u;
        auto piece_offset = [&](int cc, int k) -> unsigned {
            unsigned run = rp_run[k];
            if (!a.fwd_mode) {  // the runs are channels: those beyond R (last chunk) repeat the last one
                const int r0 = cc * a.NGW * 8;
                if (r0 + 8 * a.NGW > a.R) run = static_cast<unsigned>(max(0, min(rp_u[k], a.R - 1 - r0))) * static_cast<unsigned>(a.su);
            }
            return (((chunk_base(cc) + run) & ~1u) << 1) + rp_q16[k];
        };
        // The first kDepth requests are issued on every path (chunks past the end repeat the last one), and the last
        // pieces of the tensor are loaded from a clamped address and shifted when they are parked.
        auto raw_prefetch = [&](int cc_, u32x4 (&rr)[kMaxRP]) {
            const int cc = min(cc_, nchunks - 1);
            const char* wb = reinterpret_cast<const char*>(a.wt);
#pragma unroll
            for (int k = 0; k < kMaxRP; ++k)
                if (k * 512 < NRP) rr[k] = *reinterpret_cast<const u32x4*>(wb + min(piece_offset(cc, k), last_piece));
        };
        auto raw_commit = [&](int cc, const u32x4 (&rr)[kMaxRP]) {
            u32x4* raw = lds4 + a.wres_slots + (cc & 1) * a.raw_slots;
            // does any piece of this chunk reach into the last 16 bytes of the tensor?  (an upper bound, uniform)
            const unsigned top = static_cast<unsigned>(a.fwd_mode ? min(a.NU - 1, a.M - 1 - m0) : a.NU - 1) * static_cast<unsigned>(a.su);
            const bool tail = ((chunk_base(cc) + top) << 1) + 16u * static_cast<unsigned>(a.NPc - 1) > last_piece;
#pragma unroll
            for (int k = 0; k < kMaxRP; ++k)
                if (tid + k * 512 < NRP) {
                    u32x4 v = rr[k];
                    if (tail) {
                        const unsigned B = piece_offset(cc, k);
                        const unsigned sh = B > last_piece ? (B - last_piece) >> 2 : 0u;  // dwords the clamped load started early
                        v[0] = sh == 0 ? v[0] : (sh == 1 ? v[1] : (sh == 2 ? v[2] : v[3]));
                        v[1] = sh == 0 ? v[1] : (sh == 1 ? v[2] : v[3]);
                        v[2] = sh == 0 ? v[2] : v[3];
                    }
                    raw[tid + k * 512] = v;
                }
        };
        // entry k of the thread (filter ml of the group, plane g of the chunk, tap sx): byte offsets, within a raw
        // buffer, of its channels 0 (and 2, 4, 6: + j cs2) and 1 (3, 5, 7); 16-byte slot within the chunk's entries.
        // A run that starts at an odd element was fetched from the dword before it and lies one halfword further on.
        int wi_be[kMaxWI], wi_bo[kMaxWI], wi_lds[kMaxWI], wi_g8[kMaxWI], wi_ml[kMaxWI];
        auto entry_tables = [&]() {
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k) {
                if (k * 512 >= NWI) break;  // uniform
                const int e = min(tid + k * 512, NWI - 1);
                const int mg = fast_div(e, a.dv_s), sx = e - mg * a.S;
                const int ml = fast_div(mg, a.dv_ngw), g = mg - ml * a.NGW;
                if (a.fwd_mode) {
                    const int idx0 = ml * RSH + 8 * g * a.S + sx;
                    const int pm = static_cast<int>((ml * a.w_sm) & 1);
                    wi_be[k] = 2 * (idx0 + pm);
                    wi_bo[k] = 2 * (idx0 + pm) + cs2;
                } else {
                    const int idx0 = 8 * g * RSH + ml * a.S + (a.S - 1 - sx);
                    wi_be[k] = 2 * idx0;
                    wi_bo[k] = 2 * (idx0 + static_cast<int>(a.w_sr & 1)) + cs2;  // runs of odd channels start at the other parity
                }
                wi_lds[k] = ((g * JT + (sx >> 2)) * FB + (ml >> 4)) * kQS + 17 * (sx & 3) + (ml & 15);
                wi_g8[k] = 8 * g;
                wi_ml[k] = ml;
            }
        };
        // channels beyond R or filters beyond M anywhere in the launch?  (else no entry needs a mask)
        const bool wmask = a.ncc * a.NG * 8 != a.R || a.nfg * FB * 16 != a.M;
        auto gather = [&](int cc) {
            const char* raw = reinterpret_cast<const char*>(lds4 + a.wres_slots + (cc & 1) * a.raw_slots);
            u32x4* wgt = lds4 + cc * (a.NGW * JT * FB * kQS);
            const int r0 = cc * a.NGW * 8;
            unsigned v[kMaxWI][8];
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (k * 512 < NWI) {
#pragma unroll
                    for (int j = 0; j < 8; j += 2) {
                        v[k][j] = *reinterpret_cast<const unsigned short*>(raw + wi_be[k] + j * cs2);
                        v[k][j + 1] = *reinterpret_cast<const unsigned short*>(raw + wi_bo[k] + j * cs2);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (tid + k * 512 < NWI) {
                    if (wmask) {
                        const int nv = m0 + wi_ml[k] < a.M ? a.R - r0 - wi_g8[k] : 0;  // channels that exist
#pragma unroll
                        for (int j = 0; j < 8; ++j) v[k][j] = j < nv ? v[k][j] : 0u;
                    }
                    wgt[wi_lds[k]] = u32x4{v[k][0] | (v[k][1] << 16), v[k][2] | (v[k][3] << 16), v[k][4] | (v[k][5] << 16), v[k][6] | (v[k][7] << 16)};
                }
        };
        // Chunk cc travels in register set cc % kDepth and raw buffer cc & 1; its loads are issued kDepth chunks
        // ahead, so that only the first chunks wait for memory.  The first loads leave before anything else is
        // set up: the weights first, then (producer waves) the window of the first stage, and the tables of the
        // gather and the zeroes are written while they are in flight.
#pragma unroll
        for (int i = 0; i < kDepth; ++i) raw_prefetch(i, rreg[i]);
        if (!consumer) {
            __builtin_amdgcn_s_setprio(3);
            window_prefetch(std::integral_constant<int, kMaxWT>{}, g0, wreg[0]);
        }
        zero_padded_taps();
        entry_tables();
        // (no barrier: the slots just zeroed are no gathered entry's)
        for (int c0 = 0; c0 < nchunks; c0 += kDepth) {
#pragma unroll
            for (int i = 0; i < kDepth; ++i) {
                const int cc = c0 + i;
                if (cc < nchunks) {  // uniform
                    raw_commit(cc, rreg[i]);
                    __syncthreads();
                    gather(cc);
                    if (cc + kDepth < nchunks) raw_prefetch(cc + kDepth, rreg[i]);
                }
            }
        }
        __syncthreads();
    }

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        //   weight operand (plane gp, tap group jj, filter block fb): slot ((gp * JT + jj) * FB + fb) * 68 + 17 kb + li
        //   input operand G of plane g of the stage:  slot g * LPS + 128 cw + li + kb d + delta + U G
        const unsigned wlane = 16u * static_cast<unsigned>(17 * kb + li);
        const unsigned plane_bytes = 16u * static_cast<unsigned>(JT * FB * kQS);
        const unsigned wres_bytes = 16u * static_cast<unsigned>(a.wres_slots);
        const unsigned xlane = 16u * static_cast<unsigned>(wbase + cw * (kT * 16) + li + kb * D + a.delta);
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };
        f32x4 acc[FB][kT];
        bf16x8 W[FB][JT];
        // The bias of the lane's filters, loaded once: a load where a tile completes would wait, with the counter
        // the vector memory instructions share, for every output store still in flight.
        float bm[FB];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            const int m = (fg * FB + fb) * 16 + li;
            bm[fb] = m < a.M ? epi_bias(a.epi, m) : 0.f;
        }
        const bool plain = a.epi.bias == nullptr && !a.epi.relu;
        const long rowblk = 16L * a.Wout;
        const int mlim = a.M - fg * FB * 16 - li;  // filter block fb of this lane exists if 16 fb < mlim
        auto store_unit = [&](int fb, int t, const f32x4& v, long idx0, int o) {  // v: after the epilogue
            if (16 * fb < mlim) {
                const long idx = idx0 + fb * rowblk + 16 * t;
                if (a.vec_out && o + 16 * t + 3 < a.Wout) {
                    epi_store4(a.epi, a.out, idx, v);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (o + 16 * t + i < a.Wout) epi_store(a.epi, a.out, idx + i, v[i]);
                }
            }
        };
        // aligned rows only; with bfloat16 output the first two registers already hold the 8 bytes
        // Non-temporal stores from 37 taps on: measured on C = K = 64 they save 1.2 us per launch there (63.9 -> 62.7 us at
        // S = 51).  With fewer taps a tile is stored almost as fast as the store path accepts it, and non-temporal stores cost
        // 0.9 - 1.2 us at 5 and 9 taps and up to 4 us of 28 at 21 taps when the output is small enough to stay cached
        // (batch 56, C = K = 32, Q = 5000), against a gain of 1.1 us at 17 and 33 taps on the C = K = 64 sweep.
        constexpr bool kNtOut = JT >= 13;
        auto store_unit_vec = [&](int fb, int t, const f32x4& v, long idx0, int o) {
            if (16 * fb < mlim && o + 16 * t < a.Wout) {
                const long idx = idx0 + fb * rowblk + 16 * t;
                if (a.epi.out_bf16) {
                    f32x2* dst = reinterpret_cast<f32x2*>(reinterpret_cast<__bf16*>(a.out) + idx);
                    if constexpr (kNtOut) {
                        __builtin_nontemporal_store(f32x2{v[0], v[1]}, dst);
                    } else {
                        *dst = f32x2{v[0], v[1]};
                    }
                } else {
                    f32x4* dst = reinterpret_cast<f32x4*>(a.out + idx);
                    if constexpr (kNtOut) {
                        __builtin_nontemporal_store(v, dst);
                    } else {
                        *dst = v;
                    }
                }
            }
        };
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int t = 0; t < kT; ++t) acc[fb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        unsigned wnext = wlane + plane_bytes;  // entries of the plane after the current one
        if (wnext >= wlane + wres_bytes) wnext = wlane;

        int tile = t_begin, cc = 0;
        __syncthreads();  // the weight entries and stage 0 are in LDS
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int jj = 0; jj < JT; ++jj) W[fb][jj] = ld(wlane + 16u * static_cast<unsigned>((jj * FB + fb) * kQS));
        for (int st = 0; st < nstages; ++st) {
            const unsigned sb = xlane + 16u * static_cast<unsigned>((st & 1) * a.win_slots);
            for (int g = 0; g < a.NG; ++g) {
                const unsigned xo = sb + 16u * static_cast<unsigned>(g * a.LPS);
                bf16x8 X[XD];
#pragma unroll
                for (int i = 0; i < XD - 1; ++i)
                    if (i <= GMAX) X[i] = ld(xo + 16u * G_::U * i);
#pragma unroll
                for (int G = 0; G <= GMAX; ++G) {
                    // reads of this step: the operand XD - 1 steps ahead, and the next plane's weights for the tap
                    // groups whose last MFMA was in the step before
                    if (G + XD - 1 <= GMAX) X[(G + XD - 1) % XD] = ld(xo + 16u * G_::U * (G + XD - 1));
#pragma unroll
                    for (int jj = 0; jj < JT; ++jj)
                        if (BETA * jj + ALPHA * (kT - 1) == G - 1) {
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb) W[fb][jj] = ld(wnext + 16u * static_cast<unsigned>((jj * FB + fb) * kQS));
                        }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int t = 0; t < kT; ++t) {
                        const int r = G - ALPHA * t;
                        if (r >= 0 && r % BETA == 0 && r / BETA < JT) {
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb)
                                acc[fb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(X[G % XD], W[fb][r / BETA], acc[fb][t], 0, 0, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the last tap group's weights
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) W[fb][JT - 1] = ld(wnext + 16u * static_cast<unsigned>(((JT - 1) * FB + fb) * kQS));
                wnext += plane_bytes;
                if (wnext >= wlane + wres_bytes) wnext = wlane;
            }
            if (++cc == a.ncc) {
                // the tile is complete.  The MFMA operands are swapped (A = input slots, B = weights), so lane
                // (li, kb) holds filter li of each block at the 4 adjacent columns 4 kb .. 4 kb + 3 of each position block
                const int ct = tile;
                const int n = fast_div(ct, a.dv_tpr);
                const int o = (ct - n * a.tiles_per_row) * kTW + cw * (kT * 16) + 4 * kb;
                const long idx0 = static_cast<long>(n) * a.out_sn + static_cast<long>(fg * FB * 16 + li) * a.Wout + o;
                // Every choice below is uniform for the launch and is taken once for the whole tile, not per row
                // segment (this code runs between two stages, with the MFMAs idle); each step works in place on
                // the accumulators.
                auto finish = [&](f32x4 (&fin)[FB][kT]) {
                    if (!plain) {
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                            for (int t = 0; t < kT; ++t) fin[fb][t] = epi_apply4(a.epi, fin[fb][t], bm[fb]);
                    }
                    if (!a.vec_out) {  // rows that are not 16-byte aligned: element by element, here
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                            for (int t = 0; t < kT; ++t) store_unit(fb, t, fin[fb][t], idx0, o);
                    } else {
                        if (a.epi.out_bf16) {  // 4 bfloat16 in the first two registers
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                                for (int t = 0; t < kT; ++t) {
                                    const f32x2 h = __builtin_bit_cast(f32x2, __builtin_convertvector(fin[fb][t], epi_bf16x4));
                                    fin[fb][t][0] = h[0];
                                    fin[fb][t][1] = h[1];
                                }
                        }
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
                            for (int t = 0; t < kT; ++t) store_unit_vec(fb, t, fin[fb][t], idx0, o);
                    }
                };
                finish(acc);
#pragma unroll
                for (int fb = 0; fb < FB; ++fb)
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
        // Two register sets: the window of stage st + 2 is requested while stage st + 1 is written (a stage is
        // shorter than the memory latency under load).  Set st & 1 holds stage st.  The loop exists once per task
        // count.
        auto run = [&](auto nt_) {
            const int last = nstages - 1;
            // (a wave can have 63 loads in flight: the second window is requested only now, with the weights in LDS)
            window_prefetch(nt_, g1, wreg[1]);
            window_commit(g0, 0, wreg[0]);
            __syncthreads();  // the consumers start on stage 0
            g2 = geo(min(2, last));
            window_prefetch(nt_, g2, wreg[0]);
            // invariant at the top of iteration st: g1 = stage st + 1 (in set 1), g2 = stage st + 2 (in set 0)
            int st = 0;
            for (; st + 4 <= last; st += 2) {  // the steady state: no branch around a load
                window_commit(g1, 1, wreg[1]);
                g1 = geo(st + 3);
                window_prefetch(nt_, g1, wreg[1]);
                __syncthreads();
                window_commit(g2, 0, wreg[0]);
                g2 = geo(st + 4);
                window_prefetch(nt_, g2, wreg[0]);
                __syncthreads();
            }
            // the last stages; with an odd number of them the consumers meet the second barrier after their loop
            for (; st <= last; st += 2) {
                if (st + 1 <= last) window_commit(g1, 1, wreg[1]);
                if (st + 3 <= last) {
                    g1 = geo(st + 3);
                    window_prefetch(nt_, g1, wreg[1]);
                }
                __syncthreads();
                if (st + 2 <= last) window_commit(g2, 0, wreg[0]);
                __syncthreads();
            }
        };
        switch ((NWT + 255) / 256) {
            case 1: run(std::integral_constant<int, 1>{}); break;
            case 2: run(std::integral_constant<int, 2>{}); break;
            case 3: run(std::integral_constant<int, 3>{}); break;
            case 4: run(std::integral_constant<int, 4>{}); break;
            default: run(std::integral_constant<int, kMaxWT>{}); break;
        }
    }
}

struct RgPlan {
    bool ok;
    int D, FB, JT, KT, grid;
    size_t lds_bytes;
    RgArgs a;
};

template <int D, int FB, int JT, int KT>
hipError_t rg_launch(const RgPlan& pl, hipStream_t st) {
    auto kern = igemm_ring_bf16_kernel<D, FB, JT, KT>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

template <int D, int KT>
hipError_t rg_launch_dk(const RgPlan& pl, hipStream_t st) {
    switch (pl.FB * 100 + pl.JT) {
        case 113: return rg_launch<D, 1, 13, KT>(pl, st);
        case 213: return rg_launch<D, 2, 13, KT>(pl, st);
        case 109: return rg_launch<D, 1, 9, KT>(pl, st);
        case 209: return rg_launch<D, 2, 9, KT>(pl, st);
        case 105: return rg_launch<D, 1, 5, KT>(pl, st);
        case 205: return rg_launch<D, 2, 5, KT>(pl, st);
        // (four filter blocks only with the narrow tile: with 8 position blocks the accumulators alone take 128 registers)
        case 403: if constexpr (KT == 5) return rg_launch<D, 4, 3, KT>(pl, st); else return hipErrorInvalidValue;
        case 402: if constexpr (KT == 5) return rg_launch<D, 4, 2, KT>(pl, st); else return hipErrorInvalidValue;
        case 103: return rg_launch<D, 1, 3, KT>(pl, st);
        case 203: return rg_launch<D, 2, 3, KT>(pl, st);
        case 102: return rg_launch<D, 1, 2, KT>(pl, st);
        case 202: return rg_launch<D, 2, 2, KT>(pl, st);
        default: return hipErrorInvalidValue;
    }
}

template <int D>
hipError_t rg_launch_d(const RgPlan& pl, hipStream_t st) {
    if (pl.KT == 5) return rg_launch_dk<D, 5>(pl, st);
    return rg_launch_dk<D, 8>(pl, st);
}

hipError_t launch_d1(const RgPlan& pl, hipStream_t st);
hipError_t launch_d2(const RgPlan& pl, hipStream_t st);
hipError_t launch_d4(const RgPlan& pl, hipStream_t st);
hipError_t launch_d8(const RgPlan& pl, hipStream_t st);
hipError_t launch_d16(const RgPlan& pl, hipStream_t st);

}  // namespace rg
}  // namespace conv1d
