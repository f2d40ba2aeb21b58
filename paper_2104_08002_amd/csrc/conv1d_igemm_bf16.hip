// Forward / backward-data passes (Eq. 2; Section 3.2) for bfloat16 inputs and many channels (R or M > 16).
//
//   out[n][m][o] = sum_r sum_s in[n][r][o + s*d - P] * wt(m, r, s)
//
// is an implicit GEMM of the weight matrix (M x [R*S]) with the shifted-input matrix ([R*S] x positions), run as
// a batch-reduce over (channel chunk, tap) in the sense of Algorithm 2, but with the whole reduction of a tile
// kept in MFMA accumulators.  The reduction index is cut into "k-blocks" (8 channels of one tap); one
// v_mfma_f32_16x16x32_bf16 contracts four of them: 16 filters x 4 k-blocks times 4 k-blocks x 16 positions.
//
// Tile.  A workgroup owns 32 filters x 512 output columns of one sample: consumer wave v takes the columns
// [128 v, 128 v + 128) as 8 position blocks and both filter blocks, so every weight operand feeds 8 MFMAs and
// every input operand 2 (10 LDS reads per 16 MFMAs).  The reduction runs in stages of one channel chunk
// (8*NG channels, all S taps, NQ = ceil(NG*S/4) MFMA steps).
//
// LDS per stage (16-byte slots, double buffered):
//   window   plane g (8 channels) x LPS positions, slot = those 8 channels at one input position, so a lane's
//            k-block operand is one ds_read_b128 at (plane, position + s*d) for any dilation;
//   weights  entry (filter block, step j, lane) = wt(m, 8 channels, tap) of that lane's k-block, gathered from
//            the [K][C][S] tensor as it is (no prepared copy exists: the pass has no workspace), 68 slots per
//            step so that both the gather's writes and the operand reads are conflict free.
//
// Workgroup = 8 waves, one per CU, persistent over a contiguous strip of tiles: waves 0-3 ("consumers") read
// operands and issue MFMAs, and write the finished tile straight from the accumulators; waves 4-7 ("producers")
// fetch stage t+1 (window: 8 rows x 2 positions per task, transposed with byte permutes; weights: 8 channel
// loads per entry) into registers while stage t is computed and write it into the other LDS buffer.  One
// workgroup barrier per stage.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kFB = 2;            // filter blocks of 16 per workgroup
constexpr int kT = 8;             // position blocks of 16 per consumer wave
constexpr int kTW = 4 * kT * 16;  // output columns per tile
constexpr int kMaxNQ = 13;        // MFMA steps per stage
constexpr int kMaxWT = 5;         // window tasks per producer thread
constexpr int kMaxWI = 7;         // weight entries per producer thread
constexpr int kMaxRP = 7;         // raw 16-byte pieces per producer thread
constexpr int kQS = 68;           // slots per (filter block, step): 4 k-blocks x 17
constexpr unsigned kPermLo = 0x05040100u;  // {b.lo16, a.lo16} -> a.lo | b.lo << 16
constexpr unsigned kPermHi = 0x07060302u;  // {b.hi16, a.hi16} -> a.hi | b.hi << 16

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct IgArgs {
    const unsigned short* in;
    const unsigned short* wt;
    float* out;
    int N, R, M, Win, Wout, S, d, P;
    long w_sm, w_sr, in_sn, out_sn;
    int w_s0, w_ss;
    int tiles_per_row, nfg, nct, nteams;  // column blocks per row, filter groups, N * tiles_per_row, teams of nfg workgroups
    int NG, NQ, ncc;  // channel groups of 8 per stage, MFMA steps per stage, stages per tile
    int LP, LPS;      // window positions staged (even), plane stride in slots
    int delta;        // (o0 - P) - window origin: 0 or 1
    int stage_slots;  // NG * LPS + kFB * NQ * kQS
    int fwd_mode;     // weights are [m][r][s] (forward) or [r][m][S-1-s] (backward-data)
    int NU, NPc;      // raw runs per stage, 16-byte pieces per run
    long su;          // elements between the starts of consecutive runs
    long wbytes;      // size of the weight tensor
    int raw_slots;    // NU * NPc
    Epilogue epi;
};

__global__ __launch_bounds__(512, 2) void igemm_corr_bf16_kernel(IgArgs a) {
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

    // A tile is (column block ct of one sample, filter group fg).  nfg workgroups with consecutive logical indices
    // form a team that walks one contiguous strip of column blocks, one filter group each: the team's members
    // run side by side on one XCD, so a window is fetched from HBM once and found in L2 by the others.
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int team = lid / a.nfg, fg = lid - team * a.nfg;
    const int t_begin = static_cast<int>(static_cast<long>(team) * a.nct / a.nteams);
    const int t_end = static_cast<int>(static_cast<long>(team + 1) * a.nct / a.nteams);
    const int nstages = (t_end - t_begin) * a.ncc;
    const int wbase = a.NG * a.LPS;  // weights behind the window planes

    // zero both weight areas once: the k-blocks that pad the last MFMA step are never written again
    for (int b = 0; b < 2; ++b)
        for (int e = tid; e < kFB * a.NQ * kQS; e += 512) lds4[b * a.stage_slots + wbase + e] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        // Lane (li, kb) of step j holds k-block i = 4 j + kb = (channel group i / S, tap i % S).
        //   weight operand, filter block fb:  slot (fb * NQ + j) * 68 + 17 kb + li
        //   input operand, position block t:  plane i / S, position 128 cw + 16 t + li + (i % S) d + delta
        // k-blocks beyond NG * S (padding of the last step) re-read the last real one; their weights are zero.
        unsigned boff[kMaxNQ];
#pragma unroll
        for (int j = 0; j < kMaxNQ; ++j) {
            const int i = min(4 * j + kb, a.NG * a.S - 1);
            const int g = i / a.S, s = i - g * a.S;
            boff[j] = 16u * static_cast<unsigned>(g * a.LPS + cw * (kT * 16) + li + s * a.d + a.delta);
        }
        const unsigned aoff0 = 16u * static_cast<unsigned>(wbase + 17 * kb + li);
        const unsigned aoff1 = aoff0 + 16u * static_cast<unsigned>(a.NQ * kQS);
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };
        f32x4 acc[kFB][kT];
#pragma unroll
        for (int fb = 0; fb < kFB; ++fb)
#pragma unroll
            for (int t = 0; t < kT; ++t) acc[fb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        // The bias of the lane's filters, loaded once: a load where a tile completes would wait, with the counter
        // the vector memory instructions share, for every output store still in flight.
        float bm[kFB][4];
#pragma unroll
        for (int fb = 0; fb < kFB; ++fb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = (fg * kFB + fb) * 16 + 4 * kb + i;
                bm[fb][i] = m < a.M ? epi_bias(a.epi, m) : 0.f;
            }

        int tile = t_begin, cc = 0;
        __syncthreads();  // raw weights of stage 0 are in LDS
        __syncthreads();  // stage 0 is in LDS
        for (int st = 0; st < nstages; ++st) {
            const unsigned sb = static_cast<unsigned>((st & 1) * a.stage_slots) * 16u;
            bf16x8 wa[2][kFB], xb[2][kT];
            wa[0][0] = ld(sb + aoff0);
            wa[0][1] = ld(sb + aoff1);
#pragma unroll
            for (int t = 0; t < kT; ++t) xb[0][t] = ld(sb + boff[0] + 256 * t);
#pragma unroll
            for (int j = 0; j < kMaxNQ; ++j) {
                if (j < a.NQ) {
                    const int cur = j & 1, nxt = cur ^ 1;
                    if (j + 1 < kMaxNQ && j + 1 < a.NQ) {
                        wa[nxt][0] = ld(sb + aoff0 + 16 * kQS * (j + 1));
                        wa[nxt][1] = ld(sb + aoff1 + 16 * kQS * (j + 1));
#pragma unroll
                        for (int t = 0; t < kT; ++t) xb[nxt][t] = ld(sb + boff[j + 1 < kMaxNQ ? j + 1 : j] + 256 * t);
                    }
#pragma unroll
                    for (int t = 0; t < kT; ++t)
#pragma unroll
                        for (int fb = 0; fb < kFB; ++fb)
                            acc[fb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[cur][fb], xb[cur][t], acc[fb][t], 0, 0, 0);
                }
            }
            if (++cc == a.ncc) {
                // the tile is complete: lane (li, kb) holds filters 4 kb .. 4 kb + 3 of each block at column li
                const int ct = tile;
                const int n = ct / a.tiles_per_row;
                const int o = (ct - n * a.tiles_per_row) * kTW + cw * (kT * 16) + li;
                const long base = static_cast<long>(n) * a.out_sn;
#pragma unroll
                for (int fb = 0; fb < kFB; ++fb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int m = (fg * kFB + fb) * 16 + 4 * kb + i;
#pragma unroll
                        for (int t = 0; t < kT; ++t) {
                            if (m < a.M && o + 16 * t < a.Wout)
                                epi_store(a.epi, a.out, base + static_cast<long>(m) * a.Wout + o + 16 * t, epi_apply(a.epi, acc[fb][t][i], bm[fb][i]));
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
    } else {
        // ---- producer side -----------------------------------------------------------------------
        // Window task (plane g, pair i): positions G0 + 2i, G0 + 2i + 1 of the 8 channels of plane g; 8 dword
        // loads (row starts, the window origin and Win are even) from clamped addresses, two slots out.
        //
        // Weights travel in three steps, one stage apart each.  The weights of a stage are NU contiguous
        // runs of the [K][C][S] tensor (forward: one run of 8 NG channels x S taps per filter; backward-data:
        // one run of 32 channels-of-dx x S taps per channel-of-dy).  (1) The runs are fetched as 16-byte pieces
        // from 4-byte aligned addresses into registers, (2) written as they are into a raw LDS area, and (3)
        // the operand entries (8 channels of one tap per lane) are gathered from the raw area with 2-byte LDS
        // reads.  Sub-dword global loads would cost one memory instruction per element instead.
        const int LP2 = a.LP >> 1;
        const int NWT = a.NG * LP2;
        const int NWI = kFB * 16 * a.NG * a.S;
        const int NRP = a.NU * a.NPc;
        int wt_plane8[kMaxWT], wt_pair[kMaxWT];  // 8 * plane, pair index within the plane
#pragma unroll
        for (int k = 0; k < kMaxWT; ++k) {
            const int e = min(rtid + k * 256, NWT - 1);
            const int g = e / LP2;
            wt_plane8[k] = 8 * g;
            wt_pair[k] = e - g * LP2;
        }
        int rp_u[kMaxRP], rp_q[kMaxRP];  // run and piece of a raw-copy task
#pragma unroll
        for (int k = 0; k < kMaxRP; ++k) {
            const int e = min(rtid + k * 256, NRP - 1);
            rp_u[k] = e / a.NPc;
            rp_q[k] = e - rp_u[k] * a.NPc;
        }
        // entry (m, g, s): raw halfword index of channel c8 = idx0 + c8 * cs + (parity of the run's start), slot
        int wi_idx0[kMaxWI], wi_lds[kMaxWI], wi_g8[kMaxWI], wi_par[kMaxWI];
#pragma unroll
        for (int k = 0; k < kMaxWI; ++k) {
            const int e = min(rtid + k * 256, NWI - 1);
            const int sx = e % a.S, mg = e / a.S;
            const int g = mg % a.NG, ml = mg / a.NG;
            const int i = g * a.S + sx;
            const int RSH = a.NPc * 8;  // halfwords per raw run
            if (a.fwd_mode) {
                wi_idx0[k] = ml * RSH + 8 * g * a.S + sx;
                const int pm = static_cast<int>((ml * a.w_sm) & 1);
                wi_par[k] = pm | (pm << 1);
            } else {
                wi_idx0[k] = 8 * g * RSH + ml * a.S + (a.S - 1 - sx);
                wi_par[k] = static_cast<int>(a.w_sr & 1) << 1;  // runs of odd channels start at the other parity
            }
            wi_lds[k] = ((ml >> 4) * a.NQ + (i >> 2)) * kQS + 17 * (i & 3) + (ml & 15);
            wi_g8[k] = 8 * g;
        }
        const int cs = a.fwd_mode ? a.S : a.NPc * 8;
        struct Geo {
            int n, G0, fg, r0;  // sample, window origin, filter group, first channel of the chunk
        };
        auto geo = [&](int st) -> Geo {
            const int ct = t_begin + st / a.ncc, cc = st - (st / a.ncc) * a.ncc;
            Geo g;
            g.fg = fg;
            g.n = ct / a.tiles_per_row;
            g.G0 = (ct - g.n * a.tiles_per_row) * kTW - a.P - a.delta;
            g.r0 = cc * a.NG * 8;
            return g;
        };
        unsigned wreg[kMaxWT][8];
        u32x4 rreg[kMaxRP];
        // A stage is "interior" when its whole window lies inside the rows and all its channels exist: the
        // loads then go to scalar row bases + one per-thread constant and nothing is masked (the producer waves
        // share their SIMDs' issue slots with the MFMA waves, so every instruction they do not execute counts).
        auto interior = [&](const Geo& g) { return g.G0 >= 0 && g.G0 + a.LP <= a.Win && g.r0 + 8 * a.NG <= a.R; };
        unsigned wt_voff[kMaxWT];  // byte offset of the task's pair from the first row of its chunk at the window origin
        int wt_dst[kMaxWT];        // slot of the task's first output
#pragma unroll
        for (int k = 0; k < kMaxWT; ++k) {
            wt_voff[k] = 2u * (static_cast<unsigned>(wt_plane8[k]) * static_cast<unsigned>(a.Win) + 2u * static_cast<unsigned>(wt_pair[k]));
            wt_dst[k] = (wt_plane8[k] >> 3) * a.LPS + 2 * wt_pair[k];
        }
        auto window_prefetch = [&](const Geo& g) {
            const char* ib = reinterpret_cast<const char*>(a.in + static_cast<long>(g.n) * a.in_sn);
            const unsigned rowb = static_cast<unsigned>(a.Win) * 2u;
            if (interior(g)) {
                const char* rb = ib + 2 * (static_cast<long>(g.r0) * a.Win + g.G0);  // uniform
#pragma unroll
                for (int k = 0; k < kMaxWT; ++k)
                    if (k * 256 < NWT) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) wreg[k][j] = *reinterpret_cast<const unsigned*>(rb + j * static_cast<long>(rowb) + wt_voff[k]);
                    }
            } else {
#pragma unroll
                for (int k = 0; k < kMaxWT; ++k)
                    if (k * 256 < NWT) {
                        int pos = g.G0 + 2 * wt_pair[k];
                        pos = pos < 0 ? 0 : (pos > a.Win - 2 ? a.Win - 2 : pos);
                        const unsigned offmax = static_cast<unsigned>((a.R - 1) * a.Win + pos) * 2u;
                        unsigned off = static_cast<unsigned>((g.r0 + wt_plane8[k]) * a.Win + pos) * 2u;
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            wreg[k][j] = *reinterpret_cast<const unsigned*>(ib + min(off, offmax));
                            off += rowb;
                        }
                    }
            }
        };
        auto window_commit = [&](const Geo& g, int b) {
            u32x4* win = lds4 + b * a.stage_slots;
            const bool inner = interior(g);
#pragma unroll
            for (int k = 0; k < kMaxWT; ++k)
                if (rtid + k * 256 < NWT) {
                    const int pos = g.G0 + 2 * wt_pair[k];
                    const bool ok = inner || (pos >= 0 && pos < a.Win);  // a pair is inside or outside the row as a whole
                    u32x4 ev, od;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const unsigned lo = ok ? wreg[k][2 * q] : 0u, hi = ok ? wreg[k][2 * q + 1] : 0u;
                        ev[q] = __builtin_amdgcn_perm(hi, lo, kPermLo);
                        od[q] = __builtin_amdgcn_perm(hi, lo, kPermHi);
                    }
                    u32x4* dst = win + wt_dst[k];
                    dst[0] = ev;
                    dst[1] = od;
                }
        };
        // element offset of the stage's first run from the tensor base (runs beyond the last filter / channel
        // re-read the last one; their entries are zeroed in the gather)
        auto stage_base = [&](const Geo& g) -> long {
            return static_cast<long>(g.fg * kFB * 16) * a.w_sm + static_cast<long>(g.r0) * a.w_sr;
        };
        auto raw_prefetch = [&](const Geo& g) {
            const unsigned eb = static_cast<unsigned>(stage_base(g));  // the tensor has fewer than 2^31 elements
            const int umax = a.fwd_mode ? a.M - 1 - g.fg * kFB * 16 : a.R - 1 - g.r0;
            const char* wb = reinterpret_cast<const char*>(a.wt);
            const unsigned su = static_cast<unsigned>(a.su);
            const unsigned wb4 = static_cast<unsigned>(a.wbytes) & ~3u;
            // only the pieces of the last runs of the tensor can reach beyond its end (uniform test)
            const unsigned reach = ((eb + static_cast<unsigned>(min(a.NU - 1, umax)) * su) * 2u & ~3u) + 16u * static_cast<unsigned>(a.NPc);
            if (reach <= wb4) {
#pragma unroll
                for (int k = 0; k < kMaxRP; ++k)
                    if (k * 256 < NRP) {
                        const unsigned eu = eb + static_cast<unsigned>(min(rp_u[k], umax)) * su;
                        rreg[k] = *reinterpret_cast<const u32x4*>(wb + (((eu * 2u) & ~3u) + 16u * static_cast<unsigned>(rp_q[k])));
                    }
            } else {
                const unsigned last_dw = static_cast<unsigned>(a.wbytes - 2) & ~3u;  // the last dword that holds an element
#pragma unroll
                for (int k = 0; k < kMaxRP; ++k)
                    if (k * 256 < NRP) {
                        const unsigned eu = eb + static_cast<unsigned>(min(rp_u[k], umax)) * su;
                        const unsigned B = ((eu * 2u) & ~3u) + 16u * static_cast<unsigned>(rp_q[k]);
#pragma unroll
                        for (int i = 0; i < 4; ++i) rreg[k][i] = *reinterpret_cast<const unsigned*>(wb + min(B + 4u * i, last_dw));
                    }
            }
        };
        auto raw_commit = [&](int rb) {
            u32x4* raw = lds4 + 2 * a.stage_slots + rb * a.raw_slots;
#pragma unroll
            for (int k = 0; k < kMaxRP; ++k)
                if (rtid + k * 256 < NRP) raw[rp_u[k] * a.NPc + rp_q[k]] = rreg[k];
        };
        auto gather = [&](const Geo& g, int b) {
            const unsigned short* raw = reinterpret_cast<const unsigned short*>(lds4 + 2 * a.stage_slots + b * a.raw_slots);
            u32x4* wgt = lds4 + b * a.stage_slots + wbase;
            const int pb = static_cast<int>(stage_base(g) & 1);
            const int m0 = g.fg * kFB * 16;
            // all reads first (one LDS round trip for the lot), then the packing
            unsigned v[kMaxWI][8];
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (k * 256 < NWI) {
                    const int ie = wi_idx0[k] + (pb ^ (wi_par[k] & 1)), io = wi_idx0[k] + (pb ^ (wi_par[k] >> 1));
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[k][j] = raw[((j & 1) ? io : ie) + j * cs];
                }
            __builtin_amdgcn_sched_barrier(0);
            // channels beyond R and filters beyond M are zero: an entry keeps its first nv channels
            const bool full = (a.R % (8 * a.NG)) == 0 && (a.M % (kFB * 16)) == 0;
#pragma unroll
            for (int k = 0; k < kMaxWI; ++k)
                if (rtid + k * 256 < NWI) {
                    if (!full) {
                        const int ml = (rtid + k * 256) / (a.S * a.NG);
                        const int nv = m0 + ml < a.M ? a.R - g.r0 - wi_g8[k] : 0;
#pragma unroll
                        for (int j = 0; j < 8; ++j) v[k][j] = j < nv ? v[k][j] : 0u;
                    }
                    wgt[wi_lds[k]] = u32x4{v[k][0] | (v[k][1] << 16), v[k][2] | (v[k][3] << 16), v[k][4] | (v[k][5] << 16), v[k][6] | (v[k][7] << 16)};
                }
        };
        // iteration t: window t+1 -> LDS, window t+2 -> registers; entries t+1 <- raw[(t+1)&1],
        // raw[t&1] <- registers (stage t+2), registers <- global (stage t+3)
        // (the geometry of a stage costs four integer divisions: it is worked out once, when the stage enters
        // the pipeline, and handed down: g1, g2, g3 are the stages st + 1, st + 2, st + 3)
        Geo g1 = geo(0), g2 = geo(1 < nstages ? 1 : 0), g3 = geo(2 < nstages ? 2 : 0);
        if (nstages > 0) {
            raw_prefetch(g1);
            window_prefetch(g1);
            raw_commit(0);
            if (nstages > 1) raw_prefetch(g2);
        }
        __syncthreads();
        if (nstages > 0) {
            gather(g1, 0);
            window_commit(g1, 0);
            if (nstages > 1) {
                raw_commit(1);
                window_prefetch(g2);
            }
            if (nstages > 2) raw_prefetch(g3);
        }
        __syncthreads();
        g1 = g2;
        g2 = g3;
        for (int st = 0; st < nstages; ++st) {
            if (st + 3 < nstages) g3 = geo(st + 3);
            if (st + 1 < nstages) {
                // registers are refilled as soon as they are free, so every load has a whole stage to arrive
                window_commit(g1, (st + 1) & 1);
                if (st + 2 < nstages) window_prefetch(g2);
                if (st + 2 < nstages) raw_commit(st & 1);
                if (st + 3 < nstages) raw_prefetch(g3);
                gather(g1, (st + 1) & 1);
            }
            g1 = g2;
            g2 = g3;
            __syncthreads();
        }
    }
}

struct IgPlan {
    bool ok;
    int grid;
    size_t lds_bytes;
    IgArgs a;
};

IgPlan ig_plan(const CorrProblem& p) {
    IgPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.accumulate) return pl;
    if (p.R <= 16 && p.M <= 16) return pl;  // the small-channel kernels are built for that
    if (p.S < 4 || p.S > 4 * kMaxNQ) return pl;
    // dword loads of position pairs: even row starts and an even window origin
    if ((p.Win & 1) || (p.in_sn & 1) || (reinterpret_cast<uintptr_t>(p.in) & 3) || p.Win < 2) return pl;
    if (reinterpret_cast<uintptr_t>(p.wt) & 3) return pl;
    const bool fwd_mode = p.w_ss == 1 && p.w_sr == p.S && p.w_s0 == 0;
    const bool bwd_mode = p.w_ss == -1 && p.w_sm == p.S && p.w_s0 == p.S - 1;
    if (!fwd_mode && !bwd_mode) return pl;
    if (static_cast<long>(p.R) * p.Win >= (1L << 30)) return pl;                                  // 32-bit byte offsets within a sample
    if (static_cast<long>(p.M) * p.R * p.S >= (1L << 31) || p.M * p.w_sm >= (1L << 31) || p.R * p.w_sr >= (1L << 31)) return pl;
    IgArgs& a = pl.a;
    a.in = static_cast<const unsigned short*>(p.in);
    a.wt = static_cast<const unsigned short*>(p.wt);
    a.out = p.out;
    a.epi = p.epi;
    a.N = p.N; a.R = p.R; a.M = p.M; a.Win = p.Win; a.Wout = p.Wout; a.S = p.S; a.d = p.d; a.P = p.P;
    a.w_sm = p.w_sm; a.w_sr = p.w_sr; a.w_s0 = p.w_s0; a.w_ss = p.w_ss; a.in_sn = p.in_sn; a.out_sn = p.out_sn;
    a.delta = (p.P & 1) ? 1 : 0;  // (column block start - P) - delta is even
    const long halo = static_cast<long>(p.S - 1) * p.d;
    const long LP = (kTW + halo + a.delta + 1) / 2 * 2;
    const int ngroups = cdiv(p.R, 8);
    // as many channel groups per stage as fit (fewer, longer stages)
    for (int NG = 8; NG >= 1; NG /= 2) {
        if (NG > 1 && NG / 2 >= ngroups) continue;  // no point in planes that are never filled
        const int NQ = cdiv(static_cast<long>(NG) * p.S, 4);
        if (NQ > kMaxNQ) continue;
        if (cdiv(static_cast<long>(NG) * (LP / 2), 256) > kMaxWT) continue;
        if (cdiv(static_cast<long>(kFB) * 16 * NG * p.S, 256) > kMaxWI) continue;
        const long LPS = LP + 8;  // the operand of a padded k-block never leaves the plane; a little slack anyway
        const long stage = NG * LPS + static_cast<long>(kFB) * NQ * kQS;
        const int NU = fwd_mode ? kFB * 16 : 8 * NG;
        const long L = fwd_mode ? 8L * NG * p.S : static_cast<long>(kFB) * 16 * p.S;
        const long NPc = (2 * L + 2 + 15) / 16;
        if (cdiv(NU * NPc, 256) > kMaxRP) continue;
        const size_t bytes = static_cast<size_t>(2 * stage + 2 * NU * NPc) * 16;
        if (bytes > static_cast<size_t>(kLdsBudget)) continue;
        a.NG = NG;
        a.NQ = NQ;
        a.ncc = cdiv(ngroups, NG);
        a.LP = static_cast<int>(LP);
        a.LPS = static_cast<int>(LPS);
        a.stage_slots = static_cast<int>(stage);
        a.fwd_mode = fwd_mode;
        a.NU = NU;
        a.NPc = static_cast<int>(NPc);
        a.raw_slots = static_cast<int>(NU * NPc);
        a.su = fwd_mode ? p.w_sm : p.w_sr;
        a.wbytes = (fwd_mode ? static_cast<long>(p.M) * p.w_sm : static_cast<long>(p.R) * p.w_sr) * 2;
        a.tiles_per_row = cdiv(p.Wout, kTW);
        a.nfg = cdiv(p.M, kFB * 16);
        const long nct = static_cast<long>(p.N) * a.tiles_per_row;
        if (nct > 0x7fffffffL / 16 || a.nfg > 65535) return pl;
        a.nct = static_cast<int>(nct);
        const int fit = kNumCU / a.nfg > 0 ? kNumCU / a.nfg : 1;  // teams that run at the same time
        a.nteams = a.nct < fit ? a.nct : fit;
        pl.grid = a.nteams * a.nfg;
        pl.lds_bytes = bytes;
        pl.ok = true;
        return pl;
    }
    return pl;
}

}  // namespace

bool igemm_bf16_corr_supported(const CorrProblem& p) { return ig_plan(p).ok; }

hipError_t igemm_bf16_corr_launch(const CorrProblem& p, hipStream_t st) {
    const IgPlan pl = ig_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(igemm_corr_bf16_kernel), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(igemm_corr_bf16_kernel, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

}  // namespace conv1d
