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
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;

// ------------------------------------------------------------------------------------------------
// FP32 forward / backward-data
// ------------------------------------------------------------------------------------------------
// Workgroup = 8 waves, one per CU, persistent over a contiguous strip of tiles (4*T*16 output columns of one
// sample each).  LDS holds
//   wfrag[S*RC][64]      weights in MFMA A-operand order: entry (step = s*RC + cc, lane = m + 16*kb) is
//                        wt(m, 4*cc + kb, s)  (zero outside M x R)
//   win[b][4*RC][LPS]    input window b, row r, column i <-> input position G0 + i   (NBUF = 1 or 2 buffers)
// Waves 0-3 ("consumers") own T adjacent 16-column output tiles each and walk the (tap, channel-chunk)
// reduction with v_mfma_f32_16x16x4_f32, the LDS reads of tap s+1 interleaved with the MFMAs of tap s;
// they store their outputs themselves.  With more than 16 channels (ncb > 1 channel blocks of 16) a tile is
// reduced in ncb stages, one window per channel block, with the sums kept in the accumulators in between;
// wfrag then holds the weights of all blocks.  Waves 4-7 ("producers") fetch the window of tile t+2 from global
// memory into registers and write the window of tile t+1 into the free buffer; one workgroup barrier per
// tile hands the buffers over.  When two windows do not fit in LDS (long halos) the same kernel runs with one
// buffer and a second barrier per tile.
template <int RC, int T, int MAXS, bool FAST>
__global__ __launch_bounds__(512, 2) void smallc_corr_f32_kernel(CorrProblem p, int tiles_per_row, int ntiles, int LPS, int LP4,
                                                                 int nbuf, int raw_in_lds, int ncb, int vec_out) {
    extern __shared__ float lds[];
    constexpr int TQ = 4 * T * 16;
    const int nsteps = p.S * RC;  // MFMA steps per channel block
    float* wfrag = lds;
    auto win = [&](int b) { return lds + ncb * nsteps * 64 + b * 4 * RC * LPS; };
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;
    const int rtid = tid & 255;
    const int li = lane & 15;  // row of A / column of B and D
    const int kb = lane >> 4;  // k index of A/B; row block of D
    const float* __restrict__ in = static_cast<const float*>(p.in);
    // More than 16 filters: blockIdx.y numbers the filter blocks of 16; a workgroup computes its block's rows.
    const int mb = blockIdx.y;
    const int Mb = min(16, p.M - 16 * mb);  // filters of this block
    const float* __restrict__ wt = static_cast<const float*>(p.wt) + static_cast<long>(mb) * 16 * p.w_sm;
    const int nslots = 4 * RC * LP4;
    // window column 0 is the input position (tile start - P) rounded down to a multiple of 4, so that 16-byte
    // staging loads stay aligned for any padding; the consumers skip the psh extra columns
    const int psh = ((-p.P) % 4 + 4) % 4;

    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int t_begin = static_cast<int>(static_cast<long>(lid) * ntiles / gridDim.x) * ncb;      // first stage of the strip
    const int t_end = static_cast<int>(static_cast<long>(lid + 1) * ntiles / gridDim.x) * ncb;  // one past its last stage
    // stage u = tile * ncb + channel block (all of the strip's stages in one sequence)
    auto stage_tile = [&](int u) { return ncb == 1 ? u : u / ncb; };
    auto tile_n = [&](int u) { return stage_tile(u) / tiles_per_row; };
    auto tile_O0 = [&](int u) { const int t = stage_tile(u); return (t - (t / tiles_per_row) * tiles_per_row) * TQ; };
    auto stage_cb = [&](int u) { return ncb == 1 ? 0 : u - (u / ncb) * ncb; };
    // everything a staging slot needs to know about its stage, worked out once per stage (the divisions above
    // are not something to repeat for every slot)
    struct Geo {
        long nbase;        // element offset of the stage's sample
        int gorg;          // input position of window column 0
        unsigned rowbase;  // element offset of the stage's first channel row within the sample
    };
    auto geo = [&](int u) -> Geo {
        return Geo{static_cast<long>(tile_n(u)) * p.in_sn, tile_O0(u) - p.P - psh, static_cast<unsigned>(stage_cb(u) * 16 * p.Win)};
    };

    // ---- producer side ------------------------------------------------------------------------------
    // Staging slot e = 4 adjacent positions of row e / LP4; slot k of a producer thread is e = rtid + 256*k
    // and everything about it except the window origin is worked out once.  FAST (row starts, window origin
    // and base pointer are multiples of 4 floats, so a slot is inside or outside its row as a whole): one
    // 16-byte load from a clamped address, masked when it is written to LDS.  Otherwise element loads, done
    // when the window is written.
    constexpr int kRowBad = 1 << 29;
    struct Slot { unsigned off; int col, lds; };
    auto make_slot = [&](int e) -> Slot {
        const int r = e / LP4, i = e - r * LP4;
        return Slot{static_cast<unsigned>(min(r, p.R - 1) * p.Win), 4 * i, (r * LPS + 4 * i) | (r < p.R ? 0 : kRowBad)};
    };
    auto fetch = [&](const Geo& t, const Slot& w) -> f32x4 {
        // (rows beyond R re-read row R - 1; they are zeroed when written to LDS)
        const unsigned rowoff = min(w.off + t.rowbase, static_cast<unsigned>((p.R - 1) * p.Win));
        const float* row = in + t.nbase + rowoff;
        const int g = t.gorg + w.col;
        if constexpr (FAST) {
            const int lim = p.Win - 4;  // >= 0 on this path (checked by the host)
            return *reinterpret_cast<const f32x4*>(row + (g < 0 ? 0 : (g > lim ? lim : g)));
        } else {
            f32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int gj = g + j;
                const float tt = row[gj < 0 ? 0 : (gj > p.Win - 1 ? p.Win - 1 : gj)];
                v[j] = (gj >= 0 && gj < p.Win) ? tt : 0.f;
            }
            return v;
        }
    };
    auto commit = [&](float* wb, const Geo& t, const Slot& w, f32x4 v) {
        const int g = t.gorg + w.col;
        const bool row_ok = ncb == 1 ? !(w.lds & kRowBad) : w.off + t.rowbase < static_cast<unsigned>(p.R * p.Win);
        const bool ok = row_ok && (!FAST || (g >= 0 && g + 4 <= p.Win));
        if (!ok) v = f32x4{0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<f32x4*>(wb + (w.lds & (kRowBad - 1))) = v;
    };
    Slot slot[MAXS];
    // two stages in flight: stage u travels in register set u & 1, fetched two stages before it is written to LDS
    // (a stage of a narrow filter is shorter than the memory latency)
    f32x4 preA[FAST ? MAXS : 1], preB[FAST ? MAXS : 1];
    auto prefetch_set = [&](f32x4 (&pre)[FAST ? MAXS : 1], int u) {
        if constexpr (FAST) {
            const Geo t = geo(u);
#pragma unroll
            for (int k = 0; k < MAXS; ++k)
                if (k * 256 < nslots) pre[k] = fetch(t, slot[k]);
        }
    };
    auto commit_set = [&](const f32x4 (&pre)[FAST ? MAXS : 1], float* wb, int u) {
        const Geo t = geo(u);
#pragma unroll
        for (int k = 0; k < MAXS; ++k) {
            if (rtid + k * 256 < nslots) {
                if constexpr (FAST) {
                    commit(wb, t, slot[k], pre[k]);
                } else {
                    commit(wb, t, slot[k], fetch(t, slot[k]));
                }
            }
        }
    };
    auto commit_rest = [&](float* wb, int u) {
        const Geo t = geo(u);
        for (int e = rtid + MAXS * 256; e < nslots; e += 256) {  // long halos: beyond the register budget
            const Slot w = make_slot(e);
            commit(wb, t, w, fetch(t, w));
        }
    };

    // ---- prologue: weights (all waves), first window (producers) -------------------------------------
    if (!consumer) {
#pragma unroll
        for (int k = 0; k < MAXS; ++k) slot[k] = make_slot(min(rtid + k * 256, nslots - 1));
    }
    {
        // coalesced copy of the raw tensor into LDS (aliasing the windows), then reorder into wfrag
        const int nW = Mb * p.R * p.S;
        float* raw = win(0);
        if (raw_in_lds) {
            if ((reinterpret_cast<uintptr_t>(wt) & 15) == 0) {
                constexpr int NV = (16 * 16 * 64 / 4 + 511) / 512;  // 16-byte pieces per thread for S <= 64
                const int nvec = nW / 4;
                f32x4 tmp[NV];
#pragma unroll
                for (int k = 0; k < NV; ++k) tmp[k] = reinterpret_cast<const f32x4*>(wt)[min(tid + k * 512, nvec > 0 ? nvec - 1 : 0)];
                if (!consumer && t_begin < t_end) prefetch_set(preA, t_begin);  // queued behind the weight loads
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k = 0; k < NV; ++k)
                    if (tid + k * 512 < nvec) reinterpret_cast<f32x4*>(raw)[tid + k * 512] = tmp[k];
                for (int e = NV * 512 + tid; e < nvec; e += 512) reinterpret_cast<f32x4*>(raw)[e] = reinterpret_cast<const f32x4*>(wt)[e];
                for (int e = nvec * 4 + tid; e < nW; e += 512) raw[e] = wt[e];
            } else {
                for (int e = tid; e < nW; e += 512) raw[e] = wt[e];
                if (!consumer && t_begin < t_end) prefetch_set(preA, t_begin);
            }
            __syncthreads();
        } else if (!consumer && t_begin < t_end) {
            prefetch_set(preA, t_begin);
        }
        // Entry (channel block cb, step, lane): wave w takes the steps w, w + 8, ... of the sequence over all channel
        // blocks.  The step counter is wave-uniform and counted, not divided (this loop is most of the time a workgroup
        // spends before its first MFMA); element offsets fit 32 bits (checked by the host).
        {
            const int m = lane & 15, kbl = lane >> 4;
            const int wsr = static_cast<int>(p.w_sr), wss = static_cast<int>(p.w_ss);
            const int mbase = m * static_cast<int>(p.w_sm) + static_cast<int>(p.w_s0);
            int step = wave, cb = 0;
            while (step >= nsteps) {
                step -= nsteps;
                ++cb;
            }
            while (cb < ncb) {
                const int cc = step % RC, s = step / RC;  // (RC is a compile-time constant)
                const int r = 16 * cb + 4 * cc + kbl;
                float v = 0.f;
                if (m < Mb && r < p.R) {
                    const int idx = mbase + r * wsr + s * wss;
                    v = raw_in_lds ? raw[idx] : wt[idx];
                }
                wfrag[(cb * nsteps + step) * 64 + lane] = v;
                step += 8;
                while (step >= nsteps) {
                    step -= nsteps;
                    ++cb;
                }
            }
        }
        __syncthreads();  // raw copy is dead, wfrag is complete
    }
    if (!consumer && t_begin < t_end) {
        if (t_begin + 1 < t_end) prefetch_set(preB, t_begin + 1);
        commit_set(preA, win(0), t_begin);
        commit_rest(win(0), t_begin);
        if (t_begin + 2 < t_end) prefetch_set(preA, t_begin + 2);
    }
    __syncthreads();

    // ---- consumer side --------------------------------------------------------------------------------
    f32x4 acc[T];  // lives across the channel blocks of a tile
    auto compute = [&](const float* wb, int t) {
        const int cb = stage_cb(t);
        if (cb == 0) {
#pragma unroll
            for (int j = 0; j < T; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const int ob = cw * T * 16;
        // running LDS indices (into lds[]), one per channel chunk, bumped by d per tap: the operand reads then
        // carry immediate offsets only instead of an address add in front of each of them
        int wi[RC];
#pragma unroll
        for (int cc = 0; cc < RC; ++cc) wi[cc] = static_cast<int>(wb - lds) + (4 * cc + kb) * LPS + ob + li + psh;
        int ai = lane + cb * nsteps * 64;
        float a0[RC], b0[RC][T], a1[RC], b1[RC][T];
        auto load_tap = [&](float (&a)[RC], float (&b)[RC][T]) {  // loads the tap the indices point at
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) {
                a[cc] = lds[ai + cc * 64];
#pragma unroll
                for (int j = 0; j < T; ++j) b[cc][j] = lds[wi[cc] + j * 16];
            }
        };
        auto next_tap = [&]() {
            ai += RC * 64;
#pragma unroll
            for (int cc = 0; cc < RC; ++cc) wi[cc] += p.d;
        };
        auto mfma_tap = [&](const float (&a)[RC], const float (&b)[RC][T]) {
#pragma unroll
            for (int cc = 0; cc < RC; ++cc)
#pragma unroll
                for (int j = 0; j < T; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(b[cc][j], a[cc], acc[j], 0, 0, 0);
        };
        // the LDS reads of the next tap are spread between the MFMAs of the current one, an MFMA first (read first
        // measured 234.6 against 230.4 us on the 51-tap genomics layer: the tap's first MFMA then waits behind a read)
        auto interleave = [&]() {
#pragma unroll
            for (int i = 0; i < RC * T; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, RC, 0);
        };
        // Keeps the operands of the tap just consumed live to the end of the tap: otherwise the register an
        // MFMA has just been issued with is handed to the very next LDS read, which then cannot issue until
        // the MFMA has finished fetching its sources.
        auto keep = [&](const float (&b)[RC][T]) {
#pragma unroll
            for (int cc = 0; cc < RC; ++cc)
#pragma unroll
                for (int j = 0; j < T; ++j) asm volatile("" ::"v"(b[cc][j]));
            __builtin_amdgcn_sched_barrier(0);
        };
        load_tap(a0, b0);
        int s = 0;
        for (; s + 1 < p.S; s += 2) {
            next_tap();
            load_tap(a1, b1);
            mfma_tap(a0, b0);
            interleave();
            keep(b0);
            if (s + 2 < p.S) next_tap();  // (S even: the last look-ahead re-reads tap S-1 and is discarded)
            load_tap(a0, b0);
            mfma_tap(a1, b1);
            interleave();
            keep(b1);
        }
        if (s < p.S) mfma_tap(a0, b0);  // odd S: the last tap is already loaded
        if (cb + 1 < ncb) return;       // more channel blocks to come
        // The input fragment is the A operand and the weight fragment the B operand, so the accumulator tile is
        // [position][filter]: lane (li, kb) holds filter li at the 4 adjacent columns 4 kb .. 4 kb + 3 of each
        // 16-column block, one 16-byte store per block when the row starts allow it.
        const int n = tile_n(t), O0 = tile_O0(t);
        if (li < Mb) {
            const long rowi = static_cast<long>(n) * p.out_sn + static_cast<long>(16 * mb + li) * p.Wout;
            float* row = p.out + rowi;
            const float bm = p.accumulate ? 0.f : epi_bias(p.epi, 16 * mb + li);
#pragma unroll
            for (int j = 0; j < T; ++j) {
                const int o = O0 + ob + j * 16 + 4 * kb;
                if (p.accumulate) {  // a further channel block of a layer: float output, no epilogue
                    if (vec_out && o + 4 <= p.Wout) {
                        f32x4* dst = reinterpret_cast<f32x4*>(row + o);
                        *dst = *dst + acc[j];
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (o + i < p.Wout) row[o + i] += acc[j][i];
                    }
                } else {
                    const f32x4 v = epi_apply4(p.epi, acc[j], bm);
                    if (vec_out && o + 4 <= p.Wout) {
                        epi_store4(p.epi, p.out, rowi + o, v);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (o + i < p.Wout) epi_store(p.epi, p.out, rowi + o + i, v[i]);
                    }
                }
            }
        }
    };

    // ---- steady state -----------------------------------------------------------------------------------
    int k = 0;
    for (int t = t_begin; t < t_end; ++t, ++k) {
        const int b = nbuf == 2 ? (k & 1) : 0;
        if (consumer) {
            compute(win(b), t);
        } else if (nbuf == 2 && t + 1 < t_end) {
            if ((k + 1) & 1) {
                commit_set(preB, win(b ^ 1), t + 1);
                if (t + 3 < t_end) prefetch_set(preB, t + 3);
            } else {
                commit_set(preA, win(b ^ 1), t + 1);
                if (t + 3 < t_end) prefetch_set(preA, t + 3);
            }
            commit_rest(win(b ^ 1), t + 1);
        }
        __syncthreads();
        if (nbuf == 1 && t + 1 < t_end) {  // single buffer: refill it while the consumers wait
            if (!consumer) {
                if ((k + 1) & 1) {
                    commit_set(preB, win(0), t + 1);
                    if (t + 3 < t_end) prefetch_set(preB, t + 3);
                } else {
                    commit_set(preA, win(0), t + 1);
                    if (t + 3 < t_end) prefetch_set(preA, t + 3);
                }
                commit_rest(win(0), t + 1);
            }
            __syncthreads();
        }
    }
}

struct CorrF32Plan {
    int RC, LPS, LP4, tiles_per_row, ntiles, fast, raw_in_lds, nbuf, ncb, vec_out;
    size_t lds_bytes;
    bool ok;
};

constexpr int kCorrT = 4, kCorrMaxS = 11;

CorrF32Plan corr_f32_plan(const CorrProblem& p, bool blocks = false) {
    CorrF32Plan pl{};
    pl.ok = false;
    if (p.bf16 || (p.M > 16 && !blocks) || cdiv(p.M, 16) > 65535) return pl;
    if (static_cast<long>(p.R) * p.Win >= (1L << 30)) return pl;  // 32-bit element offsets within one sample
    {  // ... and within the weights this launch reads
        const auto mag = [](long v) { return v < 0 ? -v : v; };
        if (16 * mag(p.w_sm) + p.R * mag(p.w_sr) + p.S * mag(p.w_ss) + mag(p.w_s0) >= (1L << 31)) return pl;
    }
    constexpr int TQ = 4 * kCorrT * 16;
    // more than 16 channels: blocks of 16, reduced one after the other inside the kernel
    pl.ncb = cdiv(p.R, 16);
    if (pl.ncb > 1 && p.accumulate) return pl;
    pl.RC = pl.ncb > 1 ? 4 : (p.R + 3) / 4;
    const long halo = static_cast<long>(p.S - 1) * p.d;
    const long LP = TQ + halo + 3;  // + the columns in front of an unaligned window origin
    // row stride == 16 (mod 32) words: the four k rows of a B fragment fall on disjoint bank halves
    const long LPS = (LP + 31) / 32 * 32 + 16;
    const long wbytes = static_cast<long>(pl.ncb) * p.S * pl.RC * 64 * 4;
    const long win_bytes = 4L * pl.RC * LPS * 4;
    pl.nbuf = wbytes + 2 * win_bytes <= kLdsBudget ? 2 : 1;
    const long bytes = wbytes + pl.nbuf * win_bytes;
    if (bytes > kLdsBudget) return pl;
    pl.LPS = static_cast<int>(LPS);
    pl.LP4 = static_cast<int>((LP + 3) / 4);
    pl.tiles_per_row = cdiv(p.Wout, TQ);
    const long nt = static_cast<long>(p.N) * pl.tiles_per_row;
    if (nt > 0x7fffffffL) return pl;
    pl.ntiles = static_cast<int>(nt);
    pl.lds_bytes = static_cast<size_t>(bytes);
    // 16-byte window loads need every row start, the window origin and the base pointer aligned
    pl.fast = (p.Win % 4 == 0) && (p.in_sn % 4 == 0) && (reinterpret_cast<uintptr_t>(p.in) % 16 == 0) && p.Win >= 4;
    pl.vec_out = (p.Wout % 4 == 0) && (p.out_sn % 4 == 0) && (reinterpret_cast<uintptr_t>(p.out) % 16 == 0);
    pl.raw_in_lds = p.w_contig && p.M <= 16 && static_cast<long>(p.M) * p.R * p.S * 4 <= pl.nbuf * win_bytes;
    pl.ok = true;
    return pl;
}

template <int RC, bool FAST>
hipError_t corr_f32_launch_f(const CorrProblem& p, const CorrF32Plan& pl, hipStream_t st) {
    auto kern = smallc_corr_f32_kernel<RC, kCorrT, kCorrMaxS, FAST>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    // one workgroup per CU in total: the filter blocks (grid rows) share the strips of tiles between them
    const int strips = cdiv(kNumCU, cdiv(p.M, 16));
    const int grid = pl.ntiles < strips ? pl.ntiles : strips;
    return launch_kernel(kern, dim3(grid, cdiv(p.M, 16)), dim3(512), pl.lds_bytes, st, p, pl.tiles_per_row, pl.ntiles, pl.LPS, pl.LP4, pl.nbuf,
                       pl.raw_in_lds, pl.ncb, pl.vec_out);
}

template <int RC>
hipError_t corr_f32_launch_rc(const CorrProblem& p, const CorrF32Plan& pl, hipStream_t st) {
    return pl.fast ? corr_f32_launch_f<RC, true>(p, pl, st) : corr_f32_launch_f<RC, false>(p, pl, st);
}

// ------------------------------------------------------------------------------------------------
// FP32 backward-weight
// ------------------------------------------------------------------------------------------------
// Workgroup = 8 waves, one per CU, persistent over a contiguous strip of chunks (QC output columns of one
// sample each).  Waves 0-3 ("consumers"): wave v owns taps s = v, v+4, v+8, ... (NT slots) and keeps one
// 16 x 16 accumulator tile per tap; one MFMA k-step covers 4 positions, A = dy[m][q0 + kb],
// B = x[c][q0 + kb + s*d - P], both read from LDS with ds_read_b32 (any dilation), the reads of k-step t+1
// interleaved with the MFMAs of k-step t.  Waves 4-7 ("producers") fetch chunk i+2 from global memory into
// registers and write chunk i+1 into the free half of the double-buffered LDS:
//   dyt[b][16][LQS]  rows = filters, column j <-> q = Qs + j
//   xt [b][16][LXS]  rows = channels, column i <-> input position Qs - P + i
// One workgroup barrier per chunk hands the buffers over.  Partial sums: ws[(wg * S + s) * 256 + m * 16 + c].
template <int NT, int MAXS, bool FAST>
__global__ __launch_bounds__(512, 2) void smallc_wgrad_f32_kernel(WgradProblem p, int chunks_per_row, int nchunks, int QC, int LQS, int LXS,
                                                                  int LX4) {
    extern __shared__ float lds[];
    const int stage_floats = 16 * (LQS + LXS);
    auto dyt = [&](int b) { return lds + b * stage_floats; };
    auto xt = [&](int b) { return lds + b * stage_floats + 16 * LQS; };
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;
    const int rtid = tid & 255;
    const int li = lane & 15;
    const int kb = lane >> 4;
    // More than 16 channels or filters: blockIdx.y numbers the (filter block, channel block) pairs; a workgroup
    // works on the 16 x 16 block pair of its row of the grid and writes its own slice of the workspace.
    const int ncbp = (p.C + 15) >> 4;
    const int pair = blockIdx.y, kbi = pair / ncbp, cbi = pair - kbi * ncbp;
    const int Cb = min(16, p.C - 16 * cbi), Kb = min(16, p.K - 16 * kbi);  // channels / filters of this block
    const float* __restrict__ x = static_cast<const float*>(p.x) + static_cast<long>(cbi) * 16 * p.W;
    const float* __restrict__ dy = static_cast<const float*>(p.dy) + static_cast<long>(kbi) * 16 * p.Q;
    const int Q4 = QC / 4;
    const int ndy = 16 * Q4;
    const int nslots = ndy + 16 * LX4;

    // contiguous strip of chunks; neighbouring strips (shared halos) land on the same XCD
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int c_begin = static_cast<int>(static_cast<long>(lid) * nchunks / gridDim.x);
    const int c_end = static_cast<int>(static_cast<long>(lid + 1) * nchunks / gridDim.x);

    // Staging slot e: first the dy rows (Q4 slots each), then the x rows (LX4 slots each); 4 adjacent
    // positions per slot.  Slot k of a producer thread is e = rtid + 256*k; QC is a multiple of 64, so the
    // dy/x boundary (16*Q4) is a multiple of 256 and "is this an x slot" is uniform per k.  Everything about
    // a slot except the chunk origin is worked out once.  FAST: one clamped 16-byte load, masked at the LDS
    // write (widths, padding and pointers are multiples of 4 floats, so a slot never straddles a row end).
    constexpr int kRowBad = 1 << 29;
    struct Slot { unsigned off; int col, lds; };  // row offset in the sample, first column, LDS index (| kRowBad)
    auto slot_is_x = [&](int k) { return k * 256 >= ndy; };
    auto make_slot = [&](int k, int e) -> Slot {
        const bool is_x = slot_is_x(k);
        const int e2 = is_x ? e - ndy : e;
        const int per_row = is_x ? LX4 : Q4;
        const int r = e2 / per_row, i = e2 - r * per_row;
        const int rows = is_x ? Cb : Kb;
        Slot w;
        w.off = static_cast<unsigned>(min(r, rows - 1) * (is_x ? p.W : p.Q));
        w.col = 4 * i;
        w.lds = (r * (is_x ? LXS : LQS) + 4 * i) | (r < rows ? 0 : kRowBad);
        return w;
    };
    // x column 0 is the input position (chunk start - P) rounded down to a multiple of 4, so that 16-byte staging
    // loads stay aligned for any padding; the consumers skip the psh extra columns
    const int psh = ((-p.P) % 4 + 4) % 4;
    struct Origin { const float* xb; const float* dyb; int Qs; };
    auto origin = [&](int chunk) -> Origin {
        const int n = chunk / chunks_per_row;
        return Origin{x + static_cast<long>(n) * p.x_sn, dy + static_cast<long>(n) * p.dy_sn, (chunk - n * chunks_per_row) * QC};
    };
    auto fetch = [&](const Origin& o, int k, const Slot& w) -> f32x4 {
        const bool is_x = slot_is_x(k);
        const float* row = (is_x ? o.xb : o.dyb) + w.off;
        const int limit = is_x ? p.W : p.Q;
        const int g = (is_x ? o.Qs - p.P - psh : o.Qs) + w.col;
        if constexpr (FAST) {
            const int lim = limit - 4;
            return *reinterpret_cast<const f32x4*>(row + (g < 0 ? 0 : (g > lim ? lim : g)));
        } else {
            f32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int gj = g + j;
                const float t = row[gj < 0 ? 0 : (gj > limit - 1 ? limit - 1 : gj)];
                v[j] = (gj >= 0 && gj < limit) ? t : 0.f;
            }
            return v;
        }
    };
    auto commit = [&](int b, const Origin& o, int k, const Slot& w, f32x4 v) {
        const bool is_x = slot_is_x(k);
        const int limit = is_x ? p.W : p.Q;
        const int g = (is_x ? o.Qs - p.P - psh : o.Qs) + w.col;
        const bool ok = !(w.lds & kRowBad) && (!FAST || (g >= 0 && g + 4 <= limit));
        if (!ok) v = f32x4{0.f, 0.f, 0.f, 0.f};
        // rows are only 8-byte aligned (their stride is 2 mod 32 words, see the plan): two 8-byte stores
        f32x2* dst = reinterpret_cast<f32x2*>((is_x ? xt(b) : dyt(b)) + (w.lds & (kRowBad - 1)));
        dst[0] = f32x2{v[0], v[1]};
        dst[1] = f32x2{v[2], v[3]};
    };
    Slot slot[MAXS];
    // Two prefetch sets: the loads of a chunk are issued two chunks before it is written to LDS (with few taps a
    // chunk is shorter than the memory latency under load).  Set (chunk - c_begin) & 1 holds a chunk.
    constexpr int NPRE = (FAST && NT <= 5) ? 2 : 1;  // long chunks (many taps) need one set only
    f32x4 pre[NPRE][FAST ? MAXS : 1];
    if (!consumer) {
#pragma unroll
        for (int k = 0; k < MAXS; ++k) slot[k] = make_slot(k, min(rtid + k * 256, nslots - 1));
    }
    auto prefetch_chunk = [&](int chunk, f32x4 (&pr)[FAST ? MAXS : 1]) {
        if constexpr (FAST) {
            const Origin o = origin(chunk);
#pragma unroll
            for (int k = 0; k < MAXS; ++k) pr[k] = fetch(o, k, slot[k]);
        }
    };
    auto commit_chunk = [&](int b, int chunk, const f32x4 (&pr)[FAST ? MAXS : 1]) {
        const Origin o = origin(chunk);
#pragma unroll
        for (int k = 0; k < MAXS; ++k) {
            if (rtid + k * 256 < nslots) {
                if constexpr (FAST) {
                    commit(b, o, k, slot[k], pr[k]);
                } else {
                    commit(b, o, k, slot[k], fetch(o, k, slot[k]));
                }
            }
        }
        // slots beyond the per-thread register budget (long halos) are staged directly
        for (int k = MAXS; rtid + k * 256 < nslots; ++k) {
            const Slot w = make_slot(k, rtid + k * 256);
            commit(b, o, k, w, fetch(o, k, w));
        }
    };

    f32x4 acc[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // prologue: producers stage the first chunk and start on the second
    if (!consumer && c_begin < c_end) {
        prefetch_chunk(c_begin, pre[0]);
        if constexpr (NPRE == 2) {
            if (c_begin + 1 < c_end) prefetch_chunk(c_begin + 1, pre[1]);
            commit_chunk(0, c_begin, pre[0]);
            if (c_begin + 2 < c_end) prefetch_chunk(c_begin + 2, pre[0]);
        } else {
            commit_chunk(0, c_begin, pre[0]);
            if (c_begin + 1 < c_end) prefetch_chunk(c_begin + 1, pre[0]);
        }
    }
    __syncthreads();

    // The two roles run separate loops (with one barrier per chunk each) so that neither carries the other's
    // registers through its loop.
    if (consumer) {
        int k = 0;
        for (int chunk = c_begin; chunk < c_end; ++chunk, ++k) {
            const int b = k & 1;
            // one running LDS index per tap slot (into lds[]): the reads then need no address arithmetic in
            // front of them (a dependent v_add before every ds_read costs about a quarter of the MFMA rate)
            int ai = b * stage_floats + li * LQS + kb;
            int bi[NT];
#pragma unroll
            for (int i = 0; i < NT; ++i) bi[i] = b * stage_floats + 16 * LQS + li * LXS + kb + (cw + 4 * i) * p.d + psh;
            // NS k-steps per iteration with a ring of NS operand register sets: the LDS reads of k-step t + NS - 1
            // are issued between the MFMAs of k-step t.  With few taps per wave a k-step is only 2 - 3 MFMAs
            // long, so the reads have to run three k-steps ahead to cover the LDS latency.  The reads of the
            // last iteration run up to 4 (NS - 1) columns past the chunk (into row padding / the slack after the
            // last row) and are discarded.
            constexpr int NS = NT <= 3 ? 4 : 2;
            float av[NS], bv[NS][NT];
#pragma unroll
            for (int j = 0; j < NS - 1; ++j) {
                av[j] = lds[ai + 4 * j];
#pragma unroll
                for (int i = 0; i < NT; ++i) bv[j][i] = lds[bi[i] + 4 * j];
            }
            for (int t = 0; t < QC; t += 4 * NS) {
#pragma unroll
                for (int j = 0; j < NS; ++j) {
                    constexpr int kAhead = NS - 1;
                    const int nx = (j + kAhead) % NS;
                    av[nx] = lds[ai + 4 * (j + kAhead)];
#pragma unroll
                    for (int i = 0; i < NT; ++i) {
                        bv[nx][i] = lds[bi[i] + 4 * (j + kAhead)];
                        acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[j], bv[j][i], acc[i], 0, 0, 0);
                    }
#pragma unroll
                    for (int i = 0; i < NT; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read ...
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // ... then one MFMA
                    }
                    // Keep the consumed operands live to the end of the k-step: otherwise the register of the
                    // operand an MFMA has just been issued with is handed to the very next LDS read, and that
                    // read cannot issue until the MFMA has finished fetching its sources.
#pragma unroll
                    for (int i = 0; i < NT; ++i) asm volatile("" ::"v"(bv[j][i]));
                    __builtin_amdgcn_sched_barrier(0);
                }
                ai += 4 * NS;
#pragma unroll
                for (int i = 0; i < NT; ++i) bi[i] += 4 * NS;
            }
            __syncthreads();
        }
    } else {
        if constexpr (NPRE == 2) {
            for (int chunk = c_begin; chunk < c_end; chunk += 2) {
                if (chunk + 1 < c_end) {
                    commit_chunk(1, chunk + 1, pre[1]);
                    if (chunk + 3 < c_end) prefetch_chunk(chunk + 3, pre[1]);
                }
                __syncthreads();
                if (chunk + 1 < c_end) {
                    if (chunk + 2 < c_end) {
                        commit_chunk(0, chunk + 2, pre[0]);
                        if (chunk + 4 < c_end) prefetch_chunk(chunk + 4, pre[0]);
                    }
                    __syncthreads();
                }
            }
        } else {
            int k = 0;
            for (int chunk = c_begin; chunk < c_end; ++chunk, ++k) {
                const int b = k & 1;
                if (chunk + 1 < c_end) {
                    commit_chunk(b ^ 1, chunk + 1, pre[0]);
                    if (chunk + 2 < c_end) prefetch_chunk(chunk + 2, pre[0]);
                }
                __syncthreads();
            }
        }
    }
    if (consumer) {
        const int nt = (p.S - cw + 3) / 4;  // real taps of this wave; slots beyond hold unused sums
        float* ws = static_cast<float*>(p.ws) + (static_cast<long>(pair) * gridDim.x + blockIdx.x) * p.S * 256;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            if (i < nt) {
                const int s = cw + 4 * i;
#pragma unroll
                for (int j = 0; j < 4; ++j) ws[s * 256 + (4 * kb + j) * 16 + li] = acc[i][j];
            }
        }
    }
}

// Second stage of the backward-weight pass: dw[k][c][s] = sum over workgroups g of
// ws[(g*S + s)*256 + k*16 + c], always in the same order: 32 contiguous groups of workgroups are
// summed left to right by 16 threads each, then the 32 group sums are added left to right.
// blockIdx.y numbers the (filter block, channel block) pairs of a batched launch (K, C: totals).
__global__ __launch_bounds__(512) void smallc_wgrad_reduce_kernel(const float* __restrict__ ws, float* __restrict__ dw, int K, int C, int S, long dw_sk,
                                                                  long dw_sc, int nwg) {
    __shared__ epi_f32x4 part[kTailPartSlots];
    WgradTail t;
    {
        const int ncbp = (C + 15) >> 4;
        const int pair = blockIdx.y, kbi = pair / ncbp, cbi = pair - kbi * ncbp;
        t.ws = ws + static_cast<long>(pair) * nwg * S * 256;
        t.dw = dw + kbi * 16 * dw_sk + cbi * 16 * dw_sc;
        t.K = min(16, K - 16 * kbi);
        t.C = min(16, C - 16 * cbi);
        t.S = S; t.nwg = nwg; t.dw_sk = dw_sk; t.dw_sc = dw_sc;
    }
    wgrad_tail_phase1(t, blockIdx.x, threadIdx.x, part);
    __syncthreads();
    wgrad_tail_phase2(t, blockIdx.x, threadIdx.x, part);
}

struct WgradF32Plan {
    int QC, LQS, LXS, LX4, chunks_per_row, nchunks, grid, fast, NT;
    size_t lds_bytes;
    bool ok;
};

constexpr int kWgradNT = 13, kWgradMaxS = 15;  // most taps per wave; staging slots per producer thread held in registers
constexpr int kWgradNTs[] = {2, 3, 5, 9, 13};    // instantiated taps per wave: 4 * NT tap slots are multiplied whatever S is

WgradF32Plan wgrad_f32_plan(const WgradProblem& p, bool blocks = false) {
    WgradF32Plan pl{};
    pl.ok = false;
    if (p.bf16 || p.S > 4 * kWgradNT) return pl;
    if (!blocks && (p.C > 16 || p.K > 16)) return pl;
    if (static_cast<long>(cdiv(p.C, 16)) * cdiv(p.K, 16) > 65535) return pl;
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    pl.NT = kWgradNT;
    for (int i = 4; i >= 0; --i)
        if (4 * kWgradNTs[i] >= p.S) pl.NT = kWgradNTs[i];
    const long halo = static_cast<long>(4 * pl.NT - 1) * p.d + 3;  // every tap slot a wave may read, + an unaligned window origin
    // row stride == 2 (mod 32) words: the 32 lanes (16 rows x 2 adjacent columns) that the LDS serves together
    // fall on 32 distinct banks (a stride of 4 would pair row r with row r+8)
    auto pad = [](long v) { return (v + 31) / 32 * 32 + 2; };
    for (int QC = 256; QC >= 64; QC /= 2) {  // the largest chunk whose two stages fit in LDS
        const long LQS = pad(QC), LXS = pad(QC + halo);
        const long bytes = 2 * 16 * (LQS + LXS) * 4 + 128;  // + slack for the discarded look-ahead reads
        if (bytes > kLdsBudget) continue;
        pl.QC = QC;
        pl.LQS = static_cast<int>(LQS);
        pl.LXS = static_cast<int>(LXS);
        pl.LX4 = static_cast<int>((QC + halo + 3) / 4);
        pl.chunks_per_row = cdiv(p.Q, QC);
        const long nc = static_cast<long>(p.N) * pl.chunks_per_row;
        if (nc > 0x7fffffffL) return pl;
        pl.nchunks = static_cast<int>(nc);
        // one workgroup per CU in total: the block pairs (grid rows) share the strips of chunks between them
        const int strips = blocks ? cdiv(kNumCU, cdiv(p.C, 16) * cdiv(p.K, 16)) : kNumCU;
        pl.grid = pl.nchunks < strips ? pl.nchunks : strips;
        pl.lds_bytes = static_cast<size_t>(bytes);
        pl.fast = (p.W % 4 == 0) && (p.Q % 4 == 0) && (p.x_sn % 4 == 0) && (p.dy_sn % 4 == 0) && p.W >= 4 && p.Q >= 4 &&
                  (reinterpret_cast<uintptr_t>(p.x) % 16 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 16 == 0);
        pl.ok = true;
        return pl;
    }
    return pl;
}

template <int NT>
hipError_t wgrad_f32_launch_nt(const WgradProblem& p, const WgradF32Plan& pl, hipStream_t st) {
    auto kern = pl.fast ? smallc_wgrad_f32_kernel<NT, kWgradMaxS, true> : smallc_wgrad_f32_kernel<NT, kWgradMaxS, false>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    const int pairs = cdiv(p.K, 16) * cdiv(p.C, 16);
    return launch_kernel(kern, dim3(pl.grid, pairs), dim3(512), pl.lds_bytes, st, p, pl.chunks_per_row, pl.nchunks, pl.QC, pl.LQS, pl.LXS,
                       pl.LX4);
}

}  // namespace

hipError_t smallc_wgrad_reduce_launch(const float* ws, float* dw, int K, int C, int S, long dw_sk, long dw_sc, int nwg,
                                      hipStream_t st) {
    const int pairs = cdiv(K, 16) * cdiv(C, 16);
    return launch_kernel(smallc_wgrad_reduce_kernel, dim3(S * 4, pairs), dim3(512), 0, st, ws, dw, K, C, S, dw_sk, dw_sc, nwg);
}

hipError_t smallc_corr_launch_impl(const CorrProblem& p, bool blocks, hipStream_t st);

bool smallc_corr_supported(const CorrProblem& p) {
    if (p.bf16) return smallc_bf16_corr_supported(p);
    return corr_f32_plan(p).ok;
}

// FP32 with any M: all filter blocks of 16 in one launch (grid.y), the channel blocks reduced inside the kernel
bool smallc_corr_f32_blocks_supported(const CorrProblem& p) { return corr_f32_plan(p, true).ok; }

hipError_t smallc_corr_f32_blocks_launch(const CorrProblem& p, hipStream_t st) { return smallc_corr_launch_impl(p, true, st); }

hipError_t smallc_corr_launch(const CorrProblem& p, hipStream_t st) {
    if (p.bf16) return smallc_bf16_corr_launch(p, st);
    return smallc_corr_launch_impl(p, false, st);
}

hipError_t smallc_corr_launch_impl(const CorrProblem& p, bool blocks, hipStream_t st) {
    const CorrF32Plan pl = corr_f32_plan(p, blocks);
    if (!pl.ok) return hipErrorInvalidValue;
    switch (pl.RC) {
        case 1: return corr_f32_launch_rc<1>(p, pl, st);
        case 2: return corr_f32_launch_rc<2>(p, pl, st);
        case 3: return corr_f32_launch_rc<3>(p, pl, st);
        default: return corr_f32_launch_rc<4>(p, pl, st);
    }
}

hipError_t smallc_wgrad_launch_impl(const WgradProblem& p, bool blocks, hipStream_t st);

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

// FP32 with any C, K: all 16 x 16 block pairs in one launch (grid.y) and one second stage
size_t smallc_wgrad_f32_blocks_workspace(const WgradProblem& p) {
    const WgradF32Plan pl = wgrad_f32_plan(p, true);
    if (!pl.ok) return 0;
    return static_cast<size_t>(cdiv(p.K, 16)) * cdiv(p.C, 16) * pl.grid * p.S * 256 * sizeof(float);
}

hipError_t smallc_wgrad_f32_blocks_launch(const WgradProblem& p, hipStream_t st) { return smallc_wgrad_launch_impl(p, true, st); }

hipError_t smallc_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    if (p.bf16) return smallc_bf16_wgrad_launch(p, st);
    return smallc_wgrad_launch_impl(p, false, st);
}

hipError_t smallc_wgrad_launch_impl(const WgradProblem& p, bool blocks, hipStream_t st) {
    const WgradF32Plan pl = wgrad_f32_plan(p, blocks);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e;
    switch (pl.NT) {
        case 2: e = wgrad_f32_launch_nt<2>(p, pl, st); break;
        case 3: e = wgrad_f32_launch_nt<3>(p, pl, st); break;
        case 5: e = wgrad_f32_launch_nt<5>(p, pl, st); break;
        case 9: e = wgrad_f32_launch_nt<9>(p, pl, st); break;
        default: e = wgrad_f32_launch_nt<kWgradNT>(p, pl, st); break;
    }
    if (e != hipSuccess) return e;
    return smallc_wgrad_reduce_launch(static_cast<const float*>(p.ws), p.dw, p.K, p.C, p.S, p.dw_sk, p.dw_sc, pl.grid, st);
}

}  // namespace conv1d
