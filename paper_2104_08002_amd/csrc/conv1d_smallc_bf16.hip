// Small-channel MFMA kernels (C, K <= 16), bfloat16 inputs, FP32 accumulation and output.
//
// Forward / backward-data (Eq. 2; Section 3.2).  One v_mfma_f32_16x16x32_bf16 multiplies a
// 16 x 32 slice of the weight matrix (16 filters x [2 taps x 16 channels]) with a 32 x 16 slice of
// the shifted-input matrix (the same [2 taps x 16 channels] x 16 adjacent output columns).  All
// weight slices of a layer (NP = ceil(S/2) of them: taps p and p+NP share a slice) stay in
// registers for the lifetime of a workgroup.  The input window (tile + halo) is transposed into
// LDS as [position][8 channels] 16-byte slots so that one lane's 8 k-values are one ds_read_b128.
// A batch-reduce GEMM over taps (Algorithm 2) would re-read the window once per tap; here the
// Toeplitz structure of the shifted-input matrix is used instead: when d divides 16 (G = 16/d), the operand
// for (tile j, tap p) is the operand for (tile j+1, tap p - 16/d), so a wave that owns T adjacent
// tiles loads each operand once and feeds up to T MFMAs from it.
//
// Backward-weight (Section 3.3, Algorithm 4) for d == 8.  The contraction runs over positions:
// A = dy (16 filters x 32 positions), B = x shifted by the tap (32 positions x 16 channels), one
// 16 x 16 accumulator per tap.  With d = 8 the B operand of (k-step t, tap s) equals that of
// (t+1, s-4); wave v of a workgroup owns the taps s = v (mod 4) and keeps their 13 operands in a
// register ring, loading one new operand per k-step.
#include <type_traits>

#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr unsigned kPermLo = 0x05040100u;  // {b.lo16, a.lo16} -> a.lo | b.lo << 16
constexpr unsigned kPermHi = 0x07060302u;  // {b.hi16, a.hi16} -> a.hi | b.hi << 16

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// ------------------------------------------------------------------------------------------------
// forward / backward-data
// ------------------------------------------------------------------------------------------------
// k-slot layout of one MFMA (lane = li + 16*kb, element j of the lane's 8):
//   channel r = 8*(kb & 1) + j,  tap s = p + NP*(kb >> 1)
// LDS: plane h = kb & 1 holds channels 8h..8h+7; slot (h*LPS + i) <-> input position G0 + i.
// Block staging (L16 kernels): blocks of 8 positions per window and the block count NB per position residue
// (NB = 2 mod 16, NB > blocks staged), both fixed by the tap count bucket and the dilation.
constexpr int blk_count(int NP, int d) { return (4 * 8 * 16 + (2 * NP - 1) * d + 7) / 8; }
constexpr int blk_nb(int NP, int d) {
    int nb = blk_count(NP, d) + 1;
    while (nb % 16 != 2) ++nb;
    return nb;
}

constexpr int kOS = 132;                    // row stride (floats) of an output staging tile: 4 rows apart -> 16 banks apart
constexpr int kOstSlots = 4 * 16 * kOS / 4;  // 16-byte slots of one staging buffer (4 consumer waves x 16 rows)

// Workgroup = 8 waves with two roles, one workgroup per CU, persistent over a contiguous strip of tiles
// (512 output columns of one sample each):
//   waves 0-3 ("consumers") keep the weight slices in registers and do nothing but LDS operand reads,
//             MFMAs and parking their finished 16 x 128 output tile in LDS;
//   waves 4-7 ("producers") fetch the window of tile t+2 from global memory into registers, transpose
//             the window of tile t+1 into the free LDS window buffer, and write the parked outputs of
//             tile t-1 to global memory as 16-byte stores (two 512-byte row segments per instruction).
// One workgroup barrier per tile hands the buffers over.  The matrix pipe of every SIMD is fed by a wave
// whose instruction stream is almost pure MFMA, and the memory traffic of both directions runs under it.
// LDS (16-byte slots): window buffer b at b*2*LPS (two planes of LPS slots), staging buffer b at
// 4*LPS + b*kOstSlots; the weight-slice assembly area aliases the staging buffers before the first tile.
// L16 (d = 8 or 16, padding and width multiples of 8): the window is staged in blocks of 8 positions with 16-byte
// global loads (a quarter of the load instructions of the dword path), and the LDS window is laid out block-transposed:
//   slot(position) = (position & 7) * NB + (position >> 3),   NB = LPS / 8 = 2 (mod 16)
// A producer lane that holds block b writes its eight positions to slots k*NB + b: the 16 lanes of a pass hit 16
// adjacent slots.  A consumer's 16 lanes read 16 adjacent positions from a block boundary on: slots u + 2k (first
// block) and u + 1 + 2k (second block) modulo 16, all different.  Both are conflict-free, and a step of 8 positions
// is still a step of one slot, so the operand walk keeps its immediate offsets.
template <int NP, int G, int T, int MAXT, bool FAST, bool L16>
__global__ __launch_bounds__(512, 2) void smallc_corr_bf16_kernel(CorrProblem p, int tiles_per_row, int ntiles, int LPS, int vec_out) {
    static_assert(T == 8, "the output staging tile is 16 rows x 128 columns");
    static_assert(!L16 || (FAST && (G == 1 || G == 2)), "block staging needs tile and tap shifts that are multiples of 8 positions");
    extern __shared__ u32x4 lds4[];
    constexpr int TQ = 4 * T * 16;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;   // consumer wave index / the consumer wave this producer wave serves
    const int rtid = tid & 255;  // thread index within the role group
    // producers have little to do but sit on the critical path of the barrier: let them issue first
    if (!consumer) __builtin_amdgcn_s_setprio(3);
    const int li = lane & 15;
    const int kb = lane >> 4;
    // lane (li, kb) accumulates filter li: its sums start from that filter's bias (requested here, at the start, so
    // that the first tile does not wait for it)
    const float bias_li = (!p.accumulate && p.epi.bias && li < p.M) ? p.epi.bias[li] : 0.f;
    const unsigned short* __restrict__ in = static_cast<const unsigned short*>(p.in);
    const unsigned short* __restrict__ wt = static_cast<const unsigned short*>(p.wt);
    const int d = (G > 0) ? 16 / (G > 0 ? G : 1) : p.d;
    // window slot 0 is the input position (tile start - P) rounded down to an even one, so that the dword loads of
    // position pairs stay aligned for any padding; the consumers skip the extra slot
    const int psh = p.P & 1;
    const int LP = TQ + (2 * NP - 1) * d + psh;
    const int LP2 = (LP + 1) >> 1;
    const int ntasks = 2 * LP2;
    const int ob = cw * T * 16;
    auto win = [&](int b) { return lds4 + b * 2 * LPS; };
    auto ost = [&](int b) { return reinterpret_cast<float*>(lds4 + 4 * LPS + b * kOstSlots) + cw * 16 * kOS; };

    // Contiguous strip of tiles per workgroup.  Workgroups are dealt round-robin to the 8 XCDs, so the
    // logical index puts neighbouring strips (which share halos) on the same XCD and its L2.
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    int t_begin = static_cast<int>(static_cast<long>(lid) * ntiles / gridDim.x);
    int t_wend = static_cast<int>(static_cast<long>(lid + 1) * ntiles / gridDim.x);  // end of the whole tiles
    // Half tiles.  With ntiles = base * grid + rem the strips above hold base or base + 1 tiles and the launch lasts
    // base + 1 tile times.  Where the fast output path applies (block staging, aligned output rows, no accumulation
    // into the output) and 2 rem <= grid, every workgroup takes base whole tiles instead, and the rem tiles left over
    // are cut into halves of TQ / 2 columns, one for each of the first 2 rem workgroups: it is that workgroup's last
    // item (index t_wend), staged like any tile that starts at its first column, computed by the four consumer
    // waves on 64 columns each.  The launch then lasts base + 1/2 tile times.
    int xn = 0, xO0 = 0;  // (sample, first column) of the workgroup's half tile
    bool has_half = false;
    if constexpr (L16) {
        const int grid = static_cast<int>(gridDim.x);
        const int base = ntiles / grid, rem = ntiles - base * grid;
        const bool plain = vec_out && !p.accumulate && p.M >= 15;
        if (plain && base >= 1 && rem > 0 && 2 * rem <= grid) {
            t_begin = lid * base;
            t_wend = t_begin + base;
            if (lid < 2 * rem) {
                const int X = grid * base + (lid >> 1);
                xn = X / tiles_per_row;
                xO0 = (X - xn * tiles_per_row) * TQ + (lid & 1) * (TQ / 2);
                has_half = xO0 < p.Wout;
            }
        }
    }
    const int t_end = t_wend + (has_half ? 1 : 0);

    // ---- producer side: window staging -----------------------------------------------------------
    // One staging task = 8 channels (half h) x 2 adjacent positions: 8 dwords in, two 16-byte
    // [position][8 channels] slots out.  FAST (even row starts and window origin): branch-free dword
    // loads from clamped addresses, masked when written to LDS, fetched one tile ahead.  Otherwise
    // element loads, done when the window is written.
    struct Task { unsigned v[8]; };
    auto task_h = [&](int task) { return task >= LP2 ? 1 : 0; };
    // (producer waves share their SIMD's issue slots with an MFMA wave, so their instruction count matters:
    // one add and one min per load; rows beyond R re-read row R-1, which is harmless because the weight
    // slices are zero there and the duplicated values are as finite as the originals)
    auto fetch_task = [&](int n, int G0, int task) -> Task {
        const int h = task_h(task);
        int g = G0 + 2 * (task - h * LP2);
        g = g < 0 ? 0 : (g > p.Win - 2 ? p.Win - 2 : g);
        const char* base = reinterpret_cast<const char*>(in + static_cast<long>(n) * p.in_sn);  // uniform
        const unsigned rowb = static_cast<unsigned>(p.Win) * 2u;                                     // uniform
        const unsigned offmax = static_cast<unsigned>((p.R - 1) * p.Win + g) * 2u;
        unsigned off = static_cast<unsigned>(8 * h * p.Win + g) * 2u;
        Task t;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            t.v[j] = *reinterpret_cast<const unsigned*>(base + min(off, offmax));
            off += rowb;
        }
        return t;
    };
    auto fetch_task_slow = [&](int n, int G0, int task) -> Task {
        const int h = task_h(task);
        const int g = G0 + 2 * (task - h * LP2);
        const int g0 = g < 0 ? 0 : (g > p.Win - 1 ? p.Win - 1 : g);
        const int g1 = g + 1 < 0 ? 0 : (g + 1 > p.Win - 1 ? p.Win - 1 : g + 1);
        const unsigned short* base = in + static_cast<long>(n) * p.in_sn;
        Task t;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = min(8 * h + j, p.R - 1);
            const unsigned lo = (g >= 0 && g < p.Win) ? base[static_cast<unsigned>(r * p.Win + g0)] : 0u;
            const unsigned hi = (g + 1 >= 0 && g + 1 < p.Win) ? base[static_cast<unsigned>(r * p.Win + g1)] : 0u;
            t.v[j] = lo | (hi << 16);
        }
        return t;
    };
    // FAST windows that lie inside the row need no masking at all (see above for the channel rows);
    // `edge` is uniform per tile
    auto store_task = [&](u32x4* wb, int G0, int task, const Task& t, bool edge) {
        const int h = task_h(task);
        const int pp = task - h * LP2;
        u32x4 ev, od;
        if (FAST && !edge) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                ev[q] = __builtin_amdgcn_perm(t.v[2 * q + 1], t.v[2 * q], kPermLo);
                od[q] = __builtin_amdgcn_perm(t.v[2 * q + 1], t.v[2 * q], kPermHi);
            }
        } else {
            const int g = G0 + 2 * pp;
            // FAST: a pair is inside or outside the row as a whole (g and Win are even)
            const bool pos_ok = !FAST || (g >= 0 && g < p.Win);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned a = (pos_ok && 8 * h + 2 * q < p.R) ? t.v[2 * q] : 0u;
                const unsigned b = (pos_ok && 8 * h + 2 * q + 1 < p.R) ? t.v[2 * q + 1] : 0u;
                ev[q] = __builtin_amdgcn_perm(b, a, kPermLo);
                od[q] = __builtin_amdgcn_perm(b, a, kPermHi);
            }
        }
        wb[h * LPS + 2 * pp] = ev;
        wb[h * LPS + 2 * pp + 1] = od;
    };
    // (sample, first column) of a tile near the one the loop is at, by counting from it: a uniform integer division
    // is ~25 vector instructions, and the producers would do three per tile next to the MFMA wave of their SIMD
    const int row_w = tiles_per_row * TQ;
    int cur_t = t_begin, cur_n = t_begin / tiles_per_row, cur_O0 = (t_begin - cur_n * tiles_per_row) * TQ;
    struct TilePos {
        int n, O0;
    };
    auto tile_pos = [&](int t) -> TilePos {
        if (has_half && t >= t_wend) return TilePos{xn, xO0};
        TilePos tp{cur_n, cur_O0 + (t - cur_t) * TQ};
        while (tp.O0 >= row_w) {
            tp.O0 -= row_w;
            ++tp.n;
        }
        while (tp.O0 < 0) {
            tp.O0 += row_w;
            --tp.n;
        }
        return tp;
    };
    auto tile_advance = [&]() {
        ++cur_t;
        cur_O0 += TQ;
        if (cur_O0 >= row_w) {
            cur_O0 = 0;
            ++cur_n;
        }
    };
    // ---- block staging (L16): one task = 8 channels (half h) x 8 adjacent positions, 8 loads of 16 bytes ----------
    // (compile-time geometry: the LDS offsets of a lane's eight slots become immediates)
    constexpr int NB = L16 ? blk_nb(NP, 16 / (G > 0 ? G : 1)) : 1;     // the host passes LPS = 8 * NB
    constexpr int NBLK = L16 ? blk_count(NP, 16 / (G > 0 ? G : 1)) : 1;  // blocks staged per plane; 2 * NBLK <= 256
    u32x4 pre16[L16 ? 8 : 1];
    auto prefetch16 = [&](int t) {
        const TilePos tp = tile_pos(t);
        const int n = tp.n, G0 = tp.O0 - p.P;  // a multiple of 8
        const int task = rtid < 2 * NBLK ? rtid : 2 * NBLK - 1;
        const int h = task >= NBLK ? 1 : 0;
        int g = G0 + 8 * (task - h * NBLK);
        g = g < 0 ? 0 : (g > p.Win - 8 ? p.Win - 8 : g);
        const char* base = reinterpret_cast<const char*>(in + static_cast<long>(n) * p.in_sn);  // uniform
        const unsigned rowb = static_cast<unsigned>(p.Win) * 2u;                                     // uniform
        const unsigned offmax = static_cast<unsigned>((p.R - 1) * p.Win + g) * 2u;
        unsigned off = static_cast<unsigned>(8 * h * p.Win + g) * 2u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            pre16[j] = *reinterpret_cast<const u32x4*>(base + min(off, offmax));
            off += rowb;
        }
    };
    auto commit16 = [&](int t, u32x4* wb) {
        const TilePos tp = tile_pos(t);
        const int G0 = tp.O0 - p.P;
        const bool edge = G0 < 0 || G0 + 8 * NBLK > p.Win;  // uniform
        if (rtid < 2 * NBLK) {
            const int h = rtid >= NBLK ? 1 : 0;
            const int blk = rtid - h * NBLK;
            const int g = G0 + 8 * blk;
            // a block is inside or outside the row as a whole (row length and padding are multiples of 8)
            const bool pos_ok = g >= 0 && g + 8 <= p.Win;
            u32x4* dst = wb + h * LPS + blk;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x4 ev, od;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    unsigned a = pre16[2 * q][i], b = pre16[2 * q + 1][i];
                    if (edge) {
                        a = (pos_ok && 8 * h + 2 * q < p.R) ? a : 0u;
                        b = (pos_ok && 8 * h + 2 * q + 1 < p.R) ? b : 0u;
                    }
                    ev[q] = __builtin_amdgcn_perm(b, a, kPermLo);
                    od[q] = __builtin_amdgcn_perm(b, a, kPermHi);
                }
                dst[(2 * i) * NB] = ev;
                dst[(2 * i + 1) * NB] = od;
            }
        }
    };
    Task pre[(FAST && !L16) ? MAXT : 1];
    auto prefetch = [&](int t) {  // producers: window of tile t -> registers
        if constexpr (L16) {
            prefetch16(t);
        } else if constexpr (FAST) {
            const TilePos tp = tile_pos(t);
            const int n = tp.n, G0 = tp.O0 - p.P - psh;
#pragma unroll
            for (int k = 0; k < MAXT; ++k) {
                const int task = rtid + k * 256;
                pre[k] = fetch_task(n, G0, task < ntasks ? task : ntasks - 1);
            }
        }
    };
    auto commit = [&](int t, u32x4* wb) {  // producers: registers (or memory) -> LDS window of tile t
        if constexpr (L16) {
            commit16(t, wb);
            return;
        }
        const TilePos tp = tile_pos(t);
        const int n = tp.n, G0 = tp.O0 - p.P - psh;
        const bool edge = G0 < 0 || G0 + 2 * LP2 > p.Win;
        if constexpr (FAST) {
#pragma unroll
            for (int k = 0; k < MAXT; ++k) {
                const int task = rtid + k * 256;
                if (task < ntasks) store_task(wb, G0, task, pre[k], edge);
            }
            for (int task = rtid + MAXT * 256; task < ntasks; task += 256) store_task(wb, G0, task, fetch_task(n, G0, task), edge);
        } else {
            for (int task = rtid; task < ntasks; task += 256) store_task(wb, G0, task, fetch_task_slow(n, G0, task), true);
        }
    };
    // producers: parked outputs of tile t (staging buffer b) -> global memory
    auto flush = [&](int t, int b) {
        const TilePos tp = tile_pos(t);
        const int n = tp.n, O0 = tp.O0;
        const float* src = ost(b);
        // the bias is already in the sums (the accumulators start from it); ReLU and the bfloat16 conversion happen
        // here, behind branches that are uniform for the launch
        if (vec_out) {
            const int orow = lane >> 5, ocol = 4 * (lane & 31);
            const bool col_ok = O0 + ob + ocol < p.Wout;
            // All eight LDS reads are issued before the first store: a read-wait-store chain per row pair would put
            // eight LDS round trips in a row on the producers' critical path.  Each variant of the store loop sits
            // behind a branch that is uniform for the launch, so the plain float path has no branch inside.
            f32x4 v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = *reinterpret_cast<const f32x4*>(src + (2 * q + orow) * kOS + ocol);
            const long base = static_cast<long>(n) * p.out_sn + O0 + ob;                   // uniform
            const unsigned lane_off = static_cast<unsigned>(orow * p.Wout + ocol);
            if (!p.accumulate && !p.epi.relu && !p.epi.out_bf16) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (col_ok && 2 * q + orow < p.M)
                        __builtin_nontemporal_store(v[q], reinterpret_cast<f32x4*>(p.out + base + static_cast<long>(2 * q) * p.Wout + lane_off));
            } else if (p.accumulate) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (col_ok && 2 * q + orow < p.M) {
                        f32x4* dst = reinterpret_cast<f32x4*>(p.out + base + static_cast<long>(2 * q) * p.Wout + lane_off);
                        *dst = *dst + v[q];
                    }
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (col_ok && 2 * q + orow < p.M)
                        epi_store4_nt(p.epi, p.out, base + static_cast<long>(2 * q) * p.Wout + lane_off, epi_apply4(p.epi, v[q], 0.f));
            }
        } else {
            for (int idx = lane; idx < 16 * T * 16; idx += 64) {
                const int m = idx / (T * 16), col = idx - m * (T * 16);
                const int o = O0 + ob + col;
                if (m < p.M && o < p.Wout) {
                    const long di = static_cast<long>(n) * p.out_sn + static_cast<long>(m) * p.Wout + o;
                    if (p.accumulate) {
                        p.out[di] += src[m * kOS + col];
                    } else {
                        epi_store(p.epi, p.out, di, epi_apply(p.epi, src[m * kOS + col], 0.f));
                    }
                }
            }
        }
    };

    // ---- prologue: weight slices (all waves copy, consumers assemble) and the first window ---------
    // Entry e = slice*64 + lane holds wt(m, 8h..8h+7, s) for m = lane & 15, h = (lane >> 4) & 1,
    // s = slice + NP*(lane >> 5).  The raw tensor is copied into LDS with 16-byte loads (all of a
    // thread's loads in flight at once), the entries are gathered from that copy, and each consumer wave
    // then keeps all NP slices in registers.  Both areas alias the output staging buffers.
    u32x4* entries = lds4 + 4 * LPS;
    unsigned short* raw = reinterpret_cast<unsigned short*>(entries + NP * 64);
    // Fused backward: the first 4*S workgroups also finish the backward-weight pass that ran just before (its second
    // stage), in the shadow of this prologue's memory latency; the group sums sit behind the raw weight copy.
    epi_f32x4* tail_part = reinterpret_cast<epi_f32x4*>(entries + 2 * NP * 64);
    const bool tail_job = p.tail.ws != nullptr && static_cast<int>(blockIdx.x) < 4 * p.tail.S;
    if (p.w_contig) {
        const int nW = p.M * p.R * p.S;
        constexpr int NV = (16 * 16 * 2 * NP / 8 + 511) / 512;  // 16-byte pieces per thread, worst case
        if ((reinterpret_cast<uintptr_t>(wt) & 15) == 0) {
            const int nvec = nW / 8;
            u32x4 tmp[NV];
#pragma unroll
            for (int k = 0; k < NV; ++k) tmp[k] = reinterpret_cast<const u32x4*>(wt)[min(tid + k * 512, nvec > 0 ? nvec - 1 : 0)];
            if (!consumer && t_begin < t_end) prefetch(t_begin);  // queued behind the weight loads
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < NV; ++k)
                if (tid + k * 512 < nvec) reinterpret_cast<u32x4*>(raw)[tid + k * 512] = tmp[k];
            for (int e = nvec * 8 + tid; e < nW; e += 512) raw[e] = wt[e];
        } else {
            for (int e = tid; e < nW; e += 512) raw[e] = wt[e];
            if (!consumer && t_begin < t_end) prefetch(t_begin);
        }
    } else if (!consumer && t_begin < t_end) {
        prefetch(t_begin);
    }
    if (tail_job) wgrad_tail_phase1(p.tail, blockIdx.x, tid, tail_part);
    __syncthreads();
    if (tail_job) wgrad_tail_phase2(p.tail, blockIdx.x, tid, tail_part);
    bf16x8 wreg[NP];
    if (consumer) {
        // Entry e = rtid + 256 k: the lane part (filter m, channel half h, tap half) is the same for every k, the
        // slice advances by 4 per k.  Everything that needs a multiplication is worked out once per thread (integer
        // multiplies run at a quarter of the ALU rate, and this code is on the critical path of every workgroup).
        constexpr int NE = (NP * 64 + 255) / 256;
        const int l = rtid & 63;
        const int m = l & 15, h = (l >> 4) & 1, s0 = (rtid >> 6) + NP * (l >> 5);
        const int wsm = static_cast<int>(p.w_sm), wsr = static_cast<int>(p.w_sr), wss = static_cast<int>(p.w_ss);
        const int bm = min(m, p.M - 1) * wsm + static_cast<int>(p.w_s0);
        int roff[8];  // offset of channel 8 h + j (clamped to the last channel)
#pragma unroll
        for (int j = 0; j < 8; ++j) roff[j] = min(8 * h + j, p.R - 1) * wsr;
        unsigned wv[NE][8];
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int base = bm + min(s0 + 4 * k, p.S - 1) * wss;
            if (p.w_contig) {
#pragma unroll
                for (int j = 0; j < 8; ++j) wv[k][j] = raw[base + roff[j]];
            } else {  // a block of a larger tensor: gather straight from global memory
#pragma unroll
                for (int j = 0; j < 8; ++j) wv[k][j] = wt[base + roff[j]];
            }
        }
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const int e = rtid + k * 256;
            const bool ok = m < p.M && s0 + 4 * k < p.S;
            unsigned v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = (ok && 8 * h + j < p.R) ? wv[k][j] : 0u;
            if (e < NP * 64) entries[e] = u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        }
    } else if (t_begin < t_end) {
        commit(t_begin, win(0));
        if (t_begin + 1 < t_end) prefetch(t_begin + 1);
    }
    __syncthreads();
    if (consumer) {
#pragma unroll
        for (int pi = 0; pi < NP; ++pi) wreg[pi] = as_bf16x8(entries[pi * 64 + lane]);
    }
    __syncthreads();  // the slice entries alias the staging buffers: every wave has its copy before anyone parks

    // ---- consumer side: one tile's reduction, parked in LDS ------------------------------------------
    // (TT position blocks per wave from column obx of the tile on: T and ob for a whole tile, T / 2 and ob / 2 for a half tile)
    auto compute_tt = [&](auto tt_, int obx, const u32x4* wb, float* dst) {
        constexpr int TT = decltype(tt_)::value;
        f32x4 acc[TT];
#pragma unroll
        for (int j = 0; j < TT; ++j) acc[j] = f32x4{bias_li, bias_li, bias_li, bias_li};
        // (L16: slot(position) = (position & 7) * NB + (position >> 3); every offset but the lane's own is a multiple of 8)
        const u32x4* bbase = L16 ? wb + (kb & 1) * LPS + (li & 7) * NB + (li >> 3) + ((obx + (kb >> 1) * NP * d) >> 3)
                                 : wb + (kb & 1) * LPS + obx + li + (kb >> 1) * NP * d + psh;
        // The input fragment is the A operand and the weight slice the B operand, so the accumulator tile is
        // [position][filter]: lane (li, kb) holds filter li at the 4 adjacent columns 4 kb .. 4 kb + 3 of tile j,
        // parked with one 16-byte LDS write.
        auto park = [&](int j) { *reinterpret_cast<f32x4*>(dst + li * kOS + j * 16 + 4 * kb) = acc[j]; };
        if constexpr (G > 0) {
            // Operand m serves (tile j, slice m - G*j) for every j.  Operands are fetched PF steps ahead
            // of their MFMAs; tile j is complete after step G*j + NP - 1 and is parked two steps later.
            // The scheduling barriers pin this interleaving.
            constexpr int PF = 3;
            constexpr int D = L16 ? (16 / (G > 0 ? G : 1)) / 8 : 16 / (G > 0 ? G : 1);  // slots between consecutive operands
            constexpr int NF = G * (TT - 1) + NP;
            // rotating: operand m lives in slot m % (PF + 2); one slot more than the look-ahead needs, so that a
            // read never targets the registers of the operand whose MFMAs have only just been issued
            bf16x8 fr[PF + 2];
#pragma unroll
            for (int m = 0; m < PF && m < NF; ++m) fr[m] = as_bf16x8(bbase[m * D]);
#pragma unroll
            for (int m = 0; m < NF; ++m) {
                if (m + PF < NF) fr[(m + PF) % (PF + 2)] = as_bf16x8(bbase[(m + PF) * D]);
#pragma unroll
                for (int j = 0; j < TT; ++j)
                    if (G * j + NP - 1 == m - 2) park(j);
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    const int pi = m - G * j;
                    if (pi >= 0 && pi < NP) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fr[m % (PF + 2)], wreg[pi < 0 ? 0 : (pi >= NP ? 0 : pi)], acc[j], 0, 0, 0);
                }
                // issue order within the step: one MFMA, one LDS operation, one MFMA, ... so that the operand
                // read and the parking writes go out in the shadow of the MFMAs instead of in front of them
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x080, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int j = 0; j < TT; ++j)
                if (G * j + NP - 1 > NF - 3) park(j);
        } else {
            // dilations without operand sharing between tiles: every (tile, slice) pair reads its own operand
#pragma unroll
            for (int pi = 0; pi < NP; ++pi) {
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    const bf16x8 f = as_bf16x8(bbase[16 * j + pi * d]);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f, wreg[pi], acc[j], 0, 0, 0);
                }
            }
#pragma unroll
            for (int j = 0; j < TT; ++j) park(j);
        }
    };
    auto compute = [&](const u32x4* wb, float* dst) { compute_tt(std::integral_constant<int, T>{}, ob, wb, dst); };
    auto compute_half = [&](const u32x4* wb, float* dst) { compute_tt(std::integral_constant<int, T / 2>{}, ob / 2, wb, dst); };


    // ---- steady state, block staging ---------------------------------------------------------------
    // Measured on this kernel: every instruction a producer wave issues, vector or scalar, lengthens the tile by about
    // 4.4 cycles (it shares its SIMD's issue with the MFMA wave), so the producers' path for tiles that lie inside
    // their row is stripped to the loads, the 32 byte permutes, the LDS accesses and the stores: everything that
    // depends on the thread only (row offsets, LDS addresses, output offsets) is worked out once, what depends on the
    // tile only is scalar, and tiles at a row edge, ragged row ends and the epilogue variants take the general lambdas.
    if constexpr (L16) {
        if (consumer) {
            int k = 0;
            for (int t = t_begin; t < t_end; ++t, ++k) {
                if (t < t_wend) {
                    compute(win(k & 1), ost(k & 1));
                } else {
                    compute_half(win(k & 1), ost(k & 1));
                }
                __syncthreads();
            }
            return;
        }
        const int task = rtid < 2 * NBLK ? rtid : 2 * NBLK - 1;  // idle threads repeat the last task: same data, same slots
        const int h = task >= NBLK ? 1 : 0;
        const int blk = task - h * NBLK;
        unsigned voff_ld[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) voff_ld[j] = static_cast<unsigned>(min(8 * h + j, p.R - 1) * p.Win + 8 * blk) * 2u;
        const int ldsw = h * LPS + blk;
        const int orow = lane >> 5, ocol = 4 * (lane & 31);
        unsigned voff_st[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) voff_st[q] = static_cast<unsigned>((2 * q + orow) * p.Wout + ocol) * 4u;
        const int ldsr = orow * kOS + ocol;
        const bool plain_out = vec_out && !p.accumulate && p.M >= 15;
        // one 4-column piece of an output row: ReLU and the bfloat16 conversion behind launch-uniform branches (the bias
        // is already in the sums).  `off` is the byte offset in a float tensor.  Non-temporal stores: the outputs are not
        // read again by this launch, and measured 1.9 us per launch faster than plain stores (4.5 us with nothing cached).
        const bool relu = p.epi.relu, out16 = p.epi.out_bf16;
        auto put = [&](f32x4 v, char* base, unsigned off) {
            if (relu) {
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = v[i] < 0.f ? 0.f : v[i];  // (a comparison, not a max: NaN stays NaN)
            }
            if (out16) {
                __builtin_nontemporal_store(__builtin_convertvector(v, epi_bf16x4), reinterpret_cast<epi_bf16x4*>(base + (off >> 1)));
            } else {
                __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(base + off));
            }
        };
        const int osh = out16 ? 1 : 2;  // log2 of the output element size
        const bool last_row_ok = orow < p.M - 14;
        auto interior = [&](int O0) { return O0 - p.P >= 0 && O0 - p.P + 8 * NBLK <= p.Win; };
        auto prefetch_plain = [&](int n, int O0) {
            const char* base = reinterpret_cast<const char*>(in + static_cast<long>(n) * p.in_sn + (O0 - p.P));  // uniform
#pragma unroll
            for (int j = 0; j < 8; ++j) pre16[j] = *reinterpret_cast<const u32x4*>(base + voff_ld[j]);
        };
        auto commit_plain = [&](u32x4* wb) {
            u32x4* dst = wb + ldsw;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x4 ev, od;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    ev[q] = __builtin_amdgcn_perm(pre16[2 * q + 1][i], pre16[2 * q][i], kPermLo);
                    od[q] = __builtin_amdgcn_perm(pre16[2 * q + 1][i], pre16[2 * q][i], kPermHi);
                }
                dst[(2 * i) * NB] = ev;
                dst[(2 * i + 1) * NB] = od;
            }
        };
        auto flush_plain = [&](int n, int O0, int b) {
            const float* src = ost(b) + ldsr;
            f32x4 v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = *reinterpret_cast<const f32x4*>(src + 2 * q * kOS);
            char* base = reinterpret_cast<char*>(p.out) + ((static_cast<long>(n) * p.out_sn + O0 + ob) << osh);  // uniform
#pragma unroll
            for (int q = 0; q < 7; ++q) put(v[q], base, voff_st[q]);
            if (last_row_ok) put(v[7], base, voff_st[7]);
        };
        // the workgroup's half tile: 16 rows x 64 columns per wave, 4 rows per store instruction
        auto flush_half = [&](int b) {
            const int hrow = lane >> 4, hcol = 4 * (lane & 15);
            const float* src = ost(b) + hrow * kOS + hcol;
            f32x4 v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const f32x4*>(src + 4 * q * kOS);
            const int col = xO0 + ob / 2 + hcol;
            char* base = reinterpret_cast<char*>(p.out) + ((static_cast<long>(xn) * p.out_sn + col) << osh);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (col < p.Wout && 4 * q + hrow < p.M) put(v[q], base, static_cast<unsigned>((4 * q + hrow) * p.Wout) * 4u);
        };
        // (sample, first column) of tiles t - 1 .. t + 2, moved along with the loop
        TilePos tm1{0, 0}, t0 = tile_pos(t_begin), tp1 = tile_pos(t_begin + 1), tp2 = tile_pos(t_begin + 2);
        auto next_pos = [&](TilePos a) {
            a.O0 += TQ;
            if (a.O0 >= row_w) {
                a.O0 = 0;
                ++a.n;
            }
            return a;
        };
        int k = 0;
        for (int t = t_begin; t < t_end; ++t, ++k) {
            if (t + 1 < t_end) {
                if (interior(tp1.O0)) {
                    commit_plain(win((k + 1) & 1));
                } else {
                    commit16(t + 1, win((k + 1) & 1));
                }
                if (t + 2 < t_end) {
                    if (interior(tp2.O0)) {
                        prefetch_plain(tp2.n, tp2.O0);
                    } else {
                        prefetch16(t + 2);
                    }
                }
            }
            if (k > 0) {
                if (plain_out && tm1.O0 + TQ <= p.Wout) {
                    flush_plain(tm1.n, tm1.O0, (k - 1) & 1);
                } else {
                    flush(t - 1, (k - 1) & 1);
                }
            }
            __syncthreads();
            tile_advance();
            tm1 = t0;
            t0 = tp1;
            tp1 = tp2;
            tp2 = (has_half && t + 3 >= t_wend) ? TilePos{xn, xO0} : next_pos(tp2);
        }
        if (k > 0) {
            if (has_half) {
                flush_half((k - 1) & 1);
            } else {
                flush(t_end - 1, (k - 1) & 1);
            }
        }
        return;
    }

    // ---- steady state -----------------------------------------------------------------------------
    int k = 0;
    for (int t = t_begin; t < t_end; ++t, ++k) {
        if (consumer) {
            compute(win(k & 1), ost(k & 1));
        } else {
            if (t + 1 < t_end) {
                commit(t + 1, win((k + 1) & 1));
                if (t + 2 < t_end) prefetch(t + 2);
            }
            if (k > 0) flush(t - 1, (k - 1) & 1);
        }
        __syncthreads();
        tile_advance();
    }
    if (!consumer && k > 0) flush(t_end - 1, (k - 1) & 1);
}

constexpr int kCorrT = 8;
constexpr int kCorrMaxT = 4;
constexpr int kNPBuckets[] = {3, 5, 9, 13, 17, 26};

struct CorrPlan {
    int NP, G, LPS, tiles_per_row, ntiles, fast, vec_out, l16;
    size_t lds_bytes;
    bool ok;
};

CorrPlan corr_plan(const CorrProblem& p) {
    CorrPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.R > 16 || p.M > 16) return pl;
    if (static_cast<long>(p.R) * p.Win >= (1L << 30)) return pl;  // 32-bit element offsets within one sample
    const int need = (p.S + 1) / 2;
    pl.NP = 0;
    for (int b : kNPBuckets) {
        if (b >= need) { pl.NP = b; break; }
    }
    if (pl.NP == 0) return pl;
    // operand reuse across tiles pays when a tile shift is a few taps (d = 4, 8, 16); for d = 1, 2 the
    // shift is 16 or 8 taps, little is shared and the unrolled schedule gets very long
    pl.G = (p.d == 1 || p.d == 2 || p.d == 4 || p.d == 8 || p.d == 16) ? 16 / p.d : 0;
    constexpr int TQ = 4 * kCorrT * 16;
    const long LP = TQ + static_cast<long>(2 * pl.NP - 1) * p.d + 1;  // + the slot in front of an odd window origin
    const long LPS = (LP + 2 + 7) / 8 * 8;
    // [2 window buffers | 2 output staging buffers]; the weight-slice assembly area aliases the staging buffers
    const long slots = 4 * LPS + 2 * kOstSlots;
    if (slots * 16 > kLdsBudget) return pl;  // one workgroup per CU
    pl.LPS = static_cast<int>(LPS);
    pl.l16 = 0;
    pl.tiles_per_row = cdiv(p.Wout, TQ);
    const long nt = static_cast<long>(p.N) * pl.tiles_per_row;
    if (nt > 0x7fffffffL) return pl;
    pl.ntiles = static_cast<int>(nt);
    pl.lds_bytes = static_cast<size_t>(slots) * 16;
    // dword loads of position pairs need even row starts and an even window origin
    pl.fast = (p.Win % 2 == 0) && (p.in_sn % 2 == 0) && (reinterpret_cast<uintptr_t>(p.in) % 4 == 0) && p.Win >= 2;
    pl.vec_out = (p.Wout % 4 == 0) && (reinterpret_cast<uintptr_t>(p.out) % 16 == 0) &&
                 static_cast<long>(p.M) * p.Wout < (1L << 30);
    // block staging: see the kernel.  NB = 2 (mod 16) blocks per position residue, one plane = 8 * NB slots
    if (pl.fast && (pl.G == 1 || pl.G == 2) && p.P % 8 == 0 && p.Win % 8 == 0 && p.in_sn % 8 == 0 && p.Win >= 8 &&
        reinterpret_cast<uintptr_t>(p.in) % 16 == 0) {
        const long nblk = blk_count(pl.NP, p.d);
        const long nb = blk_nb(pl.NP, p.d);
        const long slots16 = 4 * 8 * nb + 2 * kOstSlots;
        if (2 * nblk <= 256 && slots16 * 16 <= kLdsBudget) {
            pl.l16 = 1;
            pl.LPS = static_cast<int>(8 * nb);
            pl.lds_bytes = static_cast<size_t>(slots16) * 16;
        }
    }
    pl.ok = true;
    return pl;
}

template <int NP, int G, bool FAST, bool L16 = false>
hipError_t corr_launch_f(const CorrProblem& p, const CorrPlan& pl, hipStream_t st) {
    auto kern = smallc_corr_bf16_kernel<NP, G, kCorrT, kCorrMaxT, FAST, L16>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    const int grid = pl.ntiles < kNumCU ? pl.ntiles : kNumCU;
    return launch_kernel(kern, dim3(grid), dim3(512), pl.lds_bytes, st, p, pl.tiles_per_row, pl.ntiles, pl.LPS, pl.vec_out);
}

template <int NP, int G>
hipError_t corr_launch_t(const CorrProblem& p, const CorrPlan& pl, hipStream_t st) {
    if constexpr (G == 1 || G == 2) {
        if (pl.l16) return corr_launch_f<NP, G, true, true>(p, pl, st);
    }
    return pl.fast ? corr_launch_f<NP, G, true>(p, pl, st) : corr_launch_f<NP, G, false>(p, pl, st);
}

template <int NP>
hipError_t corr_launch_np(const CorrProblem& p, const CorrPlan& pl, hipStream_t st) {
    switch (pl.G) {
        case 1: return corr_launch_t<NP, 1>(p, pl, st);
        case 4:
            return corr_launch_t<NP, 4>(p, pl, st);
        case 8: return corr_launch_t<NP, 8>(p, pl, st);
        case 16: return corr_launch_t<NP, 16>(p, pl, st);
        case 2: return corr_launch_t<NP, 2>(p, pl, st);
        default: return corr_launch_t<NP, 0>(p, pl, st);
    }
}

// ------------------------------------------------------------------------------------------------
// backward-weight, d == 8
// ------------------------------------------------------------------------------------------------
// A workgroup owns a strip of one sample: consecutive units of 416 output columns (13 k-steps of 32; the
// last unit of a strip may be shorter).  Columns are handled as 16-byte slots of 8 bf16: dy slot i <-> q = 8i..8i+7,
// x slot i <-> input positions 8i - P .. 8i - P + 7 (so tap s reads x slot = dy slot + s).
// Wave v owns taps s = v + 4i (i < 13).  In k-step t its lane (li, kb) needs, for tap slot i, the
// x operand X_f = x[li][slots 4f + v + kb], f = t + i: a sliding window of 13 operands kept in a
// register ring, refilled with X_{t+13} in step t.  The refills of unit j therefore read exactly x
// slots [52(j+1), 52(j+1) + 55): LDS holds one such "period" of x and one unit of dy at a time, and
// the halo never has to be staged again.  The next period/unit is fetched from global memory into
// registers while the MFMAs of the current unit run.
//   xbuf [16][kXR]  row = channel, slot i <-> x slot 52(j+1) + i      (kXP = 60 slots staged)
//   dybuf[16][kDR]  row = filter,  slot i <-> dy slot 52j + i         (j, and the slots, count from the strip's start)
constexpr int kNT = 13;            // taps per wave == operands in the ring == k-steps per unit
constexpr int kUnitSlots = 4 * kNT;  // 52 slots = 416 columns
constexpr int kXP = 60;            // x slots staged per period (52 + look-ahead of the highest tap slot)
constexpr int kXR = 61, kDR = 53;  // LDS row strides in slots (odd: rows spread over the bank groups)
constexpr int kWgMaxS = 7;         // 16 * (60 + 52) slots / 256 producer threads

// Workgroup = 8 waves, one workgroup per CU: waves 0-3 ("consumers", one per tap class) do the operand
// reads and MFMAs; waves 4-7 ("producers") fetch stage s+2 from global memory into registers and write
// stage s+1 into the free half of the double-buffered LDS while the consumers work on stage s.  Stage s of
// a strip is {x period s+1, dy unit s}; one workgroup barrier per unit hands the buffers over.
template <bool FAST>
__global__ __launch_bounds__(512, 2) void smallc_wgrad_bf16_d8_kernel(WgradProblem p, int SPR, int KSS, int KS) {
    __shared__ u32x4 xbuf[2][16 * kXR];
    __shared__ u32x4 dybuf[2][16 * kDR];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;  // tap class of a consumer wave
    const int rtid = tid & 255;
    // producers have little to do but sit on the critical path of the barrier: let them issue first
    if (!consumer) __builtin_amdgcn_s_setprio(3);
    const int li = lane & 15;
    const int kb = lane >> 4;
    const unsigned short* __restrict__ x = static_cast<const unsigned short*>(p.x);
    const unsigned short* __restrict__ dy = static_cast<const unsigned short*>(p.dy);
    // A strip is a run of KSS k-steps (32 columns each) of one sample, cut where the columns divide evenly over the
    // workgroups, not at unit boundaries: its units are numbered from 0, and the last one may have fewer than 13
    // k-steps (the consumers stop there; what is staged beyond the strip's last column is zero).
    const int n = blockIdx.x / SPR;
    const int ks0 = (blockIdx.x - n * SPR) * KSS;
    const int ks1 = min(ks0 + KSS, KS);
    const int sb = 4 * ks0;  // first dy slot of the strip
    const int j0 = 0;
    const int j1 = (ks1 - ks0 + kNT - 1) / kNT;
    const int last_steps = (ks1 - ks0) - (j1 - 1) * kNT;  // k-steps of the last unit: 1 .. 13
    const int Qb = min(ks1 * 32, p.Q);  // this strip's dy columns end here
    const unsigned short* xn = x + static_cast<long>(n) * p.x_sn;
    const unsigned short* dyn = dy + static_cast<long>(n) * p.dy_sn;

    constexpr int NX = 16 * kXP, NS = 16 * (kXP + kUnitSlots);
    // Staging slot e of stage j: e < NX is x period j+1 (row e / kXP), the rest is dy unit j.  Everything
    // about a slot except its column is fixed for a thread, so it is worked out once (producer waves share
    // their SIMD's issue slots with an MFMA wave: every VALU instruction they do not execute matters).
    // FAST (all widths, the padding and the pointers are multiples of 8 elements): one 16-byte load
    // from a clamped address, masked when it is written to LDS; a slot is then inside or outside
    // its row as a whole.  Otherwise element loads, done when the stage is written.
    struct Slot {
        unsigned off;  // element offset of the (clamped) source row from the sample's x or dy base
        int g0;        // column of the slot in stage 0 of this strip (advances by 416 per stage)
        int lds;       // index into xbuf[b] / dybuf[b]; bit 30: x (else dy), bit 29: row beyond C or K
    };
    constexpr int kIsX = 1 << 30, kRowBad = 1 << 29, kLdsMask = kRowBad - 1;
    auto make_slot = [&](int e) -> Slot {
        Slot w;
        if (e < NX) {
            const int r = e / kXP, i = e - r * kXP;
            w.off = static_cast<unsigned>(min(r, p.C - 1) * p.W);
            w.g0 = 8 * (sb + kUnitSlots + i) - p.P;
            w.lds = (r * kXR + i) | kIsX | (r < p.C ? 0 : kRowBad);
        } else {
            const int e2 = e - NX, r = e2 / kUnitSlots, i = e2 - r * kUnitSlots;
            w.off = static_cast<unsigned>(min(r, p.K - 1) * p.Q);
            w.g0 = 8 * (sb + i);
            w.lds = (r * kDR + i) | (r < p.K ? 0 : kRowBad);
        }
        return w;
    };
    auto fetch = [&](const Slot& w, int stage) -> u32x4 {  // stage counts from 0 at unit j0
        const int g = w.g0 + stage * (kUnitSlots * 8);
        const bool is_x = w.lds & kIsX;
        const int limit = is_x ? p.W : Qb;
        const unsigned short* row = (is_x ? xn : dyn) + w.off;
        if constexpr (FAST) {
            const int lim = limit - 8;  // >= 0 on this path (checked by the host)
            return *reinterpret_cast<const u32x4*>(row + (g < 0 ? 0 : (g > lim ? lim : g)));
        } else {
            unsigned t[8];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const int gj = g + jj;
                const int gc = gj < 0 ? 0 : (gj > limit - 1 ? limit - 1 : gj);
                t[jj] = (gj >= 0 && gj < limit) ? row[gc] : 0u;
            }
            return u32x4{t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16)};
        }
    };
    auto commit = [&](const Slot& w, int b, int stage, u32x4 v) {
        const int g = w.g0 + stage * (kUnitSlots * 8);
        const bool is_x = w.lds & kIsX;
        const int limit = is_x ? p.W : Qb;
        const bool ok = !(w.lds & kRowBad) && (!FAST || (g >= 0 && g + 8 <= limit));
        if (!ok) v = u32x4{0u, 0u, 0u, 0u};
        (is_x ? xbuf[b] : dybuf[b])[w.lds & kLdsMask] = v;
    };
    Slot slot[kWgMaxS];
#pragma unroll
    for (int k = 0; k < kWgMaxS; ++k) slot[k] = make_slot(min(rtid + k * 256, NS - 1));
    // producers keep two stages in flight (registers preA / preB, used alternately)
    u32x4 preA[FAST ? kWgMaxS : 1], preB[FAST ? kWgMaxS : 1];
    auto prefetch_stage = [&](u32x4 (&pre)[FAST ? kWgMaxS : 1], int j) {
        if constexpr (FAST) {
#pragma unroll
            for (int k = 0; k < kWgMaxS; ++k) pre[k] = fetch(slot[k], j - j0);
        }
    };
    auto commit_stage = [&](const u32x4 (&pre)[FAST ? kWgMaxS : 1], int b, int j) {
#pragma unroll
        for (int k = 0; k < kWgMaxS; ++k) {
            if (rtid + k * 256 < NS) {
                if constexpr (FAST) {
                    commit(slot[k], b, j - j0, pre[k]);
                } else {
                    commit(slot[k], b, j - j0, fetch(slot[k], j - j0));
                }
            }
        }
    };

    // prologue: every thread helps to put x period j0 into buffer 1 (stage index j0 - 1 addresses it);
    // the producers also start on stage j0
    // (all global loads of the prologue are issued before the first one is used)
    {
        constexpr int NP0 = (NX + 511) / 512;
        Slot w0[NP0];
        u32x4 v0[NP0];
#pragma unroll
        for (int k = 0; k < NP0; ++k) {
            w0[k] = make_slot(min(tid + k * 512, NX - 1));
            v0[k] = fetch(w0[k], -1);
        }
        if (!consumer) {
            prefetch_stage(preA, j0);
            prefetch_stage(preB, min(j0 + 1, j1 - 1));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < NP0; ++k)
            if (tid + k * 512 < NX) commit(w0[k], 1, -1, v0[k]);
    }
    __syncthreads();
    bf16x8 ring[kNT];
    f32x4 acc[kNT];
    if (consumer) {
        const u32x4* xp = xbuf[1] + li * kXR + cw + kb;
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
            ring[i] = as_bf16x8(xp[4 * i]);
            acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    } else {
        commit_stage(preA, 0, j0);
        prefetch_stage(preA, min(j0 + 2, j1 - 1));
    }
    __syncthreads();

    if (consumer) {
        // One unit: 13 k-steps (fewer in the last unit of a strip).  The dy operand of a k-step is read two k-steps
        // ahead (three registers in rotation): one step ahead, its latency under load showed at the head of every step.
        auto unit = [&](int b, auto partial, int nsteps) {
            const u32x4* xp = xbuf[b] + li * kXR + cw + kb;
            const u32x4* ap = dybuf[b] + li * kDR + kb;
            bf16x8 av[3];
            av[0] = as_bf16x8(ap[0]);
            av[1] = as_bf16x8(ap[4]);
#pragma unroll
            for (int u = 0; u < kNT; ++u) {
                // (a guard per step, not an early exit: the loop has to unroll completely, the ring is indexed by u)
                if (!decltype(partial)::value || u < nsteps) {
                    // ring slot u is dead once tap slot 0 has consumed it: refill it (and fetch a later dy
                    // operand) right away so the other taps' MFMAs cover the LDS latency
                    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u % 3], ring[u], acc[0], 0, 0, 0);
                    if (u + 2 < kNT) av[(u + 2) % 3] = as_bf16x8(ap[4 * (u + 2)]);
                    ring[u] = as_bf16x8(xp[4 * u]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 1; i < kNT; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[u % 3], ring[(u + i) % kNT], acc[i], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        for (int j = j0; j + 1 < j1; ++j) {
            unit((j - j0) & 1, std::false_type{}, kNT);
            __syncthreads();
        }
        unit((j1 - 1 - j0) & 1, std::true_type{}, last_steps);
        __syncthreads();
    } else {
        // Stage j + 1 sits in preB while an even stage (counted from j0) is consumed and in preA otherwise; its
        // registers then take stage j + 3.  The steady loop has no branch around a load, so the compiler can tell
        // that a set's first use has to wait for that set only, not for the requests made since.
        const int last = j1 - 1;
        int j = j0;
        for (; j + 4 <= last; j += 2) {
            commit_stage(preB, 1, j + 1);
            prefetch_stage(preB, j + 3);
            __syncthreads();
            commit_stage(preA, 0, j + 2);
            prefetch_stage(preA, j + 4);
            __syncthreads();
        }
        for (; j <= last; j += 2) {  // the last stages
            if (j + 1 <= last) {
                commit_stage(preB, 1, j + 1);
                if (j + 3 <= last) prefetch_stage(preB, j + 3);
            }
            __syncthreads();
            if (j + 1 <= last) {
                if (j + 2 <= last) commit_stage(preA, 0, j + 2);
                __syncthreads();
            }
        }
    }
    if (consumer) {
        const int nt = (p.S - cw + 3) / 4;  // real taps of this wave; the remaining slots hold unused sums
        float* ws = static_cast<float*>(p.ws) + static_cast<long>(blockIdx.x) * p.S * 256;
#pragma unroll
        for (int i = 0; i < kNT; ++i) {
            if (i < nt) {
                const int s = cw + 4 * i;
#pragma unroll
                // (non-temporal: the second stage that reads them runs on other compute units, and the lines would
                // only push input rows out of this one's L2; measured 28.5 -> 27.9 us per pass on uncached tensors)
                for (int jj = 0; jj < 4; ++jj) __builtin_nontemporal_store(acc[i][jj], &ws[s * 256 + (4 * kb + jj) * 16 + li]);
            }
        }
    }
}

struct WgradPlan {
    int SPR, KSS, KS, grid, fast;
    bool ok;
};

WgradPlan wgrad_plan(const WgradProblem& p) {
    WgradPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.C > 16 || p.K > 16 || p.d != 8 || p.S > 4 * kNT) return pl;
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    // Strips of KSS k-steps (32 columns) so that one workgroup per CU exists: the columns of a sample are dealt out
    // evenly (60000 columns over 16 strips: 118 k-steps = 9 units and 1 step each, where whole units gave 10 and 5).
    pl.KS = cdiv(p.Q, 32);
    int spr = p.N >= kNumCU ? 1 : kNumCU / p.N;
    if (spr > pl.KS) spr = pl.KS;
    pl.KSS = cdiv(pl.KS, spr);
    pl.SPR = cdiv(pl.KS, pl.KSS);
    const long grid = static_cast<long>(p.N) * pl.SPR;
    if (grid > 0x7fffffffL) return pl;
    pl.grid = static_cast<int>(grid);
    pl.fast = (p.W % 8 == 0) && (p.Q % 8 == 0) && (p.P % 8 == 0) && p.W >= 8 && p.Q >= 8 &&
              (reinterpret_cast<uintptr_t>(p.x) % 16 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 16 == 0);
    pl.ok = true;
    return pl;
}

}  // namespace

bool smallc_bf16_corr_supported(const CorrProblem& p) { return corr_plan(p).ok; }

int smallc_bf16_corr_grid(const CorrProblem& p) {
    const CorrPlan pl = corr_plan(p);
    if (!pl.ok) return 0;
    return pl.ntiles < kNumCU ? pl.ntiles : kNumCU;
}

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

hipError_t smallc_bf16_wgrad_stage1_launch(const WgradProblem& p, hipStream_t st, int* nwg) {
    const WgradPlan pl = wgrad_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    *nwg = pl.grid;
    return launch_kernel(pl.fast ? smallc_wgrad_bf16_d8_kernel<true> : smallc_wgrad_bf16_d8_kernel<false>, dim3(pl.grid),
                         dim3(512), 0, st, p, pl.SPR, pl.KSS, pl.KS);
}

hipError_t smallc_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    int nwg = 0;
    const hipError_t e = smallc_bf16_wgrad_stage1_launch(p, st, &nwg);
    if (e != hipSuccess) return e;
    return smallc_wgrad_reduce_launch(static_cast<const float*>(p.ws), p.dw, p.K, p.C, p.S, p.dw_sk, p.dw_sc, nwg, st);
}

}  // namespace conv1d
