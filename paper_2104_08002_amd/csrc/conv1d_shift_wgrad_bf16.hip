// Backward-weight pass (Section 3.3, Algorithm 4) for bfloat16 inputs, few taps and small dilations
// (d = 1 with (S - 1) d <= 16, d = 2, 4 with (S - 1) d <= 32): the tap shift is applied in registers.
//
//   dw[k][c][s] = sum_n sum_q dy[n][k][q] * x[n][c][q + s*d - P]
//
// One v_mfma_f32_16x16x32_bf16 multiplies A = dy (16 filters x 32 positions) with B = x shifted by one tap
// (32 positions x 16 channels); a lane's 8 k-values are 8 consecutive positions.  A 16-byte LDS read is fast only
// from a 16-byte address, and the other backward-weight kernels therefore stage one copy of the x rows per
// residue of the operand starts modulo 8 elements: with dilation 1 that is up to 8 copies for a handful of taps.
// Here x is staged once, in slots of 8 positions that start at multiples of 8, and the dy rows are staged P mod 8
// elements off that grid.  The x operand of tap s then starts exactly s*d elements into the slots a lane has read
// (two or three of them): a compile-time shift, made of register renaming and, for odd shifts, four
// v_alignbit_b32 per operand.  A wave reads 2 - 3 x slots and FB dy slots from LDS per k-step for SMAX * FB MFMAs.
//
// Work split.  A workgroup owns 64 channels (consumer wave v: channels 16 v .. 16 v + 15), FB blocks of 16
// filters, all taps, and a strip of the positions (units of 8 (or 4) k-steps of 32 positions); it keeps all its sums
// in registers and writes one partial tile to the workspace; a second kernel adds the strips in a fixed order
// (no floating-point atomics).  Workgroup = 8 waves: waves 0-3 consume, waves 4-7 ("producers") load the next
// unit from global memory and write it into the other half of the double-buffered LDS.  One workgroup barrier
// per unit.
#include <type_traits>

#include "conv1d_internal.h"

namespace conv1d {

namespace sw {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
// k-steps per unit: 8, or 4 with four filter blocks (the producers' two register sets hold one slot per task: 9 x and 8
// dy tasks per thread at 8 k-steps no longer fit, 5 + 4 at 4 k-steps do, and the unit is as long in MFMAs either way)
constexpr int lu_of(int FB) { return FB == 4 ? 4 : 8; }
constexpr int kBufferRsrcFlags = 0x00020000;  // fourth dword of a raw buffer descriptor (32-bit data format, no swizzle)

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct SwArgs {
    const unsigned short* x;
    const unsigned short* dy;
    float* ws;
    int C, K, W, Q, S, P;
    long x_sn, dy_sn;
    int nfg, ncg;      // filter groups of FB * 16, channel groups of 64
    int UPR;           // units per sample row
    int KSR;           // k-steps per sample row
    int nunits;        // N * UPR
    int nstrips;       // strips of consecutive units per (filter group, channel group)
    int u_base, u_rem; // units per strip, and one more for the first u_rem strips
    int RSX, RSY;      // LDS row strides in 16-byte slots (odd)
    int ybuf_slots;    // FB * 16 * RSY
    int stage_slots;   // ybuf_slots + 64 * RSX
    int fast;          // rows start at 4-byte addresses, have even lengths and at least 8 columns: 16-byte loads from even columns
    FastDiv dv_upr;
};

// Compile-time geometry: dilation D, taps computed SMAX (taps s >= S are computed and dropped), filter blocks FB.
template <int D, int SMAX, int FB>
struct Sw {
    static constexpr int LU = lu_of(FB);
    static constexpr int NSL = 1 + ((SMAX - 1) * D + 7) / 8;  // x slots a lane reads per k-step
    static constexpr int NXS = 4 * LU + NSL - 1;              // x slots per row of a unit
    static constexpr int NYS = 4 * LU;                        // dy slots per row of a unit
};

// the 8 elements of columns c .. c + 7 of a row of `limit` columns, zero outside the row: element by element, for
// rows that are not 4-byte aligned, have odd lengths or fewer than 8 columns
__device__ __forceinline__ u32x4 load_slot(const unsigned short* row, int c, int limit) {
    unsigned e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = (c + i >= 0 && c + i < limit) ? row[c + i] : 0u;
    return u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
}

template <int D, int SMAX, int FB>
__global__ __launch_bounds__(512, 1) void shift_wgrad_bf16_kernel(SwArgs a) {
    using G = Sw<D, SMAX, FB>;
    constexpr int NSL = G::NSL, NXS = G::NXS, NYS = G::NYS, LU = G::LU;
    constexpr int NXT = 64 * NXS, NYT = FB * 16 * NYS;  // staging tasks (16-byte slots) per unit
    constexpr int NT = (NXT + NYT + 255) / 256;          // per producer thread (one more when neither count is a multiple of 256)
    extern __shared__ u32x4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int v = wave & 3;
    const int rtid = tid & 255;
    const int li = lane & 15;
    const int kb = lane >> 4;

    // workgroup -> (strip, filter group, channel group).  The combinations of one strip read the same x and dy
    // columns: their logical indices are consecutive, which puts them on one XCD and its L2 (the loop runs at the
    // rate memory delivers the units, so every byte fetched twice from HBM is time).
    const int ncombos = a.nfg * a.ncg;
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int strip = lid / ncombos;
    const int combo = lid - strip * ncombos;
    const int fg = combo / a.ncg, cg = combo - fg * a.ncg;
    const int u_begin = strip * a.u_base + min(strip, a.u_rem);
    const int u_end = u_begin + a.u_base + (strip < a.u_rem ? 1 : 0);
    const int P8 = a.P >> 3, Pr = a.P & 7;

    // unit u: sample n, k-steps t0 .. t0 + ks - 1 of its row.  dy slot j of the row holds q = Pr - 8 + 8 j .. + 7,
    // x slot j the positions 8 j .. 8 j + 7; the k-step t reads dy slots 4 t .. 4 t + 3 and, for the tap shift
    // s d = 8 w + r, the x slots 4 t - 1 - P8 + w (+ 1).
    struct Unit {
        int n, t0, ks;
    };
    auto unit = [&](int u) -> Unit {
        Unit un;
        un.n = fast_div(u, a.dv_upr);
        un.t0 = (u - un.n * a.UPR) * LU;
        un.ks = min(LU, a.KSR - un.t0);
        return un;
    };

    if (consumer) {
        f32x4 acc[SMAX][FB];
#pragma unroll
        for (int s = 0; s < SMAX; ++s)
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) acc[s][fb] = f32x4{0.f, 0.f, 0.f, 0.f};
        const unsigned xlane = 16u * static_cast<unsigned>(a.ybuf_slots + (16 * v + li) * a.RSX + kb);
        const unsigned ylane = 16u * static_cast<unsigned>(li * a.RSY + kb);
        const unsigned yrow = 16u * static_cast<unsigned>(16 * a.RSY);
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return *reinterpret_cast<const u32x4*>(ldsb + off); };
        __syncthreads();  // unit u_begin is in LDS
        for (int u = u_begin; u < u_end; ++u) {
            const Unit un = unit(u);
            const unsigned sb = 16u * static_cast<unsigned>(((u - u_begin) & 1) * a.stage_slots);
            u32x4 X[2][NSL], Y[2][FB];
#pragma unroll
            for (int w = 0; w < NSL; ++w) X[0][w] = ld(sb + xlane + 16u * w);
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) Y[0][fb] = ld(sb + ylane + fb * yrow);
            // two k-steps per iteration, so that the register set of a k-step is a compile-time index
            for (int t = 0; t < un.ks; t += 2) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (t + h < un.ks) {
                        // the reads of the next k-step (of this unit; the last one reads slots nobody uses)
                        const unsigned nx = sb + 64u * static_cast<unsigned>(t + h + 1);
#pragma unroll
                        for (int w = 0; w < NSL; ++w) X[h ^ 1][w] = ld(nx + xlane + 16u * w);
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb) Y[h ^ 1][fb] = ld(nx + ylane + fb * yrow);
                        unsigned in[4 * NSL];
#pragma unroll
                        for (int w = 0; w < NSL; ++w)
#pragma unroll
                            for (int i = 0; i < 4; ++i) in[4 * w + i] = X[h][w][i];
#pragma unroll
                        for (int s = 0; s < SMAX; ++s) {
                            const int sh = s * D, m = sh >> 1;  // dwords, and one more element if sh is odd
                            u32x4 b;
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                b[i] = (sh & 1) ? __builtin_amdgcn_alignbit(in[m + i + 1], in[m + i], 16) : in[m + i];
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb)
                                acc[s][fb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(Y[h][fb]), as_bf16x8(b), acc[s][fb], 0, 0, 0);
                        }
                    }
                }
            }
            __syncthreads();
        }
        // the partial tile: element (((v FB + fb) SMAX + s) 64 + lane) 4 + r = filter 4 kb + r of block fb, channel li of
        // wave v, tap s
        float* tile = a.ws + (static_cast<long>(strip) * ncombos + combo) * (4L * FB * SMAX * 256);
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int s = 0; s < SMAX; ++s)
                *reinterpret_cast<f32x4*>(tile + (((v * FB + fb) * SMAX + s) * 64 + lane) * 4) = acc[s][fb];
    } else {
        // ---- producers: a thread's first NTX tasks are x slots (task e = rtid + 256 i: slot e % NXS of row e / NXS of
        // the channel group), the other NTY are dy slots; which is which is the same for every lane ----
        constexpr int NTX = (NXT + 255) / 256, NTY = (NYT + 255) / 256;
        static_assert(NTX + NTY == NT || NTX + NTY == NT + 1, "task split");
        constexpr int NTT = NTX + NTY;
        int t_rs[NTT], t_lds[NTT];  // 256 row + slot; LDS slot within a stage
        unsigned t_vo[NTT];         // byte offset of (row, clamped to the last real one; column 8 slot) in the sample's block
        bool t_row_ok[NTT];
#pragma unroll
        for (int i = 0; i < NTT; ++i) {
            const bool is_x = i < NTX;
            const int e = is_x ? min(rtid + 256 * i, NXT - 1) : min(rtid + 256 * (i - NTX), NYT - 1);
            const int per = is_x ? NXS : NYS;
            const int r = e / per, sl = e - r * per;
            t_rs[i] = 256 * r + sl;
            t_lds[i] = is_x ? a.ybuf_slots + r * a.RSX + sl : r * a.RSY + sl;
            const int row = is_x ? cg * 64 + r : fg * FB * 16 + r;
            const int nrows = is_x ? a.C : a.K, len = is_x ? a.W : a.Q;
            t_row_ok[i] = row < nrows;
            t_vo[i] = static_cast<unsigned>(min(row, nrows - 1) * len + 8 * sl) * 2u;
        }
        auto task_valid = [&](int i) { return i < NTX ? rtid + 256 * i < NXT : rtid + 256 * (i - NTX) < NYT; };
        // Two register sets: the loads of unit u + 2 are requested before unit u + 1 is written to LDS (a unit is
        // consumed faster than memory answers).  Set u & 1 (counted from the strip's first unit) holds unit u.
        // Every load is unconditional (a branch around a load would make the compiler wait for each load where the
        // paths join).  Units that lie inside their rows - all but the first and last of a row - take buffer
        // loads whose address is the thread's constant offset plus a scalar offset per unit, and are written to
        // LDS as they are; for the others the column is clamped into the row, and what lies outside is shifted out
        // and zeroed when the registers are written to LDS.  dy slots that start at an odd column (odd padding) are
        // the 16 bytes from the even column before plus one more element pair.
        struct Regs {
            u32x4 v[NTT];
            unsigned nxt[NTY];
        };
        Regs reg[2];
        const int podd = Pr & 1;
        const bool all_rows = cg * 64 + 64 <= a.C && (fg + 1) * FB * 16 <= a.K;
        struct Cols {
            int cx, cy;  // first column of the unit's x slots, and of its dy slots (even: one less if Pr is odd)
            bool lean;
        };
        auto cols = [&](const Unit& un) -> Cols {
            Cols c;
            c.cx = 8 * (4 * un.t0 - 1 - P8);
            c.cy = Pr - 8 + 32 * un.t0 - podd;
            c.lean = a.fast && c.cx >= 0 && c.cx + 8 * NXS <= a.W && c.cy >= 0 && c.cy + 8 * NYS + 2 <= a.Q;
            return c;
        };
        auto fetch = [&](int u, Regs& rg) {
            const Unit un = unit(u);
            const Cols c = cols(un);
            const unsigned short* xb = a.x + static_cast<long>(un.n) * a.x_sn;
            const unsigned short* yb = a.dy + static_cast<long>(un.n) * a.dy_sn;
            if (c.lean) {
                // (the range check of the descriptors is not relied upon: every address is inside the sample's block)
                const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(xb), 0, 2 * a.C * a.W, kBufferRsrcFlags);
                const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned short*>(yb), 0, 2 * a.K * a.Q, kBufferRsrcFlags);
#pragma unroll
                for (int i = 0; i < NTT; ++i) {
                    if (i < NTX) {
                        rg.v[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rx, static_cast<int>(t_vo[i]), 2 * c.cx, 0));
                    } else {
                        rg.v[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ry, static_cast<int>(t_vo[i]), 2 * c.cy, 0));
                        if (podd) rg.nxt[i - NTX] = __builtin_amdgcn_raw_buffer_load_b32(ry, static_cast<int>(t_vo[i]), 2 * c.cy + 16, 0);
                    }
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < NTT; ++i) {
                const bool is_x = i < NTX;
                const int sl = t_rs[i] & 255;
                const unsigned short* row = (is_x ? xb : yb) + ((t_vo[i] >> 1) - 8 * sl);
                const int limit = is_x ? a.W : a.Q;
                const int col = (is_x ? c.cx : c.cy) + 8 * sl;  // even
                if (a.fast) {
                    rg.v[i] = load128_clamped(row, col, limit);
                    if (!is_x) rg.nxt[is_x ? 0 : i - NTX] = podd ? load_pair(row, col + 8, limit) : 0u;
                } else {
                    rg.v[i] = load_slot(row, is_x ? col : col + podd, limit);  // element by element
                }
            }
        };
        auto commit = [&](int u, int b, const Regs& rg) {
            const Unit un = unit(u);
            const Cols c = cols(un);
            u32x4* st = lds4 + b * a.stage_slots;
#pragma unroll
            for (int i = 0; i < NTT; ++i)
                if (task_valid(i)) {
                    const bool is_x = i < NTX;
                    u32x4 v = rg.v[i];
                    if (a.fast) {
                        if (!c.lean) v = fix128(v, (is_x ? c.cx : c.cy) + 8 * (t_rs[i] & 255), is_x ? a.W : a.Q);
                        if (!is_x && podd) v = shift_one(v, rg.nxt[is_x ? 0 : i - NTX]);
                    }
                    if (!all_rows) v = t_row_ok[i] ? v : u32x4{0u, 0u, 0u, 0u};
                    st[t_lds[i]] = v;
                }
        };
        const int nu = u_end - u_begin;
        fetch(u_begin, reg[0]);
        if (nu > 1) fetch(u_begin + 1, reg[1]);
        commit(u_begin, 0, reg[0]);
        __syncthreads();
        for (int j = 0; j < nu; j += 2) {  // units u_begin + j and u_begin + j + 1
            if (j + 2 < nu) fetch(u_begin + j + 2, reg[0]);
            if (j + 1 < nu) commit(u_begin + j + 1, 1, reg[1]);
            __syncthreads();
            if (j + 1 < nu) {
                if (j + 3 < nu) fetch(u_begin + j + 3, reg[1]);
                if (j + 2 < nu) commit(u_begin + j + 2, 0, reg[0]);
                __syncthreads();
            }
        }
    }
}

// Fixed-order sum of the strips' partial tiles into dw.  Thread (g = tid >> 4, el = tid & 15) of a block adds the
// tiles of the strips g, g + 16, ... for the 4 elements 4 el .. + 3 of the block's 64; group 0 then adds the 16
// partial sums left to right.
__global__ __launch_bounds__(256) void shift_wgrad_reduce_kernel(const float* ws, float* dw, SwArgs a, int FB, int SMAX) {
    __shared__ f32x4 part[16][17];
    const int el = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int tile = 4 * FB * SMAX * 256;
    const int ncombos = a.nfg * a.ncg;
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
        const int fg = combo / a.ncg, cg = combo - fg * a.ncg;
        const int l = (e >> 2) & 63, blk = e >> 8;  // lane, (v FB + fb) SMAX + s
        const int s = blk % SMAX, fb = (blk / SMAX) % FB, v = blk / (SMAX * FB);
        const int k0 = (fg * FB + fb) * 16 + 4 * (l >> 4), c = cg * 64 + v * 16 + (l & 15);
        if (c < a.C && s < a.S) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (k0 + jj < a.K) dw[(static_cast<long>(k0 + jj) * a.C + c) * a.S + s] = t[jj];
        }
    }
}

struct SwPlan {
    bool ok;
    int D, SMAX, FB, grid;
    long tile;
    size_t lds_bytes;
    SwArgs a;
};

template <int D, int SMAX, int FB>
hipError_t sw_launch(const SwPlan& pl, hipStream_t st) {
    auto kern = shift_wgrad_bf16_kernel<D, SMAX, FB>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

template <int D, int SMAX>
hipError_t sw_launch_fb(const SwPlan& pl, hipStream_t st) {
    switch (pl.FB) {
        case 4:
            if constexpr (SMAX <= 9) return sw_launch<D, SMAX, 4>(pl, st);
            return hipErrorInvalidValue;
        case 2: return sw_launch<D, SMAX, 2>(pl, st);
        case 1: return sw_launch<D, SMAX, 1>(pl, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sw

namespace {

using sw::SwArgs;
using sw::SwPlan;

template <int D, int SMAX, int FB>
void sw_geometry_fb(SwPlan& pl) {
    using G = sw::Sw<D, SMAX, FB>;
    SwArgs& a = pl.a;
    a.RSX = G::NXS | 1;
    a.RSY = G::NYS | 1;
    a.ybuf_slots = pl.FB * 16 * a.RSY;
    a.stage_slots = a.ybuf_slots + 64 * a.RSX;
    // + slack for the reads that run one k-step ahead of the last one
    pl.lds_bytes = static_cast<size_t>(2 * a.stage_slots + 8) * 16;
}

template <int D, int SMAX>
void sw_geometry(SwPlan& pl) {
    switch (pl.FB) {
        case 4: sw_geometry_fb<D, SMAX, 4>(pl); break;
        case 2: sw_geometry_fb<D, SMAX, 2>(pl); break;
        default: sw_geometry_fb<D, SMAX, 1>(pl); break;
    }
}

SwPlan sw_plan(const WgradProblem& p) {
    SwPlan pl{};
    pl.ok = false;
    if (!p.bf16) return pl;
    if (p.d != 1 && p.d != 2 && p.d != 4) return pl;
    const int max_shift = p.d >= 2 ? 32 : 16;  // 3 x slots per lane and k-step; 5 at even dilations (shifts of whole dwords)
    if (static_cast<long>(p.S - 1) * p.d > max_shift || p.S < 2) return pl;
    if (p.dw_sc != p.S || p.dw_sk != static_cast<long>(p.C) * p.S) return pl;  // writes the whole dw tensor
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    if (static_cast<long>(p.K) * p.C * p.S >= (1L << 31)) return pl;
    if (p.P < 0 || p.W < 1 || p.Q < 1) return pl;
    const int SMAX = p.S <= 5 ? 5 : (p.S <= 9 ? 9 : 17);
    if (static_cast<long>(SMAX - 1) * p.d > max_shift) return pl;
    SwArgs& a = pl.a;
    a.x = static_cast<const unsigned short*>(p.x);
    a.dy = static_cast<const unsigned short*>(p.dy);
    a.ws = static_cast<float*>(p.ws);
    a.C = p.C; a.K = p.K; a.W = p.W; a.Q = p.Q; a.S = p.S; a.P = p.P;
    a.x_sn = p.x_sn; a.dy_sn = p.dy_sn;
    a.fast = (p.W >= 8) && (p.Q >= 8) && (p.W % 2 == 0) && (p.Q % 2 == 0) && (p.x_sn % 2 == 0) && (p.dy_sn % 2 == 0) &&
             (reinterpret_cast<uintptr_t>(p.x) % 4 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 4 == 0);
    a.ncg = cdiv(p.C, 64);
    // dy slots of a row: q = Pr - 8 + 8 j covers 0 .. Q - 1 for j < NJ
    const int Pr = p.P & 7;
    const int NJ = cdiv(p.Q - Pr + 8, 8);
    a.KSR = cdiv(NJ, 4);
    // filter blocks per workgroup: as many as the accumulators allow (every x slot staged then feeds more MFMAs),
    // fewer when that leaves compute units idle (a strip should still have some 32 k-steps: every workgroup pays a
    // start-up and writes a partial tile)
    const int fbmax = SMAX <= 9 ? 4 : 2;
    int FB = 1;
    while (FB * 2 <= fbmax && FB * 16 < p.K) FB *= 2;
    const long row_units8 = cdiv(a.KSR, 8);
    while (FB > 1 && static_cast<long>(cdiv(cdiv(p.K, 16), FB)) * a.ncg * cdiv(p.N * row_units8, 4) < sw::kNumCU) FB /= 2;
    pl.FB = FB;
    a.UPR = cdiv(a.KSR, sw::lu_of(FB));
    const long nunits = static_cast<long>(p.N) * a.UPR;
    if (nunits >= (1L << 30)) return pl;
    a.nunits = static_cast<int>(nunits);
    if (!make_fastdiv(a.dv_upr, a.UPR, nunits)) return pl;
    pl.D = p.d;
    pl.SMAX = SMAX;
    a.nfg = cdiv(cdiv(p.K, 16), FB);
    const int ncombos = a.nfg * a.ncg;
    long nstrips = sw::kNumCU / ncombos;
    if (nstrips < 1) nstrips = 1;
    if (nstrips > nunits) nstrips = nunits;
    a.nstrips = static_cast<int>(nstrips);
    a.u_base = static_cast<int>(nunits / nstrips);
    a.u_rem = static_cast<int>(nunits % nstrips);
    const long grid = nstrips * ncombos;
    if (grid > 0x7fffffffL) return pl;
    pl.grid = static_cast<int>(grid);
    pl.tile = 4L * FB * SMAX * 256;
    switch (p.d * 100 + SMAX) {
        case 105: sw_geometry<1, 5>(pl); break;
        case 109: sw_geometry<1, 9>(pl); break;
        case 117: sw_geometry<1, 17>(pl); break;
        case 205: sw_geometry<2, 5>(pl); break;
        case 209: sw_geometry<2, 9>(pl); break;
        case 217: sw_geometry<2, 17>(pl); break;
        case 405: sw_geometry<4, 5>(pl); break;
        case 409: sw_geometry<4, 9>(pl); break;
        default: return pl;
    }
    if (pl.lds_bytes > static_cast<size_t>(sw::kLdsBudget)) return pl;
    pl.ok = true;
    return pl;
}

}  // namespace

bool shift_bf16_wgrad_supported(const WgradProblem& p) { return sw_plan(p).ok; }

size_t shift_bf16_wgrad_workspace(const WgradProblem& p) {
    const SwPlan pl = sw_plan(p);
    return pl.ok ? static_cast<size_t>(pl.grid) * pl.tile * sizeof(float) : 0;
}

hipError_t shift_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const SwPlan pl = sw_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e;
    switch (pl.D * 100 + pl.SMAX) {
        case 105: e = sw::sw_launch_fb<1, 5>(pl, st); break;
        case 109: e = sw::sw_launch_fb<1, 9>(pl, st); break;
        case 117: e = sw::sw_launch_fb<1, 17>(pl, st); break;
        case 205: e = sw::sw_launch_fb<2, 5>(pl, st); break;
        case 209: e = sw::sw_launch_fb<2, 9>(pl, st); break;
        case 217: e = sw::sw_launch_fb<2, 17>(pl, st); break;
        case 405: e = sw::sw_launch_fb<4, 5>(pl, st); break;
        case 409: e = sw::sw_launch_fb<4, 9>(pl, st); break;
        default: e = hipErrorInvalidValue; break;
    }
    if (e != hipSuccess) return e;
    const long nel = static_cast<long>(pl.a.nfg) * pl.a.ncg * pl.tile;
    return launch_kernel(sw::shift_wgrad_reduce_kernel, dim3(cdiv(nel, 64)), dim3(256), 0, st, static_cast<const float*>(p.ws), p.dw, pl.a,
                         pl.FB, pl.SMAX);
}

}  // namespace conv1d
