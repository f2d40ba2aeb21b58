// Backward-weight pass (Section 3.3, Algorithm 4) for bfloat16 inputs and dilations 1, 2, 4, 8, 16, any channel
// count: the x operands of neighbouring taps and k-steps are the same registers.
//
//   dw[k][c][s] = sum_n sum_q dy[n][k][q] * x[n][c][q + s*d - P]
//
// One v_mfma_f32_16x16x32_bf16 multiplies A = dy (16 filters x 32 positions) with B = x shifted by one tap
// (32 positions x 16 channels); a lane's 8 k-values are 8 consecutive positions, one 16-byte LDS read.
//
// Operand reuse.  Consumer wave v owns the taps s = s0 + v + 4 i, i < NTW.  In k-step t (32 positions) its tap i
// needs x from element 32 t + 4 i d + E_v on, E_v = (s0 + v) d - P.  With U = min(32, 4 d), a = 32 / U and
// b = 4 d / U that start is U * G + E_v for the operand number G = a t + b i: the wave walks ONE sequence of
// operands, a k-step uses the G in [a t, a t + b (NTW - 1)] and only the a largest of them are new.  The
// operands live in a register ring of R slots, G in slot G % R; per k-step a wave reads a x operands and FB dy
// operands from LDS for FB * NTW MFMAs.
//
// Alignment.  16-byte LDS reads are fast only at 16-byte addresses, so the x rows are staged once per residue
// ("phase") of the operand starts modulo 8 elements: copy phi holds the row shifted left by phi elements.  A
// wave reads one copy (two for d = 1, where consecutive G are 4 elements apart).
//
// Work split.  dw is cut into (filter group of FB blocks of 16) x (channel block of 16) x (tap group of 4 NTW
// taps); the positions of a sample row are cut into units of LU k-steps and strips of consecutive units.  A
// workgroup owns one combination and one strip, keeps all its sums in registers and writes one partial tile
// to the workspace; a second kernel adds the strips in a fixed order (no floating-point atomics).
//
// Workgroup = 8 waves: waves 0-3 are the consumers above (every one of them walks all positions, for its own
// taps), waves 4-7 ("producers") load the next unit from global memory, build the phase copies and write them
// into the other half of the double-buffered LDS.  One workgroup barrier per unit.
#pragma once
#include <type_traits>

#include "conv1d_internal.h"

namespace conv1d {
namespace tz {


typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kMaxY = 8;   // most dy staging slots per producer thread
constexpr int kMaxI = 12;  // most x load items (slot, even phase base) per producer thread

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Compile-time geometry of one (dilation, taps per wave) pair.
template <int D, int NTW>
struct Tz {
    static constexpr int U = D >= 8 ? 32 : 4 * D;      // elements between consecutive operands
    static constexpr int A = 32 / U;                    // new operands per k-step
    static constexpr int B = 4 * D / U;                 // operands between consecutive taps of a wave
    static constexpr int NQ = U == 4 ? 2 : 1;           // phase classes of a wave (parity of G when U = 4)
    static constexpr int NG = D >= 8 ? 1 : (D == 4 ? 2 : 4);  // pairs of phases (2g, 2g + 1) in use, whatever P is
    static constexpr int SPAN = (NTW - 1) * B + 1;      // operands a k-step looks at
    static constexpr int R = (SPAN + A + A - 1) / A * A;  // ring slots: a multiple of A, >= SPAN + A
    // k-steps per unit (one LDS stage) and units per unrolled body: A * LU * NB is a multiple of R, so that the
    // ring slot of every operand is a compile-time constant
    static constexpr int BASE = R / A;                  // k-steps per revolution of the ring
    static constexpr int NB = BASE > 16 ? 2 : 1;
    static constexpr int STEP = BASE / NB;
    static constexpr int LUMAX = D == 1 ? 6 : (D == 2 ? 10 : 16);  // LDS and staging-slot budgets
    static constexpr int LU = LUMAX / STEP * STEP;
    static constexpr int WSP = (7 + 3 * D + 4 * (NQ - 1)) >> 3;  // largest slot offset between the waves' operands
    static constexpr int NXS = 4 * LU + WSP + 4;        // x slots per row and copy in a unit's stage
    static constexpr int HS = U * SPAN / 8;             // slot of operand SPAN (the first refill) ...
    static constexpr int HP = U * (SPAN - 1) / 8;       // ... and of operand SPAN - 1 (the last of the first fill)
    static constexpr int NXP = HP + WSP + 4;            // x slots per row and copy of the first fill
    static_assert((A * LU * NB) % R == 0, "ring slots must repeat from body to body");
    static_assert(R >= SPAN + A, "ring too small");
    static_assert(BASE % NB == 0 && LU >= 1, "units per body");
    static constexpr int hslot(int Gc) { return U * Gc / 8; }
    static constexpr int qcls(int Gc) { return U == 4 ? (Gc & 1) : 0; }
};

struct TzArgs {
    const unsigned short* x;
    const unsigned short* dy;
    float* ws;
    int C, K, W, Q, S, P;
    long x_sn, dy_sn;
    int BPR, BPS, SPR, nstrips;  // bodies per sample row, bodies per strip, strips per row, N * SPR
    int nfg, ncb, ntg;           // filter groups, channel blocks, tap groups
    int RSY, RSX, RSXP;          // LDS row strides in 16-byte slots (odd): dy, x, x of the first fill
    unsigned phase_mask;         // bit phi set: some wave reads the copy of phase phi
    unsigned gmask;              // bit g set: phase 2g or 2g + 1 is in use
    int xcopy_slots;             // 16 * RSX
    int pcopy_slots;             // 16 * RSXP
    int ybuf_slots;              // FB * 16 * RSY
    int stage_slots;             // ybuf_slots + ncopies * xcopy_slots
};

template <int D, int FB, int NTW, bool FAST>
__global__ __launch_bounds__(512, 1) void toeplitz_wgrad_bf16_kernel(TzArgs a) {
    using G = Tz<D, NTW>;
    constexpr int R = G::R, LU = G::LU, NB = G::NB, NQ = G::NQ, SPAN = G::SPAN;
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

    // the combinations of one strip read the same x and dy units: neighbours on one XCD and its L2
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const int strip = lid / ncombos;
    const int combo = lid - strip * ncombos;
    const int tg = combo % a.ntg;
    const int cbi = (combo / a.ntg) % a.ncb;
    const int fg = combo / (a.ntg * a.ncb);
    const int s0 = tg * 4 * NTW, c0 = cbi * 16, k0 = fg * FB * 16;
    const int E0 = s0 * D - a.P;           // operand start of wave 0, class 0, relative to 32 t
    const int fl8p = (E0 >> 3) * 8;        // window origin of the first fill ...
    const int fl8 = fl8p + 8 * G::HS;      // ... and of a unit's stage, relative to the unit's first column
    const int n = strip / a.SPR;
    const int body0 = (strip - n * a.SPR) * a.BPS;
    const int nbodies = min(a.BPS, a.BPR - body0);
    const int nunits = nbodies * NB;
    const int qs = body0 * NB * LU * 32;   // first column of the strip
    const unsigned short* xn = a.x + static_cast<long>(n) * a.x_sn;
    const unsigned short* dyn = a.dy + static_cast<long>(n) * a.dy_sn;
    const unsigned stage_bytes = static_cast<unsigned>(a.stage_slots) * 16u;

    // columns g .. g+7 of a row of `limit` columns that starts `off` elements behind `base`, zero outside the row
    auto load8 = [&](const unsigned short* base, unsigned off, int g, int limit) -> u32x4 {
        unsigned t[8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {  // unconditional loads from clamped columns: all in flight together
            const int gj = g + jj;
            t[jj] = base[off + static_cast<unsigned>(gj < 0 ? 0 : (gj > limit - 1 ? limit - 1 : gj))];
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj)
            if (g + jj < 0 || g + jj >= limit) t[jj] = 0u;
        return u32x4{t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16)};
    };

    // ---- first fill: the operands 0 .. SPAN-1 of the strip's first k-step ------------------------------------
    // Every thread helps: slot (copy, row, i) <-> x[c0 + row][qs + fl8p + phi + 8 i ..], staged in buffer 1.
    auto first_fill = [&]() {
        const int ncopies = __builtin_popcount(a.phase_mask);
        const int total = ncopies * 16 * G::NXP;
        u32x4* pbuf = lds4 + a.stage_slots;
        for (int e = tid; e < total; e += 512) {
            const int ci = e / (16 * G::NXP), r = e - ci * (16 * G::NXP);
            const int row = r / G::NXP, i = r - row * G::NXP;
            unsigned m = a.phase_mask;
            for (int g = ci; g > 0; --g) m &= m - 1;
            const int phi = __builtin_ctz(m);
            const unsigned rowoff = static_cast<unsigned>(min(c0 + row, a.C - 1)) * static_cast<unsigned>(a.W);
            const int c = qs + fl8p + phi + 8 * i;
            u32x4 v;
            if (FAST) {
                const int ce = c & ~1;
                v = fix128(load128_clamped(xn + rowoff, ce, a.W), ce, a.W);
                if (c & 1) v = shift_one(v, load_pair(xn + rowoff, ce + 8, a.W));
            } else {
                v = load8(xn, rowoff, c, a.W);
            }
            pbuf[ci * a.pcopy_slots + row * a.RSXP + i] = v;
        }
    };

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        // Byte offsets into LDS of this lane's operands:
        //   dy operand of filter block fb, k-step tt of a unit:  row 16 fb + li, slot 4 tt + kb
        //   x operand G = a t0 + Gc (t0: first k-step of the body):  copy of phase (E & 7), row li,
        //       slot hslot(Gc) + (E >> 3) + kb - (window origin >> 3),  E = E0 + v d + 4 q,  q = class of Gc
        first_fill();
        unsigned ya[FB], xo[NQ], po[NQ];
        f32x4 acc[FB][NTW];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            ya[fb] = 16u * static_cast<unsigned>((fb * 16 + li) * a.RSY + kb);
#pragma unroll
            for (int i = 0; i < NTW; ++i) acc[fb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int E = E0 + cw * D + 4 * q;
            const int ci = __builtin_popcount(a.phase_mask & ((1u << (E & 7)) - 1u));
            const int dw = (E >> 3) - (E0 >> 3);
            xo[q] = 16u * static_cast<unsigned>(a.ybuf_slots + ci * a.xcopy_slots + li * a.RSX + dw + kb);
            po[q] = stage_bytes + 16u * static_cast<unsigned>(ci * a.pcopy_slots + li * a.RSXP + dw + kb);
        }
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };

        bf16x8 ring[R];
        __syncthreads();  // first fill and unit 0 staged
#pragma unroll
        for (int Gc = 0; Gc < SPAN; ++Gc) ring[Gc % R] = ld(po[G::qcls(Gc)] + 16u * G::hslot(Gc));
        __syncthreads();  // buffer 1 may be overwritten now

        for (int body = 0; body < nbodies; ++body) {
#pragma unroll
            for (int ub = 0; ub < NB; ++ub) {
                bf16x8 acur[FB], anxt[FB];
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) acur[fb] = ld(ya[fb]);
#pragma unroll
                for (int tt = 0; tt < LU; ++tt) {
                    const int tb = ub * LU + tt;  // k-step within the body
                    // The a refills of this k-step (operands first used in the next one) and the dy operands of
                    // the next k-step are requested before the MFMAs of this k-step are issued; the scheduling
                    // barriers keep the compiler from sinking the reads to where their results are needed.
                    if (tt + 1 < LU) {
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb) anxt[fb] = ld(ya[fb] + 64u * static_cast<unsigned>(tt + 1));
                    }
#pragma unroll
                    for (int r = 0; r < G::A; ++r) {
                        const int Gc = G::A * tb + SPAN + r;
                        ring[Gc % R] = ld(xo[G::qcls(Gc)] + 16u * static_cast<unsigned>(G::hslot(Gc) - G::HS - 4 * ub * LU));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < NTW; ++i)
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
                            acc[fb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[fb], ring[(G::A * tb + G::B * i) % R], acc[fb][i], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (tt + 1 < LU) {
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb) acur[fb] = anxt[fb];
                    }
                }
                // hop to the other stage; the x offsets also absorb the 4 LU slots a unit advances inside a body
                const int u = body * NB + ub;
                const unsigned hop = (u & 1) ? 0u - stage_bytes : stage_bytes;
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) ya[fb] += hop;
#pragma unroll
                for (int q = 0; q < NQ; ++q) xo[q] += hop;
                __syncthreads();
            }
        }
        // ---- one contiguous partial tile per workgroup ---------------------------------------------
        //   tile element ((v * FB + fb) * NTW + i) * 256 + 4 * lane + jj  <->  filter k0 + 16 fb + 4 (lane >> 4) + jj,
        //   channel c0 + (lane & 15), tap s0 + v + 4 i
        f32x4* ws = reinterpret_cast<f32x4*>(a.ws + static_cast<long>(lid) * (4 * FB * NTW * 256));
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int i = 0; i < NTW; ++i) ws[((cw * FB + fb) * NTW + i) * 64 + lane] = acc[fb][i];
    } else {
        // ---- producer side -----------------------------------------------------------------------
        // A staging slot is 8 consecutive columns of one row; consecutive threads stage consecutive slots of a
        // row (coalesced loads, conflict-free LDS writes).  dy slot (row, i) <-> dy[k0 + row][q0 + 8i ..].
        // x slot (row, i) of the copy of phase phi <-> x[c0 + row][q0 + fl8 + phi + 8i ..].  16-byte global loads
        // run at full speed from any 4-byte aligned address, so an even phase is simply loaded where it starts;
        // an odd phase phi = e + 1 is made from the load of the even phase e and the dword behind it, shifted
        // by one element.  A load item is (slot, even base e); every thread owns kMaxI of them.
        // Rows beyond C or K re-read the last row: their sums are never stored and no other sum depends on them.
        // FAST (widths, sample strides and pointers multiples of 2 elements): units are fetched one or two units
        // ahead with 16-byte loads from addresses clamped into the rows; a unit whose window leaves the rows (not
        // "interior") is put right when it is written to LDS.  Otherwise every unit is loaded element by element,
        // zero outside the row, when it is written to LDS.
        constexpr int SY = 4 * LU;
        constexpr int NY = FB * 16 * SY, NXT = 16 * G::NXS;
        constexpr int ng = G::NG;
        constexpr int kMaxY = (NY + 255) >> 8;            // dy staging slots per producer thread
        constexpr int kMaxI = ((NXT + 255) >> 8) * ng;    // x load items (slot, even phase base) per producer thread
        int ylds[kMaxY], xlds[kMaxI];         // row * stride + slot
        int ycol[kMaxY], xcol[kMaxI];         // first column relative to the unit / window origin
        unsigned yrow[kMaxY], xrow[kMaxI];    // element offset of the (clamped) row from the sample's base
#pragma unroll
        for (int k = 0; k < kMaxY; ++k) {
            const int e = min(rtid + k * 256, NY - 1);
            const int row = e / SY, i = e - row * SY;
            yrow[k] = static_cast<unsigned>(min(k0 + row, a.K - 1)) * static_cast<unsigned>(a.Q);
            ycol[k] = 8 * i;
            ylds[k] = row * a.RSY + i;
        }
        // item it = (slot task it / ng, even base = 2 * (it % ng)-th set bit of gmask); all of that is uniform
        auto item_base = [&](int it) {
            unsigned m = a.gmask;
            for (int g = it % ng; g > 0; --g) m &= m - 1;
            return 2 * __builtin_ctz(m);
        };
#pragma unroll
        for (int it = 0; it < kMaxI; ++it) {
            const int e = min(rtid + (it / ng) * 256, NXT - 1);
            const int row = e / G::NXS, i = e - row * G::NXS;
            xrow[it] = static_cast<unsigned>(min(c0 + row, a.C - 1)) * static_cast<unsigned>(a.W);
            xcol[it] = 8 * i + item_base(it);
            xlds[it] = row * a.RSX + i;
        }
        struct Stage {
            u32x4 y[kMaxY];
            u32x4 x[kMaxI];
            unsigned xd[kMaxI];  // the dword behind x[it] (odd phases)
        };
        auto interior = [&](int q0) {
            const int x0 = q0 + fl8;
            return FAST && q0 + 32 * LU <= a.Q && x0 >= 0 && x0 + 8 * G::NXS + 16 <= a.W;
        };
        auto has_odd = [&](int it) { return (a.phase_mask >> (item_base(it) + 1)) & 1u; };
        // FAST: every unit is fetched one unit ahead with 16-byte loads; where the window leaves the rows the
        // loads are clamped into them and the slots are put right when they are written to LDS.
        // Whether the dwords behind the slots are loaded at all (some phase in use is odd) is a compile-time
        // choice of the caller, so no branch surrounds a load: the compiler can then count the loads that may
        // still be in flight when a register set is used instead of waiting for all of them.
        auto prefetch = [&](auto odd_, Stage& st, int u) {
            constexpr bool ODD = decltype(odd_)::value;
            if (!FAST) return;
            const int q0 = qs + u * 32 * LU;
            // (one path for interior and edge units: clamping on the vector ALU measured as fast as a second path
            // with scalar bases)
#pragma unroll
            for (int k = 0; k < kMaxY; ++k) st.y[k] = load128_clamped(dyn + yrow[k], q0 + ycol[k], a.Q);
#pragma unroll
            for (int it = 0; it < kMaxI; ++it) {
                const int c = q0 + fl8 + xcol[it];
                st.x[it] = load128_clamped(xn + xrow[it], c, a.W);
                // clamped like the slot itself; put right (zero outside the row) when it is written to LDS
                if (ODD) st.xd[it] = *reinterpret_cast<const unsigned*>(xn + xrow[it] + clampi(c + 8, 0, a.W - 2));
            }
        };
        auto commit = [&](Stage& st, int u) {
            const int q0 = qs + u * 32 * LU;
            if (FAST) {
                if (!interior(q0)) {
#pragma unroll
                    for (int k = 0; k < kMaxY; ++k)
                        if (k * 256 < NY) st.y[k] = fix128(st.y[k], q0 + ycol[k], a.Q);
#pragma unroll
                    for (int it = 0; it < kMaxI; ++it) {
                        const int c = q0 + fl8 + xcol[it];
                        st.x[it] = fix128(st.x[it], c, a.W);
                        if (has_odd(it)) st.xd[it] = (c + 8 >= 0 && c + 8 < a.W) ? st.xd[it] : 0u;
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < kMaxY; ++k)
                    if (k * 256 < NY) st.y[k] = load8(dyn, yrow[k], q0 + ycol[k], a.Q);
#pragma unroll
                for (int it = 0; it < kMaxI; ++it) {
                        const int c = q0 + fl8 + xcol[it];
                        st.x[it] = load8(xn, xrow[it], c, a.W);
                        const int c8 = c + 8;
                        const unsigned xd = xn[xrow[it] + static_cast<unsigned>(c8 < 0 ? 0 : (c8 > a.W - 1 ? a.W - 1 : c8))];
                        st.xd[it] = (c8 >= 0 && c8 < a.W) ? xd : 0u;
                    }
            }
            u32x4* ybuf = lds4 + (u & 1) * a.stage_slots;
            u32x4* xbuf = ybuf + a.ybuf_slots;
#pragma unroll
            for (int k = 0; k < kMaxY; ++k)
                if (rtid + k * 256 < NY) ybuf[ylds[k]] = st.y[k];
#pragma unroll
            for (int it = 0; it < kMaxI; ++it)
                if (rtid + (it / ng) * 256 < NXT) {
                    const int e = item_base(it);
                    const unsigned below = a.phase_mask & ((1u << e) - 1u);
                    u32x4* dst = xbuf + __builtin_popcount(below) * a.xcopy_slots + xlds[it];
                    const u32x4 v = st.x[it];
                    if ((a.phase_mask >> e) & 1u) {
                        *dst = v;
                        dst += a.xcopy_slots;
                    }
                    if ((a.phase_mask >> (e + 1)) & 1u) *dst = shift_one(v, st.xd[it]);
                }
        };
        // Two register sets where they fit: the loads of a unit are then issued two units before it is written
        // to LDS (the memory latency under load exceeds the MFMA time of one unit).  Set A holds the even units,
        // set B the odd ones.
        constexpr bool kTwoSets = FAST && !(FB == 2 && (D == 2 || D == 4));
        auto run = [&](auto odd_) {
            const int last = nunits - 1;
            Stage sa;
            // (with the dwords behind the slots, two sets of the d = 2 and d = 4 kernels no longer fit in registers)
            if constexpr (kTwoSets && !(decltype(odd_)::value && (D == 2 || D == 4))) {
                Stage sb;
                prefetch(odd_, sa, 0);
                prefetch(odd_, sb, min(1, last));
                first_fill();  // while the units' loads are on their way
                commit(sa, 0);
                prefetch(odd_, sa, min(2, last));
                __syncthreads();
                __syncthreads();
                int u = 0;
                for (; u + 4 <= last; u += 2) {  // the steady state: no branch around a load
                    commit(sb, u + 1);
                    prefetch(odd_, sb, u + 3);
                    __syncthreads();
                    commit(sa, u + 2);
                    prefetch(odd_, sa, u + 4);
                    __syncthreads();
                }
                for (; u <= last; u += 2) {  // the last units
                    if (u + 1 <= last) {
                        commit(sb, u + 1);
                        if (u + 3 <= last) prefetch(odd_, sb, u + 3);
                    }
                    __syncthreads();
                    if (u + 1 <= last) {
                        if (u + 2 <= last) commit(sa, u + 2);
                        __syncthreads();
                    }
                }
            } else {
                prefetch(odd_, sa, 0);
                first_fill();
                commit(sa, 0);
                if (nunits > 1) prefetch(odd_, sa, 1);
                __syncthreads();
                __syncthreads();
                for (int u = 0; u < nunits; ++u) {
                    if (u + 1 < nunits) {
                        commit(sa, u + 1);
                        if (u + 2 < nunits) prefetch(odd_, sa, u + 2);
                    }
                    __syncthreads();
                }
            }
        };
        if (a.phase_mask & 0xaau) run(std::true_type{});
        else run(std::false_type{});
    }
}


struct TzPlan {
    bool ok;
    int D, FB, NTW, fast, grid, tile;
    size_t lds_bytes;
    TzArgs a;
};

constexpr int kNTWs[] = {13, 9, 5, 3, 2};  // taps per consumer wave (a tap group has 4 times as many)

template <int D, int FB, int NTW>
hipError_t launch(const TzPlan& pl, hipStream_t st) {
    auto kern = pl.fast ? toeplitz_wgrad_bf16_kernel<D, FB, NTW, true> : toeplitz_wgrad_bf16_kernel<D, FB, NTW, false>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

// every (filter blocks, taps per wave) shape of one dilation; one translation unit per dilation
template <int D>
hipError_t launch_dilation(const TzPlan& pl, hipStream_t st) {
    switch (pl.FB * 100 + pl.NTW) {
        case 113: return launch<D, 1, 13>(pl, st);
        case 213: return launch<D, 2, 13>(pl, st);
        case 109: return launch<D, 1, 9>(pl, st);
        case 209: return launch<D, 2, 9>(pl, st);
        case 105: return launch<D, 1, 5>(pl, st);
        case 205: return launch<D, 2, 5>(pl, st);
        case 103: return launch<D, 1, 3>(pl, st);
        case 203: return launch<D, 2, 3>(pl, st);
        case 102: return launch<D, 1, 2>(pl, st);
        case 202: return launch<D, 2, 2>(pl, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_d1(const TzPlan& pl, hipStream_t st);
hipError_t launch_d2(const TzPlan& pl, hipStream_t st);
hipError_t launch_d4(const TzPlan& pl, hipStream_t st);
hipError_t launch_d8(const TzPlan& pl, hipStream_t st);
hipError_t launch_d16(const TzPlan& pl, hipStream_t st);

}  // namespace tz
}  // namespace conv1d
