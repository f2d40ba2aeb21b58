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
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kMaxY = 8;   // dy staging slots per producer thread
constexpr int kMaxI = 12;  // x load items (slot, even phase base) per producer thread

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// v holds the 8 elements of a row of `limit` >= 8 columns from column clamp(c, 0, limit - 8) on; returns the
// elements of columns c .. c+7, zero outside the row.
__device__ __forceinline__ u32x4 fix128(u32x4 v, int c, int limit) {
    const int sh = c - clampi(c, 0, limit - 8);
    if (sh == 0) return v;
    if (sh >= 8 || sh <= -8) return u32x4{0u, 0u, 0u, 0u};
    unsigned long lo = v.x | (static_cast<unsigned long>(v.y) << 32), hi = v.z | (static_cast<unsigned long>(v.w) << 32);
    if (sh > 0) {  // the row ends inside the slot: drop the low elements, zeros come in at the top
        const int s = 16 * sh;
        if (s < 64) {
            lo = (lo >> s) | (hi << (64 - s));
            hi >>= s;
        } else {
            lo = hi >> (s - 64);
            hi = 0;
        }
    } else {  // the row starts inside the slot
        const int s = -16 * sh;
        if (s < 64) {
            hi = (hi << s) | (lo >> (64 - s));
            lo <<= s;
        } else {
            hi = lo << (s - 64);
            lo = 0;
        }
    }
    return u32x4{static_cast<unsigned>(lo), static_cast<unsigned>(lo >> 32), static_cast<unsigned>(hi), static_cast<unsigned>(hi >> 32)};
}

// 16-byte load of the columns clamp(c, 0, limit - 8) .. + 7 of the row at `row` (c even, row 4-byte aligned)
__device__ __forceinline__ u32x4 load128_clamped(const unsigned short* row, int c, int limit) {
    return *reinterpret_cast<const u32x4*>(row + clampi(c, 0, limit - 8));
}
// the element pair at the even column c, zero outside the row (limit even)
__device__ __forceinline__ unsigned load_pair(const unsigned short* row, int c, int limit) {
    const unsigned v = *reinterpret_cast<const unsigned*>(row + clampi(c, 0, limit - 2));
    return (c >= 0 && c < limit) ? v : 0u;
}
__device__ __forceinline__ u32x4 shift_one(u32x4 v, unsigned next) {
    return u32x4{__builtin_amdgcn_alignbit(v.y, v.x, 16), __builtin_amdgcn_alignbit(v.z, v.y, 16), __builtin_amdgcn_alignbit(v.w, v.z, 16),
                 __builtin_amdgcn_alignbit(next, v.w, 16)};
}

// Compile-time geometry of one (dilation, taps per wave) pair.
template <int D, int NTW>
struct Tz {
    static constexpr int U = D >= 8 ? 32 : 4 * D;      // elements between consecutive operands
    static constexpr int A = 32 / U;                    // new operands per k-step
    static constexpr int B = 4 * D / U;                 // operands between consecutive taps of a wave
    static constexpr int NQ = U == 4 ? 2 : 1;           // phase classes of a wave (parity of G when U = 4)
    static constexpr int SPAN = (NTW - 1) * B + 1;      // operands a k-step looks at
    static constexpr int R = (SPAN + A + A - 1) / A * A;  // ring slots: a multiple of A, >= SPAN + A
    // k-steps per unit (one LDS stage) and units per unrolled body: A * LU * NB is a multiple of R, so that the
    // ring slot of every operand is a compile-time constant
    static constexpr int NB = D == 16 ? 2 : 1;
    static constexpr int LU = D == 16 ? R / 2 : (D == 8 ? R : 2 * R / A);
    static constexpr int WSP = (7 + 3 * D + 4 * (NQ - 1)) >> 3;  // largest slot offset between the waves' operands
    static constexpr int NXS = 4 * LU + WSP + 4;        // x slots per row and copy in a unit's stage
    static constexpr int HS = U * SPAN / 8;             // slot of operand SPAN (the first refill) ...
    static constexpr int HP = U * (SPAN - 1) / 8;       // ... and of operand SPAN - 1 (the last of the first fill)
    static constexpr int NXP = HP + WSP + 4;            // x slots per row and copy of the first fill
    static_assert((A * LU * NB) % R == 0, "ring slots must repeat from body to body");
    static_assert(R >= SPAN + A, "ring too small");
    static_assert(D != 16 || R % 2 == 0, "d = 16: two units per body");
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
    {
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
    }

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        // Byte offsets into LDS of this lane's operands:
        //   dy operand of filter block fb, k-step tt of a unit:  row 16 fb + li, slot 4 tt + kb
        //   x operand G = a t0 + Gc (t0: first k-step of the body):  copy of phase (E & 7), row li,
        //       slot hslot(Gc) + (E >> 3) + kb - (window origin >> 3),  E = E0 + v d + 4 q,  q = class of Gc
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
                    // the next k-step are read while the MFMAs run; the group barriers pin the interleaving.
#pragma unroll
                    for (int i = 0; i < NTW; ++i) {
                        int nreads = 0;
#pragma unroll
                        for (int r = 0; r < G::A; ++r)
                            if (r * NTW / G::A == i) {
                                const int Gc = G::A * tb + SPAN + r;
                                ring[Gc % R] = ld(xo[G::qcls(Gc)] + 16u * static_cast<unsigned>(G::hslot(Gc) - G::HS - 4 * ub * LU));
                                ++nreads;
                            }
                        if (tt + 1 < LU) {
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb)
                                if (fb * NTW / FB == i) {
                                    anxt[fb] = ld(ya[fb] + 64u * static_cast<unsigned>(tt + 1));
                                    ++nreads;
                                }
                        }
#pragma unroll
                        for (int fb = 0; fb < FB; ++fb)
                            acc[fb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[fb], ring[(G::A * tb + G::B * i) % R], acc[fb][i], 0, 0, 0);
                        if (nreads == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        if (nreads == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        if (nreads == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, FB, 0);
                    }
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
        // by one element.  A load item is (slot, even base e); every thread owns up to kMaxI of them.
        // Rows beyond C or K re-read the last row: their sums are never stored and no other sum depends on them.
        // FAST (widths, sample strides and pointers multiples of 2 elements): units are fetched one unit ahead;
        // a unit whose whole window lies inside the rows ("interior") from scalar base + per-thread constant
        // offsets.  Otherwise every unit is loaded element by element, zero outside the row, when it is written
        // to LDS.
        constexpr int SY = 4 * LU;
        constexpr int NY = FB * 16 * SY, NXT = 16 * G::NXS;
        static_assert(NY <= 256 * kMaxY, "dy staging slots");
        const int ng = __builtin_popcount(a.gmask);
        const int nitems = ((NXT + 255) >> 8) * ng;
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
            xcol[it] = 8 * i + (it < nitems ? item_base(it) : 0);
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
        auto prefetch = [&](Stage& st, int u) {
            if (!FAST) return;
            const int q0 = qs + u * 32 * LU;
            if (interior(q0)) {
                const unsigned short* yb = dyn + q0;
                const unsigned short* xb = xn + (q0 + fl8);
#pragma unroll
                for (int k = 0; k < kMaxY; ++k)
                    if (k * 256 < NY) st.y[k] = *reinterpret_cast<const u32x4*>(yb + (yrow[k] + static_cast<unsigned>(ycol[k])));
#pragma unroll
                for (int it = 0; it < kMaxI; ++it)
                    if (it < nitems) {
                        const unsigned short* src = xb + (xrow[it] + static_cast<unsigned>(xcol[it]));
                        st.x[it] = *reinterpret_cast<const u32x4*>(src);
                        if (has_odd(it)) st.xd[it] = *reinterpret_cast<const unsigned*>(src + 8);
                    }
            } else {
#pragma unroll
                for (int k = 0; k < kMaxY; ++k)
                    if (k * 256 < NY) st.y[k] = load128_clamped(dyn + yrow[k], q0 + ycol[k], a.Q);
#pragma unroll
                for (int it = 0; it < kMaxI; ++it)
                    if (it < nitems) {
                        const int c = q0 + fl8 + xcol[it];
                        st.x[it] = load128_clamped(xn + xrow[it], c, a.W);
                        if (has_odd(it)) st.xd[it] = load_pair(xn + xrow[it], c + 8, a.W);
                    }
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
                    for (int it = 0; it < kMaxI; ++it)
                        if (it < nitems) st.x[it] = fix128(st.x[it], q0 + fl8 + xcol[it], a.W);
                }
            } else {
#pragma unroll
                for (int k = 0; k < kMaxY; ++k)
                    if (k * 256 < NY) st.y[k] = load8(dyn, yrow[k], q0 + ycol[k], a.Q);
#pragma unroll
                for (int it = 0; it < kMaxI; ++it)
                    if (it < nitems) {
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
                if (it < nitems && rtid + (it / ng) * 256 < NXT) {
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
        Stage st;
        if (nunits > 0) {
            prefetch(st, 0);
            commit(st, 0);
            if (nunits > 1) prefetch(st, 1);
        }
        __syncthreads();
        __syncthreads();
        for (int u = 0; u < nunits; ++u) {
            if (u + 1 < nunits) {
                commit(st, u + 1);
                if (u + 2 < nunits) prefetch(st, u + 2);
            }
            __syncthreads();
        }
    }
}

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

struct TzPlan {
    bool ok;
    int D, FB, NTW, fast, grid, tile;
    size_t lds_bytes;
    TzArgs a;
};

template <int D, int NTW>
bool tz_geometry(const WgradProblem& p, int FB, TzPlan& pl) {
    using G = Tz<D, NTW>;
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
    if (FB * 16 * 4 * G::LU > 256 * kMaxY) return false;
    if ((16 * G::NXS + 255) / 256 * ng > kMaxI) return false;
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
    if (pl.lds_bytes > static_cast<size_t>(kLdsBudget)) return false;
    const int QB = 32 * G::LU * G::NB;  // columns per body
    a.BPR = cdiv(p.Q, QB);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const long total_bodies = static_cast<long>(p.N) * a.BPR;
    long want = kNumCU / ncombos;  // strips
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

TzPlan tz_plan(const WgradProblem& p) {
    TzPlan pl{};
    pl.ok = false;
    if (!p.bf16) return pl;
    if (p.d != 1 && p.d != 2 && p.d != 4 && p.d != 8 && p.d != 16) return pl;
    if (p.dw_sc != p.S || p.dw_sk != static_cast<long>(p.C) * p.S) return pl;  // writes the whole dw tensor
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    if (static_cast<long>(p.K) * p.C * p.S >= (1L << 31)) return pl;
    if (p.S < 27) return pl;  // too few taps per wave: the blocked kernel wastes fewer MFMAs
    pl.D = p.d;
    pl.NTW = 13;
    bool ok = false;
    for (int FB = p.K > 16 ? 2 : 1; FB >= 1 && !ok; --FB) {
        pl.FB = FB;
        switch (p.d) {
            case 1: ok = tz_geometry<1, 13>(p, FB, pl); break;
            case 2: ok = tz_geometry<2, 13>(p, FB, pl); break;
            case 4: ok = tz_geometry<4, 13>(p, FB, pl); break;
            case 8: ok = tz_geometry<8, 13>(p, FB, pl); break;
            default: ok = tz_geometry<16, 13>(p, FB, pl); break;
        }
    }
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

template <int D, int FB, int NTW>
hipError_t tz_launch(const TzPlan& pl, hipStream_t st) {
    auto kern = pl.fast ? toeplitz_wgrad_bf16_kernel<D, FB, NTW, true> : toeplitz_wgrad_bf16_kernel<D, FB, NTW, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
    return hipGetLastError();
}

template <int D>
hipError_t tz_launch_d(const TzPlan& pl, hipStream_t st) {
    if (pl.FB == 2) return tz_launch<D, 2, 13>(pl, st);
    return tz_launch<D, 1, 13>(pl, st);
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
#ifndef CONV1D_DEV_FEW_KERNELS
        case 1: e = tz_launch_d<1>(pl, st); break;
        case 2: e = tz_launch_d<2>(pl, st); break;
        case 16: e = tz_launch_d<16>(pl, st); break;
#endif
        case 4: e = tz_launch_d<4>(pl, st); break;
        case 8: e = tz_launch_d<8>(pl, st); break;
        default: e = hipErrorInvalidValue; break;
    }
    if (e != hipSuccess) return e;
    const long nel = static_cast<long>(pl.grid / pl.a.nstrips) * pl.tile;
    hipLaunchKernelGGL(toeplitz_wgrad_reduce_kernel, dim3(cdiv(nel, 64)), dim3(256), 0, st, static_cast<const float*>(p.ws), p.dw, pl.a, pl.FB,
                       pl.NTW);
    return hipGetLastError();
}

}  // namespace conv1d
