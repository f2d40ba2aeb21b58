// Backward-weight pass (Section 3.3, Algorithm 4) for bfloat16 inputs, any dilation and any channel count.
//
//   dw[k][c][s] = sum_n sum_q dy[n][k][q] * x[n][c][q + s*d - P]
//
// The contraction runs over positions.  One v_mfma_f32_16x16x32_bf16 multiplies A = dy (16 filters x 32
// positions) with B = x shifted by one tap (32 positions x 16 channels) into the 16 x 16 block of dw of that
// tap; a lane's 8 k-values are 8 consecutive positions, i.e. one 16-byte LDS read.
//
// Alignment.  LDS reads of 16 bytes are fast only at 16-byte addresses, but tap s needs the positions
// q + s*d - P, whose offset modulo 8 elements depends on s.  The x rows of a chunk are therefore staged once
// per residue ("phase") that occurs among the taps: copy phi holds the row shifted left by phi elements, so the
// operand of a tap with (s*d - P) = phi (mod 8) is an aligned slot of copy phi.  d = 8, 16 need one copy, d = 4
// two, d = 2 four, odd d eight.
//
// Work split.  The dw tensor is cut into (filter group of FB blocks of 16) x (channel block of 16) x (tap group
// of NT taps); the positions (n, q) are cut into chunks of QC columns of one sample and the chunks into
// contiguous strips.  A workgroup owns one (group, block, group) combination and one strip: it walks its chunks
// with all FB*NT accumulators of a wave in registers and writes one partial tensor block per strip to the
// workspace; a second kernel adds the strips in a fixed order (no floating-point atomics, bit-reproducible).
//
// Workgroup = 8 waves, one per CU: waves 0-3 ("consumers") each take a quarter of the chunk's positions and do
// nothing but LDS operand reads and MFMAs (x operands are shared by the FB filter blocks, dy operands by the NT
// taps); waves 4-7 ("producers") load the next chunk from global memory, build the shifted copies and write them
// into the other half of the double-buffered LDS.  One workgroup barrier per chunk.  At the end of the strip
// the four consumers' accumulators are added through LDS.
#include "conv1d_internal.h"

namespace conv1d {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kLdsBudget = 160 * 1024;
constexpr int kNumCU = 256;
constexpr int kMaxY = 8;   // dy staging slots per producer thread
constexpr int kMaxX = 6;   // x staging slots per producer thread
constexpr int kRowBad = 1 << 30;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct BlkArgs {
    const unsigned short* x;
    const unsigned short* dy;
    float* ws;
    int C, K, W, Q, S, d, P;
    long x_sn, dy_sn, KCS;
    int CPR, nchunks, nstrips;  // chunks per sample row, N * CPR, strips
    int nfg, ncb, ntg;          // filter groups, channel blocks, tap groups
    int QC, nksw;               // columns per chunk, k-steps (32 columns) per consumer wave = QC / 128
    int RSY, RSX, NXS;          // LDS row strides in 16-byte slots (odd), x slots staged per row
    unsigned phase_mask;        // bit phi set: a tap with (s*d - P - fl8) % 8 == phi exists in some tap group
    int xcopy_slots;            // 16 * RSX
    int ybuf_slots;             // FB * 16 * RSY
    int stage_slots;            // ybuf_slots + ncopies * xcopy_slots
};

// out = elements [phi, phi + 8) of the 16 consecutive elements (lo, hi)
__device__ __forceinline__ u32x4 shift_elems(u32x4 lo, u32x4 hi, int phi) {
    switch (phi) {
        case 0: return lo;
        case 1: return u32x4{__builtin_amdgcn_alignbit(lo.y, lo.x, 16), __builtin_amdgcn_alignbit(lo.z, lo.y, 16),
                             __builtin_amdgcn_alignbit(lo.w, lo.z, 16), __builtin_amdgcn_alignbit(hi.x, lo.w, 16)};
        case 2: return u32x4{lo.y, lo.z, lo.w, hi.x};
        case 3: return u32x4{__builtin_amdgcn_alignbit(lo.z, lo.y, 16), __builtin_amdgcn_alignbit(lo.w, lo.z, 16),
                             __builtin_amdgcn_alignbit(hi.x, lo.w, 16), __builtin_amdgcn_alignbit(hi.y, hi.x, 16)};
        case 4: return u32x4{lo.z, lo.w, hi.x, hi.y};
        case 5: return u32x4{__builtin_amdgcn_alignbit(lo.w, lo.z, 16), __builtin_amdgcn_alignbit(hi.x, lo.w, 16),
                             __builtin_amdgcn_alignbit(hi.y, hi.x, 16), __builtin_amdgcn_alignbit(hi.z, hi.y, 16)};
        case 6: return u32x4{lo.w, hi.x, hi.y, hi.z};
        default: return u32x4{__builtin_amdgcn_alignbit(hi.x, lo.w, 16), __builtin_amdgcn_alignbit(hi.y, hi.x, 16),
                              __builtin_amdgcn_alignbit(hi.z, hi.y, 16), __builtin_amdgcn_alignbit(hi.w, hi.z, 16)};
    }
}

template <int FB, int NT, bool FAST>
__global__ __launch_bounds__(512, 2) void blocked_wgrad_bf16_kernel(BlkArgs a) {
    extern __shared__ u32x4 lds4[];
    // operand prefetch distance in taps: the LDS latency has to be covered by PF * FB MFMAs
    constexpr int PF = FB == 1 ? 6 : (FB == 2 ? 4 : 2);
    constexpr int R = PF + 2;                  // operand ring
    constexpr int NTP = (NT + R - 1) / R * R;  // ring positions per k-step (taps padded to a multiple of R)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = wave < 4;
    const int cw = wave & 3;
    const int rtid = tid & 255;
    if (!consumer) __builtin_amdgcn_s_setprio(3);
    const int li = lane & 15;
    const int kb = lane >> 4;

    // Workgroups are dealt round-robin to the 8 XCDs: the logical index puts the combinations of one strip
    // (which read the same x and dy chunks) next to each other on one XCD and its L2.
    int lid = blockIdx.x;
    if ((gridDim.x & 7) == 0) lid = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const int strip = lid / ncombos;
    const int combo = lid - strip * ncombos;
    const int tg = combo % a.ntg;
    const int cbi = (combo / a.ntg) % a.ncb;
    const int fg = combo / (a.ntg * a.ncb);
    const int s0 = tg * NT, c0 = cbi * 16, k0 = fg * FB * 16;
    const int fl8 = ((s0 * a.d - a.P) >> 3) * 8;  // window origin relative to the chunk: floor to a multiple of 8
    const int ch_begin = static_cast<int>(static_cast<long>(strip) * a.nchunks / a.nstrips);
    const int ch_end = static_cast<int>(static_cast<long>(strip + 1) * a.nchunks / a.nstrips);

    // ---- producer side ---------------------------------------------------------------------------
    // A staging slot is 8 consecutive columns of one row.  dy slot (row, i) <-> dy[k0 + row][q0 + 8i ..];
    // x slot (row, i) <-> x[c0 + row][q0 + fl8 + 8i ..], needed with every phase shift, so the next 8 columns
    // are loaded with it.  FAST (all widths and sample strides multiples of 8 elements, 16-byte aligned
    // pointers): 16-byte loads from clamped addresses, masked when written to LDS; a slot is then inside or
    // outside its row as a whole.  Otherwise element loads, done when the stage is written.
    struct Slot {
        unsigned off;  // element offset of the (clamped) source row from the sample's base
        int col;       // column of the slot relative to the chunk's origin
        int lds;       // row * stride + i, bit 30: row beyond C or K
    };
    const int SY = a.QC >> 3;
    const int NY = FB * 16 * SY, NX = 16 * a.NXS;
    auto make_y = [&](int e) -> Slot {
        const int row = e / SY, i = e - row * SY;
        return Slot{static_cast<unsigned>(min(k0 + row, a.K - 1)) * static_cast<unsigned>(a.Q), 8 * i,
                    (row * a.RSY + i) | (k0 + row < a.K ? 0 : kRowBad)};
    };
    auto make_x = [&](int e) -> Slot {
        const int row = e / a.NXS, i = e - row * a.NXS;
        return Slot{static_cast<unsigned>(min(c0 + row, a.C - 1)) * static_cast<unsigned>(a.W), 8 * i,
                    (row * a.RSX + i) | (c0 + row < a.C ? 0 : kRowBad)};
    };
    auto load8 = [&](const unsigned short* row, int g, int limit) -> u32x4 {  // columns g .. g+7 of a row of `limit` columns
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
    auto inside = [&](int g, int limit) { return !FAST || (g >= 0 && g + 8 <= limit); };
    const u32x4 zero4 = u32x4{0u, 0u, 0u, 0u};

    Slot ys[kMaxY], xs[kMaxX];
    u32x4 ypre[FAST ? kMaxY : 1], xlo[FAST ? kMaxX : 1], xhi[FAST ? kMaxX : 1];
    if (!consumer) {
#pragma unroll
        for (int k = 0; k < kMaxY; ++k) ys[k] = make_y(min(rtid + k * 256, NY - 1));
#pragma unroll
        for (int k = 0; k < kMaxX; ++k) xs[k] = make_x(min(rtid + k * 256, NX - 1));
    }
    auto origin = [&](int ch, const unsigned short*& xn, const unsigned short*& dyn, int& q0) {
        const int n = ch / a.CPR;
        q0 = (ch - n * a.CPR) * a.QC;
        xn = a.x + static_cast<long>(n) * a.x_sn;
        dyn = a.dy + static_cast<long>(n) * a.dy_sn;
    };
    auto prefetch = [&](int ch) {
        if constexpr (FAST) {
            const unsigned short *xn, *dyn;
            int q0;
            origin(ch, xn, dyn, q0);
#pragma unroll
            for (int k = 0; k < kMaxY; ++k) ypre[k] = load8(dyn + ys[k].off, q0 + ys[k].col, a.Q);
#pragma unroll
            for (int k = 0; k < kMaxX; ++k) {
                xlo[k] = load8(xn + xs[k].off, q0 + fl8 + xs[k].col, a.W);
                xhi[k] = load8(xn + xs[k].off, q0 + fl8 + xs[k].col + 8, a.W);
            }
        }
    };
    auto commit = [&](int ch, int b) {
        const unsigned short *xn, *dyn;
        int q0;
        origin(ch, xn, dyn, q0);
        u32x4* ybuf = lds4 + b * a.stage_slots;
        u32x4* xbuf = ybuf + a.ybuf_slots;
#pragma unroll
        for (int k = 0; k < kMaxY; ++k) {
            if (rtid + k * 256 < NY) {
                const int g = q0 + ys[k].col;
                u32x4 v;
                if constexpr (FAST) v = ypre[k]; else v = load8(dyn + ys[k].off, g, a.Q);
                if ((ys[k].lds & kRowBad) || !inside(g, a.Q)) v = zero4;
                ybuf[ys[k].lds & (kRowBad - 1)] = v;
            }
        }
#pragma unroll
        for (int k = 0; k < kMaxX; ++k) {
            if (rtid + k * 256 < NX) {
                const int g = q0 + fl8 + xs[k].col;
                u32x4 lo, hi;
                if constexpr (FAST) {
                    lo = xlo[k];
                    hi = xhi[k];
                } else {
                    lo = load8(xn + xs[k].off, g, a.W);
                    hi = load8(xn + xs[k].off, g + 8, a.W);
                }
                const bool bad = xs[k].lds & kRowBad;
                if (bad || !inside(g, a.W)) lo = zero4;
                if (bad || !inside(g + 8, a.W)) hi = zero4;
                u32x4* dst = xbuf + (xs[k].lds & (kRowBad - 1));
                for (unsigned m = a.phase_mask; m != 0; m &= m - 1) {  // uniform: one copy per phase in use
                    *dst = shift_elems(lo, hi, __builtin_ctz(m));
                    dst += a.xcopy_slots;
                }
            }
        }
    };

    // ---- consumer side ---------------------------------------------------------------------------
    // Byte offsets into LDS of this lane's operands in stage 0, k-step 0 of this wave's quarter:
    //   dy operand of filter block fb:  row 16 fb + li, slot 4 ks + kb
    //   x operand of tap s0 + i:        copy of phase (delta & 7), row li, slot 4 ks + kb + (delta >> 3),
    //                                   delta = (s0 + i) d - P - fl8 >= 0
    // Taps beyond S (last tap group) are clamped to tap S - 1 for addressing; their sums are not stored.
    unsigned ay[FB], bx[NT];
    f32x4 acc[FB][NT];
    {
        const int ks0 = cw * a.nksw;
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) ay[fb] = 16u * static_cast<unsigned>((fb * 16 + li) * a.RSY + 4 * ks0 + kb);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int s = min(s0 + i, a.S - 1);
            const int delta = s * a.d - a.P - fl8;
            const int ci = __builtin_popcount(a.phase_mask & ((1u << (delta & 7)) - 1u));
            bx[i] = 16u * static_cast<unsigned>(a.ybuf_slots + ci * a.xcopy_slots + li * a.RSX + 4 * ks0 + kb + (delta >> 3));
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) acc[fb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
    const char* ldsb = reinterpret_cast<const char*>(lds4);
    auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };

    auto compute = [&](int b) {
        unsigned ko = static_cast<unsigned>(b * a.stage_slots) * 16u;
        bf16x8 acur[FB], anxt[FB], ring[R];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) acur[fb] = ld(ay[fb] + ko);
#pragma unroll
        for (int i = 0; i < PF; ++i)
            if (i < NT) ring[i % R] = ld(bx[i] + ko);
        for (int ks = 0; ks < a.nksw; ++ks) {
            // (the reads issued for "the next k-step" in the last k-step fall into the slack behind the rows)
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) anxt[fb] = ld(ay[fb] + ko + 64);
#pragma unroll
            for (int i = 0; i < NTP; ++i) {
                const int f = i + PF;  // ring position to refill
                if (f < NTP) {
                    if (f < NT) ring[f % R] = ld(bx[f] + ko);
                } else if (f - NTP < NT) {
                    ring[f % R] = ld(bx[f - NTP] + ko + 64);
                }
                if (i < NT) {
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb)
                        acc[fb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[fb], ring[i % R], acc[fb][i], 0, 0, 0);
                }
            }
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) acur[fb] = anxt[fb];
            ko += 64;
        }
    };

    // ---- pipeline (one loop per role: the register allocation of one role is not burdened by the other's) ------
    f32x4* red = reinterpret_cast<f32x4*>(lds4);
    if (consumer) {
        __syncthreads();
        for (int ch = ch_begin; ch < ch_end; ++ch) {
            compute((ch - ch_begin) & 1);
            __syncthreads();
        }
        // ---- add the four consumers' sums and write this strip's partial block ----------------------
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int i = 0; i < NT; ++i) red[((cw * FB + fb) * NT + i) * 64 + lane] = acc[fb][i];
    } else {
        if (ch_begin < ch_end) {
            prefetch(ch_begin);
            commit(ch_begin, 0);
            if (ch_begin + 1 < ch_end) prefetch(ch_begin + 1);
        }
        __syncthreads();
        for (int ch = ch_begin; ch < ch_end; ++ch) {
            if (ch + 1 < ch_end) {
                commit(ch + 1, ((ch - ch_begin) & 1) ^ 1);
                if (ch + 2 < ch_end) prefetch(ch + 2);
            }
            __syncthreads();
        }
    }
    __syncthreads();
    const float* redf = reinterpret_cast<const float*>(lds4);
    float* ws = a.ws + static_cast<long>(strip) * a.KCS;
    for (int e = tid; e < FB * NT * 256; e += 512) {
        float sum = redf[e];
#pragma unroll
        for (int w = 1; w < 4; ++w) sum += redf[w * FB * NT * 256 + e];
        const int blk = e >> 8, r = e & 255;
        const int fb = blk / NT, i = blk - fb * NT;
        const int l = r >> 2, jj = r & 3;
        const int k = k0 + 16 * fb + 4 * (l >> 4) + jj, c = c0 + (l & 15), s = s0 + i;
        if (k < a.K && c < a.C && s < a.S) ws[(static_cast<long>(k) * a.C + c) * a.S + s] = sum;
    }
}

// dw[e] = sum over strips of ws[strip][e], strips added in a fixed order: 16 interleaved running sums per
// element, then those 16 in order.
__global__ __launch_bounds__(256) void blocked_wgrad_reduce_kernel(const float* __restrict__ ws, float* __restrict__ dw, long KCS, int nstrips) {
    __shared__ float part[16][17];
    const int el = threadIdx.x & 15, g = threadIdx.x >> 4;
    const long e = static_cast<long>(blockIdx.x) * 16 + el;
    float sum = 0.f;
    if (e < KCS)
        for (int s = g; s < nstrips; s += 16) sum += ws[s * KCS + e];
    part[g][el] = sum;
    __syncthreads();
    if (g == 0 && e < KCS) {
        float t = part[0][el];
#pragma unroll
        for (int j = 1; j < 16; ++j) t += part[j][el];
        dw[e] = t;
    }
}

struct BlkPlan {
    bool ok;
    int FB, NT, fast, grid;
    size_t lds_bytes;
    BlkArgs a;
};

struct Shape { int FB, NT; };
#ifdef CONV1D_DEV_FEW_KERNELS
constexpr Shape kShapes[] = {{1, 17}, {4, 9}};
#else
constexpr Shape kShapes[] = {{1, 5}, {1, 9}, {1, 17}, {1, 26}, {2, 9}, {2, 17}, {4, 5}, {4, 9}};
#endif

BlkPlan blk_plan(const WgradProblem& p) {
    BlkPlan pl{};
    pl.ok = false;
    if (!p.bf16) return pl;
    if (p.dw_sc != p.S || p.dw_sk != static_cast<long>(p.C) * p.S) return pl;  // writes the whole dw tensor
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return pl;
    const long KCS = static_cast<long>(p.K) * p.C * p.S;
    if (KCS >= (1L << 31)) return pl;
    const int nfb = cdiv(p.K, 16);
    BlkArgs& a = pl.a;
    // shapes in order of cost: MFMA slots, an LDS operand read counted as half an MFMA
    constexpr int kNumShapes = sizeof(kShapes) / sizeof(kShapes[0]);
    int order[kNumShapes];
    double cost[kNumShapes];
    for (int i = 0; i < kNumShapes; ++i) {
        const Shape& sh = kShapes[i];
        const double slots = static_cast<double>(cdiv(nfb, sh.FB)) * sh.FB * cdiv(p.S, sh.NT) * sh.NT;
        cost[i] = slots * (1.0 + 0.5 * (sh.FB + sh.NT) / (sh.FB * sh.NT));
        int j = i;
        while (j > 0 && cost[order[j - 1]] > cost[i]) { order[j] = order[j - 1]; --j; }
        order[j] = i;
    }
    for (int oi = 0; oi < kNumShapes; ++oi) {
    pl.FB = kShapes[order[oi]].FB;
    pl.NT = kShapes[order[oi]].NT;
    a.ntg = cdiv(p.S, pl.NT);
    a.nfg = cdiv(nfb, pl.FB);
    a.ncb = cdiv(p.C, 16);
    // phases in use: delta = s*d - P - fl8(group) over all taps of all groups
    a.phase_mask = 0;
    for (int s = 0; s < p.S; ++s) {
        const long s0 = s / pl.NT * pl.NT;
        const long fl8 = ((s0 * p.d - p.P) >> 3) * 8;
        a.phase_mask |= 1u << ((static_cast<long>(s) * p.d - p.P - fl8) & 7);
    }
    const int ncopies = __builtin_popcount(a.phase_mask);
    const long span = static_cast<long>(pl.NT - 1) * p.d + 7;  // largest delta
    for (int QC = 512; QC >= 128; QC /= 2) {
        const int SY = QC / 8;
        if (pl.FB * 16 * SY > 256 * kMaxY) continue;
        const long NXS = SY + span / 8 + 1;
        if (16 * NXS > 256 * kMaxX) continue;
        a.QC = QC;
        a.nksw = QC / 128;
        a.RSY = SY + 1;
        a.NXS = static_cast<int>(NXS);
        a.RSX = static_cast<int>(NXS | 1);
        a.xcopy_slots = 16 * a.RSX;
        a.ybuf_slots = pl.FB * 16 * a.RSY;
        a.stage_slots = a.ybuf_slots + ncopies * a.xcopy_slots;
        // + slack for the look-ahead reads of the last k-step (4 slots behind the last row)
        size_t bytes = static_cast<size_t>(2 * a.stage_slots + 8) * 16;
        const size_t red = static_cast<size_t>(4) * pl.FB * pl.NT * 1024;
        if (bytes > static_cast<size_t>(kLdsBudget)) continue;
        if (red > bytes) bytes = red;
        pl.lds_bytes = bytes;
        a.CPR = cdiv(p.Q, QC);
        const long nc = static_cast<long>(p.N) * a.CPR;
        if (nc > 0x7fffffffL) return pl;
        a.nchunks = static_cast<int>(nc);
        const int ncombos = a.nfg * a.ncb * a.ntg;
        int nstrips = kNumCU / ncombos;
        if (nstrips < 1) nstrips = 1;
        if (nstrips > a.nchunks) nstrips = a.nchunks;
        a.nstrips = nstrips;
        const long grid = static_cast<long>(ncombos) * nstrips;
        if (grid > 0x7fffffffL) return pl;
        pl.grid = static_cast<int>(grid);
        a.x = static_cast<const unsigned short*>(p.x);
        a.dy = static_cast<const unsigned short*>(p.dy);
        a.ws = static_cast<float*>(p.ws);
        a.C = p.C; a.K = p.K; a.W = p.W; a.Q = p.Q; a.S = p.S; a.d = p.d; a.P = p.P;
        a.x_sn = p.x_sn; a.dy_sn = p.dy_sn; a.KCS = KCS;
        pl.fast = (p.W % 8 == 0) && (p.Q % 8 == 0) && (p.x_sn % 8 == 0) && (p.dy_sn % 8 == 0) && p.W >= 8 && p.Q >= 8 &&
                  (reinterpret_cast<uintptr_t>(p.x) % 16 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 16 == 0);
        pl.ok = true;
        return pl;
    }
    }
    return pl;
}

template <int FB, int NT>
hipError_t blk_launch(const BlkPlan& pl, hipStream_t st) {
    auto kern = pl.fast ? blocked_wgrad_bf16_kernel<FB, NT, true> : blocked_wgrad_bf16_kernel<FB, NT, false>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(pl.lds_bytes));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
    return hipGetLastError();
}

}  // namespace

bool blocked_bf16_wgrad_supported(const WgradProblem& p) { return blk_plan(p).ok; }

size_t blocked_bf16_wgrad_workspace(const WgradProblem& p) {
    const BlkPlan pl = blk_plan(p);
    return pl.ok ? static_cast<size_t>(pl.a.nstrips) * pl.a.KCS * sizeof(float) : 0;
}

hipError_t blocked_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const BlkPlan pl = blk_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
    const int key = pl.FB * 100 + pl.NT;
    switch (key) {
#ifndef CONV1D_DEV_FEW_KERNELS
        case 105: e = blk_launch<1, 5>(pl, st); break;
        case 109: e = blk_launch<1, 9>(pl, st); break;
        case 126: e = blk_launch<1, 26>(pl, st); break;
        case 209: e = blk_launch<2, 9>(pl, st); break;
        case 217: e = blk_launch<2, 17>(pl, st); break;
        case 405: e = blk_launch<4, 5>(pl, st); break;
#endif
        case 117: e = blk_launch<1, 17>(pl, st); break;
        case 409: e = blk_launch<4, 9>(pl, st); break;
        default: break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(blocked_wgrad_reduce_kernel, dim3(cdiv(pl.a.KCS, 16)), dim3(256), 0, st, static_cast<const float*>(p.ws), p.dw, pl.a.KCS,
                       pl.a.nstrips);
    return hipGetLastError();
}

}  // namespace conv1d
