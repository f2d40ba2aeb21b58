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
constexpr int kMaxI = 12;  // x load items (slot, even phase base) per producer thread

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct BlkArgs {
    const unsigned short* x;
    const unsigned short* dy;
    float* ws;
    int C, K, W, Q, S, d, P;
    long x_sn, dy_sn;
    int CPR, nchunks, nstrips;  // chunks per sample row, N * CPR, strips
    int nfg, ncb, ntg;          // filter groups, channel groups, tap groups
    int ncbw;                   // channel blocks per workgroup (1, 2 or 4): consumer wave v works on block v % ncbw
    int QC, nksw;               // columns per chunk, k-steps (32 columns) per consumer wave = QC / 32 * ncbw / 4
    int RSY, RSX, NXS;          // LDS row strides in 16-byte slots (odd), x slots staged per row
    unsigned phase_mask;        // bit phi set: a tap with (s*d - P - fl8) % 8 == phi exists in some tap group
    unsigned gmask;             // bit g set: phase 2g or 2g + 1 is in use
    int xcopy_slots;            // 16 * ncbw * RSX
    int ybuf_slots;             // FB * 16 * RSY
    int stage_slots;            // ybuf_slots + ncopies * xcopy_slots
};

template <int FB, int NT, bool FAST>
__global__ __launch_bounds__(512, 2) void blocked_wgrad_bf16_kernel(BlkArgs a) {
    extern __shared__ u32x4 lds4[];
    // x operands live in a ring of R registers that is refilled PF = R - 2 taps ahead of its use (the LDS
    // latency has to be covered by PF * FB MFMAs).  R divides the taps of a k-step wherever the registers
    // allow, so that the refills run on seamlessly into the next k-step.
    constexpr int R = NT == 26 ? 13 : ((FB == 2 && NT == 17) ? 6 : NT);
    constexpr int PF = R - 2;
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
    const int lid = xcd_logical_id(blockIdx.x, gridDim.x);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    const int strip = lid / ncombos;
    const int combo = lid - strip * ncombos;
    const int tg = combo % a.ntg;
    const int cbi = (combo / a.ntg) % a.ncb;
    const int fg = combo / (a.ntg * a.ncb);
    const int xrows = 16 * a.ncbw;
    const int s0 = tg * NT, c0 = cbi * xrows, k0 = fg * FB * 16;
    const int fl8 = ((s0 * a.d - a.P) >> 3) * 8;  // window origin relative to the chunk: floor to a multiple of 8
    const int ch_begin = static_cast<int>(static_cast<long>(strip) * a.nchunks / a.nstrips);
    const int ch_end = static_cast<int>(static_cast<long>(strip + 1) * a.nchunks / a.nstrips);
    f32x4* red = reinterpret_cast<f32x4*>(lds4);

    if (consumer) {
        // ---- consumer side -----------------------------------------------------------------------
        // Wave cw works on channel block cw % ncbw and on the k-steps [ks0, ks0 + nksw) of every chunk.
        // Byte offsets into LDS of this lane's operands in stage 0, k-step ks0:
        //   dy operand of filter block fb:  row 16 fb + li, slot 4 ks + kb
        //   x operand of tap s0 + i:        copy of phase (delta & 7), row 16 (cw % ncbw) + li,
        //                                   slot 4 ks + kb + (delta >> 3),  delta = (s0 + i) d - P - fl8 >= 0
        // Taps beyond S (last tap group) are clamped to tap S - 1 for addressing; their sums are not stored.
        const int cbl = cw % a.ncbw;
        const int ks0 = (cw / a.ncbw) * a.nksw;
        unsigned ay[FB], bx[NT];
        f32x4 acc[FB][NT];
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) ay[fb] = 16u * static_cast<unsigned>((fb * 16 + li) * a.RSY + 4 * ks0 + kb);
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int s = min(s0 + i, a.S - 1);
            const int delta = s * a.d - a.P - fl8;
            const int ci = __builtin_popcount(a.phase_mask & ((1u << (delta & 7)) - 1u));
            bx[i] = 16u * static_cast<unsigned>(a.ybuf_slots + ci * a.xcopy_slots + (cbl * 16 + li) * a.RSX + 4 * ks0 + kb + (delta >> 3));
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) acc[fb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const char* ldsb = reinterpret_cast<const char*>(lds4);
        auto ld = [&](unsigned off) { return as_bf16x8(*reinterpret_cast<const u32x4*>(ldsb + off)); };

        __syncthreads();
        for (int ch = ch_begin; ch < ch_end; ++ch) {
            {
                // The operand addresses run along with the k-steps (one add per operand and k-step, off the
                // critical path) and hop to the other stage at the end of the chunk.  Within a k-step the x
                // operand of tap i + PF and, in the first FB positions, the dy operands of the next k-step are
                // read while the MFMAs of tap i run; the group barriers pin that interleaving.
                bf16x8 acur[FB], anxt[FB], ring[R];
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) acur[fb] = ld(ay[fb]);
#pragma unroll
                for (int i = 0; i < PF; ++i)
                    if (i < NT) ring[i % R] = ld(bx[i]);
                for (int ks = 0; ks < a.nksw; ++ks) {
                    // (the reads issued for "the next k-step" in the last k-step fall into the slack behind the rows)
#pragma unroll
                    for (int i = 0; i < NTP; ++i) {
                        const int f = i + PF;  // ring position to refill
                        int nreads = 0;
                        if (f < NTP) {
                            if (f < NT) {
                                ring[f % R] = ld(bx[f]);
                                ++nreads;
                            }
                        } else if (f - NTP < NT) {
                            ring[f % R] = ld(bx[f - NTP] + 64);
                            ++nreads;
                        }
                        if (i < FB) {
                            anxt[i] = ld(ay[i] + 64);
                            ++nreads;
                        }
                        if (i < NT) {
#pragma unroll
                            for (int fb = 0; fb < FB; ++fb)
                                acc[fb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(acur[fb], ring[i % R], acc[fb][i], 0, 0, 0);
                        }
                        if (nreads == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        if (nreads == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        if (i < NT) __builtin_amdgcn_sched_group_barrier(0x008, FB, 0);
                    }
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) {
                        acur[fb] = anxt[fb];
                        ay[fb] += 64;
                    }
#pragma unroll
                    for (int i = 0; i < NT; ++i) bx[i] += 64;
                }
                const unsigned hop = (((ch - ch_begin) & 1) ? 0u - static_cast<unsigned>(a.stage_slots) : static_cast<unsigned>(a.stage_slots)) * 16u -
                                     static_cast<unsigned>(a.nksw) * 64u;
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) ay[fb] += hop;
#pragma unroll
                for (int i = 0; i < NT; ++i) bx[i] += hop;
            }
            __syncthreads();
        }
        // park the sums: the waves that share a channel block are added below
#pragma unroll
        for (int fb = 0; fb < FB; ++fb)
#pragma unroll
            for (int i = 0; i < NT; ++i) red[((cw * FB + fb) * NT + i) * 64 + lane] = acc[fb][i];
    } else {
        // ---- producer side -----------------------------------------------------------------------
        // A staging slot is 8 consecutive columns of one row; consecutive threads stage consecutive slots of a
        // row (coalesced loads, conflict-free LDS writes).  dy slot (row, i) <-> dy[k0 + row][q0 + 8i ..].
        // x slot (row, i) of the copy of phase phi <-> x[c0 + row][q0 + fl8 + phi + 8i ..].  16-byte global loads
        // run at full speed from any 4-byte aligned address, so an even phase is simply loaded where it starts;
        // an odd phase phi = e + 1 is made from the load of the even phase e and the dword behind it, shifted
        // by one element.  A load item is (slot, even base e); every thread owns up to kMaxI of them.
        // Rows beyond C or K re-read the last row: their sums are never stored and no other sum depends on them.
        // FAST (widths, sample strides and pointers multiples of 2 elements) and the chunk "interior" (its whole
        // window inside the rows: all but the first and last chunks of a row): loads from scalar base +
        // per-thread constant offsets, fetched one chunk ahead, written unmasked.  Every other chunk is loaded
        // element by element, zero outside the row, when it is written to LDS.
        const int SY = a.QC >> 3;
        const int NY = FB * 16 * SY, NXT = xrows * a.NXS;
        const int ng = __builtin_popcount(a.gmask);
        const int nitems = ((NXT + 255) >> 8) * ng;
        unsigned yoffb[kMaxY], xoffb[kMaxI];  // byte offset of the slot's first column (phase 0) from the chunk origin of the sample
        int ylds[kMaxY], xlds[kMaxI];         // row * stride + slot
        int ycol[kMaxY], xcol[kMaxI];         // first column relative to the chunk / window origin
        unsigned yrow[kMaxY], xrow[kMaxI];    // element offset of the (clamped) row from the sample's base
#pragma unroll
        for (int k = 0; k < kMaxY; ++k) {
            const int e = min(rtid + k * 256, NY - 1);
            const int row = e / SY, i = e - row * SY;
            yrow[k] = static_cast<unsigned>(min(k0 + row, a.K - 1)) * static_cast<unsigned>(a.Q);
            ycol[k] = 8 * i;
            yoffb[k] = 2u * (yrow[k] + 8u * static_cast<unsigned>(i));
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
            const int row = e / a.NXS, i = e - row * a.NXS;
            xrow[it] = static_cast<unsigned>(min(c0 + row, a.C - 1)) * static_cast<unsigned>(a.W);
            xcol[it] = 8 * i + (it < nitems ? item_base(it) : 0);
            xoffb[it] = 2u * (xrow[it] + static_cast<unsigned>(xcol[it]));
            xlds[it] = row * a.RSX + i;
        }
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
        struct Stage {
            u32x4 y[kMaxY];
            u32x4 x[kMaxI];
            unsigned xd[kMaxI];  // the dword behind x[it] (odd phases)
        };
        struct Geo {
            const unsigned short* xn;
            const unsigned short* dyn;
            int q0;
            bool interior;
        };
        auto geo = [&](int ch) -> Geo {
            Geo g;
            const int n = ch / a.CPR;
            g.q0 = (ch - n * a.CPR) * a.QC;
            g.xn = a.x + static_cast<long>(n) * a.x_sn;
            g.dyn = a.dy + static_cast<long>(n) * a.dy_sn;
            const int x0 = g.q0 + fl8;
            g.interior = FAST && g.q0 + a.QC <= a.Q && x0 >= 0 && x0 + 8 * a.NXS + 16 <= a.W;
            return g;
        };
        auto has_odd = [&](int it) { return (a.phase_mask >> (item_base(it) + 1)) & 1u; };
        auto prefetch = [&](Stage& st, int ch) {
            const Geo g = geo(ch);
            if (!g.interior) return;
            const char* yb = reinterpret_cast<const char*>(g.dyn + g.q0);
            const char* xb = reinterpret_cast<const char*>(g.xn + (g.q0 + fl8));
#pragma unroll
            for (int k = 0; k < kMaxY; ++k)
                if (k * 256 < NY) st.y[k] = *reinterpret_cast<const u32x4*>(yb + yoffb[k]);
#pragma unroll
            for (int it = 0; it < kMaxI; ++it)
                if (it < nitems) {
                    st.x[it] = *reinterpret_cast<const u32x4*>(xb + xoffb[it]);
                    if (has_odd(it)) st.xd[it] = *reinterpret_cast<const unsigned*>(xb + xoffb[it] + 16);
                }
        };
        auto commit = [&](Stage& st, int ch, int b) {
            const Geo g = geo(ch);
            if (!g.interior) {
#pragma unroll
                for (int k = 0; k < kMaxY; ++k)
                    if (k * 256 < NY) st.y[k] = load8(g.dyn, yrow[k], g.q0 + ycol[k], a.Q);
#pragma unroll
                for (int it = 0; it < kMaxI; ++it)
                    if (it < nitems) {
                        const int c = g.q0 + fl8 + xcol[it];
                        st.x[it] = load8(g.xn, xrow[it], c, a.W);
                        const int c8 = c + 8;
                        const unsigned xd = g.xn[xrow[it] + static_cast<unsigned>(c8 < 0 ? 0 : (c8 > a.W - 1 ? a.W - 1 : c8))];
                        st.xd[it] = (c8 >= 0 && c8 < a.W) ? xd : 0u;
                    }
            }
            u32x4* ybuf = lds4 + b * a.stage_slots;
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
                    if ((a.phase_mask >> (e + 1)) & 1u)
                        *dst = u32x4{__builtin_amdgcn_alignbit(v.y, v.x, 16), __builtin_amdgcn_alignbit(v.z, v.y, 16),
                                     __builtin_amdgcn_alignbit(v.w, v.z, 16), __builtin_amdgcn_alignbit(st.xd[it], v.w, 16)};
                }
        };
        Stage st;
        if (ch_begin < ch_end) {
            prefetch(st, ch_begin);
            commit(st, ch_begin, 0);
            if (ch_begin + 1 < ch_end) prefetch(st, ch_begin + 1);
        }
        __syncthreads();
        for (int ch = ch_begin; ch < ch_end; ++ch) {
            if (ch + 1 < ch_end) {
                commit(st, ch + 1, ((ch - ch_begin) & 1) ^ 1);
                    if (ch + 2 < ch_end) prefetch(st, ch + 2);
            }
            __syncthreads();
        }
    }

    // ---- add the sums of the waves that share a channel block; one contiguous tile per workgroup ----------
    //   tile element ((cbl * FB + fb) * NT + i) * 256 + 4 * lane + jj  <->  filter k0 + 16 fb + 4 (lane >> 4) + jj,
    //   channel c0 + 16 cbl + (lane & 15), tap s0 + i
    __syncthreads();
    const float* redf = reinterpret_cast<const float*>(lds4);
    const int tile = a.ncbw * FB * NT * 256;
    float* ws = a.ws + static_cast<long>(lid) * tile;
    const int nparts = 4 / a.ncbw;
    for (int e = tid; e < tile; e += 512) {
        const int cbl = e / (FB * NT * 256), r = e - cbl * (FB * NT * 256);
        float sum = redf[cbl * (FB * NT * 256) + r];
        for (int part = 1; part < nparts; ++part) sum += redf[(cbl + part * a.ncbw) * (FB * NT * 256) + r];
        ws[e] = sum;
    }
}

// Adds the strips in a fixed order (16 interleaved running sums per element, then those 16 in order) and
// scatters the tiles into dw[k][c][s].  A block of 16 x 16 threads handles 64 consecutive tile elements: thread
// (g, el) adds the strips g, g + 16, ... of the 4 elements 4 el .. 4 el + 3 with 16-byte loads.  The tile size is
// a multiple of 256, so a block never straddles two combinations.
__global__ __launch_bounds__(256) void blocked_wgrad_reduce_kernel(const float* __restrict__ ws, float* __restrict__ dw, BlkArgs a, int FB, int NT) {
    __shared__ f32x4 part[16][17];
    const int el = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int tile = a.ncbw * FB * NT * 256;
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
        const int i = blk % NT, fb = (blk / NT) % FB, cbl = blk / (NT * FB);
        const int k0 = (fg * FB + fb) * 16 + 4 * (l >> 4), c = (cbi * a.ncbw + cbl) * 16 + (l & 15), s = tg * NT + i;
        if (c < a.C && s < a.S) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
                if (k0 + jj < a.K) dw[(static_cast<long>(k0 + jj) * a.C + c) * a.S + s] = t[jj];
        }
    }
}

struct BlkPlan {
    bool ok;
    int FB, NT, fast, grid, tile;
    size_t lds_bytes;
    BlkArgs a;
};

struct Shape { int FB, NT; };
constexpr Shape kShapes[] = {{1, 5}, {1, 9}, {1, 17}, {1, 26}, {2, 9}, {2, 17}, {4, 5}, {4, 9}};

// Geometry of one candidate (shape, channel blocks per workgroup, chunk length); false if it does not fit.
bool blk_geometry(const WgradProblem& p, int FB, int NT, int ncbw, int QC, BlkPlan& pl) {
    BlkArgs& a = pl.a;
    const int nfb = cdiv(p.K, 16);
    pl.FB = FB;
    pl.NT = NT;
    a.ntg = cdiv(p.S, NT);
    a.nfg = cdiv(nfb, FB);
    // phases in use: delta = s*d - P - fl8(group) over all taps of all groups
    a.phase_mask = 0;
    for (int s = 0; s < p.S; ++s) {
        const long s0 = s / NT * NT;
        const long fl8 = ((s0 * p.d - p.P) >> 3) * 8;
        a.phase_mask |= 1u << ((static_cast<long>(s) * p.d - p.P - fl8) & 7);
    }
    const int ncopies = __builtin_popcount(a.phase_mask);
    a.gmask = 0;
    for (int g = 0; g < 4; ++g)
        if ((a.phase_mask >> (2 * g)) & 3u) a.gmask |= 1u << g;
    const int ng = __builtin_popcount(a.gmask);
    const long span = static_cast<long>(NT - 1) * p.d + 7;  // largest delta
    const int SY = QC / 8;
    if (FB * 16 * SY > 256 * kMaxY) return false;
    const long NXS = SY + span / 8 + 1;
    if ((16 * ncbw * NXS + 255) / 256 * ng > kMaxI) return false;
    a.ncbw = ncbw;
    a.ncb = cdiv(p.C, 16 * ncbw);
    a.QC = QC;
    a.nksw = QC / 32 * ncbw / 4;
    a.RSY = SY + 1;
    a.NXS = static_cast<int>(NXS);
    a.RSX = a.NXS | 1;
    a.xcopy_slots = 16 * ncbw * a.RSX;
    a.ybuf_slots = FB * 16 * a.RSY;
    a.stage_slots = a.ybuf_slots + ncopies * a.xcopy_slots;
    // + slack for the look-ahead reads of the last k-step (4 slots behind the last row)
    size_t bytes = static_cast<size_t>(2 * a.stage_slots + 8) * 16;
    const size_t red = static_cast<size_t>(4) * FB * NT * 1024;
    if (bytes > static_cast<size_t>(kLdsBudget)) return false;
    if (red > bytes) bytes = red;
    pl.lds_bytes = bytes;
    a.CPR = cdiv(p.Q, QC);
    const long nc = static_cast<long>(p.N) * a.CPR;
    if (nc > 0x7fffffffL) return false;
    a.nchunks = static_cast<int>(nc);
    const int ncombos = a.nfg * a.ncb * a.ntg;
    int nstrips = kNumCU / ncombos;
    if (nstrips < 1) nstrips = 1;
    if (nstrips > a.nchunks) nstrips = a.nchunks;
    a.nstrips = nstrips;
    const long grid = static_cast<long>(ncombos) * nstrips;
    if (grid > 0x7fffffffL) return false;
    pl.grid = static_cast<int>(grid);
    pl.tile = ncbw * FB * NT * 256;
    return true;
}

// Estimated time of a candidate in microseconds: MFMA slots (an LDS operand read counted as half an MFMA, the pipe
// at 60 %), the bytes staged into LDS (served mostly by L2), and the partial tiles written and read once.
double blk_cost(const WgradProblem& p, const BlkPlan& pl) {
    const BlkArgs& a = pl.a;
    const double ksteps = static_cast<double>(a.nchunks) * a.QC / 32;
    const double slots = static_cast<double>(a.nfg) * pl.FB * a.ncb * a.ncbw * a.ntg * pl.NT;
    const double reads = 1.0 + 0.5 * (pl.FB + pl.NT) / (pl.FB * pl.NT);
    const int waves = pl.grid < kNumCU ? pl.grid : kNumCU;  // busy CUs
    const double mfma_us = ksteps * slots * reads * 16 / (4.0 * waves) / 2400 / 0.6;
    const int ncopies = __builtin_popcount(a.phase_mask);
    const double staged = static_cast<double>(a.nchunks) * a.nfg * a.ncb * a.ntg * (pl.FB * 16 + ncopies * 16 * a.ncbw) * a.QC * 2;
    const double stage_us = staged / 15e6;
    const double ws_us = 2.0 * pl.grid * pl.tile * 4 / 4e6;
    (void)p;
    return mfma_us + stage_us + ws_us;
}

BlkPlan blk_plan(const WgradProblem& p) {
    BlkPlan best{};
    best.ok = false;
    if (!p.bf16) return best;
    if (p.dw_sc != p.S || p.dw_sk != static_cast<long>(p.C) * p.S) return best;  // writes the whole dw tensor
    if (static_cast<long>(p.C) * p.W >= (1L << 30) || static_cast<long>(p.K) * p.Q >= (1L << 30)) return best;
    if (static_cast<long>(p.K) * p.C * p.S >= (1L << 31)) return best;
    double best_cost = 0;
    for (const Shape& sh : kShapes)
        for (int ncbw = p.C > 32 ? 4 : (p.C > 16 ? 2 : 1); ncbw >= 1; ncbw /= 2)
            for (int QC = 512; QC >= 128; QC /= 2) {
                BlkPlan pl{};
                if (!blk_geometry(p, sh.FB, sh.NT, ncbw, QC, pl)) continue;
                const double c = blk_cost(p, pl);
                if (!best.ok || c < best_cost) {
                    best = pl;
                    best.ok = true;
                    best_cost = c;
                }
                break;  // the longest chunk that fits
            }
    if (!best.ok) return best;
    BlkArgs& a = best.a;
    a.x = static_cast<const unsigned short*>(p.x);
    a.dy = static_cast<const unsigned short*>(p.dy);
    a.ws = static_cast<float*>(p.ws);
    a.C = p.C; a.K = p.K; a.W = p.W; a.Q = p.Q; a.S = p.S; a.d = p.d; a.P = p.P;
    a.x_sn = p.x_sn; a.dy_sn = p.dy_sn;
    best.fast = (p.W % 2 == 0) && (p.Q % 2 == 0) && (p.x_sn % 2 == 0) && (p.dy_sn % 2 == 0) &&
                (reinterpret_cast<uintptr_t>(p.x) % 4 == 0) && (reinterpret_cast<uintptr_t>(p.dy) % 4 == 0);
    return best;
}

template <int FB, int NT>
hipError_t blk_launch(const BlkPlan& pl, hipStream_t st) {
    auto kern = pl.fast ? blocked_wgrad_bf16_kernel<FB, NT, true> : blocked_wgrad_bf16_kernel<FB, NT, false>;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), pl.lds_bytes);
    if (e != hipSuccess) return e;
    return launch_kernel(kern, dim3(pl.grid), dim3(512), pl.lds_bytes, st, pl.a);
}

}  // namespace

bool blocked_bf16_wgrad_supported(const WgradProblem& p) { return blk_plan(p).ok; }

size_t blocked_bf16_wgrad_workspace(const WgradProblem& p) {
    const BlkPlan pl = blk_plan(p);
    return pl.ok ? static_cast<size_t>(pl.grid) * pl.tile * sizeof(float) : 0;
}

hipError_t blocked_bf16_wgrad_launch(const WgradProblem& p, hipStream_t st) {
    const BlkPlan pl = blk_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
    const int key = pl.FB * 100 + pl.NT;
    switch (key) {
        case 105: e = blk_launch<1, 5>(pl, st); break;
        case 109: e = blk_launch<1, 9>(pl, st); break;
        case 126: e = blk_launch<1, 26>(pl, st); break;
        case 209: e = blk_launch<2, 9>(pl, st); break;
        case 217: e = blk_launch<2, 17>(pl, st); break;
        case 405: e = blk_launch<4, 5>(pl, st); break;
        case 117: e = blk_launch<1, 17>(pl, st); break;
        case 409: e = blk_launch<4, 9>(pl, st); break;
        default: break;
    }
    if (e != hipSuccess) return e;
    const long nel = static_cast<long>(pl.grid / pl.a.nstrips) * pl.tile;
    return launch_kernel(blocked_wgrad_reduce_kernel, dim3(cdiv(nel, 64)), dim3(256), 0, st, static_cast<const float*>(p.ws), p.dw, pl.a, pl.FB,
                       pl.NT);
}

}  // namespace conv1d
