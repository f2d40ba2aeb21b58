// Forward / backward-data, bfloat16, many channels, dilations 1, 2, 4, 8, 16: launch plan and dispatch of the
// resident-weight kernels (the kernel template and its description are in the header; every dilation is
// instantiated in a translation unit of its own).
#include "conv1d_igemm_ring_bf16.h"

namespace conv1d {

namespace {

using rg::RgArgs;
using rg::RgPlan;
using rg::kLdsBudget;
using rg::kNumCU;
using rg::kMaxWT;
using rg::kMaxWI;
using rg::kMaxRP;
using rg::kQS;

RgPlan rg_plan_kt(const CorrProblem& p, int kT) {
    const int kTW = 64 * kT;
    RgPlan pl{};
    pl.ok = false;
    if (!p.bf16 || p.accumulate) return pl;
    if (p.R <= 16 && p.M <= 16) return pl;
    if (p.d != 1 && p.d != 2 && p.d != 4 && p.d != 8 && p.d != 16) return pl;
    if (p.S < 5 || p.S > 52) return pl;
    if ((p.Win & 1) || (p.in_sn & 1) || (reinterpret_cast<uintptr_t>(p.in) & 3) || p.Win < 2) return pl;
    if (reinterpret_cast<uintptr_t>(p.wt) & 3) return pl;
    const bool fwd_mode = p.w_ss == 1 && p.w_sr == p.S && p.w_s0 == 0;
    const bool bwd_mode = p.w_ss == -1 && p.w_sm == p.S && p.w_s0 == p.S - 1;
    if (!fwd_mode && !bwd_mode) return pl;
    if (static_cast<long>(p.R) * p.Win >= (1L << 30)) return pl;
    if (static_cast<long>(p.M) * p.R * p.S >= (1L << 31) || p.M * p.w_sm >= (1L << 31) || p.R * p.w_sr >= (1L << 31)) return pl;
    const int JT = p.S <= 8 ? 2 : (p.S <= 12 ? 3 : (p.S <= 20 ? 5 : (p.S <= 36 ? 9 : 13)));
    RgArgs& a = pl.a;
    a.in = static_cast<const unsigned short*>(p.in);
    a.wt = static_cast<const unsigned short*>(p.wt);
    a.out = p.out;
    a.epi = p.epi;
    a.N = p.N; a.R = p.R; a.M = p.M; a.Win = p.Win; a.Wout = p.Wout; a.S = p.S; a.P = p.P;
    a.w_sm = p.w_sm; a.w_sr = p.w_sr; a.in_sn = p.in_sn; a.out_sn = p.out_sn;
    a.delta = (p.P & 1) ? 1 : 0;
    const long halo = static_cast<long>(4 * JT - 1) * p.d;  // padded taps read (and multiply by zero) real positions
    const long LP = (kTW + halo + a.delta + 1) / 2 * 2;
    const long LPS = LP + 8;
    const int planes = cdiv(p.R, 8);
    // Four filter blocks per workgroup with few taps: the window of a tile is then staged once for 64 filters, and
    // staging, not the MFMAs, is what a stage with few taps waits for.
    for (int FB = (p.M > 32 && JT <= 3 && kT == 5) ? 4 : (p.M > 16 ? 2 : 1); FB >= 1; FB /= 2) {
        // one filter block per workgroup pays off only with many taps per input operand (measured: C = K = 256,
        // S = 9 ran 1.4 times slower than the staged kernel with its two filter blocks)
        if (FB == 1 && p.M > 16 && JT < 5) break;
        for (int NG = 8; NG >= 1; NG /= 2) {
            if (NG > 1 && NG / 2 >= planes) continue;
            const int ncc = cdiv(planes, NG);
            const long wres = static_cast<long>(ncc) * NG * JT * FB * kQS;
            const long win = NG * LPS;
            if (cdiv(NG * (LP / 2), 256) > kMaxWT) continue;
            // the prologue gathers the weights in chunks of NGW planes: as many as its per-thread task lists hold
            // (all planes at once where the lists and the LDS allow it: every chunk costs a barrier and a round
            // trip through LDS).  The two raw buffers of the prologue lie where the two window buffers will be.
            int NGW = 0, NU = 0;
            long NPc = 0;
            size_t bytes = 0;
            // few weights: the direct prologue (no raw buffers)
            const long NE = static_cast<long>(FB) * 16 * ncc * NG * p.S;
            const bool direct = NE <= 512L * rg::kMaxDE && static_cast<size_t>(wres + 2 * win) * 16 <= static_cast<size_t>(kLdsBudget);
            if (direct) {
                NGW = NG; NU = 1; NPc = 1; bytes = static_cast<size_t>(wres + 2 * win) * 16;
            }
            for (int w = ncc * NG; w >= 1 && NGW == 0; --w) {
                if ((ncc * NG) % w != 0) continue;  // whole chunks
                if (cdiv(static_cast<long>(FB) * 16 * w * p.S, 512) > kMaxWI) continue;
                const int nu = fwd_mode ? FB * 16 : 8 * w;
                const long L = fwd_mode ? 8L * w * p.S : static_cast<long>(FB) * 16 * p.S;
                const long npc = (2 * L + 2 + 15) / 16;
                if (cdiv(nu * npc, 512) > kMaxRP) continue;
                const long behind = 2 * win > 2 * nu * npc ? 2 * win : 2 * nu * npc;
                const size_t need = static_cast<size_t>(wres + behind) * 16;
                if (need > static_cast<size_t>(kLdsBudget)) continue;
                NGW = w; NU = nu; NPc = npc; bytes = need;
            }
            if (NGW == 0) continue;
            pl.D = p.d; pl.FB = FB; pl.JT = JT; pl.KT = kT;
            a.NG = NG;
            a.NGW = NGW;
            a.ncc = ncc;
            a.LP = static_cast<int>(LP);
            a.LPS = static_cast<int>(LPS);
            a.win_slots = static_cast<int>(win);
            a.wres_slots = static_cast<int>(wres);
            a.fwd_mode = fwd_mode;
            a.direct = direct ? 1 : 0;
            a.NU = NU;
            a.NPc = static_cast<int>(NPc);
            a.raw_slots = static_cast<int>(NU * NPc);
            a.su = fwd_mode ? p.w_sm : p.w_sr;
            a.wbytes = (fwd_mode ? static_cast<long>(p.M) * p.w_sm : static_cast<long>(p.R) * p.w_sr) * 2;
            a.vec_out = (p.Wout % 4 == 0) && (p.out_sn % 4 == 0) && (reinterpret_cast<uintptr_t>(p.out) % 16 == 0);
            a.tiles_per_row = cdiv(p.Wout, kTW);
            a.nfg = cdiv(p.M, FB * 16);
            const long nct = static_cast<long>(p.N) * a.tiles_per_row;
            if (nct > 0x7fffffffL / 64 || a.nfg > 65535) return pl;
            a.nct = static_cast<int>(nct);
            const int fit = kNumCU / a.nfg > 0 ? kNumCU / a.nfg : 1;  // teams that run at the same time
            a.nteams = a.nct < fit ? a.nct : fit;
            a.t_base = a.nct / a.nteams;
            a.t_rem = a.nct % a.nteams;
            {
                // the divisions of the kernel, and the largest number each of them divides
                const long max_stages = static_cast<long>(a.t_base + 1) * ncc;
                const long NWI = static_cast<long>(FB) * 16 * NGW * p.S;
                bool ok = make_fastdiv(a.dv_nfg, a.nfg, static_cast<long>(a.nteams) * a.nfg);
                ok = make_fastdiv(a.dv_tpr, a.tiles_per_row, nct) && ok;
                ok = make_fastdiv(a.dv_ncc, ncc, max_stages + 4) && ok;
                ok = make_fastdiv(a.dv_lp2, LP / 2, 256L * kMaxWT + static_cast<long>(NG) * (LP / 2)) && ok;
                ok = make_fastdiv(a.dv_npc, NPc, 512L * kMaxRP + NU * NPc) && ok;
                ok = make_fastdiv(a.dv_s, p.S, 512L * kMaxWI + NWI) && ok;
                ok = make_fastdiv(a.dv_ngw, NGW, (512L * kMaxWI + NWI) / p.S + 1) && ok;
                ok = make_fastdiv(a.dv_pl, ncc * NG, (512L * rg::kMaxDE + NE) / p.S + 1) && ok;
                ok = make_fastdiv(a.dv_s, p.S, 512L * (kMaxWI > rg::kMaxDE ? kMaxWI : rg::kMaxDE) + NWI + NE) && ok;
                if (!ok) return pl;
            }
            pl.grid = a.nteams * a.nfg;
            pl.lds_bytes = bytes;
            pl.ok = true;
            return pl;
        }
    }
    return pl;
}

// Tile width: 8 position blocks per wave, or 5 when that spreads the tiles more evenly over the workgroups (a
// workgroup walks whole tiles; 2.5 tiles per workgroup cost as much as 3), or when only the narrow tile leaves
// room for four filter blocks.
RgPlan rg_plan(const CorrProblem& p) {
    RgPlan best = rg_plan_kt(p, 8);
    if (best.ok) {
        const RgPlan alt = rg_plan_kt(p, 5);
        auto makespan = [](const RgPlan& pl) { return static_cast<long>(cdiv(pl.a.nct, pl.a.nteams)) * (2 * pl.KT + 1); };
        if (alt.ok && (alt.FB > best.FB || (alt.FB == best.FB && makespan(alt) * 10 < makespan(best) * 9))) best = alt;
    }
    return best;
}

}  // namespace

bool igemm_ring_bf16_corr_supported(const CorrProblem& p) { return rg_plan(p).ok; }

hipError_t igemm_ring_bf16_corr_launch(const CorrProblem& p, hipStream_t st) {
    const RgPlan pl = rg_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    switch (pl.D) {
        case 1: return rg::launch_d1(pl, st);
        case 2: return rg::launch_d2(pl, st);
        case 4: return rg::launch_d4(pl, st);
        case 8: return rg::launch_d8(pl, st);
        case 16: return rg::launch_d16(pl, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace conv1d
