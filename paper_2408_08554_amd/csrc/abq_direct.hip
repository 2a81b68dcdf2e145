// Host side of the direct decode kernel (abq_direct_kernels.h): which problems it takes, the launch plan
// (operand rows per slice set, super-chunks per wave, waves per workgroup), single and grouped launches.
#include "abq_direct_kernels.h"

#include <vector>

namespace abq {

static int next_pow2(int v) { int p = 1; while (p < v) p <<= 1; return p; }

// Launch plan of one problem: MR operand rows per slice set, R super-chunks per wave, S waves per workgroup.
// R is the smallest of 1, 2, 4 that keeps the workgroup within 16 waves and has a kernel variant (direct_has).
// Narrow weights (p <= 2) over ten or more super-chunks take two per wave (measured on 5120 -> 13824: a 2 KiB item
// per wave leaves the reduction across waves too large a share), and over more than 24 super-chunks the variants
// with four per wave are ahead of two (K = 13824, M = 1: W2A8 6.5 vs 7.3 us, W4A8 9.2 vs 9.9; W4A8 M = 4: 11.0 vs 11.6;
// W1A8 M = 4: 7.2 vs 8.1; but W2A8 M = 4: 8.3 vs 8.0, which keeps two).  forced_r > 0 (plan table) replaces the rule where it fits.
bool direct_plan(int p, int M, int nsuper, int forced_r, DirectPlan* out)
{
    if (M < 1 || M > 16 || nsuper < 1) return false;
    const int MR = next_pow2(M) > direct_min_rows(p) ? next_pow2(M) : direct_min_rows(p);
    auto has = [&](int R) { return direct_has(p, MR, R); };
    auto fits = [&](int R) { return has(R) && (nsuper + R - 1) / R <= 16; };
    int R = 0;
    if (forced_r > 0 && fits(forced_r)) R = forced_r;
    if (R == 0) {
        for (int cand : {1, 2, 4})
            if (fits(cand)) { R = cand; break; }
        if (R == 1 && p <= 2 && nsuper >= 10 && fits(2)) R = 2;
        if (R == 2 && nsuper > 24 && fits(4) && (M == 1 || p == 4 || p == 1)) R = 4;
    }
    if (R == 0) return false;
    out->MR = MR; out->R = R; out->S = (nsuper + R - 1) / R;
    return true;
}

static void fill_problem(DirectProblem& d, const GemmArgs& g, const ActLayout& A, const WeightLayout& W, int rsplit)
{
    for (int i = 0; i < 3; ++i) d.fields[i] = (const u4v*)(g.w_blob + W.off_fields[i]);
    if (g.a_raw) {
        d.a_codes = nullptr; d.aparams = nullptr;
        d.a_raw = g.a_raw; d.a_scale = g.a_scale; d.a_zero = g.a_zero;
    } else {
        d.a_codes = (const int8_t*)(g.act_blob + A.off_codes);
        d.aparams = (const RowParams*)(g.act_blob + A.off_params);
        d.a_raw = nullptr; d.a_scale = nullptr; d.a_zero = nullptr;
    }
    d.wparams = (const RowParams*)(g.w_blob + W.off_params);
    d.gparams = W.g128 ? (const u4v*)(g.w_blob + W.off_gparams) : nullptr;
    d.y = g.y; d.acc = g.acc; d.rq = g.rq;
    d.N = g.N; d.K = g.K; d.Kp = A.Kp; d.nsuper = A.Kp / kSuperK;
    d.rsplit = rsplit;
}

static hipError_t launch_p(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    if (p <= 2) return direct_launch_p12(p, gp, MR, R, raw, grid, waves, s);
    if (p <= 4) return direct_launch_p34(p, gp, MR, R, raw, grid, waves, s);
    if (p <= 6) return direct_launch_p56(p, gp, MR, R, raw, grid, waves, s);
    return direct_launch_p78(p, gp, MR, R, raw, grid, waves, s);
}

hipError_t launch_gemm_direct(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, const DirectPlan& pl, hipStream_t s)
{
    DirectParams gp;
    gp.count = 1;
    for (int i = 0; i <= kDirectMaxGroup; ++i) gp.first_tile[i] = i == 0 ? 0 : W.NT;
    gp.M = g.M;
    gp.oa = g.q == 8 ? 128 : 0;
    gp.ow = g.p == 8 ? 128 : 0;
    gp.a_mask = ((1u << g.q) - 1u) * 0x01010101u;
    for (int i = 0; i < kDirectMaxGroup; ++i) fill_problem(gp.d[i], g, A, W, pl.R);   // unused slots repeat a valid descriptor
    return launch_p(g.p, gp, pl.MR, pl.R, g.a_raw != nullptr, (unsigned)W.NT, pl.S, s);
}

// A group runs as direct launches when every problem has a plan.
bool gemm_direct_grouped_fits(int p, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W)
{
    if (count < 1) return false;
    for (int i = 0; i < count; ++i) {
        DirectPlan pl;
        if (!W[i].has_fields || W[i].g128) return false;
        if (probs[i].a_raw ? (probs[i].K % 16 != 0) : !A[i].has_fields) return false;
        if ((probs[i].a_raw != nullptr) != (probs[0].a_raw != nullptr)) return false;
        if (!direct_plan(p, M, A[i].Kp / kSuperK, 0, &pl)) return false;
    }
    return true;
}

// Plan for per-group (g128) blobs, one row of A: one super-chunk per wave where sixteen waves cover K, else two (the
// widths with a single plane group only).
bool direct_plan_g128(int p, int nsuper, DirectPlan* out)
{
    for (int R : {1, 2})
        if (direct_has_gq(p, 1, R) && direct_plan(p, 1, nsuper, R, out) && out->R == R) return true;
    return false;
}

// Per-group (g128) blobs: the direct kernel's variant takes one row of A, p <= 4 and at most 16 super-chunks of K
// (32 for p = 1, 2, 4).
bool gemm_direct_g128_fits(int p, int M, const GemmArgs& g, const ActLayout& A, const WeightLayout& W)
{
    DirectPlan pl;
    if (!W.g128 || !W.has_fields || M != 1 || p > 4 || g.acc || g.rq.codes) return false;
    if (g.a_raw ? (g.K % 16 != 0) : !A.has_fields) return false;
    return direct_plan_g128(p, A.Kp / kSuperK, &pl);
}

hipError_t launch_gemm_direct_grouped(int p, int q, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W, hipStream_t s)
{
    // Problems with the same plan (super-chunks per wave, waves per workgroup) share a launch, eight at most: one
    // workgroup size fits them all, so no wave idles.  A decoder block's layers have two lengths of K, hence two launches.
    std::vector<DirectPlan> plans(count);
    std::vector<char> done(count, 0);
    for (int i = 0; i < count; ++i)
        if (!(W[i].g128 ? direct_plan_g128(p, A[i].Kp / kSuperK, &plans[i]) : direct_plan(p, M, A[i].Kp / kSuperK, 0, &plans[i])))
            return hipErrorInvalidValue;   // (callers check the fits functions)
    for (int lead = 0; lead < count; ++lead) {
        if (done[lead]) continue;
        const DirectPlan pl = plans[lead];
        DirectParams gp;
        gp.M = M;
        gp.oa = q == 8 ? 128 : 0;
        gp.ow = p == 8 ? 128 : 0;
        gp.a_mask = ((1u << q) - 1u) * 0x01010101u;
        int n = 0, tiles = 0;
        for (int i = lead; i < count && n < kDirectMaxGroup; ++i) {
            if (done[i] || plans[i].R != pl.R || plans[i].S != pl.S) continue;
            done[i] = 1;
            fill_problem(gp.d[n], probs[i], A[i], W[i], pl.R);
            gp.first_tile[n] = tiles;
            tiles += W[i].NT;
            ++n;
        }
        gp.count = n;
        for (int i = n; i < kDirectMaxGroup; ++i) { gp.d[i] = gp.d[0]; gp.first_tile[i] = tiles; }   // unused slots start at the end of the grid
        gp.first_tile[kDirectMaxGroup] = tiles;
        const hipError_t e = launch_p(p, gp, pl.MR, pl.R, probs[lead].a_raw != nullptr, (unsigned)tiles, pl.S, s);
        if (e != hipSuccess) return e;
        if (n == kDirectMaxGroup) --lead;   // more problems of this plan may be left: look again from the same place
    }
    return hipSuccess;
}

}  // namespace abq
