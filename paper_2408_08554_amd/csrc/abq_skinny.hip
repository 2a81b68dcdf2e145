// Decode-shaped matmul (M = 1 .. 64): the packed weight plane groups are streamed from HBM
// exactly once with 128-bit coalesced non-temporal loads, expanded to signed bytes in
// registers with one AND per dword, and contracted against the int8 activation codes on the
// 16x16x64 int8 MFMA.  Bit reduction (Sec. 3.4 step 5 / Appendix B: the 2^(s+t) factors)
// happens in registers: the activation side carries all q planes at once as the int8 code,
// the weight side one plane group per accumulator, recombined with shifts after the K loop.
// The dequant epilogue is fused (Fig. 3b).
//
// Work decomposition: a workgroup of S waves owns one 16-row tile of W at a time (and walks
// several tiles when the grid is smaller than the tile count).  Its waves split K in units
// of 512 (a "super-chunk": every plane group tiles 512 k-values with whole 1 KiB wave loads),
// wave w taking super-chunks w, w+S, ...  Each wave keeps a ring of D super-chunks of weight
// loads in flight, running ahead across tile boundaries, so the stream never drains between
// tiles.  The rows of A a wave needs are staged once into its own part of LDS (no barrier on
// the way to the first MFMA).  Per tile the S partial tiles are summed through LDS.
#include "abq_skinny_kernels.h"

#include <math.h>
#include <atomic>

namespace abq {

// ---- host side -------------------------------------------------------------------------------------

static std::atomic<int> g_num_cus{0};   // a cached device property (every thread would store the same value)

int num_cus()
{
    int n = g_num_cus.load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0;
        if (!(hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0))
            n = 256;
        g_num_cus.store(n, std::memory_order_relaxed);
    }
    return n;
}

// The kernels use up to 256 VGPRs, i.e. two waves per SIMD, eight per CU.
static const int kWavesPerCu = 8;
static const size_t kLdsPerCu = 160 * 1024;
static const int kMaxWalk = 64;   // most tiles one workgroup walks (their epilogue parameters live in LDS)
static const size_t kAsumBytes = 8 * 16 * sizeof(int32_t) + 512;   // per-wave partial row sums of A and 512 zero bytes, kept at the end of the parameter area

// Launch plan: S waves per workgroup (= K split of a tile) and gx workgroups walking the tiles.
// What it trades off (the analogue of the paper's tile-shape search, Appendix D "Auto Kernel
// Search", as a closed-form score instead of timed trials):
//   - waves resident per CU (LDS for the staged rows of A and the 8-wave register limit bound it),
//   - idle wave-slots in the last round over K when S does not divide the super-chunk count,
//   - idle workgroup-slots in the last round over the tiles.
struct SkinnyPlan { int waves, gx, mrows, kgroups, cap, rounds; size_t a_stride, par_bytes, red_bytes, part_bytes, lds_bytes; };

// G > 1 (K groups): only the columns of one run of super-chunks per wave are staged at a time, so up to 16
// rows of A fit whatever K is and W is streamed once; the price is a drained ring at every group boundary
// and S * rounds KiB of LDS for the partial sums.
static bool make_plan(int S, int G, int M, int Kp, int ntiles, int cus, SkinnyPlan* out, double* score)
{
    const int nsuper = Kp / kSuperK;
    if (S > nsuper) return false;
    const int nsw_min = nsuper / S, nsw_max = (nsuper + S - 1) / S;
    if (G > 1 && (S < 4 || nsw_min < G)) return false;   // every wave needs a super-chunk in every group
    const int cap = (nsw_max + G - 1) / G;
    const size_t a_stride = (G > 1 ? (size_t)S * cap * kSuperK : (size_t)Kp) + 16;
    const size_t red_bytes = 2 * (size_t)S * 1024;
    const int m16 = M < 16 ? M : 16;
    int mrows = m16;
    // the per-workgroup tile count (rounds) sizes the parameter and partial-sum areas, which bound how many
    // workgroups fit a CU, which sets rounds: iterate to the fixed point (rounds only grows)
    int rounds = 1;
    for (int pass = 0; pass < 8; ++pass) {
        const size_t par_bytes = (size_t)(16 + rounds * 16) * sizeof(RowParams) + kAsumBytes;
        const size_t part_bytes = G > 1 ? (size_t)S * rounds * 1024 : 0;
        if (red_bytes + par_bytes + part_bytes + 64 >= kLdsPerCu) return false;
        const size_t budget = kLdsPerCu - red_bytes - par_bytes - part_bytes - 64;
        if ((size_t)mrows * a_stride > budget) mrows = (int)(budget / a_stride);
        if (mrows < 1) return false;
        const size_t lds = align_up((size_t)mrows * a_stride, 16) + par_bytes + red_bytes + part_bytes;
        int per_cu = (int)(kLdsPerCu / lds);
        if (per_cu > kWavesPerCu / S) per_cu = kWavesPerCu / S;
        if (per_cu < 1) per_cu = 1;
        // M > mrows: the launch has one set of gx workgroups per group of mrows rows.  All sets together should be
        // resident at once, each workgroup walking more tiles (A staged once per workgroup, the ring running
        // across its tiles), rather than several rounds of workgroups that each stage their rows of A afresh.
        const int row_groups = (M + mrows - 1) / mrows;
        int slots = cus * per_cu / row_groups;
        if (slots < 1) slots = 1;
        int gx = ntiles < slots ? ntiles : slots;
        if ((ntiles + gx - 1) / gx > kMaxWalk) gx = (ntiles + kMaxWalk - 1) / kMaxWalk;   // (many row groups: several rounds after all)
        const int new_rounds = (ntiles + gx - 1) / gx;
        if (new_rounds > rounds) { rounds = new_rounds; continue; }
        out->waves = S; out->gx = gx; out->mrows = mrows; out->kgroups = G; out->cap = cap; out->rounds = rounds;
        out->a_stride = a_stride; out->par_bytes = par_bytes; out->red_bytes = red_bytes; out->part_bytes = part_bytes;
        out->lds_bytes = lds;
        if (lds > kLdsPerCu) return false;
        const double waves_cu = (double)per_cu * S < kWavesPerCu ? (double)per_cu * S : kWavesPerCu;
        const double occupancy = (double)gx * row_groups * S / cus < waves_cu ? (double)gx * row_groups * S / cus : waves_cu;
        const double k_eff = (double)nsuper / (nsw_max * S);
        // tiles the busiest CU works through (its workgroups, each walking `rounds` tiles) against an even spread
        const long wgs_busiest = ((long)gx * row_groups + cus - 1) / cus;
        const double t_eff = ((double)ntiles * row_groups / cus) / ((double)wgs_busiest * rounds) < 1.0
                                 ? ((double)ntiles * row_groups / cus) / ((double)wgs_busiest * rounds) : 1.0;
        const double m_eff = (double)((M + 15) / 16) / row_groups;   // passes over W against the fewest possible
        const double g_eff = 1.0 / (1.0 + 0.1 * (G - 1));
        // Staging A: one load instruction covers a row over TWO of the wave's super-chunks, so a wave with an odd
        // count wastes half an instruction per row, all of it when it owns a single super-chunk; it matters as
        // the rows grow (measured with the plan search at K = 4096: from four rows on, four waves with two
        // super-chunks each beat eight waves with one by 13-20 %; at one or two rows eight stay ahead).  For the
        // same reason half-filled CUs cost less than their share of idle wave slots (the exponent below).
        const int run = (nsw_max + G - 1) / G;
        const double stage_eff = (double)run / (2 * ((run + 1) / 2));
        const double row_weight = mrows >= 4 ? 1.0 : (mrows - 1) / 3.0;
        const double s_eff = 1.0 - row_weight * (1.0 - stage_eff);
        *score = pow(occupancy / kWavesPerCu, 0.75) * k_eff * t_eff * m_eff * g_eff * s_eff;
        return true;
    }
    return false;
}

// one_group: the kernel variant at hand has no K groups (then long K with many rows takes more passes over W).
// forced / forced_g > 0: the K split / group count to use if it fits (from the plan table or the environment).
static bool pick_plan(int M, int Kp, int ntiles, int cus, size_t stream_bytes, bool one_group, int forced, int forced_g,
                      SkinnyPlan* best)
{
    static const int candidates[] = {8, 7, 6, 5, 4, 2, 1};
    const int m16 = M < 16 ? M : 16;
    // K groups are used only where one group cannot hold all (up to 16) rows of A, and then as few as possible.
    // Long streams over many tiles (measured: >= 48 MB, >= 2 tiles per CU) run best as one resident
    // workgroup per CU that walks its tiles with 6..8 waves: the ring never drains between tiles and
    // A is staged once per workgroup.  Among 6..8 the split that wastes the fewest wave-slots over K.
    if (forced <= 0 && forced_g <= 0 && stream_bytes >= ((size_t)48 << 20) && ntiles >= 2 * cus) {
        const int nsuper = Kp / kSuperK;
        int order[3] = {8, 7, 6};
        for (int i = 0; i < 3; ++i)   // sort by wasted wave-slots, ties to the larger S
            for (int j = i + 1; j < 3; ++j) {
                const int wi = (nsuper + order[i] - 1) / order[i] * order[i] - nsuper;
                const int wj = (nsuper + order[j] - 1) / order[j] * order[j] - nsuper;
                if (wj < wi) { const int t = order[i]; order[i] = order[j]; order[j] = t; }
            }
        double sc;
        for (int G = 1; G <= (one_group ? 1 : 4); ++G)
            for (int S : order)
                if (make_plan(S, G, M, Kp, ntiles, cus, best, &sc) && best->mrows == m16) return true;
        for (int S : order)
            if (make_plan(S, 1, M, Kp, ntiles, cus, best, &sc)) return true;
    }
    auto search = [&](int g_lo, int g_hi, bool all_rows, SkinnyPlan* out) {
        double best_score = -1.0;
        bool ok = false;
        for (int G = g_lo; G <= g_hi; ++G) {
            if (forced_g > 0 && G != forced_g) continue;
            for (int S : candidates) {
                if (forced > 0 && S != forced) continue;
                SkinnyPlan pl;
                double sc;
                if (!make_plan(S, G, M, Kp, ntiles, cus, &pl, &sc)) continue;
                if (all_rows && pl.mrows != m16) continue;
                if (sc > best_score + 1e-9) { best_score = sc; *out = pl; ok = true; }
            }
        }
        return ok;
    };
    if (one_group) {
        if (search(1, 1, false, best)) return true;
    } else {
        if (forced_g > 1 && search(forced_g, forced_g, false, best)) return true;
        const bool one = search(1, 1, false, best);
        // (no K groups where they save no pass over W: all rows fit, or M > 16 needs as many passes anyway)
        if (one && (best->mrows == m16 || (M + best->mrows - 1) / best->mrows == (M + 15) / 16)) return true;
        SkinnyPlan grouped;
        if (forced_g <= 0 && search(2, 4, true, &grouped)) { *best = grouped; return true; }
        if (one) return true;
    }
    if (forced > 0 || forced_g > 0) return pick_plan(M, Kp, ntiles, cus, stream_bytes, one_group, 0, 0, best);   // does not fit: the rule
    return false;
}

static void fill_operands(SkinnyParams& prm, const GemmArgs& g, const ActLayout& A, const WeightLayout& W)
{
    for (int i = 0; i < 3; ++i) {
        prm.fields[i] = (const u4v*)(g.w_blob + W.off_fields[i]);
        prm.chunks[i] = W.chunks[i];
    }
    if (g.a_raw) {
        prm.a_codes = nullptr; prm.aparams = nullptr;
        prm.a_raw = g.a_raw; prm.a_scale = g.a_scale; prm.a_zero = g.a_zero;
    } else {
        prm.a_codes = (const int8_t*)(g.act_blob + A.off_codes);
        prm.aparams = (const RowParams*)(g.act_blob + A.off_params);
        prm.a_raw = nullptr; prm.a_scale = nullptr; prm.a_zero = nullptr;
    }
    prm.wparams = (const RowParams*)(g.w_blob + W.off_params);
    prm.gparams = W.g128 ? (const u4v*)(g.w_blob + W.off_gparams) : nullptr;
    prm.y = g.y;
    prm.acc = g.acc;
    prm.rq = g.rq;
    prm.M = g.M; prm.N = g.N; prm.K = g.K; prm.Kp = A.Kp;
    prm.oa = (g.q == 8) ? 128 : 0;
    prm.ow = (g.p == 8) ? 128 : 0;
    prm.a_mask = ((1u << g.q) - 1u) * 0x01010101u;
    prm.ntiles = W.NT;
}

hipError_t launch_gemm_skinny(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s)
{
    SkinnyParams prm;
    fill_operands(prm, g, A, W);
    const int cus = num_cus();
    const int nsuper = A.Kp / kSuperK;
    SkinnyPlan pl;
    const size_t stream_bytes = (size_t)g.p * W.NT * 16 * (size_t)A.Kp / 8;
    // override: the plan table entry of this exact problem (K split, K group count)
    PlanOverride ov;
    lookup_plan(g.p, g.q, g.M, g.N, g.K, &ov);
    const int forced = ov.skinny_waves > 0 ? ov.skinny_waves : tuning_env("ABQ_SKINNY_WAVES");
    const int forced_g = ov.skinny_kgroups > 0 ? ov.skinny_kgroups : tuning_env("ABQ_SKINNY_KGROUPS");
    if (!pick_plan(g.M, A.Kp, W.NT, cus, stream_bytes, W.g128, forced, forced_g, &pl)) return hipErrorInvalidValue;   // cannot happen for K <= ABQ_MAX_K
    const int waves = pl.waves, gx = pl.gx, mrows = pl.mrows;
    // LDS: staged rows of A (all of K, or one K group of it), the epilogue parameters, two reduction buffers
    // of 1 KiB per wave, the partial sums of the K groups
    prm.a_stride = (int)pl.a_stride;
    prm.mrows = mrows;
    prm.par_off = (int)align_up((size_t)mrows * pl.a_stride, 16);
    prm.red_off = prm.par_off + (int)pl.par_bytes;
    prm.asum_off = prm.red_off - (int)kAsumBytes;
    prm.zero_off = prm.red_off - 512;
    prm.part_off = prm.red_off + (int)pl.red_bytes;
    prm.kgroups = pl.kgroups;
    prm.col_w = pl.kgroups > 1 ? pl.cap * kSuperK : kSuperK;
    prm.col_s = pl.kgroups > 1 ? kSuperK : waves * kSuperK;
    prm.nmy_max = pl.rounds;
    const size_t lds_bytes = pl.lds_bytes;
    prm.nsuper = nsuper;
    prm.sc_q = nsuper / waves; prm.sc_r = nsuper % waves;
    prm.tl_q = W.NT / gx; prm.tl_r = W.NT % gx;
    dim3 grid((unsigned)gx, (unsigned)((g.M + mrows - 1) / mrows));
    // the kernels live in one translation unit per pair of weight widths
    if (g.p <= 2) return skinny_launch_p12(g.p, prm, grid, waves, lds_bytes, s);
    if (g.p <= 4) return skinny_launch_p34(g.p, prm, grid, waves, lds_bytes, s);
    if (g.p <= 6) return skinny_launch_p56(g.p, prm, grid, waves, lds_bytes, s);
    return skinny_launch_p78(g.p, prm, grid, waves, lds_bytes, s);
}

// ---- grouped launch ----------------------------------------------------------------------------

// One launch serves a group when every problem can run as "one workgroup of S waves per tile, all of
// A staged at once": M <= 16, every K spans at least four super-chunks (S = 4..8 waves, the same for
// all), the rows of A fit LDS, field-packed weights, and for unpacked codes K a multiple of 16.
// Shape of a grouped launch, measured on the seven layer shapes of a LLaMA-7B block (W1/W2/W4/W8, M = 1, 4, 8):
// few rows of A -> small workgroups (two waves for M <= 2, four for M <= 4) and four of them per CU, so that
// the prologue and tail of one run hide behind the streams of the others; more rows -> eight waves, one
// workgroup per CU, so that the rows of A are staged as seldom as possible.  A run never exceeds kMaxRun tiles
// (the epilogue parameters of a run live in LDS).
constexpr int kMaxRun = 64;
static int group_waves(int M) { return M <= 2 ? 2 : (M <= 4 ? 4 : 8); }
static int group_workgroups(int tiles, int M, int cus)
{
    const int forced = tuning_env("ABQ_GROUP_WGS");
    int gx = forced > 0 ? forced : (M <= 4 ? 4 * cus : cus);
    if (gx > tiles) gx = tiles;
    if ((tiles + gx - 1) / gx > kMaxRun) gx = (tiles + kMaxRun - 1) / kMaxRun;
    return gx;
}

static size_t group_par_bytes(int run_max) { return (size_t)(16 + 16 * run_max) * sizeof(RowParams) + kAsumBytes; }

// Fills the tile list and the work-balanced partition of problems first .. first+n-1 and picks the workgroup
// count; returns the most tiles any workgroup's run holds.
static int group_partition(GroupedParams& gp, int first, int n, int M, const ActLayout* A, const WeightLayout* W, int cus, int* wgs_out)
{
    gp.count = n;
    int tiles = 0;
    double cost = 0;
    // Measured on the LLaMA-7B block (same box, A/B): with many small workgroups per CU (M <= 4) equal tile
    // counts, the longer runs first, beat every equal-work cut by 3-8 %; with one eight-wave workgroup per CU
    // (M > 4) equal work (super-chunks + a fixed cost of 16 per tile) is 10 % faster than equal counts.
    const int overhead = tuning_env("ABQ_GROUP_TILE_COST");   // > 0 forces the equal-work cut with that fixed cost
    gp.by_work = (overhead > 0 || M > 4) ? 1 : 0;
    for (int i = 0; i < kMaxGroup; ++i) {
        const int src = first + (i < n ? i : 0);
        const int tile_cost = A[src].Kp / kSuperK + (overhead > 0 ? overhead : kTileOverheadCost);
        gp.first_tile[i] = tiles;
        gp.cost_first[i] = (float)cost;
        gp.inv_tile_cost[i] = 1.0f / (float)tile_cost;
        if (i < n) { tiles += W[src].NT; cost += (double)W[src].NT * tile_cost; }
    }
    gp.first_tile[kMaxGroup] = tiles;
    gp.cost_first[kMaxGroup] = (float)cost;
    int wgs = group_workgroups(tiles, M, cus);
    for (;;) {
        gp.cost_per_wg = (float)(cost / wgs);
        gp.run_q = tiles / wgs; gp.run_r = tiles % wgs;
        int run_max = 0, prev = grouped_run_start(gp, 0, wgs);
        for (int b = 1; b <= wgs; ++b) {
            const int next = grouped_run_start(gp, b, wgs);
            if (next - prev > run_max) run_max = next - prev;
            prev = next;
        }
        if (run_max <= kMaxRun || wgs >= tiles) { *wgs_out = wgs; return run_max + 1; }   // (+1: margin for the parameter area)
        wgs = wgs * 2 < tiles ? wgs * 2 : tiles;
    }
}

// One launch serves a group when every problem can run as "S waves per tile, all of A staged at once":
// M <= 16, every K spans at least four super-chunks (and at least S of them: S is the same for all), the
// rows of A fit LDS, field-packed weights, and for unpacked codes K a multiple of 16.
bool gemm_grouped_fits(int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W, int* waves, size_t* lds_bytes)
{
    if (M > 16 || count < 1) return false;
    const int forced = tuning_env("ABQ_GROUP_WAVES");
    int S = forced >= 2 && forced <= 8 && forced != 3 ? forced : group_waves(M);
    for (int i = 0; i < count; ++i) {
        if (!W[i].has_fields) return false;
        if (probs[i].a_raw ? (probs[i].K % 16 != 0) : !A[i].has_fields) return false;
        if ((probs[i].a_raw != nullptr) != (probs[0].a_raw != nullptr)) return false;
        const int nsuper = A[i].Kp / kSuperK;
        if (nsuper < 4) return false;
        if (nsuper < S) S = nsuper;
    }
    const int cus = num_cus();
    size_t lds = 0;
    for (int first = 0; first < count; first += kMaxGroup) {
        const int n = count - first < kMaxGroup ? count - first : kMaxGroup;
        GroupedParams gp;
        int gx = 0;
        const int run_max = group_partition(gp, first, n, M, A, W, cus, &gx);
        if (run_max > kMaxRun + 1) return false;
        for (int i = first; i < first + n; ++i) {
            const size_t need = align_up((size_t)M * ((size_t)A[i].Kp + 16), 16) + group_par_bytes(run_max) + 2 * (size_t)S * 1024;
            if (need > kLdsPerCu) return false;
            if (need > lds) lds = need;
        }
    }
    *waves = S;
    *lds_bytes = lds;
    return true;
}

hipError_t launch_gemm_grouped(int p, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W,
                               int waves, size_t lds_bytes, hipStream_t s)
{
    for (int first = 0; first < count; first += kMaxGroup) {
        const int n = count - first < kMaxGroup ? count - first : kMaxGroup;
        GroupedParams gp;
        int wgs = 0;
        const int run_max = group_partition(gp, first, n, M, A, W, num_cus(), &wgs);
        for (int i = 0; i < kMaxGroup; ++i) {
            const int src = first + (i < n ? i : 0);   // unused slots repeat a valid descriptor
            SkinnyParams& prm = gp.d[i];
            fill_operands(prm, probs[src], A[src], W[src]);
            const int nsuper = A[src].Kp / kSuperK;
            prm.a_stride = A[src].Kp + 16;
            prm.mrows = M;
            prm.par_off = (int)align_up((size_t)M * prm.a_stride, 16);
            prm.red_off = prm.par_off + (int)group_par_bytes(run_max);
            prm.asum_off = prm.red_off - (int)kAsumBytes;
            prm.zero_off = prm.red_off - 512;
            prm.part_off = prm.red_off + 2 * waves * 1024;
            prm.kgroups = 1;
            prm.col_w = kSuperK;
            prm.col_s = waves * kSuperK;
            prm.nmy_max = run_max;
            prm.nsuper = nsuper;
            prm.sc_q = nsuper / waves; prm.sc_r = nsuper % waves;
            prm.tl_q = 0; prm.tl_r = 0;   // (not used: the kernel hands each workgroup its run)
        }
        hipError_t e;
        const bool raw = probs[first].a_raw != nullptr;
        if (p <= 2) e = grouped_launch_p12(p, gp, raw, (unsigned)wgs, waves, lds_bytes, s);
        else if (p <= 4) e = grouped_launch_p34(p, gp, raw, (unsigned)wgs, waves, lds_bytes, s);
        else if (p <= 6) e = grouped_launch_p56(p, gp, raw, (unsigned)wgs, waves, lds_bytes, s);
        else e = grouped_launch_p78(p, gp, raw, (unsigned)wgs, waves, lds_bytes, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace abq
