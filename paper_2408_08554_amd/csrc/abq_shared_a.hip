// Host side of the shared-operand decode kernel: launch plan and launch.
#include "abq_shared_a_kernels.h"

namespace abq {

// Plan: one workgroup of sixteen waves per compute unit (the copy of A takes most of a unit's LDS, and the weight stream
// needs every unit pulling), the tiles dealt out evenly, so a workgroup's run is T or T - 1 tiles with T = ceil(NT / units);
// its waves split into 16 / run waves per tile, each with ceil(nsuper / that) super-chunks of K.  Where A is larger than
// LDS, K is cut in two phases whose halves of A take turns there.  False where the kernel does not fit: no more tiles
// than units (the direct kernel's case), a phase of A larger than LDS or more loads per lane than a wave holds, a run
// of weights that the registers do not hold.  forced: two tiles per workgroup at least, for problems of few tiles.
bool shared_a_plan(int p, int M, int NT, int Kp, bool raw, int K, bool forced, SharedAPlan* out)
{
    if (M < 1 || M > 16 || NT < 1 || Kp < kSuperK || (raw && K % 16 != 0)) return false;
    const int cus = num_cus(), nsuper = Kp / kSuperK, S = 16;
    int nwg = NT < cus ? NT : cus;
    if (forced && NT < 2 * cus) nwg = (NT + 1) / 2;   // (a plan-table entry asks for this kernel on a problem of few tiles)
    const int T = (NT + nwg - 1) / nwg;
    if (T < 2 || T > 8) return false;
    const int wpt = S / T;
    for (int phases = 1; phases <= 2; ++phases) {
        const int H = (nsuper + phases - 1) / phases;            // super-chunks per phase
        if (phases == 2 && nsuper < 2) break;
        const int R = (H + wpt - 1) / wpt;
        const int quads = (8 * H + S - 1) / S;
        if (R > shared_a_max_r(p, phases)) continue;
        if (quads > (phases == 1 ? kSharedAMaxQuads : kSharedAMaxQuads2)) continue;
        if (shared_a_lds_bytes(H, S) > (size_t)160 * 1024) continue;
        out->nwg = nwg; out->S = S; out->R = R; out->phases = phases; out->H = H;
        return true;
    }
    return false;
}

hipError_t launch_gemm_shared_a(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, const SharedAPlan& pl, hipStream_t s)
{
    SharedAParams gp;
    DirectProblem& d = gp.d;
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
    d.gparams = nullptr;
    d.y = g.y; d.acc = g.acc; d.rq = g.rq;
    d.N = g.N; d.K = g.K; d.Kp = A.Kp; d.nsuper = A.Kp / kSuperK;
    d.rsplit = 0;
    gp.M = g.M;
    gp.oa = g.q == 8 ? 128 : 0;
    gp.ow = g.p == 8 ? 128 : 0;
    gp.a_mask = ((1u << g.q) - 1u) * 0x01010101u;
    // runs of T and T - 1 tiles, and per kind of run the split of the sixteen waves
    gp.H = pl.H;
    gp.T = (W.NT + pl.nwg - 1) / pl.nwg;
    gp.nbig = W.NT - pl.nwg * (gp.T - 1);   // (nwg when the tiles divide evenly)
    for (int kind = 0; kind < 2; ++kind) {
        const int cnt = gp.T - kind > 0 ? gp.T - kind : 1;
        const int wpt = pl.S / cnt;
        gp.wpt[kind] = wpt;
        gp.rsplit[kind] = (pl.H + wpt - 1) / wpt;
        gp.inv[kind] = (256 + wpt - 1) / wpt;   // (wave * inv) >> 8 == wave / wpt for wave < 16, wpt <= 16
        for (int wv = 0; wv < 16; ++wv)
            if (((wv * gp.inv[kind]) >> 8) != wv / wpt) return hipErrorInvalidValue;
    }
    const unsigned grid = (unsigned)pl.nwg;
    const int waves = pl.S;
    return g.p <= 4 ? shared_a_launch_p1234(g.p, gp, pl.phases, pl.R, g.a_raw != nullptr, grid, waves, s)
                    : shared_a_launch_p5678(g.p, gp, pl.phases, pl.R, g.a_raw != nullptr, grid, waves, s);
}

}  // namespace abq
