// Device code of the direct decode kernel and the templates that launch its variants.  Included by the host-side
// translation unit (abq_direct.hip) for the argument structures and by one translation unit per pair of weight
// widths (abq_direct_p12.hip ...), which hold the kernel instantiations, so that they compile in parallel.
//
// Decode-shaped matmul for few rows of A (M = 1 .. 16, built for M = 1 .. 8): the GEMV of Sec. 3.4 ("GEMV
// elimination" / Table 4: a decode step is bound by the weight stream).  Nothing but the packed weights moves in
// volume: they go HBM -> registers with 128-bit non-temporal loads, all of a wave's loads issued before its first
// multiply, and the activation operand is loaded straight into the MFMA's register layout — no LDS staging, no
// load ring, no loop.
//
// The A operand of the 16x16x64 int8 MFMA holds 16 rows.  With MR = 1, 2, 4, 8 or 16 rows of A in use (M <= MR)
// the operand rows are filled with SL = 16/MR different 64-k slices of those rows (at most four for p >= 5, whose
// wider streams leave fewer registers for the accumulators that every slice of a set needs): operand row i*MR + m
// is row m of A over slice i of a set of SL consecutive slices, so one 16-byte load per lane serves SL slices.  An MFMA of that operand against the weights of slice i yields the
// wanted products in rows i*MR .. i*MR+MR-1 of the accumulator and unrelated ones elsewhere; slices with the same
// i (and, for field-packed weights, the same field position) share an accumulator, and after the last MFMA the
// rows that belong to each accumulator are picked out (one select chain per lane) and summed.  Bit reduction
// (Sec. 3.4 step 5 / Appendix B) happens in registers as in the streaming kernel: the activation side carries all q
// planes as the int8 code, the weight side one plane group per accumulator set, recombined with shifts.
//
// Work decomposition: one workgroup per 16-channel tile of W; its S waves split K in runs of super-chunks (512 k).
// The S partial tiles meet in LDS (one barrier) and 16*M threads apply the fused dequant epilogue (Fig. 3b).
// A grouped launch is the same grid over the tiles of several problems.
#pragma once
#include "abq_internal.h"
#include "../../include/abq.h"

#include <hip/hip_fp16.h>

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

constexpr int kDirectMaxGroup = 8;

struct DirectProblem {
    const u4v* fields[3];      // per plane group
    const int8_t* a_codes;     // [M][Kp] packed activations (code less oa), or null with a_raw
    const RowParams* aparams;
    const uint8_t* a_raw;      // [M][K] unpacked codes with a_scale / a_zero (activation pack fused in), K a multiple of 16
    const float* a_scale;
    const int32_t* a_zero;
    const RowParams* wparams;
    uint16_t* y;               // may be null when rq.codes is given
    int32_t* acc;              // may be null
    Requant rq;                // output codes of the next layer (codes == null: off)
    int N, K, Kp, nsuper;
    int rsplit;                // super-chunks per wave (<= R): wave w owns [w*rsplit, w*rsplit + rsplit) clipped to nsuper
    const u4v* gparams;        // per-group weight parameters (g128 blobs; null otherwise): [tiles][nsuper][16 channels] records
};

struct DirectParams {
    int count;                              // problems in this launch
    int first_tile[kDirectMaxGroup + 1];    // where each problem's tiles start in the grid
    int M, oa, ow;
    uint32_t a_mask;                        // (2^q - 1) in every byte (unpacked codes are masked to q bits)
    DirectProblem d[kDirectMaxGroup];
};

constexpr int dmax(int a, int b) { return a > b ? a : b; }
constexpr int dmin(int a, int b) { return a < b ? a : b; }

// Fewest operand rows per slice set for weight width p: every width takes a single row.
__host__ __device__ constexpr int direct_min_rows(int) { return 1; }
// Which (weight width, operand rows, super-chunks per wave) variants exist: those the kernel's 128 registers hold
// without spilling (the kernel runs up to sixteen waves per workgroup).  Two super-chunks per wave spill at p = 7 and,
// with sixteen operand rows, at every width that has two plane groups or eight bits; four fit only single-group widths
// up to four bits with at most four operand rows.  (A spilling variant is 2x slower: measured at p = 3, R = 4.)
__host__ __device__ constexpr bool direct_has(int p, int MR, int R)
{
    const bool narrow_single_group = p == 1 || p == 2 || p == 4;
    return R == 1 || (R == 2 && p != 7 && (MR < 16 || narrow_single_group)) || (R == 4 && narrow_single_group && MR <= 4);
}

// Variants for per-group (g128) weight parameters: one row of A; one super-chunk per wave for p <= 4, two for the
// single-group widths (sixteen slices, sixteen accumulators: two plane groups would need thirty-two).
__host__ __device__ constexpr bool direct_has_gq(int p, int MR, int R)
{
    return MR == 1 && ((R == 1 && p <= 4) || (R == 2 && (p == 1 || p == 2 || p == 4)));
}

// Field t of a b-bit group as a signed-byte MFMA operand dword, and the shift that undoes its scale (as in the
// streaming kernel: the field that would touch the byte's sign bit is taken one bit lower, or as weight -128).
template <int B, int T>
__device__ __forceinline__ uint32_t dfield_bytes(uint32_t x)
{
    if constexpr (B == 8) return x;
    else if constexpr (B == 4) return T == 0 ? (x & 0x0F0F0F0Fu) : ((x >> 1) & 0x78787878u);
    else if constexpr (B == 2) return T == 3 ? ((x >> 1) & 0x60606060u) : (x & (0x03030303u << (2 * T)));
    else return x & (0x01010101u << T);
}
template <int B, int T>
__device__ __forceinline__ int32_t dfield_unscale(int32_t acc)
{
    if constexpr (B == 8) return acc;
    else if constexpr (B == 4) return T == 0 ? acc : (acc >> 3);
    else if constexpr (B == 2) return T == 3 ? (acc >> 5) : (acc >> (2 * T));
    else return T == 7 ? -(acc >> 7) : (acc >> T);
}
template <int B, int T>
__device__ __forceinline__ v4i dfield_operand(const u4v& w)
{
    return v4i{(int)dfield_bytes<B, T>(w.x), (int)dfield_bytes<B, T>(w.y), (int)dfield_bytes<B, T>(w.z), (int)dfield_bytes<B, T>(w.w)};
}

// Compile-time shape of one variant.
template <int P, int MR, int R>
struct DirectShape {
    static constexpr int NG = group_count(P);
    static constexpr int SL = dmin(16 / MR, P <= 4 ? 16 : 4);   // slices per A operand quad (operand rows past SL*MR stay zero)
    static constexpr int NSL = 8 * R;                     // slices per wave
    static constexpr int NQ = (NSL + SL - 1) / SL;        // A operand quads per wave
    static constexpr int NI = dmin(SL, NSL);              // slice sets in use
    __host__ __device__ static constexpr int b(int g) { return group_width(P, g); }
    __host__ __device__ static constexpr int t(int g) { return 8 / group_width(P, g); }
    __host__ __device__ static constexpr int na(int g) { return dmax(NI, t(g)); }                       // accumulators of group g
    __host__ __device__ static constexpr int acc_base(int g) { return g == 0 ? 0 : (g == 1 ? na(0) : na(0) + na(1)); }
    static constexpr int NACC = acc_base(NG - 1) + na(NG - 1);
    __host__ __device__ static constexpr int load_base(int g) { return group_shift(P, g); }            // 1 KiB loads below group g in a super-chunk
};

// All MFMAs of one super-chunk (index RR of the wave's run) for plane group GI: chunk c holds slices c*T .. c*T+T-1.
template <int P, int MR, int R, int RR, int GI, int C = 0, int T0 = 0>
__device__ __forceinline__ void direct_group_mfma(const u4v* w, const v4i* aq, v4i* acc)
{
    using SH = DirectShape<P, MR, R>;
    constexpr int B = SH::b(GI), T = SH::t(GI);
    if constexpr (C < B) {
        constexpr int s = RR * 8 + C * T + T0;            // slice inside the wave's run
        v4i& a = acc[SH::acc_base(GI) + s % SH::na(GI)];
        a = __builtin_amdgcn_mfma_i32_16x16x64_i8(aq[s / SH::SL], dfield_operand<B, T0>(w[SH::load_base(GI) + C]), a, 0, 0, 0);
        if constexpr (T0 + 1 < T) direct_group_mfma<P, MR, R, RR, GI, C, T0 + 1>(w, aq, acc);
        else direct_group_mfma<P, MR, R, RR, GI, C + 1, 0>(w, aq, acc);
    }
}

// Every super-chunk of the wave's run (RR < nsc, wave-uniform) and every plane group.
template <int P, int MR, int R, int RR = 0>
__device__ __forceinline__ void direct_all_mfma(const u4v (*w)[P], const v4i* aq, v4i* acc, int nsc)
{
    using SH = DirectShape<P, MR, R>;
    if constexpr (RR < R) {
        if (RR < nsc) {
            direct_group_mfma<P, MR, R, RR, 0>(w[RR], aq, acc);
            if constexpr (SH::NG > 1) direct_group_mfma<P, MR, R, RR, 1>(w[RR], aq, acc);
            if constexpr (SH::NG > 2) direct_group_mfma<P, MR, R, RR, 2>(w[RR], aq, acc);
        }
        direct_all_mfma<P, MR, R, RR + 1>(w, aq, acc, nsc);
    }
}

// Per-slice sums of the weights for the per-group path with two super-chunks per wave (single-group widths): the A operand
// of MFMA s holds ones in row s only, so row s of accW[field position] collects sum_k w' of slice s and nothing else.
template <int P, int R, int RR = 0, int C = 0, int T0 = 0>
__device__ __forceinline__ void direct_wsum_mfma(const u4v (*w)[P], int r, int nsc, v4i* accW)
{
    constexpr int B = group_width(P, 0), T = 8 / B;
    if constexpr (RR < R) {
        if constexpr (C < B) {
            constexpr int s = RR * 8 + C * T + T0;
            if (RR < nsc) {
                const int one = r == s ? 0x01010101 : 0;
                accW[T0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(v4i{one, one, one, one}, dfield_operand<B, T0>(w[RR][C]), accW[T0], 0, 0, 0);
            }
            if constexpr (T0 + 1 < T) direct_wsum_mfma<P, R, RR, C, T0 + 1>(w, r, nsc, accW);
            else direct_wsum_mfma<P, R, RR, C + 1, 0>(w, r, nsc, accW);
        } else {
            direct_wsum_mfma<P, R, RR + 1, 0, 0>(w, r, nsc, accW);
        }
    }
}
template <int B, int T0 = 0>
__device__ __forceinline__ v4i direct_wsum_unscale(const v4i* accW)
{
    constexpr int T = 8 / B;
    const v4i& a = accW[T0];
    v4i v{dfield_unscale<B, T0>(a.x), dfield_unscale<B, T0>(a.y), dfield_unscale<B, T0>(a.z), dfield_unscale<B, T0>(a.w)};
    if constexpr (T0 + 1 < T) v += direct_wsum_unscale<B, T0 + 1>(accW);
    return v;
}

// accI[i] += (sum of group GI's accumulators of slice set i, each unscaled by its field position) << shift of the group
template <int P, int MR, int R, int GI, int A = 0>
__device__ __forceinline__ void direct_fold(const v4i* acc, v4i* accI)
{
    using SH = DirectShape<P, MR, R>;
    constexpr int B = SH::b(GI), T = SH::t(GI);
    if constexpr (A < SH::na(GI)) {
        const v4i& a = acc[SH::acc_base(GI) + A];
        constexpr int sh = group_shift(P, GI);
        accI[A % SH::NI] += v4i{dfield_unscale<B, A % T>(a.x) << sh, dfield_unscale<B, A % T>(a.y) << sh, dfield_unscale<B, A % T>(a.z) << sh,
                                dfield_unscale<B, A % T>(a.w) << sh};
        direct_fold<P, MR, R, GI, A + 1>(acc, accI);
    }
}

// Lane (G, reg) of an accumulator holds operand row 4G + reg = slice set (4G+reg)/MR, row (4G+reg) % MR of A.  Picks
// this lane's element of the accumulator of its slice set, then folds the registers that hold the same row of A
// (MR = 1: all four; MR = 2: pairs).  Returns the number of values left in v[].
template <int MR, int NI>
__device__ __forceinline__ void direct_pick(const v4i* accI, int G, int32_t* v)
{
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) {
        int32_t val = 0;
        if constexpr (MR >= 4) {
            // (4G + reg) / MR does not depend on reg
#pragma unroll
            for (int i = 0; i < NI; ++i) val = (4 * G / MR == i) ? accI[i][reg] : val;
        } else {
#pragma unroll
            for (int i = 0; i < NI; ++i) val = ((4 * G + reg) / MR == i) ? accI[i][reg] : val;
        }
        v[reg] = val;
    }
    if constexpr (MR == 1) v[0] = (v[0] + v[1]) + (v[2] + v[3]);
    else if constexpr (MR == 2) { v[0] += v[2]; v[1] += v[3]; }
}

// R = super-chunks per wave at most (all loaded before the first MFMA); RAW: the activation BitPacking step is fused
// in (Fig. 3b packs activations online; Sec. 3.4 folds that cost into existing operators): A arrives as unpacked
// codes, is masked to q bits and offset to signed bytes in registers, and its row sums for the zero-point correction
// come from one more MFMA per operand quad against a B operand of ones.
// GROUPED: several problems in one grid (the workgroup finds its problem from the tile starts); otherwise problem 0.
// Either way the problem's descriptor is copied from the kernel arguments in one batch of scalar loads at the top:
// read field by field where it is used, every first use would wait for a scalar load of its own.
// GQ: per-group weight parameters (groups of 128 along K, Appendix C), built for one row of A and p <= 4.  Every 64-k
// slice of the wave's run then has an accumulator of its own, so the integer sum of every group of 128 k is there after
// the MFMAs without any change to them.  sum_k a' per slice comes from one MFMA of the operand against ones.  sum_k w'
// per slice — the operand sum that the activation zero-point needs — comes, with one super-chunk per wave (eight slices,
// eight operand rows), for free: the other eight operand rows, unused at M = 1, are filled with ones, and row 8 of
// accumulator s then holds it for every channel.  With two super-chunks per wave (p = 1, 2, 4; K up to 16384) all
// sixteen rows are slices, and the sums come from one more MFMA per slice whose A operand holds ones in that slice's
// row only.  Per group: t = c - z * sum a' - zc * (sum w' - 128 z) in exact integers (z: the group's zero-point, zc: the
// token's, both less the stored offsets; padded k hold a' = 0 and w' = z), then one conversion and one fma with the
// group's scale; the lanes of a wave add their groups by lane exchange, and the 16 threads of the epilogue add the
// waves in a fixed order.
template <int P, int MR, int R, bool RAW, bool GROUPED, bool GQ = false>
__global__ __launch_bounds__(1024) void direct_kernel(DirectParams gp)
{
    static_assert(!GQ || direct_has_gq(P, MR, R), "per-group parameters: one row of A and an accumulator per slice");
    using SH = DirectShape<P, MR, R>;
    constexpr int SL = SH::SL, NQ = SH::NQ, NI = SH::NI;
    constexpr int NV = MR == 1 ? 1 : (MR == 2 ? 2 : 4);             // values per lane after direct_pick
    constexpr int C = MR <= 4 ? 4 : (MR == 8 ? 2 : 1);              // lane groups G that hold partials of the same (row, channel)
    extern __shared__ __align__(16) int32_t red[];                   // [S][MR][16][C] partial sums, then [S][MR][C] partial row sums of A
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, G = lane >> 4;
    int g = 0, tile = (int)blockIdx.x;
    if constexpr (GROUPED) {   // (slots past count start at the end of the grid)
#pragma unroll
        for (int i = 1; i < kDirectMaxGroup; ++i) g = (int)blockIdx.x >= gp.first_tile[i] ? i : g;
        tile -= gp.first_tile[g];
    }
    const DirectProblem pr = gp.d[g];
    // (pins the pointers in scalar registers here, so that the compiler fetches them with the sizes above in one
    // batch instead of sinking each load next to its first use behind a branch)
    const int S = (int)blockDim.x >> 6;
    asm volatile("" ::"s"(pr.fields[0]), "s"(pr.fields[1]), "s"(pr.fields[2]), "s"(pr.wparams), "s"(pr.y), "s"(pr.acc), "s"(pr.rq.codes), "s"(pr.N), "s"(pr.K),
                 "s"(gp.oa), "s"(gp.ow), "s"(gp.a_mask), "s"(S));
    if constexpr (RAW) asm volatile("" ::"s"(pr.a_raw), "s"(pr.a_scale), "s"(pr.a_zero));
    else asm volatile("" ::"s"(pr.a_codes), "s"(pr.aparams));
    if constexpr (GQ) asm volatile("" ::"s"(pr.gparams));
    const int M = gp.M, nsuper = pr.nsuper, Kp = pr.Kp;
    const int sc0 = wave * pr.rsplit;
    const int nsc = max(0, min(pr.rsplit, nsuper - sc0));            // this wave's super-chunks (<= R), wave-uniform

    // ---- epilogue parameters of the first 16*M outputs' threads (requested first: cold lines of the blob, used after the barrier)
    const int t0 = (int)threadIdx.x;
    RowParams pa0{0, 0.f, 0, 0}, pw0{0, 0.f, 0, 0};
    if (t0 < 16 * M) {
        const int m = t0 >> 4;
        if constexpr (RAW) pa0 = RowParams{0, pr.a_scale[m], pr.a_zero[m], 0};
        else pa0 = pr.aparams[m];
        pw0 = pr.wparams[min(tile * kTileN + (t0 & 15), pr.N - 1)];
    }

    // ---- the A operand quads: lane (r, G) holds row r % MR of A over 16 k of slice q*SL + r/MR of the wave's run
    v4i aq[NQ];
    const int m_l = r % MR, i_l = r / MR;                            // (i_l >= SL: an operand row that stays zero)
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int sl = i_l < SL ? q * SL + i_l : 8 * R;
        const int k = (sc0 * 8 + sl) * 64 + G * 16;
        v4i v{0, 0, 0, 0};
        if constexpr (RAW) {   // (masked and offset further down, behind the last load of this prologue: nothing waits in between)
            if (m_l < M && sl < 8 * nsc && k < pr.K) v = *reinterpret_cast<const v4i*>(pr.a_raw + (size_t)m_l * pr.K + k);
        } else {
            if (m_l < M && sl < 8 * nsc) v = *reinterpret_cast<const v4i*>(pr.a_codes + (size_t)m_l * Kp + k);
        }
        aq[q] = v;
    }
    u4v grec{0, 0, 0, 0};       // GQ: the group record of this lane's channel and super-chunk
    int zc_all = 0;             // GQ: the token's zero-point less oa (M = 1: the same for every lane)
    if constexpr (GQ) {
        // (R = 2: lanes of G = 2, 3 work on the wave's second super-chunk and take its record)
        grec = __builtin_nontemporal_load(pr.gparams + ((size_t)tile * nsuper + min(sc0 + (R == 2 ? (G >> 1) : 0), nsuper - 1)) * 16 + r);
        if constexpr (RAW) zc_all = pr.a_zero[0] - gp.oa;
        else zc_all = pr.aparams[0].zero - gp.oa;
    }
    // ---- the weight stream, last in program order: everything above can be waited for while it is in flight.  The
    // loads are unconditional (a wave with fewer than R super-chunks re-reads its last one, or the problem's last one
    // when it has none: lines another wave of the tile fetches anyway) so that the wait counts in front of them are exact.
    u4v w[R][P];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int sc = min(sc0 + rr, nsuper - 1);
#pragma unroll
        for (int gi = 0; gi < SH::NG; ++gi) {
            const int b = SH::b(gi);
            const u4v* base = pr.fields[gi] + ((size_t)tile * nsuper + sc) * (b * 64) + lane;
#pragma unroll
            for (int i = 0; i < b; ++i) w[rr][SH::load_base(gi) + i] = __builtin_nontemporal_load(base + i * 64);
        }
    }
    if constexpr (RAW) {
        // unpacked codes -> operand bytes: bits above q dropped (as the packers drop them), less oa; positions that were
        // not loaded (rows past M, k past K) become -oa here and are cleared again
        const uint32_t flip = gp.oa ? 0x80808080u : 0u;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int sl = i_l < SL ? q * SL + i_l : 8 * R;
            const bool live = m_l < M && sl < 8 * nsc && (sc0 * 8 + sl) * 64 + G * 16 < pr.K;
            const v4i c = aq[q];
            aq[q] = live ? v4i{(int)(((uint32_t)c.x & gp.a_mask) ^ flip), (int)(((uint32_t)c.y & gp.a_mask) ^ flip),
                               (int)(((uint32_t)c.z & gp.a_mask) ^ flip), (int)(((uint32_t)c.w & gp.a_mask) ^ flip)}
                         : v4i{0, 0, 0, 0};
        }
    }

    if constexpr (GQ) {
        // R = 1: operand rows 8..15 (no slice lives there) become rows of ones
        if (R == 1 && r >= 8) aq[0] = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};
    }
    v4i asum_acc{0, 0, 0, 0};
    if constexpr (RAW || GQ) {   // row sums of the operand bytes, while the weights are still on their way
        const v4i ones{0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
        for (int q = 0; q < NQ; ++q) asum_acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(aq[q], ones, asum_acc, 0, 0, 0);
    }

    // ---- multiply
    v4i acc[SH::NACC];
#pragma unroll
    for (int i = 0; i < SH::NACC; ++i) acc[i] = v4i{0, 0, 0, 0};
    direct_all_mfma<P, MR, R>(w, aq, acc, nsc);

    if constexpr (GQ) {
        v4i accS[NI];           // accS[s]: accumulator of slice s, fields and plane groups recombined
#pragma unroll
        for (int i = 0; i < NI; ++i) accS[i] = v4i{0, 0, 0, 0};
        direct_fold<P, MR, R, 0>(acc, accS);
        if constexpr (SH::NG > 1) direct_fold<P, MR, R, 1>(acc, accS);
        if constexpr (SH::NG > 2) direct_fold<P, MR, R, 2>(acc, accS);
        // R = 1: lane (G, reg) holds operand row 4G + reg: rows 0..7 = slice 4G + reg against itself (the wanted product
        // sum), rows 8..15 = the ones rows (sum of the weights of slice 4(G-2) + reg).  Either way the lane takes element
        // reg of accumulator 4(G & 1) + reg and adds the two slices of each group: lanes of G = 0, 1 then hold the product
        // sums of groups 2G, 2G+1 of their channel, lanes of G = 2, 3 the weight sums of the same groups, 32 lanes further up.
        int c0, c1, ws0, ws1;
        bool live = true;
        if constexpr (R == 1) {
            int32_t e[4];
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) e[reg] = (G & 1) ? accS[4 + reg][reg] : accS[reg][reg];
            c0 = e[0] + e[1]; c1 = e[2] + e[3];
            ws0 = __shfl(c0, (lane + 32) & 63); ws1 = __shfl(c1, (lane + 32) & 63);
        } else {
            // R = 2: all sixteen operand rows are slices; lane (G, reg) takes element reg of accumulator 4G + reg, and the
            // weight sums come from MFMAs of their own whose A operand holds ones in one row only
            v4i accW[8 / group_width(P, 0)];
#pragma unroll
            for (int i = 0; i < 8 / group_width(P, 0); ++i) accW[i] = v4i{0, 0, 0, 0};
            direct_wsum_mfma<P, R>(w, r, nsc, accW);
            const v4i wsv = direct_wsum_unscale<group_width(P, 0)>(accW);
            int32_t e[4] = {0, 0, 0, 0};
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) e[reg] = G == g4 ? accS[4 * g4 + reg][reg] : e[reg];
            c0 = e[0] + e[1]; c1 = e[2] + e[3];
            ws0 = wsv.x + wsv.y; ws1 = wsv.z + wsv.w;
            live = (G >> 1) < nsc;                                     // (a wave with one super-chunk: its second half adds nothing)
        }
        // every column of asum_acc holds the row sums of the operand: this lane's rows are slices 4G .. 4G+3
        const int as0 = asum_acc.x + asum_acc.y, as1 = asum_acc.z + asum_acc.w;
        const int g0 = 2 * (G & 1);                                    // this lane's first group of the super-chunk
        const int z0 = ((int)(grec.z << (24 - 8 * g0))) >> 24, z1 = ((int)(grec.z << (16 - 8 * g0))) >> 24;
        const uint32_t sb = (G & 1) ? grec.y : grec.x;                 // the two binary16 scales of groups g0, g0 + 1
        const float s0 = __half2float(__ushort_as_half((unsigned short)(sb & 0xFFFFu)));
        const float s1 = __half2float(__ushort_as_half((unsigned short)(sb >> 16)));
        const int t0g = c0 - z0 * as0 - zc_all * (ws0 - 128 * z0);
        const int t1g = c1 - z1 * as1 - zc_all * (ws1 - 128 * z1);
        float f = (float)t0g * s0;
        f = __builtin_fmaf((float)t1g, s1, f);
        if (!live) f = 0.f;
        f += __shfl(f, lane ^ 16);                                      // groups 0, 1 (G = 0) + groups 2, 3 (G = 1): same order in both lanes
        if constexpr (R == 2) f += __shfl(f, lane ^ 32);               // + the second super-chunk's four groups
        float* fpart = reinterpret_cast<float*>(red);                  // [wave][channel]
        if (G == 0) fpart[wave * 16 + r] = f;
        __syncthreads();
        if (t0 < 16) {           // (M = 1: one output per channel of the tile); the waves' sums are added in a fixed order
            const int n = tile * kTileN + t0;
            float fsum = 0.f;
            for (int ww = 0; ww < S; ++ww) fsum += fpart[ww * 16 + t0];
            if (n < pr.N) pr.y[n] = __half_as_ushort(__float2half_rn(pa0.scale * fsum));
        }
        return;
    }

    // ---- bit reduction over fields and plane groups, then the rows that belong to each accumulator
    v4i accI[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) accI[i] = v4i{0, 0, 0, 0};
    direct_fold<P, MR, R, 0>(acc, accI);
    if constexpr (SH::NG > 1) direct_fold<P, MR, R, 1>(acc, accI);
    if constexpr (SH::NG > 2) direct_fold<P, MR, R, 2>(acc, accI);
    int32_t v[4];
    direct_pick<MR, NI>(accI, G, v);
    // lane (G, r): v[i] is a partial sum for row m of A and channel r of the tile, m = i (MR <= 4), 4*(G&1)+i (MR = 8),
    // 4*G+i (MR = 16); C lane groups hold partials of the same element: red[((wave*MR + m)*16 + r)*C + c]
    const int c_l = MR <= 4 ? G : (MR == 8 ? (G >> 1) : 0);
    const int m_base = MR <= 4 ? 0 : (MR == 8 ? 4 * (G & 1) : 4 * G);
#pragma unroll
    for (int i = 0; i < NV; ++i) red[((wave * MR + m_base + i) * 16 + r) * C + c_l] = v[i];
    int32_t* reda = red + S * MR * 16 * C;
    if constexpr (RAW) {
        // every row of asum_acc holds the sum of its operand row over the wave's quads, the same in all 16 columns
        int32_t s4[4] = {asum_acc.x, asum_acc.y, asum_acc.z, asum_acc.w};
        if constexpr (MR == 1) s4[0] = (s4[0] + s4[1]) + (s4[2] + s4[3]);
        else if constexpr (MR == 2) { s4[0] += s4[2]; s4[1] += s4[3]; }
        if (r == 0) {
#pragma unroll
            for (int i = 0; i < NV; ++i) reda[(wave * MR + m_base + i) * C + c_l] = s4[i];
        }
    }
    __syncthreads();

    // ---- sum over waves (and lane groups), fused dequant epilogue
    for (int t = t0; t < 16 * M; t += (int)blockDim.x) {
        const int m = t >> 4, nl = t & 15, n = tile * kTileN + nl;
        int32_t sum = 0;
        for (int ww = 0; ww < S; ++ww) {
            const int32_t* p = red + ((ww * MR + m) * 16 + nl) * C;
            if constexpr (C == 4) { const v4i x = *reinterpret_cast<const v4i*>(p); sum += (x.x + x.y) + (x.z + x.w); }
            else if constexpr (C == 2) sum += p[0] + p[1];
            else sum += p[0];
        }
        RowParams pa = pa0, pw = pw0;
        if (t != t0) {   // (more outputs than threads: M > 4 with fewer than four waves)
            if constexpr (RAW) pa = RowParams{0, pr.a_scale[m], pr.a_zero[m], 0};
            else pa = pr.aparams[m];
            pw = pr.wparams[min(n, pr.N - 1)];
        }
        if constexpr (RAW) {
            int32_t as = 0;
            for (int ww = 0; ww < S; ++ww) {
                const int32_t* p = reda + (ww * MR + m) * C;
                if constexpr (C == 4) { const v4i x = *reinterpret_cast<const v4i*>(p); as += (x.x + x.y) + (x.z + x.w); }
                else if constexpr (C == 2) as += p[0] + p[1];
                else as += p[0];
            }
            pa.sum = as + gp.oa * pr.K;   // the operand bytes are the codes less oa; padding holds zero bytes
        }
        if (n < pr.N) epilogue_store(sum, gp.oa, gp.ow, pr.K, pa, pw, (size_t)m * pr.N + n, pr.y, pr.acc, pr.rq, m);
    }
}

inline size_t direct_lds_bytes(int S, int MR, bool gq)
{
    if (gq) return (size_t)S * 16 * 4;   // one binary32 partial per wave and channel (MR = 1)
    const int C = MR <= 4 ? 4 : (MR == 8 ? 2 : 1);
    return (size_t)S * MR * 16 * C * 4 + (size_t)S * MR * C * 4;
}

template <int P, int MR, int R, bool RAW>
static hipError_t direct_launch_one(const DirectParams& gp, unsigned grid, int waves, hipStream_t s)
{
    if (gp.d[0].gparams) {   // per-group weight parameters (every problem of a launch is of the same kind)
        if constexpr (direct_has_gq(P, MR, R)) {
            if (gp.count > 1) direct_kernel<P, MR, R, RAW, true, true><<<grid, waves * 64, direct_lds_bytes(waves, MR, true), s>>>(gp);
            else direct_kernel<P, MR, R, RAW, false, true><<<grid, waves * 64, direct_lds_bytes(waves, MR, true), s>>>(gp);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (gp.count > 1) direct_kernel<P, MR, R, RAW, true><<<grid, waves * 64, direct_lds_bytes(waves, MR, false), s>>>(gp);
    else direct_kernel<P, MR, R, RAW, false><<<grid, waves * 64, direct_lds_bytes(waves, MR, false), s>>>(gp);
    return hipGetLastError();
}

template <int P, int MR, int R>
static hipError_t direct_launch_r(const DirectParams& gp, bool raw, unsigned grid, int waves, hipStream_t s)
{
    return raw ? direct_launch_one<P, MR, R, true>(gp, grid, waves, s) : direct_launch_one<P, MR, R, false>(gp, grid, waves, s);
}

template <int P, int MR>
static hipError_t direct_launch_mr(const DirectParams& gp, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    if constexpr (MR < direct_min_rows(P)) return hipErrorInvalidValue;
    else {
        if (R == 1) return direct_launch_r<P, MR, 1>(gp, raw, grid, waves, s);
        if constexpr (direct_has(P, MR, 2)) { if (R == 2) return direct_launch_r<P, MR, 2>(gp, raw, grid, waves, s); }
        if constexpr (direct_has(P, MR, 4)) { if (R == 4) return direct_launch_r<P, MR, 4>(gp, raw, grid, waves, s); }
        return hipErrorInvalidValue;
    }
}

template <int P>
static hipError_t direct_launch_p(const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s)
{
    switch (MR) {
        case 1: return direct_launch_mr<P, 1>(gp, R, raw, grid, waves, s);
        case 2: return direct_launch_mr<P, 2>(gp, R, raw, grid, waves, s);
        case 4: return direct_launch_mr<P, 4>(gp, R, raw, grid, waves, s);
        case 8: return direct_launch_mr<P, 8>(gp, R, raw, grid, waves, s);
        case 16: return direct_launch_mr<P, 16>(gp, R, raw, grid, waves, s);
        default: return hipErrorInvalidValue;
    }
}

// Entry points of the per-width translation units.
hipError_t direct_launch_p12(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s);
hipError_t direct_launch_p34(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s);
hipError_t direct_launch_p56(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s);
hipError_t direct_launch_p78(int p, const DirectParams& gp, int MR, int R, bool raw, unsigned grid, int waves, hipStream_t s);

}  // namespace abq
