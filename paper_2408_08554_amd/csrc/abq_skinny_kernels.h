// Device code of the streaming decode kernel and the templates that launch its variants.  Included by the
// host-side translation unit (abq_skinny.hip) for the argument structures and by one translation unit per
// pair of weight widths (abq_skinny_p12.hip ...), which hold the kernel instantiations, so that they
// compile in parallel.
//
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
#pragma once
#include "abq_internal.h"
#include "../../include/abq.h"

#include <hip/hip_fp16.h>
#include <stdlib.h>
#include <atomic>

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

struct SkinnyParams {
    const u4v* fields[3];     // per plane group
    int chunks[3];
    const int8_t* a_codes;    // [M][Kp]  (packed activations)
    const RowParams* aparams;
    const uint8_t* a_raw;     // [M][K] unpacked codes, with a_scale / a_zero: the fused-pack variant reads these instead
    const float* a_scale;
    const int32_t* a_zero;
    const RowParams* wparams;
    uint16_t* y;              // may be null when rq.codes is given
    int32_t* acc;
    Requant rq;               // output codes of the next layer (codes == null: off)
    int M, N, K, Kp;
    int oa, ow;
    uint32_t a_mask;          // (2^q - 1) in every byte: applied to unpacked activation codes while they are staged
    int ntiles;               // 16-row tiles of W
    int nsuper;               // Kp / 512
    int sc_q, sc_r;           // nsuper = sc_q * S + sc_r   (S = waves per workgroup): wave w owns sc_q + (w < sc_r) super-chunks
    int tl_q, tl_r;           // ntiles = tl_q * gridDim.x + tl_r: workgroup b owns tl_q + (b < tl_r) tiles
    int mrows;                // rows of A per workgroup (<= 16); blockIdx.y walks row groups
    int a_stride;             // bytes per staged row of A (Kp + 16: rows land 16 B apart in bank space)
    int par_off;              // byte offset in LDS of the staged per-row / per-channel parameters
    int red_off;              // byte offset in LDS of the two reduction buffers
    int asum_off;             // byte offset in LDS of the per-wave partial row sums of A ([S][16] int32, fused-pack variant)
    int zero_off;             // byte offset in LDS of 512 zero bytes
    // K groups (long K with up to 16 rows of A: all of A does not fit LDS at once).  A wave's nsw super-chunks
    // are cut into kgroups runs [g*nsw/kgroups, (g+1)*nsw/kgroups); the workgroup walks its tiles once per
    // run with only that run's columns of A staged, keeping per-tile partial sums in LDS in between.
    int kgroups;              // 1: everything staged once
    int col_w, col_s;         // LDS column of (wave, slot) = wave*col_w + slot*col_s  (slot = super-chunk index inside the run)
    int part_off;             // byte offset in LDS of the partial sums [S][nmy_max][256] int32 (kgroups > 1)
    int nmy_max;              // most tiles any workgroup owns
    // Per-group weight parameters (groups of 128 k; null for per-channel weights): [ntiles][nsuper][16 channels]
    // records of 16 B = four binary16 scales, four int8 zero-points (already less ow), 4 B unused.
    const u4v* gparams;
};

// g * n / G for the few group counts the host uses (constant divisors).
__device__ __forceinline__ int group_bound(int g, int n, int G)
{
    const int x = g * n;
    switch (G) {
        case 1: return x;
        case 2: return x >> 1;
        case 3: return x / 3;
        default: return x >> 2;
    }
}
// Field t of a b-bit group as a signed-byte MFMA operand dword, and the power of two it is
// scaled by.  The field that would touch the byte's sign bit is moved down one bit instead
// (b = 2, 4) or taken as is with weight -128 (b = 1).
template <int B, int T>
__device__ __forceinline__ uint32_t field_bytes(uint32_t x)
{
    if constexpr (B == 8) return x;
    else if constexpr (B == 4) return T == 0 ? (x & 0x0F0F0F0Fu) : ((x >> 1) & 0x78787878u);
    else if constexpr (B == 2) return T == 3 ? ((x >> 1) & 0x60606060u) : (x & (0x03030303u << (2 * T)));
    else return x & (0x01010101u << T);
}
template <int B, int T>
__device__ __forceinline__ int32_t field_unscale(int32_t acc)
{
    if constexpr (B == 8) return acc;
    else if constexpr (B == 4) return T == 0 ? acc : (acc >> 3);
    else if constexpr (B == 2) return T == 3 ? (acc >> 5) : (acc >> (2 * T));
    else return T == 7 ? -(acc >> 7) : (acc >> T);
}

template <int B, int T>
__device__ __forceinline__ v4i field_operand(const u4v& w)
{
    v4i r;
    r.x = (int)field_bytes<B, T>(w.x);
    r.y = (int)field_bytes<B, T>(w.y);
    r.z = (int)field_bytes<B, T>(w.z);
    r.w = (int)field_bytes<B, T>(w.w);
    return r;
}

// Per-group compile-time bookkeeping for weight width P.
template <int P> struct GroupInfo {
    static constexpr int NG = group_count(P);
    static constexpr int loads = P;   // sum_g b_g chunks of 1 KiB per super-chunk
    __host__ __device__ static constexpr int b(int g) { return group_width(P, g); }
    __host__ __device__ static constexpr int load_base(int g) { return group_shift(P, g); }   // sum of widths below g
    __host__ __device__ static constexpr int acc_base(int g)
    {
        return g == 0 ? 0 : (g == 1 ? 8 / b(0) : 8 / b(0) + 8 / b(1));
    }
    static constexpr int NACC = acc_base(NG - 1) + 8 / b(NG - 1);
};

// MFMAs of one chunk (index I inside the super-chunk) of group width B: slices I*T .. I*T+T-1.
template <int B, int I, int T0 = 0>
__device__ __forceinline__ void chunk_mfma(const u4v& w, const v4i* aop, v4i* acc)
{
    constexpr int T = 8 / B;
    if constexpr (T0 < T) {
        acc[T0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[I * T + T0], field_operand<B, T0>(w), acc[T0], 0, 0, 0);
        chunk_mfma<B, I, T0 + 1>(w, aop, acc);
    }
}
template <int B, int I = 0>
__device__ __forceinline__ void group_mfma(const u4v* w, const v4i* aop, v4i* acc)
{
    if constexpr (I < B) {   // a b-bit group has b chunks per super-chunk
        chunk_mfma<B, I>(w[I], aop, acc);
        group_mfma<B, I + 1>(w, aop, acc);
    }
}
template <int B, int T0 = 0>
__device__ __forceinline__ v4i group_combine(const v4i* acc)
{
    constexpr int T = 8 / B;
    v4i r;
    r.x = field_unscale<B, T0>(acc[T0].x);
    r.y = field_unscale<B, T0>(acc[T0].y);
    r.z = field_unscale<B, T0>(acc[T0].z);
    r.w = field_unscale<B, T0>(acc[T0].w);
    if constexpr (T0 + 1 < T) r += group_combine<B, T0 + 1>(acc);
    return r;
}

// Sum of v over the 64 lanes, returned in every lane: four DPP steps inside each row of 16
// lanes, then the four row totals are read out as scalars.
__device__ __forceinline__ int32_t wave_sum(int32_t v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);   // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false);   // row_mirror
    return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
           (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}

// One super-chunk of one tile: P wave loads of 1 KiB.  Every group stores whole super-chunks
// (chunk count = b * Kp/512), so no load is conditional.
template <int P, bool GQ = false>
__device__ __forceinline__ void load_super(const SkinnyParams& prm, int nsuper, int tile, int sc, int lane, u4v* w)
{
    using GI = GroupInfo<P>;
    if constexpr (GQ)   // the super-chunk's group parameters of this lane's channel ride in the ring slot's last entry
        w[P] = __builtin_nontemporal_load(prm.gparams + ((size_t)tile * nsuper + sc) * 16 + (lane & 15));
#pragma unroll
    for (int g = 0; g < GI::NG; ++g) {
        const int b = GI::b(g);
        const u4v* base = prm.fields[g] + ((size_t)tile * nsuper + sc) * (b * 64) + lane;
#pragma unroll
        for (int i = 0; i < b; ++i)   // read once: non-temporal, so the stream does not displace A and the parameters in L2
            w[GI::load_base(g) + i] = __builtin_nontemporal_load(base + i * 64);
    }
}

template <int P>
__device__ __forceinline__ void compute_super(const u4v* w, const uint8_t* lds_row, v4i* acc)
{
    using GI = GroupInfo<P>;
    v4i aop[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) aop[j] = *reinterpret_cast<const v4i*>(lds_row + j * 64);
    group_mfma<GI::b(0)>(w + GI::load_base(0), aop, acc + GI::acc_base(0));
    if constexpr (GI::NG > 1) group_mfma<GI::b(1)>(w + GI::load_base(1), aop, acc + GI::acc_base(1));
    if constexpr (GI::NG > 2) group_mfma<GI::b(2)>(w + GI::load_base(2), aop, acc + GI::acc_base(2));
}

// ---- per-group weight parameters: one super-chunk = four groups of 128 k = four pairs of 64-k slices --------
typedef float v4f __attribute__((ext_vector_type(4)));

// Field T0 of a b-bit plane group placed at bit position SH of the operand byte (the plane group's shift inside
// the weight): the bit reduction over plane groups then happens inside the MFMA, every group adding into one
// accumulator.  p <= 7 keeps the byte below 128; an 8-bit group is the stored signed byte itself.
template <int B, int T0, int SH>
__device__ __forceinline__ uint32_t placed_bytes(uint32_t x)
{
    if constexpr (B == 8) return x;
    else {
        constexpr uint32_t mask = (0x01010101u * ((1u << B) - 1u)) << SH;
        constexpr int from = B * T0;
        if constexpr (from == SH) return x & mask;
        else if constexpr (from > SH) return (x >> (from - SH)) & mask;
        else return (x << (SH - from)) & mask;
    }
}
template <int B, int T0, int SH>
__device__ __forceinline__ v4i placed_operand(const u4v& w)
{
    return v4i{(int)placed_bytes<B, T0, SH>(w.x), (int)placed_bytes<B, T0, SH>(w.y), (int)placed_bytes<B, T0, SH>(w.z),
               (int)placed_bytes<B, T0, SH>(w.w)};
}
// acc += sum_k a * (field << SH) over the 128 k of pair J for one plane group of width B.  Slice SL lives in chunk
// SL / T at field position SL % T (T = 8 / B).
template <int B, int SH, int J>
__device__ __forceinline__ v4i pair_add(const u4v* w, const v4i* aop, v4i acc)
{
    constexpr int T = 8 / B, S0 = 2 * J, S1 = 2 * J + 1;
    acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[S0], placed_operand<B, S0 % T, SH>(w[S0 / T]), acc, 0, 0, 0);
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[S1], placed_operand<B, S1 % T, SH>(w[S1 / T]), acc, 0, 0, 0);
}
// Group J of the super-chunk: the exact integer sum_k (a' - zc)(w' - z) over its 128 k, then one conversion and one
// multiply-add per element with the group's scale into the single-precision sum over groups.  a' = a - oa and
// w' = w - ow are the stored operands, z the group's zero-point less ow, zc the token's zero-point less oa.
//   c = sum_k a' w' + sum_k a' (-z): every plane group (fields placed at their bit positions) and then one more
//       MFMA pair against a B operand whose bytes all hold -z of the lane's channel (p <= 7: -z fits a signed byte);
//   d = sum_k zc w' + sum_k zc (-z): the same B operands against an A operand whose bytes all hold zc of the lane's
//       row (zc fits a signed byte; -zc would not when zc = -128, hence the second accumulator and c - d).
// At p = 8 (z down to -128) the z terms come from an MFMA pair against ones and integer multiplies instead:
//   sum = c - d - z (sum_k a' - 128 zc).
// Every term is an exact integer before the first float operation, so nothing large cancels in floating point.
// Padding: k past K holds a' = 0 and w' = z (the packer pads a g128 blob's last group with its zero-point), so
// padded k add nothing to either accumulator; groups wholly past K carry scale 0.
template <int P, int J>
__device__ __forceinline__ void group_step(const u4v* w, const v4i* aop, const u4v gp, const v4i& zc_op, const v4i& zc128, v4f& facc)
{
    using GI = GroupInfo<P>;
    v4i c{0, 0, 0, 0}, d{0, 0, 0, 0};
    const v4i zaop[8] = {zc_op, zc_op, zc_op, zc_op, zc_op, zc_op, zc_op, zc_op};
    c = pair_add<GI::b(0), 0, J>(w + GI::load_base(0), aop, c);
    d = pair_add<GI::b(0), 0, J>(w + GI::load_base(0), zaop, d);
    if constexpr (GI::NG > 1) {
        c = pair_add<GI::b(1), GI::load_base(1), J>(w + GI::load_base(1), aop, c);
        d = pair_add<GI::b(1), GI::load_base(1), J>(w + GI::load_base(1), zaop, d);
    }
    if constexpr (GI::NG > 2) {
        c = pair_add<GI::b(2), GI::load_base(2), J>(w + GI::load_base(2), aop, c);
        d = pair_add<GI::b(2), GI::load_base(2), J>(w + GI::load_base(2), zaop, d);
    }
    const int z = ((int)(gp.z << (24 - 8 * J))) >> 24;
    if constexpr (P < 8) {
        const int zb = (int)(((uint32_t)(-z) & 0xFFu) * 0x01010101u);
        const v4i zop{zb, zb, zb, zb};
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[2 * J], zop, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[2 * J + 1], zop, c, 0, 0, 0);
        d = __builtin_amdgcn_mfma_i32_16x16x64_i8(zc_op, zop, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_i32_16x16x64_i8(zc_op, zop, d, 0, 0, 0);
        c -= d;
    } else {
        const v4i zero{0, 0, 0, 0}, ones{0x01010101, 0x01010101, 0x01010101, 0x01010101};
        const v4i asum = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[2 * J + 1], ones,
                             __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[2 * J], ones, zero, 0, 0, 0), 0, 0, 0);
        c -= d;
        c = v4i{c.x - z * (asum.x - zc128.x), c.y - z * (asum.y - zc128.y), c.z - z * (asum.z - zc128.z), c.w - z * (asum.w - zc128.w)};
    }
    const uint32_t sbits = (J < 2 ? gp.x : gp.y) >> (16 * (J & 1));
    const float sc = __half2float(__ushort_as_half((unsigned short)(sbits & 0xFFFFu)));
    facc.x = fmaf((float)c.x, sc, facc.x);
    facc.y = fmaf((float)c.y, sc, facc.y);
    facc.z = fmaf((float)c.z, sc, facc.z);
    facc.w = fmaf((float)c.w, sc, facc.w);
}
template <int P>
__device__ __forceinline__ void compute_super_gq(const u4v* w, const uint8_t* lds_row, const v4i& zc_op, const v4i& zc128, v4f& facc)
{
    v4i aop[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) aop[j] = *reinterpret_cast<const v4i*>(lds_row + j * 64);
    const u4v gp = w[P];
    group_step<P, 0>(w, aop, gp, zc_op, zc128, facc);
    group_step<P, 1>(w, aop, gp, zc_op, zc128, facc);
    group_step<P, 2>(w, aop, gp, zc_op, zc128, facc);
    group_step<P, 3>(w, aop, gp, zc_op, zc128, facc);
}

// Per-wave streaming state (lives in registers once everything is inlined).
template <int P>
struct WaveState {
    int nsuper, S, nsw, nitems;
    int tile0, tstride;            // this workgroup's tiles: tile0 + i * tstride
    int p_ti, p_lsc;               // next item to prefetch
    int ti, lsc, parity;           // item being consumed
    int nmy;                       // tiles this workgroup owns
    int g, gs, ge;                 // K group being consumed and its run [gs, ge) of this wave's super-chunks
    int p_g, p_gs, p_ge;           // the same for the prefetch side
    int32_t* part;                 // LDS: this wave's partial sums [nmy_max][256] (kgroups > 1)
    int lane, wave, tid, m0, mt;   // mt = rows of A this workgroup owns (<= 16)
    const uint8_t* lds_lane;       // this lane's A operand base in LDS: its row of A, or a block of zeros for rows past mt
    int k_mask;                    // ~0 for a row of A, 0 for the zero block (which has no k extent)
    const RowParams* par;          // LDS: [16] rows of A, then [nmy][16] channels
    const int32_t* asum;           // LDS: [S][16] partial row sums of A (fused-pack variant)
    int32_t* red;
    v4i acc[GroupInfo<P>::NACC];
    v4f facc;                      // per-group weight parameters: this wave's single-precision sum over its groups
    v4i zc_op, zc128;              // the same: zero-point less oa of the lane's row of A in every operand byte; 128 times that of the lane's four accumulator rows
};

// Item order: (K group,) tile, super-chunk.
template <int P, bool KG = false, bool GQ = false>
__device__ __forceinline__ void prefetch_item(const SkinnyParams& prm, WaveState<P>& st, u4v* slot)
{
    load_super<P, GQ>(prm, st.nsuper, st.tile0 + st.p_ti * st.tstride, st.wave + st.p_lsc * st.S, st.lane, slot);
    if constexpr (!KG) {
        if (++st.p_lsc == st.nsw) { st.p_lsc = 0; ++st.p_ti; }
    } else {
        if (++st.p_lsc == st.p_ge) {
            if (++st.p_ti == st.nmy) {
                st.p_ti = 0;
                ++st.p_g;
                st.p_gs = st.p_ge;
                st.p_ge = group_bound(st.p_g + 1, st.nsw, prm.kgroups);
            }
            st.p_lsc = st.p_gs;
        }
    }
}

// LDS address of this lane's A operand for the super-chunk being consumed.
template <int P, bool KG>
__device__ __forceinline__ const uint8_t* operand_row(const SkinnyParams& prm, const WaveState<P>& st)
{
    if constexpr (!KG) return st.lds_lane + (((st.wave + st.lsc * st.S) * kSuperK) & st.k_mask);
    else return st.lds_lane + ((st.wave * prm.col_w + (st.lsc - st.gs) * prm.col_s) & st.k_mask);
}

// End of a tile on this wave: bit reduction over the plane groups, sum over the S waves
// through LDS (two buffers alternate, so one barrier per tile is enough), fused epilogue.
template <int P, int EPT, bool RAW, bool KG = false, bool GQ = false>
__device__ __forceinline__ void finish_tile(const SkinnyParams& prm, WaveState<P>& st)
{
    using GI = GroupInfo<P>;
    static_assert(!(GQ && KG), "per-group weight parameters are not combined with K groups");
    v4i total;
    if constexpr (GQ) {
        // the wave's partial result is a single-precision sum; it travels through LDS as its bit pattern
        total = v4i{__float_as_int(st.facc.x), __float_as_int(st.facc.y), __float_as_int(st.facc.z), __float_as_int(st.facc.w)};
        st.facc = v4f{0.f, 0.f, 0.f, 0.f};
    } else {
        total = group_combine<GI::b(0)>(st.acc + GI::acc_base(0));
        if constexpr (GI::NG > 1) total += group_combine<GI::b(1)>(st.acc + GI::acc_base(1)) << GI::load_base(1);
        if constexpr (GI::NG > 2) total += group_combine<GI::b(2)>(st.acc + GI::acc_base(2)) << GI::load_base(2);
#pragma unroll
        for (int i = 0; i < GI::NACC; ++i) st.acc[i] = v4i{0, 0, 0, 0};
    }
    if constexpr (KG) {
        // all but the last K group: the tile's sum so far stays in this wave's own part of LDS
        int32_t* pp = st.part + st.ti * 256 + st.lane;
        if (st.g > 0) {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) total[reg] += pp[reg * 64];
        }
        if (st.g < prm.kgroups - 1) {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) pp[reg * 64] = total[reg];
            ++st.ti;
            return;
        }
    }
    int32_t* rb = st.red + st.parity * (st.S * 256);
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) rb[(st.wave * 4 + reg) * 64 + st.lane] = total[reg];
    __syncthreads();
    // thread t finishes C elements e = t + i*blockDim < 256; element e is register e/64 of lane e%64:
    // row 4*((e%64)/16) + e/64 of A, column e%16 of the tile (the 16x16 MFMA accumulator layout)
    const int tile = st.tile0 + st.ti * st.tstride;
    const int n = tile * kTileN + (st.tid & 15);
    const RowParams pw = st.par[16 + st.ti * 16 + (st.tid & 15)];
    if constexpr (GQ) {
        // Y = a_scale * (sum over waves and groups); the waves' sums are added in a fixed order.  Any workgroup
        // size: thread t takes elements t, t + blockDim, ...
        for (int e = st.tid; e < 256; e += (int)blockDim.x) {
            const int row = 4 * ((e & 63) >> 4) + (e >> 6);
            if (row < st.mt && n < prm.N) {
                float part[8];
#pragma unroll
                for (int ww = 0; ww < 8; ++ww) part[ww] = ww < st.S ? __int_as_float(rb[ww * 256 + e]) : 0.f;
                const float sum = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
                const RowParams pa = st.par[row];
                const float v = pa.scale * sum;
                prm.y[(size_t)(st.m0 + row) * prm.N + n] = __half_as_ushort(__float2half_rn(v));
            }
        }
        st.parity ^= 1;
        ++st.ti;
        return;
    }
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int e = st.tid + i * (int)blockDim.x;
        const int row = 4 * ((e & 63) >> 4) + (e >> 6);
        const int m = st.m0 + row;
        if ((EPT > 1 || e < 256) && row < st.mt && n < prm.N) {   // rows past mt belong to the next row group's workgroup
            int32_t part[8];
#pragma unroll
            for (int ww = 0; ww < 8; ++ww) part[ww] = ww < st.S ? rb[ww * 256 + e] : 0;   // independent reads, one wait
            const int32_t s = ((part[0] + part[1]) + (part[2] + part[3])) + ((part[4] + part[5]) + (part[6] + part[7]));
            RowParams pa = st.par[row];
            if constexpr (RAW) {   // the row sum of A was taken while staging, one part per wave
                int32_t sp[8];
#pragma unroll
                for (int ww = 0; ww < 8; ++ww) sp[ww] = ww < st.S ? st.asum[ww * 16 + row] : 0;
                pa.sum = ((sp[0] + sp[1]) + (sp[2] + sp[3])) + ((sp[4] + sp[5]) + (sp[6] + sp[7]));
            }
            epilogue_store(s, prm.oa, prm.ow, prm.K, pa, pw, (size_t)m * prm.N + n, prm.y, prm.acc, prm.rq, m);
        }
    }
    st.parity ^= 1;
    ++st.ti;
}

// One item: MFMAs, refill of its ring slot, end-of-tile work.  With K groups, the end of a group's last
// tile moves on to the next run of super-chunks and stages its columns of A (next_group).
template <int P, int EPT, bool RAW, bool KG, bool REFILL, bool GQ, typename F>
__device__ __forceinline__ void item_step(const SkinnyParams& prm, WaveState<P>& st, u4v* slot, bool refill, F&& next_group)
{
    if constexpr (GQ) compute_super_gq<P>(slot, operand_row<P, KG>(prm, st), st.zc_op, st.zc128, st.facc);
    else compute_super<P>(slot, operand_row<P, KG>(prm, st), st.acc);
    if (REFILL) prefetch_item<P, KG, GQ>(prm, st, slot);
    else if (refill) prefetch_item<P, KG, GQ>(prm, st, slot);
    if constexpr (!KG) {
        if (++st.lsc == st.nsw) { finish_tile<P, EPT, RAW, false, GQ>(prm, st); st.lsc = 0; }
    } else {
        if (++st.lsc == st.ge) {
            finish_tile<P, EPT, RAW, true>(prm, st);
            if (st.ti == st.nmy) {
                st.ti = 0;
                ++st.g;
                st.gs = st.ge;
                st.ge = group_bound(st.g + 1, st.nsw, prm.kgroups);
                if (st.g < prm.kgroups) next_group();
            }
            st.lsc = st.gs;
        }
    }
}

// D = super-chunks of weight loads each wave keeps in flight; EPT = C elements per thread in
// the epilogue (1 for >= 4 waves, 2 for two waves, 4 for one).  RAW: the activation BitPacking
// step is fused in (Fig. 3b packs activations online; Sec. 3.4 folds that cost into existing
// operators): A arrives as unpacked codes, is offset to signed bytes while it is staged, and
// its row sums for the zero-point correction are taken on the way.
// FULL: every wave of the launch has at least D items, so the ring prologue needs no conditions.
// KG: K groups (see SkinnyParams); never together with FULL.
// The body takes the workgroup's share of the problem as arguments (tiles tile0 + i * tstride, i < nmy; row
// group by) so that the grouped launch below can run it on one problem of several.
template <int P, int D, int EPT, bool RAW, bool FULL, bool KG, bool R16, bool GQ = false>
__device__ __forceinline__ void skinny_body(const SkinnyParams& prm, const int tile0, const int tstride, const int nmy, const int by)
{
    static_assert(!(FULL && KG), "the K-group variant uses the conditional ring prologue");
    static_assert(!(GQ && (KG || R16)), "per-group weight parameters: plain and FULL variants only");
    using GI = GroupInfo<P>;
    extern __shared__ __align__(16) uint8_t lds[];
    WaveState<P> st;
    st.tid = threadIdx.x; st.lane = st.tid & 63; st.wave = st.tid >> 6; st.S = blockDim.x >> 6;
    st.m0 = by * prm.mrows;
    const int mt = min(prm.mrows, prm.M - st.m0);
    st.mt = mt;
    const int r = st.lane & 15, G = st.lane >> 4;
    st.nsuper = prm.nsuper;
    st.tile0 = tile0; st.tstride = tstride;
    st.p_ti = 0; st.p_lsc = 0; st.ti = 0; st.lsc = 0; st.parity = 0;

    st.nsw = prm.sc_q + (st.wave < prm.sc_r ? 1 : 0);                       // this wave's super-chunks per tile (>= 1)
    st.nitems = nmy * st.nsw;
    st.nmy = nmy;
    st.g = 0; st.gs = 0; st.ge = KG ? group_bound(1, st.nsw, prm.kgroups) : st.nsw;
    st.p_g = 0; st.p_gs = 0; st.p_ge = st.ge;

    // ---- epilogue parameters: entry i < 16 is row m0+i of A, entry 16 + 16*t + c is channel c of this
    // workgroup's t-th tile.  Loads use clamped indices so that none is conditional.
    RowParams* par = reinterpret_cast<RowParams*>(lds + prm.par_off);
    const int npar = 16 + nmy * 16;
    auto load_par = [&](int i) -> RowParams {
        if constexpr (RAW) {
            const int m = min(st.m0 + min(i, 15), prm.M - 1);
            const RowParams pa{0, prm.a_scale[m], prm.a_zero[m], 0};
            const RowParams pw = prm.wparams[min((st.tile0 + (max(i - 16, 0) >> 4) * st.tstride) * kTileN + (i & 15), prm.N - 1)];
            return i < 16 ? pa : pw;
        } else {
            const RowParams* src = i < 16 ? prm.aparams + min(st.m0 + i, prm.M - 1)
                                          : prm.wparams + min((st.tile0 + ((i - 16) >> 4) * st.tstride) * kTileN + (i & 15), prm.N - 1);
            return *src;   // one unconditional load
        }
    };
    const RowParams par_first = load_par(min(st.tid, npar - 1));
    if constexpr (GQ) {
        // zero-points of the rows of A, less oa: of the lane's operand row (lane % 16) and of its four accumulator rows
        auto zc_of = [&](int row) -> int {
            const int m = min(st.m0 + row, prm.M - 1);
            const int z = RAW ? prm.a_zero[m] : prm.aparams[m].zero;
            return row < mt ? z - prm.oa : 0;
        };
        const int zb = (int)(((uint32_t)zc_of(r) & 0xFFu) * 0x01010101u);
        st.zc_op = v4i{zb, zb, zb, zb};
        st.zc128 = v4i{128 * zc_of(4 * G), 128 * zc_of(4 * G + 1), 128 * zc_of(4 * G + 2), 128 * zc_of(4 * G + 3)};
    }

    // ---- this wave's part of A: columns of its own super-chunks, in every row (wave-private: only this
    // wave reads what it writes, so no barrier is needed before the first MFMA).  A load instruction
    // covers two super-chunks of one row (2 x 32 vectors of 16 B); a batch is four rows of that.
    // RAW: unpacked codes with K a multiple of 16, so a 16-byte vector is either all inside the row or
    // all padding.  Valid bytes become a - oa (a xor 0x80 when q = 8), padding becomes 0, and lane `row`
    // keeps that row's partial sum over this wave's super-chunks.
    const int half = st.lane >> 5, vec = st.lane & 31;
    const uint8_t* a_base = RAW ? prm.a_raw + (size_t)st.m0 * prm.K : (const uint8_t*)prm.a_codes + (size_t)st.m0 * prm.Kp;
    const int a_ld = RAW ? prm.K : prm.Kp;
    const uint32_t flip = (RAW && prm.oa) ? 0x80808080u : 0u;
    const uint32_t qmask = prm.a_mask;   // RAW: bits above q are ignored, as the packers ignore them
    int32_t my_sum = 0;
    // column of A in global memory / in LDS for slot pr + half of the run [st.gs, st.ge) being staged
    auto batch_col = [&](int pr) { return (st.wave + (st.gs + min(pr + half, st.ge - st.gs - 1)) * st.S) * kSuperK + vec * 16; };
    auto batch_lds_col = [&](int pr) {
        if constexpr (!KG) return batch_col(pr);
        else return st.wave * prm.col_w + min(pr + half, st.ge - st.gs - 1) * prm.col_s + vec * 16;
    };
    auto batch_load = [&](int pr, int row0, uint4* areg) {
        const int col = batch_col(pr);
        const int colc = RAW ? min(col, prm.K - 16) : col;
#pragma unroll
        for (int u = 0; u < 4; ++u)   // row0 itself is always a row of A; the others are skipped when past mt (wave-uniform)
            if (u == 0 || row0 + u < mt) areg[u] = *reinterpret_cast<const uint4*>(a_base + (size_t)(row0 + u) * a_ld + colc);
    };
    auto batch_store = [&](int pr, int row0, const uint4* areg) {
        const int col = batch_col(pr);
        const int lcol = batch_lds_col(pr);
        const bool lv = pr + half < st.ge - st.gs;
        const bool inside = !RAW || col < prm.K;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u > 0 && row0 + u >= mt) break;   // wave-uniform
            uint4 v = areg[u];
            if constexpr (RAW) {
                v = uint4{v.x & qmask, v.y & qmask, v.z & qmask, v.w & qmask};
                {
                    uint32_t part = 0;
                    part = __builtin_amdgcn_udot4(v.x, 0x01010101u, part, false);
                    part = __builtin_amdgcn_udot4(v.y, 0x01010101u, part, false);
                    part = __builtin_amdgcn_udot4(v.z, 0x01010101u, part, false);
                    part = __builtin_amdgcn_udot4(v.w, 0x01010101u, part, false);
                    const int32_t tot = wave_sum((lv && inside) ? (int32_t)part : 0);
                    if (st.lane == row0 + u) my_sum += tot;
                }
                v = inside ? uint4{v.x ^ flip, v.y ^ flip, v.z ^ flip, v.w ^ flip} : uint4{0, 0, 0, 0};
            }
            if (lv) *reinterpret_cast<uint4*>(lds + (row0 + u) * prm.a_stride + lcol) = v;
        }
    };
    // The first batches (rows 0..7, or all 16 with R16, of the wave's first two super-chunks: all of A for
    // K <= 1024 * S) are loaded in straight-line code ahead of the weight stream, so that waiting for
    // them does not wait for the stream behind them.  (R16 is a variant of its own: the extra code costs
    // the single-token launches 2 %.)
    uint4 a0[4], a1[4], a2[4], a3[4];
    batch_load(0, 0, a0);
    const bool second = mt > 4, third = R16 && mt > 8, fourth = R16 && mt > 12;
    if (second) batch_load(0, 4, a1);
    if constexpr (R16) {
        if (third) batch_load(0, 8, a2);
        if (fourth) batch_load(0, 12, a3);
    }
    auto store_first = [&]() {
        batch_store(0, 0, a0);
        if (second) batch_store(0, 4, a1);
        if constexpr (R16) {
            if (third) batch_store(0, 8, a2);
            if (fourth) batch_store(0, 12, a3);
        }
    };

    // ---- the weight stream: first item = (tile0, super-chunk `wave`), then the rest of the ring
    u4v w[D][P + (GQ ? 1 : 0)];
    prefetch_item<P, KG, GQ>(prm, st, w[0]);
    if constexpr (FULL) {
        // every wave has at least D items: the whole ring is issued unconditionally, the number of
        // loads behind A is known, and the wait for A is exact
#pragma unroll
        for (int d = 1; d < D; ++d) prefetch_item<P, KG, GQ>(prm, st, w[d]);
        store_first();
    } else {
        // short streams: A is staged behind the first item only (again an exact wait), the rest of
        // the ring follows
        store_first();
#pragma unroll
        for (int d = 1; d < D; ++d)
            if (d < st.nitems) prefetch_item<P, KG, GQ>(prm, st, w[d]);
    }
    // whatever is left of A (more than two super-chunks per wave); with K groups also
    // every later run, staged over the columns of the run before it once that run's last tile is done
    auto stage_rest = [&](int first_row0) {
        for (int pr = 0; pr < st.ge - st.gs; pr += 2) {
            for (int row0 = (pr == 0 ? first_row0 : 0); row0 < mt; row0 += 4) {
                uint4 areg[4];
                batch_load(pr, row0, areg);
                batch_store(pr, row0, areg);
            }
        }
        if constexpr (RAW) {
            if (st.lane < 16) reinterpret_cast<int32_t*>(lds + prm.asum_off)[st.wave * 16 + st.lane] = my_sum;
        }
    };
    stage_rest(R16 ? 16 : 8);
    if (st.tid < npar) par[st.tid] = par_first;
    for (int i = st.tid + blockDim.x; i < npar; i += blockDim.x) par[i] = load_par(i);
    // MFMA rows past mt read a 512-byte block of zeros instead of A (every wave writes the same zeros,
    // so this needs no barrier either)
    if (st.lane < 32) *reinterpret_cast<uint4*>(lds + prm.zero_off + st.lane * 16) = uint4{0, 0, 0, 0};
    // same-wave LDS accesses execute in order; keep the compiler from moving the operand reads above
    // the staging writes (the parameters are read only after the first per-tile barrier)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    st.lds_lane = (r < mt ? lds + r * prm.a_stride : lds + prm.zero_off) + G * 16;
    st.k_mask = r < mt ? ~0 : 0;
    st.par = par;
    st.red = reinterpret_cast<int32_t*>(lds + prm.red_off);
    st.asum = reinterpret_cast<const int32_t*>(lds + prm.asum_off);
    st.part = reinterpret_cast<int32_t*>(lds + prm.part_off) + st.wave * prm.nmy_max * 256;
    auto next_group = [&]() {
        stage_rest(0);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
#pragma unroll
    for (int i = 0; i < GI::NACC; ++i) st.acc[i] = v4i{0, 0, 0, 0};
    st.facc = v4f{0.f, 0.f, 0.f, 0.f};
    auto compute = [&](const u4v* slot, const uint8_t* row) {
        if constexpr (GQ) compute_super_gq<P>(slot, row, st.zc_op, st.zc128, st.facc);
        else compute_super<P>(slot, row, st.acc);
    };

    int it = 0;
    if (!KG && nmy == 1) {
        // One tile per workgroup (the usual case): the K loop holds loads only, so the compiler's
        // waits are exact and P*(D-1) loads stay in flight; the tile is finished after the loop.
        for (; it + 2 * D <= st.nitems; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                compute(w[d], st.lds_lane + (((st.wave + st.lsc * st.S) * kSuperK) & st.k_mask));
                prefetch_item<P, false, GQ>(prm, st, w[d]);
                ++st.lsc;
            }
        }
        for (; it < st.nitems; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (it + d < st.nitems) {
                    compute(w[d], st.lds_lane + (((st.wave + st.lsc * st.S) * kSuperK) & st.k_mask));
                    if (it + d + D < st.nitems) prefetch_item<P, false, GQ>(prm, st, w[d]);
                    ++st.lsc;
                }
        }
        finish_tile<P, EPT, RAW, false, GQ>(prm, st);
    } else {
        // Several tiles per workgroup: the ring runs ahead across tile boundaries.
        for (; it + 2 * D <= st.nitems; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) item_step<P, EPT, RAW, KG, true, GQ>(prm, st, w[d], true, next_group);
        }
        for (; it < st.nitems; it += D) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (it + d < st.nitems) item_step<P, EPT, RAW, KG, false, GQ>(prm, st, w[d], it + d + D < st.nitems, next_group);
        }
    }
}

template <int P, int D, int EPT, bool RAW, bool FULL, bool KG, bool R16, bool GQ = false>
__global__ __launch_bounds__(512) void skinny_kernel(SkinnyParams prm)
{
    // workgroup b owns tl_q + (b < tl_r) tiles: b, b + gridDim.x, ...
    skinny_body<P, D, EPT, RAW, FULL, KG, R16, GQ>(prm, (int)blockIdx.x, (int)gridDim.x, prm.tl_q + ((int)blockIdx.x < prm.tl_r ? 1 : 0),
                                          (int)blockIdx.y);
}

// Grouped decode launch: up to kMaxGroup independent problems (same p, q and M <= 16; own A, W, Y, N, K)
// in ONE launch.  The 16-row tiles of all problems form one list (problem after problem); a resident set
// of workgroups cuts it into equal contiguous runs, and a workgroup streams its run problem by problem
// with the load ring running across the tiles of a problem (a run mostly lies inside one problem; where
// it crosses into the next, the workgroup drains, stages that problem's rows of A and goes on).
// Microsecond-sized matmuls then share one launch ramp and tail instead of paying one each (Sec. 3.4:
// the engine replaces all the linear layers of a decoder block).  Descriptors are read from the kernel
// arguments.
constexpr int kMaxGroup = 8;
constexpr int kTileOverheadCost = 16;  // fixed work per tile (sum over waves, epilogue), in units of one super-chunk
struct GroupedParams {
    int count;
    int first_tile[kMaxGroup + 1];    // where each problem's tiles start in the list
    // Two ways to cut the list into runs, as the host chooses.  by_work = 0: equal tile counts, workgroup b
    // owning run_q + (b < run_r) tiles.  by_work = 1: equal work; a tile of problem g costs its super-chunks +
    // a fixed overhead (a tile of a long-K problem is several tiles' worth of a short-K one), cost_first[g] is
    // the cost of all tiles before problem g, and workgroup b starts at the first tile whose preceding cost
    // reaches b * cost_per_wg.  Single precision is enough: neighbours evaluate the same expression for
    // their common boundary, so the runs tile the list whatever the rounding.
    int by_work, run_q, run_r;
    float cost_per_wg;
    float inv_tile_cost[kMaxGroup];
    float cost_first[kMaxGroup + 1];
    SkinnyParams d[kMaxGroup];
};

// Index in the tile list where the run of workgroup b (of n) starts; b = n gives the end of the list.
// (Select chains over constant indices instead of indexing by the problem found: the kernel arguments are
// then fetched with a few wide scalar loads up front rather than one dependent load after another.)
__host__ __device__ inline int grouped_run_start(const GroupedParams& gp, int b, int n)
{
    if (!gp.by_work) return b * gp.run_q + (b < gp.run_r ? b : gp.run_r);
    const float target = (float)b * gp.cost_per_wg;
    float cf = gp.cost_first[0], inv = gp.inv_tile_cost[0];
    int ft = gp.first_tile[0], ft_next = gp.first_tile[1];
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) {
        const bool in = i < gp.count && target >= gp.cost_first[i];
        cf = in ? gp.cost_first[i] : cf;
        inv = in ? gp.inv_tile_cost[i] : inv;
        ft = in ? gp.first_tile[i] : ft;
        ft_next = in ? gp.first_tile[i + 1] : ft_next;
    }
    const int within = (int)ceilf((target - cf) * inv);
    const int start = ft + (within < ft_next - ft ? within : ft_next - ft);
    return b >= n ? gp.first_tile[kMaxGroup] : start;
}

template <int P, int D, int EPT, bool RAW, bool GQ = false>
__global__ __launch_bounds__(512) void grouped_kernel(GroupedParams gp)
{
    const int b = (int)blockIdx.x;
    const int t0 = grouped_run_start(gp, b, (int)gridDim.x), t1 = grouped_run_start(gp, b + 1, (int)gridDim.x);
    bool first = true;
#pragma nounroll
    for (int g = 0; g < gp.count; ++g) {
        const int lo = max(t0, gp.first_tile[g]), hi = min(t1, gp.first_tile[g + 1]);
        if (lo >= hi) continue;   // the same for the whole workgroup
        if (!first) __syncthreads();   // every wave is done with the LDS contents of the problem before
        first = false;
        skinny_body<P, D, EPT, RAW, false, false, (EPT == 1 && !GQ), GQ>(gp.d[g], lo - gp.first_tile[g], 1, hi - lo, 0);
    }
}

template <int P, int D, int EPT, bool RAW, bool FULL, bool KG, bool R16, bool GQ = false>
static hipError_t launch_variant_r(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    static std::atomic<bool> attr_set{false};   // (an idempotent call: a lost race only repeats it)
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)skinny_kernel<P, D, EPT, RAW, FULL, KG, R16, GQ>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    skinny_kernel<P, D, EPT, RAW, FULL, KG, R16, GQ><<<grid, waves * 64, lds_bytes, s>>>(prm);
    return hipGetLastError();
}

// More than 8 rows of A per workgroup (only with four or more waves): the variant that loads all 16 rows ahead of the ring.
template <int P, int D, int EPT, bool RAW, bool FULL, bool KG>
static hipError_t launch_variant(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    if constexpr (EPT == 1) {
        if (prm.mrows > 8) return launch_variant_r<P, D, EPT, RAW, FULL, KG, true>(prm, grid, waves, lds_bytes, s);
    }
    return launch_variant_r<P, D, EPT, RAW, FULL, KG, false>(prm, grid, waves, lds_bytes, s);
}

template <int P, int D, int EPT>
static hipError_t launch_pde(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    if constexpr (EPT == 1) {   // K groups come with long K, hence with at least four waves
        if (prm.kgroups > 1)
            return prm.a_raw ? launch_variant<P, D, EPT, true, false, true>(prm, grid, waves, lds_bytes, s)
                             : launch_variant<P, D, EPT, false, false, true>(prm, grid, waves, lds_bytes, s);
    }
    if (prm.kgroups > 1) return hipErrorInvalidValue;
    const bool full = prm.tl_q * prm.sc_q >= D;   // the fewest items any wave has
    if (prm.a_raw)
        return full ? launch_variant<P, D, EPT, true, true, false>(prm, grid, waves, lds_bytes, s)
                    : launch_variant<P, D, EPT, true, false, false>(prm, grid, waves, lds_bytes, s);
    return full ? launch_variant<P, D, EPT, false, true, false>(prm, grid, waves, lds_bytes, s)
                : launch_variant<P, D, EPT, false, false, false>(prm, grid, waves, lds_bytes, s);
}

// Per-group weight parameters: one epilogue serves every workgroup size (instantiated as EPT = 1), no K groups.
// Ring depth, measured against deeper and shallower rings on one box (5120->13824, 11008<->4096, the LLaMA-7B
// block): four super-chunks at p <= 2 (eight spill), two above (at p = 3, 4 two beat four by 4-11 % in single
// launches and tie in the grouped launch).
__host__ __device__ constexpr int gq_depth(int p, int d) { return p <= 2 ? (d > 4 ? 4 : d) : (d > 2 ? 2 : d); }
template <int P, int D>
static hipError_t launch_gq(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    if (prm.kgroups > 1) return hipErrorInvalidValue;
    const bool full = prm.tl_q * prm.sc_q >= D;
    if (prm.a_raw)
        return full ? launch_variant_r<P, D, 1, true, true, false, false, true>(prm, grid, waves, lds_bytes, s)
                    : launch_variant_r<P, D, 1, true, false, false, false, true>(prm, grid, waves, lds_bytes, s);
    return full ? launch_variant_r<P, D, 1, false, true, false, false, true>(prm, grid, waves, lds_bytes, s)
                : launch_variant_r<P, D, 1, false, false, false, false, true>(prm, grid, waves, lds_bytes, s);
}

template <int P, int D>
static hipError_t launch_pd(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    if (prm.gparams) return launch_gq<P, gq_depth(P, D)>(prm, grid, waves, lds_bytes, s);
    if (waves >= 4) return launch_pde<P, D, 1>(prm, grid, waves, lds_bytes, s);
    if (waves == 2) return launch_pde<P, D, 2>(prm, grid, waves, lds_bytes, s);
    return launch_pde<P, D, 4>(prm, grid, waves, lds_bytes, s);
}

// Grouped launch on blobs with per-group weight parameters (all problems of a launch alike): one variant per
// activation form, any workgroup size.
template <int P, int D>
static hipError_t launch_grouped_gq(const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s)
{
    static std::atomic<bool> attr_set{false};   // (an idempotent call: a lost race only repeats it)
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 1, true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 1, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    if (raw) grouped_kernel<P, D, 1, true, true><<<grid, waves * 64, lds_bytes, s>>>(gp);
    else grouped_kernel<P, D, 1, false, true><<<grid, waves * 64, lds_bytes, s>>>(gp);
    return hipGetLastError();
}

template <int P, int D>
static hipError_t launch_grouped_pd(const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s)
{
    if (gp.d[0].gparams) return launch_grouped_gq<P, gq_depth(P, D)>(gp, raw, grid, waves, lds_bytes, s);
    static std::atomic<bool> attr_set{false};   // (an idempotent call: a lost race only repeats it)
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 1, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)grouped_kernel<P, D, 2, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    if (waves >= 4) {
        if (raw) grouped_kernel<P, D, 1, true><<<grid, waves * 64, lds_bytes, s>>>(gp);
        else grouped_kernel<P, D, 1, false><<<grid, waves * 64, lds_bytes, s>>>(gp);
    } else if (waves == 2) {
        if (raw) grouped_kernel<P, D, 2, true><<<grid, waves * 64, lds_bytes, s>>>(gp);
        else grouped_kernel<P, D, 2, false><<<grid, waves * 64, lds_bytes, s>>>(gp);
    } else {
        return hipErrorInvalidValue;   // (the plan never asks for one or three waves)
    }
    return hipGetLastError();
}

// Callers check gemm_grouped_fits first; count may exceed kMaxGroup (then several launches follow each other).
// Entry points of the per-width translation units (P_LO..P_HI each).
hipError_t skinny_launch_p12(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t skinny_launch_p34(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t skinny_launch_p56(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t skinny_launch_p78(int p, const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t grouped_launch_p12(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t grouped_launch_p34(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t grouped_launch_p56(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s);
hipError_t grouped_launch_p78(int p, const GroupedParams& gp, bool raw, unsigned grid, int waves, size_t lds_bytes, hipStream_t s);

}  // namespace abq
