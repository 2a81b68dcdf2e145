// Device code of the shared-operand decode kernel and the templates that launch its variants.  Included by the host
// translation unit (abq_shared_a.hip) and by the translation units that hold the instantiations.
//
// Decode-shaped matmul for 9 .. 16 rows of A over more 16-channel tiles of W than the chip has compute units (Sec. 3.4:
// the GEMV / small-batch case, bound by the weight stream).  With sixteen rows in use the MFMA's A operand has no spare
// rows to fill with further K slices, so a workgroup per tile (the direct kernel) would fetch the rows of A once per
// tile, sixteen times the weight bytes at p = 1.  Here there is one workgroup of sixteen waves per compute unit; the
// tiles are dealt out evenly (runs of T or T - 1 tiles) and the workgroup shares one copy of A among its run: its waves
// are a grid of (tile of the run) x (part of K).  Every wave requests its share of A (whole cache lines: eight rows x 128
// k per load), then all its weights (all loads up front, as in the direct kernel: no loop, no ring), writes its share of
// A to LDS in the MFMA operand's own layout (1 KiB per 64-k slice, lane L's 16 bytes at 16 L: one conflict-free 128-bit
// read per lane and MFMA), and after the one barrier multiplies its weights against operands read from LDS.  The partial
// tiles of the waves that share a tile meet in LDS (second barrier) and 256 threads per tile run the fused dequant
// epilogue (Fig. 3b).  Bit reduction (Sec. 3.4 step 5 / Appendix B) is the direct kernel's: the activation code rides as
// one int8, the weight side one plane group per accumulator set with the fields of a byte masked in place, recombined
// with shifts.  With sixteen waves on every unit the kernel is bound by the weight stream plus what each wave executes
// around it (every hundred vector instructions per wave are 0.7 us at this occupancy), so the prologue holds no division
// (the host works out the runs and the wave grid) and the row sums of A come from byte sums on the way to LDS.
#pragma once
#include "abq_direct_kernels.h"

#include <atomic>

namespace abq {

constexpr int kSharedAMaxQuads = 6;    // 16-byte loads of A per lane that a wave holds in registers while staging (one phase of K)
constexpr int kSharedAMaxQuads2 = 7;   // the same with two phases of K

struct SharedAParams {
    DirectProblem d;      // (rsplit: unused, the kernel derives it from its run of tiles)
    int M, oa, ow;
    uint32_t a_mask;      // (2^q - 1) in every byte (unpacked codes are masked to q bits)
    // The 16-channel tiles of W are dealt out evenly: the first nbig workgroups take runs of T tiles, the others T - 1.
    // Per kind of run (index 0: T tiles, 1: T - 1) the host works out the waves per tile, the super-chunks per wave and
    // a multiplier that divides a wave number by the waves per tile ((wave * inv) >> 8), so that the kernel's prologue
    // holds no division.
    int T, nbig;
    int H;                // super-chunks of K per phase (one phase: all of them)
    int wpt[2], rsplit[2], inv[2];
};

// Widest run of super-chunks per phase that a wave holds in registers without spilling: phases * R * p KiB of weights per
// wave beside its share of A, 128 registers per lane (sixteen waves per workgroup); the widths with two or three plane
// groups need more registers for the recombination.  Two phases exist for p = 1 and 2.
__host__ __device__ constexpr int shared_a_max_r(int p, int phases)
{
    if (phases == 2) return p == 1 ? 3 : (p == 2 ? 2 : 0);   // (p = 4 with two super-chunks per phase spills 60 bytes and loses to the streaming kernel)
    return p <= 2 ? 6 : (p == 3 ? 4 : (p == 4 ? 5 : (p <= 6 ? 3 : 2)));
}

// All MFMAs of one super-chunk for plane group GI: chunk c holds slices c*T .. c*T+T-1; the A operand of slice s is
// the lane's 16 bytes of LDS block s.
template <int P, int R, int GI, int C = 0, int T0 = 0>
__device__ __forceinline__ void shared_a_group_mfma(const u4v* w, const uint8_t* a_sc, v4i* acc)
{
    using SH = DirectShape<P, 16, R>;
    constexpr int B = SH::b(GI), T = SH::t(GI);
    if constexpr (C < B) {
        constexpr int s = C * T + T0;
        const v4i a = *reinterpret_cast<const v4i*>(a_sc + s * 1024);
        v4i& ac = acc[SH::acc_base(GI) + T0];
        ac = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, dfield_operand<B, T0>(w[SH::load_base(GI) + C]), ac, 0, 0, 0);
        if constexpr (T0 + 1 < T) shared_a_group_mfma<P, R, GI, C, T0 + 1>(w, a_sc, acc);
        else shared_a_group_mfma<P, R, GI, C + 1, 0>(w, a_sc, acc);
    }
}

template <int P, int R, int RR = 0>
__device__ __forceinline__ void shared_a_all_mfma(const u4v (*w)[P], const uint8_t* a_wave, v4i* acc, int nsc)
{
    using SH = DirectShape<P, 16, R>;
    if constexpr (RR < R) {
        if (RR < nsc) {
            shared_a_group_mfma<P, R, 0>(w[RR], a_wave + RR * 8 * 1024, acc);
            if constexpr (SH::NG > 1) shared_a_group_mfma<P, R, 1>(w[RR], a_wave + RR * 8 * 1024, acc);
            if constexpr (SH::NG > 2) shared_a_group_mfma<P, R, 2>(w[RR], a_wave + RR * 8 * 1024, acc);
        }
        shared_a_all_mfma<P, R, RR + 1>(w, a_wave, acc, nsc);
    }
}

// Requests a wave's share of one phase's A: units (eight rows x 128 k, whole cache lines: a pair of slices) wave, wave + S,
// ... of the phase's nunits, counted from unit0 of the problem; lane -> row 8 (unit & 1) + lane % 8, 16 k from 16 (lane /
// 8).  Rows past M: row M-1 again, their outputs are never stored.  The loads are unconditional, positions past the end
// clamped to valid ones, so that the wait counts stay exact.
template <bool RAW, int NAQ>
__device__ __forceinline__ void shared_a_load_a(const DirectProblem& pr, v4i* aq, int wave, int S, int unit0, int nunits, int M, int lane)
{
#pragma unroll
    for (int i = 0; i < NAQ; ++i) {
        const int u = unit0 + min(wave + i * S, nunits - 1);
        const int row = min(8 * (u & 1) + (lane & 7), M - 1);
        const int k = (u >> 1) * 128 + (lane >> 3) * 16;
        if constexpr (RAW) aq[i] = *reinterpret_cast<const v4i*>(pr.a_raw + (size_t)row * pr.K + min(k, pr.K - 16));
        else aq[i] = *reinterpret_cast<const v4i*>(pr.a_codes + (size_t)row * pr.Kp + k);
    }
}

// A -> LDS in the operand layout, [slice of the phase][k block of 16][row][16 bytes]: the lane's 16 bytes belong to slice
// 2 (unit / 2) + (lane / 8) / 4, k block (lane / 8) % 4, row as above; eight neighbouring lanes write 128 contiguous
// bytes.  RAW: unpacked codes -> operand bytes on the way (bits above q dropped, as the packers drop them, less oa; k past
// K stay zero) and the lane's codes are added up (all units of a wave lie in the same rows: S and unit0 are even).
template <bool RAW, int NAQ>
__device__ __forceinline__ void shared_a_store_a(const DirectProblem& pr, const v4i* aq, uint8_t* lds_a, int wave, int S, int unit0, int nunits, int lane,
                                                 uint32_t a_mask, uint32_t flip, uint32_t& code_sum)
{
    const int a_j = lane >> 3, a_row = lane & 7;
#pragma unroll
    for (int i = 0; i < NAQ; ++i) {
        const int ul = wave + i * S, u = unit0 + ul;
        v4i c = aq[i];
        if constexpr (RAW) {
            const bool live = ul < nunits && (u >> 1) * 128 + a_j * 16 < pr.K;
            const uint32_t m0 = live ? (uint32_t)c.x & a_mask : 0u, m1 = live ? (uint32_t)c.y & a_mask : 0u;
            const uint32_t m2 = live ? (uint32_t)c.z & a_mask : 0u, m3 = live ? (uint32_t)c.w & a_mask : 0u;
            code_sum = __builtin_amdgcn_sad_u8(m0, 0u, code_sum);
            code_sum = __builtin_amdgcn_sad_u8(m1, 0u, code_sum);
            code_sum = __builtin_amdgcn_sad_u8(m2, 0u, code_sum);
            code_sum = __builtin_amdgcn_sad_u8(m3, 0u, code_sum);
            c = live ? v4i{(int)(m0 ^ flip), (int)(m1 ^ flip), (int)(m2 ^ flip), (int)(m3 ^ flip)} : v4i{0, 0, 0, 0};
        }
        if (ul < nunits)
            *reinterpret_cast<v4i*>(lds_a + (size_t)(2 * (ul >> 1) + (a_j >> 2)) * 1024 + (a_j & 3) * 256 + (8 * (ul & 1) + a_row) * 16) = c;
    }
}

// The weights of a wave's run of super-chunks from sc_first: unconditional loads (a wave with fewer than R super-chunks
// re-reads its last one, or the problem's last one), so that the wait counts in front of them are exact.
template <int P, int R>
__device__ __forceinline__ void shared_a_load_w(const DirectProblem& pr, u4v (*w)[P], int tile, int sc_first, int lane)
{
    using SH = DirectShape<P, 16, R>;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int sc = min(sc_first + rr, pr.nsuper - 1);
#pragma unroll
        for (int gi = 0; gi < SH::NG; ++gi) {
            const int b = SH::b(gi);
            const u4v* base = pr.fields[gi] + ((size_t)tile * pr.nsuper + sc) * (b * 64) + lane;
#pragma unroll
            for (int i = 0; i < b; ++i) w[rr][SH::load_base(gi) + i] = __builtin_nontemporal_load(base + i * 64);
        }
    }
}

// R: super-chunks (512 k) per wave and phase at most.  PH: phases of K (1: all of A fits LDS; 2: K is cut at gp.H
// super-chunks and the halves of A take turns in LDS — the second half is requested while the first is multiplied, and
// the weights of both phases are requested at the start).  RAW: the activation BitPacking step is fused in (Fig. 3b): A
// arrives as unpacked codes, is masked to q bits and offset to signed bytes on its way to LDS, and the row sums of the
// codes for the zero-point correction are taken on the way (byte sums per lane, three lane exchanges, one partial per
// wave and row).
template <int P, int R, bool RAW, int PH>
__global__ __launch_bounds__(1024) void shared_a_kernel(SharedAParams gp)
{
    using SH = DirectShape<P, 16, R>;
    constexpr int NAQ = PH == 1 ? kSharedAMaxQuads : kSharedAMaxQuads2;
    extern __shared__ __align__(16) uint8_t lds_raw[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, G = lane >> 4;
    const DirectProblem pr = gp.d;
    const int S = (int)blockDim.x >> 6;
    asm volatile("" ::"s"(pr.fields[0]), "s"(pr.fields[1]), "s"(pr.fields[2]), "s"(pr.wparams), "s"(pr.y), "s"(pr.acc), "s"(pr.rq.codes), "s"(pr.N), "s"(pr.K),
                 "s"(gp.oa), "s"(gp.ow), "s"(gp.a_mask), "s"(S), "s"(gp.T), "s"(gp.nbig), "s"(gp.H));
    if constexpr (RAW) asm volatile("" ::"s"(pr.a_raw), "s"(pr.a_scale), "s"(pr.a_zero));
    else asm volatile("" ::"s"(pr.a_codes), "s"(pr.aparams));
    const int M = gp.M, nsuper = pr.nsuper, H = gp.H;
    // this workgroup's run of tiles (the tiles are dealt out evenly: runs differ by one at most) and its waves as a grid
    // of (tile of the run) x (part of K)
    const int b = (int)blockIdx.x, kind = b < gp.nbig ? 0 : 1;
    const int first = kind == 0 ? b * gp.T : gp.nbig * gp.T + (b - gp.nbig) * (gp.T - 1);
    const int cnt = gp.T - kind;
    const int wpt = gp.wpt[kind];                                        // waves per tile
    const int rsplit = gp.rsplit[kind];                                  // super-chunks per wave and phase (<= R)
    const int ti = (wave * gp.inv[kind]) >> 8, kpart = wave - ti * wpt;
    const int tile = first + min(ti, cnt - 1);                           // (a wave past the run: a valid tile again, nothing kept)
    const int scl = kpart * rsplit;                                      // this wave's first super-chunk inside a phase
    uint8_t* lds_a = lds_raw;                                            // one phase of A: [8 H slices][4 k blocks][16 rows][16 bytes]: slice s = 1 KiB, lane (r, G) of the operand at 256 G + 16 r
    int32_t* red = reinterpret_cast<int32_t*>(lds_raw + (size_t)H * 8192);   // [S][16 rows][16 channels]
    int32_t* reda = red + S * 256;                                       // [S][8 rows] partial row sums of A (RAW): wave w holds rows 8 (w & 1) ..

    // ---- epilogue parameters of this thread's first output (requested first, used after the last barrier):
    // thread t -> tile t >> 8 of the run, row (t >> 4) & 15, channel t & 15
    const int t0 = (int)threadIdx.x;
    RowParams pa0{0, 0.f, 0, 0}, pw0{0, 0.f, 0, 0};
    {
        const int m = min((t0 >> 4) & 15, M - 1);
        const int n = min((first + (t0 >> 8)) * kTileN + (t0 & 15), pr.N - 1);
        if constexpr (RAW) pa0 = RowParams{0, pr.a_scale[m], pr.a_zero[m], 0};
        else pa0 = pr.aparams[m];
        pw0 = pr.wparams[n];
    }

    // ---- every load of the first phase, and the weights of the second: A first, so that the wait for it leaves the
    // weights in flight
    const int n0 = min(H, nsuper), n1 = nsuper - n0;                     // super-chunks of the two phases
    v4i aq[NAQ];
    shared_a_load_a<RAW, NAQ>(pr, aq, wave, S, 0, 8 * n0, M, lane);
    u4v w[PH][R][P];
    shared_a_load_w<P, R>(pr, w[0], tile, scl, lane);
    if constexpr (PH == 2) shared_a_load_w<P, R>(pr, w[1], tile, H + scl, lane);
    const uint32_t flip = gp.oa ? 0x80808080u : 0u;
    uint32_t code_sum = 0;
    shared_a_store_a<RAW, NAQ>(pr, aq, lds_a, wave, S, 0, 8 * n0, lane, gp.a_mask, flip, code_sum);
    if constexpr (RAW && PH == 1) {
        // the row sums of the codes for the zero-point correction: lanes L, L + 8, ... hold parts of the same row
        code_sum += __shfl_xor(code_sum, 8);
        code_sum += __shfl_xor(code_sum, 16);
        code_sum += __shfl_xor(code_sum, 32);
        if (lane < 8) reda[wave * 8 + lane] = (int32_t)code_sum;
    }
    __syncthreads();
    if constexpr (PH == 2) shared_a_load_a<RAW, NAQ>(pr, aq, wave, S, 8 * H, 8 * max(n1, 1), M, lane);   // (in flight under the MFMAs)

    // ---- multiply
    const uint8_t* a_wave = lds_a + (size_t)scl * 8 * 1024 + lane * 16;
    v4i acc[SH::NACC];
#pragma unroll
    for (int i = 0; i < SH::NACC; ++i) acc[i] = v4i{0, 0, 0, 0};
    shared_a_all_mfma<P, R>(w[0], a_wave, acc, ti < cnt ? max(0, min(rsplit, n0 - scl)) : 0);
    if constexpr (PH == 2) {
        __syncthreads();                                                 // every wave is done with the first half of A
        shared_a_store_a<RAW, NAQ>(pr, aq, lds_a, wave, S, 8 * H, 8 * n1, lane, gp.a_mask, flip, code_sum);
        if constexpr (RAW) {
            code_sum += __shfl_xor(code_sum, 8);
            code_sum += __shfl_xor(code_sum, 16);
            code_sum += __shfl_xor(code_sum, 32);
            if (lane < 8) reda[wave * 8 + lane] = (int32_t)code_sum;
        }
        __syncthreads();
        shared_a_all_mfma<P, R>(w[1], a_wave, acc, ti < cnt ? max(0, min(rsplit, n1 - scl)) : 0);
    }

    // ---- bit reduction over fields and plane groups; lane (G, reg) holds row 4G + reg, channel r
    v4i accI[1] = {v4i{0, 0, 0, 0}};
    direct_fold<P, 16, R, 0>(acc, accI);
    if constexpr (SH::NG > 1) direct_fold<P, 16, R, 1>(acc, accI);
    if constexpr (SH::NG > 2) direct_fold<P, 16, R, 2>(acc, accI);
#pragma unroll
    for (int i = 0; i < 4; ++i) red[(wave * 16 + 4 * G + i) * 16 + r] = accI[0][i];
    __syncthreads();

    // ---- sum over the waves of a tile, fused dequant epilogue
    for (int t = t0; t < cnt * 256; t += (int)blockDim.x) {
        const int tw = t >> 8, m = (t >> 4) & 15, nl = t & 15;
        const int n = (first + tw) * kTileN + nl;
        if (m >= M || n >= pr.N) continue;
        int32_t sum = 0;
        for (int kk = 0; kk < wpt; ++kk) sum += red[((tw * wpt + kk) * 16 + m) * 16 + nl];
        RowParams pa = pa0, pw = pw0;
        if (t != t0) {
            if constexpr (RAW) pa = RowParams{0, pr.a_scale[m], pr.a_zero[m], 0};
            else pa = pr.aparams[m];
            pw = pr.wparams[n];
        }
        if constexpr (RAW) {
            int32_t as = 0;
            for (int ww = m >> 3; ww < S; ww += 2) as += reda[ww * 8 + (m & 7)];
            pa.sum = as;   // sum of the row's codes (rows past M are never stored)
        }
        epilogue_store(sum, gp.oa, gp.ow, pr.K, pa, pw, (size_t)m * pr.N + n, pr.y, pr.acc, pr.rq, m);
    }
}

inline size_t shared_a_lds_bytes(int H, int S) { return (size_t)H * 8192 + (size_t)S * 1024 + (size_t)S * 64; }   // H: super-chunks per phase

template <int P, int R, bool RAW, int PH>
static hipError_t shared_a_launch_one(const SharedAParams& gp, unsigned grid, int waves, hipStream_t s)
{
    static std::atomic<bool> attr_set{false};   // (an idempotent call: a lost race only repeats it)
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute((const void*)shared_a_kernel<P, R, RAW, PH>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    shared_a_kernel<P, R, RAW, PH><<<grid, waves * 64, shared_a_lds_bytes(gp.H, waves), s>>>(gp);
    return hipGetLastError();
}

template <int P, int PH, int R = 1>
static hipError_t shared_a_launch_r(const SharedAParams& gp, int Rwant, bool raw, unsigned grid, int waves, hipStream_t s)
{
    if constexpr (R > shared_a_max_r(P, PH)) return hipErrorInvalidValue;
    else {
        if (Rwant == R) return raw ? shared_a_launch_one<P, R, true, PH>(gp, grid, waves, s) : shared_a_launch_one<P, R, false, PH>(gp, grid, waves, s);
        return shared_a_launch_r<P, PH, R + 1>(gp, Rwant, raw, grid, waves, s);
    }
}

template <int P>
static hipError_t shared_a_launch_p(const SharedAParams& gp, int phases, int Rwant, bool raw, unsigned grid, int waves, hipStream_t s)
{
    return phases == 2 ? shared_a_launch_r<P, 2>(gp, Rwant, raw, grid, waves, s) : shared_a_launch_r<P, 1>(gp, Rwant, raw, grid, waves, s);
}

// Entry points of the per-width translation units.
hipError_t shared_a_launch_p1234(int p, const SharedAParams& gp, int phases, int R, bool raw, unsigned grid, int waves, hipStream_t s);
hipError_t shared_a_launch_p5678(int p, const SharedAParams& gp, int phases, int R, bool raw, unsigned grid, int waves, hipStream_t s);

}  // namespace abq
