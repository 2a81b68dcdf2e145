// Prefill-shaped matmul (M > 16): a dense int8 contraction on the 16x16x64 MFMA.
//
// Workgroup tile (16*MT rows of A) x (64*NTW rows of W), four waves side by side along N, each owning
// NTW 16-row tiles of W for all rows of A (MT x NTW accumulator tiles).  The packed weight plane
// groups go from HBM straight into registers in the same tiled layout the decode kernel streams
// (one 256-k phase ahead) and are expanded there: for every 64-k slice the fields of all groups are
// shifted to their bit position and OR-ed into one signed byte per weight, so a slice costs one
// MFMA per accumulator tile whatever p is.  (This is the bit reduction of Sec. 3.4 step 5 /
// Appendix B folded into the operand: the 2^s factors are bit positions inside the byte, the 2^t
// factors are the activation code itself.)  The rows of A go from global memory straight into LDS
// (direct 128-bit loads, XOR-swizzled so that operand reads have no bank conflicts) in 256-k steps,
// double buffered, one barrier per step.  The dequant epilogue is fused (Fig. 3b) and leaves
// through LDS so that rows of Y are written in 16-byte pieces.
#include "abq_internal.h"
#include "../../include/abq.h"

#include <stdlib.h>
#include <type_traits>

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

// Tile shape: MT 16-row tiles of A per workgroup (4 or 8: 64 or 128 rows), NTW 16-row tiles of W per
// wave (1, 2 or 4: workgroup covers 64, 128 or 256 rows of W).  Narrow shapes give more workgroups
// when M and N are small; wide ones reuse each A operand read for more MFMAs.
constexpr int kStepK = 256;          // one step = one phase = four 64-k slices
constexpr int kARow = kStepK;        // LDS row stride (unpadded; the 16-B vectors of a row are XOR-swizzled by the row index)


struct TiledParams {
    const u4v* fields[3];
    const int8_t* a_codes;
    const RowParams* aparams;
    const RowParams* wparams;
    uint16_t* y;              // may be null when rq.codes is given
    int32_t* acc;
    Requant rq;               // output codes of the next layer (codes == null: off)
    int M, N, K, Kp, nsuper, ntiles;
    int oa, ow;
    const u4v* gparams;       // per-group weight parameters (g128 blobs; null otherwise): [ntiles][nsuper][16 channels] records
    int tiles_m, tiles_n;     // workgroup tiles along M and N (1-D grid of tiles_m * tiles_n workgroups)
    int band_m;               // row blocks per band of the tile order (see the kernel's tile mapping)
    int narrow_sums;          // 1: every row sum of codes is below 2^23 (the epilogue then multiplies at the 24-bit rate)
};

// Weights are held one phase (half a super-chunk, 256 k, four 64-k slices) at a time.  A b-bit
// group needs max(b/2, 1) of its 1 KiB chunks per phase (a 1-bit chunk spans both phases and is
// simply fetched for each).
__host__ __device__ constexpr int phase_chunks(int b) { return b >= 2 ? b / 2 : 1; }
__host__ __device__ constexpr int phase_base(int p, int g)
{
    return g == 0 ? 0 : (g == 1 ? phase_chunks(group_width(p, 0)) : phase_chunks(group_width(p, 0)) + phase_chunks(group_width(p, 1)));
}
__host__ __device__ constexpr int phase_regs(int p) { return phase_base(p, group_count(p) - 1) + phase_chunks(group_width(p, group_count(p) - 1)); }

// Operand dword of k-slice `SL` (0..7 inside a super-chunk) for one 16-row tile: all plane groups
// merged into one byte per weight.  `w` is the tile's register set of the phase SL/4.
template <int P, int SL, int G0 = 0>
__device__ __forceinline__ uint32_t merged_dword(const u4v* w, int j)
{
    constexpr int b = group_width(P, G0), shift = group_shift(P, G0), T = 8 / b;
    constexpr int chunk = SL / T, t = SL % T;
    constexpr int local = b == 1 ? 0 : chunk - phase_chunks(b) * (SL / 4);
    const uint32_t x = w[phase_base(P, G0) + local][j];
    uint32_t v;
    if constexpr (b == 8) {
        v = x;
    } else {
        constexpr int sh = b * t - shift;
        constexpr uint32_t mask = (((1u << b) - 1u) * 0x01010101u) << shift;
        if constexpr (sh > 0) v = (x >> sh) & mask;
        else if constexpr (sh < 0) v = (x << (-sh)) & mask;
        else v = x & mask;
    }
    if constexpr (G0 + 1 < group_count(P)) v |= merged_dword<P, SL, G0 + 1>(w, j);
    return v;
}

template <int P, int SL>
__device__ __forceinline__ v4i merged_operand(const u4v* w)
{
    v4i r;
    r.x = (int)merged_dword<P, SL>(w, 0);
    r.y = (int)merged_dword<P, SL>(w, 1);
    r.z = (int)merged_dword<P, SL>(w, 2);
    r.w = (int)merged_dword<P, SL>(w, 3);
    return r;
}

// A tile in LDS: [128 rows][16 vectors of 16 B], vector v of row `row` stored at position v ^ (row & 15),
// so that the 16 rows an operand read touches (same v) land in 16 different 16-byte bank groups.
// Lane (r = lane%16, G = lane/16) reads, for m-tile mt and slice sl, vector 4*sl + G of row 16*mt + r.
template <int MT>
__device__ __forceinline__ void read_a_operands(const uint8_t* a_buf, int r, int G, int sl, v4i* aop)
{
    const uint8_t* p = a_buf + r * kARow + (((4 * sl + G) ^ r) << 4);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) aop[mt] = *reinterpret_cast<const v4i*>(p + mt * 16 * kARow);
}

template <int P, int NTW, int MT, int SL>
__device__ __forceinline__ void slice_mfma(const u4v (*w)[phase_regs(P)], const v4i* aop, v4i (*acc)[NTW])
{
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const v4i bop = merged_operand<P, SL>(w[nt]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[mt], bop, acc[mt][nt], 0, 0, 0);
    }
}

// The four 64-k slices of one step (phase PH of a super-chunk): the A operands of two slices are
// requested from LDS, then their 2 x 32 MFMAs run as one uninterrupted burst.  The scheduling
// barriers pin that order: left alone, the machine scheduler sinks the reads next to their uses
// and the matrix pipe idles on every wait.
template <int P, int NTW, int MT, int PH>
__device__ __forceinline__ void step_mfma(const u4v (*w)[phase_regs(P)], const uint8_t* a_buf, int r, int G, v4i (*acc)[NTW])
{
    v4i a0[MT], a1[MT];
    read_a_operands<MT>(a_buf, r, G, 0, a0);
    read_a_operands<MT>(a_buf, r, G, 1, a1);
    __builtin_amdgcn_sched_barrier(0);
    slice_mfma<P, NTW, MT, 4 * PH + 0>(w, a0, acc);
    __builtin_amdgcn_sched_barrier(0);
    read_a_operands<MT>(a_buf, r, G, 2, a0);      // (travels under the MFMAs of slice 1)
    __builtin_amdgcn_sched_barrier(0);
    slice_mfma<P, NTW, MT, 4 * PH + 1>(w, a1, acc);
    __builtin_amdgcn_sched_barrier(0);
    read_a_operands<MT>(a_buf, r, G, 3, a1);      // (under those of slice 2)
    __builtin_amdgcn_sched_barrier(0);
    slice_mfma<P, NTW, MT, 4 * PH + 2>(w, a0, acc);
    slice_mfma<P, NTW, MT, 4 * PH + 3>(w, a1, acc);
    __builtin_amdgcn_sched_barrier(0);
}

// Loads phase `ph` (0 or 1) of super-chunk `sc` for this wave's tiles.
template <int P, int NTW>
__device__ __forceinline__ void load_tiles(const TiledParams& prm, int tile0, int sc, int ph, int lane, u4v (*w)[phase_regs(P)])
{
    // tile0, sc and ph are wave-uniform: the chunk base is a scalar address, the lane adds 16*lane
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const int tile = min(tile0 + nt, prm.ntiles - 1);   // past the last tile: re-read a valid one, never stored
#pragma unroll
        for (int g = 0; g < group_count(P); ++g) {
            const int b = group_width(P, g), cpp = phase_chunks(b);
            const int first = b == 1 ? 0 : cpp * ph;
            const u4v* base = prm.fields[g] + (((size_t)tile * prm.nsuper + sc) * b + first) * 64;
#pragma unroll
            for (int i = 0; i < cpp; ++i) w[nt][phase_base(P, g) + i] = base[i * 64 + lane];
        }
    }
}

// Up to two 16-row tiles of W per wave the kernel is held to 256 registers, so that two workgroups
// share a CU and each hides the other's waits; the four-tile shape takes the whole register file.
// WD = steps of operands in flight per wave: 2 (the next step is fetched while the current one is multiplied)
// or 4 (weights and rows of A three steps ahead, both through registers: for the small tile shapes on
// problems with few workgroups, where a step's MFMAs are much shorter than a load's latency and the K loop
// would otherwise advance one load latency per step).
template <int P, int NTW, int MT, int WD>
__global__ __launch_bounds__(256, (WD == 4 ? 2 : (NTW <= 2 ? (MT == 4 ? 3 : 2) : (MT == 4 ? 2 : 1)))) void tiled_kernel(TiledParams prm)
{
    constexpr int kBM = MT * 16, kBN = 4 * NTW * kTileN;
    __shared__ __align__(16) uint8_t lds_a0[kBM * kARow];   // two separate objects: the loads that fill one must
    __shared__ __align__(16) uint8_t lds_a1[kBM * kARow];   // not be taken to alias the reads of the other
    __shared__ RowParams par_a[kBM], par_w[kBN];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps the weight addresses scalar
    const int r = lane & 15, G = lane >> 4;
    // Workgroup b runs on XCD b % 8 (round-robin dispatch) and each XCD has its own L2.  Give every
    // XCD a contiguous run of the tile order.  The order goes band by band (band_m row blocks of A), and
    // inside a band column block by column block with M fastest: the workgroups resident on one XCD then
    // cover band_m row blocks of A times a few column blocks of W and share both through that L2.  A band
    // of all row blocks would make every XCD stream the whole of A once per handful of column blocks.
    const int nwg = prm.tiles_m * prm.tiles_n;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;                     // XCD x owns per + (x < rem) workgroups
    const int vid = xcd * per + min(xcd, rem) + slot;
    const int band = vid / (prm.band_m * prm.tiles_n), in_band = vid - band * prm.band_m * prm.tiles_n;
    const int band_rows = min(prm.band_m, prm.tiles_m - band * prm.band_m);
    const int m_blk = band * prm.band_m + in_band % band_rows, n_blk = in_band / band_rows;
    const int m0 = m_blk * kBM, n0 = n_blk * kBN;
    const int tile0 = n_blk * (kBN / kTileN) + wave * NTW;

    // weights of the first phase (WD = 2) or the first three (WD = 4)
    u4v wa[NTW][phase_regs(P)], wb[NTW][phase_regs(P)];
    u4v wc[WD == 4 ? NTW : 1][phase_regs(P)], wd[WD == 4 ? NTW : 1][phase_regs(P)];
    const int nsteps = prm.nsuper * 2;
    auto load_phase = [&](int j, u4v (*w)[phase_regs(P)]) {   // phase j of the K loop, clamped to the last one
        const int jc = min(j, nsteps - 1);
        load_tiles<P, NTW>(prm, tile0, jc >> 1, jc & 1, lane, w);
    };
    load_tiles<P, NTW>(prm, tile0, 0, 0, lane, wa);
    if constexpr (WD == 4) {
        load_phase(1, wb);
        load_phase(2, wc);
    }

    // epilogue parameters
    if (tid < kBM) par_a[tid] = prm.aparams[min(m0 + tid, prm.M - 1)];
    if (tid < kBN) par_w[tid] = prm.wparams[min(n0 + tid, prm.N - 1)];

    // A tile of one 256-k step goes from global memory straight into LDS (128-bit direct loads, no
    // registers in between): wave w issues loads j = MT*w .. MT*w+MT-1, load j fills rows 4j .. 4j+3 (1 KiB,
    // lane L -> LDS position 16*L of that KiB = row 4j + L/16, position L%16, which holds vector
    // (L%16) ^ (row & 15) of the row).  Rows past M re-read row M-1; their outputs are never stored.
    unsigned a_goff[MT];
#pragma unroll
    for (int u = 0; u < MT; ++u) {
        const int row = 4 * (wave * MT + u) + (lane >> 4);
        const int vec = (lane & 15) ^ (row & 15);
        a_goff[u] = (unsigned)(min(m0 + row, prm.M - 1) - m0) * (unsigned)prm.Kp + vec * 16;
    }
    const int8_t* a_tile = prm.a_codes + (size_t)m0 * prm.Kp;   // uniform
    auto a_prefetch = [&](int step, uint8_t* buf) {
        const int8_t* base = a_tile + (size_t)step * kStepK;     // uniform
#pragma unroll
        for (int u = 0; u < MT; ++u)
            __builtin_amdgcn_global_load_lds((const void*)(base + a_goff[u]),
                                             (__attribute__((address_space(3))) void*)(buf + (wave * MT + u) * 1024), 16, 0, 0);
    };

    v4i acc[MT][NTW];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) acc[mt][nt] = v4i{0, 0, 0, 0};

    // A wave's direct loads into an LDS buffer have to have landed before the wave enters the barrier behind which the other
    // waves read that buffer.  The barrier's own fence covers LDS instructions, not these loads, so the wait is written out
    // here and in the loop (the compiler usually places its own wait for the weight registers there too, but need not).
    a_prefetch(0, lds_a0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    if constexpr (WD == 4) {
        // two super-chunks per iteration, four steps; in every step the A tile of the next step is requested
        // first and the weights of the step three ahead after it, so that the wait for A before the barrier
        // leaves those weights in flight
        // Here the A tiles travel through registers (global -> VGPR three steps ahead, VGPR -> LDS after the
        // MFMAs of the step before their own) instead of straight into LDS: the compiler waits for direct loads
        // with vmcnt(0) before a barrier, which would drain the rings every step, whereas for register loads
        // its wait counts are exact and leave the younger loads in flight.
        u4v ar0[MT], ar1[MT], ar2[MT], ar3[MT];
#define ABQ_A_LOAD(STEP, AR)                                                                       \
        {                                                                                          \
            const int8_t* a_src = a_tile + (size_t)min((STEP), nsteps - 1) * kStepK;               \
            _Pragma("unroll") for (int u = 0; u < MT; ++u)                                         \
                AR[u] = *reinterpret_cast<const u4v*>(a_src + a_goff[u]);                          \
        }
        ABQ_A_LOAD(1, ar1)
        ABQ_A_LOAD(2, ar2)
#define ABQ_STEP(J, W_NEXT, W_CUR, PH, BUF_CUR, BUF_NEXT, AR_LOAD, AR_STORE)                   \
        {                                                                                          \
            ABQ_A_LOAD((J) + 3, AR_LOAD)                                                           \
            load_phase((J) + 3, W_NEXT);                                                           \
            __builtin_amdgcn_sched_barrier(0);                                                     \
            step_mfma<P, NTW, MT, PH>(W_CUR, BUF_CUR, r, G, acc);                                  \
            _Pragma("unroll") for (int u = 0; u < MT; ++u)                                         \
                *reinterpret_cast<u4v*>(BUF_NEXT + (wave * MT + u) * 1024 + lane * 16) = AR_STORE[u]; \
            __syncthreads();                                                                       \
        }
        for (int sc = 0; sc < prm.nsuper; sc += 2) {
            const int j = 2 * sc;
            ABQ_STEP(j, wd, wa, 0, lds_a0, lds_a1, ar3, ar1)
            ABQ_STEP(j + 1, wa, wb, 1, lds_a1, lds_a0, ar0, ar2)
            if (sc + 1 < prm.nsuper) {   // (the same for every thread)
                ABQ_STEP(j + 2, wb, wc, 0, lds_a0, lds_a1, ar1, ar3)
                ABQ_STEP(j + 3, wc, wd, 1, lds_a1, lds_a0, ar2, ar0)
            }
        }
#undef ABQ_STEP
#undef ABQ_A_LOAD
    } else
    // one super-chunk per iteration: two steps (= phases) of four 64-k slices; the weights and the A
    // tile of the next step are fetched while the current one is multiplied.  Loads past the end are
    // clamped to the last step instead of being skipped, so that every load in the loop is unconditional.
    for (int sc = 0; sc < prm.nsuper; ++sc) {
        const int scn = min(sc + 1, prm.nsuper - 1);
        {   // step 2*sc: weights in wa, A in buffer 0
            load_tiles<P, NTW>(prm, tile0, sc, 1, lane, wb);
            a_prefetch(2 * sc + 1, lds_a1);
            step_mfma<P, NTW, MT, 0>(wa, lds_a0, r, G, acc);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        {   // step 2*sc+1: weights in wb, A in buffer 1
            load_tiles<P, NTW>(prm, tile0, scn, 0, lane, wa);
            a_prefetch(min(2 * sc + 2, nsteps - 1), lds_a0);
            step_mfma<P, NTW, MT, 1>(wb, lds_a1, r, G, acc);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    }

    // Fused epilogue.  Lane l, register reg of accumulator tile (mt, nt) is row 16*mt + 4*(l/16) + reg,
    // column 16*nt + l%16.  The fp16 values are transposed through LDS (the A buffers are free now; waves
    // 0,1 use the first, waves 2,3 the second) so that each lane then stores 16 contiguous bytes of a row
    // of Y instead of 2: full 32..128-byte row segments per wave instead of scattered halves.
    __syncthreads();   // every wave is done reading A
    constexpr int kWCols = NTW * kTileN;                       // columns of Y this wave owns
    uint16_t* stage = reinterpret_cast<uint16_t*>((wave < 2 ? lds_a0 : lds_a1) + (wave & 1) * (kBM * kWCols * 2));
    // Eq. 3's affine dequant in the integers, with everything that depends on the row or on the column alone taken out of
    // the element loop:  raw = S + ow sumA + oa sumW - K oa ow  (the sum over the codes themselves; S is over the stored,
    // offset operands) and centered = raw - wz sumA - az (sumW - K wz), all modulo 2^32 as in epilogue_value.  That
    // leaves two multiplies per element.  32-bit integer multiplies run at a quarter of the vector rate and made this
    // epilogue a third of a prefill launch; where every factor fits 24 bits (sums of codes below 2^23: the host checks
    // K (2^p - 1) and K (2^q - 1)) the 24-bit multiply-add gives the same low 32 bits at the full rate.
    RowParams pw[NTW];
    int32_t col_raw[NTW], col_cw[NTW], col_nwz[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        pw[nt] = par_w[wave * kWCols + nt * 16 + r];
        col_raw[nt] = (int32_t)((uint32_t)prm.oa * (uint32_t)pw[nt].sum - (uint32_t)prm.K * (uint32_t)prm.oa * (uint32_t)prm.ow);
        col_cw[nt] = (int32_t)((uint32_t)pw[nt].sum - (uint32_t)prm.K * (uint32_t)pw[nt].zero);
        col_nwz[nt] = -pw[nt].zero;
    }
    auto dequant_tile = [&](auto narrow, auto plain) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int ml = mt * 16 + 4 * G + reg;
                const int m = m0 + ml;
                const RowParams pa = par_a[ml];
                const int32_t row_raw = (int32_t)((uint32_t)prm.ow * (uint32_t)pa.sum), naz = -pa.zero;
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    const int32_t raw = (int32_t)((uint32_t)acc[mt][nt][reg] + (uint32_t)row_raw + (uint32_t)col_raw[nt]);
                    int32_t centered;
                    if constexpr (decltype(narrow)::value)
                        centered = __mul24(naz, col_cw[nt]) + (__mul24(col_nwz[nt], pa.sum) + raw);
                    else
                        centered = (int32_t)((uint32_t)raw + (uint32_t)col_nwz[nt] * (uint32_t)pa.sum + (uint32_t)naz * (uint32_t)col_cw[nt]);
                    const float v = ((float)centered * pa.scale) * pw[nt].scale;
                    uint32_t hv;
                    asm("v_cvt_f16_f32 %0, %1" : "=v"(hv) : "v"(v));   // (the instruction itself: see epilogue_value)
                    const uint16_t h = (uint16_t)hv;
                    stage[ml * kWCols + nt * 16 + r] = h;
                    if constexpr (!decltype(plain)::value) {
                        const int n = n0 + wave * kWCols + nt * 16 + r;
                        if (prm.acc && m < prm.M && n < prm.N) prm.acc[(size_t)m * prm.N + n] = raw;
                        if (prm.rq.codes && m < prm.M && n < prm.N)
                            prm.rq.codes[(size_t)m * prm.N + n] = requant_code(h, prm.rq.scale[m], prm.rq.zero[m], prm.rq.qmax);
                    }
                }
            }
        }
    };
    const bool plain_out = prm.acc == nullptr && prm.rq.codes == nullptr;   // (the same for every thread, as is narrow_sums)
    if (prm.narrow_sums && plain_out) dequant_tile(std::true_type{}, std::true_type{});
    else if (prm.narrow_sums) dequant_tile(std::true_type{}, std::false_type{});
    else dequant_tile(std::false_type{}, std::false_type{});
    // only this wave reads what it wrote; same-wave LDS accesses execute in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int kPieces = kWCols / 8;                        // 16-byte pieces per row of the wave's block
    const bool vec_ok = (prm.N & 7) == 0;                       // rows of Y 16-byte aligned
#pragma unroll
    for (int it = 0; it < kBM * kPieces / 64; ++it) {
        const int idx = it * 64 + lane;
        const int ml = idx / kPieces, piece = idx % kPieces;
        const int m = m0 + ml, n = n0 + wave * kWCols + piece * 8;
        if (prm.y && m < prm.M && n < prm.N) {
            const uint4 v = *reinterpret_cast<const uint4*>(stage + ml * kWCols + piece * 8);
            uint16_t* dst = prm.y + (size_t)m * prm.N + n;
            if (vec_ok && n + 8 <= prm.N) {
                *reinterpret_cast<uint4*>(dst) = v;
            } else {
                const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (n + e < prm.N) dst[e] = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}


// ---- per-group weight parameters (groups of 128 along K, Appendix C) in the prefill shape ------------------------
// Same tiling and operand paths as tiled_kernel (64 rows of A x 64*NTW rows of W per workgroup, weights HBM -> registers
// one 256-k step ahead, rows of A global -> LDS double buffered), but a 256-k step is two groups of 128 k and every group
// gets fresh integer accumulators that are flushed through the group's scale into a binary32 tile sum:
//   sum_k (a' - zc)(w' - z) = c - z * sum_k a' - zc * (sum_k w' - 128 z)          (exact integers)
// with c the MFMA sum of the stored operands a' = a - oa, w' = w - ow, z the group's zero-point less ow, zc the token's
// zero-point less oa.  The two operand sums come from the matrix pipe as well: an MFMA of the A operand against ones
// gives sum_k a' of every row in every column, an MFMA of ones against the B operand gives sum_k w' of every column
// in every row — both already in the accumulator layout.  k past K holds a' = 0 and w' = z (the packer pads the last
// group of a g128 blob with its zero-point), so padded k add nothing; groups wholly past K carry scale 0.
// Then two 24-bit integer multiply-adds, one conversion and one fused multiply-add per element and group: M*N*K/128
// of each, which is what bounds this kernel (the vector ALU, not the matrix pipe).
typedef float v4f __attribute__((ext_vector_type(4)));

template <int P, int NTW, int MT, int PH>
__device__ __forceinline__ void step_g128(const u4v (*w)[phase_regs(P)], const u4v* gq, const uint8_t* a_buf, int r, int G,
                                          const v4i* zc, v4f (*facc)[NTW])
{
    const v4i ones{0x01010101, 0x01010101, 0x01010101, 0x01010101}, zero4{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 2; ++j) {                      // group 2*PH + j of the super-chunk
        v4i c[MT][NTW], asum[MT], wsum[NTW];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            asum[mt] = zero4;
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) c[mt][nt] = zero4;
        }
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) wsum[nt] = zero4;
        auto slice = [&](auto SLC) {
            constexpr int SL = decltype(SLC)::value;   // slice inside the super-chunk
            v4i aop[MT];
            read_a_operands<MT>(a_buf, r, G, SL & 3, aop);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) asum[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[mt], ones, asum[mt], 0, 0, 0);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const v4i bop = merged_operand<P, SL>(w[nt]);
                wsum[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, bop, wsum[nt], 0, 0, 0);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) c[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[mt], bop, c[mt][nt], 0, 0, 0);
            }
        };
        if (j == 0) { slice(std::integral_constant<int, 4 * PH + 0>{}); slice(std::integral_constant<int, 4 * PH + 1>{}); }
        else { slice(std::integral_constant<int, 4 * PH + 2>{}); slice(std::integral_constant<int, 4 * PH + 3>{}); }
        const int gj = 2 * PH + j;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int z = ((int)(gq[nt].z << (24 - 8 * gj))) >> 24;
            const uint32_t sbits = (gj < 2 ? gq[nt].x : gq[nt].y) >> (16 * (gj & 1));
            const float sc = __half2float(__ushort_as_half((unsigned short)(sbits & 0xFFFFu)));
            const int wz = wsum[nt].x - 128 * z;       // (every row of wsum holds the column's sum)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    // (24-bit multiply-adds, full rate: a group's sums are below 2^17 and the zero-points below 2^8, and the
                    // products are exact in 32 bits; 32-bit multiplies run at a quarter of the rate and were this kernel's bound)
                    const int t = __mul24(-zc[mt][reg], wz) + (__mul24(-z, asum[mt][reg]) + c[mt][nt][reg]);
                    facc[mt][nt][reg] = fmaf((float)t, sc, facc[mt][nt][reg]);
                }
            }
        }
    }
}

template <int P, int NTW>
__global__ __launch_bounds__(256, 2) void tiled_g128_kernel(TiledParams prm)
{
    constexpr int MT = 4;
    constexpr int kBM = MT * 16, kBN = 4 * NTW * kTileN;
    __shared__ __align__(16) uint8_t lds_a0[kBM * kARow];
    __shared__ __align__(16) uint8_t lds_a1[kBM * kARow];
    __shared__ RowParams par_a[kBM];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, G = lane >> 4;
    // tile order: as in tiled_kernel (a contiguous run of the banded order per XCD)
    const int nwg = prm.tiles_m * prm.tiles_n;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    const int vid = xcd * per + min(xcd, rem) + slot;
    const int band = vid / (prm.band_m * prm.tiles_n), in_band = vid - band * prm.band_m * prm.tiles_n;
    const int band_rows = min(prm.band_m, prm.tiles_m - band * prm.band_m);
    const int m_blk = band * prm.band_m + in_band % band_rows, n_blk = in_band / band_rows;
    const int m0 = m_blk * kBM, n0 = n_blk * kBN;
    const int tile0 = n_blk * (kBN / kTileN) + wave * NTW;

    u4v wa[NTW][phase_regs(P)], wb[NTW][phase_regs(P)], gq[NTW], gq_next[NTW];
    auto load_records = [&](int sc, u4v* out) {   // the super-chunk's group parameters of this lane's channel, per tile
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
            out[nt] = prm.gparams[((size_t)min(tile0 + nt, prm.ntiles - 1) * prm.nsuper + sc) * 16 + r];
    };
    load_tiles<P, NTW>(prm, tile0, 0, 0, lane, wa);
    load_records(0, gq);
    if (tid < kBM) par_a[tid] = prm.aparams[min(m0 + tid, prm.M - 1)];

    unsigned a_goff[MT];
#pragma unroll
    for (int u = 0; u < MT; ++u) {
        const int row = 4 * (wave * MT + u) + (lane >> 4);
        const int vec = (lane & 15) ^ (row & 15);
        a_goff[u] = (unsigned)(min(m0 + row, prm.M - 1) - m0) * (unsigned)prm.Kp + vec * 16;
    }
    const int8_t* a_tile = prm.a_codes + (size_t)m0 * prm.Kp;
    auto a_prefetch = [&](int step, uint8_t* buf) {
        const int8_t* base = a_tile + (size_t)step * kStepK;
#pragma unroll
        for (int u = 0; u < MT; ++u)
            __builtin_amdgcn_global_load_lds((const void*)(base + a_goff[u]),
                                             (__attribute__((address_space(3))) void*)(buf + (wave * MT + u) * 1024), 16, 0, 0);
    };
    v4f facc[MT][NTW];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) facc[mt][nt] = v4f{0.f, 0.f, 0.f, 0.f};

    a_prefetch(0, lds_a0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (a wave's direct loads land before it enters a barrier, here and below: see tiled_kernel)
    __syncthreads();
    // zero-points of this lane's accumulator rows, less oa
    v4i zc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) zc[mt][reg] = par_a[mt * 16 + 4 * G + reg].zero - prm.oa;

    const int nsteps = prm.nsuper * 2;
    for (int sc = 0; sc < prm.nsuper; ++sc) {
        const int scn = min(sc + 1, prm.nsuper - 1);
        {
            load_tiles<P, NTW>(prm, tile0, sc, 1, lane, wb);
            load_records(scn, gq_next);
            a_prefetch(2 * sc + 1, lds_a1);
            step_g128<P, NTW, MT, 0>(wa, gq, lds_a0, r, G, zc, facc);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        {
            load_tiles<P, NTW>(prm, tile0, scn, 0, lane, wa);
            a_prefetch(min(2 * sc + 2, nsteps - 1), lds_a0);
            step_g128<P, NTW, MT, 1>(wb, gq, lds_a1, r, G, zc, facc);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) gq[nt] = gq_next[nt];
    }

    // epilogue: Y = half(a_scale * sum over groups), rows leave in 16-byte pieces through LDS as in tiled_kernel
    __syncthreads();
    constexpr int kWCols = NTW * kTileN;
    uint16_t* stage = reinterpret_cast<uint16_t*>((wave < 2 ? lds_a0 : lds_a1) + (wave & 1) * (kBM * kWCols * 2));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int ml = mt * 16 + 4 * G + reg;
            const float sa = par_a[ml].scale;
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const float v = sa * facc[mt][nt][reg];
                uint32_t h;
                asm("v_cvt_f16_f32 %0, %1" : "=v"(h) : "v"(v));
                stage[ml * kWCols + nt * 16 + r] = (uint16_t)h;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int kPieces = kWCols / 8;
    const bool vec_ok = (prm.N & 7) == 0;
#pragma unroll
    for (int it = 0; it < kBM * kPieces / 64; ++it) {
        const int idx = it * 64 + lane;
        const int ml = idx / kPieces, piece = idx % kPieces;
        const int m = m0 + ml, n = n0 + wave * kWCols + piece * 8;
        if (m < prm.M && n < prm.N) {
            const uint4 v = *reinterpret_cast<const uint4*>(stage + ml * kWCols + piece * 8);
            uint16_t* dst = prm.y + (size_t)m * prm.N + n;
            if (vec_ok && n + 8 <= prm.N) {
                *reinterpret_cast<uint4*>(dst) = v;
            } else {
                const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (n + e < prm.N) dst[e] = (uint16_t)(w4[e >> 1] >> (16 * (e & 1)));
            }
        }
    }
}

template <int P>
static hipError_t launch_g128_p(const TiledParams& prm, int ntw, dim3 grid, hipStream_t s)
{
    if (ntw == 1) tiled_g128_kernel<P, 1><<<grid, 256, 0, s>>>(prm);
    else tiled_g128_kernel<P, 2><<<grid, 256, 0, s>>>(prm);
    return hipGetLastError();
}

template <int P, int NTW, int MT>
static hipError_t launch_shape(const TiledParams& prm, dim3 grid, int cus, int plan_wd, hipStream_t s)
{
    // The deep rings exist for the small tile shapes (for two tiles of W per wave only up to p = 6: beyond, the
    // registers run out) and run two workgroups per CU instead of three.  Measured: with at most one workgroup
    // per CU (M = 64..128 on a 4096-wide layer) they are 20 % faster, with more workgroups (M = 128 on an
    // 11008-wide layer and up) the traffic through L2, not the latency of a step, is the bound and they lose.
    // With long K (13824) and p = 8 the plan search found them ahead up to 2.5 workgroups per CU (M = 512, 5120 channels:
    // 75 vs 84 us); narrower weights lose or tie there (between one and two workgroups per CU, K = 11008..13824: W1A8
    // 38 vs 33 us, W2A8 35 vs 28, W4A8 and W6A8 within 1 %), because the deep rings hold two workgroups per CU, not three.
    // Override: the plan table (plan_wd).
    constexpr bool has_deep = MT == 4 && (NTW == 1 || (NTW == 2 && P <= 6));
    const int forced = plan_wd > 0 ? plan_wd : tuning_env("ABQ_TILED_WD");
    if constexpr (has_deep) {
        if (forced == 4 || (forced != 2 && ((long)grid.x <= (long)cus || (P == 8 && (long)grid.x <= 3L * cus && prm.K >= 8192)))) {
            tiled_kernel<P, NTW, MT, 4><<<grid, 256, 0, s>>>(prm);
            return hipGetLastError();
        }
    }
    tiled_kernel<P, NTW, MT, 2><<<grid, 256, 0, s>>>(prm);
    return hipGetLastError();
}

template <int P>
static hipError_t launch_p(const TiledParams& prm, int ntw, int mt, dim3 grid, int cus, int plan_wd, hipStream_t s)
{
    if (mt == 4) {
        if (ntw == 1) return launch_shape<P, 1, 4>(prm, grid, cus, plan_wd, s);
        if (ntw == 2) return launch_shape<P, 2, 4>(prm, grid, cus, plan_wd, s);
        return launch_shape<P, 4, 4>(prm, grid, cus, plan_wd, s);
    }
    if (ntw == 1) return launch_shape<P, 1, 8>(prm, grid, cus, plan_wd, s);
    if (ntw == 2) return launch_shape<P, 2, 8>(prm, grid, cus, plan_wd, s);
    return launch_shape<P, 4, 8>(prm, grid, cus, plan_wd, s);
}

hipError_t launch_gemm_tiled(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s)
{
    TiledParams prm;
    for (int i = 0; i < 3; ++i) prm.fields[i] = (const u4v*)(g.w_blob + W.off_fields[i]);
    prm.a_codes = (const int8_t*)(g.act_blob + A.off_codes);
    prm.aparams = (const RowParams*)(g.act_blob + A.off_params);
    prm.wparams = (const RowParams*)(g.w_blob + W.off_params);
    prm.y = g.y;
    prm.acc = g.acc;
    prm.rq = g.rq;
    prm.M = g.M; prm.N = g.N; prm.K = g.K; prm.Kp = A.Kp;
    prm.nsuper = A.Kp / kSuperK;
    prm.ntiles = W.NT;
    prm.oa = (g.q == 8) ? 128 : 0;
    prm.ow = (g.p == 8) ? 128 : 0;
    prm.gparams = W.g128 ? (const u4v*)(g.w_blob + W.off_gparams) : nullptr;
    prm.narrow_sums = ((long)g.K * ((1 << g.p) - 1) < (1L << 23) && (long)g.K * ((1 << g.q) - 1) < (1L << 23)) ? 1 : 0;
    if (W.g128) {
        // per-group weight parameters: 64 rows of A against 128 (or, for few workgroups, 64) rows of W per workgroup
        int cus_g = 256, dev_g = 0;
        if (hipGetDevice(&dev_g) != hipSuccess || hipDeviceGetAttribute(&cus_g, hipDeviceAttributeMultiprocessorCount, dev_g) != hipSuccess || cus_g <= 0) cus_g = 256;
        const long wg2 = (long)((g.M + 63) / 64) * ((g.N + 127) / 128);
        const int ntw_g = 2 * wg2 >= 3L * cus_g ? 2 : 1;
        prm.tiles_m = (g.M + 63) / 64;
        prm.tiles_n = (g.N + 64 * ntw_g - 1) / (64 * ntw_g);
        const int cap = (g.p <= 4 ? 512 : 1024) / 64;
        const int bands = (prm.tiles_m + cap - 1) / cap;
        prm.band_m = (prm.tiles_m + bands - 1) / bands;
        dim3 grid_g((unsigned)(prm.tiles_m * prm.tiles_n));
        switch (g.p) {
            case 1: return launch_g128_p<1>(prm, ntw_g, grid_g, s);
            case 2: return launch_g128_p<2>(prm, ntw_g, grid_g, s);
            case 3: return launch_g128_p<3>(prm, ntw_g, grid_g, s);
            case 4: return launch_g128_p<4>(prm, ntw_g, grid_g, s);
            case 5: return launch_g128_p<5>(prm, ntw_g, grid_g, s);
            case 6: return launch_g128_p<6>(prm, ntw_g, grid_g, s);
            case 7: return launch_g128_p<7>(prm, ntw_g, grid_g, s);
            default: return launch_g128_p<8>(prm, ntw_g, grid_g, s);
        }
    }
    // Tile shape (rows of A x rows of W per workgroup), measured on LLaMA-7B/13B prefill shapes: 128x128
    // while it yields at least 1.5 workgroups per CU (two or three share a CU), else 64x128, else 64x64.
    // Narrow weights (p <= 4) with M >= 1024 do better with 64 rows of A against 256 (or 128) rows of W: the
    // launch-plan search on M = 1024..8192 found 64x256 3-19 % ahead of 128x128 at p = 2, 4 where it still
    // yields three workgroups per CU, and 64x128 ahead of both where it does not (N = 5120: 124 vs 144 us);
    // at M = 512 and at p = 8 128x128 stays ahead.
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    auto wgs = [&](int mt_, int ntw_) { return (long)((g.M + mt_ * 16 - 1) / (mt_ * 16)) * ((g.N + 64 * ntw_ - 1) / (64 * ntw_)); };
    int mt = 8, ntw = 2;
    // (p = 8: 128 x 128 also with 0.8..1 workgroups per CU, where it halves the weight bytes through L2 and every CU still
    // has one: M = 256 on 13824 channels 40 -> 37 us, M = 1024 on 4096 channels 71 -> 67; with 1.25 per CU it loses 8 %.  64 x 256 also where it fills the chip exactly once
    // at two workgroups per CU, 1.5..2 per CU: M = 2048 on 4096 channels, W4A8 K = 11008 95 -> 83 us.)
    const bool mt8 = 2 * wgs(8, 2) >= 3L * cus || (g.p == 8 && 5 * wgs(8, 2) >= 4L * cus && wgs(8, 2) <= (long)cus);
    if (g.M <= 64 || !mt8) { mt = 4; ntw = 2; }
    else if (g.p <= 4 && g.M >= 1024) { mt = 4; ntw = (wgs(4, 4) >= 3L * cus || (wgs(4, 4) <= 2L * cus && 2 * wgs(4, 4) > 3L * cus)) ? 4 : 2; }
    // K >= 5120, p = 4..6 and between 0.5 and 1.25 workgroups of 64 x 128 per CU: that tile on the deep rings is
    // 4-11 % ahead of 64 x 64 (plan search, K = 5120, 11008, 13824: M = 128 on 13824 channels, M = 256 on 5120, M = 512 on
    // 4096 and 5120; at K = 4096, M = 128 on 11008 channels, it is 3 % behind); with
    // fewer workgroups 64 x 64 on the deep rings wins by a wide margin (M = 256 on 4096 channels: 24 vs 33 us), with two
    // per CU the shallow rings do (M = 1024 on 4096 channels: 60 vs 66 us), and narrower weights prefer those anyway.
    int rule_wd = 0;
    if (mt == 4 && ntw == 2 && g.p >= 4 && g.p <= 6 && g.K >= 5120 && 2 * wgs(4, 2) > (long)cus && 4 * wgs(4, 2) <= 5L * cus) rule_wd = 4;
    if (mt == 4 && ntw == 2 && rule_wd == 0 && 2 * wgs(4, 2) < 3L * cus) ntw = 1;
    {
        const int forced_mt = tuning_env("ABQ_TILED_MT"), forced_ntw = tuning_env("ABQ_TILED_NTW");
        if (forced_mt == 4 || forced_mt == 8) mt = forced_mt;
        if (forced_ntw == 1 || forced_ntw == 2 || forced_ntw == 4) ntw = forced_ntw;
    }
    PlanOverride ov;   // the plan table entry of this exact problem
    lookup_plan(g.p, g.q, g.M, g.N, g.K, &ov);
    if (ov.tiled_mt > 0) mt = ov.tiled_mt;
    if (ov.tiled_ntw > 0) ntw = ov.tiled_ntw;
    const int wd_arg = ov.tiled_wd > 0 ? ov.tiled_wd : ((mt == 4 && ntw == 2) ? rule_wd : 0);
    prm.tiles_m = (g.M + mt * 16 - 1) / (mt * 16);
    prm.tiles_n = (g.N + 64 * ntw - 1) / (64 * ntw);
    // Bands of equal height.  The workgroups resident on one XCD (about 64) form a band_m x (64 / band_m)
    // patch of tiles whose L2 fills cost band_m row blocks of A (one byte per element) plus 64 / band_m
    // column blocks of W (p/8 byte per element): least near band_m = sqrt(8p) blocks of 128 rows, and measured
    // so on M = 2048 and 8192: bands of 512 rows of A for p <= 4, 1024 above.
    {
        const int forced_band = tuning_env("ABQ_TILED_BAND");
        const int cap = ov.tiled_band > 0 ? ov.tiled_band : (forced_band > 0 ? forced_band : (g.p <= 4 ? 512 : 1024) / (mt * 16));
        const int bands = (prm.tiles_m + cap - 1) / cap;
        prm.band_m = (prm.tiles_m + bands - 1) / bands;
    }
    dim3 grid((unsigned)(prm.tiles_m * prm.tiles_n));
    switch (g.p) {
        case 1: return launch_p<1>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 2: return launch_p<2>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 3: return launch_p<3>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 4: return launch_p<4>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 5: return launch_p<5>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 6: return launch_p<6>(prm, ntw, mt, grid, cus, wd_arg, s);
        case 7: return launch_p<7>(prm, ntw, mt, grid, cus, wd_arg, s);
        default: return launch_p<8>(prm, ntw, mt, grid, cus, wd_arg, s);
    }
}

}  // namespace abq
