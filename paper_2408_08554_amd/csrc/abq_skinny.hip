// Decode-shaped matmul (M = 1 .. 64): the packed weight plane groups are streamed from HBM
// exactly once with 128-bit coalesced loads, expanded to signed bytes in registers with one
// AND per dword, and contracted against the int8 activation codes on the 16x16x64 int8 MFMA.
// Bit reduction (Sec. 3.4 step 5 / Appendix B: the 2^(s+t) factors) happens in registers:
// the activation side carries all q planes at once as the int8 code, the weight side one
// plane group per accumulator, recombined with shifts after the K loop.  The dequant
// epilogue is fused (Fig. 3b).
//
// Work decomposition: one workgroup per 16 output channels (one MFMA tile of W rows); its
// waves split K in units of 512 (a "super-chunk": every plane group tiles 512 k-values with
// whole 1 KiB wave loads) and are summed through LDS at the end.  The M <= 16 rows of A for
// the K range in flight are staged in LDS once per workgroup.
#include "abq_internal.h"
#include "../../include/abq.h"

#include <hip/hip_fp16.h>

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));

struct SkinnyParams {
    const uint4* fields[3];   // per plane group
    int chunks[3];
    const int8_t* a_codes;    // [M][Kp]
    const RowParams* aparams;
    const RowParams* wparams;
    uint16_t* y;
    int32_t* acc;
    int M, N, K, Kp;
    int oa, ow;
    int kseg;                 // k-extent of A staged in LDS at a time (multiple of 512)
    int lds_stride;           // bytes per staged row (kseg + 16: rows land 16 B apart in bank space)
};

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
__device__ __forceinline__ v4i field_operand(const uint4& w)
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
__device__ __forceinline__ void chunk_mfma(const uint4& w, const v4i* aop, v4i* acc)
{
    constexpr int T = 8 / B;
    if constexpr (T0 < T) {
        acc[T0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[I * T + T0], field_operand<B, T0>(w), acc[T0], 0, 0, 0);
        chunk_mfma<B, I, T0 + 1>(w, aop, acc);
    }
}
template <int B, int I = 0>
__device__ __forceinline__ void group_mfma(const uint4* w, const v4i* aop, v4i* acc)
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

template <int P>
__device__ __forceinline__ void load_super(const SkinnyParams& prm, int nt, int sc, int lane, uint4* w)
{
    using GI = GroupInfo<P>;
#pragma unroll
    for (int g = 0; g < GI::NG; ++g) {
        const int b = GI::b(g);
#pragma unroll
        for (int i = 0; i < b; ++i) {
            const int c = sc * b + i;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (c < prm.chunks[g]) v = prm.fields[g][((size_t)nt * prm.chunks[g] + c) * 64 + lane];
            w[GI::load_base(g) + i] = v;
        }
    }
}

template <int P>
__device__ __forceinline__ void compute_super(const uint4* w, const uint8_t* lds_row, bool row_valid, v4i* acc)
{
    using GI = GroupInfo<P>;
    v4i aop[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        v4i v = {0, 0, 0, 0};
        if (row_valid) v = *reinterpret_cast<const v4i*>(lds_row + j * 64);
        aop[j] = v;
    }
    group_mfma<GI::b(0)>(w + GI::load_base(0), aop, acc + GI::acc_base(0));
    if constexpr (GI::NG > 1) group_mfma<GI::b(1)>(w + GI::load_base(1), aop, acc + GI::acc_base(1));
    if constexpr (GI::NG > 2) group_mfma<GI::b(2)>(w + GI::load_base(2), aop, acc + GI::acc_base(2));
}

template <int P>
__global__ __launch_bounds__(512) void skinny_kernel(SkinnyParams prm)
{
    using GI = GroupInfo<P>;
    extern __shared__ __align__(16) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int nt = blockIdx.x;
    const int m0 = blockIdx.y * 16;
    const int mt = min(16, prm.M - m0);
    const int r = lane & 15, G = lane >> 4;
    const bool row_valid = r < mt;
    const int nsuper = prm.Kp / kSuperK;

    v4i acc[GI::NACC];
#pragma unroll
    for (int i = 0; i < GI::NACC; ++i) acc[i] = v4i{0, 0, 0, 0};

    // epilogue operands are fetched up front so that their latency hides under the stream
    RowParams ep_a = {0, 0.0f, 0, 0}, ep_w = {0, 0.0f, 0, 0};
    const int ep_m = m0 + 4 * ((tid & 63) >> 4) + (tid >> 6);   // thread tid < 256 finishes C register tid/64 of lane tid%64
    const int ep_n = nt * kTileN + (tid & 15);
    const bool ep_valid = tid < 256 && ep_m < prm.M && ep_n < prm.N;
    if (ep_valid) { ep_a = prm.aparams[ep_m]; ep_w = prm.wparams[ep_n]; }

    const int super_per_seg = prm.kseg / kSuperK;
    for (int seg0 = 0; seg0 < nsuper; seg0 += super_per_seg) {
        const int seg1 = min(nsuper, seg0 + super_per_seg);
        const int vec_per_row = (seg1 - seg0) * (kSuperK / 16);
        const int nvec = mt * vec_per_row;
        const int8_t* a_seg = prm.a_codes + (size_t)m0 * prm.Kp + (size_t)seg0 * kSuperK;
        // order of issue: first slice of A, then this wave's first weight loads, so that waiting
        // for A leaves the weight loads in flight
        uint4 a_first = make_uint4(0, 0, 0, 0);
        if (tid < nvec) a_first = *reinterpret_cast<const uint4*>(a_seg + (size_t)(tid / vec_per_row) * prm.Kp + (tid % vec_per_row) * 16);
        uint4 wa[P], wb[P];
        int sc = seg0 + wave;
        if (sc < seg1) load_super<P>(prm, nt, sc, lane, wa);
        if (seg0 > 0) __syncthreads();   // every wave is done reading the previous segment
        if (tid < nvec) *reinterpret_cast<uint4*>(lds + (tid / vec_per_row) * prm.lds_stride + (tid % vec_per_row) * 16) = a_first;
        for (int i = tid + blockDim.x; i < nvec; i += blockDim.x) {
            const int row = i / vec_per_row, col = (i % vec_per_row) * 16;
            *reinterpret_cast<uint4*>(lds + row * prm.lds_stride + col) =
                *reinterpret_cast<const uint4*>(a_seg + (size_t)row * prm.Kp + col);
        }
        __syncthreads();
        const uint8_t* lds_lane = lds + r * prm.lds_stride + G * 16;
        // double-buffered stream over this wave's super-chunks
        for (; sc < seg1; sc += 2 * nwaves) {
            const int sc_b = sc + nwaves;
            if (sc_b < seg1) load_super<P>(prm, nt, sc_b, lane, wb);
            compute_super<P>(wa, lds_lane + (sc - seg0) * kSuperK, row_valid, acc);
            if (sc_b < seg1) {
                const int sc_c = sc_b + nwaves;
                if (sc_c < seg1) load_super<P>(prm, nt, sc_c, lane, wa);
                compute_super<P>(wb, lds_lane + (sc_b - seg0) * kSuperK, row_valid, acc);
            }
        }
    }

    // bit reduction across the plane groups of this wave
    v4i total = group_combine<GI::b(0)>(acc + GI::acc_base(0));
    if constexpr (GI::NG > 1) {
        v4i t1 = group_combine<GI::b(1)>(acc + GI::acc_base(1));
        total += t1 << GroupInfo<P>::load_base(1);
    }
    if constexpr (GI::NG > 2) {
        v4i t2 = group_combine<GI::b(2)>(acc + GI::acc_base(2));
        total += t2 << GroupInfo<P>::load_base(2);
    }

    // sum over the waves (split K) through LDS, then the fused epilogue
    __syncthreads();
    int32_t* red = reinterpret_cast<int32_t*>(lds);
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) red[(wave * 4 + reg) * 64 + lane] = total[reg];
    __syncthreads();
    if (tid < 256) {
        int32_t s = 0;
        for (int w = 0; w < nwaves; ++w) s += red[w * 256 + tid];
        // MFMA C layout: lane l, register reg holds row 4*(l/16)+reg (A side: m), column l%16 (B side: n);
        // thread tid sums register tid/64 of lane tid%64
        if (ep_valid) epilogue_store(s, prm.oa, prm.ow, prm.K, ep_a, ep_w, (size_t)ep_m * prm.N + ep_n, prm.y, prm.acc);
    }
}

// Waves per workgroup (4..8): as many as there are super-chunks to split when K is short (one
// memory round trip), otherwise the count that leaves the fewest idle wave-slots.
static int pick_waves(int nsuper)
{
    if (nsuper <= 8) return nsuper < 4 ? 4 : nsuper;
    int best = 8, best_waste = 1 << 30;
    for (int w = 8; w >= 4; --w) {
        const int rounds = (nsuper + w - 1) / w;
        const int waste = rounds * w - nsuper;
        if (waste < best_waste) { best_waste = waste; best = w; }
    }
    return best;
}

template <int P>
static hipError_t launch_p(const SkinnyParams& prm, dim3 grid, int waves, size_t lds_bytes, hipStream_t s)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)skinny_kernel<P>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    skinny_kernel<P><<<grid, waves * 64, lds_bytes, s>>>(prm);
    return hipGetLastError();
}

hipError_t launch_gemm_skinny(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s)
{
    SkinnyParams prm;
    for (int i = 0; i < 3; ++i) {
        prm.fields[i] = (const uint4*)(g.w_blob + W.off_fields[i]);
        prm.chunks[i] = W.chunks[i];
    }
    prm.a_codes = (const int8_t*)(g.act_blob + A.off_codes);
    prm.aparams = (const RowParams*)(g.act_blob + A.off_params);
    prm.wparams = (const RowParams*)(g.w_blob + W.off_params);
    prm.y = g.y;
    prm.acc = g.acc;
    prm.M = g.M; prm.N = g.N; prm.K = g.K; prm.Kp = A.Kp;
    prm.oa = (g.q == 8) ? 128 : 0;
    prm.ow = (g.p == 8) ? 128 : 0;
    const int nsuper = A.Kp / kSuperK;
    const int waves = pick_waves(nsuper);
    const int mt = g.M < 16 ? g.M : 16;
    // LDS: staged rows (<= 128 KiB) and, afterwards, the 1 KiB per wave reduction buffer
    const int budget = 128 * 1024;
    int super_per_seg = (budget / mt - 16) / kSuperK;
    if (super_per_seg > nsuper) super_per_seg = nsuper;
    if (super_per_seg < 1) super_per_seg = 1;
    prm.kseg = super_per_seg * kSuperK;
    prm.lds_stride = prm.kseg + 16;
    size_t lds_bytes = (size_t)mt * prm.lds_stride;
    const size_t red_bytes = (size_t)waves * 1024;
    if (lds_bytes < red_bytes) lds_bytes = red_bytes;
    dim3 grid((unsigned)W.NT, (unsigned)((g.M + 15) / 16));
    switch (g.p) {
        case 1: return launch_p<1>(prm, grid, waves, lds_bytes, s);
        case 2: return launch_p<2>(prm, grid, waves, lds_bytes, s);
        case 3: return launch_p<3>(prm, grid, waves, lds_bytes, s);
        case 4: return launch_p<4>(prm, grid, waves, lds_bytes, s);
        case 5: return launch_p<5>(prm, grid, waves, lds_bytes, s);
        case 6: return launch_p<6>(prm, grid, waves, lds_bytes, s);
        case 7: return launch_p<7>(prm, grid, waves, lds_bytes, s);
        default: return launch_p<8>(prm, grid, waves, lds_bytes, s);
    }
}

}  // namespace abq
