// The activation quantizer fused into its producers: the producer-side fusion of Sec. 3.4 / Fig. 3b (the
// online quantization of a linear layer's input is folded into the operator in front of it, which in
// the LLaMA models the paper evaluates is RMSNorm for the attention and gate/up projections and
// SiLU(gate) * up for down_proj).  One kernel takes a token's fp16 row to q-bit codes with their
// per-token scale and zero-point, ready for abq_gemm_act_codes.
//
// RMSNorm (KIND 0).
// Every step that decides a code is a single, stated IEEE operation, so the codes are reproducible
// bit for bit whatever the order of the parallel reductions:
//   sum_k x^2 exactly (x is binary16: 2^48 x^2 is an integer below 2^81, summed in 128 bits),
//   ss = (double(hi) * 2^64 + double(lo)) * 2^-48;  mean = ss / K;  r = float(1 / sqrt(mean + eps)),
//   y = half_rne((float(x) * r) * float(gamma)),
//   then the per-token quantizer of abq_quant_pack_act on y (lo/hi include 0, Delta = (hi - lo) / (2^q - 1),
//   z = clamp(rint(-lo / Delta)), code = clamp(rint(y / Delta) + z)).
// SiLU * up (KIND 1): h = half_rne((g / (1 + e)) * up) with e = exp(-g) as a fixed sequence of binary32
// operations (no math library, no fused multiply-add): t = clamp(-g * log2(e), -126, 126), n = rint(t),
// f = t - n, 2^f by a degree-6 Horner polynomial with coefficients ln(2)^k / k!, e = ldexp(2^f, n).
#include "abq_internal.h"
#include "../../include/abq.h"

namespace abq {

__device__ __forceinline__ float half_to_f32(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// A binary16 value is mant * 2^(max(e,1) - 25), so 2^48 * value^2 = mant^2 * 2^sh with sh = 2 max(e,1) - 2 = 0 .. 58
// and mant^2 < 2^22.

__device__ __forceinline__ void add128(uint64_t& lo, uint64_t& hi, uint64_t l, uint64_t h)
{
    lo += l;
    hi += h + (lo < l ? 1ull : 0ull);
}

// The same sum with one shift and one add per element: squares with a shift below 32 go to one 64-bit
// accumulator (each below 2^54), the others, shifted by 32 less, to a second one (each below 2^48); a
// thread adds at most 512 of them, so neither overflows.  fold() turns the pair into the 128-bit sum.
struct SquareSum {
    uint64_t small = 0, large = 0;
    __device__ __forceinline__ void add(uint16_t h)
    {
        const uint32_t e = (h >> 10) & 31u, frac = h & 1023u;
        const uint32_t mant = e ? frac + 1024u : frac;
        const uint32_t sh = 2u * (e ? e : 1u) - 2u;
        const uint64_t sq = (uint64_t)(mant * mant);
        small += sh < 32u ? (sq << sh) : 0ull;
        large += sh < 32u ? 0ull : (sq << (sh - 32u));
    }
    __device__ __forceinline__ void fold(uint64_t& lo, uint64_t& hi) const
    {
        lo = small;
        hi = 0;
        add128(lo, hi, large << 32, large >> 32);
    }
};

// value of r for a row from the exact 128-bit sum of squares (in units of 2^-48)
__device__ __forceinline__ float inv_rms(uint64_t lo, uint64_t hi, int K, float eps)
{
    const double ss = __dmul_rn(__dadd_rn(__dmul_rn(__ull2double_rn(hi), 18446744073709551616.0), __ull2double_rn(lo)),
                                1.0 / 281474976710656.0);
    const double mean = __ddiv_rn(ss, (double)K);
    return __double2float_rn(__ddiv_rn(1.0, __dsqrt_rn(__dadd_rn(mean, (double)eps))));
}

// y = half_rne((float(x) * r) * float(gamma)) as binary16 bits.  The conversion is written as the instruction
// itself: left to the compiler, the second product and the conversion are merged into one mixed-precision
// operation with a single rounding, which lands on the other neighbour whenever the float product is an exact
// tie between two binary16 values.
__device__ __forceinline__ uint16_t normalized_half(uint16_t xb, uint16_t gb, float r)
{
    const float t = __fmul_rn(half_to_f32(xb), r);
    const float u = __fmul_rn(t, half_to_f32(gb));
    uint32_t hb;
    asm("v_cvt_f16_f32 %0, %1" : "=v"(hb) : "v"(u));
    return (uint16_t)hb;
}

// silu(g) * u as binary16 bits (see the head of the file for the definition of exp).
__device__ __forceinline__ uint16_t silu_mul_half(uint16_t gb, uint16_t ub)
{
    const float g = half_to_f32(gb), u = half_to_f32(ub);
    float t = __fmul_rn(-g, 0x1.715476p+0f);
    t = t < -126.0f ? -126.0f : (t > 126.0f ? 126.0f : t);
    const float n = rintf(t);
    const float f = __fsub_rn(t, n);
    float p = __fmul_rn(f, 0x1.430912p-13f);
    p = __fmul_rn(__fadd_rn(p, 0x1.5d87fep-10f), f);
    p = __fmul_rn(__fadd_rn(p, 0x1.3b2ab6p-7f), f);
    p = __fmul_rn(__fadd_rn(p, 0x1.c6b08ep-5f), f);
    p = __fmul_rn(__fadd_rn(p, 0x1.ebfbe0p-3f), f);
    p = __fmul_rn(__fadd_rn(p, 0x1.62e430p-1f), f);
    p = __fadd_rn(p, 1.0f);
    const float e = ldexpf(p, (int)n);
    const float sg = __fdiv_rn(g, __fadd_rn(1.0f, e));
    const float h = __fmul_rn(sg, u);
    uint32_t hb;
    asm("v_cvt_f16_f32 %0, %1" : "=v"(hb) : "v"(h));   // (kept apart from the product, as above)
    return (uint16_t)hb;
}

// h = half_rne(float(a) + float(b)): the residual add in front of the normalization (one binary32 addition, then the
// conversion as its own instruction, for the reason given above).
__device__ __forceinline__ uint16_t add_half(uint16_t ab, uint16_t bb)
{
    const float s = __fadd_rn(half_to_f32(ab), half_to_f32(bb));
    uint32_t hb;
    asm("v_cvt_f16_f32 %0, %1" : "=v"(hb) : "v"(s));
    return (uint16_t)hb;
}
__device__ __forceinline__ uint32_t add_half2(uint32_t a, uint32_t b)
{
    return (uint32_t)add_half((uint16_t)(a & 0xFFFFu), (uint16_t)(b & 0xFFFFu)) |
           ((uint32_t)add_half((uint16_t)(a >> 16), (uint16_t)(b >> 16)) << 16);
}

// KIND 0: RMSNorm, operand b = gamma [K];  KIND 1: SiLU(a) * b, operand b = up [M,K].
template <int KIND>
__device__ __forceinline__ uint16_t produce_half(uint16_t ab, uint16_t bb, float r)
{
    if constexpr (KIND == 0) return normalized_half(ab, bb, r);
    else return silu_mul_half(ab, bb);
}

// Fast path: K a multiple of 8 and at most 8 * BLOCK * VPT.  A thread keeps its VPT 16-byte vectors of x and
// of gamma in registers across the three passes (sum of squares, range, codes): the row is read once.
template <int KIND, int VPT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void producer_quant_rows_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma,
                                                                 float eps, int q, int K, uint8_t* __restrict__ codes,
                                                                 float* __restrict__ scale, int32_t* __restrict__ zero,
                                                                 uint16_t* __restrict__ y_out,
                                                                 const uint16_t* residual, uint16_t* sum_out)   /* may be one buffer */
{
    constexpr int W = BLOCK / 64;
    __shared__ uint64_t s_lo64[W], s_hi64[W];
    __shared__ float s_r, s_min[W], s_max[W];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nvec = K >> 3, qmax = (1 << q) - 1;
    const uint4* xrow = reinterpret_cast<const uint4*>(x + (size_t)m * K);
    const uint4* grow = reinterpret_cast<const uint4*>(KIND == 0 ? gamma : gamma + (size_t)m * K);
    uint32_t xv[VPT][4], gv[VPT][4];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int v = tid + i * BLOCK;
        const uint4 a = xrow[v < nvec ? v : nvec - 1], b = grow[v < nvec ? v : nvec - 1];   // clamped: no conditional load
        const bool in = v < nvec;
        xv[i][0] = in ? a.x : 0u; xv[i][1] = in ? a.y : 0u; xv[i][2] = in ? a.z : 0u; xv[i][3] = in ? a.w : 0u;
        gv[i][0] = b.x; gv[i][1] = b.y; gv[i][2] = b.z; gv[i][3] = b.w;
    }
    if constexpr (KIND == 0) {
        if (residual) {   // x + residual first; the sum is the row that is normalized and the next residual
            const uint4* rrow = reinterpret_cast<const uint4*>(residual + (size_t)m * K);
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                const int v = tid + i * BLOCK;
                const uint4 c = rrow[v < nvec ? v : nvec - 1];
                xv[i][0] = add_half2(xv[i][0], c.x); xv[i][1] = add_half2(xv[i][1], c.y);
                xv[i][2] = add_half2(xv[i][2], c.z); xv[i][3] = add_half2(xv[i][3], c.w);
                if (v < nvec) reinterpret_cast<uint4*>(sum_out + (size_t)m * K)[v] = uint4{xv[i][0], xv[i][1], xv[i][2], xv[i][3]};
                else { xv[i][0] = 0u; xv[i][1] = 0u; xv[i][2] = 0u; xv[i][3] = 0u; }
            }
        }
    }
    float r = 0.0f;
    if constexpr (KIND == 0) {
        SquareSum acc;
#pragma unroll
        for (int i = 0; i < VPT; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) { acc.add((uint16_t)(xv[i][j] & 0xFFFFu)); acc.add((uint16_t)(xv[i][j] >> 16)); }
        uint64_t lo, hi;
        acc.fold(lo, hi);
        for (int off = 32; off > 0; off >>= 1) {
            const uint64_t l = (uint64_t)__shfl_xor((unsigned long long)lo, off, 64);
            const uint64_t h = (uint64_t)__shfl_xor((unsigned long long)hi, off, 64);
            add128(lo, hi, l, h);
        }
        if (lane == 0) { s_lo64[wave] = lo; s_hi64[wave] = hi; }
        __syncthreads();
        if (tid == 0) {
            uint64_t tl = 0, th = 0;
            for (int w = 0; w < W; ++w) add128(tl, th, s_lo64[w], s_hi64[w]);
            s_r = inv_rms(tl, th, K, eps);
        }
        __syncthreads();
        r = s_r;
    }

    // produced row (kept as binary16 bits in place of x) and its range, 0 included; padding lanes hold zeros
    float vmin = 0.0f, vmax = 0.0f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint16_t y0 = produce_half<KIND>((uint16_t)(xv[i][j] & 0xFFFFu), (uint16_t)(gv[i][j] & 0xFFFFu), r);
            const uint16_t y1 = produce_half<KIND>((uint16_t)(xv[i][j] >> 16), (uint16_t)(gv[i][j] >> 16), r);
            xv[i][j] = (uint32_t)y0 | ((uint32_t)y1 << 16);
            const float f0 = half_to_f32(y0), f1 = half_to_f32(y1);
            vmin = fminf(vmin, fminf(f0, f1));
            vmax = fmaxf(vmax, fmaxf(f0, f1));
        }
        const int v = tid + i * BLOCK;
        if (y_out && v < nvec)
            reinterpret_cast<uint4*>(y_out + (size_t)m * K)[v] = uint4{xv[i][0], xv[i][1], xv[i][2], xv[i][3]};
    }
    for (int off = 32; off > 0; off >>= 1) {
        vmin = fminf(vmin, __shfl_xor(vmin, off, 64));
        vmax = fmaxf(vmax, __shfl_xor(vmax, off, 64));
    }
    if (lane == 0) { s_min[wave] = vmin; s_max[wave] = vmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < W; ++w) { vmin = fminf(vmin, s_min[w]); vmax = fmaxf(vmax, s_max[w]); }
    float delta = 1.0f;
    int z = 0;
    if (vmax != vmin) {
        delta = __fdiv_rn(__fsub_rn(vmax, vmin), (float)qmax);
        const float zf = rintf(__fdiv_rn(-vmin, delta));
        z = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);
    }
    if (tid == 0) { scale[m] = delta; zero[m] = z; }
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        uint32_t out[2] = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int hsel = 0; hsel < 2; ++hsel) {
                const float f = half_to_f32((uint16_t)(hsel ? xv[i][j] >> 16 : xv[i][j] & 0xFFFFu));
                int c = (int)rintf(__fdiv_rn(f, delta)) + z;
                c = c < 0 ? 0 : (c > qmax ? qmax : c);
                const int e = 2 * j + hsel;
                out[e >> 2] |= (uint32_t)c << (8 * (e & 3));
            }
        }
        const int v = tid + i * BLOCK;
        if (v < nvec) reinterpret_cast<uint2*>(codes + (size_t)m * K)[v] = uint2{out[0], out[1]};
    }
}

template <int KIND, int BLOCK>
__global__ __launch_bounds__(BLOCK) void producer_quant_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ gamma,
                                                              float eps, int q, int K, uint8_t* __restrict__ codes,
                                                              float* __restrict__ scale, int32_t* __restrict__ zero,
                                                              uint16_t* __restrict__ y_out,
                                                              const uint16_t* residual, uint16_t* sum_out)   /* may be one buffer */
{
    constexpr int W = BLOCK / 64;
    __shared__ uint64_t s_lo64[W], s_hi64[W];
    __shared__ float s_r, s_min[W], s_max[W];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint16_t* row = x + (size_t)m * K;
    const int qmax = (1 << q) - 1;
    if constexpr (KIND == 0) {
        if (residual) {   // x + residual first; every later pass reads the sum (each thread re-reads only what it wrote)
            for (int k = tid; k < K; k += BLOCK) sum_out[(size_t)m * K + k] = add_half(row[k], residual[(size_t)m * K + k]);
            row = sum_out + (size_t)m * K;
        }
    }

    const uint16_t* brow = KIND == 0 ? gamma : gamma + (size_t)m * K;
    float r = 0.0f;
    if constexpr (KIND == 0) {
        // exact sum of squares (at most K / BLOCK <= 512 terms per thread)
        SquareSum acc;
        for (int k = tid; k < K; k += BLOCK) acc.add(row[k]);
        uint64_t lo, hi;
        acc.fold(lo, hi);
        for (int off = 32; off > 0; off >>= 1) {
            const uint64_t l = (uint64_t)__shfl_xor((unsigned long long)lo, off, 64);
            const uint64_t h = (uint64_t)__shfl_xor((unsigned long long)hi, off, 64);
            add128(lo, hi, l, h);
        }
        if (lane == 0) { s_lo64[wave] = lo; s_hi64[wave] = hi; }
        __syncthreads();
        if (tid == 0) {
            uint64_t tl = 0, th = 0;
            for (int w = 0; w < W; ++w) add128(tl, th, s_lo64[w], s_hi64[w]);
            s_r = inv_rms(tl, th, K, eps);
        }
        __syncthreads();
        r = s_r;
    }

    auto normalized = [&](int k) -> uint16_t { return produce_half<KIND>(row[k], brow[k], r); };

    // range of the normalized row (0 included)
    float vmin = 0.0f, vmax = 0.0f;
    for (int k = tid; k < K; k += BLOCK) {
        const uint16_t yb = normalized(k);
        if (y_out) y_out[(size_t)m * K + k] = yb;
        const float f = half_to_f32(yb);
        vmin = fminf(vmin, f);
        vmax = fmaxf(vmax, f);
    }
    for (int off = 32; off > 0; off >>= 1) {
        vmin = fminf(vmin, __shfl_xor(vmin, off, 64));
        vmax = fmaxf(vmax, __shfl_xor(vmax, off, 64));
    }
    if (lane == 0) { s_min[wave] = vmin; s_max[wave] = vmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < W; ++w) { vmin = fminf(vmin, s_min[w]); vmax = fmaxf(vmax, s_max[w]); }
    float delta = 1.0f;
    int z = 0;
    if (vmax != vmin) {
        delta = __fdiv_rn(__fsub_rn(vmax, vmin), (float)qmax);
        const float zf = rintf(__fdiv_rn(-vmin, delta));
        z = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);
    }
    if (tid == 0) { scale[m] = delta; zero[m] = z; }

    // codes
    for (int k = tid; k < K; k += BLOCK) {
        const float f = half_to_f32(normalized(k));
        int c = (int)rintf(__fdiv_rn(f, delta)) + z;
        c = c < 0 ? 0 : (c > qmax ? qmax : c);
        codes[(size_t)m * K + k] = (uint8_t)c;
    }
}

// KIND 0: b = gamma [K], eps used;  KIND 1: b = up [M,K], eps ignored.
template <int KIND>
static hipError_t launch_producer_quant(int q, int M, int K, const uint16_t* a, const uint16_t* b, float eps, uint8_t* codes,
                                        float* scale, int32_t* zero, uint16_t* y_out, hipStream_t s,
                                        const uint16_t* residual = nullptr, uint16_t* sum_out = nullptr)
{
    // rows of whole, 16-byte aligned vectors that fit a workgroup's registers take the fast path
    const bool vec_ok = K % 8 == 0 && K <= 16384 && ((uintptr_t)y_out & 15u) == 0;
    if (vec_ok && K <= 2048) producer_quant_rows_kernel<KIND, 1, 256><<<M, 256, 0, s>>>(a, b, eps, q, K, codes, scale, zero, y_out, residual, sum_out);
    else if (vec_ok && K <= 4096) producer_quant_rows_kernel<KIND, 1, 512><<<M, 512, 0, s>>>(a, b, eps, q, K, codes, scale, zero, y_out, residual, sum_out);
    else if (vec_ok && K <= 8192) producer_quant_rows_kernel<KIND, 2, 512><<<M, 512, 0, s>>>(a, b, eps, q, K, codes, scale, zero, y_out, residual, sum_out);
    else if (vec_ok) producer_quant_rows_kernel<KIND, 4, 512><<<M, 512, 0, s>>>(a, b, eps, q, K, codes, scale, zero, y_out, residual, sum_out);
    else producer_quant_kernel<KIND, 256><<<M, 256, 0, s>>>(a, b, eps, q, K, codes, scale, zero, y_out, residual, sum_out);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_quant(int q, int M, int K, const uint16_t* x, const uint16_t* gamma, float eps, uint8_t* codes,
                                float* scale, int32_t* zero, uint16_t* y_out, hipStream_t s)
{
    return launch_producer_quant<0>(q, M, K, x, gamma, eps, codes, scale, zero, y_out, s);
}

hipError_t launch_add_rmsnorm_quant(int q, int M, int K, const uint16_t* x, const uint16_t* residual, const uint16_t* gamma, float eps,
                                    uint8_t* codes, float* scale, int32_t* zero, uint16_t* sum_out, uint16_t* y_out, hipStream_t s)
{
    return launch_producer_quant<0>(q, M, K, x, gamma, eps, codes, scale, zero, y_out, s, residual, sum_out);
}

hipError_t launch_silu_mul_quant(int q, int M, int K, const uint16_t* gate, const uint16_t* up, uint8_t* codes, float* scale,
                                 int32_t* zero, uint16_t* h_out, hipStream_t s)
{
    return launch_producer_quant<1>(q, M, K, gate, up, 0.0f, codes, scale, zero, h_out, s);
}

}  // namespace abq
