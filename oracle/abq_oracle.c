/*
 * CPU oracle for the arbitrary-precision quantized matmul of ABQ-LLM (arXiv 2408.08554).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP path and the
 * product never calls it: only tests, the smoke check and the bench's cpu_baseline leg do.
 *
 * Notation (Appendix B of the paper; p = weight bits, q = activation bits):
 *   A  uint8 [M,K] row-major activation codes, 0 <= A < 2^q
 *   W  uint8 [N,K] row-major weight codes,     0 <= W < 2^p
 *   acc[m,n] = sum_k A[m,k] * W[n,k]                         ("32-bit output Y = W X", Sec. 3.4)
 *
 * The bit-plane method of Sec. 3.4 / Appendix B (Eq. "formula:matrix") reaches this integer
 * exactly, so the oracle for the accumulator is the plain product sum in int64;
 * abq_oracle_acc_bitplane() is the literal decomposition, kept as an independent second path.
 *
 * Affine semantics (Eq. 3: codes are clamp(round(x/Delta)+z, 0, 2^n-1), so the real value
 * of a code c is Delta*(c - z); weights per output channel, activations per token, Sec. 4.1):
 *   accc[m,n] = sum_k (A[m,k]-az[m]) * (W[n,k]-wz[n])         computed directly, term by term
 *   Y[m,n]    = (double)accc * (double)a_scale[m] * (double)w_scale[n], then RNE to binary16.
 * The paper names the DeQuant step (Fig. 3b) but prints no formula; the lines above are the
 * reading this build takes.
 *
 * Parity status: accumulator, centered accumulator, dequant, half rounding, plane packing are
 * pinned by tests (brute force, library matmul, closed forms, long-double dequantise-then-
 * multiply, numpy's float16 conversion).  abq_oracle_quant_act: PARITY UNPINNED by the paper
 * (it only says "per-token"); pinned by invariants only.  abq_oracle_rmsnorm_half (the producer
 * the quantizer is fused into): the paper prints no formula; pinned against a float64 numpy
 * evaluation of the standard definition, closed forms and invariances.  abq_oracle_silu_mul_half
 * (the second producer): pinned against a float64 evaluation with the library exp and closed forms.
 * abq_oracle_add_half (the residual add in front of the normalization): pinned against numpy's float32
 * addition and float16 conversion, identities, ties and overflow.  abq_oracle_dequant_grouped (per-group
 * weight scales and zero-points, Appendix C): pinned by its reductions to the per-channel result (one group;
 * equal parameters in every group), a long-double dequantise-then-multiply with every weight under its own
 * group's parameters, and single-live-group closed forms including the short last group.
 * abq_oracle_requant (the matmul output quantized again with given per-token parameters): PARITY UNPINNED by the
 * paper; pinned by its reduction to abq_oracle_quant_act, grid round trips, saturation, ties and monotonicity.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int abq_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* acc[m,n] = sum_k A[m,k]*W[n,k]  (Sec. 3.4: Y = W X with a 32-bit result; here int64). */
void abq_oracle_acc(int M, int N, int K, const uint8_t* A, const uint8_t* W, int64_t* acc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int k = 0; k < K; ++k)
                s += (int64_t)A[(size_t)m * K + k] * (int64_t)W[(size_t)n * K + k];
            acc[(size_t)m * N + n] = s;
        }
    }
}

/* Same sum, but only at the listed (m,n) pairs: for sampled checks at sizes where the full
 * triple loop would take minutes. */
void abq_oracle_acc_sampled(int M, int N, int K, const uint8_t* A, const uint8_t* W,
                            int64_t count, const int32_t* ms, const int32_t* ns, int64_t* acc)
{
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const uint8_t* a = A + (size_t)ms[i] * K;
        const uint8_t* w = W + (size_t)ns[i] * K;
        int64_t s = 0;
        for (int k = 0; k < K; ++k) s += (int64_t)a[k] * (int64_t)w[k];
        acc[i] = s;
    }
}

/* accc[m,n] = sum_k (A[m,k]-az[m]) * (W[n,k]-wz[n])   (Eq. 3 semantics, direct form). */
void abq_oracle_acc_centered(int M, int N, int K, const uint8_t* A, const uint8_t* W,
                             const int32_t* az, const int32_t* wz, int64_t* accc)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int k = 0; k < K; ++k)
                s += ((int64_t)A[(size_t)m * K + k] - az[m]) * ((int64_t)W[(size_t)n * K + k] - wz[n]);
            accc[(size_t)m * N + n] = s;
        }
    }
}

void abq_oracle_acc_centered_sampled(int M, int N, int K, const uint8_t* A, const uint8_t* W,
                                     const int32_t* az, const int32_t* wz, int64_t count,
                                     const int32_t* ms, const int32_t* ns, int64_t* accc)
{
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int m = ms[i], n = ns[i];
        int64_t s = 0;
        for (int k = 0; k < K; ++k)
            s += ((int64_t)A[(size_t)m * K + k] - az[m]) * ((int64_t)W[(size_t)n * K + k] - wz[n]);
        accc[i] = s;
    }
}

/* Round a double to IEEE binary16, round-to-nearest-even, returned as its bit pattern.
 * Written from the format definition: 1 sign, 5 exponent (bias 15), 10 fraction bits;
 * smallest subnormal 2^-24, largest finite 65504, overflow to infinity. */
uint16_t abq_oracle_half_bits(double v)
{
    uint16_t sign = 0;
    if (signbit(v)) { sign = 0x8000u; v = -v; }
    if (isnan(v)) return (uint16_t)(sign | 0x7E00u);
    if (isinf(v)) return (uint16_t)(sign | 0x7C00u);
    if (v == 0.0) return sign;
    int e;
    (void)frexp(v, &e);            /* v = f * 2^e with f in [0.5,1)  =>  v in [2^(e-1), 2^e) */
    int ex = e - 1;                /* unbiased exponent of the leading bit */
    if (ex < -14) ex = -14;        /* subnormal range: fixed quantum 2^-24 */
    /* quantum of the target grid at this exponent */
    const double quantum = ldexp(1.0, ex - 10);
    double scaled = v / quantum;   /* exact: division by a power of two */
    double r = nearbyint(scaled);  /* default rounding mode = nearest-even */
    /* r is an integer in [0, 2048]; 2048 means carry into the next binade */
    double back = r * quantum;
    if (back >= 65520.0) return (uint16_t)(sign | 0x7C00u);   /* rounds past the largest finite */
    if (back == 0.0) return sign;
    int e2;
    (void)frexp(back, &e2);
    int ex2 = e2 - 1;
    if (ex2 < -14) {
        /* subnormal: fraction field counts multiples of 2^-24 */
        uint16_t frac = (uint16_t)(back / ldexp(1.0, -24));
        return (uint16_t)(sign | frac);
    }
    uint16_t frac = (uint16_t)(back / ldexp(1.0, ex2 - 10) - 1024.0);
    return (uint16_t)(sign | (uint16_t)((ex2 + 15) << 10) | frac);
}

/* Y = accc * a_scale[m] * w_scale[n] in double; y16 = RNE(binary16).  Either output may be NULL. */
void abq_oracle_dequant(int M, int N, const int64_t* accc, const float* a_scale,
                        const float* w_scale, double* y, uint16_t* y16)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double v = (double)accc[(size_t)m * N + n] * (double)a_scale[m] * (double)w_scale[n];
            if (y) y[(size_t)m * N + n] = v;
            if (y16) y16[(size_t)m * N + n] = abq_oracle_half_bits(v);
        }
    }
}

/* Per-group weight quantization (Appendix C: the weight row is cut along K into groups of gs
 * values, e.g. 128, each with its own scale and zero-point; activations stay per token):
 *   Y[m][n] = a_scale[m] * sum_g w_scale[n][g] * sum_{k in group g} (A[m][k] - az[m]) * (W[n][k] - wz[n][g])
 * with group g = k / gs (the last group may be short), G = ceil(K / gs) groups per row.  The inner
 * sums are exact integers; the sum over groups is taken in double in the order g = 0, 1, ...
 * Group scales are binary16 values (given as bit patterns), the way deployed group formats store them.
 * y, y16 and mag may be NULL; mag[m][n] = a_scale[m] * sum_g |w_scale[n][g] * inner_g| is the size of
 * the terms the sum is made of (what a single-precision evaluation's rounding error scales with). */
static float half_to_float(uint16_t h);
void abq_oracle_dequant_grouped(int M, int N, int K, int gs, const uint8_t* A, const uint8_t* W,
                                const int32_t* az, const float* a_scale, const int32_t* wz,
                                const uint16_t* w_scale_half, double* y, uint16_t* y16, double* mag)
{
    const int G = (K + gs - 1) / gs;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            double total = 0.0, size = 0.0;
            for (int g = 0; g < G; ++g) {
                const int k_end = (g + 1) * gs < K ? (g + 1) * gs : K;
                int64_t inner = 0;
                for (int k = g * gs; k < k_end; ++k)
                    inner += ((int64_t)A[(size_t)m * K + k] - az[m]) * ((int64_t)W[(size_t)n * K + k] - wz[(size_t)n * G + g]);
                const double term = (double)half_to_float(w_scale_half[(size_t)n * G + g]) * (double)inner;
                total += term;
                size += fabs(term);
            }
            const double v = (double)a_scale[m] * total;
            if (y) y[(size_t)m * N + n] = v;
            if (y16) y16[(size_t)m * N + n] = abq_oracle_half_bits(v);
            if (mag) mag[(size_t)m * N + n] = fabs((double)a_scale[m]) * size;
        }
    }
}

/* BitPacking (Sec. 3.4 step 1): bit view [R,K,bits] -> [bits,R,K]; plane s holds
 * (code >> s) & 1 (Appendix B).  Each plane row is stored as 32-bit words, bit (k mod 32) of
 * word k/32, zero padded to Kw words (the word order inside a plane is this build's choice,
 * the paper only fixes the [bits,R,K] order). */
void abq_oracle_pack_planes(int bits, int R, int K, int Kw, const uint8_t* codes, uint32_t* planes)
{
    memset(planes, 0, (size_t)bits * R * Kw * sizeof(uint32_t));
    for (int s = 0; s < bits; ++s)
        for (int r = 0; r < R; ++r)
            for (int k = 0; k < K; ++k)
                if ((codes[(size_t)r * K + k] >> s) & 1u)
                    planes[((size_t)s * R + r) * Kw + (k >> 5)] |= (uint32_t)1u << (k & 31);
}

void abq_oracle_unpack_planes(int bits, int R, int K, int Kw, const uint32_t* planes, uint8_t* codes)
{
    for (int r = 0; r < R; ++r)
        for (int k = 0; k < K; ++k) {
            unsigned c = 0;
            for (int s = 0; s < bits; ++s)
                c |= ((planes[((size_t)s * R + r) * Kw + (k >> 5)] >> (k & 31)) & 1u) << s;
            codes[(size_t)r * K + k] = (uint8_t)c;
        }
}

static int popcount32(uint32_t v)
{
    int c = 0;
    while (v) { c += (int)(v & 1u); v >>= 1; }
    return c;
}

/* The literal method (Appendix B): Y = sum_{s<p} sum_{t<q} 2^(s+t) * BMMA(W^s, X^t), where the
 * 1-bit product is AND and the 1-bit matmul counts the set bits of (A_t AND W_s) along K.
 * Takes host-packed planes as laid out by abq_oracle_pack_planes. */
void abq_oracle_acc_bitplane(int p, int q, int M, int N, int Kw,
                             const uint32_t* a_planes, const uint32_t* w_planes, int64_t* acc)
{
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int64_t y = 0;
            for (int s = 0; s < p; ++s)
                for (int t = 0; t < q; ++t) {
                    int64_t yst = 0;
                    const uint32_t* wr = w_planes + ((size_t)s * N + n) * Kw;
                    const uint32_t* ar = a_planes + ((size_t)t * M + m) * Kw;
                    for (int kw = 0; kw < Kw; ++kw) yst += popcount32(ar[kw] & wr[kw]);
                    y += yst * ((int64_t)1 << (s + t));
                }
            acc[(size_t)m * N + n] = y;
        }
}

/* binary16 bit pattern -> float (exact). */
static float half_to_float(uint16_t h)
{
    const int sign = (h >> 15) & 1, ex = (h >> 10) & 0x1F, fr = h & 0x3FF;
    double v;
    if (ex == 0) v = ldexp((double)fr, -24);
    else if (ex == 31) v = fr ? NAN : INFINITY;
    else v = ldexp((double)(fr + 1024), ex - 25);
    return (float)(sign ? -v : v);
}

/* ReQuant of a matmul output with parameters fixed ahead of the call (Fig. 3b: the kernel's output is quantized
 * again for the next layer; the last paragraph of Sec. 3.4 folds that step into a neighbouring operator, here the
 * matmul's own epilogue).  A token's range is not known before its whole output row exists, so the fused step takes
 * Delta and z per token from the caller (a calibrated or previous-step range) and applies Eq. 3's
 * clamp(round(x/Delta)+z) to the binary16 output value, in IEEE binary32 like the per-token quantizer below:
 *   code[m,n] = clamp( clamp(rint(y[m,n] / Delta[m]), -2^24, 2^24) + z[m], 0, 2^q-1 )
 * (the inner clamp only keeps the integer sum in range for any Delta > 0).  PARITY UNPINNED by the paper (it prints
 * no formula for ReQuant); pinned by its reduction to abq_oracle_quant_act when Delta and z are that function's own,
 * grid round trips, saturation, ties and monotonicity.  NaN/Inf inputs and Delta <= 0 are undefined. */
void abq_oracle_requant(int q, int M, int N, const uint16_t* y_half, const float* scale, const int32_t* zero,
                        uint8_t* codes)
{
    const int qmax = (1 << q) - 1;
    for (int m = 0; m < M; ++m) {
        volatile float delta = scale[m];
        const int z = zero[m];
        for (int n = 0; n < N; ++n) {
            float y = half_to_float(y_half[(size_t)m * N + n]);
            volatile float t = y / delta;
            float rn = nearbyintf(t);
            if (rn < -16777216.0f) rn = -16777216.0f;
            if (rn > 16777216.0f) rn = 16777216.0f;
            int c = (int)rn + z;
            codes[(size_t)m * N + n] = (uint8_t)(c < 0 ? 0 : (c > qmax ? qmax : c));
        }
    }
}

/* Per-token activation quantizer (the paper says only "per-token", Sec. 4.1; Eq. 3 gives the
 * clamp(round(x/Delta)+z) form).  PARITY UNPINNED by the paper.  Reading taken here, all in
 * IEEE binary32 because the float results decide integer codes:
 *   lo = min(min_k x, 0), hi = max(max_k x, 0); Delta = (hi-lo)/(2^q-1); if hi==lo: Delta=1,z=0
 *   z = clamp(rint(-lo/Delta), 0, 2^q-1); code = clamp(rint(x/Delta)+z, 0, 2^q-1)
 * rint = round-half-to-even.  NaN/Inf inputs are undefined. */
void abq_oracle_quant_act(int q, int M, int K, const uint16_t* x_half, uint8_t* codes,
                          float* a_scale, int32_t* a_zero)
{
    const int qmax = (1 << q) - 1;
    for (int m = 0; m < M; ++m) {
        float lo = 0.0f, hi = 0.0f;
        for (int k = 0; k < K; ++k) {
            float x = half_to_float(x_half[(size_t)m * K + k]);
            if (x < lo) lo = x;
            if (x > hi) hi = x;
        }
        volatile float delta;
        int z;
        if (hi == lo) { delta = 1.0f; z = 0; }
        else {
            volatile float range = hi - lo;
            delta = range / (float)qmax;
            volatile float zr = (-lo) / delta;
            float zf = nearbyintf(zr);
            z = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);
        }
        a_scale[m] = delta;
        a_zero[m] = z;
        for (int k = 0; k < K; ++k) {
            float x = half_to_float(x_half[(size_t)m * K + k]);
            volatile float t = x / delta;
            float r = nearbyintf(t);
            /* r is integral and |r| <= 2^q-1 here, so the int sum is exact */
            int c = (int)r + z;
            codes[(size_t)m * K + k] = (uint8_t)(c < 0 ? 0 : (c > qmax ? qmax : c));
        }
    }
}

/* Residual add in front of the normalization (the LLaMA block adds a sub-layer's output to the hidden state and
 * normalizes the sum; the sum is also the next residual, so it is materialised in binary16):
 *     h[i] = half_rne( float(a[i]) + float(b[i]) )          one binary32 addition, then one rounding to binary16
 * (two binary16 values can be 40 binades apart, so the binary32 sum is not always exact: the two roundings are
 * part of the definition). */
void abq_oracle_add_half(size_t n, const uint16_t* a_half, const uint16_t* b_half, uint16_t* h_half)
{
    for (size_t i = 0; i < n; ++i) {
        volatile float s = half_to_float(a_half[i]) + half_to_float(b_half[i]);
        h_half[i] = abq_oracle_half_bits((double)s);
    }
}

/* RMSNorm to binary16, the producer that Sec. 3.4 / Fig. 3b fuse the activation quantizer into
 * (the paper quantizes the input of every linear layer of LLaMA, whose normalization is RMSNorm;
 * the paper prints no formula for it, so this is the standard definition):
 *     y[k] = x[k] / sqrt(mean_k(x[k]^2) + eps) * gamma[k]
 * The results feed a quantizer, i.e. they decide integer codes, so every rounding is spelled out:
 *   - sum_k x[k]^2 is taken EXACTLY (x is binary16, so 2^48 * x^2 is an integer below 2^81; the sum
 *     is an integer in 128 bits and does not depend on the order of summation),
 *   - ss   = double(high 64 bits) * 2^64 + double(low 64 bits), scaled by 2^-48   (one rounding at most)
 *   - mean = ss / K;  r = (float)(1.0 / sqrt(mean + (double)eps))                (double ops, then one rounding)
 *   - y[k] = half_rne( (float(x[k]) * r) * float(gamma[k]) )                    (two float products)
 * NaN/Inf inputs are undefined. */
void abq_oracle_rmsnorm_half(int M, int K, const uint16_t* x_half, const uint16_t* gamma_half, float eps,
                             uint16_t* y_half)
{
    for (int m = 0; m < M; ++m) {
        unsigned __int128 sum = 0;
        for (int k = 0; k < K; ++k) {
            const double x = (double)half_to_float(x_half[(size_t)m * K + k]);
            const double scaled = x * x * 281474976710656.0;      /* 2^48: exact, an integer */
            sum += (unsigned __int128)scaled;
        }
        const uint64_t hi = (uint64_t)(sum >> 64), lo = (uint64_t)sum;
        const double ss = ((double)hi * 18446744073709551616.0 + (double)lo) * (1.0 / 281474976710656.0);
        const double mean = ss / (double)K;
        volatile float r = (float)(1.0 / sqrt(mean + (double)eps));
        for (int k = 0; k < K; ++k) {
            volatile float t = half_to_float(x_half[(size_t)m * K + k]) * r;
            volatile float u = t * half_to_float(gamma_half[k]);
            y_half[(size_t)m * K + k] = abq_oracle_half_bits((double)u);
        }
    }
}

/* SiLU(gate) * up to binary16: the producer in front of down_proj in the LLaMA MLP, the other operator
 * Sec. 3.4 / Fig. 3b fuse the activation quantizer into.  silu(g) = g / (1 + exp(-g)).  The result
 * decides integer codes, so exp is not left to a math library (two libraries differ in the last bits);
 * it is the following sequence of single IEEE binary32 operations, the same on every machine:
 *   t = clamp(-g * log2(e), -126, 126);  n = rint(t);  f = t - n      (f in [-1/2, 1/2], exact)
 *   2^f = 1 + f*(c1 + f*(c2 + f*(c3 + f*(c4 + f*(c5 + f*c6)))))        (c_k = ln(2)^k / k!, Horner, no fma)
 *   e = 2^f * 2^n;   h = half_rne( (g / (1 + e)) * up )
 * Its distance from the real exp is below 2 * 10^-7 relative, far inside half an ulp of binary16.
 * NaN/Inf inputs are undefined. */
static float oracle_exp2_poly(float f)
{
    static const float c1 = 0x1.62e430p-1f, c2 = 0x1.ebfbe0p-3f, c3 = 0x1.c6b08ep-5f, c4 = 0x1.3b2ab6p-7f,
                       c5 = 0x1.5d87fep-10f, c6 = 0x1.430912p-13f;
    volatile float p = f * c6;
    p = p + c5; p = p * f;
    p = p + c4; p = p * f;
    p = p + c3; p = p * f;
    p = p + c2; p = p * f;
    p = p + c1; p = p * f;
    p = p + 1.0f;
    return p;
}

void abq_oracle_silu_mul_half(int M, int K, const uint16_t* gate_half, const uint16_t* up_half, uint16_t* h_half)
{
    for (size_t i = 0; i < (size_t)M * K; ++i) {
        const float g = half_to_float(gate_half[i]), u = half_to_float(up_half[i]);
        volatile float t = -g * 0x1.715476p+0f;
        if (t < -126.0f) t = -126.0f;
        if (t > 126.0f) t = 126.0f;
        const float n = nearbyintf(t);
        volatile float f = t - n;
        volatile float e = ldexpf(oracle_exp2_poly(f), (int)n);
        volatile float s = 1.0f + e;
        volatile float sg = g / s;
        volatile float h = sg * u;
        h_half[i] = abq_oracle_half_bits((double)h);
    }
}
