// Packing kernels: weight BitPacking (offline), activation BitPacking / ReQuant (online),
// and the decode hooks the tests use.  Sec. 3.4 step 1 and Fig. 3b of the paper.
#include "abq_internal.h"
#include "../../include/abq.h"

#include <hip/hip_fp16.h>

namespace abq {

// ---- blob header -----------------------------------------------------------------------------
__global__ void write_header_kernel(uint32_t* hdr, uint32_t magic, int bits, int R, int K, int layout)
{
    const int t = threadIdx.x;
    uint32_t v = 0;
    if (t == 0) v = magic;
    else if (t == 1) v = 1;          // format version
    else if (t == 2) v = (uint32_t)bits;
    else if (t == 3) v = (uint32_t)R;
    else if (t == 4) v = (uint32_t)K;
    else if (t == 5) v = (uint32_t)layout;
    if (t < kHeaderBytes / 4) hdr[t] = v;
}

// ---- 1-bit planes: [bits][R][Kw] words, bit (k mod 32) of word k/32 ---------------------------
// One thread per output word; codes above K are zero bits.
__global__ void pack_planes_kernel(const uint8_t* __restrict__ codes, int bits, int R, int K, int Kw,
                                   uint32_t* __restrict__ planes)
{
    const size_t total = (size_t)R * Kw;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int r = (int)(idx / Kw), kw = (int)(idx % Kw);
    uint32_t word[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int k0 = kw * 32;
    for (int i = 0; i < 32; ++i) {
        const int k = k0 + i;
        const uint32_t c = (k < K) ? codes[(size_t)r * K + k] : 0u;
#pragma unroll
        for (int s = 0; s < 8; ++s) word[s] |= ((c >> s) & 1u) << i;
    }
    for (int s = 0; s < bits; ++s) planes[((size_t)s * R + r) * Kw + kw] = word[s];
}

__global__ void unpack_planes_kernel(const uint32_t* __restrict__ planes, int bits, int R, int K, int Kw,
                                     uint8_t* __restrict__ codes)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)R * K) return;
    const int r = (int)(idx / K), k = (int)(idx % K);
    uint32_t c = 0;
    for (int s = 0; s < bits; ++s) c |= ((planes[((size_t)s * R + r) * Kw + (k >> 5)] >> (k & 31)) & 1u) << s;
    codes[idx] = (uint8_t)c;
}

// ---- weight plane groups, tiled for the 16x16x64 int8 MFMA -------------------------------------
// One group of width b (planes shift..shift+b-1 of every weight) is stored as 1 KiB chunks,
// chunk (nt, c) = rows nt*16..+15, k = c*(512/b) .. +512/b-1.  Inside a chunk lane l = 16*G + r
// owns 16 bytes (dwords j = 0..3, bytes cc = 0..3); byte (j,cc) carries the 8/b fields
// t = 0..8/b-1 at bit b*t, field t being weight (row nt*16+r, k = c*(512/b) + t*64 + G*16 + 4*j + cc).
// Masking all four dwords with the mask of field t therefore yields the B operand of one MFMA
// over the 64 k-values of slice t.  8-bit groups are stored as w - 128 (the MFMA is signed).
// pad_zero (null for per-channel blobs): per-group zero-points [N][G]; k from K up to the end of the last group of
// 128 is then filled with that group's zero-point instead of 0, so that (w - zero) vanishes there.
__global__ void pack_fields_kernel(const uint8_t* __restrict__ w, int N, int K, int b, int shift, int chunks,
                                   size_t total_dwords, uint32_t* __restrict__ out, const int32_t* __restrict__ pad_zero = nullptr,
                                   int ngroups128 = 0)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total_dwords) return;
    const int j = (int)(idx & 3), l = (int)((idx >> 2) & 63);
    const size_t chunk = idx >> 8;
    const int c = (int)(chunk % chunks), nt = (int)(chunk / chunks);
    const int G = l >> 4, r = l & 15;
    const int n = nt * kTileN + r;
    const int T = 8 / b, kchunk = kSuperK / b;
    const uint32_t fmask = (1u << b) - 1u;
    uint32_t dword = 0;
    for (int cc = 0; cc < 4; ++cc) {
        uint32_t byte = 0;
        for (int t = 0; t < T; ++t) {
            const int k = c * kchunk + t * 64 + G * 16 + 4 * j + cc;
            uint32_t code = (n < N && k < K) ? w[(size_t)n * K + k] : 0u;
            if (pad_zero && n < N && k >= K && k < ngroups128 * 128) code = (uint32_t)pad_zero[(size_t)n * ngroups128 + (ngroups128 - 1)];
            uint32_t f = (code >> shift) & fmask;
            if (b == 8) f ^= 0x80u;
            byte |= f << (b * t);
        }
        dword |= byte << (8 * cc);
    }
    out[idx] = dword;
}

__global__ void unpack_fields_kernel(const uint8_t* __restrict__ blob, WeightLayout L, uint8_t* __restrict__ codes)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)L.N * L.K) return;
    const int n = (int)(idx / L.K), k = (int)(idx % L.K);
    uint32_t code = 0;
    for (int g = 0; g < L.ngroups; ++g) {
        const int b = L.gb[g], kchunk = kSuperK / b;
        const int c = k / kchunk, rem = k % kchunk;
        const int t = rem / 64, G = (rem % 64) / 16, j = (rem % 16) / 4, cc = rem % 4;
        const int l = G * 16 + (n % kTileN);
        const uint32_t* base = (const uint32_t*)(blob + L.off_fields[g]);
        const uint32_t dword = base[(((size_t)(n / kTileN) * L.chunks[g] + c) * 64 + l) * 4 + j];
        uint32_t f = ((dword >> (8 * cc)) >> (b * t)) & ((1u << b) - 1u);
        if (b == 8) f ^= 0x80u;
        code |= f << L.gs[g];
    }
    codes[idx] = (uint8_t)code;
}

// ---- per-row parameters ------------------------------------------------------------------------
// One wave per row: sum of the (masked) codes, plus copies of scale and zero.
__global__ void row_params_kernel(const uint8_t* __restrict__ codes, int bits, int R, int K,
                                  const float* __restrict__ scale, const int32_t* __restrict__ zero,
                                  RowParams* __restrict__ out)
{
    const int row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= R) return;
    const uint32_t mask = (1u << bits) - 1u;
    int32_t s = 0;
    for (int k = lane; k < K; k += 64) s += (int32_t)(codes[(size_t)row * K + k] & mask);
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) out[row] = RowParams{s, scale[row], zero[row], 0};
}

// ---- per-group weight parameters (groups of 128 along K, Appendix C) ------------------------------
// One thread per (tile, super-chunk, channel): the 16-byte record the streaming kernel loads with the
// super-chunk's weights.  Groups past ceil(K/128) and channels past N get scale 0 and zero-point 0.
__global__ void group_params_kernel(const uint16_t* __restrict__ scale_half, const int32_t* __restrict__ zero, int N, int G,
                                    int nsuper, int NT, int ow, uint4* __restrict__ out)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)NT * nsuper * 16) return;
    const int c = (int)(idx & 15), sc = (int)((idx >> 4) % nsuper), nt = (int)((idx >> 4) / nsuper);
    const int n = nt * kTileN + c;
    uint32_t sh[4], zz = 0;
    for (int j = 0; j < 4; ++j) {
        const int g = sc * 4 + j;
        const bool live = n < N && g < G;
        sh[j] = live ? scale_half[(size_t)n * G + g] : 0u;
        const int z = live ? zero[(size_t)n * G + g] - ow : 0;
        zz |= ((uint32_t)z & 0xFFu) << (8 * j);
    }
    out[idx] = uint4{sh[0] | (sh[1] << 16), sh[2] | (sh[3] << 16), zz, 0u};
}

// g128 blobs keep the per-channel parameter area (all zero: every parameter lives in the group records).
__global__ void zero_params_kernel(RowParams* __restrict__ out, int N)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) out[i] = RowParams{0, 0.0f, 0, 0};
}

// ---- activation rows: codes (given, or quantized here) -> int8 rows + 1-bit planes ---------------
// One workgroup per token m.  Thread units of 32 consecutive k: 32 codes -> two uint4 of int8
// (a - oa, oa = 128 when q == 8 so that the value fits the signed MFMA operand; zero beyond K
// up to Kp) and one word per plane.  SRC_HALF: the codes come from the per-token quantizer
//   lo = min(min_k x,0), hi = max(max_k x,0), Delta = (hi-lo)/(2^q-1) (1 if hi==lo),
//   z = clamp(rint(-lo/Delta)), code = clamp(rint(x/Delta)+z)
// with every float step a single correctly rounded binary32 operation, since they decide
// integer codes.
__device__ __forceinline__ float half_bits_to_float(uint16_t h) { return __half2float(__ushort_as_half(h)); }

template <bool SRC_HALF, int BLOCK>
__global__ __launch_bounds__(BLOCK) void act_rows_kernel(const void* __restrict__ src, const float* __restrict__ a_scale,
                                                         const int32_t* __restrict__ a_zero, ActLayout L,
                                                         uint8_t* __restrict__ blob)
{
    __shared__ float s_lo[BLOCK / 64], s_hi[BLOCK / 64];
    __shared__ int32_t s_sum[BLOCK / 64];
    __shared__ float s_delta;
    __shared__ int s_zero;
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = L.q, K = L.K, qmax = (1 << q) - 1;
    if (m == 0 && tid < kHeaderBytes / 4) {
        uint32_t v = 0;
        if (tid == 0) v = kMagicA; else if (tid == 1) v = 1; else if (tid == 2) v = (uint32_t)q;
        else if (tid == 3) v = (uint32_t)L.M; else if (tid == 4) v = (uint32_t)K; else if (tid == 5) v = (uint32_t)L.layout;
        ((uint32_t*)blob)[tid] = v;
    }
    float delta = 1.0f;
    int z = 0;
    if (SRC_HALF) {
        const uint16_t* row = (const uint16_t*)src + (size_t)m * K;
        float lo = 0.0f, hi = 0.0f;
        for (int k = tid; k < K; k += BLOCK) {
            const float v = half_bits_to_float(row[k]);
            lo = fminf(lo, v);
            hi = fmaxf(hi, v);
        }
        for (int off = 32; off > 0; off >>= 1) {
            lo = fminf(lo, __shfl_xor(lo, off, 64));
            hi = fmaxf(hi, __shfl_xor(hi, off, 64));
        }
        if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < BLOCK / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
            float d = 1.0f;
            int zz = 0;
            if (hi != lo) {
                d = __fdiv_rn(__fsub_rn(hi, lo), (float)qmax);
                const float zf = rintf(__fdiv_rn(-lo, d));
                zz = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);
            }
            s_delta = d;
            s_zero = zz;
        }
        __syncthreads();
        delta = s_delta;
        z = s_zero;
    }
    const int oa = (q == 8) ? 128 : 0;
    const uint32_t mask = (uint32_t)qmax;
    const int units = L.Kp / 32;
    int8_t* out_bytes = L.has_fields ? (int8_t*)(blob + L.off_codes) + (size_t)m * L.Kp : nullptr;
    uint32_t* out_planes = L.has_planes ? (uint32_t*)(blob + L.off_planes) : nullptr;
    int32_t sum = 0;
    for (int u = tid; u < units; u += BLOCK) {
        const int k0 = u * 32;
        uint32_t dw[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        uint32_t pl[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int i = 0; i < 32; ++i) {
            const int k = k0 + i;
            if (k < K) {
                uint32_t c;
                if (SRC_HALF) {
                    const float v = half_bits_to_float(((const uint16_t*)src)[(size_t)m * K + k]);
                    int ci = (int)rintf(__fdiv_rn(v, delta)) + z;
                    c = (uint32_t)(ci < 0 ? 0 : (ci > qmax ? qmax : ci));
                } else {
                    c = ((const uint8_t*)src)[(size_t)m * K + k] & mask;
                }
                sum += (int32_t)c;
                dw[i >> 2] |= ((uint32_t)((int)c - oa) & 0xFFu) << (8 * (i & 3));
#pragma unroll
                for (int s = 0; s < 8; ++s) pl[s] |= ((c >> s) & 1u) << i;
            }
        }
        if (out_bytes) {
            uint4* o = reinterpret_cast<uint4*>(out_bytes + k0);
            o[0] = make_uint4(dw[0], dw[1], dw[2], dw[3]);
            o[1] = make_uint4(dw[4], dw[5], dw[6], dw[7]);
        }
        if (out_planes && u < L.Kw)
            for (int s = 0; s < q; ++s) out_planes[((size_t)s * L.M + m) * L.Kw + u] = pl[s];
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) s_sum[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        int32_t t = 0;
        for (int w = 0; w < BLOCK / 64; ++w) t += s_sum[w];
        RowParams* params = (RowParams*)(blob + L.off_params);
        params[m] = SRC_HALF ? RowParams{t, delta, z, 0} : RowParams{t, a_scale[m], a_zero[m], 0};
    }
}

// ---- fast path of the same step: int8 rows only (no planes), rows 16-byte aligned -----------------
// One workgroup per token; a thread handles 16 consecutive k per step with 128-bit loads and
// stores.  The first two steps of a thread stay in registers between the min/max pass and the
// quantizing pass (rows up to 32*BLOCK elements are read once).
__device__ __forceinline__ void half8_to_float(const uint4& v, float* f)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
        f[2 * i + 1] = half_bits_to_float((uint16_t)(w[i] >> 16));
    }
}

template <bool SRC_HALF, int BLOCK>
__global__ __launch_bounds__(BLOCK) void act_rows_fast_kernel(const void* __restrict__ src, const float* __restrict__ a_scale,
                                                              const int32_t* __restrict__ a_zero, ActLayout L,
                                                              uint8_t* __restrict__ blob)
{
    __shared__ float s_lo[BLOCK / 64], s_hi[BLOCK / 64];
    __shared__ int32_t s_sum[BLOCK / 64];
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = L.q, K = L.K, qmax = (1 << q) - 1;
    const int nvalid = K / 16, nblk = L.Kp / 16;       // 16-element blocks with data / in the padded row
    if (m == 0 && tid < kHeaderBytes / 4) {
        uint32_t v = 0;
        if (tid == 0) v = kMagicA; else if (tid == 1) v = 1; else if (tid == 2) v = (uint32_t)q;
        else if (tid == 3) v = (uint32_t)L.M; else if (tid == 4) v = (uint32_t)K; else if (tid == 5) v = (uint32_t)L.layout;
        ((uint32_t*)blob)[tid] = v;
    }
    // SRC_HALF: 16 halves = two uint4; codes: one uint4
    constexpr int VPB = SRC_HALF ? 2 : 1;
    const uint4* row = (const uint4*)src + (size_t)m * nvalid * VPB;
    uint4 keep[2][VPB];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + i * BLOCK;
#pragma unroll
        for (int v = 0; v < VPB; ++v) keep[i][v] = e < nvalid ? row[(size_t)e * VPB + v] : make_uint4(0, 0, 0, 0);
    }
    float delta = 1.0f;
    int z = 0;
    if (SRC_HALF) {
        float lo = 0.0f, hi = 0.0f;
        for (int e = tid; e < nvalid; e += BLOCK) {
            float f[16];
            if (e < 2 * BLOCK) {
                half8_to_float(keep[e >= BLOCK ? 1 : 0][0], f);
                half8_to_float(keep[e >= BLOCK ? 1 : 0][VPB - 1], f + 8);
            } else {
                half8_to_float(row[(size_t)e * VPB], f);
                half8_to_float(row[(size_t)e * VPB + VPB - 1], f + 8);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) { lo = fminf(lo, f[i]); hi = fmaxf(hi, f[i]); }
        }
        for (int off = 32; off > 0; off >>= 1) {
            lo = fminf(lo, __shfl_xor(lo, off, 64));
            hi = fmaxf(hi, __shfl_xor(hi, off, 64));
        }
        if (lane == 0) { s_lo[wave] = lo; s_hi[wave] = hi; }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < BLOCK / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
        if (hi != lo) {
            delta = __fdiv_rn(__fsub_rn(hi, lo), (float)qmax);
            const float zf = rintf(__fdiv_rn(-lo, delta));
            z = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);
        }
    }
    const uint32_t oa4 = (q == 8) ? 0x80808080u : 0u;           // a - 128 as a byte == a ^ 0x80
    const uint32_t mask4 = (uint32_t)qmax * 0x01010101u;
    int8_t* out = (int8_t*)(blob + L.off_codes) + (size_t)m * L.Kp;
    uint32_t sum = 0;
    for (int e = tid; e < nblk; e += BLOCK) {
        uint32_t dw[4] = {0, 0, 0, 0};
        if (e < nvalid) {
            if (SRC_HALF) {
                float f[16];
                if (e < 2 * BLOCK) {
                    half8_to_float(keep[e >= BLOCK ? 1 : 0][0], f);
                    half8_to_float(keep[e >= BLOCK ? 1 : 0][VPB - 1], f + 8);
                } else {
                    half8_to_float(row[(size_t)e * VPB], f);
                    half8_to_float(row[(size_t)e * VPB + VPB - 1], f + 8);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    int c = (int)rintf(__fdiv_rn(f[i], delta)) + z;
                    c = c < 0 ? 0 : (c > qmax ? qmax : c);
                    dw[i >> 2] |= (uint32_t)c << (8 * (i & 3));
                }
            } else {
                const uint4 v = e < 2 * BLOCK ? keep[e >= BLOCK ? 1 : 0][0] : row[e];
                dw[0] = v.x & mask4; dw[1] = v.y & mask4; dw[2] = v.z & mask4; dw[3] = v.w & mask4;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                sum = __builtin_amdgcn_udot4(dw[i], 0x01010101u, sum, false);   // sum of the four codes
                dw[i] ^= oa4;
            }
        }
        *reinterpret_cast<uint4*>(out + (size_t)e * 16) = make_uint4(dw[0], dw[1], dw[2], dw[3]);
    }
    int32_t isum = (int32_t)sum;
    for (int off = 32; off > 0; off >>= 1) isum += __shfl_xor(isum, off, 64);
    if (lane == 0) s_sum[wave] = isum;
    __syncthreads();
    if (tid == 0) {
        int32_t t = 0;
#pragma unroll
        for (int w = 0; w < BLOCK / 64; ++w) t += s_sum[w];
        RowParams* params = (RowParams*)(blob + L.off_params);
        params[m] = SRC_HALF ? RowParams{t, delta, z, 0} : RowParams{t, a_scale[m], a_zero[m], 0};
    }
}

__global__ void unpack_act_bytes_kernel(const int8_t* __restrict__ in, int q, int M, int K, int Kp,
                                        uint8_t* __restrict__ codes)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * K) return;
    const int m = (int)(idx / K), k = (int)(idx % K);
    const int oa = (q == 8) ? 128 : 0;
    codes[idx] = (uint8_t)((int)in[(size_t)m * Kp + k] + oa);
}

__global__ void read_params_kernel(const RowParams* __restrict__ p, int R, float* scale, int32_t* zero, int32_t* sum)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= R) return;
    const RowParams v = p[i];
    if (scale) scale[i] = v.scale;
    if (zero) zero[i] = v.zero;
    if (sum) sum[i] = v.sum;
}

// ---- launchers -----------------------------------------------------------------------------------
static inline unsigned blocks_for(size_t n, int block) { return (unsigned)((n + block - 1) / block); }

hipError_t launch_pack_weights(const WeightLayout& L, const uint8_t* w, const float* w_scale, const int32_t* w_zero,
                               uint8_t* blob, hipStream_t s)
{
    write_header_kernel<<<1, 64, 0, s>>>((uint32_t*)blob, kMagicW, L.p, L.N, L.K, L.layout);
    row_params_kernel<<<blocks_for(L.N, 4), 256, 0, s>>>(w, L.p, L.N, L.K, w_scale, w_zero, (RowParams*)(blob + L.off_params));
    if (L.has_planes) {
        const size_t words = (size_t)L.N * L.Kw;
        pack_planes_kernel<<<blocks_for(words, 256), 256, 0, s>>>(w, L.p, L.N, L.K, L.Kw, (uint32_t*)(blob + L.off_planes));
    }
    if (L.has_fields) {
        for (int g = 0; g < L.ngroups; ++g) {
            const size_t dwords = (size_t)L.NT * L.chunks[g] * 256;
            pack_fields_kernel<<<blocks_for(dwords, 256), 256, 0, s>>>(w, L.N, L.K, L.gb[g], L.gs[g], L.chunks[g], dwords,
                                                                      (uint32_t*)(blob + L.off_fields[g]));
        }
    }
    return hipGetLastError();
}

hipError_t launch_pack_weights_g128(const WeightLayout& L, const uint8_t* w, const uint16_t* w_scale_half, const int32_t* w_zero,
                                    uint8_t* blob, hipStream_t s)
{
    const int G = (L.K + 127) / 128, nsuper = (L.K + kSuperK - 1) / kSuperK;
    write_header_kernel<<<1, 64, 0, s>>>((uint32_t*)blob, kMagicW, L.p, L.N, L.K, L.layout);
    zero_params_kernel<<<blocks_for(L.N, 256), 256, 0, s>>>((RowParams*)(blob + L.off_params), L.N);
    for (int g = 0; g < L.ngroups; ++g) {
        const size_t dwords = (size_t)L.NT * L.chunks[g] * 256;
        pack_fields_kernel<<<blocks_for(dwords, 256), 256, 0, s>>>(w, L.N, L.K, L.gb[g], L.gs[g], L.chunks[g], dwords,
                                                                  (uint32_t*)(blob + L.off_fields[g]), w_zero, G);
    }
    const size_t records = (size_t)L.NT * nsuper * 16;
    group_params_kernel<<<blocks_for(records, 256), 256, 0, s>>>(w_scale_half, w_zero, L.N, G, nsuper, L.NT, L.p == 8 ? 128 : 0,
                                                                (uint4*)(blob + L.off_gparams));
    return hipGetLastError();
}

hipError_t launch_unpack_weights(const WeightLayout& L, const uint8_t* blob, int which, uint8_t* out, hipStream_t s)
{
    const size_t n = (size_t)L.N * L.K;
    if (which == ABQ_LAYOUT_PLANES)
        unpack_planes_kernel<<<blocks_for(n, 256), 256, 0, s>>>((const uint32_t*)(blob + L.off_planes), L.p, L.N, L.K, L.Kw, out);
    else
        unpack_fields_kernel<<<blocks_for(n, 256), 256, 0, s>>>(blob, L, out);
    return hipGetLastError();
}

hipError_t launch_pack_act_codes(const ActLayout& L, const uint8_t* codes, const float* a_scale, const int32_t* a_zero,
                                 uint8_t* blob, hipStream_t s)
{
    if (!L.has_planes && L.K % 16 == 0)
        act_rows_fast_kernel<false, 256><<<L.M, 256, 0, s>>>(codes, a_scale, a_zero, L, blob);
    else
        act_rows_kernel<false, 256><<<L.M, 256, 0, s>>>(codes, a_scale, a_zero, L, blob);
    return hipGetLastError();
}

hipError_t launch_quant_pack_act(const ActLayout& L, const uint16_t* x, uint8_t* blob, hipStream_t s)
{
    if (!L.has_planes && L.K % 16 == 0)
        act_rows_fast_kernel<true, 256><<<L.M, 256, 0, s>>>(x, nullptr, nullptr, L, blob);
    else
        act_rows_kernel<true, 256><<<L.M, 256, 0, s>>>(x, nullptr, nullptr, L, blob);
    return hipGetLastError();
}

hipError_t launch_unpack_act(const ActLayout& L, const uint8_t* blob, int which, uint8_t* codes, float* scale,
                             int32_t* zero, int32_t* sum, hipStream_t s)
{
    if (scale || zero || sum)
        read_params_kernel<<<blocks_for(L.M, 256), 256, 0, s>>>((const RowParams*)(blob + L.off_params), L.M, scale, zero, sum);
    if (codes) {
        const size_t n = (size_t)L.M * L.K;
        if (which == ABQ_LAYOUT_PLANES)
            unpack_planes_kernel<<<blocks_for(n, 256), 256, 0, s>>>((const uint32_t*)(blob + L.off_planes), L.q, L.M, L.K, L.Kw, codes);
        else
            unpack_act_bytes_kernel<<<blocks_for(n, 256), 256, 0, s>>>((const int8_t*)(blob + L.off_codes), L.q, L.M, L.K, L.Kp, codes);
    }
    return hipGetLastError();
}

}  // namespace abq
