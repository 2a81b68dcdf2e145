// Measurement aids, not part of the method: a plain streaming read and an int8 MFMA issue loop, so that
// achieved figures can be priced against what this machine delivers for the same kind of work, beside
// the published peaks (HBM 8 TB/s, dense int8 5 POP/s).  The caller times the launches.  A library of its own
// (libabq_probe.so); status values: 0 ok, -1 null pointer, -3 bad size, -4 misaligned pointer, -7 launch failed.
#include "../../../include/abq_probe.h"

#include <hip/hip_runtime.h>

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

// Every thread reads U 16-byte vectors a workgroup-stride apart with non-temporal loads (what the decode
// kernel issues for its weights) and folds them; the fold is stored only for a value that does not occur.
template <int U>
__global__ __launch_bounds__(512) void stream_read_kernel(const u4v* src, size_t nvec, uint32_t* sink)
{
    const size_t base = (size_t)blockIdx.x * (blockDim.x * U) + threadIdx.x;
    u4v v[U];
#pragma unroll
    for (int i = 0; i < U; ++i) {
        const size_t idx = base + (size_t)i * blockDim.x;
        v[i] = __builtin_nontemporal_load(src + (idx < nvec ? idx : nvec - 1));   // clamped: no conditional load
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < U; ++i) s ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    if (s == 0x9E3779B9u) sink[threadIdx.x] = s;
}

// Reads that hit in L2: workgroup b (on XCD b % 8: round-robin dispatch) reads the region of its XCD, `region_vecs`
// 16-byte vectors, `passes` times with ordinary 128-bit loads, eight in flight per lane, every workgroup starting at a
// different offset.  After the first pass a region of a megabyte or two lives in that XCD's L2, so the rate of a
// launch is the rate at which the compute units can pull operands that hit there.
__global__ __launch_bounds__(256) void l2_read_kernel(const u4v* src, unsigned region_vecs, int passes, uint32_t* sink)
{
    const u4v* region = src + (size_t)(blockIdx.x & 7) * region_vecs;
    const unsigned chunk = 256u * 8u;                                    // vectors a workgroup reads per round
    const unsigned rounds = region_vecs / chunk;
    unsigned at = ((blockIdx.x >> 3) * 7u) % rounds;
    uint32_t s = 0;
    for (int p = 0; p < passes; ++p)
        for (unsigned i = 0; i < rounds; ++i) {
            const u4v* base = region + (size_t)at * chunk + threadIdx.x;
            u4v v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = base[u * 256];
#pragma unroll
            for (int u = 0; u < 8; ++u) s ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
            at = at + 1 == rounds ? 0 : at + 1;
        }
    if (s == 0x9E3779B9u) sink[threadIdx.x] = s;
}

// Eight independent 16x16x64 int8 MFMA chains per wave, `iters` rounds.  pattern 0: three of four operand
// bytes are zero; pattern 1: every operand byte is non-zero and differs from lane to lane.  The sustained
// rate depends on the data: measured on MI355X, the chip holds its clock on the former (4.1-4.9 POP/s)
// and lowers it on the latter (2.3-2.9 POP/s), which is the rate real operands see.
__global__ void mfma_i8_kernel(int iters, int pattern, uint32_t* sink)   // (no launch bounds: with a 512-register budget the allocator moves the accumulators through AGPRs every round)
{
    v4i acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4i{0, 0, 0, 0};
    const int t = (int)threadIdx.x;
    const int h = (t * 0x9E3779B1) ^ (t << 13);
    const v4i a = pattern ? v4i{h, h * 3 + 0x5A5A5A5A, ~h, h * 7 + 0x33CC33CC} : v4i{t, 1, 2, 3};
    const v4i b = pattern ? v4i{h * 5, ~(h * 11), h * 13 + 0x0F0F0F0F, h * 17} : v4i{4, 5, 6, t};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s ^= acc[j].x ^ acc[j].y ^ acc[j].z ^ acc[j].w;
    if (s == 0x12345 && iters < 0) sink[t] = (uint32_t)s;
}

// The same issue loop on the 4-bit floating-point MFMA of gfx950 (16x16x128, E2M1 operands, binary32 accumulate, block
// scales of one): the codes 0..3 of a 1- or 2-bit operand are E2M1 values, and sums of their products stay exact in
// binary32 far beyond any K here, so this is the rate a W<=2 A<=2 prefill kernel could price itself against.  Operand
// patterns as above (E2M1 has no infinity or NaN encodings).
typedef int v8i_probe __attribute__((ext_vector_type(8)));
typedef float v4f_probe __attribute__((ext_vector_type(4)));
__global__ void mfma_f4_kernel(int iters, int pattern, uint32_t* sink)
{
    v4f_probe acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = v4f_probe{0.f, 0.f, 0.f, 0.f};
    const int t = (int)threadIdx.x;
    const int h = (t * 0x9E3779B1) ^ (t << 13);
    // (32 E2M1 values per lane: the low four of the eight operand registers)
    const v8i_probe a = pattern ? v8i_probe{h, h * 3 + 0x5A5A5A5A, ~h, h * 7 + 0x33CC33CC, 0, 0, 0, 0} : v8i_probe{t & 0x22, 2, 0, 0x20, 0, 0, 0, 0};
    const v8i_probe b = pattern ? v8i_probe{h * 5, ~(h * 11), h * 13 + 0x0F0F0F0F, h * 17, 0, 0, 0, 0} : v8i_probe{0x200, 0, 2, t & 0x22, 0, 0, 0, 0};
    const int one = 0x7F7F7F7F;   // E8M0 block scales of 2^0
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc[j], 4, 4, 0, one, 0, one);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j].x + acc[j].y + acc[j].z + acc[j].w;
    if (s == 12345.f && iters < 0) sink[t] = (uint32_t)s;
}

static const int kProbeWaveMfmas = 8;          // per round
static const int kProbeWgsPerCu = 8, kProbeWaves = 4;

}  // namespace abq

using namespace abq;

extern "C" {

int abq_probe_stream_read(const void* buf, size_t bytes, void* sink, void* stream)
{
    if (!buf || !sink) return -1;
    if (bytes < 16 || bytes % 16 != 0) return -3;
    if (((uintptr_t)buf & 15u) || ((uintptr_t)sink & 15u)) return -4;
    // 256 threads; the most loads per thread (8, 4, 2, 1) that still leaves four workgroups per CU
    constexpr int threads = 256;
    const size_t nvec = bytes / 16;
    int U = 8;
    while (U > 1 && nvec / ((size_t)threads * U) < 1024) U >>= 1;
    const size_t per_wg = (size_t)threads * U;
    const size_t grid = (nvec + per_wg - 1) / per_wg;
    if (grid > 0x7fffffffu) return -3;
    hipStream_t s = (hipStream_t)stream;
    switch (U) {
        case 8: stream_read_kernel<8><<<(unsigned)grid, threads, 0, s>>>((const u4v*)buf, nvec, (uint32_t*)sink); break;
        case 4: stream_read_kernel<4><<<(unsigned)grid, threads, 0, s>>>((const u4v*)buf, nvec, (uint32_t*)sink); break;
        case 2: stream_read_kernel<2><<<(unsigned)grid, threads, 0, s>>>((const u4v*)buf, nvec, (uint32_t*)sink); break;
        default: stream_read_kernel<1><<<(unsigned)grid, threads, 0, s>>>((const u4v*)buf, nvec, (uint32_t*)sink); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

int abq_probe_l2_read(const void* buf, size_t region_bytes, int passes, int wgs_per_cu, void* sink, void* stream)
{
    if (!buf || !sink) return -1;
    if (region_bytes < 32768 || region_bytes % 32768 != 0 || region_bytes > (64u << 20) || passes < 1 || passes > 4096 || wgs_per_cu < 1 || wgs_per_cu > 8) return -3;
    if (((uintptr_t)buf & 15u) || ((uintptr_t)sink & 15u)) return -4;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    l2_read_kernel<<<(unsigned)(cus * wgs_per_cu), 256, 0, (hipStream_t)stream>>>((const u4v*)buf, (unsigned)(region_bytes / 16), passes, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

double abq_probe_l2_read_bytes(size_t region_bytes, int passes, int wgs_per_cu)
{
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    return (double)region_bytes * passes * wgs_per_cu * cus;
}

double abq_probe_mfma_i8_ops(int iters)
{
    if (iters < 1) return 0.0;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    return 2.0 * 16 * 16 * 64 * (double)kProbeWaveMfmas * iters * kProbeWaves * kProbeWgsPerCu * cus;
}

double abq_probe_mfma_f4_ops(int iters)
{
    return 2.0 * abq_probe_mfma_i8_ops(iters);   // (twice the K per instruction)
}

int abq_probe_mfma_f4(int iters, int pattern, void* sink, void* stream)
{
    if (!sink) return -1;
    if (iters < 1 || iters > (1 << 20) || pattern < 0 || pattern > 1) return -3;
    if ((uintptr_t)sink & 15u) return -4;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    mfma_f4_kernel<<<(unsigned)(cus * kProbeWgsPerCu), kProbeWaves * 64, 0, (hipStream_t)stream>>>(iters, pattern, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

int abq_probe_mfma_i8(int iters, int pattern, void* sink, void* stream)
{
    if (!sink) return -1;
    if (iters < 1 || iters > (1 << 20) || pattern < 0 || pattern > 1) return -3;
    if ((uintptr_t)sink & 15u) return -4;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    mfma_i8_kernel<<<(unsigned)(cus * kProbeWgsPerCu), kProbeWaves * 64, 0, (hipStream_t)stream>>>(iters, pattern, (uint32_t*)sink);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

}  // extern "C"
