// Internal declarations shared by the HIP translation units of libabq (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

namespace abq {

// ---- plane groups ---------------------------------------------------------------------------
// A p-bit weight is stored as 1..3 "plane groups": runs of 4, 2 or 1 adjacent bit-planes
// (8 planes when p == 8) kept interleaved per element, lowest planes first:
//   p : 1:(1)  2:(2)  3:(2,1)  4:(4)  5:(4,1)  6:(4,2)  7:(4,2,1)  8:(8)
// w = sum_g field_g << shift_g is the bit-plane sum of Appendix B with the inner sum over the
// planes of one group already carried out by the storage format.
__host__ __device__ constexpr int group_count(int p) { return (p == 7) ? 3 : ((p == 3 || p == 5 || p == 6) ? 2 : 1); }
__host__ __device__ constexpr int group_width(int p, int g)
{
    return p == 8 ? 8
         : p >= 4 ? (g == 0 ? 4 : (p == 5 ? 1 : (p == 6 ? 2 : (g == 1 ? 2 : 1))))   // 4 | 4,1 | 4,2 | 4,2,1
         : p == 3 ? (g == 0 ? 2 : 1)
         : p;                                                                      // 1 or 2
}
__host__ __device__ constexpr int group_shift(int p, int g)
{
    return g == 0 ? 0 : (g == 1 ? group_width(p, 0) : group_width(p, 0) + group_width(p, 1));
}

constexpr int kTileN = 16;        // rows of W per MFMA tile
constexpr int kSuperK = 512;      // k-extent all groups tile evenly: one 1 KiB wave load of a b-bit group spans 512/b
constexpr int kHeaderBytes = 256;
constexpr uint32_t kMagicW = 0x57514241u;   // "ABQW"
constexpr uint32_t kMagicA = 0x41514241u;   // "ABQA"

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The library reads no environment variable: launch plans come from closed-form rules and from the plan table of
// the ABI.  Only a build made with -DABQ_TUNING_ENV (the tuner's own A/B experiments) looks at ABQ_* variables,
// afresh on every call, so that no mutable state is kept.
static inline int tuning_env(const char* name)
{
#ifdef ABQ_TUNING_ENV
    const char* e = getenv(name);
    return e ? atoi(e) : 0;
#else
    (void)name;
    return 0;
#endif
}

// Packed-weight blob:
//   [header 256 B][wparams N x {int32 wsum, float scale, int32 zero, int32 0}]
//   [planes  uint32 [p][N][Kw]]                               if PLANES/BOTH   (Kw = ceil(K/128)*4)
//   [group g: uint4 [NT][C_g][64 lanes]] for each group       if FIELDS/BOTH   (NT = ceil(N/16), C_g = b_g*ceil(K/512))
//   [uint4 [NT][ceil(K/512)][16 channels]]                    if FIELDS_G128: per channel of a tile and super-chunk of 512 k
//                                                             the four 128-k groups' binary16 scales (8 B), their zero-points
//                                                             as int8 (zero - 128 when p == 8; 4 B), 4 B unused.  wparams is
//                                                             all zero then, and k from K to the end of the last group holds
//                                                             that group's zero-point instead of 0.
struct WeightLayout {
    int p, N, K, layout;
    bool has_planes, has_fields, g128;
    int ngroups, gb[3], gs[3], chunks[3];
    int NT, Kw;
    size_t off_params, off_planes, off_fields[3], off_gparams, total;
};

// Packed-activation blob:
//   [header 256 B][aparams M x {int32 asum, float scale, int32 zero, int32 0}]
//   [planes uint32 [q][M][Kw]]                                if PLANES/BOTH
//   [codes  int8 [M][Kp], value a - (q==8 ? 128 : 0), zero padded to Kp = ceil(K/512)*512]   if FIELDS/BOTH
struct ActLayout {
    int q, M, K, layout;
    bool has_planes, has_fields;
    int Kp, Kw;
    size_t off_params, off_planes, off_codes, total;
};

bool make_weight_layout(int p, int N, int K, int layout, WeightLayout* out);
bool make_act_layout(int q, int M, int K, int layout, ActLayout* out);

// ---- kernel launchers (each returns the hipError_t of the launch) --------------------------
hipError_t launch_pack_weights(const WeightLayout& L, const uint8_t* w_codes, const float* w_scale,
                               const int32_t* w_zero, uint8_t* blob, hipStream_t s);
hipError_t launch_pack_weights_g128(const WeightLayout& L, const uint8_t* w_codes, const uint16_t* w_scale_half,
                                    const int32_t* w_zero, uint8_t* blob, hipStream_t s);
hipError_t launch_unpack_weights(const WeightLayout& L, const uint8_t* blob, int which, uint8_t* out, hipStream_t s);
hipError_t launch_pack_act_codes(const ActLayout& L, const uint8_t* codes, const float* a_scale,
                                 const int32_t* a_zero, uint8_t* blob, hipStream_t s);
hipError_t launch_quant_pack_act(const ActLayout& L, const uint16_t* x, uint8_t* blob, hipStream_t s);
hipError_t launch_unpack_act(const ActLayout& L, const uint8_t* blob, int which, uint8_t* codes, float* scale,
                             int32_t* zero, int32_t* sum, hipStream_t s);

hipError_t launch_rmsnorm_quant(int q, int M, int K, const uint16_t* x, const uint16_t* gamma, float eps, uint8_t* codes,
                                float* scale, int32_t* zero, uint16_t* y_out, hipStream_t s);

hipError_t launch_add_rmsnorm_quant(int q, int M, int K, const uint16_t* x, const uint16_t* residual, const uint16_t* gamma,
                                    float eps, uint8_t* codes, float* scale, int32_t* zero, uint16_t* sum_out, uint16_t* y_out,
                                    hipStream_t s);

hipError_t launch_silu_mul_quant(int q, int M, int K, const uint16_t* gate, const uint16_t* up, uint8_t* codes, float* scale,
                                 int32_t* zero, uint16_t* h_out, hipStream_t s);

// Launch-plan override for one exact problem size (0 = keep the library's rule); see abq_plan in the ABI header.
struct PlanOverride { int skinny_waves, skinny_kgroups, tiled_mt, tiled_ntw, tiled_wd, tiled_band, direct_r; };
bool lookup_plan(int p, int q, int M, int N, int K, PlanOverride* out);   // false (and *out all zero) when none is set

// ReQuant fused into the matmul epilogue (Fig. 3b; the last paragraph of Sec. 3.4): besides (or instead of) the
// binary16 output, the codes of the next layer's activations under per-token parameters the caller fixes ahead of
// the call.  codes == nullptr: off.
struct Requant {
    uint8_t* codes;        // [M,N] uint8
    const float* scale;    // [M] Delta of the output row
    const int32_t* zero;   // [M] zero-point of the output row
    int qmax;              // 2^q_out - 1
};

struct GemmArgs {
    int p, q, M, N, K;
    const uint8_t* act_blob;   // packed activations, or null when a_raw is given (streaming kernel only)
    const uint8_t* a_raw;      // unpacked codes [M][K] with a_scale[M], a_zero[M]: activation packing fused into the kernel
    const float* a_scale;
    const int32_t* a_zero;
    const uint8_t* w_blob;
    uint16_t* y;       // may be null when rq.codes is given
    int32_t* acc;      // may be null
    void* workspace;
    size_t workspace_bytes;
    Requant rq = Requant{nullptr, nullptr, nullptr, 0};
};
hipError_t launch_gemm_skinny(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s);
bool gemm_grouped_fits(int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W, int* waves,
                       size_t* lds_bytes);
hipError_t launch_gemm_grouped(int p, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W,
                               int waves, size_t lds_bytes, hipStream_t s);
int num_cus();   // compute units of the current device (cached)
// The direct decode kernel (few rows of A): plan = operand rows per slice set, super-chunks per wave, waves per workgroup.
struct DirectPlan { int MR, R, S; };
bool direct_plan(int p, int M, int nsuper, int forced_r, DirectPlan* out);   // false: the problem does not fit this kernel
hipError_t launch_gemm_direct(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, const DirectPlan& pl, hipStream_t s);
bool gemm_direct_grouped_fits(int p, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W);
// The very-low-bit path on the 4-bit floating-point MFMA (operands of one or two bits): one packed layout for both operands.
size_t f4_packed_bytes(int rows, int K);
hipError_t launch_f4_pack(int bits, int rows, int K, const uint8_t* codes, const float* scale, const int32_t* zero, uint8_t* blob, hipStream_t s);
hipError_t launch_f4_gemm(int M, int N, int K, const uint8_t* act_blob, const uint8_t* w_blob, uint16_t* y, int32_t* acc, hipStream_t s);
// The shared-operand decode kernel (9 .. 16 rows of A over more tiles than compute units): workgroups, waves per
// workgroup, super-chunks per wave and phase at most, phases of K (1 or 2), super-chunks per phase.
struct SharedAPlan { int nwg, S, R, phases, H; };
bool shared_a_plan(int p, int M, int NT, int Kp, bool raw, int K, bool forced, SharedAPlan* out);   // false: the problem does not fit this kernel
hipError_t launch_gemm_shared_a(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, const SharedAPlan& pl, hipStream_t s);
bool direct_plan_g128(int p, int nsuper, DirectPlan* out);   // per-group blobs, one row of A
bool gemm_direct_g128_fits(int p, int M, const GemmArgs& g, const ActLayout& A, const WeightLayout& W);
hipError_t launch_gemm_direct_grouped(int p, int q, int M, int count, const GemmArgs* probs, const ActLayout* A, const WeightLayout* W,
                                      hipStream_t s);
hipError_t launch_gemm_tiled(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s);
hipError_t launch_gemm_bitserial(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s);

// ---- device helpers -------------------------------------------------------------------------
struct alignas(16) RowParams { int32_t sum; float scale; int32_t zero; int32_t pad; };

// Fused dequant epilogue (the "DeQuant" box of Fig. 3b with the affine semantics of Eq. 3).
// S is the kernel's sum over (a - oa)(w - ow); the exact integer zero-point correction is
// applied before any float operation.  Unsigned arithmetic: intermediate wrap-around is
// harmless because the final value fits in int32.
__device__ __forceinline__ uint16_t epilogue_value(int32_t S, int oa, int ow, int K, const RowParams& ap,
                                                   const RowParams& wp, int32_t* raw_out)
{
    const uint32_t asum = (uint32_t)ap.sum, wsum = (uint32_t)wp.sum;
    const uint32_t uK = (uint32_t)K, uoa = (uint32_t)oa, uow = (uint32_t)ow;
    const uint32_t raw = (uint32_t)S + uow * asum + uoa * wsum - uK * uoa * uow;
    *raw_out = (int32_t)raw;
    const uint32_t az = (uint32_t)ap.zero, wz = (uint32_t)wp.zero;
    const int32_t centered = (int32_t)(raw - wz * asum - az * wsum + uK * az * wz);
    const float v = ((float)centered * ap.scale) * wp.scale;
    // the conversion as the instruction itself: left to the compiler, the last product and the conversion may merge
    // into one mixed-precision operation with a single rounding, which differs from the stated two roundings when
    // the binary32 product is a tie between two binary16 values, and then kernels would not agree bit for bit
    uint32_t h;
    asm("v_cvt_f16_f32 %0, %1" : "=v"(h) : "v"(v));
    return (uint16_t)h;
}

// code = clamp(clamp(rint(y / Delta), -2^24, 2^24) + z, 0, qmax) on the binary16 output value, every float step one
// IEEE binary32 operation (Eq. 3's clamp(round(x/Delta)+z); the float results decide integer codes).
__device__ __forceinline__ uint8_t requant_code(uint16_t h, float delta, int z, int qmax)
{
    const float yv = __half2float(__ushort_as_half(h));
    float r = rintf(__fdiv_rn(yv, delta));
    r = fminf(fmaxf(r, -16777216.0f), 16777216.0f);
    const int c = (int)r + z;
    return (uint8_t)(c < 0 ? 0 : (c > qmax ? qmax : c));
}

// m: the output row (for the ReQuant parameters).
__device__ __forceinline__ void epilogue_store(int32_t S, int oa, int ow, int K, const RowParams& ap,
                                               const RowParams& wp, size_t idx, uint16_t* y, int32_t* acc,
                                               const Requant& rq = Requant{nullptr, nullptr, nullptr, 0}, int m = 0)
{
    int32_t raw;
    const uint16_t h = epilogue_value(S, oa, ow, K, ap, wp, &raw);
    if (y) y[idx] = h;
    if (acc) acc[idx] = raw;
    if (rq.codes) rq.codes[idx] = requant_code(h, rq.scale[m], rq.zero[m], rq.qmax);
}

}  // namespace abq
