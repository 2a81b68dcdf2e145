// Host side of the C ABI (include/abq.h): argument validation, blob layouts, dispatch.
// No device code here; validation runs before the first HIP call so that every error path
// can be exercised on a machine without a GPU.
#include "abq_internal.h"
#include "../../include/abq.h"

#include <limits.h>
#include <stdlib.h>
#include <array>
#include <atomic>
#include <map>
#include <mutex>
#include <vector>

// Scratch of abq_gemm_act_codes_static: the packed activations of its two-kernel path live here instead of in
// a caller's workspace.  In host code this name is a stand-in, not a device address: host code uses the
// per-device pointer that static_scratch_ptr() obtains with hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[ABQ_STATIC_SCRATCH_BYTES];

namespace abq {

static thread_local int g_last_hip_error = 0;
static thread_local int g_last_decode_kernel = 0;   // test hook: which decode kernel the last single-problem call on this thread launched

static int hip_status(hipError_t e)
{
    if (e == hipSuccess) return ABQ_OK;
    g_last_hip_error = (int)e;
    return ABQ_ERR_HIP;
}

static bool layout_bits(int layout, bool* planes, bool* fields)
{
    switch (layout) {
        case ABQ_LAYOUT_AUTO:
        case ABQ_LAYOUT_FIELDS: *planes = false; *fields = true; return true;
        case ABQ_LAYOUT_PLANES: *planes = true; *fields = false; return true;
        case ABQ_LAYOUT_BOTH: *planes = true; *fields = true; return true;
        case ABQ_LAYOUT_FIELDS_G128: *planes = false; *fields = true; return true;
        default: return false;
    }
}

bool make_weight_layout(int p, int N, int K, int layout, WeightLayout* L)
{
    if (p < 1 || p > 8 || N < 1 || K < 1 || K > ABQ_MAX_K) return false;
    if (!layout_bits(layout, &L->has_planes, &L->has_fields)) return false;
    L->p = p; L->N = N; L->K = K; L->layout = layout;
    L->g128 = layout == ABQ_LAYOUT_FIELDS_G128;
    L->NT = (N + kTileN - 1) / kTileN;
    L->Kw = (K + 127) / 128 * 4;
    L->ngroups = group_count(p);
    size_t off = kHeaderBytes;
    L->off_params = off;
    off = align_up(off + (size_t)N * sizeof(RowParams), 256);
    L->off_planes = 0;
    if (L->has_planes) {
        L->off_planes = off;
        off = align_up(off + (size_t)p * N * L->Kw * 4, 256);
    }
    for (int g = 0; g < 3; ++g) { L->gb[g] = 0; L->gs[g] = 0; L->chunks[g] = 0; L->off_fields[g] = 0; }
    if (L->has_fields) {
        for (int g = 0; g < L->ngroups; ++g) {
            L->gb[g] = group_width(p, g);
            L->gs[g] = group_shift(p, g);
            L->chunks[g] = (K + kSuperK - 1) / kSuperK * L->gb[g];   // whole super-chunks of 512 k
            L->off_fields[g] = off;
            off = align_up(off + (size_t)L->NT * L->chunks[g] * 1024, 256);
        }
    }
    L->off_gparams = 0;
    if (L->g128) {
        L->off_gparams = off;
        off = align_up(off + (size_t)L->NT * ((K + kSuperK - 1) / kSuperK) * 256, 256);
    }
    L->total = off;
    return true;
}

bool make_act_layout(int q, int M, int K, int layout, ActLayout* L)
{
    if (q < 1 || q > 8 || M < 1 || K < 1 || K > ABQ_MAX_K) return false;
    if (layout == ABQ_LAYOUT_FIELDS_G128 || !layout_bits(layout, &L->has_planes, &L->has_fields)) return false;
    L->q = q; L->M = M; L->K = K; L->layout = layout;
    L->Kp = (K + kSuperK - 1) / kSuperK * kSuperK;
    L->Kw = (K + 127) / 128 * 4;
    size_t off = kHeaderBytes;
    L->off_params = off;
    off = align_up(off + (size_t)M * sizeof(RowParams), 256);
    L->off_planes = 0;
    L->off_codes = 0;
    if (L->has_planes) {
        L->off_planes = off;
        off = align_up(off + (size_t)q * M * L->Kw * 4, 256);
    }
    if (L->has_fields) {
        L->off_codes = off;
        off = align_up(off + (size_t)M * L->Kp, 256);
    }
    L->total = off;
    return true;
}

// ---- launch-plan table --------------------------------------------------------------------------
static std::mutex g_plan_mutex;
static std::map<std::array<int, 5>, PlanOverride> g_plans;
static std::atomic<int> g_plan_count{0};   // launches skip the lock while the table is empty

bool lookup_plan(int p, int q, int M, int N, int K, PlanOverride* out)
{
    *out = PlanOverride{0, 0, 0, 0, 0, 0, 0};
    if (g_plan_count.load(std::memory_order_relaxed) == 0) return false;
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    auto it = g_plans.find({p, q, M, N, K});
    if (it == g_plans.end()) return false;
    *out = it->second;
    return true;
}

static bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// Device address of `scratch` on the current device (each GPU holds its own copy of the array at its own
// address): looked up once per device, with that device current, and kept.
static hipError_t static_scratch_ptr(void** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void* ptrs[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mutex);
    if (!ptrs[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return hipSuccess;
}

static int check_bits_shape(int bits, int R, int K)
{
    if (bits < 1 || bits > 8) return ABQ_ERR_BITS;
    if (R < 1 || K < 1 || K > ABQ_MAX_K) return ABQ_ERR_SHAPE;
    return ABQ_OK;
}

}  // namespace abq

using namespace abq;

extern "C" {

int abq_version(void) { return 100; }

const char* abq_status_string(int status)
{
    switch (status) {
        case ABQ_OK: return "ok";
        case ABQ_ERR_NULL: return "a required pointer is NULL";
        case ABQ_ERR_BITS: return "bit width outside 1..8";
        case ABQ_ERR_SHAPE: return "invalid shape (M,N,K must be >= 1, K <= ABQ_MAX_K, K*(2^p-1)*(2^q-1) <= INT32_MAX)";
        case ABQ_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case ABQ_ERR_SIZE: return "caller buffer smaller than its size query";
        case ABQ_ERR_LAYOUT: return "unknown layout or the blob lacks the representation this call needs";
        case ABQ_ERR_HIP: return "a HIP call failed (see abq_last_hip_error)";
        default: return "unknown status";
    }
}

int abq_last_hip_error(void) { return g_last_hip_error; }
int abq_last_decode_kernel(void) { return g_last_decode_kernel; }

size_t abq_packed_weight_bytes(int p, int N, int K, int layout)
{
    WeightLayout L;
    return make_weight_layout(p, N, K, layout, &L) ? L.total : 0;
}

size_t abq_packed_act_bytes(int q, int M, int K, int layout)
{
    ActLayout L;
    return make_act_layout(q, M, K, layout, &L) ? L.total : 0;
}

int abq_pack_weights(int p, int N, int K, const uint8_t* w_codes, const float* w_scale, const int32_t* w_zero,
                     int layout, void* packed_out, size_t packed_bytes, void* stream)
{
    if (!w_codes || !w_scale || !w_zero || !packed_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(p, N, K)) return e;
    WeightLayout L;
    if (!make_weight_layout(p, N, K, layout, &L) || L.g128) return ABQ_ERR_LAYOUT;
    if (misaligned(w_codes) || misaligned(w_scale) || misaligned(w_zero) || misaligned(packed_out)) return ABQ_ERR_ALIGN;
    if (packed_bytes < L.total) return ABQ_ERR_SIZE;
    return hip_status(launch_pack_weights(L, w_codes, w_scale, w_zero, (uint8_t*)packed_out, (hipStream_t)stream));
}

int abq_pack_weights_g128(int p, int N, int K, const uint8_t* w_codes, const uint16_t* w_scale_fp16, const int32_t* w_zero,
                          void* packed_out, size_t packed_bytes, void* stream)
{
    if (!w_codes || !w_scale_fp16 || !w_zero || !packed_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(p, N, K)) return e;
    WeightLayout L;
    if (!make_weight_layout(p, N, K, ABQ_LAYOUT_FIELDS_G128, &L)) return ABQ_ERR_LAYOUT;
    if (misaligned(w_codes) || misaligned(w_scale_fp16) || misaligned(w_zero) || misaligned(packed_out)) return ABQ_ERR_ALIGN;
    if (packed_bytes < L.total) return ABQ_ERR_SIZE;
    return hip_status(launch_pack_weights_g128(L, w_codes, w_scale_fp16, w_zero, (uint8_t*)packed_out, (hipStream_t)stream));
}

int abq_unpack_weights(int p, int N, int K, int layout, const void* packed, int which, uint8_t* w_codes_out, void* stream)
{
    if (!packed || !w_codes_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(p, N, K)) return e;
    WeightLayout L;
    if (!make_weight_layout(p, N, K, layout, &L)) return ABQ_ERR_LAYOUT;
    if (!((which == ABQ_LAYOUT_PLANES && L.has_planes) || (which == ABQ_LAYOUT_FIELDS && L.has_fields))) return ABQ_ERR_LAYOUT;
    if (misaligned(packed) || misaligned(w_codes_out)) return ABQ_ERR_ALIGN;
    return hip_status(launch_unpack_weights(L, (const uint8_t*)packed, which, w_codes_out, (hipStream_t)stream));
}

int abq_quant_pack_act(int q, int M, int K, const uint16_t* x_fp16, int layout, void* packed_out, size_t packed_bytes,
                       void* stream)
{
    if (!x_fp16 || !packed_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    ActLayout L;
    if (!make_act_layout(q, M, K, layout, &L)) return ABQ_ERR_LAYOUT;
    if (misaligned(x_fp16) || misaligned(packed_out)) return ABQ_ERR_ALIGN;
    if (packed_bytes < L.total) return ABQ_ERR_SIZE;
    return hip_status(launch_quant_pack_act(L, x_fp16, (uint8_t*)packed_out, (hipStream_t)stream));
}

int abq_pack_act_codes(int q, int M, int K, const uint8_t* a_codes, const float* a_scale, const int32_t* a_zero,
                       int layout, void* packed_out, size_t packed_bytes, void* stream)
{
    if (!a_codes || !a_scale || !a_zero || !packed_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    ActLayout L;
    if (!make_act_layout(q, M, K, layout, &L)) return ABQ_ERR_LAYOUT;
    if (misaligned(a_codes) || misaligned(a_scale) || misaligned(a_zero) || misaligned(packed_out)) return ABQ_ERR_ALIGN;
    if (packed_bytes < L.total) return ABQ_ERR_SIZE;
    return hip_status(launch_pack_act_codes(L, a_codes, a_scale, a_zero, (uint8_t*)packed_out, (hipStream_t)stream));
}

int abq_unpack_act(int q, int M, int K, int layout, const void* packed, int which, uint8_t* a_codes_out,
                   float* a_scale_out, int32_t* a_zero_out, int32_t* a_sum_out, void* stream)
{
    if (!packed) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    ActLayout L;
    if (!make_act_layout(q, M, K, layout, &L)) return ABQ_ERR_LAYOUT;
    if (a_codes_out && !((which == ABQ_LAYOUT_PLANES && L.has_planes) || (which == ABQ_LAYOUT_FIELDS && L.has_fields)))
        return ABQ_ERR_LAYOUT;
    if (misaligned(packed) || misaligned(a_codes_out) || misaligned(a_scale_out) || misaligned(a_zero_out) ||
        misaligned(a_sum_out))
        return ABQ_ERR_ALIGN;
    return hip_status(launch_unpack_act(L, (const uint8_t*)packed, which, a_codes_out, a_scale_out, a_zero_out,
                                        a_sum_out, (hipStream_t)stream));
}

int abq_rmsnorm_quant_act(int q, int M, int K, const uint16_t* x_fp16, const uint16_t* gamma_fp16, float eps,
                          uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out, uint16_t* y_fp16_out, void* stream)
{
    if (!x_fp16 || !gamma_fp16 || !a_codes_out || !a_scale_out || !a_zero_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    if (!(eps >= 0.0f)) return ABQ_ERR_SHAPE;
    if (misaligned(x_fp16) || misaligned(gamma_fp16) || misaligned(a_codes_out) || misaligned(a_scale_out) ||
        misaligned(a_zero_out) || misaligned(y_fp16_out))
        return ABQ_ERR_ALIGN;
    return hip_status(launch_rmsnorm_quant(q, M, K, x_fp16, gamma_fp16, eps, a_codes_out, a_scale_out, a_zero_out, y_fp16_out,
                                           (hipStream_t)stream));
}

int abq_add_rmsnorm_quant_act(int q, int M, int K, const uint16_t* x_fp16, const uint16_t* residual_fp16, const uint16_t* gamma_fp16,
                              float eps, uint8_t* a_codes_out, float* a_scale_out, int32_t* a_zero_out, uint16_t* sum_fp16_out,
                              uint16_t* y_fp16_out, void* stream)
{
    if (!x_fp16 || !residual_fp16 || !gamma_fp16 || !a_codes_out || !a_scale_out || !a_zero_out || !sum_fp16_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    if (!(eps >= 0.0f)) return ABQ_ERR_SHAPE;
    if (misaligned(x_fp16) || misaligned(residual_fp16) || misaligned(gamma_fp16) || misaligned(a_codes_out) ||
        misaligned(a_scale_out) || misaligned(a_zero_out) || misaligned(sum_fp16_out) || misaligned(y_fp16_out))
        return ABQ_ERR_ALIGN;
    return hip_status(launch_add_rmsnorm_quant(q, M, K, x_fp16, residual_fp16, gamma_fp16, eps, a_codes_out, a_scale_out, a_zero_out,
                                               sum_fp16_out, y_fp16_out, (hipStream_t)stream));
}

int abq_silu_mul_quant_act(int q, int M, int K, const uint16_t* gate_fp16, const uint16_t* up_fp16, uint8_t* a_codes_out,
                           float* a_scale_out, int32_t* a_zero_out, uint16_t* h_fp16_out, void* stream)
{
    if (!gate_fp16 || !up_fp16 || !a_codes_out || !a_scale_out || !a_zero_out) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(q, M, K)) return e;
    if (misaligned(gate_fp16) || misaligned(up_fp16) || misaligned(a_codes_out) || misaligned(a_scale_out) ||
        misaligned(a_zero_out) || misaligned(h_fp16_out))
        return ABQ_ERR_ALIGN;
    return hip_status(launch_silu_mul_quant(q, M, K, gate_fp16, up_fp16, a_codes_out, a_scale_out, a_zero_out, h_fp16_out,
                                            (hipStream_t)stream));
}

int abq_check_packed(int kind, int bits, int rows, int K, int layout, const void* packed, size_t packed_bytes, void* stream)
{
    if (!packed) return ABQ_ERR_NULL;
    if (int e = check_bits_shape(bits, rows, K)) return e;
    size_t total = 0;
    if (kind == 0) {
        WeightLayout L;
        if (!make_weight_layout(bits, rows, K, layout, &L)) return ABQ_ERR_LAYOUT;
        total = L.total;
    } else if (kind == 1) {
        ActLayout L;
        if (!make_act_layout(bits, rows, K, layout, &L)) return ABQ_ERR_LAYOUT;
        total = L.total;
    } else {
        return ABQ_ERR_LAYOUT;
    }
    if (misaligned(packed)) return ABQ_ERR_ALIGN;
    if (packed_bytes < total) return ABQ_ERR_SIZE;
    uint32_t hdr[6] = {0, 0, 0, 0, 0, 0};   // magic, format version, bits, rows, K, layout
    hipStream_t s = (hipStream_t)stream;
    if (int e = hip_status(hipMemcpyAsync(hdr, packed, sizeof(hdr), hipMemcpyDeviceToHost, s))) return e;
    if (int e = hip_status(hipStreamSynchronize(s))) return e;
    const uint32_t want[6] = {kind == 0 ? kMagicW : kMagicA, 1u, (uint32_t)bits, (uint32_t)rows, (uint32_t)K, (uint32_t)layout};
    for (int i = 0; i < 6; ++i)
        if (hdr[i] != want[i]) return ABQ_ERR_LAYOUT;
    return ABQ_OK;
}

static int check_gemm_shape(int p, int q, int M, int N, int K)
{
    if (p < 1 || p > 8 || q < 1 || q > 8) return ABQ_ERR_BITS;
    if (M < 1 || N < 1 || K < 1 || K > ABQ_MAX_K) return ABQ_ERR_SHAPE;
    const int64_t bound = (int64_t)K * ((1 << p) - 1) * ((1 << q) - 1);
    if (bound > (int64_t)INT32_MAX) return ABQ_ERR_SHAPE;
    return ABQ_OK;
}

// Kernel family for a problem: true = int8-MFMA on field-packed operands, false = bit-serial
// AND+popcount on the 1-bit planes.  Where a blob carries both representations the MFMA path is taken: measured on
// MI355X over p, q in {1, 2, 4} it is the faster one everywhere (W1A1 M = 1 5120 -> 13824: 4.65 vs 4.58 us, the only
// near tie; W2A2 5.5 vs 6.1; W1A1 M = 16 9.4 vs 48.9; M = 256 23.5 vs 55.4), and only it runs the fused one-launch
// decode step.  The literal form runs on blobs that hold nothing but planes, or when forced (ABQ_USE_PLANES).
static bool choose_fields(bool can_fields, bool can_planes, int force, int p, int q, int M, int N)
{
    (void)can_planes; (void)p; (void)q; (void)M; (void)N;
    if (force == ABQ_USE_PLANES) return false;
    if (force == ABQ_USE_FIELDS) return true;
    return can_fields;
}

static const int kSkinnyMaxM = 16;   // one MFMA tile of activation rows: the streaming kernel; above it the tiled kernel

// Streaming kernel or tiled kernel (both on field-packed operands).  Few output tiles and M <= 64:
// the tiled kernel would occupy a fraction of the chip with long K loops; the streaming kernel
// splits K over waves instead (one pass over W per 16 rows of A).
static bool streaming_shape(int M, int N)
{
    if (M <= kSkinnyMaxM) return true;
    const int env_m = tuning_env("ABQ_STREAM_MAX_M"), env_wgs = tuning_env("ABQ_STREAM_MAX_WGS");
    const int max_m = env_m > 0 ? env_m : 64, max_wgs = env_wgs > 0 ? env_wgs : 128;
    const long tiled_wgs = (long)((M + 63) / 64) * ((N + 63) / 64);
    return M <= max_m && tiled_wgs < max_wgs;
}

// The two decode kernels (both on field-packed operands, M <= 16).  The direct kernel (A operand loaded straight into
// registers, every load of a wave up front, no ring, one workgroup per 16-channel tile) is ahead while its operand loads
// stay few against the weight loads; the streaming kernel (A staged in LDS once per workgroup and shared by all the tiles
// it walks, a ring of weight loads) is ahead for many rows of A over many tiles and for the longest streams.  The rule
// follows the launch-plan search over LLaMA-7B/13B shapes (p = 2, 3, 4, 6, 8; M = 1, 4, 8, 16; direct / streaming in us):
//   M <= 4: direct (W4A8 M = 4 13824 ch: 8.6 / 11.2; W3A8 M = 1 11008 ch: 5.4 / 8.2), except
//     p = 8 over more than 48 MiB (13824 x 5120, M = 1: 14.7 / 13.0; M = 4: 15.7 / 13.4), p = 5 and 7 over more than
//     40 MiB (W7A8 13824 x 5120 M = 1: 14.9 / 13.2, M = 4: 16.8 / 13.7; W5A8: 11.3 / 10.8, 13.8 / 12.5; W6A8 stays: 10.6 / 11.2) and
//     p >= 5 with K > 12288 (W6A8 5120 x 13824: 14.5 / 13.0; W8A8: 16.8 / 14.6);
//   4 < M <= 16 with K > 12288: streaming (W4A8 M = 8: 14.2 / 12.3);
//   4 < M <= 16, at most one tile per CU: direct at every width (4096 ch, K = 11008, M = 8: W3A8 7.1 / 9.1, W6A8 9.3 / 11.4,
//     W8A8 10.4 / 11.5; M = 16: W4A8 9.8 / 11.7, W2A8 8.6 / 11.5);
//   4 < M <= 8, more tiles: direct for the single-group widths 1, 2, 4 (W4A8 13824 ch: 10.2 / 10.9; W2A8: 8.8 / 10.2),
//     streaming for the others (W3A8 13824 ch: 14.1 / 11.8; W6A8: 14.3 / 12.4);
//   8 < M <= 16, more tiles: streaming (W2A8 11008 ch: 8.9 / 8.0; W4A8: 10.0 / 8.7).
// A plan-table entry can force either (direct_r = -1: streaming; 1, 2, 4: direct with that many super-chunks per wave).
static bool direct_by_rule(int p, int M, int nsuper, const WeightLayout& W)
{
    const bool long_k = nsuper > 24;
    if (M <= 4) {
        const size_t stream = (size_t)p * W.NT * kTileN * (size_t)nsuper * kSuperK / 8;
        if (p == 8 && stream > ((size_t)48 << 20)) return false;
        if ((p == 5 || p == 7) && stream > ((size_t)40 << 20)) return false;   // (widths with a 1-bit group beside wider ones)
        return !(p >= 5 && long_k);
    }
    if (long_k) return false;
    if (W.NT <= num_cus()) return true;
    return M <= 8 && (p == 1 || p == 2 || p == 4);
}
static bool choose_direct(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, DirectPlan* pl)
{
    if (g.M > 16 || !W.has_fields) return false;
    if (W.g128)   // per-group weight parameters: the direct kernel has a variant for one row of A, one super-chunk per wave and
                  // p <= 4 (wider weights share accumulators between slices there, which the per-group sums cannot)
        return gemm_direct_g128_fits(g.p, g.M, g, A, W) && direct_plan_g128(g.p, A.Kp / kSuperK, pl);
    PlanOverride ov;
    lookup_plan(g.p, g.q, g.M, g.N, g.K, &ov);
    const int env = tuning_env("ABQ_DIRECT_R");
    const int forced = ov.direct_r != 0 ? ov.direct_r : env;
    if (forced < 0) return false;
    if (forced == 0 && !direct_by_rule(g.p, g.M, A.Kp / kSuperK, W)) return false;
    return direct_plan(g.p, g.M, A.Kp / kSuperK, forced, pl);
}
// The shared-operand kernel (one copy of A in LDS per workgroup, several tiles per workgroup, every load up front): where
// neither of the two above is at home — more than eight rows of A over more tiles than compute units, narrow weights.
// Measured (shared / streaming / direct, us; M = 16 unless said): 13824 ch x 5120: W1A8 8.0 / 10.5 / 14.1, W2A8 8.8 / 11.0 /
// 14.5, W3A8 11.4 / 12.5 / 18.1, W4A8 11.4 / 12.2 / 16.2 (M = 9: 10.7 / 10.8), W5A8 14.0 / 13.2; 11008 ch x 4096: W1A8 7.1 / 7.9 /
// 8.8, W2A8 7.4 / 8.0, W3A8 8.8 / 9.1, W4A8 8.8 / 8.7, W8A8 11.7 / 10.7.  Hence: p <= 3, and p = 4 over more than three
// tiles per compute unit.  Where A is larger than LDS (K > 6144) the kernel cuts K in two phases; those variants exist
// for p <= 2 (5120 ch x 13824, M = 16: W1A8 11.9 / 14.3, W2A8 13.2 / 14.4; W4A8 would spill: 20.7 / 16.2).  A plan-table entry
// direct_r = -2 forces it wherever it fits.
static bool choose_shared_a(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, SharedAPlan* pl)
{
    if (g.M > 16 || !W.has_fields || W.g128) return false;
    if (g.a_raw ? (g.K % 16 != 0) : !A.has_fields) return false;
    PlanOverride ov;
    lookup_plan(g.p, g.q, g.M, g.N, g.K, &ov);
    const int env = tuning_env("ABQ_DIRECT_R");
    const int forced = ov.direct_r != 0 ? ov.direct_r : env;
    if (forced != 0 && forced != -2) return false;
    if (forced == 0 && (g.M <= 8 || g.p > 4 || (g.p == 4 && W.NT <= 3 * num_cus()))) return false;
    return shared_a_plan(g.p, g.M, W.NT, A.Kp, g.a_raw != nullptr, g.K, forced == -2, pl);
}
static hipError_t launch_decode(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s)
{
    DirectPlan pl;
    SharedAPlan sp;
    if (choose_direct(g, A, W, &pl)) { g_last_decode_kernel = ABQ_DECODE_DIRECT; return launch_gemm_direct(g, A, W, pl, s); }
    if (choose_shared_a(g, A, W, &sp)) { g_last_decode_kernel = ABQ_DECODE_SHARED_OPERAND; return launch_gemm_shared_a(g, A, W, sp, s); }
    g_last_decode_kernel = ABQ_DECODE_STREAMING;
    return launch_gemm_skinny(g, A, W, s);
}

size_t abq_f4_packed_bytes(int bits, int rows, int K)
{
    if (bits < 1 || bits > 2 || rows < 1 || K < 1 || K > ABQ_MAX_K) return 0;
    return f4_packed_bytes(rows, K);
}

int abq_f4_pack_codes(int bits, int rows, int K, const uint8_t* codes, const float* scale, const int32_t* zero, void* packed_out,
                      size_t packed_bytes, void* stream)
{
    if (!codes || !scale || !zero || !packed_out) return ABQ_ERR_NULL;
    if (bits < 1 || bits > 2) return ABQ_ERR_BITS;
    if (rows < 1 || K < 1 || K > ABQ_MAX_K) return ABQ_ERR_SHAPE;
    if (misaligned(codes) || misaligned(scale) || misaligned(zero) || misaligned(packed_out)) return ABQ_ERR_ALIGN;
    if (packed_bytes < f4_packed_bytes(rows, K)) return ABQ_ERR_SIZE;
    return hip_status(launch_f4_pack(bits, rows, K, codes, scale, zero, (uint8_t*)packed_out, (hipStream_t)stream));
}

int abq_f4_gemm(int p, int q, int M, int N, int K, const void* packed_act, const void* packed_w, uint16_t* y_fp16, int32_t* acc_i32,
                void* stream)
{
    if (!packed_act || !packed_w || !y_fp16) return ABQ_ERR_NULL;
    if (p < 1 || p > 2 || q < 1 || q > 2) return ABQ_ERR_BITS;
    if (M < 1 || N < 1 || K < 1 || K > ABQ_MAX_K) return ABQ_ERR_SHAPE;
    if (misaligned(packed_act) || misaligned(packed_w) || misaligned(y_fp16) || misaligned(acc_i32)) return ABQ_ERR_ALIGN;
    return hip_status(launch_f4_gemm(M, N, K, (const uint8_t*)packed_act, (const uint8_t*)packed_w, y_fp16, acc_i32, (hipStream_t)stream));
}

int abq_plan_set(int p, int q, int M, int N, int K, const abq_plan* plan)
{
    if (int e = check_gemm_shape(p, q, M, N, K)) return e;
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    if (!plan) {
        g_plans.erase({p, q, M, N, K});
    } else {
        const int w = plan->skinny_waves, g = plan->skinny_kgroups, mt = plan->tiled_mt, nt = plan->tiled_ntw, wd = plan->tiled_wd;
        const int dr = plan->direct_r;
        const bool ok = (w == 0 || w == 1 || w == 2 || (w >= 4 && w <= 8)) && g >= 0 && g <= 4 && (mt == 0 || mt == 4 || mt == 8) &&
                        (nt == 0 || nt == 1 || nt == 2 || nt == 4) && (wd == 0 || wd == 2 || wd == 4) && plan->tiled_band >= 0 &&
                        (dr == -2 || dr == -1 || dr == 0 || dr == 1 || dr == 2 || dr == 4);
        if (!ok) return ABQ_ERR_LAYOUT;
        g_plans[{p, q, M, N, K}] = PlanOverride{w, g, mt, nt, wd, plan->tiled_band, dr};
    }
    g_plan_count.store((int)g_plans.size(), std::memory_order_relaxed);
    return ABQ_OK;
}

int abq_plan_get(int p, int q, int M, int N, int K, abq_plan* out)
{
    if (!out) return ABQ_ERR_NULL;
    if (int e = check_gemm_shape(p, q, M, N, K)) return e;
    PlanOverride o;
    lookup_plan(p, q, M, N, K, &o);
    *out = abq_plan{o.skinny_waves, o.skinny_kgroups, o.tiled_mt, o.tiled_ntw, o.tiled_wd, o.tiled_band, o.direct_r};
    return ABQ_OK;
}

void abq_plan_clear(void)
{
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    g_plans.clear();
    g_plan_count.store(0, std::memory_order_relaxed);
}

size_t abq_gemm_workspace_bytes(int p, int q, int M, int N, int K)
{
    if (check_gemm_shape(p, q, M, N, K) != ABQ_OK) return 0;
    return 0;   // no kernel needs scratch at present
}

static const Requant kNoRequant{nullptr, nullptr, nullptr, 0};

static int gemm_impl(int p, int q, int M, int N, int K, const void* packed_act, int a_layout, const void* packed_w,
                     int w_layout, uint16_t* y_fp16, int32_t* acc_i32, void* workspace, size_t workspace_bytes, void* stream,
                     const Requant& rq)
{
    if (!packed_act || !packed_w || (!y_fp16 && !rq.codes)) return ABQ_ERR_NULL;
    if (int e = check_gemm_shape(p, q, M, N, K)) return e;
    const int force = w_layout & (ABQ_USE_PLANES | ABQ_USE_FIELDS);
    w_layout &= ~(ABQ_USE_PLANES | ABQ_USE_FIELDS);
    if (force == (ABQ_USE_PLANES | ABQ_USE_FIELDS)) return ABQ_ERR_LAYOUT;
    ActLayout A;
    WeightLayout W;
    if (!make_act_layout(q, M, K, a_layout, &A) || !make_weight_layout(p, N, K, w_layout, &W)) return ABQ_ERR_LAYOUT;
    const bool can_fields = A.has_fields && W.has_fields, can_planes = A.has_planes && W.has_planes;
    if (!can_fields && !can_planes) return ABQ_ERR_LAYOUT;
    if ((force == ABQ_USE_PLANES && !can_planes) || (force == ABQ_USE_FIELDS && !can_fields)) return ABQ_ERR_LAYOUT;
    if (misaligned(packed_act) || misaligned(packed_w) || misaligned(y_fp16) || misaligned(acc_i32) || misaligned(workspace))
        return ABQ_ERR_ALIGN;
    const size_t need = abq_gemm_workspace_bytes(p, q, M, N, K);
    if (need > 0 && (!workspace || workspace_bytes < need)) return workspace ? ABQ_ERR_SIZE : ABQ_ERR_NULL;
    if (W.g128 && (acc_i32 || force == ABQ_USE_PLANES || rq.codes)) return ABQ_ERR_LAYOUT;

    GemmArgs g{p, q, M, N, K, (const uint8_t*)packed_act, nullptr, nullptr, nullptr, (const uint8_t*)packed_w, y_fp16, acc_i32,
               workspace, workspace_bytes, rq};
    hipStream_t s = (hipStream_t)stream;
    if (W.g128)   // per-group weight parameters: the streaming kernel up to 16 rows of A, the tiled per-group kernel above
        return hip_status(M <= kSkinnyMaxM ? launch_decode(g, A, W, s) : launch_gemm_tiled(g, A, W, s));
    if (!choose_fields(can_fields, can_planes, force, p, q, M, N)) return hip_status(launch_gemm_bitserial(g, A, W, s));
    if (streaming_shape(M, N)) return hip_status(launch_decode(g, A, W, s));
    return hip_status(launch_gemm_tiled(g, A, W, s));
}

int abq_gemm(int p, int q, int M, int N, int K, const void* packed_act, int a_layout, const void* packed_w,
             int w_layout, uint16_t* y_fp16, int32_t* acc_i32, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!y_fp16) return ABQ_ERR_NULL;
    return gemm_impl(p, q, M, N, K, packed_act, a_layout, packed_w, w_layout, y_fp16, acc_i32, workspace, workspace_bytes, stream, kNoRequant);
}

// The fused call runs as one kernel when abq_gemm on the same problem would pick the streaming kernel
// and the rows of A can be read as whole 16-byte vectors.
static bool fused_act_direct(const WeightLayout& W, int force, int p, int q, int M, int N, int K)
{
    if (!W.has_fields || force == ABQ_USE_PLANES) return false;
    if (W.g128) return M <= kSkinnyMaxM && K % 16 == 0;
    if (!choose_fields(true, W.has_planes, force, p, q, M, N)) return false;
    return streaming_shape(M, N) && K % 16 == 0;
}

size_t abq_gemm_act_codes_workspace_bytes(int p, int q, int M, int N, int K, int w_layout)
{
    if (check_gemm_shape(p, q, M, N, K) != ABQ_OK) return 0;
    const int force = w_layout & (ABQ_USE_PLANES | ABQ_USE_FIELDS);
    w_layout &= ~(ABQ_USE_PLANES | ABQ_USE_FIELDS);
    WeightLayout W;
    if (force == (ABQ_USE_PLANES | ABQ_USE_FIELDS) || !make_weight_layout(p, N, K, w_layout, &W)) return 0;
    if (fused_act_direct(W, force, p, q, M, N, K)) return 0;
    return abq_packed_act_bytes(q, M, K, W.g128 ? ABQ_LAYOUT_FIELDS : w_layout) + abq_gemm_workspace_bytes(p, q, M, N, K);
}

static int gemm_act_codes_impl(int p, int q, int M, int N, int K, const uint8_t* a_codes, const float* a_scale,
                               const int32_t* a_zero, const void* packed_w, int w_layout, uint16_t* y_fp16, int32_t* acc_i32,
                               void* workspace, size_t workspace_bytes, void* stream, const Requant& rq)
{
    if (!a_codes || !a_scale || !a_zero || !packed_w || (!y_fp16 && !rq.codes)) return ABQ_ERR_NULL;
    if (int e = check_gemm_shape(p, q, M, N, K)) return e;
    const int force = w_layout & (ABQ_USE_PLANES | ABQ_USE_FIELDS);
    const int base_layout = w_layout & ~(ABQ_USE_PLANES | ABQ_USE_FIELDS);
    if (force == (ABQ_USE_PLANES | ABQ_USE_FIELDS)) return ABQ_ERR_LAYOUT;
    WeightLayout W;
    if (!make_weight_layout(p, N, K, base_layout, &W)) return ABQ_ERR_LAYOUT;
    if ((force == ABQ_USE_PLANES && !W.has_planes) || (force == ABQ_USE_FIELDS && !W.has_fields)) return ABQ_ERR_LAYOUT;
    if (misaligned(a_codes) || misaligned(a_scale) || misaligned(a_zero) || misaligned(packed_w) || misaligned(y_fp16) ||
        misaligned(acc_i32) || misaligned(workspace))
        return ABQ_ERR_ALIGN;
    if (W.g128 && (acc_i32 || rq.codes)) return ABQ_ERR_LAYOUT;
    hipStream_t s = (hipStream_t)stream;
    if (fused_act_direct(W, force, p, q, M, N, K)) {
        ActLayout A;
        if (!make_act_layout(q, M, K, ABQ_LAYOUT_FIELDS, &A)) return ABQ_ERR_LAYOUT;
        GemmArgs g{p, q, M, N, K, nullptr, a_codes, a_scale, a_zero, (const uint8_t*)packed_w, y_fp16, acc_i32, nullptr, 0, rq};
        return hip_status(launch_decode(g, A, W, s));
    }
    // Otherwise the two steps run back to back, the packed activations living in the caller's workspace.
    const int act_layout = W.g128 ? ABQ_LAYOUT_FIELDS : base_layout;
    const size_t act_bytes = abq_packed_act_bytes(q, M, K, act_layout);
    const size_t need = act_bytes + abq_gemm_workspace_bytes(p, q, M, N, K);
    if (!workspace) return ABQ_ERR_NULL;
    if (workspace_bytes < need) return ABQ_ERR_SIZE;
    if (int e = abq_pack_act_codes(q, M, K, a_codes, a_scale, a_zero, act_layout, workspace, act_bytes, stream)) return e;
    return gemm_impl(p, q, M, N, K, workspace, act_layout, packed_w, w_layout, y_fp16, acc_i32,
                     (uint8_t*)workspace + act_bytes, workspace_bytes - act_bytes, stream, rq);
}

int abq_gemm_act_codes(int p, int q, int M, int N, int K, const uint8_t* a_codes, const float* a_scale,
                       const int32_t* a_zero, const void* packed_w, int w_layout, uint16_t* y_fp16, int32_t* acc_i32,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!y_fp16) return ABQ_ERR_NULL;
    return gemm_act_codes_impl(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, y_fp16, acc_i32, workspace, workspace_bytes,
                               stream, kNoRequant);
}

int abq_gemm_act_codes_requant(int p, int q, int M, int N, int K, const uint8_t* a_codes, const float* a_scale,
                               const int32_t* a_zero, const void* packed_w, int w_layout, int q_out, const float* out_scale,
                               const int32_t* out_zero, uint8_t* codes_out, uint16_t* y_fp16, void* workspace,
                               size_t workspace_bytes, void* stream)
{
    if (!out_scale || !out_zero || !codes_out) return ABQ_ERR_NULL;
    if (q_out < 1 || q_out > 8) return ABQ_ERR_BITS;
    if (misaligned(out_scale) || misaligned(out_zero) || misaligned(codes_out)) return ABQ_ERR_ALIGN;
    const Requant rq{codes_out, out_scale, out_zero, (1 << q_out) - 1};
    return gemm_act_codes_impl(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, y_fp16, nullptr, workspace, workspace_bytes,
                               stream, rq);
}

int abq_gemm_act_codes_static(int p, int q, int M, int N, int K, const uint8_t* a_codes, const float* a_scale,
                              const int32_t* a_zero, const void* packed_w, int w_layout, uint16_t* y_fp16, int32_t* acc_i32,
                              void* stream)
{
    if (!a_codes || !a_scale || !a_zero || !packed_w || !y_fp16) return ABQ_ERR_NULL;
    if (int e = check_gemm_shape(p, q, M, N, K)) return e;
    const int force = w_layout & (ABQ_USE_PLANES | ABQ_USE_FIELDS);
    WeightLayout W;
    if (force == (ABQ_USE_PLANES | ABQ_USE_FIELDS) || !make_weight_layout(p, N, K, w_layout & ~(ABQ_USE_PLANES | ABQ_USE_FIELDS), &W))
        return ABQ_ERR_LAYOUT;
    const size_t need = abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, w_layout);
    if (need > (size_t)ABQ_STATIC_SCRATCH_BYTES) return ABQ_ERR_SIZE;
    void* ws = nullptr;
    if (need > 0) {
        if (int e = hip_status(static_scratch_ptr(&ws))) return e;
    }
    // every byte of the scratch that the matmul reads is written by the pack step of the same call first, so
    // nothing needs clearing between calls
    return abq_gemm_act_codes(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, y_fp16, acc_i32, ws, need, stream);
}

// Validation and layouts of a group; fills the per-problem arrays (sized by the caller) and says whether one
// launch can serve it.
static int prepare_group(int p, int q, int M, int count, const abq_problem* pr, int a_layout, int w_layout,
                         GemmArgs* args, ActLayout* A, WeightLayout* W, bool* raw, bool* fits, int* waves, size_t* lds)
{
    if (!pr) return ABQ_ERR_NULL;
    if (count < 1 || count > 4096) return ABQ_ERR_SHAPE;
    const int force = w_layout & (ABQ_USE_PLANES | ABQ_USE_FIELDS);
    const int base_w = w_layout & ~(ABQ_USE_PLANES | ABQ_USE_FIELDS);
    if (force == (ABQ_USE_PLANES | ABQ_USE_FIELDS)) return ABQ_ERR_LAYOUT;
    *raw = pr[0].a_codes != nullptr;
    for (int i = 0; i < count; ++i) {
        const abq_problem& c = pr[i];
        if (!c.packed_w || !c.y_fp16) return ABQ_ERR_NULL;
        if ((c.a_codes != nullptr) != *raw) return ABQ_ERR_LAYOUT;
        if (*raw ? (!c.a_scale || !c.a_zero || c.packed_act) : !c.packed_act) return *raw && c.packed_act ? ABQ_ERR_LAYOUT : ABQ_ERR_NULL;
        if (int e = check_gemm_shape(p, q, M, c.N, c.K)) return e;
        if (!make_weight_layout(p, c.N, c.K, base_w, &W[i])) return ABQ_ERR_LAYOUT;
        if (W[i].g128 && (c.acc_i32 || force == ABQ_USE_PLANES)) return ABQ_ERR_LAYOUT;
        if (!make_act_layout(q, M, c.K, *raw ? ABQ_LAYOUT_FIELDS : a_layout, &A[i])) return ABQ_ERR_LAYOUT;
        if (misaligned(c.packed_w) || misaligned(c.packed_act) || misaligned(c.a_codes) || misaligned(c.a_scale) ||
            misaligned(c.a_zero) || misaligned(c.y_fp16) || misaligned(c.acc_i32))
            return ABQ_ERR_ALIGN;
        args[i] = GemmArgs{p, q, M, c.N, c.K, (const uint8_t*)c.packed_act, c.a_codes, c.a_scale, c.a_zero,
                           (const uint8_t*)c.packed_w, c.y_fp16, c.acc_i32, nullptr, 0};
    }
    // one launch only where every problem would go to the streaming kernel of the int8-MFMA family anyway
    *fits = force != ABQ_USE_PLANES && M <= kSkinnyMaxM;
    for (int i = 0; i < count && *fits; ++i)
        *fits = W[i].g128 || choose_fields(W[i].has_fields && (*raw || A[i].has_fields), W[i].has_planes && !*raw && A[i].has_planes, force, p, q, M, pr[i].N);
    if (*fits) *fits = gemm_grouped_fits(M, count, args, A, W, waves, lds);
    return ABQ_OK;
}

size_t abq_gemm_grouped_workspace_bytes(int p, int q, int M, int count, const abq_problem* host_problems, int a_layout,
                                        int w_layout)
{
    if (!host_problems || count < 1 || count > 4096) return 0;
    std::vector<GemmArgs> args(count);
    std::vector<ActLayout> A(count);
    std::vector<WeightLayout> W(count);
    bool raw = false, fits = false;
    int waves = 0;
    size_t lds = 0;
    if (prepare_group(p, q, M, count, host_problems, a_layout, w_layout, args.data(), A.data(), W.data(), &raw, &fits, &waves, &lds) != ABQ_OK)
        return 0;
    if (fits || !raw) return 0;
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        const size_t n = abq_gemm_act_codes_workspace_bytes(p, q, M, host_problems[i].N, host_problems[i].K, w_layout);
        if (n > need) need = n;
    }
    return need;
}

int abq_gemm_grouped(int p, int q, int M, int count, const abq_problem* host_problems, int a_layout, int w_layout,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!host_problems) return ABQ_ERR_NULL;
    if (count < 1 || count > 4096) return ABQ_ERR_SHAPE;
    std::vector<GemmArgs> args(count);
    std::vector<ActLayout> A(count);
    std::vector<WeightLayout> W(count);
    bool raw = false, fits = false;
    int waves = 0;
    size_t lds = 0;
    if (int e = prepare_group(p, q, M, count, host_problems, a_layout, w_layout, args.data(), A.data(), W.data(), &raw, &fits, &waves, &lds))
        return e;
    if (misaligned(workspace)) return ABQ_ERR_ALIGN;
    // grouped: the direct kernel for up to eight rows of A below p = 8 (measured on the LLaMA-7B block: W4A8 M = 1 19.6 vs
    // 22.0 us, W2A8 13.9 vs 17.9, W4A8 M = 8 26.0 vs 25.1; at p = 8 its two launches, one per length of K, cost more than
    // they gain: 34.8 vs 33.3 us)
    if (fits && M <= 8 && p < 8 && tuning_env("ABQ_DIRECT_R") >= 0 && gemm_direct_grouped_fits(p, M, count, args.data(), A.data(), W.data()))
        return hip_status(launch_gemm_direct_grouped(p, q, M, count, args.data(), A.data(), W.data(), (hipStream_t)stream));
    if (fits && W[0].g128 && tuning_env("ABQ_DIRECT_R") >= 0) {
        // per-group blobs: the members the direct kernel's g128 variant takes (K <= 8192) go there in one launch, the others
        // to the streaming kernel's grouped launch (LLaMA-7B block W4A8 g128 M = 1: 28.2 us as one streaming launch)
        std::vector<GemmArgs> a1, a2;
        std::vector<ActLayout> A1, A2;
        std::vector<WeightLayout> W1, W2;
        for (int i = 0; i < count; ++i) {
            const bool d = gemm_direct_g128_fits(p, M, args[i], A[i], W[i]);
            (d ? a1 : a2).push_back(args[i]);
            (d ? A1 : A2).push_back(A[i]);
            (d ? W1 : W2).push_back(W[i]);
        }
        if (!a1.empty()) {
            if (int e = hip_status(launch_gemm_direct_grouped(p, q, M, (int)a1.size(), a1.data(), A1.data(), W1.data(), (hipStream_t)stream))) return e;
            if (a2.empty()) return ABQ_OK;
            if (a2.size() == 1) return hip_status(launch_gemm_skinny(a2[0], A2[0], W2[0], (hipStream_t)stream));   // (a set of one: the single launch's plan)
            int waves2 = 0;
            size_t lds2 = 0;
            if (!gemm_grouped_fits(M, (int)a2.size(), a2.data(), A2.data(), W2.data(), &waves2, &lds2)) return ABQ_ERR_SHAPE;   // (a subset of a set that fits)
            return hip_status(launch_gemm_grouped(p, M, (int)a2.size(), a2.data(), A2.data(), W2.data(), waves2, lds2, (hipStream_t)stream));
        }
    }
    if (fits) return hip_status(launch_gemm_grouped(p, M, count, args.data(), A.data(), W.data(), waves, lds, (hipStream_t)stream));
    if (raw) {   // every problem's workspace need is checked before the first launch
        size_t need = 0;
        for (int i = 0; i < count; ++i) {
            const size_t n = abq_gemm_act_codes_workspace_bytes(p, q, M, host_problems[i].N, host_problems[i].K, w_layout);
            if (n > need) need = n;
        }
        if (need > 0 && !workspace) return ABQ_ERR_NULL;
        if (workspace_bytes < need) return ABQ_ERR_SIZE;
    }
    for (int i = 0; i < count; ++i) {
        const abq_problem& c = host_problems[i];
        const int e = raw ? abq_gemm_act_codes(p, q, M, c.N, c.K, c.a_codes, c.a_scale, c.a_zero, c.packed_w, w_layout, c.y_fp16,
                                               c.acc_i32, workspace, workspace_bytes, stream)
                          : abq_gemm(p, q, M, c.N, c.K, c.packed_act, a_layout, c.packed_w, w_layout, c.y_fp16, c.acc_i32,
                                     workspace, workspace_bytes, stream);
        if (e != ABQ_OK) return e;
    }
    return ABQ_OK;
}

}  // extern "C"
