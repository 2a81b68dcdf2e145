// Prefill-shaped matmul (M > 64): a dense int8 contraction on the 16x16x64 MFMA.
//
// Workgroup tile 128 (rows of A) x 128 (rows of W), four waves side by side along N, each owning
// two 16-row tiles of W for all 128 rows of A (8 x 2 accumulator tiles).  The packed weight
// plane groups go from HBM straight into registers in the same tiled layout the decode kernel
// streams (one super-chunk of 512 k ahead) and are expanded there: for every 64-k slice the
// fields of all groups are shifted to their bit position and OR-ed into one signed byte per
// weight, so a slice costs one MFMA per accumulator tile whatever p is.  (This is the bit
// reduction of Sec. 3.4 step 5 / Appendix B folded into the operand: the 2^s factors are bit
// positions inside the byte, the 2^t factors are the activation code itself.)  The rows of A
// pass through LDS in 128-k steps, double buffered, one barrier per step.  The dequant epilogue
// is fused (Fig. 3b).
#include "abq_internal.h"
#include "../../include/abq.h"

namespace abq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBN = 128, kStepK = 128;
constexpr int kARow = kStepK + 16;   // LDS row stride: the 16 rows of an operand read fall into distinct 16-B bank groups

struct TiledParams {
    const u4v* fields[3];
    const int8_t* a_codes;
    const RowParams* aparams;
    const RowParams* wparams;
    uint16_t* y;
    int32_t* acc;
    int M, N, K, Kp, nsuper, ntiles;
    int oa, ow;
};

// Operand dword of k-slice `SL` (0..7 inside a super-chunk) for one 16-row tile: all plane groups
// merged into one byte per weight.
template <int P, int SL, int G0 = 0>
__device__ __forceinline__ uint32_t merged_dword(const u4v* w, int j)
{
    constexpr int b = group_width(P, G0), shift = group_shift(P, G0), T = 8 / b;
    constexpr int chunk = SL / T, t = SL % T;
    const uint32_t x = w[shift + chunk][j];   // the group's chunks start at index `shift` (= sum of lower widths)
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

template <int P, int SL>
__device__ __forceinline__ void slice_mfma(const u4v (*w)[P], const uint8_t* a_lane, v4i (*acc)[2])
{
    // a_lane: this lane's A operand address for m-tile 0 of the slice; m-tiles are 16 rows apart
    v4i aop[8];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) aop[mt] = *reinterpret_cast<const v4i*>(a_lane + mt * 16 * kARow);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const v4i bop = merged_operand<P, SL>(w[nt]);
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[mt], bop, acc[mt][nt], 0, 0, 0);
    }
}

template <int P>
__device__ __forceinline__ void load_tiles(const TiledParams& prm, int tile0, int sc, int lane, u4v (*w)[P])
{
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int tile = min(tile0 + nt, prm.ntiles - 1);   // past the last tile: re-read a valid one, never stored
#pragma unroll
        for (int g = 0; g < group_count(P); ++g) {
            const int b = group_width(P, g);
            const u4v* base = prm.fields[g] + ((size_t)tile * prm.nsuper + sc) * (b * 64) + lane;
#pragma unroll
            for (int i = 0; i < b; ++i) w[nt][group_shift(P, g) + i] = base[i * 64];
        }
    }
}

template <int P>
__global__ __launch_bounds__(256) void tiled_kernel(TiledParams prm)
{
    __shared__ __align__(16) uint8_t lds_a[2][kBM * kARow];
    __shared__ RowParams par_a[kBM], par_w[kBN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, G = lane >> 4;
    const int m0 = blockIdx.y * kBM, n0 = blockIdx.x * kBN;
    const int tile0 = blockIdx.x * (kBN / kTileN) + wave * 2;

    // weights of super-chunk 0
    u4v wa[2][P], wb[2][P];
    load_tiles<P>(prm, tile0, 0, lane, wa);

    // epilogue parameters
    if (tid < kBM) par_a[tid] = prm.aparams[min(m0 + tid, prm.M - 1)];
    else par_w[tid - kBM] = prm.wparams[min(n0 + tid - kBM, prm.N - 1)];

    // A tile of one 128-k step: 128 rows x 8 vectors of 16 B; thread t moves vectors t, t+256, t+512, t+768
    int a_row[4], a_vec[4];
    bool a_ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int idx = tid + 256 * u;
        a_row[u] = idx >> 3; a_vec[u] = idx & 7;
        a_ok[u] = m0 + a_row[u] < prm.M;
    }
    const int8_t* a_src[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a_src[u] = prm.a_codes + (size_t)min(m0 + a_row[u], prm.M - 1) * prm.Kp + a_vec[u] * 16;
    uint4 areg[4];
    auto a_load = [&](int step) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint4 v = *reinterpret_cast<const uint4*>(a_src[u] + (size_t)step * kStepK);
            areg[u] = a_ok[u] ? v : make_uint4(0, 0, 0, 0);
        }
    };
    auto a_store = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) *reinterpret_cast<uint4*>(&lds_a[buf][a_row[u] * kARow + a_vec[u] * 16]) = areg[u];
    };

    v4i acc[8][2];
#pragma unroll
    for (int mt = 0; mt < 8; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = v4i{0, 0, 0, 0};

    a_load(0);
    a_store(0);
    __syncthreads();

    const int nsteps = prm.nsuper * 4;
    // one super-chunk (4 steps of 128 k, 8 slices of 64 k) per iteration; weights one super-chunk ahead
    auto super_chunk = [&](const u4v (*wc)[P], u4v (*wn)[P], int sc) {
        if (sc + 1 < prm.nsuper) load_tiles<P>(prm, tile0, sc + 1, lane, wn);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const int step = sc * 4 + st, buf = st & 1;   // 4 steps per super-chunk: the buffer parity is static
            if (step + 1 < nsteps) a_load(step + 1);
            const uint8_t* a_lane = &lds_a[buf][r * kARow + G * 16];
            if (st == 0) { slice_mfma<P, 0>(wc, a_lane, acc); slice_mfma<P, 1>(wc, a_lane + 64, acc); }
            if (st == 1) { slice_mfma<P, 2>(wc, a_lane, acc); slice_mfma<P, 3>(wc, a_lane + 64, acc); }
            if (st == 2) { slice_mfma<P, 4>(wc, a_lane, acc); slice_mfma<P, 5>(wc, a_lane + 64, acc); }
            if (st == 3) { slice_mfma<P, 6>(wc, a_lane, acc); slice_mfma<P, 7>(wc, a_lane + 64, acc); }
            if (step + 1 < nsteps) a_store(buf ^ 1);
            __syncthreads();
        }
    };
    for (int sc = 0; sc < prm.nsuper; sc += 2) {
        super_chunk(wa, wb, sc);
        if (sc + 1 < prm.nsuper) super_chunk(wb, wa, sc + 1);
    }

    // fused epilogue: lane l, register reg of accumulator tile (mt, nt) is row 16*mt + 4*(l/16) + reg, column 16*nt + l%16
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int nl = wave * 32 + nt * 16 + r;
        const int n = n0 + nl;
        const RowParams pw = par_w[nl];
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int ml = mt * 16 + 4 * G + reg;
                const int m = m0 + ml;
                if (m < prm.M && n < prm.N)
                    epilogue_store(acc[mt][nt][reg], prm.oa, prm.ow, prm.K, par_a[ml], pw, (size_t)m * prm.N + n, prm.y, prm.acc);
            }
        }
    }
}

size_t gemm_tiled_workspace_bytes(int, int, int, int, int) { return 0; }

template <int P>
static hipError_t launch_p(const TiledParams& prm, dim3 grid, hipStream_t s)
{
    tiled_kernel<P><<<grid, 256, 0, s>>>(prm);
    return hipGetLastError();
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
    prm.M = g.M; prm.N = g.N; prm.K = g.K; prm.Kp = A.Kp;
    prm.nsuper = A.Kp / kSuperK;
    prm.ntiles = W.NT;
    prm.oa = (g.q == 8) ? 128 : 0;
    prm.ow = (g.p == 8) ? 128 : 0;
    dim3 grid((unsigned)((g.N + kBN - 1) / kBN), (unsigned)((g.M + kBM - 1) / kBM));
    switch (g.p) {
        case 1: return launch_p<1>(prm, grid, s);
        case 2: return launch_p<2>(prm, grid, s);
        case 3: return launch_p<3>(prm, grid, s);
        case 4: return launch_p<4>(prm, grid, s);
        case 5: return launch_p<5>(prm, grid, s);
        case 6: return launch_p<6>(prm, grid, s);
        case 7: return launch_p<7>(prm, grid, s);
        default: return launch_p<8>(prm, grid, s);
    }
}

}  // namespace abq
