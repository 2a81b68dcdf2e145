// The very-low-bit matmul on gfx950's 4-bit floating-point MFMA: operands of one or two bits (weights AND activations).
//
// Appendix B decomposes a p x q-bit matmul into p*q binary ones because the tensor cores it targets multiply 1-bit
// planes; the point of Sec. 3.4 / Table 4 is that narrower operands should run faster.  The int8 MFMA path of this
// library carries a whole byte per operand whatever p and q are.  gfx950 has a 16x16x128 MFMA on 4-bit E2M1 operands at
// twice the int8 rate, and the codes 0..3 are E2M1 values (0, 1, 2, 3 = 0b0000, 0b0010, 0b0100, 0b0101): their products
// (<= 9) and the sums of them are exact in the instruction's binary32 accumulator as long as K * 9 < 2^24, far beyond
// any K the library accepts, so the accumulator converts to the same int32 the other kernels produce, and the fused
// dequant epilogue (Fig. 3b) is theirs.  Block scales of the instruction are 2^0.
//
// Both operands use ONE packed layout (so one packer serves weights and activations): after the header and the row
// parameters, [row tiles of 16][K blocks of 128][64 lanes][16 bytes] — 1 KiB per (16 rows x 128 k), lane L holding row
// L % 16, k = 128 block + 32 (L / 16) .. + 31 as 32 nibbles, which is the MFMA operand of that block as it stands.
// Rows past the end and k past K hold code 0.
//
// Kernel: workgroup tile 256 rows of A x 128 channels of W, four waves of 64 x 128 each (32 accumulator tiles; 64 x 128
// with waves of 16 x 128 for problems of few tiles), K in
// steps of 128: the step's 16 + 8 operand blocks go global -> LDS with direct 128-bit loads (a block is one wave
// instruction and lands in LDS as the operand layout: conflict-free 128-bit reads), one barrier per step; three workgroups
// share a compute unit with two operand buffers each, or two with three buffers each (launch_f4_gemm says when), and
// hide each other's waits.
#include "abq_internal.h"
#include "../../include/abq.h"

#include <atomic>

namespace abq {

typedef int v4i_f4 __attribute__((ext_vector_type(4)));
typedef int v8i_f4 __attribute__((ext_vector_type(8)));
typedef float v4f_f4 __attribute__((ext_vector_type(4)));

constexpr int kF4BlockK = 128;                 // k per operand block
constexpr int kF4TileN = 128;                  // channels of W per workgroup tile (the rows of A: F4Shape)

static inline int f4_row_tiles(int rows) { return (rows + 15) / 16; }
static inline int f4_k_blocks(int K) { return (K + kF4BlockK - 1) / kF4BlockK; }

size_t f4_packed_bytes(int rows, int K)
{
    return kHeaderBytes + align_up((size_t)rows * sizeof(RowParams), 256) + (size_t)f4_row_tiles(rows) * f4_k_blocks(K) * 1024;
}
static inline size_t f4_off_params() { return kHeaderBytes; }
static inline size_t f4_off_blocks(int rows) { return kHeaderBytes + align_up((size_t)rows * sizeof(RowParams), 256); }

// ---- packer ---------------------------------------------------------------------------------------------------------
// Four codes in the bytes of a dword (already masked to 0..3) -> their four E2M1 nibbles in the low 16 bits: a code c
// becomes c << 1, except 3, which becomes 5 (0, 1, 2, 3 = 0b0000, 0b0010, 0b0100, 0b0101).
__device__ __forceinline__ uint32_t f4_nibbles(uint32_t x)
{
    const uint32_t three = x & (x >> 1) & 0x01010101u;             // 1 in the bytes that hold 3
    const uint32_t nib = (x << 1) ^ (three * 3u);                  // one E2M1 value per byte
    const uint32_t pairs = (nib | (nib >> 4)) & 0x00FF00FFu;       // bytes 0, 2: nibble pairs (0,1), (2,3)
    return (pairs | (pairs >> 8)) & 0xFFFFu;
}

// One thread per (row tile, K block, lane): 32 codes of one row -> 32 E2M1 nibbles (16 bytes).  vec: K is a multiple
// of 16 and the rows are 16-byte aligned, so the 32 codes are two 128-bit loads.
__global__ void f4_pack_blocks_kernel(const uint8_t* codes, int rows, int K, int kblocks, uint32_t mask, int vec, v4i_f4* out, size_t nvec)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nvec) return;
    const int lane = (int)(i & 63);
    const size_t blk = i >> 6;
    const int kb = (int)(blk % kblocks), rt = (int)(blk / kblocks);
    const int row = rt * 16 + (lane & 15), k0 = kb * kF4BlockK + (lane >> 4) * 32;
    uint32_t w[4] = {0, 0, 0, 0};
    if (row < rows) {
        const uint8_t* src = codes + (size_t)row * K;
        if (vec && k0 + 32 <= K) {
            const uint32_t m4 = mask * 0x01010101u;
            const v4i_f4 lo = *reinterpret_cast<const v4i_f4*>(src + k0), hi = *reinterpret_cast<const v4i_f4*>(src + k0 + 16);
            w[0] = f4_nibbles((uint32_t)lo.x & m4) | (f4_nibbles((uint32_t)lo.y & m4) << 16);
            w[1] = f4_nibbles((uint32_t)lo.z & m4) | (f4_nibbles((uint32_t)lo.w & m4) << 16);
            w[2] = f4_nibbles((uint32_t)hi.x & m4) | (f4_nibbles((uint32_t)hi.y & m4) << 16);
            w[3] = f4_nibbles((uint32_t)hi.z & m4) | (f4_nibbles((uint32_t)hi.w & m4) << 16);
        } else {
            for (int e = 0; e < 32; ++e) {
                const int k = k0 + e;
                const uint32_t c = k < K ? (src[k] & mask) : 0u;
                const uint32_t nib = c == 3 ? 5u : (c << 1);
                w[e >> 3] |= nib << (4 * (e & 7));
            }
        }
    }
    out[i] = v4i_f4{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
}

// Row parameters {sum of the row's codes, scale, zero}: one workgroup per row.
__global__ void f4_row_params_kernel(const uint8_t* codes, int K, uint32_t mask, int vec, const float* scale, const int32_t* zero, RowParams* out)
{
    __shared__ int32_t part[256];
    const int row = (int)blockIdx.x;
    const uint8_t* src = codes + (size_t)row * K;
    uint32_t s = 0;
    int done = 0;
    if (vec) {   // 128-bit loads, byte sums four at a time
        const uint32_t m4 = mask * 0x01010101u;
        done = K & ~15;
        for (int k = (int)threadIdx.x * 16; k < done; k += (int)blockDim.x * 16) {
            const v4i_f4 x = *reinterpret_cast<const v4i_f4*>(src + k);
            s = __builtin_amdgcn_sad_u8((uint32_t)x.x & m4, 0u, s);
            s = __builtin_amdgcn_sad_u8((uint32_t)x.y & m4, 0u, s);
            s = __builtin_amdgcn_sad_u8((uint32_t)x.z & m4, 0u, s);
            s = __builtin_amdgcn_sad_u8((uint32_t)x.w & m4, 0u, s);
        }
    }
    for (int k = done + (int)threadIdx.x; k < K; k += (int)blockDim.x) s += (uint32_t)(src[k] & mask);
    part[threadIdx.x] = (int32_t)s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[row] = RowParams{part[0], scale[row], zero[row], 0};
}

__global__ void f4_header_kernel(uint32_t* hdr, uint32_t magic, int bits, int rows, int K)
{
    const int t = (int)threadIdx.x;
    if (t < 64) hdr[t] = t == 0 ? magic : (t == 1 ? 0x34460001u : (t == 2 ? (uint32_t)bits : (t == 3 ? (uint32_t)rows : (t == 4 ? (uint32_t)K : 0u))));
}

hipError_t launch_f4_pack(int bits, int rows, int K, const uint8_t* codes, const float* scale, const int32_t* zero, uint8_t* blob, hipStream_t s)
{
    const uint32_t mask = (1u << bits) - 1u;
    f4_header_kernel<<<1, 64, 0, s>>>((uint32_t*)blob, 0x34514241u /* "ABQ4" */, bits, rows, K);
    const int vec = (K % 16 == 0) ? 1 : 0;   // (the entry point checks that `codes` is 16-byte aligned)
    f4_row_params_kernel<<<(unsigned)rows, 256, 0, s>>>(codes, K, mask, vec, scale, zero, (RowParams*)(blob + f4_off_params()));
    const size_t nvec = (size_t)f4_row_tiles(rows) * f4_k_blocks(K) * 64;
    f4_pack_blocks_kernel<<<(unsigned)((nvec + 255) / 256), 256, 0, s>>>(codes, rows, K, f4_k_blocks(K), mask, vec, (v4i_f4*)(blob + f4_off_blocks(rows)), nvec);
    return hipGetLastError();
}

// ---- matmul ---------------------------------------------------------------------------------------------------------
struct F4Params {
    const v4i_f4* a_blocks;    // [row tiles][kblocks][64]
    const v4i_f4* w_blocks;
    const RowParams* aparams;
    const RowParams* wparams;
    uint16_t* y;
    int32_t* acc;              // may be null
    int M, N, K, kblocks;
    int a_tiles, w_tiles;      // 16-row tiles of the two operands
    int tiles_m, tiles_n;      // workgroup tiles
};

// RT: 16-row tiles of A per wave (4: workgroup tile 256 x 128, the shape for large M; 1: 64 x 128, for problems that would
// otherwise leave compute units idle).  NBUF: operand buffers (2: requested one step ahead; 3: two steps ahead).
template <int RT> struct F4Shape {
    static constexpr int kTileM = 64 * RT;
    static constexpr int kABlocks = 4 * RT, kBlocks = kABlocks + 8;     // operand blocks of a step (A rows, then W channels)
    static constexpr int kStepBytes = kBlocks * 1024;
    static constexpr int kLoads = kBlocks / 4;                          // blocks a wave requests per step
    static constexpr int kPassRows = RT >= 2 ? 32 : 16;                 // rows a wave stages per pass of the epilogue
    static constexpr int kStageBytes = 4 * kPassRows * 272;
    static constexpr int kParamOffset = (kStageBytes + 1023) / 1024 * 1024;
    static constexpr int kEpilogueBytes = kParamOffset + (kTileM + kF4TileN) * (int)sizeof(RowParams);
    static constexpr int lds_bytes(int nbuf) { return nbuf * kStepBytes > kEpilogueBytes ? nbuf * kStepBytes : kEpilogueBytes; }
    static constexpr int wgs_per_cu(int nbuf) { return RT == 4 ? (nbuf == 2 ? 3 : 2) : 4; }
};

template <int NBUF, int RT>
__global__ __launch_bounds__(256, F4Shape<RT>::wgs_per_cu(NBUF)) void f4_gemm_kernel(F4Params prm)
{
    using SH = F4Shape<RT>;
    // NBUF buffers of a step's operands, 1 KiB per block.  After the K loop the same memory holds the epilogue's staging
    // area and, behind it, the parameters.
    extern __shared__ __align__(16) uint8_t lds_f4[];
    uint8_t* const buf0 = lds_f4;
    uint8_t* const buf1 = lds_f4 + SH::kStepBytes;
    uint8_t* const buf2 = lds_f4 + (NBUF - 1) * SH::kStepBytes;   // (NBUF = 2: unused)
    RowParams* const par_a = reinterpret_cast<RowParams*>(lds_f4 + SH::kParamOffset);
    RowParams* const par_w = par_a + SH::kTileM;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroup b runs on XCD b % 8 and each XCD has its own L2: give every XCD a contiguous run of the tile order, row
    // blocks fastest, so that the workgroups resident on one XCD share their column blocks of W and a few row blocks of A.
    const int nwg = prm.tiles_m * prm.tiles_n;
    const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    const int vid = xcd * per + min(xcd, rem) + slot;
    const int m_blk = vid % prm.tiles_m, n_blk = vid / prm.tiles_m;
    const int m0 = m_blk * SH::kTileM, n0 = n_blk * kF4TileN;

    // this wave's blocks of a step: kLoads consecutive ones of the kBlocks (first the A row tiles, then the W tiles); tiles
    // past the operand's end re-read its last tile (their outputs are never stored)
    const v4i_f4* src[SH::kLoads];
#pragma unroll
    for (int u = 0; u < SH::kLoads; ++u) {
        const int blk = wave * SH::kLoads + u;   // wave-uniform
        if (blk < SH::kABlocks) src[u] = prm.a_blocks + ((size_t)min(m0 / 16 + blk, prm.a_tiles - 1) * prm.kblocks) * 64 + lane;
        else src[u] = prm.w_blocks + ((size_t)min(n0 / 16 + (blk - SH::kABlocks), prm.w_tiles - 1) * prm.kblocks) * 64 + lane;
    }
    auto prefetch = [&](int step, uint8_t* buf) {
#pragma unroll
        for (int u = 0; u < SH::kLoads; ++u)
            __builtin_amdgcn_global_load_lds((const void*)(src[u] + (size_t)step * 64),
                                             (__attribute__((address_space(3))) void*)(buf + (wave * SH::kLoads + u) * 1024), 16, 0, 0);
    };

    v4f_f4 acc[RT][8];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = v4f_f4{0.f, 0.f, 0.f, 0.f};

    const int one = 0x7F7F7F7F;   // block scales of 2^0
    auto multiply = [&](const uint8_t* buf) {
        // wave w: rows 16 RT w .. + 16 RT - 1 of the workgroup tile (A blocks RT w ..), all eight W blocks
        v8i_f4 a[RT];
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const v4i_f4 x = *reinterpret_cast<const v4i_f4*>(buf + (wave * RT + i) * 1024 + lane * 16);
            a[i] = v8i_f4{x.x, x.y, x.z, x.w, 0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const v4i_f4 x = *reinterpret_cast<const v4i_f4*>(buf + (SH::kABlocks + j) * 1024 + lane * 16);
            const v8i_f4 b = v8i_f4{x.x, x.y, x.z, x.w, 0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < RT; ++i) acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[i], b, acc[i][j], 4, 4, 0, one, 0, one);
        }
    };
    // wait until all but the youngest step's loads of this wave have landed
    auto wait_all_but_one_step = [&]() {
        if constexpr (SH::kLoads == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
    };
    static_assert(SH::kLoads == 6 || SH::kLoads == 3, "the wait counts above");

    // Operands are requested NBUF - 1 steps ahead.  The direct loads of a buffer have to have landed before the barrier
    // behind which the other waves read it (the barrier's own fence covers LDS instructions, not these loads), so the wait
    // is written out: with three buffers all but the youngest step's loads, which stay in flight across the barrier.
    const int nsteps = prm.kblocks;
    prefetch(0, buf0);
    if constexpr (NBUF == 2) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        for (int step = 0; step < nsteps; step += 2) {
            if (step + 1 < nsteps) prefetch(step + 1, buf1);
            multiply(buf0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (step + 1 < nsteps) {
                if (step + 2 < nsteps) prefetch(step + 2, buf0);
                multiply(buf1);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                __syncthreads();
            }
        }
    } else {
        if (nsteps > 1) prefetch(1, buf1);
        if (nsteps > 1) wait_all_but_one_step();
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        auto one_step = [&](int step, uint8_t* cur, uint8_t* ahead) {   // ahead: the buffer read in step - 1
            if (step + 2 < nsteps) prefetch(step + 2, ahead);
            multiply(cur);
            if (step + 2 < nsteps) wait_all_but_one_step();
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        };
        for (int step = 0; step < nsteps; step += 3) {
            one_step(step, buf0, buf2);
            if (step + 1 < nsteps) one_step(step + 1, buf1, buf0);
            if (step + 2 < nsteps) one_step(step + 2, buf2, buf1);
        }
    }
    // epilogue parameters into the freed operand memory (the other workgroups of the unit hide this round trip)
    if (tid < SH::kTileM) par_a[tid] = prm.aparams[min(m0 + tid, prm.M - 1)];
    if (tid < kF4TileN) par_w[tid] = prm.wparams[min(n0 + tid, prm.N - 1)];
    __syncthreads();

    // ---- epilogue: lane (G, r) of accumulator (i, j) holds rows 16 RT wave + 16 i + 4 G + reg, channel 16 j + r.
    // With up to 128 outputs per lane the epilogue is a third of the kernel if every output is stored on its own (2 bytes
    // per lane and instruction), so the usual case (no accumulator output, rows of Y a whole number of 16-byte vectors)
    // goes through LDS: every wave stages its binary16 results, up to 32 rows x 128 at a time, in its own part of the
    // operand buffers (free after the loop's last barrier; row stride 272 bytes keeps the four row groups of a write on
    // different banks) and writes them out as 128-bit vectors.  The arithmetic is the fused dequant of the other kernels
    // (Fig. 3b), with the terms that depend on the column only taken out of the inner loop:
    // centered = S - wz asum - az (wsum - K wz).
    const int r = lane & 15, G = lane >> 4;
    constexpr int kWaveRows = 16 * RT;
    if (prm.acc == nullptr && (prm.N & 7) == 0) {
        constexpr int kRowBytes = 272, kPassRows = SH::kPassRows, kPassTiles = kPassRows / 16;
        uint8_t* const stage = lds_f4 + wave * (kPassRows * kRowBytes);
        uint32_t wz[8], cw[8];
        float sw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const RowParams pw = par_w[16 * j + r];
            wz[j] = (uint32_t)pw.zero;
            cw[j] = (uint32_t)pw.sum - (uint32_t)prm.K * (uint32_t)pw.zero;
            sw[j] = pw.scale;
        }
#pragma unroll
        for (int pass = 0; pass < kWaveRows / kPassRows; ++pass) {
#pragma unroll
            for (int i2 = 0; i2 < kPassTiles; ++i2)
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    const int i = kPassTiles * pass + i2;
                    const int rl = 16 * i2 + 4 * G + reg;            // row inside this pass
                    const RowParams pa = par_a[kWaveRows * wave + kPassRows * pass + rl];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t S = (uint32_t)(int32_t)acc[i][j][reg];
                        const int32_t centered = (int32_t)(S - wz[j] * (uint32_t)pa.sum - (uint32_t)pa.zero * cw[j]);
                        const float v = ((float)centered * pa.scale) * sw[j];
                        uint32_t h;
                        asm("v_cvt_f16_f32 %0, %1" : "=v"(h) : "v"(v));   // (the instruction itself: see epilogue_value)
                        *reinterpret_cast<uint16_t*>(stage + rl * kRowBytes + (16 * j + r) * 2) = (uint16_t)h;
                    }
                }
            // (the wave reads back what its own lanes wrote, and rewrites the area only after it has read it: no barrier,
            // the LDS counter orders it)
#pragma unroll
            for (int it = 0; it < kPassRows / 4; ++it) {
                const int c = it * 64 + lane, rl = c >> 4, cc = c & 15;
                const v4i_f4 x = *reinterpret_cast<const v4i_f4*>(stage + rl * kRowBytes + cc * 16);
                const int m = m0 + kWaveRows * wave + kPassRows * pass + rl, n = n0 + 8 * cc;
                if (m < prm.M && n < prm.N) *reinterpret_cast<v4i_f4*>(prm.y + (size_t)m * prm.N + n) = x;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int nl = 16 * j + r, n = n0 + nl;
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int ml = kWaveRows * wave + 16 * i + 4 * G + reg, m = m0 + ml;
                if (m < prm.M && n < prm.N)
                    epilogue_store((int32_t)acc[i][j][reg], 0, 0, prm.K, par_a[ml], par_w[nl], (size_t)m * prm.N + n, prm.y, prm.acc);
            }
        }
}

template <int NBUF, int RT>
static hipError_t f4_launch(const F4Params& prm, unsigned grid, hipStream_t s)
{
    constexpr int lds = F4Shape<RT>::lds_bytes(NBUF);
    if constexpr (lds > 64 * 1024) {
        static std::atomic<bool> attr_set{false};   // (an idempotent call: a lost race only repeats it)
        if (!attr_set.load(std::memory_order_acquire)) {
            const hipError_t e = hipFuncSetAttribute((const void*)f4_gemm_kernel<NBUF, RT>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
            attr_set.store(true, std::memory_order_release);
        }
    }
    f4_gemm_kernel<NBUF, RT><<<grid, 256, lds, s>>>(prm);
    return hipGetLastError();
}

hipError_t launch_f4_gemm(int M, int N, int K, const uint8_t* act_blob, const uint8_t* w_blob, uint16_t* y, int32_t* acc, hipStream_t s)
{
    F4Params prm;
    prm.a_blocks = (const v4i_f4*)(act_blob + f4_off_blocks(M));
    prm.w_blocks = (const v4i_f4*)(w_blob + f4_off_blocks(N));
    prm.aparams = (const RowParams*)(act_blob + f4_off_params());
    prm.wparams = (const RowParams*)(w_blob + f4_off_params());
    prm.y = y; prm.acc = acc;
    prm.M = M; prm.N = N; prm.K = K; prm.kblocks = f4_k_blocks(K);
    prm.a_tiles = f4_row_tiles(M); prm.w_tiles = f4_row_tiles(N);
    prm.tiles_n = (N + kF4TileN - 1) / kF4TileN;
    const long cus = num_cus();
    // Workgroup tile: 256 rows where that still gives every compute unit a workgroup, else 64 rows (four times the
    // workgroups; more LDS reads per MFMA, but the chip is busy).
    const long nwg_big = (long)((M + 255) / 256) * prm.tiles_n;
    if (nwg_big < cus) {
        prm.tiles_m = (M + 63) / 64;
        return f4_launch<3, 1>(prm, (unsigned)(prm.tiles_m * prm.tiles_n), s);
    }
    prm.tiles_m = (M + 255) / 256;
    // Two or three workgroups per compute unit: three hide more latency, but the grid runs in rounds of (units x resident
    // workgroups) and a nearly empty last round costs a whole one, so the count that wastes fewer workgroup slots is
    // taken (M = 8192, 4096 x 4096: 1024 workgroups are two full rounds of 512 but 1.33 rounds of 768: 73 vs 85 us); with
    // two, the LDS left over holds a third operand buffer.
    const long nwg = nwg_big;
    const long slots3 = (nwg + 3 * cus - 1) / (3 * cus) * 3, slots2 = (nwg + 2 * cus - 1) / (2 * cus) * 2;
    if (nwg > 2 * cus && slots2 < slots3) return f4_launch<3, 4>(prm, (unsigned)nwg, s);
    return f4_launch<2, 4>(prm, (unsigned)nwg, s);
}

}  // namespace abq
