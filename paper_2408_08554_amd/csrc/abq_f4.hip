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

// The whole blob in one launch (a pack of the activations sits in front of every matmul: three dependent launches
// cost more than the work).  One workgroup of sixteen waves per tile of 16 rows; wave w packs the K blocks w, w + 16, ...:
// lane L takes 32 codes of row L % 16 at k = 128 kb + 32 (L / 16) -> 32 E2M1 nibbles (16 bytes, the operand layout), and
// keeps the sum of its codes; the sums meet across the lanes of a row, then across the waves through LDS, and become the
// rows' parameter records {sum of codes, scale, zero}.  vec: K is a multiple of 16 and the rows are 16-byte aligned, so
// the 32 codes are two 128-bit loads.  Workgroup 0 also writes the header.
constexpr int kF4PackWaves = 16;
__global__ __launch_bounds__(64 * kF4PackWaves) void f4_pack_kernel(const uint8_t* codes, int rows, int K, int kblocks, uint32_t mask, int vec,
                                                                    const float* scale, const int32_t* zero, int bits, uint32_t* hdr,
                                                                    RowParams* params, v4i_f4* out, int ksplit)
{
    __shared__ uint32_t part[kF4PackWaves][16];
    const int tid = (int)threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // ksplit = 2: two workgroups per row tile, one per half of the K blocks (a pack of 2048 rows is otherwise 128
    // workgroups: half the chip); the second writes its sums of codes into the record's spare word
    const int rt = (int)blockIdx.x / ksplit, half = (int)blockIdx.x % ksplit;
    const int kb_per = (kblocks + ksplit - 1) / ksplit, kb_lo = half * kb_per, kb_hi = min(kblocks, kb_lo + kb_per);
    const int row = rt * 16 + (lane & 15);
    const uint8_t* src = codes + (size_t)min(row, rows - 1) * K;   // (rows past the end: a valid row is read, zeros are stored)
    const uint32_t m4 = mask * 0x01010101u;
    uint32_t sum = 0;
    // up to four K blocks of the wave at a time: their loads are all requested before the first is packed
    constexpr int NB = 4;
    for (int kb0 = kb_lo + wave; kb0 < kb_hi; kb0 += kF4PackWaves * NB) {
        v4i_f4 lo[NB], hi[NB];
        bool fast[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int kb = kb0 + kF4PackWaves * u, k0 = kb * kF4BlockK + (lane >> 4) * 32;
            fast[u] = vec && kb < kb_hi && k0 + 32 <= K;
            lo[u] = hi[u] = v4i_f4{0, 0, 0, 0};
            if (fast[u]) {
                lo[u] = *reinterpret_cast<const v4i_f4*>(src + k0);
                hi[u] = *reinterpret_cast<const v4i_f4*>(src + k0 + 16);
            }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int kb = kb0 + kF4PackWaves * u, k0 = kb * kF4BlockK + (lane >> 4) * 32;
            if (kb >= kb_hi) break;   // (the same for the whole wave)
            uint32_t w[4] = {0, 0, 0, 0};
            if (fast[u]) {
                const uint32_t c[8] = {(uint32_t)lo[u].x & m4, (uint32_t)lo[u].y & m4, (uint32_t)lo[u].z & m4, (uint32_t)lo[u].w & m4,
                                       (uint32_t)hi[u].x & m4, (uint32_t)hi[u].y & m4, (uint32_t)hi[u].z & m4, (uint32_t)hi[u].w & m4};
#pragma unroll
                for (int e = 0; e < 8; ++e) sum = __builtin_amdgcn_sad_u8(c[e], 0u, sum);
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = f4_nibbles(c[2 * e]) | (f4_nibbles(c[2 * e + 1]) << 16);
            } else {
                for (int e = 0; e < 32; ++e) {
                    const int k = k0 + e;
                    const uint32_t c = k < K ? (src[k] & mask) : 0u;
                    sum += c;
                    const uint32_t nib = c == 3 ? 5u : (c << 1);
                    w[e >> 3] |= nib << (4 * (e & 7));
                }
            }
            if (row >= rows) w[0] = w[1] = w[2] = w[3] = 0;
            out[((size_t)rt * kblocks + kb) * 64 + lane] = v4i_f4{(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        }
    }
    sum += (uint32_t)__shfl_xor((int)sum, 16);
    sum += (uint32_t)__shfl_xor((int)sum, 32);
    if (lane < 16) part[wave][lane] = sum;
    __syncthreads();
    if (tid < 16 && row < rows) {
        uint32_t total = 0;
#pragma unroll
        for (int w = 0; w < kF4PackWaves; ++w) total += part[w][tid];
        if (half == 0) {
            params[row].sum = (int32_t)total;
            params[row].scale = scale[row];
            params[row].zero = zero[row];
            if (ksplit == 1) params[row].pad = 0;
        } else {
            params[row].pad = (int32_t)total;   // (the matmul adds the two)
        }
    }
    if (blockIdx.x == 0 && tid >= 64 && tid < 128) {
        const int t = tid - 64;
        hdr[t] = t == 0 ? 0x34514241u /* "ABQ4" */ : (t == 1 ? 0x34460001u : (t == 2 ? (uint32_t)bits : (t == 3 ? (uint32_t)rows : (t == 4 ? (uint32_t)K : 0u))));
    }
}

hipError_t launch_f4_pack(int bits, int rows, int K, const uint8_t* codes, const float* scale, const int32_t* zero, uint8_t* blob, hipStream_t s)
{
    const uint32_t mask = (1u << bits) - 1u;
    const int vec = (K % 16 == 0) ? 1 : 0;   // (the entry point checks that `codes` is 16-byte aligned)
    const int ksplit = (f4_k_blocks(K) >= 32 && 2L * f4_row_tiles(rows) <= (long)num_cus()) ? 2 : 1;
    f4_pack_kernel<<<(unsigned)(f4_row_tiles(rows) * ksplit), 64 * kF4PackWaves, 0, s>>>(codes, rows, K, f4_k_blocks(K), mask, vec, scale, zero, bits, (uint32_t*)blob,
                                                                                         (RowParams*)(blob + f4_off_params()), (v4i_f4*)(blob + f4_off_blocks(rows)), ksplit);
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
// otherwise leave compute units idle).
template <int RT> struct F4Shape {
    static constexpr int kTileM = 64 * RT;
    static constexpr int kWBufBytes = 8 * 1024;                         // the eight W blocks of a step
    static constexpr int kPassRows = RT >= 2 ? 32 : 16;                 // rows a wave stages per pass of the epilogue
    static constexpr int kStageBytes = 4 * kPassRows * 272;
    static constexpr int kParamOffset = (kStageBytes + 1023) / 1024 * 1024;
    static constexpr int kEpilogueBytes = kParamOffset + (kTileM + kF4TileN) * (int)sizeof(RowParams);
    static constexpr int kLdsBytes = 3 * kWBufBytes > kEpilogueBytes ? 3 * kWBufBytes : kEpilogueBytes;
};

// The epilogue of the matmul kernel: parameters of the tile's rows and columns into LDS, then the dequantised
// outputs, staged through LDS for 128-bit stores where the output allows it.  lds_f4 is free for reuse when it starts (the
// caller has passed a barrier after its last read, and none of its loads into LDS is in flight).
template <int RT>
__device__ __forceinline__ void f4_epilogue(const F4Params& prm, v4f_f4 (*acc)[8], uint8_t* lds_f4, int tid, int lane, int wave, int m0, int n0,
                                            v4i_f4 my_a, v4i_f4 my_w)
{
    using SH = F4Shape<RT>;
    RowParams* const par_a = reinterpret_cast<RowParams*>(lds_f4 + SH::kParamOffset);
    RowParams* const par_w = par_a + SH::kTileM;
    // epilogue parameters (fetched by the kernel before its K loop: no memory round trip here) into the freed operand memory
    // (a record's sum of codes may come in two parts, the second in its spare word: see f4_pack_kernel)
    if (tid < SH::kTileM) *reinterpret_cast<v4i_f4*>(par_a + tid) = v4i_f4{my_a.x + my_a.w, my_a.y, my_a.z, 0};
    if (tid < kF4TileN) *reinterpret_cast<v4i_f4*>(par_w + tid) = v4i_f4{my_w.x + my_w.w, my_w.y, my_w.z, 0};
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
        // Every term here is an integer below 2^24 in magnitude (K * 9 < 2^24: the entry point checks it), and so is every
        // partial sum, so binary32 fused multiply-adds give the int32 arithmetic's value exactly, at four times the rate
        // of 32-bit integer multiplies; the accumulator needs no conversion either.
        float wz[8], cw[8], sw[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const RowParams pw = par_w[16 * j + r];
            wz[j] = -(float)pw.zero;
            cw[j] = (float)(pw.sum - prm.K * pw.zero);
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
                    const float asum = (float)pa.sum, az = -(float)pa.zero;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float centered = __builtin_fmaf(az, cw[j], __builtin_fmaf(wz[j], asum, acc[i][j][reg]));
                        const float v = (centered * pa.scale) * sw[j];
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

// Y = dequant(A W^T) on the 4-bit floating-point MFMA.  Four waves; wave w owns rows 16 RT w .. of the tile and all 128
// columns.  Its A blocks go global -> registers (a wave's rows are its own: nothing to share), the eight W blocks of a step
// go global -> LDS, where every wave reads them: per MFMA a wave reads 0.25 KiB of LDS.
template <int RT>
__global__ __launch_bounds__(256, RT == 4 ? 2 : 4) void f4_gemm_kernel(F4Params prm)
{
    using SH = F4Shape<RT>;
    // Three buffers of a step's W blocks, 1 KiB per block.  After the K loop the same memory holds the epilogue's staging
    // area and, behind it, the parameters.
    extern __shared__ __align__(16) uint8_t lds_f4[];
    uint8_t* const buf0 = lds_f4;
    uint8_t* const buf1 = lds_f4 + SH::kWBufBytes;
    uint8_t* const buf2 = lds_f4 + 2 * SH::kWBufBytes;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Workgroup b runs on XCD b % 8 and each XCD has its own L2: give every XCD a contiguous run of the tile order, so
    // that the workgroups resident on one XCD share their column blocks of W and their row blocks of A.
    const int nwg = prm.tiles_m * prm.tiles_n;
    const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    const int vid = xcd * per + min(xcd, rem) + slot;
    // Within the order, row tiles go in panels of eight: the workgroups resident on an XCD at one time then cover about as
    // many row tiles as column tiles, which is the least operand traffic into its L2 for that many tiles.
    const int panel_wgs = 8 * prm.tiles_n, panel = vid / panel_wgs, in_panel = vid - panel * panel_wgs;
    const int panel_rows = min(8, prm.tiles_m - 8 * panel);
    const int m_blk = 8 * panel + in_panel % panel_rows, n_blk = in_panel / panel_rows;
    const int m0 = m_blk * SH::kTileM, n0 = n_blk * kF4TileN;

    // the epilogue's parameters of this tile's rows and channels, one record per thread: on their way during the K loop
    v4i_f4 my_a = v4i_f4{0, 0, 0, 0}, my_w = my_a;   // (a record is 16 bytes)
    if (tid < SH::kTileM) my_a = *reinterpret_cast<const v4i_f4*>(prm.aparams + min(m0 + tid, prm.M - 1));
    if (tid < kF4TileN) my_w = *reinterpret_cast<const v4i_f4*>(prm.wparams + min(n0 + tid, prm.N - 1));

    const v4i_f4* a_src[RT];
#pragma unroll
    for (int i = 0; i < RT; ++i) a_src[i] = prm.a_blocks + ((size_t)min(m0 / 16 + wave * RT + i, prm.a_tiles - 1) * prm.kblocks) * 64 + lane;
    const v4i_f4* w_src[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) w_src[u] = prm.w_blocks + ((size_t)min(n0 / 16 + wave * 2 + u, prm.w_tiles - 1) * prm.kblocks) * 64 + lane;

    v4f_f4 acc[RT][8];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = v4f_f4{0.f, 0.f, 0.f, 0.f};

    const int one = 0x7F7F7F7F;   // block scales of 2^0
    // One step of K: the W blocks are read from LDS two at a time, one pair ahead of the MFMAs that use them, so that a
    // wave's LDS latency runs under its own MFMAs (the scheduling barriers keep the reads where they are written).
    auto multiply = [&](const uint8_t* buf, const v4i_f4* ar) {
        v8i_f4 a[RT];
#pragma unroll
        for (int i = 0; i < RT; ++i) a[i] = v8i_f4{ar[i].x, ar[i].y, ar[i].z, ar[i].w, 0, 0, 0, 0};
        const uint8_t* const mine = buf + lane * 16;
        v4i_f4 x[2][2];
        x[0][0] = *reinterpret_cast<const v4i_f4*>(mine);
        x[0][1] = *reinterpret_cast<const v4i_f4*>(mine + 1024);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g < 3) {
                x[(g + 1) & 1][0] = *reinterpret_cast<const v4i_f4*>(mine + (2 * g + 2) * 1024);
                x[(g + 1) & 1][1] = *reinterpret_cast<const v4i_f4*>(mine + (2 * g + 3) * 1024);
            }
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(1);   // (the wave that has its operands goes first: 1-2 % with two workgroups per unit)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const v4i_f4 xb = x[g & 1][h];
                const v8i_f4 b = v8i_f4{xb.x, xb.y, xb.z, xb.w, 0, 0, 0, 0};
#pragma unroll
                for (int i = 0; i < RT; ++i)
                    acc[i][2 * g + h] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[i], b, acc[i][2 * g + h], 4, 4, 0, one, 0, one);
            }
            __builtin_amdgcn_s_setprio(0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Two steps ahead: three LDS buffers for W and three register sets for A, used in rotation.  A wave issues RT + 2
    // vector-memory loads per step, in order, so "at most RT + 2 outstanding" means the step before the newest has landed.
    // The body of the main loop has no branch: past the last step it loads that step again into a buffer and a register
    // set that nothing reads any more.  The wait and the barrier are written out: a workgroup fence would wait for every
    // outstanding load (the loads into LDS count as LDS writes), the newest included, and the scheduling barriers keep
    // the MFMAs above the wait.
    const int nsteps = prm.kblocks;
    v4i_f4 a0[RT], a1[RT], a2[RT];
    auto load_step = [&](int step, v4i_f4* ar, uint8_t* buf) {
        const size_t off = (size_t)min(step, nsteps - 1) * 64;
        // The register loads are written as instructions: the compiler, seeing register loads and loads into LDS mixed
        // on one counter, would wait for all of them before the first use of these registers.  It does not know that
        // the registers fill later: between here and the MFMAs that read them it must neither copy nor spill them,
        // which the build checks (no scratch memory for this kernel).
#pragma unroll
        for (int i = 0; i < RT; ++i) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(ar[i]) : "v"(a_src[i] + off));
#pragma unroll
        for (int u = 0; u < 2; ++u)
            __builtin_amdgcn_global_load_lds((const void*)(w_src[u] + off), (__attribute__((address_space(3))) void*)(buf + (wave * 2 + u) * 1024), 16, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto sync_keep_newest = [&]() {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (RT == 4) asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(RT == 4 || RT == 1, "the wait counts above are RT + 2");
    load_step(0, a0, buf0);
    load_step(1, a1, buf1);
    sync_keep_newest();
    int step = 0;
    for (; step + 3 <= nsteps; step += 3) {
        load_step(step + 2, a2, buf2);   // (each buffer and register set was last read one step before it is loaded again)
        multiply(buf0, a0);
        sync_keep_newest();
        load_step(step + 3, a0, buf0);
        multiply(buf1, a1);
        sync_keep_newest();
        load_step(step + 4, a1, buf1);
        multiply(buf2, a2);
        sync_keep_newest();
    }
    // the steps left are in a0 / buf0 and a1 / buf1; no load is in flight when the epilogue reuses LDS
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    if (step < nsteps) multiply(buf0, a0);
    if (step + 1 < nsteps) multiply(buf1, a1);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    f4_epilogue<RT>(prm, acc, lds_f4, tid, lane, wave, m0, n0, my_a, my_w);
}

template <int RT>
static hipError_t f4_launch(const F4Params& prm, unsigned grid, hipStream_t s)
{
    f4_gemm_kernel<RT><<<grid, 256, F4Shape<RT>::kLdsBytes, s>>>(prm);   // (under 64 KiB: no attribute to raise)
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
        return f4_launch<1>(prm, (unsigned)(prm.tiles_m * prm.tiles_n), s);
    }
    prm.tiles_m = (M + 255) / 256;
    return f4_launch<4>(prm, (unsigned)nwg_big, s);
}

}  // namespace abq
