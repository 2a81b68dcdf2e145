// The paper's decomposition taken literally (Appendix B): for every weight plane s and
// activation plane t, AND the 1-bit rows and count the set bits along K; the counts are
// weighted by 2^(s+t) and summed ("Bit Reduction", Sec. 3.4 step 5).  gfx950 has no 1-bit
// matrix instruction, so BMMA becomes wavefront-wide v_and + v_bcnt (popcount-accumulate) on
// 128-bit loads of the [bits][rows][K] planes.  Counts of equal s+t share one accumulator,
// which leaves p+q-1 accumulators per output instead of p*q.
//
// Few rows of A (M < 8): a wave owns 4 output channels, 16 lanes per channel; each lane walks the 128-bit
// quads of its channel's planes, then the 16 partial sums are added with in-row shuffles.
// MB rows of A are processed per pass over the weights.  More rows: bitserial_rows_kernel below.
#include "abq_internal.h"
#include "../../include/abq.h"

namespace abq {

struct BitSerialParams {
    const uint4* w_planes;   // [p][N][Kq] quads
    const uint4* a_planes;   // [q][M][Kq]
    const RowParams* aparams;
    const RowParams* wparams;
    uint16_t* y;
    int32_t* acc;
    Requant rq;
    int M, N, K, Kq;
};

template <int P, int Q, int MB>
__global__ __launch_bounds__(256) void bitserial_kernel(BitSerialParams prm)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15;
    const int n = blockIdx.x * 16 + wave * 4 + (lane >> 4);
    const int m0 = blockIdx.y * MB;
    const bool n_valid = n < prm.N;
    constexpr int ND = P + Q - 1;
    int32_t cnt[MB][ND];
#pragma unroll
    for (int mm = 0; mm < MB; ++mm)
#pragma unroll
        for (int d = 0; d < ND; ++d) cnt[mm][d] = 0;

    if (n_valid) {
        for (int kq = sub; kq < prm.Kq; kq += 16) {
            uint4 w[P];
#pragma unroll
            for (int s = 0; s < P; ++s) w[s] = prm.w_planes[((size_t)s * prm.N + n) * prm.Kq + kq];
#pragma unroll
            for (int mm = 0; mm < MB; ++mm) {
                const int m = min(m0 + mm, prm.M - 1);   // rows past M repeat the last one; never stored
#pragma unroll
                for (int t = 0; t < Q; ++t) {
                    const uint4 a = prm.a_planes[((size_t)t * prm.M + m) * prm.Kq + kq];
#pragma unroll
                    for (int s = 0; s < P; ++s) {
                        int32_t c = cnt[mm][s + t];
                        c += __popc(a.x & w[s].x);
                        c += __popc(a.y & w[s].y);
                        c += __popc(a.z & w[s].z);
                        c += __popc(a.w & w[s].w);
                        cnt[mm][s + t] = c;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int mm = 0; mm < MB; ++mm) {
        uint32_t total = 0;
#pragma unroll
        for (int d = 0; d < ND; ++d) total += (uint32_t)cnt[mm][d] << d;   // the 2^(s+t) factors
        int32_t v = (int32_t)total;
#pragma unroll
        for (int off = 8; off > 0; off >>= 1) v += __shfl_xor(v, off, 16);
        const int m = m0 + mm;
        if (sub == 0 && n_valid && m < prm.M)
            epilogue_store(v, 0, 0, prm.K, prm.aparams[m], prm.wparams[n], (size_t)m * prm.N + n, prm.y, prm.acc, prm.rq, m);
    }
}


// ---- many rows of A (M >= 8): one output channel per lane, the activation planes in scalar registers ----------------
// A lane owns one channel and walks all of K for BM rows of A, so nothing is reduced across lanes.  The A planes of a
// row are the same for every lane: they are fetched with scalar loads (wave-uniform addresses) and enter the
// v_and as scalar operands, which leaves the vector ALU exactly the two operations per 32 bit-products that the
// method needs (v_and_b32 + v_bcnt_u32_b32) and no LDS traffic at all.  Per 256 k a lane holds two 128-bit quads
// of each weight plane; a workgroup takes BM rows of A and the grid's second dimension the rest (the weights are
// read again per BM rows, from the caches).
// acc + popcount(a & w): the accumulating form of the popcount instruction (left to the compiler, the counts of
// a quad are taken against zero and added in a tree: five instructions per two words instead of four)
__device__ __forceinline__ int32_t and_count(uint32_t a, uint32_t w, int32_t acc)
{
    const uint32_t x = a & w;
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(x));
    return acc;
}

template <int P, int Q>
struct RowsShape {
    static constexpr int ND = P + Q - 1;
    // NC channels per lane: an A quad, once in scalar registers, meets the weight quads of NC channels, which divides
    // the scalar-load traffic per vector operation by NC (at P = 1 a quad is otherwise used for eight operations only)
    static constexpr int NC = P * Q <= 4 ? 2 : 1;
    // rows of A per workgroup: bounded by the counters (NC * (P + Q - 1) * BM registers) and by the unrolled body
    // (16 * NC * P * Q * BM vector instructions per 256 k)
    static constexpr int BM = P * Q >= 64 ? 1 : (P * Q >= 32 ? 2 : (P * Q >= 16 ? 4 : (P * Q >= 8 ? 8 : (P * Q >= 2 ? 8 : 16))));
};

template <int P, int Q>
__global__ __launch_bounds__(256) void bitserial_rows_kernel(BitSerialParams prm)
{
    using SH = RowsShape<P, Q>;
    constexpr int BM = SH::BM, ND = SH::ND, NC = SH::NC;
    // Workgroup b runs on XCD b % 8 (round-robin dispatch) and each XCD has its own L2: every XCD gets a contiguous run
    // of the order (channel block, row block) with the row blocks fastest, so that the workgroups that read the same
    // weight planes run next to each other on one XCD and the planes leave HBM once.  (With the channel blocks fastest
    // every row block streamed all of W again: measured 1.39 GB of fetches for 17.7 MB of planes at W2A2 M = 256.)
    const int row_blocks = (prm.M + BM - 1) / BM;
    const int nwg = gridDim.x;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    const int vid = xcd * per + min(xcd, rem) + slot;
    const int n0 = (vid / row_blocks) * (256 * NC) + threadIdx.x;  // this lane's channels: n0, n0 + 256, ...
    const int m0 = (vid % row_blocks) * BM;
    const uint4* __restrict__ wp = prm.w_planes;
    const uint4* __restrict__ ap = prm.a_planes;
    const int Kq = prm.Kq;
    int32_t cnt[NC][BM][ND];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int mm = 0; mm < BM; ++mm)
#pragma unroll
            for (int d = 0; d < ND; ++d) cnt[c][mm][d] = 0;

    for (int kq0 = 0; kq0 < Kq; kq0 += 2) {
        const bool two = kq0 + 1 < Kq;                     // (block-uniform)
        uint4 w[NC][P][2];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int s = 0; s < P; ++s) {
                const int nc = min(n0 + c * 256, prm.N - 1);   // lanes past N repeat the last channel; never stored
                const uint4* wrow = wp + ((size_t)s * prm.N + nc) * Kq + kq0;
                w[c][s][0] = wrow[0];
                w[c][s][1] = two ? wrow[1] : uint4{0, 0, 0, 0};
            }
        // The (row, plane) pairs of this step in groups of GP: the A quads of the next group are requested (scalar loads:
        // the addresses are wave-uniform) before the current group is counted, so that a wave waits once per group and
        // mostly finds its operands there.  A quad past the row's end is re-read from its last one (the weight quad it
        // meets is zero); rows past M repeat the last one and are never stored.
        constexpr int NP = BM * Q, GP = NP < 4 ? NP : 4, NGRP = (NP + GP - 1) / GP;
        uint4 cur[GP][2], nxt[GP][2];
        auto load_group = [&](int g, uint4 (*dst)[2]) {
#pragma unroll
            for (int j = 0; j < GP; ++j) {
                const int pr = min(g * GP + j, NP - 1);
                const int m = min(m0 + pr / Q, prm.M - 1);
                const uint4* arow = ap + ((size_t)(pr % Q) * prm.M + m) * Kq;
                dst[j][0] = arow[kq0];
                dst[j][1] = arow[min(kq0 + 1, Kq - 1)];
            }
        };
        load_group(0, cur);
#pragma unroll
        for (int g = 0; g < NGRP; ++g) {
            if (g + 1 < NGRP) load_group(g + 1, nxt);
#pragma unroll
            for (int j = 0; j < GP; ++j) {
                const int pr = g * GP + j;
                if (pr < NP) {
                    const int mm = pr / Q, t = pr % Q;
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int s = 0; s < P; ++s) {
                            int32_t v = cnt[c][mm][s + t];
                            v = and_count(cur[j][0].x, w[c][s][0].x, v);
                            v = and_count(cur[j][0].y, w[c][s][0].y, v);
                            v = and_count(cur[j][0].z, w[c][s][0].z, v);
                            v = and_count(cur[j][0].w, w[c][s][0].w, v);
                            v = and_count(cur[j][1].x, w[c][s][1].x, v);
                            v = and_count(cur[j][1].y, w[c][s][1].y, v);
                            v = and_count(cur[j][1].z, w[c][s][1].z, v);
                            v = and_count(cur[j][1].w, w[c][s][1].w, v);
                            cnt[c][mm][s + t] = v;
                        }
                }
            }
#pragma unroll
            for (int j = 0; j < GP; ++j) { cur[j][0] = nxt[j][0]; cur[j][1] = nxt[j][1]; }
        }
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int n = n0 + c * 256;
        if (n < prm.N) {
            const RowParams pw = prm.wparams[n];
#pragma unroll
            for (int mm = 0; mm < BM; ++mm) {
                const int m = m0 + mm;
                if (m < prm.M) {
                    uint32_t total = 0;
#pragma unroll
                    for (int d = 0; d < ND; ++d) total += (uint32_t)cnt[c][mm][d] << d;   // the 2^(s+t) factors
                    epilogue_store((int32_t)total, 0, 0, prm.K, prm.aparams[m], pw, (size_t)m * prm.N + n, prm.y, prm.acc, prm.rq, m);
                }
            }
        }
    }
}

template <int P, int Q>
static hipError_t launch_pq(const BitSerialParams& prm, hipStream_t s)
{
    if (prm.M >= 8) {
        constexpr int BM = RowsShape<P, Q>::BM, CH = 256 * RowsShape<P, Q>::NC;
        bitserial_rows_kernel<P, Q><<<dim3((unsigned)(((prm.N + CH - 1) / CH) * ((prm.M + BM - 1) / BM))), 256, 0, s>>>(prm);
        return hipGetLastError();
    }
    const unsigned gx = (unsigned)((prm.N + 15) / 16);
    if (prm.M == 1)
        bitserial_kernel<P, Q, 1><<<dim3(gx, 1), 256, 0, s>>>(prm);
    else
        bitserial_kernel<P, Q, 4><<<dim3(gx, (unsigned)((prm.M + 3) / 4)), 256, 0, s>>>(prm);
    return hipGetLastError();
}

template <int P>
static hipError_t launch_p(int q, const BitSerialParams& prm, hipStream_t s)
{
    switch (q) {
        case 1: return launch_pq<P, 1>(prm, s);
        case 2: return launch_pq<P, 2>(prm, s);
        case 3: return launch_pq<P, 3>(prm, s);
        case 4: return launch_pq<P, 4>(prm, s);
        case 5: return launch_pq<P, 5>(prm, s);
        case 6: return launch_pq<P, 6>(prm, s);
        case 7: return launch_pq<P, 7>(prm, s);
        default: return launch_pq<P, 8>(prm, s);
    }
}

hipError_t launch_gemm_bitserial(const GemmArgs& g, const ActLayout& A, const WeightLayout& W, hipStream_t s)
{
    BitSerialParams prm;
    prm.w_planes = (const uint4*)(g.w_blob + W.off_planes);
    prm.a_planes = (const uint4*)(g.act_blob + A.off_planes);
    prm.aparams = (const RowParams*)(g.act_blob + A.off_params);
    prm.wparams = (const RowParams*)(g.w_blob + W.off_params);
    prm.y = g.y;
    prm.acc = g.acc;
    prm.rq = g.rq;
    prm.M = g.M; prm.N = g.N; prm.K = g.K; prm.Kq = W.Kw / 4;
    switch (g.p) {
        case 1: return launch_p<1>(g.q, prm, s);
        case 2: return launch_p<2>(g.q, prm, s);
        case 3: return launch_p<3>(g.q, prm, s);
        case 4: return launch_p<4>(g.q, prm, s);
        case 5: return launch_p<5>(g.q, prm, s);
        case 6: return launch_p<6>(g.q, prm, s);
        case 7: return launch_p<7>(g.q, prm, s);
        default: return launch_p<8>(g.q, prm, s);
    }
}

}  // namespace abq
