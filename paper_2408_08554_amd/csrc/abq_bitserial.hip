// The paper's decomposition taken literally (Appendix B): for every weight plane s and
// activation plane t, AND the 1-bit rows and count the set bits along K; the counts are
// weighted by 2^(s+t) and summed ("Bit Reduction", Sec. 3.4 step 5).  gfx950 has no 1-bit
// matrix instruction, so BMMA becomes wavefront-wide v_and + v_bcnt (popcount-accumulate) on
// 128-bit loads of the [bits][rows][K] planes.  Counts of equal s+t share one accumulator,
// which leaves p+q-1 accumulators per output instead of p*q.
//
// Mapping: a wave owns 4 output channels, 16 lanes per channel; each lane walks the 128-bit
// quads of its channel's planes, then the 16 partial sums are added with in-row shuffles.
// MB rows of A are processed per pass over the weights.
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

template <int P, int Q>
static hipError_t launch_pq(const BitSerialParams& prm, hipStream_t s)
{
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
