// Log-sum-exp combine: merges the split-KV partial states of every sequence that was cut
// over several waves into its output rows, and writes zero rows for empty requests.
//
//   M = max_i m_i,   out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i
//
// (scores are kept in the exp2 domain by the partial pass).  Which waves hold pieces of
// stream (b, kv) follows from the partition alone: the stream owns page-units [a, a+n)
// of the work line, wave w owns [w*span, (w+1)*span), so the pieces sit in waves
// a/span .. (a+n-1)/span; a piece that starts before its wave's span is that wave's
// record 0, otherwise record 1.  Streams that fit one wave were written by the partial
// pass directly and are left alone.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

constexpr int kWavesPerBlock = 4;

template <int D>
__global__ __launch_bounds__(kWavesPerBlock * 64) void combine_kernel(Params p)
{
    constexpr int EPL = D / 64;  // output elements per lane
    const int lane = threadIdx.x & 63;
    const int row = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (row >= p.B * p.Hq) return;
    const int b = row / p.Hq, h = row % p.Hq;
    const int kv = h / p.G, g = h % p.G;
    float* o = p.out + static_cast<size_t>(row) * D + lane * EPL;

    const int n = uniform_load(p.cum_pages + b + 1) - uniform_load(p.cum_pages + b);
    if (n == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[e] = 0.f;
        return;
    }
    const int span = uniform_load(p.header + kHdrSpan);
    const int a = uniform_load(p.cum_pages + b) * p.Hkv + kv * n;
    const int w0 = a / span, w1 = (a + n - 1) / span;
    if (w0 == w1) return;

    const int rec_floats = record_floats(p.G, D);
    float M = -__builtin_inff();
    for (int w = w0; w <= w1; ++w) {
        const int slot = (a < w * span) ? 0 : 1;
        const float* rec = p.partials + static_cast<size_t>(w * 2 + slot) * rec_floats;
        M = fmaxf(M, rec[p.G * D + g]);
    }
    float den = 0.f, num[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) num[e] = 0.f;
    for (int w = w0; w <= w1; ++w) {
        const int slot = (a < w * span) ? 0 : 1;
        const float* rec = p.partials + static_cast<size_t>(w * 2 + slot) * rec_floats;
        const float sc = __builtin_amdgcn_exp2f(rec[p.G * D + g] - M);
        den = fmaf(sc, rec[p.G * D + p.G + g], den);
#pragma unroll
        for (int e = 0; e < EPL; ++e) num[e] = fmaf(sc, rec[g * D + lane * EPL + e], num[e]);
    }
    const float inv = 1.f / den;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = num[e] * inv;
}

}  // namespace

hipError_t launch_combine(const Params& p, hipStream_t stream)
{
    const int rows = p.B * p.Hq;
    const int blocks = (rows + kWavesPerBlock - 1) / kWavesPerBlock;
    if (p.D == 128)
        hipLaunchKernelGGL(combine_kernel<128>, dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream, p);
    else
        hipLaunchKernelGGL(combine_kernel<64>, dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace jd
