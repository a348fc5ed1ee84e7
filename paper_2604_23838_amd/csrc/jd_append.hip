// KV append: the write half of a decode step.  The new token's K and V rows of every active
// request go into slot (L % 16) of the page block_table[b][L / 16], and the request's length
// becomes L + 1, so that the attention call that follows sees the token (seq_lens counts the
// token being decoded).  One block per request: it reads L once, writes the Hkv rows of both
// tensors with 16-byte stores, and only then publishes the new length.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

constexpr int kThreads = 128;

__global__ __launch_bounds__(kThreads) void append_kv_kernel(Params p, const uint16_t* k_new, const uint16_t* v_new,
                                                              uint16_t* k_pages, uint16_t* v_pages, int32_t* seq_lens,
                                                              const int32_t* active)
{
    const int b = blockIdx.x;
    const int L = seq_lens[b];
    const bool on = active ? active[b] != 0 : L > 0;
    __syncthreads();  // every thread holds the old length before anyone publishes the new one
    if (!on || L < 0) return;
    const int pg = L / kPage, slot = L % kPage;
    if (pg >= p.maxp) {
        if (threadIdx.x == 0) atomicOr(&p.header[kHdrBadInput], kBadLength);
        return;
    }
    const int id = p.block_table[static_cast<size_t>(b) * p.maxp + pg];
    if (static_cast<unsigned>(id) >= static_cast<unsigned>(p.NP)) {
        if (threadIdx.x == 0) atomicOr(&p.header[kHdrBadInput], kBadPage);
        return;
    }
    const int chunks_per_row = p.D / 8;  // 16-byte chunks of one token row
    for (int i = threadIdx.x; i < p.Hkv * chunks_per_row; i += kThreads) {
        const int kv = i / chunks_per_row, c = i % chunks_per_row;
        const size_t src = (static_cast<size_t>(b) * p.Hkv + kv) * p.D + c * 8;
        const size_t dst = ((static_cast<size_t>(id) * p.Hkv + kv) * kPage + slot) * p.D + c * 8;
        *reinterpret_cast<uint4*>(k_pages + dst) = *reinterpret_cast<const uint4*>(k_new + src);
        *reinterpret_cast<uint4*>(v_pages + dst) = *reinterpret_cast<const uint4*>(v_new + src);
    }
    if (threadIdx.x == 0) seq_lens[b] = L + 1;
}

}  // namespace

hipError_t launch_append_kv(const Params& p, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pages,
                            uint16_t* v_pages, int32_t* seq_lens, const int32_t* active, hipStream_t stream)
{
    hipLaunchKernelGGL(append_kv_kernel, dim3(p.B), dim3(kThreads), 0, stream, p, k_new, v_new, k_pages, v_pages,
                       seq_lens, active);
    return hipGetLastError();
}

}  // namespace jd
