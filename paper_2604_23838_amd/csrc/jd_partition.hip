// Work partitioner: turns the ragged seq_lens of one decode step into equal shares of
// KV pages, one share per wave of the split-KV partial pass.
//
// The imbalance it answers is the one the paper describes for rollout (Motivation,
// "Varied Decoding Lengths": a few long sequences dominate and the effective batch
// shrinks; Sub-stage Merging migrates such stragglers between workers).  Inside one GPU
// the same imbalance is removed by cutting the step's work, not its requests: all
// (request, kv head, page) units are laid on one line, request-major then kv head then
// page, and the line is cut into `active` spans of `span` units.  A span may end in the
// middle of a sequence (the sequence is then split over consecutive waves and merged by
// the combine pass) and may hold several short sequences.  Every wave gets the same
// number of pages to stream (+-1 span rounding), whatever the length distribution.
#include "jd_internal.h"

namespace jd {

namespace {

constexpr int kThreads = 1024;

__device__ inline int2 block_scan_inclusive(int2 v, int2* warp_tot, int tid)
{
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int a = __shfl_up(v.x, d, 64), b = __shfl_up(v.y, d, 64);
        if (lane >= d) { v.x += a; v.y += b; }
    }
    if (lane == 63) warp_tot[wv] = v;
    __syncthreads();
    int2 add = make_int2(0, 0);
    for (int i = 0; i < wv; ++i) { add.x += warp_tot[i].x; add.y += warp_tot[i].y; }
    v.x += add.x; v.y += add.y;
    __syncthreads();
    return v;
}

__global__ __launch_bounds__(kThreads) void partition_kernel(Params p)
{
    __shared__ int2 warp_tot[kThreads / 64];
    __shared__ int2 carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = make_int2(0, 0);
    __syncthreads();

    // 1. pages per request, their exclusive prefix, and the compacted list of non-empty requests
    for (int base = 0; base < p.B; base += kThreads) {
        const int b = base + tid;
        int n = 0;
        if (b < p.B) {
            const int L = p.seq_lens[b];
            n = L > 0 ? (L + kPage - 1) / kPage : 0;
            if (n > p.maxp) { n = p.maxp; atomicOr(&p.header[kHdrBadInput], kBadLength); }
        }
        const int2 c = carry;
        int2 inc = block_scan_inclusive(make_int2(n, n > 0 ? 1 : 0), warp_tot, tid);
        if (b < p.B) {
            p.cum_pages[b] = c.x + inc.x - n;
            const int r = c.y + inc.y - (n > 0 ? 1 : 0);
            p.rank[b] = r;
            if (n > 0) p.req[r] = b;
        }
        __syncthreads();
        if (tid == kThreads - 1) carry = make_int2(c.x + inc.x, c.y + inc.y);
        __syncthreads();
    }
    const int total_pages = carry.x;
    const int units = total_pages * p.Hkv;
    const int span = span_for(units, p.slots);
    const int active = (units + span - 1) / span;
    if (tid == 0) {
        p.cum_pages[p.B] = total_pages;
        p.header[kHdrUnits] = units;
        p.header[kHdrSpan] = span;
        p.header[kHdrActive] = active;
        p.header[kHdrSlots] = p.slots;
        p.header[kHdrNonEmpty] = carry.y;
        p.header[kHdrGroup] = 1;
    }
    // cum_pages was written by other threads of this block: make it visible before searching it
    __threadfence();
    __syncthreads();

    // 2. first unit of every active wave: the last request whose first unit is <= w*span
    for (int w = tid; w < active; w += kThreads) {
        const int u = w * span;
        int lo = 0, hi = p.B - 1;  // invariant: cum[lo]*Hkv <= u
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            const int c = __hip_atomic_load(&p.cum_pages[mid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (c * p.Hkv <= u) lo = mid; else hi = mid - 1;
        }
        const int c0 = __hip_atomic_load(&p.cum_pages[lo], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int c1 = __hip_atomic_load(&p.cum_pages[lo + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int n = c1 - c0;
        const int within = u - c0 * p.Hkv;
        int4 ws;
        ws.x = __hip_atomic_load(&p.rank[lo], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ws.y = within / n;
        ws.z = within % n;
        ws.w = lo;  // the request id itself, for inspection
        reinterpret_cast<int4*>(p.wave_start)[w] = ws;
    }
}

}  // namespace

hipError_t launch_partition(const Params& p, hipStream_t stream)
{
    hipLaunchKernelGGL(partition_kernel, dim3(1), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace jd
