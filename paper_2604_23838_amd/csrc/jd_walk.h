// Wave-uniform cursor over the (request, kv head, page) units of one wave's span.
#pragma once
#include "jd_internal.h"

namespace jd {

// Read-only data written before the kernel started is fetched through the scalar data
// path when the address is wave-uniform; the constant address space tells the compiler so.
template <typename T>
__device__ inline T uniform_load(const T* ptr)
{
    return *reinterpret_cast<const __attribute__((address_space(4))) T*>(reinterpret_cast<uintptr_t>(ptr));
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// Reductions over the four lanes {l, l^16, l^32, l^48}: the four 16-lane rows of a wave hold the
// four slices of one column of a 16x16 matrix-core result.  A row swap exchanges rows between two
// registers inside the vector ALU (after it, the two registers hold a lane's own value and its
// partner's, in either order), so the chain never waits on the LDS crossbar that a general
// cross-lane shuffle goes through.  max and + are commutative: the result has the shuffle's bits.
__device__ inline float rows_max(float x)
{
    const unsigned xb = __float_as_uint(x);
    const u32x2 a = __builtin_amdgcn_permlane16_swap(xb, xb, false, false);
    const unsigned yb = __float_as_uint(__builtin_fmaxf(__uint_as_float(a.x), __uint_as_float(a.y)));
    const u32x2 b = __builtin_amdgcn_permlane32_swap(yb, yb, false, false);
    return __builtin_fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}

__device__ inline float rows_sum(float x)
{
    const unsigned xb = __float_as_uint(x);
    const u32x2 a = __builtin_amdgcn_permlane16_swap(xb, xb, false, false);
    const unsigned yb = __float_as_uint(__uint_as_float(a.x) + __uint_as_float(a.y));
    const u32x2 b = __builtin_amdgcn_permlane32_swap(yb, yb, false, false);
    return __uint_as_float(b.x) + __uint_as_float(b.y);
}

struct Stream {
    int b;  // request
    int L;  // tokens of the request
    int n;  // pages of the request (clamped to the block-table width)
    int a;  // first page-unit of stream (b, kv) on the work line
};

__device__ inline Stream open_stream(const Params& p, int r, int kv)
{
    Stream s;
    s.b = uniform_load(p.req + r);
    s.L = uniform_load(p.seq_lens + s.b);
    int n = (s.L + kPage - 1) / kPage;
    if (n > p.maxp) { n = p.maxp; s.L = n * kPage; }
    s.n = n;
    s.a = uniform_load(p.cum_pages + s.b) * p.Hkv + kv * n;
    return s;
}

// A physical page id that is safe to dereference; raises the sticky flag otherwise.
__device__ inline int checked_page(const Params& p, int id)
{
    if (static_cast<unsigned>(id) >= static_cast<unsigned>(p.NP)) {
        if ((threadIdx.x & 63) == 0) atomicOr(&p.header[kHdrBadInput], kBadPage);
        id = 0;
    }
    return id;
}

}  // namespace jd
