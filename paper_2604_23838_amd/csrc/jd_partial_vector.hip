// Split-KV partial attention, vector-ALU variant.
//
// One wave streams the pages of its span.  A 16-token page of one kv head is D*32 bytes
// of K and as many of V; each wave-wide load moves 1 KiB with 16 bytes per lane, so a
// token row is spread over D/8 neighbouring lanes and a load covers 64/(D/8) tokens.
// Every lane multiplies its 8 K elements with the matching 8 elements of each of the G
// query heads of the kv head (bf16 pair dot products accumulated in fp32), the partial
// dot products are summed over the row's lanes with DPP adds, and the softmax is kept
// online per lane group: a lane group only ever sees the tokens that fall to it, so no
// traffic between groups is needed until the end of a segment, where the groups' states
// are merged by the log-sum-exp rule.  The probability-weighted V rows are accumulated in
// fp32 in the same lane layout as they were loaded.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
// 16 bytes of K or V, read once per step: a streaming (non-temporal) load
__device__ inline uint4 load_stream16(const uint16_t* ptr)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(ptr));
    return make_uint4(v.x, v.y, v.z, v.w);
}
}  // namespace


namespace {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kWavesPerBlock = 4;
constexpr int kBlocksPerCu = 2;

template <int CTRL>
__device__ inline float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true);
    return x + __builtin_bit_cast(float, y);
}

// Sum over the LPT (8 or 16) neighbouring lanes that hold one token row; every lane gets the total.
template <int LPT>
__device__ inline float row_sum(float x)
{
    x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
    x = dpp_add<0x141>(x);  // row_half_mirror
    if (LPT == 16) x = dpp_add<0x140>(x);  // row_mirror
    return x;
}

__device__ inline float dot8(const uint4& a, const uint4& b)
{
    float d = 0.f;
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.x), __builtin_bit_cast(bf16x2, b.x), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.y), __builtin_bit_cast(bf16x2, b.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.z), __builtin_bit_cast(bf16x2, b.z), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a.w), __builtin_bit_cast(bf16x2, b.w), d, false);
    return d;
}

__device__ inline void unpack8(const uint4& v, float* f)
{
    f[0] = __builtin_bit_cast(float, v.x << 16); f[1] = __builtin_bit_cast(float, v.x & 0xffff0000u);
    f[2] = __builtin_bit_cast(float, v.y << 16); f[3] = __builtin_bit_cast(float, v.y & 0xffff0000u);
    f[4] = __builtin_bit_cast(float, v.z << 16); f[5] = __builtin_bit_cast(float, v.z & 0xffff0000u);
    f[6] = __builtin_bit_cast(float, v.w << 16); f[7] = __builtin_bit_cast(float, v.w & 0xffff0000u);
}

template <int D, int G>
__global__ __launch_bounds__(kWavesPerBlock * 64) void partial_vector_kernel(Params p)
{
    constexpr int LPT = D / 8;       // lanes per token row
    constexpr int TPL = 64 / LPT;    // tokens per wave-wide load
    constexpr int NL = kPage / TPL;  // loads per page and tensor
    constexpr float kNegInf = -__builtin_inff();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int units = uniform_load(p.header + kHdrUnits);
    const int span = uniform_load(p.header + kHdrSpan);
    const int active = uniform_load(p.header + kHdrActive);
    if (wave >= active) return;
    const int u0 = wave * span;
    const int u1 = min(u0 + span, units);
    const i32x4 ws = uniform_load(reinterpret_cast<const i32x4*>(p.wave_start) + wave);
    int r = ws.x, kv = ws.y, pg = ws.z, u = u0;
    const int c = lane % LPT, tg = lane / LPT;
    const size_t page_elems = static_cast<size_t>(p.Hkv) * kPage * D;

    while (u < u1) {
        const Stream st = open_stream(p, r, kv);
        const int pend = min(st.n, pg + (u1 - u));
        const int32_t* bt = p.block_table + static_cast<size_t>(st.b) * p.maxp;
        const size_t lane_off = static_cast<size_t>(kv) * kPage * D + static_cast<size_t>(lane) * 8;

        uint4 qr[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
            qr[g] = *reinterpret_cast<const uint4*>(p.q + (static_cast<size_t>(st.b) * p.Hq + kv * G + g) * D + c * 8);

        float m[G], l[G], acc[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m[g] = kNegInf; l[g] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
        }

        uint4 kr[NL], vr[NL];
        {
            const size_t base = static_cast<size_t>(checked_page(p, uniform_load(bt + pg))) * page_elems + lane_off;
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                kr[j] = load_stream16(p.k_pages + base + j * 512);
                vr[j] = load_stream16(p.v_pages + base + j * 512);
            }
        }
        for (int i = pg; i < pend; ++i) {
            uint4 kn[NL], vn[NL];
            if (i + 1 < pend) {
                const size_t base = static_cast<size_t>(checked_page(p, uniform_load(bt + i + 1))) * page_elems + lane_off;
#pragma unroll
                for (int j = 0; j < NL; ++j) {
                    kn[j] = load_stream16(p.k_pages + base + j * 512);
                    vn[j] = load_stream16(p.v_pages + base + j * 512);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NL; ++j) { kn[j] = kr[j]; vn[j] = vr[j]; }
            }

            float s[NL][G];
#pragma unroll
            for (int j = 0; j < NL; ++j)
#pragma unroll
                for (int g = 0; g < G; ++g)
                    s[j][g] = row_sum<LPT>(dot8(qr[g], kr[j])) * p.scale_log2e;

            const int valid = st.L - i * kPage;  // tokens of this page that exist
            if (valid < kPage) {
#pragma unroll
                for (int j = 0; j < NL; ++j) {
                    if (j * TPL + tg >= valid) {
#pragma unroll
                        for (int g = 0; g < G; ++g) s[j][g] = kNegInf;
                        vr[j] = make_uint4(0, 0, 0, 0);
                    }
                }
            }

            float vf[NL][8];
#pragma unroll
            for (int j = 0; j < NL; ++j) unpack8(vr[j], vf[j]);

#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mx = s[0][g];
#pragma unroll
                for (int j = 1; j < NL; ++j) mx = fmaxf(mx, s[j][g]);
                const float mn = fmaxf(m[g], mx);
                const float ms = (mn == kNegInf) ? 0.f : mn;
                const float alpha = __builtin_amdgcn_exp2f(m[g] - ms);
                m[g] = mn;
                float pj[NL], ps = 0.f;
#pragma unroll
                for (int j = 0; j < NL; ++j) { pj[j] = __builtin_amdgcn_exp2f(s[j][g] - ms); ps += pj[j]; }
                l[g] = l[g] * alpha + ps;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float a = acc[g][e] * alpha;
#pragma unroll
                    for (int j = 0; j < NL; ++j) a = fmaf(pj[j], vf[j][e], a);
                    acc[g][e] = a;
                }
            }
#pragma unroll
            for (int j = 0; j < NL; ++j) { kr[j] = kn[j]; vr[j] = vn[j]; }
        }

        // merge the lane groups' states (each saw a disjoint subset of the tokens)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float M = m[g];
#pragma unroll
            for (int mask = LPT; mask < 64; mask <<= 1) M = fmaxf(M, __shfl_xor(M, mask, 64));
            const float w = __builtin_amdgcn_exp2f(m[g] - M);  // M is finite: a segment holds at least one token
            float lt = l[g] * w;
#pragma unroll
            for (int mask = LPT; mask < 64; mask <<= 1) lt += __shfl_xor(lt, mask, 64);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float a = acc[g][e] * w;
#pragma unroll
                for (int mask = LPT; mask < 64; mask <<= 1) a += __shfl_xor(a, mask, 64);
                acc[g][e] = a;
            }
            m[g] = M; l[g] = lt;
        }

        const bool complete = (pg == 0 && pend == st.n);
        if (tg == 0) {
            if (complete) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float inv = 1.f / l[g];
                    float* o = p.out + (static_cast<size_t>(st.b) * p.Hq + kv * G + g) * D + c * 8;
                    reinterpret_cast<float4*>(o)[0] = make_float4(acc[g][0] * inv, acc[g][1] * inv, acc[g][2] * inv, acc[g][3] * inv);
                    reinterpret_cast<float4*>(o)[1] = make_float4(acc[g][4] * inv, acc[g][5] * inv, acc[g][6] * inv, acc[g][7] * inv);
                }
            } else {
                const int slot = (st.a < u0) ? 0 : 1;
                float* rec = p.partials + static_cast<size_t>(wave * 2 + slot) * record_floats(G, D);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float* o = rec + g * D + c * 8;
                    reinterpret_cast<float4*>(o)[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
                    reinterpret_cast<float4*>(o)[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
                    if (lane == 0) { rec[G * D + g] = m[g]; rec[G * D + G + g] = l[g]; }
                }
            }
        }

        u += pend - pg;
        pg = 0;
        if (++kv == p.Hkv) { kv = 0; ++r; }
    }
}

template <int D, int G>
hipError_t launch(const Params& p, hipStream_t stream)
{
    const int blocks = p.slots / kWavesPerBlock;
    hipLaunchKernelGGL((partial_vector_kernel<D, G>), dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream, p);
    return hipGetLastError();
}

template <int D>
hipError_t dispatch_g(const Params& p, hipStream_t stream)
{
    switch (p.G) {
    case 1: return launch<D, 1>(p, stream);
    case 2: return launch<D, 2>(p, stream);
    case 4: return launch<D, 4>(p, stream);
    case 7: return launch<D, 7>(p, stream);
    case 8: return launch<D, 8>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

int vector_waves_per_cu() { return kWavesPerBlock * kBlocksPerCu; }
int vector_waves_per_block() { return kWavesPerBlock; }

hipError_t launch_partial_vector(const Params& p, hipStream_t stream)
{
    return p.D == 128 ? dispatch_g<128>(p, stream) : dispatch_g<64>(p, stream);
}

}  // namespace jd
