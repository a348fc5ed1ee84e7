// Causal prefill attention over the paged cache (KV recomputation after a migration, new turns of a
// multi-turn rollout): the last q_lens[b] tokens of request b attend to everything before them and to
// each other causally.  Unlike decode this is bound by the matrix cores, not by HBM.
//
// One block serves one (request, kv head, block of query tokens).  Its kNW waves each hold kNT
// tiles of 16 query rows in registers (a row is a (token, query head of the group) pair, the group
// padded to a power of two), and all of them sweep the same K/V pages, which the block stages once
// per page in a shared LDS ring with direct loads (each wave issues its share of a page).  Per page
// and tile the arithmetic is the decode kernel's:
//   S^T[token][row] = K . Q^T (v_mfma_f32_16x16x32_bf16), online softmax in the exp2 domain,
//   O^T[d][row]    += V^T . P^T (v_mfma_f32_16x16x16_bf16, P as bf16 head + bf16 remainder),
// with V read transposed from LDS.  Keys after a row's own position are excluded by selection; pages
// wholly above the block's last position are never fetched, pages wholly above a wave's last
// position are skipped by that wave.  Query blocks of a request are launched heaviest first.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int kNW = 8;   // waves per block
constexpr int kNS = 4;   // ring stages (pages in flight per block)

__device__ inline void dma16(unsigned lds_addr, unsigned lane_off, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Wait until at most `ahead` of this wave's own younger page loads (one instruction each) are in flight.
__device__ inline void wait_pages(int ahead)
{
    if (ahead >= 3) { wait_vmcnt<3>(); return; }
    if (ahead == 2) { wait_vmcnt<2>(); return; }
    if (ahead == 1) { wait_vmcnt<1>(); return; }
    wait_vmcnt<0>();
}

__device__ inline const char* scalar_ptr(const char* ptr)
{
    const uint64_t v = reinterpret_cast<uint64_t>(ptr);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

struct PrefillArgs {
    const uint16_t* q;        // bf16 [TQ, Hq, D]
    const int32_t* q_lens;    // [B]
    const int32_t* q_offsets; // [B]
    float* out;               // fp32 [TQ, Hq, D]
    int32_t gp;               // group size padded to a power of two (query heads per token in a tile)
    int32_t nqb;              // query blocks per (request, kv head)
};

template <int D, int NT>
__global__ __launch_bounds__(kNW * 64) void prefill_kernel(Params p, PrefillArgs a)
{
    constexpr int kRowBytes = D * 2;
    constexpr int kPageBytes = kPage * kRowBytes;
    constexpr int kLoadsPerTensor = kPageBytes / 1024;   // 4 (D=128) or 2 (D=64)
    constexpr int kStageBytes = 2 * kPageBytes;
    constexpr int CPR = kRowBytes / 16, RPL = 1024 / kRowBytes;
    constexpr int kRowShift = D == 128 ? 8 : 7;
    constexpr float kNegInf = -__builtin_inff();
    __shared__ __attribute__((aligned(1024))) char ring[kNS * kStageBytes];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int bkv = blockIdx.x / a.nqb;
    const int b = bkv / p.Hkv, kv = bkv % p.Hkv;
    const int L0 = uniform_load(p.seq_lens + b);
    int n = uniform_load(a.q_lens + b);
    const int npages = min(L0 > 0 ? (L0 + kPage - 1) / kPage : 0, p.maxp);
    const int L = min(L0, npages * kPage);
    if (n > L) n = L;                      // malformed: more new tokens than the cache holds
    const int c = L - n;                   // tokens of context in front of the new ones
    const int tpt = 16 / a.gp;             // tokens per tile
    const int tw = NT * tpt;               // tokens per wave
    const int qb = a.nqb - 1 - static_cast<int>(blockIdx.x % a.nqb);   // heaviest query block first
    const int t0 = qb * tw * kNW;
    if (t0 >= n) return;
    const int qoff = uniform_load(a.q_offsets + b);
    const int tw0 = t0 + w * tw;                       // first token of this wave
    const int blk_last = c + min(n, t0 + tw * kNW) - 1;   // last position any row of the block attends to
    const int wave_last = c + min(n, tw0 + tw) - 1;       // same for this wave (below c + tw0: wave idle)
    const bool wave_live = tw0 < n;
    const int pend = blk_last / kPage + 1;             // pages the block sweeps

    // ---- lane tables (same placement as the decode kernel: rows XOR-swizzled by token) ----
    const int t16 = lane % 16, kg = lane / 16;
    unsigned k_rd[D / 32], v_rd[D / 16];
#pragma unroll
    for (int i = 0; i < D / 32; ++i) k_rd[i] = t16 * kRowBytes + (((4 * i + kg) ^ (t16 & (CPR - 1))) * 16);
    {
        const int row = 4 * kg + t16 / 4, cc = lane % 4;
        const int vs = D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) v_rd[jd] = row * kRowBytes + (((2 * jd + cc / 2) ^ vs) * 16) + (cc % 2) * 8;
    }
    // this wave's share of a page: one 1 KiB direct load (K parts first, then V parts)
    const int my_part = w;
    const bool loader = my_part < 2 * kLoadsPerTensor;
    const int part_j = my_part % kLoadsPerTensor;
    const bool part_is_v = my_part >= kLoadsPerTensor;
    unsigned part_src, part_dst;
    {
        const int t = part_j * RPL + lane / CPR, cp = lane % CPR;
        const int swz = part_is_v ? (D == 128 ? ((t & 7) << 1) : (((t >> 1) & 3) << 1)) : (t & (CPR - 1));
        part_src = t * kRowBytes + ((cp ^ swz) * 16);
        part_dst = (part_is_v ? kPageBytes : 0) + part_j * 1024;
    }
    const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)ring));
    const char* pool = reinterpret_cast<const char*>(part_is_v ? p.v_pages : p.k_pages);
    const int32_t* bt = p.block_table + static_cast<size_t>(b) * p.maxp;

    auto issue = [&](int pg) {
        if (!loader) return;
        const int id = checked_page(p, uniform_load(bt + pg));
        const uint64_t off = static_cast<uint64_t>(static_cast<unsigned>(id * p.Hkv + kv)) << (kRowShift + 4);
        dma16(lds_base + (pg % kNS) * kStageBytes + part_dst, part_src, scalar_ptr(pool + off));
    };

    // ---- queries of this wave: NT tiles of 16 rows, row = (token, head of the group) ----
    bf16x8 qreg[NT][D / 32];
    int row_pos[NT];      // position of this lane's query row in the sequence (c + token)
    bool row_ok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tok = tw0 + nt * tpt + t16 / a.gp, g = t16 % a.gp;
        row_ok[nt] = tok < n && g < p.G;
        const int tk = min(tok, n - 1), gg = min(g, p.G - 1);   // padding rows repeat a real row
        row_pos[nt] = c + tk;
        const uint16_t* src = a.q + (static_cast<size_t>(qoff + tk) * p.Hq + kv * p.G + gg) * D;
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
            qreg[nt][i] = *reinterpret_cast<const bf16x8*>(src + (4 * i + kg) * 8);
    }
    f32x4 acc[NT][D / 16];
    float m[NT], l[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m[nt] = kNegInf;
        l[nt] = 0.f;
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) acc[nt][jd] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the query loads are in before the page ring starts

    // ---- sweep the pages ----
    for (int s = 0; s < kNS - 1 && s < pend; ++s) issue(s);
    for (int pg = 0; pg < pend; ++pg) {
        if (loader) wait_pages(min(kNS - 2, pend - 1 - pg));
        __syncthreads();   // every part of page pg has landed; everybody is done with page pg - 1
        if (pg + kNS - 1 < pend) issue(pg + kNS - 1);
        if (!wave_live || pg * kPage > wave_last) continue;

        lds_char* stage = (lds_char*)ring + (pg % kNS) * kStageBytes;
        bf16x8 kf[D / 32];
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
            kf[i] = *reinterpret_cast<__attribute__((address_space(3))) bf16x8*>(stage + k_rd[i]);
        s16x4 vf[D / 16];
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            vf[jd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                reinterpret_cast<__attribute__((address_space(3))) s16x4*>(stage + kPageBytes + v_rd[jd]));
        const int valid = L - pg * kPage;   // tokens of this page that exist
        if (valid < kPage) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int jd = 0; jd < D / 16; ++jd)
                    if (4 * kg + r >= valid) vf[jd][r] = 0;
        }
        const bool diagonal = pg * kPage + kPage - 1 > c + tw0;   // some row of the wave ends inside or before this page
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < D / 32; ++i) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i], qreg[nt][i], s, 0, 0, 0);
            float sc[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) sc[r] = s[r] * p.scale_log2e;
            if (diagonal) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (pg * kPage + 4 * kg + r > row_pos[nt]) sc[r] = kNegInf;   // keys after the row's own position
            }
            float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float mn = fmaxf(m[nt], mx);   // finite from the first page on: position 0 is visible to every row
            const float alpha = __builtin_amdgcn_exp2f(m[nt] - mn);
            float pr[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) pr[r] = __builtin_amdgcn_exp2f(sc[r] - mn);
            l[nt] = l[nt] * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
            if (__builtin_amdgcn_ballot_w64(mn > m[nt]) != 0) {
#pragma unroll
                for (int jd = 0; jd < D / 16; ++jd)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[nt][jd][r] *= alpha;
            }
            m[nt] = mn;
            s16x4 ph, pl;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const __bf16 hi = static_cast<__bf16>(pr[r]);
                const __bf16 lo = static_cast<__bf16>(pr[r] - static_cast<float>(hi));
                ph[r] = __builtin_bit_cast(short, hi);
                pl[r] = __builtin_bit_cast(short, lo);
            }
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd) {
                acc[nt][jd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[jd], ph, acc[nt][jd], 0, 0, 0);
                acc[nt][jd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[jd], pl, acc[nt][jd], 0, 0, 0);
            }
        }
    }

    // ---- normalise and store ----
    if (!wave_live) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        float lt = l[nt];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (!row_ok[nt]) continue;
        const int tok = tw0 + nt * tpt + t16 / a.gp, g = t16 % a.gp;
        const float inv = 1.f / lt;
        float* o = a.out + (static_cast<size_t>(qoff + tok) * p.Hq + kv * p.G + g) * D + 4 * kg;
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            *reinterpret_cast<float4*>(o + 16 * jd) =
                make_float4(acc[nt][jd][0] * inv, acc[nt][jd][1] * inv, acc[nt][jd][2] * inv, acc[nt][jd][3] * inv);
    }
}

}  // namespace

// Tokens of one request a block covers, for a group size G.
int prefill_block_tokens(int G, int D)
{
    int gp = 1;
    while (gp < G) gp *= 2;
    const int nt = D == 128 ? 2 : 4;
    return kNW * nt * (16 / gp);
}

hipError_t launch_prefill(const Params& p, const uint16_t* q, const int32_t* q_lens, const int32_t* q_offsets,
                          int max_q_len, float* out, hipStream_t stream)
{
    PrefillArgs a;
    a.q = q; a.q_lens = q_lens; a.q_offsets = q_offsets; a.out = out;
    a.gp = 1;
    while (a.gp < p.G) a.gp *= 2;
    const int qb = prefill_block_tokens(p.G, p.D);
    a.nqb = (max_q_len + qb - 1) / qb;
    if (a.nqb == 0 || p.B == 0) return hipSuccess;
    if (static_cast<int64_t>(a.nqb) * p.B * p.Hkv > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(a.nqb * p.B * p.Hkv));
    if (p.D == 128)
        hipLaunchKernelGGL((prefill_kernel<128, 2>), grid, dim3(kNW * 64), 0, stream, p, a);
    else
        hipLaunchKernelGGL((prefill_kernel<64, 4>), grid, dim3(kNW * 64), 0, stream, p, a);
    return hipGetLastError();
}

}  // namespace jd
