// Causal prefill attention over the paged cache (KV recomputation after a migration, new turns of a
// multi-turn rollout): the last q_lens[b] tokens of request b attend to everything before them and to
// each other causally.  Unlike decode this is bound by the matrix cores, not by HBM.
//
// One block serves one (request, kv head, block of query tokens).  Its kNW waves each hold kNT
// tiles of 16 query rows in registers (a row is a (token, query head of the group) pair, the group
// padded to a power of two), and all of them sweep the same K/V pages, which the block stages in a
// shared LDS ring of 64-key stages with direct loads (each wave issues its share of a stage; one
// barrier and one softmax update per stage).  Per page and tile the arithmetic is the decode kernel's:
//   S^T[token][row] = K . Q^T (v_mfma_f32_16x16x32_bf16), online softmax in the exp2 domain,
//   O^T[d][row]    += V^T . P^T (v_mfma_f32_16x16x32_bf16 over two pages at once, P as bf16 head + bf16 remainder),
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
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int kNW = 4;   // waves per block (two blocks share a compute unit and drift out of step, so that one's
                         // matrix work overlaps the other's softmax arithmetic)
constexpr int kSP = 4;   // pages (16 keys each) per ring stage: one barrier and one softmax update per 64 keys
constexpr int kNS = 2;   // ring stages

__device__ inline void dma16(unsigned lds_addr, unsigned lane_off, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

template <typename T>
__device__ inline __attribute__((address_space(3))) T* lds_ptr(unsigned addr)
{
    return (__attribute__((address_space(3))) T*)(uintptr_t)addr;
}

// max of three floats without the canonicalising moves fmaxf brings (inputs are never signalling NaNs here)
__device__ inline float max3(float a, float b, float c)
{
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Wait until only the loads of `ahead` younger stages (N instructions of this wave each) are in flight.
template <int N>
__device__ inline void wait_stages(int ahead)
{
    static_assert(kNS <= 4, "one case per possible number of younger stages");
    if (ahead >= 2) { wait_vmcnt<2 * N>(); return; }
    if (ahead == 1) { wait_vmcnt<N>(); return; }
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
__global__ __launch_bounds__(kNW * 64, 2) void prefill_kernel(Params p, PrefillArgs a)
{
    constexpr int kRowBytes = D * 2;
    constexpr int kPageBytes = kPage * kRowBytes;
    constexpr int kPartsPerPage = 2 * kPageBytes / 1024;      // 1 KiB direct loads per page: 8 (D=128) or 4 (D=64)
    constexpr int kSlotBytes = 2 * kPageBytes;                // K then V of one page
    constexpr int kStageBytes = kSP * kSlotBytes;
    constexpr int kHalfParts = kPartsPerPage / 2;             // parts of one tensor's page
    constexpr int kLoadsPerWave = kSP * kPartsPerPage / kNW;  // direct loads a wave issues per stage (a K and a V part each time)
    constexpr int kPageStride = kNW / kHalfParts;             // pages between two part pairs of a wave
    static_assert(kNW % kHalfParts == 0 && kLoadsPerWave >= 2 && kLoadsPerWave % 2 == 0, "a wave keeps one part index");
    constexpr int CPR = kRowBytes / 16, RPL = 1024 / kRowBytes;
    constexpr int kRowShift = D == 128 ? 8 : 7;
    constexpr float kNegInf = -__builtin_inff();
    static_assert(kLoadsPerWave * (kNS - 1) <= 63, "vmcnt is a 6-bit counter");
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
    const int tw0 = t0 + w * tw;                          // first token of this wave
    const int blk_last = c + min(n, t0 + tw * kNW) - 1;   // last position any row of the block attends to
    const int wave_last = c + min(n, tw0 + tw) - 1;       // same for this wave
    const bool wave_live = tw0 < n;
    const int pend = blk_last / kPage + 1;                // pages the block sweeps (<= npages)
    const int nsteps = (pend + kSP - 1) / kSP;            // stages of kSP pages

    // ---- lane tables (same placement as the decode kernel: rows XOR-swizzled by token) ----
    const int t16 = lane % 16, kg = lane / 16;
    unsigned k_rd[D / 32], v_rd[D / 16];
#pragma unroll
    for (int i = 0; i < D / 32; ++i) k_rd[i] = t16 * kRowBytes + (((4 * i + kg) ^ (t16 & (CPR - 1))) * 16);
    {
        const int row = 4 * kg + t16 / 4, cc = lane % 4;
        const int vs = D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            v_rd[jd] = kPageBytes + row * kRowBytes + (((2 * jd + cc / 2) ^ vs) * 16) + (cc % 2) * 8;
    }
    // this wave's share of a stage: the same 1 KiB part of K and of V of every kPageStride-th page,
    // starting at page w / kHalfParts
    const int part_j = w % kHalfParts;
    const int first_page = w / kHalfParts;
    unsigned src_k, src_v;
    {
        const int t = part_j * RPL + lane / CPR, cp = lane % CPR;
        src_k = t * kRowBytes + ((cp ^ (t & (CPR - 1))) * 16);
        src_v = t * kRowBytes + ((cp ^ (D == 128 ? ((t & 7) << 1) : (((t >> 1) & 3) << 1))) * 16);
    }
    const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)ring));
    const char* kpool = reinterpret_cast<const char*>(p.k_pages);
    const char* vpool = reinterpret_cast<const char*>(p.v_pages);
    const int32_t* bt = p.block_table + static_cast<size_t>(b) * p.maxp;

    // Every wave issues the same number of loads for every stage: slots past the block's last page
    // get that last page again (never read uninitialised memory, never count loads per wave).
    auto issue = [&](int st) {
#pragma unroll
        for (int i = 0; i < kLoadsPerWave / 2; ++i) {
            const int j = first_page + kPageStride * i;
            const int pg = min(st * kSP + j, pend - 1);
            const int id = checked_page(p, uniform_load(bt + pg));
            const uint64_t off = static_cast<uint64_t>(static_cast<unsigned>(id * p.Hkv + kv)) << (kRowShift + 4);
            const unsigned dst = lds_base + (st % kNS) * kStageBytes + j * kSlotBytes + part_j * 1024;
            dma16(dst, src_k, scalar_ptr(kpool + off));
            dma16(dst + kPageBytes, src_v, scalar_ptr(vpool + off));
        }
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
    f32x4 lacc[NT];       // softmax denominators (every register of a lane holds its row's)
    float m[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m[nt] = kNegInf;
        lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) acc[nt][jd] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the query loads are in before the page ring starts

    // ---- sweep the stages ----
    for (int s = 0; s < kNS - 1 && s < nsteps; ++s) issue(s);
    for (int st = 0; st < nsteps; ++st) {
        wait_stages<kLoadsPerWave>(min(kNS - 2, nsteps - 1 - st));
        __syncthreads();   // every part of stage st has landed; everybody is done with stage st - 1
        if (st + kNS - 1 < nsteps) issue(st + kNS - 1);
        const int key0 = st * kSP * kPage;
        if (!wave_live || key0 > wave_last) continue;

        const unsigned stage = lds_base + (st % kNS) * kStageBytes;
        // S^T of every tile against the stage's keys (raw dot products; the scale is applied inside the exponent)
        f32x4 sc[NT][kSP];
        {
            unsigned ka[D / 32];
#pragma unroll
            for (int i = 0; i < D / 32; ++i) {
                ka[i] = stage + k_rd[i];
                asm volatile("" : "+v"(ka[i]));   // one add per stage; the page offset rides in the instruction
            }
#pragma unroll
            for (int j = 0; j < kSP; ++j) {
                bf16x8 kf[D / 32];
#pragma unroll
                for (int i = 0; i < D / 32; ++i) kf[i] = *lds_ptr<bf16x8>(ka[i] + j * kSlotBytes);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < D / 32; ++i)
                        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i], qreg[nt][i], s, 0, 0, 0);
                    sc[nt][j] = s;
                }
            }
        }
        // keys after a row's own position (and the slots past the sequence's end) are excluded by selection
        if (key0 + kSP * kPage - 1 > c + tw0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < kSP; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (key0 + j * kPage + 4 * kg + r > row_pos[nt]) sc[nt][j][r] = kNegInf;
        }
        // online softmax per tile (the scale is positive, so the maximum can be taken before scaling);
        // probabilities as bf16 head + bf16 remainder, two pages side by side: the 8 keys a lane holds
        // of a page pair are one k-group of a 32-deep contraction
        u32x4 ph[NT][kSP / 2], pl[NT][kSP / 2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float mx = max3(sc[nt][0][0], sc[nt][0][1], sc[nt][0][2]);
#pragma unroll
            for (int e = 3; e < 4 * kSP; e += 2)   // two more values per instruction; the odd one out pairs with itself
                mx = max3(mx, sc[nt][e / 4][e % 4], e + 1 < 4 * kSP ? sc[nt][(e + 1) / 4][(e + 1) % 4] : mx);
            mx = max3(mx, __shfl_xor(mx, 16, 64), mx);
            mx = max3(mx, __shfl_xor(mx, 32, 64), mx);
            const float mn = max3(m[nt], mx * p.scale_log2e, m[nt]);   // finite from the first stage on: position 0 is visible to every row
            const float alpha = __builtin_amdgcn_exp2f(m[nt] - mn);
#pragma unroll
            for (int j = 0; j < kSP; ++j)
#pragma unroll
                for (int r = 0; r < 4; r += 2) {
                    f32x2 pr;
                    pr[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[nt][j][r], p.scale_log2e, -mn));
                    pr[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[nt][j][r + 1], p.scale_log2e, -mn));
                    const bf16x2 hi = __builtin_convertvector(pr, bf16x2);
                    const bf16x2 lo = __builtin_convertvector(pr - __builtin_convertvector(hi, f32x2), bf16x2);
                    ph[nt][j / 2][2 * (j % 2) + r / 2] = __builtin_bit_cast(uint32_t, hi);
                    pl[nt][j / 2][2 * (j % 2) + r / 2] = __builtin_bit_cast(uint32_t, lo);
                }
            if (__builtin_amdgcn_ballot_w64(mn > m[nt]) != 0) {   // nobody's maximum moved: alpha is exactly 1 everywhere
                lacc[nt] *= alpha;
#pragma unroll
                for (int jd = 0; jd < D / 16; ++jd) acc[nt][jd] *= alpha;
            }
            m[nt] = mn;
        }
        // O^T += V^T P^T, 32 keys per instruction; the row sums of P come from the same unit (V^T replaced by ones)
        unsigned va_[D / 16];
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) {
            va_[jd] = stage + v_rd[jd];
            asm volatile("" : "+v"(va_[jd]));
        }
        const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
#pragma unroll
        for (int jp = 0; jp < kSP / 2; ++jp) {
            const bool ragged = L - (key0 + (2 * jp + 1) * kPage) < kPage;   // the pair reaches past the sequence's end
            bf16x8 bh[NT], bl[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                bh[nt] = __builtin_bit_cast(bf16x8, ph[nt][jp]);
                bl[nt] = __builtin_bit_cast(bf16x8, pl[nt][jp]);
                lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bh[nt], lacc[nt], 0, 0, 0);
                lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bl[nt], lacc[nt], 0, 0, 0);
            }
#pragma unroll
            for (int q4 = 0; q4 < D / 64; ++q4) {   // four 16-wide slices of the head dimension at a time
                u32x4 vf[4];   // per lane: 4 keys of page 2 jp, then 4 keys of page 2 jp + 1
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            lds_ptr<s16x4>(va_[4 * q4 + e] + (2 * jp + h) * kSlotBytes)));
                        vf[e][2 * h] = t[0];
                        vf[e][2 * h + 1] = t[1];
                    }
                if (ragged) {
                    uint32_t keep[2][2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int valid = L - (key0 + (2 * jp + h) * kPage);   // tokens of this page that exist (<= 0: a repeated page)
                        keep[h][0] = (4 * kg + 0 < valid ? 0x0000ffffu : 0u) | (4 * kg + 1 < valid ? 0xffff0000u : 0u);
                        keep[h][1] = (4 * kg + 2 < valid ? 0x0000ffffu : 0u) | (4 * kg + 3 < valid ? 0xffff0000u : 0u);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        vf[e][0] &= keep[0][0]; vf[e][1] &= keep[0][1];
                        vf[e][2] &= keep[1][0]; vf[e][3] &= keep[1][1];
                    }
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bf16x8 va = __builtin_bit_cast(bf16x8, vf[e]);
                        acc[nt][4 * q4 + e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, bh[nt], acc[nt][4 * q4 + e], 0, 0, 0);
                        acc[nt][4 * q4 + e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, bl[nt], acc[nt][4 * q4 + e], 0, 0, 0);
                    }
            }
        }
    }

    // ---- normalise and store ----
    if (!wave_live) return;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float lt = lacc[nt][0];
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
