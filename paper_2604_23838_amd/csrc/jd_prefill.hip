// Causal prefill attention over the paged cache (KV recomputation after a migration, new turns of a
// multi-turn rollout): the last q_lens[b] tokens of request b attend to everything before them and to
// each other causally.  Unlike decode this is bound by the matrix cores, not by HBM.
//
// One block of kNW waves serves one (request, kv head, block of query tokens); two blocks share a
// compute unit, so that one's matrix work runs while the other's softmax arithmetic does.  Each wave
// holds NT tiles of 16 query rows in registers (row r of a request's kv head is query head r % G of new
// token r / G, packed densely whatever G is), and all waves sweep the same K/V pages, which the block stages in
// shared LDS rings of 64-key stages with direct loads (each wave issues its share of a stage; one
// barrier and one softmax update per stage).  The block table reaches LDS the same way, a window of
// 64 page ids at a time, so no round waits for a table read.  Per stage and tile:
//   S^T[key][row]  = K . Q^T (v_mfma_f32_16x16x32_bf16), online softmax in the exp2 domain,
//   O^T[d][row]   += V^T . P^T (same instruction over two pages at once: the 8 keys a lane holds of a
//                    page pair are one k-group of the 32-deep contraction; P as bf16 head + bf16 remainder),
//   l[row]        += 1 . P^T   (row sums from the matrix unit, V^T replaced by ones),
// with V read transposed from LDS.  Keys after a row's own position are excluded by selection (only
// in the rounds that reach the diagonal); pages wholly above the block's last position are never
// fetched.  Requests are dispatched by decreasing work (a small ranking kernel runs first), the query
// blocks of a request heaviest first.
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

constexpr int kNW = 4;    // waves per block; two blocks share a compute unit
constexpr int kDist = 1;  // rounds between a stage's loads and its use
constexpr int kPrefillBlockRows = kNW * 2 * 16;   // query rows (token x head of the group) per block: 2 tiles of 16 per wave

__device__ inline void dma16(unsigned lds_addr, unsigned lane_off, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

__device__ inline void dma4(unsigned lds_addr, unsigned lane_off, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

template <typename T>
__device__ inline __attribute__((address_space(3))) T* lds_ptr(unsigned addr)
{
    return (__attribute__((address_space(3))) T*)(uintptr_t)addr;
}

// Row maximum of the scores a lane group holds.  Plain compiler-visible maxima on purpose: the compiler
// places the wait states that a read of a fresh matrix result needs, which it cannot do for an
// instruction hidden in inline assembly (a hand-written v_max3 here once read scores before the matrix
// unit had written them: right to rounding, since only the reference maximum moved, but not repeatable).
template <int N>
__device__ inline float row_max(const f32x4 (&s)[N])
{
    float mx = __builtin_fmaxf(__builtin_fmaxf(s[0][0], s[0][1]), s[0][2]);
#pragma unroll
    for (int e = 3; e < 4 * N; e += 2) {
        const float x = s[e / 4][e % 4];
        mx = e + 1 < 4 * N ? __builtin_fmaxf(__builtin_fmaxf(mx, x), s[(e + 1) / 4][(e + 1) % 4]) : __builtin_fmaxf(mx, x);
    }
    mx = rows_max(mx);   // the lanes of the other key groups hold the rest of the row
    return mx;
}

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
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
    int32_t tq;               // rows of q and out
    int32_t nqb;              // query blocks per (request, kv head)
    const int32_t* order;     // [B] requests by decreasing work
};

// Requests by decreasing work (query-key pairs under the causal mask), so that the blocks of the heaviest
// request are dispatched first and the launch ends on light ones.  Rank by counting: ties go to the lower
// index, so the ranks are a permutation whatever the lengths hold.
__global__ __launch_bounds__(256) void prefill_order_kernel(Params p, const int32_t* q_lens, int32_t* order)
{
    __shared__ long long tile[256];
    const int b = blockIdx.x * 256 + threadIdx.x;
    auto work = [&](int i) -> long long {
        const int L0 = p.seq_lens[i];
        const long long L = min(max(L0, 0), p.maxp * kPage);
        const long long n = min(static_cast<long long>(max(q_lens[i], 0)), L);
        return n * (2 * (L - n) + n + 1);
    };
    const long long mine = b < p.B ? work(b) : -1;
    int rank = 0;
    for (int base = 0; base < p.B; base += 256) {
        __syncthreads();
        tile[threadIdx.x] = base + threadIdx.x < p.B ? work(base + threadIdx.x) : -1;
        __syncthreads();
        const int m = min(256, p.B - base);
        for (int i = 0; i < m; ++i) {
            const long long o = tile[i];
            rank += (o > mine || (o == mine && base + i < b)) ? 1 : 0;
        }
    }
    if (b < p.B) order[rank] = b;
}

template <bool B>
struct Flag { static constexpr bool value = B; };

template <int D, int NT>
__global__ __launch_bounds__(kNW * 64, 2) void prefill_kernel(Params p, PrefillArgs a)
{
    constexpr int kSP = 4;   // pages (16 keys each) per ring stage: one barrier and one softmax update per 64 keys
    constexpr int kRowBytes = D * 2;
    constexpr int kPageBytes = kPage * kRowBytes;
    constexpr int kStageBytes = kSP * kPageBytes;             // one tensor's share of a stage
    constexpr int kHalfParts = kPageBytes / 1024;             // 1 KiB direct loads per page and tensor: 4 (D=128) or 2 (D=64)
    constexpr int kLoadsPerWave = kSP * kHalfParts / kNW;     // direct loads a wave issues per stage and tensor
    constexpr int kPageStride = kNW / kHalfParts;             // pages between two parts of a wave
    static_assert(kNW % kHalfParts == 0 && kLoadsPerWave >= 1, "a wave keeps one part index");
    constexpr int CPR = kRowBytes / 16, RPL = 1024 / kRowBytes;
    constexpr int kRowShift = D == 128 ? 8 : 7;
    constexpr float kNegInf = -__builtin_inff();
    // K and V rings of kDist + 1 stages: the loads of a stage are issued kDist rounds before its round
    constexpr int kSlots = kDist + 1;
    constexpr int kInFlight = (kDist - 1) * 2 * kLoadsPerWave;   // a wave's loads of the last kDist - 1 rounds
    static_assert(kDist * 2 * kLoadsPerWave <= 63, "vmcnt is a 6-bit counter");
    __shared__ __attribute__((aligned(1024))) char kring[kSlots * kStageBytes];
    __shared__ __attribute__((aligned(1024))) char vring[kSlots * kStageBytes];
    // page ids of the request, two windows of 64 pages: page q sits at idring[q % 128]
    __shared__ __attribute__((aligned(256))) int32_t idring[128];
    constexpr int kWin = 64 / kSP;   // stages per window

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int bkv = blockIdx.x / a.nqb;
    const int b = min(max(uniform_load(a.order + bkv / p.Hkv), 0), p.B - 1), kv = bkv % p.Hkv;
    const int L0 = uniform_load(p.seq_lens + b);
    int n = uniform_load(a.q_lens + b);
    const int npages = min(L0 > 0 ? (L0 + kPage - 1) / kPage : 0, p.maxp);
    const int L = min(L0, npages * kPage);
    if (n > L) n = L;                      // malformed: more new tokens than the cache holds
    const int c = L - n;                   // tokens of context in front of the new ones
    // query rows of the request: row r is head r % G of new token r / G (no padding of the group)
    constexpr int kWaveRows = NT * 16;
    static_assert(kNW * kWaveRows == kPrefillBlockRows, "the launch and the kernel agree on the rows of a block");
    const int nrows = n * p.G;
    const int qb = a.nqb - 1 - static_cast<int>(blockIdx.x % a.nqb);   // heaviest query block first
    const int r0 = qb * kPrefillBlockRows;
    if (r0 >= nrows) return;
    const int qoff = uniform_load(a.q_offsets + b);
    // the rows of the request's new tokens lie inside q and out, or the request is skipped and flagged
    if (qoff < 0 || static_cast<int64_t>(qoff) + n > a.tq) {
        if (threadIdx.x == 0 && (p.header[kHdrBadInput] & kBadQueryRows) == 0) atomicOr(&p.header[kHdrBadInput], kBadQueryRows);
        return;
    }
    const int rw0 = min(r0 + w * kWaveRows, nrows - 1);   // first row of this wave (a wave past the end repeats the last row)
    const bool wave_live = r0 + w * kWaveRows < nrows;
    const int tw0 = rw0 / p.G;                            // the token of that row
    const int blk_last = c + (min(nrows, r0 + kPrefillBlockRows) - 1) / p.G;   // last position any row of the block attends to
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
        for (int jd = 0; jd < D / 16; ++jd) v_rd[jd] = row * kRowBytes + (((2 * jd + cc / 2) ^ vs) * 16) + (cc % 2) * 8;
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
    const unsigned k_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)kring));
    const unsigned v_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)vring));
    const char* kpool = reinterpret_cast<const char*>(p.k_pages);
    const char* vpool = reinterpret_cast<const char*>(p.v_pages);
    const int32_t* bt = p.block_table + static_cast<size_t>(b) * p.maxp;

    // Every wave issues the same loads for every stage: slots past the block's last page get that
    // last page again (no uninitialised memory is ever multiplied).  The block table reaches LDS through
    // the same direct loads, a window of 64 page ids at a time and long before they are needed, so
    // that no round waits for a table read; wave 0 refills the window everybody has left.
    const unsigned id_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char*)idring));
    auto fill_ids = [&](int win) __attribute__((always_inline)) {
        if (w != 0) return;
        const int pg = min(win * 64 + lane, pend - 1);
        dma4(id_base + (win % 2) * 256, static_cast<unsigned>(pg) * 4u, bt);
    };
    auto load_ids = [&](int st, int (&ids)[kLoadsPerWave]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i)
            ids[i] = __builtin_amdgcn_readfirstlane(idring[(st * kSP + first_page + kPageStride * i) & 127]);
    };
    bool bad_seen = false;
    auto issue = [&](auto always, int st, int (&ids)[kLoadsPerWave]) __attribute__((always_inline)) {
        if (!decltype(always)::value && st >= nsteps) return;
        bool bad = false;
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            const int j = first_page + kPageStride * i;
            const bool ok = static_cast<unsigned>(ids[i]) < static_cast<unsigned>(p.NP);
            bad |= !ok;
            // a page id out of range reads page 0 and raises the sticky flag
            const unsigned id = __builtin_amdgcn_readfirstlane(ok ? static_cast<unsigned>(ids[i]) : 0u);
            const unsigned row = id * static_cast<unsigned>(p.Hkv) + static_cast<unsigned>(kv);
            const uint64_t off = static_cast<uint64_t>(row) << (kRowShift + 4);
            const unsigned dst = __builtin_amdgcn_readfirstlane((st % kSlots) * kStageBytes + j * kPageBytes + part_j * 1024);
            dma16(k_base + dst, src_k, scalar_ptr(kpool + off));
            dma16(v_base + dst, src_v, scalar_ptr(vpool + off));
        }
        bad_seen |= bad;
    };
    int ids[kLoadsPerWave];   // page ids of the next stage to issue

    // ---- queries of this wave: NT tiles of 16 rows, row = (token, head of the group) ----
    bf16x8 qreg[NT][D / 32];
    int row_pos[NT];      // position of this lane's query row in the sequence (c + token)
    bool row_ok[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int r = r0 + w * kWaveRows + nt * 16 + t16;
        row_ok[nt] = wave_live && r < nrows;
        const int rc = min(r, nrows - 1);   // rows past the end repeat the last real row
        const int tk = rc / p.G, gg = rc % p.G;
        row_pos[nt] = c + tk;
        const uint16_t* src = a.q + (static_cast<size_t>(qoff + tk) * p.Hq + kv * p.G + gg) * D;
#pragma unroll
        for (int i = 0; i < D / 32; ++i)
            qreg[nt][i] = *reinterpret_cast<const bf16x8*>(src + (4 * i + kg) * 8);
    }
    f32x4 acc[NT][D / 16];
    f32x4 lacc[NT];       // softmax denominators (every register of a lane holds its row's)
    float m[NT], alpha[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m[nt] = kNegInf;
        alpha[nt] = 1.f;
        lacc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) acc[nt][jd] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the query loads are in before the page rings start

    f32x4 sc[NT][kSP];                       // raw scores of the stage whose softmax comes next
    u32x4 ph[NT][kSP / 2], pl[NT][kSP / 2];  // probabilities of the stage whose PV product comes next
    const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});

    // S^T = K Q^T of stage st for every tile (raw dot products; the scale is applied inside the exponent)
    auto qk = [&](int st) __attribute__((always_inline)) {
        unsigned ka[D / 32];
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            ka[i] = k_base + (st % kSlots) * kStageBytes + k_rd[i];
            asm volatile("" : "+v"(ka[i]));   // one add per stage; the page offset rides in the instruction
        }
#pragma unroll
        for (int j = 0; j < kSP; ++j) {
            bf16x8 kf[D / 32];
#pragma unroll
            for (int i = 0; i < D / 32; ++i) kf[i] = *lds_ptr<bf16x8>(ka[i] + j * kPageBytes);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < D / 32; ++i)
                    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[i], qreg[nt][i], s, 0, 0, 0);
                sc[nt][j] = s;
            }
        }
    };

    // Online softmax of stage st: sc -> ph, pl (bf16 head + bf16 remainder, two pages side by side: the
    // 8 keys a lane holds of a page pair are one k-group of a 32-deep contraction), m, alpha.  With
    // `masked`, keys after a row's own position (and slots past the sequence's end) are excluded by selection.
    auto softmax = [&](auto masked, int st) __attribute__((always_inline)) {
        const int key0 = st * kSP * kPage;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (decltype(masked)::value) {
#pragma unroll
                for (int j = 0; j < kSP; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (key0 + j * kPage + 4 * kg + r > row_pos[nt]) sc[nt][j][r] = kNegInf;
            }
            // the scale is positive, so the maximum can be taken before scaling; mn is finite from the
            // first stage on, because position 0 is visible to every row
            const float mx = row_max<kSP>(sc[nt]);
            const float mn = __builtin_fmaxf(m[nt], mx * p.scale_log2e);
            alpha[nt] = __builtin_amdgcn_exp2f(m[nt] - mn);
            m[nt] = mn;
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
        }
    };

    // O^T += V^T P^T of stage st, 32 keys per instruction; the row sums of P come from the same unit
    // (V^T replaced by ones).  With `ragged`, value rows past the sequence's end are zeroed first.
    auto pv = [&](auto ragged, int st) __attribute__((always_inline)) {
        const int key0 = st * kSP * kPage;
        unsigned va[D / 16];
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) {
            va[jd] = v_base + (st % kSlots) * kStageBytes + v_rd[jd];
            asm volatile("" : "+v"(va[jd]));
        }
#pragma unroll
        for (int jp = 0; jp < kSP / 2; ++jp) {
            bf16x8 bh[NT], bl[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                bh[nt] = __builtin_bit_cast(bf16x8, ph[nt][jp]);
                bl[nt] = __builtin_bit_cast(bf16x8, pl[nt][jp]);
                lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bh[nt], lacc[nt], 0, 0, 0);
                lacc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, bl[nt], lacc[nt], 0, 0, 0);
            }
            uint32_t keep[2][2];
            if (decltype(ragged)::value) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int valid = L - (key0 + (2 * jp + h) * kPage);   // tokens of this page that exist (<= 0: a repeated page)
                    keep[h][0] = (4 * kg + 0 < valid ? 0x0000ffffu : 0u) | (4 * kg + 1 < valid ? 0xffff0000u : 0u);
                    keep[h][1] = (4 * kg + 2 < valid ? 0x0000ffffu : 0u) | (4 * kg + 3 < valid ? 0xffff0000u : 0u);
                }
            }
#pragma unroll
            for (int q4 = 0; q4 < D / 64; ++q4) {   // four 16-wide slices of the head dimension at a time
                u32x4 vf[4];   // per lane: 4 keys of page 2 jp, then 4 keys of page 2 jp + 1
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            lds_ptr<s16x4>(va[4 * q4 + e] + (2 * jp + h) * kPageBytes)));
                        vf[e][2 * h] = t[0];
                        vf[e][2 * h + 1] = t[1];
                    }
                if (decltype(ragged)::value) {
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
                        const bf16x8 vt = __builtin_bit_cast(bf16x8, vf[e]);
                        acc[nt][4 * q4 + e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, bh[nt], acc[nt][4 * q4 + e], 0, 0, 0);
                        acc[nt][4 * q4 + e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, bl[nt], acc[nt][4 * q4 + e], 0, 0, 0);
                    }
            }
        }
    };

    // alpha of the last softmax is applied once the PV product issued before it is through
    auto rescale = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (__builtin_amdgcn_ballot_w64(alpha[nt] != 1.f) != 0) {   // nobody's maximum moved: alpha is exactly 1 everywhere
                lacc[nt] *= alpha[nt];
#pragma unroll
                for (int jd = 0; jd < D / 16; ++jd) acc[nt][jd] *= alpha[nt];
            }
        }
    };

    // One round: the scores of stage st, its softmax, its PV product.  The loads of stage st + kDist go
    // out among the matrix instructions of the scores.
    auto round = [&](auto steady, auto masked, auto ragged, int st) __attribute__((always_inline)) {
        if (decltype(steady)::value || st + kDist - 1 < nsteps) wait_vmcnt<kInFlight>(); else wait_vmcnt<0>();
        __syncthreads();   // stage st has landed; everybody is through round st - 1
        // every id of window (st + kDist) / kWin - 1 has been read by now: its slot takes the window after next
        // (a window no stage of which will be issued is not fetched: no load may be in flight when the block ends)
        if ((st + kDist) % kWin == 0 && ((st + kDist) / kWin + 1) * kWin < nsteps) fill_ids((st + kDist) / kWin + 1);
        qk(st);
        issue(steady, st + kDist, ids);
        load_ids(st + kDist + 1, ids);
        softmax(masked, st);
        rescale();
        pv(ragged, st);
    };

    // ---- prologue: the first kDist stages ----
    fill_ids(0);
    fill_ids(1);
    wait_vmcnt<0>();
    __syncthreads();
#pragma unroll
    for (int x = 0; x < kDist; ++x) {
        load_ids(x, ids);
        issue(Flag<false>{}, x, ids);
    }
    load_ids(kDist, ids);

    // ---- rounds ----
    // the softmax of stage st needs the mask once the stage reaches past the wave's first row
    const int first_masked = (c + tw0 >= kSP * kPage - 1) ? (c + tw0 - (kSP * kPage - 1)) / (kSP * kPage) + 1 : 0;
    int st = 0;
    // steady rounds: the stage they issue exists, no softmax needs the mask, no value row lies past the end
    for (; st + kDist < nsteps && st < first_masked; ++st) round(Flag<true>{}, Flag<false>{}, Flag<false>{}, st);
    for (; st < nsteps - 1; ++st) round(Flag<false>{}, Flag<true>{}, Flag<false>{}, st);
    round(Flag<false>{}, Flag<true>{}, Flag<true>{}, nsteps - 1);
    wait_vmcnt<0>();   // nothing of this wave's may still be on its way into LDS when the block retires
    if (bad_seen && lane == 0) atomicOr(&p.header[kHdrBadInput], kBadPage);

    // ---- normalise and store ----
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float lt = lacc[nt][0];
        if (!row_ok[nt]) continue;
        const int r = r0 + w * kWaveRows + nt * 16 + t16;
        const int tok = r / p.G, g = r % p.G;
        const float inv = 1.f / lt;
        float* o = a.out + (static_cast<size_t>(qoff + tok) * p.Hq + kv * p.G + g) * D + 4 * kg;
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            *reinterpret_cast<float4*>(o + 16 * jd) =
                make_float4(acc[nt][jd][0] * inv, acc[nt][jd][1] * inv, acc[nt][jd][2] * inv, acc[nt][jd][3] * inv);
    }
}

}  // namespace

// Query blocks per (request, kv head) for requests of up to max_q_len new tokens.
int prefill_query_blocks(int max_q_len, int G)
{
    return static_cast<int>((static_cast<int64_t>(max_q_len) * G + kPrefillBlockRows - 1) / kPrefillBlockRows);
}


hipError_t launch_prefill(const Params& p, const uint16_t* q, const int32_t* q_lens, const int32_t* q_offsets,
                          int total_q_rows, int max_q_len, float* out, hipStream_t stream)
{
    PrefillArgs a;
    a.q = q; a.q_lens = q_lens; a.q_offsets = q_offsets; a.out = out; a.tq = total_q_rows;
    a.nqb = prefill_query_blocks(max_q_len, p.G);
    if (a.nqb == 0 || p.B == 0) return hipSuccess;
    if (static_cast<int64_t>(a.nqb) * p.B * p.Hkv > 0x7fffffff) return hipErrorInvalidValue;
    a.order = p.order;
    hipLaunchKernelGGL(prefill_order_kernel, dim3((p.B + 255) / 256), dim3(256), 0, stream, p, q_lens, p.order);
    const dim3 grid(static_cast<unsigned>(a.nqb * p.B * p.Hkv));
    if (p.D == 128)
        hipLaunchKernelGGL((prefill_kernel<128, 2>), grid, dim3(kNW * 64), 0, stream, p, a);
    else
        hipLaunchKernelGGL((prefill_kernel<64, 2>), grid, dim3(kNW * 64), 0, stream, p, a);
    return hipGetLastError();
}

}  // namespace jd
