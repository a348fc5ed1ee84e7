// Causal prefill attention over the paged cache (KV recomputation after a migration, new turns of a
// multi-turn rollout): the last q_lens[b] tokens of request b attend to everything before them and to
// each other causally.  Unlike decode this is bound by the matrix cores, not by HBM.
//
// One block of kNW waves serves one (request, kv head, block of query tokens); two blocks (three at
// head_dim 64) share a compute unit.  Each wave holds one tile of 32 query rows in registers (row r of a
// request's kv head is query head r % G of new token r / G, packed densely whatever G is), and all waves
// sweep the same K/V pages, which the block stages in shared LDS rings of 64-key stages with direct loads
// (every wave loads one page of a stage; one barrier per stage).  The block table reaches LDS the same
// way, a window of 64 page ids at a time, so no round waits for a table read.  Per 32-key tile, with 32x32
// matrix tiles (v_mfma_f32_32x32x16_bf16, one query row per lane):
//   S^T[key][row]  = K . Q^T; a lane ends up with 16 keys of its query row, its partner lane (l ^ 32)
//                    with the other 16,
//   online softmax in the exp2 domain against the reference exponent the row already has; row maxima,
//                    a new reference and rescaled accumulators only when a row has outgrown it,
//   O^T[d][row]   += V^T . P^T, one page (16 keys) per instruction: the 8 keys a lane holds of a page are
//                    its k-group of the contraction, so P needs no shuffle; P as bf16 head + bf16 remainder,
//                    V read transposed from LDS.
// The three are software-pipelined over consecutive tiles and their instructions ordered by hand.
// Keys after a row's own position are excluded by selection (only in the rounds that reach the
// diagonal); pages wholly above the block's last position are never fetched.  Requests are dispatched
// by decreasing work (a small ranking kernel runs first), the query blocks of a request heaviest first.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int kNW = 4;    // waves per block; two blocks share a compute unit
constexpr int kWaveRows = 32;                     // query rows of a wave: one 32-wide matrix tile
constexpr int kPrefillBlockRows = kNW * kWaveRows;   // query rows (token x head of the group) per block

// The direct loads of one tensor's page: one LDS base in m0, the j-th load 1 KiB further on.  The instruction
// offset moves the global address and the LDS address alike, so the per-lane source offsets come with j KiB
// taken off.
__device__ inline void dma_page(unsigned lds_addr, const unsigned (&o)[4], const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %5\n\t"
                 "global_load_lds_dwordx4 %2, %5 offset:1024\n\t"
                 "global_load_lds_dwordx4 %3, %5 offset:2048\n\t"
                 "global_load_lds_dwordx4 %4, %5 offset:3072"
                 :: "s"(lds_addr), "v"(o[0]), "v"(o[1]), "v"(o[2]), "v"(o[3]), "s"(base) : "memory");
}

__device__ inline void dma_page(unsigned lds_addr, const unsigned (&o)[2], const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %3\n\t"
                 "global_load_lds_dwordx4 %2, %3 offset:1024"
                 :: "s"(lds_addr), "v"(o[0]), "v"(o[1]), "s"(base) : "memory");
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

// Maximum of the 16 scores a lane holds of its query row in a tile, then of its partner's (lane ^ 32 holds
// the other keys of the row).  Plain compiler-visible maxima on purpose: the compiler places the wait
// states that a read of a fresh matrix result needs, which it cannot do for an instruction hidden in
// inline assembly (a hand-written v_max3 here once read scores before the matrix unit had written
// them: right to rounding, since only the reference maximum moved, but not repeatable).
__device__ inline float row_max(const f32x16& s)
{
    float mx = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), s[2]);
#pragma unroll
    for (int e = 3; e < 15; e += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[e]), s[e + 1]);
    mx = __builtin_fmaxf(mx, s[15]);
    const unsigned xb = __float_as_uint(mx);
    const u32x2 b = __builtin_amdgcn_permlane32_swap(xb, xb, false, false);
    return __builtin_fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
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
template <int T>
struct Tensor { static constexpr int value = T; };

template <int D>
__global__ __launch_bounds__(kNW * 64, D == 64 ? 3 : 2) void prefill_kernel(Params p, PrefillArgs a)
{
    constexpr int kSP = 4;   // pages (16 keys each) per ring stage: one barrier per 64 keys, two 32-key tiles
    constexpr int kRowBytes = D * 2;
    constexpr int kPageBytes = kPage * kRowBytes;
    constexpr int kStageBytes = kSP * kPageBytes;             // one tensor's share of a stage
    constexpr int kHalfParts = kPageBytes / 1024;             // 1 KiB direct loads per page and tensor: 4 (D=128) or 2 (D=64)
    static_assert(kSP == kNW, "every wave loads one page of a stage");
    constexpr int CPR = kRowBytes / 16, RPL = 1024 / kRowBytes;
    constexpr int kRowShift = D == 128 ? 8 : 7;
    constexpr float kNegInf = -__builtin_inff();
    // K and V rings of two stages each; the loads of a stage are in flight for one round (see the rounds below)
    constexpr int kSlots = 2;
    static_assert(2 * 2 * kHalfParts <= 63, "vmcnt is a 6-bit counter");
    __shared__ __attribute__((aligned(1024))) char kring[kSlots * kStageBytes];
    __shared__ __attribute__((aligned(1024))) char vring[kSlots * kStageBytes];
    // page ids of the request, two windows of 64 pages: page q sits at idring[q % 128]
    __shared__ __attribute__((aligned(256))) int32_t idring[128];
    constexpr int kWin = 64 / kSP;   // stages per window

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Blocks go to the chip's eight dies in turn (block i to die i % 8), each die with an L2 of its own.  When the
    // kv heads come in eights, die d takes the kv heads congruent to d of every request: all query blocks of a
    // (request, kv head) then read its K/V pages through one L2, and every die gets the same share of every request.
    const bool by_die = p.Hkv % 8 == 0;
    const int lin = by_die ? static_cast<int>(blockIdx.x / 8) : static_cast<int>(blockIdx.x);
    const int bkv = by_die ? (lin / a.nqb) * 8 + static_cast<int>(blockIdx.x % 8) : lin / a.nqb;
    const int b = min(max(uniform_load(a.order + bkv / p.Hkv), 0), p.B - 1), kv = bkv % p.Hkv;
    const int L0 = uniform_load(p.seq_lens + b);
    int n = uniform_load(a.q_lens + b);
    const int npages = min(L0 > 0 ? (L0 + kPage - 1) / kPage : 0, p.maxp);
    const int L = min(L0, npages * kPage);
    if (n > L) n = L;                      // malformed: more new tokens than the cache holds
    const int c = L - n;                   // tokens of context in front of the new ones
    // query rows of the request: row r is head r % G of new token r / G (no padding of the group)
    const int nrows = n * p.G;
    const int qb = a.nqb - 1 - lin % a.nqb;   // heaviest query block first
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

    // ---- lane tables (same placement in LDS as the decode kernel: rows XOR-swizzled by token) ----
    // lane = (kh, j32): j32 is the lane's query row in the tile and, for a matrix A operand, its key
    // (K) or head-dimension element (V^T); kh picks the 8-wide half of a 16-deep contraction step.
    const int j32 = lane % 32, kh = lane / 32, t16 = lane % 16;
    // K as A operand of step i: key j32 of a 32-key tile (two pages), elements 16 i + 8 kh .. + 7
    // (chunk 2 i + kh, swizzled by the token).
    const unsigned k_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)kring));
    const unsigned v_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_char*)vring));
    constexpr int NDT = D / 32, NK = D / 16;
    // Step i toggles address bits above the half only, so one register serves every step (exclusive-or with 32 i);
    // likewise the head-dimension tile of a V^T operand (exclusive-or with 64 dt).
    const unsigned k_rd = k_base + (j32 / 16) * kPageBytes + t16 * kRowBytes + ((kh ^ (t16 & (CPR - 1))) * 16);
    // V^T as A operand of head-dimension tile dt: the transposing read hands lane i of a 16-lane group element i
    // of 4 keys; the group reads keys 4 kh .. + 3 (and 8 more for the second half of the k-group) of
    // elements 32 dt + 16 (j32 / 16) .. + 15.
    unsigned v_rd;
    {
        const int key = 4 * kh + t16 / 4, cc = t16 % 4;
        const int vs = D == 128 ? ((key & 7) << 1) : (((key >> 1) & 3) << 1);
        v_rd = v_base + key * kRowBytes + (((2 * (j32 / 16) + cc / 2) ^ vs) * 16) + (cc % 2) * 8;
    }
    // this wave's share of a stage: page w of K and of V, in 1 KiB direct loads; lane l of load q fills
    // row q RPL + l / CPR, chunk position l % CPR, with the chunk the swizzle puts there.  The loads of a
    // page differ by a constant exclusive-or at most (the row's swizzle moves with q): one register a tensor.
    unsigned src_k, src_v;
    {
        const int t = lane / CPR, cp = lane % CPR;
        src_k = t * kRowBytes + ((cp ^ (t & (CPR - 1))) * 16);
        src_v = t * kRowBytes + ((cp ^ (D == 128 ? ((t & 7) << 1) : (((t >> 1) & 3) << 1))) * 16);
    }
    auto page_sources = [&](auto which, unsigned (&o)[kHalfParts]) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < kHalfParts; ++q) {
            // row q RPL + t: the instruction offset supplies q KiB on both sides, the swizzle term of q RPL stays
            const int tq = q * RPL;
            const unsigned flip = decltype(which)::value == 0 ? (tq & (CPR - 1)) * 16u
                                                               : (D == 128 ? ((tq & 7) << 1) : (((tq >> 1) & 3) << 1)) * 16u;
            o[q] = (decltype(which)::value == 0 ? src_k : src_v) ^ flip;
        }
    };
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
    auto load_id = [&](int st) __attribute__((always_inline)) -> int {
        return __builtin_amdgcn_readfirstlane(idring[(st * kSP + w) & 127]);
    };
    bool bad_seen = false;
    // this wave's direct loads of stage st of one tensor (K: which = 0, V: which = 1), the page with id `id`;
    // with `sure` the stage is known to exist
    auto issue = [&](auto which, auto sure, int st, int id) __attribute__((always_inline)) {
        if (!decltype(sure)::value && st >= nsteps) return;
        const bool ok = static_cast<unsigned>(id) < static_cast<unsigned>(p.NP);
        bad_seen |= !ok;
        // a page id out of range reads page 0 and raises the sticky flag
        const unsigned idc = __builtin_amdgcn_readfirstlane(ok ? static_cast<unsigned>(id) : 0u);
        const unsigned row = idc * static_cast<unsigned>(p.Hkv) + static_cast<unsigned>(kv);
        const uint64_t off = static_cast<uint64_t>(row) << (kRowShift + 4);
        const unsigned dst = __builtin_amdgcn_readfirstlane((st % kSlots) * kStageBytes + w * kPageBytes);
        unsigned o[kHalfParts];
        page_sources(which, o);
        if (decltype(which)::value == 0) dma_page(k_base + dst, o, scalar_ptr(kpool + off));
        else dma_page(v_base + dst, o, scalar_ptr(vpool + off));
    };
    int id_k, id_v;   // page ids of this wave's page of the next K stage and of the next V stage to issue

    // ---- queries of this wave: 32 rows, row = (token, head of the group); B operand of step i ----
    bf16x8 qreg[D / 16];
    int row_pos;      // position of this lane's query row in the sequence (c + token)
    bool row_ok;
    {
        const int r = r0 + w * kWaveRows + j32;
        row_ok = wave_live && r < nrows;
        const int rc = min(r, nrows - 1);   // rows past the end repeat the last real row
        const int tk = rc / p.G, gg = rc % p.G;
        row_pos = c + tk;
        const uint16_t* src = a.q + (static_cast<size_t>(qoff + tk) * p.Hq + kv * p.G + gg) * D;
#pragma unroll
        for (int i = 0; i < D / 16; ++i)
            qreg[i] = *reinterpret_cast<const bf16x8*>(src + (2 * i + kh) * 8);
    }
    f32x16 acc[D / 32];   // O^T: register r of tile dt is element 32 dt + 8 (r / 4) + 4 kh + r % 4 of row j32
    float lsum = 0.f;     // softmax denominator over this lane's keys (the partner lane holds the rest)
    float m = kNegInf;    // reference exponent of the row's probabilities (log2 domain)
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the query loads are in before the page rings start

    f32x16 sc[2];              // raw scores of a 32-key tile, by tile parity: register r is key 8 (r / 4) + 4 kh + r % 4 of the tile
    u32x4 ph[2][2], pl[2][2];  // probabilities of a tile, by tile parity and page: the lane's 8 keys of the page as bf16 pairs

    // S^T = K Q^T of tile kt of stage st (raw dot products; the scale is applied inside the exponent)
    auto qk = [&](int st, int kt) __attribute__((always_inline)) {
        const unsigned ka = k_rd + (st % kSlots) * kStageBytes + kt * 2 * kPageBytes;
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            const bf16x8 kf = *lds_ptr<bf16x8>(ka ^ (i * 32));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qreg[i], s, 0, 0, 0);
        }
        sc[kt] = s;
    };

    // Probabilities of scores 2 j, 2 j + 1 of tile kt against the reference exponent mref: -> ph[kt], pl[kt]
    // (bf16 head + bf16 remainder; the remainder p - head comes from one packed dot product per score:
    // head . (-1, 0) + p), their sum joins part[j % 4].
    // (the two constants live in scalar registers: written as an immediate, the pair (-1, 0) is encoded as
    // the inline constant -1.0, which the instruction reads as the pair (0, -1))
    uint32_t minus_first_bits = 0x0000bf80u, minus_second_bits = 0xbf800000u;
    asm volatile("" : "+s"(minus_first_bits), "+s"(minus_second_bits));
    const bf16x2 minus_first = __builtin_bit_cast(bf16x2, minus_first_bits), minus_second = __builtin_bit_cast(bf16x2, minus_second_bits);
    auto probability_pair = [&](int kt, int j, float mref, float (&part)[4]) __attribute__((always_inline)) {
        const int r = 2 * j;
        f32x2 pr;
        pr[0] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][r], p.scale_log2e, -mref));
        pr[1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][r + 1], p.scale_log2e, -mref));
        part[j % 4] += pr[0];
        part[j % 4] += pr[1];
        const bf16x2 hi = __builtin_convertvector(pr, bf16x2);
        f32x2 rem;
        rem[0] = __builtin_amdgcn_fdot2_f32_bf16(hi, minus_first, pr[0], false);
        rem[1] = __builtin_amdgcn_fdot2_f32_bf16(hi, minus_second, pr[1], false);
        const bf16x2 lo = __builtin_convertvector(rem, bf16x2);
        ph[kt][r / 8][(r % 8) / 2] = __builtin_bit_cast(uint32_t, hi);
        pl[kt][r / 8][(r % 8) / 2] = __builtin_bit_cast(uint32_t, lo);
    };
    auto probabilities = [&](int kt, float mref) __attribute__((always_inline)) -> float {
        float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 8; ++j) probability_pair(kt, j, mref, part);
        return (part[0] + part[1]) + (part[2] + part[3]);
    };

    // Keys after the row's own position (and slots past the sequence's end) are excluded by selection.
    auto mask = [&](int st, int kt) __attribute__((always_inline)) {
        const int key0 = (st * kSP + 2 * kt) * kPage + 4 * kh;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (key0 + 8 * (r / 4) + r % 4 > row_pos) sc[kt][r] = kNegInf;
    };

    // Online softmax of a tile.  Any reference exponent m gives the same result as long as nothing
    // overflows, so the tile is first evaluated against the m the row already has (no row maximum, no
    // rescaling of the accumulators: the common case once the first tiles have set m): `part` is that
    // evaluation's sum.  Only when some row's probabilities have outgrown 2^16 (or m is still unset, or
    // a sum is not a number) does the wave take the exact path: row maxima, new m, accumulators and
    // sums rescaled, probabilities again.  The accumulators hold exactly the tiles before this one.
    auto settle = [&](int kt, float part) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(!(part < 65536.f)) != 0) {
            // the scale is positive, so the maximum can be taken before scaling; mn is finite,
            // because position 0 is visible to every row
            const float mx = row_max(sc[kt]);
            const float mn = __builtin_fmaxf(m, mx * p.scale_log2e);
            const float alpha = __builtin_amdgcn_exp2f(m - mn);
            m = mn;
            lsum *= alpha;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt) acc[dt] *= alpha;
            part = probabilities(kt, m);
        }
        lsum += part;
    };

    // V^T operands of one page of a tile: read k of the page is half k % 2 of the k-group of head-dimension tile k / 2;
    // va is this lane's address in the tile for head-dimension tile 0
    auto read_v = [&](unsigned va, int pg, int k, u32x4 (&vf)[2][NDT]) __attribute__((always_inline)) {
        const int dt = k / 2, h = k % 2;
        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            lds_ptr<s16x4>((va ^ (dt * 64)) + pg * kPageBytes + h * 8 * kRowBytes)));
        vf[pg][dt][2 * h] = t[0];
        vf[pg][dt][2 * h + 1] = t[1];
    };

    // O^T += V^T P^T of tile kt of stage st on its own (the last tile of a block), value rows past the
    // sequence's end zeroed first.
    auto pv_last = [&](int st, int kt) __attribute__((always_inline)) {
        const int key0 = (st * kSP + 2 * kt) * kPage + 4 * kh;
        const unsigned va = v_rd + (st % kSlots) * kStageBytes + kt * 2 * kPageBytes;
        u32x4 vf[2][NDT];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
#pragma unroll
            for (int k = 0; k < 2 * NDT; ++k) read_v(va, pg, k, vf);
            const int valid = L - (key0 + pg * kPage);   // tokens from this lane's first key on that exist (<= 0: a repeated page)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k0 = 8 * (e / 2) + 2 * (e % 2);
                const uint32_t keep = (k0 < valid ? 0x0000ffffu : 0u) | (k0 + 1 < valid ? 0xffff0000u : 0u);
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) vf[pg][dt][e] &= keep;
            }
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[pg][dt]), __builtin_bit_cast(bf16x8, ph[kt][pg]), acc[dt], 0, 0, 0);
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[pg][dt]), __builtin_bit_cast(bf16x8, pl[kt][pg]), acc[dt], 0, 0, 0);
        }
    };

    // Half a round: the PV product of the tile before tile (st, KT), the softmax of tile (st, KT), the scores of
    // the tile after it: matrix work and vector work that do not depend on each other, in one stretch of
    // straight-line code (a SIMD overlaps the two kinds only when one wave's instruction stream offers both).
    // The order is fixed by hand, group by group: one matrix instruction, the LDS reads that later groups need
    // (the second page's V operands during the first page's products, each K operand three groups ahead), and a
    // share of the 8 probability pairs; the compiler's own order bunches the matrix instructions.
    auto half = [&](auto kt_c, auto with_pv, auto masked, auto ragged, auto sure, int st) __attribute__((always_inline)) {
        constexpr int KT = decltype(kt_c)::value, OT = 1 - KT;
        constexpr int NPV = decltype(with_pv)::value ? 4 * NDT : 0, NM = NPV + NK, kLead = NPV >= 3 ? 3 : 0;
        const int st_pv = st - 1 + KT, st_qk = st + KT;   // the tile before is (st - 1, 1) or (st, 0), the tile after (st, 1) or (st + 1, 0)
        // this lane's addresses in the two tiles (one add per tile; the rest rides in the instructions)
        unsigned va = v_rd + (st_pv % kSlots) * kStageBytes + OT * 2 * kPageBytes;
        unsigned ka = k_rd + (st_qk % kSlots) * kStageBytes + OT * 2 * kPageBytes;
        asm volatile("" : "+v"(va), "+v"(ka));
        if (decltype(masked)::value) mask(st, KT);
        u32x4 vf[2][NDT];
        bf16x8 kf[NK];
        uint32_t keep[2][4];
        if (NPV != 0) {
#pragma unroll
            for (int k = 0; k < 2 * NDT; ++k) read_v(va, 0, k, vf);
            if (decltype(ragged)::value) {
                const int key0 = (st_pv * kSP + 2 * OT) * kPage + 4 * kh;
#pragma unroll
                for (int pg = 0; pg < 2; ++pg) {
                    const int valid = L - (key0 + pg * kPage);   // tokens from this lane's first key on that exist (<= 0: a repeated page)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int k0 = 8 * (e / 2) + 2 * (e % 2);
                        keep[pg][e] = (k0 < valid ? 0x0000ffffu : 0u) | (k0 + 1 < valid ? 0xffff0000u : 0u);
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NK; ++i)
            if (i - kLead < 0 || NPV == 0) kf[i] = *lds_ptr<bf16x8>(ka ^ (i * 32));
        float part[4] = {0.f, 0.f, 0.f, 0.f};
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < NM; ++g) {
            if (g < NPV) {
                const int pg = g / (2 * NDT), dt = (g % (2 * NDT)) / 2, lo = g % 2;   // head then remainder on one accumulator
                if (decltype(ragged)::value && lo == 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) vf[pg][dt][e] &= keep[pg][e];
                }
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[pg][dt]),
                                                                  __builtin_bit_cast(bf16x8, lo ? pl[OT][pg] : ph[OT][pg]), acc[dt], 0, 0, 0);
                if (g < 2 * NDT) read_v(va, 1, g, vf);
            } else {
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[g - NPV], qreg[g - NPV], s, 0, 0, 0);
            }
            if (NPV != 0 && g - (NPV - kLead) >= 0 && g - (NPV - kLead) < NK) kf[g - (NPV - kLead)] = *lds_ptr<bf16x8>(ka ^ ((g - (NPV - kLead)) * 32));
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (g == j * NM / 8) probability_pair(KT, j, m, part);
            // the second half carries the round's direct loads (K of stage st + 2, then V of stage st + 1: their
            // slots are free since the barrier in front of it) and fetches the page id of the round after
            if (KT == 1) {
                if (g == 0) issue(Tensor<0>{}, sure, st + 2, id_k);
                else if (g == 2) issue(Tensor<1>{}, sure, st + 1, id_v);
                else if (g == 4) { id_v = id_k; id_k = load_id(st + 3); }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        sc[OT] = s;
        // the probabilities are complete before the branch of `settle` (the compiler would sink their bf16
        // split behind it, where no matrix instruction runs)
        asm volatile("" :: "v"(ph[KT][0]), "v"(ph[KT][1]), "v"(pl[KT][0]), "v"(pl[KT][1]));
        settle(KT, (part[0] + part[1]) + (part[2] + part[3]));
    };

    // One round = the two 32-key tiles of stage st, software-pipelined:
    //   first half:   PV of tile (st - 1, 1)   softmax of tile (st, 0)   scores of tile (st, 1)
    //   middle:       every wave's loads have landed, barrier
    //   second half:  PV of tile (st, 0)       softmax of tile (st, 1)   scores of tile (st + 1, 0)   the next loads
    // So K of stage st + 1 and V of stage st must be in LDS at the middle of round st; they were issued at the
    // middle of round st - 1, into the slots that K of stage st - 1 and V of stage st - 2 had left by then, and
    // have a whole round to arrive.  One barrier per round.
    auto round = [&](auto first, auto masked, auto ragged, auto sure, int st) __attribute__((always_inline)) {
        half(Tensor<0>{}, Flag<!decltype(first)::value>{}, masked, Flag<false>{}, sure, st);
        wait_vmcnt<0>();
        __syncthreads();   // K of stage st + 1 and V of stage st have landed; everybody has left K of stage st and V of stage st - 1
        // every id of window (st + 1) / kWin - 1 has been read by now: its slot takes the window after next
        // (a window no stage of which will be issued is not fetched: no load may be in flight when the block ends)
        if ((st + 1) % kWin == 0 && ((st + 1) / kWin + 1) * kWin < nsteps) fill_ids((st + 1) / kWin + 1);
        half(Tensor<1>{}, Flag<true>{}, masked, ragged, sure, st);   // past the last stage: scores of whatever the slot holds, never used
    };

    // ---- prologue: K and V of stage 0, K of stage 1, the scores of the first tile ----
    fill_ids(0);
    fill_ids(1);
    wait_vmcnt<0>();
    __syncthreads();
    id_k = load_id(0);
    issue(Tensor<0>{}, Flag<false>{}, 0, id_k);
    issue(Tensor<1>{}, Flag<false>{}, 0, id_k);
    id_v = load_id(1);
    issue(Tensor<0>{}, Flag<false>{}, 1, id_v);
    id_k = load_id(2);
    wait_vmcnt<0>();
    __syncthreads();
    qk(0, 0);

    // ---- rounds ----
    // the softmax of stage st needs the mask once the stage reaches past the wave's first row
    const int first_masked = (c + tw0 >= kSP * kPage - 1) ? (c + tw0 - (kSP * kPage - 1)) / (kSP * kPage) + 1 : 0;
    if (nsteps == 1) {
        round(Flag<true>{}, Flag<true>{}, Flag<true>{}, Flag<false>{}, 0);
    } else {
        round(Flag<true>{}, Flag<true>{}, Flag<false>{}, Flag<false>{}, 0);
        int st = 1;
        // steady rounds: the stages they load exist, no softmax needs the mask, no value row lies past the end
        for (; st < nsteps - 2 && st < first_masked; ++st) round(Flag<false>{}, Flag<false>{}, Flag<false>{}, Flag<true>{}, st);
        for (; st < nsteps - 1; ++st) round(Flag<false>{}, Flag<true>{}, Flag<false>{}, Flag<false>{}, st);
        round(Flag<false>{}, Flag<true>{}, Flag<true>{}, Flag<false>{}, nsteps - 1);
    }
    pv_last(nsteps - 1, 1);
    wait_vmcnt<0>();   // nothing of this wave's may still be on its way into LDS when the block retires
    if (bad_seen && lane == 0) atomicOr(&p.header[kHdrBadInput], kBadPage);

    // ---- normalise and store ----
    {
        const unsigned lb = __float_as_uint(lsum);
        const u32x2 both = __builtin_amdgcn_permlane32_swap(lb, lb, false, false);   // the partner's share of the row sum
        const float lt = __uint_as_float(both.x) + __uint_as_float(both.y);
        if (row_ok) {
            const int r = r0 + w * kWaveRows + j32;
            const int tok = r / p.G, g = r % p.G;
            const float inv = 1.f / lt;
            float* o = a.out + (static_cast<size_t>(qoff + tok) * p.Hq + kv * p.G + g) * D + 4 * kh;
#pragma unroll
            for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<float4*>(o + 32 * dt + 8 * e) =
                        make_float4(acc[dt][4 * e] * inv, acc[dt][4 * e + 1] * inv, acc[dt][4 * e + 2] * inv, acc[dt][4 * e + 3] * inv);
        }
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
        hipLaunchKernelGGL((prefill_kernel<128>), grid, dim3(kNW * 64), 0, stream, p, a);
    else
        hipLaunchKernelGGL((prefill_kernel<64>), grid, dim3(kNW * 64), 0, stream, p, a);
    return hipGetLastError();
}

}  // namespace jd
