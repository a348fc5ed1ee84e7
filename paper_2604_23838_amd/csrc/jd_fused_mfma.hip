// Fused decode-attention kernel, matrix-core variant: work partition, split-KV partial
// attention and log-sum-exp combine in ONE launch.
//
// Prologue (work partition).  Every block scans seq_lens in LDS (exclusive prefix of pages
// per request) and each wave finds, by binary search, the (request, kv head, page) at
// which its equal share of the work line begins.  The scan is repeated by every block
// instead of being produced by a separate kernel: it costs a few KiB of L2 reads and
// removes a launch and a dependency from the critical path of short steps.  Rows of empty
// requests are zeroed here.
//
// Main loop (split-KV partial attention).  Each wave streams the KV pages of its span
// through a private ring of LDS stages.  A stage holds one 16-token page of K and of V for
// one kv head (D*32 bytes each) and, when the page opens a segment, the G query rows of
// that kv head.  Pages are moved HBM -> LDS by direct loads (16 bytes per lane, 1 KiB per
// instruction, fully coalesced) that bypass the vector registers, so the bytes a wave keeps
// in flight are set by the ring depth, not by register pressure; a wave only ever waits on
// the vector-memory counter for the oldest stage while the younger ones stay in flight.
// Block-table entries are fetched through the scalar data path one page ahead.
//
// Per page the GQA group is packed into matrix-core tiles (query rows padded to 16):
//   S^T[token][q]  = K[token][:] . Q[q][:]         D/32 x  v_mfma_f32_16x16x32_bf16
//   O^T[d][q]     += V^T[d][token] . P^T[token][q]  D/16 x  v_mfma_f32_16x16x16_bf16
// The accumulator layout of the first product (lane = query row, 4 consecutive tokens per
// lane) is exactly the B-operand layout of the second, so the probabilities never leave
// the registers; V is stored token-major, and the transposing LDS read delivers the
// token-minor A operand.  The probabilities are split into a bf16 head and a bf16
// remainder (two products), which keeps the result at fp32 accuracy.  Softmax is online in
// the exp2 domain with fp32 running maximum and sum per query row.
//
// Epilogue (combine).  A sequence that fits one wave is normalised and written directly.
// A sequence cut over several waves leaves one partial state (m, l, acc) per piece in the
// workspace; after its last page each wave bumps the sequence's arrival counter, and the
// wave that arrives last merges all pieces by the log-sum-exp rule and writes the rows.
// Nobody ever waits for anybody: the pattern cannot deadlock, and the counters reset
// themselves for the next call.
//
// LDS placement: the 16-byte chunks of a token row are XOR-swizzled with the token index
// so that both the row-wise K reads and the transposing V reads spread over all banks; the
// swizzle costs nothing because every lane of a direct load picks its own source address.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int kWaves = 4;  // waves per block; one block per compute unit (LDS-limited)
constexpr int kLdsBudget = 160 * 1024;

// meta word of a stage
constexpr int kMetaValidMask = 0x1f;
constexpr int kMetaFirst = 1 << 8;
constexpr int kMetaLast = 1 << 9;
constexpr int kMetaComplete = 1 << 10;
constexpr int kMetaSlot1 = 1 << 11;

template <int D, int QKB, int NS>
struct Geometry {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kPageBytes = kPage * kRowBytes;       // one tensor, one kv head
    static constexpr int kLoadsPerTensor = kPageBytes / 1024;  // wave-wide 1 KiB direct loads
    static constexpr int kQBytes = QKB * 1024;
    static constexpr int kQLoads = QKB;
    static constexpr int kStageBytes = kQBytes + 2 * kPageBytes;
    static constexpr int kWaveBytes = NS * kStageBytes;
    static constexpr int kLoadsPerStage = 2 * kLoadsPerTensor;  // Q loads come on top, only when a segment opens
    static constexpr int kChunksPerRow = kRowBytes / 16;
    static constexpr int kRowsPerLoad = 1024 / kRowBytes;
    static_assert(kWaves * kWaveBytes <= kLdsBudget, "LDS ring does not fit");
    static_assert(kWaves * kWaveBytes >= (2 * 8192 + 2 * kWaves * 64 + 256) * 4, "ring too small for the prologue tables");
};

__device__ inline void dma16(unsigned lds_addr, unsigned lane_off, const void* base)
{
    // LDS[lds_addr + 16 * lane] <- 16 bytes at base + lane_off; counted by vmcnt
    // nt: every K/V byte is read once per step, so the load is marked streaming; without it the pages
    // compete for the caches with themselves and the step is a tenth slower
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

// The same for a partial record that another compute unit has written: a device-coherent load (sc1), which
// bypasses the cache levels that are not coherent between dies.
__device__ inline void dma16_shared(unsigned lds_addr, unsigned lane_off, const void* base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 sc1"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
}

// The direct loads of one tensor's page, or of both tensors' pages when they fit the instruction's offset range:
// one LDS base in m0, the j-th load 1 KiB further on.  The instruction offset moves the global address and
// the LDS address alike, so the per-lane source offsets come with j KiB taken off (see init_lane_tables).
__device__ inline void dma16x4(unsigned lds_addr, unsigned o0, unsigned o1, unsigned o2, unsigned o3, const void* base01,
                               const void* base23)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, %5 nt\n\t"
                 "global_load_lds_dwordx4 %2, %5 offset:1024 nt\n\t"
                 "global_load_lds_dwordx4 %3, %6 offset:2048 nt\n\t"
                 "global_load_lds_dwordx4 %4, %6 offset:3072 nt"
                 :: "s"(lds_addr), "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(base01), "s"(base23) : "memory");
}

template <int N>
__device__ inline void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// Wait until at most `ahead` younger stages (of LPS loads each) are still in flight.
template <int LPS, int NS>
__device__ inline void wait_stage(int ahead)
{
    if constexpr (NS >= 8) { if (ahead >= 7) { wait_vmcnt<7 * LPS>(); return; } }
    if constexpr (NS >= 7) { if (ahead == 6) { wait_vmcnt<6 * LPS>(); return; } }
    if constexpr (NS >= 6) { if (ahead == 5) { wait_vmcnt<5 * LPS>(); return; } }
    if constexpr (NS >= 5) { if (ahead == 4) { wait_vmcnt<4 * LPS>(); return; } }
    if constexpr (NS >= 4) { if (ahead == 3) { wait_vmcnt<3 * LPS>(); return; } }
    if constexpr (NS >= 3) { if (ahead == 2) { wait_vmcnt<2 * LPS>(); return; } }
    if constexpr (NS >= 2) { if (ahead == 1) { wait_vmcnt<1 * LPS>(); return; } }
    wait_vmcnt<0>();
}

// Producer cursor: the next page-unit to fetch.
struct Cursor {
    int upos;           // position on the work line
    int r;              // index of the request among those that own pages
    int b, kv, pg;      // request, kv head, page within the request
    const int32_t* bt;  // block-table row of request b
    int L, n;           // tokens and pages of request b
    int seg_pg0;        // page at which the current segment began
    int seg_at_start;   // the current segment began at the first unit of the span
    int last_bkv, last_n, last_a;  // the stream the newest segment belongs to: b*Hkv+kv, pages, first unit
};

// One planned page-unit: everything issue() needs, with the block-table entry already on its way.
struct Planned {
    int meta, dest, id, kv;
    unsigned qrow;
};

__device__ inline int pages_of(const Params& p, int L)
{
    int n = L > 0 ? (L + kPage - 1) / kPage : 0;
    return n > p.maxp ? p.maxp : n;
}

template <int D, int QKB, int NS>
struct Wave {
    using Geo = Geometry<D, QKB, NS>;
    const Params& p;
    int lane, u0, u1;
    unsigned lds_wave;           // LDS byte address of this wave's ring
    lds_char* lds_ptr;           // same, as a pointer for the compiler-visible reads
    unsigned k_src[Geo::kLoadsPerTensor], v_src[Geo::kLoadsPerTensor], q_src[Geo::kQLoads];
    unsigned k_rd[D / 32], v_rd[D / 16], q_rd[D / 32];
    int meta[NS], dest[NS];
    bool bad_page = false;
    Cursor cur;
    Planned nx, nx2, rs[NS];
    // consumer state (lane = query row q = lane % 16; token group tg = lane / 16)
    bf16x8 qreg[D / 32];
    f32x4 acc[D / 16];
    float m, l;

    __device__ Wave(const Params& prm) : p(prm) {}

    __device__ void init_lane_tables()
    {
        const int G = p.G;
        constexpr int CPR = Geo::kChunksPerRow;   // 16-byte chunks per token row: 16 (D=128) or 8 (D=64)
        constexpr int RPL = Geo::kRowsPerLoad;    // token rows per direct load: 4 or 8
        // direct-load sources: LDS chunk (row t, position c') of load j is fed from source chunk c' ^ swizzle(t)
#pragma unroll
        for (int j = 0; j < Geo::kLoadsPerTensor; ++j) {
            const int t = j * RPL + lane / CPR;
            const int cp = lane % CPR;
            // load j is issued with an instruction offset of j KiB, which also moves its global address:
            // t * kRowBytes holds exactly those j KiB, so what is left is never negative
            k_src[j] = t * Geo::kRowBytes + ((cp ^ kswz(t)) * 16) - j * 1024;
            v_src[j] = t * Geo::kRowBytes + ((cp ^ vswz(t)) * 16) - j * 1024;
        }
        const int qbytes = G * Geo::kRowBytes;
#pragma unroll
        for (int j = 0; j < Geo::kQLoads; ++j) {
            int off = j * 1024 + lane * 16;
            q_src[j] = off < qbytes ? off : qbytes - 16;  // never read past the group's rows
        }
        // operand reads
        const int t = lane % 16, kg = lane / 16;
        const int qrow = t < G ? t : G - 1;
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            k_rd[i] = t * Geo::kRowBytes + (((4 * i + kg) ^ kswz(t)) * 16);
            q_rd[i] = qrow * Geo::kRowBytes + (4 * i + kg) * 16;
        }
        const int row = 4 * kg + (lane % 16) / 4, c = lane % 4;
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            v_rd[jd] = row * Geo::kRowBytes + (((2 * jd + c / 2) ^ vswz(row)) * 16) + (c % 2) * 8;
    }

    static constexpr int kRowShift = D == 128 ? 8 : 7;  // log2 of the bytes of one token row

    // A wave-uniform pointer, pinned to scalar registers (the direct loads take their base there).
    static __device__ inline const char* scalar_ptr(const char* ptr)
    {
        const uint64_t v = reinterpret_cast<uint64_t>(ptr);
        const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
        const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
        return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
    }

    static __device__ inline int kswz(int t) { return t & (Geo::kChunksPerRow - 1); }
    static __device__ inline int vswz(int t)
    {
        return D == 128 ? ((t & 7) << 1) : (((t >> 1) & 3) << 1);
    }

    // ---- producer -------------------------------------------------------------------------------
    // Move to the next request that owns pages (only called while units remain, so one exists): its id
    // comes from the compacted list the prologue stored, so finished rows cost nothing here.
    __device__ inline void next_request()
    {
        int r = cur.r + 1;
        if (r >= live) {  // seq_lens changed under the kernel: stay in bounds, flag it
            r = live - 1;
            if (lane == 0) atomicOr(&p.header[kHdrBadInput], kBadLensMoved);
        }
        // The list was stored earlier in this kernel, so the compiler will not take it through the scalar
        // path by itself; a vector load here would make it drain the page ring.  The block's own stores
        // completed before its first wave got here.
        int b;
        asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(b)
                     : "s"(scalar_ptr(reinterpret_cast<const char*>(p.req) + (static_cast<uint64_t>(static_cast<unsigned>(r)) << 2)))
                     : "memory");
        const int L = uniform_load(p.seq_lens + b);
        int n = pages_of(p, L);
        if (n == 0) n = 1;  // same cause; a one-page request keeps every index in range
        cur.r = r;
        cur.b = b;
        cur.bt = p.block_table + static_cast<size_t>(b) * p.maxp;
        cur.n = n;
        cur.L = L > n * kPage ? n * kPage : (L < 1 ? 1 : L);
    }

    // Describe the unit at the cursor, request its block-table entry, and move the cursor on.
    __device__ inline void plan(Planned& r)
    {
        r.id = uniform_load(cur.bt + cur.pg);
        r.dest = cur.b * p.Hkv + cur.kv;
        r.kv = cur.kv;
        r.qrow = static_cast<unsigned>(cur.b * p.Hq + cur.kv * p.G);
        // the common case, a full page in the middle of a sequence and of the span: nothing begins or ends
        if (cur.pg != 0 && cur.pg + 1 != cur.n && cur.upos != u0 && cur.upos + 1 != u1) {
            r.meta = kPage;
            ++cur.upos;
            ++cur.pg;
            return;
        }
        const bool first = (cur.upos == u0) || (cur.pg == 0);
        const bool last = (cur.pg == cur.n - 1) || (cur.upos == u1 - 1);
        if (first) {
            cur.seg_pg0 = cur.pg;
            cur.seg_at_start = (cur.upos == u0);
            cur.last_bkv = cur.b * p.Hkv + cur.kv;
            cur.last_n = cur.n;
            cur.last_a = cur.upos - cur.pg;
        }
        int mt = min(kPage, cur.L - cur.pg * kPage);
        if (first) mt |= kMetaFirst;
        if (last) {
            mt |= kMetaLast;
            if (cur.seg_pg0 == 0 && cur.pg == cur.n - 1) mt |= kMetaComplete;
            // a piece that starts before its wave's span is record 0, any other record 1
            if (!(cur.seg_at_start && cur.seg_pg0 > 0)) mt |= kMetaSlot1;
        }
        r.meta = mt;

        ++cur.upos;
        if (++cur.pg == cur.n) {
            cur.pg = 0;
            cur.kv += p.wg;                 // the next kv head of this wave's lane in the group
            if (cur.kv >= p.Hkv) {
                cur.kv = member;
                if (cur.upos < u1) next_request();
            }
        }
    }

    // Start the direct loads of a planned unit into stage S.
    template <int S>
    __device__ inline void issue(const Planned& r)
    {
        // a page id out of range reads page 0 and raises the sticky flag when the wave ends; the id stays
        // on the scalar unit (no divergent branch here)
        const bool ok = static_cast<unsigned>(r.id) < static_cast<unsigned>(p.NP);
        bad_page |= !ok;
        const unsigned id = __builtin_amdgcn_readfirstlane(ok ? static_cast<unsigned>(r.id) : 0u);
        meta[S] = r.meta;
        dest[S] = r.dest;
        const unsigned kv = static_cast<unsigned>(r.kv);
        const unsigned stage = lds_wave + S * Geo::kStageBytes;
        // every read of this stage's previous contents has returned before it is overwritten
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // byte offsets are 32-bit indices shifted left, so the address arithmetic stays on the scalar unit
        if (r.meta & kMetaFirst) {
            const char* qb = scalar_ptr(reinterpret_cast<const char*>(p.q) + (static_cast<uint64_t>(r.qrow) << kRowShift));
#pragma unroll
            for (int j = 0; j < Geo::kQLoads; ++j) dma16(stage + j * 1024, q_src[j], qb);
        }
        const uint64_t page_off = static_cast<uint64_t>(id * static_cast<unsigned>(p.Hkv) + kv) << (kRowShift + 4);
        const char* kb = scalar_ptr(reinterpret_cast<const char*>(p.k_pages) + page_off);
        const char* vb = scalar_ptr(reinterpret_cast<const char*>(p.v_pages) + page_off);
        if constexpr (Geo::kLoadsPerTensor == 2) {
            // K and V of the page behind one LDS base: V's slot lies 2 KiB behind K's, so V's global base goes 2 KiB back
            dma16x4(stage + Geo::kQBytes, k_src[0], k_src[1], v_src[0], v_src[1], kb, vb - Geo::kPageBytes);
        } else {
            static_assert(Geo::kLoadsPerTensor == 4, "four 1 KiB loads per tensor at head_dim 128");
            dma16x4(stage + Geo::kQBytes, k_src[0], k_src[1], k_src[2], k_src[3], kb, kb);
            dma16x4(stage + Geo::kQBytes + Geo::kPageBytes, v_src[0], v_src[1], v_src[2], v_src[3], vb, vb);
        }
    }

    // ---- consumer -------------------------------------------------------------------------------
    template <int S>
    __device__ inline void consume()
    {
        constexpr float kNegInf = -__builtin_inff();
        lds_char* stage = lds_ptr + S * Geo::kStageBytes;
        const int mt = meta[S];
        const int valid = mt & kMetaValidMask;
        const int tg = lane >> 4;

        if (mt & kMetaFirst) {
#pragma unroll
            for (int i = 0; i < D / 32; ++i)
                qreg[i] = *reinterpret_cast<__attribute__((address_space(3))) bf16x8*>(stage + q_rd[i]);
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd) acc[jd] = f32x4{0.f, 0.f, 0.f, 0.f};
            m = kNegInf;
            l = 0.f;
        }

        // S^T = K Q^T
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        lds_char* kbase = stage + Geo::kQBytes;
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            const bf16x8 kf = *reinterpret_cast<__attribute__((address_space(3))) bf16x8*>(kbase + k_rd[i]);
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qreg[i], s, 0, 0, 0);
        }
        // V^T operands (issued early; the softmax arithmetic overlaps their latency)
        s16x4 vf[D / 16];
        lds_char* vbase = stage + Geo::kQBytes + Geo::kPageBytes;
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd)
            vf[jd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                reinterpret_cast<__attribute__((address_space(3))) s16x4*>(vbase + v_rd[jd]));

        float sc[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) sc[r] = s[r] * p.scale_log2e;
        if (valid < kPage) {
            // slots past the end of the sequence: excluded by selection (their bits may be anything)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool dead = 4 * tg + r >= valid;
                if (dead) sc[r] = kNegInf;
#pragma unroll
                for (int jd = 0; jd < D / 16; ++jd)
                    if (dead) vf[jd][r] = 0;
            }
        }
        float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
        mx = rows_max(mx);
        const float mn = fmaxf(m, mx);  // finite: every page holds at least one live token
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        float pr[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) pr[r] = __builtin_amdgcn_exp2f(sc[r] - mn);
        l = l * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
        if (__builtin_amdgcn_ballot_w64(mn > m) != 0) {
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[jd][r] *= alpha;
        }
        m = mn;

        // probabilities as bf16 head + bf16 remainder
        s16x4 ph, pl;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const __bf16 h = static_cast<__bf16>(pr[r]);
            const __bf16 lo = static_cast<__bf16>(pr[r] - static_cast<float>(h));
            ph[r] = __builtin_bit_cast(short, h);
            pl[r] = __builtin_bit_cast(short, lo);
        }
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) {
            acc[jd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[jd], ph, acc[jd], 0, 0, 0);
            acc[jd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf[jd], pl, acc[jd], 0, 0, 0);
        }

        if (mt & kMetaLast) finalize(mt, dest[S]);
    }

    // Two full pages from the middle of one segment, in slots S and S + 1, as one softmax update over their 32
    // tokens.  A wave is alone on its SIMD, so every latency in the chain LDS read -> scores -> maximum ->
    // exponentials -> P.V is idle time; two pages side by side give the scheduler independent work to fill it,
    // and the row maximum, the rescale and the bookkeeping of the running sum are paid once.  The 8 tokens a
    // lane holds of the two pages are one k-group of a 32-deep contraction, so P.V takes half the instructions.
    template <int S>
    __device__ inline void consume_pair()
    {
        lds_char* st0 = lds_ptr + S * Geo::kStageBytes + Geo::kQBytes;
        lds_char* st1 = st0 + Geo::kStageBytes;
        bf16x8 k0[D / 32], k1[D / 32];
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            k0[i] = *reinterpret_cast<__attribute__((address_space(3))) bf16x8*>(st0 + k_rd[i]);
            k1[i] = *reinterpret_cast<__attribute__((address_space(3))) bf16x8*>(st1 + k_rd[i]);
        }
        s16x4 v0[D / 16], v1[D / 16];
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) {
            v0[jd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                reinterpret_cast<__attribute__((address_space(3))) s16x4*>(st0 + Geo::kPageBytes + v_rd[jd]));
            v1[jd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                reinterpret_cast<__attribute__((address_space(3))) s16x4*>(st1 + Geo::kPageBytes + v_rd[jd]));
        }
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < D / 32; ++i) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0[i], qreg[i], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1[i], qreg[i], s1, 0, 0, 0);
        }
        float sc[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            sc[r] = s0[r] * p.scale_log2e;
            sc[4 + r] = s1[r] * p.scale_log2e;
        }
        float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        mx = rows_max(mx);
        const float mn = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - mn);
        float pr[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) pr[r] = __builtin_amdgcn_exp2f(sc[r] - mn);
        l = l * alpha + (((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7])));
        if (__builtin_amdgcn_ballot_w64(mn > m) != 0) {
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[jd][r] *= alpha;
        }
        m = mn;
        s16x8 ph, pl;   // bf16 head and bf16 remainder of the probabilities
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const __bf16 h = static_cast<__bf16>(pr[r]);
            const __bf16 lo = static_cast<__bf16>(pr[r] - static_cast<float>(h));
            ph[r] = __builtin_bit_cast(short, h);
            pl[r] = __builtin_bit_cast(short, lo);
        }
#pragma unroll
        for (int jd = 0; jd < D / 16; ++jd) {
            const s16x8 vt = {v0[jd][0], v0[jd][1], v0[jd][2], v0[jd][3], v1[jd][0], v1[jd][1], v1[jd][2], v1[jd][3]};
            acc[jd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt), __builtin_bit_cast(bf16x8, ph), acc[jd], 0, 0, 0);
            acc[jd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt), __builtin_bit_cast(bf16x8, pl), acc[jd], 0, 0, 0);
        }
    }

    __device__ inline void finalize(int mt, int bkv)
    {
        const int qh = lane & 15, tg = lane >> 4;
        const float lt = rows_sum(l);
        if (qh >= p.G) return;
        const int b = bkv / p.Hkv, kv = bkv % p.Hkv;
        if (mt & kMetaComplete) {
            const float inv = 1.f / lt;
            float* o = p.out + (static_cast<size_t>(b) * p.Hq + kv * p.G + qh) * D + 4 * tg;
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd)
                *reinterpret_cast<float4*>(o + 16 * jd) =
                    make_float4(acc[jd][0] * inv, acc[jd][1] * inv, acc[jd][2] * inv, acc[jd][3] * inv);
        } else {
            // Records are shared between compute units that sit behind different L2 caches.  They are
            // written and read with device-scope atomic accesses, which go through to memory, so
            // that no cache-wide write-back or invalidate is ever needed.
            const int slot = (mt & kMetaSlot1) ? 1 : 0;
            const unsigned rec = static_cast<unsigned>(wave * 2 + slot) * record_floats(p.G, D) * 4u;  // byte offset
            const unsigned o = rec + (qh * D + 4 * tg) * 4u;
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd) shared_store4(o + 64 * jd, acc[jd]);
            if (tg == 0) shared_store2(rec + (p.G * D + 2 * qh) * 4u, m, lt);   // (m, l) of a row side by side
        }
    }

    // Records are shared between compute units that sit behind different L2 caches.  They are
    // written and read with device-coherent accesses (sc1: write-through stores here, loads that
    // bypass the non-coherent cache levels in the merge), so that no cache-wide write-back or
    // invalidate is ever needed.  `off` is a byte offset into the record area; the buffer
    // descriptor bounds every store to that area.
    static constexpr int kDeviceCoherent = 16;  // cache-policy bit sc1
    __device__ inline void shared_store4(unsigned off, f32x4 v) const
    {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), records, off, 0, kDeviceCoherent);
    }
    __device__ inline void shared_store2(unsigned off, float a, float b) const
    {
        __builtin_amdgcn_raw_buffer_store_b64(u32x2{__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b)}, records, off, 0,
                                              kDeviceCoherent);
    }

    // ---- epilogue: arrival counters and last-arriver merge -------------------------------------
    // Count this wave's piece of stream bkv (units [a, a+n) of the work line) with add = 1, or, with add = 0,
    // look at the count of a stream whose piece was announced earlier; whoever finds every piece counted
    // merges them.  The caller has waited for its record stores to complete.  A piece announced without
    // an answer may have been the last to be counted, which only its own later look (add = 0) can find
    // out; that look may also come just before another wave, which counted last, resets the counter:
    // the stream is then merged twice, to the same bits.
    //
    // A stream of kFlatMergePieces pieces or more is merged in two levels, so that no single wave has to
    // fold them all: the piece is counted in its cluster of kMergeCluster wave groups; the last one there
    // merges the cluster's pieces into the cluster's record, waits for its stores and counts the cluster in the
    // stream's counter; the last cluster merges the cluster records.  Every count at both levels is an add whose
    // answer is awaited (pieces of such streams are never announced early), so each merge happens once.
    static constexpr int kWholeStream = -1;
    // more than kFlatMergePieces - 1 spans long: cut into kFlatMergePieces pieces at least, i.e. over two clusters or more
    __device__ inline bool two_levels(int n) const { return n > (kFlatMergePieces - 1) * span; }
    __device__ inline void arrive(int bkv, int a, int n, int add)
    {
        const int w0 = a / span, w1 = (a + n - 1) / span;
        // the only level: all pieces of the stream
        int first = w0, last = w1, into = kWholeStream;
        int* counter = p.counters + bkv;
        if (two_levels(n)) {   // the first level of two: the cluster's part of the stream
            const int c = group / kMergeCluster;
            first = max(w0, c * kMergeCluster);
            last = min(w1, c * kMergeCluster + kMergeCluster - 1);
            into = cluster_record(c, w0);
            counter = p.counters + p.B * p.Hkv + into;
        }
        bool from_clusters = false;
#pragma unroll 1
        for (;;) {
            int old = 0;
            if (lane == 0) old = __hip_atomic_fetch_add(counter, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            old = __builtin_amdgcn_readfirstlane(old);
            if (old + add != last - first + 1) return;
            if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("" ::: "memory");  // the record loads below stay behind the counter read
            // the record of item i: of wave group i, the first of its wave's two if the piece began before that wave's
            // span (a < i*span), the second otherwise; of cluster i, behind all of those, by the same rule (w0 < i*8)
            merge(bkv, first, last, from_clusters ? 2 * p.slots : 0, from_clusters ? w0 : a, from_clusters ? kMergeCluster : span, into);
            if (into == kWholeStream) return;
            // second level: the cluster's record is complete in memory before the cluster is counted
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            first = w0 / kMergeCluster;
            last = w1 / kMergeCluster;
            counter = p.counters + bkv;
            into = kWholeStream;
            from_clusters = true;
            add = 1;
        }
    }

    // Index of the record (and counter) of cluster c for the part of a stream that begins in wave group w0.
    __device__ inline int cluster_record(int c, int w0) const
    {
        return ((c * p.wg + member) * 2 + (w0 < c * kMergeCluster ? 0 : 1));
    }

    // Log-sum-exp merge of records first..last of one stream, by one wave: its pieces (the records of the wave
    // groups first..last) or the records of its clusters first..last (item i is record
    // base + (i*wg + member)*2 + (start < i*stride ? 0 : 1)); the result goes to the output rows, normalised,
    // or, as it is, into cluster record `into`.  The G*D accumulator floats of a
    // record are contiguous; lane j owns the float4 groups j, j+64, ... of them (each group lies in
    // one query row).  The wave's page ring is empty by now and takes the records: a batch of them is
    // copied into it whole by direct loads, 16 bytes a lane and load, as many records as fit the ring
    // and the counter of loads in flight, so that all of them overlap; then they are folded in one
    // after the other from LDS.  The direct loads are inline assembly with one explicit wait behind
    // them: compiler-visible loads into registers inside the loop over batches get a full wait in front
    // of each of them from the compiler (their registers may still be the target of a load of the trip
    // before), which turns a merge of 13 pieces into 26 round trips to memory, one after the other.
    // The loops are rolled and short: a wave that is alone on its SIMD issues one instruction every
    // four cycles, so at the end of a step the length of this code in instructions is its time.
    __device__ inline void merge(int bkv, int first, int last, int base, int start, int stride, int into)
    {
        constexpr int K = 2 * QKB;           // float4 groups per lane: G*D*2 <= QKB KiB, so G*D/4 <= 128*QKB groups
        constexpr int NL = K + 1;            // 1 KiB loads per record: its G*D*4 <= K KiB, its (m, l) pairs another 8*G bytes
        const int G = p.G;
        const int groups = G * D / 4;
        const unsigned rec_bytes = record_floats(G, D) * 4u;   // a whole number of 16-byte units
        const int fit = min(static_cast<int>(Geo::kWaveBytes / rec_bytes), 60 / NL);   // records per batch
        // A lane without a k-th group folds group 0 in its place and stores nothing for it: the loop below
        // then has no divergent parts, and the reads of a lane's groups are issued together.
        int idx[K], grp[K], qrow[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            idx[k] = lane + 64 * k;
            if (idx[k] >= groups) idx[k] = -1;
            grp[k] = idx[k] < 0 ? 0 : idx[k];
            qrow[k] = grp[k] * 4 / D;
        }
        float M[K], den[K];
        f32x4 num[K];
#pragma unroll
        for (int k = 0; k < K; ++k) { M[k] = -__builtin_inff(); den[k] = 0.f; num[k] = f32x4{0.f, 0.f, 0.f, 0.f}; }

        for (int w = first; w <= last; w += fit) {
            const int nb = min(fit, last - w + 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the LDS reads of the batch before have returned
#pragma unroll 1
            for (int i = 0; i < nb; ++i) {
                const int wi = w + i;
                const int r = base + (wi * p.wg + member) * 2 + (start < wi * stride ? 0 : 1);
                const char* src = scalar_ptr(reinterpret_cast<const char*>(p.partials) + static_cast<unsigned>(r) * rec_bytes);
                const unsigned dst = lds_wave + static_cast<unsigned>(i) * rec_bytes;
#pragma unroll
                for (int j = 0; j < NL; ++j) {
                    const unsigned off = j * 1024u + lane * 16u;
                    if (off < rec_bytes) dma16_shared(dst + j * 1024u, off, src);
                }
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll 1
            for (int i = 0; i < nb; ++i) {
                const lds_char* rec = lds_ptr + static_cast<unsigned>(i) * rec_bytes;
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    const f32x2 ml = *reinterpret_cast<const __attribute__((address_space(3))) f32x2*>(rec + (G * D + 2 * qrow[k]) * 4);
                    const f32x4 aa = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(rec + grp[k] * 16);
                    const float mb = fmaxf(M[k], ml[0]);
                    const float c_old = __builtin_amdgcn_exp2f(M[k] - mb);
                    const float c = __builtin_amdgcn_exp2f(ml[0] - mb);
                    M[k] = mb;
                    den[k] = fmaf(c, ml[1], den[k] * c_old);
#pragma unroll
                    for (int r = 0; r < 4; ++r) num[k][r] = fmaf(c, aa[r], num[k][r] * c_old);
                }
            }
        }
        if (into != kWholeStream) {
            // a record like a wave's own: the sums as they are, and (m, l) from the lane that owns a row's first group
            const unsigned rec = static_cast<unsigned>(2 * p.slots + into) * rec_bytes;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (idx[k] < 0) continue;
                shared_store4(rec + idx[k] * 16u, num[k]);
                if (idx[k] * 4 % D == 0) shared_store2(rec + (G * D + 2 * qrow[k]) * 4u, M[k], den[k]);
            }
            return;
        }
        const int b = bkv / p.Hkv, kv = bkv % p.Hkv;
        float* o = p.out + (static_cast<size_t>(b) * p.Hq + kv * G) * D;  // the group's rows are contiguous, like the record's
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (idx[k] < 0) continue;
            const float inv = 1.f / den[k];
            *reinterpret_cast<float4*>(o + idx[k] * 4) =
                make_float4(num[k][0] * inv, num[k][1] * inv, num[k][2] * inv, num[k][3] * inv);
        }
    }

    __amdgpu_buffer_rsrc_t records;  // the record area of the workspace
    int wave;       // index of this wave
    int group;      // index of its group of wg waves
    int member;     // its place in its group of wg waves: it serves the kv heads congruent to member mod wg
    int span;       // group-units per group of waves
    int live;       // requests that own pages
    int first_bkv, first_n, first_pg0;  // the stream the span begins in, and the page it begins at

    template <int S>
    __device__ inline void plan_stage(int total, Planned* rs)
    {
        if (S < total) plan(rs[S]);
        if constexpr (S + 1 < NS) plan_stage<S + 1>(total, rs);
    }

    template <int S>
    __device__ inline void issue_stage(int total, const Planned* rs)
    {
        if (S < total) issue<S>(rs[S]);
        if constexpr (S + 1 < NS) issue_stage<S + 1>(total, rs);
    }

    template <int S>
    __device__ inline void round_stage(int base, int total)
    {
        const int i = base + S;
        if (i < total) {
            wait_stage<Geo::kLoadsPerStage, NS>(min(NS - 1, total - 1 - i));
            consume<S>();
            if (i + NS < total) {
                issue<S>(nx);                       // its block-table entry was requested a page ago
                if constexpr (kPairs) {             // two units are kept planned: the second moves up
                    nx = nx2;
                    if (i + NS + 2 < total) plan(nx2);
                } else {
                    if (i + NS + 1 < total) plan(nx);
                }
            }
        }
        if constexpr (S + 1 < NS) round_stage<S + 1>(base, total);
    }

    // A round in which every stage still has a full ring behind it: the wait is the same each time,
    // a unit is always issued and the next one always planned (no comparisons against the span's end).
    template <int S>
    __device__ inline void steady_stage()
    {
        wait_vmcnt<(NS - 1) * Geo::kLoadsPerStage>();
        consume<S>();
        issue<S>(nx);
        plan(nx);
        if constexpr (S + 1 < NS) steady_stage<S + 1>();
    }

    // Two such rounds at once where the ring is deep enough to spare a slot: both pages have landed, and if they are
    // full pages from the middle of one segment (nothing begins or ends in either) they are consumed as a pair.
    // Two units are then kept planned (nx, nx2), so that each block-table entry is still requested a pair ahead
    // of its use.  Not with a 2 KiB query slot (64-wide heads, more than 8 query heads per kv head): in that
    // instantiation the compiler takes the wave-uniform loads of lengths and page ids in the loop through the
    // vector path, with a full wait behind each of them, which drains the ring (4.2 against 6.0 TB/s measured).
    static constexpr bool kPairs = NS >= 6 && NS % 2 == 0 && QKB == 1;
    template <int S>
    __device__ inline void steady_pair()
    {
        wait_vmcnt<(NS - 2) * Geo::kLoadsPerStage>();
        if (meta[S] == kPage && meta[S + 1] == kPage) {
            consume_pair<S>();
        } else {
            consume<S>();
            consume<S + 1>();
        }
        issue<S>(nx);
        issue<S + 1>(nx2);
        plan(nx);
        plan(nx2);
        if constexpr (S + 2 < NS) steady_pair<S + 2>();
    }
    __device__ inline void steady_round()
    {
        if constexpr (kPairs) steady_pair<0>(); else steady_stage<0>();
    }

    // Request the block-table entries of the first stages, all at once.  Touches no LDS, so it can run
    // while the block is still busy with the partition tables.
    __device__ inline void begin()
    {
        plan_stage<0>(u1 - u0, rs);
    }

    __device__ inline void run()
    {
        const int total = u1 - u0;
        issue_stage<0>(total, rs);
        if (NS < total) plan(nx);
        if constexpr (kPairs) {
            if (NS + 1 < total) plan(nx2);
        }
        // a steady round issues NS units and plans as many beyond them: they must all exist
        constexpr int kSteady = 2 * NS + (kPairs ? 1 : 0);

        // Pieces of sequences shared with other waves: at most the first and the last stream of the span.
        const int first_a = u0 - first_pg0;
        const bool first_partial = first_pg0 > 0 || first_a + first_n > u1;
        // When the first stream ends inside the span, its piece (the stream's last) is stored early in the
        // span.  Vector memory operations complete in issue order, so once NS - 1 further stages have gone
        // through the steady wait the record stores are known to have completed, and the piece is announced
        // right there, without draining the ring and without waiting for an answer.  The wave that holds
        // the stream's earlier piece then finds every piece in place at the end of its own span and merges;
        // this wave owes at most one merge when it ends (for the stream its span ends in) instead of two.
        const int first_end = first_a + first_n - u0;   // stages the first stream takes in this span, if it ends inside
        bool announced = false;
        // stages after which the piece may be announced (never reached when there is nothing to announce)
        const int stop = (first_partial && first_end < total && !two_levels(first_n)) ? first_end + NS - 1 : total;
        int base = 0;
        for (; base + kSteady < total; base += NS) {   // one copy of the steady round in the kernel's code
            if (base >= stop && !announced) {
                if (lane == 0) (void)__hip_atomic_fetch_add(p.counters + first_bkv, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                announced = true;
            }
            steady_round();
        }
        if (base >= stop && !announced) {
            if (lane == 0) (void)__hip_atomic_fetch_add(p.counters + first_bkv, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            announced = true;
        }
        for (; base < total; base += NS) round_stage<0>(base, total);

        const bool last_partial = cur.last_a != first_a && cur.last_a + cur.last_n > u1;
        if (first_partial || last_partial) {
            // release: the write-through record stores of this wave have completed before it is counted
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (first_partial) arrive(first_bkv, first_a, first_n, announced ? 0 : 1);
            if (last_partial) arrive(cur.last_bkv, cur.last_a, cur.last_n, 1);
        }
        if (bad_page && lane == 0) atomicOr(&p.header[kHdrBadInput], kBadPage);
    }
};

constexpr int kThreads = kWaves * 64;


// The partition tables, by all threads of the block: the requests that own pages are compacted, in
// order, into c_req[0..R) (their ids) and c_cum[0..R] (pages before each, total at the end), both in
// LDS; the id list is also stored to the workspace (every block stores the same values), where the
// waves find the next live request when they walk off the end of one.  Returns R.
__device__ inline int build_tables(const Params& p, int* c_cum, int* c_req, int* s_part)
{
    const int tid = threadIdx.x;
    const int chunk = (p.B + kThreads - 1) / kThreads;
    const int b0 = min(tid * chunk, p.B), b1 = min(b0 + chunk, p.B);
    int pages = 0, live = 0;
    for (int b = b0; b < b1; ++b) {
        const int L = p.seq_lens[b];
        if (L > p.maxp * kPage && (p.header[kHdrBadInput] & kBadLength) == 0) atomicOr(&p.header[kHdrBadInput], kBadLength);
        const int n = pages_of(p, L);
        pages += n;
        live += n > 0;
    }
    s_part[tid] = pages;
    s_part[kThreads + tid] = live;
    __syncthreads();
    if (tid < 64) {
        constexpr int per = kThreads / 64;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            int* arr = s_part + which * kThreads;
            int v[per], sum = 0;
#pragma unroll
            for (int i = 0; i < per; ++i) { v[i] = arr[tid * per + i]; sum += v[i]; }
            int inc = sum;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int t = __shfl_up(inc, d, 64);
                if (tid >= d) inc += t;
            }
            int run = inc - sum;
#pragma unroll
            for (int i = 0; i < per; ++i) { arr[tid * per + i] = run; run += v[i]; }
        }
    }
    __syncthreads();
    int run_p = s_part[tid], run_r = s_part[kThreads + tid];
    for (int b = b0; b < b1; ++b) {
        const int n = pages_of(p, p.seq_lens[b]);
        if (n > 0) {
            c_cum[run_r] = run_p;
            c_req[run_r] = b;
            p.req[run_r] = b;
            ++run_r;
            run_p += n;
        }
    }
    if (tid == kThreads - 1) {  // the last thread ends on the totals
        c_cum[run_r] = run_p;
        s_part[2 * kThreads] = run_r;
    }
    __syncthreads();
    return s_part[2 * kThreads];
}

template <int D, int QKB, int NS>
__global__ __launch_bounds__(kThreads) void decode_fused_kernel(Params p, int partition_only)
{
    using W = Wave<D, QKB, NS>;
    __shared__ __attribute__((aligned(1024))) char ring[kWaves * W::Geo::kWaveBytes];
    // ---- prologue: work partition (the ring doubles as scratch until the first page is fetched) ----
    int* c_cum = reinterpret_cast<int*>(ring);
    int* c_req = c_cum + ((p.B + 1 + 63) & ~63);
    int* s_part = c_req + ((p.B + 63) & ~63);
    // (values read from LDS are wave-uniform here; saying so keeps everything derived from them on the scalar unit)
    const int live = __builtin_amdgcn_readfirstlane(build_tables(p, c_cum, c_req, s_part));
    // Waves work in groups of wg: the waves of a group walk the same (request, page) sequence, each on its
    // own kv heads (member, member + wg, ...), so that together they read neighbouring kv heads of the
    // same physical page at about the same time.  The work line is counted in group-units
    // (request, kv-head group, page); a group of waves owns a span of it.
    const int hg = p.Hkv / p.wg;
    const int units = __builtin_amdgcn_readfirstlane(c_cum[live]) * hg;
    const int span = span_for(units, p.slots / p.wg);
    const int active = (units + span - 1) / span;   // groups that own at least one unit

    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Blocks go to the chip's eight dies in turn (block i to die i % 8).  Waves are numbered die by die, so that
    // consecutive spans of the work line, and with them the pieces of a sequence, sit on one die.
    const int nblocks = static_cast<int>(gridDim.x);
    const int block = nblocks % 8 == 0 ? static_cast<int>(blockIdx.x % 8) * (nblocks / 8) + static_cast<int>(blockIdx.x / 8)
                                       : static_cast<int>(blockIdx.x);
    const int wave = __builtin_amdgcn_readfirstlane(block * kWaves + wave_in_block);
    const int group = wave / p.wg, member = wave % p.wg;
    int sr = 0, sb = 0, skv = 0, spg = 0;
    if (group < active) {
        const int u = group * span;
        int lo = 0, hi = live - 1;  // the last live request whose first unit is <= u
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (c_cum[mid] * hg <= u) lo = mid; else hi = mid - 1;
        }
        const int n = c_cum[lo + 1] - c_cum[lo];
        const int within = u - c_cum[lo] * hg;
        sr = lo;
        sb = c_req[lo];
        skv = (within / n) * p.wg + member;
        spg = within % n;
    }
    sr = __builtin_amdgcn_readfirstlane(sr);
    sb = __builtin_amdgcn_readfirstlane(sb);
    skv = __builtin_amdgcn_readfirstlane(skv);
    spg = __builtin_amdgcn_readfirstlane(spg);
    // Touch the block-table line and the length this wave starts with now: the first access is a cold miss
    // all the way to HBM, and the rest of the prologue hides it.
    int warm = 0;
    if (group < active && !partition_only)
        warm = uniform_load(p.block_table + static_cast<size_t>(sb) * p.maxp + spg) ^ uniform_load(p.seq_lens + sb);

    if (partition_only) {
        // tables for inspection
        if (blockIdx.x == 0) {
            for (int b = threadIdx.x; b <= p.B; b += kThreads) {
                int lo = 0, hi = live;  // pages before request b = pages before the first live request at or after b
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (c_req[mid] < b) lo = mid + 1; else hi = mid;
                }
                p.cum_pages[b] = c_cum[lo];
            }
            if (threadIdx.x == 0) {
                p.header[kHdrUnits] = units;
                p.header[kHdrSpan] = span;
                p.header[kHdrActive] = active;
                p.header[kHdrSlots] = p.slots;
                p.header[kHdrGroup] = p.wg;
            }
        }
        if (group < active && (threadIdx.x & 63) == 0) {
            i32x4 ws = {sb, skv, spg, sb};
            reinterpret_cast<i32x4*>(p.wave_start)[wave] = ws;
        }
    }
    // Every wave's stores of the request list have reached the L2 before the barrier, so after it the whole
    // block's copy is there for the scalar loads that walk it (the barrier alone does not wait for stores).
    asm volatile("s_waitcnt vmcnt(0)" :: "s"(warm) : "memory");
    __syncthreads();  // the scratch is dead from here on
    if (!partition_only) {
        // Rows of requests without tokens.  Nobody waits for these stores: they drain while the page ring
        // starts (older operations in flight only make the ring's counter waits err on the safe side).
        for (int b = blockIdx.x; b < p.B; b += gridDim.x) {
            if (pages_of(p, uniform_load(p.seq_lens + b)) == 0) {
                float4* o = reinterpret_cast<float4*>(p.out + static_cast<size_t>(b) * p.Hq * D);
                for (int i = threadIdx.x; i < p.Hq * D / 4; i += kThreads) o[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    }
    if (partition_only || group >= active) return;

    W w(p);
    w.lane = threadIdx.x & 63;
    w.wave = wave;
    w.member = member;
    w.group = group;
    w.span = span;
    w.live = live;
    w.u0 = group * span;
    w.u1 = min(w.u0 + span, units);
    w.lds_ptr = (lds_char*)ring + wave_in_block * W::Geo::kWaveBytes;
    w.lds_wave = static_cast<unsigned>(reinterpret_cast<uintptr_t>(w.lds_ptr));
    w.init_lane_tables();
    w.records = __builtin_amdgcn_make_buffer_rsrc(p.partials, 0, static_cast<int>((2u * p.slots + cluster_records(p.slots)) * record_floats(p.G, D) * 4u), 0x00020000);
    w.m = 0.f;
    w.l = 0.f;
    w.cur.upos = w.u0;
    w.cur.r = sr;
    w.cur.b = sb;
    w.cur.bt = p.block_table + static_cast<size_t>(sb) * p.maxp;
    w.cur.kv = skv;
    w.cur.pg = spg;
    const int L = uniform_load(p.seq_lens + sb);
    w.cur.n = pages_of(p, L);
    w.cur.L = L > w.cur.n * kPage ? w.cur.n * kPage : L;
    w.cur.seg_pg0 = spg;
    w.cur.seg_at_start = 1;
    w.cur.last_bkv = sb * p.Hkv + skv;
    w.cur.last_n = w.cur.n;
    w.cur.last_a = w.u0 - spg;
    w.first_bkv = w.cur.last_bkv;
    w.first_n = w.cur.n;
    w.first_pg0 = spg;
    w.begin();

    // ---- main loop and epilogue ----
    w.run();
}

// Ring depth: as many stages as the LDS of one compute unit holds for kWaves waves, at most 8.
constexpr int stages_for(int D, int qkb)
{
    const int stage = qkb * 1024 + 2 * kPage * D * 2;
    const int n = kLdsBudget / (kWaves * stage);
    return n > 8 ? 8 : n;
}

template <int D, int QKB, int NS>
hipError_t launch(const Params& p, hipStream_t stream, int partition_only)
{
    hipLaunchKernelGGL((decode_fused_kernel<D, QKB, NS>), dim3(p.slots / kWaves), dim3(kThreads), 0, stream, p,
                       partition_only);
    return hipGetLastError();
}

}  // namespace

int mfma_waves_per_cu() { return kWaves; }
int mfma_waves_per_block() { return kWaves; }

// Waves per group: the largest power of two, at most 8, that divides the kv-head count and the wave slots
// (with 8 kv heads every wave of a group serves one head, and a sequence is cut into half as many pieces
// as with two heads a wave).
int mfma_group_waves(int num_kv_heads, int slots)
{
    int wg = 1;
    while (wg * 2 <= 2 * kWaves && num_kv_heads % (wg * 2) == 0 && slots % (wg * 2) == 0) wg *= 2;
    return wg;
}

int mfma_max_batch()
{
    // the prologue keeps 2B + 1 table entries and two entries per thread in the ring (at least 96 KiB)
    return 8192;
}

hipError_t launch_fused_mfma(const Params& p, hipStream_t stream, int partition_only)
{
    // query slot of a stage: G rows of D bf16, rounded up to whole 1 KiB direct loads
    const int qkb = (p.G * p.D * 2 + 1023) / 1024;
    if (p.D == 128) {
        if (qkb <= 1) return launch<128, 1, stages_for(128, 1)>(p, stream, partition_only);
        if (qkb <= 2) return launch<128, 2, stages_for(128, 2)>(p, stream, partition_only);
        return launch<128, 4, stages_for(128, 4)>(p, stream, partition_only);
    }
    if (qkb <= 1) return launch<64, 1, stages_for(64, 1)>(p, stream, partition_only);
    return launch<64, 2, stages_for(64, 2)>(p, stream, partition_only);
}

}  // namespace jd
