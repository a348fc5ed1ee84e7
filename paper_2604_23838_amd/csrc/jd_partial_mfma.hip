// Split-KV partial attention, matrix-core variant.
//
// Each wave streams the KV pages of its span through a private ring of LDS stages.  A
// stage holds one 16-token page of K and of V for one kv head (D*32 bytes each) and,
// when the page opens a segment, the G query rows of that kv head.  Pages are moved
// HBM -> LDS by direct loads (16 bytes per lane, 1 KiB per instruction, fully coalesced)
// that bypass the vector registers, so the number of bytes a wave keeps in flight is set
// by the ring depth, not by register pressure; a wave only ever waits on the vector-memory
// counter for the oldest stage while the younger ones stay in flight.
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
// LDS placement: the 16-byte chunks of a token row are XOR-swizzled with the token index
// so that both the row-wise K reads and the transposing V reads spread over all banks; the
// swizzle costs nothing because every lane of a direct load picks its own source address.
#include "jd_internal.h"
#include "jd_walk.h"

namespace jd {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int kWaves = 4;  // waves per block, one per SIMD; one block per compute unit

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
    static_assert(kWaves * kWaveBytes <= 160 * 1024, "LDS ring does not fit");
};

__device__ inline void dma16(unsigned lds_addr, unsigned lane_off, const void* base)
{
    // LDS[lds_addr + 16 * lane] <- 16 bytes at base + lane_off; counted by vmcnt
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory");
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
    int upos;     // position on the work line
    int r, kv, pg;
    Stream st;
    int seg_pg0;  // page of the stream at which the current segment began
};

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
    Cursor cur;
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
            k_src[j] = t * Geo::kRowBytes + ((cp ^ kswz(t)) * 16);
            v_src[j] = t * Geo::kRowBytes + ((cp ^ vswz(t)) * 16);
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
    template <int S>
    __device__ inline void produce()
    {
        const Stream& st = cur.st;
        const int id = checked_page(p, uniform_load(p.block_table + static_cast<size_t>(st.b) * p.maxp + cur.pg));
        const bool first = (cur.upos == u0) || (cur.pg == 0);
        const bool last = (cur.pg == st.n - 1) || (cur.upos == u1 - 1);
        if (first) cur.seg_pg0 = cur.pg;
        int mt = min(kPage, st.L - cur.pg * kPage);
        if (first) mt |= kMetaFirst;
        if (last) {
            mt |= kMetaLast;
            if (cur.seg_pg0 == 0 && cur.pg == st.n - 1) mt |= kMetaComplete;
            if (!(st.a < u0)) mt |= kMetaSlot1;
        }
        meta[S] = mt;
        dest[S] = st.b * p.Hkv + cur.kv;

        const unsigned stage = lds_wave + S * Geo::kStageBytes;
        // every read of this stage's previous contents has returned before it is overwritten
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        // byte offsets are 32-bit indices shifted left, so the address arithmetic stays on the scalar unit
        if (first) {
            const unsigned qrow = static_cast<unsigned>(st.b * p.Hq + cur.kv * p.G);
            const char* qb = scalar_ptr(reinterpret_cast<const char*>(p.q) + (static_cast<uint64_t>(qrow) << kRowShift));
#pragma unroll
            for (int j = 0; j < Geo::kQLoads; ++j) dma16(stage + j * 1024, q_src[j], qb);
        }
        const uint64_t page_off = static_cast<uint64_t>(static_cast<unsigned>(id * p.Hkv + cur.kv)) << (kRowShift + 4);
        const char* kb = scalar_ptr(reinterpret_cast<const char*>(p.k_pages) + page_off);
        const char* vb = scalar_ptr(reinterpret_cast<const char*>(p.v_pages) + page_off);
#pragma unroll
        for (int j = 0; j < Geo::kLoadsPerTensor; ++j) dma16(stage + Geo::kQBytes + j * 1024, k_src[j], kb);
#pragma unroll
        for (int j = 0; j < Geo::kLoadsPerTensor; ++j)
            dma16(stage + Geo::kQBytes + Geo::kPageBytes + j * 1024, v_src[j], vb);

        // advance to the next unit
        ++cur.upos;
        if (++cur.pg == st.n) {
            cur.pg = 0;
            if (++cur.kv == p.Hkv) { cur.kv = 0; ++cur.r; }
            if (cur.upos < u1) cur.st = open_stream(p, cur.r, cur.kv);
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
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
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

    __device__ inline void finalize(int mt, int bkv)
    {
        const int qh = lane & 15, tg = lane >> 4;
        float lt = l;
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
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
            const int wave = u0_wave;
            const int slot = (mt & kMetaSlot1) ? 1 : 0;
            float* rec = p.partials + static_cast<size_t>(wave * 2 + slot) * record_floats(p.G, D);
            float* o = rec + qh * D + 4 * tg;
#pragma unroll
            for (int jd = 0; jd < D / 16; ++jd)
                *reinterpret_cast<float4*>(o + 16 * jd) = make_float4(acc[jd][0], acc[jd][1], acc[jd][2], acc[jd][3]);
            if (tg == 0) {
                rec[p.G * D + qh] = m;
                rec[p.G * D + p.G + qh] = lt;
            }
        }
    }

    int u0_wave;  // index of this wave on the work line

    template <int S>
    __device__ inline void prologue_stage(int total)
    {
        if (S < total) produce<S>();
        if constexpr (S + 1 < NS) prologue_stage<S + 1>(total);
    }

    template <int S>
    __device__ inline void round_stage(int base, int total)
    {
        const int i = base + S;
        if (i < total) {
            wait_stage<Geo::kLoadsPerStage, NS>(min(NS - 1, total - 1 - i));
            consume<S>();
            if (i + NS < total) produce<S>();
        }
        if constexpr (S + 1 < NS) round_stage<S + 1>(base, total);
    }

    __device__ inline void run()
    {
        const int total = u1 - u0;
        prologue_stage<0>(total);
        for (int base = 0; base < total; base += NS) round_stage<0>(base, total);
    }
};

template <int D, int QKB, int NS>
__global__ __launch_bounds__(kWaves * 64) void partial_mfma_kernel(Params p)
{
    using W = Wave<D, QKB, NS>;
    __shared__ __attribute__((aligned(1024))) char ring[kWaves * W::Geo::kWaveBytes];

    const int wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWaves + wave_in_block);
    const int units = uniform_load(p.header + kHdrUnits);
    const int span = uniform_load(p.header + kHdrSpan);
    const int active = uniform_load(p.header + kHdrActive);
    if (wave >= active) return;

    W w(p);
    w.lane = threadIdx.x & 63;
    w.u0_wave = wave;
    w.u0 = wave * span;
    w.u1 = min(w.u0 + span, units);
    w.lds_ptr = (lds_char*)ring + wave_in_block * W::Geo::kWaveBytes;
    w.lds_wave = static_cast<unsigned>(reinterpret_cast<uintptr_t>(w.lds_ptr));
    w.init_lane_tables();
    const i32x4 ws = uniform_load(reinterpret_cast<const i32x4*>(p.wave_start) + wave);
    w.cur.upos = w.u0;
    w.cur.r = ws.x;
    w.cur.kv = ws.y;
    w.cur.pg = ws.z;
    w.cur.seg_pg0 = ws.z;
    w.cur.st = open_stream(p, ws.x, ws.y);
    w.m = 0.f;
    w.l = 0.f;
    w.run();
}

template <int D, int QKB, int NS>
hipError_t launch(const Params& p, hipStream_t stream)
{
    hipLaunchKernelGGL((partial_mfma_kernel<D, QKB, NS>), dim3(p.slots / kWaves), dim3(kWaves * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

int mfma_waves_per_cu() { return kWaves; }
int mfma_waves_per_block() { return kWaves; }

hipError_t launch_partial_mfma(const Params& p, hipStream_t stream)
{
    // query slot of a stage: G rows of D bf16, rounded up to whole 1 KiB direct loads
    const int qkb = (p.G * p.D * 2 + 1023) / 1024;
    if (p.D == 128) {
        if (qkb <= 1) return launch<128, 1, 4>(p, stream);
        if (qkb <= 2) return launch<128, 2, 4>(p, stream);
        return launch<128, 4, 3>(p, stream);
    }
    if (qkb <= 1) return launch<64, 1, 8>(p, stream);
    return launch<64, 2, 6>(p, stream);
}

}  // namespace jd
