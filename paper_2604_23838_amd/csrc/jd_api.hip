// Host side of libjigsaw_decode: configuration checks, the handle, the workspace and the
// three launches of one decode step.  See include/jigsaw_decode.h for the contract.
#include "../../include/jigsaw_decode.h"
#include "jd_internal.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

struct jd_handle {
    jd_config cfg;
    jd::Params params;      // workspace pointers and sizes filled in; per-call pointers patched per call
    void* workspace;
    size_t workspace_bytes;
    int variant;            // resolved: JD_VARIANT_VECTOR or JD_VARIANT_MFMA
    int device;
    std::vector<hipEvent_t> events;  // 4 per profiled call
    int prof_max = 0, prof_calls = 0, prof_every = 1, prof_seen = 0;
    std::string error;
};

namespace {

thread_local std::string g_error = "no error";

struct Layout {
    size_t header, cum, rank, req, wave_start, counters, partials, total;
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Layout make_layout(const jd_config& c, int slots)
{
    Layout l;
    size_t off = 0;
    l.header = off; off = align_up(off + sizeof(int32_t) * jd::kHeaderInts, 256);
    l.cum = off; off = align_up(off + sizeof(int32_t) * (static_cast<size_t>(c.batch) + 1), 256);
    l.rank = off; off = align_up(off + sizeof(int32_t) * static_cast<size_t>(c.batch), 256);
    l.req = off; off = align_up(off + sizeof(int32_t) * static_cast<size_t>(c.batch), 256);
    l.wave_start = off; off = align_up(off + sizeof(int32_t) * 4 * static_cast<size_t>(slots), 256);
    l.counters = off; off = align_up(off + sizeof(int32_t) * static_cast<size_t>(c.batch) * c.num_kv_heads, 256);
    const int G = c.num_q_heads / c.num_kv_heads;
    l.partials = off;
    off = align_up(off + sizeof(float) * 2 * static_cast<size_t>(slots) * jd::record_floats(G, c.head_dim), 256);
    l.total = off;
    return l;
}

jd_status fail(jd_handle* h, jd_status st, const std::string& msg)
{
    if (h) h->error = msg;
    g_error = msg;
    return st;
}

bool vector_supports(int G) { return G == 1 || G == 2 || G == 4 || G == 7 || G == 8; }

jd_status validate(const jd_config* c, std::string& msg)
{
    if (!c) { msg = "config is NULL"; return JD_ERR_INVALID_ARG; }
    if (c->batch <= 0 || c->num_q_heads <= 0 || c->num_kv_heads <= 0 || c->max_pages_per_seq <= 0 || c->num_pages <= 0) {
        msg = "batch, head counts, max_pages_per_seq and num_pages must be positive";
        return JD_ERR_INVALID_ARG;
    }
    if (c->num_q_heads % c->num_kv_heads) { msg = "num_kv_heads must divide num_q_heads"; return JD_ERR_INVALID_ARG; }
    if (!(c->softmax_scale >= 0.f) || std::isinf(c->softmax_scale)) { msg = "softmax_scale must be finite and >= 0"; return JD_ERR_INVALID_ARG; }
    if (c->cu_budget < 0) { msg = "cu_budget must be >= 0"; return JD_ERR_INVALID_ARG; }
    const long long line = static_cast<long long>(c->batch) * c->max_pages_per_seq * c->num_kv_heads;
    if (line >= (1ll << 31)) { msg = "batch * max_pages_per_seq * num_kv_heads must stay below 2^31"; return JD_ERR_INVALID_ARG; }
    if (static_cast<long long>(c->batch) * c->num_q_heads >= (1ll << 31)) { msg = "batch * num_q_heads must stay below 2^31"; return JD_ERR_INVALID_ARG; }
    if (static_cast<long long>(c->num_pages) * c->num_kv_heads >= (1ll << 31)) { msg = "num_pages * num_kv_heads must stay below 2^31"; return JD_ERR_INVALID_ARG; }
    if (c->head_dim != 64 && c->head_dim != 128) { msg = "head_dim must be 64 or 128"; return JD_ERR_UNSUPPORTED; }
    if (c->page_size != jd::kPage) { msg = "page_size must be 16"; return JD_ERR_UNSUPPORTED; }
    const int G = c->num_q_heads / c->num_kv_heads;
    if (G > 16) { msg = "group size num_q_heads / num_kv_heads must be <= 16"; return JD_ERR_UNSUPPORTED; }
    if (c->variant != JD_VARIANT_DEFAULT && c->variant != JD_VARIANT_VECTOR && c->variant != JD_VARIANT_MFMA) {
        msg = "unknown variant"; return JD_ERR_UNSUPPORTED;
    }
    if (c->variant == JD_VARIANT_VECTOR && !vector_supports(G)) {
        msg = "the vector variant supports group sizes 1, 2, 4, 7 and 8"; return JD_ERR_UNSUPPORTED;
    }
    if (c->variant != JD_VARIANT_VECTOR && c->batch > jd::mfma_max_batch()) {
        msg = "the matrix-core variant supports batches up to 8192"; return JD_ERR_UNSUPPORTED;
    }
    return JD_OK;
}

int resolve_variant(const jd_config& c)
{
    if (c.variant != JD_VARIANT_DEFAULT) return c.variant;
    return JD_VARIANT_MFMA;  // measured faster than the vector variant on every benchmark shape
}

// Wave slots for a handle: waves per CU of the variant times the CU budget, a multiple of the block size.
int wave_slots(int variant, int cus)
{
    const int per_cu = variant == JD_VARIANT_VECTOR ? jd::vector_waves_per_cu() : jd::mfma_waves_per_cu();
    int slots = per_cu * cus;
    if (slots > jd::kMaxWaveSlots) slots = jd::kMaxWaveSlots;
    return slots;
}

constexpr int kAssumedCus = 256;  // MI355X; used only by the pure-host size query

// Compute units a handle spreads the partial pass over, of `device_cus` present.
int effective_cus(const jd_config& c, int variant, int device_cus)
{
    if (c.cu_budget > 0) return c.cu_budget < device_cus ? c.cu_budget : device_cus;
    // measured: with 128-wide heads three quarters of the compute units already keep HBM saturated,
    // and the step is 2-3 % faster without the contention of the rest (which stay free for a co-located job)
    if (variant == JD_VARIANT_MFMA && c.head_dim == 128) return device_cus * 3 / 4;
    return device_cus;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

// The workspace and the kernels' launches belong to the device the handle was created on.
jd_status check_device(jd_handle* h)
{
    int dev = -1;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("hipGetDevice failed: ") + hipGetErrorString(e));
    if (dev != h->device)
        return fail(h, JD_ERR_INVALID_ARG, "the current HIP device is not the one the handle was created on");
    return JD_OK;
}

}  // namespace

extern "C" {

jd_status jd_validate_config(const jd_config* cfg)
{
    std::string msg;
    jd_status st = validate(cfg, msg);
    if (st != JD_OK) return fail(nullptr, st, msg);
    return JD_OK;
}

size_t jd_workspace_bytes(const jd_config* cfg)
{
    std::string msg;
    if (validate(cfg, msg) != JD_OK) return 0;
    const int variant = resolve_variant(*cfg);
    return make_layout(*cfg, wave_slots(variant, effective_cus(*cfg, variant, kAssumedCus))).total;
}

jd_status jd_create(const jd_config* cfg, jd_handle** out)
{
    if (!out) return fail(nullptr, JD_ERR_INVALID_ARG, "out handle pointer is NULL");
    std::string msg;
    jd_status st = validate(cfg, msg);
    if (st != JD_OK) return fail(nullptr, st, msg);

    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    hipDeviceProp_t prop;
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("no usable HIP device: ") + hipGetErrorString(e));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(nullptr, JD_ERR_UNSUPPORTED, std::string("built for gfx950, device is ") + prop.gcnArchName);

    jd_handle* h = new (std::nothrow) jd_handle();
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "out of host memory");
    h->cfg = *cfg;
    h->device = dev;
    h->variant = resolve_variant(*cfg);
    const int cus = effective_cus(*cfg, h->variant, prop.multiProcessorCount);
    const int slots = wave_slots(h->variant, cus);
    const Layout lay = make_layout(*cfg, slots);
    h->workspace_bytes = lay.total;
    e = hipMalloc(&h->workspace, lay.total);
    if (e == hipSuccess) e = hipMemset(h->workspace, 0, lay.total);
    if (e != hipSuccess) {
        if (h->workspace) (void)hipFree(h->workspace);
        delete h;
        return fail(nullptr, JD_ERR_HIP, std::string("workspace allocation failed: ") + hipGetErrorString(e));
    }
    char* ws = static_cast<char*>(h->workspace);
    jd::Params& p = h->params;
    std::memset(&p, 0, sizeof p);
    p.header = reinterpret_cast<int32_t*>(ws + lay.header);
    p.cum_pages = reinterpret_cast<int32_t*>(ws + lay.cum);
    p.rank = reinterpret_cast<int32_t*>(ws + lay.rank);
    p.req = reinterpret_cast<int32_t*>(ws + lay.req);
    p.wave_start = reinterpret_cast<int32_t*>(ws + lay.wave_start);
    p.counters = reinterpret_cast<int32_t*>(ws + lay.counters);
    p.partials = reinterpret_cast<float*>(ws + lay.partials);
    p.B = cfg->batch; p.Hq = cfg->num_q_heads; p.Hkv = cfg->num_kv_heads;
    p.G = p.Hq / p.Hkv; p.D = cfg->head_dim; p.maxp = cfg->max_pages_per_seq; p.NP = cfg->num_pages;
    p.slots = slots;
    p.wg = h->variant == JD_VARIANT_VECTOR ? 1 : jd::mfma_group_waves(p.Hkv);
    const double scale = cfg->softmax_scale > 0.f ? static_cast<double>(cfg->softmax_scale) : 1.0 / std::sqrt(static_cast<double>(p.D));
    p.scale_log2e = static_cast<float>(scale * 1.4426950408889634);
    *out = h;
    return JD_OK;
}

jd_status jd_decode_attention(jd_handle* h, const void* q, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, const int32_t* seq_lens, float* out, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !out)
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages, block_table, seq_lens and out must be non-NULL");
    if (misaligned(q) || misaligned(k_pages) || misaligned(v_pages) || misaligned(out))
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages and out must be 16-byte aligned");
    if (misaligned4(block_table) || misaligned4(seq_lens))
        return fail(h, JD_ERR_INVALID_ARG, "block_table and seq_lens must be 4-byte aligned");
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    p.q = static_cast<const uint16_t*>(q);
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.out = out;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t* ev = (h->prof_calls < h->prof_max && h->prof_seen++ % h->prof_every == 0) ? &h->events[4 * h->prof_calls] : nullptr;
    const bool fused = h->variant != JD_VARIANT_VECTOR;  // one launch does partition, partial pass and combine
    hipError_t e = ev ? hipEventRecord(ev[0], s) : hipSuccess;
    if (e == hipSuccess && !fused) e = jd::launch_partition(p, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[1], s);
    if (e == hipSuccess) e = fused ? jd::launch_fused_mfma(p, s, 0) : jd::launch_partial_vector(p, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[2], s);
    if (e == hipSuccess && !fused) e = jd::launch_combine(p, s);
    if (e == hipSuccess && ev) { e = hipEventRecord(ev[3], s); ++h->prof_calls; }
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return JD_OK;
}

jd_status jd_append_kv(jd_handle* h, const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                       const int32_t* block_table, int32_t* seq_lens, const int32_t* active, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!k_new || !v_new || !k_pages || !v_pages || !block_table || !seq_lens)
        return fail(h, JD_ERR_INVALID_ARG, "k_new, v_new, k_pages, v_pages, block_table and seq_lens must be non-NULL");
    if (misaligned(k_new) || misaligned(v_new) || misaligned(k_pages) || misaligned(v_pages))
        return fail(h, JD_ERR_INVALID_ARG, "k_new, v_new, k_pages and v_pages must be 16-byte aligned");
    if (misaligned4(block_table) || misaligned4(seq_lens) || misaligned4(active))
        return fail(h, JD_ERR_INVALID_ARG, "block_table, seq_lens and active must be 4-byte aligned");
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    p.block_table = block_table;
    hipError_t e = jd::launch_append_kv(p, static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                                        static_cast<uint16_t*>(k_pages), static_cast<uint16_t*>(v_pages), seq_lens,
                                        active, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return JD_OK;
}

jd_status jd_prefill_attention(jd_handle* h, const void* q, const void* k_pages, const void* v_pages,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* q_lens,
                               const int32_t* q_offsets, int32_t max_q_len, float* out, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !q_lens || !q_offsets || !out)
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets and out must be non-NULL");
    if (misaligned(q) || misaligned(k_pages) || misaligned(v_pages) || misaligned(out))
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages and out must be 16-byte aligned");
    if (misaligned4(block_table) || misaligned4(seq_lens) || misaligned4(q_lens) || misaligned4(q_offsets))
        return fail(h, JD_ERR_INVALID_ARG, "block_table, seq_lens, q_lens and q_offsets must be 4-byte aligned");
    if (max_q_len < 0) return fail(h, JD_ERR_INVALID_ARG, "max_q_len must be >= 0");
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    // a request never has more new tokens than its table holds; the launch is sized for the bound
    const int64_t cap = static_cast<int64_t>(p.maxp) * jd::kPage;
    if (max_q_len > cap) max_q_len = static_cast<int32_t>(cap);
    if (cap * p.G > 0x7fffffff) return fail(h, JD_ERR_UNSUPPORTED, "max_pages_per_seq x 16 x group size exceeds the row index range");
    const int64_t blocks = static_cast<int64_t>(jd::prefill_query_blocks(max_q_len, p.G)) * p.B * p.Hkv;
    if (blocks > 0x7fffffff) return fail(h, JD_ERR_UNSUPPORTED, "batch x kv heads x query blocks exceeds the launch limit");
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    hipError_t e = jd::launch_prefill(p, static_cast<const uint16_t*>(q), q_lens, q_offsets, max_q_len, out,
                                      static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return JD_OK;
}

jd_status jd_check_device_flags(jd_handle* h, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (jd_status st = check_device(h)) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, h->params.header + jd::kHdrBadInput, sizeof flag, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess && flag) e = hipMemsetAsync(h->params.header + jd::kHdrBadInput, 0, sizeof flag, s);
    if (e == hipSuccess && flag) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("reading device flags failed: ") + hipGetErrorString(e));
    if (flag) {
        std::string msg = "device-side input check failed:";
        if (flag & 1) msg += " a sequence length exceeds 16 * max_pages_per_seq (clamped);";
        if (flag & 2) msg += " a block-table entry lies outside [0, num_pages) (page 0 read instead);";
        return fail(h, JD_ERR_BAD_INPUT, msg);
    }
    return JD_OK;
}

jd_status jd_debug_partition(jd_handle* h, const int32_t* seq_lens, int32_t* header_host,
                             int32_t* wave_start_host, int32_t* cum_pages_host, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!seq_lens) return fail(h, JD_ERR_INVALID_ARG, "seq_lens is NULL");
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    p.seq_lens = seq_lens;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = h->variant == JD_VARIANT_VECTOR ? jd::launch_partition(p, s) : jd::launch_fused_mfma(p, s, 1);
    int32_t hdr[8] = {0};
    if (e == hipSuccess) e = hipMemcpyAsync(hdr, p.header, sizeof hdr, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess && wave_start_host)
        e = hipMemcpyAsync(wave_start_host, p.wave_start, sizeof(int32_t) * 4 * p.slots, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess && cum_pages_host)
        e = hipMemcpyAsync(cum_pages_host, p.cum_pages, sizeof(int32_t) * (p.B + 1), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("partition failed: ") + hipGetErrorString(e));
    if (header_host) {
        std::memcpy(header_host, hdr, sizeof hdr);
        header_host[4] = hdr[jd::kHdrGroup];
        header_host[5] = header_host[6] = header_host[7] = 0;
    }
    if (wave_start_host) {  // report {request, kv head, page, 0}
        const int active_waves = hdr[jd::kHdrActive] * hdr[jd::kHdrGroup];
        for (int w = 0; w < p.slots; ++w) {
            int32_t* r = wave_start_host + 4 * w;
            r[0] = w < active_waves ? r[3] : 0;
            if (w >= active_waves) r[1] = r[2] = 0;
            r[3] = 0;
        }
    }
    return JD_OK;
}

jd_status jd_profile_enable(jd_handle* h, int32_t max_calls, int32_t every)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (max_calls < 0 || max_calls > (1 << 20) || every < 1) return fail(h, JD_ERR_INVALID_ARG, "max_calls or every out of range");
    for (hipEvent_t ev : h->events) (void)hipEventDestroy(ev);
    h->events.clear();
    h->prof_max = h->prof_calls = 0;
    for (int i = 0; i < 4 * max_calls; ++i) {
        hipEvent_t ev;
        hipError_t e = hipEventCreate(&ev);
        if (e != hipSuccess) {
            for (hipEvent_t x : h->events) (void)hipEventDestroy(x);
            h->events.clear();
            return fail(h, JD_ERR_HIP, std::string("hipEventCreate failed: ") + hipGetErrorString(e));
        }
        h->events.push_back(ev);
    }
    h->prof_max = max_calls;
    h->prof_every = every;
    h->prof_seen = 0;
    return JD_OK;
}

jd_status jd_profile_read(jd_handle* h, float ms_sum[3], int32_t* calls)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!ms_sum || !calls) return fail(h, JD_ERR_INVALID_ARG, "ms_sum and calls must be non-NULL");
    ms_sum[0] = ms_sum[1] = ms_sum[2] = 0.f;
    *calls = h->prof_calls;
    if (h->prof_calls == 0) return JD_OK;
    hipError_t e = hipEventSynchronize(h->events[4 * h->prof_calls - 1]);
    for (int c = 0; c < h->prof_calls && e == hipSuccess; ++c)
        for (int k = 0; k < 3 && e == hipSuccess; ++k) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, h->events[4 * c + k], h->events[4 * c + k + 1]);
            ms_sum[k] += ms;
        }
    h->prof_calls = 0;
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("reading event times failed: ") + hipGetErrorString(e));
    return JD_OK;
}

jd_status jd_debug_schedule(int32_t units, int32_t wave_slots, int32_t out[2])
{
    if (units < 0 || wave_slots <= 0 || !out) return fail(nullptr, JD_ERR_INVALID_ARG, "units >= 0, wave_slots > 0 and out != NULL required");
    out[0] = jd::span_for(units, wave_slots);
    out[1] = (units + out[0] - 1) / out[0];
    return JD_OK;
}

int32_t jd_wave_slots(const jd_handle* h) { return h ? h->params.slots : 0; }

jd_status jd_destroy(jd_handle* h)
{
    if (!h) return JD_OK;
    for (hipEvent_t ev : h->events) (void)hipEventDestroy(ev);
    hipError_t e = hipFree(h->workspace);
    delete h;
    if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("hipFree failed: ") + hipGetErrorString(e));
    return JD_OK;
}

const char* jd_last_error_string(const jd_handle* h)
{
    return h ? (h->error.empty() ? "no error" : h->error.c_str()) : g_error.c_str();
}

}  // extern "C"
