// Host side of libjigsaw_decode: configuration checks, the handle, the workspace and the
// launches of the entry points.  See include/jigsaw_decode.h for the contract; the inspection
// and measurement calls of include/jigsaw_decode_bench.h are at the end.
#include "../../include/jigsaw_decode_bench.h"
#include "jd_internal.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

struct jd_handle {
    jd_config cfg;
    jd::Params params;      // workspace pointers and sizes filled in; per-call pointers patched per call
    void* workspace;
    size_t workspace_bytes;
    int device;
    // the vector-ALU comparison path (jigsaw_decode_bench.h): its own tables, allocated on first use
    void* vector_workspace = nullptr;
    jd::Params vector_params;
    std::string error;
};

namespace {

thread_local std::string g_error = "no error";

// Byte offsets of the workspace arrays of the decode kernel (and of the prefill's dispatch order).
struct Layout {
    size_t header, cum, req, order, wave_start, counters, partials, total;
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

Layout make_layout(const jd_config& c, int slots)
{
    Layout l;
    size_t off = 0;
    l.header = off; off = align_up(off + sizeof(int32_t) * jd::kHeaderInts, 256);
    l.cum = off; off = align_up(off + sizeof(int32_t) * (static_cast<size_t>(c.batch) + 1), 256);
    l.req = off; off = align_up(off + sizeof(int32_t) * static_cast<size_t>(c.batch), 256);
    l.order = off; off = align_up(off + sizeof(int32_t) * static_cast<size_t>(c.batch), 256);
    l.wave_start = off; off = align_up(off + sizeof(int32_t) * 4 * static_cast<size_t>(slots), 256);
    l.counters = off;
    off = align_up(off + sizeof(int32_t) * (static_cast<size_t>(c.batch) * c.num_kv_heads + jd::cluster_records(slots)), 256);
    const int G = c.num_q_heads / c.num_kv_heads;
    l.partials = off;
    off = align_up(off + sizeof(float) * (2 * static_cast<size_t>(slots) + jd::cluster_records(slots)) * jd::record_floats(G, c.head_dim), 256);
    l.total = off;
    return l;
}

jd_status fail(jd_handle* h, jd_status st, const std::string& msg)
{
    if (h) h->error = msg;
    g_error = msg;
    return st;
}

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
    if (c->batch > jd::mfma_max_batch()) { msg = "batches up to 8192 rows are supported"; return JD_ERR_UNSUPPORTED; }
    return JD_OK;
}

// Wave slots of the decode kernel for a CU budget: one block per compute unit.
int wave_slots(int cus)
{
    int slots = jd::mfma_waves_per_cu() * cus;
    if (slots > jd::kMaxWaveSlots) slots = jd::kMaxWaveSlots;
    return slots;
}

constexpr int kAssumedCus = 256;  // MI355X; used only by the pure-host size query

// Compute units a handle spreads the decode kernel over, of `device_cus` present.
int effective_cus(const jd_config& c, int device_cus)
{
    if (c.cu_budget > 0) return c.cu_budget < device_cus ? c.cu_budget : device_cus;
    // measured: three quarters of the compute units (13/16 with 64-wide heads) already keep HBM saturated,
    // and the step is 2-4 % faster without the contention of the rest (with all units busy the dies no
    // longer get equal shares of the bandwidth and the slowest die sets the step time); the rest stay
    // free for a co-located job
    if (c.head_dim == 128) return device_cus * 3 / 4;
    return device_cus * 13 / 16;
}

// Everything of Params that does not change from call to call.
void fill_params(jd::Params& p, char* ws, const Layout& lay, const jd_config& c, int slots)
{
    std::memset(&p, 0, sizeof p);
    p.header = reinterpret_cast<int32_t*>(ws + lay.header);
    p.cum_pages = reinterpret_cast<int32_t*>(ws + lay.cum);
    p.req = reinterpret_cast<int32_t*>(ws + lay.req);
    p.order = reinterpret_cast<int32_t*>(ws + lay.order);
    p.wave_start = reinterpret_cast<int32_t*>(ws + lay.wave_start);
    p.counters = reinterpret_cast<int32_t*>(ws + lay.counters);
    p.partials = reinterpret_cast<float*>(ws + lay.partials);
    p.B = c.batch; p.Hq = c.num_q_heads; p.Hkv = c.num_kv_heads;
    p.G = p.Hq / p.Hkv; p.D = c.head_dim; p.maxp = c.max_pages_per_seq; p.NP = c.num_pages;
    p.slots = slots;
    p.wg = jd::mfma_group_waves(p.Hkv, slots);
    const double scale = c.softmax_scale > 0.f ? static_cast<double>(c.softmax_scale) : 1.0 / std::sqrt(static_cast<double>(p.D));
    p.scale_log2e = static_cast<float>(scale * 1.4426950408889634);
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

jd_status check_decode_args(jd_handle* h, const void* q, const void* k_pages, const void* v_pages,
                            const int32_t* block_table, const int32_t* seq_lens, const float* out)
{
    if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !out)
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages, block_table, seq_lens and out must be non-NULL");
    if (misaligned(q) || misaligned(k_pages) || misaligned(v_pages) || misaligned(out))
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages and out must be 16-byte aligned");
    if (misaligned4(block_table) || misaligned4(seq_lens))
        return fail(h, JD_ERR_INVALID_ARG, "block_table and seq_lens must be 4-byte aligned");
    return JD_OK;
}

// ---- the allocation-free entry point's workspace ---------------------------------------------------
// jd_decode_attention_static keeps what a handle keeps in its hipMalloc'ed workspace (partition tables,
// arrival counters, partial records) in this array instead.  Every GPU the library runs on holds its own
// copy of it, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = 12u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
struct StaticSlot {
    void* ptr = nullptr;   // device address of this GPU's copy of `scratch`
    int cus = 0;
};
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mutex;

// Zeroes what must start a call at zero: the flag word and the arrival counters.  A kernel, not a memset,
// so that a caller may capture the call into a graph.
__global__ __launch_bounds__(256) void static_clear_kernel(int32_t* header, int32_t* counters, int n_counters)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < jd::kHeaderInts) header[i] = 0;
    if (i < n_counters) counters[i] = 0;
}

// The address of the current device's copy of the scratch array and its compute-unit count, resolved
// once per device with that device current.
jd_status static_slot(int dev, hipStream_t stream, StaticSlot& out)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(nullptr, JD_ERR_UNSUPPORTED, "device index beyond the 64 the static workspace table holds");
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticSlot& slot = g_static[dev];
    if (!slot.ptr) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        hipError_t e = hipStreamIsCapturing(stream, &cap);
        if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("hipStreamIsCapturing failed: ") + hipGetErrorString(e));
        if (cap != hipStreamCaptureStatusNone)
            return fail(nullptr, JD_ERR_INVALID_ARG, "the first jd_decode_attention_static call on a device resolves the "
                        "workspace address and must come outside a stream capture");
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("no usable HIP device: ") + hipGetErrorString(e));
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return fail(nullptr, JD_ERR_UNSUPPORTED, std::string("built for gfx950, device is ") + prop.gcnArchName);
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(nullptr, JD_ERR_HIP, std::string("hipGetSymbolAddress failed: ") + hipGetErrorString(e));
        slot.cus = prop.multiProcessorCount;
        slot.ptr = ptr;
    }
    out = slot;
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
    return make_layout(*cfg, wave_slots(effective_cus(*cfg, kAssumedCus))).total;
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
    const int slots = wave_slots(effective_cus(*cfg, prop.multiProcessorCount));
    const Layout lay = make_layout(*cfg, slots);
    h->workspace_bytes = lay.total;
    e = hipMalloc(&h->workspace, lay.total);
    // the arrival counters and the flag word start at zero; the clear has completed before the handle is
    // handed out, whatever stream (blocking or not) the first call comes on
    if (e == hipSuccess) e = hipMemset(h->workspace, 0, lay.total);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (h->workspace) (void)hipFree(h->workspace);
        delete h;
        return fail(nullptr, JD_ERR_HIP, std::string("workspace allocation failed: ") + hipGetErrorString(e));
    }
    fill_params(h->params, static_cast<char*>(h->workspace), lay, *cfg, slots);
    *out = h;
    return JD_OK;
}

jd_status jd_decode_attention(jd_handle* h, const void* q, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, const int32_t* seq_lens, float* out, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (jd_status st = check_decode_args(h, q, k_pages, v_pages, block_table, seq_lens, out)) return st;
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    p.q = static_cast<const uint16_t*>(q);
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.out = out;
    // one launch: work partition, split-KV partial pass and combine
    const hipError_t e = jd::launch_fused_mfma(p, static_cast<hipStream_t>(stream), 0);
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return JD_OK;
}

jd_status jd_decode_attention_static(const jd_config* cfg, const void* q, const void* k_pages, const void* v_pages,
                                     const int32_t* block_table, const int32_t* seq_lens, float* out, void* stream)
{
    std::string msg;
    if (jd_status st = validate(cfg, msg)) return fail(nullptr, st, msg);
    if (jd_status st = check_decode_args(nullptr, q, k_pages, v_pages, block_table, seq_lens, out)) return st;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("hipGetDevice failed: ") + hipGetErrorString(e));
    hipStream_t s = static_cast<hipStream_t>(stream);
    StaticSlot slot;
    if (jd_status st = static_slot(dev, s, slot)) return st;
    const int slots = wave_slots(effective_cus(*cfg, slot.cus));
    const Layout lay = make_layout(*cfg, slots);
    if (lay.total > kStaticScratchBytes)
        return fail(nullptr, JD_ERR_UNSUPPORTED, "this configuration needs " + std::to_string(lay.total) +
                    " bytes of workspace, the static array holds " + std::to_string(kStaticScratchBytes) +
                    " (use a handle, or a smaller cu_budget)");
    jd::Params p;
    fill_params(p, static_cast<char*>(slot.ptr), lay, *cfg, slots);
    p.q = static_cast<const uint16_t*>(q);
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.out = out;
    // the array keeps the last call's contents, and that call may have had another configuration
    const int n_counters = p.B * p.Hkv + jd::cluster_records(p.slots);
    const int n_clear = n_counters > jd::kHeaderInts ? n_counters : jd::kHeaderInts;
    hipLaunchKernelGGL(static_clear_kernel, dim3((n_clear + 255) / 256), dim3(256), 0, s, p.header, p.counters, n_counters);
    e = hipGetLastError();
    if (e == hipSuccess) e = jd::launch_fused_mfma(p, s, 0);
    if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
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
                               const int32_t* q_offsets, int32_t total_q_rows, int32_t max_q_len, float* out,
                               void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!q || !k_pages || !v_pages || !block_table || !seq_lens || !q_lens || !q_offsets || !out)
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages, block_table, seq_lens, q_lens, q_offsets and out must be non-NULL");
    if (misaligned(q) || misaligned(k_pages) || misaligned(v_pages) || misaligned(out))
        return fail(h, JD_ERR_INVALID_ARG, "q, k_pages, v_pages and out must be 16-byte aligned");
    if (misaligned4(block_table) || misaligned4(seq_lens) || misaligned4(q_lens) || misaligned4(q_offsets))
        return fail(h, JD_ERR_INVALID_ARG, "block_table, seq_lens, q_lens and q_offsets must be 4-byte aligned");
    if (max_q_len < 0) return fail(h, JD_ERR_INVALID_ARG, "max_q_len must be >= 0");
    if (total_q_rows < 0) return fail(h, JD_ERR_INVALID_ARG, "total_q_rows must be >= 0");
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
    hipError_t e = jd::launch_prefill(p, static_cast<const uint16_t*>(q), q_lens, q_offsets, total_q_rows, max_q_len, out,
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
        if (flag & jd::kBadLength) msg += " a sequence length exceeds 16 * max_pages_per_seq (clamped);";
        if (flag & jd::kBadPage) msg += " a block-table entry lies outside [0, num_pages) (page 0 read instead, or the append skipped);";
        if (flag & jd::kBadLensMoved) msg += " seq_lens changed while a decode kernel was running (its rows are meaningless);";
        if (flag & jd::kBadQueryRows) msg += " a prefill request's query rows leave [0, total_q_rows) (request skipped);";
        return fail(h, JD_ERR_BAD_INPUT, msg);
    }
    return JD_OK;
}

jd_status jd_destroy(jd_handle* h)
{
    if (!h) return JD_OK;
    hipError_t e = hipFree(h->workspace);
    if (h->vector_workspace) {
        const hipError_t e2 = hipFree(h->vector_workspace);
        if (e == hipSuccess) e = e2;
    }
    delete h;
    if (e != hipSuccess) return fail(nullptr, JD_ERR_HIP, std::string("hipFree failed: ") + hipGetErrorString(e));
    return JD_OK;
}

const char* jd_last_error_string(const jd_handle* h)
{
    return h ? (h->error.empty() ? "no error" : h->error.c_str()) : g_error.c_str();
}

// ---- inspection and measurement (include/jigsaw_decode_bench.h) ------------------------------------

jd_status jd_debug_partition(jd_handle* h, const int32_t* seq_lens, int32_t* header_host,
                             int32_t* wave_start_host, int32_t* cum_pages_host, void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (!seq_lens) return fail(h, JD_ERR_INVALID_ARG, "seq_lens is NULL");
    if (jd_status st = check_device(h)) return st;
    jd::Params p = h->params;
    p.seq_lens = seq_lens;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = jd::launch_fused_mfma(p, s, 1);
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
            if (w >= active_waves) r[0] = r[1] = r[2] = 0;
            r[3] = 0;
        }
    }
    return JD_OK;
}

jd_status jd_debug_schedule(int32_t units, int32_t groups, int32_t out[2])
{
    if (units < 0 || groups <= 0 || !out) return fail(nullptr, JD_ERR_INVALID_ARG, "units >= 0, groups > 0 and out != NULL required");
    out[0] = jd::span_for(units, groups);
    out[1] = (units + out[0] - 1) / out[0];
    return JD_OK;
}

int32_t jd_wave_slots(const jd_handle* h) { return h ? h->params.slots : 0; }

jd_status jd_bench_decode_attention_vector(jd_handle* h, const void* q, const void* k_pages, const void* v_pages,
                                           const int32_t* block_table, const int32_t* seq_lens, float* out,
                                           void* stream)
{
    if (!h) return fail(nullptr, JD_ERR_INVALID_ARG, "handle is NULL");
    if (jd_status st = check_decode_args(h, q, k_pages, v_pages, block_table, seq_lens, out)) return st;
    if (jd_status st = check_device(h)) return st;
    const int G = h->cfg.num_q_heads / h->cfg.num_kv_heads;
    if (!(G == 1 || G == 2 || G == 4 || G == 7 || G == 8))
        return fail(h, JD_ERR_UNSUPPORTED, "the vector-ALU kernels support group sizes 1, 2, 4, 7 and 8");
    if (!h->vector_workspace) {
        int cus = 0;
        hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device);
        if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("hipDeviceGetAttribute failed: ") + hipGetErrorString(e));
        if (h->cfg.cu_budget > 0 && h->cfg.cu_budget < cus) cus = h->cfg.cu_budget;
        int slots = jd::vector_waves_per_cu() * cus;
        if (slots > jd::kMaxWaveSlots) slots = jd::kMaxWaveSlots;
        // same arrays as the decode kernel's workspace plus the rank table, in one allocation
        const Layout lay = make_layout(h->cfg, slots);
        const size_t rank_off = lay.total;
        const size_t total = align_up(rank_off + sizeof(int32_t) * static_cast<size_t>(h->cfg.batch), 256);
        e = hipMalloc(&h->vector_workspace, total);
        if (e == hipSuccess) e = hipMemset(h->vector_workspace, 0, total);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            if (h->vector_workspace) (void)hipFree(h->vector_workspace);
            h->vector_workspace = nullptr;
            return fail(h, JD_ERR_HIP, std::string("workspace allocation failed: ") + hipGetErrorString(e));
        }
        fill_params(h->vector_params, static_cast<char*>(h->vector_workspace), lay, h->cfg, slots);
        h->vector_params.rank = reinterpret_cast<int32_t*>(static_cast<char*>(h->vector_workspace) + rank_off);
        h->vector_params.wg = 1;
        // both paths report through the flag word jd_check_device_flags reads (calls on a handle are
        // stream-ordered, and the decode kernel reads nothing else of the header)
        h->vector_params.header = h->params.header;
    }
    jd::Params p = h->vector_params;
    p.q = static_cast<const uint16_t*>(q);
    p.k_pages = static_cast<const uint16_t*>(k_pages);
    p.v_pages = static_cast<const uint16_t*>(v_pages);
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.out = out;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = jd::launch_partition(p, s);
    if (e == hipSuccess) e = jd::launch_partial_vector(p, s);
    if (e == hipSuccess) e = jd::launch_combine(p, s);
    if (e != hipSuccess) return fail(h, JD_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return JD_OK;
}

}  // extern "C"
