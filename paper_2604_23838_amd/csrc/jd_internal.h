// Internal declarations shared by the translation units of libjigsaw_decode.
// Nothing here is part of the C ABI (see include/jigsaw_decode.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jd {

constexpr int kPage = 16;          // tokens per KV page
constexpr int kMinSpan = 16;       // smallest share of work (page-units) a wave is given
constexpr int kMaxWaveSlots = 4096;
constexpr int kHeaderInts = 64;

// Header words of the work-partition table (device, int32).
enum HeaderWord {
    kHdrUnits = 0,      // page-units of work: sum_b ceil(L_b/16) * Hkv
    kHdrSpan = 1,       // page-units per wave
    kHdrActive = 2,     // waves that own at least one unit
    kHdrSlots = 3,      // wave slots the partial pass is launched with
    kHdrNonEmpty = 4,   // requests with at least one token
    kHdrBadInput = 5,   // sticky flags, see BadInputBit
    kHdrGroup = 6,      // waves per group (fused kernel; 1 = every wave on its own)
};

// Bits of the sticky device-side input-check word header[kHdrBadInput].
enum BadInputBit {
    kBadLength = 1,      // a sequence length beyond 16 * max_pages_per_seq (clamped)
    kBadPage = 2,        // a block-table entry outside [0, num_pages) (page 0 read / append skipped)
    kBadLensMoved = 4,   // seq_lens changed while the decode kernel was walking it
    kBadQueryRows = 8,   // a prefill request whose query rows leave [0, total_q_rows) (skipped)
};

// Device pointers and sizes every kernel receives by value.
struct Params {
    const uint16_t* q;          // bf16 [B, Hq, D]
    const uint16_t* k_pages;    // bf16 [NP, Hkv, 16, D]
    const uint16_t* v_pages;    // bf16 [NP, Hkv, 16, D]
    const int32_t* block_table; // [B, MAXP]
    const int32_t* seq_lens;    // [B]
    float* out;                 // fp32 [B, Hq, D]
    // workspace
    int32_t* header;            // [kHeaderInts]
    int32_t* cum_pages;         // [B + 1] exclusive prefix of pages per request
    int32_t* rank;              // [B] index of request b among the non-empty ones (vector-ALU kernels only)
    int32_t* req;               // [B] request id of the r-th non-empty request
    int32_t* order;             // [B] requests by decreasing prefill work
    int32_t* wave_start;        // [slots * 4] {r, kv, page, 0}
    float* partials;            // [slots * 2 + cluster_records(slots)] records, record_floats(G, D) floats apart: G*D accumulator
                                // values, then m and l of the G rows; two per wave, then the clusters' records
    int32_t* counters;          // [B * Hkv + cluster_records(slots)] arrival counters of the fused kernel, per stream and then
                                // per cluster record (zero between calls)
    int32_t B, Hq, Hkv, G, D, maxp, NP, slots;
    int32_t wg;                 // waves per group in the fused kernel (divides Hkv and slots)
    float scale_log2e;          // softmax_scale * log2(e): scores are kept in the exp2 domain
};

// Page-units per wave for a work line of `units`, and the number of waves that get any.
inline __host__ __device__ int span_for(int units, int slots)
{
    int span = (units + slots - 1) / slots;
    return span < kMinSpan ? kMinSpan : span;
}

// The merge of a stream longer than kFlatMergePieces - 1 spans (kFlatMergePieces pieces or more) goes in two levels: the pieces of
// each cluster of kMergeCluster consecutive wave groups are merged, by the last wave of the cluster to finish,
// into one record of the same format, and the last cluster to finish merges those.  A cluster holds at most two
// such parts per wave of a group: of a stream that began before the cluster (side 0) and of one that begins in
// it and goes on beyond it (side 1).  cluster_records(slots) bounds ((cluster * wg + member) * 2 + side) + 1.
constexpr int kMergeCluster = 8;
constexpr int kFlatMergePieces = 16;
inline __host__ __device__ int cluster_records(int slots) { return 2 * (slots / kMergeCluster) + 16; }

// Floats from one partial record to the next: G*D accumulator values, then G (m, l) pairs, rounded up to a whole
// number of 16-byte units (the merge copies records 16 bytes a lane).
inline __host__ __device__ int record_floats(int G, int D) { return (G * (D + 2) + 3) & ~3; }

// Launchers (each enqueues on `stream` and returns hipGetLastError()).
hipError_t launch_partition(const Params& p, hipStream_t stream);
hipError_t launch_partial_vector(const Params& p, hipStream_t stream);
hipError_t launch_fused_mfma(const Params& p, hipStream_t stream, int partition_only);
int mfma_max_batch();
int mfma_group_waves(int num_kv_heads, int slots);
hipError_t launch_combine(const Params& p, hipStream_t stream);
hipError_t launch_append_kv(const Params& p, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pages,
                            uint16_t* v_pages, int32_t* seq_lens, const int32_t* active, hipStream_t stream);

hipError_t launch_prefill(const Params& p, const uint16_t* q, const int32_t* q_lens, const int32_t* q_offsets,
                          int total_q_rows, int max_q_len, float* out, hipStream_t stream);
int prefill_query_blocks(int max_q_len, int G);

// Wave slots each variant wants per compute unit.
int vector_waves_per_cu();
int mfma_waves_per_cu();
int vector_waves_per_block();
int mfma_waves_per_block();

}  // namespace jd
