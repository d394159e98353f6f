// Internal declarations shared by the C-ABI translation unit and the kernel files.
// Not part of the public boundary (that is include/matkv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "matkv.h"

namespace matkv {

// Query heads per KV head the kernels are instantiated for (3: Llama-3.2-3B's 24 / 8).
inline bool group_size_built(int g) { return g == 1 || g == 2 || g == 3 || g == 4 || g == 8; }

// ---------------------------------------------------------------- cache table (device) ----
// One table describes the assembled cache of a batch (paper Section IV, put_KV): for each
// instance its pages cut into work items, then one item for its tail.  Built on the host by
// matkv_assemble, read by the attention and tail-materialize kernels.

constexpr int kMaxDecodeUnitsPerInstance = 256;
constexpr int kDecodeCounterStride = 32;         // ints: decode arrival counters sit 128 bytes apart
constexpr int kMaxPrefillUnitsPerInstance = 32;
constexpr int kMaxPrefillItemsPerUnit = 64;      // item list the matrix-core prefill kernel keeps in LDS

struct Item {              // 32 bytes: a run of tokens inside one page, or the tail
    uint64_t base;         // device address of the page's blob; 0 = the instance's tail
    int32_t page_tokens;   // tokens of the whole page (stride of a head inside the blob)
    int32_t tok0;          // first token of this piece
    int32_t ntok;          // tokens of this piece (tail: capacity, clipped by tail_len)
    int32_t fmt;           // matkv_page_format of the page
    int32_t scales16;      // compressed page: byte offset of its scale table inside the blob, / 16
    int32_t umask;         // shared decode units: bit k = the unit's k-th user sees this piece
};

struct Unit {              // 64 bytes: the work of one workgroup = consecutive items of one instance
    int32_t inst;
    int32_t item0;         // global index of the first item
    int32_t n_items;
    int32_t idx_in_inst;
    int32_t n_units_inst;  // units of this instance in this partition
    int32_t unit0_inst;    // global index of the instance's first unit
    int32_t has_tail;      // the last item is the tail
    int32_t page_tokens;   // token rows of the unit's page items together
    Item first;            // copy of items[item0]: one fetch is enough to start streaming
};

// A shared decode unit (instances of a batch that retrieved the same chunk read it once): a run
// of pieces of the batch's distinct pages (and at most one tail) and the instances whose newest
// tokens attend to some of them in this workgroup; Item::umask says which of the unit's users
// see a piece.  Every (unit, user) pair owns one partial slot of that user; an instance's slots
// are consecutive (InstanceInfo::sslot0 .. + n_sslots).
constexpr int kMaxSharedUsers = 16;             // rows of one matrix tile / smallest group size
constexpr int kMaxSharedUnitsPerInstance = 64;  // table capacity per instance of max_batch

struct SUnit {             // 208 bytes
    Unit u;                // its pieces (pages of several users, at most one tail: u.inst names that tail's instance)
    int32_t n_users;
    int32_t pad[3];
    struct { int32_t inst, slot; } users[kMaxSharedUsers];
};

struct InstanceInfo {      // 48 bytes
    int64_t pos_base;      // position of tail row 0
    int32_t tail_len;      // valid tail rows (advanced on the device)
    int32_t q_len;         // question rows
    int32_t cu_q;          // first row of this instance in the packed Q / O / hidden
    int32_t dunit0, n_dunits;   // decode units of this instance (global unit index, count)
    int32_t punit0, n_punits;   // prefill units
    int32_t sslot0, n_sslots;   // shared decode partition: this instance's partial slots
    int32_t pad;
};

struct TableHeader {       // 64 bytes
    int32_t batch;
    int32_t n_items;
    int32_t n_dunits;
    int32_t n_punits;
    int32_t total_q;
    int32_t max_q;
    int32_t pad[10];
};

// Byte offsets of the table's sections, all derived from the configuration.
struct TableLayout {
    size_t off_inst, off_items, off_dunits, off_punits, off_sunits, bytes;
    int max_items, max_dunits, max_punits, max_sunits;
};

inline TableLayout table_layout(const matkv_config& c) {
    TableLayout L;
    // every unit boundary and every page boundary starts a new item, in both partitions
    // (and once more for the private runs of the shared decode partition)
    L.max_items = c.max_batch * (kMaxDecodeUnitsPerInstance + kMaxPrefillUnitsPerInstance + kMaxDecodeUnitsPerInstance / 2 + 3 * c.max_pages + 4);
    L.max_dunits = c.max_batch * kMaxDecodeUnitsPerInstance;
    L.max_punits = c.max_batch * kMaxPrefillUnitsPerInstance;
    size_t o = sizeof(TableHeader);
    L.off_inst = o;   o += sizeof(InstanceInfo) * (size_t)c.max_batch;
    o = (o + 63) & ~(size_t)63;
    L.off_items = o;  o += sizeof(Item) * (size_t)L.max_items;
    L.off_dunits = o; o += sizeof(Unit) * (size_t)L.max_dunits;
    L.off_punits = o; o += sizeof(Unit) * (size_t)L.max_punits;
    L.max_sunits = c.max_batch * (kMaxSharedUnitsPerInstance + 1);
    L.off_sunits = o; o += sizeof(SUnit) * (size_t)L.max_sunits;
    L.bytes = (o + 255) & ~(size_t)255;
    return L;
}

// The one-instance table of a chunk's own prefill attention (matkv_chunk_attn): the chunk is
// an instance without pages whose "tail" is the chunk's K/V of one layer inside its blob.
constexpr size_t kChunkOffInst = 0, kChunkOffItem = 64, kChunkOffUnit = 128, kChunkTableBytes = 256;

// ---------------------------------------------------------------- workspace (device) ------
// [ rope table | chunk table | counters | partials ]
struct WorkspaceLayout {
    size_t off_rope, off_chunk, off_counters, off_partials, bytes;
    size_t n_counters, partial_floats;
};

inline int max_q_rows(const matkv_config& c) { return c.max_tail_tokens; }
constexpr int kSplitTiles = 128;    // half the compute units: two workgroups per tile

inline WorkspaceLayout workspace_layout(const matkv_config& c) {
    WorkspaceLayout W;
    size_t o = 0;
    W.off_rope = o;      o += 4096;   // D/2 entries of {double inv_freq; float hi, lo (turns)}
    W.off_chunk = o;     o += kChunkTableBytes;
    W.off_counters = o;
    // prefill: one per (instance, KV head, question row); decode: one per (instance, KV head), each
    // on a 128-byte line of its own (the two kinds of launch never overlap, and every counter is
    // back at zero when its launch ends)
    W.n_counters = (size_t)c.max_batch * c.n_kv_heads * (size_t)std::max(max_q_rows(c), kDecodeCounterStride);
    // (bf16, head_dim 128: the projection GEMM may split the hidden axis over two workgroups per
    // 128 x 128 tile, up to kSplitTiles tiles: a counter line and two fp32 partial tiles each)
    const bool gemm_split = c.dtype == MATKV_BF16 && c.head_dim == 128;
    if (gemm_split) W.n_counters = std::max(W.n_counters, (size_t)kSplitTiles * kDecodeCounterStride);
    o += ((W.n_counters * sizeof(int32_t)) + 255) & ~(size_t)255;
    W.off_partials = o;
    size_t stride = (size_t)c.n_q_heads * (c.head_dim + 4);   // acc[D] + {m, l} (padded)
    size_t dec = (size_t)c.max_batch * kMaxDecodeUnitsPerInstance * stride;
    size_t pre = (size_t)c.max_batch * kMaxPrefillUnitsPerInstance * (size_t)max_q_rows(c) * stride;
    W.partial_floats = dec > pre ? dec : pre;
    if (gemm_split) W.partial_floats = std::max(W.partial_floats, (size_t)kSplitTiles * 2 * 128 * 128);
    o += W.partial_floats * sizeof(float);
    W.bytes = (o + 255) & ~(size_t)255;
    return W;
}

struct RopeEntry {         // 16 bytes, one per pair j < D/2
    double inv_freq;       // base^(-2j/D)                       (fp32 path: angle in fp64)
    float turns_hi;        // inv_freq / (2 pi), split hi + lo   (bf16 path: fp32 in turns)
    float turns_lo;
};

// ---------------------------------------------------------------- kernel launchers ---------
struct AttnArgs {
    const void* q;
    void* out;
    const void* tail_k;
    const void* tail_v;
    const char* table;         // device table
    float* partials;           // [unit][row][Hq][D + 4]: accumulator, running max, sum, pad
    int32_t* counters;
    int32_t layer, n_layers;
    int32_t Hq, Hkv, D;
    int32_t max_tail;
    int32_t rows;              // 1 = decode; > 1 = prefill rows (grid.z)
    int32_t n_units;           // grid.x
    int32_t max_units_inst;    // most units any one instance is cut into
    int32_t batch, total_q;    // instances; rows of the packed Q / O tensors (prefill)
    int32_t max_unit_items;    // most items in any one unit of this launch
    int32_t prefill;           // 0: decode units + whole tail; 1: prefill units + causal tail;
                               // 2: as 1 for a chunk's own attention (longest row tiles first)
    float scale_log2e;
    int32_t kv_fmt;            // matkv_page_format of every page of the table
    int32_t shared;            // decode over the shared partition (units = SUnit records)
    int32_t out_f32;           // bf16 configurations: q / out of the attention calls: out is float
    int32_t variant;           // kernel shape: 0 = default; 9000 + waves = matrix-core kernel;
                               // waves * 100 + loads in flight = plain-ALU kernel
    size_t off_inst, off_items, off_units;
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load of the wave (loads and stores share one counter on this chip), which
// drains a register-staged prefetch at every step; this one leaves those loads in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

hipError_t launch_attn_rows(const AttnArgs& a, int dtype, hipStream_t s);     // plain ALU, any dtype
bool attn_prefill_supported(const AttnArgs& a, int dtype);
hipError_t launch_attn_prefill(const AttnArgs& a, int dtype, hipStream_t s);  // matrix cores, rows split over waves
bool attn_mfma_supported(const AttnArgs& a, int dtype);
hipError_t launch_attn_mfma(const AttnArgs& a, int dtype, hipStream_t s);     // matrix cores, bf16 D=128

struct MaterializeArgs {
    const void* hidden;
    const void* w_k;
    const void* w_v;
    void* k_out;
    void* v_out;
    const RopeEntry* rope;
    const char* table;          // tail form only, else nullptr
    size_t off_inst;
    int64_t pos0;
    int64_t token_stride;       // rows between heads in the destination
    int32_t n_tokens;           // direct form: rows; tail form: upper bound on total rows
    int32_t rows_per_instance;  // tail form: <0 ragged question rows, >0 uniform newest rows
    int32_t batch;              // tail form
    int32_t Hkv, D, Hd;
    // scratch for launches that split the hidden axis over two workgroups (null: none): partial
    // tiles and arrival counters (all zero between launches), shared with the attention kernels
    float* ws_partials;
    int32_t* ws_counters;
    int64_t ws_partial_floats;
    int32_t ws_n_counters;
};

hipError_t launch_materialize(const MaterializeArgs& a, int dtype, hipStream_t s);
bool materialize_mfma_supported(const MaterializeArgs& a, int dtype, int total_rows);
hipError_t launch_materialize_mfma(const MaterializeArgs& a, int total_rows, hipStream_t s);
bool materialize_fewrows_supported(const MaterializeArgs& a, int dtype, int total_rows);
hipError_t launch_materialize_fewrows(const MaterializeArgs& a, int total_rows, hipStream_t s);
bool decode_step_supported(const AttnArgs& a, const MaterializeArgs& m, int dtype);
hipError_t launch_decode_step(const AttnArgs& a, const MaterializeArgs& m, int dtype, hipStream_t s);   // projection + attention
hipError_t launch_probe_read(const void* src, size_t bytes, unsigned* sink, hipStream_t s);
hipError_t launch_advance(char* table, size_t off_inst, int batch, int n, int max_tail, hipStream_t s);
hipError_t launch_chunk_table(char* table, int n_tokens, hipStream_t s);
hipError_t launch_compress(const void* blob, void* out, int n_layers, int Hkv, int n_tokens, int D, hipStream_t s);

// Compressed blob: codes, then the scale table [layer][K|V][Hkv] (float), both padded to 16 bytes.
inline size_t compressed_codes_bytes(const matkv_config& c, int n_tokens) {
    return ((size_t)c.n_layers * 2 * c.n_kv_heads * (size_t)n_tokens * c.head_dim + 15) & ~(size_t)15;
}
inline size_t compressed_scales_bytes(const matkv_config& c) {
    return ((size_t)c.n_layers * 2 * c.n_kv_heads * sizeof(float) + 15) & ~(size_t)15;
}

}  // namespace matkv
