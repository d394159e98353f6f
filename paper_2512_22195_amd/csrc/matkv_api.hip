// C-ABI of libmatkv: argument validation, host bookkeeping (tickets, slot states, cache
// tables, captured graphs) and the enqueue of copies and kernels.  See include/matkv.h for
// the contract of every entry point.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <errno.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <list>
#include <mutex>
#include <exception>
#include <new>
#include <thread>
#include <unordered_map>
#include <vector>

#include "matkv_internal.h"

using namespace matkv;

namespace {

constexpr int kTicketRing = 4096;
constexpr int kStagingRing = 4;
constexpr int kReleaseRing = 8;                // events marking "work on a table's old contents is enqueued"
constexpr int kBounceRing = 6;                 // pinned pieces between a file and the load stream
constexpr size_t kBounceBytes = 8u << 20;

struct Ticket {
    hipEvent_t ev = nullptr;
    uint64_t id = 0;          // 0 = never used
    void* slot = nullptr;
    bool done = true;         // observed complete
    // loads from a file: the event is recorded by a reader thread once the last piece's copy is on
    // the load stream.  Guarded by the context's io mutex.
    bool queued = false;      // pieces still to be read or enqueued: the event is not recorded yet
    bool failed = false;      // a read failed (the reason is in io_err)
};

struct SlotState {
    uint64_t pending = 0;     // ticket id of the last load into the slot (0 = none)
    bool waited = true;       // compute stream has been ordered after that load
    int refs = 0;             // live cache tables that point into it
    hipEvent_t release = nullptr;   // recorded on the compute stream when its last table let go of it
};

struct TableHost {
    int batch = 0, n_items = 0, n_dunits = 0, n_punits = 0, total_q = 0, max_q = 0;
    int max_punits_inst = 0;  // most prefill units of any one instance
    int max_punit_items = 0;  // most items of any one prefill unit
    int kv_fmt = 0;           // matkv_page_format of its pages
    int n_sunits = 0;         // units of the shared decode partition; 0 = the batch shares no page
    uint64_t sig_decode = 0, sig_prefill = 0;   // of what a recorded decode / prefill launch bakes in
    int max_tail_len = 0;     // largest tail_len of any instance (host mirror)
    int min_tail_len = 0;
    int n_decode_slots = 0;   // partial slots a decode launch writes (units, or (unit, user) pairs when shared)
    std::vector<const void*> slots;   // distinct slots its pages point into
};

struct Staging {
    char* host = nullptr;     // pinned
    hipEvent_t ev = nullptr;
    bool used = false;
};

}  // namespace

// Scratch of matkv_decode_attn_static (the decode attention for callers that cannot allocate or
// pass a workspace): arrival counters, 128 bytes apart, then the units' partial results.  Every
// device the library runs on holds its own copy until the process ends.
constexpr size_t kStaticCounterBytes = 1u << 20;    // 8192 (instance, KV head) pairs
constexpr size_t kStaticPartialBytes = 7u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticCounterBytes + kStaticPartialBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.  In host code the
// array's name is only a handle; the address comes from the runtime, once per device.
hipError_t scratch_address(int device, char** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = static_cast<char*>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

__global__ void zero_ints_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

struct matkv_graph {
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    std::vector<std::pair<void*, int>> advances;   // (table, n) recorded during capture
    struct TableUse { const void* table; bool decode, prefill; uint64_t sig_decode, sig_prefill; };
    std::vector<TableUse> tables;                  // every table the recording reads, with its partition signatures
};

struct matkv_ctx {
    matkv_config cfg;
    int device = 0;
    hipStream_t compute = nullptr, load = nullptr;
    char* workspace = nullptr;
    char* static_scratch = nullptr;           // this device's copy of `scratch`
    WorkspaceLayout wl;
    TableLayout tl;
    float scale_log2e = 0.f;
    char err[512];
    bool sticky_hip = false;
    uint64_t next_ticket = 1;
    std::vector<Ticket> tickets;
    std::unordered_map<const void*, SlotState> slots;
    std::unordered_map<const void*, TableHost> tables;
    Staging staging[kStagingRing];
    int staging_next = 0;
    Staging bounce[kBounceRing];              // allocated at the first matkv_load_file / matkv_store_file
    int bounce_next = 0;
    char* plain_buf = nullptr;                // matkv_store_file: direct writes that cannot come from pinned memory
    std::atomic<bool> read_via_plain{false};  // direct I/O cannot target the pinned buffers on this system
    // file loads: requests wait in a queue, reader threads take them piece by piece
    struct FileReq {
        int fd; uint64_t offset; size_t bytes; char* dst; Ticket* ticket;
        size_t n_pieces, next_piece, pieces_done;
    };
    std::mutex io_mu;
    std::condition_variable io_work, io_done;
    std::list<FileReq> io_queue;              // front = the oldest request (a list: readers keep pointers into it)
    std::vector<std::thread> io_readers;
    bool io_stop = false;
    char io_err[256] = {0};                   // reason of the last failed read
    hipEvent_t fence_ev = nullptr;
    hipEvent_t release_ev[kReleaseRing] = {};
    int release_next = 0;
    bool capturing = false;
    int chunk_table_tokens = -1;   // chunk length the workspace's one-instance table was last written for (-1: unknown)
    matkv_graph* cap = nullptr;
    std::vector<matkv_graph*> graphs;
};

namespace {

matkv_status fail(matkv_ctx* c, matkv_status s, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

matkv_status hip_fail(matkv_ctx* c, hipError_t e, const char* what) {
    (void)hipGetLastError();
    if (c) {
        c->sticky_hip = true;
        snprintf(c->err, sizeof(c->err), "%s: %s", what, hipGetErrorString(e));
    }
    return MATKV_EHIP;
}

#define HIP_TRY(ctx, call)                                     \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(ctx, e_, #call); \
    } while (0)

// No C++ exception crosses the boundary: host containers and std::thread can throw
// (allocation failure, no thread to be had); every entry point that reaches them runs between
// these two and turns the exception into a status.
#define MATKV_TRY try {
#define MATKV_CATCH(ctx, name)                                                                     \
    } catch (const std::bad_alloc&) {                                                              \
        return fail(ctx, MATKV_ENOMEM, "%s: out of host memory", name);                            \
    } catch (const std::exception& ex_) {                                                          \
        return fail(ctx, MATKV_ENOMEM, "%s: %s", name, ex_.what());                                \
    } catch (...) {                                                                                \
        return fail(ctx, MATKV_ENOMEM, "%s: unexpected C++ exception", name);                      \
    }
#define MATKV_CATCH_INT                                                                            \
    } catch (...) {                                                                                \
        return -1;                                                                                 \
    }

int elem_bytes(const matkv_config& c) { return c.dtype == MATKV_F32 ? 4 : 2; }

matkv_status check_config(const matkv_config* c, const char** why) {
    static const char* ok = "";
    *why = ok;
    if (!c) { *why = "config is null"; return MATKV_EINVAL; }
    if (c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->hidden < 1 ||
        c->max_batch < 1 || c->max_pages < 0 || c->max_tail_tokens < 1) {
        *why = "sizes must be positive"; return MATKV_EINVAL;
    }
    if (c->dtype != MATKV_F32 && c->dtype != MATKV_BF16) { *why = "unknown dtype"; return MATKV_EINVAL; }
    if (c->n_q_heads % c->n_kv_heads) { *why = "n_q_heads not a multiple of n_kv_heads"; return MATKV_EINVAL; }
    if (!(c->rope_base > 1.0f)) { *why = "rope_base must exceed 1"; return MATKV_EINVAL; }
    if (c->softmax_scale < 0.f || isnan(c->softmax_scale)) { *why = "softmax_scale negative"; return MATKV_EINVAL; }
    if (c->hidden % 64) { *why = "hidden must be a multiple of 64"; return MATKV_EINVAL; }
    if (c->max_tail_tokens % 8) { *why = "max_tail_tokens must be a multiple of 8"; return MATKV_EINVAL; }
    if (c->decode_units < 0 || c->decode_units > kMaxDecodeUnitsPerInstance) { *why = "decode_units outside 0..256"; return MATKV_EINVAL; }
    if (c->decode_variant < 0) { *why = "decode_variant negative"; return MATKV_EINVAL; }
    if (c->out_f32 != 0 && c->out_f32 != 1) { *why = "out_f32 must be 0 or 1"; return MATKV_EINVAL; }
    if (c->max_batch > 1024 || c->max_pages > 4096) { *why = "max_batch <= 1024, max_pages <= 4096"; return MATKV_EINVAL; }
    if (c->head_dim != 64 && c->head_dim != 128) { *why = "head_dim must be 64 or 128"; return MATKV_EUNSUPPORTED; }
    const int g = c->n_q_heads / c->n_kv_heads;
    if (!group_size_built(g)) { *why = "group size must be 1, 2, 3, 4 or 8"; return MATKV_EUNSUPPORTED; }
    return MATKV_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Decode workgroups per (instance, KV head) when the configuration does not fix it: one
// workgroup per compute unit over the whole batch and never more than there are compute units
// (a compute unit that holds two runs a third longer, and the launch ends with it: batch 3,
// 8 KV heads: 240 workgroups 19.7 us, 264 workgroups 24.9 us), each with at least 128 tokens.
int choose_decode_units(const matkv_config& c, int batch, long inst_tokens) {
    int u = c.decode_units;
    if (u <= 0) {
        const int per_head = batch * c.n_kv_heads;
        u = 256 / per_head;
        const long cap = inst_tokens / 128;
        if (u > cap) u = (int)cap;
    }
    if (u < 1) u = 1;
    if (u > kMaxDecodeUnitsPerInstance) u = kMaxDecodeUnitsPerInstance;
    return u;
}

// Units one instance's cache is cut into for the question prefill.  The matrix-core kernel runs
// one workgroup per (unit, KV head, row tile); every extra unit costs a partial per question row
// and a share of the fold launch.  Four-wave workgroups (128-row tiles, questions of up to 128
// (row, head) rows): as many units as it takes to give every compute unit a workgroup (none
// shorter than 256 tokens), and twice that - two resident workgroups per compute unit overlap
// each other's matrix and vector phases - only while a unit keeps at least 4096 tokens to
// amortise its partial over.  Eight-wave workgroups (256-row tiles): see below.
// The other kernels launch a workgroup per question row and want few units.
int choose_prefill_units(const matkv_config& cfg, long tiles_in_batch, long tile_rows, long tokens) {
    const int g = cfg.n_q_heads / cfg.n_kv_heads;
    const bool mfma = cfg.dtype == MATKV_BF16 && cfg.head_dim == 128 && group_size_built(g);
    long pu;
    if (mfma && tile_rows > 128) {
        // eight-wave workgroups fill a compute unit alone: about 256 of them, and rather a few
        // compute units idle than one more cut (config 3, 216 workgroups uncut: 187 us against
        // 218 us in two units; config 4, 128 uncut: 376 us in two units against 414 us in four)
        const long wgs_per_unit = std::max<long>(1, tiles_in_batch * cfg.n_kv_heads);
        pu = (256 + wgs_per_unit / 2) / wgs_per_unit;
        pu = std::max<long>(1, std::min<long>(pu, tokens / 256));
    } else if (mfma) {
        const long wgs_per_unit = std::max<long>(1, tiles_in_batch * cfg.n_kv_heads);
        pu = (256 + wgs_per_unit - 1) / wgs_per_unit;
        pu = std::max<long>(1, std::min<long>(pu, tokens / 256));
        if (wgs_per_unit * pu < 512 && tokens / (2 * pu) >= 4096) pu *= 2;
    } else {
        pu = tokens / 1024;
    }
    return (int)std::max<long>(1, std::min<long>(pu, kMaxPrefillUnitsPerInstance));
}

// Cuts one instance's cache (its pages in order, then its tail) into n_units runs of nearly
// equal token counts, in 8-token granules.  A run is a list of items (page pieces); the tail
// is one item and belongs to the last run.  Appends to items / units; returns the number of
// units made (runs that would hold no tokens are dropped).
template <typename ScalesOff>
int build_units(const matkv_page* pages, int n_pages, int inst, int n_units, int tail_estimate,
                int max_tail, Item* items, int* n_items, Unit* units, int* n_units_out, ScalesOff scales_off) {
    long page_gran = 0;
    for (int p = 0; p < n_pages; ++p) page_gran += (pages[p].n_tokens + 7) / 8;
    const long tail_gran = (tail_estimate + 7) / 8;
    const long total = page_gran + tail_gran;
    int made = 0;
    int p = 0;            // current page
    long p_g0 = 0;        // first granule (in the instance's page stream) of page p
    for (int u = 0; u < n_units; ++u) {
        long g0 = total * u / n_units, g1 = total * (u + 1) / n_units;
        const bool last = (u == n_units - 1);
        if (g0 > page_gran) g0 = page_gran;
        if (g1 > page_gran || last) g1 = page_gran;
        if (g1 <= g0 && !last) continue;
        Unit un;
        memset(&un, 0, sizeof(un));
        un.inst = inst; un.item0 = *n_items; un.idx_in_inst = made;
        long g = g0;
        while (g < g1) {
            long pg = (pages[p].n_tokens + 7) / 8;
            while (g >= p_g0 + pg) { p_g0 += pg; ++p; pg = (pages[p].n_tokens + 7) / 8; }
            const long e = (g1 < p_g0 + pg) ? g1 : p_g0 + pg;
            Item it;
            memset(&it, 0, sizeof(it));
            it.base = reinterpret_cast<uint64_t>(pages[p].slot);
            it.page_tokens = pages[p].n_tokens;
            it.tok0 = (int)((g - p_g0) * 8);
            const int t1 = (int)((e - p_g0) * 8);
            it.ntok = (t1 < pages[p].n_tokens ? t1 : pages[p].n_tokens) - it.tok0;
            it.fmt = pages[p].format;
            it.scales16 = (int32_t)(scales_off(pages[p].n_tokens) / 16);
            un.page_tokens += it.ntok;
            items[(*n_items)++] = it;
            g = e;
        }
        if (last) {
            Item it;
            memset(&it, 0, sizeof(it));
            it.base = 0; it.page_tokens = max_tail; it.tok0 = 0; it.ntok = max_tail;
            items[(*n_items)++] = it;
        }
        un.n_items = *n_items - un.item0;
        un.has_tail = last ? 1 : 0;
        un.first = items[un.item0];
        units[(*n_units_out)++] = un;
        ++made;
    }
    for (int k = 0; k < made; ++k) {
        Unit& un = units[*n_units_out - made + k];
        un.n_units_inst = made;
        un.unit0_inst = *n_units_out - made;
    }
    return made;
}

// Shared decode partition (instances of a batch that retrieved the same chunk read it once).
// The batch's DISTINCT pages and its tails form one stream of token rows - per instance its
// private pages, then the shared pages it uses first, then its tail - which is cut into equal
// runs, one workgroup (per KV head) each, never more workgroups than compute units.  A run is a
// list of pieces like any decode unit; every piece carries the set of the unit's users that
// may see it (Item::umask), the unit lists its users (at most 16 / G: the rows of its matrix
// tile are (user, query head) pairs) and each (unit, user) pair gets one of that user's
// consecutive partial slots.  A run ends early where one more piece would bring a user too many
// or a second tail.  tokens_out (may be null): [unit][kMaxSharedUsers] page tokens each user sees.
// Returns the number of units, 0 if the batch shares no page worth the trouble or the
// partition does not fit the table (then the per-instance partition is used).
int build_shared_units(const matkv_config& cfg, const matkv_page* pages, const int32_t* n_pages, int batch,
                       int max_sunits, int max_items, InstanceInfo* insts, Item* items, int* n_items, SUnit* sunits,
                       int kv_fmt, int32_t* tokens_out = nullptr) {
    struct PageUse { const void* slot; int n_tokens; std::vector<int> users; };
    std::vector<PageUse> distinct;
    std::unordered_map<const void*, std::vector<int>> by_slot;   // slot -> indices into distinct
    for (int b = 0; b < batch; ++b)
        for (int p = 0; p < n_pages[b]; ++p) {
            const matkv_page& pg = pages[(size_t)b * cfg.max_pages + p];
            // (an instance that lists one page twice attends to it twice: the second occurrence is a
            // page of its own)
            int found = -1;
            for (int i : by_slot[pg.slot])
                if (distinct[i].n_tokens == pg.n_tokens &&
                    std::find(distinct[i].users.begin(), distinct[i].users.end(), b) == distinct[i].users.end()) { found = i; break; }
            if (found < 0) {
                found = (int)distinct.size();
                distinct.push_back(PageUse{pg.slot, pg.n_tokens, {}});
                by_slot[pg.slot].push_back(found);
            }
            distinct[found].users.push_back(b);
        }
    // Worth it when the distinct pages are at least a twentieth fewer tokens than all uses together
    // (measured at batch 16, five 1000-token chunks each, per layer, per-instance against shared
    // partition: 81 % of the page tokens distinct 58.3 against 54.8 us, 41 % 43.4 against 35.5,
    // 6 % 33.5 against 18.3).
    long all_tokens = 0, distinct_tokens = 0;
    for (const PageUse& pu : distinct) {
        distinct_tokens += pu.n_tokens;
        all_tokens += (long)pu.n_tokens * (long)pu.users.size();
    }
    if (distinct_tokens * 20 > all_tokens * 19) return 0;

    const int G = cfg.n_q_heads / cfg.n_kv_heads;
    const int cap_users = kMaxSharedUsers / G;
    // a page with more users than a tile has rows for is streamed once per group of them: each
    // group becomes a page of its own from here on
    {
        std::vector<PageUse> split;
        for (const PageUse& pu : distinct)
            for (size_t u0 = 0; u0 < pu.users.size(); u0 += cap_users)
                split.push_back(PageUse{pu.slot, pu.n_tokens,
                                        std::vector<int>(pu.users.begin() + u0, pu.users.begin() + std::min(pu.users.size(), u0 + cap_users))});
        distinct.swap(split);
    }
    // the stream: per instance the pages it is the first user of (private ones first), then its
    // tail; an instance that is the first user of no page gets its tail behind a page it uses (one
    // tail per page at most), so that tails stay apart: a unit holds at most one
    struct Piece { int page; int inst; long gran; std::vector<int> users; };    // page < 0: the tail of inst
    std::vector<Piece> stream;
    std::vector<char> tail_placed(batch, 0), owns(batch, 0);
    for (const PageUse& pu : distinct) owns[pu.users[0]] = 1;
    long total_gran = 0;
    auto push_tail = [&](int b) {
        const int tail_est = insts[b].q_len + (cfg.max_tail_tokens - insts[b].q_len) / 2;
        stream.push_back(Piece{-1, b, (tail_est + 7) / 8, {b}});
        total_gran += stream.back().gran;
        tail_placed[b] = 1;
    };
    for (int b = 0; b < batch; ++b) {
        for (int pass = 0; pass < 2; ++pass)                     // private pages first
            for (size_t di = 0; di < distinct.size(); ++di) {
                const PageUse& pu = distinct[di];
                if (pu.users[0] != b || (pass == 0) != (pu.users.size() == 1)) continue;
                stream.push_back(Piece{(int)di, b, (pu.n_tokens + 7) / 8, pu.users});
                total_gran += stream.back().gran;
                for (int u : pu.users)
                    if (!tail_placed[u] && !owns[u]) { push_tail(u); break; }
            }
        if (owns[b]) push_tail(b);
    }
    for (int b = 0; b < batch; ++b)
        if (!tail_placed[b]) push_tail(b);
    int n_target = 256 / cfg.n_kv_heads;
    if (n_target > total_gran * 8 / 128) n_target = (int)(total_gran * 8 / 128);
    if (n_target < 1) n_target = 1;

    // Cuts the stream into units of `per` granules; returns the number of units, or -1 if they do
    // not fit.  emit = false only counts.
    std::vector<std::vector<int>> slot_of;                       // [unit][user index] -> partial slot (second pass)
    auto cut = [&](long per, bool emit, int first_item) -> int {
        int n = 0, n_it = first_item;
        long room = 0;                                           // granules the open unit may still take
        std::vector<int> users;                                  // of the open unit
        bool open = false, has_tail = false;
        SUnit* su = nullptr;
        auto close_unit = [&]() {
            if (!open) return;
            if (emit) {
                su->u.n_items = n_it - su->u.item0;
                // the unit's tail, if it has one, goes last (compressed pages: the kernel walks the
                // code pages and then the plain tail)
                for (int i = su->u.item0; i + 1 < n_it; ++i)
                    if (items[i].base == 0) std::rotate(items + i, items + i + 1, items + n_it);
                su->u.first = items[su->u.item0];
                su->n_users = (int)users.size();
                for (size_t k = 0; k < users.size(); ++k) su->users[k].inst = users[k];
            }
            ++n; open = false;
        };
        auto open_unit = [&]() {
            if (emit) {
                su = &sunits[n];
                memset(su, 0, sizeof(*su));
                su->u.item0 = n_it;
            }
            users.clear(); room = per; open = true; has_tail = false;
        };
        for (const Piece& pc : stream) {
            const std::vector<int>& pusers = pc.users;
            long g = 0;
            while (g < pc.gran) {
                if (open) {
                    int fresh = 0;
                    for (int u : pusers) if (std::find(users.begin(), users.end(), u) == users.end()) ++fresh;
                    if ((int)users.size() + fresh > cap_users || (pc.page < 0 && has_tail) || room <= 0) close_unit();
                }
                if (!open) {
                    if (n >= max_sunits) return -1;
                    open_unit();
                }
                uint32_t mask = 0;
                for (int u : pusers) {
                    auto it = std::find(users.begin(), users.end(), u);
                    if (it == users.end()) { users.push_back(u); it = users.end() - 1; }
                    mask |= 1u << (int)(it - users.begin());
                }
                // a tail is never cut; a page piece takes what room there is
                const long take = pc.page < 0 ? pc.gran : std::min(pc.gran - g, room);
                if (emit) {
                    if (n_it >= max_items) return -1;
                    Item it;
                    memset(&it, 0, sizeof(it));
                    if (pc.page < 0) {
                        it.base = 0; it.page_tokens = cfg.max_tail_tokens; it.tok0 = 0; it.ntok = cfg.max_tail_tokens;
                        su->u.has_tail = 1; su->u.inst = pc.inst;
                    } else {
                        const PageUse& pu = distinct[pc.page];
                        it.base = reinterpret_cast<uint64_t>(pu.slot);
                        it.page_tokens = pu.n_tokens;
                        it.tok0 = (int)(g * 8);
                        it.ntok = (int)std::min<long>(pu.n_tokens, (g + take) * 8) - it.tok0;
                        it.fmt = kv_fmt;
                        it.scales16 = kv_fmt == MATKV_PAGE_E4M3 ? (int32_t)(compressed_codes_bytes(cfg, pu.n_tokens) / 16) : 0;
                        su->u.page_tokens += it.ntok;
                        if (tokens_out)
                            for (int k = 0; k < kMaxSharedUsers; ++k)
                                if (mask >> k & 1) tokens_out[(size_t)n * kMaxSharedUsers + k] += it.ntok;
                    }
                    it.umask = (int32_t)mask;
                    items[n_it] = it;
                }
                ++n_it;
                if (pc.page < 0) has_tail = true;
                g += take; room -= take;
            }
        }
        close_unit();
        if (emit) *n_items = n_it;
        return n;
    };
    // unit size: the smallest with which the launch has no more workgroups than compute units
    long per = std::max<long>(16, (total_gran + n_target - 1) / n_target);
    int n = cut(per, false, *n_items);
    for (int it = 0; it < 64 && (n < 0 || n * cfg.n_kv_heads > 256); ++it) {
        per += std::max<long>(1, per / 32);
        n = cut(per, false, *n_items);
    }
    if (n <= 0 || n > max_sunits || n * cfg.n_kv_heads > 256) return 0;
    if (tokens_out) memset(tokens_out, 0, sizeof(int32_t) * (size_t)n * kMaxSharedUsers);
    n = cut(per, true, *n_items);
    if (n <= 0) return 0;
    // partial slots: every (unit, user) pair one, an instance's slots consecutive
    std::vector<int> count(batch, 0), next(batch, 0);
    for (int u = 0; u < n; ++u)
        for (int k = 0; k < sunits[u].n_users; ++k) ++count[sunits[u].users[k].inst];
    int slot0 = 0;
    for (int b = 0; b < batch; ++b) {
        if (count[b] > kMaxDecodeUnitsPerInstance) return 0;
        insts[b].sslot0 = slot0; insts[b].n_sslots = count[b];
        next[b] = slot0;
        slot0 += count[b];
    }
    for (int u = 0; u < n; ++u) {
        sunits[u].u.idx_in_inst = u;
        for (int k = 0; k < sunits[u].n_users; ++k) sunits[u].users[k].slot = next[sunits[u].users[k].inst]++;
    }
    return n;
}

TableHost* find_table(matkv_ctx* c, const void* t) {
    auto it = c->tables.find(t);
    return it == c->tables.end() ? nullptr : &it->second;
}

// Launch shapes and kernel choices are fixed when a call is recorded; they follow from these.
uint64_t fnv(std::initializer_list<int> f) {
    uint64_t h = 1469598103934665603ull;
    for (int v : f) { h ^= (uint64_t)(uint32_t)v; h *= 1099511628211ull; }
    return h;
}
void sign_partition(TableHost& th) {
    th.sig_decode = fnv({th.batch, th.n_dunits, th.n_sunits, th.kv_fmt});
    th.sig_prefill = fnv({th.batch, th.n_punits, th.total_q, th.max_q, th.max_punits_inst, th.max_punit_items, th.kv_fmt});
}
// While a graph is being recorded: remember that it reads this table's decode or prefill side.
void note_table_use(matkv_ctx* c, const void* table, const TableHost& th, bool prefill) {
    if (!c->capturing || !c->cap) return;
    for (auto& e : c->cap->tables)
        if (e.table == table) { (prefill ? e.prefill : e.decode) = true; return; }
    c->cap->tables.push_back({table, !prefill, prefill, th.sig_decode, th.sig_prefill});
}

matkv_status precheck(matkv_ctx* c) {
    if (!c) return MATKV_EINVAL;
    if (c->sticky_hip) return MATKV_EHIP;
    return MATKV_OK;
}

}  // namespace

extern "C" {

const char* matkv_status_string(matkv_status s) {
    switch (s) {
        case MATKV_OK: return "MATKV_OK";
        case MATKV_EINVAL: return "MATKV_EINVAL";
        case MATKV_EUNSUPPORTED: return "MATKV_EUNSUPPORTED";
        case MATKV_ENOTREADY: return "MATKV_ENOTREADY";
        case MATKV_EBUSY: return "MATKV_EBUSY";
        case MATKV_EHIP: return "MATKV_EHIP";
        case MATKV_ENOMEM: return "MATKV_ENOMEM";
        case MATKV_EIO: return "MATKV_EIO";
    }
    return "MATKV_?";
}

matkv_status matkv_config_check(const matkv_config* cfg) {
    const char* why;
    return check_config(cfg, &why);
}

size_t matkv_blob_bytes(const matkv_config* cfg, int32_t n_tokens) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK || n_tokens < 0) return 0;
    return (size_t)cfg->n_layers * 2 * cfg->n_kv_heads * (size_t)n_tokens * cfg->head_dim * elem_bytes(*cfg);
}

size_t matkv_compressed_blob_bytes(const matkv_config* cfg, int32_t n_tokens) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK || n_tokens < 0) return 0;
    return compressed_codes_bytes(*cfg, n_tokens) + compressed_scales_bytes(*cfg);
}

size_t matkv_tail_bytes(const matkv_config* cfg) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK) return 0;
    return (size_t)cfg->max_batch * cfg->n_kv_heads * (size_t)cfg->max_tail_tokens * cfg->head_dim * elem_bytes(*cfg);
}

size_t matkv_workspace_bytes(const matkv_config* cfg) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK) return 0;
    return workspace_layout(*cfg).bytes;
}

size_t matkv_table_bytes(const matkv_config* cfg) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK) return 0;
    return table_layout(*cfg).bytes;
}

matkv_status matkv_create(const matkv_config* cfg, void* workspace, size_t workspace_bytes,
                          void* compute_stream, void* load_stream, matkv_ctx** out) {
    if (!out) return MATKV_EINVAL;
    *out = nullptr;
    const char* why;
    matkv_status st = check_config(cfg, &why);
    if (st != MATKV_OK) return st;
    const WorkspaceLayout wl = workspace_layout(*cfg);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return MATKV_EINVAL;
    if (workspace_bytes < wl.bytes) return MATKV_ENOMEM;

    matkv_ctx* c = new (std::nothrow) matkv_ctx();
    if (!c) return MATKV_ENOMEM;
    c->cfg = *cfg;
    c->err[0] = 0;
    c->compute = reinterpret_cast<hipStream_t>(compute_stream);
    c->load = reinterpret_cast<hipStream_t>(load_stream);
    c->workspace = reinterpret_cast<char*>(workspace);
    c->wl = wl;
    c->tl = table_layout(*cfg);
    const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
    c->scale_log2e = scale * 1.4426950408889634f;
    try {
        c->tickets.resize(kTicketRing);
    } catch (...) {
        delete c;
        return MATKV_ENOMEM;
    }

    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = scratch_address(c->device, &c->static_scratch);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->fence_ev, hipEventDisableTiming);
    // rotary table: inv_freq in double, and inv_freq / 2pi split into two floats
    RopeEntry rope[64];
    const int half = cfg->head_dim / 2;
    for (int j = 0; j < half; ++j) {
        const double f = pow((double)cfg->rope_base, -2.0 * j / (double)cfg->head_dim);
        const double turns = f / 6.283185307179586476925286766559;
        rope[j].inv_freq = f;
        rope[j].turns_hi = (float)turns;
        rope[j].turns_lo = (float)(turns - (double)rope[j].turns_hi);
    }
    if (e == hipSuccess) e = hipMemcpy(c->workspace + wl.off_rope, rope, sizeof(RopeEntry) * half, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemsetAsync(c->workspace + wl.off_counters, 0, wl.off_partials - wl.off_counters, c->compute);
    for (int i = 0; i < kStagingRing && e == hipSuccess; ++i) {
        e = hipHostMalloc(reinterpret_cast<void**>(&c->staging[i].host), c->tl.bytes, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->staging[i].ev, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        matkv_destroy(c);
        return MATKV_EHIP;
    }
    *out = c;
    return MATKV_OK;
}

matkv_status matkv_destroy(matkv_ctx* c) {
    if (!c) return MATKV_EINVAL;
    {
        std::lock_guard<std::mutex> lk(c->io_mu);
        c->io_stop = true;                   // requests still queued are dropped with the context
    }
    c->io_work.notify_all();
    for (std::thread& th : c->io_readers) th.join();
    (void)hipStreamSynchronize(c->load);
    (void)hipStreamSynchronize(c->compute);
    for (matkv_graph* g : c->graphs) {
        if (g->exec) (void)hipGraphExecDestroy(g->exec);
        if (g->graph) (void)hipGraphDestroy(g->graph);
        delete g;
    }
    for (Ticket& t : c->tickets)
        if (t.ev) (void)hipEventDestroy(t.ev);
    for (int i = 0; i < kStagingRing; ++i) {
        if (c->staging[i].ev) (void)hipEventDestroy(c->staging[i].ev);
        if (c->staging[i].host) (void)hipHostFree(c->staging[i].host);
    }
    for (int i = 0; i < kBounceRing; ++i) {
        if (c->bounce[i].ev) (void)hipEventDestroy(c->bounce[i].ev);
        if (c->bounce[i].host) (void)hipHostFree(c->bounce[i].host);
    }
    free(c->plain_buf);
    for (int i = 0; i < kReleaseRing; ++i)
        if (c->release_ev[i]) (void)hipEventDestroy(c->release_ev[i]);
    if (c->fence_ev) (void)hipEventDestroy(c->fence_ev);
    (void)hipGetLastError();
    delete c;
    return MATKV_OK;
}

const char* matkv_last_error(const matkv_ctx* c) { return c ? c->err : "context is null"; }

// ------------------------------------------------------------------------------------ M ----

// The workspace's partial and counter regions as scratch of a projection launch (every call runs
// on the compute stream, so it never overlaps an attention launch that uses them).
static void materialize_scratch(matkv_ctx* c, MaterializeArgs& a) {
    a.ws_partials = reinterpret_cast<float*>(c->workspace + c->wl.off_partials);
    a.ws_counters = reinterpret_cast<int32_t*>(c->workspace + c->wl.off_counters);
    a.ws_partial_floats = (int64_t)c->wl.partial_floats;
    a.ws_n_counters = (int32_t)std::min<size_t>(c->wl.n_counters, 1u << 30);
}

matkv_status matkv_materialize(matkv_ctx* c, const void* hidden, const void* w_k, const void* w_v,
                               int32_t n_tokens, int64_t pos0, void* k_out, void* v_out,
                               int64_t token_stride) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!hidden || !w_k || !w_v || !k_out || !v_out) return fail(c, MATKV_EINVAL, "materialize: null pointer");
    if (!aligned16(hidden) || !aligned16(w_k) || !aligned16(w_v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(c, MATKV_EINVAL, "materialize: pointers must be 16-byte aligned");
    if (n_tokens < 0 || pos0 < 0 || token_stride < n_tokens)
        return fail(c, MATKV_EINVAL, "materialize: n_tokens=%d pos0=%lld token_stride=%lld", n_tokens,
                    (long long)pos0, (long long)token_stride);
    if (pos0 + n_tokens > (1ll << 24)) return fail(c, MATKV_EINVAL, "materialize: positions beyond 2^24");
    if (n_tokens == 0) return MATKV_OK;
    MaterializeArgs a{};
    a.hidden = hidden; a.w_k = w_k; a.w_v = w_v; a.k_out = k_out; a.v_out = v_out;
    a.rope = reinterpret_cast<const RopeEntry*>(c->workspace + c->wl.off_rope);
    a.table = nullptr; a.off_inst = 0;
    a.pos0 = pos0; a.token_stride = token_stride; a.n_tokens = n_tokens;
    a.rows_per_instance = 0; a.batch = 1;
    a.Hkv = c->cfg.n_kv_heads; a.D = c->cfg.head_dim; a.Hd = c->cfg.hidden;
    materialize_scratch(c, a);
    HIP_TRY(c, launch_materialize(a, c->cfg.dtype, c->compute));
    return MATKV_OK;
}

matkv_status matkv_compress(matkv_ctx* c, const void* blob, int32_t n_tokens, void* out) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!blob || !out) return fail(c, MATKV_EINVAL, "compress: null pointer");
    if (!aligned16(blob) || !aligned16(out)) return fail(c, MATKV_EINVAL, "compress: pointers must be 16-byte aligned");
    if (c->cfg.dtype != MATKV_BF16) return fail(c, MATKV_EUNSUPPORTED, "compress: bf16 configurations only");
    if (n_tokens < 1) return fail(c, MATKV_EINVAL, "compress: n_tokens=%d", n_tokens);
    const char* a = static_cast<const char*>(blob);
    const char* b = static_cast<const char*>(out);
    if (a < b + matkv_compressed_blob_bytes(&c->cfg, n_tokens) && b < a + matkv_blob_bytes(&c->cfg, n_tokens))
        return fail(c, MATKV_EINVAL, "compress: output overlaps the blob");
    HIP_TRY(c, launch_compress(blob, out, c->cfg.n_layers, c->cfg.n_kv_heads, n_tokens, c->cfg.head_dim, c->compute));
    return MATKV_OK;
}

matkv_status matkv_materialize_tail(matkv_ctx* c, const void* hidden, const void* w_k, const void* w_v,
                                    const void* table, int32_t rows_per_instance, void* tail_k,
                                    void* tail_v) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    MATKV_TRY
    if (!hidden || !w_k || !w_v || !table || !tail_k || !tail_v)
        return fail(c, MATKV_EINVAL, "materialize_tail: null pointer");
    if (!aligned16(hidden) || !aligned16(w_k) || !aligned16(w_v) || !aligned16(tail_k) || !aligned16(tail_v))
        return fail(c, MATKV_EINVAL, "materialize_tail: pointers must be 16-byte aligned");
    TableHost* th = find_table(c, table);
    if (!th) return fail(c, MATKV_EINVAL, "materialize_tail: table was not built by matkv_assemble");
    if (rows_per_instance == 0) return fail(c, MATKV_EINVAL, "materialize_tail: rows_per_instance is 0");
    note_table_use(c, table, *th, rows_per_instance < 0);
    if (rows_per_instance > 0 && rows_per_instance > th->min_tail_len)
        return fail(c, MATKV_EINVAL, "materialize_tail: %d newest rows but a tail holds only %d",
                    rows_per_instance, th->min_tail_len);
    MaterializeArgs a{};
    a.hidden = hidden; a.w_k = w_k; a.w_v = w_v; a.k_out = tail_k; a.v_out = tail_v;
    a.rope = reinterpret_cast<const RopeEntry*>(c->workspace + c->wl.off_rope);
    a.table = reinterpret_cast<const char*>(table); a.off_inst = c->tl.off_inst;
    a.pos0 = 0; a.token_stride = c->cfg.max_tail_tokens;
    a.rows_per_instance = rows_per_instance; a.batch = th->batch;
    a.n_tokens = rows_per_instance > 0 ? th->batch * rows_per_instance : th->total_q;
    a.Hkv = c->cfg.n_kv_heads; a.D = c->cfg.head_dim; a.Hd = c->cfg.hidden;
    materialize_scratch(c, a);
    HIP_TRY(c, launch_materialize(a, c->cfg.dtype, c->compute));
    return MATKV_OK;
    MATKV_CATCH(c, "materialize_tail")
}

// ------------------------------------------------------------------------------------ L ----

// Where a file load stands: 0 = all its copies are on the load stream (or it is no file load),
// 1 = pieces still to be read, 2 = a read failed.  block: wait until it is not 1.
static int file_state(matkv_ctx* c, Ticket* t, bool block) {
    std::unique_lock<std::mutex> lk(c->io_mu);
    if (block) c->io_done.wait(lk, [&] { return !t->queued; });
    if (t->queued) return 1;
    return t->failed ? 2 : 0;
}
static matkv_status file_failed(matkv_ctx* c) {
    std::lock_guard<std::mutex> lk(c->io_mu);
    return fail(c, MATKV_EIO, "%s", c->io_err);
}

// Checks shared by both load entry points; on success *t_out is the ticket record to fill and
// the load stream has been ordered after compute work that may still read the slot.
static matkv_status load_prepare(matkv_ctx* c, const char* name, size_t bytes, int32_t n_tokens,
                                 void* device_slot, size_t slot_bytes, Ticket** t_out) {
    // a copy ordered behind the compute stream would pull the load stream and the ticket's event
    // into the recording
    if (c->capturing) return fail(c, MATKV_EBUSY, "%s: not allowed while a graph is being captured", name);
    if (n_tokens < 1) return fail(c, MATKV_EINVAL, "%s: n_tokens=%d", name, n_tokens);
    const size_t want = matkv_blob_bytes(&c->cfg, n_tokens), want_c = matkv_compressed_blob_bytes(&c->cfg, n_tokens);
    if (bytes != want && bytes != want_c)
        return fail(c, MATKV_EINVAL, "%s: %zu bytes given, a %d-token blob has %zu (compressed: %zu)", name, bytes, n_tokens, want, want_c);
    if (slot_bytes < bytes) return fail(c, MATKV_EINVAL, "%s: slot of %zu bytes cannot hold %zu", name, slot_bytes, bytes);
    if (!aligned16(device_slot)) return fail(c, MATKV_EINVAL, "%s: pointers must be 16-byte aligned", name);
    hipPointerAttribute_t attr;
    hipError_t pe = hipPointerGetAttributes(&attr, device_slot);
    if (pe != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(c, MATKV_EINVAL, "%s: slot is not device memory", name);
    }
    Ticket& t = c->tickets[c->next_ticket % kTicketRing];
    if (t.id != 0 && !t.done) {
        if (file_state(c, &t, false) == 1) return fail(c, MATKV_EBUSY, "%s: %d tickets outstanding", name, kTicketRing);
        hipError_t q = hipEventQuery(t.ev);
        if (q == hipErrorNotReady) { (void)hipGetLastError(); return fail(c, MATKV_EBUSY, "%s: %d tickets outstanding", name, kTicketRing); }
        if (q != hipSuccess) return hip_fail(c, q, "hipEventQuery");
        t.done = true;
    }
    if (!t.ev) HIP_TRY(c, hipEventCreateWithFlags(&t.ev, hipEventDisableTiming));
    SlotState& s = c->slots[device_slot];
    if (s.pending) {
        // a file load into this slot whose pieces are still being read: a second load would mix
        // its copies with theirs on the load stream
        Ticket& prev = c->tickets[s.pending % kTicketRing];
        if (prev.id == s.pending && file_state(c, &prev, false) == 1)
            return fail(c, MATKV_EBUSY, "%s: a load from a file into this slot is still being read", name);
    }
    if (s.refs > 0) {
        // a live table still points into the slot: order the copy after all compute work so far
        HIP_TRY(c, hipEventRecord(c->fence_ev, c->compute));
        HIP_TRY(c, hipStreamWaitEvent(c->load, c->fence_ev, 0));
    } else if (s.release) {
        // its last table was re-assembled onto other slots: the copy waits for the work that was
        // enqueued up to that moment, not for what has been enqueued since
        HIP_TRY(c, hipStreamWaitEvent(c->load, s.release, 0));
    }
    s.release = nullptr;
    *t_out = &t;
    return MATKV_OK;
}

// The copies of a load are on the load stream: record the ticket's event behind them.
static matkv_status load_finish(matkv_ctx* c, Ticket* t, void* device_slot, matkv_ticket* out) {
    HIP_TRY(c, hipEventRecord(t->ev, c->load));
    t->id = c->next_ticket++;
    t->slot = device_slot;
    t->done = false; t->queued = false; t->failed = false;
    SlotState& s = c->slots[device_slot];
    s.pending = t->id;
    s.waited = false;
    out->id = t->id;
    return MATKV_OK;
}

matkv_status matkv_load(matkv_ctx* c, const void* host_blob, size_t bytes, int32_t n_tokens,
                        void* device_slot, size_t slot_bytes, matkv_ticket* out) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    MATKV_TRY
    if (!host_blob || !device_slot || !out) return fail(c, MATKV_EINVAL, "load: null pointer");
    if (!aligned16(host_blob)) return fail(c, MATKV_EINVAL, "load: pointers must be 16-byte aligned");
    hipPointerAttribute_t attr;
    hipError_t pe = hipPointerGetAttributes(&attr, host_blob);
    if (pe != hipSuccess) { (void)hipGetLastError(); return fail(c, MATKV_EINVAL, "load: host blob is not pinned memory"); }
    if (attr.type != hipMemoryTypeHost) return fail(c, MATKV_EINVAL, "load: host blob is not pinned host memory");
    Ticket* t;
    st = load_prepare(c, "load", bytes, n_tokens, device_slot, slot_bytes, &t);
    if (st != MATKV_OK) return st;
    HIP_TRY(c, hipMemcpyAsync(device_slot, host_blob, bytes, hipMemcpyHostToDevice, c->load));
    return load_finish(c, t, device_slot, out);
    MATKV_CATCH(c, "load")
}

// ---- loads from a file: reader threads owned by the context -------------------------------
// matkv_load_file queues a request and returns.  kIoReaders threads take the queued requests
// piece by piece (8 MiB, several preads in flight at different offsets), each into one of its own
// two pinned bounce buffers - through a plain page-aligned buffer of its own where direct I/O
// cannot target pinned memory - and enqueue the piece's copy on the load stream.  The thread
// that finishes a request's last piece records the ticket's event behind all its copies.
constexpr int kIoReaders = 3;
static_assert(kBounceRing >= 2 * kIoReaders, "two bounce buffers per reader");

static void io_reader_main(matkv_ctx* c, int reader) {
    (void)hipSetDevice(c->device);
    char* plain = nullptr;
    int flip = 0;
    std::unique_lock<std::mutex> lk(c->io_mu);
    for (;;) {
        matkv_ctx::FileReq* rq = nullptr;
        c->io_work.wait(lk, [&] {
            if (c->io_stop) return true;
            for (auto& r : c->io_queue) if (r.next_piece < r.n_pieces) { rq = &r; return true; }
            return false;
        });
        if (c->io_stop) break;
        const size_t k = rq->next_piece++;
        const bool skip = rq->ticket->failed;           // an earlier piece failed: nothing more is read
        lk.unlock();

        char why[200] = {0};
        if (!skip) {
            Staging& b = c->bounce[2 * reader + flip];
            flip ^= 1;
            hipError_t he = b.used ? hipEventSynchronize(b.ev) : hipSuccess;     // its last copy has left the buffer
            const size_t piece = std::min(kBounceBytes, rq->bytes - k * kBounceBytes);
            const uint64_t at = rq->offset + k * kBounceBytes;
            size_t got = 0;
            while (he == hipSuccess && !why[0] && got < piece) {
                const bool via_plain = c->read_via_plain.load();
                if (via_plain && !plain && posix_memalign(reinterpret_cast<void**>(&plain), 4096, kBounceBytes) != 0) {
                    plain = nullptr;
                    snprintf(why, sizeof(why), "out of host memory");
                    break;
                }
                char* dest = via_plain ? plain : b.host;
                const ssize_t r = pread(rq->fd, dest + got, piece - got, (off_t)(at + got));
                if (r < 0 && errno == EINTR) continue;
                if (r < 0 && errno == EFAULT && !via_plain) {
                    // direct I/O cannot pin the device-mapped bounce buffer on this system: from now
                    // on read into plain page-aligned memory and copy into the bounce buffer
                    c->read_via_plain.store(true);
                    got = 0;
                    continue;
                }
                if (r < 0) snprintf(why, sizeof(why), "pread at %llu: %s", (unsigned long long)(at + got), strerror(errno));
                else if (r == 0) snprintf(why, sizeof(why), "file ends %llu bytes short of the blob",
                                          (unsigned long long)(rq->offset + rq->bytes - (at + got)));
                else got += (size_t)r;
            }
            if (he == hipSuccess && !why[0]) {
                if (c->read_via_plain.load()) memcpy(b.host, plain, piece);
                he = hipMemcpyAsync(rq->dst + k * kBounceBytes, b.host, piece, hipMemcpyHostToDevice, c->load);
                if (he == hipSuccess) he = hipEventRecord(b.ev, c->load);
                b.used = true;
            }
            if (he != hipSuccess) {
                (void)hipGetLastError();
                snprintf(why, sizeof(why), "copy of a piece: %s", hipGetErrorString(he));
            }
        }

        lk.lock();
        if (why[0] && !rq->ticket->failed) {
            rq->ticket->failed = true;
            snprintf(c->io_err, sizeof(c->io_err), "load_file: %s", why);
        }
        if (++rq->pieces_done == rq->n_pieces) {
            // every copy of this request is on the load stream (or the request was given up)
            if (hipEventRecord(rq->ticket->ev, c->load) != hipSuccess) {
                (void)hipGetLastError();
                rq->ticket->failed = true;
            }
            rq->ticket->queued = false;
            for (auto it = c->io_queue.begin(); it != c->io_queue.end(); ++it)
                if (&*it == rq) { c->io_queue.erase(it); break; }
            c->io_done.notify_all();
        }
    }
    free(plain);
}

// Blocks until no file load is queued or being read (the store path and the destructor share
// the bounce buffers with the readers).
static void io_drain(matkv_ctx* c) {
    std::unique_lock<std::mutex> lk(c->io_mu);
    c->io_done.wait(lk, [&] { return c->io_queue.empty(); });
}

static matkv_status bounce_buffers(matkv_ctx* c) {
    for (int i = 0; i < kBounceRing; ++i) {
        if (c->bounce[i].host) continue;
        HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&c->bounce[i].host), kBounceBytes, hipHostMallocDefault));
        HIP_TRY(c, hipEventCreateWithFlags(&c->bounce[i].ev, hipEventDisableTiming));
    }
    return MATKV_OK;
}

matkv_status matkv_load_file(matkv_ctx* c, int fd, uint64_t offset, size_t bytes, int32_t n_tokens,
                             void* device_slot, size_t slot_bytes, matkv_ticket* out) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    MATKV_TRY
    if (fd < 0 || !device_slot || !out) return fail(c, MATKV_EINVAL, "load_file: bad descriptor or null pointer");
    Ticket* t;
    st = load_prepare(c, "load_file", bytes, n_tokens, device_slot, slot_bytes, &t);
    if (st != MATKV_OK) return st;
    st = bounce_buffers(c);
    if (st != MATKV_OK) return st;
    if (c->io_readers.empty()) {
        c->io_readers.reserve(kIoReaders);
        for (int r = 0; r < kIoReaders; ++r) c->io_readers.emplace_back(io_reader_main, c, r);
    }
    {
        std::lock_guard<std::mutex> lk(c->io_mu);
        t->id = c->next_ticket++;
        t->slot = device_slot;
        t->done = false; t->queued = true; t->failed = false;
        matkv_ctx::FileReq rq{};
        rq.fd = fd; rq.offset = offset; rq.bytes = bytes; rq.dst = static_cast<char*>(device_slot); rq.ticket = t;
        rq.n_pieces = (bytes + kBounceBytes - 1) / kBounceBytes; rq.next_piece = 0; rq.pieces_done = 0;
        c->io_queue.push_back(rq);
    }
    c->io_work.notify_all();
    SlotState& s = c->slots[device_slot];
    s.pending = t->id;
    s.waited = false;
    out->id = t->id;
    return MATKV_OK;
    MATKV_CATCH(c, "load_file")
}

matkv_status matkv_store_file(matkv_ctx* c, int fd, uint64_t offset, const void* device_blob, size_t bytes) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (fd < 0 || !device_blob || bytes == 0) return fail(c, MATKV_EINVAL, "store_file: bad descriptor, null pointer or no bytes");
    if (c->capturing) return fail(c, MATKV_EBUSY, "store_file: not allowed while a graph is being captured");
    hipPointerAttribute_t attr;
    hipError_t pe = hipPointerGetAttributes(&attr, device_blob);
    if (pe != hipSuccess || attr.type != hipMemoryTypeDevice) {
        (void)hipGetLastError();
        return fail(c, MATKV_EINVAL, "store_file: blob is not device memory");
    }
    st = bounce_buffers(c);
    if (st != MATKV_OK) return st;
    io_drain(c);                             // the reader threads use the same bounce buffers
    // the blob was produced on the compute stream: the copies out follow what is enqueued there
    HIP_TRY(c, hipEventRecord(c->fence_ev, c->compute));
    HIP_TRY(c, hipStreamWaitEvent(c->load, c->fence_ev, 0));
    // piece k is written to the file while the copy of piece k+1 is in flight
    const size_t n_pieces = (bytes + kBounceBytes - 1) / kBounceBytes;
    auto piece_bytes = [&](size_t k) { return std::min(kBounceBytes, bytes - k * kBounceBytes); };
    auto enqueue = [&](size_t k) -> hipError_t {
        Staging& b = c->bounce[k % kBounceRing];
        if (b.used) { hipError_t e = hipEventSynchronize(b.ev); if (e != hipSuccess) return e; }
        hipError_t e = hipMemcpyAsync(b.host, static_cast<const char*>(device_blob) + k * kBounceBytes, piece_bytes(k),
                                      hipMemcpyDeviceToHost, c->load);
        if (e == hipSuccess) e = hipEventRecord(b.ev, c->load);
        b.used = true;
        return e;
    };
    HIP_TRY(c, enqueue(0));
    for (size_t k = 0; k < n_pieces; ++k) {
        if (k + 1 < n_pieces) HIP_TRY(c, enqueue(k + 1));
        Staging& b = c->bounce[k % kBounceRing];
        HIP_TRY(c, hipEventSynchronize(b.ev));
        const char* src = b.host;
        const size_t piece = piece_bytes(k);
        if (c->read_via_plain.load()) {
            if (!c->plain_buf && posix_memalign(reinterpret_cast<void**>(&c->plain_buf), 4096, kBounceBytes) != 0) {
                c->plain_buf = nullptr;
                return fail(c, MATKV_ENOMEM, "store_file: out of host memory");
            }
            memcpy(c->plain_buf, b.host, piece);
            src = c->plain_buf;
        }
        size_t put = 0;
        while (put < piece) {
            ssize_t r = pwrite(fd, src + put, piece - put, (off_t)(offset + k * kBounceBytes + put));
            if (r < 0 && errno == EINTR) continue;
            if (r < 0 && errno == EFAULT && !c->read_via_plain.load()) {
                // direct I/O cannot pin the device-mapped bounce buffer on this system (see the reader threads)
                if (!c->plain_buf && posix_memalign(reinterpret_cast<void**>(&c->plain_buf), 4096, kBounceBytes) != 0) {
                    c->plain_buf = nullptr;
                    return fail(c, MATKV_ENOMEM, "store_file: out of host memory");
                }
                c->read_via_plain.store(true);
                memcpy(c->plain_buf, b.host, piece);
                src = c->plain_buf;
                continue;
            }
            if (r <= 0) return fail(c, MATKV_EIO, "store_file: pwrite at %llu: %s", (unsigned long long)(offset + k * kBounceBytes + put),
                                    r < 0 ? strerror(errno) : "no progress");
            put += (size_t)r;
        }
    }
    return MATKV_OK;
}

static matkv_status ticket_lookup(matkv_ctx* c, matkv_ticket tk, Ticket** out) {
    if (tk.id == 0 || tk.id >= c->next_ticket) return fail(c, MATKV_EINVAL, "ticket %llu was never issued", (unsigned long long)tk.id);
    Ticket& t = c->tickets[tk.id % kTicketRing];
    if (t.id != tk.id) { *out = nullptr; return MATKV_OK; }   // ring slot reused: that copy finished long ago
    *out = &t;
    return MATKV_OK;
}

matkv_status matkv_wait(matkv_ctx* c, matkv_ticket tk) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    Ticket* t;
    st = ticket_lookup(c, tk, &t);
    if (st != MATKV_OK || !t) return st;
    // a file load still being read: the event is not recorded yet, so the host waits here until
    // the last piece's copy is on the load stream (the copies themselves are not waited for)
    if (!t->done && file_state(c, t, true) == 2) return file_failed(c);
    if (!t->done) HIP_TRY(c, hipStreamWaitEvent(c->compute, t->ev, 0));
    auto it = c->slots.find(t->slot);
    if (it != c->slots.end() && it->second.pending == tk.id) it->second.waited = true;
    return MATKV_OK;
}

matkv_status matkv_query(matkv_ctx* c, matkv_ticket tk) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    Ticket* t;
    st = ticket_lookup(c, tk, &t);
    if (st != MATKV_OK || !t) return st;
    if (t->done) return MATKV_OK;
    const int fs = file_state(c, t, false);
    if (fs == 1) return MATKV_ENOTREADY;
    if (fs == 2) return file_failed(c);
    hipError_t q = hipEventQuery(t->ev);
    if (q == hipErrorNotReady) { (void)hipGetLastError(); return MATKV_ENOTREADY; }
    if (q != hipSuccess) return hip_fail(c, q, "hipEventQuery");
    t->done = true;
    return MATKV_OK;
}

matkv_status matkv_sync(matkv_ctx* c, matkv_ticket tk) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    Ticket* t;
    st = ticket_lookup(c, tk, &t);
    if (st != MATKV_OK || !t) return st;
    if (!t->done && file_state(c, t, true) == 2) {
        (void)hipEventSynchronize(t->ev);     // the pieces that did get enqueued
        return file_failed(c);
    }
    if (!t->done) { HIP_TRY(c, hipEventSynchronize(t->ev)); t->done = true; }
    return MATKV_OK;
}

// A slot that was the target of a load nobody has waited for: if the copy has finished, the
// compute stream is ordered behind it (while a graph is being recorded nothing is ordered: a
// finished copy needs no edge) and the slot counts as waited for; if not, MATKV_ENOTREADY.
static matkv_status slot_ready(matkv_ctx* c, const void* slot, const char* name) {
    auto it = c->slots.find(slot);
    if (it == c->slots.end() || !it->second.pending || it->second.waited) return MATKV_OK;
    Ticket& t = c->tickets[it->second.pending % kTicketRing];
    bool done = (t.id != it->second.pending) || t.done;
    if (!done) {
        const int fs = file_state(c, &t, false);
        if (fs == 1) return fail(c, MATKV_ENOTREADY, "%s: a page's load from a file is still being read", name);
        if (fs == 2) return fail(c, MATKV_EIO, "%s: a page's load from a file failed", name);
        hipError_t q = hipEventQuery(t.ev);
        if (q == hipSuccess) { t.done = true; done = true; }
        else if (q == hipErrorNotReady) (void)hipGetLastError();
        else return hip_fail(c, q, "hipEventQuery");
    }
    if (!done) return fail(c, MATKV_ENOTREADY, "%s: a page's load has neither finished nor been waited for", name);
    if (t.id == it->second.pending && !c->capturing) HIP_TRY(c, hipStreamWaitEvent(c->compute, t.ev, 0));
    it->second.waited = true;
    return MATKV_OK;
}

// Every slot a table points into, before work that reads the table is enqueued: a load into one
// of them after the table was assembled must not race with that work.
static matkv_status table_pages_ready(matkv_ctx* c, const TableHost& th, const char* name) {
    for (const void* sl : th.slots) {
        matkv_status st = slot_ready(c, sl, name);
        if (st != MATKV_OK) return st;
    }
    return MATKV_OK;
}

// ------------------------------------------------------------------------------------ A ----

matkv_status matkv_assemble(matkv_ctx* c, const matkv_page* pages, const int32_t* n_pages,
                            const int32_t* q_len, const int64_t* pos_base, int32_t batch, void* table) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (c->capturing) return fail(c, MATKV_EBUSY, "assemble: not allowed while a graph is being captured");
    MATKV_TRY
    if (!n_pages || !q_len || !table) return fail(c, MATKV_EINVAL, "assemble: null pointer");
    if (!aligned16(table)) return fail(c, MATKV_EINVAL, "assemble: table must be 16-byte aligned");
    if (batch < 1 || batch > c->cfg.max_batch) return fail(c, MATKV_EINVAL, "assemble: batch=%d, max_batch=%d", batch, c->cfg.max_batch);
    const matkv_config& cfg = c->cfg;
    long total_tokens = 0;
    int kv_fmt = -1;                   // format of the table's pages (-1: none seen yet)
    for (int b = 0; b < batch; ++b) {
        if (n_pages[b] < 0 || n_pages[b] > cfg.max_pages) return fail(c, MATKV_EINVAL, "assemble: instance %d has %d pages, max_pages=%d", b, n_pages[b], cfg.max_pages);
        if (n_pages[b] > 0 && !pages) return fail(c, MATKV_EINVAL, "assemble: pages is null");
        if (q_len[b] < 1 || q_len[b] > cfg.max_tail_tokens) return fail(c, MATKV_EINVAL, "assemble: instance %d question length %d outside 1..%d", b, q_len[b], cfg.max_tail_tokens);
        if (pos_base && (pos_base[b] < 0 || pos_base[b] + cfg.max_tail_tokens > (1ll << 24))) return fail(c, MATKV_EINVAL, "assemble: instance %d pos_base out of range", b);
        for (int p = 0; p < n_pages[b]; ++p) {
            const matkv_page& pg = pages[(size_t)b * cfg.max_pages + p];
            if (!pg.slot || !aligned16(pg.slot) || pg.n_tokens < 1)
                return fail(c, MATKV_EINVAL, "assemble: instance %d page %d is invalid", b, p);
            if (pg.format != MATKV_PAGE_PLAIN && pg.format != MATKV_PAGE_E4M3)
                return fail(c, MATKV_EINVAL, "assemble: instance %d page %d has unknown format %d", b, p, pg.format);
            if (kv_fmt < 0) kv_fmt = pg.format;
            if (pg.format != kv_fmt) return fail(c, MATKV_EUNSUPPORTED, "assemble: plain and compressed pages in one table");
            st = slot_ready(c, pg.slot, "assemble");
            if (st == MATKV_ENOTREADY) return fail(c, MATKV_ENOTREADY, "assemble: instance %d page %d: load neither finished nor waited for", b, p);
            if (st != MATKV_OK) return st;
            total_tokens += pg.n_tokens;
        }
    }

    (void)total_tokens;
    if (kv_fmt < 0) kv_fmt = MATKV_PAGE_PLAIN;
    if (kv_fmt == MATKV_PAGE_E4M3 && !(cfg.dtype == MATKV_BF16 && cfg.head_dim == 128))
        return fail(c, MATKV_EUNSUPPORTED, "assemble: compressed pages need bf16 and head_dim 128");
    auto scales_off = [&](int n_tokens) { return kv_fmt == MATKV_PAGE_E4M3 ? compressed_codes_bytes(cfg, n_tokens) : (size_t)0; };
    Staging& sg = c->staging[c->staging_next];
    c->staging_next = (c->staging_next + 1) % kStagingRing;
    if (sg.used) HIP_TRY(c, hipEventSynchronize(sg.ev));
    char* h = sg.host;
    TableHeader* hdr = reinterpret_cast<TableHeader*>(h);
    InstanceInfo* insts = reinterpret_cast<InstanceInfo*>(h + c->tl.off_inst);
    Item* items = reinterpret_cast<Item*>(h + c->tl.off_items);
    Unit* dunits = reinterpret_cast<Unit*>(h + c->tl.off_dunits);
    Unit* punits = reinterpret_cast<Unit*>(h + c->tl.off_punits);
    memset(hdr, 0, sizeof(*hdr));
    int n_items = 0, n_dunits = 0, n_punits = 0, cu = 0, max_q = 0;
    TableHost th;
    th.min_tail_len = cfg.max_tail_tokens;
    // row tiles of (question row, query head of one KV head) over the batch: the matrix-core prefill
    // kernel takes 256-row workgroups once the longest question has more than 128 such rows
    long prefill_tiles = 0, max_rg = 0;
    for (int b = 0; b < batch; ++b) max_rg = std::max<long>(max_rg, (long)q_len[b] * (cfg.n_q_heads / cfg.n_kv_heads));
    const long tile_rows = max_rg > 128 ? 256 : 128;
    for (int b = 0; b < batch; ++b)
        prefill_tiles += ((long)q_len[b] * (cfg.n_q_heads / cfg.n_kv_heads) + tile_rows - 1) / tile_rows;
    for (int b = 0; b < batch; ++b) {
        InstanceInfo& in = insts[b];
        memset(&in, 0, sizeof(in));
        const matkv_page* pg = pages ? pages + (size_t)b * cfg.max_pages : nullptr;
        long inst_tokens = 0;
        for (int p = 0; p < n_pages[b]; ++p) {
            inst_tokens += pg[p].n_tokens;
        }
        in.pos_base = pos_base ? pos_base[b] : inst_tokens;
        if (in.pos_base + cfg.max_tail_tokens > (1ll << 24)) return fail(c, MATKV_EINVAL, "assemble: positions beyond 2^24");
        in.tail_len = q_len[b];
        in.q_len = q_len[b];
        in.cu_q = cu;
        cu += q_len[b];
        if (q_len[b] > max_q) max_q = q_len[b];
        if (q_len[b] > th.max_tail_len) th.max_tail_len = q_len[b];
        if (q_len[b] < th.min_tail_len) th.min_tail_len = q_len[b];
        const int tail_est = q_len[b] + (cfg.max_tail_tokens - q_len[b]) / 2;
        // decode: fine partition, one workgroup per (unit, KV head)
        in.dunit0 = n_dunits;
        in.n_dunits = build_units(pg, n_pages[b], b, choose_decode_units(cfg, batch, inst_tokens + tail_est),
                                  tail_est, cfg.max_tail_tokens, items, &n_items, dunits, &n_dunits, scales_off);
        // prefill: coarse partition (the question rows supply most of the parallelism)
        const int pu = choose_prefill_units(cfg, prefill_tiles, tile_rows, inst_tokens + q_len[b]);
        in.punit0 = n_punits;
        in.n_punits = build_units(pg, n_pages[b], b, pu, q_len[b], cfg.max_tail_tokens, items, &n_items,
                                  punits, &n_punits, scales_off);
        if (in.n_punits > th.max_punits_inst) th.max_punits_inst = in.n_punits;
        for (int u = in.punit0; u < n_punits; ++u)
            if (punits[u].n_items > th.max_punit_items) th.max_punit_items = punits[u].n_items;
    }
    // decode over shared pages: only where the default matrix-core decode kernel runs
    const int grp = cfg.n_q_heads / cfg.n_kv_heads;
    int n_sunits = 0;
    if (batch >= 2 && pages && cfg.decode_units == 0 && cfg.decode_variant == 0 &&
        cfg.dtype == MATKV_BF16 && cfg.head_dim == 128 && group_size_built(grp))
        n_sunits = build_shared_units(cfg, pages, n_pages, batch, c->tl.max_sunits, c->tl.max_items, insts, items, &n_items,
                                      reinterpret_cast<SUnit*>(h + c->tl.off_sunits), kv_fmt);
    hdr->batch = batch; hdr->n_items = n_items; hdr->n_dunits = n_dunits; hdr->n_punits = n_punits;
    hdr->total_q = cu; hdr->max_q = max_q;

    char* d = reinterpret_cast<char*>(table);
    HIP_TRY(c, hipMemcpyAsync(d, h, c->tl.off_inst + sizeof(InstanceInfo) * batch, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(d + c->tl.off_items, h + c->tl.off_items, sizeof(Item) * n_items, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(d + c->tl.off_dunits, h + c->tl.off_dunits, sizeof(Unit) * n_dunits, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipMemcpyAsync(d + c->tl.off_punits, h + c->tl.off_punits, sizeof(Unit) * n_punits, hipMemcpyHostToDevice, c->compute));
    if (n_sunits > 0)
        HIP_TRY(c, hipMemcpyAsync(d + c->tl.off_sunits, h + c->tl.off_sunits, sizeof(SUnit) * n_sunits, hipMemcpyHostToDevice, c->compute));
    HIP_TRY(c, hipEventRecord(sg.ev, c->compute));
    sg.used = true;

    th.batch = batch; th.n_items = n_items; th.n_dunits = n_dunits; th.n_punits = n_punits;
    th.total_q = cu; th.max_q = max_q; th.kv_fmt = kv_fmt; th.n_sunits = n_sunits;
    th.n_decode_slots = n_dunits;
    if (n_sunits > 0) {
        th.n_decode_slots = 0;
        for (int b = 0; b < batch; ++b) th.n_decode_slots = std::max(th.n_decode_slots, insts[b].sslot0 + insts[b].n_sslots);
    }
    sign_partition(th);
    // Slot bookkeeping: the table's old contents are dead from here on in stream order, so the
    // slots only they pointed into may be overwritten once the work enqueued so far is done.
    for (int b = 0; b < batch; ++b) {
        const matkv_page* pg = pages ? pages + (size_t)b * cfg.max_pages : nullptr;
        for (int p = 0; p < n_pages[b]; ++p)
            if (std::find(th.slots.begin(), th.slots.end(), pg[p].slot) == th.slots.end()) th.slots.push_back(pg[p].slot);
    }
    auto old = c->tables.find(table);
    if (old != c->tables.end() && !old->second.slots.empty()) {
        hipEvent_t& ev = c->release_ev[c->release_next];
        c->release_next = (c->release_next + 1) % kReleaseRing;
        if (!ev) HIP_TRY(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        HIP_TRY(c, hipEventRecord(ev, c->compute));
        for (const void* sl : old->second.slots) {
            SlotState& ss = c->slots[sl];
            if (ss.refs > 0) --ss.refs;
            if (ss.refs == 0) ss.release = ev;
        }
    }
    for (const void* sl : th.slots) ++c->slots[sl].refs;
    c->tables[table] = th;
    return MATKV_OK;
    MATKV_CATCH(c, "assemble")
}

int32_t matkv_plan_decode_units(const matkv_config* cfg, const int32_t* page_tokens, int32_t n_pages,
                                int32_t batch, int32_t q_len, int32_t* unit_tokens_out,
                                int32_t* unit_items_out, int32_t cap) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK) return -1;
    MATKV_TRY
    if (n_pages < 0 || n_pages > cfg->max_pages || (n_pages > 0 && !page_tokens) || batch < 1 ||
        batch > cfg->max_batch || q_len < 1 || q_len > cfg->max_tail_tokens || cap < 0)
        return -1;
    std::vector<matkv_page> pages((size_t)(n_pages > 0 ? n_pages : 1));
    long inst_tokens = 0;
    for (int p = 0; p < n_pages; ++p) {
        if (page_tokens[p] < 1) return -1;
        pages[p].slot = reinterpret_cast<const void*>((uintptr_t)0x1000);   // never dereferenced
        pages[p].n_tokens = page_tokens[p];
        pages[p].format = MATKV_PAGE_PLAIN;
        inst_tokens += page_tokens[p];
    }
    const int tail_est = q_len + (cfg->max_tail_tokens - q_len) / 2;
    std::vector<Item> items((size_t)kMaxDecodeUnitsPerInstance + n_pages + 2);
    std::vector<Unit> units((size_t)kMaxDecodeUnitsPerInstance);
    int n_items = 0, n_units = 0;
    const int made = build_units(pages.data(), n_pages, 0, choose_decode_units(*cfg, batch, inst_tokens + tail_est),
                                 tail_est, cfg->max_tail_tokens, items.data(), &n_items, units.data(), &n_units,
                                 [](int) { return (size_t)0; });
    for (int u = 0; u < made && u < cap; ++u) {
        if (unit_tokens_out) unit_tokens_out[u] = units[u].page_tokens;
        if (unit_items_out) unit_items_out[u] = units[u].n_items - units[u].has_tail;
    }
    return made < cap ? made : cap;
    MATKV_CATCH_INT
}

int32_t matkv_plan_shared_units(const matkv_config* cfg, const int32_t* page_ids, const int32_t* page_tokens,
                                const int32_t* n_pages, const int32_t* q_len, int32_t batch,
                                int32_t* units_out, int32_t cap, int32_t* slots_out) {
    const char* why;
    if (check_config(cfg, &why) != MATKV_OK) return -1;
    if (!n_pages || !q_len || batch < 1 || batch > cfg->max_batch || cap < 0 || (cap > 0 && !units_out)) return -1;
    MATKV_TRY
    const int grp = cfg->n_q_heads / cfg->n_kv_heads;
    std::vector<matkv_page> pages((size_t)batch * std::max(cfg->max_pages, 1));
    std::vector<InstanceInfo> insts((size_t)batch);
    for (int b = 0; b < batch; ++b) {
        if (n_pages[b] < 0 || n_pages[b] > cfg->max_pages || q_len[b] < 1 || q_len[b] > cfg->max_tail_tokens) return -1;
        if (n_pages[b] > 0 && (!page_ids || !page_tokens)) return -1;
        memset(&insts[b], 0, sizeof(InstanceInfo));
        insts[b].q_len = q_len[b];
        for (int p = 0; p < n_pages[b]; ++p) {
            const size_t i = (size_t)b * cfg->max_pages + p;
            if (page_ids[i] < 0 || page_tokens[i] < 1) return -1;
            pages[i].slot = reinterpret_cast<const void*>(((uintptr_t)page_ids[i] + 1) * 4096);   // never dereferenced
            pages[i].n_tokens = page_tokens[i];
            pages[i].format = MATKV_PAGE_PLAIN;
        }
    }
    // the conditions of matkv_assemble
    if (batch < 2 || cfg->decode_units != 0 || cfg->decode_variant != 0 || cfg->dtype != MATKV_BF16 ||
        cfg->head_dim != 128 || !group_size_built(grp))
        return 0;
    const TableLayout tl = table_layout(*cfg);
    std::vector<Item> items((size_t)tl.max_items);
    std::vector<SUnit> sunits((size_t)tl.max_sunits);
    int n_items = 0;
    std::vector<int32_t> user_tokens((size_t)tl.max_sunits * kMaxSharedUsers);
    const int n = build_shared_units(*cfg, pages.data(), n_pages, batch, tl.max_sunits, tl.max_items, insts.data(),
                                     items.data(), &n_items, sunits.data(), MATKV_PAGE_PLAIN, user_tokens.data());
    for (int u = 0; u < n && u < cap; ++u) {
        const SUnit& su = sunits[u];
        int32_t* o = units_out + (size_t)u * (4 + 3 * kMaxSharedUsers);
        const uintptr_t base = (uintptr_t)su.u.first.base;
        o[0] = base ? (int32_t)(base / 4096 - 1) : -1;     // id of the unit's first page; -1: it starts with a tail
        o[1] = su.u.page_tokens;                            // page tokens the unit streams (all its pieces)
        o[2] = su.u.has_tail ? su.u.inst : -1;              // the instance whose tail it holds, or -1
        o[3] = su.n_users;
        for (int k = 0; k < kMaxSharedUsers; ++k) {
            o[4 + 3 * k] = k < su.n_users ? su.users[k].inst : -1;
            o[5 + 3 * k] = k < su.n_users ? su.users[k].slot : -1;
            o[6 + 3 * k] = k < su.n_users ? user_tokens[(size_t)u * kMaxSharedUsers + k] : 0;
        }
    }
    if (slots_out && n > 0)
        for (int b = 0; b < batch; ++b) { slots_out[2 * b] = insts[b].sslot0; slots_out[2 * b + 1] = insts[b].n_sslots; }
    return n < cap ? n : cap;
    MATKV_CATCH_INT
}

int32_t matkv_table_shared_units(matkv_ctx* c, const void* table) {
    if (!c) return -1;
    TableHost* th = find_table(c, table);
    return th ? th->n_sunits : -1;
}

matkv_status matkv_advance(matkv_ctx* c, void* table, int32_t n) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    TableHost* th = find_table(c, table);
    if (!th) return fail(c, MATKV_EINVAL, "advance: table was not built by matkv_assemble");
    if (n < 1) return fail(c, MATKV_EINVAL, "advance: n=%d", n);
    MATKV_TRY
    note_table_use(c, table, *th, false);
    if (c->capturing) {
        c->cap->advances.emplace_back(table, n);
    } else {
        if (th->max_tail_len + n > c->cfg.max_tail_tokens)
            return fail(c, MATKV_EINVAL, "advance: tail would hold %d tokens, max_tail_tokens=%d", th->max_tail_len + n, c->cfg.max_tail_tokens);
        th->max_tail_len += n; th->min_tail_len += n;
    }
    HIP_TRY(c, launch_advance(reinterpret_cast<char*>(table), c->tl.off_inst, th->batch, n, c->cfg.max_tail_tokens, c->compute));
    return MATKV_OK;
    MATKV_CATCH(c, "advance")
}

// -------------------------------------------------------------------------------- P / D ----

static matkv_status attn_args(matkv_ctx* c, const char* name, int prefill, int32_t layer, const void* q,
                              const void* table, const void* tail_k, const void* tail_v, void* out, AttnArgs* out_args) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!q || !table || !tail_k || !tail_v || !out) return fail(c, MATKV_EINVAL, "%s: null pointer", name);
    if (!aligned16(q) || !aligned16(tail_k) || !aligned16(tail_v) || !aligned16(out))
        return fail(c, MATKV_EINVAL, "%s: pointers must be 16-byte aligned", name);
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, MATKV_EINVAL, "%s: layer %d outside 0..%d", name, layer, c->cfg.n_layers - 1);
    TableHost* th = find_table(c, table);
    if (!th) return fail(c, MATKV_EINVAL, "%s: table was not built by matkv_assemble", name);
    MATKV_TRY
    st = table_pages_ready(c, *th, name);
    if (st != MATKV_OK) return st;
    note_table_use(c, table, *th, prefill != 0);
    MATKV_CATCH(c, name)
    AttnArgs a{};
    a.q = q; a.out = out; a.tail_k = tail_k; a.tail_v = tail_v;
    a.table = reinterpret_cast<const char*>(table);
    a.partials = reinterpret_cast<float*>(c->workspace + c->wl.off_partials);
    a.variant = prefill ? 0 : c->cfg.decode_variant;
    a.counters = reinterpret_cast<int32_t*>(c->workspace + c->wl.off_counters);
    a.layer = layer; a.n_layers = c->cfg.n_layers;
    a.Hq = c->cfg.n_q_heads; a.Hkv = c->cfg.n_kv_heads; a.D = c->cfg.head_dim;
    a.max_tail = c->cfg.max_tail_tokens;
    a.prefill = prefill;
    a.rows = prefill ? th->max_q : 1;
    a.shared = !prefill && th->n_sunits > 0;
    a.n_units = prefill ? th->n_punits : (a.shared ? th->n_sunits : th->n_dunits);
    a.max_units_inst = prefill ? th->max_punits_inst : 0;
    a.batch = th->batch; a.total_q = th->total_q; a.kv_fmt = th->kv_fmt;
    a.max_unit_items = prefill ? th->max_punit_items : 0;
    a.scale_log2e = c->scale_log2e;
    a.out_f32 = c->cfg.dtype == MATKV_BF16 && c->cfg.out_f32;
    a.off_inst = c->tl.off_inst; a.off_items = c->tl.off_items;
    a.off_units = prefill ? c->tl.off_punits : (a.shared ? c->tl.off_sunits : c->tl.off_dunits);
    *out_args = a;
    return MATKV_OK;
}

static matkv_status attn_common(matkv_ctx* c, const char* name, int prefill, int32_t layer, const void* q,
                                const void* table, const void* tail_k, const void* tail_v, void* out,
                                bool static_scratch = false) {
    AttnArgs a;
    matkv_status st = attn_args(c, name, prefill, layer, q, table, tail_k, tail_v, out, &a);
    if (st != MATKV_OK) return st;
    if (static_scratch) {
        const TableHost* th = find_table(c, table);
        const size_t need_p = (size_t)th->n_decode_slots * a.Hq * (a.D + 4) * sizeof(float);
        const size_t need_c = (size_t)a.batch * a.Hkv * kDecodeCounterStride * sizeof(int32_t);
        if (need_p > kStaticPartialBytes || need_c > kStaticCounterBytes)
            return fail(c, MATKV_ENOMEM, "%s: this batch needs %zu bytes of partial results and %zu bytes of counters, the static scratch holds %zu and %zu",
                        name, need_p, need_c, kStaticPartialBytes, kStaticCounterBytes);
        a.counters = reinterpret_cast<int32_t*>(c->static_scratch);
        a.partials = reinterpret_cast<float*>(c->static_scratch + kStaticCounterBytes);
        // the array keeps whatever the last call on this device left: the counters start at zero
        // (a fill kernel, so that the call can be recorded into a graph)
        const int n_ints = (int)(need_c / sizeof(int32_t));
        hipLaunchKernelGGL(zero_ints_kernel, dim3((n_ints + 255) / 256), dim3(256), 0, c->compute, a.counters, n_ints);
        HIP_TRY(c, hipGetLastError());
    }
    const bool want_mfma = prefill || a.variant == 0 || a.variant >= 9000;
    if (attn_prefill_supported(a, c->cfg.dtype)) HIP_TRY(c, launch_attn_prefill(a, c->cfg.dtype, c->compute));
    else if (want_mfma && attn_mfma_supported(a, c->cfg.dtype)) HIP_TRY(c, launch_attn_mfma(a, c->cfg.dtype, c->compute));
    else if (a.kv_fmt != MATKV_PAGE_PLAIN) return fail(c, MATKV_EUNSUPPORTED, "%s: compressed pages need the matrix-core kernels (decode_variant 0 or 90xx)", name);
    else HIP_TRY(c, launch_attn_rows(a, c->cfg.dtype, c->compute));
    return MATKV_OK;
}

matkv_status matkv_prefill_attn(matkv_ctx* c, int32_t layer, const void* q, const void* table,
                                const void* tail_k, const void* tail_v, void* out) {
    return attn_common(c, "prefill_attn", 1, layer, q, table, tail_k, tail_v, out);
}

matkv_status matkv_decode_attn(matkv_ctx* c, int32_t layer, const void* q, const void* table,
                               const void* tail_k, const void* tail_v, void* out) {
    return attn_common(c, "decode_attn", 0, layer, q, table, tail_k, tail_v, out);
}

matkv_status matkv_decode_attn_static(matkv_ctx* c, int32_t layer, const void* q, const void* table,
                                      const void* tail_k, const void* tail_v, void* out) {
    return attn_common(c, "decode_attn_static", 0, layer, q, table, tail_k, tail_v, out, true);
}

matkv_status matkv_decode_step(matkv_ctx* c, int32_t layer, const void* hidden, const void* w_k, const void* w_v,
                               const void* q, const void* table, void* tail_k, void* tail_v, void* out) {
    if (c && (!hidden || !w_k || !w_v)) return fail(c, MATKV_EINVAL, "decode_step: null pointer");
    if (c && (!aligned16(hidden) || !aligned16(w_k) || !aligned16(w_v)))
        return fail(c, MATKV_EINVAL, "decode_step: pointers must be 16-byte aligned");
    AttnArgs a;
    matkv_status st = attn_args(c, "decode_step", 0, layer, q, table, tail_k, tail_v, out, &a);
    if (st != MATKV_OK) return st;
    TableHost* th = find_table(c, table);
    if (th->min_tail_len < 1) return fail(c, MATKV_EINVAL, "decode_step: a tail holds no row for the new token");
    MaterializeArgs m{};
    m.hidden = hidden; m.w_k = w_k; m.w_v = w_v; m.k_out = tail_k; m.v_out = tail_v;
    m.rope = reinterpret_cast<const RopeEntry*>(c->workspace + c->wl.off_rope);
    m.table = reinterpret_cast<const char*>(table); m.off_inst = c->tl.off_inst;
    m.pos0 = 0; m.token_stride = c->cfg.max_tail_tokens;
    m.rows_per_instance = 1; m.batch = th->batch; m.n_tokens = th->batch;
    m.Hkv = c->cfg.n_kv_heads; m.D = c->cfg.head_dim; m.Hd = c->cfg.hidden;
    if (decode_step_supported(a, m, c->cfg.dtype)) {
        HIP_TRY(c, launch_decode_step(a, m, c->cfg.dtype, c->compute));
        return MATKV_OK;
    }
    // shapes the fused kernel does not cover: the two launches it stands for
    const bool want_mfma = a.variant == 0 || a.variant >= 9000;
    if (a.kv_fmt != MATKV_PAGE_PLAIN && !(want_mfma && attn_mfma_supported(a, c->cfg.dtype)))
        return fail(c, MATKV_EUNSUPPORTED, "decode_step: compressed pages need the matrix-core kernels (decode_variant 0 or 90xx)");
    HIP_TRY(c, launch_materialize(m, c->cfg.dtype, c->compute));
    if (want_mfma && attn_mfma_supported(a, c->cfg.dtype)) HIP_TRY(c, launch_attn_mfma(a, c->cfg.dtype, c->compute));
    else HIP_TRY(c, launch_attn_rows(a, c->cfg.dtype, c->compute));
    return MATKV_OK;
}

matkv_status matkv_chunk_attn(matkv_ctx* c, int32_t layer, const void* q, const void* blob, int32_t n_tokens, void* out) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!q || !blob || !out) return fail(c, MATKV_EINVAL, "chunk_attn: null pointer");
    if (!aligned16(q) || !aligned16(blob) || !aligned16(out)) return fail(c, MATKV_EINVAL, "chunk_attn: pointers must be 16-byte aligned");
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, MATKV_EINVAL, "chunk_attn: layer %d outside 0..%d", layer, c->cfg.n_layers - 1);
    if (n_tokens < 0 || n_tokens > 65535) return fail(c, MATKV_EINVAL, "chunk_attn: n_tokens=%d outside 0..65535", n_tokens);
    if (n_tokens == 0) return MATKV_OK;
    const matkv_config& cfg = c->cfg;
    const size_t head_bytes = (size_t)n_tokens * cfg.head_dim * elem_bytes(cfg);
    const char* k_layer = static_cast<const char*>(blob) + (size_t)layer * 2 * cfg.n_kv_heads * head_bytes;
    AttnArgs a{};
    a.q = q; a.out = out;
    a.tail_k = k_layer; a.tail_v = k_layer + (size_t)cfg.n_kv_heads * head_bytes;
    a.table = c->workspace + c->wl.off_chunk;
    a.off_inst = kChunkOffInst; a.off_items = kChunkOffItem; a.off_units = kChunkOffUnit;
    a.partials = reinterpret_cast<float*>(c->workspace + c->wl.off_partials);
    a.counters = reinterpret_cast<int32_t*>(c->workspace + c->wl.off_counters);
    a.layer = 0; a.n_layers = cfg.n_layers;      // the layer is in the pointers: the kernels see a tail, not a blob
    a.Hq = cfg.n_q_heads; a.Hkv = cfg.n_kv_heads; a.D = cfg.head_dim;
    a.max_tail = n_tokens;
    a.prefill = 2; a.rows = n_tokens; a.n_units = 1; a.max_units_inst = 1;
    a.batch = 1; a.total_q = n_tokens; a.max_unit_items = 1;
    a.scale_log2e = c->scale_log2e;
    a.out_f32 = cfg.dtype == MATKV_BF16 && cfg.out_f32;
    const bool tiles = attn_prefill_supported(a, cfg.dtype);
    if (!tiles) {
        // the row-per-workgroup kernel leaves a partial and a counter per (row, head) in the workspace
        const size_t need_f = (size_t)n_tokens * cfg.n_q_heads * (cfg.head_dim + 4);
        const size_t need_c = (size_t)n_tokens * cfg.n_kv_heads;
        if (need_f > c->wl.partial_floats || need_c > c->wl.n_counters)
            return fail(c, MATKV_ENOMEM, "chunk_attn: the workspace of this configuration holds the partial results of %zu rows, the chunk has %d",
                        std::min(c->wl.partial_floats / ((size_t)cfg.n_q_heads * (cfg.head_dim + 4)), c->wl.n_counters / cfg.n_kv_heads), n_tokens);
    }
    // the one-instance table depends on the chunk's length alone: written again only when that
    // changes (a launch of its own costs 4-5 us per layer), always inside a capture (a replay
    // must not depend on what ran before it), and after any replay
    if (c->capturing || c->chunk_table_tokens != n_tokens) {
        HIP_TRY(c, launch_chunk_table(c->workspace + c->wl.off_chunk, n_tokens, c->compute));
        c->chunk_table_tokens = c->capturing ? -1 : n_tokens;
    }
    if (tiles) HIP_TRY(c, launch_attn_prefill(a, cfg.dtype, c->compute));
    else HIP_TRY(c, launch_attn_rows(a, cfg.dtype, c->compute));
    return MATKV_OK;
}

matkv_status matkv_probe_read(matkv_ctx* c, const void* src, size_t bytes) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!src || !aligned16(src) || bytes == 0 || (bytes % 16)) return fail(c, MATKV_EINVAL, "probe_read: src / bytes");
    // sink: the last word of the rotary-table page of the workspace (never read by any kernel)
    unsigned* sink = reinterpret_cast<unsigned*>(c->workspace + c->wl.off_rope + 4096 - 4);
    HIP_TRY(c, launch_probe_read(src, bytes, sink, c->compute));
    return MATKV_OK;
}

// -------------------------------------------------------------------------------- graphs ----

matkv_status matkv_graph_begin(matkv_ctx* c) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (c->capturing) return fail(c, MATKV_EBUSY, "graph_begin: a capture is already open");
    matkv_graph* g = new (std::nothrow) matkv_graph();
    if (!g) return fail(c, MATKV_ENOMEM, "graph_begin: out of host memory");
    hipError_t e = hipStreamBeginCapture(c->compute, hipStreamCaptureModeRelaxed);
    if (e != hipSuccess) { delete g; return hip_fail(c, e, "hipStreamBeginCapture"); }
    c->capturing = true;
    c->cap = g;
    return MATKV_OK;
}

matkv_status matkv_graph_end(matkv_ctx* c, matkv_graph** out) {
    if (!c || !out) return MATKV_EINVAL;
    if (!c->capturing) return fail(c, MATKV_EINVAL, "graph_end: no capture is open");
    matkv_graph* g = c->cap;
    c->capturing = false;
    c->cap = nullptr;
    hipError_t e = hipStreamEndCapture(c->compute, &g->graph);
    if (e == hipSuccess) e = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (e != hipSuccess) {
        if (g->graph) (void)hipGraphDestroy(g->graph);
        delete g;
        return hip_fail(c, e, "graph_end");
    }
    try {
        c->graphs.push_back(g);
    } catch (...) {
        (void)hipGraphExecDestroy(g->exec);
        (void)hipGraphDestroy(g->graph);
        delete g;
        return fail(c, MATKV_ENOMEM, "graph_end: out of host memory");
    }
    *out = g;
    return MATKV_OK;
}

matkv_status matkv_graph_launch(matkv_ctx* c, matkv_graph* g) {
    matkv_status st = precheck(c);
    if (st != MATKV_OK) return st;
    if (!g || !g->exec) return fail(c, MATKV_EINVAL, "graph_launch: null graph");
    if (c->capturing) return fail(c, MATKV_EBUSY, "graph_launch: a capture is open");
    // the tables must still be cut the way they were when the calls were recorded
    for (auto& e : g->tables) {
        TableHost* th = find_table(c, e.table);
        if (!th) return fail(c, MATKV_EINVAL, "graph_launch: a recorded table no longer exists");
        if ((e.decode && th->sig_decode != e.sig_decode) || (e.prefill && th->sig_prefill != e.sig_prefill))
            return fail(c, MATKV_EINVAL, "graph_launch: a table has been re-assembled into a different partition since the recording");
        // a load into one of its slots since the recording: the replay must not race with the copy
        st = table_pages_ready(c, *th, "graph_launch");
        if (st != MATKV_OK) return st;
    }
    // the recorded tail advances must still fit
    for (auto& adv : g->advances) {
        TableHost* th = find_table(c, adv.first);
        if (!th) return fail(c, MATKV_EINVAL, "graph_launch: a recorded table no longer exists");
        if (th->max_tail_len + adv.second > c->cfg.max_tail_tokens)
            return fail(c, MATKV_EINVAL, "graph_launch: tail would hold %d tokens, max_tail_tokens=%d", th->max_tail_len + adv.second, c->cfg.max_tail_tokens);
    }
    for (auto& adv : g->advances) {
        TableHost* th = find_table(c, adv.first);
        th->max_tail_len += adv.second; th->min_tail_len += adv.second;
    }
    c->chunk_table_tokens = -1;                // the replay may hold a chunk attention of another length
    HIP_TRY(c, hipGraphLaunch(g->exec, c->compute));
    return MATKV_OK;
}

matkv_status matkv_graph_destroy(matkv_ctx* c, matkv_graph* g) {
    if (!c || !g) return MATKV_EINVAL;
    for (size_t i = 0; i < c->graphs.size(); ++i) {
        if (c->graphs[i] == g) {
            (void)hipStreamSynchronize(c->compute);
            if (g->exec) (void)hipGraphExecDestroy(g->exec);
            if (g->graph) (void)hipGraphDestroy(g->graph);
            delete g;
            c->graphs.erase(c->graphs.begin() + i);
            return MATKV_OK;
        }
    }
    return fail(c, MATKV_EINVAL, "graph_destroy: unknown graph");
}

}  // extern "C"
