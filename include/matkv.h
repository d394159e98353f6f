/*
 * libmatkv - the inference-time hot path of MatKV on one MI355X (gfx950).
 *
 * MatKV (paper Section III) precomputes the key/value tensors of every RAG
 * chunk once ("materialization"), stores them, and at query time loads them
 * instead of recomputing them; the question's tokens and every generated token
 * then attend over a cache assembled from the loaded chunk KVs followed by their
 * own KVs.  This library is that path and nothing else:
 *
 *   matkv_materialize       K = RoPE(X Wk^T), V = X Wv^T of one layer   (III-B steps 1-3)
 *   matkv_chunk_attn        a chunk's own causal attention while it is materialized (III-B step 2)
 *   matkv_compress          blob -> E4M3 codes + per-head power-of-two scales (III-C, compression)
 *   matkv_load              pinned-host KV blob -> HBM slot, side stream (IV, load_KV)
 *   matkv_load_file         the same from a file, through pinned bounce buffers (IV, load_KV)
 *   matkv_store_file        device blob -> file, through the same buffers       (IV, store_KV)
 *   matkv_assemble          page table of a batch, no data movement      (IV, put_KV)
 *   matkv_prefill_attn      question rows over [chunks | question]       (V-A "prefill time")
 *   matkv_decode_attn       newest token over [chunks | tail]            (V-A "decode time")
 *   matkv_decode_step       new token's K/V projection + decode attention, one launch
 *
 * Conventions
 *   - Plain C ABI.  Pointers are DEVICE pointers unless the name or the comment
 *     says "host".  The library allocates no device memory: slots, tails, Q/O,
 *     the workspace and cache tables belong to the caller.
 *   - All compute entry points enqueue on the compute stream given at creation
 *     and return without waiting; matkv_load enqueues on the load stream.
 *   - Every entry point returns a matkv_status; nothing aborts or prints, and no C++
 *     exception leaves the library (host allocation failures become MATKV_ENOMEM).
 *     After a failure matkv_last_error() holds a one-line reason.  Arguments are
 *     validated before anything is enqueued.
 *   - Element type (config.dtype): MATKV_BF16 (bf16 storage, fp32 arithmetic,
 *     one round-to-nearest-even on store) or MATKV_F32.
 *
 * Layouts (s = bytes per element)
 *   blob / slot   [layer][K|V][Hkv][n_tokens][D]        dense, no header; one chunk is
 *                 one contiguous copy and each (layer, K|V, head) is a contiguous stream
 *   tail (layer)  [max_batch][Hkv][max_tail_tokens][D]  one buffer for K, one for V;
 *                 holds the question's and the generated tokens' KVs
 *   Q, O prefill  [sum of question lengths][Hq][D]      instances back to back
 *   Q, O decode   [batch][Hq][D]
 *   hidden        [tokens][hidden]   weights [Hkv*D][hidden] (row = output feature)
 *
 * Positions: every chunk is rotated from position 0, whatever place it later takes
 * in a prompt (Section III-B), so a chunk is materialized with pos0 = 0; tail token j
 * of instance b sits at position pos_base[b] + j.  Attention takes Q already rotated.
 */
#ifndef MATKV_H
#define MATKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct matkv_ctx matkv_ctx;      /* opaque, host memory, owned by the library */
typedef struct matkv_graph matkv_graph;  /* opaque captured command sequence */

typedef enum {
    MATKV_OK = 0,
    MATKV_EINVAL = 1,        /* bad argument (null, misaligned, out of range, wrong size) */
    MATKV_EUNSUPPORTED = 2,  /* valid but not built (head_dim, group size, dtype) */
    MATKV_ENOTREADY = 3,     /* a page's load has neither completed nor been waited for */
    MATKV_EBUSY = 4,         /* resource in use (capture already open, ticket ring full) */
    MATKV_EHIP = 5,          /* a HIP call failed; sticky until the context is destroyed */
    MATKV_ENOMEM = 6,        /* host allocation failed or caller's buffer too small */
    MATKV_EIO = 7            /* reading a file failed or it ended early */
} matkv_status;

typedef enum { MATKV_F32 = 0, MATKV_BF16 = 1 } matkv_dtype;

typedef struct {
    int32_t n_layers;
    int32_t n_q_heads;        /* Hq, multiple of n_kv_heads; Hq/Hkv in {1,2,3,4,8} */
    int32_t n_kv_heads;       /* Hkv */
    int32_t head_dim;         /* D in {64, 128} */
    int32_t hidden;           /* Hd, multiple of 64 */
    int32_t dtype;            /* matkv_dtype */
    float rope_base;          /* theta_j = rope_base^(-2j/D), half-split pairing (j, j+D/2) */
    float softmax_scale;      /* 0 selects 1/sqrt(D) */
    int32_t max_batch;        /* instances per cache table */
    int32_t max_pages;        /* chunks per instance */
    int32_t max_tail_tokens;  /* question + generated tokens per instance, multiple of 8 */
    int32_t decode_units;     /* decode workgroups per (instance, KV head); 0 = chosen per table */
    int32_t decode_variant;   /* decode kernel shape; 0 = default.  9000 + 10 * (blocks of loads in flight)
                               * + waves = matrix-core kernel (9024, 9034, 9028, 9022 are built);
                               * 100 * waves + loads in flight = plain-ALU kernel (402 .. 108) */
    int32_t out_f32;          /* 1: the attention entry points of a bf16 configuration write `out` as float
                               * ([..][Hq][D] floats, unrounded; Q, K and V stay bf16); 0: out has the
                               * configuration's element type.  Ignored for MATKV_F32. */
} matkv_config;

/* One loaded chunk: the device slot that holds its blob and its token count (host struct). */
typedef struct {
    const void* slot;
    int32_t n_tokens;
    int32_t format;           /* matkv_page_format of the blob in the slot */
} matkv_page;

/* A slot holds either the blob as matkv_materialize writes it, or its compressed form
 * (matkv_compress): one E4M3 byte per element and one power-of-two scale per
 * (layer, K or V, KV head).  The pages of one cache table share one format. */
typedef enum { MATKV_PAGE_PLAIN = 0, MATKV_PAGE_E4M3 = 1 } matkv_page_format;

typedef struct { uint64_t id; } matkv_ticket;

/* ---- sizes (pure host arithmetic; usable without a GPU) ------------------------------ */

/* Bytes of one chunk blob: n_layers * 2 * Hkv * n_tokens * D * s.  0 on a bad config. */
size_t matkv_blob_bytes(const matkv_config* cfg, int32_t n_tokens);
/* Bytes of the compressed form of a chunk blob (matkv_compress): the codes
 * [n_layers][2][Hkv][n_tokens][D], one byte each, padded to 16 bytes; then the scales
 * [n_layers][2][Hkv] as float, padded to 16 bytes.  0 on a bad config. */
size_t matkv_compressed_blob_bytes(const matkv_config* cfg, int32_t n_tokens);
/* Bytes of one layer's tail buffer (K or V): max_batch * Hkv * max_tail_tokens * D * s. */
size_t matkv_tail_bytes(const matkv_config* cfg);
/* Device bytes the caller must provide as workspace: rotary table, arrival counters and the
 * split partials of the attention kernels; for bf16 / head_dim 128 at least 16 MiB of partials,
 * which the tiled projection uses when two workgroups share a tile. */
size_t matkv_workspace_bytes(const matkv_config* cfg);
/* Device bytes of one cache table (matkv_assemble's output). */
size_t matkv_table_bytes(const matkv_config* cfg);
/* MATKV_OK if the configuration is supported, else EINVAL / EUNSUPPORTED. */
matkv_status matkv_config_check(const matkv_config* cfg);
const char* matkv_status_string(matkv_status s);

/* ---- context -------------------------------------------------------------------------- */

/* Creates a context on the current device.  workspace: device buffer of at least
 * matkv_workspace_bytes(cfg), 256-byte aligned, zeroed by this call (on the compute
 * stream) and owned by the caller for the context's lifetime.  compute_stream and
 * load_stream are hipStream_t handles (0 = the null stream); they must differ for loads
 * to overlap compute and must both have default priority.  The runtime deals a process's
 * streams onto a few hardware queues (four by default) in creation order: two streams that
 * land on one queue run one behind the other, so create the pair early and keep it. */
matkv_status matkv_create(const matkv_config* cfg, void* workspace, size_t workspace_bytes,
                          void* compute_stream, void* load_stream, matkv_ctx** out);
/* Waits for both streams, destroys events and open graphs, frees host bookkeeping. */
matkv_status matkv_destroy(matkv_ctx* ctx);
/* Reason of the last failure on this context ("" if none).  Valid until the next call. */
const char* matkv_last_error(const matkv_ctx* ctx);

/* ---- M: materialization (Section III-B steps 2-3; Section IV store_KV's compute half) --- */

/* One layer, n_tokens rows:  K[g][i][:] = RoPE(Wk_g hidden[i], pos0 + i),
 * V[g][i][:] = Wv_g hidden[i].  k_out / v_out point at element [0][0][0] of a
 * [Hkv][token_stride][D] region (inside a blob, a slot or a private buffer); rows
 * 0..n_tokens-1 of each head are written.  A chunk uses pos0 = 0.  No bias, no norm:
 * hidden is whatever the layer would feed its K/V projections. */
matkv_status matkv_materialize(matkv_ctx* ctx, const void* hidden, const void* w_k,
                               const void* w_v, int32_t n_tokens, int64_t pos0,
                               void* k_out, void* v_out, int64_t token_stride);

/* The attention a chunk performs on itself while it is materialized (Section III-B: each chunk
 * is prefilled on its own, its tokens at positions 0, 1, ...): row i, head h
 * (KV head h / (Hq/Hkv)) = softmax over the chunk's own tokens j <= i of scale * q.k, times V.
 * Together with matkv_materialize this is the part of a chunk's forward pass that reads and
 * writes K/V; the rest of the layer (norms, output projection, MLP) is the caller's.
 * q, out: device [n_tokens][Hq][D], q already rotated to positions 0..n_tokens-1.  blob: device
 * blob of n_tokens tokens whose `layer` section matkv_materialize has written (same stream, or
 * ordered before this call).  Runs on the compute stream; capturable.  n_tokens = 0 is a no-op;
 * at most 65535.  Shapes outside the matrix-core kernel (fp32, head_dim 64) keep one partial
 * result per (row, head) in the workspace: MATKV_ENOMEM when the chunk has more rows than the
 * configuration's workspace covers (max_batch * max_tail_tokens). */
matkv_status matkv_chunk_attn(matkv_ctx* ctx, int32_t layer, const void* q, const void* blob,
                              int32_t n_tokens, void* out);

/* Compressed form of a materialized chunk (the paper leaves KV compression as its lever on
 * storage cost and load time, Section III-C; the scheme is this library's): for every
 * (layer, K or V, KV head) the scale s is the smallest power of two with max|x| <= 448 s over
 * the head's n_tokens x D values (1 if they are all zero, never below 2^-60), and every value
 * becomes the E4M3 code (OCP FP8, largest value 448, round to nearest even) of x / s.  A reader
 * sees code * s.  blob: device, bf16, matkv_blob_bytes(cfg, n_tokens); out: device,
 * matkv_compressed_blob_bytes(cfg, n_tokens), 16-byte aligned, must not overlap blob.  Runs
 * on the compute stream; capturable.  bf16 configurations only (else MATKV_EUNSUPPORTED).
 * Load it like any blob (matkv_load / matkv_load_file accept either size) and name the format
 * in matkv_page.format; attention over compressed pages needs bf16 and head_dim 128. */
matkv_status matkv_compress(matkv_ctx* ctx, const void* blob, int32_t n_tokens, void* out);

/* The same projection for the newest tail rows of every instance of a cache table
 * (question tokens at prefill, the generated token at each decode step); where rows go
 * and which positions they take is read on the device from the table, so the call can
 * be captured and replayed.  rows_per_instance < 0: instance b contributes its whole
 * question (q_len[b] rows, hidden = [sum q_len][Hd], written to tail rows 0..q_len[b]-1);
 * rows_per_instance = r > 0: every instance contributes r rows (hidden = [batch*r][Hd])
 * written to tail rows tail_len[b]-r .. tail_len[b]-1.  Row j takes position
 * pos_base[b] + j.  tail_k / tail_v: this layer's tail buffers. */
matkv_status matkv_materialize_tail(matkv_ctx* ctx, const void* hidden, const void* w_k,
                                    const void* w_v, const void* table,
                                    int32_t rows_per_instance, void* tail_k, void* tail_v);

/* ---- L: load (Section IV load_KV, host-memory-to-HBM half) ------------------------------ */

/* Asynchronous byte-exact copy of one blob, pinned host memory -> device slot, on the load
 * stream.  host_blob must be pinned (hipHostMalloc) and stay valid until the ticket
 * completes; bytes must equal matkv_blob_bytes(cfg, n_tokens) or
 * matkv_compressed_blob_bytes(cfg, n_tokens) and fit slot_bytes.  If a cache
 * table still points into the slot, the copy is ordered after all compute work enqueued so
 * far; if that table has since been re-assembled onto other slots, only after the work that
 * was enqueued up to that re-assembly (so the next instance's load runs beside the current
 * instance's kernels whichever of the two is enqueued first).  A table that still points
 * into the slot cannot be read again (attention, graph replay) until the new copy has been
 * waited for or has finished: such a call returns MATKV_ENOTREADY instead of racing with
 * the copy.  Errors: EINVAL (null, size mismatch, not pinned, slot too small), EBUSY (more than
 * 4096 tickets outstanding; a graph is being recorded), EHIP. */
matkv_status matkv_load(matkv_ctx* ctx, const void* host_blob, size_t bytes, int32_t n_tokens,
                        void* device_slot, size_t slot_bytes, matkv_ticket* out);
/* The storage half of load_KV (Section IV: materialized KVs live as raw bytes on flash storage):
 * the blob is `bytes` bytes at `offset` of the open file descriptor fd.  The call validates its
 * arguments, queues the request and returns; it does not read.  Reader threads owned by the
 * context (started at the first call) take the queued requests in order, piece by piece (8 MiB,
 * three preads in flight at different offsets), each piece into a pinned bounce buffer and from
 * there onto the load stream; the ticket completes when the last piece's copy does.  fd must
 * stay open, and the file unchanged, until then.  matkv_query never blocks (MATKV_ENOTREADY
 * while pieces are still being read); matkv_wait and matkv_sync block the host until the last
 * piece has been enqueued (matkv_sync: until it has landed) - work already enqueued on the compute
 * stream keeps running meanwhile.  A descriptor opened with O_DIRECT needs offset and bytes to
 * be multiples of the device's block size (4096 is safe; a blob of a multiple of 8 tokens is a
 * multiple of 4096 at head_dim 128); where the system cannot do direct I/O into pinned
 * GPU-visible memory the pieces pass through one more host copy in the reader thread.  A read
 * error or a file shorter than the blob makes the TICKET fail: matkv_wait / matkv_query /
 * matkv_sync on it return MATKV_EIO (reason in matkv_last_error), part of the slot may have been
 * overwritten, and a table over the slot is refused with MATKV_EIO until another load into it
 * succeeds.  One load per slot at a time: a load (of either kind) into a slot whose file load is
 * still being read returns MATKV_EBUSY.  Requests still queued when the context is destroyed are
 * dropped.  Other errors as matkv_load. */
matkv_status matkv_load_file(matkv_ctx* ctx, int fd, uint64_t offset, size_t bytes, int32_t n_tokens,
                             void* device_slot, size_t slot_bytes, matkv_ticket* out);
/* The storage half of store_KV (Section IV): writes `bytes` of device memory (a materialized blob
 * or any part of one) to the open file descriptor at `offset`, through the same pinned bounce
 * buffers, after all work enqueued on the compute stream so far and after every queued file load
 * has been read.  Synchronous: returns when the last byte has been handed to pwrite (no fsync).  O_DIRECT descriptors: as for matkv_load_file.
 * Errors: EINVAL, EIO, EHIP, ENOMEM. */
matkv_status matkv_store_file(matkv_ctx* ctx, int fd, uint64_t offset, const void* device_blob, size_t bytes);
/* Makes the compute stream wait for the ticket's copy (does not block the host). */
matkv_status matkv_wait(matkv_ctx* ctx, matkv_ticket t);
/* MATKV_OK if the copy has finished, MATKV_ENOTREADY if not; never blocks. */
matkv_status matkv_query(matkv_ctx* ctx, matkv_ticket t);
/* Blocks the host until the ticket's copy has finished. */
matkv_status matkv_sync(matkv_ctx* ctx, matkv_ticket t);

/* ---- A: cache assembly (Section IV put_KV) ---------------------------------------------- */

/* Builds the cache table of a batch: per instance the ordered list of loaded pages followed
 * by its tail.  No KV bytes move.  pages_host [batch][cfg.max_pages] and n_pages_host,
 * q_len_host [batch] are host arrays; pos_base_host [batch] may be NULL (then the first
 * question token of instance b takes position sum of its pages' n_tokens).  The table's
 * tail_len starts at q_len.  Every page whose slot was a matkv_load target must have been
 * waited for or completed, else MATKV_ENOTREADY (the attention entry points and
 * matkv_graph_launch make the same check for loads issued after the table was built).
 * A slot that a live table points into may be the target of a new load at any time: the copy
 * is ordered behind the work already enqueued instead of being refused.  table: device buffer
 * of matkv_table_bytes(cfg), written on the compute stream. */
matkv_status matkv_assemble(matkv_ctx* ctx, const matkv_page* pages_host,
                            const int32_t* n_pages_host, const int32_t* q_len_host,
                            const int64_t* pos_base_host, int32_t batch, void* table);
/* Host-only preview of the decode work partition matkv_assemble builds for one instance of a
 * batch of `batch` instances like it (no GPU is touched): page_tokens_host[n_pages] are the
 * chunk lengths, q_len the question length.  Unit u streams unit_tokens_out[u] page tokens and
 * is made of unit_items_out[u] page pieces; the last unit also owns the tail.  Returns the
 * number of units (at most cap), or -1 on a bad argument.  Either output may be NULL. */
int32_t matkv_plan_decode_units(const matkv_config* cfg, const int32_t* page_tokens_host,
                                int32_t n_pages, int32_t batch, int32_t q_len,
                                int32_t* unit_tokens_out, int32_t* unit_items_out, int32_t cap);
/* Host-only preview of the shared decode partition (see matkv_table_shared_units) that
 * matkv_assemble would build for a batch (no GPU is touched).  page_ids_host /
 * page_tokens_host: [batch][max_pages], instance b uses its first n_pages_host[b] entries;
 * equal ids mean the same slot.  Unit u is written to units_out[u * 52 ..]: id of its first
 * page (-1: it starts with a tail), page tokens it streams, the instance whose tail it holds
 * (-1: none), number of users, then 16 triples (instance, partial slot, page tokens of the
 * unit that this user sees), -1 / -1 / 0 where unused.  slots_out (may be NULL): [batch][2] =
 * first partial slot and number of slots of each instance.  Returns the number of units (at
 * most cap), 0 if no shared partition would be built, -1 on a bad argument. */
int32_t matkv_plan_shared_units(const matkv_config* cfg, const int32_t* page_ids_host,
                                const int32_t* page_tokens_host, const int32_t* n_pages_host,
                                const int32_t* q_len_host, int32_t batch, int32_t* units_out,
                                int32_t cap, int32_t* slots_out);
/* Decode work units of the table's shared partition, 0 if matkv_assemble built none, -1 if the
 * table is unknown.  When two or more instances of a batch point at the same slot (the same
 * chunk, retrieved by several requests), matkv_assemble cuts the batch's DISTINCT pages and its
 * tails into equal work units and notes with every piece the instances that use it: the decode
 * attention then reads a shared chunk once for up to 16 / (Hq/Hkv) instances at a time instead
 * of once per instance.  Built when the distinct pages are at least a twentieth fewer tokens
 * than all uses together, for plain or compressed pages, bf16, head_dim 128, decode_units = 0
 * and decode_variant = 0; results are the same as without it (every instance still gets exact
 * attention over its own cache). */
int32_t matkv_table_shared_units(matkv_ctx* ctx, const void* table);
/* tail_len[b] += n for every instance of the table (a one-wave kernel; capturable). */
matkv_status matkv_advance(matkv_ctx* ctx, void* table, int32_t n);

/* ---- P / D: attention over the assembled cache (one layer, whole batch) ------------------- */

/* Question row i of instance b, head h (KV head h / (Hq/Hkv)):
 *   softmax over { every token of every page } U { tail tokens j <= i } of scale * q.k,
 *   times V.  q/out: [sum q_len][Hq][D] in the table's instance order. */
matkv_status matkv_prefill_attn(matkv_ctx* ctx, int32_t layer, const void* q, const void* table,
                                const void* tail_k, const void* tail_v, void* out);
/* The newest token of each instance: all page tokens and tail tokens 0..tail_len[b]-1.
 * q/out: [batch][Hq][D]. */
matkv_status matkv_decode_attn(matkv_ctx* ctx, int32_t layer, const void* q, const void* table,
                               const void* tail_k, const void* tail_v, void* out);
/* matkv_decode_attn for callers that cannot allocate device memory or hand the library a
 * scratch buffer of their own choosing at this point: code under stream capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, same result.  The split partial
 * results and arrival counters that matkv_decode_attn keeps in the context's workspace live
 * here in an 8 MiB array inside the library's device image (1 MiB of counters: at most 8192
 * (instance, KV head) pairs; 7 MiB of partial results: decode units of the batch x Hq x
 * (D + 4) floats), which every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing (no hipMalloc, hipFree, hipHostMalloc), clears the counters it
 * uses with a fill kernel and can be recorded by matkv_graph_begin / end.  A batch that needs
 * more than the array holds is refused with MATKV_ENOMEM before anything is enqueued.  All
 * calls on one GPU share the array: two calls that overlap in time (other streams, other
 * contexts) race; calls on one compute stream are ordered and safe. */
matkv_status matkv_decode_attn_static(matkv_ctx* ctx, int32_t layer, const void* q, const void* table,
                                      const void* tail_k, const void* tail_v, void* out);
/* One decode step of one layer in a single launch (Section III-B steps 2-3 for the new token,
 * then Section V-A's decode attention): the same result as
 *   matkv_materialize_tail(hidden, w_k, w_v, table, 1, tail_k, tail_v) followed by
 *   matkv_decode_attn(layer, q, table, tail_k, tail_v, out),
 * i.e. K = RoPE(Wk x_b, pos_base[b] + tail_len[b] - 1) and V = Wv x_b are written (rounded to
 * the storage type) at tail row tail_len[b] - 1 of every instance, and the new token attends
 * to all page tokens and tail rows 0..tail_len[b]-1, the row just written included.
 * hidden: device [batch][hidden]; w_k, w_v: [Hkv*D][hidden]; q/out: [batch][Hq][D].
 * Call matkv_advance first, as before matkv_materialize_tail.  On bf16, head_dim 128, hidden a
 * multiple of 4096 and the default decode kernel the projection's weight reads overlap the
 * cache reads inside one kernel; other configurations run the two launches above.
 * MATKV_EINVAL if some tail is empty. */
matkv_status matkv_decode_step(matkv_ctx* ctx, int32_t layer, const void* hidden, const void* w_k,
                               const void* w_v, const void* q, const void* table, void* tail_k,
                               void* tail_v, void* out);

/* ---- measurement aid ------------------------------------------------------------------------ */

/* Streams `bytes` of device memory at `src` once with 16-byte loads (no output besides a
 * checksum sink inside the workspace) on the compute stream: the practical ceiling of a read
 * of that size on this device, to set beside the attention kernels' achieved bandwidth.
 * src 16-byte aligned, bytes a multiple of 16. */
matkv_status matkv_probe_read(matkv_ctx* ctx, const void* src, size_t bytes);

/* ---- command capture: replay a fixed sequence of the calls above without host cost ------ */

/* Between begin and end, calls to materialize_tail / advance / prefill_attn / decode_attn /
 * decode_step are recorded from the compute stream instead of executed.  Captured work reads tail
 * lengths and positions from the table on the device, so one recording of a decode step
 * serves every step.  Launch shapes are fixed at recording time: a table may be re-assembled
 * between replays (other slots, other chunk and question lengths), but if the new batch is cut
 * differently where the recording looks - for recorded decode calls another number of
 * instances or decode units or another page format, for recorded prefill calls also another
 * number of question rows - matkv_graph_launch returns MATKV_EINVAL and the calls have to be
 * recorded again. */
matkv_status matkv_graph_begin(matkv_ctx* ctx);
matkv_status matkv_graph_end(matkv_ctx* ctx, matkv_graph** out);
matkv_status matkv_graph_launch(matkv_ctx* ctx, matkv_graph* g);
matkv_status matkv_graph_destroy(matkv_ctx* ctx, matkv_graph* g);

#ifdef __cplusplus
}
#endif
#endif /* MATKV_H */
