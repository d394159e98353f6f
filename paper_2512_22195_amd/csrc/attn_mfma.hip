// Matrix-core attention over the assembled cache with the unit's TOKENS split over the waves,
// bf16, head_dim 128: the decode step (paper Section V-A "decode time": the newest token of
// each instance over every chunk key and the whole tail), alone or fused with the projection of
// that token's K/V (Section III-B steps 2-3), and - as the fallback of the row-parallel kernel in
// attn_prefill.hip - the question prefill (rows i of the question over every chunk key and
// question keys j <= i).
//
// The M dimension of the tiles is the flattened (question row, query head of one KV head)
// index, so the G query heads that share a KV head ride in the same matrix-core operation.
// Per wave and per block of 32 token rows:
//   S^T = K Q^T     mfma 16x16x32: A = K rows straight from HBM in operand layout (16 tokens x
//                   8 consecutive dims per lane), B = Q held in registers for the whole unit
//   softmax         per lane on its own column (one (row, head)) with a running maximum that
//                   the four 16-lane groups agree on through register swaps
//   O^T += V^T P^T  A = V transposed on the fly: V rows land in a private LDS strip as loaded
//                   (coalesced 16-byte loads) and come back through the transposing LDS read,
//                   B = P rounded to bf16, already sitting in operand layout
// Waves of a workgroup split the unit's tokens; workgroups split the cache; merging is the
// same as in the plain-ALU kernel.
#include "attn_common.h"
#include "gemv_common.h"

namespace matkv {
namespace {

using namespace attn;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int D = 128;
constexpr int BLK = 32;             // token rows per wave step
constexpr int VSTR = D + 16;        // bf16 elements per LDS row of the V strip (bank spread)
constexpr int ACCS = D + 4;         // floats per LDS row of the merge buffer

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& r) { return __builtin_bit_cast(bf16x8, r); }

// Transposing LDS read: the 16 lanes of a group each name 8 bytes (4 bf16); lane i of the group
// receives element i of the group's four 16-element rows.
__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t* p) {
    typedef s16x4 __attribute__((address_space(3))) * lptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(uintptr_t)p);
}

// What a fused decode step adds to the attention launch (paper Section III-B steps 2-3 for the
// newest token of every instance, then Section V-A's decode attention over everything).
struct StepArgs {
    const void* hidden;         // [batch][Hd]
    const void* w_k;            // [Hkv * D][Hd]
    const void* w_v;
    const RopeEntry* rope;
    int32_t Hd, batch;
};

// Last arrival of a fused decode step at instance b, KV head kvh: folds the units' partials and
// the newest token into the G output rows.  Wave w owns row w (query head kvh*G + w), lane l
// the dims 2l, 2l+1.  The newest token's K/V row is read back from the tail cache, where the
// projection waves left it with agent-scope stores; its loads and the partials' loads are all
// issued before anything is consumed (one memory round trip), its score is a 64-lane dot
// product, and it enters as one more contribution of weight 1.  No barrier: waves past G leave.
template <int G, int NT>
__device__ __forceinline__ void merge_decode_step(const KernelArgs& a, const InstanceInfo& inst, int b, int kvh) {
    typedef uint16_t T;
    constexpr int PSTRIDE = kPartialStride(D);
    constexpr int UPC = 32;                             // units per pass: the default partition (up to 32 units) folds in one
    const int w0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    for (int w = w0; w < G; w += NT / 64) {             // more rows than waves: a wave takes several in turn
    const int head = kvh * G + w, d = 2 * lane;

    const size_t toff = (((size_t)b * a.Hkv + kvh) * (size_t)a.max_tail + (size_t)(inst.tail_len - 1)) * D + d;
    const uint32_t kw = __hip_atomic_load(reinterpret_cast<const uint32_t*>(reinterpret_cast<const T*>(a.tail_k) + toff),
                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t vw = __hip_atomic_load(reinterpret_cast<const uint32_t*>(reinterpret_cast<const T*>(a.tail_v) + toff),
                                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t qw = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const T*>(a.q) + ((size_t)b * a.Hq + head) * D + d);

    const int n_units = inst.n_dunits;
    const float* src = a.partials + ((size_t)inst.dunit0 * a.rows * a.Hq + head) * PSTRIDE;
    const size_t ustride = (size_t)a.rows * a.Hq * PSTRIDE;
    float M = kNegBig, L = 0.f, ox = 0.f, oy = 0.f;
    for (int u0 = 0; u0 < n_units; u0 += UPC) {
        float2 av[UPC], ml[UPC];
#pragma unroll
        for (int k = 0; k < UPC; ++k) {
            const size_t uo = (size_t)min(u0 + k, n_units - 1) * ustride;
            ml[k] = ld_agent2(src + uo + D);
            av[k] = ld_agent2(src + uo + d);
        }
        float mn = M;
#pragma unroll
        for (int k = 0; k < UPC; ++k) mn = fmaxf(mn, (u0 + k < n_units) ? ml[k].x : kNegBig);
        const float cold = fast_exp2(M - mn);
        L *= cold; ox *= cold; oy *= cold;
        M = mn;
#pragma unroll
        for (int k = 0; k < UPC; ++k) {
            const float c = (u0 + k < n_units) ? fast_exp2(ml[k].x - mn) : 0.f;
            L = fmaf(ml[k].y, c, L);
            ox = fmaf(av[k].x, c, ox);
            oy = fmaf(av[k].y, c, oy);
        }
    }
    const float sx = gemv::wave_sum(gemv::dot2(qw, kw, 0.f), lane) * a.scale_log2e;
    const float mn = fmaxf(M, sx);
    const float cold = fast_exp2(M - mn), cx = fast_exp2(sx - mn);
    L = fmaf(L, cold, cx);
    ox = fmaf(ox, cold, __uint_as_float(vw << 16) * cx);
    oy = fmaf(oy, cold, __uint_as_float(vw & 0xffff0000u) * cx);
    const float inv = 1.0f / L;
    store_out2(a.out, a.out_f32, ((size_t)b * a.Hq + head) * D + d, ox * inv, oy * inv);
    }
}

// A projection wave of a fused decode step: one task = one rotary pair of K or of V of KV head
// kvh for a group of FR instances; the pair is stored (bf16, agent scope) at the newest tail
// row of each instance.  The n_waves projection waves of this KV head share the tasks round-robin.
template <int FR>
__device__ __forceinline__ void projection_tasks(const KernelArgs& a, const StepArgs& f, const InstanceInfo* __restrict__ insts,
                                                 int kvh, int wave_id, int n_waves, int lane) {
    typedef uint16_t T;
    const int groups = (f.batch + FR - 1) / FR;
    for (int task = wave_id; task < groups * D; task += n_waves) {
        const int b0 = (task / D) * FR;
        const int kv = (task % D) / (D / 2), j = task % (D / 2);
        const T* w = reinterpret_cast<const T*>(kv == 0 ? f.w_k : f.w_v);
        const T* w0 = w + ((size_t)kvh * D + j) * f.Hd;
        const T* w1 = w0 + (size_t)(D / 2) * f.Hd;
        const T* x = reinterpret_cast<const T*>(f.hidden) + (size_t)b0 * f.Hd;
        float acc0[FR], acc1[FR];
        if (f.Hd % 4096 == 0) gemv::pair_dots<FR, 8>(w0, w1, x, (size_t)f.Hd, f.batch - b0, f.Hd, lane, acc0, acc1);
        else                  gemv::pair_dots<FR, 6>(w0, w1, x, (size_t)f.Hd, f.batch - b0, f.Hd, lane, acc0, acc1);   // multiples of 3072
        if (lane < FR && b0 + lane < f.batch) {
            float r0 = 0.f, r1 = 0.f;
#pragma unroll
            for (int r = 0; r < FR; ++r) if (lane == r) { r0 = acc0[r]; r1 = acc1[r]; }
            const int b = b0 + lane;
            const int row = insts[b].tail_len - 1;
            if (row >= 0 && row < a.max_tail) {
                if (kv == 0) gemv::rotate_pair(f.rope[j], (float)(insts[b].pos_base + row), r0, r1);
                T* out = reinterpret_cast<T*>(const_cast<void*>(kv == 0 ? a.tail_k : a.tail_v)) +
                         (((size_t)b * a.Hkv + kvh) * (size_t)a.max_tail + (size_t)row) * D + j;
                __hip_atomic_store(out, f32_to_bf16_rne(r0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(out + D / 2, f32_to_bf16_rne(r1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

constexpr int kFusedMaxBatch = 4;

// Shared decode units: fold, for every user of this unit at whose counter the workgroup arrived
// last, that instance's partial slots into its G output rows - all such users at once.  A thread
// owns pairs of output elements; a wave's 64 pairs are one (user, head) row, so the number of
// slots is uniform within a wave.  users[u] = {instance, this unit's slot, first slot, slots}.
template <int G, int NT>
__device__ __forceinline__ void merge_shared(const KernelArgs& a, const int4* users, const int* lastv, int n_users, int kvh) {
    typedef uint16_t T;
    constexpr int PSTRIDE = kPartialStride(D), CB = 4, UPC = 8;
    const int total = n_users * G * (D / 2);
    const size_t ustride = (size_t)a.Hq * PSTRIDE;                     // decode: one row per slot
    for (int c0 = threadIdx.x; c0 < total; c0 += NT * CB) {
        float M[CB], L[CB], ox[CB], oy[CB];
        const float* src[CB];
        int n[CB], inst[CB], head[CB], dd[CB];
        int nmax = 0;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int col = min(c0 + cb * NT, total - 1);
            const int row = col / (D / 2), u = row / G;
            const int4 us = users[u];
            const bool live = c0 + cb * NT < total && lastv[u];
            inst[cb] = us.x; head[cb] = kvh * G + row % G; dd[cb] = (col % (D / 2)) * 2;
            n[cb] = live ? us.w : 0;
            nmax = max(nmax, n[cb]);
            src[cb] = a.partials + ((size_t)us.z * a.Hq + head[cb]) * PSTRIDE;
            M[cb] = kNegBig; L[cb] = 0.f; ox[cb] = 0.f; oy[cb] = 0.f;
        }
        for (int u0 = 0; u0 < nmax; u0 += UPC) {
            float2 av[CB][UPC], ml[CB][UPC];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int k = 0; k < UPC; ++k) {
                    const size_t uo = (size_t)min(u0 + k, max(n[cb], 1) - 1) * ustride;
                    ml[cb][k] = ld_agent2(src[cb] + uo + D);
                    av[cb][k] = ld_agent2(src[cb] + uo + dd[cb]);
                }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                float mn = M[cb];
#pragma unroll
                for (int k = 0; k < UPC; ++k) mn = fmaxf(mn, (u0 + k < n[cb]) ? ml[cb][k].x : kNegBig);
                const float cold = fast_exp2(M[cb] - mn);
                L[cb] *= cold; ox[cb] *= cold; oy[cb] *= cold;
                M[cb] = mn;
#pragma unroll
                for (int k = 0; k < UPC; ++k) {
                    const float c = (u0 + k < n[cb]) ? fast_exp2(ml[cb][k].x - mn) : 0.f;
                    L[cb] = fmaf(ml[cb][k].y, c, L[cb]);
                    ox[cb] = fmaf(av[cb][k].x, c, ox[cb]);
                    oy[cb] = fmaf(av[cb][k].y, c, oy[cb]);
                }
            }
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            if (n[cb] == 0) continue;
            const float inv = 1.0f / L[cb];
            store_out2(a.out, a.out_f32, ((size_t)inst[cb] * a.Hq + head[cb]) * D + dd[cb], ox[cb] * inv, oy[cb] * inv);
        }
    }
}

// (Second launch bound: two waves per SIMD, i.e. at most 256 registers, wherever the decode
// tile fits them - a few registers more would halve the workgroups resident per compute unit.)
// FR = 0: attention only, NW waves.  FR > 0: fused decode step - the workgroup has NW more
// waves, which project the newest token's K/V (FR instances per task) while the first NW walk
// the cache; every compute unit then holds both kinds of work side by side.  In that form each
// workgroup of a KV head arrives at the counter of EVERY instance of the batch once all its
// work is out, so the last arrival at an instance's counter knows that instance's partials and
// its newest K/V row are complete, whichever workgroups produced them.
// F8: the pages hold E4M3 codes with per-head power-of-two scales; a block's codes are widened
// to bf16 in registers (exact), the K scale multiplies the block's scores and the V scale its
// weights on their way to bf16 (exact too: powers of two), the row sums stay unscaled.
// SH: decode over the shared partition - `units` are SUnit records: one piece of a page (or one
// instance's tail) and up to 16 / G instances whose newest tokens attend to it; the rows of the
// tile are (user, query head) pairs, the piece is streamed once for all of them, every user gets
// its own partial, and the workgroup arrives at every user's counter: the last arrival at an
// instance's counter folds that instance's partial slots.
template <int G, int NW, int MS, int PF, int FR, bool F8, bool SH = false>
__global__ __launch_bounds__((FR > 0 ? 2 : 1) * NW * 64, (FR > 0 || (MS == 1 && PF <= 2)) ? 2 : 1) void attn_mfma_kernel(
        KernelArgs a, StepArgs f, const InstanceInfo* __restrict__ insts, const Item* __restrict__ items,
        const Unit* __restrict__ units) {
    constexpr int ROWS = 16 * MS;                       // (row, head) pairs per workgroup
    constexpr int NT = (FR > 0 ? 2 : 1) * NW * 64;      // threads of the workgroup
    typedef uint16_t T;
    static_assert(!SH || (FR == 0 && MS == 1), "shared units: decode tiles only");
    __shared__ int sm_last, sm_lastv[SH ? kMaxSharedUsers : (FR > 0 ? kFusedMaxBatch : 1)];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int kvh = blockIdx.y, tile = blockIdx.z;
    const int m0 = tile * ROWS;

    const SUnit* const su = reinterpret_cast<const SUnit*>(units) + blockIdx.x;     // SH only
    const Unit unit = SH ? su->u : units[blockIdx.x];

    int n_m, q_row0, tail_len = 0, tail_visible;
    if (SH) {
        n_m = su->n_users * G;
        q_row0 = 0;
        if (unit.has_tail) tail_len = insts[unit.inst].tail_len;
        tail_visible = tail_len;
    } else if (a.prefill) {
        const InstanceInfo inst = insts[unit.inst];
        n_m = inst.q_len * G;
        if (m0 >= n_m) return;                          // whole workgroup leaves together
        q_row0 = inst.cu_q;
        const int r_last = (min(m0 + ROWS, n_m) - 1) / G;
        tail_visible = r_last + 1;                      // the most any row of this tile may see
    } else {
        n_m = G;
        q_row0 = unit.inst;
        if (unit.has_tail) tail_len = insts[unit.inst].tail_len - (FR > 0 ? 1 : 0);   // fused: the newest row is not in the cache yet
        tail_visible = tail_len;
    }

    f32x4 ot[MS][8];                                    // O^T: dims 16s + 4*g4 + i of row 16j + c16
    float mrow[MS], lrow[MS];
#pragma unroll
    for (int j = 0; j < MS; ++j) {
        mrow[j] = kNegBig; lrow[j] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) ot[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // LDS: per-wave V strips during the walk, the merge buffer afterwards (same bytes).
    constexpr int V_BYTES = NW * BLK * VSTR * 2;
    constexpr int ACC_BYTES = NW * ROWS * ACCS * 4;
    __shared__ __attribute__((aligned(16))) char smem[V_BYTES > ACC_BYTES ? V_BYTES : ACC_BYTES];
    __shared__ float sm_m[NW * ROWS], sm_l[NW * ROWS];

    // shared unit: its users with their slot ranges, for the publishing and folding at the end
    __shared__ int4 sm_users[SH ? kMaxSharedUsers : 1];
    if (SH && tid < su->n_users) {
        const int inst = su->users[tid].inst;
        sm_users[tid] = make_int4(inst, su->users[tid].slot, insts[inst].sslot0, insts[inst].n_sslots);
    }

    if (FR > 0 && wave >= NW) {
        if constexpr (FR > 0)
            projection_tasks<FR>(a, f, insts, kvh, (int)blockIdx.x * NW + (wave - NW), (int)gridDim.x * NW, lane);
    } else {
    // Q in operand layout: lane (c16, g4) holds, for sub-tile j and chunk c of the head
    // dimension, the 8 dims dim0(c) .. +8 of row m0 + 16j + c16: 32c + 8*g4 for plain pages; with
    // compressed pages 16*g4 + 8*(c%2) + 64*(c/2), so that the two chunks of a pair are the 16
    // codes of one 16-byte load.  Padding rows repeat the last real row.
    auto dim0 = [&](int c) { return F8 ? 16 * g4 + 8 * (c & 1) + 64 * (c >> 1) : 32 * c + 8 * g4; };
    bf16x8 bq[MS][4];
    int vis[MS];                                        // tail rows this lane's row may see
    int row_user[MS];                                   // shared units: index of the row's user in the unit's list
#pragma unroll
    for (int j = 0; j < MS; ++j) {
        const int m = min(m0 + 16 * j + c16, n_m - 1);
        const int r = m / G, g = m % G;
        row_user[j] = r;
        int q_row = a.prefill ? q_row0 + r : q_row0;
        if (SH) {           // the record's user list comes through scalar loads; pick this lane's
#pragma unroll
            for (int k = 0; k < kMaxSharedUsers; ++k) {
                const int v = su->users[k].inst;
                q_row = (r == k) ? v : q_row;
            }
        }
        const T* qp = reinterpret_cast<const T*>(a.q) + ((size_t)q_row * a.Hq + (size_t)kvh * G + g) * D;
#pragma unroll
        for (int c = 0; c < 4; ++c) bq[j][c] = as_bf16x8(ldg16(qp + dim0(c)));
        vis[j] = (a.prefill && !SH) ? r + 1 : tail_len;
    }

    uint16_t* const vstrip = reinterpret_cast<uint16_t*>(smem) + (size_t)wave * BLK * VSTR;

    // One block's loads in registers.  Plain rows: lane (c16, g4) holds, per 16-token half, the
    // 8 dims of each of the 4 chunks of its token row, and 8 V rows' worth of 8 dims.  Code rows
    // (one byte per element): 16 dims per load, so half as many loads carry the same tokens.
    struct PlainBuf { uint4 k[2][4], v[8]; };
    struct CodeBuf { uint4 k[2][2], v[4]; };

    // Rows past the block's end are clamped to its last row and masked in the softmax.
    auto issue_plain = [&](const BlockRef<T>& r, PlainBuf& b) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const T* kp = r.k + (size_t)min(r.t0 + 16 * h + c16, r.tok_end - 1) * D;
#pragma unroll
            for (int c = 0; c < 4; ++c) b.k[h][c] = ldg16(kp + dim0(c));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            b.v[u] = ldg16(r.v + (size_t)min(r.t0 + 4 * u + g4, r.tok_end - 1) * D + 8 * c16);
    };
    // K: the two 16-byte pieces of the lane's token row that hold its dims (chunks 0-1, 2-3);
    // V: lane l takes 16 dims (l % 8) of token row 8u + l / 8.
    auto issue_codes = [&](const BlockRef<T>& r, CodeBuf& b) {
        const uint8_t* kc = reinterpret_cast<const uint8_t*>(r.k);
        const uint8_t* vc = reinterpret_cast<const uint8_t*>(r.v);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint8_t* kp = kc + (size_t)min(r.t0 + 16 * h + c16, r.tok_end - 1) * D + 16 * g4;
            b.k[h][0] = ldg16(kp);
            b.k[h][1] = ldg16(kp + 64);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            b.v[u] = ldg16(vc + (size_t)min(r.t0 + 8 * u + (lane >> 3), r.tok_end - 1) * D + 16 * (lane & 7));
    };

    // Scores, online softmax and P V of one block whose K operands are in ak and whose V rows
    // are in this wave's strip.  sc_blk: score scale of the block; pv_scale: factor of its
    // weights on their way to bf16 (both carry a compressed page's power-of-two scales).
    auto attend = [&](const BlockRef<T>& r, const uint4 (*ak)[4], float sc_blk, float pv_scale) {
        bf16x8 pb[MS];
#pragma unroll
        for (int j = 0; j < MS; ++j) {
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ak[0][c]), bq[j][c], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ak[1][c]), bq[j][c], s1, 0, 0, 0);
            }
            // lane holds tokens t0 + 4*g4 + i (s0) and t0 + 16 + 4*g4 + i (s1) of its row
            // (shared units: a row whose user does not use this piece sees none of it)
            const int limit = (SH && !((r.umask >> row_user[j]) & 1)) ? 0 : (r.is_tail ? min(r.tok_end, vis[j]) : r.tok_end);
            const int tb = r.t0 + 4 * g4;
            float sv[8];
            bool ok[8];
            float mx = kNegBig;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ok[i] = tb + i < limit;
                ok[4 + i] = tb + 16 + i < limit;
                sv[i] = ok[i] ? s0[i] * sc_blk : kNegBig;
                sv[4 + i] = ok[4 + i] ? s1[i] * sc_blk : kNegBig;
                mx = fmaxf(mx, fmaxf(sv[i], sv[4 + i]));
            }
            mx = fmaxf(mx, lane_xor(mx, 16, lane));
            mx = fmaxf(mx, lane_xor(mx, 32, lane));
            const float mn = fmaxf(mrow[j], mx);
            const float alpha = fast_exp2(mrow[j] - mn);
            mrow[j] = mn;
            float psum = 0.f;
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = ok[i] ? fast_exp2(sv[i] - mn) : 0.f;
                psum += p[i];
            }
            lrow[j] = lrow[j] * alpha + psum;
#pragma unroll
            for (int i = 0; i < 8; ++i) pb[j][i] = (__bf16)(p[i] * pv_scale);
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {   // wave-uniform: some row's maximum moved
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    ot[j][s][0] *= alpha; ot[j][s][1] *= alpha; ot[j][s][2] *= alpha; ot[j][s][3] *= alpha;
                }
            }
        }

        __builtin_amdgcn_wave_barrier();                // strip writes stay ahead of the reads below
        // lane (c16, g4) names 4 dims (4*(c16%4) ..) of token 4*g4 + c16/4 (+16 for the second
        // half) and receives dim 16s + c16 of tokens 4*g4 .. 4*g4+3: the k order of P above
        const uint16_t* vp = vstrip + (4 * g4 + (c16 >> 2)) * VSTR + 4 * (c16 & 3);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const s16x4 lo = lds_read_tr(vp + 16 * s);
            const s16x4 hi = lds_read_tr(vp + 16 * VSTR + 16 * s);
            const bf16x8 av = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int j = 0; j < MS; ++j)
                ot[j][s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[j], ot[j][s], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();                // and the next block's writes behind them
    };

    auto consume_plain = [&](const BlockRef<T>& r, const PlainBuf& b) {
        // V rows into this wave's strip, as loaded
#pragma unroll
        for (int u = 0; u < 8; ++u)
            *reinterpret_cast<uint4*>(vstrip + (4 * u + g4) * VSTR + 8 * c16) = b.v[u];
        attend(r, b.k, a.scale_log2e, 1.0f);
    };
    auto consume_codes = [&](const BlockRef<T>& r, const CodeBuf& b) {
        uint4 ak[2][4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            ak[h][0] = e4m3x8_to_bf16x8(make_uint2(b.k[h][0].x, b.k[h][0].y));
            ak[h][1] = e4m3x8_to_bf16x8(make_uint2(b.k[h][0].z, b.k[h][0].w));
            ak[h][2] = e4m3x8_to_bf16x8(make_uint2(b.k[h][1].x, b.k[h][1].y));
            ak[h][3] = e4m3x8_to_bf16x8(make_uint2(b.k[h][1].z, b.k[h][1].w));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint16_t* dst = vstrip + (8 * u + (lane >> 3)) * VSTR + 16 * (lane & 7);
            *reinterpret_cast<uint4*>(dst) = e4m3x8_to_bf16x8(make_uint2(b.v[u].x, b.v[u].y));
            *reinterpret_cast<uint4*>(dst + 8) = e4m3x8_to_bf16x8(make_uint2(b.v[u].z, b.v[u].w));
        }
        attend(r, ak, a.scale_log2e * r.sk, r.sv);
    };

    // PF blocks of loads stay in flight: block i + PF is issued right after block i is consumed.
    // The loads are issued without a branch (past the end of the wave's share they all fall on
    // one row) and the loop has one exit: only then can the compiler count the loads in flight
    // exactly, instead of waiting for all of them before each block.
    auto stream = [&](auto& walk, auto buf_tag, auto issue, auto consume) {
        decltype(buf_tag) b[PF];
        BlockRef<T> rb[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            rb[i] = walk.next_safe();
            issue(rb[i], b[i]);
        }
        do {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                if (rb[i].valid) consume(rb[i], b[i]);
                rb[i] = walk.next_safe();
                issue(rb[i], b[i]);
            }
        } while (rb[0].valid);
    };
    if constexpr (!F8) {
        Walker<T, D, NW, BLK, 8> walk(a, unit, items, kvh, tail_visible, wave);
        stream(walk, PlainBuf{}, issue_plain, consume_plain);
    } else {
        // Compressed pages first, then the (plain) tail, each in a loop of its own: one loop
        // over both kinds would put the two load patterns under a branch.
        {
            Walker<T, D, NW, BLK, 8, true> walk(a, unit, items, kvh, 0, wave);
            stream(walk, CodeBuf{}, issue_codes, consume_codes);
        }
        if (unit.has_tail && tail_visible > 0) {
            Unit tu = unit;                             // the unit's last item, alone
            tu.item0 = unit.item0 + unit.n_items - 1; tu.n_items = 1; tu.page_tokens = 0;
            tu.first.base = 0; tu.first.page_tokens = a.max_tail; tu.first.tok0 = 0; tu.first.ntok = a.max_tail;
            tu.first.fmt = 0; tu.first.scales16 = 0;
            if (SH) tu.first.umask = items[tu.item0].umask;     // the users that see it (its owner)
            Walker<T, D, NW, BLK, 8> walk(a, tu, items, kvh, tail_visible, wave);
            stream(walk, PlainBuf{}, issue_plain, consume_plain);
        }
    }

#pragma unroll
    for (int j = 0; j < MS; ++j) {
        lrow[j] += lane_xor(lrow[j], 16, lane);
        lrow[j] += lane_xor(lrow[j], 32, lane);
    }
    }   // attention waves

    // ---- per-wave states to LDS (the strips are dead now), then the common merge ----
    __syncthreads();                                    // every wave is done with its strip
    float* const sm_acc = reinterpret_cast<float*>(smem);
    if (wave < NW) {
#pragma unroll
        for (int j = 0; j < MS; ++j) {
            float* dst = sm_acc + ((size_t)wave * ROWS + 16 * j + c16) * ACCS + 4 * g4;
#pragma unroll
            for (int s = 0; s < 8; ++s)
                *reinterpret_cast<float4*>(dst + 16 * s) = make_float4(ot[j][s][0], ot[j][s][1], ot[j][s][2], ot[j][s][3]);
            if (g4 == 0) { sm_m[wave * ROWS + 16 * j + c16] = mrow[j]; sm_l[wave * ROWS + 16 * j + c16] = lrow[j]; }
        }
    }
    const int prefill = a.prefill;
    auto map = [&](int i) {
        RowMap rm;
        const int m = m0 + i;
        const int r = m / G, g = m % G;
        rm.slot_row = (prefill && !SH) ? r : 0;
        rm.head = kvh * G + g;
        rm.q_row = prefill ? q_row0 + r : q_row0;
        if (SH) { const int4 us = sm_users[r]; rm.q_row = us.x; rm.unit_slot = us.y; }
        return rm;
    };
    if constexpr (SH) {
        publish_partial<T, D, NT, NW, ROWS, ACCS>(a, sm_acc, sm_m, sm_l, n_m, map);
        // arrival at the counter of every user of this unit
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        const int n_users = n_m / G;
        if (tid < n_users) {
            const int4 us = sm_users[tid];
            const int prev = __hip_atomic_fetch_add(&a.counters[counter_index(a, us.x, kvh, 0)], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sm_lastv[tid] = (prev == us.w - 1);
            if (prev == us.w - 1)                       // ready for the next launch
                __hip_atomic_store(&a.counters[counter_index(a, us.x, kvh, 0)], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        merge_shared<G, NT>(a, sm_users, sm_lastv, n_users, kvh);
    } else if constexpr (FR == 0) {
        finish_unit<T, D, NW, NW, ROWS, ACCS>(a, unit, kvh, tile, sm_acc, sm_m, sm_l, &sm_last, min(ROWS, n_m - m0), map);
    } else {
        publish_partial<T, D, NT, NW, ROWS, ACCS>(a, sm_acc, sm_m, sm_l, G, map);
        // arrival at every instance's counter of this KV head
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (tid < f.batch) {
            const int prev = __hip_atomic_fetch_add(&a.counters[counter_index(a, tid, kvh, 0)], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sm_lastv[tid] = (prev == (int)gridDim.x - 1);
        }
        __syncthreads();
        for (int b = 0; b < f.batch; ++b) {
            if (!sm_lastv[b]) continue;                 // uniform
            merge_decode_step<G, NT>(a, insts[b], b, kvh);
            reset_counter(a, counter_index(a, b, kvh, 0));
        }
    }
}

template <int G, int NW, int MS, int PF, bool F8 = false>
hipError_t launch_v(const AttnArgs& a, int tiles, hipStream_t s) {
    const KernelArgs k = make_kernel_args(a);
    dim3 grid(a.n_units, a.Hkv, tiles), block(NW * 64);
    hipLaunchKernelGGL((attn_mfma_kernel<G, NW, MS, PF, 0, F8>), grid, block, 0, s, k, StepArgs{},
                       reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst),
                       reinterpret_cast<const Item*>(a.table + a.off_items),
                       reinterpret_cast<const Unit*>(a.table + a.off_units));
    return hipGetLastError();
}

template <int G, int NW, int FR>
hipError_t launch_step_v(const AttnArgs& a, const MaterializeArgs& m, hipStream_t s) {
    const KernelArgs k = make_kernel_args(a);
    StepArgs f;
    f.hidden = m.hidden; f.w_k = m.w_k; f.w_v = m.w_v; f.rope = m.rope;
    f.Hd = m.Hd; f.batch = a.batch;
    dim3 grid(a.n_units, a.Hkv, 1), block(2 * NW * 64);
    auto kern = a.kv_fmt == MATKV_PAGE_E4M3 ? attn_mfma_kernel<G, NW, 1, 2, FR, true> : attn_mfma_kernel<G, NW, 1, 2, FR, false>;
    hipLaunchKernelGGL(kern, grid, block, 0, s, k, f,
                       reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst),
                       reinterpret_cast<const Item*>(a.table + a.off_items),
                       reinterpret_cast<const Unit*>(a.table + a.off_units));
    return hipGetLastError();
}

template <int G>
hipError_t launch_step_g(const AttnArgs& a, const MaterializeArgs& m, hipStream_t s) {
    if constexpr (G <= 4) return a.batch == 1 ? launch_step_v<G, 4, 1>(a, m, s) : launch_step_v<G, 4, 4>(a, m, s);
    return hipErrorInvalidValue;
}

template <int G>
hipError_t launch_g(const AttnArgs& a, hipStream_t s) {
    const bool f8 = a.kv_fmt == MATKV_PAGE_E4M3;        // compressed pages: the default shapes only
    if (a.prefill) {
        const int tiles = (a.rows * G + 31) / 32;
        return f8 ? launch_v<G, 4, 2, 2, true>(a, tiles, s) : launch_v<G, 4, 2, 2>(a, tiles, s);
    }
    if (a.shared) {
        const KernelArgs k = make_kernel_args(a);
        auto kern = f8 ? attn_mfma_kernel<G, 4, 1, 2, 0, true, true> : attn_mfma_kernel<G, 4, 1, 2, 0, false, true>;
        hipLaunchKernelGGL(kern, dim3(a.n_units, a.Hkv, 1), dim3(4 * 64), 0, s, k, StepArgs{},
                           reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst),
                           reinterpret_cast<const Item*>(a.table + a.off_items),
                           reinterpret_cast<const Unit*>(a.table + a.off_units));
        return hipGetLastError();
    }
    if (f8) return launch_v<G, 4, 1, 2, true>(a, 1, s);
    // decode: variant 9000 + 10 * (blocks in flight) + waves
    switch (a.variant % 100) {
        case 24: return launch_v<G, 4, 1, 2>(a, 1, s);
        case 34: return launch_v<G, 4, 1, 3>(a, 1, s);
        case 28: return launch_v<G, 8, 1, 2>(a, 1, s);
        case 22: return launch_v<G, 2, 1, 2>(a, 1, s);
        default: break;
    }
    // measured: four waves are ahead for every group size (config 4, G = 8: 62.7 us against
    // 65.1 us with eight)
    return launch_v<G, 4, 1, 2>(a, 1, s);
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a, int dtype) {
    const int g = a.Hq / a.Hkv;
    return dtype == MATKV_BF16 && a.D == 128 && group_size_built(g);
}

hipError_t launch_attn_mfma(const AttnArgs& a, int dtype, hipStream_t s) {
    if (a.n_units <= 0) return hipSuccess;
    if (!attn_mfma_supported(a, dtype)) return hipErrorInvalidValue;
    switch (a.Hq / a.Hkv) {
        case 1: return launch_g<1>(a, s);
        case 2: return launch_g<2>(a, s);
        case 3: return launch_g<3>(a, s);
        case 4: return launch_g<4>(a, s);
        case 8: return launch_g<8>(a, s);
    }
    return hipErrorInvalidValue;
}


// Fused decode step: K/V projection of every instance's newest token and the decode attention
// in one launch (default kernel shape only).
bool decode_step_supported(const AttnArgs& a, const MaterializeArgs& m, int dtype) {
    // Measured: the single launch wins while every projection wave has one task (up to four
    // instances) at the 8B shape; at group size 8 with hidden 8192 (config 4) it is 3 % behind
    // the two launches (it halves the attention waves per compute unit), so it stops at group
    // size 4.  Projection workgroups of their own beside the attention workgroups (for larger
    // batches) lose outright: the decode kernel wants exactly one attention workgroup per
    // compute unit - a second resident workgroup of any kind on a compute unit stretches the
    // launch by a third (batch 16: 57 us with 256 workgroups, 83 us with 264).
    return attn_mfma_supported(a, dtype) && !a.prefill && !a.shared && a.variant == 0 &&
           ((m.Hd % 4096) == 0 || (m.Hd % 3072) == 0) &&
           a.batch >= 1 && a.batch <= kFusedMaxBatch && a.Hq / a.Hkv <= 4;
}

hipError_t launch_decode_step(const AttnArgs& a, const MaterializeArgs& m, int dtype, hipStream_t s) {
    if (a.n_units <= 0 || !decode_step_supported(a, m, dtype)) return hipErrorInvalidValue;
    switch (a.Hq / a.Hkv) {
        case 1: return launch_step_g<1>(a, m, s);
        case 2: return launch_step_g<2>(a, m, s);
        case 3: return launch_step_g<3>(a, m, s);
        case 4: return launch_step_g<4>(a, m, s);
        case 8: return launch_step_g<8>(a, m, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace matkv
