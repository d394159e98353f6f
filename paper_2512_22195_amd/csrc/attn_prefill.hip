// Question prefill attention on the matrix cores, bf16, head_dim 128 (paper Section V-A "prefill
// time": row i of the question attends to every chunk key and to question keys j <= i).
//
// The M dimension is the flattened (question row, query head of one KV head) index.  A
// workgroup owns a tile of NW*16*MS such rows (NW = 4 or 8 waves) and one work unit of the cache;
// its waves split the ROWS (16*MS each) and walk the unit's tokens TOGETHER, 64 at a time: each
// K/V block is fetched from HBM once per workgroup with coalesced 16-byte loads into double-buffered LDS
// tiles and shared by all waves -
//   S^T = K Q^T     A = K rows from the LDS tile (padded rows, conflict-free 16-byte reads),
//                   B = Q held in registers
//   softmax         online, per lane on its own column; the four 16-lane groups agree on the
//                   running maximum through register swaps
//   O^T += V^T P^T  A = V through the transposing LDS read, B = P rounded to bf16
// The next block's loads are in flight (in registers) while the current one is computed out of
// LDS; eight waves share a compute unit (two four-wave workgroups, or one of eight).
// A wave owns its rows outright, so nothing is merged between waves.  An instance whose cache
// is one unit gets its output rows straight from the registers; otherwise every unit leaves an
// unnormalised partial (accumulator, running maximum, sum) per row and a second, chip-wide
// launch folds the units of each row together (the last-arrival merge of the decode kernels
// would leave that work to a handful of compute units here: the partials of a question are
// megabytes, not kilobytes).
#include "attn_common.h"

namespace matkv {
namespace {

using namespace attn;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
// Row strides of the LDS tiles, measured on the chip with the three access patterns used here
// (16-byte operand reads of 16 rows, transposing 8-byte reads, 16-byte staging writes of whole
// rows; cycles per instruction with eight waves): K 272 bytes 8.8, 288 bytes 5.4; V 288 bytes
// 6.7, 304 bytes 6.2.
constexpr int KSTR = D + 16;        // bf16 per LDS row of the K tile
constexpr int VSTR = D + 24;        // bf16 per LDS row of the V tile
constexpr float kLazyLog2 = 8.0f;     // slack of the running reference exponent, in powers of two

__device__ __forceinline__ s16x4 lds_read_tr(const uint16_t* p) {
    typedef s16x4 __attribute__((address_space(3))) * lptr;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(uintptr_t)p);
}

// TB = token rows per step (a multiple of 32).  64 against 32 halves the per-step costs that do
// not depend on the number of tokens (walking the items, addresses, barrier, reference update)
// and measured 5-12 % ahead.
// F8: the pages hold E4M3 codes with per-head power-of-two scales (the tail stays bf16).  Codes
// are widened to bf16 on their way into the LDS tiles (exact).  The K scale multiplies a block's
// maximum and its exponent factor instead of its scores; the V scale goes into the weights as
// they are rounded to bf16 (exact: a power of two) and is taken out of the row sums by summing
// with 1/scale instead of 1 - so the per-element work is the same as for plain pages.
template <int G, int MS, int TB, bool F8, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_prefill_kernel(
        KernelArgs a, const InstanceInfo* __restrict__ insts, const Item* __restrict__ items,
        const Unit* __restrict__ units) {
    constexpr int WR = 16 * MS;                         // rows per wave
    constexpr int RT = NW * WR;                         // rows per workgroup
    constexpr int NH = TB / 32;                         // 32-token halves of a step
    typedef uint16_t T;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    // a chunk's own attention: tile t walks (t + 1) * RT / G keys, so the longest go first
    const int kvh = blockIdx.y, tile = a.prefill == 2 ? gridDim.z - 1 - blockIdx.z : blockIdx.z;
    const int m0 = tile * RT;

    const Unit unit = units[blockIdx.x];
    const InstanceInfo inst = insts[unit.inst];
    const int n_m = inst.q_len * G;
    if (m0 >= n_m) return;                              // whole workgroup leaves together
    const int r_last = (min(m0 + RT, n_m) - 1) / G;
    const bool wave_live = m0 + WR * wave < n_m;        // this wave has at least one real row
    const int vis_min = (m0 + WR * wave) / G + 1;       // tail rows every row of this wave may see

    // Q in operand layout; padding rows repeat the last real row
    bf16x8 bq[MS][4];
    int vis[MS];                                        // tail rows this lane's row may see
#pragma unroll
    for (int j = 0; j < MS; ++j) {
        const int m = min(m0 + WR * wave + 16 * j + c16, n_m - 1);
        const int r = m / G, g = m % G;
        const T* qp = reinterpret_cast<const T*>(a.q) + ((size_t)(inst.cu_q + r) * a.Hq + (size_t)kvh * G + g) * D + 8 * g4;
#pragma unroll
        for (int c = 0; c < 4; ++c) bq[j][c] = __builtin_bit_cast(bf16x8, ldg16(qp + 32 * c));
        vis[j] = r + 1;
    }

    f32x4 ot[MS][8], ol[MS];          // O^T accumulators; row sums (every element of a lane the same)
    float mrow[MS];                   // reference score of the lane's row, unscaled
#pragma unroll
    for (int j = 0; j < MS; ++j) {
        mrow[j] = kNegBig;
        ol[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 8; ++s) ot[j][s] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    constexpr int TILE_ELEMS = TB * KSTR + TB * VSTR;               // one K tile + one V tile
    __shared__ __attribute__((aligned(16))) uint16_t tiles[2 * TILE_ELEMS];

    // The unit's item list sits in LDS: fetching an item from global memory inside the loop
    // would put a memory wait there that also drains the block loads in flight.
    __shared__ __attribute__((aligned(16))) Item sm_items[kMaxPrefillItemsPerUnit];
    __shared__ float sm_scale[F8 ? kMaxPrefillItemsPerUnit : 1][2];    // K and V scale of every item
    for (int i = tid; i < unit.n_items * 2; i += NW * 64)
        reinterpret_cast<uint4*>(sm_items)[i] = reinterpret_cast<const uint4*>(items + unit.item0)[i];
    if (F8 && tid < unit.n_items) {
        const Item it = items[unit.item0 + tid];
        float sk = 1.f, sv = 1.f;
        if (it.base) page_scales(it, a.layer, a.Hkv, kvh, sk, sv);
        sm_scale[tid][0] = sk; sm_scale[tid][1] = sv;
    }
    __syncthreads();

    // Every wave walks the same blocks: the unit's items end to end (the tail clipped to the
    // rows this tile may see), TB token rows at a time, never across two items.
    struct {
        Item item;
        int item_i, rows, left;         // current item, its visible rows, rows of it not yet handed out
    } wk;
    const int tail_visible = r_last + 1;
    auto rows_of = [&](const Item& it) { return it.base ? it.ntok : min(min(it.ntok, tail_visible), a.max_tail); };
    wk.item = unit.first; wk.item_i = 0; wk.rows = rows_of(wk.item); wk.left = wk.rows;
    // Past the unit's end the previous block comes back marked invalid: still safe to load,
    // so that the loop below can issue its loads unconditionally.
    BlockRef<T> last_block;
    last_block.valid = false; last_block.is_tail = false; last_block.k = nullptr; last_block.v = nullptr;
    last_block.t0 = 0; last_block.tok_end = 0; last_block.sk = 1.f; last_block.sv = 1.f;
    auto next_block = [&]() {
        BlockRef<T> r = last_block;
        r.valid = false;
        while (wk.left <= 0) {
            if (++wk.item_i >= unit.n_items) return r;
            wk.item = sm_items[wk.item_i];
            wk.rows = rows_of(wk.item);
            wk.left = wk.rows;
        }
        r.sk = 1.f; r.sv = 1.f;
        if (wk.item.base) {
            const size_t head_elems = (size_t)wk.item.page_tokens * D;
            if (F8) {
                const uint8_t* codes = reinterpret_cast<const uint8_t*>(wk.item.base);
                r.k = reinterpret_cast<const T*>(codes + ((size_t)(a.layer * 2 + 0) * a.Hkv + kvh) * head_elems);
                r.v = reinterpret_cast<const T*>(codes + ((size_t)(a.layer * 2 + 1) * a.Hkv + kvh) * head_elems);
                r.sk = sm_scale[wk.item_i][0]; r.sv = sm_scale[wk.item_i][1];
            } else {
                const T* blob = reinterpret_cast<const T*>(wk.item.base);
                r.k = blob + ((size_t)(a.layer * 2 + 0) * a.Hkv + kvh) * head_elems;
                r.v = blob + ((size_t)(a.layer * 2 + 1) * a.Hkv + kvh) * head_elems;
            }
        } else {
            const size_t off = ((size_t)unit.inst * a.Hkv + kvh) * (size_t)a.max_tail * D;
            r.k = reinterpret_cast<const T*>(a.tail_k) + off;
            r.v = reinterpret_cast<const T*>(a.tail_v) + off;
            r.is_tail = true;
        }
        if (wk.item.base) r.is_tail = false;
        const int n = min(TB, wk.left);
        r.t0 = wk.item.tok0 + (wk.rows - wk.left);
        r.tok_end = r.t0 + n;
        r.valid = true;
        wk.left -= n;
        last_block = r;
        return r;
    };

    // cooperative staging: thread t moves rows t/16 + RPP*i, columns 8*(t%16), of K and of V
    constexpr int RPP = NW * 4;                         // rows the workgroup moves per pass
    const int st_row = tid >> 4, st_col = (tid & 15) * 8;
    constexpr int SR = TB / RPP;
    struct Stage { uint4 k[SR], v[SR]; };
    auto load_global = [&](const BlockRef<T>& r, Stage& g) {
        if (F8 && !r.is_tail) {      // the same number of loads, half as wide (see the loop below)
#pragma unroll
            for (int i = 0; i < SR; ++i) {
                const size_t off = (size_t)min(r.t0 + st_row + RPP * i, r.tok_end - 1) * D + st_col;
                const uint2 kw = ldg8(reinterpret_cast<const uint8_t*>(r.k) + off);
                const uint2 vw = ldg8(reinterpret_cast<const uint8_t*>(r.v) + off);
                g.k[i] = make_uint4(kw.x, kw.y, 0u, 0u);
                g.v[i] = make_uint4(vw.x, vw.y, 0u, 0u);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < SR; ++i) {
            const size_t off = (size_t)min(r.t0 + st_row + RPP * i, r.tok_end - 1) * D + st_col;
            g.k[i] = ldg16(r.k + off);
            g.v[i] = ldg16(r.v + off);
        }
    };
    auto store_lds = [&](int buf, const Stage& g, bool codes) {
        uint16_t* kt = tiles + buf * TILE_ELEMS;
        uint16_t* vt = kt + TB * KSTR;
#pragma unroll
        for (int i = 0; i < SR; ++i) {
            uint4 kw = g.k[i], vw = g.v[i];
            if (F8 && codes) {
                kw = e4m3x8_to_bf16x8(make_uint2(kw.x, kw.y));
                vw = e4m3x8_to_bf16x8(make_uint2(vw.x, vw.y));
            }
            *reinterpret_cast<uint4*>(kt + (st_row + RPP * i) * KSTR + st_col) = kw;
            *reinterpret_cast<uint4*>(vt + (st_row + RPP * i) * VSTR + st_col) = vw;
        }
    };

    // Scores stay unscaled until the exponent: 2^((s - m) c) is one multiply-add and one
    // exponential per element, with m the row's reference score (unscaled too).  The row sums
    // come from the matrix cores as well - P times a block of ones - which sums the weights
    // exactly as the output uses them (rounded to bf16) and spares the vector ALU the adds.
    const float sc = a.scale_log2e;
    const float lazy_raw = kLazyLog2 / sc;
    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;

    // masked: the block is ragged, or lies in the tail and reaches past what the wave's first
    // row may see (per-row causal limit); otherwise all TB rows are visible to every question
    // row of the wave and no element needs a test.
    auto compute = [&](const BlockRef<T>& r, int buf) {
        const bool masked = r.tok_end - r.t0 != TB || (r.is_tail && r.tok_end > vis_min);
        const uint16_t* kt = tiles + buf * TILE_ELEMS;
        const uint16_t* vt = kt + TB * KSTR;
        // compressed page: scores carry the factor 1 / sk until the exponent, weights the factor
        // sv from the exponent on (nsv = log2 sv goes into the exponent's offset)
        const float scb = F8 ? sc * r.sk : sc;
        const float nsv = F8 ? __builtin_amdgcn_frexp_expf(r.sv) - 1.0f : 0.f;
        bf16x8 ones_b = ones;
        if (F8) {
            const __bf16 iv = (__bf16)(1.0f / r.sv);
#pragma unroll
            for (int i = 0; i < 8; ++i) ones_b[i] = iv;
        }
        // S^T in 16-token quarters q: lane holds tokens t0 + 16q + 4*g4 + i of its row
        f32x4 st[MS][2 * NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            bf16x8 ak[2][4];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    ak[hh][c] = *reinterpret_cast<const bf16x8*>(kt + (32 * h + 16 * hh + c16) * KSTR + 32 * c + 8 * g4);
#pragma unroll
            for (int j = 0; j < MS; ++j) {
                st[j][2 * h] = f32x4{0.f, 0.f, 0.f, 0.f};
                st[j][2 * h + 1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            // dim chunk outermost: 2 * MS independent accumulation chains are interleaved, so no
            // matrix instruction waits for the result of the one just before it
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int j = 0; j < MS; ++j) {
                    st[j][2 * h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[0][c], bq[j][c], st[j][2 * h], 0, 0, 0);
                    st[j][2 * h + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[1][c], bq[j][c], st[j][2 * h + 1], 0, 0, 0);
                }
        }
        bf16x8 pb[MS][NH];
#pragma unroll
        for (int j = 0; j < MS; ++j) {
            float sv[8 * NH];
#pragma unroll
            for (int q = 0; q < 2 * NH; ++q)
#pragma unroll
                for (int i = 0; i < 4; ++i) sv[4 * q + i] = st[j][q][i];
            if (masked) {           // wave-uniform
                const int limit = r.is_tail ? min(r.tok_end, vis[j]) : r.tok_end;
                const int tb = r.t0 + 4 * g4;
#pragma unroll
                for (int q = 0; q < 2 * NH; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) sv[4 * q + i] = tb + 16 * q + i < limit ? sv[4 * q + i] : kNegBig;
            }
            float mx = sv[0];
#pragma unroll
            for (int i = 1; i < 8 * NH; ++i) mx = fmaxf(mx, sv[i]);
            mx = fmaxf(mx, lane_xor(mx, 16, lane));
            mx = fmaxf(mx, lane_xor(mx, 32, lane));
            if (F8) mx = mx > 0.5f * kNegBig ? mx * r.sk : kNegBig;     // into the units of the reference
            // The reference score of a row moves only when the block's maximum exceeds it by
            // more than kLazyLog2 powers of two: weights stay below 2^kLazyLog2, and the
            // accumulators are rescaled on few blocks instead of on most.
            const float mn = mx > mrow[j] + lazy_raw ? mx : mrow[j];
            const float alpha = fast_exp2((mrow[j] - mn) * sc);
            mrow[j] = mn;
            // a row that has seen no key yet keeps the floor as its reference; its masked
            // scores must still come out as weight 0, not 2^0
            const float nmc = mn > 0.5f * kNegBig ? -mn * sc : 0.f;
#pragma unroll
            for (int h = 0; h < NH; ++h)
#pragma unroll
                for (int i = 0; i < 8; ++i) pb[j][h][i] = (__bf16)fast_exp2(fmaf(sv[8 * h + i], scb, nmc + nsv));
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {   // wave-uniform: some row's reference moved
                ol[j][0] *= alpha;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    ot[j][s][0] *= alpha; ot[j][s][1] *= alpha; ot[j][s][2] *= alpha; ot[j][s][3] *= alpha;
                }
            }
#pragma unroll
            for (int h = 0; h < NH; ++h) ol[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones_b, pb[j][h], ol[j], 0, 0, 0);
        }
        // lane (c16, g4) names 4 dims (4*(c16%4) ..) of token 4*g4 + c16/4 (+16 for the second
        // quarter) of a half and receives dim 16s + c16 of tokens 4*g4 .. 4*g4+3: the k order of P
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const uint16_t* vp = vt + (32 * h + 4 * g4 + (c16 >> 2)) * VSTR + 4 * (c16 & 3);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const s16x4 lo = lds_read_tr(vp + 16 * s);
                const s16x4 hi = lds_read_tr(vp + 16 * VSTR + 16 * s);
                const bf16x8 av = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int j = 0; j < MS; ++j)
                    ot[j][s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[j][h], ot[j][s], 0, 0, 0);
            }
        }
    };

    // Loads and LDS stores are unconditional (a block past the end repeats the last one) and the
    // loops have one exit at the bottom: a load under a branch, or a break half way, would leave
    // the compiler no exact count of the loads in flight, and it would then wait for all of them.
    // Every load before the loop (Q above all) is waited for once, ahead of it: otherwise each
    // first use of Q inside the loop is guarded with a wait that, loads completing in order, would
    // also drain the block just requested.
    BlockRef<T> r0 = next_block();
    if (r0.valid) {
        // one register stage: the next block's loads are in flight while this one is computed,
        // then move into the other LDS tile
        Stage g;
        load_global(r0, g);
        store_lds(0, g, !r0.is_tail);
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0) only
        lds_barrier();
        int buf = 0;
        do {
            const BlockRef<T> r1 = next_block();
            load_global(r1, g);
            if (wave_live) compute(r0, buf);
            store_lds(buf ^ 1, g, !r1.is_tail);
            lds_barrier();
            r0 = r1;
            buf ^= 1;
        } while (r0.valid);
    }
    if (!wave_live) return;

    // ---- a wave owns its rows: results leave straight from the registers ----
    // lane (c16, g4) holds, for row 16j + c16 of the wave, dims 16s + 4*g4 + {0..3}
    const bool single = unit.n_units_inst == 1;
#pragma unroll
    for (int j = 0; j < MS; ++j) {
        const int m = m0 + WR * wave + 16 * j + c16;
        if (m >= n_m) continue;
        const int r = m / G, head = kvh * G + m % G;
        if (single) {
            const float inv = 1.0f / ol[j][0];
            const size_t oidx = ((size_t)(inst.cu_q + r) * a.Hq + head) * D + 4 * g4;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                store_out2(a.out, a.out_f32, oidx + 16 * s, ot[j][s][0] * inv, ot[j][s][1] * inv);
                store_out2(a.out, a.out_f32, oidx + 16 * s + 2, ot[j][s][2] * inv, ot[j][s][3] * inv);
            }
        } else {
            float* prow = a.partials + (((size_t)blockIdx.x * a.rows + r) * a.Hq + head) * kPartialStride(D);
#pragma unroll
            for (int s = 0; s < 8; ++s)
                *reinterpret_cast<float4*>(prow + 16 * s + 4 * g4) = make_float4(ot[j][s][0], ot[j][s][1], ot[j][s][2], ot[j][s][3]);
            if (g4 == 0) *reinterpret_cast<float2*>(prow + D) = make_float2(mrow[j] * sc, ol[j][0]);
        }
    }
}

// Folds the units' partials of every (question row, query head) of instances cut into several
// units: out = sum_u 2^(m_u - M) acc_u / sum_u 2^(m_u - M) l_u,  M = max_u m_u.
// Half a wave owns one row: lane k first fetches (m, l) of unit k, the half wave agrees on M
// and on every unit's weight, then each lane accumulates its 4 dims over the units.
// NU: units requested per round (the smallest of 2, 4, 8, 16 that covers the launch's largest
// instance: rounds beyond an instance's units would only re-read its last partial).
template <int NU>
__global__ __launch_bounds__(256) void prefill_merge_kernel(
        KernelArgs a, const InstanceInfo* __restrict__ insts, int batch, int total_pairs) {
    constexpr int PS = kPartialStride(D);
    const int lane = threadIdx.x & 63, hl = lane & 31;
    const int pair = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 2 + (lane >> 5);
    const bool in_range = pair < total_pairs;
    const int q_row = in_range ? pair / a.Hq : 0, head = in_range ? pair % a.Hq : 0;
    int b = 0;
    for (int i = 1; i < batch; ++i) if (q_row >= insts[i].cu_q) b = i;
    const InstanceInfo inst = insts[b];
    const int n_units = (in_range && inst.n_punits > 1) ? inst.n_punits : 0;     // 0: nothing to do
    const float* base = a.partials + (((size_t)inst.punit0 * a.rows + (q_row - inst.cu_q)) * a.Hq + head) * PS;
    const size_t ustride = (size_t)a.rows * a.Hq * PS;

    // the first NU units' accumulators are requested together with the (m, l) pairs, before
    // anything is consumed: one memory round trip for up to NU units, two for up to 2 NU
    auto load16 = [&](int u0, float4 (&v)[NU]) {
#pragma unroll
        for (int k = 0; k < NU; ++k) {
            const int u = min(u0 + k, max(n_units, 1) - 1);
            v[k] = *reinterpret_cast<const float4*>(base + (size_t)u * ustride + 4 * hl);
        }
    };
    float2 ml = make_float2(kNegBig, 0.f);
    if (hl < n_units) ml = *reinterpret_cast<const float2*>(base + (size_t)hl * ustride + D);
    float4 v[NU];
    load16(0, v);
    float M = ml.x;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float w = hl < n_units ? fast_exp2(ml.x - M) : 0.f;
    float L = w * ml.y;
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) L += __shfl_xor(L, off);

    // both halves of the wave run the same number of steps (shuffles need every lane)
    const int steps = max(n_units, __shfl_xor(n_units, 32));
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int u0 = 0; u0 < steps; u0 += NU) {
        if (u0 > 0) load16(u0, v);
#pragma unroll
        for (int k = 0; k < NU; ++k) {
            const float c = __shfl(w, (lane & 32) + ((u0 + k) & 31));
            const float cc = (u0 + k < n_units) ? c : 0.f;
            acc.x = fmaf(v[k].x, cc, acc.x); acc.y = fmaf(v[k].y, cc, acc.y);
            acc.z = fmaf(v[k].z, cc, acc.z); acc.w = fmaf(v[k].w, cc, acc.w);
        }
    }
    if (n_units == 0) return;
    const float inv = 1.0f / L;
    const size_t oidx = ((size_t)q_row * a.Hq + head) * D + 4 * hl;
    store_out2(a.out, a.out_f32, oidx, acc.x * inv, acc.y * inv);
    store_out2(a.out, a.out_f32, oidx + 2, acc.z * inv, acc.w * inv);
}

template <int G, int MS, int TB, bool F8, int NW = 4>
hipError_t launch_v(const AttnArgs& a, hipStream_t s) {
    const KernelArgs k = make_kernel_args(a);
    const int tiles = (a.rows * G + NW * 16 * MS - 1) / (NW * 16 * MS);
    dim3 grid(a.n_units, a.Hkv, tiles), block(NW * 64);
    hipLaunchKernelGGL((attn_prefill_kernel<G, MS, TB, F8, NW>), grid, block, 0, s, k,
                       reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst),
                       reinterpret_cast<const Item*>(a.table + a.off_items),
                       reinterpret_cast<const Unit*>(a.table + a.off_units));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.max_units_inst <= 1) return e;
    const int total_pairs = a.total_q * a.Hq;
    const dim3 mgrid((total_pairs + 7) / 8), mblock(256);
    const InstanceInfo* insts = reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst);
    if (a.max_units_inst <= 2)      hipLaunchKernelGGL(prefill_merge_kernel<2>, mgrid, mblock, 0, s, k, insts, a.batch, total_pairs);
    else if (a.max_units_inst <= 4) hipLaunchKernelGGL(prefill_merge_kernel<4>, mgrid, mblock, 0, s, k, insts, a.batch, total_pairs);
    else if (a.max_units_inst <= 8) hipLaunchKernelGGL(prefill_merge_kernel<8>, mgrid, mblock, 0, s, k, insts, a.batch, total_pairs);
    else                            hipLaunchKernelGGL(prefill_merge_kernel<16>, mgrid, mblock, 0, s, k, insts, a.batch, total_pairs);
    return hipGetLastError();
}

template <int G>
hipError_t launch_g(const AttnArgs& a, hipStream_t s) {
    const long rg = (long)a.rows * G;                   // (row, head) rows of the longest question
    if (a.prefill == 2) {
        // A chunk's own attention has one workgroup per (row tile, KV head) and the last tile walks
        // the whole chunk: until 128-row tiles give every compute unit two workgroups, 64-row
        // tiles do (1024 tokens, 8 KV heads: 31 us against 36 us; 4096 tokens: 269 against 210).
        // (from 512 eight-wave workgroups on, 256-row tiles are a little ahead: 4096 tokens 188 against 196 us)
        if (((rg + 255) / 256) * a.Hkv >= 512) return launch_v<G, 2, 64, false, 8>(a, s);
        if (rg <= 64 || ((rg + 127) / 128) * a.Hkv < 512) return launch_v<G, 1, 64, false>(a, s);
        return launch_v<G, 2, 64, false>(a, s);
    }
    // Up to 64 rows: one 16-row block per wave.  Up to 128: two.  Beyond: eight waves share the
    // K/V tiles of a 256-row workgroup, which halves the reads of the cache per question row
    // (config 3: 202 -> 187 us per layer, config 4: 418 -> 376 us; config 2, exactly 256 rows:
    // 33.2 -> 32.3 us).
    if (a.kv_fmt == MATKV_PAGE_E4M3) {
        if (rg <= 64) return launch_v<G, 1, 64, true>(a, s);
        if (rg <= 128) return launch_v<G, 2, 64, true>(a, s);
        return launch_v<G, 2, 64, true, 8>(a, s);
    }
    if (rg <= 64) return launch_v<G, 1, 64, false>(a, s);
    if (rg <= 128) return launch_v<G, 2, 64, false>(a, s);
    return launch_v<G, 2, 64, false, 8>(a, s);
}

}  // namespace

bool attn_prefill_supported(const AttnArgs& a, int dtype) {
    const int g = a.Hq / a.Hkv;
    return a.prefill && dtype == MATKV_BF16 && a.D == 128 && group_size_built(g) &&
           a.max_unit_items <= kMaxPrefillItemsPerUnit;
}

hipError_t launch_attn_prefill(const AttnArgs& a, int dtype, hipStream_t s) {
    if (a.n_units <= 0) return hipSuccess;
    if (!attn_prefill_supported(a, dtype)) return hipErrorInvalidValue;
    switch (a.Hq / a.Hkv) {
        case 1: return launch_g<1>(a, s);
        case 2: return launch_g<2>(a, s);
        case 3: return launch_g<3>(a, s);
        case 4: return launch_g<4>(a, s);
        case 8: return launch_g<8>(a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace matkv
