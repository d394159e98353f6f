// Pieces shared by the two attention kernels (plain-ALU rows and matrix-core tiles): the walk
// over a work unit's token rows, and the merge of partial results across waves and across the
// units of one (instance, KV head).
#pragma once

#include "device_util.h"

namespace matkv {
namespace attn {

constexpr float kNegBig = -1.0e30f;   // "no key seen yet": finite, so that exp2(m - m) = 1
constexpr int kPartialStride(int D) { return D + 4; }   // floats: accumulator, max, sum, pad

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

using dev::f32_to_bf16_rne;
using dev::ldg16;
using dev::ldg8;
using dev::st_agent2;
using dev::ld_agent2;

// exp2 of a non-positive argument: the bare hardware instruction (results below the normal
// range flush to zero, which is what a softmax weight that small should be).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Eight E4M3 codes to eight bf16 (exact: three mantissa bits fit seven), through fp32.
__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint2 w) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, true);
    const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, true);
    return make_uint4(__builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2)),
                      __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2)),
                      __builtin_bit_cast(uint32_t, __builtin_convertvector(c, bf16x2)),
                      __builtin_bit_cast(uint32_t, __builtin_convertvector(d, bf16x2)));
}

// Value of the lane whose index differs in bit log2(off); off in {32, 16, 8}.  Distances 32
// and 16 are register swaps on this chip; 8 goes through the LDS crossbar.
__device__ __forceinline__ float lane_xor(float v, int off, int lane) {
    const unsigned x = __float_as_uint(v);
    if (off == 32) {
        const u32x2 r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return __uint_as_float((lane & 32) ? r.x : r.y);
    }
    if (off == 16) {
        const u32x2 r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return __uint_as_float((lane & 16) ? r.x : r.y);
    }
    return __shfl_xor(v, off);
}

// One pair of output elements of a bf16 launch: rounded to bf16, or as they are when the
// configuration asks for float outputs.
__device__ __forceinline__ void store_out2(void* out, bool f32, size_t idx, float x, float y);

struct KernelArgs {
    const void* __restrict__ q;
    void* __restrict__ out;
    const void* tail_k;          // a fused decode step also writes the newest row of each instance
    const void* tail_v;
    float* __restrict__ partials;
    int32_t* __restrict__ counters;
    int32_t layer, Hq, Hkv, max_tail, rows, prefill;
    int32_t cstride;             // ints between two arrival counters
    int32_t out_f32;             // bf16 path: outputs leave as float, unrounded
    float scale_log2e;
};

__device__ __forceinline__ void store_out2(void* out, bool f32, size_t idx, float x, float y) {
    if (f32) *reinterpret_cast<float2*>(reinterpret_cast<float*>(out) + idx) = make_float2(x, y);
    else *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(out) + idx) = (uint32_t)f32_to_bf16_rne(x) | ((uint32_t)f32_to_bf16_rne(y) << 16);
}

// Arrival counter of (instance, KV head, row z).  Decode launches keep every counter on a
// 128-byte line of its own: agent-scope atomics on one line are served one after the other, and
// a launch's workgroups arrive within a microsecond or two of each other.
__device__ __forceinline__ int counter_index(const KernelArgs& a, int inst, int kvh, int z) {
    return ((inst * a.Hkv + kvh) * a.rows + z) * a.cstride;
}

inline KernelArgs make_kernel_args(const AttnArgs& a) {
    KernelArgs k;
    k.q = a.q; k.out = a.out; k.tail_k = a.tail_k; k.tail_v = a.tail_v;
    k.partials = a.partials; k.counters = a.counters;
    k.layer = a.layer; k.Hq = a.Hq; k.Hkv = a.Hkv; k.max_tail = a.max_tail; k.rows = a.rows;
    k.prefill = a.prefill; k.scale_log2e = a.scale_log2e;
    k.cstride = a.prefill ? 1 : kDecodeCounterStride;
    k.out_f32 = a.out_f32;
    return k;
}

// Where a wave's next block of token rows lives.
template <typename T>
struct BlockRef {
    const T* k;      // row 0 of the item's K stream for this head
    const T* v;
    int t0;          // first token row of the block (index inside the page, or inside the tail)
    int tok_end;     // one past the block's last valid row
    bool is_tail;
    bool valid;
    float sk, sv;    // compressed page: scale of this head's K and V codes (else unused)
    int umask;       // shared decode units: which of the unit's users see this block
};

// Scales of KV head kvh of a compressed page at `layer`: the blob's scale table is
// [layer][K|V][Hkv] floats, scales16 * 16 bytes behind its base.
__device__ __forceinline__ void page_scales(const Item& it, int layer, int Hkv, int kvh, float& sk, float& sv) {
    // read through the constant address space: with a wave-uniform address these are scalar
    // loads, which do not touch the counter of the vector loads in flight
    typedef const __attribute__((address_space(4))) float* cptr;
    const cptr t = (cptr)(uintptr_t)(it.base + (uint64_t)it.scales16 * 16) + ((size_t)layer * 2 * Hkv + kvh);
    sk = t[0];
    sv = t[Hkv];
}

// The unit's items, end to end, form one run of token rows (the tail clipped to tail_visible).
// Each wave takes an equal contiguous share of the run, rounded up to ALIGN rows, and walks it
// in blocks of at most BLK rows that never straddle two items.  All state is wave-uniform.
// F8: the pages are compressed (one E4M3 byte per element): k / v of a page block then point at
// the head's codes (row stride D bytes) and sk / sv carry the head's scales; the tail stays in T.
template <typename T, int D, int NW, int BLK, int ALIGN, bool F8 = false>
struct Walker {
    const KernelArgs& a;
    const Unit& unit;
    const Item* __restrict__ items;
    int kvh, tail_visible;
    Item item;
    int item_i, item_pos0, pos, pos_end;
    float sk, sv;                // scales of the current item (compressed pages)

    __device__ __forceinline__ Walker(const KernelArgs& a_, const Unit& u_, const Item* items_, int kvh_,
                                      int tail_visible_, int wave)
        : a(a_), unit(u_), items(items_), kvh(kvh_), tail_visible(tail_visible_), item(u_.first),
          item_i(0), item_pos0(0), sk(1.f), sv(1.f) {
        if (F8 && item.base) page_scales(item, a.layer, a.Hkv, kvh, sk, sv);
        int total = unit.page_tokens;
        if (unit.has_tail) total += min(a.max_tail, tail_visible);
        const int share = ((total + NW - 1) / NW + ALIGN - 1) / ALIGN * ALIGN;
        pos = wave * share;
        pos_end = min(total, pos + share);
    }
    __device__ __forceinline__ int rows_of(const Item& it) const {
        return it.base ? it.ntok : min(it.ntok, tail_visible);
    }
    // row 0 of this KV head's K and V inside a page's blob
    __device__ __forceinline__ void page_heads(const Item& it, BlockRef<T>& r) const {
        const size_t head_elems = (size_t)it.page_tokens * D;
        if (F8) {
            const uint8_t* codes = reinterpret_cast<const uint8_t*>(it.base);
            r.k = reinterpret_cast<const T*>(codes + ((size_t)(a.layer * 2 + 0) * a.Hkv + kvh) * head_elems);
            r.v = reinterpret_cast<const T*>(codes + ((size_t)(a.layer * 2 + 1) * a.Hkv + kvh) * head_elems);
        } else {
            const T* blob = reinterpret_cast<const T*>(it.base);
            r.k = blob + ((size_t)(a.layer * 2 + 0) * a.Hkv + kvh) * head_elems;
            r.v = blob + ((size_t)(a.layer * 2 + 1) * a.Hkv + kvh) * head_elems;
        }
    }
    __device__ __forceinline__ BlockRef<T> next() {
        BlockRef<T> r;
        r.valid = false; r.is_tail = false; r.k = nullptr; r.v = nullptr; r.t0 = 0; r.tok_end = 0; r.umask = 0;
        if (pos >= pos_end) return r;
        int rows = rows_of(item);
        while (pos >= item_pos0 + rows) {
            item_pos0 += rows;
            if (++item_i >= unit.n_items) return r;
            item = items[unit.item0 + item_i];
            rows = rows_of(item);
            if (F8) {
                sk = 1.f; sv = 1.f;
                if (item.base) page_scales(item, a.layer, a.Hkv, kvh, sk, sv);
            }
        }
        r.sk = sk; r.sv = sv;
        r.umask = item.umask;
        if (item.base) {
            page_heads(item, r);
        } else {
            const size_t off = ((size_t)unit.inst * a.Hkv + kvh) * (size_t)a.max_tail * D;
            r.k = reinterpret_cast<const T*>(a.tail_k) + off;
            r.v = reinterpret_cast<const T*>(a.tail_v) + off;
            r.is_tail = true;
        }
        const int in_item = pos - item_pos0;
        const int n = min(BLK, min(rows - in_item, pos_end - pos));
        r.t0 = item.tok0 + in_item;
        r.tok_end = r.t0 + n;
        r.valid = true;
        pos += n;
        return r;
    }
    // next(), except that past the end it hands out a one-row block (the first row of the
    // unit's first item) marked invalid: a loop can then issue its loads without a branch, and
    // the loads of such a block all fall on one row.
    __device__ __forceinline__ BlockRef<T> next_safe() {
        BlockRef<T> r = next();
        if (r.valid) return r;
        const Item& f = unit.first;
        r.sk = 1.f; r.sv = 1.f;
        if (f.base) {
            page_heads(f, r);
        } else {
            const size_t off = ((size_t)unit.inst * a.Hkv + kvh) * (size_t)a.max_tail * D;
            r.k = reinterpret_cast<const T*>(a.tail_k) + off;
            r.v = reinterpret_cast<const T*>(a.tail_v) + off;
        }
        r.is_tail = f.base == 0;
        r.t0 = f.tok0;
        r.tok_end = f.tok0 + 1;
        return r;
    }
};

// What a local result row of a workgroup stands for.
struct RowMap {
    int slot_row;    // row index inside the partial buffer (question row; 0 for decode)
    int head;        // query head
    int q_row;       // row of the packed Q / O tensors
    int unit_slot = -1;   // partial slot of the row's unit; -1 = the workgroup's own (blockIdx.x)
};

// Last-arrival merge of all units' partials into the output rows (see finish_unit).
// unit0 = the instance's first unit.
template <typename T, int D, int NT, int CB, typename MapFn>
__device__ __forceinline__ void merge_units(const KernelArgs& a, int unit0, int cols_valid, int n_units, MapFn map) {
    constexpr int PSTRIDE = kPartialStride(D);
    constexpr int UPC = 32 / CB;                               // units per column and pass
    const int tid = threadIdx.x;
    const size_t ustride = (size_t)a.rows * a.Hq * PSTRIDE;
    for (int c0 = tid; c0 < cols_valid; c0 += NT * CB) {
        float M[CB], Lsum[CB], ox[CB], oy[CB];
        const float* src[CB];
        int dd[CB];
        RowMap rms[CB];
        bool live[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int col = c0 + cb * NT;
            live[cb] = col < cols_valid;
            const int cc = live[cb] ? col : c0;
            const int i = cc / (D / 2);
            dd[cb] = (cc % (D / 2)) * 2;
            rms[cb] = map(i);
            src[cb] = a.partials + (((size_t)unit0 * a.rows + rms[cb].slot_row) * a.Hq + rms[cb].head) * PSTRIDE;
            M[cb] = kNegBig; Lsum[cb] = 0.f; ox[cb] = 0.f; oy[cb] = 0.f;
        }
        for (int u0 = 0; u0 < n_units; u0 += UPC) {
            float2 av[CB][UPC], ml[CB][UPC];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int k = 0; k < UPC; ++k) {
                    const size_t uo = (size_t)min(u0 + k, n_units - 1) * ustride;
                    ml[cb][k] = ld_agent2(src[cb] + uo + D);
                    av[cb][k] = ld_agent2(src[cb] + uo + dd[cb]);
                }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                float mn = M[cb];
#pragma unroll
                for (int k = 0; k < UPC; ++k) mn = fmaxf(mn, (u0 + k < n_units) ? ml[cb][k].x : kNegBig);
                const float cold = fast_exp2(M[cb] - mn);
                Lsum[cb] *= cold; ox[cb] *= cold; oy[cb] *= cold;
                M[cb] = mn;
#pragma unroll
                for (int k = 0; k < UPC; ++k) {
                    const float c = (u0 + k < n_units) ? fast_exp2(ml[cb][k].x - mn) : 0.f;
                    Lsum[cb] = fmaf(ml[cb][k].y, c, Lsum[cb]);
                    ox[cb] = fmaf(av[cb][k].x, c, ox[cb]);
                    oy[cb] = fmaf(av[cb][k].y, c, oy[cb]);
                }
            }
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            if (!live[cb]) continue;
            const float inv = 1.0f / Lsum[cb];
            const size_t oidx = ((size_t)rms[cb].q_row * a.Hq + rms[cb].head) * D + dd[cb];
            T* op = reinterpret_cast<T*>(a.out) + oidx;
            if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<float2*>(op) = make_float2(ox[cb] * inv, oy[cb] * inv);
            } else if (a.out_f32) {
                *reinterpret_cast<float2*>(reinterpret_cast<float*>(a.out) + oidx) = make_float2(ox[cb] * inv, oy[cb] * inv);
            } else {
                *reinterpret_cast<uint32_t*>(op) =
                    (uint32_t)f32_to_bf16_rne(ox[cb] * inv) | ((uint32_t)f32_to_bf16_rne(oy[cb] * inv) << 16);
            }
        }
    }
}

// A thread owns pairs of output elements (columns).  Per pass it takes CB of its columns and
// up to 32 / CB units and issues all those loads - the pairs and the (max, sum) of their rows -
// at once: one memory round trip per pass.  Few units means many columns per pass.
template <typename T, int D, int NT, typename MapFn>
__device__ __forceinline__ void merge_dispatch(const KernelArgs& a, int unit0, int n_units, int cols_valid, MapFn map) {
    if (n_units <= 4)       merge_units<T, D, NT, 8>(a, unit0, cols_valid, n_units, map);
    else if (n_units <= 8)  merge_units<T, D, NT, 4>(a, unit0, cols_valid, n_units, map);
    else if (n_units <= 16) merge_units<T, D, NT, 2>(a, unit0, cols_valid, n_units, map);
    else                    merge_units<T, D, NT, 1>(a, unit0, cols_valid, n_units, map);
}

// One workgroup's arrival at the counter of (instance, KV head, z index): every thread has
// waited for its own agent-scope stores, the barrier orders them before thread 0's ticket.
// Returns true in every thread of the workgroup that arrived last of `expected`.
__device__ __forceinline__ bool arrive(const KernelArgs& a, int cidx, int expected, int* sm_last) {
    return dev::arrive_at(&a.counters[cidx], expected, sm_last);
}
__device__ __forceinline__ void reset_counter(const KernelArgs& a, int cidx) { dev::reset_counter_at(&a.counters[cidx]); }

// Merge of one workgroup's NS partial states per row (already in LDS: accumulators
// sm_acc[w][row][..] with row stride ACC_STRIDE floats, running maxima sm_m[w][row], sums
// sm_l[w][row]; NS = the waves when they split the tokens, 1 when they split the rows) into the
// unit's partial, written with agent-scope stores (coherent across the chip's L2 slices; no
// L2 write-back or invalidate is involved), followed by the workgroup's arrival.  Returns true
// in the workgroup that arrived last of `expected`: it then folds all partials (merge_dispatch)
// and resets the counter.
template <typename T, int D, int NT, int NS, int ROWS, int ACC_STRIDE, typename MapFn>
__device__ __forceinline__ void publish_partial(const KernelArgs& a, const float* sm_acc, const float* sm_m,
                                                const float* sm_l, int n_valid_rows, MapFn map) {
    constexpr int PSTRIDE = kPartialStride(D);
    const int tid = threadIdx.x;
    __syncthreads();

    const int cols_valid = n_valid_rows * (D / 2);            // valid rows are a prefix of the local rows
    for (int col = tid; col < cols_valid; col += NT) {
        const int i = col / (D / 2), d = (col % (D / 2)) * 2;
        const RowMap rm = map(i);
        float mn = sm_m[i];
#pragma unroll
        for (int w = 1; w < NS; ++w) mn = fmaxf(mn, sm_m[w * ROWS + i]);
        float ax = 0.f, ay = 0.f, lv = 0.f;
#pragma unroll
        for (int w = 0; w < NS; ++w) {
            const float c = fast_exp2(sm_m[w * ROWS + i] - mn);
            const float* src = sm_acc + ((size_t)w * ROWS + i) * ACC_STRIDE + d;
            ax = fmaf(src[0], c, ax);
            ay = fmaf(src[1], c, ay);
            lv = fmaf(sm_l[w * ROWS + i], c, lv);
        }
        const size_t uslot = rm.unit_slot >= 0 ? (size_t)rm.unit_slot : (size_t)blockIdx.x;
        float* prow = a.partials + ((uslot * a.rows + rm.slot_row) * a.Hq + rm.head) * PSTRIDE;
        st_agent2(prow + d, ax, ay);
        if (d == 0) st_agent2(prow + D, mn, lv);
    }
}

template <typename T, int D, int NW, int NS, int ROWS, int ACC_STRIDE, typename MapFn>
__device__ __forceinline__ bool publish_unit(const KernelArgs& a, int cidx, int expected,
                                             const float* sm_acc, const float* sm_m, const float* sm_l,
                                             int* sm_last, int n_valid_rows, MapFn map) {
    publish_partial<T, D, NW * 64, NS, ROWS, ACC_STRIDE>(a, sm_acc, sm_m, sm_l, n_valid_rows, map);
    return arrive(a, cidx, expected, sm_last);
}

template <typename T, int D, int NW, int NS, int ROWS, int ACC_STRIDE, typename MapFn>
__device__ __forceinline__ void finish_unit(const KernelArgs& a, const Unit& unit, int kvh, int zidx,
                                            const float* sm_acc, const float* sm_m, const float* sm_l,
                                            int* sm_last, int n_valid_rows, MapFn map) {
    const int cidx = counter_index(a, unit.inst, kvh, zidx);
    if (!publish_unit<T, D, NW, NS, ROWS, ACC_STRIDE>(a, cidx, unit.n_units_inst, sm_acc, sm_m, sm_l, sm_last, n_valid_rows, map))
        return;
    merge_dispatch<T, D, NW * 64>(a, unit.unit0_inst, unit.n_units_inst, n_valid_rows * (D / 2), map);
    reset_counter(a, cidx);
}

}  // namespace attn
}  // namespace matkv
