// Split-KV attention of single query rows over the assembled cache (decode attention, paper
// Section V-A "decode time"; also the plain-FMA form of the question prefill).
//
// No matrix cores: one row against N keys is a bandwidth problem.  A workgroup streams the
// K rows and the V rows of its work unit (page pieces and/or the tail) for ONE KV head from
// HBM with 16-byte loads, serves all G = Hq/Hkv query heads of that KV head from the same
// registers, and keeps a running (max, sum, accumulator) per head.  Lanes that share a token
// reduce their partial dot products with DPP adds inside a 16-lane row.  The next block's
// loads are issued before the current block is consumed.  Units of one (instance, KV head,
// row) are merged by the last workgroup to arrive (atomic ticket), so a layer's attention is
// one launch; partials travel through agent-scope (cache-bypassing) accesses, which keeps
// the chip's separate L2 slices coherent without flushing them.
#include "attn_common.h"

namespace matkv {
namespace {

using namespace attn;

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> { static constexpr int kPerLoad = 4; };
template <> struct ElemTraits<uint16_t> { static constexpr int kPerLoad = 8; };   // bf16 bits

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(o);
}

// Sum over the LPT consecutive lanes that share a token; every lane of the group gets it.
template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
    static_assert(LPT == 8 || LPT == 16 || LPT == 32, "lanes per token");
    v = dpp_add<0xB1>(v);     // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);     // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);    // row_half_mirror: other quad of the 8
    if (LPT >= 16) v = dpp_add<0x140>(v);   // row_mirror: other half of the 16-lane row
    if (LPT >= 32) v += __shfl_xor(v, 16);
    return v;
}

// ---- per-element-type arithmetic on one 16-byte piece of a K or V row -----------------------
// Q is kept in the form the dot product wants: fp32 for the fp32 path, packed bf16 pairs for
// the bf16 path (exact: Q arrives as bf16), where v_dot2_f32_bf16 does two multiply-adds per
// lane and instruction with an fp32 accumulator.
template <typename T> struct RowMath;

template <> struct RowMath<float> {
    static constexpr int QREGS = 4;
    typedef float qreg_t;
    static __device__ __forceinline__ void load_q(const uint4& raw, qreg_t* q) {
        q[0] = __uint_as_float(raw.x); q[1] = __uint_as_float(raw.y);
        q[2] = __uint_as_float(raw.z); q[3] = __uint_as_float(raw.w);
    }
    static __device__ __forceinline__ float dot(const qreg_t* q, const uint4& k) {
        float d = q[0] * __uint_as_float(k.x);
        d = fmaf(q[1], __uint_as_float(k.y), d);
        d = fmaf(q[2], __uint_as_float(k.z), d);
        d = fmaf(q[3], __uint_as_float(k.w), d);
        return d;
    }
};

template <> struct RowMath<uint16_t> {
    static constexpr int QREGS = 4;
    typedef uint32_t qreg_t;
    static __device__ __forceinline__ void load_q(const uint4& raw, qreg_t* q) {
        q[0] = raw.x; q[1] = raw.y; q[2] = raw.z; q[3] = raw.w;
    }
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
    }
    static __device__ __forceinline__ float dot(const qreg_t* q, const uint4& k) {
        float d = dot2(q[0], k.x, 0.f);
        d = dot2(q[1], k.y, d);
        d = dot2(q[2], k.z, d);
        d = dot2(q[3], k.w, d);
        return d;
    }
};

// acc[g][e] += sum_u p[u][g] * v[u][e]
template <typename T, int G, int U> struct PV;

template <int G, int U> struct PV<float, G, U> {
    static __device__ __forceinline__ void run(const uint4* vraw, const float (*p)[G], float (*acc)[4]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float vf[4] = {__uint_as_float(vraw[u].x), __uint_as_float(vraw[u].y),
                                 __uint_as_float(vraw[u].z), __uint_as_float(vraw[u].w)};
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[g][e] = fmaf(p[u][g], vf[e], acc[g][e]);
        }
    }
};

// bf16: two tokens at a time.  The two rows' elements are interleaved with byte permutes into
// (token u, token u+1) pairs per element, the two probabilities are rounded to one bf16 pair,
// and one dot2 per (head, element) adds both tokens.
template <int G, int U> struct PV<uint16_t, G, U> {
    static_assert(U % 2 == 0, "tokens are consumed in pairs");
    static __device__ __forceinline__ void run(const uint4* vraw, const float (*p)[G], float (*acc)[8]) {
#pragma unroll
        for (int u = 0; u < U; u += 2) {
            const uint32_t a[4] = {vraw[u].x, vraw[u].y, vraw[u].z, vraw[u].w};
            const uint32_t b[4] = {vraw[u + 1].x, vraw[u + 1].y, vraw[u + 1].z, vraw[u + 1].w};
            uint32_t ev[4], od[4];     // element 2w of both tokens, element 2w+1 of both tokens
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                ev[w] = __builtin_amdgcn_perm(b[w], a[w], 0x05040100u);   // {a.lo, b.lo}
                od[w] = __builtin_amdgcn_perm(b[w], a[w], 0x07060302u);   // {a.hi, b.hi}
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const f32x2 pf = {p[u][g], p[u + 1][g]};
                const uint32_t pp = __builtin_bit_cast(uint32_t, __builtin_convertvector(pf, bf16x2));
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    acc[g][2 * w] = RowMath<uint16_t>::dot2(pp, ev[w], acc[g][2 * w]);
                    acc[g][2 * w + 1] = RowMath<uint16_t>::dot2(pp, od[w], acc[g][2 * w + 1]);
                }
            }
        }
    }
};

template <typename T, int D, int G, int NW, int U>
__global__ __launch_bounds__(NW * 64) void attn_rows_kernel(
        KernelArgs a, const InstanceInfo* __restrict__ insts, const Item* __restrict__ items,
        const Unit* __restrict__ units) {
    constexpr int EPL = ElemTraits<T>::kPerLoad;        // elements per 16-byte load
    constexpr int LPT = D / EPL;                        // lanes that share one token row
    constexpr int TPW = 64 / LPT;                       // token rows per wave-wide load
    constexpr int BLK = TPW * U;                        // token rows one wave handles per step
    typedef RowMath<T> RM;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps the block walk scalar
    const int lane = tid & 63;
    const int grp = lane / LPT, sub = lane % LPT;
    const int kvh = blockIdx.y, row = blockIdx.z;

    const Unit unit = units[blockIdx.x];

    int q_row, tail_visible = 0;
    if (a.prefill) {
        const InstanceInfo inst = insts[unit.inst];
        if (row >= inst.q_len) return;                  // whole workgroup leaves together
        q_row = inst.cu_q + row;
        tail_visible = row + 1;
    } else {
        q_row = unit.inst;
        if (unit.has_tail) tail_visible = insts[unit.inst].tail_len;
    }

    // This lane's slice of the G query vectors.
    typename RM::qreg_t qr[G][RM::QREGS];
    {
        const T* qp = reinterpret_cast<const T*>(a.q) + ((size_t)q_row * a.Hq + (size_t)kvh * G) * D + sub * EPL;
#pragma unroll
        for (int g = 0; g < G; ++g) RM::load_q(ldg16(qp + (size_t)g * D), qr[g]);
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    Walker<T, D, NW, BLK, TPW> walk(a, unit, items, kvh, tail_visible, wave);
    auto next_block = [&]() { return walk.next(); };
    // Rows past the end are clamped to the last valid row (a cached re-read, no extra HBM
    // traffic) and masked later, so all 2*U loads issue back to back without branches.
    auto issue = [&](const BlockRef<T>& r, uint4* kraw, uint4* vraw) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t eoff = (size_t)min(r.t0 + u * TPW + grp, r.tok_end - 1) * D + sub * EPL;
            kraw[u] = ldg16(r.k + eoff);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t eoff = (size_t)min(r.t0 + u * TPW + grp, r.tok_end - 1) * D + sub * EPL;
            vraw[u] = ldg16(r.v + eoff);
        }
    };
    auto consume = [&](const BlockRef<T>& r, const uint4* kraw, const uint4* vraw) {
        float s[U][G];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = r.t0 + u * TPW + grp < r.tok_end;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float d = group_sum<LPT>(RM::dot(qr[g], kraw[u]));
                s[u][g] = ok ? d * a.scale_log2e : kNegBig;
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mn = m[g];
#pragma unroll
            for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][g]);
            const float alpha = fast_exp2(m[g] - mn);
            m[g] = mn;
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool ok = r.t0 + u * TPW + grp < r.tok_end;
                s[u][g] = ok ? fast_exp2(s[u][g] - mn) : 0.f;
                psum += s[u][g];
            }
            l[g] = l[g] * alpha + psum;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
        }
        PV<T, G, U>::run(vraw, s, acc);
    };

    {
        uint4 k0[U], v0[U], k1[U], v1[U];
        BlockRef<T> r0 = next_block(), r1;
        if (r0.valid) issue(r0, k0, v0);
        while (r0.valid) {
            r1 = next_block();
            if (r1.valid) issue(r1, k1, v1);
            consume(r0, k0, v0);
            if (!r1.valid) break;
            r0 = next_block();
            if (r0.valid) issue(r0, k0, v0);
            consume(r1, k1, v1);
        }
    }

    // ---- merge the TPW token groups of the wave (each kept its own running state) ----
    // Lane exchanges at distance 32 and 16 are register swaps on this chip; distance 8 (only
    // when a row holds two tokens) goes through the LDS crossbar.
#pragma unroll
    for (int off = 32; off >= LPT; off >>= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = lane_xor(m[g], off, lane);
            const float lo = lane_xor(l[g], off, lane);
            const float mn = fmaxf(m[g], mo);
            const float ca = fast_exp2(m[g] - mn), cb = fast_exp2(mo - mn);
            l[g] = l[g] * ca + lo * cb;
            m[g] = mn;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float ao = lane_xor(acc[g][e], off, lane);
                acc[g][e] = acc[g][e] * ca + ao * cb;
            }
        }
    }

    // ---- per-wave states to LDS, then the common merge ----
    __shared__ float sm_acc[NW][G][D];
    __shared__ float sm_m[NW][G], sm_l[NW][G];
    __shared__ int sm_last;
    if (grp == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) sm_acc[wave][g][sub * EPL + e] = acc[g][e];
            if (sub == 0) { sm_m[wave][g] = m[g]; sm_l[wave][g] = l[g]; }
        }
    }
    auto map = [&](int g) {
        RowMap rm;
        rm.slot_row = row; rm.head = kvh * G + g; rm.q_row = q_row;
        return rm;
    };
    finish_unit<T, D, NW, NW, G, D>(a, unit, kvh, row, &sm_acc[0][0][0], &sm_m[0][0], &sm_l[0][0], &sm_last, G, map);
}

template <typename T, int D, int G, int NW, int U>
hipError_t launch_v(const AttnArgs& a, hipStream_t s) {
    const KernelArgs k = make_kernel_args(a);
    dim3 grid(a.n_units, a.Hkv, a.rows), block(NW * 64);
    hipLaunchKernelGGL((attn_rows_kernel<T, D, G, NW, U>), grid, block, 0, s, k,
                       reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst),
                       reinterpret_cast<const Item*>(a.table + a.off_items),
                       reinterpret_cast<const Unit*>(a.table + a.off_units));
    return hipGetLastError();
}

// variant = NW * 100 + U for the shapes built below; 0 picks the default
template <typename T, int D, int G>
hipError_t launch_t(const AttnArgs& a, hipStream_t s) {
    if constexpr (sizeof(T) == 2 && D == 128 && (G == 4 || G == 8)) {
        switch (a.variant) {
            case 402: return launch_v<T, D, G, 4, 2>(a, s);
            case 408: return launch_v<T, D, G, 4, 8>(a, s);
            case 802: return launch_v<T, D, G, 8, 2>(a, s);
            case 804: return launch_v<T, D, G, 8, 4>(a, s);
            case 202: return launch_v<T, D, G, 2, 2>(a, s);
            case 204: return launch_v<T, D, G, 2, 4>(a, s);
            case 208: return launch_v<T, D, G, 2, 8>(a, s);
            case 102: return launch_v<T, D, G, 1, 2>(a, s);
            case 104: return launch_v<T, D, G, 1, 4>(a, s);
            case 108: return launch_v<T, D, G, 1, 8>(a, s);
            default: break;
        }
    }
    return launch_v<T, D, G, 4, 4>(a, s);
}

template <typename T, int D>
hipError_t launch_g(const AttnArgs& a, hipStream_t s) {
    switch (a.Hq / a.Hkv) {
        case 1: return launch_t<T, D, 1>(a, s);
        case 2: return launch_t<T, D, 2>(a, s);
        case 3: return launch_t<T, D, 3>(a, s);
        case 4: return launch_t<T, D, 4>(a, s);
        case 8: return launch_t<T, D, 8>(a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn_rows(const AttnArgs& a, int dtype, hipStream_t s) {
    if (a.n_units <= 0) return hipSuccess;
    if (dtype == MATKV_F32) {
        if (a.D == 64) return launch_g<float, 64>(a, s);
        if (a.D == 128) return launch_g<float, 128>(a, s);
    } else {
        if (a.D == 64) return launch_g<uint16_t, 64>(a, s);
        if (a.D == 128) return launch_g<uint16_t, 128>(a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace matkv
