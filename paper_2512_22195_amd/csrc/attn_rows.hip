// Split-KV attention of single query rows over the assembled cache (decode attention, paper
// Section V-A "decode time"; also the plain-FMA form of the question prefill).
//
// No matrix cores: one row against N keys is a bandwidth problem.  A workgroup streams the
// K rows, then the V rows, of its work unit (a run of page pieces, or the tail) for ONE KV
// head from HBM with 16-byte loads, serves all G = Hq/Hkv query heads of that KV head from
// the same registers, and keeps a running (max, sum, accumulator) per head.  Lanes that share
// a token reduce their partial dot products with DPP adds inside a 16-lane row.  Units of one
// (instance, KV head, row) are merged by the last workgroup to arrive (atomic ticket), so a
// layer's attention is one launch.
#include "matkv_internal.h"

namespace matkv {
namespace {

constexpr float kNegBig = -1.0e30f;   // "no key seen yet": finite, so that exp2(m - m) = 1

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> { static constexpr int kPerLoad = 4; };
template <> struct ElemTraits<uint16_t> { static constexpr int kPerLoad = 8; };   // bf16 bits

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// 16 bytes -> kPerLoad floats
template <typename T> struct Vec16;
template <> struct Vec16<float> {
    static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
};
template <> struct Vec16<uint16_t> {
    static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
};

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

template <typename T, int D, int G, int NW, int U>
__global__ __launch_bounds__(NW * 64) void attn_rows_kernel(AttnArgs a) {
    constexpr int EPL = ElemTraits<T>::kPerLoad;        // elements per 16-byte load
    constexpr int LPT = D / EPL;                        // lanes that share one token row
    constexpr int TPW = 64 / LPT;                       // token rows per wave-wide load
    constexpr int PSTRIDE = D + 2;                      // floats of one partial: acc, m, l

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int grp = lane / LPT, sub = lane % LPT;
    const int kvh = blockIdx.y, row = blockIdx.z;

    const InstanceInfo* insts = reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst);
    const Item* items = reinterpret_cast<const Item*>(a.table + a.off_items);
    const Unit unit = reinterpret_cast<const Unit*>(a.table + a.off_units)[blockIdx.x];
    const InstanceInfo inst = insts[unit.inst];

    int q_row, tail_visible, n_units_inst, unit0_inst;
    if (a.prefill) {
        if (row >= inst.q_len) return;                  // whole workgroup leaves together
        q_row = inst.cu_q + row;
        tail_visible = row + 1;
        n_units_inst = inst.n_punits; unit0_inst = inst.punit0;
    } else {
        q_row = unit.inst;
        tail_visible = inst.tail_len;
        n_units_inst = inst.n_dunits; unit0_inst = inst.dunit0;
    }

    // This lane's slice of the G query vectors, scaled so that exp2 can be used.
    float qf[G][EPL];
    {
        const T* qp = reinterpret_cast<const T*>(a.q) + ((size_t)q_row * a.Hq + (size_t)kvh * G) * D + sub * EPL;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            uint4 raw = *reinterpret_cast<const uint4*>(qp + (size_t)g * D);
            Vec16<T>::unpack(raw, qf[g]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) qf[g][e] *= a.scale_log2e;
        }
    }

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    for (int it = 0; it < unit.n_items; ++it) {
        const Item item = items[unit.item0 + it];
        const T* kbase;
        const T* vbase;
        int tok_end = item.tok0 + item.ntok;
        if (item.base) {
            const size_t head_elems = (size_t)item.page_tokens * D;
            const T* blob = reinterpret_cast<const T*>(item.base);
            kbase = blob + ((size_t)(a.layer * 2 + 0) * a.Hkv + kvh) * head_elems;
            vbase = blob + ((size_t)(a.layer * 2 + 1) * a.Hkv + kvh) * head_elems;
        } else {
            const size_t off = ((size_t)unit.inst * a.Hkv + kvh) * (size_t)a.max_tail * D;
            kbase = reinterpret_cast<const T*>(a.tail_k) + off;
            vbase = reinterpret_cast<const T*>(a.tail_v) + off;
            tok_end = min(tok_end, tail_visible);
        }
        for (int t0 = item.tok0 + wave * (TPW * U); t0 < tok_end; t0 += NW * TPW * U) {
            uint4 kraw[U], vraw[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int tok = t0 + u * TPW + grp;
                ok[u] = tok < tok_end;
                const size_t eoff = (size_t)tok * D + sub * EPL;
                kraw[u] = ok[u] ? *reinterpret_cast<const uint4*>(kbase + eoff) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int tok = t0 + u * TPW + grp;
                const size_t eoff = (size_t)tok * D + sub * EPL;
                vraw[u] = ok[u] ? *reinterpret_cast<const uint4*>(vbase + eoff) : make_uint4(0, 0, 0, 0);
            }
            float s[U][G];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float kf[EPL];
                Vec16<T>::unpack(kraw[u], kf);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) d = fmaf(qf[g][e], kf[e], d);
                    d = group_sum<LPT>(d);
                    s[u][g] = ok[u] ? d : kNegBig;
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mn = m[g];
#pragma unroll
                for (int u = 0; u < U; ++u) mn = fmaxf(mn, s[u][g]);
                const float alpha = exp2f(m[g] - mn);
                m[g] = mn;
                float psum = 0.f;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    s[u][g] = ok[u] ? exp2f(s[u][g] - mn) : 0.f;
                    psum += s[u][g];
                }
                l[g] = l[g] * alpha + psum;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[EPL];
                Vec16<T>::unpack(vraw[u], vf);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(s[u][g], vf[e], acc[g][e]);
            }
        }
    }

    // ---- merge the TPW token groups of the wave (each kept its own running state) ----
#pragma unroll
    for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(m[g], off);
            const float lo = __shfl_xor(l[g], off);
            const float mn = fmaxf(m[g], mo);
            const float ca = exp2f(m[g] - mn), cb = exp2f(mo - mn);
            l[g] = l[g] * ca + lo * cb;
            m[g] = mn;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const float ao = __shfl_xor(acc[g][e], off);
                acc[g][e] = acc[g][e] * ca + ao * cb;
            }
        }
    }

    // ---- merge the waves of the workgroup through LDS ----
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
    __syncthreads();

    const size_t pbase = (((size_t)blockIdx.x * a.rows + row) * a.Hq + (size_t)kvh * G) * PSTRIDE;
    for (int idx = tid; idx < G * D; idx += NW * 64) {
        const int g = idx / D, d = idx % D;
        float mn = sm_m[0][g];
#pragma unroll
        for (int w = 1; w < NW; ++w) mn = fmaxf(mn, sm_m[w][g]);
        float accv = 0.f, lv = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float c = exp2f(sm_m[w][g] - mn);
            accv = fmaf(sm_acc[w][g][d], c, accv);
            lv = fmaf(sm_l[w][g], c, lv);
        }
        float* pp = a.partials + pbase + (size_t)g * PSTRIDE;
        pp[d] = accv;
        if (d == 0) { pp[D] = mn; pp[D + 1] = lv; }
    }

    // ---- the last workgroup of this (instance, KV head, row) merges all units ----
    const int cidx = ((unit.inst * a.Hkv) + kvh) * a.rows + row;
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int prev = atomicAdd(&a.counters[cidx], 1);
        sm_last = (prev == n_units_inst - 1);
    }
    __syncthreads();
    if (!sm_last) return;
    __threadfence();

    for (int idx = tid; idx < G * D; idx += NW * 64) {
        const int g = idx / D, d = idx % D;
        const size_t hoff = ((size_t)kvh * G + g) * PSTRIDE;
        const size_t ustride = (size_t)a.rows * a.Hq * PSTRIDE;
        const float* p0 = a.partials + ((size_t)unit0_inst * a.rows + row) * a.Hq * PSTRIDE + hoff;
        float mn = kNegBig;
        for (int u = 0; u < n_units_inst; ++u)
            mn = fmaxf(mn, p0[(size_t)u * ustride + D]);
        float accv = 0.f, lv = 0.f;
        for (int u = 0; u < n_units_inst; ++u) {
            const float* pu = p0 + (size_t)u * ustride;
            const float c = exp2f(pu[D] - mn);
            accv = fmaf(pu[d], c, accv);
            lv = fmaf(pu[D + 1], c, lv);
        }
        const float o = accv / lv;
        T* op = reinterpret_cast<T*>(a.out) + ((size_t)q_row * a.Hq + (size_t)kvh * G + g) * D + d;
        if constexpr (sizeof(T) == 4) *reinterpret_cast<float*>(op) = o;
        else *reinterpret_cast<uint16_t*>(op) = f32_to_bf16_rne(o);
    }
    if (tid == 0) a.counters[cidx] = 0;   // ready for the next launch on this stream
}

template <typename T, int D, int G>
hipError_t launch_t(const AttnArgs& a, hipStream_t s) {
    constexpr int NW = 4, U = 4;
    dim3 grid(a.n_units, a.Hkv, a.rows), block(NW * 64);
    hipLaunchKernelGGL((attn_rows_kernel<T, D, G, NW, U>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_g(const AttnArgs& a, hipStream_t s) {
    switch (a.Hq / a.Hkv) {
        case 1: return launch_t<T, D, 1>(a, s);
        case 2: return launch_t<T, D, 2>(a, s);
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
