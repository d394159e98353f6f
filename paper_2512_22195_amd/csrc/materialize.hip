// K/V materialization of one layer (paper Section III-B steps 2-3, cut to the K/V projection):
//   K[g][i][:] = RoPE(Wk_g x_i, pos_i),  V[g][i][:] = Wv_g x_i
// This file holds the row-streaming form: one wave owns one rotary pair (features j and
// j + D/2 of one head, K or V) and reads those two weight rows once for a small tile of
// tokens.  With one token per instance (a decode step) it is a GEMV bound by reading the
// weights once from HBM; it is also the fp32 path.  The tile-GEMM form for long token
// runs lives in materialize_mfma.hip.
#include "gemv_common.h"

namespace matkv {
namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

using dev::f32_to_bf16_rne;

template <typename T> struct Ld;
template <> struct Ld<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void get(const float* p, float* f) {
        const float4 r = *reinterpret_cast<const float4*>(p);
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
};
template <> struct Ld<uint16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void get(const uint16_t* p, float* f) {
        const uint4 r = *reinterpret_cast<const uint4*>(p);
        f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
        f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Where a row of the hidden-state matrix goes and which position it takes.
struct RowDest {
    int64_t pos;        // rotary position
    size_t elem_off;    // element offset of [head 0][row][0] in the destination
    bool valid;
};

__device__ __forceinline__ RowDest resolve_row(const MaterializeArgs& a, int r) {
    RowDest d;
    d.valid = false; d.pos = 0; d.elem_off = 0;
    if (a.table == nullptr) {
        if (r < a.n_tokens) { d.valid = true; d.pos = a.pos0 + r; d.elem_off = (size_t)r * a.D; }
        return d;
    }
    const InstanceInfo* insts = reinterpret_cast<const InstanceInfo*>(a.table + a.off_inst);
    int b = -1, j = 0;
    if (a.rows_per_instance > 0) {
        if (r < a.batch * a.rows_per_instance) {
            b = r / a.rows_per_instance;
            j = insts[b].tail_len - a.rows_per_instance + (r % a.rows_per_instance);
        }
    } else {
        for (int i = 0; i < a.batch; ++i) {
            const int c0 = insts[i].cu_q;
            if (r >= c0 && r < c0 + insts[i].q_len) { b = i; j = r - c0; break; }
        }
    }
    if (b < 0 || j < 0 || j >= a.token_stride) return d;
    d.valid = true;
    d.pos = insts[b].pos_base + j;
    d.elem_off = ((size_t)b * a.Hkv * a.token_stride + (size_t)j) * a.D;
    return d;
}

template <typename T>
__device__ __forceinline__ void rope_cs(const RopeEntry& e, int64_t pos, float& c, float& s) {
    if constexpr (sizeof(T) == 4) {
        // fp32 path: the angle in double, so that the 1e-5 parity bar holds at any position
        double sd, cd;
        sincos((double)pos * e.inv_freq, &sd, &cd);
        c = (float)cd; s = (float)sd;
    } else {
        // bf16 path: the angle in turns, hi/lo split product, whole turns dropped exactly (no
        // contraction: p * turns_hi - rint(t) as one multiply-add would count t's rounding error twice)
#pragma clang fp contract(off)
        const float p = (float)pos;
        const float t = p * e.turns_hi;
        const float err = fmaf(p, e.turns_hi, -t);
        float fr = t - rintf(t);
        fr += fmaf(p, e.turns_lo, err);
        const float ang = fr * 6.283185307179586f;
        c = cosf(ang); s = sinf(ang);
    }
}

constexpr int kWavesPerBlock = 4;

template <typename T, int TT>
__global__ __launch_bounds__(kWavesPerBlock * 64) void materialize_rows_kernel(MaterializeArgs a) {
    constexpr int N = Ld<T>::N;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int half = a.D / 2;
    const int task = blockIdx.x * kWavesPerBlock + wave;     // (kv, head, pair)
    const int n_tasks = 2 * a.Hkv * half;
    if (task >= n_tasks) return;
    const int kv = task / (a.Hkv * half);
    const int head = (task / half) % a.Hkv;
    const int j = task % half;
    const int row0 = blockIdx.y * TT;

    const T* w = reinterpret_cast<const T*>(kv == 0 ? a.w_k : a.w_v);
    const T* w0 = w + ((size_t)head * a.D + j) * a.Hd;
    const T* w1 = w0 + (size_t)half * a.Hd;
    const T* x = reinterpret_cast<const T*>(a.hidden) + (size_t)row0 * a.Hd;

    RowDest dest[TT];
    bool any = false;
#pragma unroll
    for (int t = 0; t < TT; ++t) { dest[t] = resolve_row(a, row0 + t); any |= dest[t].valid; }
    if (!any) return;

    float acc0[TT], acc1[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) { acc0[t] = 0.f; acc1[t] = 0.f; }

#pragma unroll 8
    for (int c = lane * N; c < a.Hd; c += 64 * N) {
        float f0[N], f1[N];
        Ld<T>::get(w0 + c, f0);
        Ld<T>::get(w1 + c, f1);
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            if (!dest[t].valid) continue;
            float xf[N];
            Ld<T>::get(x + (size_t)t * a.Hd + c, xf);
#pragma unroll
            for (int e = 0; e < N; ++e) {
                acc0[t] = fmaf(f0[e], xf[e], acc0[t]);
                acc1[t] = fmaf(f1[e], xf[e], acc1[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < TT; ++t) { acc0[t] = wave_sum(acc0[t]); acc1[t] = wave_sum(acc1[t]); }

    if (lane < TT) {
        RowDest d; float r0 = 0.f, r1 = 0.f;
#pragma unroll
        for (int t = 0; t < TT; ++t) if (lane == t) { d = dest[t]; r0 = acc0[t]; r1 = acc1[t]; }
        if (d.valid) {
            if (kv == 0) {
                float c, s;
                rope_cs<T>(a.rope[j], d.pos, c, s);
                const float k0 = r0 * c - r1 * s;
                const float k1 = r0 * s + r1 * c;
                r0 = k0; r1 = k1;
            }
            T* out = reinterpret_cast<T*>(kv == 0 ? a.k_out : a.v_out) + d.elem_off +
                     (size_t)head * a.token_stride * a.D + j;
            if constexpr (sizeof(T) == 4) { out[0] = r0; out[half] = r1; }
            else { out[0] = f32_to_bf16_rne(r0); out[half] = f32_to_bf16_rne(r1); }
        }
    }
}

// ---- bf16 GEMV form: a handful of token rows (a decode step), hidden a multiple of 4096 ------
// (NL = 8) or of 3072 (NL = 6: Llama-3.2-3B).
// One wave per rotary pair, as above, but shaped for latency (see gemv_common.h).
// KS = 2: the hidden axis is cut in two and a pair is the work of two waves of the workgroup
// (eight waves, two per SIMD), each with one pass of 512 * NL columns - all weight loads of the
// launch are then requested at once instead of in two dependent rounds (hidden 8192, four
// rows: 11.3 -> 10.9 us); the odd wave hands its sums over through LDS.
template <int R, int NL, int KS>
__global__ __launch_bounds__(kWavesPerBlock * KS * 64) void materialize_gemv_kernel(MaterializeArgs a) {
    typedef uint16_t T;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int half = a.D / 2;
    const int task = blockIdx.x * kWavesPerBlock + wave / KS;     // (kv, head, pair)
    const int part = wave % KS;                                   // which slice of the hidden axis
    const bool live = task < 2 * a.Hkv * half;
    const int kv = task / (a.Hkv * half);
    const int head = (task / half) % a.Hkv;
    const int j = task % half;
    const int row0 = blockIdx.y * R;
    const int Hd_part = a.Hd / KS;

    __shared__ float sm_part[KS > 1 ? kWavesPerBlock : 1][2][R];
    float acc0[R], acc1[R];
    if (live) {
        const T* w = reinterpret_cast<const T*>(kv == 0 ? a.w_k : a.w_v);
        const T* w0 = w + ((size_t)head * a.D + j) * a.Hd + (size_t)part * Hd_part;
        const T* w1 = w0 + (size_t)half * a.Hd;
        const T* x = reinterpret_cast<const T*>(a.hidden) + (size_t)row0 * a.Hd + (size_t)part * Hd_part;
        gemv::pair_dots<R, NL>(w0, w1, x, (size_t)a.Hd, a.n_tokens - row0, Hd_part, lane, acc0, acc1);
    }
    if constexpr (KS > 1) {
        if (live && part == 1 && lane < R) {
#pragma unroll
            for (int r = 0; r < R; ++r) if (lane == r) { sm_part[wave / KS][0][r] = acc0[r]; sm_part[wave / KS][1][r] = acc1[r]; }
        }
        __syncthreads();
        if (part != 0) return;
    }
    if (!live) return;

    if (lane < R) {
        float r0 = 0.f, r1 = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r) if (lane == r) { r0 = acc0[r]; r1 = acc1[r]; }
        if constexpr (KS > 1) { r0 += sm_part[wave / KS][0][lane]; r1 += sm_part[wave / KS][1][lane]; }
        const RowDest d = resolve_row(a, row0 + lane);
        if (d.valid) {
            if (kv == 0) gemv::rotate_pair(a.rope[j], (float)d.pos, r0, r1);
            T* out = reinterpret_cast<T*>(kv == 0 ? a.k_out : a.v_out) + d.elem_off +
                     (size_t)head * a.token_stride * a.D + j;
            out[0] = f32_to_bf16_rne(r0);
            out[half] = f32_to_bf16_rne(r1);
        }
    }
}

constexpr int kGemmMinRows = 64;
constexpr int kSkinnyMinRows = 32;

bool gemv_supported(const MaterializeArgs& a, int dtype) {
    return dtype == MATKV_BF16 && ((a.Hd % 4096) == 0 || (a.Hd % 3072) == 0);
}

template <int NL, int KS>
hipError_t launch_gemv_nl(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    const int n_tasks = 2 * a.Hkv * (a.D / 2);
    const int bx = (n_tasks + kWavesPerBlock - 1) / kWavesPerBlock;
    const dim3 block(kWavesPerBlock * KS * 64);
    if (total_rows == 1) hipLaunchKernelGGL((materialize_gemv_kernel<1, NL, KS>), dim3(bx, 1), block, 0, s, a);
    else if (total_rows == 2) hipLaunchKernelGGL((materialize_gemv_kernel<2, NL, KS>), dim3(bx, 1), block, 0, s, a);
    else hipLaunchKernelGGL((materialize_gemv_kernel<4, NL, KS>), dim3(bx, (total_rows + 3) / 4), block, 0, s, a);
    return hipGetLastError();
}
hipError_t launch_gemv(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    // two passes of columns per wave become one pass in each of two waves
    if (a.Hd == 8192) return launch_gemv_nl<8, 2>(a, total_rows, s);
    if (a.Hd == 6144) return launch_gemv_nl<6, 2>(a, total_rows, s);
    return (a.Hd % 4096) == 0 ? launch_gemv_nl<8, 1>(a, total_rows, s) : launch_gemv_nl<6, 1>(a, total_rows, s);
}

__global__ void advance_kernel(char* table, size_t off_inst, int batch, int n, int max_tail) {
    InstanceInfo* insts = reinterpret_cast<InstanceInfo*>(table + off_inst);
    for (int b = threadIdx.x; b < batch; b += blockDim.x) {
        const int v = insts[b].tail_len + n;
        insts[b].tail_len = v > max_tail ? max_tail : v;   // never walks off the tail buffer
    }
}

template <typename T>
hipError_t launch_rows(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    const int n_tasks = 2 * a.Hkv * (a.D / 2);
    const int bx = (n_tasks + kWavesPerBlock - 1) / kWavesPerBlock;
    if (total_rows <= 1) {
        hipLaunchKernelGGL((materialize_rows_kernel<T, 1>), dim3(bx, 1), dim3(kWavesPerBlock * 64), 0, s, a);
    } else {
        constexpr int TT = 4;
        hipLaunchKernelGGL((materialize_rows_kernel<T, TT>), dim3(bx, (total_rows + TT - 1) / TT),
                           dim3(kWavesPerBlock * 64), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_materialize(const MaterializeArgs& a, int dtype, hipStream_t s) {
    const int total_rows = a.n_tokens;
    if (total_rows <= 0) return hipSuccess;
    // a decode step of a batch: the GEMV form reads the weights once per 4 rows; from 16 rows on
    // the matrix cores take over where the skinny form that stages rows through LDS exists (hidden
    // a multiple of 1024; 16 rows at hidden 4096 / 8192: 8.0 / 14.8 us against 9.7 / 20.7, 31 rows
    // 8.0 / 13.5 against 16.1 / 33.6), from 32 rows on elsewhere (skinny forms, then the tiled GEMM)
    // up to 16 rows (a decode step): the staged form cut into 256 workgroups where it is ahead of the
    // GEMV form (per layer, every layer's weights from HBM: 4 rows at hidden 8192 10.9 -> 9.0 us,
    // 16 rows at hidden 4096 10.4 -> 7.9 us; one row at hidden 4096 5.8 us against 6.1: GEMV kept)
    if ((total_rows >= 8 || a.Hd >= 8192) && materialize_fewrows_supported(a, dtype, total_rows))
        return launch_materialize_fewrows(a, total_rows, s);
    const int skinny_min = (a.Hd % 1024) == 0 ? 16 : kSkinnyMinRows;
    if (gemv_supported(a, dtype) && total_rows < kGemmMinRows &&
        !(total_rows >= skinny_min && materialize_mfma_supported(a, dtype, total_rows) && (a.Hd % 512) == 0))
        return launch_gemv(a, total_rows, s);
    if (materialize_mfma_supported(a, dtype, total_rows)) return launch_materialize_mfma(a, total_rows, s);
    if (dtype == MATKV_F32) return launch_rows<float>(a, total_rows, s);
    if (gemv_supported(a, dtype)) return launch_gemv(a, total_rows, s);
    return launch_rows<uint16_t>(a, total_rows, s);
}

// Plain streaming read (measurement aid): every workgroup sums one contiguous slice.
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t vec_per_wg, size_t n_vec, unsigned* sink) {
    const size_t v0 = (size_t)blockIdx.x * vec_per_wg;
    const size_t v1 = v0 + vec_per_wg < n_vec ? v0 + vec_per_wg : n_vec;
    unsigned acc = 0;
    for (size_t i = v0 + threadIdx.x; i < v1; i += 256 * 8) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { const size_t j = i + (size_t)u * 256; v[u] = j < v1 ? src[j] : make_uint4(0, 0, 0, 0); }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;          // keeps the loads alive; practically never taken
}

hipError_t launch_probe_read(const void* src, size_t bytes, unsigned* sink, hipStream_t s) {
    const size_t n_vec = bytes / 16;
    const int grid = 2048;
    const size_t vec_per_wg = (n_vec + grid - 1) / grid;
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<const uint4*>(src), vec_per_wg, n_vec, sink);
    return hipGetLastError();
}

// One instance, no pages, a "tail" of n_tokens rows all of which are question rows; one unit
// whose single item is that tail.  Written by one thread: the three records are 160 bytes.
__global__ void chunk_table_kernel(char* table, int n_tokens) {
    if (threadIdx.x != 0) return;
    InstanceInfo in;
    in.pos_base = 0; in.tail_len = n_tokens; in.q_len = n_tokens; in.cu_q = 0;
    in.dunit0 = 0; in.n_dunits = 0; in.punit0 = 0; in.n_punits = 1;
    in.sslot0 = 0; in.n_sslots = 0; in.pad = 0;
    Item it;
    it.base = 0; it.page_tokens = n_tokens; it.tok0 = 0; it.ntok = n_tokens;
    it.fmt = 0; it.scales16 = 0; it.umask = 0;
    Unit un;
    un.inst = 0; un.item0 = 0; un.n_items = 1; un.idx_in_inst = 0; un.n_units_inst = 1;
    un.unit0_inst = 0; un.has_tail = 1; un.page_tokens = 0; un.first = it;
    *reinterpret_cast<InstanceInfo*>(table + kChunkOffInst) = in;
    *reinterpret_cast<Item*>(table + kChunkOffItem) = it;
    *reinterpret_cast<Unit*>(table + kChunkOffUnit) = un;
}

hipError_t launch_chunk_table(char* table, int n_tokens, hipStream_t s) {
    hipLaunchKernelGGL(chunk_table_kernel, dim3(1), dim3(64), 0, s, table, n_tokens);
    return hipGetLastError();
}

hipError_t launch_advance(char* table, size_t off_inst, int batch, int n, int max_tail, hipStream_t s) {
    hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(64), 0, s, table, off_inst, batch, n, max_tail);
    return hipGetLastError();
}

}  // namespace matkv
