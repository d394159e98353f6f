// K/V materialization of one layer as a matrix-core GEMM with the rotary embedding in the
// epilogue (paper Section III-B steps 2-3, cut to the K/V projection):
//   [T, Hd] x [2*Hkv*D, Hd]^T  ->  K = RoPE(X Wk^T, pos), V = X Wv^T,   bf16, D = 128.
// Both operands are contiguous along the contraction (hidden) axis, which is what the
// matrix-core operand layout wants: a lane's 8 consecutive bf16 of one row.
//
// A workgroup owns 128 (or 64) tokens x one head of K or of V (128 features, so both halves of
// every rotary pair are in the tile), stepping 64 hidden columns at a time through double-buffered
// LDS tiles fed from four rotating register stages (two steps' loads stay in flight).  Its four
// waves form a 2 x 2 grid of sub-tiles 64 features wide; a wave's features are the 16-wide
// blocks {2w, 2w+1} and their rotary partners {2w+4, 2w+5}, so the rotation is lane-local on
// the fp32 accumulators.  One rounding to bf16 on store.
#include <type_traits>

#include "matkv_internal.h"

namespace matkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 16;         // bf16 per LDS row: 160 bytes (the 16-byte operand reads measured 4.5 cycles per instruction, 8.6 with 144 bytes)

__device__ __forceinline__ uint4 ldg16(const void* p) {
    typedef const __attribute__((address_space(1))) u32x4* gptr;
    const u32x4 r = *(gptr)(uintptr_t)p;
    return make_uint4(r.x, r.y, r.z, r.w);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

struct RowDest {
    float pos;          // rotary position (exact in fp32: below 2^24)
    size_t elem_off;    // element offset of [head 0][row][0] in the destination
    bool valid;
};

__device__ __forceinline__ RowDest resolve_row(const MaterializeArgs& a, int r) {
    RowDest d;
    d.valid = false; d.pos = 0.f; d.elem_off = 0;
    if (a.table == nullptr) {
        if (r < a.n_tokens) { d.valid = true; d.pos = (float)(a.pos0 + r); d.elem_off = (size_t)r * D; }
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
    d.pos = (float)(insts[b].pos_base + j);
    d.elem_off = ((size_t)b * a.Hkv * a.token_stride + (size_t)j) * D;
    return d;
}

// cos / sin of pos * theta_j with the angle kept in turns: hi/lo split product, whole turns
// dropped exactly, then the hardware sine / cosine (which take turns).
__device__ __forceinline__ void rope_cs(const RopeEntry& e, float p, float& c, float& s) {
    // no contraction here: were p * turns_hi - rint(t) fused into one multiply-add, the product
    // would enter exactly and the rounding error of t, added back below, would count twice
    // (half an ulp of t: 1e-4 turns at position 20 000)
#pragma clang fp contract(off)
    const float t = p * e.turns_hi;
    const float err = fmaf(p, e.turns_hi, -t);
    float fr = t - rintf(t);
    fr += fmaf(p, e.turns_lo, err);
    c = __builtin_amdgcn_cosf(fr);
    s = __builtin_amdgcn_sinf(fr);
}

// BM = token rows per workgroup (128, or 64 when 128-row tiles would leave compute units idle)
template <int BM>
__global__ __launch_bounds__(256) void materialize_mfma_kernel(MaterializeArgs a, int total_rows) {
    constexpr int MI = BM / 32;              // 16-row token blocks per wave
    constexpr int LR = BM / 32;              // staging rows per thread for the token tile
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][D * LDS_STRIDE];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int wm = wave >> 1, wn = wave & 1;
    const int kv = blockIdx.x / a.Hkv, head = blockIdx.x % a.Hkv;
    const int row0 = blockIdx.y * BM;

    const uint16_t* X = reinterpret_cast<const uint16_t*>(a.hidden);
    const uint16_t* W = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) + (size_t)head * D * a.Hd;

    // global -> LDS staging: thread t moves 16 bytes of rows t/8 + 32i (i < 4), columns 8*(t%8)
    const int ld_row = tid >> 3, ld_col = (tid & 7) * 8;
    const uint16_t* xg[LR];
    const uint16_t* wg[4];
#pragma unroll
    for (int i = 0; i < LR; ++i) {
        const int r = min(row0 + ld_row + 32 * i, total_rows - 1);       // rows past the end repeat the last
        xg[i] = X + (size_t)r * a.Hd + ld_col;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) wg[i] = W + (size_t)(ld_row + 32 * i) * a.Hd + ld_col;
    // NS register stages rotate through the hidden axis: while block k is multiplied out of one
    // LDS tile, block k+1 moves from its stage into the other tile and blocks k+2 .. k+NS-1 are
    // in flight - a step of 64 columns is far shorter than a trip to the L2, so several steps'
    // worth of loads have to be outstanding.  Loads and LDS stores carry no branch (past the end
    // they repeat the last block) and the loop has one exit, so that the compiler can count the
    // loads in flight instead of draining them at every step.
    constexpr int NS = 4;                       // measured: 6 stages gain nothing over 4
    struct Stage { uint4 x[LR], w[4]; };
    Stage st[NS];
    const int nk = a.Hd / BK;
    auto load_global = [&](Stage& g, int ks) {
        const int k0 = min(ks, nk - 1) * BK;
#pragma unroll
        for (int i = 0; i < LR; ++i) g.x[i] = ldg16(xg[i] + k0);
#pragma unroll
        for (int i = 0; i < 4; ++i) g.w[i] = ldg16(wg[i] + k0);
    };
    auto store_lds = [&](int buf, const Stage& g) {
#pragma unroll
        for (int i = 0; i < LR; ++i)
            *reinterpret_cast<uint4*>(&As[buf][(ld_row + 32 * i) * LDS_STRIDE + ld_col]) = g.x[i];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<uint4*>(&Bs[buf][(ld_row + 32 * i) * LDS_STRIDE + ld_col]) = g.w[i];
    };

    f32x4 acc[MI][4];           // [token block mi][feature block: 2wn, 2wn+1, 2wn+4, 2wn+5]
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
#pragma unroll
        for (int k2 = 0; k2 < BK / 32; ++k2) {
            bf16x8 av[MI], bv[4];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                av[mi] = *reinterpret_cast<const bf16x8*>(&As[buf][(16 * MI * wm + 16 * mi + c16) * LDS_STRIDE + 32 * k2 + 8 * g4]);
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int tn = 2 * wn + (ni & 1) + 4 * (ni >> 1);
                bv[ni] = *reinterpret_cast<const bf16x8*>(&Bs[buf][(16 * tn + c16) * LDS_STRIDE + 32 * k2 + 8 * g4]);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
        }
    };

#pragma unroll
    for (int i = 0; i < NS - 1; ++i) load_global(st[i], i);
    store_lds(0, st[0]);
    lds_barrier();
    int ks = 0;
    // block ks sits in LDS tile ks & 1; its stage index S = ks % NS is a compile-time constant
    auto step = [&](auto stage_tag) {
        constexpr int S = decltype(stage_tag)::value;
        load_global(st[(S + NS - 1) % NS], ks + NS - 1);
        if (ks < nk) compute(ks & 1);
        store_lds((ks + 1) & 1, st[(S + 1) % NS]);
        lds_barrier();
        ++ks;
    };
    do {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
    } while (ks < nk);

    // epilogue: lane holds tokens 16*MI*wm + 16mi + 4*g4 + i, features 16*tn + c16
    uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const RowDest d = resolve_row(a, row0 + 16 * MI * wm + 16 * mi + 4 * g4 + i);
            if (!d.valid) continue;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int j = 16 * (2 * wn + p) + c16;           // rotary pair index, features j and j + 64
                float lo = acc[mi][p][i], hi = acc[mi][p + 2][i];
                if (kv == 0) {
                    float c, s;
                    rope_cs(a.rope[j], d.pos, c, s);
                    const float k0 = lo * c - hi * s;
                    const float k1 = lo * s + hi * c;
                    lo = k0; hi = k1;
                }
                out[d.elem_off + j] = f32_to_bf16_rne(lo);
                out[d.elem_off + j + 64] = f32_to_bf16_rne(hi);
            }
        }
    }
}

// ---- the same tile on eight waves ------------------------------------------------------------
// One wave per SIMD leaves every latency of a step in the open: the operand reads from LDS, the
// matrix instructions that wait for them, the stores of the next tile and the barrier follow
// one another (measured: about 980 cycles per 64-column step around 256 cycles of matrix work).
// Here the workgroup has two wave groups of 2 x 2 waves each; a step covers 128 hidden columns
// and group g multiplies columns 64g .. 64g+63 of it, so every SIMD holds two waves whose
// reads and matrix instructions overlap, and there is one barrier per 128 columns.  Rows of the
// LDS tiles are 256 + 32 bytes: 16 lanes store one whole row at a time and 16 lanes read 16
// bytes of 16 different rows without a bank conflict.  The two groups' partial sums meet in LDS
// once, at the end: each group hands over the token blocks the other one finishes, so all eight
// waves share the rotary epilogue.  (128-row tiles in this form - 238 registers, 139 KB of LDS -
// measured 167 us for a 1000-token chunk against 37 us: not built.)
constexpr int BK8 = 128;
constexpr int STR8 = BK8 + 16;      // 288-byte rows: the 16-byte operand reads measured 5.4 cycles against 8.8 with 272

template <int BM>
__global__ __launch_bounds__(512, 2) void materialize_mfma8_kernel(MaterializeArgs a, int total_rows) {
    constexpr int MI = BM / 32;              // 16-row token blocks per wave
    constexpr int LRA = BM / 32;             // 16-byte pieces per thread and step: token tile
    constexpr int LRB = D / 32;              //                                    weight tile
    constexpr int A_ELEMS = BM * STR8, B_ELEMS = D * STR8;
    __shared__ __attribute__((aligned(16))) uint16_t tiles[2 * (A_ELEMS + B_ELEMS)];
    static_assert(MI == 2, "the two wave groups split the token blocks of a wave in the epilogue");
    static_assert(sizeof(float) * 8 * (MI / 2) * 4 * 64 * 4 <= sizeof(uint16_t) * 2 * (A_ELEMS + B_ELEMS), "exchange buffer");

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int kg = wave >> 2, wm = (wave >> 1) & 1, wn = wave & 1;
    const int kv = blockIdx.x / a.Hkv, head = blockIdx.x % a.Hkv;
    const int row0 = blockIdx.y * BM;

    const uint16_t* X = reinterpret_cast<const uint16_t*>(a.hidden);
    const uint16_t* W = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) + (size_t)head * D * a.Hd;

    // global -> LDS staging: thread t moves 16 bytes of rows t/16 + 32i, columns 8*(t%16)
    const int ld_row = tid >> 4, ld_col = (tid & 15) * 8;
    const uint16_t* xg[LRA];
    const uint16_t* wg[LRB];
#pragma unroll
    for (int i = 0; i < LRA; ++i) {
        const int r = min(row0 + ld_row + 32 * i, total_rows - 1);       // rows past the end repeat the last
        xg[i] = X + (size_t)r * a.Hd + ld_col;
    }
#pragma unroll
    for (int i = 0; i < LRB; ++i) wg[i] = W + (size_t)(ld_row + 32 * i) * a.Hd + ld_col;

    constexpr int NS = 4;
    struct Stage { uint4 x[LRA], w[LRB]; };
    Stage st[NS];
    const int nk = a.Hd / BK8;
    auto load_global = [&](Stage& g, int ks) {
        const int k0 = min(ks, nk - 1) * BK8;
#pragma unroll
        for (int i = 0; i < LRA; ++i) g.x[i] = ldg16(xg[i] + k0);
#pragma unroll
        for (int i = 0; i < LRB; ++i) g.w[i] = ldg16(wg[i] + k0);
    };
    auto a_tile = [&](int buf) { return tiles + buf * (A_ELEMS + B_ELEMS); };
    auto b_tile = [&](int buf) { return tiles + buf * (A_ELEMS + B_ELEMS) + A_ELEMS; };
    auto store_lds = [&](int buf, const Stage& g) {
#pragma unroll
        for (int i = 0; i < LRA; ++i)
            *reinterpret_cast<uint4*>(a_tile(buf) + (ld_row + 32 * i) * STR8 + ld_col) = g.x[i];
#pragma unroll
        for (int i = 0; i < LRB; ++i)
            *reinterpret_cast<uint4*>(b_tile(buf) + (ld_row + 32 * i) * STR8 + ld_col) = g.w[i];
    };

    f32x4 acc[MI][4];           // [token block mi][feature block: 2wn, 2wn+1, 2wn+4, 2wn+5]
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int buf) {
        const uint16_t* At = a_tile(buf) + (16 * MI * wm + c16) * STR8 + 64 * kg + 8 * g4;
        const uint16_t* Bt = b_tile(buf) + c16 * STR8 + 64 * kg + 8 * g4;
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            bf16x8 av[MI], bv[4];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                av[mi] = *reinterpret_cast<const bf16x8*>(At + 16 * mi * STR8 + 32 * k2);
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const int tn = 2 * wn + (ni & 1) + 4 * (ni >> 1);
                bv[ni] = *reinterpret_cast<const bf16x8*>(Bt + 16 * tn * STR8 + 32 * k2);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
        }
    };

#pragma unroll
    for (int i = 0; i < NS - 1; ++i) load_global(st[i], i);
    store_lds(0, st[0]);
    lds_barrier();
    int ks = 0;
    auto step = [&](auto stage_tag) {
        constexpr int S = decltype(stage_tag)::value;
        load_global(st[(S + NS - 1) % NS], ks + NS - 1);
        if (ks < nk) compute(ks & 1);
        store_lds((ks + 1) & 1, st[(S + 1) % NS]);
        lds_barrier();
        ++ks;
    };
    do {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
    } while (ks < nk);

    // the two groups' sums meet: group g keeps token blocks [g * MI/2, (g+1) * MI/2) and hands
    // the others to its partner wave (same wm, wn; the tiles are dead after the last barrier)
    constexpr int MH = MI / 2;
    float4* xch = reinterpret_cast<float4*>(tiles);
    __syncthreads();
#pragma unroll
    for (int m = 0; m < MH; ++m)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const f32x4 v = acc[(1 - kg) * MH + m][ni];
            xch[((wave * MH + m) * 4 + ni) * 64 + lane] = make_float4(v[0], v[1], v[2], v[3]);
        }
    __syncthreads();
    // epilogue: lane holds tokens 16*MI*wm + 16mi + 4*g4 + i, features 16*tn + c16
    uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
#pragma unroll
    for (int m = 0; m < MH; ++m) {
        const int mi = kg * MH + m;
        f32x4 sum[4];
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const float4 o = xch[(((wave ^ 4) * MH + m) * 4 + ni) * 64 + lane];
            sum[ni] = acc[mi][ni];
            sum[ni][0] += o.x; sum[ni][1] += o.y; sum[ni][2] += o.z; sum[ni][3] += o.w;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const RowDest d = resolve_row(a, row0 + 16 * MI * wm + 16 * mi + 4 * g4 + i);
            if (!d.valid) continue;
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const int j = 16 * (2 * wn + p) + c16;           // rotary pair index, features j and j + 64
                float lo = sum[p][i], hi = sum[p + 2][i];
                if (kv == 0) {
                    float c, s;
                    rope_cs(a.rope[j], d.pos, c, s);
                    const float k0 = lo * c - hi * s;
                    const float k1 = lo * s + hi * c;
                    lo = k0; hi = k1;
                }
                out[d.elem_off + j] = f32_to_bf16_rne(lo);
                out[d.elem_off + j + 64] = f32_to_bf16_rne(hi);
            }
        }
    }
}

// ---- skinny form: 16 .. 255 token rows (a question, a decode step of a large batch) ----------
// (The form for hidden sizes that are a multiple of 512 but not of 1024; multiples of 1024 take
// the staged form below.)
// Too few rows for the tiled GEMM to fill the chip (64 rows make 16 tiles).  Here a workgroup owns
// up to 64 rows x 16 rotary pairs (features 16g .. 16g+15 and their partners 64 further) of one
// head of K or of V, and its eight waves split the HIDDEN axis: each wave multiplies its slice
// with operands loaded straight from global memory in matrix-core layout (tokens as A rows,
// weight rows as B columns; 16 bytes per lane, no LDS staging: the weights are read once, the
// few token rows come from the caches), the eight partial tiles meet in LDS, and the rotation
// and the single rounding to bf16 follow.  Grid: 64 x row tiles workgroups of 8 waves.
template <int MI>
__global__ __launch_bounds__(512) void materialize_skinny_kernel(MaterializeArgs a, int total_rows) {
    constexpr int NWV = 8, CH = 2;                      // waves; matrix-core steps per staged chunk (fixed by the lane layout below)
    constexpr int TM = 16 * MI;
    __shared__ float red[NWV][TM][33];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int pg = blockIdx.x & 3, head = (blockIdx.x >> 2) % a.Hkv, kv = (blockIdx.x >> 2) / a.Hkv;
    const int row0 = blockIdx.y * TM;
    const int kslice = a.Hd / NWV;                      // a multiple of 32 * CH (checked by the launcher)
    const int n_chunks = kslice / (32 * CH);

    // Columns: a chunk is 64 columns per wave; lane (c16, g4) takes the 16 consecutive columns
    // 16 g4 .. 16 g4 + 15 of its row as two adjacent 16-byte loads, the first for one matrix-core
    // step and the second for the next (the contraction order is free as long as tokens and
    // weights agree), so that the four lanes of a row consume one whole 128-byte line at once
    // instead of half of it now and half a step later.  The eight waves take adjacent 64-column
    // pieces: together they read 1 KB of every row per chunk.
    const uint16_t* W = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) +
                        ((size_t)head * D + 16 * pg + c16) * a.Hd + 64 * wave + 16 * g4;
    const uint16_t* Whi = W + (size_t)(D / 2) * a.Hd;
    const uint16_t* X = reinterpret_cast<const uint16_t*>(a.hidden) + 64 * wave + 16 * g4;
    const uint16_t* xr[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) xr[mi] = X + (size_t)min(row0 + 16 * mi + c16, total_rows - 1) * a.Hd;

    // a thread's output column in the epilogue is fixed (16 pg + tid % 16): its rotary entry is
    // requested now, not after the reduction
    const RopeEntry rope_e = a.rope[16 * pg + (tid & 15)];

    struct Chunk { uint4 x[MI][CH], wl[CH], wh[CH]; };
    auto load = [&](Chunk& c, int ci) {
        const int off = min(ci, n_chunks - 1) * (32 * CH * NWV);
#pragma unroll
        for (int s = 0; s < CH; ++s) {
            c.wl[s] = ldg16(W + off + 8 * s);
            c.wh[s] = ldg16(Whi + off + 8 * s);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) c.x[mi][s] = ldg16(xr[mi] + off + 8 * s);
        }
    };
    f32x4 acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) { acc[mi][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[mi][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    auto mma = [&](const Chunk& c) {
#pragma unroll
        for (int s = 0; s < CH; ++s)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const bf16x8 xa = __builtin_bit_cast(bf16x8, c.x[mi][s]);
                acc[mi][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, __builtin_bit_cast(bf16x8, c.wl[s]), acc[mi][0], 0, 0, 0);
                acc[mi][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, __builtin_bit_cast(bf16x8, c.wh[s]), acc[mi][1], 0, 0, 0);
            }
    };
    // NCH chunks in flight; loads carry no branch (past the end they repeat the last chunk) and
    // the loop has one exit, so the compiler counts the loads in flight exactly
    {
        constexpr int NCH = MI == 1 ? 4 : 2;
        Chunk c[NCH];
#pragma unroll
        for (int i = 0; i < NCH; ++i) load(c[i], i);
        int ci = 0;
        do {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                if (ci + i < n_chunks) mma(c[i]);
                load(c[i], ci + i + NCH);
            }
            ci += NCH;
        } while (ci < n_chunks);
    }

    // lane holds tokens 16mi + 4*g4 + i, feature c16 of the low (h = 0) or high (h = 1) half
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][16 * mi + 4 * g4 + i][16 * h + c16] = acc[mi][h][i];
    __syncthreads();

    uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
    for (int idx = tid; idx < TM * 16; idx += NWV * 64) {
        const int t = idx >> 4, p = idx & 15;
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) { lo += red[w][t][p]; hi += red[w][t][16 + p]; }
        const RowDest d = resolve_row(a, row0 + t);
        if (!d.valid) continue;
        const int j = 16 * pg + p;
        if (kv == 0) {
            float c, s;
            rope_cs(rope_e, d.pos, c, s);
            const float k0 = lo * c - hi * s;
            const float k1 = lo * s + hi * c;
            lo = k0; hi = k1;
        }
        out[d.elem_off + j] = f32_to_bf16_rne(lo);
        out[d.elem_off + j + 64] = f32_to_bf16_rne(hi);
    }
}


// ---- skinny form with coalesced loads ---------------------------------------------------------
// The kernel above loads operands straight into matrix-core layout: consecutive lanes then sit on
// sixteen different rows, every lane's 16 bytes is a request of its own to the vector cache, and
// the launch is bound by that request rate (64 rows, hidden 4096: 98 MB in 17 us).  Here a wave
// loads its slice of the hidden axis row-wise instead - sixteen consecutive lanes take 256
// consecutive bytes of one row - parks the rows in a private LDS region (272-byte rows: sixteen
// lanes write one whole row, sixteen lanes read 16 bytes of sixteen different rows, both without a
// bank conflict) and reads them back in operand layout.  The region belongs to one wave: no
// workgroup barrier in the loop.  Same tile, same split of the hidden axis, same epilogue.
template <int MI, int NB>
__global__ __launch_bounds__(512) void materialize_skinny_staged_kernel(MaterializeArgs a, int total_rows) {
    constexpr int NWV = 8, SC = 128;                    // waves; hidden columns per wave and round
    constexpr int TM = 16 * MI;
    constexpr int NR = 32 + TM;                         // rows staged per round: 16 + 16 weight rows, TM token rows
    constexpr int NL = NR / 4;                          // 16-byte loads per lane and round (a load covers 4 rows)
    constexpr int RS = SC + 8;                          // bf16 per staged row
    constexpr int STAGE_BYTES = NWV * NR * RS * 2, RED_BYTES = NWV * TM * 33 * 4;
    __shared__ __attribute__((aligned(16))) char smem[STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int pg = blockIdx.x & 3, head = (blockIdx.x >> 2) % a.Hkv, kv = (blockIdx.x >> 2) / a.Hkv;
    const int row0 = blockIdx.y * TM;
    const int kslice = a.Hd / NWV;                      // a multiple of SC (checked by the launcher)
    const int n_rounds = kslice / SC;

    // the epilogue's row and rotary entry of this thread are fixed: asked for now, not after the sums
    static_assert(TM * 16 <= NWV * 64, "one output pair per thread");
    const int et = tid >> 4, ep = tid & 15;
    const RopeEntry rope_e = a.rope[16 * pg + ep];
    RowDest edest = resolve_row(a, row0 + min(et, TM - 1));
    if (et >= TM) edest.valid = false;

    // load i of a round: row 4 i + lane / 16 of the staged rows, 16 bytes at column 8 (lane % 16)
    const int lr = lane >> 4, lc = 8 * (lane & 15);
    const size_t col0 = (size_t)wave * kslice + lc;
    const uint16_t* wbase = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) + ((size_t)head * D + 16 * pg + lr) * a.Hd + col0;
    const uint16_t* xp[MI * 4];
#pragma unroll
    for (int i = 0; i < MI * 4; ++i)
        xp[i] = reinterpret_cast<const uint16_t*>(a.hidden) + (size_t)min(row0 + 4 * i + lr, total_rows - 1) * a.Hd + col0;
    auto load = [&](uint4 (&b)[NL], int r) {
        const int off = min(r, n_rounds - 1) * SC;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            b[i] = ldg16(wbase + (size_t)(4 * i) * a.Hd + off);
            b[4 + i] = ldg16(wbase + (size_t)(D / 2 + 4 * i) * a.Hd + off);
        }
#pragma unroll
        for (int i = 0; i < MI * 4; ++i) b[8 + i] = ldg16(xp[i] + off);
    };

    uint16_t* const st = reinterpret_cast<uint16_t*>(smem) + (size_t)wave * NR * RS;
    f32x4 acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) { acc[mi][0] = f32x4{0.f, 0.f, 0.f, 0.f}; acc[mi][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    auto process = [&](const uint4 (&b)[NL]) {
        __builtin_amdgcn_wave_barrier();                // the last round's reads stay ahead of these writes
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<uint4*>(st + (4 * i + lr) * RS + lc) = b[i];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < SC / 32; ++j) {
            const bf16x8 wl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(st + c16 * RS + 32 * j + 8 * g4));
            const bf16x8 wh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(st + (16 + c16) * RS + 32 * j + 8 * g4));
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const bf16x8 xa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(st + (32 + 16 * mi + c16) * RS + 32 * j + 8 * g4));
                acc[mi][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wl, acc[mi][0], 0, 0, 0);
                acc[mi][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wh, acc[mi][1], 0, 0, 0);
            }
        }
    };
    // NB rounds of loads in flight; no load under a branch (the launcher sees to it that the rounds
    // are a multiple of NB), the last NB rounds are consumed without asking for more
    {
        uint4 b[NB][NL];
#pragma unroll
        for (int i = 0; i < NB; ++i) load(b[i], i);
        for (int r = NB; r < n_rounds; r += NB) {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                process(b[i]);
                load(b[i], r + i);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) process(b[i]);
    }

    // the eight partial tiles meet in LDS (over the staging rows, once every wave is done with its own)
    __syncthreads();
    float (*red)[TM][33] = reinterpret_cast<float (*)[TM][33]>(smem);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][16 * mi + 4 * g4 + i][16 * h + c16] = acc[mi][h][i];
    __syncthreads();

    uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
    if (edest.valid) {
        const RowDest d = edest;
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) { lo += red[w][et][ep]; hi += red[w][et][16 + ep]; }
        const int j = 16 * pg + ep;
        if (kv == 0) {
            float c, s;
            rope_cs(rope_e, d.pos, c, s);
            const float k0 = lo * c - hi * s;
            const float k1 = lo * s + hi * c;
            lo = k0; hi = k1;
        }
        out[d.elem_off + j] = f32_to_bf16_rne(lo);
        out[d.elem_off + j + 64] = f32_to_bf16_rne(hi);
    }
}

}  // namespace

bool materialize_mfma_supported(const MaterializeArgs& a, int dtype, int total_rows) {
    return dtype == MATKV_BF16 && a.D == 128 && (a.Hd % BK) == 0 && total_rows >= 16;
}

// Skinny forms: measured ahead of the tiled GEMM below a few hundred rows, where the GEMM's grid
// leaves most compute units idle.  The staged form (hidden a multiple of 1024), us per launch at
// hidden 4096 / 8192 against the form with direct operand loads: 64 rows 8.1 / 13.8 (17.2 / -),
// 128 rows 10.6 / 17.4, 255 rows 18.8 / 30.1 (33.9 / 61.6); against the tiled GEMM: 384 rows
// 27.1 / 44.6 (33.1 / 59.0), 512 rows 35.3 / 57.3 (33.2 / 60.5), 768 rows 50.6 / 80.2 (33.8 / 61.6).
constexpr int kSkinnyMaxRows = 256;
constexpr int kStagedMaxRows = 448;

hipError_t launch_materialize_mfma(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    const bool staged = (a.Hd % 1024) == 0;
    if ((a.Hd % 512) == 0 && (total_rows < kSkinnyMaxRows || (staged && (total_rows <= kStagedMaxRows || (total_rows <= 512 && a.Hd >= 8192))))) {
        const dim3 block(512);
        const int gx = 2 * a.Hkv * 4;
        if (staged) {
            // rows staged through LDS: 16-row tiles up to 64 rows (64 x 4 workgroups fill the chip),
            // 32-row tiles beyond (half the workgroups, the weights re-read half as often)
            const int rounds = a.Hd / 1024;             // per wave: an eighth of the hidden axis, 128 columns a round
            const bool mi2 = total_rows > 64;
            const dim3 grid(gx, mi2 ? (total_rows + 31) / 32 : (total_rows + 15) / 16);
            if (rounds % 2 == 0) {
                if (mi2) hipLaunchKernelGGL((materialize_skinny_staged_kernel<2, 2>), grid, block, 0, s, a, total_rows);
                else     hipLaunchKernelGGL((materialize_skinny_staged_kernel<1, 2>), grid, block, 0, s, a, total_rows);
            } else {
                if (mi2) hipLaunchKernelGGL((materialize_skinny_staged_kernel<2, 1>), grid, block, 0, s, a, total_rows);
                else     hipLaunchKernelGGL((materialize_skinny_staged_kernel<1, 1>), grid, block, 0, s, a, total_rows);
            }
            return hipGetLastError();
        }
        // 16-row tiles keep every compute unit busy from 64 rows on (64 x 4 workgroups) and leave
        // registers for four chunks of loads in flight; from 512 workgroups on, 32-row tiles halve
        // the re-reading of the weights
        if (total_rows <= 128) hipLaunchKernelGGL(materialize_skinny_kernel<1>, dim3(gx, (total_rows + 15) / 16), block, 0, s, a, total_rows);
        else                   hipLaunchKernelGGL(materialize_skinny_kernel<2>, dim3(gx, (total_rows + 31) / 32), block, 0, s, a, total_rows);
        return hipGetLastError();
    }
    // Measured (8 KV heads, TFLOP/s at hidden 4096 / 8192): the launch is bound by what the L2 can
    // hand to the compute units (64 x 128 tiles re-read every operand 16 times: 454 MB for a
    // 1000-token chunk at hidden 4096, 81 % of it L2 hits, about 12 TB/s), so larger tiles win as
    // soon as there are enough of them: 128-row tiles 715 / 765 at 4096 rows and 721 / 817 at 8192,
    // against 549 / 610 and 585 / 666 with 64-row tiles.  While 64-row tiles make no more
    // workgroups than there are compute units, the eight-wave form of the same tile is ahead
    // (1000 rows: 444 / 519 against 394 / 440); with more, it holds one workgroup per compute unit
    // where the four-wave form holds two or three, and falls behind (1206 rows: 295 against 335).
    const int wgs64 = 2 * a.Hkv * ((total_rows + 63) / 64);
    if ((a.Hd % BK8) == 0 && wgs64 <= 256) {
        hipLaunchKernelGGL(materialize_mfma8_kernel<64>, dim3(2 * a.Hkv, (total_rows + 63) / 64), dim3(512), 0, s, a, total_rows);
        return hipGetLastError();
    }
    const dim3 block(256);
    if (2 * a.Hkv * ((total_rows + 127) / 128) >= 256)
        hipLaunchKernelGGL(materialize_mfma_kernel<128>, dim3(2 * a.Hkv, (total_rows + 127) / 128), block, 0, s, a, total_rows);
    else
        hipLaunchKernelGGL(materialize_mfma_kernel<64>, dim3(2 * a.Hkv, (total_rows + 63) / 64), block, 0, s, a, total_rows);
    return hipGetLastError();
}

}  // namespace matkv
