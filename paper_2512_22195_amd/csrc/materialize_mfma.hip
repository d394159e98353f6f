// K/V materialization of one layer as a matrix-core GEMM with the rotary embedding in the
// epilogue (paper Section III-B steps 2-3, cut to the K/V projection):
//   [T, Hd] x [2*Hkv*D, Hd]^T  ->  K = RoPE(X Wk^T, pos), V = X Wv^T,   bf16, D = 128.
// Both operands are contiguous along the contraction (hidden) axis, which is what the
// matrix-core operand layout wants: a lane's 8 consecutive bf16 of one row.
//
// Three forms by row count: the tiled GEMM (128 x 128 tiles, below), and two skinny forms for a
// few hundred rows at most (a question, a decode step of a large batch), whose eight waves split
// the hidden axis.  In all of them the two features of a rotary pair sit in the same lane, so the
// rotation is lane-local on the fp32 accumulators, and values are rounded to bf16 once, on store.
#include <type_traits>

#include "device_util.h"

namespace matkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128, BK = 64;             // BK: hidden columns per step of the tiled GEMM

using dev::ldg16;
using dev::f32_to_bf16_rne;

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

// ---- tiled GEMM: 128 x 128 tiles, the hidden axis split over SK workgroups ---------------------
// A workgroup owns 128 tokens x one head of K or of V (128 features: both halves of every rotary
// pair); 64 hidden columns per step through double-buffered LDS tiles fed from four rotating
// register stages (loads carry no branch - past the end they repeat the last step - and the
// loop has one exit, so the compiler counts the loads in flight instead of draining them).
// LDS rows are 160 bytes: the 16-byte operand reads of 16 rows measured 4.5 cycles per
// instruction with them, 8.6 with 144.
// The launch is bound by what the L2s hand to the compute units, every workgroup reading its
// token rows and its weight rows over the whole hidden axis: 64 x 128 tiles (the earlier form)
// moved 393 MB for a 1000-token chunk at hidden 4096 against 25 MB of distinct operands, these
// tiles a third less.  Where 128 x 128 tiles alone would leave half of the chip idle (up to 1024
// rows with 8 KV heads), two workgroups share a tile, each over half of the hidden axis: both
// leave their fp32 partial in the workspace (agent-scope stores), arrive at the tile's counter,
// and the one that arrives second adds the other's partial to its own and runs the epilogue.
// Measured, us per launch at hidden 4096 / 8192 (8 KV heads), against the 64 x 128 forms this
// replaced (eight waves up to 1000 rows, four waves beyond): 512 rows 30.6 / - (33.1 / -),
// 1000 rows 34.0 / 57.9 (35.9 / 67.6), 1206 rows 46.9 / 88.7 (56.7 / 103.4), 2048 rows
// 50.2 / 96.0 (62.8 / 111.4), 8192 rows 173 / 315 (185 / 327).
// The work is split between waves.  In a first form every wave did everything - requested the
// next operands, moved a tile into LDS, read operands back, multiplied - and the barrier kept
// all eight in the same phase, so a step lasted as long as its phases added up.  Now waves 4-7
// only move data (global -> registers -> LDS, four steps of loads in flight) and waves 0-3, one
// per SIMD, only read operands and multiply (2 x 2 waves, 64 tokens x the 16-feature blocks
// {2wn, 2wn+1, 2wn+4, 2wn+5} each), so the load path and the LDS writes of step i + 1 run beside
// the matrix work of step i (1206 rows at hidden 4096 / 8192: 48.9 / 90.0 -> 45.8 / 80.0 us, 2048
// rows 52.1 / 95.4 -> 48.5 / 86.0; 1000 rows and 8192 rows unchanged).
template <int SK>
__global__ __launch_bounds__(512, 2) void materialize_mfma128_kernel(MaterializeArgs a, int total_rows) {
    constexpr int BM = 128, BKS = BK, STR = BKS + 16;
    constexpr int A_ELEMS = BM * STR, B_ELEMS = D * STR;
    __shared__ __attribute__((aligned(16))) uint16_t tiles[2 * (A_ELEMS + B_ELEMS)];
    RowDest* const sm_dest = reinterpret_cast<RowDest*>(tiles);
    int* const sm_last = reinterpret_cast<int*>(sm_dest + BM);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int kv = blockIdx.x / a.Hkv, head = blockIdx.x % a.Hkv;
    const int row0 = blockIdx.y * BM;
    const int part = blockIdx.z;
    const int nk = a.Hd / (BKS * SK);                   // steps of this workgroup
    const size_t kbase = (size_t)part * nk * BKS;
    auto a_tile = [&](int buf) { return tiles + buf * (A_ELEMS + B_ELEMS); };
    auto b_tile = [&](int buf) { return tiles + buf * (A_ELEMS + B_ELEMS) + A_ELEMS; };

    const int wm = (wave >> 1) & 1, wn = wave & 1;      // of the multiplying waves
    f32x4 acc[4][4];            // [token block 4 wm + mi][feature block 2wn, 2wn+1, 2wn+4, 2wn+5]
    // where the tile's rows go and their rotary positions: looked up once per row, now
    const RowDest my_dest = resolve_row(a, row0 + min(tid, BM - 1));

    if (wave >= 4) {
        // ---- moving waves: thread t of 256 moves 16 bytes of rows t/8 + 32i, columns 8*(t%8) ----
        const int lt = tid - 256;
        const int ld_row = lt >> 3, ld_col = (lt & 7) * 8;
        const uint16_t* X = reinterpret_cast<const uint16_t*>(a.hidden) + kbase;
        const uint16_t* W = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) + (size_t)head * D * a.Hd + kbase;
        const uint16_t* xg[4];
        const uint16_t* wg[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = min(row0 + ld_row + 32 * i, total_rows - 1);   // rows past the end repeat the last
            xg[i] = X + (size_t)r * a.Hd + ld_col;
            wg[i] = W + (size_t)(ld_row + 32 * i) * a.Hd + ld_col;
        }
        constexpr int NS = 4;
        struct Stage { uint4 x[4], w[4]; };
        Stage st[NS];
        auto load_global = [&](Stage& g, int ks) {
            const int k0 = min(ks, nk - 1) * BKS;
#pragma unroll
            for (int i = 0; i < 4; ++i) { g.x[i] = ldg16(xg[i] + k0); g.w[i] = ldg16(wg[i] + k0); }
        };
        auto store_lds = [&](int buf, const Stage& g) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                *reinterpret_cast<uint4*>(a_tile(buf) + (ld_row + 32 * i) * STR + ld_col) = g.x[i];
                *reinterpret_cast<uint4*>(b_tile(buf) + (ld_row + 32 * i) * STR + ld_col) = g.w[i];
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
    } else {
        // ---- multiplying waves ----
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) acc[mi][ni] = f32x4{0.f, 0.f, 0.f, 0.f};
        auto compute = [&](int buf) {
            const uint16_t* At = a_tile(buf) + (64 * wm + c16) * STR + 8 * g4;
            const uint16_t* Bt = b_tile(buf) + c16 * STR + 8 * g4;
#pragma unroll
            for (int k2 = 0; k2 < BKS / 32; ++k2) {
                bf16x8 av[4], bv[4];
#pragma unroll
                for (int mi = 0; mi < 4; ++mi) av[mi] = *reinterpret_cast<const bf16x8*>(At + 16 * mi * STR + 32 * k2);
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) {
                    const int tn = 2 * wn + (ni & 1) + 4 * (ni >> 1);
                    bv[ni] = *reinterpret_cast<const bf16x8*>(Bt + 16 * tn * STR + 32 * k2);
                }
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 4; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
            }
        };
        lds_barrier();                                  // tile 0 is in place
        const int n_bar = (nk + 3) / 4 * 4;             // the moving waves run whole rounds of four steps
        for (int ks = 0; ks < n_bar; ++ks) {
            if (ks < nk) compute(ks & 1);
            lds_barrier();
        }
    }
    if (tid < BM) sm_dest[tid] = my_dest;               // (the loop's last barrier is behind every read of the tiles)
    __syncthreads();

    if constexpr (SK > 1) {
        static_assert(SK == 2, "two workgroups per tile");
        const int tile = blockIdx.y * gridDim.x + blockIdx.x;
        if (wave < 4) {
            float* mine = a.ws_partials + ((size_t)(tile * SK + part) * 4 + wave) * (32 * 128) + lane * 2;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) {
                    dev::st_agent2(mine + ((mi * 4 + ni) * 2 + 0) * 128, acc[mi][ni][0], acc[mi][ni][1]);
                    dev::st_agent2(mine + ((mi * 4 + ni) * 2 + 1) * 128, acc[mi][ni][2], acc[mi][ni][3]);
                }
        }
        int32_t* counter = a.ws_counters + (size_t)tile * kDecodeCounterStride;
        if (!dev::arrive_at(counter, SK, sm_last)) return;
        dev::reset_counter_at(counter);
        if (wave < 4) {
            const float* theirs = a.ws_partials + ((size_t)(tile * SK + (part ^ 1)) * 4 + wave) * (32 * 128) + lane * 2;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi) {
                float2 o[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) o[r] = dev::ld_agent2(theirs + (mi * 8 + r) * 128);
#pragma unroll
                for (int ni = 0; ni < 4; ++ni) {
                    acc[mi][ni][0] += o[2 * ni].x; acc[mi][ni][1] += o[2 * ni].y;
                    acc[mi][ni][2] += o[2 * ni + 1].x; acc[mi][ni][3] += o[2 * ni + 1].y;
                }
            }
        }
    }
    if (wave >= 4) return;

    // epilogue: lane holds tokens 64 wm + 16 mi + 4 g4 + i, features 16 tn + c16
    uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const RowDest d = sm_dest[64 * wm + 16 * mi + 4 * g4 + i];
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


// ---- a handful of rows (a decode step) on the staged form ---------------------------------------
// The same scheme cut finer, so that a launch with 1 .. 16 token rows still has 256 workgroups: a
// workgroup owns NP rotary pairs (2 NP weight rows: NP "low" features and their partners) and TMR
// token rows, which together fill part of one 16 x 16 matrix tile - lanes beyond repeat a row and
// their results are dropped.  Eight waves split the hidden axis as above; only the TMR real token
// rows are staged.
template <int NP, int TMR, int NB>
__global__ __launch_bounds__(512) void materialize_fewrows_kernel(MaterializeArgs a, int total_rows) {
    constexpr int NWV = 8, SC = 128;                    // waves; hidden columns per wave and round
    constexpr int NR = 2 * NP + TMR;                    // rows staged per round
    static_assert(NP % 4 == 0 && TMR % 4 == 0 && 2 * NP <= 16 && TMR <= 16, "whole loads of four rows; one matrix tile");
    constexpr int NL = NR / 4;                          // 16-byte loads per lane and round
    constexpr int RS = SC + 8;                          // bf16 per staged row
    constexpr int STAGE_BYTES = NWV * NR * RS * 2, RED_BYTES = NWV * TMR * (2 * NP + 1) * 4;
    __shared__ __attribute__((aligned(16))) char smem[STAGE_BYTES > RED_BYTES ? STAGE_BYTES : RED_BYTES];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c16 = lane & 15, g4 = lane >> 4;
    constexpr int GPH = (D / 2) / NP;                   // pair groups per head
    const int pg = blockIdx.x % GPH, head = (blockIdx.x / GPH) % a.Hkv, kv = (blockIdx.x / GPH) / a.Hkv;
    const int row0 = blockIdx.y * TMR;
    const int kslice = a.Hd / NWV;                      // a multiple of SC (checked by the launcher)
    const int n_rounds = kslice / SC;

    // the epilogue's row and rotary entry of this thread are fixed: asked for now, not after the sums
    const int et = tid / NP, ep = tid % NP;
    const RopeEntry rope_e = a.rope[NP * pg + ep];
    RowDest edest = resolve_row(a, row0 + min(et, TMR - 1));
    if (et >= TMR) edest.valid = false;

    // load i of a round: staged row 4 i + lane / 16, 16 bytes at column 8 (lane % 16)
    const int lr = lane >> 4, lc = 8 * (lane & 15);
    const size_t col0 = (size_t)wave * kslice + lc;
    const uint16_t* wbase = reinterpret_cast<const uint16_t*>(kv == 0 ? a.w_k : a.w_v) + ((size_t)head * D + NP * pg + lr) * a.Hd + col0;
    const uint16_t* xp[TMR / 4];
#pragma unroll
    for (int i = 0; i < TMR / 4; ++i)
        xp[i] = reinterpret_cast<const uint16_t*>(a.hidden) + (size_t)min(row0 + 4 * i + lr, total_rows - 1) * a.Hd + col0;
    auto load = [&](uint4 (&b)[NL], int r) {
        const int off = min(r, n_rounds - 1) * SC;
#pragma unroll
        for (int i = 0; i < NP / 4; ++i) {
            b[i] = ldg16(wbase + (size_t)(4 * i) * a.Hd + off);
            b[NP / 4 + i] = ldg16(wbase + (size_t)(D / 2 + 4 * i) * a.Hd + off);
        }
#pragma unroll
        for (int i = 0; i < TMR / 4; ++i) b[NP / 2 + i] = ldg16(xp[i] + off);
    };

    uint16_t* const st = reinterpret_cast<uint16_t*>(smem) + (size_t)wave * NR * RS;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int brow = c16 < 2 * NP ? c16 : 0;            // weight row of this lane's column (columns beyond: dropped)
    const int arow = 2 * NP + min(c16, TMR - 1);        // token row of this lane's operand row
    auto process = [&](const uint4 (&b)[NL]) {
        __builtin_amdgcn_wave_barrier();                // the last round's reads stay ahead of these writes
#pragma unroll
        for (int i = 0; i < NL; ++i) *reinterpret_cast<uint4*>(st + (4 * i + lr) * RS + lc) = b[i];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < SC / 32; ++j) {
            const bf16x8 wv = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(st + brow * RS + 32 * j + 8 * g4));
            const bf16x8 xa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(st + arow * RS + 32 * j + 8 * g4));
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wv, acc, 0, 0, 0);
        }
    };
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
    float (*red)[TMR][2 * NP + 1] = reinterpret_cast<float (*)[TMR][2 * NP + 1]>(smem);
    // lane holds tokens 4 g4 + i, column c16
    if (c16 < 2 * NP)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * g4 + i < TMR) red[wave][4 * g4 + i][c16] = acc[i];
    __syncthreads();

    if (edest.valid) {
        float lo = 0.f, hi = 0.f;
#pragma unroll
        for (int w = 0; w < NWV; ++w) { lo += red[w][et][ep]; hi += red[w][et][NP + ep]; }
        const int j = NP * pg + ep;
        if (kv == 0) {
            float c, s;
            rope_cs(rope_e, edest.pos, c, s);
            const float k0 = lo * c - hi * s;
            const float k1 = lo * s + hi * c;
            lo = k0; hi = k1;
        }
        uint16_t* out = reinterpret_cast<uint16_t*>(kv == 0 ? a.k_out : a.v_out) + (size_t)head * a.token_stride * D;
        out[edest.elem_off + j] = f32_to_bf16_rne(lo);
        out[edest.elem_off + j + 64] = f32_to_bf16_rne(hi);
    }
}

template <int TMR>
hipError_t launch_fewrows_t(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    constexpr int NP = 4;
    const dim3 grid(2 * a.Hkv * (64 / NP), (total_rows + TMR - 1) / TMR), block(512);
    const int rounds = a.Hd / 1024;
    if (rounds % 4 == 0) hipLaunchKernelGGL((materialize_fewrows_kernel<NP, TMR, 4>), grid, block, 0, s, a, total_rows);
    else if (rounds % 2 == 0) hipLaunchKernelGGL((materialize_fewrows_kernel<NP, TMR, 2>), grid, block, 0, s, a, total_rows);
    else hipLaunchKernelGGL((materialize_fewrows_kernel<NP, TMR, 1>), grid, block, 0, s, a, total_rows);
    return hipGetLastError();
}

}  // namespace

bool materialize_fewrows_supported(const MaterializeArgs& a, int dtype, int total_rows) {
    return dtype == MATKV_BF16 && a.D == 128 && (a.Hd % 1024) == 0 && total_rows >= 1 && total_rows <= 16;
}
hipError_t launch_materialize_fewrows(const MaterializeArgs& a, int total_rows, hipStream_t s) {
    if (total_rows <= 4) return launch_fewrows_t<4>(a, total_rows, s);
    if (total_rows <= 8) return launch_fewrows_t<8>(a, total_rows, s);
    return launch_fewrows_t<16>(a, total_rows, s);
}

bool materialize_mfma_supported(const MaterializeArgs& a, int dtype, int total_rows) {
    return dtype == MATKV_BF16 && a.D == 128 && (a.Hd % BK) == 0 && total_rows >= 16;
}

// Skinny forms: measured ahead of the tiled GEMM below a few hundred rows, where the GEMM's grid
// leaves most compute units idle.  The staged form (hidden a multiple of 1024), us per launch at
// hidden 4096 / 8192 against the form with direct operand loads: 64 rows 8.1 / 13.8 (17.2 / -),
// 128 rows 10.6 / 17.4, 255 rows 18.8 / 30.1 (33.9 / 61.6); against the tiled GEMM: 384 rows
// 27.1 / 44.6 (about 30 / 58), 512 rows 35.3 / 57.3 (30.6 / 58), 768 rows 50.6 / 80.2 (about 33 / 58).
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
    // two workgroups per tile while that fills the chip at most once (and the workspace has room)
    const int tiles = 2 * a.Hkv * ((total_rows + 127) / 128);
    const bool room = a.ws_partials && (int64_t)tiles * 2 * 128 * 128 <= a.ws_partial_floats &&
                      (int64_t)tiles * kDecodeCounterStride <= a.ws_n_counters;
    if (tiles * 2 <= 256 && (a.Hd % (2 * BK)) == 0 && room)
        hipLaunchKernelGGL(materialize_mfma128_kernel<2>, dim3(2 * a.Hkv, (total_rows + 127) / 128, 2), dim3(512), 0, s, a, total_rows);
    else
        hipLaunchKernelGGL(materialize_mfma128_kernel<1>, dim3(2 * a.Hkv, (total_rows + 127) / 128, 1), dim3(512), 0, s, a, total_rows);
    return hipGetLastError();
}

}  // namespace matkv
