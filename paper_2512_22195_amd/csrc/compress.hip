// Compressed form of a materialized chunk blob (the paper names KV compression as its lever on
// storage cost and load time, Section III-C; the scheme is this library's): per (layer, K or V,
// KV head) one power-of-two scale s - the smallest with max|x| <= 448 s - and per element the
// E4M3 code (OCP FP8: 4 exponent bits of bias 7, 3 mantissa bits, no infinities, largest value
// 448) of x / s, rounded to nearest even by the hardware conversion.  x / s is exact in fp32, so
// the codes depend on nothing but the format.  HBM bound.  A head of up to 1024 tokens (256 KB)
// is held in the registers of its workgroup between the two passes - every load of the launch is
// requested before anything is consumed, and the blob is read once; longer heads are read twice
// (the second pass mostly from L2).  Written once at half the size.
#include "matkv_internal.h"

namespace matkv {
namespace {

constexpr int NT = 256;

__device__ __forceinline__ uint32_t max_mag2(uint32_t acc, uint32_t w) {
    // two bf16 per word: magnitudes order like their bit patterns
    return max(acc, max(w & 0x7fffu, (w >> 16) & 0x7fffu));
}

// Scale exponent k of a head whose largest magnitude has the bf16 pattern amax (s = 2^k).
__device__ __forceinline__ int scale_exponent(uint32_t amax) {
    // amax = f 2^E, f in [1, 2): 448 = 1.75 * 2^8, so s = 2^(E - 8) if f <= 1.75, else 2^(E - 7)
    if (amax == 0) return 0;
    const int E = (int)(amax >> 7) - 127, m7 = (int)(amax & 0x7f);
    return max(m7 <= 96 ? E - 8 : E - 7, -60);            // floor 2^-60 (a subnormal amax lands there too)
}
__device__ __forceinline__ uint2 encode8(const uint4& v, float inv) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(__uint_as_float(w[0] << 16) * inv, __uint_as_float(w[0] & 0xffff0000u) * inv, lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(__uint_as_float(w[1] << 16) * inv, __uint_as_float(w[1] & 0xffff0000u) * inv, lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(__uint_as_float(w[2] << 16) * inv, __uint_as_float(w[2] & 0xffff0000u) * inv, hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(__uint_as_float(w[3] << 16) * inv, __uint_as_float(w[3] & 0xffff0000u) * inv, hi, true);
    return make_uint2((uint32_t)lo, (uint32_t)hi);
}

__global__ __launch_bounds__(NT) void compress_kernel(const uint16_t* __restrict__ blob, uint8_t* __restrict__ out,
                                                      size_t head_elems, size_t scales_off) {
    const int kvh = blockIdx.x, kv = blockIdx.y, layer = blockIdx.z;
    const size_t head = ((size_t)layer * 2 + kv) * gridDim.x + kvh;
    const uint4* src = reinterpret_cast<const uint4*>(blob + head * head_elems);
    uint2* dst = reinterpret_cast<uint2*>(out + head * head_elems);
    const size_t n_vec = head_elems / 8;                  // head_dim is a multiple of 64

    uint32_t amax = 0;
    for (size_t i = threadIdx.x; i < n_vec; i += NT) {
        const uint4 v = src[i];
        amax = max_mag2(max_mag2(max_mag2(max_mag2(amax, v.x), v.y), v.z), v.w);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off));
    __shared__ uint32_t sm[NT / 64];
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = max(max(sm[0], sm[1]), max(sm[2], sm[3]));

    const int k = scale_exponent(amax);
    const float inv = __uint_as_float((uint32_t)(127 - k) << 23);
    if (threadIdx.x == 0)
        reinterpret_cast<float*>(out + scales_off)[head] = __uint_as_float((uint32_t)(127 + k) << 23);

    for (size_t i = threadIdx.x; i < n_vec; i += NT) {
        dst[i] = encode8(src[i], inv);
    }
}

// Heads of at most NV * 512 vectors of eight values: the whole head in registers.
constexpr int NTR = 512, NV = 32;
__global__ __launch_bounds__(NTR) void compress_resident_kernel(const uint16_t* __restrict__ blob, uint8_t* __restrict__ out,
                                                                size_t head_elems, size_t scales_off) {
    const int kvh = blockIdx.x, kv = blockIdx.y, layer = blockIdx.z;
    const size_t head = ((size_t)layer * 2 + kv) * gridDim.x + kvh;
    const uint4* src = reinterpret_cast<const uint4*>(blob + head * head_elems);
    uint2* dst = reinterpret_cast<uint2*>(out + head * head_elems);
    const int n_vec = (int)(head_elems / 8);              // at most NV * NTR (checked by the launcher)

    uint4 v[NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) v[u] = src[min(u * NTR + (int)threadIdx.x, n_vec - 1)];   // past the end: the last vector again
    uint32_t amax = 0;
#pragma unroll
    for (int u = 0; u < NV; ++u) amax = max_mag2(max_mag2(max_mag2(max_mag2(amax, v[u].x), v[u].y), v[u].z), v[u].w);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off));
    __shared__ uint32_t sm[NTR / 64];
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = sm[0];
#pragma unroll
    for (int w = 1; w < NTR / 64; ++w) amax = max(amax, sm[w]);

    const int k = scale_exponent(amax);
    const float inv = __uint_as_float((uint32_t)(127 - k) << 23);
    if (threadIdx.x == 0)
        reinterpret_cast<float*>(out + scales_off)[head] = __uint_as_float((uint32_t)(127 + k) << 23);
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int i = u * NTR + (int)threadIdx.x;
        if (i < n_vec) dst[i] = encode8(v[u], inv);
    }
}

}  // namespace

hipError_t launch_compress(const void* blob, void* out, int n_layers, int Hkv, int n_tokens, int D, hipStream_t s) {
    const size_t head_elems = (size_t)n_tokens * D;
    const size_t scales_off = ((size_t)n_layers * 2 * Hkv * head_elems + 15) & ~(size_t)15;
    if (head_elems / 8 <= (size_t)NV * NTR && head_elems >= 8)
        hipLaunchKernelGGL(compress_resident_kernel, dim3(Hkv, 2, n_layers), dim3(NTR), 0, s,
                           reinterpret_cast<const uint16_t*>(blob), reinterpret_cast<uint8_t*>(out), head_elems, scales_off);
    else
        hipLaunchKernelGGL(compress_kernel, dim3(Hkv, 2, n_layers), dim3(NT), 0, s,
                           reinterpret_cast<const uint16_t*>(blob), reinterpret_cast<uint8_t*>(out), head_elems, scales_off);
    return hipGetLastError();
}

}  // namespace matkv
