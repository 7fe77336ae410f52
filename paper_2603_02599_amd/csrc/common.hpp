// Shared device/host helpers of the SUN shared-decode library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/sun.h"

namespace sun {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kWave = 64;
constexpr int kPageTokens = 16;     // tokens per KV page
constexpr int kAttnChunk = 256;  // tokens per full split-K work item
constexpr int kAttnSmall = 64;   // tokens per small work item at the end of a request
// Length of a request's full chunks.  From 64 requests up it is kAttnChunk.  A smaller batch has too few
// chunks of that length to occupy the chip (and one wave walks a chunk step by step, a memory latency per
// step), so there the length is the power of two in [kAttnSmall, kAttnChunk] that gives about 2048 items over
// the whole batch if every request were like this one.  It depends on the request's own length, the batch
// size and the number of KV heads, never on the other requests, so a request's result does not depend on its
// batch-mates.
__host__ __device__ inline int attn_full_chunk(int n, int batch, int Hkv) {
    if (batch >= 64) return kAttnChunk;
    const long long target = (long long)n * Hkv * batch / 2048;
    int ch = kAttnSmall;
    while (2 * ch <= target && 2 * ch <= kAttnChunk) ch *= 2;
    return ch;
}
// All but the last full chunk's worth of tokens go into full chunks of length ch, the remaining
// 1 .. 2*ch-1 tokens into small chunks.
__host__ __device__ inline void attn_chunking(int n, int batch, int Hkv, int& n_full, int& n_small, int& ch) {
    ch = attn_full_chunk(n, batch, Hkv);
    const int f = n / ch;
    n_full = f > 1 ? f - 1 : 0;
    n_small = (n - n_full * ch + kAttnSmall - 1) / kAttnSmall;
}
constexpr int kGroup = 128;         // quantisation group along K (Appendix A.1)
constexpr int kMaxBatchTile = 256;  // rows one projection launch covers

// ---- bf16 <-> f32 (round to nearest even) ----
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

// ---- projection activations: "fragment-tiled" two-plane bf16 layout ----
// An fp32 activation x is carried into the matrix cores as two bf16 values, hi = bf16(x) and
// lo = bf16(x - hi) (16 significant bits together); the projection multiplies both planes with
// the same weight fragment and adds the two results.  Rounding activations to a single bf16
// would make the result depend on which way values near a rounding boundary fall, and a deep
// stack amplifies that noise beyond the parity tolerance.
// A [rows, K] is stored so that one staging step of the MFMA projection kernels is a linear
// copy into LDS and each 16-byte unit (8 consecutive k of one row) is one lane's A operand of a
// 32x32x16 MFMA.  With MB = number of 32-row blocks of real rows (1, 2, 4 or 8) the tiling has
// 2*MB blocks, plane p of row block r at block p*MB + r:
//   unit(p, b, k/8) = ((chunk * 8 + kk) * 2*MB + p*MB + b/32) * 64 + half * 32 + b%32
// with chunk = k / 128, g = (k % 128) / 8, half = g / 8, kk = g % 8.  Lane-half `half` of k-step
// kk of a 128-wide chunk therefore carries k = chunk*128 + half*64 + kk*8 .. +7; the packed
// weights use the same assignment, and any bijection is valid because the MFMA sums over k.
struct ATile {
    int MB;
};
__host__ __device__ __forceinline__ ATile atile_for_rows(int rows) {
    return ATile{rows <= 32 ? 1 : rows <= 64 ? 2 : rows <= 128 ? 4 : 8};
}
__host__ __device__ __forceinline__ size_t atile_unit(ATile t, int plane, int b, int k8) {
    const int chunk = k8 >> 4, g = k8 & 15;
    const int half = g >> 3, kk = g & 7;
    return ((size_t)(chunk * 8 + kk) * (2 * t.MB) + plane * t.MB + (b >> 5)) * 64 + half * 32 + (b & 31);
}
__host__ __device__ __forceinline__ size_t atile_elem(ATile t, int plane, int b, int k) {
    return atile_unit(t, plane, b, k >> 3) * 8 + (k & 7);
}
__host__ __device__ __forceinline__ size_t atile_bytes(ATile t, int K) { return (size_t)2 * t.MB * 32 * K * 2; }
// hi/lo split of one value; returns hi bits, lo bits via reference
__device__ __forceinline__ uint16_t split_bf16(float x, uint16_t& lo) {
    const uint16_t hi = f32_to_bf16_bits(x);
    lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
    return hi;
}

// ---- 4-bit projections: activations as 16-bit fixed point in two int8 planes ----
// The 4-bit codes are integers, so the quantised projections run on the int8 matrix cores with exact
// int32 sums (Eq. 8 evaluated on the integer grid; the scales are applied to the sums in fp32).  Per row
// and 128-wide group (the weights' group) an activation is x ~ sx * xi with sx = max|x| / kQMax and the
// integer xi = 256 * hi + lo, hi and lo in [-128, 127]: 16 bits below the group's largest value.  The
// producer of the activations also stores sx and sum_k xi (for the zero point) per row and group.
// Tile: 16-byte units of 16 consecutive k of one row and plane, ordered [group][k-step 0..3][plane]
// [32-row block][lane = half * 32 + row % 32] with k = group * 128 + half * 64 + step * 16 + (0..15):
// a unit is one lane's operand of a 32x32x32 int8 MFMA.
constexpr float kQMax = 32639.f;  // 127 * 256 + 127
__host__ __device__ __forceinline__ size_t qtile_unit(ATile t, int plane, int b, int k16) {
    const int c = k16 >> 3, g = k16 & 7, half = g >> 2, s = g & 3;
    return ((size_t)((c * 4 + s) * 2 + plane) * t.MB + (b >> 5)) * 64 + half * 32 + (b & 31);
}
// eight consecutive values of one row (k8 = index of the octet) -> their bytes in both planes; returns sum of xi
__device__ __forceinline__ int qtile_store8(uint8_t* tile, ATile t, int b, int k8, const float (&x)[8], float inv) {
    uint32_t hi[2] = {0u, 0u}, lo[2] = {0u, 0u};
    int sum = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int xi = (int)rintf(x[e] * inv);
        const int l = ((xi + 128) & 255) - 128, h = (xi - l) >> 8;
        sum += xi;
        hi[e >> 2] |= (uint32_t)(h & 255) << (8 * (e & 3));
        lo[e >> 2] |= (uint32_t)(l & 255) << (8 * (e & 3));
    }
    *reinterpret_cast<uint2*>(tile + qtile_unit(t, 0, b, k8 >> 1) * 16 + (k8 & 1) * 8) = uint2{hi[0], hi[1]};
    *reinterpret_cast<uint2*>(tile + qtile_unit(t, 1, b, k8 >> 1) * 16 + (k8 & 1) * 8) = uint2{lo[0], lo[1]};
    return sum;
}
// 1 / sx for a group whose largest magnitude is amax (an all-zero group maps to zeros with sx = 0)
__device__ __forceinline__ float qtile_inv(float amax) { return amax > 0.f ? kQMax / amax : 0.f; }

// 16-byte load of data that is read once and never again by this launch (the cached V of the attention kernel):
// streamed past the caches (the "nt" form of the load), which also leaves what the neighbouring kernels exchange
// in place.  Pays where an instruction reads long contiguous runs; see the attention kernel.
typedef uint32_t u32x4_s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_s load_stream(const u32x4_s* p) { return __builtin_nontemporal_load(p); }

// ---- wave reductions (all lanes receive the result; fixed order => deterministic) ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// ---- handles ----
struct KvPool {
    sun_model_cfg cfg;
    uint16_t* base;
    sun_kv_layout lay;
    int n_source_models;
    std::vector<int64_t> ingested;  // tokens ingested per source model (host side)
};

enum MatKind { MAT_NONE = 0, MAT_F32 = 1, MAT_BF16_PACKED = 2, MAT_W4_PACKED = 3, MAT_W4_LOGICAL = 4 };

// One projection matrix as the kernels consume it.
struct Mat {
    int kind = MAT_NONE;
    int N = 0, K = 0;          // logical out/in features (N counts gate+up rows for the fused pair)
    const void* w = nullptr;   // F32: row-major fp32; BF16_PACKED / W4_PACKED: packed codes
    const void* sz = nullptr;  // W4_PACKED: half2 (scale, zero) per (32-row block, group, row); or, with
                               // s_only, the fp16 scales alone, two groups per dword (zero point 8 everywhere)
    bool s_only = false;
    // W4_LOGICAL (fp32 activations): logical arrays, up to two stacked sources (gate, up)
    const uint8_t* q[3] = {nullptr, nullptr, nullptr};
    const uint16_t* s[3] = {nullptr, nullptr, nullptr};
    const uint16_t* z[3] = {nullptr, nullptr, nullptr};
    const void* wsrc[3] = {nullptr, nullptr, nullptr};  // F32: separate row-major sources
    int nsrc = 0;
    int src_rows[3] = {0, 0, 0};
};

struct LayerW {
    const void* g1;
    const void* g2;
    const void* qn = nullptr;  // head-norm gains [head_dim], only with cfg.qk_norm
    const void* kn = nullptr;
    const void *bq = nullptr, *bk = nullptr, *bv = nullptr;  // projection biases, only with cfg.qkv_bias
    Mat qkv, o, gu, down;
};

struct Weights {
    sun_model_cfg cfg;
    bool quant;
    const void* embed;
    const void* gf;
    Mat lm;
    LayerW* layers;
};

void set_error(const char* fmt, ...);

}  // namespace sun

#define SUN_HIP_CHECK(expr)                                                              \
    do {                                                                                 \
        hipError_t e_ = (expr);                                                          \
        if (e_ != hipSuccess) {                                                          \
            sun::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
            return SUN_ERR_HIP;                                                          \
        }                                                                                \
    } while (0)
