// Small kernels of the decode step (Eq. 3): embedding gather, residual + RMSNorm,
// rotary embedding + KV append (Eq. 4), SwiGLU (fp32 path), greedy argmax, and the
// layout helpers around the projection kernels.
#include "kernels.hpp"

namespace sun {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---------------- embedding: x[b] = E[token_b] ----------------
__global__ __launch_bounds__(256) void embed_kernel(const void* __restrict__ E, int is_bf16, int H, int V,
                                                    const int32_t* __restrict__ tokens, float* __restrict__ x) {
    const int b = blockIdx.x;
    int tok = tokens[b];
    tok = min(max(tok, 0), V - 1);  // ids are validated on the host under SUN_VALIDATE; never fault here
    for (int j = threadIdx.x; j < H; j += 256)
        x[(size_t)b * H + j] = is_bf16 ? bf16_bits_to_f32(((const uint16_t*)E)[(size_t)tok * H + j])
                                       : ((const float*)E)[(size_t)tok * H + j];
}

hipError_t launch_embed(const sun_model_cfg& cfg, const void* embed, const int32_t* tokens, int batch, float* x,
                        hipStream_t st) {
    hipLaunchKernelGGL(embed_kernel, dim3(batch), dim3(256), 0, st, embed, cfg.act_dtype == SUN_BF16, cfg.hidden,
                       cfg.vocab, tokens, x);
    return hipGetLastError();
}

// Writes eight consecutive values of row b (unit u = k / 8) into the fixed-point tile of a 4-bit projection.
// The 16 lanes that hold one 128-wide group share its scale (largest magnitude over the group); the first of
// them stores the scale and the sum of the group's integers.  Every lane of the wave must call it.
__device__ __forceinline__ void qtile_group16(uint8_t* tile, float2* qscale, ATile t, int b, int u, bool live,
                                              const float (&y)[8]) {
    float am = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) am = fmaxf(am, fabsf(y[e]));
    am = fmaxf(am, __shfl_xor(am, 1));
    am = fmaxf(am, __shfl_xor(am, 2));
    am = fmaxf(am, __shfl_xor(am, 4));
    am = fmaxf(am, __shfl_xor(am, 8));
    int sum = live ? qtile_store8(tile, t, b, u, y, qtile_inv(am)) : 0;
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    sum += __shfl_xor(sum, 4);
    sum += __shfl_xor(sum, 8);
    if (live && (threadIdx.x & 15) == 0) qscale[(size_t)(u >> 4) * (t.MB * 32) + b] = float2{am / kQMax, __int_as_float(sum)};
}

// ---------------- residual add + RMSNorm ----------------
// One block per row.  x += sum_s partial[s] (s ascending), h = x * rsqrt(mean(x^2) + eps) * g.
struct NormArgs {
    float* x;
    const float* partial;
    const void* gain;
    float* h_f32;
    uint16_t* h_tiled;
    float2* qscale;  // not NULL: h_tiled is the fixed-point tile of a 4-bit projection, and this its scales and sums
    int nparts, ld_rows, H, gain_bf16, mb;
    float eps;
};

// One 8-element unit per thread and pass (up to two passes, i.e. hidden <= 16 * blockDim), all
// slab loads of a unit independent of one another so that they are in flight together.
__global__ __launch_bounds__(1024) void residual_norm_kernel(NormArgs a) {
    __shared__ float red[16];
    const int b = blockIdx.x, tid = threadIdx.x, H = a.H, nunits = H / 8, nthreads = blockDim.x;
    float* xr = a.x + (size_t)b * H;
    float v[2][8];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int u = tid + it * nthreads;
        if (u < nunits) {
            f32x4 lo = *reinterpret_cast<const f32x4*>(xr + u * 8), hi = *reinterpret_cast<const f32x4*>(xr + u * 8 + 4);
            const float* p = a.partial + (size_t)b * H + u * 8;
            const size_t slab = (size_t)a.ld_rows * H;
            for (int s0 = 0; s0 < a.nparts; s0 += 4) {
                f32x4 pl[4], ph[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int s = min(s0 + j, a.nparts - 1);
                    pl[j] = *reinterpret_cast<const f32x4*>(p + s * slab);
                    ph[j] = *reinterpret_cast<const f32x4*>(p + s * slab + 4);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (s0 + j < a.nparts) {  // slabs are added in ascending order
                        lo += pl[j];
                        hi += ph[j];
                    }
            }
            if (a.nparts > 0) {
                *reinterpret_cast<f32x4*>(xr + u * 8) = lo;
                *reinterpret_cast<f32x4*>(xr + u * 8 + 4) = hi;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[it][e] = lo[e];
                v[it][4 + e] = hi[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = fmaf(v[it][e], v[it][e], ss);
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < nthreads / 64; ++w) tot += red[w];
    const float rinv = 1.0f / sqrtf(tot / (float)H + a.eps);
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int u = tid + it * nthreads;
        float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (u < nunits) {
            float g[8];
            if (a.gain_bf16) {
                const u32x4 gw = *reinterpret_cast<const u32x4*>((const uint16_t*)a.gain + u * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    g[2 * e] = bf16_lo(gw[e]);
                    g[2 * e + 1] = bf16_hi(gw[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) g[e] = ((const float*)a.gain)[u * 8 + e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = v[it][e] * rinv * g[e];
            if (a.h_f32) {
                *reinterpret_cast<f32x4*>(a.h_f32 + (size_t)b * H + u * 8) = f32x4{y[0], y[1], y[2], y[3]};
                *reinterpret_cast<f32x4*>(a.h_f32 + (size_t)b * H + u * 8 + 4) = f32x4{y[4], y[5], y[6], y[7]};
            }
            if (a.h_tiled && !a.qscale) {
                u32x4 o, ol;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    o[e] = pack_bf16(y[2 * e], y[2 * e + 1]);
                    ol[e] = pack_bf16(y[2 * e] - bf16_lo(o[e]), y[2 * e + 1] - bf16_hi(o[e]));
                }
                reinterpret_cast<u32x4*>(a.h_tiled)[atile_unit(ATile{a.mb}, 0, b, u)] = o;
                reinterpret_cast<u32x4*>(a.h_tiled)[atile_unit(ATile{a.mb}, 1, b, u)] = ol;
            }
        }
        if (a.qscale)  // fixed-point tile of a 4-bit projection: 16 consecutive units (lanes) form one 128-wide group
            qtile_group16((uint8_t*)a.h_tiled, a.qscale, ATile{a.mb}, b, u, u < nunits, y);
    }
}

hipError_t launch_residual_norm(const sun_model_cfg& cfg, float* x, const float* partial, int nparts, int ld_rows,
                                const void* gain, int batch, float* h_f32, void* h_tiled, float* qscale, hipStream_t st) {
    NormArgs a{};
    a.x = x;
    a.partial = partial;
    a.gain = gain;
    a.h_f32 = h_f32;
    a.h_tiled = (uint16_t*)h_tiled;
    a.qscale = (float2*)qscale;
    a.nparts = nparts;
    a.ld_rows = ld_rows;
    a.H = cfg.hidden;
    a.gain_bf16 = cfg.act_dtype == SUN_BF16;
    a.mb = atile_for_rows(batch).MB;
    a.eps = cfg.rms_eps;
    if (cfg.hidden % 8 || cfg.hidden > 16 * 1024) return hipErrorInvalidValue;
    const int units = cfg.hidden / 8;
    const int threads = units <= 1024 ? (units + 63) / 64 * 64 : ((units + 1) / 2 + 63) / 64 * 64;
    hipLaunchKernelGGL(residual_norm_kernel, dim3(batch), dim3(threads), 0, st, a);
    return hipGetLastError();
}

// ---------------- rotary table: cos/sin of pos * theta_j, angle in double ----------------
// theta_j = base^(-2j/d); with the wavelength-dependent scaling rule of the LLaMA-3.1 class (scaling = 1) it
// is kept, divided by `factor`, or blended between the two, depending on where 2*pi/theta_j lies relative to
// orig/high_freq and orig/low_freq.
struct RopeScale {
    int scaling, orig_max;
    double factor, low_freq, high_freq;
};

__global__ __launch_bounds__(64) void rope_table_kernel(const int32_t* __restrict__ seq_lens, int d, double base,
                                                        RopeScale rs, float* __restrict__ table) {
    const int b = blockIdx.x;
    const double pos = (double)seq_lens[b];
    for (int j = threadIdx.x; j < d / 2; j += 64) {
        double theta = pow(base, -2.0 * (double)j / (double)d);
        if (rs.scaling == 1) {
            const double wavelen = 2.0 * 3.14159265358979323846 / theta, orig = (double)rs.orig_max;
            if (wavelen > orig / rs.low_freq) {
                theta = theta / rs.factor;
            } else if (wavelen >= orig / rs.high_freq) {
                const double smooth = (orig / wavelen - rs.low_freq) / (rs.high_freq - rs.low_freq);
                theta = (1.0 - smooth) * theta / rs.factor + smooth * theta;
            }
        }
        const double ang = pos * theta;
        table[((size_t)b * (d / 2) + j) * 2] = (float)cos(ang);
        table[((size_t)b * (d / 2) + j) * 2 + 1] = (float)sin(ang);
    }
}

hipError_t launch_rope_table(const sun_model_cfg& cfg, const int32_t* seq_lens, int batch, float* table,
                             hipStream_t st) {
    const RopeScale rs{cfg.rope_scaling, cfg.rope_original_max_position, (double)cfg.rope_factor,
                       (double)cfg.rope_low_freq_factor, (double)cfg.rope_high_freq_factor};
    hipLaunchKernelGGL(rope_table_kernel, dim3(batch), dim3(64), 0, st, seq_lens, cfg.head_dim, (double)cfg.rope_base, rs,
                       table);
    return hipGetLastError();
}

// ---------------- rotary embedding + KV append ----------------
// grid (Hq + 2*Hkv, batch): head index < Hq -> q head; next Hkv -> k head; last Hkv -> v head.
struct RopeArgs {
    const float* qkv;
    const float* table;
    const int32_t* seq_lens;
    const int32_t* page_tables;
    float* q_out;
    uint16_t* pool;
    int64_t k_base, k_page, k_head, k_token, k_dim, v_base, v_page, v_head, v_token, v_dim;
    int nparts, ld_rows, Hq, Hkv, D, max_pages, n_pages;
    const void* qn;  // head-norm gains [D] for q and k heads, or NULL (no head norm)
    const void* kn;
    const void *bq, *bk, *bv;  // projection biases [Hq*D], [Hkv*D], [Hkv*D] (element type as the gains), or NULL
    int gain_bf16;
    float eps;
};

__global__ __launch_bounds__(64) void rope_append_kernel(RopeArgs a) {
    const int b = blockIdx.y, hh = blockIdx.x, D = a.D, half = D / 2;
    const int Nqkv = (a.Hq + 2 * a.Hkv) * D;
    // lengths and page ids are validated on the host under SUN_VALIDATE; clamp so bad input cannot fault
    const int L = min(max(a.seq_lens[b], 0), a.max_pages * kPageTokens - 1);
    const int page = min(max(a.page_tables[(size_t)b * a.max_pages + L / kPageTokens], 0), a.n_pages - 1);
    const int slot = L % kPageTokens;
    const float* src = a.qkv + (size_t)b * Nqkv + (size_t)hh * D;
    const size_t pstride = (size_t)a.ld_rows * Nqkv;
    // head_dim <= 128: lane j owns elements j and j + D/2; lanes past D/2 carry zeros through the norm
    const int j = threadIdx.x;
    const bool act = j < half;
    float lo = 0.f, hi = 0.f;
    if (act) {
        for (int s = 0; s < a.nparts; ++s) {
            lo += src[s * pstride + j];
            hi += src[s * pstride + j + half];
        }
    }
    if (a.bq && act) {  // bias of this head's slice of the q, k or v projection
        const void* bias = hh < a.Hq ? a.bq : hh < a.Hq + a.Hkv ? a.bk : a.bv;
        const int h0 = (hh < a.Hq ? hh : hh < a.Hq + a.Hkv ? hh - a.Hq : hh - a.Hq - a.Hkv) * D;
        lo += a.gain_bf16 ? bf16_bits_to_f32(((const uint16_t*)bias)[h0 + j]) : ((const float*)bias)[h0 + j];
        hi += a.gain_bf16 ? bf16_bits_to_f32(((const uint16_t*)bias)[h0 + j + half]) : ((const float*)bias)[h0 + j + half];
    }
    if (a.qn && hh < a.Hq + a.Hkv) {  // RMSNorm over the head's D elements (uniform branch: all lanes take part)
        const float ss = wave_sum(lo * lo + hi * hi);
        const float r = 1.0f / sqrtf(ss / (float)D + a.eps);
        if (act) {
            const void* g = hh < a.Hq ? a.qn : a.kn;
            const float gl = a.gain_bf16 ? bf16_bits_to_f32(((const uint16_t*)g)[j]) : ((const float*)g)[j];
            const float gh = a.gain_bf16 ? bf16_bits_to_f32(((const uint16_t*)g)[j + half]) : ((const float*)g)[j + half];
            lo = lo * r * gl;
            hi = hi * r * gh;
        }
    }
    if (!act) return;
    if (hh < a.Hq + a.Hkv) {
        const float c = a.table[((size_t)b * half + j) * 2], sn = a.table[((size_t)b * half + j) * 2 + 1];
        const float rl = lo * c - hi * sn, rh = hi * c + lo * sn;
        lo = rl;
        hi = rh;
    }
    if (hh < a.Hq) {
        a.q_out[((size_t)b * a.Hq + hh) * D + j] = lo;
        a.q_out[((size_t)b * a.Hq + hh) * D + j + half] = hi;
    } else if (hh < a.Hq + a.Hkv) {
        uint16_t* kd = a.pool + a.k_base + (int64_t)page * a.k_page + (int64_t)(hh - a.Hq) * a.k_head + slot * a.k_token;
        kd[j * a.k_dim] = f32_to_bf16_bits(lo);
        kd[(j + half) * a.k_dim] = f32_to_bf16_bits(hi);
    } else {
        uint16_t* vd = a.pool + a.v_base + (int64_t)page * a.v_page + (int64_t)(hh - a.Hq - a.Hkv) * a.v_head + slot * a.v_token;
        vd[j * a.v_dim] = f32_to_bf16_bits(lo);
        vd[(j + half) * a.v_dim] = f32_to_bf16_bits(hi);
    }
}

hipError_t launch_rope_append(const KvPool& pool, int layer, const float* qkv, int nparts, int ld_rows,
                              const float* table, const int32_t* seq_lens, const int32_t* page_tables, int max_pages,
                              int batch, float* q_out, const void* q_norm, const void* k_norm, const void* bq, const void* bk,
                              const void* bv, hipStream_t st) {
    const sun_model_cfg& c = pool.cfg;
    if (c.head_dim > 128) return hipErrorInvalidValue;
    const sun_kv_layout& L = pool.lay;
    RopeArgs a{};
    a.qkv = qkv;
    a.table = table;
    a.seq_lens = seq_lens;
    a.page_tables = page_tables;
    a.q_out = q_out;
    a.pool = pool.base;
    a.k_base = L.k_off + (int64_t)layer * L.k_layer;
    a.k_page = L.k_page;
    a.k_head = L.k_head;
    a.k_token = L.k_token;
    a.k_dim = L.k_dim;
    a.v_base = L.v_off + (int64_t)layer * L.v_layer;
    a.v_page = L.v_page;
    a.v_head = L.v_head;
    a.v_token = L.v_token;
    a.v_dim = L.v_dim;
    a.nparts = nparts;
    a.ld_rows = ld_rows;
    a.Hq = c.n_q_heads;
    a.Hkv = c.n_kv_heads;
    a.D = c.head_dim;
    a.max_pages = max_pages;
    a.n_pages = (int)L.n_pages;
    a.qn = c.qk_norm ? q_norm : nullptr;
    a.kn = c.qk_norm ? k_norm : nullptr;
    a.gain_bf16 = c.act_dtype == SUN_BF16;
    a.eps = c.rms_eps;
    a.bq = c.qkv_bias ? bq : nullptr;
    a.bk = c.qkv_bias ? bk : nullptr;
    a.bv = c.qkv_bias ? bv : nullptr;
    if (c.qk_norm && (!q_norm || !k_norm)) return hipErrorInvalidValue;
    if (c.qkv_bias && (!bq || !bk || !bv)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rope_append_kernel, dim3(c.n_q_heads + 2 * c.n_kv_heads, batch), dim3(64), 0, st, a);
    return hipGetLastError();
}

// ---------------- SwiGLU on fp32 [batch, 2*ffn] (gate columns first) ----------------
__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float* __restrict__ gu, int ffn, float* __restrict__ u) {
    const int b = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= ffn) return;
    const float g = gu[(size_t)b * 2 * ffn + j], up = gu[(size_t)b * 2 * ffn + ffn + j];
    u[(size_t)b * ffn + j] = g / (1.0f + expf(-g)) * up;
}

hipError_t launch_swiglu_f32(const float* gu, int batch, int ffn, float* u, hipStream_t st) {
    hipLaunchKernelGGL(swiglu_f32_kernel, dim3((ffn + 255) / 256, batch), dim3(256), 0, st, gu, ffn, u);
    return hipGetLastError();
}

// ---------------- SwiGLU over the gate/up projection's partial sums ----------------
// part: [nparts][ld_rows][2*ffn] fp32 with the projection's column order (blocks of 16 gate
// columns followed by their 16 up columns).  Writes u = silu(sum g) * (sum u) [rows, ffn] as the down
// projection's input: two-plane tiled bf16, or (qscale given) the fixed-point tile of a 4-bit projection.
__global__ __launch_bounds__(256) void swiglu_tile_kernel(const float* __restrict__ part, int nparts, int ld_rows,
                                                          int ffn, int mb, u32x4* __restrict__ tiled,
                                                          float* __restrict__ qscale) {
    const int b = blockIdx.y, u = blockIdx.x * 256 + threadIdx.x;  // unit = 8 consecutive u columns
    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (u < ffn / 8) {
        const int j = u * 8;
        const float* p = part + (size_t)b * 2 * ffn + (j >> 4) * 32 + (j & 15);
        const size_t slab = (size_t)ld_rows * 2 * ffn;
        f32x4 g0 = {0.f, 0.f, 0.f, 0.f}, g1 = g0, u0 = g0, u1 = g0;
        for (int s = 0; s < nparts; ++s) {  // slabs in ascending order
            g0 += *reinterpret_cast<const f32x4*>(p + s * slab);
            g1 += *reinterpret_cast<const f32x4*>(p + s * slab + 4);
            u0 += *reinterpret_cast<const f32x4*>(p + s * slab + 16);
            u1 += *reinterpret_cast<const f32x4*>(p + s * slab + 20);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            y[e] = g0[e] / (1.f + __expf(-g0[e])) * u0[e];
            y[4 + e] = g1[e] / (1.f + __expf(-g1[e])) * u1[e];
        }
        if (!qscale) {
            u32x4 o, ol;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = pack_bf16(y[2 * e], y[2 * e + 1]);
                ol[e] = pack_bf16(y[2 * e] - bf16_lo(o[e]), y[2 * e + 1] - bf16_hi(o[e]));
            }
            tiled[atile_unit(ATile{mb}, 0, b, u)] = o;
            tiled[atile_unit(ATile{mb}, 1, b, u)] = ol;
        }
    }
    if (qscale) qtile_group16((uint8_t*)tiled, (float2*)qscale, ATile{mb}, b, u, u < ffn / 8, y);
}

hipError_t launch_swiglu_tile(const float* part, int nparts, int ld_rows, int rows, int ffn, void* tiled, float* qscale,
                              hipStream_t st) {
    if (ffn % 128) return hipErrorInvalidValue;
    const int mb = atile_for_rows(rows).MB;
    hipLaunchKernelGGL(swiglu_tile_kernel, dim3((ffn / 8 + 255) / 256, rows), dim3(256), 0, st, part, nparts, ld_rows, ffn,
                       mb, (u32x4*)tiled, qscale);
    return hipGetLastError();
}

// ---------------- greedy argmax, lowest index on ties ----------------
// Two passes so that all compute units read the logits: kArgmaxParts slices of a row are
// searched by one workgroup each, then one thread per row picks among the slice winners
// (slices in index order, strict comparison, so the lowest index wins ties).
__global__ __launch_bounds__(256) void argmax_part_kernel(const float* __restrict__ logits, int V,
                                                          float* __restrict__ pval, int32_t* __restrict__ pidx) {
    __shared__ float bv[4];
    __shared__ int bi[4];
    const int b = blockIdx.y, part = blockIdx.x, tid = threadIdx.x;
    const int per = (V + kArgmaxParts - 1) / kArgmaxParts;
    const int j0 = part * per, j1 = min(V, j0 + per);
    const float* row = logits + (size_t)b * V;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int j = j0 + tid; j < j1; j += 256) {
        const float v = row[j];
        if (v > best) {  // a thread meets its indices in ascending order
            best = v;
            idx = j;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(idx, o);
        if (ov > best || (ov == best && oi < idx)) {
            best = ov;
            idx = oi;
        }
    }
    if ((tid & 63) == 0) {
        bv[tid >> 6] = best;
        bi[tid >> 6] = idx;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) {
                best = bv[w];
                idx = bi[w];
            }
        pval[(size_t)b * kArgmaxParts + part] = best;
        pidx[(size_t)b * kArgmaxParts + part] = idx;
    }
}

__global__ __launch_bounds__(256) void argmax_pick_kernel(const float* __restrict__ pval, const int32_t* __restrict__ pidx,
                                                          int batch, int32_t* __restrict__ next) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= batch) return;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int p = 0; p < kArgmaxParts; ++p) {
        const float v = pval[(size_t)b * kArgmaxParts + p];
        const int i = pidx[(size_t)b * kArgmaxParts + p];
        if (v > best || (v == best && i < idx)) {
            best = v;
            idx = i;
        }
    }
    next[b] = idx == 0x7fffffff ? 0 : idx;
}

hipError_t launch_argmax(const float* logits, int batch, int vocab, float* part_val, int32_t* part_idx, int32_t* next,
                         hipStream_t st) {
    hipLaunchKernelGGL(argmax_part_kernel, dim3(kArgmaxParts, batch), dim3(256), 0, st, logits, vocab, part_val, part_idx);
    hipLaunchKernelGGL(argmax_pick_kernel, dim3((batch + 255) / 256), dim3(256), 0, st, part_val, part_idx, batch, next);
    return hipGetLastError();
}

// ---------------- KV ingest: a contiguous cache into a request's pages ----------------
// One workgroup per (logical page, kv head, layer).  Source [layer][token][head][dim] bf16; token t is
// position first_pos + t.  K rows are copied 16 bytes at a time; V goes through an LDS tile because the
// pool keeps it transposed ([dim][token]).  Only the positions of the source are written, so a chunk can
// be appended to a partly filled page.  A page id outside the pool skips the page.
struct IngestArgs {
    uint16_t* kbase;  // pool base + k_off
    uint16_t* vbase;
    int64_t k_layer, k_page, k_head, v_layer, v_page, v_head;
    const uint16_t* k_src;
    const uint16_t* v_src;
    const int32_t* page_table;
    int n_tokens, first_pos, Hkv, D, n_pages;
};

__global__ __launch_bounds__(256) void kv_ingest_kernel(IngestArgs a) {
    __shared__ uint16_t tile[kPageTokens][128 + 8];
    const int lp = a.first_pos / kPageTokens + blockIdx.x, h = blockIdx.y, l = blockIdx.z, tid = threadIdx.x;
    const int page = a.page_table[lp];
    if (page < 0 || page >= a.n_pages) return;
    const int p0 = lp * kPageTokens;
    const int s_lo = max(a.first_pos - p0, 0), s_hi = min(a.first_pos + a.n_tokens - p0, kPageTokens);  // valid slots
    const int D = a.D, cpt = D / 8;                                                                    // 16-byte chunks per token
    uint16_t* kd = a.kbase + l * a.k_layer + page * a.k_page + h * a.k_head;
    uint16_t* vd = a.vbase + l * a.v_layer + page * a.v_page + h * a.v_head;
    for (int idx = tid; idx < kPageTokens * cpt; idx += 256) {
        const int s = idx / cpt, c = idx % cpt;
        if (s < s_lo || s >= s_hi) continue;
        const size_t so = (((size_t)l * a.n_tokens + (p0 + s - a.first_pos)) * a.Hkv + h) * D + c * 8;
        *reinterpret_cast<u32x4*>(kd + s * D + c * 8) = *reinterpret_cast<const u32x4*>(a.k_src + so);
        const u32x4 v = *reinterpret_cast<const u32x4*>(a.v_src + so);
        *reinterpret_cast<u32x4*>(&tile[s][c * 8]) = v;
    }
    __syncthreads();
    // V^T: thread <-> (dim, half of the page's 16 slots)
    for (int idx = tid; idx < D * 2; idx += 256) {
        const int dim = idx >> 1, half = idx & 1, s0 = half * 8;
        if (s0 >= s_lo && s0 + 8 <= s_hi) {
            uint16_t e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = tile[s0 + j][dim];
            u32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) o[j] = (uint32_t)e[2 * j] | ((uint32_t)e[2 * j + 1] << 16);
            *reinterpret_cast<u32x4*>(vd + dim * kPageTokens + s0) = o;
        } else {
            for (int j = 0; j < 8; ++j)
                if (s0 + j >= s_lo && s0 + j < s_hi) vd[dim * kPageTokens + s0 + j] = tile[s0 + j][dim];
        }
    }
}

hipError_t launch_kv_ingest(const KvPool& pool, const void* k_src, const void* v_src, int n_tokens, int first_pos,
                            const int32_t* page_table, hipStream_t st) {
    const sun_model_cfg& c = pool.cfg;
    const sun_kv_layout& L = pool.lay;
    if (L.k_dim != 1 || L.k_token != c.head_dim || L.v_token != 1 || L.v_dim != kPageTokens || c.head_dim > 128 ||
        c.head_dim % 8)
        return hipErrorInvalidValue;
    IngestArgs a{};
    a.kbase = pool.base + L.k_off;
    a.vbase = pool.base + L.v_off;
    a.k_layer = L.k_layer; a.k_page = L.k_page; a.k_head = L.k_head;
    a.v_layer = L.v_layer; a.v_page = L.v_page; a.v_head = L.v_head;
    a.k_src = (const uint16_t*)k_src;
    a.v_src = (const uint16_t*)v_src;
    a.page_table = page_table;
    a.n_tokens = n_tokens;
    a.first_pos = first_pos;
    a.Hkv = c.n_kv_heads;
    a.D = c.head_dim;
    a.n_pages = (int)L.n_pages;
    const int pages = (first_pos + n_tokens - 1) / kPageTokens - first_pos / kPageTokens + 1;
    hipLaunchKernelGGL(kv_ingest_kernel, dim3(pages, c.n_kv_heads, c.n_layers), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ---------------- per-row inputs of a prefill block ----------------
__global__ __launch_bounds__(256) void prefill_rows_kernel(const int32_t* __restrict__ page_table, int max_pages,
                                                           int first_pos, int model_id, int32_t* __restrict__ tables,
                                                           int32_t* __restrict__ lens, int32_t* __restrict__ ids) {
    const int r = blockIdx.x;
    for (int c = threadIdx.x; c < max_pages; c += 256) tables[(size_t)r * max_pages + c] = page_table[c];
    if (threadIdx.x == 0) {
        lens[r] = first_pos + r;
        ids[r] = model_id;
    }
}

hipError_t launch_prefill_rows(const int32_t* page_table, int max_pages, int first_pos, int model_id, int rows,
                               int32_t* tables, int32_t* lens, int32_t* ids, hipStream_t st) {
    hipLaunchKernelGGL(prefill_rows_kernel, dim3(rows), dim3(256), 0, st, page_table, max_pages, first_pos, model_id,
                       tables, lens, ids);
    return hipGetLastError();
}

// ---------------- bookkeeping between the steps of a run ----------------
// One workgroup.  Request b feeds its generated token back and grows by one position.  If that
// position opens a page its table does not have yet, it takes the next unused entry of the free
// list; requests are served in index order (an exclusive scan over the requests that need a page).
// A request that finds the list empty, or whose table is full, keeps its length and re-decodes the
// same position; status bit 0 / bit 1 records that.
__global__ __launch_bounds__(1024) void advance_kernel(const int32_t* __restrict__ next, int batch, int max_pages,
                                                       const int32_t* __restrict__ free_pages, int n_free,
                                                       int32_t* __restrict__ token_ids, int32_t* __restrict__ page_tables,
                                                       int32_t* __restrict__ seq_lens, int32_t* __restrict__ free_head,
                                                       int32_t* __restrict__ status, int clear_status) {
    __shared__ int scan[1024];
    const int t = threadIdx.x;
    if (clear_status && t == 0) *status = 0;  // ordered before the atomicOr below by the barriers in between
    int new_len = 0, slot_page = 0, wants = 0, full = 0;
    if (t < batch) {
        token_ids[t] = next[t];
        new_len = seq_lens[t] + 1;
        slot_page = new_len / kPageTokens;
        full = slot_page >= max_pages;
        wants = !full && new_len % kPageTokens == 0 && page_tables[(size_t)t * max_pages + slot_page] < 0;
    }
    scan[t] = wants;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int v = t >= o ? scan[t - o] : 0;
        __syncthreads();
        scan[t] += v;
        __syncthreads();
    }
    const int head = *free_head;
    const int rank = scan[t] - wants;  // requests before this one that take a page
    int flags = 0;
    if (t < batch) {
        if (full) {
            flags = 2;
        } else if (wants && head + rank >= n_free) {
            flags = 1;
        } else {
            if (wants) page_tables[(size_t)t * max_pages + slot_page] = free_pages[head + rank];
            seq_lens[t] = new_len;
        }
    }
    if (flags) atomicOr(status, flags);
    __syncthreads();  // every thread has read *free_head
    if (t == 1023) *free_head = min(head + scan[1023], n_free);
}

hipError_t launch_advance(const int32_t* next, int batch, int max_pages, const int32_t* free_pages, int n_free,
                          int32_t* token_ids, int32_t* page_tables, int32_t* seq_lens, int32_t* free_head,
                          int32_t* status, bool clear_status, hipStream_t st) {
    if (batch > 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(advance_kernel, dim3(1), dim3(1024), 0, st, next, batch, max_pages, free_pages, n_free, token_ids,
                       page_tables, seq_lens, free_head, status, clear_status ? 1 : 0);
    return hipGetLastError();
}

// ---------------- continuous batching: retire, advance, admit between two steps ----------------
// One workgroup of 1024 threads; thread t < slots owns row t, and all 16 waves share the walks over page-table
// rows (a wave per row, 64 columns per load), so that no thread walks a row alone.  All orders are row order
// (exclusive scans) and column order (ballots), so the result does not depend on scheduling.  The phases
// follow the declaration of sun_decode_serve.
constexpr int kServeThreads = 1024;
constexpr int kServeWaves = kServeThreads / 64;

// exclusive prefix sum over the workgroup in thread order; total = the sum over all threads
__device__ __forceinline__ int block_scan_excl(int v, int* sc, int& total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(inc, o);
        if (lane >= o) inc += u;
    }
    __syncthreads();  // sc may still be read from the previous scan
    if (lane == 63) sc[w] = inc;
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kServeWaves; ++i) {
        const int part = sc[i];
        before += i < w ? part : 0;
        tot += part;
    }
    total = tot;
    return before + inc - v;
}

// pages (entries >= 0) in one table row, counted by a whole wave; the same value in every lane
__device__ __forceinline__ int wave_count_row(const int32_t* row, int max_pages) {
    const int lane = threadIdx.x & 63;
    int n = 0;
    for (int c0 = 0; c0 < max_pages; c0 += 64) {
        const int c = c0 + lane;
        const bool have = c < max_pages && row[c] >= 0;
        n += __popcll(__ballot(have));
    }
    return n;
}

__global__ __launch_bounds__(kServeThreads) void serve_kernel(ServeArgs a, const int32_t* __restrict__ next,
                                                              int32_t* __restrict__ tokens_out,
                                                              int32_t* __restrict__ req_out, int do_reset, int do_advance) {
    __shared__ int sc[kServeWaves];
    __shared__ int held[256];  // pages per row, later pages per admission candidate
    __shared__ int roff[256];  // ring offset of a retiring row's first page, else -1
    __shared__ int act[256];   // what happens to a row's table: -1 nothing, -2 written as idle, q >= 0 copied from waiting q
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const bool row = t < a.slots;
    int whead = a.counters[0], head = a.counters[1], tail = a.counters[2];
    int32_t* tab = a.page_tables + (size_t)(row ? t : 0) * a.max_pages;
    int req = -1, left = 0, len = 0, status = 0, retired = 0, generated = 0;
    if (row && !do_reset) {
        req = a.slot_req[t];
        left = a.slot_left[t];
        len = a.seq_lens[t];
    }
    if (!do_reset)
        for (int r = wave; r < a.slots; r += kServeWaves) {
            const int n = wave_count_row(a.page_tables + (size_t)r * a.max_pages, a.max_pages);
            if (lane == 0) held[r] = n;
        }
    __syncthreads();
    int my_held = (row && !do_reset) ? held[t] : 0;
    bool occ = req >= 0;
    bool clear = row && do_reset;  // rows to be written as idle
    if (do_advance) {
        const int tok = row ? next[t] : 0;
        if (row) {
            tokens_out[t] = occ ? tok : -1;
            req_out[t] = req;
        }
        bool fin = false;
        if (occ) {
            left -= 1;
            generated = 1;
            fin = left == 0 || tok == a.eos_id;
        }
        // retire: pages to the ring's tail, rows in order, columns in order
        int give_total;
        const int give = (occ && fin) ? my_held : 0;
        const int off = block_scan_excl(give, sc, give_total);
        if (t < 256) roff[t] = (occ && fin) ? off : -1;
        __syncthreads();
        for (int r = wave; r < a.slots; r += kServeWaves) {
            if (roff[r] < 0) continue;  // the same for the whole wave
            const int32_t* src = a.page_tables + (size_t)r * a.max_pages;
            int at = tail + roff[r];
            for (int c0 = 0; c0 < a.max_pages; c0 += 64) {
                const int c = c0 + lane;
                const int pg = c < a.max_pages ? src[c] : -1;
                const unsigned long long m = __ballot(pg >= 0);
                if (pg >= 0) a.ring[(unsigned)(at + __popcll(m & ((1ull << lane) - 1ull))) % (unsigned)a.ring_cap] = pg;
                at += __popcll(m);
            }
        }
        if (occ && fin) {
            retired = 1;
            clear = true;
        }
        tail += give_total;
        __syncthreads();  // the ring entries written above may be taken below
        // advance the others
        const bool cont = occ && !fin;
        const int new_len = len + 1, col = new_len / kPageTokens;
        const int wants = cont && col < a.max_pages && new_len % kPageTokens == 0 && tab[col] < 0;
        int want_total;
        const int rank = block_scan_excl(wants, sc, want_total);
        if (cont) {
            if (col >= a.max_pages) {
                status |= 2;
            } else if (wants && head + rank >= tail) {
                status |= 1;
            } else {
                if (wants) {
                    tab[col] = a.ring[(unsigned)(head + rank) % (unsigned)a.ring_cap];
                    my_held += 1;
                }
                len = new_len;
            }
            a.token_ids[t] = tok;
            a.slot_left[t] = left;
            a.seq_lens[t] = len;
        }
        head = min(head + want_total, tail);
        if (fin) occ = false;
    }
    if (do_reset) occ = false;
    if (clear) {
        a.token_ids[t] = 0;
        a.seq_lens[t] = 0;
        a.model_ids[t] = 0;
        a.slot_req[t] = -1;
        a.slot_left[t] = 0;
    }
    // admission
    int out_total, idle_total, need_total, ok_total;
    const int outst = occ ? max(0, (len + left - 1) / kPageTokens + 1 - my_held) : 0;
    block_scan_excl(outst, sc, out_total);
    const int avail = (tail - head) - out_total;
    const bool idle = row && !occ;
    const int idle_rank = block_scan_excl(idle ? 1 : 0, sc, idle_total);
    const int ncand = max(0, min(idle_total, a.n_wait - whead));
    for (int q = wave; q < ncand; q += kServeWaves) {  // the scans above separate this from the last use of held[]
        const int n = wave_count_row(a.w_tables + (size_t)(whead + q) * a.max_pages, a.max_pages);
        if (lane == 0) held[q] = n;
    }
    __syncthreads();
    auto cut_budget = [&](int q, bool& cut) {
        const int room = a.max_pages * kPageTokens - a.w_lens[q];
        const int b = a.w_budget[q];
        cut = b > room;
        return max(1, min(b, room));
    };
    int need = 0;
    if (t < ncand) {
        const int q = whead + t;
        bool cut;
        const int b = cut_budget(q, cut);
        need = max(0, (a.w_lens[q] + b - 1) / kPageTokens + 1 - held[t]);
    }
    const int before = block_scan_excl(need, sc, need_total);
    // candidate t is admitted if it and all before it fit (needs are >= 0, so the admitted ones are a prefix)
    const int ok = t < ncand && before + need <= avail;
    block_scan_excl(ok, sc, ok_total);
    int what = clear ? -2 : -1;
    if (idle && idle_rank < ok_total) {
        const int q = whead + idle_rank;
        bool cut;
        const int b = cut_budget(q, cut);
        if (cut) status |= 2;
        what = q;
        a.token_ids[t] = a.w_token[q];
        a.seq_lens[t] = a.w_lens[q];
        a.model_ids[t] = a.w_model[q];
        a.slot_req[t] = a.w_req[q];
        a.slot_left[t] = b;
    }
    if (t < 256) act[t] = what;
    __syncthreads();  // also: every read of the old tables (retirement, tab[col]) is behind us
    for (int r = wave; r < a.slots; r += kServeWaves) {
        const int w = act[r];
        if (w == -1) continue;
        int32_t* dst = a.page_tables + (size_t)r * a.max_pages;
        const int32_t* src = w >= 0 ? a.w_tables + (size_t)w * a.max_pages : nullptr;
        for (int c = lane; c < a.max_pages; c += 64) dst[c] = src ? src[c] : (c == 0 ? a.idle_page : -1);
    }
    int ret_total, gen_total;
    block_scan_excl(retired, sc, ret_total);
    block_scan_excl(generated, sc, gen_total);
    if (status) atomicOr(&a.counters[3], status);
    if (t == 0) {
        a.counters[0] = whead + ok_total;
        a.counters[1] = head;
        a.counters[2] = tail;
        a.counters[4] += ret_total;
        a.counters[5] += ok_total;
        a.counters[6] += gen_total;
        a.counters[7] += do_advance;
    }
}

hipError_t launch_serve(const ServeArgs& a, const int32_t* next, int32_t* tokens_out, int32_t* req_out, bool reset,
                        bool advance, hipStream_t st) {
    if (a.slots < 1 || a.slots > 256) return hipErrorInvalidValue;
    hipLaunchKernelGGL(serve_kernel, dim3(1), dim3(kServeThreads), 0, st, a, next, tokens_out, req_out, reset ? 1 : 0,
                       advance ? 1 : 0);
    return hipGetLastError();
}

// ---------------- HBM read probe (measurement only) ----------------
// Reads `n_blocks` blocks of `block_units` 16-byte units each, in the order perm gives (or in address order),
// and does nothing with them but fold them into one word per thread: what a kernel that only streams from HBM
// reaches on this device, contiguous or in scattered blocks the size of one (page, head) K or V block.
template <int STREAM>
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4* __restrict__ src, long long n_blocks,
                                                             int block_units, const int32_t* __restrict__ perm,
                                                             uint32_t* __restrict__ sink) {
    auto ld = [](const u32x4* p) { return STREAM ? load_stream(p) : *p; };
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long gw = (long long)blockIdx.x * 4 + wave, nw = (long long)gridDim.x * 4;
    uint32_t acc = 0;
    for (long long b = gw; b < n_blocks; b += nw) {     // one block per wave and turn, four 16-byte loads per lane in flight
        const long long blk = perm ? perm[b] : b;
        const u32x4* p = src + blk * block_units;
        for (int u = lane; u < block_units; u += 256) {
            const u32x4 v0 = ld(p + u), v1 = ld(p + min(u + 64, block_units - 1)), v2 = ld(p + min(u + 128, block_units - 1)),
                        v3 = ld(p + min(u + 192, block_units - 1));
            acc ^= v0[0] ^ v0[3] ^ v1[1] ^ v1[2] ^ v2[0] ^ v2[2] ^ v3[1] ^ v3[3];
        }
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

hipError_t launch_hbm_read_probe(const void* src, long long n_blocks, int block_units, const int32_t* perm, int grid,
                                 bool stream, uint32_t* sink, hipStream_t st) {
    if (stream) hipLaunchKernelGGL(hbm_read_probe_kernel<1>, dim3(grid), dim3(256), 0, st, (const u32x4*)src, n_blocks, block_units, perm, sink);
    else hipLaunchKernelGGL(hbm_read_probe_kernel<0>, dim3(grid), dim3(256), 0, st, (const u32x4*)src, n_blocks, block_units, perm, sink);
    return hipGetLastError();
}

// ---------------- layout helpers ----------------
__global__ __launch_bounds__(256) void tile_rows_kernel(const float* __restrict__ x, int rows, int K, int mb,
                                                        u32x4* __restrict__ tiled, float* __restrict__ qscale) {
    const int b = blockIdx.y;
    const int u = blockIdx.x * 256 + threadIdx.x;
    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (u < K / 8) {
        const float* p = x + (size_t)b * K + u * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = p[e];
        if (!qscale) {
            u32x4 o, ol;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = pack_bf16(y[2 * e], y[2 * e + 1]);
                ol[e] = pack_bf16(y[2 * e] - bf16_lo(o[e]), y[2 * e + 1] - bf16_hi(o[e]));
            }
            tiled[atile_unit(ATile{mb}, 0, b, u)] = o;
            tiled[atile_unit(ATile{mb}, 1, b, u)] = ol;
        }
    }
    if (qscale) qtile_group16((uint8_t*)tiled, (float2*)qscale, ATile{mb}, b, u, u < K / 8, y);
}

hipError_t launch_tile_rows(const float* x, int rows, int K, void* tiled, float* qscale, hipStream_t st) {
    if (K % 128) return hipErrorInvalidValue;
    const int mb = atile_for_rows(rows).MB;
    hipLaunchKernelGGL(tile_rows_kernel, dim3((K / 8 + 255) / 256, rows), dim3(256), 0, st, x, rows, K, mb,
                       (u32x4*)tiled, qscale);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int nparts,
                                                              int ld_rows, int N, float* __restrict__ out) {
    const int b = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    float v = 0.f;
    for (int s = 0; s < nparts; ++s) v += partial[((size_t)s * ld_rows + b) * N + n];
    out[(size_t)b * N + n] = v;
}

hipError_t launch_reduce_partials(const float* partial, int nparts, int ld_rows, int rows, int N, float* out,
                                  hipStream_t st) {
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((N + 255) / 256, rows), dim3(256), 0, st, partial, nparts, ld_rows,
                       N, out);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void untile_rows_kernel(const uint16_t* __restrict__ tiled, int K, int mb,
                                                          float* __restrict__ out) {
    const int b = blockIdx.y, k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    out[(size_t)b * K + k] = bf16_bits_to_f32(tiled[atile_elem(ATile{mb}, 0, b, k)]) +
                             bf16_bits_to_f32(tiled[atile_elem(ATile{mb}, 1, b, k)]);
}

hipError_t launch_untile_rows(const void* tiled, int rows, int K, float* out, hipStream_t st) {
    const int mb = atile_for_rows(rows).MB;
    hipLaunchKernelGGL(untile_rows_kernel, dim3((K + 255) / 256, rows), dim3(256), 0, st, (const uint16_t*)tiled, K, mb,
                       out);
    return hipGetLastError();
}

}  // namespace sun
