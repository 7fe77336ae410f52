// Paged GQA decode attention over the shared KV pool (the cache-reading part of
// Eq. 3; the cache is prompt KV from any task's prefill module followed by
// decode-generated KV, Eq. 4).  One query position per request attends to all
// n_i cached positions of that request; requests of different source models are
// handled identically, the pool is addressed through the page table only.
//
// Work decomposition: a work item is (request, kv head, chunk of positions).  All but the last
// 256..511 positions of a request form full chunks of 256, the rest small chunks of 64 (below 64
// requests the full chunks are shorter, see attn_full_chunk); the chunk grid of a request depends on
// its own length and the batch size only, so a request's result does not depend on its batch-mates.  One persistent workgroup of 8 waves per compute unit works through a
// statically dealt item list, full chunks first; a wave streams an item's K and V^T pages with
// 16-byte loads straight into matrix-core operand registers:
//   S^T[token, head] = K[token, :] . q[head, :]      (16x16x32 MFMA, q split hi+lo bf16)
//   O[head, dim]    += P[head, token] V^T[dim, token] (16x16x32 MFMA, P split hi+lo bf16)
// The group's q heads occupy the first G of the 16 MFMA columns.  Softmax runs in
// fp32 in the log2 domain with a running maximum; partial (O, m, l) per item are
// merged by a second kernel in chunk order.  The matrix cores are used because at
// ~13 HBM bytes per CU-clock the vector ALUs cannot also convert, multiply and
// reduce 256 bf16 values per token for several query heads; the kernel stays HBM
// bound.  An fp32 vector-ALU variant serves the fp32 parity configuration.
#include "kernels.hpp"

namespace sun {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int CH = kAttnChunk;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kRecInts = 24;  // ints per item record
constexpr int kTopUp = CH / kAttnSmall;  // small chunks that stand for one full chunk in a wave's item list

size_t attn_max_chunks(int batch, int max_pages, int Hkv) {
    // An upper bound for every batch size up to `batch` (a workspace sized for a larger batch serves a smaller
    // one).  Full chunks of a request: n / ch with ch = 256, or a shorter ch only while n * Hkv * b / 2048 < 256,
    // which bounds b * n / ch by 4096 / Hkv over the b < 64 requests; small chunks: at most
    // (2 * 256 - 1) / 64 + 1 = 8 per request.
    const size_t max_tokens = (size_t)max_pages * kPageTokens;
    return (size_t)batch * (max_tokens / CH + 2 * CH / kAttnSmall + 1) + 4096 / (size_t)Hkv + 64;
}

// ---------------------------------------------------------------------------------
// plan: chunk counts of every request and their prefix sums (one block)
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void attn_plan_kernel(const int32_t* __restrict__ n_or_len, int len_plus, int batch,
                                                         int32_t* __restrict__ chunk_off, int32_t* __restrict__ full_off,
                                                         int32_t* __restrict__ small_off, int max_tokens, int Hkv) {
    __shared__ int scan_f[1024], scan_s[1024];
    const int t = threadIdx.x;
    int nf = 0, ns = 0, ch = 0;
    if (t < batch) attn_chunking(min(max(n_or_len[t] + len_plus, 1), max_tokens), batch, Hkv, nf, ns, ch);
    scan_f[t] = nf;
    scan_s[t] = ns;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int vf = t >= o ? scan_f[t - o] : 0, vs = t >= o ? scan_s[t - o] : 0;
        __syncthreads();
        scan_f[t] += vf;
        scan_s[t] += vs;
        __syncthreads();
    }
    if (t < batch) {
        full_off[t + 1] = scan_f[t];
        small_off[t + 1] = scan_s[t];
        chunk_off[t + 1] = scan_f[t] + scan_s[t];
        if (t == 0) full_off[0] = small_off[0] = chunk_off[0] = 0;
    }
}

// One record per work item.  Items of all full chunks come first, ordered (request, kv head,
// chunk), then the items of all small chunks in the same order.  Record: the chunk's page ids
// (clamped into the pool, -1 where the chunk has no page), then request, kv head, first and
// one-past-last token, and the chunk's slot in the partial array (chunks of a request in token
// order).
__global__ __launch_bounds__(256) void attn_records_kernel(const int32_t* __restrict__ n_or_len, int len_plus, int batch,
                                                           const int32_t* __restrict__ chunk_off,
                                                           const int32_t* __restrict__ full_off,
                                                           const int32_t* __restrict__ small_off,
                                                           const int32_t* __restrict__ page_tables, int max_pages,
                                                           int n_pages, int Hkv, int32_t* __restrict__ records) {
    const int total_full = full_off[batch] * Hkv, total = chunk_off[batch] * Hkv;
    for (int item = blockIdx.x * 16 + (threadIdx.x >> 4); item < total; item += gridDim.x * 16) {
        const int slot = threadIdx.x & 15;
        const bool is_full = item < total_full;
        const int32_t* off = is_full ? full_off : small_off;
        const int idx = is_full ? item : item - total_full;
        int lo = 0, hi = batch;  // request whose item range [off[r]*Hkv, off[r+1]*Hkv) holds idx
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (off[mid] * Hkv <= idx) lo = mid; else hi = mid;
        }
        const int req = lo, nc = off[req + 1] - off[req];
        const int local = idx - off[req] * Hkv, head = local / nc, cj = local % nc;
        const int n = min(max(n_or_len[req] + len_plus, 1), max_pages * kPageTokens);
        const int nfull = full_off[req + 1] - full_off[req];
        const int ch = attn_full_chunk(n, batch, Hkv);
        const int t0 = is_full ? cj * ch : nfull * ch + cj * kAttnSmall;
        const int t1 = is_full ? t0 + ch : min(n, t0 + kAttnSmall);
        const int npages = (t1 - t0 + kPageTokens - 1) / kPageTokens;
        int32_t* rec = records + (size_t)item * kRecInts;
        rec[slot] = slot < npages ? min(max(page_tables[(size_t)req * max_pages + t0 / kPageTokens + slot], 0), n_pages - 1) : -1;
        if (slot < 8) {
            const int vals[8] = {req, head, t0, t1, chunk_off[req] + (is_full ? cj : nfull + cj), 0, 0, 0};
            rec[16 + slot] = vals[slot];
        }
    }
}

hipError_t launch_attn_plan(const AttnPlan& plan, const int32_t* n_or_len, int len_plus, int batch,
                            const int32_t* page_tables, int max_pages, int n_pages, int Hkv, hipStream_t st) {
    if (batch > 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(1024), 0, st, n_or_len, len_plus, batch, plan.chunk_off,
                       plan.full_off, plan.small_off, max_pages * kPageTokens, Hkv);
    const long long items = (long long)plan.max_chunks * Hkv;
    const int grid = (int)max(1LL, min((items + 15) / 16, 1024LL));
    hipLaunchKernelGGL(attn_records_kernel, dim3(grid), dim3(256), 0, st, n_or_len, len_plus, batch, plan.chunk_off,
                       plan.full_off, plan.small_off, page_tables, max_pages, n_pages, Hkv, plan.records);
    return hipGetLastError();
}

struct AttnArgs {
    const uint16_t* kbase;  // pool base + k_off + layer * k_layer
    const uint16_t* vbase;
    int64_t k_page, k_head, v_page, v_head;
    const float* q;         // [batch, Hq*D]
    const int32_t* page_tables;
    const int32_t* n_or_len;
    const int32_t* chunk_off;
    const int32_t* full_off;
    const int32_t* records;
    float* partial;
    int len_plus, max_pages, batch, Hq, Hkv, n_pages;
    int n_full_items, total_items;  // item counts when the host knows the lengths, else -1: read from the plan
    float qscale;           // log2(e) / sqrt(D)
};

__device__ __forceinline__ uint32_t bf16_pair_hi(float a, float b, float& ra, float& rb) {
    const uint32_t ha = f32_to_bf16_bits(a), hb = f32_to_bf16_bits(b);
    ra = a - __uint_as_float(ha << 16);
    rb = b - __uint_as_float(hb << 16);
    return ha | (hb << 16);
}

// ---------------------------------------------------------------------------------
// split kernel, matrix-core variant
// ---------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_split_kernel(AttnArgs a) {
    constexpr int NS = D / 32;  // dim slices of a QK MFMA
    constexpr int NB = D / 16;  // dim blocks of a PV MFMA
    const int lane = threadIdx.x & 63;
    const int c16 = lane & 15, kq = lane >> 4;
    // One workgroup of 8 waves per compute unit.  Items are dealt to workgroups statically: full
    // chunks (all of one size) round-robin; the workgroups that got one full chunk fewer are
    // topped up with a block of kTopUp small chunks, the remaining small chunks go round-robin.
    // Inside a workgroup the waves take the list's entries in order through a counter in LDS, so
    // they run out of work within one small chunk of each other however unevenly the hardware
    // serves them.  Which wave computes an item has no effect on its value.
    __shared__ int list_cursor;
    if (threadIdx.x == 0) list_cursor = 0;
    __syncthreads();
    const int n_full = a.n_full_items >= 0 ? a.n_full_items : a.full_off[a.batch] * a.Hkv;
    const int total_items = a.total_items >= 0 ? a.total_items : a.chunk_off[a.batch] * a.Hkv;
    const int n_small = total_items - n_full;
    const int wg = blockIdx.x, nwg = gridDim.x;
    const int fq = n_full / nwg, fr = n_full % nwg;
    auto next_item = [&]() -> int {  // next unclaimed entry of this workgroup's list, total_items when it is over
        int c = 0;
        if (lane == 0) c = atomicAdd(&list_cursor, 1);
        c = __builtin_amdgcn_readfirstlane(c);
        const int mine_full = fq + (wg < fr ? 1 : 0);
        if (c < mine_full) return wg + c * nwg;
        c -= mine_full;
        const int top = wg >= fr ? min(max(n_small - kTopUp * (wg - fr), 0), kTopUp) : 0;
        if (c < top) return n_full + kTopUp * (wg - fr) + c;
        c -= top;
        const long long j = (long long)kTopUp * (nwg - fr) + wg + (long long)c * nwg;
        return j < n_small ? n_full + (int)j : total_items;
    };
    int item = next_item();
    if (item >= total_items) return;
    int item_n = next_item();

    // K operand rows: MFMA row i of tile 0 <-> page (i>>3), token 8*((i>>2)&1) + (i&3); tile 1: +4
    const int k_psel = c16 >> 3, k_tok = 8 * ((c16 >> 2) & 1) + (c16 & 3);
    const int64_t k_lane_off = (int64_t)k_tok * D + kq * 8;
    // V^T operand: lane (dim c16 of a 16-dim block, token octet kq): page (kq>>1), tokens 8*(kq&1)..+7
    const int v_psel = kq >> 1;
    const int64_t v_lane_off = (int64_t)c16 * kPageTokens + 8 * (kq & 1);

    auto load_rec = [&](int it) { return lane < kRecInts ? a.records[(size_t)it * kRecInts + lane] : 0; };
    u32x4 kr[2][NS], vr[NB];  // K and V^T operand registers of one 32-token page pair
    auto load_k = [&](int recv, int head, int pp) {
        const int pA = __builtin_amdgcn_readlane(recv, 2 * pp);
        int pB = __builtin_amdgcn_readlane(recv, 2 * pp + 1);
        if (pB < 0) pB = pA;
        const uint16_t* kp = a.kbase + head * a.k_head + (int64_t)(k_psel ? pB : pA) * a.k_page + k_lane_off;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            kr[0][s] = *reinterpret_cast<const u32x4*>(kp + s * 32);
            kr[1][s] = *reinterpret_cast<const u32x4*>(kp + 4 * D + s * 32);
        }
    };
    // V^T is requested with streaming loads (every instruction reads two runs of 512 contiguous bytes, which
    // such loads move 10 % faster than cached ones and without displacing what the neighbouring kernels exchange
    // through the caches); K with plain loads: an instruction of K reads 64 bytes of each of 16 token rows, half a
    // cache line at a time, and streaming loads are slower than cached ones on that pattern (measured with a
    // read-only kernel: 6.7 against 6.1 TB/s on contiguous kilobytes, 5.95 against 6.2 on the K pattern)
    auto load_v = [&](int recv, int head, int pp) {
        const int pA = __builtin_amdgcn_readlane(recv, 2 * pp);
        int pB = __builtin_amdgcn_readlane(recv, 2 * pp + 1);
        if (pB < 0) pB = pA;
        const uint16_t* vp = a.vbase + head * a.v_head + (int64_t)(v_psel ? pB : pA) * a.v_page + v_lane_off;
#pragma unroll
        for (int b = 0; b < NB; ++b) vr[b] = load_stream(reinterpret_cast<const u32x4*>(vp + b * 16 * kPageTokens));
    };

    bf16x8 qhi[NS], qlo[NS];
    // q as MFMA B operand: lane (head g = c16, dim octet kq) per 32-dim slice, hi + lo bf16
    auto load_q = [&](int req, int head) {
        const float* qp = a.q + ((size_t)req * a.Hq + head * G + (c16 < G ? c16 : 0)) * D;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            u32x4 h, l;
            const f32x4 v0 = *reinterpret_cast<const f32x4*>(qp + s * 32 + kq * 8);
            const f32x4 v1 = *reinterpret_cast<const f32x4*>(qp + s * 32 + kq * 8 + 4);
            float x[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const float xa = c16 < G ? x[2 * p] * a.qscale : 0.f;
                const float xb = c16 < G ? x[2 * p + 1] * a.qscale : 0.f;
                float ra, rb;
                h[p] = bf16_pair_hi(xa, xb, ra, rb);
                l[p] = pack_bf16(ra, rb);
            }
            qhi[s] = __builtin_bit_cast(bf16x8, h);
            qlo[s] = __builtin_bit_cast(bf16x8, l);
        }
    };

    // current item state (wave-uniform scalars) and accumulators
    int rec = load_rec(item);
    int req = __builtin_amdgcn_readlane(rec, 16), head = __builtin_amdgcn_readlane(rec, 17);
    int t0 = __builtin_amdgcn_readlane(rec, 18), t1 = __builtin_amdgcn_readlane(rec, 19);
    int cidx = __builtin_amdgcn_readlane(rec, 20);
    int npairs = ((t1 - t0 + kPageTokens - 1) / kPageTokens + 1) / 2, pp = 0;
    load_k(rec, head, 0);
    load_v(rec, head, 0);
    int rec_n = load_rec(item_n < total_items ? item_n : item);
    load_q(req, head);
    int head_n = __builtin_amdgcn_readlane(rec_n, 17);

    f32x4 O[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) O[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

    // bf16 hi/lo split of two fp32 values with the hardware converter (round to nearest even)
    auto split2 = [&](float x0, float x1, uint32_t& hi, uint32_t& lo) {
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        typedef float fl2 __attribute__((ext_vector_type(2)));
        const bf2 h = __builtin_convertvector(fl2{x0, x1}, bf2);
        hi = __builtin_bit_cast(uint32_t, h);
        const bf2 l = __builtin_convertvector(fl2{x0 - bf16_lo(hi), x1 - bf16_hi(hi)}, bf2);
        lo = __builtin_bit_cast(uint32_t, l);
    };

    // One pipeline step = one 32-token page pair.  On entry K of the pair has been requested
    // earlier and V is still in flight.  K of the following pair (of this item or of the wave's
    // next item) is requested as soon as the score MFMAs have consumed the K registers, V of the
    // following pair right after the output MFMAs.  Returns false when the wave's range is done.
    auto step = [&]() -> bool {
        f32x4 sx = {0.f, 0.f, 0.f, 0.f}, sy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const bf16x8 kx = __builtin_bit_cast(bf16x8, kr[0][s]), ky = __builtin_bit_cast(bf16x8, kr[1][s]);
            sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kx, qhi[s], sx, 0, 0, 0);
            sy = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ky, qhi[s], sy, 0, 0, 0);
            sx = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kx, qlo[s], sx, 0, 0, 0);
            sy = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ky, qlo[s], sy, 0, 0, 0);
        }
        // The following pair is requested unconditionally (branch-free, so that the K and V
        // requests can stay in flight across each other); past the end of the wave's range it
        // re-reads a valid pair that is never used.
        const bool more_pairs = pp + 1 < npairs;
        const int nrec = more_pairs ? rec : rec_n, nhead = more_pairs ? head : head_n, npp = more_pairs ? pp + 1 : 0;
        load_k(nrec, nhead, npp);

        // this lane: head c16, tokens tb + r (tile X) and tb + 4 + r (tile Y)
        const int tb = t0 + pp * 32 + (kq >> 1) * 16 + 8 * (kq & 1);
        float mloc = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            sx[r] = (tb + r < t1) ? sx[r] : -INFINITY;
            sy[r] = (tb + 4 + r < t1) ? sy[r] : -INFINITY;
            mloc = fmaxf(mloc, fmaxf(sx[r], sy[r]));
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run, mloc);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float p[8], psum = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            p[r] = __builtin_amdgcn_exp2f(sx[r] - m_new);
            p[4 + r] = __builtin_amdgcn_exp2f(sy[r] - m_new);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) psum += p[e];
        l_run = l_run * alpha + psum;
        u32x4 ph, pl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t hi, lo;
            split2(p[2 * e], p[2 * e + 1], hi, lo);
            ph[e] = hi;
            pl[e] = lo;
        }
        const bf16x8 phi = __builtin_bit_cast(bf16x8, ph), plo = __builtin_bit_cast(bf16x8, pl);
        // rescale O only when some head's running maximum moved (rare after the first pairs);
        // row (head) 4*kq + r of the output tile needs alpha of lane (head)
        if (__any(alpha != 1.f)) {
            float al[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) al[r] = __shfl(alpha, 4 * kq + r);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) O[b][r] *= al[r];
        }
        // pool slots past the end of the cache may hold anything: zero their V
        if (t0 + pp * 32 + 32 > t1) {
            const int vt = t0 + pp * 32 + (kq >> 1) * 16 + 8 * (kq & 1);
            uint32_t msk[4];
#pragma unroll
            for (int w = 0; w < 4; ++w)
                msk[w] = (vt + 2 * w < t1 ? 0x0000ffffu : 0u) | (vt + 2 * w + 1 < t1 ? 0xffff0000u : 0u);
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int w = 0; w < 4; ++w) vr[b][w] &= msk[w];
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const bf16x8 vt8 = __builtin_bit_cast(bf16x8, vr[b]);
            O[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(phi, vt8, O[b], 0, 0, 0);
            O[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(plo, vt8, O[b], 0, 0, 0);
        }
        load_v(nrec, nhead, npp);
        if (++pp < npairs) return true;

        float l_tot = l_run + __shfl_xor(l_run, 16);
        l_tot += __shfl_xor(l_tot, 32);
        float* pbase = a.partial + ((size_t)cidx * a.Hq + head * G) * (D + 2);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int g = 4 * kq + r;
            if (g < G) {
#pragma unroll
                for (int b = 0; b < NB; ++b) pbase[(size_t)g * (D + 2) + b * 16 + c16] = O[b][r];
            }
        }
        if (kq == 0 && c16 < G) {
            pbase[(size_t)c16 * (D + 2) + D] = m_run;
            pbase[(size_t)c16 * (D + 2) + D + 1] = l_tot;
        }
        if (item_n >= total_items) return false;
        item = item_n;
        item_n = next_item();
        rec = rec_n;
        req = __builtin_amdgcn_readlane(rec, 16);
        head = __builtin_amdgcn_readlane(rec, 17);
        t0 = __builtin_amdgcn_readlane(rec, 18);
        t1 = __builtin_amdgcn_readlane(rec, 19);
        cidx = __builtin_amdgcn_readlane(rec, 20);
        npairs = ((t1 - t0 + kPageTokens - 1) / kPageTokens + 1) / 2;
        pp = 0;
        rec_n = load_rec(item_n < total_items ? item_n : item);
        load_q(req, head);  // also drains every outstanding request before the steady state resumes
        head_n = __builtin_amdgcn_readlane(rec_n, 17);
#pragma unroll
        for (int b = 0; b < NB; ++b) O[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = -INFINITY;
        l_run = 0.f;
        return true;
    };

    while (step()) {
    }
}

// ---------------------------------------------------------------------------------
// split kernel, fp32 vector-ALU variant (parity configuration); one wave per item
// ---------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attn_split_f32_kernel(AttnArgs a, int G) {
    __shared__ float sc[8][CH];
    const int lane = threadIdx.x;
    const int total_items = a.chunk_off[a.batch] * a.Hkv;
    for (int item = blockIdx.x; item < total_items; item += gridDim.x) {
        const int32_t* rec = a.records + (size_t)item * kRecInts;
        const int req = rec[16], head = rec[17], t0 = rec[18], t1 = rec[19], chunk_idx = rec[20], cnt = t1 - t0;
        const int32_t* pt = a.page_tables + (size_t)req * a.max_pages;
        const uint16_t* kb = a.kbase + head * a.k_head;
        const uint16_t* vb = a.vbase + head * a.v_head;
        __syncthreads();
        // scores: lane <-> token
        for (int g = 0; g < G; ++g) {
            const float* qp = a.q + ((size_t)req * a.Hq + head * G + g) * D;
            for (int tt = lane; tt < cnt; tt += 64) {
                const int t = t0 + tt;
                const uint16_t* kr = kb + (int64_t)min(max(pt[t / kPageTokens], 0), a.n_pages - 1) * a.k_page + (t % kPageTokens) * D;
                float acc = 0.f;
                for (int j = 0; j < D; ++j) acc = fmaf(qp[j], bf16_bits_to_f32(kr[j]), acc);
                sc[g][tt] = acc * a.qscale;
            }
        }
        __syncthreads();
        float* pbase = a.partial + ((size_t)chunk_idx * a.Hq + head * G) * (D + 2);
        for (int g = 0; g < G; ++g) {
            float mx = -INFINITY;
            for (int tt = lane; tt < cnt; tt += 64) mx = fmaxf(mx, sc[g][tt]);
            mx = wave_max(mx);
            float sum = 0.f;
            for (int tt = lane; tt < cnt; tt += 64) {
                const float p = exp2f(sc[g][tt] - mx);
                sc[g][tt] = p;
                sum += p;
            }
            sum = wave_sum(sum);
            __syncthreads();
            // output: lane <-> dim
            for (int j = lane; j < D; j += 64) {
                float acc = 0.f;
                for (int tt = 0; tt < cnt; ++tt) {
                    const int t = t0 + tt;
                    const uint16_t* vr = vb + (int64_t)min(max(pt[t / kPageTokens], 0), a.n_pages - 1) * a.v_page + j * kPageTokens + (t % kPageTokens);
                    acc = fmaf(sc[g][tt], bf16_bits_to_f32(*vr), acc);
                }
                pbase[(size_t)g * (D + 2) + j] = acc;
            }
            if (lane == 0) {
                pbase[(size_t)g * (D + 2) + D] = mx;
                pbase[(size_t)g * (D + 2) + D + 1] = sum;
            }
        }
    }
}

template <int D>
static hipError_t launch_split_d(const AttnArgs& a, int G, int grid, hipStream_t st) {
    switch (G) {
#define SUN_CASE(g) \
    case g: hipLaunchKernelGGL((attn_split_kernel<D, g>), dim3(grid), dim3(512), 0, st, a); break;
        SUN_CASE(1) SUN_CASE(2) SUN_CASE(3) SUN_CASE(4) SUN_CASE(5) SUN_CASE(6) SUN_CASE(7) SUN_CASE(8)
#undef SUN_CASE
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attn_split(const KvPool& pool, int layer, const AttnPlan& plan, const float* q,
                             const int32_t* page_tables, int max_pages, const int32_t* n_or_len, int len_plus,
                             int batch, int total_chunks_hint, int full_chunks_hint, bool f32_exact, hipStream_t st) {
    const sun_model_cfg& c = pool.cfg;
    const sun_kv_layout& L = pool.lay;
    const int D = c.head_dim, G = c.n_q_heads / c.n_kv_heads;
    if (L.k_dim != 1 || L.k_token != D || L.v_token != 1 || L.v_dim != kPageTokens) return hipErrorInvalidValue;
    AttnArgs a{};
    a.kbase = pool.base + L.k_off + (int64_t)layer * L.k_layer;
    a.vbase = pool.base + L.v_off + (int64_t)layer * L.v_layer;
    a.k_page = L.k_page;
    a.k_head = L.k_head;
    a.v_page = L.v_page;
    a.v_head = L.v_head;
    a.q = q;
    a.page_tables = page_tables;
    a.n_or_len = n_or_len;
    a.chunk_off = plan.chunk_off;
    a.full_off = plan.full_off;
    a.records = plan.records;
    a.partial = plan.partial;
    a.len_plus = len_plus;
    a.max_pages = max_pages;
    a.batch = batch;
    a.Hq = c.n_q_heads;
    a.Hkv = c.n_kv_heads;
    a.n_pages = (int)L.n_pages;
    a.qscale = kLog2e / sqrtf((float)D);
    a.n_full_items = a.total_items = -1;
    const long long chunks = total_chunks_hint >= 0 ? total_chunks_hint : plan.max_chunks;
    const long long items = chunks * c.n_kv_heads;
    if (f32_exact) {
        if (G > 8) return hipErrorInvalidValue;
        const int grid = (int)max(1LL, min(items, 4096LL));
        if (D == 64) hipLaunchKernelGGL(attn_split_f32_kernel<64>, dim3(grid), dim3(64), 0, st, a, G);
        else if (D == 128) hipLaunchKernelGGL(attn_split_f32_kernel<128>, dim3(grid), dim3(64), 0, st, a, G);
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    // persistent workgroups of 8 waves, one per compute unit (fewer only when there are fewer
    // items than waves)
    // the item counts travel as kernel arguments when the host knows them: one dependent load less before a
    // wave's first request for K and V
    if (full_chunks_hint >= 0 && total_chunks_hint >= 0) {
        a.n_full_items = full_chunks_hint * c.n_kv_heads;
        a.total_items = total_chunks_hint * c.n_kv_heads;
    }
    const int grid = (int)max(1LL, min((items + 7) / 8, 256LL));
    if (D == 64) return launch_split_d<64>(a, G, grid, st);
    if (D == 128) return launch_split_d<128>(a, G, grid, st);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------
// combine: merge the chunk partials of a request in chunk order
// ---------------------------------------------------------------------------------
struct CombineArgs {
    const int32_t* chunk_off;
    const float* partial;
    float* out_f32;
    uint16_t* out_tiled;
    float* qscale;
    int Hq, D, batch, out_mb;
};

__global__ __launch_bounds__(128) void attn_combine_kernel(CombineArgs a) {
    const int b = blockIdx.y, col = blockIdx.x * 128 + threadIdx.x;
    const int h = col / a.D, j = col % a.D;
    const int c0 = a.chunk_off[b], c1 = a.chunk_off[b + 1];
    const size_t stride = (size_t)a.Hq * (a.D + 2);
    const float* p = a.partial + (size_t)c0 * stride + (size_t)h * (a.D + 2);
    // chunks are merged in order, eight at a time so that their loads are in flight together
    float M = -INFINITY, num = 0.f, den = 0.f;
    for (int cb = 0; cb < c1 - c0; cb += 8) {
        float m8[8], l8[8], o8[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c = min(cb + i, c1 - c0 - 1);
            m8[i] = p[c * stride + a.D];
            l8[i] = p[c * stride + a.D + 1];
            o8[i] = p[c * stride + j];
        }
        float Mn = M;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (cb + i < c1 - c0) Mn = fmaxf(Mn, m8[i]);
        const float sc = exp2f(M - Mn);
        num *= sc;
        den *= sc;
        M = Mn;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (cb + i < c1 - c0) {
                const float w = exp2f(m8[i] - M);
                den = fmaf(w, l8[i], den);
                num = fmaf(w, o8[i], num);
            }
    }
    const float v = num / den;
    if (a.out_f32) a.out_f32[(size_t)b * a.Hq * a.D + col] = v;
    if (a.out_tiled && !a.qscale) {
        uint16_t lo;
        const uint16_t hi = split_bf16(v, lo);
        a.out_tiled[atile_elem(ATile{a.out_mb}, 0, b, col)] = hi;
        a.out_tiled[atile_elem(ATile{a.out_mb}, 1, b, col)] = lo;
    }
    if (a.out_tiled && a.qscale) {
        // fixed-point tile of the 4-bit O projection: the workgroup's 128 columns are one group
        __shared__ float red_max[2];
        __shared__ int red_sum[2];
        const float wm = wave_max(fabsf(v));
        if ((threadIdx.x & 63) == 0) red_max[threadIdx.x >> 6] = wm;
        __syncthreads();
        const float am = fmaxf(red_max[0], red_max[1]);
        const int xi = (int)rintf(v * qtile_inv(am));
        const int l = ((xi + 128) & 255) - 128, hq = (xi - l) >> 8;
        uint8_t* tile = reinterpret_cast<uint8_t*>(a.out_tiled);
        tile[qtile_unit(ATile{a.out_mb}, 0, b, col >> 4) * 16 + (col & 15)] = (uint8_t)(hq & 255);
        tile[qtile_unit(ATile{a.out_mb}, 1, b, col >> 4) * 16 + (col & 15)] = (uint8_t)(l & 255);
        int sum = xi;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if ((threadIdx.x & 63) == 0) red_sum[threadIdx.x >> 6] = sum;
        __syncthreads();
        if (threadIdx.x == 0)
            reinterpret_cast<float2*>(a.qscale)[(size_t)blockIdx.x * (a.out_mb * 32) + b] =
                float2{am / kQMax, __int_as_float(red_sum[0] + red_sum[1])};
    }
}

hipError_t launch_attn_combine(const sun_model_cfg& cfg, const AttnPlan& plan, int batch, float* out_f32,
                               void* out_tiled, float* qscale, hipStream_t st) {
    CombineArgs a{};
    a.chunk_off = plan.chunk_off;
    a.partial = plan.partial;
    a.out_f32 = out_f32;
    a.out_tiled = (uint16_t*)out_tiled;
    a.qscale = qscale;
    a.Hq = cfg.n_q_heads;
    a.D = cfg.head_dim;
    a.batch = batch;
    a.out_mb = atile_for_rows(batch).MB;
    const int cols = cfg.n_q_heads * cfg.head_dim;
    if (cols % 128) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(cols / 128, batch), dim3(128), 0, st, a);
    return hipGetLastError();
}

}  // namespace sun
