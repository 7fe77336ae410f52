// Projections of the decode step: out[b, n] = sum_k W[n, k] x[b, k] for the skinny
// batch (b <= 256) against the shared decode weights (Section 3.1, Eq. 3), and the
// QSUN variant with W_hat = (Q - Z) * S, 4-bit codes in groups of 128 along k
// (Section 3.3, Eq. 8; Appendix A.1).
//
// bf16 path: each weight byte is read from HBM once.  Weights are pre-tiled so that a
// wave's 16-byte-per-lane load is 1 KiB contiguous and already is the B operand of a
// 32x32x16 MFMA (lane n%32 <-> weight row, lane half <-> k octet).  Activations are
// pre-tiled by their producer, staged through LDS (double buffered) and shared by the
// waves of a workgroup; wave w owns 32 output columns and all batch rows.
//
// W4 path (proj_w4_kernel): the codes stay integers.  Activations arrive as 16-bit fixed point in two
// int8 planes with one scale per row and group (see common.hpp), the 4-bit codes are widened to bytes
// (an and, a shift-and per four codes) and both go through the 32x32x32 int8 MFMA, whose int32 sums
// are exact.  Per 128-wide group:  acc += (S * sx) * (256 * sum_k q_k hi_k + sum_k q_k lo_k - Z * sum_k xi_k),
// which is sum_k (q_k - Z) S (sx xi_k) up to the rounding of one int -> fp32 conversion and one fma.
#include <hip/hip_fp16.h>

#include <type_traits>

#include "kernels.hpp"

namespace sun {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct ProjArgs {
    const u32x4* W;
    const uint32_t* SZ;
    int s_only;    // W4: SZ holds fp16 scales only, two 128-wide groups per dword; the zero point is 8 everywhere
    const u32x4* A;
    const float* qscale;
    float* out;
    int rows, N, K;
    int n_stages, stages_per_split;
    int ldo, ld_rows;
    int mb_rows;   // 32-row blocks of real rows in the activation tiling (it holds twice as many: hi and lo plane)
};

// MB counts the 32-row operand blocks of the workgroup: MR = MB/2 blocks of rows, each present
// as a hi and a lo bf16 plane (operand block m < MR is the hi plane of row block m, block MR+m
// its lo plane); both are multiplied with the same weight fragment into the same accumulator.
template <int MB, int KS, int NW, int EPI, int NBUF>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2)))
void proj_kernel(ProjArgs a) {
    constexpr int MR = MB / 2;
    static_assert(MB % 2 == 0, "operand blocks come in hi/lo pairs");
    constexpr int KK = KS / 16;                // MFMA k-steps per stage
    constexpr int STAGE_UNITS = KK * MB * 64;  // 16-byte units of activations per stage
    constexpr int NT = NW * 64;
    constexpr int UPT = (STAGE_UNITS + NT - 1) / NT;  // the last round of a stage may be partial
    constexpr int WREGS = KK;                  // 16-byte weight loads per lane per stage

    __shared__ u32x4 lds[NBUF][STAGE_UNITS];  // ring of staged activation tiles (prefetch distance NBUF-1)

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5;
    const int nb = blockIdx.x * NW + wave;
    const bool active = nb < a.N / 32;
    const int split = blockIdx.y;
    const int mb_off = blockIdx.z * MR;  // first row block of this workgroup
    const int s0 = split * a.stages_per_split;
    const int s1 = min(a.n_stages, s0 + a.stages_per_split);
    const int kch = a.K / 128;

    // waves past the last column block work on block 0 and drop their result (keeps the loop branch-free)
    const u32x4* Wl = a.W + ((size_t)(active ? nb : 0) * kch) * 8 * 64 + lane;

    f32x16 acc[MR];
#pragma unroll
    for (int m = 0; m < MR; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;

    u32x4 w0[WREGS], w1[WREGS], w2[NBUF == 3 ? WREGS : 1], areg[UPT];

    auto load_w = [&](u32x4(&w)[WREGS], int st) {
#pragma unroll
        for (int j = 0; j < WREGS; ++j) w[j] = Wl[((size_t)st * WREGS + j) * 64];
    };
    auto load_a = [&](int st) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = min(i * NT + tid, STAGE_UNITS - 1);  // past the stage: re-read its last unit, never stored
            const int kk = u / (MB * 64), rem = u % (MB * 64);
            const int m = rem >> 6;  // operand block: hi plane of row block m, or lo plane of row block m - MR
            const int gb = m < MR ? mb_off + m : a.mb_rows + mb_off + (m - MR);
            areg[i] = a.A[((size_t)(st * KK + kk) * (2 * a.mb_rows) + gb) * 64 + (rem & 63)];
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < UPT; ++i)
            if (STAGE_UNITS % NT == 0 || i * NT + tid < STAGE_UNITS) lds[buf][i * NT + tid] = areg[i];
    };
    auto compute = [&](int buf, const u32x4(&w)[WREGS]) {
        // A operands are read from LDS one k-step ahead of the MFMAs that use them; the 128-row
        // kernel reads them just in time instead: with the second fragment set it would not fit two
        // waves per SIMD, and the second wave hides more latency than the early read
        constexpr int AF = MB == 8 ? 1 : 2;
        u32x4 afr[AF][MB];
        if constexpr (AF == 2) {
#pragma unroll
            for (int m = 0; m < MB; ++m) afr[0][m] = lds[buf][m * 64 + lane];
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if constexpr (AF == 2) {
                if (kk + 1 < KK) {
#pragma unroll
                    for (int m = 0; m < MB; ++m) afr[(kk + 1) & 1][m] = lds[buf][((kk + 1) * MB + m) * 64 + lane];
                }
            } else {
#pragma unroll
                for (int m = 0; m < MB; ++m) afr[0][m] = lds[buf][(kk * MB + m) * 64 + lane];
            }
            __builtin_amdgcn_sched_barrier(0);
            const bf16x8 bfrag = __builtin_bit_cast(bf16x8, w[kk]);
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)  // hi plane, then lo plane, into the same accumulators
#pragma unroll
                for (int m = 0; m < MR; ++m) {
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, afr[kk & (AF - 1)][pl * MR + m]);
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag, acc[m], 0, 0, 0);
                }
        }
    };

    // Steady state without branches around the loads, so that the requests of the following
    // stages stay in flight while this stage is computed; past the end the last stage is
    // re-read and never used.
    if (s0 < s1) {
        if constexpr (NBUF == 3) {
            auto phase = [&](const u32x4(&wc)[WREGS], u32x4(&wn)[WREGS], int bufc, int bufn, int st) {
                const int nx = min(st + 2, s1 - 1);
                load_a(nx);  // before the weights: the LDS store below then waits for these only
                load_w(wn, nx);
                compute(bufc, wc);
                store_a(bufn);
                __syncthreads();
            };
            const int sA = min(s0 + 1, s1 - 1);
            load_w(w0, s0);
            load_a(s0);
            store_a(0);
            load_w(w1, sA);
            load_a(sA);
            store_a(1);
            __syncthreads();
            for (int st = s0; st < s1; st += 3) {
                phase(w0, w2, 0, 2, st);
                if (st + 1 >= s1) break;
                phase(w1, w0, 1, 0, st + 1);
                if (st + 2 >= s1) break;
                phase(w2, w1, 2, 1, st + 2);
            }
        } else {
            load_w(w0, s0);
            load_a(s0);
            store_a(0);
            __syncthreads();
            for (int st = s0; st < s1; st += 2) {
                const int n1 = min(st + 1, s1 - 1);
                load_a(n1);
                load_w(w1, n1);
                compute(0, w0);
                store_a(1);
                __syncthreads();
                if (st + 1 >= s1) break;
                const int n2 = min(st + 2, s1 - 1);
                load_a(n2);
                load_w(w0, n2);
                compute(1, w1);
                store_a(0);
                __syncthreads();
            }
        }
    }
    if (!active) return;

    const int col = lane & 31;
    if constexpr (EPI == EPI_SWIGLU) {
        // The wave's 32 columns are 16 gate columns followed by the 16 up columns of the same u columns (the
        // packing order of the pair): lane c < 16 fetches its up value from lane c + 16 and owns u column
        // nb*16 + c.  The results leave as the tile the down projection reads: hi and lo plane, 16-byte units
        // of 8 consecutive u columns of one row, gathered through the wave's own piece of the (now idle)
        // activation ring.  Every wave has passed the barrier that follows the last stage.
        uint16_t* sw = reinterpret_cast<uint16_t*>(&lds[0][0]) + (size_t)wave * (MR * 32 * 16 * 2);
#pragma unroll
        for (int m = 0; m < MR; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float g = acc[m][r];
                const float up = __shfl_xor(g, 16);
                const float y = g / (1.f + __expf(-g)) * up;
                const uint16_t hi = f32_to_bf16_bits(y);
                const uint16_t lo = f32_to_bf16_bits(y - bf16_bits_to_f32(hi));
                const int rl = m * 32 + 8 * (r >> 2) + 4 * half + (r & 3);  // row inside the workgroup's tile
                if (col < 16) {
                    sw[(0 * MR * 32 + rl) * 16 + col] = hi;
                    sw[(1 * MR * 32 + rl) * 16 + col] = lo;
                }
            }
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's LDS writes have landed (no other wave reads them)
        __builtin_amdgcn_wave_barrier();
        u32x4* tile = reinterpret_cast<u32x4*>(a.out);
#pragma unroll
        for (int i = 0; i < MR * 2; ++i) {       // MR*32 rows x 2 units x 2 planes = MR*128 units, 64 lanes
            const int idx = i * 64 + lane;
            const int plane = idx / (MR * 64), rem = idx % (MR * 64), rl = rem >> 1, un = rem & 1;
            const int b = mb_off * 32 + rl;
            const u32x4 v = *reinterpret_cast<const u32x4*>(sw + ((size_t)plane * MR * 32 + rl) * 16 + un * 8);
            if (b < a.rows) tile[atile_unit(ATile{a.mb_rows}, plane, b, nb * 2 + un)] = v;
        }
    } else {
        float* o = a.out + (size_t)split * a.ld_rows * a.ldo + nb * 32 + col;
#pragma unroll
        for (int m = 0; m < MR; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int b = (mb_off + m) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                if (b < a.rows) o[(size_t)b * a.ldo] = acc[m][r];
            }
    }
}

// ---------------------------------------------------------------------------------
// bf16 weights, more than 128 rows
// ---------------------------------------------------------------------------------
// Above 64 rows the projection is no longer bound by the weight stream, and the workgroup shape above would
// be bound by LDS just as much: there every operand fragment read from LDS feeds one matrix
// instruction (1 KiB per 32 cycles and SIMD = the 128 bytes per cycle the LDS delivers).  Here a
// wave owns 64 columns (two strips), so a fragment of the activations feeds two instructions.
// A workgroup is eight waves, two per SIMD, and covers 256 columns and 64 * MRW rows: wave (c, h)
// owns column pair c and row group h (MRW row blocks of 32; 2 in every launch: 128-row
// workgroups).  The two row groups of a column pair request the same weights (HBM sees them once).
// The activation stage is 64 wide (four k-steps) and shared by all waves.
// Used above 128 rows.  Up to 128 rows the strip kernel stays (measured on the 14B shape at batch
// 128: gate/up 103 against 119 us, the rest equal).  A variant with four waves of 128 rows x 64
// columns, one per SIMD with its accumulators in the upper half of the register file, requests no
// weight twice but was 10 to 90 % slower: one wave per SIMD cannot cover its own waits.
template <int MRW, int EPI>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void proj_tall_kernel(ProjArgs a) {
    constexpr int RH = 2, NWC = 4;             // row groups and column pairs of a workgroup
    constexpr int MRT = RH * MRW;              // row blocks of the workgroup
    constexpr int MB = 2 * MRT;                // operand blocks of a k-step in LDS: hi planes, then lo planes
    constexpr int KK = 4;                      // k-steps per stage (64 of k)
    constexpr int STAGE_UNITS = KK * MB * 64;
    constexpr int NT = RH * NWC * 64;
    constexpr int NBUF = (MRT <= 2) ? 3 : 2;   // a third weight stage in registers does not fit beside 64 + 64 accumulators
    constexpr int UPT = (STAGE_UNITS + NT - 1) / NT;
    static_assert(STAGE_UNITS % NT == 0, "every thread stages the same number of units");
    __shared__ u32x4 lds_all[NBUF * STAGE_UNITS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5;
    const int wc = wave % NWC, rh = wave / NWC;
    const int cp = blockIdx.x * NWC + wc;      // column pair: strips 2 cp and 2 cp + 1
    const int n_strips = a.N / 32;
    const bool act0 = 2 * cp < n_strips, act1 = 2 * cp + 1 < n_strips;
    const int split = blockIdx.y;
    const int mb_off = blockIdx.z * MRT;       // first row block of this workgroup
    const int s0 = split * a.stages_per_split;
    const int s1 = min(a.n_stages, s0 + a.stages_per_split);
    const int kch = a.K / 128;

    // a stage is half a 128-wide chunk of the packed weights: four of its eight k-steps
    const u32x4* Wl0 = a.W + ((size_t)(act0 ? 2 * cp : 0) * kch) * 8 * 64 + lane;
    const u32x4* Wl1 = a.W + ((size_t)(act1 ? 2 * cp + 1 : 0) * kch) * 8 * 64 + lane;

    f32x16 acc[2][MRW];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int m = 0; m < MRW; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[s][m][r] = 0.f;

    u32x4 w0[2][KK], w1[2][KK], w2[NBUF == 3 ? 2 : 1][NBUF == 3 ? KK : 1], areg[UPT];

    auto load_w = [&](u32x4(&w)[2][KK], int st) {
        const size_t off = ((size_t)st * KK) * 64;   // in k-steps of 64 lanes
#pragma unroll
        for (int j = 0; j < KK; ++j) {
            w[0][j] = Wl0[off + (size_t)j * 64];
            w[1][j] = Wl1[off + (size_t)j * 64];
        }
    };
    auto load_a = [&](int st) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = i * NT + tid;
            const int kk = u / (MB * 64), rem = u % (MB * 64);
            const int m = rem >> 6;  // operand block: hi plane of row block m, or lo plane of row block m - MRT
            const int gb = m < MRT ? mb_off + m : a.mb_rows + mb_off + (m - MRT);
            areg[i] = a.A[((size_t)(st * KK + kk) * (2 * a.mb_rows) + gb) * 64 + (rem & 63)];
        }
    };
    auto store_a = [&](int buf) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) lds_all[buf * STAGE_UNITS + i * NT + tid] = areg[i];
    };
    auto compute = [&](int buf, const u32x4(&w)[2][KK]) {
        // this wave's operand blocks of a k-step: hi and lo plane of its MRW row blocks
        const u32x4* src = lds_all + buf * STAGE_UNITS + lane;
        u32x4 afr[2][2 * MRW];
        auto read_a = [&](int kk, u32x4(&dst)[2 * MRW]) {
#pragma unroll
            for (int pl = 0; pl < 2; ++pl)
#pragma unroll
                for (int m = 0; m < MRW; ++m) dst[pl * MRW + m] = src[(kk * MB + pl * MRT + rh * MRW + m) * 64];
        };
        read_a(0, afr[0]);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk + 1 < KK) read_a(kk + 1, afr[(kk + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 bfrag = __builtin_bit_cast(bf16x8, w[s][kk]);
#pragma unroll
                for (int pl = 0; pl < 2; ++pl)  // hi plane, then lo plane, into the same accumulators
#pragma unroll
                    for (int m = 0; m < MRW; ++m) {
                        const bf16x8 afrag = __builtin_bit_cast(bf16x8, afr[kk & 1][pl * MRW + m]);
                        acc[s][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag, acc[s][m], 0, 0, 0);
                    }
            }
        }
    };

    if (s0 < s1) {
        if constexpr (NBUF == 3) {
            auto phase = [&](const u32x4(&wcur)[2][KK], u32x4(&wn)[2][KK], int bufc, int bufn, int st) {
                const int nx = min(st + 2, s1 - 1);
                load_a(nx);  // before the weights: the LDS store below then waits for these only
                load_w(wn, nx);
                compute(bufc, wcur);
                store_a(bufn);
                __syncthreads();
            };
            const int sA = min(s0 + 1, s1 - 1);
            load_w(w0, s0);
            load_a(s0);
            store_a(0);
            load_w(w1, sA);
            load_a(sA);
            store_a(1);
            __syncthreads();
            for (int st = s0; st < s1; st += 3) {
                phase(w0, w2, 0, 2, st);
                if (st + 1 >= s1) break;
                phase(w1, w0, 1, 0, st + 1);
                if (st + 2 >= s1) break;
                phase(w2, w1, 2, 1, st + 2);
            }
        } else {
            load_w(w0, s0);
            load_a(s0);
            store_a(0);
            __syncthreads();
            for (int st = s0; st < s1; st += 2) {
                const int n1 = min(st + 1, s1 - 1);
                load_a(n1);
                load_w(w1, n1);
                compute(0, w0);
                store_a(1);
                __syncthreads();
                if (st + 1 >= s1) break;
                const int n2 = min(st + 2, s1 - 1);
                load_a(n2);
                load_w(w0, n2);
                compute(1, w1);
                store_a(0);
                __syncthreads();
            }
        }
    }

    const int col = lane & 31;
    if constexpr (EPI == EPI_SWIGLU) {
        // A strip's 32 columns are 16 gate columns followed by the 16 up columns of the same u columns (the
        // packing order of the pair): lane c < 16 fetches its up value from lane c + 16 and owns u column
        // strip*16 + c.  The results leave as the tile the down projection reads: hi and lo plane, 16-byte units
        // of 8 consecutive u columns of one row, gathered through the wave's own piece of the (now idle)
        // activation ring.  Every wave has passed the barrier that follows the last stage.
        uint16_t* sw = reinterpret_cast<uint16_t*>(lds_all) + (size_t)wave * (MRW * 32 * 16 * 2);
        u32x4* tile = reinterpret_cast<u32x4*>(a.out);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int nb = 2 * cp + s;
#pragma unroll
            for (int m = 0; m < MRW; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float g = acc[s][m][r];
                    const float up = __shfl_xor(g, 16);
                    const float y = g / (1.f + __expf(-g)) * up;
                    const uint16_t hi = f32_to_bf16_bits(y);
                    const uint16_t lo = f32_to_bf16_bits(y - bf16_bits_to_f32(hi));
                    const int rl = m * 32 + 8 * (r >> 2) + 4 * half + (r & 3);  // row inside the wave's rows
                    if (col < 16) {
                        sw[(0 * MRW * 32 + rl) * 16 + col] = hi;
                        sw[(1 * MRW * 32 + rl) * 16 + col] = lo;
                    }
                }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the wave's LDS writes have landed (no other wave reads them)
            __builtin_amdgcn_wave_barrier();
            if (nb < n_strips) {
#pragma unroll
                for (int i = 0; i < MRW * 2; ++i) {       // MRW*32 rows x 2 units x 2 planes = MRW*128 units, 64 lanes
                    const int idx = i * 64 + lane;
                    const int plane = idx / (MRW * 64), rem = idx % (MRW * 64), rl = rem >> 1, un = rem & 1;
                    const int b = (mb_off + rh * MRW) * 32 + rl;
                    const u32x4 v = *reinterpret_cast<const u32x4*>(sw + ((size_t)plane * MRW * 32 + rl) * 16 + un * 8);
                    if (b < a.rows) tile[atile_unit(ATile{a.mb_rows}, plane, b, nb * 2 + un)] = v;
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // the reads are done before the second strip overwrites the piece
            __builtin_amdgcn_wave_barrier();
        }
    } else {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int nb = 2 * cp + s;
            if (nb >= n_strips) continue;
            float* o = a.out + (size_t)split * a.ld_rows * a.ldo + nb * 32 + col;
#pragma unroll
            for (int m = 0; m < MRW; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int b = (mb_off + rh * MRW + m) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                    if (b < a.rows) o[(size_t)b * a.ldo] = acc[s][m][r];
                }
        }
    }
}

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));

// 4-bit weights: MR 32-row blocks per workgroup (the launches use MR = 1: 32-row tiles, see proj_tiling), one
// stage = one 128-wide group = four int8 MFMA k-steps, three stages of activations in the LDS ring.
template <int MR, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, MR == 1 ? 4 : 2)))
void proj_w4_kernel(ProjArgs a) {
    constexpr int STEPS = 4;
    constexpr int STAGE_UNITS = STEPS * 2 * MR * 64;  // 16-byte units of activations per stage (two planes)
    constexpr int NT = NW * 64;
    constexpr int UPT = (STAGE_UNITS + NT - 1) / NT;
    __shared__ u32x4 lds[3][STAGE_UNITS];
    __shared__ __attribute__((aligned(16))) float sx_lds[4][MR * 32];  // ring over groups: scale of each row ...
    __shared__ __attribute__((aligned(16))) int xs_lds[4][MR * 32];    // ... and its sum of integers

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5;
    const int nb = blockIdx.x * NW + wave;
    const bool active = nb < a.N / 32;
    const int split = blockIdx.y;
    const int mb_off = blockIdx.z * MR;
    const int s0 = split * a.stages_per_split;
    const int s1 = min(a.n_stages, s0 + a.stages_per_split);
    const int kch = a.K / 128;

    // waves past the last column block work on block 0 and drop their result (keeps the loop branch-free)
    const u32x4* Wl = a.W + ((size_t)(active ? nb : 0) * kch) * 2 * 64 + lane;
    const uint32_t* SZl = a.SZ + ((size_t)(active ? nb : 0) * (a.s_only ? (kch + 1) >> 1 : kch)) * 32 + (lane & 31);
    const float2* QS = reinterpret_cast<const float2*>(a.qscale);

    f32x16 acc[MR];
    i32x16 ih[MR], il[MR];
#pragma unroll
    for (int m = 0; m < MR; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;

    u32x4 w0[2], w1[2], w2[2], areg[UPT];
    uint32_t sz0 = 0, sz1 = 0, sz2 = 0;
    float2 qreg = float2{0.f, 0.f};

    auto load_w = [&](u32x4(&w)[2], uint32_t& sz, int st) {
        w[0] = Wl[((size_t)st * 2) * 64];
        w[1] = Wl[((size_t)st * 2 + 1) * 64];
        sz = SZl[(size_t)(a.s_only ? st >> 1 : st) * 32];
    };
    auto load_a = [&](int st) {
#pragma unroll
        for (int i = 0; i < UPT; ++i) {
            const int u = min(i * NT + tid, STAGE_UNITS - 1);  // past the stage: re-read its last unit, never stored
            const int sp = u / (MR * 64), rem = u % (MR * 64);  // sp = step * 2 + plane
            areg[i] = a.A[((size_t)(st * 8 + sp) * a.mb_rows + mb_off + (rem >> 6)) * 64 + (rem & 63)];
        }
        if (tid < MR * 32) qreg = QS[(size_t)st * (a.mb_rows * 32) + mb_off * 32 + tid];
    };
    auto store_a = [&](int buf, int st) {
#pragma unroll
        for (int i = 0; i < UPT; ++i)
            if (STAGE_UNITS % NT == 0 || i * NT + tid < STAGE_UNITS) lds[buf][i * NT + tid] = areg[i];
        if (tid < MR * 32) {
            sx_lds[st & 3][tid] = qreg.x;
            xs_lds[st & 3][tid] = __float_as_int(qreg.y);
        }
    };
    auto compute = [&](int buf, const u32x4(&w)[2], uint32_t sz, int st) {
        u32x4 afr[2][2 * MR];  // operands of one k-step (both planes), read one step ahead
#pragma unroll
        for (int i = 0; i < 2 * MR; ++i) afr[0][i] = lds[buf][i * 64 + lane];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            if (s + 1 < STEPS) {
#pragma unroll
                for (int i = 0; i < 2 * MR; ++i) afr[(s + 1) & 1][i] = lds[buf][((s + 1) * 2 * MR + i) * 64 + lane];
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint32_t wa = w[s >> 1][(s & 1) * 2], wb = w[s >> 1][(s & 1) * 2 + 1];
            const i32x4 bfrag = {(int)(wa & 0x0F0F0F0Fu), (int)((wa >> 4) & 0x0F0F0F0Fu), (int)(wb & 0x0F0F0F0Fu),
                                 (int)((wb >> 4) & 0x0F0F0F0Fu)};
#pragma unroll
            for (int m = 0; m < MR; ++m) {
                const i32x4 ah = __builtin_bit_cast(i32x4, afr[s & 1][m]), al = __builtin_bit_cast(i32x4, afr[s & 1][MR + m]);
                if (s == 0) {
                    i32x16 zero;
#pragma unroll
                    for (int r = 0; r < 16; ++r) zero[r] = 0;
                    ih[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bfrag, zero, 0, 0, 0);
                    il[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bfrag, zero, 0, 0, 0);
                } else {
                    ih[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ah, bfrag, ih[m], 0, 0, 0);
                    il[m] = __builtin_amdgcn_mfma_i32_32x32x32_i8(al, bfrag, il[m], 0, 0, 0);
                }
            }
        }
        // scale-only layout: pick this group's half of the dword; the zero point is 8 everywhere
        const uint32_t szg = a.s_only ? (((sz >> (16 * (st & 1))) & 0xffffu) | 0x48000000u) : sz;
        const __half2 h2 = __builtin_bit_cast(__half2, szg);
        const float sc = __low2float(h2);
        const int nzi = -(int)__high2float(h2);  // zero points are integer codes (Appendix A.1)
        const float* sxp = sx_lds[st & 3];
        const int* xsp = xs_lds[st & 3];
#pragma unroll
        for (int m = 0; m < MR; ++m)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const f32x4 sx4 = *reinterpret_cast<const f32x4*>(sxp + m * 32 + 8 * rr + 4 * half);
                const i32x4 xs4 = *reinterpret_cast<const i32x4*>(xsp + m * 32 + 8 * rr + 4 * half);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int e = rr * 4 + q;
                    int tot = (ih[m][e] << 8) + il[m][e];
                    asm("v_mad_i32_i24 %0, %1, %2, %0" : "+v"(tot) : "v"(nzi), "v"(xs4[q]));  // tot -= Z * sum xi, one instruction
                    acc[m][e] = fmaf((float)tot, sc * sx4[q], acc[m][e]);
                }
            }
    };

    // Steady state without branches around the loads, so that the requests of the following stages stay in
    // flight while this stage is computed; past the end the last stage is re-read and never used.
    if (s0 < s1) {
        auto phase = [&](const u32x4(&wc)[2], uint32_t szc, u32x4(&wn)[2], uint32_t& szn, int bufc, int bufn, int st) {
            const int nx = min(st + 2, s1 - 1);
            load_a(nx);  // before the weights: the LDS store below then waits for these only
            load_w(wn, szn, nx);
            compute(bufc, wc, szc, st);
            store_a(bufn, nx);
            __syncthreads();
        };
        const int sA = min(s0 + 1, s1 - 1);
        load_w(w0, sz0, s0);
        load_a(s0);
        store_a(0, s0);
        load_w(w1, sz1, sA);
        load_a(sA);
        store_a(1, sA);
        __syncthreads();
        for (int st = s0; st < s1; st += 3) {
            phase(w0, sz0, w2, sz2, 0, 2, st);
            if (st + 1 >= s1) break;
            phase(w1, sz1, w0, sz0, 1, 0, st + 1);
            if (st + 2 >= s1) break;
            phase(w2, sz2, w1, sz1, 2, 1, st + 2);
        }
    }
    if (!active) return;
    const int col = lane & 31;
    float* o = a.out + (size_t)split * a.ld_rows * a.ldo + nb * 32 + col;
#pragma unroll
    for (int m = 0; m < MR; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int b = (mb_off + m) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (b < a.rows) o[(size_t)b * a.ldo] = acc[m][r];
        }
}

template <int MR>
static hipError_t launch_proj_w4(const ProjArgs& a, int nw, int splits, int mtiles, hipStream_t st) {
    const auto go = [&](auto nwc) {
        constexpr int NW = decltype(nwc)::value;
        dim3 grid((a.N / 32 + NW - 1) / NW, splits, mtiles), block(NW * 64);
        hipLaunchKernelGGL((proj_w4_kernel<MR, NW>), grid, block, 0, st, a);
        return hipGetLastError();
    };
    switch (nw) {
    case 4: return go(std::integral_constant<int, 4>{});
    case 5: return go(std::integral_constant<int, 5>{});
    case 6: return go(std::integral_constant<int, 6>{});
    case 7: return go(std::integral_constant<int, 7>{});
    }
    return hipErrorInvalidValue;
}

template <int MB, int KS, int NW = 4>
static hipError_t launch_proj_t(const ProjArgs& a, int epilogue, int splits, int mtiles, hipStream_t st) {
    constexpr int NBUF = (MB * KS * 64 * 3 <= 49152) ? 3 : 2;  // LDS ring: 3 stages when they fit in 48 KB
    dim3 grid((a.N / 32 + NW - 1) / NW, splits, mtiles), block(NW * 64);
    if (epilogue == EPI_SWIGLU) {
        if (splits != 1) return hipErrorInvalidValue;
        hipLaunchKernelGGL((proj_kernel<MB, KS, NW, EPI_SWIGLU, NBUF>), grid, block, 0, st, a);
        return hipGetLastError();
    }
    if (epilogue != EPI_STORE) return hipErrorInvalidValue;
    hipLaunchKernelGGL((proj_kernel<MB, KS, NW, EPI_STORE, NBUF>), grid, block, 0, st, a);
    return hipGetLastError();
}

static hipError_t launch_proj_tall(const ProjArgs& a, int epilogue, int splits, int mtiles, hipStream_t st) {
    const int pairs = (a.N / 32 + 1) / 2;
    dim3 grid((pairs + 3) / 4, splits, mtiles);
    if (epilogue == EPI_SWIGLU) {
        if (splits != 1) return hipErrorInvalidValue;
        hipLaunchKernelGGL((proj_tall_kernel<2, EPI_SWIGLU>), grid, dim3(512), 0, st, a);
        return hipGetLastError();
    }
    if (epilogue != EPI_STORE) return hipErrorInvalidValue;
    hipLaunchKernelGGL((proj_tall_kernel<2, EPI_STORE>), grid, dim3(512), 0, st, a);
    return hipGetLastError();
}

// Split-K factor of the launch above 128 rows (bf16; workgroups of 128 rows x 256 columns).  All workgroups do
// equal work and one round of at most 256 of them is wanted: the largest split that stays within the round
// (each split costs a slab of partial sums, but the matrix-core time of a workgroup goes with its stages;
// measured on the 8B shape at 256 rows: qkv 5 splits 32.7 us against 37.7 with 4, down 8 against 4: 64 / 125).
static int tall_pick_splits(const Mat& W, int rows, int max_splits) {
    const int pairs = (W.N / 32 + 1) / 2, stages = W.K / 64, colwgs = (pairs + 3) / 4;
    const int mtiles = (atile_for_rows(rows).MB + 3) / 4;
    int best = 1;
    for (int s = 1; s <= max(1, min(max_splits, stages / 4)); ++s) {
        const int sps = (stages + s - 1) / s;
        if ((stages + sps - 1) / sps != s) continue;
        if ((long long)colwgs * mtiles * s <= 256) best = s;
    }
    return best;
}

static int chunks_per_split(int kch, int splits) { return (kch + splits - 1) / splits; }

// Waves per workgroup (each wave owns 32 columns) and split-K factor.  A compute unit's share of
// the HBM bandwidth does not grow with the number of workgroups it hosts, so the launch is only
// as fast as the most loaded unit: the pair is chosen to spread the weight bytes evenly over the
// 256 compute units (N = 6144 -> 6 waves x 8 splits, N = 28672 -> 7 waves x 2 splits, ...), with a
// fixed charge per workgroup for filling and draining its pipeline.  Depends on the matrix and the
// row-count class only.  The bf16 kernel above 64 rows keeps 4 waves; 4-bit launches of several row tiles have
// a rule of their own (w4_tiles_pick).
struct ProjShape {
    int nw, splits;
};
// Row tiling: operand blocks per workgroup (2 planes x 32-row blocks) and row tiles per launch.
// bf16 weights: up to 64 rows one tile holds all rows; above, 128-row tiles (every tile streams the
// weights from HBM again).  4-bit weights: 32-row tiles at every batch size.  Their kernel is bound by
// its vector-ALU epilogue and by the wait for the matrix cores between epilogues, not by the weight
// stream (a quarter of the bytes, and the row tiles of a column strip run side by side and share
// their fetches); with one row block a wave needs 128 registers instead of 230, four waves share a
// SIMD instead of two and cover each other's waits (8B shape, qkv / o / gate-up / down in us: batch 64
// 16.2 / 11.9 / 32.7 / 21.6 -> 15.0 / 11.1 / 30.0 / 20.5; batch 256 30.9 / 22.7 / 104.6 / 60.2 -> 27.8 / 20.6 /
// 90.9 / 50.7; results bit-identical).
struct ProjTiling {
    int mb, mtiles;
};
static ProjTiling proj_tiling(const Mat& W, int rows) {
    const int mbr = atile_for_rows(rows).MB;  // 32-row blocks of the activation tiling: 1, 2, 4 or 8
    if (W.kind == MAT_W4_PACKED) return ProjTiling{2, mbr};
    if (mbr <= 2) return ProjTiling{2 * mbr, 1};
    return ProjTiling{8, mbr / 4};
}
static long long proj_cost(int strips, int kch, int mtiles, int nw, int s) {
    const int cps = chunks_per_split(kch, s), real_s = (kch + cps - 1) / cps;
    const long long wgs = (long long)((strips + nw - 1) / nw) * real_s * mtiles;
    const long long rounds = (wgs + 255) / 256;
    return rounds * ((long long)nw * cps + 6) * 16 + real_s;  // ties: fewer splits
}
// 4-bit weights with more than one 32-row tile: several workgroups share a compute unit (16 waves at 128
// registers), so the launch wants two to four times 256 workgroups rather than exactly 256.  Four waves per
// workgroup (seven for a matrix of 512 strips or more while there are only two row tiles), and the smallest
// split into equal shares that gives at least 512 workgroups without leaving a workgroup more than 32 stages.  Measured on the 8B
// shape (us, best of the shapes tried): batch 64 qkv 4 x 8: 13.5 (6 x 8: 14.7, 4 x 4: 15.3), o 4 x 8: 10.8
// (4 x 4: 12.0, 4 x 16: 12.6), gate/up 7 x 2: 30.0 (4 x 2: 31.8, 7 x 1: 35.6), down 4 x 8: 19.7 (4 x 4: 26.8);
// batch 256 qkv 4 x 2: 25.8 (4 x 4: 27.5, 4 x 8: 30.3), o 4 x 4: 20.4, gate/up 4 x 1: 92.4 (4 x 2: 95.4, 4 x 4: 105),
// down 4 x 4: 49.4 (4 x 2: 52.4, 4 x 8: 51.3).
static ProjShape w4_tiles_pick(const Mat& W, int mtiles, int max_splits) {
    const int strips = W.N / 32, kch = W.K / 128;
    const int nw = (strips >= 512 && mtiles <= 2) ? 7 : 4;
    const long long colwgs = (strips + nw - 1) / nw;
    ProjShape best{nw, 1};
    for (int s = 1; s <= max(1, min(max_splits, kch / 2)); ++s) {
        if (kch % s) continue;  // equal shares only: the launch ends with its longest workgroup
        best = ProjShape{nw, s};
        if (colwgs * mtiles * s >= 448 && kch / s <= 32) break;  // "at least 512", with a little give
    }
    return best;
}
static ProjShape proj_pick(const Mat& W, int rows, int max_splits) {
    const int strips = W.N / 32, kch = W.K / 128;
    const ProjTiling t = proj_tiling(W, rows);
    const int mtiles = t.mtiles;
    if (W.kind == MAT_W4_PACKED && mtiles >= 2) return w4_tiles_pick(W, mtiles, max_splits);
    const int smax = max(1, min(max_splits, kch / 2));
    ProjShape best{4, 1};
    long long best_cost = -1;
    for (int nw = 4; nw <= (t.mb <= 4 ? 7 : 4); ++nw)
        for (int s = 1; s <= smax; ++s) {
            const long long c = proj_cost(strips, kch, mtiles, nw, s);
            if (best_cost < 0 || c < best_cost) {
                best_cost = c;
                const int cps = chunks_per_split(kch, s);
                best = ProjShape{nw, (kch + cps - 1) / cps};
            }
        }
    return best;
}

static bool use_tall(const Mat& W, int rows) {
    // the wide vocabulary projection runs several rounds of workgroups, two of the strip kernel's on a compute unit
    // at a time: measured faster there than one of these
    return W.kind == MAT_BF16_PACKED && rows > 128 && (W.N / 32 + 7) / 8 <= 256;
}

int proj_pick_splits(const Mat& W, int rows, int max_splits) {
    if (use_tall(W, rows)) return tall_pick_splits(W, rows, max_splits);
    return proj_pick(W, rows, max_splits).splits;
}

// the wave count that goes with a given split factor
static int proj_pick_waves(const Mat& W, int rows, int splits) {
    const int strips = W.N / 32, kch = W.K / 128;
    const ProjTiling t = proj_tiling(W, rows);
    const int mtiles = t.mtiles;
    if (W.kind == MAT_W4_PACKED && mtiles >= 2) return W.N / 32 >= 512 && mtiles <= 2 ? 7 : 4;
    int best = 4;
    long long best_cost = -1;
    for (int nw = 4; nw <= (t.mb <= 4 ? 7 : 4); ++nw) {
        const long long c = proj_cost(strips, kch, mtiles, nw, splits);
        if (best_cost < 0 || c < best_cost) {
            best_cost = c;
            best = nw;
        }
    }
    return best;
}

template <int MB, int KS>
static hipError_t launch_proj_nw(const ProjArgs& a, int nw, int epilogue, int splits, int mtiles, hipStream_t st) {
    switch (nw) {
    case 4: return launch_proj_t<MB, KS, 4>(a, epilogue, splits, mtiles, st);
    case 5: return launch_proj_t<MB, KS, 5>(a, epilogue, splits, mtiles, st);
    case 6: return launch_proj_t<MB, KS, 6>(a, epilogue, splits, mtiles, st);
    case 7: return launch_proj_t<MB, KS, 7>(a, epilogue, splits, mtiles, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_proj(const ProjLaunch& p, hipStream_t st) {
    const Mat& W = *p.W;
    const bool w4 = W.kind == MAT_W4_PACKED;
    if (!w4 && W.kind != MAT_BF16_PACKED) return hipErrorInvalidValue;
    if (p.rows < 1 || p.rows > kMaxBatchTile || W.N % 32 || W.K % 128) return hipErrorInvalidValue;
    const ATile at = atile_for_rows(p.rows);
    ProjArgs a{};
    a.W = (const u32x4*)W.w;
    a.SZ = (const uint32_t*)W.sz;
    a.s_only = W.s_only ? 1 : 0;
    a.A = (const u32x4*)p.A;
    a.qscale = p.qscale;
    a.out = p.out;
    a.rows = p.rows;
    a.N = W.N;
    a.K = W.K;
    a.ldo = p.ldo;
    a.ld_rows = p.ld_rows;
    a.mb_rows = at.MB;
    const int kch = W.K / 128;
    int splits = max(1, p.splits);
    const int cps = chunks_per_split(kch, splits);
    splits = (kch + cps - 1) / cps;
    if (w4 && p.qscale == nullptr) return hipErrorInvalidValue;
    const ProjTiling t = proj_tiling(W, p.rows);
    // Up to 64-row tiles a stage is a whole 128-wide group: three 16 KB stages in LDS for 32-row tiles,
    // two 32 KB stages for 64-row tiles (long stages amortise the workgroup barrier better than a
    // third buffer does); the 128-row bf16 tile has 64-wide stages.
    if (t.mb <= 4) {
        a.n_stages = kch;
        a.stages_per_split = cps;
        const int nw = proj_pick_waves(W, p.rows, splits);
        if (w4) {
            if (p.epilogue != EPI_STORE) return hipErrorInvalidValue;
            return launch_proj_w4<1>(a, nw, splits, t.mtiles, st);
        }
        if (t.mb == 2) return launch_proj_nw<2, 128>(a, nw, p.epilogue, splits, t.mtiles, st);
        return launch_proj_nw<4, 128>(a, nw, p.epilogue, splits, t.mtiles, st);
    }
    if (use_tall(W, p.rows)) {
        const int want = p.epilogue == EPI_SWIGLU ? 1 : max(1, p.splits);
        const int stg = kch * 2, per = (stg + want - 1) / want, real_s = (stg + per - 1) / per;
        a.n_stages = stg;
        a.stages_per_split = per;
        return launch_proj_tall(a, p.epilogue, real_s, (at.MB + 3) / 4, st);
    }
    a.n_stages = kch * 2;
    a.stages_per_split = cps * 2;
    return launch_proj_t<8, 64>(a, p.epilogue, splits, t.mtiles, st);
}

// ---------------------------------------------------------------------------------
// fp32 path (parity configuration): plain vector-ALU dot products, one wave per column
// ---------------------------------------------------------------------------------

struct F32Mat {
    const float* w[3];
    const uint8_t* q[3];
    const uint16_t* s[3];
    const uint16_t* z[3];
    int rows[3];
    int nsrc, N, K, quant;
};

template <int BT>
__global__ __launch_bounds__(256) void proj_f32_kernel(F32Mat m, const float* __restrict__ x, int nrows,
                                                       float* __restrict__ out) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    if (n >= m.N) return;
    const int b0 = blockIdx.y * BT;
    int src = 0, r = n;
    while (src + 1 < m.nsrc && r >= m.rows[src]) {
        r -= m.rows[src];
        ++src;
    }
    float acc[BT];
#pragma unroll
    for (int j = 0; j < BT; ++j) acc[j] = 0.f;
    const int ng = m.K / kGroup;
    for (int k = lane; k < m.K; k += 64) {
        float wv;
        if (m.quant) {
            const uint8_t byte = m.q[src][(size_t)r * (m.K / 2) + (k >> 1)];
            const float code = (float)((k & 1) ? (byte >> 4) : (byte & 15));
            const size_t g = (size_t)r * ng + k / kGroup;
            const float zf = m.z[src] ? __half2float(__ushort_as_half(m.z[src][g])) : 8.f;
            const float sf = __half2float(__ushort_as_half(m.s[src][g]));
            wv = (code - zf) * sf;  // exact: 5-bit integer times an 11-bit significand
        } else {
            wv = m.w[src][(size_t)r * m.K + k];
        }
#pragma unroll
        for (int j = 0; j < BT; ++j) {
            const int b = min(b0 + j, nrows - 1);
            acc[j] = fmaf(wv, x[(size_t)b * m.K + k], acc[j]);
        }
    }
#pragma unroll
    for (int j = 0; j < BT; ++j) {
        const float v = wave_sum(acc[j]);
        if (lane == 0 && b0 + j < nrows) out[(size_t)(b0 + j) * m.N + n] = v;
    }
}

hipError_t launch_proj_f32(const Mat& W, const float* x, int rows, float* out, hipStream_t st) {
    F32Mat m{};
    m.nsrc = W.nsrc;
    m.N = W.N;
    m.K = W.K;
    m.quant = W.kind == MAT_W4_LOGICAL;
    if (!m.quant && W.kind != MAT_F32) return hipErrorInvalidValue;
    for (int i = 0; i < 3; ++i) {
        m.w[i] = (const float*)W.wsrc[i];
        m.q[i] = W.q[i];
        m.s[i] = W.s[i];
        m.z[i] = W.z[i];
        m.rows[i] = W.src_rows[i];
    }
    constexpr int BT = 8;
    dim3 grid((W.N + 3) / 4, (rows + BT - 1) / BT);
    hipLaunchKernelGGL(proj_f32_kernel<BT>, grid, dim3(256), 0, st, m, x, rows, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// packing
// ---------------------------------------------------------------------------------

size_t packed_bf16_bytes(int N, int K) { return (size_t)N * K * 2; }
size_t packed_w4_bytes(int N, int K) { return (size_t)N * K / 2; }
size_t packed_w4_sz_bytes(int N, int K) { return (size_t)N * (K / 128) * 4; }

struct PackSrc {
    const void* p[3];
    const void* s[3];
    const void* z[3];
    int rows[3];
    int nsrc, mode, K, N;
};

// packed row pn -> (source, row).  mode 0: stacked.  mode 1: blocks of 16 rows alternate
// between source 0 (gate) and source 1 (up).
__device__ __forceinline__ void pack_row(const PackSrc& s, int pn, int& src, int& row) {
    if (s.mode == 1) {
        src = (pn >> 4) & 1;
        row = (pn >> 5) * 16 + (pn & 15);
    } else {
        src = 0;
        row = pn;
        while (src + 1 < s.nsrc && row >= s.rows[src]) {
            row -= s.rows[src];
            ++src;
        }
    }
}

// one thread per 16-byte unit of the packed matrix: [N/32][K/128][8][64] x 8 bf16
__global__ __launch_bounds__(256) void pack_bf16_kernel(PackSrc s, u32x4* __restrict__ dst) {
    const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)s.N * s.K / 8;
    if (u >= total) return;
    const int lane = (int)(u & 63), kk = (int)((u >> 6) & 7);
    const size_t t = u >> 9;
    const int kch = s.K / 128;
    const int c = (int)(t % kch), nb = (int)(t / kch);
    const int pn = nb * 32 + (lane & 31), half = lane >> 5;
    const int k = c * 128 + half * 64 + kk * 8;
    int src, row;
    pack_row(s, pn, src, row);
    dst[u] = *reinterpret_cast<const u32x4*>((const uint16_t*)s.p[src] + (size_t)row * s.K + k);
}

// one thread per packed dword (8 codes): [N/32][K/128][2][64][4 dwords]
__global__ __launch_bounds__(256) void pack_w4_kernel(PackSrc s, uint32_t* __restrict__ dst,
                                                      uint32_t* __restrict__ dst_sz) {
    const size_t u = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)s.N * s.K / 8;
    if (u >= total) return;
    const int comp = (int)(u & 3), lane = (int)((u >> 2) & 63), j = (int)((u >> 8) & 1);
    const size_t t = u >> 9;
    const int kch = s.K / 128;
    const int c = (int)(t % kch), nb = (int)(t / kch);
    const int kk = j * 4 + comp;
    const int pn = nb * 32 + (lane & 31), half = lane >> 5;
    const int k = c * 128 + half * 64 + kk * 8;
    int src, row;
    pack_row(s, pn, src, row);
    const uint32_t word = *reinterpret_cast<const uint32_t*>((const uint8_t*)s.p[src] + ((size_t)row * s.K + k) / 2);
    // logical: code e at bits [4e, 4e+4).  packed: the low nibbles of the four bytes hold e = 0..3, the
    // high nibbles e = 4..7, so that "and 0x0F0F0F0F" and "shift by 4, and" give the codes as bytes in order
    uint32_t o = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) o |= ((word >> (4 * e)) & 15u) << (e < 4 ? 8 * e : 8 * (e - 4) + 4);
    dst[u] = o;
    if (kk == 0 && half == 0) {
        const size_t g = (size_t)row * kch + c;
        const uint32_t sv = ((const uint16_t*)s.s[src])[g];
        if (s.z[src]) {
            const uint32_t zv = ((const uint16_t*)s.z[src])[g];
            dst_sz[((size_t)nb * kch + c) * 32 + (lane & 31)] = sv | (zv << 16);
        } else {  // scales only: groups 2i and 2i+1 share a dword
            ((uint16_t*)dst_sz)[(((size_t)nb * ((kch + 1) >> 1) + (c >> 1)) * 32 + (lane & 31)) * 2 + (c & 1)] = (uint16_t)sv;
        }
    }
}

static PackSrc make_src(const void* const p[3], const void* const s[3], const void* const z[3],
                        const int rows[3], int nsrc, int mode, int K) {
    PackSrc ps{};
    ps.nsrc = nsrc;
    ps.mode = mode;
    ps.K = K;
    ps.N = 0;
    for (int i = 0; i < 3; ++i) {
        ps.p[i] = p[i];
        ps.s[i] = s ? s[i] : nullptr;
        ps.z[i] = z ? z[i] : nullptr;
        ps.rows[i] = i < nsrc ? rows[i] : 0;
        ps.N += ps.rows[i];
    }
    return ps;
}

hipError_t launch_pack_bf16(const void* const src[3], const int src_rows[3], int nsrc, int mode, int K, void* dst,
                            hipStream_t st) {
    PackSrc ps = make_src(src, nullptr, nullptr, src_rows, nsrc, mode, K);
    const size_t total = (size_t)ps.N * K / 8;
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, ps, (u32x4*)dst);
    return hipGetLastError();
}

hipError_t launch_pack_w4(const sun_qmat src[3], const int src_rows[3], int nsrc, int mode, int K, void* dst_codes,
                          void* dst_sz, hipStream_t st) {
    const void *p[3] = {nullptr, nullptr, nullptr}, *s[3] = {nullptr, nullptr, nullptr}, *z[3] = {nullptr, nullptr, nullptr};
    for (int i = 0; i < nsrc; ++i) {
        p[i] = src[i].q;
        s[i] = src[i].s;
        z[i] = src[i].z;
    }
    PackSrc ps = make_src(p, s, z, src_rows, nsrc, mode, K);
    const size_t total = (size_t)ps.N * K / 8;
    hipLaunchKernelGGL(pack_w4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, ps,
                       (uint32_t*)dst_codes, (uint32_t*)dst_sz);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// round-to-nearest group quantiser (one wave per group of 128 weights)
// ---------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void quantize_w4_kernel(const void* __restrict__ w, int dtype, int rows, int cols,
                                                          int mode, uint8_t* __restrict__ q, uint16_t* __restrict__ s,
                                                          uint16_t* __restrict__ z) {
    const int lane = threadIdx.x & 63;
    const size_t grp = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int ng = cols / kGroup;
    if (grp >= (size_t)rows * ng) return;
    const size_t row = grp / ng;
    const int g = (int)(grp % ng);
    const size_t e0 = row * cols + (size_t)g * kGroup + 2 * lane;
    float a, b;
    if (dtype == SUN_BF16) {
        const uint32_t pr = *reinterpret_cast<const uint32_t*>((const uint16_t*)w + e0);
        a = bf16_lo(pr);
        b = bf16_hi(pr);
    } else {
        a = ((const float*)w)[e0];
        b = ((const float*)w)[e0 + 1];
    }
    const float mn = -wave_max(-fminf(a, b)), mx = wave_max(fmaxf(a, b));
    const float amax = wave_max(fmaxf(fabsf(a), fabsf(b)));
    const float sf = mode == 0 ? __fdiv_rn(mx - mn, 15.0f) : __fdiv_rn(amax, 7.0f);
    __half sh = __float2half_rn(sf);
    float S = __half2float(sh);
    if (S == 0.f) {
        S = 1.f;
        sh = __float2half_rn(1.f);
    }
    const float Z = mode == 0 ? fminf(fmaxf(rintf(__fdiv_rn(-mn, S)), 0.f), 15.f) : 8.f;
    const int qa = (int)fminf(fmaxf(rintf(__fdiv_rn(a, S)) + Z, 0.f), 15.f);
    const int qb = (int)fminf(fmaxf(rintf(__fdiv_rn(b, S)) + Z, 0.f), 15.f);
    q[(row * cols + (size_t)g * kGroup) / 2 + lane] = (uint8_t)(qa | (qb << 4));
    if (lane == 0) {
        s[grp] = __half_as_ushort(sh);
        if (z) z[grp] = __half_as_ushort(__float2half_rn(Z));
    }
}

hipError_t launch_quantize_w4(const void* w, int dtype, int rows, int cols, int group, int mode, void* q, void* s,
                              void* z, hipStream_t st) {
    if (group != kGroup || cols % kGroup) return hipErrorInvalidValue;
    const size_t groups = (size_t)rows * (cols / kGroup);
    hipLaunchKernelGGL(quantize_w4_kernel, dim3((unsigned)((groups + 3) / 4)), dim3(256), 0, st, w, dtype, rows, cols,
                       mode, (uint8_t*)q, (uint16_t*)s, (uint16_t*)z);
    return hipGetLastError();
}

}  // namespace sun
