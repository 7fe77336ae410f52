// Host-side launchers of the HIP kernels (one translation unit per kernel family).
#pragma once
#include "common.hpp"

namespace sun {

// ---------------- projections (proj.hip) ----------------

enum ProjEpilogue {
    EPI_STORE = 0,   // fp32 partial sums: out[(split * ld_rows + b) * ldo + n]
    EPI_SWIGLU = 1   // gate/up pair, bf16 weights, no split: out is the two-plane tile of silu(gate) * up [rows, N/2]
};

struct ProjLaunch {
    const Mat* W;
    const void* A;         // tiled bf16 activations [rows, K]
    const float* qscale;   // W4 only: [K/128][MB*32] pairs (scale, sum of integers as int bits) of the fixed-point tile A
    int rows;              // valid rows (<= 256)
    int epilogue;
    int splits;            // split-K factor (EPI_STORE only); partial s is written at out + s*ld_rows*ldo
    float* out;
    int ldo;               // leading dimension of out (>= N)
    int ld_rows;           // rows per split slab
};
// Chooses the split-K factor the step uses for this matrix and row count.
int proj_pick_splits(const Mat& W, int rows, int max_splits);
hipError_t launch_proj(const ProjLaunch& p, hipStream_t st);

// fp32 activations path (vector ALU): out[b][n] = sum_k W[n][k] x[b][k], out row-major [rows, N].
hipError_t launch_proj_f32(const Mat& W, const float* x, int rows, float* out, hipStream_t st);

// packing (weights load time)
size_t packed_bf16_bytes(int N, int K);
size_t packed_w4_bytes(int N, int K);     // codes
size_t packed_w4_sz_bytes(int N, int K);  // scales / zero points
// mode 0: rows of up to three sources stacked; mode 1: two sources interleaved in blocks of 16 rows.
hipError_t launch_pack_bf16(const void* const src[3], const int src_rows[3], int nsrc, int mode, int K,
                            void* dst, hipStream_t st);
hipError_t launch_pack_w4(const sun_qmat src[3], const int src_rows[3], int nsrc, int mode, int K,
                          void* dst_codes, void* dst_sz, hipStream_t st);
hipError_t launch_quantize_w4(const void* w, int dtype, int rows, int cols, int group, int mode, void* q,
                              void* s, void* z, hipStream_t st);

// ---------------- attention (attention.hip) ----------------

struct AttnPlan {           // device arrays inside the workspace
    int32_t* chunk_off;     // [batch+1] prefix sum of chunks (full + small) per request
    int32_t* full_off;      // [batch+1] prefix sum of full chunks per request
    int32_t* small_off;     // [batch+1] prefix sum of small chunks per request
    int32_t* records;       // [max_chunks * Hkv][24] per-item records
    float* partial;         // [max_chunks][Hq][d+2]  (o[d], m, l)
    int max_chunks;
};
size_t attn_max_chunks(int batch, int max_pages, int Hkv);
hipError_t launch_attn_plan(const AttnPlan& plan, const int32_t* n_or_len, int len_plus, int batch,
                            const int32_t* page_tables, int max_pages, int n_pages, int Hkv, hipStream_t st);
// n_tokens(i) = n_or_len[i] + len_plus.  q fp32 [batch, Hq*d].  The chunk counts of the batch (all chunks, full
// chunks) when the host knows the lengths, else < 0.
hipError_t launch_attn_split(const KvPool& pool, int layer, const AttnPlan& plan, const float* q,
                             const int32_t* page_tables, int max_pages, const int32_t* n_or_len, int len_plus,
                             int batch, int total_chunks_hint, int full_chunks_hint, bool f32_exact, hipStream_t st);
// out: fp32 row-major [batch, Hq*d] (out_f32) and/or the O projection's input: two-plane tiled bf16, or, with
// qscale given, the fixed-point tile of a 4-bit projection and its (scale, integer sum) pairs.
hipError_t launch_attn_combine(const sun_model_cfg& cfg, const AttnPlan& plan, int batch, float* out_f32,
                               void* out_tiled, float* qscale, hipStream_t st);

// ---------------- everything else (misc.hip) ----------------

hipError_t launch_embed(const sun_model_cfg& cfg, const void* embed, const int32_t* tokens, int batch, float* x,
                        hipStream_t st);
// x[b] += sum_s partial[s][b] (s ascending; nparts may be 0); then h = rmsnorm(x; g).
// h_f32: row-major fp32 or NULL; h_tiled: tiled bf16 or NULL; with qscale given h_tiled is the fixed-point tile of a
// 4-bit projection instead and qscale receives its (scale, integer sum) pairs.
hipError_t launch_residual_norm(const sun_model_cfg& cfg, float* x, const float* partial, int nparts, int ld_rows,
                                const void* gain, int batch, float* h_f32, void* h_tiled, float* qscale, hipStream_t st);
// k_src, v_src: bf16 [n_layers][n_tokens][Hkv][d]; token t lands at position first_pos + t of the request whose
// page-table row is given.
hipError_t launch_kv_ingest(const KvPool& pool, const void* k_src, const void* v_src, int n_tokens, int first_pos,
                            const int32_t* page_table, hipStream_t st);
// Between two steps of a run: token feedback, length + 1, page allocation in request order.
hipError_t launch_advance(const int32_t* next, int batch, int max_pages, const int32_t* free_pages, int n_free,
                          int32_t* token_ids, int32_t* page_tables, int32_t* seq_lens, int32_t* free_head,
                          int32_t* status, bool clear_status, hipStream_t st);
// Per-row inputs of one block of a prefill: row r gets a copy of the request's page-table row, length
// first_pos + r and the source-model id.
hipError_t launch_prefill_rows(const int32_t* page_table, int max_pages, int first_pos, int model_id, int rows,
                               int32_t* tables, int32_t* lens, int32_t* ids, hipStream_t st);
// Rows, waiting queue and page ring of a decode worker with continuous batching (sun_serve_state plus sizes).
struct ServeArgs {
    int32_t *token_ids, *page_tables, *seq_lens, *model_ids, *slot_req, *slot_left;
    const int32_t *w_req, *w_token, *w_tables, *w_lens, *w_model, *w_budget;
    int32_t *ring, *counters;
    int n_wait, ring_cap, idle_page, eos_id, slots, max_pages;
};
// Between two steps (advance) and/or before the first (reset): record tokens, retire, grow, admit.
hipError_t launch_serve(const ServeArgs& a, const int32_t* next, int32_t* tokens_out, int32_t* req_out, bool reset,
                        bool advance, hipStream_t st);
hipError_t launch_rope_table(const sun_model_cfg& cfg, const int32_t* seq_lens, int batch, float* table,
                             hipStream_t st);
// qkv partial sums [nparts][ld_rows][Nqkv] -> rotated q fp32 [batch, Hq*d]; K,V (bf16) appended to the pool.
hipError_t launch_rope_append(const KvPool& pool, int layer, const float* qkv, int nparts, int ld_rows,
                              const float* table, const int32_t* seq_lens, const int32_t* page_tables, int max_pages,
                              int batch, float* q_out, const void* q_norm, const void* k_norm, const void* bq, const void* bk,
                              const void* bv, hipStream_t st);
hipError_t launch_swiglu_f32(const float* gu, int batch, int ffn, float* u, hipStream_t st);
// gate/up partial sums (projection column order) -> silu(g)*u as two-plane tiled bf16, or as fixed-point tile + qscale
hipError_t launch_swiglu_tile(const float* part, int nparts, int ld_rows, int rows, int ffn, void* tiled, float* qscale,
                              hipStream_t st);
// measurement only: read n_blocks blocks of block_units 16-byte units (order given by perm, or address order),
// with plain loads or with the streaming loads the attention kernel uses for K and V
hipError_t launch_hbm_read_probe(const void* src, long long n_blocks, int block_units, const int32_t* perm, int grid,
                                 bool stream, uint32_t* sink, hipStream_t st);
constexpr int kArgmaxParts = 16;  // slices of a logits row searched by separate workgroups
// part_val / part_idx: scratch [batch][kArgmaxParts]
hipError_t launch_argmax(const float* logits, int batch, int vocab, float* part_val, int32_t* part_idx, int32_t* next,
                         hipStream_t st);
// fp32 [rows, K] -> two-plane tiled bf16, or fixed-point tile + qscale
hipError_t launch_tile_rows(const float* x, int rows, int K, void* tiled, float* qscale, hipStream_t st);
// out[b][n] = sum_s partial[s][b][n]
hipError_t launch_reduce_partials(const float* partial, int nparts, int ld_rows, int rows, int N, float* out,
                                  hipStream_t st);
// tiled bf16 [rows, K] -> fp32 row-major
hipError_t launch_untile_rows(const void* tiled, int rows, int K, float* out, hipStream_t st);

}  // namespace sun
