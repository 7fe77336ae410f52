/*
 * libsun — one decode step of SUN's frozen, shared decode module on one MI355X.
 *
 * The library evaluates D_theta_d of Section 3.1, Eq. 3: for every request of a
 * batch it consumes the most recent token and the request's KV cache, appends
 * the KV entry of the new position (Eq. 4) and returns next-token logits and
 * the greedy next token.  The requests of one batch may come from different
 * task-specific prefill models; because all tasks decode with the same
 * parameters (Section 3.2.1) and decode routing ignores task identity
 * (Section 3.2.3), the source-model id of a request is a tag that is validated
 * and otherwise ignored, and all caches live in one paged pool addressed only
 * through per-request page tables.  sun_qdecode_step is the QSUN variant
 * (Section 3.3, Eq. 8): the same step with 4-bit, group-128 weight-only
 * quantised projections; lm_head, embedding and norm gains stay dense
 * (Appendix A.1, "Quantization Configurations").
 *
 * Conventions
 *  - "dev" pointers are device (HBM) addresses owned by the caller; "host"
 *    pointers are ordinary host memory.  The library never allocates or frees
 *    device memory and never synchronises unless stated; work is enqueued on the
 *    caller's hipStream_t (passed as void*; NULL = the null stream).
 *  - Every function returns a status (SUN_OK = 0) and sun_last_error() describes
 *    a failure (thread-local).  Every check of arguments and, under SUN_VALIDATE,
 *    of device arrays happens before the first launch: such an error enqueues
 *    nothing.  SUN_ERR_HIP is the exception: a launch the runtime refuses in the
 *    middle of a step leaves the earlier kernels of that step enqueued, and the
 *    workspace, the outputs and the positions of the pool the step writes are
 *    then undefined; the multi-step calls (sun_decode_run, sun_decode_serve,
 *    sun_prefill) may in that case have completed earlier steps, which have
 *    updated token ids, lengths, page tables and the pool.
 *  - All matrices are row-major [out_features, in_features].
 *  - A process uses the library from one thread per stream; calls that share a
 *    workspace or a pool must not overlap.
 */
#ifndef SUN_H_
#define SUN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SUN_OK = 0,
    SUN_ERR_NULL = 1,       /* a required pointer is NULL */
    SUN_ERR_SHAPE = 2,      /* unsupported or inconsistent model shape / batch */
    SUN_ERR_POOL_SIZE = 3,  /* pool memory too small for the requested pages */
    SUN_ERR_WORKSPACE = 4,  /* workspace too small */
    SUN_ERR_PAGE_RANGE = 5, /* page table entry outside [0, n_pages) or table too short */
    SUN_ERR_SEQ_LEN = 6,    /* negative length or length beyond the page table */
    SUN_ERR_MODEL_ID = 7,   /* source-model id outside [0, n_source_models) */
    SUN_ERR_HIP = 8,        /* a HIP runtime call failed */
    SUN_ERR_TOKEN = 9       /* token id outside [0, vocab) */
};

enum { SUN_F32 = 0, SUN_BF16 = 1 };

/* step flags */
enum {
    SUN_VALIDATE = 1u, /* copy token ids, lengths, page tables and model ids to the host
                          (synchronises the stream) and check them before enqueueing */
    SUN_PROFILE = 2u,  /* record HIP events around each kernel class; see sun_profile_read */
    SUN_SERVE_RESET = 4u /* sun_decode_serve only: before the first iteration make every row idle
                            and admit from the queue */
};

/*
 * Decoder shape (pre-norm Llama-style block: RMSNorm, GQA attention with rotary
 * embedding in half-split pairing, SwiGLU, untied lm_head).  act_dtype selects the
 * arithmetic: SUN_F32 = fp32 weights and activations on the vector ALUs (parity
 * configuration), SUN_BF16 = bf16 weights, activations as two bf16 planes (value +
 * remainder) into the matrix cores, fp32 accumulators / residual stream / softmax;
 * with 4-bit weights (sun_qweights_create) the projections run on the int8 matrix
 * cores instead: the codes as integers, the activations as 16-bit fixed point with
 * one scale per row and 128-wide group, exact int32 sums per group, scales applied
 * in fp32.  The KV pool is bf16 in all of them.
 * Supported: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads with ratio
 * <= 8; SUN_BF16 additionally needs hidden, ffn and n_q_heads*head_dim multiples
 * of 128 and vocab a multiple of 32.
 */
typedef struct sun_model_cfg {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rms_eps, rope_base;
    int32_t act_dtype;
    /* Options of the backbone families the paper evaluates (Section 4.1); all zero = plain block. */
    int32_t qk_norm;       /* Qwen3 class: RMSNorm over head_dim (eps = rms_eps, own gain per layer) on every
                              q and k head before the rotation; needs q_norm / k_norm in the weight table */
    int32_t rope_scaling;  /* LLaMA-3.1 class: 1 = rotation frequencies rescaled by wavelength: pairs with
                              wavelength < rope_original_max_position / rope_high_freq_factor keep their
                              frequency, those above rope_original_max_position / rope_low_freq_factor are
                              divided by rope_factor, in between the two are blended linearly in
                              rope_original_max_position / wavelength */
    int32_t rope_original_max_position;
    float rope_factor, rope_low_freq_factor, rope_high_freq_factor;
    int32_t qkv_bias;      /* Qwen2 class: 1 = the q, k and v projections add a bias vector (before the head norm
                              and the rotation); needs bq / bk / bv in the weight table.  Neither family of
                              Section 4.1 uses it; it is here for the same backbone interface. */
} sun_model_cfg;

/* ------------------------------------------------------------------ KV pool */

/*
 * Element (bf16) offsets into the pool:
 *   K(layer,page,head,token,dim) = k_off + layer*k_layer + page*k_page + head*k_head + token*k_token + dim*k_dim
 * and the same with v_.  K is stored [token][dim], V transposed [dim][token] inside
 * a (layer, page, head) block, so that both are matrix-core operands after a
 * 16-byte load.  A prefill producer writes through these strides.
 */
typedef struct sun_kv_layout {
    int64_t n_pages;
    int32_t page_tokens, reserved;
    int64_t k_off, k_layer, k_page, k_head, k_token, k_dim;
    int64_t v_off, v_layer, v_page, v_head, v_token, v_dim;
    int64_t total_elems;
} sun_kv_layout;

typedef struct sun_kv_pool sun_kv_pool;

/* Bytes of device memory a pool of n_pages pages needs. */
size_t sun_kv_pool_bytes(const sun_model_cfg* cfg, int64_t n_pages, int page_tokens);

/*
 * Wraps caller-owned device memory as ONE paged KV pool shared by the caches of
 * all source models (Section 3.2.3: decode requests are pooled whatever model
 * prefilled them).  dev_mem: device, 256-byte aligned, borrowed until destroy
 * and never freed by the library.  bytes / page size gives n_pages.
 * page_tokens must be 16.  n_source_models bounds the model ids accepted by
 * SUN_VALIDATE.  Errors: SUN_ERR_NULL, SUN_ERR_SHAPE, SUN_ERR_POOL_SIZE (no page fits).
 */
int sun_kv_pool_create(const sun_model_cfg* cfg, void* dev_mem, size_t bytes, int page_tokens,
                       int n_source_models, sun_kv_pool** out);
int sun_kv_pool_layout(const sun_kv_pool* pool, sun_kv_layout* out);
void sun_kv_pool_destroy(sun_kv_pool* pool);

/*
 * Places a cache produced elsewhere into the pages a request owns: the prompt's cache C_T that a
 * task-specific prefill module computed (Eq. 2) and handed to this decode worker (Section 3.2.2,
 * disaggregated serving), or a later chunk of it.  After the call the decode step can consume
 * the request like any other (the cache of Eq. 4 is prompt KV followed by decode-generated KV).
 *   model_id   source model that produced the cache; a tag: it is counted, never used for addressing
 *   k_src, v_src  dev bf16 [n_layers, n_tokens, n_kv_heads, head_dim], contiguous, 16-byte aligned;
 *              K already rotated, as the decode step stores it
 *   first_pos  position of the source's token 0 in the request (0 for a whole prompt)
 *   page_table dev int32 [max_pages], the request's row; entries first_pos/16 .. (first_pos+n_tokens-1)/16
 *              must name pages of the pool that no other request writes
 * A byte-exact scatter: only the n_tokens positions are written (a chunk may start or end inside a
 * page).  Enqueued on `stream`.  Without SUN_VALIDATE a page id outside the pool skips that page;
 * with it the row is copied to the host (synchronises) and checked: SUN_ERR_PAGE_RANGE.
 * Errors: SUN_ERR_NULL, SUN_ERR_MODEL_ID, SUN_ERR_SEQ_LEN (n_tokens < 1, first_pos < 0, or the row is
 * too short), SUN_ERR_SHAPE (misaligned source).
 */
int sun_kv_pool_ingest(sun_kv_pool* pool, int model_id, const void* k_src, const void* v_src,
                       int n_tokens, int first_pos, const int32_t* page_table, int max_pages,
                       void* stream, unsigned flags);

/* Tokens ingested so far for one source model (host-side count; the pool itself is not partitioned
 * by model).  Errors: SUN_ERR_NULL, SUN_ERR_MODEL_ID. */
int sun_kv_pool_model_tokens(const sun_kv_pool* pool, int model_id, int64_t* tokens);

/* ------------------------------------------------------------------ weights */

/*
 * Dense decode parameters theta_d (Eq. 3).  embed [vocab, hidden]; per layer
 * (host arrays of n_layers device pointers) g1 [hidden], wq [Hq*d, hidden],
 * wk, wv [Hkv*d, hidden], wo [hidden, Hq*d], g2 [hidden], wg, wu [ffn, hidden],
 * wd [hidden, ffn]; gf [hidden]; wlm [vocab, hidden].  Element type is fp32
 * (SUN_F32) or bf16 (SUN_BF16) for every tensor.
 */
typedef struct sun_weight_ptrs {
    const void* embed;
    const void* const* g1;
    const void* const* wq;
    const void* const* wk;
    const void* const* wv;
    const void* const* wo;
    const void* const* g2;
    const void* const* wg;
    const void* const* wu;
    const void* const* wd;
    const void* gf;
    const void* wlm;
    const void* const* q_norm; /* per layer [head_dim]; read only if cfg.qk_norm, else may be NULL */
    const void* const* k_norm;
    const void* const* bq;     /* per layer [Hq*d], [Hkv*d], [Hkv*d], element type as the weights; read only if */
    const void* const* bk;     /* cfg.qkv_bias, else may be NULL */
    const void* const* bv;
} sun_weight_ptrs;

typedef struct sun_weights sun_weights;

/*
 * SUN_BF16: projection matrices are re-tiled into the matrix-core operand order
 * inside pack_mem (device, 256-byte aligned, at least sun_weights_pack_bytes(cfg)
 * bytes, borrowed until destroy); the packing kernels run on `stream` and the call
 * returns after synchronising it, after which the caller may free the row-major
 * matrices (embed, gains are still referenced).  SUN_F32: pack_mem may be NULL,
 * the row-major arrays are used in place.
 */
size_t sun_weights_pack_bytes(const sun_model_cfg* cfg);
int sun_weights_create(const sun_model_cfg* cfg, const sun_weight_ptrs* dev, void* pack_mem,
                       size_t pack_bytes, void* stream, sun_weights** out);
void sun_weights_destroy(sun_weights* w);

/*
 * QSUN parameters q(theta_d) (Eq. 8; Appendix A.1): every projection of the block is
 * W_hat[n,k] = (Q[n,k] - Z[n,k/128]) * S[n,k/128] with Q 4-bit codes packed two per
 * byte along k (low nibble = even k) [out, in/2], S and Z fp16 [out, in/128], Z
 * holding an integer in [0,15].  embed, gains and wlm are dense as in
 * sun_weight_ptrs (lm_head is not quantised).
 * Symmetric layout (the quantisation Appendix A.1 names): z = NULL in every sun_qmat means
 * Z = 8 everywhere, W_hat = (Q - 8) * S; no zero points are stored or read, which leaves
 * 0.5 + 2/128 = 0.516 bytes per weight.  z must be given for every matrix or for none.
 */
typedef struct sun_qmat {
    const void* q;
    const void* s;
    const void* z;
} sun_qmat;

typedef struct sun_qweight_ptrs {
    const void* embed;
    const void* const* g1;
    const sun_qmat* wq; /* host arrays of n_layers entries */
    const sun_qmat* wk;
    const sun_qmat* wv;
    const sun_qmat* wo;
    const void* const* g2;
    const sun_qmat* wg;
    const sun_qmat* wu;
    const sun_qmat* wd;
    const void* gf;
    const void* wlm;
    const void* const* q_norm; /* as in sun_weight_ptrs */
    const void* const* k_norm;
    const void* const* bq;     /* as in sun_weight_ptrs (biases are not quantised) */
    const void* const* bk;
    const void* const* bv;
} sun_qweight_ptrs;

size_t sun_qweights_pack_bytes(const sun_model_cfg* cfg, int group);
/* group must be 128.  Packing as in sun_weights_create (codes, scales and lm_head
 * are re-tiled into pack_mem under SUN_BF16). */
int sun_qweights_create(const sun_model_cfg* cfg, const sun_qweight_ptrs* dev, int group,
                        void* pack_mem, size_t pack_bytes, void* stream, sun_weights** out);

/*
 * Round-to-nearest group quantiser producing the QSUN format from a dense matrix
 * (device; dtype SUN_F32 or SUN_BF16; [rows, cols], cols a multiple of `group`,
 * group a multiple of 8).  mode 0 (affine): S = fp16((max-min)/15) (1 if 0),
 * Z = clamp(rne(-min/S),0,15), Q = clamp(rne(w/S)+Z,0,15).  mode 1 (symmetric,
 * the wording of Appendix A.1): S = fp16(max|w|/7) (1 if 0), Z = 8,
 * Q = clamp(rne(w/S)+8,0,15).  Divisions use the stored fp16 S, in fp32.
 * Outputs (device): q [rows, cols/2] bytes, s and z fp16 [rows, cols/group]; z may be NULL in
 * mode 1 (it would hold 8 everywhere).
 */
int sun_quantize_w4(const void* w, int dtype, int rows, int cols, int group, int mode, void* q,
                    void* s, void* z, void* stream);

/* ------------------------------------------------------------------ decode step */

/* Bytes of device workspace a step with up to max_batch requests and max_pages
 * page-table columns needs. */
size_t sun_workspace_bytes(const sun_model_cfg* cfg, int max_batch, int max_pages);

/*
 * One decode step (Eq. 3) for `batch` requests, enqueued on `stream`.
 *   token_ids   dev int32 [batch]             y_{t-1} of each request
 *   page_tables dev int32 [batch, max_pages]  physical page per 16 tokens, -1 = unused
 *   seq_lens    dev int32 [batch]             L_i = tokens cached BEFORE the step; the new
 *                                             token takes position L_i and attention spans
 *                                             positions 0..L_i
 *   seq_lens_host host int32 [batch] or NULL  optional copy, used only to size the launch
 *   model_ids   dev int32 [batch]             source-model tag (checked under SUN_VALIDATE,
 *                                             never read by a kernel)
 *   logits_out  dev fp32 [batch, vocab] or NULL
 *   next_tokens_out dev int32 [batch]         greedy argmax, lowest index on ties
 *   workspace   dev, 256-byte aligned, >= sun_workspace_bytes(cfg, batch, max_pages)
 * The step writes K/V of the new position into slot L_i % 16 of page
 * page_tables[i][L_i / 16] in every layer (Eq. 4) and does not change seq_lens.
 * Preconditions: the table of request i has ceil((L_i+1)/16) valid entries; the page
 * written this step is not referenced by any other request of the batch (history
 * pages may be shared read-only).  Outputs are valid after the stream is
 * synchronised.  With flags = 0 device array contents are not checked.
 * Errors: SUN_ERR_NULL, SUN_ERR_SHAPE (batch < 1, or a pool / weights pair of
 * different shape), SUN_ERR_WORKSPACE; under SUN_VALIDATE also SUN_ERR_TOKEN,
 * SUN_ERR_SEQ_LEN, SUN_ERR_PAGE_RANGE, SUN_ERR_MODEL_ID.
 */
int sun_decode_step(sun_kv_pool* pool, const sun_weights* weights, int batch,
                    const int32_t* token_ids, const int32_t* page_tables, int max_pages,
                    const int32_t* seq_lens, const int32_t* seq_lens_host, const int32_t* model_ids,
                    float* logits_out, int32_t* next_tokens_out, void* workspace,
                    size_t workspace_bytes, void* stream, unsigned flags);

/* QSUN step (Eq. 8): identical arguments; `weights` must come from sun_qweights_create. */
int sun_qdecode_step(sun_kv_pool* pool, const sun_weights* weights, int batch,
                     const int32_t* token_ids, const int32_t* page_tables, int max_pages,
                     const int32_t* seq_lens, const int32_t* seq_lens_host, const int32_t* model_ids,
                     float* logits_out, int32_t* next_tokens_out, void* workspace,
                     size_t workspace_bytes, void* stream, unsigned flags);

/* ------------------------------------------------------------------ multi-step run */

/*
 * n_steps decode steps in a row for a fixed set of requests, enqueued on `stream` without any
 * host synchronisation in between: the step of Eq. 3 applied repeatedly with greedy feedback,
 * every step extending each cache by one entry (Eq. 4).  This is the loop whose per-step time
 * the paper reports as TPOT (Appendix A.2).  `weights` may come from sun_weights_create or
 * sun_qweights_create.
 *
 * After each step, on the device: token_ids[i] = the generated token; seq_lens[i] += 1; if
 * the position the request writes next opens a page (seq_lens[i] % 16 == 0) that its table
 * does not have (entry < 0), the entry is set to free_pages[*free_head] and *free_head
 * advances; within a step requests are served in index order.  A request that finds the free
 * list empty, or whose table has no column left, keeps its length: nothing is ever written through a
 * missing page, but its fed-back token is still replaced, so from that step on it decodes every new
 * token at the same position, over its own earlier entry there, and the tokens it produces are not a
 * continuation of its sequence; bit 0 (list empty) or bit 1 (table full) of *run_status is set and the
 * caller must discard that request's outputs from the step it was starved in (sun_decode_serve avoids
 * the situation by reserving pages at admission).  *run_status is cleared at the start of the run.
 *
 *   token_ids   dev int32 [batch]             in: y_{t-1}; out: the last generated token
 *   page_tables dev int32 [batch, max_pages]  in/out
 *   seq_lens    dev int32 [batch]             in/out
 *   free_pages  dev int32 [n_free]            pages no table references (read only)
 *   free_head   dev int32 [1]                 in/out: first unused entry of free_pages
 *   run_status  dev int32 [1]                 out
 *   tokens_out  dev int32 [n_steps, batch]    the generated token of every step
 *   logits_out  dev fp32 [batch, vocab] or NULL: logits of the last step
 * Other arguments, preconditions and errors as for sun_decode_step; n_steps >= 1.  Under
 * SUN_VALIDATE the inputs of the first step are checked as there, and free_pages[*free_head..]
 * must lie in the pool, be distinct and not be referenced by any table (SUN_ERR_PAGE_RANGE).
 */
int sun_decode_run(sun_kv_pool* pool, const sun_weights* weights, int batch, int n_steps,
                   int32_t* token_ids, int32_t* page_tables, int max_pages, int32_t* seq_lens,
                   const int32_t* model_ids, const int32_t* free_pages, int n_free,
                   int32_t* free_head, int32_t* run_status, int32_t* tokens_out, float* logits_out,
                   void* workspace, size_t workspace_bytes, void* stream, unsigned flags);

/* ------------------------------------------------------------------ continuous batching */

/*
 * State of a decode worker that admits and retires requests between steps (the continuous
 * batching of Section 2.1.1) entirely on the device.  All pointers are device memory owned by
 * the caller; the struct itself is read on the host.  `slots` batch rows are decoded every
 * step; a row is either occupied by a request or idle.
 *
 * Rows (in/out, kept between calls):
 *   token_ids, seq_lens, model_ids  int32 [slots]; page_tables int32 [slots, max_pages]
 *   slot_req   int32 [slots]  id of the request in the row, -1 = idle
 *   slot_left  int32 [slots]  tokens the request may still generate (>= 1 while occupied)
 * Waiting requests (read only), already prefilled: their caches are in the pool under the
 * pages their table row lists.  Served first in, first out, starting at counters[0]:
 *   w_req, w_token, w_lens, w_model, w_budget int32 [n_wait]; w_tables int32 [n_wait, max_pages]
 *   (w_token: the first input token; w_lens: positions cached; w_budget >= 1: tokens to generate)
 * Pages: `ring` int32 [ring_cap] is a circular list of pages no table references; entries
 *   counters[1] .. counters[2]-1 (indices modulo ring_cap) are valid.  ring_cap must be at
 *   least the number of pages that can ever be free at once (the pool's page count is enough).
 *   `idle_page` is one page set aside for idle rows: it is in no table and not in the ring.
 * counters int32 [8] (in/out): 0 first unserved waiting request, 1 ring head (take),
 *   2 ring tail (put), 3 status bits, 4 requests retired, 5 requests admitted,
 *   6 tokens generated, 7 steps run.  Heads and tails only grow.
 * eos_id: a request also ends when it generates this token (-1: never).
 *
 * One iteration = one decode step over all rows (idle rows decode token 0 at position 0 of
 * idle_page; what they produce is dropped), then, in this order and in row order within each:
 *  1. every occupied row records its token and has one token less left; it is finished if
 *     none is left or the token is eos_id;
 *  2. finished rows retire: the pages of their table, in column order, go to the ring's
 *     tail, and the row becomes idle;
 *  3. the other occupied rows feed their token back and grow by one position; a row whose
 *     next position opens a page its table lacks takes the page at the ring's head;
 *  4. idle rows take waiting requests, first in first out, as long as the head of the queue
 *     fits: a request is admitted only if the pages it may still need,
 *     floor((len + budget - 1) / 16) + 1 minus the pages its table row holds, are available
 *     in the ring beyond what the rows already admitted may still need.  So an admitted
 *     request never waits for a page, and a request that does not fit blocks those behind it
 *     until pages come back.  A budget that would run past the table (max_pages * 16
 *     positions) is cut to fit and status bit 1 is set.
 * Status bit 0: step 3 found the ring empty (possible only if rows were placed by hand without
 * enough pages; the row then keeps its length, as in sun_decode_run).
 */
typedef struct sun_serve_state {
    int32_t* token_ids;
    int32_t* page_tables;
    int32_t* seq_lens;
    int32_t* model_ids;
    int32_t* slot_req;
    int32_t* slot_left;
    const int32_t* w_req;
    const int32_t* w_token;
    const int32_t* w_tables;
    const int32_t* w_lens;
    const int32_t* w_model;
    const int32_t* w_budget;
    int32_t* ring;
    int32_t* counters;
    int32_t n_wait;
    int32_t ring_cap;
    int32_t idle_page;
    int32_t eos_id;
} sun_serve_state;

/* Bytes of device workspace sun_decode_serve needs for `slots` rows. */
size_t sun_serve_workspace_bytes(const sun_model_cfg* cfg, int slots, int max_pages);

/*
 * n_steps iterations of the loop above, enqueued on `stream` with no host synchronisation in
 * between.  `weights` may come from sun_weights_create or sun_qweights_create.
 *   tokens_out dev int32 [n_steps, slots]: the token each row generated, -1 for an idle row
 *   req_out    dev int32 [n_steps, slots]: the request that generated it, -1 for an idle row
 *   logits_out dev fp32 [slots, vocab] or NULL: logits of the last step
 * With SUN_SERVE_RESET the rows' arrays need not be initialised (counters must be: zero for a
 * fresh start, with counters[2] = number of pages in the ring).  Without it the call continues
 * from the state a previous call left; two calls of n and m steps equal one of n + m.
 * Errors: SUN_ERR_NULL, SUN_ERR_SHAPE (slots outside [1, 256], n_steps < 1, n_wait < 0,
 * ring_cap < 1, shapes), SUN_ERR_WORKSPACE; under SUN_VALIDATE also SUN_ERR_PAGE_RANGE
 * (idle_page, ring entries or waiting tables outside the pool, a page listed twice),
 * SUN_ERR_SEQ_LEN, SUN_ERR_TOKEN, SUN_ERR_MODEL_ID for waiting requests not yet served.
 */
int sun_decode_serve(sun_kv_pool* pool, const sun_weights* weights, int slots, int max_pages, int n_steps,
                     const sun_serve_state* state, int32_t* tokens_out, int32_t* req_out, float* logits_out,
                     void* workspace, size_t workspace_bytes, void* stream, unsigned flags);

/* ------------------------------------------------------------------ prefill */

/* Bytes of device workspace a prefill of n_tokens positions with max_pages page-table columns needs. */
size_t sun_prefill_workspace_bytes(const sun_model_cfg* cfg, int n_tokens, int max_pages);

/*
 * The prefill module of Eq. 2 for one request, enqueued on `stream`: the causal forward of
 * `weights` (the task-specific theta_p of Section 3.2.1, or the base model) over n_tokens prompt
 * tokens at positions first_pos .. first_pos + n_tokens - 1.  It writes the K/V of those positions
 * into the request's pages in every layer (the prompt part C_X of Eq. 4) and returns the
 * distribution of the first generated token.  Positions 0 .. first_pos - 1 must already be cached
 * (first_pos > 0 continues a prompt that was prefilled in pieces); the result does not depend on
 * how a prompt is cut into pieces.
 *
 * It runs through the decode step's own kernels: the prompt is taken in blocks of up to 256
 * positions, row r of a block being the decode step of position first + r over the shared page
 * table, so it is exact but not tuned for long prompts (attention reads the cache once per row).
 *
 *   token_ids   dev int32 [n_tokens]
 *   page_table  dev int32 [max_pages]   the request's row; entries 0 .. (first_pos+n_tokens-1)/16
 *                                       must be valid pages that no other request writes
 *   model_id    source-model tag; n_tokens is added to that model's count in the pool
 *   logits_out  dev fp32 [vocab] or NULL: logits after the last prompt token
 *   next_token_out dev int32 [1] or NULL: their greedy argmax
 *   workspace   dev, 256-byte aligned, >= sun_prefill_workspace_bytes(cfg, n_tokens, max_pages)
 * `weights` must come from sun_weights_create (the prefill side stays in full precision, also
 * when decode is quantised: Section 3.3) and have the pool's shape.
 * Errors: SUN_ERR_NULL, SUN_ERR_SHAPE (also for 4-bit weights), SUN_ERR_MODEL_ID, SUN_ERR_SEQ_LEN (n_tokens < 1,
 * first_pos < 0, positions beyond the table), SUN_ERR_WORKSPACE; under SUN_VALIDATE also
 * SUN_ERR_PAGE_RANGE and SUN_ERR_TOKEN.
 */
int sun_prefill(sun_kv_pool* pool, const sun_weights* weights, int n_tokens, const int32_t* token_ids,
                const int32_t* page_table, int max_pages, int first_pos, int model_id,
                float* logits_out, int32_t* next_token_out, void* workspace, size_t workspace_bytes,
                void* stream, unsigned flags);

/* ------------------------------------------------------------------ single operations */

/*
 * The attention sub-step of the decode step on its own (same kernels, same launch
 * shape): for each request, softmax(q K^T / sqrt(d)) V over the first n_tokens[i]
 * cached positions of `layer`, GQA mapping q-head h -> kv-head h / (Hq/Hkv).
 *   q dev fp32 [batch, Hq*d] (already rotated); out dev fp32 [batch, Hq*d];
 *   n_tokens dev int32 [batch], each >= 1; n_tokens_host optional as above.
 * Reads the pool only.  Workspace as for a step.
 */
int sun_paged_attention(sun_kv_pool* pool, int layer, int batch, const float* q,
                        const int32_t* page_tables, int max_pages, const int32_t* n_tokens,
                        const int32_t* n_tokens_host, float* out, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * sun_paged_attention for callers that cannot allocate or hand over device memory for a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * the workspace, same kernels, same result.  The plan arrays, item records and split partials live in an
 * array inside the library instead (sun_paged_attention_static_limit() bytes, 16 MiB, one copy on every GPU
 * the library runs on, held until the process ends); the call allocates nothing, on the host or the device.
 *   sun_paged_attention_static_bytes(cfg, batch, max_pages): the scratch such a call needs; a call that needs
 *   more than the limit fails with SUN_ERR_WORKSPACE before anything is enqueued (use sun_paged_attention).
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (nothing in it has to be
 * cleared: every entry a kernel reads has been written by an earlier kernel of the same call).  Two calls
 * whose kernels overlap on one GPU (different streams, no ordering) race on it; calls on one stream are safe.
 * Errors: SUN_ERR_NULL, SUN_ERR_SHAPE, SUN_ERR_WORKSPACE (over the limit), SUN_ERR_HIP.
 */
size_t sun_paged_attention_static_limit(void);
size_t sun_paged_attention_static_bytes(const sun_model_cfg* cfg, int batch, int max_pages);
int sun_paged_attention_static(sun_kv_pool* pool, int layer, int batch, const float* q,
                               const int32_t* page_tables, int max_pages, const int32_t* n_tokens,
                               const int32_t* n_tokens_host, float* out, void* stream);

/*
 * out[b, n] = sum_k W[n, k] x[b, k]  through the projection kernels of the step.
 *   mat: index into the projection list of layer `layer`: 0 = [Wq;Wk;Wv] stacked,
 *        1 = Wo, 2 = fused silu(Wg x) * (Wu x) (out has ffn columns), 3 = Wd, 4 = lm_head
 *        (layer ignored).  x dev fp32 [batch, in]; out dev fp32 [batch, out].
 * Under SUN_BF16 x enters the matrix cores as in the step: two bf16 values per element (the rounded value and
 * the rounded remainder, 16 significant bits together); the output of mat 2 passes through the same split.
 */
int sun_linear(const sun_weights* weights, int layer, int mat, int batch, const float* x, float* out,
               void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------ misc */

/*
 * Measurement only (the yardstick the step's HBM-bound kernels are held against; Section 2.1: decode "must read
 * ... a growing KV cache with little compute per byte"): a kernel that does nothing but read `bytes` of device
 * memory at src in blocks of block_bytes (a multiple of 1024; 4096 = one (page, kv head) block of K or of V),
 * 16 bytes per lane and load, one block per wave and turn, in address order or in the order perm gives
 * (dev int32 [bytes / block_bytes], a permutation of the block indices), on `workgroups` workgroups of 256
 * threads; streaming_loads != 0: with the loads that pass the caches by, which the attention kernel uses for K
 * and V, else plain loads.  sink: dev, workgroups * 1024 bytes, receives one folded word per thread.
 * Asynchronous on stream.  Errors: SUN_ERR_NULL, SUN_ERR_SHAPE, SUN_ERR_HIP.
 */
int sun_hbm_read_probe(const void* src, size_t bytes, int block_bytes, const int32_t* perm, int workgroups,
                       int streaming_loads, void* sink, void* stream);

/*
 * With SUN_PROFILE the step brackets each kernel class with HIP events.  After the
 * stream is synchronised, sun_profile_read returns, for class `kind`, the summed
 * elapsed milliseconds and the number of launches since sun_profile_reset().
 * kinds: 0 attention split kernel, 1 attention combine, 2 qkv proj, 3 o proj,
 * 4 gate/up proj, 5 down proj, 6 lm_head, 7 everything else.
 */
int sun_profile_read(int kind, double* ms, int64_t* launches);
void sun_profile_reset(void);

const char* sun_last_error(void);
const char* sun_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SUN_H_ */
