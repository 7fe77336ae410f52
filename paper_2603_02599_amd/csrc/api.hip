// C ABI of libsun: handles, argument validation and the per-step launch sequence of the
// shared decode module (Section 3.1, Eq. 3; QSUN: Section 3.3, Eq. 8).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <exception>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"

namespace sun {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Host-side checks allocate with std::vector; no C++ exception may leave through the C ABI.
template <class F>
static int guarded(F&& f) {
    try {
        return f();
    } catch (const std::bad_alloc&) {
        return fail(SUN_ERR_NULL, "out of host memory");
    } catch (const std::exception& e) {
        return fail(SUN_ERR_NULL, "host error: %s", e.what());
    }
}

static int check_cfg(const sun_model_cfg* c) {
    if (!c) return fail(SUN_ERR_NULL, "cfg is NULL");
    if (c->n_layers < 1 || c->hidden < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->ffn < 1 || c->vocab < 1)
        return fail(SUN_ERR_SHAPE, "non-positive model dimension");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(SUN_ERR_SHAPE, "head_dim must be 64 or 128");
    if (c->n_q_heads % c->n_kv_heads || c->n_q_heads / c->n_kv_heads > 8)
        return fail(SUN_ERR_SHAPE, "n_q_heads must be a multiple (<= 8x) of n_kv_heads");
    if (c->hidden % 8 || (c->n_q_heads * c->head_dim) % 128)
        return fail(SUN_ERR_SHAPE, "hidden must be a multiple of 8 and n_q_heads*head_dim of 128");
    if (c->act_dtype == SUN_BF16) {
        if (c->hidden % 128 || c->ffn % 128 || c->vocab % 32)
            return fail(SUN_ERR_SHAPE, "bf16 path needs hidden, ffn multiples of 128 and vocab a multiple of 32");
    } else if (c->act_dtype != SUN_F32) {
        return fail(SUN_ERR_SHAPE, "act_dtype must be SUN_F32 or SUN_BF16");
    }
    if (c->qk_norm != 0 && c->qk_norm != 1) return fail(SUN_ERR_SHAPE, "qk_norm must be 0 or 1");
    if (c->qkv_bias != 0 && c->qkv_bias != 1) return fail(SUN_ERR_SHAPE, "qkv_bias must be 0 or 1");
    if (c->rope_scaling != 0 && c->rope_scaling != 1) return fail(SUN_ERR_SHAPE, "rope_scaling must be 0 or 1");
    if (c->rope_scaling == 1 && (!(c->rope_factor > 0.f) || !(c->rope_low_freq_factor > 0.f) ||
                                 !(c->rope_high_freq_factor > c->rope_low_freq_factor) || c->rope_original_max_position < 1))
        return fail(SUN_ERR_SHAPE, "rope scaling needs factor > 0, 0 < low_freq_factor < high_freq_factor, original length >= 1");
    return SUN_OK;
}

static bool same_shape(const sun_model_cfg& a, const sun_model_cfg& b) {
    return a.n_layers == b.n_layers && a.hidden == b.hidden && a.n_q_heads == b.n_q_heads &&
           a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim && a.ffn == b.ffn && a.vocab == b.vocab &&
           a.qk_norm == b.qk_norm && a.qkv_bias == b.qkv_bias && a.rope_scaling == b.rope_scaling &&
           (a.rope_scaling == 0 || (a.rope_original_max_position == b.rope_original_max_position &&
                                    a.rope_factor == b.rope_factor && a.rope_low_freq_factor == b.rope_low_freq_factor &&
                                    a.rope_high_freq_factor == b.rope_high_freq_factor));
}

static sun_kv_layout make_layout(const sun_model_cfg& c, int64_t n_pages) {
    sun_kv_layout L{};
    const int64_t blk = (int64_t)kPageTokens * c.head_dim;  // one (page, head) block of K or of V
    L.n_pages = n_pages;
    L.page_tokens = kPageTokens;
    L.k_page = 2 * c.n_kv_heads * blk;
    L.k_layer = n_pages * L.k_page;
    L.k_head = blk;
    L.k_token = c.head_dim;
    L.k_dim = 1;
    L.k_off = 0;
    L.v_page = L.k_page;
    L.v_layer = L.k_layer;
    L.v_head = blk;
    L.v_token = 1;
    L.v_dim = kPageTokens;
    L.v_off = c.n_kv_heads * blk;
    L.total_elems = (int64_t)c.n_layers * L.k_layer;
    return L;
}

// ---------------------------------------------------------------- workspace
struct Workspace {
    float* x;
    void *hA, *aA, *uA;         // bf16 tiled activations
    float *h32, *a32, *u32, *gu32, *qkv32, *o32;  // fp32 path
    float* qs;           // 4-bit path: (scale, integer sum) of every row and 128-wide group of the current activations
    float* part;
    float* q;
    float* table;
    AttnPlan plan;
    float* logits;
    float* amax_val;      // [batch][kArgmaxParts] slice winners of the greedy argmax
    int32_t* amax_idx;
    size_t bytes;
};

constexpr int kMaxSplits = 16;
constexpr int kMaxSplitsWide = 4;   // gate/up (2*ffn columns)

static Workspace carve(const sun_model_cfg& c, int batch, int max_pages, char* base) {
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t n) {
        char* p = base ? base + off : nullptr;
        off += align_up(n);
        return (void*)p;
    };
    const int H = c.hidden, QD = c.n_q_heads * c.head_dim, KD = c.n_kv_heads * c.head_dim, F = c.ffn;
    const int Nqkv = QD + 2 * KD;
    const int mb = atile_for_rows(batch).MB;
    w.x = (float*)take((size_t)batch * H * 4);
    w.q = (float*)take((size_t)batch * QD * 4);
    w.table = (float*)take((size_t)batch * c.head_dim * 4);
    if (c.act_dtype == SUN_BF16) {
        w.hA = take(atile_bytes(ATile{mb}, H));
        w.aA = take(atile_bytes(ATile{mb}, QD));
        w.uA = take(atile_bytes(ATile{mb}, F));
        w.qs = (float*)take((size_t)(std::max(std::max(H, QD), F) / 128 + 1) * mb * 32 * 8);  // scale and integer sum per row and group
        w.part = (float*)take(std::max((size_t)kMaxSplits * batch * std::max(Nqkv, H), (size_t)kMaxSplitsWide * batch * 2 * F) * 4);
    } else {
        w.h32 = (float*)take((size_t)batch * H * 4);
        w.a32 = (float*)take((size_t)batch * QD * 4);
        w.u32 = (float*)take((size_t)batch * F * 4);
        w.gu32 = (float*)take((size_t)batch * 2 * F * 4);
        w.qkv32 = (float*)take((size_t)batch * Nqkv * 4);
        w.o32 = (float*)take((size_t)batch * H * 4);
    }
    const size_t mc = attn_max_chunks(batch, max_pages, c.n_kv_heads);
    w.plan.max_chunks = (int)std::min<size_t>(mc, 0x7fffffff);
    w.plan.chunk_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.full_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.small_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.records = (int32_t*)take(mc * c.n_kv_heads * 24 * 4);
    w.plan.partial = (float*)take(mc * c.n_q_heads * (c.head_dim + 2) * 4);
    w.logits = (float*)take((size_t)batch * c.vocab * 4);
    w.amax_val = (float*)take((size_t)batch * kArgmaxParts * 4);
    w.amax_idx = (int32_t*)take((size_t)batch * kArgmaxParts * 4);
    w.bytes = off;
    return w;
}

// ---------------------------------------------------------------- profiling
struct ProfRec {
    int kind;
    hipEvent_t a, b;
};
static std::vector<ProfRec> g_prof;   // shared by all threads of the process
static std::mutex g_prof_mu;

struct ProfScope {
    bool on;
    hipStream_t st;
    ProfRec rec;
    ProfScope(bool enable, int kind, hipStream_t s) : on(enable), st(s) {
        if (!on) return;
        rec.kind = kind;
        if (hipEventCreate(&rec.a) != hipSuccess || hipEventCreate(&rec.b) != hipSuccess) {
            on = false;
            return;
        }
        (void)hipEventRecord(rec.a, st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(rec.b, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        try {
            g_prof.push_back(rec);
        } catch (const std::exception&) {   // this launch goes untimed
            (void)hipEventDestroy(rec.a);
            (void)hipEventDestroy(rec.b);
        }
    }
};

}  // namespace sun

using namespace sun;

// ---------------------------------------------------------------- library-owned scratch
// Scratch of sun_paged_attention_static: the plan arrays, item records and split partials that
// sun_paged_attention takes from the caller's workspace.  One copy per GPU, held until the process ends.
// In host code the array's name is only a stand-in for the symbol; the device address comes from
// hipGetSymbolAddress, once per device, and is what the kernels and carve() are given.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_static_scratch_ptr[kMaxDevices] = {};
static std::mutex g_static_scratch_mu;

// device address of this GPU's copy of the scratch array (looked up on the first call on each device)
static int static_scratch(void** out) {
    int dev = -1;
    SUN_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return sun::set_error("device %d outside [0, %d)", dev, kMaxDevices), SUN_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_static_scratch_mu);
    if (!g_static_scratch_ptr[dev]) {
        void* p = nullptr;
        SUN_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
        if (!p || (uintptr_t)p % 256) return sun::set_error("scratch symbol has no usable device address"), SUN_ERR_HIP;
        g_static_scratch_ptr[dev] = p;
    }
    *out = g_static_scratch_ptr[dev];
    return SUN_OK;
}

extern "C" {

const char* sun_last_error(void) { return g_err; }
const char* sun_version(void) { return "libsun 0.1 (gfx950)"; }

void sun_profile_reset(void) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
}

int sun_hbm_read_probe(const void* src, size_t bytes, int block_bytes, const int32_t* perm, int workgroups,
                       int streaming_loads, void* sink, void* stream) {
    if (!src || !sink) return fail(SUN_ERR_NULL, "NULL argument");
    if (block_bytes < 1024 || block_bytes % 1024 || bytes < (size_t)block_bytes || workgroups < 1 || workgroups > 65536)
        return fail(SUN_ERR_SHAPE, "block_bytes must be a multiple of 1024, bytes at least one block, workgroups in [1, 65536]");
    if ((uintptr_t)src % 16) return fail(SUN_ERR_SHAPE, "src must be 16-byte aligned");
    SUN_HIP_CHECK(launch_hbm_read_probe(src, (long long)(bytes / block_bytes), block_bytes / 16, perm, workgroups,
                                        streaming_loads != 0, (uint32_t*)sink, (hipStream_t)stream));
    return SUN_OK;
}

int sun_profile_read(int kind, double* ms, int64_t* launches) {
    if (!ms || !launches) return fail(SUN_ERR_NULL, "NULL output");
    double tot = 0;
    int64_t n = 0;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto& r : g_prof)
        if (r.kind == kind) {
            float t = 0;
            SUN_HIP_CHECK(hipEventSynchronize(r.b));
            SUN_HIP_CHECK(hipEventElapsedTime(&t, r.a, r.b));
            tot += t;
            ++n;
        }
    *ms = tot;
    *launches = n;
    return SUN_OK;
}

// ---------------------------------------------------------------- pool
size_t sun_kv_pool_bytes(const sun_model_cfg* cfg, int64_t n_pages, int page_tokens) {
    if (!cfg || n_pages < 0 || page_tokens != kPageTokens) return 0;
    return (size_t)make_layout(*cfg, n_pages).total_elems * 2;
}

int sun_kv_pool_create(const sun_model_cfg* cfg, void* dev_mem, size_t bytes, int page_tokens, int n_source_models,
                       sun_kv_pool** out) {
    if (!out) return fail(SUN_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (int rc = check_cfg(cfg)) return rc;
    if (!dev_mem) return fail(SUN_ERR_NULL, "pool memory is NULL");
    if (page_tokens != kPageTokens) return fail(SUN_ERR_SHAPE, "page_tokens must be %d", kPageTokens);
    if (n_source_models < 1) return fail(SUN_ERR_MODEL_ID, "n_source_models must be >= 1");
    if ((uintptr_t)dev_mem % 256) return fail(SUN_ERR_POOL_SIZE, "pool memory must be 256-byte aligned");
    const size_t page_bytes = sun_kv_pool_bytes(cfg, 1, page_tokens);
    const int64_t n_pages = (int64_t)(bytes / page_bytes);
    if (n_pages < 1) return fail(SUN_ERR_POOL_SIZE, "pool of %zu bytes holds no page of %zu bytes", bytes, page_bytes);
    if (n_pages > 0x7fffffff) return fail(SUN_ERR_POOL_SIZE, "too many pages");
    KvPool* p = new (std::nothrow) KvPool();
    if (!p) return fail(SUN_ERR_NULL, "out of host memory");
    p->cfg = *cfg;
    p->base = (uint16_t*)dev_mem;
    p->lay = make_layout(*cfg, n_pages);
    p->n_source_models = n_source_models;
    if (int rc = guarded([&] { p->ingested.assign((size_t)n_source_models, 0); return (int)SUN_OK; })) {
        delete p;
        return rc;
    }
    *out = (sun_kv_pool*)p;
    return SUN_OK;
}

int sun_kv_pool_layout(const sun_kv_pool* pool, sun_kv_layout* out) {
    if (!pool || !out) return fail(SUN_ERR_NULL, "NULL argument");
    *out = ((const KvPool*)pool)->lay;
    return SUN_OK;
}

void sun_kv_pool_destroy(sun_kv_pool* pool) { delete (KvPool*)pool; }

int sun_kv_pool_ingest(sun_kv_pool* pool_, int model_id, const void* k_src, const void* v_src, int n_tokens,
                       int first_pos, const int32_t* page_table, int max_pages, void* stream, unsigned flags) {
    if (!pool_ || !k_src || !v_src || !page_table) return fail(SUN_ERR_NULL, "NULL argument");
    KvPool& pool = *(KvPool*)pool_;
    if (model_id < 0 || model_id >= pool.n_source_models)
        return fail(SUN_ERR_MODEL_ID, "source-model id %d outside [0, %d)", model_id, pool.n_source_models);
    if (n_tokens < 1 || first_pos < 0 || max_pages < 1) return fail(SUN_ERR_SEQ_LEN, "n_tokens must be >= 1, first_pos >= 0");
    const long long last = (long long)first_pos + n_tokens - 1;
    if (last / kPageTokens >= max_pages)
        return fail(SUN_ERR_SEQ_LEN, "positions up to %lld need %lld page-table entries, the row has %d", last,
                    last / kPageTokens + 1, max_pages);
    if (((uintptr_t)k_src | (uintptr_t)v_src) % 16) return fail(SUN_ERR_SHAPE, "k_src and v_src must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    if (flags & SUN_VALIDATE) {
        const int rc = guarded([&]() -> int {
            std::vector<int32_t> row((size_t)max_pages);
            SUN_HIP_CHECK(hipMemcpyAsync(row.data(), page_table, row.size() * 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipStreamSynchronize(st));
            for (long long lp = first_pos / kPageTokens; lp <= last / kPageTokens; ++lp)
                if (row[lp] < 0 || row[lp] >= pool.lay.n_pages)
                    return fail(SUN_ERR_PAGE_RANGE, "page-table entry %lld = %d outside [0, %lld)", lp, row[lp],
                                (long long)pool.lay.n_pages);
            return SUN_OK;
        });
        if (rc != SUN_OK) return rc;
    }
    SUN_HIP_CHECK(launch_kv_ingest(pool, k_src, v_src, n_tokens, first_pos, page_table, st));
    pool.ingested[model_id] += n_tokens;
    return SUN_OK;
}

int sun_kv_pool_model_tokens(const sun_kv_pool* pool_, int model_id, int64_t* tokens) {
    if (!pool_ || !tokens) return fail(SUN_ERR_NULL, "NULL argument");
    const KvPool& pool = *(const KvPool*)pool_;
    if (model_id < 0 || model_id >= pool.n_source_models)
        return fail(SUN_ERR_MODEL_ID, "source-model id %d outside [0, %d)", model_id, pool.n_source_models);
    *tokens = pool.ingested[model_id];
    return SUN_OK;
}

// ---------------------------------------------------------------- weights
static void mat_dims(const sun_model_cfg& c, int which, int& N, int& K) {
    const int H = c.hidden, QD = c.n_q_heads * c.head_dim, KD = c.n_kv_heads * c.head_dim;
    switch (which) {
    case 0: N = QD + 2 * KD; K = H; break;
    case 1: N = H; K = QD; break;
    case 2: N = 2 * c.ffn; K = H; break;
    case 3: N = H; K = c.ffn; break;
    default: N = c.vocab; K = H; break;
    }
}

size_t sun_weights_pack_bytes(const sun_model_cfg* cfg) {
    if (!cfg || cfg->act_dtype != SUN_BF16) return 0;
    size_t tot = 0;
    int N, K;
    for (int m = 0; m < 4; ++m) {
        mat_dims(*cfg, m, N, K);
        tot += align_up(packed_bf16_bytes(N, K));
    }
    tot *= cfg->n_layers;
    mat_dims(*cfg, 4, N, K);
    return tot + align_up(packed_bf16_bytes(N, K));
}

size_t sun_qweights_pack_bytes(const sun_model_cfg* cfg, int group) {
    if (!cfg || cfg->act_dtype != SUN_BF16 || group != kGroup) return 0;
    size_t tot = 0;
    int N, K;
    for (int m = 0; m < 4; ++m) {
        mat_dims(*cfg, m, N, K);
        tot += align_up(packed_w4_bytes(N, K)) + align_up(packed_w4_sz_bytes(N, K));
    }
    tot *= cfg->n_layers;
    mat_dims(*cfg, 4, N, K);
    return tot + align_up(packed_bf16_bytes(N, K));
}

static Weights* new_weights(const sun_model_cfg& c, bool quant) {
    Weights* w = new (std::nothrow) Weights();
    if (!w) return nullptr;
    w->cfg = c;
    w->quant = quant;
    w->layers = new (std::nothrow) LayerW[c.n_layers]();
    if (!w->layers) {
        delete w;
        return nullptr;
    }
    return w;
}

void sun_weights_destroy(sun_weights* w) {
    Weights* p = (Weights*)w;
    if (!p) return;
    delete[] p->layers;
    delete p;
}

static int check_ptr_arrays(const void* const* const arrs[], int n_arrs, int n_layers) {
    for (int a = 0; a < n_arrs; ++a) {
        if (!arrs[a]) return fail(SUN_ERR_NULL, "a per-layer pointer array is NULL");
        for (int l = 0; l < n_layers; ++l)
            if (!arrs[a][l]) return fail(SUN_ERR_NULL, "weight pointer of layer %d is NULL", l);
    }
    return SUN_OK;
}

int sun_weights_create(const sun_model_cfg* cfg, const sun_weight_ptrs* d, void* pack_mem, size_t pack_bytes,
                       void* stream, sun_weights** out) {
    if (!out) return fail(SUN_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (int rc = check_cfg(cfg)) return rc;
    if (!d || !d->embed || !d->gf || !d->wlm) return fail(SUN_ERR_NULL, "weight table or one of embed/gf/wlm is NULL");
    const void* const* const arrs[] = {d->g1, d->wq, d->wk, d->wv, d->wo, d->g2, d->wg, d->wu, d->wd};
    if (int rc = check_ptr_arrays(arrs, 9, cfg->n_layers)) return rc;
    if (cfg->qk_norm) {
        const void* const* const narrs[] = {d->q_norm, d->k_norm};
        if (int rc = check_ptr_arrays(narrs, 2, cfg->n_layers)) return rc;
    }
    if (cfg->qkv_bias) {
        const void* const* const barrs[] = {d->bq, d->bk, d->bv};
        if (int rc = check_ptr_arrays(barrs, 3, cfg->n_layers)) return rc;
    }
    const sun_model_cfg& c = *cfg;
    const bool bf = c.act_dtype == SUN_BF16;
    if (bf) {
        if (!pack_mem) return fail(SUN_ERR_NULL, "pack_mem is NULL");
        if ((uintptr_t)pack_mem % 256 || pack_bytes < sun_weights_pack_bytes(cfg))
            return fail(SUN_ERR_WORKSPACE, "pack_mem too small or misaligned (need %zu bytes)", sun_weights_pack_bytes(cfg));
    }
    Weights* w = new_weights(c, false);
    if (!w) return fail(SUN_ERR_NULL, "out of host memory");
    hipStream_t st = (hipStream_t)stream;
    const int QD = c.n_q_heads * c.head_dim, KD = c.n_kv_heads * c.head_dim;
    char* pm = (char*)pack_mem;
    size_t off = 0;
    w->embed = d->embed;
    w->gf = d->gf;
    hipError_t e = hipSuccess;
    auto pack = [&](Mat& m, int which, const void* s0, const void* s1, const void* s2, int r0, int r1, int r2, int nsrc,
                    int mode) {
        mat_dims(c, which, m.N, m.K);
        const void* src[3] = {s0, s1, s2};
        const int rows[3] = {r0, r1, r2};
        if (bf) {
            m.kind = MAT_BF16_PACKED;
            m.w = pm + off;
            if (e == hipSuccess) e = launch_pack_bf16(src, rows, nsrc, mode, m.K, pm + off, st);
            off += align_up(packed_bf16_bytes(m.N, m.K));
        } else {
            m.kind = MAT_F32;
            m.nsrc = nsrc;
            for (int i = 0; i < 3; ++i) {
                m.wsrc[i] = src[i];
                m.src_rows[i] = rows[i];
            }
        }
    };
    for (int l = 0; l < c.n_layers; ++l) {
        LayerW& L = w->layers[l];
        L.g1 = d->g1[l];
        L.g2 = d->g2[l];
        if (c.qk_norm) {
            L.qn = d->q_norm[l];
            L.kn = d->k_norm[l];
        }
        if (c.qkv_bias) {
            L.bq = d->bq[l];
            L.bk = d->bk[l];
            L.bv = d->bv[l];
        }
        pack(L.qkv, 0, d->wq[l], d->wk[l], d->wv[l], QD, KD, KD, 3, 0);
        pack(L.o, 1, d->wo[l], nullptr, nullptr, c.hidden, 0, 0, 1, 0);
        pack(L.gu, 2, d->wg[l], d->wu[l], nullptr, c.ffn, c.ffn, 0, 2, bf ? 1 : 0);
        pack(L.down, 3, d->wd[l], nullptr, nullptr, c.hidden, 0, 0, 1, 0);
    }
    pack(w->lm, 4, d->wlm, nullptr, nullptr, c.vocab, 0, 0, 1, 0);
    if (e == hipSuccess && bf) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        sun_weights_destroy((sun_weights*)w);
        return fail(SUN_ERR_HIP, "weight packing failed: %s", hipGetErrorString(e));
    }
    *out = (sun_weights*)w;
    return SUN_OK;
}

int sun_qweights_create(const sun_model_cfg* cfg, const sun_qweight_ptrs* d, int group, void* pack_mem,
                        size_t pack_bytes, void* stream, sun_weights** out) {
    if (!out) return fail(SUN_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (int rc = check_cfg(cfg)) return rc;
    if (group != kGroup) return fail(SUN_ERR_SHAPE, "group must be %d", kGroup);
    if (!d || !d->embed || !d->gf || !d->wlm) return fail(SUN_ERR_NULL, "weight table or one of embed/gf/wlm is NULL");
    const void* const* const arrs[] = {d->g1, d->g2};
    if (int rc = check_ptr_arrays(arrs, 2, cfg->n_layers)) return rc;
    if (cfg->qk_norm) {
        const void* const* const narrs[] = {d->q_norm, d->k_norm};
        if (int rc = check_ptr_arrays(narrs, 2, cfg->n_layers)) return rc;
    }
    if (cfg->qkv_bias) {
        const void* const* const barrs[] = {d->bq, d->bk, d->bv};
        if (int rc = check_ptr_arrays(barrs, 3, cfg->n_layers)) return rc;
    }
    const sun_qmat* const qarrs[] = {d->wq, d->wk, d->wv, d->wo, d->wg, d->wu, d->wd};
    int with_z = 0, without_z = 0;
    for (auto qa : qarrs) {
        if (!qa) return fail(SUN_ERR_NULL, "a per-layer quantised matrix array is NULL");
        for (int l = 0; l < cfg->n_layers; ++l) {
            if (!qa[l].q || !qa[l].s) return fail(SUN_ERR_NULL, "quantised matrix of layer %d has a NULL part", l);
            ++(qa[l].z ? with_z : without_z);
        }
    }
    if (with_z && without_z)
        return fail(SUN_ERR_NULL, "zero points must be given for every quantised matrix or for none (symmetric layout)");
    const bool s_only = without_z > 0;
    const sun_model_cfg& c = *cfg;
    const int QD = c.n_q_heads * c.head_dim;
    if (c.hidden % kGroup || c.ffn % kGroup || QD % kGroup)
        return fail(SUN_ERR_SHAPE, "every projection input width must be a multiple of the group (%d)", kGroup);
    const bool bf = c.act_dtype == SUN_BF16;
    if (bf) {
        if (!pack_mem) return fail(SUN_ERR_NULL, "pack_mem is NULL");
        if ((uintptr_t)pack_mem % 256 || pack_bytes < sun_qweights_pack_bytes(cfg, group))
            return fail(SUN_ERR_WORKSPACE, "pack_mem too small or misaligned (need %zu bytes)",
                        sun_qweights_pack_bytes(cfg, group));
    }
    Weights* w = new_weights(c, true);
    if (!w) return fail(SUN_ERR_NULL, "out of host memory");
    hipStream_t st = (hipStream_t)stream;
    const int KD = c.n_kv_heads * c.head_dim;
    char* pm = (char*)pack_mem;
    size_t off = 0;
    w->embed = d->embed;
    w->gf = d->gf;
    hipError_t e = hipSuccess;
    auto pack = [&](Mat& m, int which, const sun_qmat* s0, const sun_qmat* s1, const sun_qmat* s2, int r0, int r1, int r2,
                    int nsrc, int mode) {
        mat_dims(c, which, m.N, m.K);
        sun_qmat src[3] = {s0 ? *s0 : sun_qmat{}, s1 ? *s1 : sun_qmat{}, s2 ? *s2 : sun_qmat{}};
        const int rows[3] = {r0, r1, r2};
        if (bf) {
            m.kind = MAT_W4_PACKED;
            m.s_only = s_only;
            m.w = pm + off;
            m.sz = pm + off + align_up(packed_w4_bytes(m.N, m.K));
            if (e == hipSuccess) e = launch_pack_w4(src, rows, nsrc, mode, m.K, (void*)m.w, (void*)m.sz, st);
            off += align_up(packed_w4_bytes(m.N, m.K)) + align_up(packed_w4_sz_bytes(m.N, m.K));
        } else {
            m.kind = MAT_W4_LOGICAL;
            m.nsrc = nsrc;
            for (int i = 0; i < 3; ++i) {
                m.q[i] = (const uint8_t*)src[i].q;
                m.s[i] = (const uint16_t*)src[i].s;
                m.z[i] = (const uint16_t*)src[i].z;
                m.src_rows[i] = rows[i];
            }
        }
    };
    for (int l = 0; l < c.n_layers; ++l) {
        LayerW& L = w->layers[l];
        L.g1 = d->g1[l];
        L.g2 = d->g2[l];
        if (c.qk_norm) {
            L.qn = d->q_norm[l];
            L.kn = d->k_norm[l];
        }
        if (c.qkv_bias) {
            L.bq = d->bq[l];
            L.bk = d->bk[l];
            L.bv = d->bv[l];
        }
        pack(L.qkv, 0, &d->wq[l], &d->wk[l], &d->wv[l], QD, KD, KD, 3, 0);
        pack(L.o, 1, &d->wo[l], nullptr, nullptr, c.hidden, 0, 0, 1, 0);
        pack(L.gu, 2, &d->wg[l], &d->wu[l], nullptr, c.ffn, c.ffn, 0, 2, bf ? 1 : 0);
        pack(L.down, 3, &d->wd[l], nullptr, nullptr, c.hidden, 0, 0, 1, 0);
    }
    {   // lm_head stays dense (Appendix A.1)
        Mat& m = w->lm;
        mat_dims(c, 4, m.N, m.K);
        const void* src[3] = {d->wlm, nullptr, nullptr};
        const int rows[3] = {c.vocab, 0, 0};
        if (bf) {
            m.kind = MAT_BF16_PACKED;
            m.w = pm + off;
            if (e == hipSuccess) e = launch_pack_bf16(src, rows, 1, 0, m.K, pm + off, st);
            off += align_up(packed_bf16_bytes(m.N, m.K));
        } else {
            m.kind = MAT_F32;
            m.nsrc = 1;
            m.wsrc[0] = d->wlm;
            m.src_rows[0] = c.vocab;
        }
    }
    if (e == hipSuccess && bf) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        sun_weights_destroy((sun_weights*)w);
        return fail(SUN_ERR_HIP, "weight packing failed: %s", hipGetErrorString(e));
    }
    *out = (sun_weights*)w;
    return SUN_OK;
}

int sun_quantize_w4(const void* w, int dtype, int rows, int cols, int group, int mode, void* q, void* s, void* z,
                    void* stream) {
    if (!w || !q || !s || (!z && mode != 1)) return fail(SUN_ERR_NULL, "NULL argument");
    if (dtype != SUN_F32 && dtype != SUN_BF16) return fail(SUN_ERR_SHAPE, "dtype must be SUN_F32 or SUN_BF16");
    if (group != kGroup || rows < 1 || cols < kGroup || cols % kGroup) return fail(SUN_ERR_SHAPE, "group must be 128 and divide cols");
    if (mode != 0 && mode != 1) return fail(SUN_ERR_SHAPE, "mode must be 0 (affine) or 1 (symmetric)");
    SUN_HIP_CHECK(launch_quantize_w4(w, dtype, rows, cols, group, mode, q, s, z, (hipStream_t)stream));
    return SUN_OK;
}

// ---------------------------------------------------------------- step
size_t sun_workspace_bytes(const sun_model_cfg* cfg, int max_batch, int max_pages) {
    if (!cfg || max_batch < 1 || max_pages < 1 || check_cfg(cfg) != SUN_OK) return 0;
    return carve(*cfg, max_batch, max_pages, nullptr).bytes;
}

static int validate_device_arrays(const KvPool& pool, int batch, const int32_t* token_ids, const int32_t* page_tables,
                                  int max_pages, const int32_t* seq_lens, const int32_t* model_ids, int len_plus,
                                  hipStream_t st) {
    std::vector<int32_t> tok(batch), len(batch), ids(batch), pt((size_t)batch * max_pages);
    if (token_ids) SUN_HIP_CHECK(hipMemcpyAsync(tok.data(), token_ids, batch * 4, hipMemcpyDeviceToHost, st));
    SUN_HIP_CHECK(hipMemcpyAsync(len.data(), seq_lens, batch * 4, hipMemcpyDeviceToHost, st));
    if (model_ids) SUN_HIP_CHECK(hipMemcpyAsync(ids.data(), model_ids, batch * 4, hipMemcpyDeviceToHost, st));
    SUN_HIP_CHECK(hipMemcpyAsync(pt.data(), page_tables, pt.size() * 4, hipMemcpyDeviceToHost, st));
    SUN_HIP_CHECK(hipStreamSynchronize(st));
    std::vector<int32_t> tails;
    for (int b = 0; b < batch; ++b) {
        if (token_ids && (tok[b] < 0 || tok[b] >= pool.cfg.vocab))
            return fail(SUN_ERR_TOKEN, "request %d: token id %d outside [0, %d)", b, tok[b], pool.cfg.vocab);
        if (model_ids && (ids[b] < 0 || ids[b] >= pool.n_source_models))
            return fail(SUN_ERR_MODEL_ID, "request %d: source-model id %d outside [0, %d)", b, ids[b], pool.n_source_models);
        const int64_t n = (int64_t)len[b] + len_plus;
        if (len[b] < 0 || n < 1) return fail(SUN_ERR_SEQ_LEN, "request %d: length %d is invalid", b, len[b]);
        const int64_t need = (n + kPageTokens - 1) / kPageTokens;
        if (need > max_pages)
            return fail(SUN_ERR_SEQ_LEN, "request %d: %lld positions need %lld pages, table has %d", b, (long long)n,
                        (long long)need, max_pages);
        for (int64_t p = 0; p < need; ++p) {
            const int32_t id = pt[(size_t)b * max_pages + p];
            if (id < 0 || id >= pool.lay.n_pages)
                return fail(SUN_ERR_PAGE_RANGE, "request %d: page table entry %lld is %d, pool has %lld pages", b,
                            (long long)p, id, (long long)pool.lay.n_pages);
        }
        if (len_plus) tails.push_back(pt[(size_t)b * max_pages + need - 1]);
    }
    if (len_plus) {  // the page written this step must not be referenced by another request
        std::vector<int32_t> sorted = tails;
        std::sort(sorted.begin(), sorted.end());
        for (size_t i = 1; i < sorted.size(); ++i)
            if (sorted[i] == sorted[i - 1])
                return fail(SUN_ERR_PAGE_RANGE, "page %d is the write target of two requests", sorted[i]);
    }
    return SUN_OK;
}

// Chunk counts of the batch (all chunks; full chunks) from lengths the host knows, as the plan kernel computes
// them on the device; -1 when the host has no lengths.
struct ChunkHint {
    int total, full;
};
static ChunkHint chunks_from_host(const int32_t* host, int len_plus, int batch, int max_pages, int Hkv) {
    if (!host) return ChunkHint{-1, -1};
    long long tot = 0, full = 0;
    const long long cap = (long long)max_pages * kPageTokens;
    for (int b = 0; b < batch; ++b) {
        const long long n = std::min(std::max<long long>((long long)host[b] + len_plus, 1), cap);
        int nf, ns, ch;
        attn_chunking((int)n, batch, Hkv, nf, ns, ch);
        tot += nf + ns;
        full += nf;
    }
    return ChunkHint{(int)std::min<long long>(tot, 0x7fffffff), (int)std::min<long long>(full, 0x7fffffff)};
}

static int step_impl(sun_kv_pool* pool_, const sun_weights* weights_, bool want_quant, int batch,
                     const int32_t* token_ids, const int32_t* page_tables, int max_pages, const int32_t* seq_lens,
                     const int32_t* seq_lens_host, const int32_t* model_ids, float* logits_out,
                     int32_t* next_tokens_out, void* workspace, size_t workspace_bytes, void* stream, unsigned flags,
                     bool with_head = true) {
    if (!pool_ || !weights_) return fail(SUN_ERR_NULL, "pool or weights is NULL");
    if (!token_ids || !page_tables || !seq_lens || !model_ids || !next_tokens_out || !workspace)
        return fail(SUN_ERR_NULL, "a required device pointer is NULL");
    KvPool& pool = *(KvPool*)pool_;
    const Weights& W = *(const Weights*)weights_;
    const sun_model_cfg& c = W.cfg;
    if (W.quant != want_quant)
        return fail(SUN_ERR_SHAPE, want_quant ? "sun_qdecode_step needs weights from sun_qweights_create"
                                              : "sun_decode_step needs weights from sun_weights_create");
    if (!same_shape(c, pool.cfg)) return fail(SUN_ERR_SHAPE, "pool and weights were created for different shapes");
    if (batch < 1 || batch > kMaxBatchTile) return fail(SUN_ERR_SHAPE, "batch must be in [1, %d]", kMaxBatchTile);
    if (max_pages < 1) return fail(SUN_ERR_SHAPE, "max_pages must be >= 1");
    if ((uintptr_t)workspace % 256) return fail(SUN_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const Workspace ws = carve(c, batch, max_pages, (char*)workspace);
    if (ws.bytes > workspace_bytes)
        return fail(SUN_ERR_WORKSPACE, "workspace has %zu bytes, step needs %zu", workspace_bytes, ws.bytes);
    hipStream_t st = (hipStream_t)stream;
    if (flags & SUN_VALIDATE)
        if (int rc = guarded([&] {
                return validate_device_arrays(pool, batch, token_ids, page_tables, max_pages, seq_lens, model_ids, 1, st);
            }))
            return rc;
    const bool prof = flags & SUN_PROFILE;
    const bool bf = c.act_dtype == SUN_BF16;
    const int H = c.hidden;
    const ChunkHint hint = chunks_from_host(seq_lens_host, 1, batch, max_pages, c.n_kv_heads);
    float* logits = logits_out ? logits_out : ws.logits;

    {
        ProfScope p(prof, 7, st);
        SUN_HIP_CHECK(launch_embed(c, W.embed, token_ids, batch, ws.x, st));
        SUN_HIP_CHECK(launch_rope_table(c, seq_lens, batch, ws.table, st));
        SUN_HIP_CHECK(launch_attn_plan(ws.plan, seq_lens, 1, batch, page_tables, max_pages, (int)pool.lay.n_pages, c.n_kv_heads, st));
    }
    int down_parts = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW& L = W.layers[l];
        const float* attn_q = ws.q;
        if (bf) {
            {
                ProfScope p(prof, 7, st);
                SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.part, down_parts, batch, L.g1, batch, nullptr, ws.hA,
                                                   W.quant ? ws.qs : nullptr, st));
            }
            const int sq = proj_pick_splits(L.qkv, batch, kMaxSplits);
            {
                ProfScope p(prof, 2, st);
                ProjLaunch pl{&L.qkv, ws.hA, ws.qs, batch, EPI_STORE, sq, ws.part, L.qkv.N, batch};
                SUN_HIP_CHECK(launch_proj(pl, st));
            }
            {
                ProfScope p(prof, 7, st);
                SUN_HIP_CHECK(launch_rope_append(pool, l, ws.part, sq, batch, ws.table, seq_lens, page_tables, max_pages,
                                                 batch, ws.q, L.qn, L.kn, L.bq, L.bk, L.bv, st));
            }
        } else {
            ProfScope p(prof, 7, st);
            if (l > 0) SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.o32, 1, batch, L.g1, batch, ws.h32, nullptr, nullptr, st));
            else SUN_HIP_CHECK(launch_residual_norm(c, ws.x, nullptr, 0, batch, L.g1, batch, ws.h32, nullptr, nullptr, st));
            SUN_HIP_CHECK(launch_proj_f32(L.qkv, ws.h32, batch, ws.qkv32, st));
            SUN_HIP_CHECK(launch_rope_append(pool, l, ws.qkv32, 1, batch, ws.table, seq_lens, page_tables, max_pages,
                                             batch, ws.q, L.qn, L.kn, L.bq, L.bk, L.bv, st));
        }
        {
            ProfScope p(prof, 0, st);
            SUN_HIP_CHECK(launch_attn_split(pool, l, ws.plan, attn_q, page_tables, max_pages, seq_lens, 1, batch, hint.total,
                                            hint.full, !bf, st));
        }
        {
            ProfScope p(prof, 1, st);
            SUN_HIP_CHECK(launch_attn_combine(c, ws.plan, batch, bf ? nullptr : ws.a32, bf ? ws.aA : nullptr,
                                              (bf && W.quant) ? ws.qs : nullptr, st));
        }
        if (bf) {
            const int so = proj_pick_splits(L.o, batch, kMaxSplits);
            {
                ProfScope p(prof, 3, st);
                ProjLaunch pl{&L.o, ws.aA, ws.qs, batch, EPI_STORE, so, ws.part, H, batch};
                SUN_HIP_CHECK(launch_proj(pl, st));
            }
            {
                ProfScope p(prof, 7, st);
                SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.part, so, batch, L.g2, batch, nullptr, ws.hA,
                                                   W.quant ? ws.qs : nullptr, st));
            }
            if (!W.quant && batch > 64) {
                // bf16 above 64 rows (no split-K there): SwiGLU in the epilogue, the down projection's tile as
                // output.  Up to 64 rows the two-way split over 256 workgroups plus a separate SwiGLU kernel is
                // faster: unsplit, the 28672 columns make 224 workgroups and leave 32 compute units idle.
                ProfScope p(prof, 4, st);
                ProjLaunch pl{&L.gu, ws.hA, nullptr, batch, EPI_SWIGLU, 1, (float*)ws.uA, L.gu.N, batch};
                SUN_HIP_CHECK(launch_proj(pl, st));
            } else {
                const int sg = proj_pick_splits(L.gu, batch, kMaxSplitsWide);
                {
                    ProfScope p(prof, 4, st);
                    ProjLaunch pl{&L.gu, ws.hA, ws.qs, batch, EPI_STORE, sg, ws.part, L.gu.N, batch};
                    SUN_HIP_CHECK(launch_proj(pl, st));
                }
                {
                    ProfScope p(prof, 7, st);
                    SUN_HIP_CHECK(launch_swiglu_tile(ws.part, sg, batch, batch, c.ffn, ws.uA, W.quant ? ws.qs : nullptr, st));
                }
            }
            const int sd = proj_pick_splits(L.down, batch, kMaxSplits);
            {
                ProfScope p(prof, 5, st);
                ProjLaunch pl{&L.down, ws.uA, ws.qs, batch, EPI_STORE, sd, ws.part, H, batch};
                SUN_HIP_CHECK(launch_proj(pl, st));
            }
            down_parts = sd;
        } else {
            ProfScope p(prof, 7, st);
            SUN_HIP_CHECK(launch_proj_f32(L.o, ws.a32, batch, ws.o32, st));
            SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.o32, 1, batch, L.g2, batch, ws.h32, nullptr, nullptr, st));
            SUN_HIP_CHECK(launch_proj_f32(L.gu, ws.h32, batch, ws.gu32, st));
            SUN_HIP_CHECK(launch_swiglu_f32(ws.gu32, batch, c.ffn, ws.u32, st));
            SUN_HIP_CHECK(launch_proj_f32(L.down, ws.u32, batch, ws.o32, st));
        }
    }
    if (!with_head) return SUN_OK;  // a caller that only wants the cache entries (all but the last prefill block)
    {
        ProfScope p(prof, 7, st);
        if (bf) SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.part, down_parts, batch, W.gf, batch, nullptr, ws.hA, nullptr, st));
        else SUN_HIP_CHECK(launch_residual_norm(c, ws.x, ws.o32, 1, batch, W.gf, batch, ws.h32, nullptr, nullptr, st));
    }
    {
        ProfScope p(prof, 6, st);
        if (bf) {
            ProjLaunch pl{&W.lm, ws.hA, nullptr, batch, EPI_STORE, 1, logits, c.vocab, batch};
            SUN_HIP_CHECK(launch_proj(pl, st));
        } else {
            SUN_HIP_CHECK(launch_proj_f32(W.lm, ws.h32, batch, logits, st));
        }
    }
    {
        ProfScope p(prof, 7, st);
        SUN_HIP_CHECK(launch_argmax(logits, batch, c.vocab, ws.amax_val, ws.amax_idx, next_tokens_out, st));
    }
    return SUN_OK;
}

int sun_decode_step(sun_kv_pool* pool, const sun_weights* weights, int batch, const int32_t* token_ids,
                    const int32_t* page_tables, int max_pages, const int32_t* seq_lens, const int32_t* seq_lens_host,
                    const int32_t* model_ids, float* logits_out, int32_t* next_tokens_out, void* workspace,
                    size_t workspace_bytes, void* stream, unsigned flags) {
    return step_impl(pool, weights, false, batch, token_ids, page_tables, max_pages, seq_lens, seq_lens_host, model_ids,
                     logits_out, next_tokens_out, workspace, workspace_bytes, stream, flags);
}

int sun_qdecode_step(sun_kv_pool* pool, const sun_weights* weights, int batch, const int32_t* token_ids,
                     const int32_t* page_tables, int max_pages, const int32_t* seq_lens, const int32_t* seq_lens_host,
                     const int32_t* model_ids, float* logits_out, int32_t* next_tokens_out, void* workspace,
                     size_t workspace_bytes, void* stream, unsigned flags) {
    return step_impl(pool, weights, true, batch, token_ids, page_tables, max_pages, seq_lens, seq_lens_host, model_ids,
                     logits_out, next_tokens_out, workspace, workspace_bytes, stream, flags);
}

// ---------------------------------------------------------------- multi-step run
int sun_decode_run(sun_kv_pool* pool_, const sun_weights* weights_, int batch, int n_steps, int32_t* token_ids,
                   int32_t* page_tables, int max_pages, int32_t* seq_lens, const int32_t* model_ids,
                   const int32_t* free_pages, int n_free, int32_t* free_head, int32_t* run_status, int32_t* tokens_out,
                   float* logits_out, void* workspace, size_t workspace_bytes, void* stream, unsigned flags) {
    if (!pool_ || !weights_) return fail(SUN_ERR_NULL, "pool or weights is NULL");
    if (!free_head || !run_status || !tokens_out) return fail(SUN_ERR_NULL, "free_head, run_status or tokens_out is NULL");
    if (n_free < 0 || (n_free > 0 && !free_pages)) return fail(SUN_ERR_NULL, "free_pages is NULL but n_free > 0");
    if (n_steps < 1) return fail(SUN_ERR_SHAPE, "n_steps must be >= 1");
    const Weights& W = *(const Weights*)weights_;
    if (flags & SUN_VALIDATE) {
        const int vrc = guarded([&]() -> int {
            const KvPool& pool = *(const KvPool*)pool_;
            if (!token_ids || !page_tables || !seq_lens || !model_ids) return fail(SUN_ERR_NULL, "a required device pointer is NULL");
            if (batch < 1 || batch > kMaxBatchTile || max_pages < 1) return fail(SUN_ERR_SHAPE, "bad batch or max_pages");
            hipStream_t st = (hipStream_t)stream;
            std::vector<int32_t> fp((size_t)n_free), tabs((size_t)batch * max_pages);
            int32_t head = 0;
            if (n_free) SUN_HIP_CHECK(hipMemcpyAsync(fp.data(), free_pages, fp.size() * 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipMemcpyAsync(tabs.data(), page_tables, tabs.size() * 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipMemcpyAsync(&head, free_head, 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipStreamSynchronize(st));
            if (head < 0 || head > n_free) return fail(SUN_ERR_PAGE_RANGE, "free_head %d outside [0, %d]", head, n_free);
            std::vector<char> used((size_t)pool.lay.n_pages, 0);
            for (int32_t pg : tabs)
                if (pg >= 0 && pg < pool.lay.n_pages) used[pg] = 1;
            for (int i = head; i < n_free; ++i) {
                const int32_t pg = fp[i];
                if (pg < 0 || pg >= pool.lay.n_pages) return fail(SUN_ERR_PAGE_RANGE, "free_pages[%d] = %d outside the pool", i, pg);
                if (used[pg]) return fail(SUN_ERR_PAGE_RANGE, "free_pages[%d] = %d is referenced by a page table or listed twice", i, pg);
                used[pg] = 1;
            }
            return SUN_OK;
        });
        if (vrc != SUN_OK) return vrc;
    }
    for (int s = 0; s < n_steps; ++s) {
        const bool last = s + 1 == n_steps;
        // only the first step can be validated from the host: later inputs exist on the device only
        const int rc = step_impl(pool_, weights_, W.quant, batch, token_ids, page_tables, max_pages, seq_lens, nullptr,
                                 model_ids, last ? logits_out : nullptr, tokens_out + (size_t)s * batch, workspace,
                                 workspace_bytes, stream, s == 0 ? flags : (flags & ~SUN_VALIDATE));
        if (rc != SUN_OK) return rc;
        SUN_HIP_CHECK(launch_advance(tokens_out + (size_t)s * batch, batch, max_pages, free_pages, n_free, token_ids,
                                     page_tables, seq_lens, free_head, run_status, s == 0, (hipStream_t)stream));
    }
    return SUN_OK;
}

// ---------------------------------------------------------------- continuous batching
static int validate_serve(const KvPool& pool, const sun_serve_state& s, int slots, int max_pages, bool reset,
                          hipStream_t st) {
    const int64_t n_pages = pool.lay.n_pages;
    if (s.idle_page < 0 || s.idle_page >= n_pages)
        return fail(SUN_ERR_PAGE_RANGE, "idle_page %d outside [0, %lld)", s.idle_page, (long long)n_pages);
    int32_t cnt[8];
    SUN_HIP_CHECK(hipMemcpyAsync(cnt, s.counters, sizeof cnt, hipMemcpyDeviceToHost, st));
    SUN_HIP_CHECK(hipStreamSynchronize(st));
    const int whead = cnt[0], head = cnt[1], tail = cnt[2];
    if (whead < 0 || whead > s.n_wait) return fail(SUN_ERR_SHAPE, "counters[0] = %d outside [0, n_wait]", whead);
    if (head < 0 || tail < head || tail - head > s.ring_cap)
        return fail(SUN_ERR_PAGE_RANGE, "ring head %d / tail %d do not fit a ring of %d", head, tail, s.ring_cap);
    const int n_ring = tail - head, n_q = s.n_wait - whead;
    std::vector<int32_t> ring((size_t)s.ring_cap), wt((size_t)n_q * max_pages), wl(n_q), wtok(n_q), wm(n_q), wb(n_q);
    SUN_HIP_CHECK(hipMemcpyAsync(ring.data(), s.ring, ring.size() * 4, hipMemcpyDeviceToHost, st));
    if (n_q) {
        SUN_HIP_CHECK(hipMemcpyAsync(wt.data(), s.w_tables + (size_t)whead * max_pages, wt.size() * 4, hipMemcpyDeviceToHost, st));
        SUN_HIP_CHECK(hipMemcpyAsync(wl.data(), s.w_lens + whead, n_q * 4, hipMemcpyDeviceToHost, st));
        SUN_HIP_CHECK(hipMemcpyAsync(wtok.data(), s.w_token + whead, n_q * 4, hipMemcpyDeviceToHost, st));
        SUN_HIP_CHECK(hipMemcpyAsync(wm.data(), s.w_model + whead, n_q * 4, hipMemcpyDeviceToHost, st));
        SUN_HIP_CHECK(hipMemcpyAsync(wb.data(), s.w_budget + whead, n_q * 4, hipMemcpyDeviceToHost, st));
    }
    std::vector<int32_t> rows, rreq;
    if (!reset) {
        rows.resize((size_t)slots * max_pages);
        rreq.resize(slots);
        SUN_HIP_CHECK(hipMemcpyAsync(rows.data(), s.page_tables, rows.size() * 4, hipMemcpyDeviceToHost, st));
        SUN_HIP_CHECK(hipMemcpyAsync(rreq.data(), s.slot_req, slots * 4, hipMemcpyDeviceToHost, st));
    }
    SUN_HIP_CHECK(hipStreamSynchronize(st));
    std::vector<char> used((size_t)n_pages, 0);
    used[s.idle_page] = 1;
    auto claim = [&](int32_t pg, const char* what, int idx) -> int {
        if (pg < 0 || pg >= n_pages) return fail(SUN_ERR_PAGE_RANGE, "%s %d: page %d outside the pool", what, idx, pg);
        if (used[pg]) return fail(SUN_ERR_PAGE_RANGE, "%s %d: page %d is listed twice (or is the idle page)", what, idx, pg);
        used[pg] = 1;
        return SUN_OK;
    };
    for (int i = 0; i < n_ring; ++i)
        if (int rc = claim(ring[(size_t)((unsigned)(head + i) % (unsigned)s.ring_cap)], "ring entry", i)) return rc;
    for (int q = 0; q < n_q; ++q) {
        if (wtok[q] < 0 || wtok[q] >= pool.cfg.vocab) return fail(SUN_ERR_TOKEN, "waiting request %d: token %d", whead + q, wtok[q]);
        if (wm[q] < 0 || wm[q] >= pool.n_source_models) return fail(SUN_ERR_MODEL_ID, "waiting request %d: model id %d", whead + q, wm[q]);
        if (wl[q] < 0 || wl[q] / kPageTokens >= max_pages || wb[q] < 1)
            return fail(SUN_ERR_SEQ_LEN, "waiting request %d: length %d / budget %d do not fit", whead + q, wl[q], wb[q]);
        for (int c = 0; c < max_pages; ++c) {
            const int32_t pg = wt[(size_t)q * max_pages + c];
            if (pg < 0) {
                if (c <= wl[q] / kPageTokens)
                    return fail(SUN_ERR_PAGE_RANGE, "waiting request %d: no page for position %d", whead + q, c * kPageTokens);
                continue;
            }
            if (int rc = claim(pg, "waiting request", whead + q)) return rc;
        }
    }
    for (int i = 0; i < (reset ? 0 : slots); ++i) {
        if (rreq[i] < 0) continue;
        for (int c = 0; c < max_pages; ++c)
            if (rows[(size_t)i * max_pages + c] >= 0)
                if (int rc = claim(rows[(size_t)i * max_pages + c], "row", i)) return rc;
    }
    return SUN_OK;
}

size_t sun_serve_workspace_bytes(const sun_model_cfg* cfg, int slots, int max_pages) {
    const size_t step = sun_workspace_bytes(cfg, slots, max_pages);
    return step ? step + align_up((size_t)slots * 4) : 0;
}

int sun_decode_serve(sun_kv_pool* pool_, const sun_weights* weights_, int slots, int max_pages, int n_steps,
                     const sun_serve_state* state, int32_t* tokens_out, int32_t* req_out, float* logits_out,
                     void* workspace, size_t workspace_bytes, void* stream, unsigned flags) {
    if (!pool_ || !weights_ || !state) return fail(SUN_ERR_NULL, "pool, weights or state is NULL");
    const sun_serve_state& s = *state;
    if (!s.token_ids || !s.page_tables || !s.seq_lens || !s.model_ids || !s.slot_req || !s.slot_left || !s.ring ||
        !s.counters || !tokens_out || !req_out || !workspace)
        return fail(SUN_ERR_NULL, "a required device pointer is NULL");
    if (s.n_wait < 0 || (s.n_wait > 0 && (!s.w_req || !s.w_token || !s.w_tables || !s.w_lens || !s.w_model || !s.w_budget)))
        return fail(s.n_wait < 0 ? SUN_ERR_SHAPE : SUN_ERR_NULL, "waiting queue: n_wait < 0 or a NULL array");
    if (slots < 1 || slots > kMaxBatchTile || max_pages < 1 || n_steps < 1 || s.ring_cap < 1)
        return fail(SUN_ERR_SHAPE, "slots must be in [1, %d], max_pages, n_steps and ring_cap >= 1", kMaxBatchTile);
    KvPool& pool = *(KvPool*)pool_;
    const Weights& W = *(const Weights*)weights_;
    if (!same_shape(W.cfg, pool.cfg)) return fail(SUN_ERR_SHAPE, "pool and weights were created for different shapes");
    if ((uintptr_t)workspace % 256) return fail(SUN_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const size_t step_bytes = carve(W.cfg, slots, max_pages, nullptr).bytes;
    const size_t next_bytes = align_up((size_t)slots * 4);
    if (step_bytes + next_bytes > workspace_bytes)
        return fail(SUN_ERR_WORKSPACE, "workspace has %zu bytes, serving needs %zu", workspace_bytes, step_bytes + next_bytes);
    hipStream_t st = (hipStream_t)stream;
    const bool reset = flags & SUN_SERVE_RESET;
    if (flags & SUN_VALIDATE)
        if (int rc = guarded([&] { return validate_serve(pool, s, slots, max_pages, reset, st); })) return rc;
    int32_t* next = (int32_t*)((char*)workspace + step_bytes);
    ServeArgs a{s.token_ids, s.page_tables, s.seq_lens, s.model_ids, s.slot_req, s.slot_left, s.w_req, s.w_token,
                s.w_tables, s.w_lens, s.w_model, s.w_budget, s.ring, s.counters, s.n_wait, s.ring_cap, s.idle_page,
                s.eos_id, slots, max_pages};
    if (reset) SUN_HIP_CHECK(launch_serve(a, nullptr, nullptr, nullptr, true, false, st));
    const unsigned step_flags = flags & SUN_PROFILE;
    for (int i = 0; i < n_steps; ++i) {
        const bool last = i + 1 == n_steps;
        const int rc = step_impl(pool_, weights_, W.quant, slots, s.token_ids, s.page_tables, max_pages, s.seq_lens, nullptr,
                                 s.model_ids, last ? logits_out : nullptr, next, workspace, step_bytes, stream, step_flags);
        if (rc != SUN_OK) return rc;
        SUN_HIP_CHECK(launch_serve(a, next, tokens_out + (size_t)i * slots, req_out + (size_t)i * slots, false, true, st));
    }
    return SUN_OK;
}

// ---------------------------------------------------------------- prefill
// Extra device memory of a prefill behind the step's workspace: per-row page tables, lengths,
// model ids and next tokens of one block of rows.
struct PrefillExtra {
    int32_t *tables, *lens, *ids, *next;
    size_t bytes;
};

static PrefillExtra carve_prefill(int rows, int max_pages, char* base) {
    PrefillExtra e{};
    size_t off = 0;
    auto take = [&](size_t n) {
        char* p = base ? base + off : nullptr;
        off += align_up(n);
        return (int32_t*)p;
    };
    e.tables = take((size_t)rows * max_pages * 4);
    e.lens = take((size_t)rows * 4);
    e.ids = take((size_t)rows * 4);
    e.next = take((size_t)rows * 4);
    e.bytes = off;
    return e;
}

size_t sun_prefill_workspace_bytes(const sun_model_cfg* cfg, int n_tokens, int max_pages) {
    if (!cfg || n_tokens < 1 || max_pages < 1 || check_cfg(cfg) != SUN_OK) return 0;
    const int rows = std::min(n_tokens, kMaxBatchTile);
    return carve(*cfg, rows, max_pages, nullptr).bytes + carve_prefill(rows, max_pages, nullptr).bytes;
}

int sun_prefill(sun_kv_pool* pool_, const sun_weights* weights_, int n_tokens, const int32_t* token_ids,
                const int32_t* page_table, int max_pages, int first_pos, int model_id, float* logits_out,
                int32_t* next_token_out, void* workspace, size_t workspace_bytes, void* stream, unsigned flags) {
    if (!pool_ || !weights_) return fail(SUN_ERR_NULL, "pool or weights is NULL");
    if (!token_ids || !page_table || !workspace) return fail(SUN_ERR_NULL, "a required device pointer is NULL");
    KvPool& pool = *(KvPool*)pool_;
    const Weights& W = *(const Weights*)weights_;
    const sun_model_cfg& c = W.cfg;
    if (!same_shape(c, pool.cfg)) return fail(SUN_ERR_SHAPE, "pool and weights were created for different shapes");
    if (W.quant) return fail(SUN_ERR_SHAPE, "prefill runs in full precision: weights must come from sun_weights_create");
    if (model_id < 0 || model_id >= pool.n_source_models)
        return fail(SUN_ERR_MODEL_ID, "source-model id %d outside [0, %d)", model_id, pool.n_source_models);
    if (n_tokens < 1 || first_pos < 0 || max_pages < 1) return fail(SUN_ERR_SEQ_LEN, "n_tokens must be >= 1, first_pos >= 0");
    const long long last = (long long)first_pos + n_tokens - 1;
    if (last / kPageTokens >= max_pages)
        return fail(SUN_ERR_SEQ_LEN, "positions up to %lld need %lld page-table entries, the row has %d", last,
                    last / kPageTokens + 1, max_pages);
    if ((uintptr_t)workspace % 256) return fail(SUN_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const int rows_max = std::min(n_tokens, kMaxBatchTile);
    const size_t step_bytes = carve(c, rows_max, max_pages, nullptr).bytes;
    const PrefillExtra ex = carve_prefill(rows_max, max_pages, (char*)workspace + step_bytes);
    if (step_bytes + ex.bytes > workspace_bytes)
        return fail(SUN_ERR_WORKSPACE, "workspace has %zu bytes, prefill needs %zu", workspace_bytes, step_bytes + ex.bytes);
    hipStream_t st = (hipStream_t)stream;
    if (flags & SUN_VALIDATE) {
        const int vrc = guarded([&]() -> int {
            std::vector<int32_t> row((size_t)max_pages), tok((size_t)n_tokens);
            SUN_HIP_CHECK(hipMemcpyAsync(row.data(), page_table, row.size() * 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipMemcpyAsync(tok.data(), token_ids, tok.size() * 4, hipMemcpyDeviceToHost, st));
            SUN_HIP_CHECK(hipStreamSynchronize(st));
            for (long long lp = 0; lp <= last / kPageTokens; ++lp)
                if (row[lp] < 0 || row[lp] >= pool.lay.n_pages)
                    return fail(SUN_ERR_PAGE_RANGE, "page-table entry %lld = %d outside [0, %lld)", lp, row[lp],
                                (long long)pool.lay.n_pages);
            for (int i = 0; i < n_tokens; ++i)
                if (tok[i] < 0 || tok[i] >= c.vocab)
                    return fail(SUN_ERR_TOKEN, "prompt token %d: id %d outside [0, %d)", i, tok[i], c.vocab);
            return SUN_OK;
        });
        if (vrc != SUN_OK) return vrc;
    }
    // Row r of a block is the decode step of position first + r over the one page table: its
    // attention spans positions 0..first + r, and the K/V of all rows of the block are in the
    // pool before the block's attention starts, which is the causal forward of Eq. 2.
    const unsigned step_flags = flags & ~SUN_VALIDATE;
    for (int done = 0; done < n_tokens; done += kMaxBatchTile) {
        const int rows = std::min(n_tokens - done, kMaxBatchTile);
        const bool last_block = done + rows == n_tokens;
        SUN_HIP_CHECK(launch_prefill_rows(page_table, max_pages, first_pos + done, model_id, rows, ex.tables, ex.lens, ex.ids, st));
        const int rc = step_impl(pool_, weights_, false, rows, token_ids + done, ex.tables, max_pages, ex.lens, nullptr,
                                 ex.ids, nullptr, ex.next, workspace, step_bytes, stream, step_flags,
                                 last_block && (logits_out || next_token_out));
        if (rc != SUN_OK) return rc;
        if (last_block) {
            const Workspace ws = carve(c, rows, max_pages, (char*)workspace);
            if (logits_out)
                SUN_HIP_CHECK(hipMemcpyAsync(logits_out, ws.logits + (size_t)(rows - 1) * c.vocab, (size_t)c.vocab * 4,
                                             hipMemcpyDeviceToDevice, st));
            if (next_token_out)
                SUN_HIP_CHECK(hipMemcpyAsync(next_token_out, ex.next + rows - 1, 4, hipMemcpyDeviceToDevice, st));
        }
    }
    pool.ingested[model_id] += n_tokens;
    return SUN_OK;
}

// ---------------------------------------------------------------- single operations
int sun_paged_attention(sun_kv_pool* pool_, int layer, int batch, const float* q, const int32_t* page_tables,
                        int max_pages, const int32_t* n_tokens, const int32_t* n_tokens_host, float* out,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (!pool_ || !q || !page_tables || !n_tokens || !out || !workspace) return fail(SUN_ERR_NULL, "NULL argument");
    KvPool& pool = *(KvPool*)pool_;
    const sun_model_cfg& c = pool.cfg;
    if (layer < 0 || layer >= c.n_layers) return fail(SUN_ERR_SHAPE, "layer out of range");
    if (batch < 1 || batch > 1024 || max_pages < 1) return fail(SUN_ERR_SHAPE, "batch must be in [1,1024], max_pages >= 1");
    if ((uintptr_t)workspace % 256) return fail(SUN_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const Workspace ws = carve(c, batch, max_pages, (char*)workspace);
    if (ws.bytes > workspace_bytes) return fail(SUN_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, ws.bytes);
    hipStream_t st = (hipStream_t)stream;
    const ChunkHint hint = chunks_from_host(n_tokens_host, 0, batch, max_pages, c.n_kv_heads);
    SUN_HIP_CHECK(launch_attn_plan(ws.plan, n_tokens, 0, batch, page_tables, max_pages, (int)pool.lay.n_pages, c.n_kv_heads, st));
    SUN_HIP_CHECK(launch_attn_split(pool, layer, ws.plan, q, page_tables, max_pages, n_tokens, 0, batch, hint.total, hint.full,
                                    c.act_dtype == SUN_F32, st));
    SUN_HIP_CHECK(launch_attn_combine(c, ws.plan, batch, out, nullptr, nullptr, st));
    return SUN_OK;
}

// The part of the workspace the attention sub-step uses: plan arrays, item records, split partials.
static Workspace carve_attention(const sun_model_cfg& c, int batch, int max_pages, char* base) {
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t n) {
        char* p = base ? base + off : nullptr;
        off += align_up(n);
        return (void*)p;
    };
    const size_t mc = attn_max_chunks(batch, max_pages, c.n_kv_heads);
    w.plan.max_chunks = (int)std::min<size_t>(mc, 0x7fffffff);
    w.plan.chunk_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.full_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.small_off = (int32_t*)take((size_t)(batch + 1) * 4);
    w.plan.records = (int32_t*)take(mc * c.n_kv_heads * 24 * 4);
    w.plan.partial = (float*)take(mc * c.n_q_heads * (c.head_dim + 2) * 4);
    w.bytes = off;
    return w;
}

size_t sun_paged_attention_static_limit(void) { return kStaticScratchBytes; }

size_t sun_paged_attention_static_bytes(const sun_model_cfg* cfg, int batch, int max_pages) {
    if (!cfg || batch < 1 || max_pages < 1 || check_cfg(cfg) != SUN_OK) return 0;
    return carve_attention(*cfg, batch, max_pages, nullptr).bytes;
}

int sun_paged_attention_static(sun_kv_pool* pool_, int layer, int batch, const float* q, const int32_t* page_tables,
                               int max_pages, const int32_t* n_tokens, const int32_t* n_tokens_host, float* out,
                               void* stream) {
    if (!pool_ || !q || !page_tables || !n_tokens || !out) return fail(SUN_ERR_NULL, "NULL argument");
    KvPool& pool = *(KvPool*)pool_;
    const sun_model_cfg& c = pool.cfg;
    if (layer < 0 || layer >= c.n_layers) return fail(SUN_ERR_SHAPE, "layer out of range");
    if (batch < 1 || batch > 1024 || max_pages < 1) return fail(SUN_ERR_SHAPE, "batch must be in [1,1024], max_pages >= 1");
    const size_t need = carve_attention(c, batch, max_pages, nullptr).bytes;
    if (need > kStaticScratchBytes)
        return fail(SUN_ERR_WORKSPACE, "batch %d x %d pages needs %zu bytes of scratch, the library's array holds %zu: "
                    "use sun_paged_attention with a workspace", batch, max_pages, need, kStaticScratchBytes);
    void* base = nullptr;
    if (int rc = static_scratch(&base)) return rc;
    const Workspace ws = carve_attention(c, batch, max_pages, (char*)base);
    hipStream_t st = (hipStream_t)stream;
    const ChunkHint hint = chunks_from_host(n_tokens_host, 0, batch, max_pages, c.n_kv_heads);
    // nothing in the scratch has to start at zero: the plan kernels write every prefix sum and every record the
    // split kernel reads, the split kernel every partial the combine kernel reads
    SUN_HIP_CHECK(launch_attn_plan(ws.plan, n_tokens, 0, batch, page_tables, max_pages, (int)pool.lay.n_pages, c.n_kv_heads, st));
    SUN_HIP_CHECK(launch_attn_split(pool, layer, ws.plan, q, page_tables, max_pages, n_tokens, 0, batch, hint.total, hint.full,
                                    c.act_dtype == SUN_F32, st));
    SUN_HIP_CHECK(launch_attn_combine(c, ws.plan, batch, out, nullptr, nullptr, st));
    return SUN_OK;
}

int sun_linear(const sun_weights* weights_, int layer, int mat, int batch, const float* x, float* out, void* workspace,
               size_t workspace_bytes, void* stream) {
    if (!weights_ || !x || !out || !workspace) return fail(SUN_ERR_NULL, "NULL argument");
    const Weights& W = *(const Weights*)weights_;
    const sun_model_cfg& c = W.cfg;
    if (mat < 0 || mat > 4 || (mat < 4 && (layer < 0 || layer >= c.n_layers))) return fail(SUN_ERR_SHAPE, "bad layer/mat");
    if (batch < 1 || batch > kMaxBatchTile) return fail(SUN_ERR_SHAPE, "batch must be in [1, %d]", kMaxBatchTile);
    if ((uintptr_t)workspace % 256) return fail(SUN_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    const Workspace ws = carve(c, batch, 1, (char*)workspace);
    if (ws.bytes > workspace_bytes) return fail(SUN_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", workspace_bytes, ws.bytes);
    hipStream_t st = (hipStream_t)stream;
    const Mat& M = mat == 4 ? W.lm : mat == 0 ? W.layers[layer].qkv : mat == 1 ? W.layers[layer].o
                                 : mat == 2 ? W.layers[layer].gu : W.layers[layer].down;
    if (c.act_dtype == SUN_F32) {
        if (mat == 2) {
            SUN_HIP_CHECK(launch_proj_f32(M, x, batch, ws.gu32, st));
            SUN_HIP_CHECK(launch_swiglu_f32(ws.gu32, batch, c.ffn, out, st));
        } else {
            SUN_HIP_CHECK(launch_proj_f32(M, x, batch, out, st));
        }
        return SUN_OK;
    }
    // the tiled input goes to the buffer the step uses for this projection's input
    void* in = mat == 1 ? ws.aA : mat == 3 ? ws.uA : ws.hA;
    const bool w4 = M.kind == MAT_W4_PACKED;
    SUN_HIP_CHECK(launch_tile_rows(x, batch, M.K, in, w4 ? ws.qs : nullptr, st));
    if (mat == 2) {
        if (!w4) {
            ProjLaunch pl{&M, in, nullptr, batch, EPI_SWIGLU, 1, (float*)ws.uA, M.N, batch};
            SUN_HIP_CHECK(launch_proj(pl, st));
        } else {
            const int s = proj_pick_splits(M, batch, kMaxSplitsWide);
            ProjLaunch pl{&M, in, ws.qs, batch, EPI_STORE, s, ws.part, M.N, batch};
            SUN_HIP_CHECK(launch_proj(pl, st));
            SUN_HIP_CHECK(launch_swiglu_tile(ws.part, s, batch, batch, c.ffn, ws.uA, nullptr, st));
        }
        SUN_HIP_CHECK(launch_untile_rows(ws.uA, batch, c.ffn, out, st));
    } else if (mat == 4) {
        ProjLaunch pl{&M, in, nullptr, batch, EPI_STORE, 1, out, M.N, batch};
        SUN_HIP_CHECK(launch_proj(pl, st));
    } else {
        const int s = proj_pick_splits(M, batch, kMaxSplits);
        ProjLaunch pl{&M, in, ws.qs, batch, EPI_STORE, s, ws.part, M.N, batch};
        SUN_HIP_CHECK(launch_proj(pl, st));
        SUN_HIP_CHECK(launch_reduce_partials(ws.part, s, batch, batch, M.N, out, st));
    }
    return SUN_OK;
}

}  // extern "C"
