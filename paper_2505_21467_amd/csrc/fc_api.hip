// C-ABI host layer of libfreecache: argument validation, launch planning, kernel enqueue.
// Every check happens before the first HIP call of an entry point.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "fc_internal.h"

namespace {

thread_local char g_err[512] = "";

fc_status fail(fc_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

size_t esize_of(int dtype) { return dtype == FC_F32 ? 4 : 2; }

// Validate a configuration; on failure fills the error text and returns the status.
fc_status check_config(const fc_config *c)
{
    if (!c) return fail(FC_ERR_INVALID_ARG, "config is NULL");
    if (c->dtype != FC_F32 && c->dtype != FC_BF16)
        return fail(FC_ERR_INVALID_ARG, "dtype %d is neither FC_F32 nor FC_BF16", c->dtype);
    if (c->n_layers < 1 || c->batch < 1 || c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 ||
        c->head_dim < 1 || c->max_seq < 1)
        return fail(FC_ERR_INVALID_ARG, "config sizes must be positive");
    if (!(c->rope_base > 1.0f) || !isfinite(c->rope_base))
        return fail(FC_ERR_INVALID_ARG, "rope_base must be finite and > 1");
    if (c->softmax_scale < 0.0f || !isfinite(c->softmax_scale))
        return fail(FC_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    if (c->n_q_heads % c->n_kv_heads != 0)
        return fail(FC_ERR_UNSUPPORTED, "n_q_heads %d is not a multiple of n_kv_heads %d", c->n_q_heads,
                    c->n_kv_heads);
    if (c->head_dim != 64 && c->head_dim != 128)
        return fail(FC_ERR_UNSUPPORTED, "head_dim %d not supported (64 or 128)", c->head_dim);
    if (c->hidden % 8 != 0) return fail(FC_ERR_UNSUPPORTED, "hidden %d is not a multiple of 8", c->hidden);
    if (c->max_seq > (1 << 24)) return fail(FC_ERR_UNSUPPORTED, "max_seq %d exceeds 2^24", c->max_seq);
    if (c->batch > 65535 || c->n_q_heads > 65535)
        return fail(FC_ERR_UNSUPPORTED, "batch and n_q_heads are limited to 65535");
    return FC_OK;
}

int spad_of(const fc_config &c) { return (c.max_seq + FC_VTILE - 1) / FC_VTILE * FC_VTILE; }

FcGeom geom_of(const fc_cache *cache)
{
    const fc_config &c = cache->cfg;
    FcGeom G;
    G.B = c.batch;
    G.d = c.hidden;
    G.Hq = c.n_q_heads;
    G.Hkv = c.n_kv_heads;
    G.Dh = c.head_dim;
    G.max_seq = c.max_seq;
    G.spad = cache->spad;
    G.g = c.n_q_heads / c.n_kv_heads;
    G.scale = c.softmax_scale > 0.f ? c.softmax_scale : (float)(1.0 / sqrt((double)c.head_dim));
    G.log_base = log((double)c.rope_base);
    return G;
}

void *layer_ptr(const fc_cache *c, void *base, int layer)
{
    return (char *)base + (size_t)layer * c->layer_elems * c->esize;
}

fc_status check_cache_layer(const fc_cache *cache, int32_t layer)
{
    if (!cache) return fail(FC_ERR_INVALID_ARG, "cache is NULL");
    if (layer < 0 || layer >= cache->cfg.n_layers)
        return fail(FC_ERR_BOUNDS, "layer %d outside [0, %d)", layer, cache->cfg.n_layers);
    return FC_OK;
}

fc_status hip_fail(hipError_t e, const char *what)
{
    return fail(FC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Launch planning (pure host functions).

// Tuning knobs (see FcKnobs): read from the environment once, then changed only by fc_tuning_set.
namespace {

FcKnobs g_knobs;
bool g_knobs_init = false;

void knobs_defaults(FcKnobs &k)
{
    memset(&k, 0, sizeof k);
    k.lin_wide_shape = -1;
    k.proj_gemm_shape = -1;
}

// Apply one "NAME", "value" pair (value NULL = back to the default).  False for an unknown name.
bool knob_apply(FcKnobs &k, const char *name, const char *value)
{
    FcKnobs d;
    knobs_defaults(d);
    const int v = value ? atoi(value) : 0;
    if (!strcmp(name, "FC_ATTN_TILES")) {
        k.attn_r = k.attn_w = 0;
        if (value) sscanf(value, "%d,%d", &k.attn_r, &k.attn_w);
    } else if (!strcmp(name, "FC_ATTN_WGS")) k.attn_wgs = value ? v : d.attn_wgs;
    else if (!strcmp(name, "FC_LIN_WGS")) k.lin_wgs = value ? v : d.lin_wgs;
    else if (!strcmp(name, "FC_LIN_NO_ROWS")) k.lin_no_rows = value ? 1 : 0;
    else if (!strcmp(name, "FC_LIN_WIDE_SHAPE")) k.lin_wide_shape = value ? v : d.lin_wide_shape;
    else if (!strcmp(name, "FC_LIN_KSPLIT")) k.lin_ksplit = value ? v : d.lin_ksplit;
    else if (!strcmp(name, "FC_GEMM_NO_SPLIT")) k.gemm_no_split = value ? 1 : 0;
    else if (!strcmp(name, "FC_PROJ_GEMM_SHAPE")) k.proj_gemm_shape = value ? v : d.proj_gemm_shape;
    else if (!strcmp(name, "FC_PROJ_NO_HEADSPLIT")) k.proj_no_headsplit = value ? 1 : 0;
    else if (!strcmp(name, "FC_ACCEPT_WGS")) k.accept_wgs = value ? v : d.accept_wgs;
    else return false;
    return true;
}

const char *const KNOB_NAMES[] = {"FC_ATTN_TILES", "FC_ATTN_WGS", "FC_LIN_WGS", "FC_LIN_NO_ROWS", "FC_LIN_WIDE_SHAPE",
                                  "FC_LIN_KSPLIT", "FC_GEMM_NO_SPLIT", "FC_PROJ_GEMM_SHAPE", "FC_PROJ_NO_HEADSPLIT",
                                  "FC_ACCEPT_WGS"};

FcKnobs &knobs_mut()
{
    if (!g_knobs_init) {
        knobs_defaults(g_knobs);
        for (const char *n : KNOB_NAMES)
            if (const char *e = getenv(n)) knob_apply(g_knobs, n, e);
        g_knobs_init = true;
    }
    return g_knobs;
}

}  // namespace

const FcKnobs &fc_knobs() { return knobs_mut(); }

FcAttnPlan fc_plan_attention(const fc_config &cfg, int A, int kv_len)
{
    FcAttnPlan p;
    memset(&p, 0, sizeof p);
    p.splits = p.splits_bound = 1;
    if (cfg.dtype != FC_BF16 || cfg.head_dim != 128) return p;  // kind 0: generic kernel
    p.kind = 1;
    const int g = cfg.n_q_heads / cfg.n_kv_heads;
    p.row_tiles = (int)(((int64_t)g * A + 31) / 32);
    // Row tiles per workgroup: 2 (four waves share one tile pair), 4 or 8 (each wave its own pair).
    // One workgroup per compute unit (its LDS ring takes 128 KB), so aim for one wave of them.
    const int r_default = p.row_tiles <= 2 ? 2 : (p.row_tiles <= 7 ? 4 : 8);
    int R = r_default, W = 8, target = 256;
    {
        // A short cache cannot give 256 eight-wave workgroups (a split takes at least 128 keys): with
        // 3..7 row tiles, four-wave workgroups of two tiles, two per compute unit, then fill the chip
        // better (one sequence, 28/4 heads, 32 rows: 10.7 against 12.7 us at 1056 keys, 11.4 against
        // 13.9 at 2112; from about 4000 keys on the eight-wave shape is as fast or faster).
        const int64_t n_rg8 = (p.row_tiles + r_default - 1) / r_default;
        const int64_t base8 = (int64_t)cfg.batch * cfg.n_kv_heads * n_rg8;
        const int64_t st = (kv_len + 63) / 64, by_len8 = st / 2 > 1 ? st / 2 : 1;
        int64_t sp8 = (256 + base8 / 2) / base8;
        if (sp8 > by_len8) sp8 = by_len8;
        if (sp8 < 1) sp8 = 1;
        if (r_default == 4 && base8 * sp8 < 256) {
            R = 2;
            W = 4;
        }
    }
    {
        const FcKnobs &kn = fc_knobs();
        if (kn.attn_r > 0 && kn.attn_w > 0) {
            R = kn.attn_r;
            W = kn.attn_w;
        }
        if (kn.attn_wgs > 0) target = kn.attn_wgs;
    }
    if (R != 2 && R != 4 && R != 8) R = r_default;
    if (W != 4 && W != 8) W = 8;
    if (W == 4) {  // four-wave workgroups: two or four tiles, two workgroups per compute unit
        if (R == 8) R = 4;
        if (target == 256) target = 512;
    }
    p.tiles_per_wg = R;
    p.waves = W;  // one row tile per wave group either way
    const int64_t n_rg = (p.row_tiles + R - 1) / R;
    const int64_t base = (int64_t)cfg.batch * cfg.n_kv_heads * n_rg;
    const int n_stages = (kv_len + 63) / 64;
    // enough workgroups to fill the chip; rounded to nearest, so that a grid that nearly fills it
    // already is not doubled (the partial results of a split are extra traffic)
    int64_t splits = (target + base / 2) / base;
    const int64_t by_len = n_stages / 2 > 1 ? n_stages / 2 : 1;  // at least 128 keys per split
    if (splits > by_len) splits = by_len;
    if (splits < 1) splits = 1;
    p.splits_bound = (int)splits;
    const int stages_per_split = (int)((n_stages + splits - 1) / splits);
    p.keys_per_split = stages_per_split * 64;
    p.splits = (n_stages + stages_per_split - 1) / stages_per_split;
    return p;
}

size_t fc_plan_workspace(const fc_config &cfg, const FcAttnPlan &p, int A)
{
    if (p.kind == 0 || p.splits_bound <= 1) return 0;
    // per (32-row tile, split): 32 x Dh partial outputs as half floats + 32 x 4 floats of row state
    (void)A;
    return (size_t)cfg.batch * cfg.n_kv_heads * p.row_tiles * p.splits_bound * 32 *
           (cfg.head_dim * 2 + 4 * sizeof(float));
}

extern "C" {

const char *fc_last_error(void) { return g_err; }

fc_status fc_tuning_set(const char *name, const char *value)
{
    if (!name) return fail(FC_ERR_INVALID_ARG, "name is NULL");
    if (!knob_apply(knobs_mut(), name, value)) return fail(FC_ERR_INVALID_ARG, "unknown tuning knob %s", name);
    return FC_OK;
}

fc_status fc_attention_plan(const fc_config *cfg, int32_t A, int32_t kv_len, int32_t *plan)
{
    fc_status st = check_config(cfg);
    if (st != FC_OK) return st;
    if (!plan) return fail(FC_ERR_INVALID_ARG, "plan is NULL");
    if (A < 1) return fail(FC_ERR_INVALID_ARG, "A %d must be >= 1", A);
    if (kv_len < 1 || kv_len > cfg->max_seq) return fail(FC_ERR_BOUNDS, "kv_len %d outside [1, %d]", kv_len, cfg->max_seq);
    const FcAttnPlan p = fc_plan_attention(*cfg, A, kv_len);
    plan[0] = p.kind;
    plan[1] = p.splits;
    plan[2] = p.keys_per_split;
    plan[3] = p.row_tiles;
    plan[4] = p.tiles_per_wg;
    plan[5] = p.waves;
    return FC_OK;
}

size_t fc_cache_storage_bytes(const fc_config *cfg)
{
    if (check_config(cfg) != FC_OK) return 0;
    return (size_t)cfg->n_layers * cfg->batch * cfg->n_kv_heads * spad_of(*cfg) * cfg->head_dim *
           esize_of(cfg->dtype);
}

fc_status fc_cache_alloc(const fc_config *cfg, void *k_storage, void *v_storage, fc_cache **out)
{
    if (!out) return fail(FC_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    fc_status st = check_config(cfg);
    if (st != FC_OK) return st;
    if ((k_storage == nullptr) != (v_storage == nullptr))
        return fail(FC_ERR_INVALID_ARG, "k_storage and v_storage must both be given or both be NULL");
    if (k_storage && (((uintptr_t)k_storage | (uintptr_t)v_storage) & 15))
        return fail(FC_ERR_INVALID_ARG, "cache storage must be 16-byte aligned");
    fc_cache *c = new (std::nothrow) fc_cache;
    if (!c) return fail(FC_ERR_OOM, "host allocation failed");
    c->cfg = *cfg;
    c->spad = spad_of(*cfg);
    c->esize = esize_of(cfg->dtype);
    c->layer_elems = (size_t)cfg->batch * cfg->n_kv_heads * c->spad * cfg->head_dim;
    c->k = k_storage;
    c->v = v_storage;
    c->owned = false;
    c->ws_A = c->ws_d_ff = 0;
    for (int i = 0; i < 64; ++i)
        c->inv_freq[i] = i < cfg->head_dim / 2 ? pow((double)cfg->rope_base, -2.0 * i / cfg->head_dim) : 0.0;
    if (!k_storage) {
        const size_t bytes = fc_cache_storage_bytes(cfg);
        void *k = nullptr, *v = nullptr;
        if (hipMalloc(&k, bytes) != hipSuccess || hipMalloc(&v, bytes) != hipSuccess ||
            hipMemset(k, 0, bytes) != hipSuccess || hipMemset(v, 0, bytes) != hipSuccess) {
            (void)hipGetLastError();
            if (k) (void)hipFree(k);
            if (v) (void)hipFree(v);
            delete c;
            return fail(FC_ERR_OOM, "could not allocate 2 x %zu bytes of cache storage", bytes);
        }
        c->k = k;
        c->v = v;
        c->owned = true;
    }
    // Scratch for kernels that hand partial results between workgroups.  On a host without a GPU
    // (argument-validation tests) the handle is still created; compute calls then fail at launch.
    c->scratch = nullptr;
    {
        void *s = nullptr;
        const hipError_t e = hipMalloc(&s, FC_SCRATCH_BYTES);
        if (e == hipSuccess) {
            c->scratch = s;
        } else {
            (void)hipGetLastError();
            if (s) (void)hipFree(s);
            int ndev = 0;
            if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) {
                if (c->owned) {
                    (void)hipFree(c->k);
                    (void)hipFree(c->v);
                }
                delete c;
                return fail(FC_ERR_OOM, "could not allocate %u bytes of device scratch", FC_SCRATCH_BYTES);
            }
            (void)hipGetLastError();
        }
    }
    *out = c;
    return FC_OK;
}

fc_status fc_cache_free(fc_cache *cache)
{
    if (!cache) return FC_OK;
    fc_status st = FC_OK;
    if (cache->owned) {
        hipError_t e1 = hipFree(cache->k), e2 = hipFree(cache->v);
        if (e1 != hipSuccess || e2 != hipSuccess) st = hip_fail(e1 != hipSuccess ? e1 : e2, "hipFree");
    }
    if (cache->scratch) {
        hipError_t e = hipFree(cache->scratch);
        if (e != hipSuccess && st == FC_OK) st = hip_fail(e, "hipFree");
    }
    delete cache;
    return st;
}

fc_status fc_cache_ptrs(const fc_cache *cache, int32_t layer, void **k, void **v)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!k || !v) return fail(FC_ERR_INVALID_ARG, "k or v is NULL");
    *k = layer_ptr(cache, cache->k, layer);
    *v = layer_ptr(cache, cache->v, layer);
    return FC_OK;
}

static fc_status copy_rows(const fc_cache *cache, int32_t layer, void *k_rows, void *v_rows,
                           int32_t start, int32_t rows, void *stream, bool to_cache)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!k_rows || !v_rows) return fail(FC_ERR_INVALID_ARG, "k_rows or v_rows is NULL");
    if (rows < 1) return fail(FC_ERR_INVALID_ARG, "rows %d must be >= 1", rows);
    if (start < 0 || start > cache->cfg.max_seq - rows)
        return fail(FC_ERR_BOUNDS, "rows [%d, %d+%d) outside the cache of %d rows", start, start, rows,
                    cache->cfg.max_seq);
    hipError_t e = fc_launch_copy_rows(geom_of(cache), cache->cfg.dtype, layer_ptr(cache, cache->k, layer),
                                       layer_ptr(cache, cache->v, layer), k_rows, v_rows, start, rows,
                                       to_cache, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "row copy launch");
}

fc_status fc_cache_write_rows(fc_cache *cache, int32_t layer, const void *k_rows, const void *v_rows,
                              int32_t start, int32_t rows, void *stream)
{
    return copy_rows(cache, layer, (void *)k_rows, (void *)v_rows, start, rows, stream, true);
}

fc_status fc_cache_read_rows(const fc_cache *cache, int32_t layer, void *k_rows, void *v_rows,
                             int32_t start, int32_t rows, void *stream)
{
    return copy_rows(cache, layer, k_rows, v_rows, start, rows, stream, false);
}

fc_status fc_window(int32_t step, int32_t P, int32_t G, int32_t Bk, int32_t steps_per_block,
                    int32_t refresh_every, int32_t mode, int32_t *win_start, int32_t *rows,
                    int32_t *refresh_after)
{
    if (!win_start || !rows || !refresh_after) return fail(FC_ERR_INVALID_ARG, "output pointer is NULL");
    if (step < 0 || P < 0 || G < 1 || Bk < 1 || steps_per_block < 1 || refresh_every < 0)
        return fail(FC_ERR_INVALID_ARG, "step/P >= 0, G/Bk/steps_per_block >= 1, refresh_every >= 0 required");
    if (mode != 0 && mode != 1) return fail(FC_ERR_INVALID_ARG, "mode %d is neither 0 nor 1", mode);
    const int64_t n_blocks = ((int64_t)G + Bk - 1) / Bk;
    const int64_t blk = step / steps_per_block;
    if (blk >= n_blocks)
        return fail(FC_ERR_BOUNDS, "step %d lies past the last of %lld blocks", step, (long long)n_blocks);
    const int64_t first = blk * Bk;  // offset of the block inside the generation region
    const int64_t rest = (int64_t)G - first;
    if ((int64_t)P + G > INT32_MAX) return fail(FC_ERR_INVALID_ARG, "P + G overflows int32");
    *win_start = (int32_t)(P + first);
    *rows = (int32_t)(mode == 1 ? rest : (rest < Bk ? rest : Bk));
    *refresh_after = (refresh_every > 0 && ((int64_t)step + 1) % refresh_every == 0) ? 1 : 0;
    return FC_OK;
}

fc_status fc_qkv_project_scatter(fc_cache *cache, int32_t layer, const void *x, const void *w_qkv,
                                 const void *b_qkv, int32_t win_start, int32_t A, const int32_t *pos,
                                 void *q_out, void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!x || !w_qkv || !q_out) return fail(FC_ERR_INVALID_ARG, "x, w_qkv or q_out is NULL");
    if (A < 1) return fail(FC_ERR_INVALID_ARG, "A %d must be >= 1", A);
    if ((int64_t)A * cache->cfg.batch > (1 << 24))
        return fail(FC_ERR_UNSUPPORTED, "batch * A exceeds 2^24 rows");
    if (!pos && (win_start < 0 || win_start > cache->cfg.max_seq - A))
        return fail(FC_ERR_BOUNDS, "window [%d, %d+%d) outside the cache of %d rows", win_start, win_start,
                    A, cache->cfg.max_seq);
    const FcGeom G = geom_of(cache);
    void *kl = layer_ptr(cache, cache->k, layer), *vl = layer_ptr(cache, cache->v, layer);
    // wide windows: tiled GEMM; short windows: weight-streaming kernels; other shapes: plain ALU kernel
    hipError_t e;
    if (fc_project_gemm_supported(cache->cfg, cache->cfg.batch * A))
        e = fc_launch_project_gemm(G, x, w_qkv, b_qkv, pos, win_start, A, q_out, kl, vl, (hipStream_t)stream);
    else if (fc_project_mfma_supported(cache->cfg, A))
        e = fc_launch_project_mfma(G, cache->inv_freq, x, w_qkv, b_qkv, pos, win_start, A, q_out, kl, vl,
                                   cache->scratch, (hipStream_t)stream);
    else
        e = fc_launch_project_generic(G, cache->cfg.dtype, x, w_qkv, b_qkv, pos, win_start, A, q_out, kl, vl,
                                      (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "projection launch");
}

size_t fc_workspace_bytes(const fc_config *cfg, int32_t max_rows)
{
    if (check_config(cfg) != FC_OK || max_rows < 1) return 0;
    size_t best = 0;
    for (int a = 1; a <= max_rows; ++a) {
        const FcAttnPlan p = fc_plan_attention(*cfg, a, cfg->max_seq);
        const size_t b = fc_plan_workspace(*cfg, p, a);
        if (b > best) best = b;
    }
    return best;
}

fc_status fc_active_attention(fc_cache *cache, int32_t layer, const void *q, int32_t A, int32_t kv_len,
                              const int32_t *pos, void *out, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!q || !out) return fail(FC_ERR_INVALID_ARG, "q or out is NULL");
    if (A < 1) return fail(FC_ERR_INVALID_ARG, "A %d must be >= 1", A);
    if ((int64_t)A * cache->cfg.batch > (1 << 24))
        return fail(FC_ERR_UNSUPPORTED, "batch * A exceeds 2^24 rows");
    if (kv_len < 1 || kv_len > cache->cfg.max_seq)
        return fail(FC_ERR_BOUNDS, "kv_len %d outside [1, %d]", kv_len, cache->cfg.max_seq);
    const FcAttnPlan plan = fc_plan_attention(cache->cfg, A, kv_len);
    const size_t need = fc_plan_workspace(cache->cfg, plan, A);
    if (need > 0 && (!workspace || workspace_bytes < need))
        return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : (size_t)0);
    const FcGeom G = geom_of(cache);
    void *kl = layer_ptr(cache, cache->k, layer), *vl = layer_ptr(cache, cache->v, layer);
    hipError_t e = plan.kind == 1
                       ? fc_launch_attention_mfma(G, plan, q, kl, vl, pos, A, kv_len, out, workspace,
                                                  (hipStream_t)stream)
                       : fc_launch_attention_generic(G, cache->cfg.dtype, q, kl, vl, pos, A, kv_len, out,
                                                     (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "attention launch");
}

// ---------------------------------------------------------------------------------------------
// Attention for callers that cannot allocate: the split-KV partial results live in a static device
// array instead of a caller-provided workspace.  The array's name is only a host-side stand-in for
// the symbol; its device address is looked up once per device and kept.
}  // extern "C"

#define FC_STATIC_SCRATCH_BYTES (16u * 1024u * 1024u)
#define FC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char fc_static_scratch[FC_STATIC_SCRATCH_BYTES];

namespace {

// Device address of fc_static_scratch on the current device (each GPU holds its own copy of the
// array at its own address).  On failure *out stays nullptr and the status (error text set) is returned.
fc_status static_scratch_ptr(void **out)
{
    *out = nullptr;
    static void *ptrs[FC_MAX_DEVICES];  // zero-initialised; a slot is written once and then only read
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= FC_MAX_DEVICES)
        return fail(FC_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, FC_MAX_DEVICES);
    void *p = __atomic_load_n(&ptrs[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(fc_static_scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(fc_static_scratch)");
        if (!p) return fail(FC_ERR_HIP, "hipGetSymbolAddress(fc_static_scratch) returned a null address");
        __atomic_store_n(&ptrs[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return FC_OK;
}

}  // namespace

extern "C" {

size_t fc_active_attention_static_max_bytes(void) { return FC_STATIC_SCRATCH_BYTES; }

fc_status fc_active_attention_static(fc_cache *cache, int32_t layer, const void *q, int32_t A, int32_t kv_len,
                                     const int32_t *pos, void *out, void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!q || !out) return fail(FC_ERR_INVALID_ARG, "q or out is NULL");
    if (A < 1) return fail(FC_ERR_INVALID_ARG, "A %d must be >= 1", A);
    if ((int64_t)A * cache->cfg.batch > (1 << 24))
        return fail(FC_ERR_UNSUPPORTED, "batch * A exceeds 2^24 rows");
    if (kv_len < 1 || kv_len > cache->cfg.max_seq)
        return fail(FC_ERR_BOUNDS, "kv_len %d outside [1, %d]", kv_len, cache->cfg.max_seq);
    const FcAttnPlan plan = fc_plan_attention(cache->cfg, A, kv_len);
    const size_t need = fc_plan_workspace(cache->cfg, plan, A);
    if (need > FC_STATIC_SCRATCH_BYTES)
        return fail(FC_ERR_WORKSPACE, "this shape needs %zu bytes of partial results, the static scratch holds %u",
                    need, FC_STATIC_SCRATCH_BYTES);
    void *scratch = nullptr;
    if (need > 0) {
        st = static_scratch_ptr(&scratch);
        if (st != FC_OK) return st;
    }
    // Nothing in the scratch has to start at zero: every (row tile, split) slot the merge kernel
    // reads is written by the first kernel of the same call.
    return fc_active_attention(cache, layer, q, A, kv_len, pos, out, scratch, need, stream);
}

fc_status fc_refresh(fc_cache *cache, int32_t layer, const void *x, const void *w_qkv, const void *b_qkv,
                     int32_t start, int32_t R, int32_t kv_len, void *q_scratch, void *out,
                     void *workspace, size_t workspace_bytes, void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!x || !w_qkv || !q_scratch) return fail(FC_ERR_INVALID_ARG, "x, w_qkv or q_scratch is NULL");
    if (R < 1) return fail(FC_ERR_INVALID_ARG, "R %d must be >= 1", R);
    if (start < 0 || start > cache->cfg.max_seq - R)
        return fail(FC_ERR_BOUNDS, "rows [%d, %d+%d) outside the cache of %d rows", start, start, R,
                    cache->cfg.max_seq);
    if (out) {
        // validate the attention half before anything is enqueued, so a failure has no side effects
        if (kv_len < 1 || kv_len > cache->cfg.max_seq)
            return fail(FC_ERR_BOUNDS, "kv_len %d outside [1, %d]", kv_len, cache->cfg.max_seq);
        if (start + R > kv_len)
            return fail(FC_ERR_BOUNDS, "refreshed rows end at %d, beyond kv_len %d", start + R, kv_len);
        const FcAttnPlan plan = fc_plan_attention(cache->cfg, R, kv_len);
        const size_t need = fc_plan_workspace(cache->cfg, plan, R);
        if (need > 0 && (!workspace || workspace_bytes < need))
            return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                        workspace ? workspace_bytes : (size_t)0);
    }
    st = fc_qkv_project_scatter(cache, layer, x, w_qkv, b_qkv, start, R, nullptr, q_scratch, stream);
    if (st != FC_OK || !out) return st;
    return fc_active_attention(cache, layer, q_scratch, R, kv_len, nullptr, out, workspace, workspace_bytes,
                               stream);
}

// ---------------------------------------------------------------------------------------------
// The rest of the layer on the window rows.

static fc_status check_dtype(int32_t dtype)
{
    if (dtype != FC_F32 && dtype != FC_BF16)
        return fail(FC_ERR_INVALID_ARG, "dtype %d is neither FC_F32 nor FC_BF16", dtype);
    return FC_OK;
}

fc_status fc_rmsnorm(int32_t dtype, const void *x, const void *weight, float eps, int32_t rows,
                     int32_t hidden, void *out, void *stream)
{
    fc_status st = check_dtype(dtype);
    if (st != FC_OK) return st;
    if (!x || !weight || !out) return fail(FC_ERR_INVALID_ARG, "x, weight or out is NULL");
    if (rows < 1 || hidden < 1) return fail(FC_ERR_INVALID_ARG, "rows and hidden must be >= 1");
    if (!(eps >= 0.0f) || !isfinite(eps)) return fail(FC_ERR_INVALID_ARG, "eps must be finite and >= 0");
    hipError_t e = fc_launch_rmsnorm(dtype, x, weight, eps, rows, hidden, out, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "rmsnorm launch");
}

static fc_status check_linear_shape(int32_t M, int32_t K, int32_t N)
{
    if (M < 1 || K < 1 || N < 1) return fail(FC_ERR_INVALID_ARG, "M, K and N must be >= 1");
    if (K % 8 != 0) return fail(FC_ERR_UNSUPPORTED, "K %d is not a multiple of 8", K);
    if (M > (1 << 24) || N > (1 << 22)) return fail(FC_ERR_UNSUPPORTED, "M is limited to 2^24 rows, N to 2^22");
    return FC_OK;
}

// Workspace of one linear call: tiled GEMM for more than 32 rows, streaming kernels otherwise.
static size_t linear_need(int dtype, int mode, int M, int K, int N)
{
    const FcWidePlan wide = fc_plan_wide(dtype, mode, M, K, N);
    if (wide.kind == 1) return fc_wide_workspace(wide, M, N);
    return fc_skinny_workspace(fc_plan_skinny(dtype, mode, M, K, N));
}

size_t fc_linear_workspace_bytes(int32_t dtype, int32_t M, int32_t K, int32_t N)
{
    if ((dtype != FC_F32 && dtype != FC_BF16) || M < 1 || K < 1 || N < 1) return 0;
    // the gated W_1 is planned on its F = N / 2 outputs; its slabs hold half as many outputs, so the
    // two plans need the same space and one query serves both calls
    const size_t a = linear_need(dtype, FC_LIN_RESIDUAL, M, K, N);
    const size_t b = N % 2 == 0 ? linear_need(dtype, FC_LIN_GATE_UP, M, K, N / 2) : 0;
    return a > b ? a : b;
}

static fc_status linear_common(int32_t dtype, int mode, const void *x, const void *w, const void *w2,
                               const void *res, int32_t M, int32_t K, int32_t N, void *out, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    fc_status st = check_dtype(dtype);
    if (st != FC_OK) return st;
    if (!x || !w || !out || (mode == FC_LIN_GATE_UP && !w2))
        return fail(FC_ERR_INVALID_ARG, "x, a weight matrix or out is NULL");
    st = check_linear_shape(M, K, N);
    if (st != FC_OK) return st;
    if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)w2 | (uintptr_t)res | (uintptr_t)out | (uintptr_t)workspace) & 15)
        return fail(FC_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    const FcWidePlan wide = fc_plan_wide(dtype, mode, M, K, N);
    const FcSkinnyPlan plan = fc_plan_skinny(dtype, mode, M, K, N);
    const size_t need = wide.kind == 1 ? fc_wide_workspace(wide, M, N) : fc_skinny_workspace(plan);
    if (need > 0 && (!workspace || workspace_bytes < need))
        return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need,
                    workspace ? workspace_bytes : (size_t)0);
    hipError_t e;
    if (wide.kind == 1)
        e = fc_launch_linear_wide(wide, mode, x, w, w2, res, M, K, N, out, workspace, (hipStream_t)stream);
    else if (plan.kind >= 1)
        e = fc_launch_linear_skinny(plan, mode, x, w, w2, res, M, K, N, out, workspace, (hipStream_t)stream);
    else
        e = fc_launch_linear_generic(dtype, mode, x, w, mode == FC_LIN_GATE_UP ? w2 : res, M, K, N, out,
                                     (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "linear launch");
}

fc_status fc_linear_residual(int32_t dtype, const void *x, const void *w, const void *residual, int32_t M,
                             int32_t K, int32_t N, void *out, void *workspace, size_t workspace_bytes,
                             void *stream)
{
    return linear_common(dtype, FC_LIN_RESIDUAL, x, w, nullptr, residual, M, K, N, out, workspace,
                         workspace_bytes, stream);
}

fc_status fc_ffn_gate_up(int32_t dtype, const void *x, const void *w_gate, const void *w_up, int32_t M,
                         int32_t K, int32_t F, void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return linear_common(dtype, FC_LIN_GATE_UP, x, w_gate, w_up, nullptr, M, K, F, out, workspace,
                         workspace_bytes, stream);
}

namespace {

// Carve-up of the whole-layer workspace for M = B * A rows (every part 256-byte aligned).
struct LayerWs {
    size_t h, q, o, x2, act, attn, lin, total;
    size_t attn_bytes, lin_bytes;
};

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

LayerWs layer_ws(const fc_config &c, int32_t d_ff, int32_t A)
{
    LayerWs w;
    const size_t es = esize_of(c.dtype);
    const size_t M = (size_t)c.batch * A, d = c.hidden, E = (size_t)c.n_q_heads * c.head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align256(bytes);
        return at;
    };
    w.h = take(M * d * es);
    w.q = take(M * E * es);
    w.o = take(M * E * es);
    w.x2 = take(M * d * es);
    w.act = take(M * (size_t)d_ff * es);
    w.attn_bytes = fc_workspace_bytes(&c, A);
    w.attn = take(w.attn_bytes);
    size_t lin = fc_linear_workspace_bytes(c.dtype, (int)M, (int)E, c.hidden);
    const size_t l2 = fc_linear_workspace_bytes(c.dtype, (int)M, c.hidden, 2 * d_ff);
    const size_t l3 = fc_linear_workspace_bytes(c.dtype, (int)M, d_ff, c.hidden);
    if (l2 > lin) lin = l2;
    if (l3 > lin) lin = l3;
    w.lin_bytes = lin;
    w.lin = take(lin);
    w.total = off;
    return w;
}

}  // namespace

size_t fc_full_layer_workspace_bytes(const fc_config *cfg, int32_t d_ff, int32_t max_rows)
{
    if (check_config(cfg) != FC_OK || d_ff < 1 || max_rows < 1 || (int64_t)max_rows * cfg->batch > (1 << 24))
        return 0;
    return layer_ws(*cfg, d_ff, max_rows).total;
}

fc_status fc_full_layer_step(fc_cache *cache, int32_t layer, const fc_layer_weights *wt, const void *x,
                             int32_t win_start, int32_t A, const int32_t *pos, int32_t kv_len, void *y,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!wt || !x || !y) return fail(FC_ERR_INVALID_ARG, "weights, x or y is NULL");
    if (!wt->norm1 || !wt->w_qkv || !wt->w_out || !wt->norm2 || !wt->w_gate || !wt->w_up || !wt->w_down)
        return fail(FC_ERR_INVALID_ARG, "a required weight pointer is NULL");
    if (wt->d_ff < 1 || wt->d_ff % 8 != 0) return fail(FC_ERR_INVALID_ARG, "d_ff %d must be a positive multiple of 8", wt->d_ff);
    if (!(wt->eps >= 0.0f) || !isfinite(wt->eps)) return fail(FC_ERR_INVALID_ARG, "eps must be finite and >= 0");
    if (A < 1) return fail(FC_ERR_INVALID_ARG, "A %d must be >= 1", A);
    const fc_config &c = cache->cfg;
    if ((int64_t)A * c.batch > (1 << 24)) return fail(FC_ERR_UNSUPPORTED, "batch * A exceeds 2^24 rows");
    if ((c.n_q_heads * c.head_dim) % 8 != 0) return fail(FC_ERR_UNSUPPORTED, "Hq * Dh must be a multiple of 8");
    if (!pos && (win_start < 0 || win_start > c.max_seq - A))
        return fail(FC_ERR_BOUNDS, "window [%d, %d+%d) outside the cache of %d rows", win_start, win_start, A,
                    c.max_seq);
    if (kv_len < 1 || kv_len > c.max_seq) return fail(FC_ERR_BOUNDS, "kv_len %d outside [1, %d]", kv_len, c.max_seq);
    LayerWs w;
    static_assert(sizeof(LayerWs) == sizeof(cache->ws_part), "cached carve-up");
    if (cache->ws_A == A && cache->ws_d_ff == wt->d_ff) {
        memcpy(&w, cache->ws_part, sizeof w);
    } else {
        w = layer_ws(c, wt->d_ff, A);
        memcpy(cache->ws_part, &w, sizeof w);
        cache->ws_A = A;
        cache->ws_d_ff = wt->d_ff;
    }
    if (!workspace || workspace_bytes < w.total)
        return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", w.total,
                    workspace ? workspace_bytes : (size_t)0);
    if ((uintptr_t)workspace & 15) return fail(FC_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    char *ws = (char *)workspace;
    const int M = c.batch * A, d = c.hidden, E = c.n_q_heads * c.head_dim;
    void *h = ws + w.h, *q = ws + w.q, *o = ws + w.o, *x2 = ws + w.x2, *act = ws + w.act;
    void *lin = w.lin_bytes ? ws + w.lin : nullptr, *attn = w.attn_bytes ? ws + w.attn : nullptr;

    st = fc_rmsnorm(c.dtype, x, wt->norm1, wt->eps, M, d, h, stream);
    if (st == FC_OK) st = fc_qkv_project_scatter(cache, layer, h, wt->w_qkv, wt->b_qkv, win_start, A, pos, q, stream);
    if (st == FC_OK) st = fc_active_attention(cache, layer, q, A, kv_len, pos, o, attn, w.attn_bytes, stream);
    if (st == FC_OK) st = fc_linear_residual(c.dtype, o, wt->w_out, x, M, E, d, x2, lin, w.lin_bytes, stream);
    if (st == FC_OK) st = fc_rmsnorm(c.dtype, x2, wt->norm2, wt->eps, M, d, h, stream);
    if (st == FC_OK) st = fc_ffn_gate_up(c.dtype, h, wt->w_gate, wt->w_up, M, d, wt->d_ff, act, lin, w.lin_bytes, stream);
    if (st == FC_OK) st = fc_linear_residual(c.dtype, act, wt->w_down, x2, M, wt->d_ff, d, y, lin, w.lin_bytes, stream);
    return st;
}

// ---------------------------------------------------------------------------------------------
// Unmasking step.

namespace {

// Carve-up of the lm-head workspace: [partial tiles of the streaming kernels][mx][arg][sm], each
// [parts][M].
struct LmHeadWs {
    FcWidePlan wide;
    FcSkinnyPlan plan;
    int parts;
    size_t tiles, mx, arg, sm, total;
};

LmHeadWs lm_head_ws(int dtype, int M, int K, int V)
{
    LmHeadWs w;
    w.wide = fc_plan_wide(dtype, FC_LIN_VOCAB, M, K, V);  // more than 32 rows: tiled GEMM
    w.plan = fc_plan_skinny(dtype, FC_LIN_VOCAB, M, K, V);
    if (w.wide.kind == 1) w.plan.kind = 0;
    w.parts = w.wide.kind == 1 ? V / 128
                               : (w.plan.kind == 1 ? w.plan.slabs
                                                   : (w.plan.kind == 2 ? w.plan.G  // one running triple per workgroup
                                                                       : (V + FC_LMHEAD_GENERIC_CHUNK - 1) / FC_LMHEAD_GENERIC_CHUNK));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align256(bytes);
        return at;
    };
    w.tiles = take(fc_skinny_workspace(w.plan));
    w.mx = take((size_t)w.parts * M * 4);
    w.arg = take((size_t)w.parts * M * 4);
    w.sm = take((size_t)w.parts * M * 4);
    w.total = off;
    return w;
}

}  // namespace

size_t fc_lm_head_workspace_bytes(int32_t dtype, int32_t M, int32_t K, int32_t V)
{
    if ((dtype != FC_F32 && dtype != FC_BF16) || M < 1 || K < 1 || V < 1 || M > (1 << 24) || V > (1 << 24)) return 0;
    return lm_head_ws(dtype, M, K, V).total;
}

fc_status fc_lm_head_argmax(int32_t dtype, const void *x, const void *w_vocab, int32_t M, int32_t K, int32_t V,
                            int32_t *tok, float *conf, void *workspace, size_t workspace_bytes, void *stream)
{
    fc_status st = check_dtype(dtype);
    if (st != FC_OK) return st;
    if (!x || !w_vocab || !tok || !conf) return fail(FC_ERR_INVALID_ARG, "x, w_vocab, tok or conf is NULL");
    if (M < 1 || K < 1 || V < 1) return fail(FC_ERR_INVALID_ARG, "M, K and V must be >= 1");
    if (K % 8 != 0) return fail(FC_ERR_UNSUPPORTED, "K %d is not a multiple of 8", K);
    if (M > (1 << 24) || V > (1 << 24)) return fail(FC_ERR_UNSUPPORTED, "M and V are limited to 2^24");
    if (((uintptr_t)x | (uintptr_t)w_vocab | (uintptr_t)workspace) & 15)
        return fail(FC_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    const LmHeadWs w = lm_head_ws(dtype, M, K, V);
    if (!workspace || workspace_bytes < w.total)
        return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", w.total,
                    workspace ? workspace_bytes : (size_t)0);
    char *ws = (char *)workspace;
    FcArgmaxPart am;
    am.mx = (float *)(ws + w.mx);
    am.arg = (int32_t *)(ws + w.arg);
    am.sm = (float *)(ws + w.sm);
    hipError_t e;
    if (w.wide.kind == 1)
        e = fc_launch_linear_wide(w.wide, FC_LIN_VOCAB, x, w_vocab, nullptr, nullptr, M, K, V, nullptr, nullptr,
                                  (hipStream_t)stream, &am);
    else if (w.plan.kind >= 1)
        e = fc_launch_linear_skinny(w.plan, FC_LIN_VOCAB, x, w_vocab, nullptr, nullptr, M, K, V, nullptr, ws + w.tiles,
                                    (hipStream_t)stream, &am);
    else
        e = fc_launch_lmhead_generic(dtype, x, w_vocab, M, K, V, am, (hipStream_t)stream);
    if (e == hipSuccess) e = fc_launch_lmhead_reduce(am, w.parts, M, tok, conf, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "lm-head launch");
}

fc_status fc_unmask_select(const int32_t *tok, const float *conf, const int32_t *pos, int32_t win_start, int32_t B,
                           int32_t A, int32_t n_unmask, int32_t mask_id, int32_t *tokens, int32_t L,
                           int32_t *pos_next, int32_t *count_next, void *stream)
{
    if (!tok || !conf || !tokens || !pos_next || !count_next)
        return fail(FC_ERR_INVALID_ARG, "tok, conf, tokens, pos_next or count_next is NULL");
    if (B < 1 || A < 1 || L < 1 || n_unmask < 0) return fail(FC_ERR_INVALID_ARG, "B, A, L >= 1 and n_unmask >= 0 required");
    if (B > 65535) return fail(FC_ERR_UNSUPPORTED, "B is limited to 65535");
    if (A > FC_UNMASK_MAX_ROWS) return fail(FC_ERR_UNSUPPORTED, "A %d exceeds %d rows", A, FC_UNMASK_MAX_ROWS);
    if (pos == pos_next) return fail(FC_ERR_INVALID_ARG, "pos_next must not be pos");
    if (!pos && (win_start < 0 || win_start > L - A))
        return fail(FC_ERR_BOUNDS, "window [%d, %d+%d) outside the sequence of %d tokens", win_start, win_start, A, L);
    hipError_t e = fc_launch_unmask_select(tok, conf, pos, win_start, B, A, n_unmask, mask_id, tokens, L, pos_next,
                                           count_next, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "unmask launch");
}

fc_status fc_gather_rows(int32_t dtype, const void *table, int32_t rows, int32_t width, const int32_t *idx, int32_t n,
                         void *out, void *stream)
{
    fc_status st = check_dtype(dtype);
    if (st != FC_OK) return st;
    if (!table || !idx || !out) return fail(FC_ERR_INVALID_ARG, "table, idx or out is NULL");
    if (rows < 1 || width < 1 || n < 1) return fail(FC_ERR_INVALID_ARG, "rows, width and n must be >= 1");
    const size_t row_bytes = (size_t)width * esize_of(dtype);
    if (row_bytes % 16 != 0) return fail(FC_ERR_UNSUPPORTED, "row size %zu is not a multiple of 16 bytes", row_bytes);
    if (((uintptr_t)table | (uintptr_t)out) & 15) return fail(FC_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
    hipError_t e = fc_launch_gather_rows(table, rows, (int)row_bytes, idx, n, out, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "gather launch");
}

size_t fc_guided_accept_workspace_bytes(int32_t B, int32_t A, int32_t V)
{
    if (B < 1 || A < 1 || V < 1 || B > 65535 || A > 65535) return 0;
    return fc_accept_workspace(B, A, V);
}

fc_status fc_guided_accept(const float *dlm, const float *ar, const int32_t *pos, int32_t win_start, int32_t B, int32_t A,
                           int32_t V, int32_t topk, float tau, int32_t mask_id, int32_t *tokens, int32_t L,
                           int32_t *n_accept, int32_t *pos_next, int32_t *count_next, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (!dlm || !ar || !tokens || !n_accept || !pos_next || !count_next)
        return fail(FC_ERR_INVALID_ARG, "dlm, ar, tokens, n_accept, pos_next or count_next is NULL");
    if (B < 1 || A < 1 || V < 1 || L < 1 || topk < 1 || topk > V) return fail(FC_ERR_INVALID_ARG, "B, A, V, L >= 1 and 1 <= topk <= V required");
    if (!isfinite(tau)) return fail(FC_ERR_INVALID_ARG, "tau must be finite");
    if (topk > FC_ACCEPT_MAX_TOPK) return fail(FC_ERR_UNSUPPORTED, "topk %d exceeds %d", topk, FC_ACCEPT_MAX_TOPK);
    if (B > 65535 || A > 65535) return fail(FC_ERR_UNSUPPORTED, "B and A are limited to 65535");
    if (pos == pos_next) return fail(FC_ERR_INVALID_ARG, "pos_next must not be pos");
    if (!pos && (win_start < 0 || win_start > L - A))
        return fail(FC_ERR_BOUNDS, "window [%d, %d+%d) outside the sequence of %d tokens", win_start, win_start, A, L);
    const size_t need = fc_guided_accept_workspace_bytes(B, A, V);
    if (!workspace || workspace_bytes < need)
        return fail(FC_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    if (((uintptr_t)dlm | (uintptr_t)ar | (uintptr_t)workspace) & 15)
        return fail(FC_ERR_INVALID_ARG, "dlm, ar and workspace must be 16-byte aligned");
    hipError_t e = fc_launch_guided_accept(dlm, ar, pos, win_start, B, A, V, topk, tau, mask_id, tokens, L, n_accept,
                                           pos_next, count_next, workspace, (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "acceptance launch");
}

fc_status fc_kv_similarity(const fc_cache *cache, int32_t layer, const void *k_prev, const void *v_prev, int32_t start,
                           int32_t rows, float *sim_k, float *sim_v, void *stream)
{
    fc_status st = check_cache_layer(cache, layer);
    if (st != FC_OK) return st;
    if (!k_prev || !v_prev || !sim_k || !sim_v) return fail(FC_ERR_INVALID_ARG, "k_prev, v_prev, sim_k or sim_v is NULL");
    if (rows < 1) return fail(FC_ERR_INVALID_ARG, "rows %d must be >= 1", rows);
    if (start < 0 || start > cache->cfg.max_seq - rows)
        return fail(FC_ERR_BOUNDS, "rows [%d, %d+%d) outside the cache of %d rows", start, start, rows,
                    cache->cfg.max_seq);
    hipError_t e = fc_launch_kv_similarity(geom_of(cache), cache->cfg.dtype, layer_ptr(cache, cache->k, layer),
                                           layer_ptr(cache, cache->v, layer), k_prev, v_prev, start, rows, sim_k, sim_v,
                                           (hipStream_t)stream);
    return e == hipSuccess ? FC_OK : hip_fail(e, "similarity launch");
}

}  // extern "C"
