// C ABI of libpod: argument validation, the host mirror of sequence lengths, and
// dispatch to the kernel launchers.  No device memory is allocated or freed here.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "pod_internal.h"

static thread_local char g_err[512] = "";

int pod_fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int pod_hip_fail(hipError_t e, const char *what)
{
    return pod_fail(POD_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The block table of cfg as two arrays [L][Hkv] (caller frees with free()): lowest layer of each (layer, head)'s
// block and the distant-key slot it reads; slots are numbered in (layer, head) order of the lowest layers.
static int make_tables(const pod_config *cfg, int32_t **lowest_out, int32_t **kslot_out, int *nslots, bool *uniform)
{
    const int L = cfg->num_layers, H = cfg->num_kv_heads;
    int32_t *lowest = (int32_t *)malloc((size_t)L * H * sizeof(int32_t));
    int32_t *kslot = (int32_t *)malloc((size_t)L * H * sizeof(int32_t));
    if (!lowest || !kslot) { free(lowest); free(kslot); return pod_fail(POD_ERR_CAPACITY, "out of host memory"); }
    int slots = 0;
    bool uni = true;
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < H; ++h) {
            const int lo = cfg->block_lowest ? cfg->block_lowest[(size_t)l * H + h] : l - l % cfg->group_size;
            const int prev = l > 0 ? lowest[(size_t)(l - 1) * H + h] : 0;
            if ((l == 0 && lo != 0) || (l > 0 && lo != prev && lo != l)) {
                free(lowest); free(kslot);
                return pod_fail(POD_ERR_INVALID_ARG, "block_lowest[%d][%d] = %d: blocks must be runs of consecutive layers", l, h, lo);
            }
            lowest[(size_t)l * H + h] = lo;
            kslot[(size_t)l * H + h] = lo == l ? slots++ : kslot[(size_t)lo * H + h];
            if (lo != lowest[(size_t)l * H]) uni = false;
        }
    *nslots = slots;
    if (uniform) *uniform = uni;
    if (lowest_out) *lowest_out = lowest; else free(lowest);
    if (kslot_out) *kslot_out = kslot; else free(kslot);
    return POD_OK;
}

static int make_layout(const pod_config *cfg, pod_layout *ly)
{
    if (!cfg) return pod_fail(POD_ERR_INVALID_ARG, "config is NULL");
    if (cfg->num_layers < 1 || (!cfg->block_lowest && (cfg->group_size < 1 || cfg->num_layers % cfg->group_size)))
        return pod_fail(POD_ERR_INVALID_ARG, "num_layers (%d) must be a positive multiple of group_size (%d)",
                        cfg->num_layers, cfg->group_size);
    if (cfg->num_kv_heads < 1 || cfg->num_q_heads < 1 || cfg->num_q_heads % cfg->num_kv_heads)
        return pod_fail(POD_ERR_INVALID_ARG, "num_q_heads (%d) must be a positive multiple of num_kv_heads (%d)",
                        cfg->num_q_heads, cfg->num_kv_heads);
    if (cfg->num_q_heads / cfg->num_kv_heads > 16)
        return pod_fail(POD_ERR_INVALID_ARG, "more than 16 query heads per KV head is not supported");
    if (cfg->num_kv_heads > kMaxKvHeads)
        return pod_fail(POD_ERR_INVALID_ARG, "at most %d kv heads are supported", kMaxKvHeads);
    if (cfg->head_dim != 64 && cfg->head_dim != 128)
        return pod_fail(POD_ERR_INVALID_ARG, "head_dim must be 64 or 128, got %d", cfg->head_dim);
    if (cfg->sink < 0 || cfg->window < 1)
        return pod_fail(POD_ERR_INVALID_ARG, "need sink >= 0 and window >= 1");
    if (cfg->max_batch < 1 || cfg->max_batch > 65535 || cfg->max_context < 1)
        return pod_fail(POD_ERR_INVALID_ARG, "need 1 <= max_batch <= 65535 and max_context >= 1");
    if ((int64_t)cfg->sink + cfg->window > (int64_t)INT32_MAX / 2)
        return pod_fail(POD_ERR_INVALID_ARG, "sink + window too large");
    int nslots = 0;
    {
        const int rc = make_tables(cfg, nullptr, nullptr, &nslots, nullptr);
        if (rc) return rc;
    }
    memset(ly, 0, sizeof *ly);
    ly->nslots = nslots;
    ly->L = cfg->num_layers; ly->G = cfg->block_lowest ? 1 : cfg->group_size; ly->Hq = cfg->num_q_heads; ly->Hkv = cfg->num_kv_heads;
    ly->D = cfg->head_dim; ly->S = cfg->sink; ly->W = cfg->window; ly->B = cfg->max_batch;
    ly->maxctx = cfg->max_context;
    ly->P = ly->S + ly->W;
    ly->Cd = ly->maxctx > ly->P ? ly->maxctx - ly->P : 0;
    ly->rep = ly->Hq / ly->Hkv;
    const size_t row = (size_t)ly->D * 2;
    const size_t per_layer_heads = (size_t)ly->L * ly->B * ly->Hkv;
    size_t off = 0;
    ly->off_lens = off; off += (size_t)ly->L * ly->B * sizeof(int32_t);
    off = align_up(off, 16);
    ly->off_flag = off; off += 16;
    ly->off_tickets = off; off += (size_t)ly->B * ly->Hkv * sizeof(uint64_t);
    ly->off_stepdone = off; off += (size_t)ly->B * sizeof(int32_t);
    off = align_up(off, 256);
    ly->off_proxK = off; off = align_up(off + per_layer_heads * ly->P * row, 256);
    ly->off_proxV = off; off = align_up(off + per_layer_heads * ly->P * row, 256);
    ly->off_distV = off; off = align_up(off + per_layer_heads * ly->Cd * row, 256);
    ly->off_distK = off; off = align_up(off + (size_t)ly->nslots * ly->B * ly->Cd * row, 256);
    ly->total_bytes = off;
    return POD_OK;
}

pod_headmap pod_make_headmap(const pod_cache *c, int layer)
{
    pod_headmap hm;
    memset(&hm, 0, sizeof hm);
    const int H = c->ly.Hkv;
    for (int h = 0; h < H; ++h) {
        hm.kslot_row[h] = c->kslot[(size_t)layer * H + h] * c->ly.B;
        if (c->lowest[(size_t)layer * H + h] == layer) hm.lowest_mask |= (uint64_t)1 << h;
    }
    // uniform blocks: the slots of one block are consecutive over the heads
    hm.uniform_row0 = c->uniform ? hm.kslot_row[0] : -1;
    return hm;
}

// is `layer` the lowest of its block for every / for some kv head?
static bool layer_lowest_all(const pod_cache *c, int layer)
{
    for (int h = 0; h < c->ly.Hkv; ++h) if (c->lowest[(size_t)layer * c->ly.Hkv + h] != layer) return false;
    return true;
}
static bool layer_lowest_any(const pod_cache *c, int layer)
{
    for (int h = 0; h < c->ly.Hkv; ++h) if (c->lowest[(size_t)layer * c->ly.Hkv + h] == layer) return true;
    return false;
}

extern "C" const char *pod_last_error(void) { return g_err; }

extern "C" int pod_cache_bytes(const pod_config *cfg, size_t *bytes)
{
    pod_layout ly;
    if (!bytes) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL");
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    *bytes = ly.total_bytes;
    return POD_OK;
}

extern "C" int pod_cache_live_bytes(const pod_config *cfg, int64_t n, size_t *pod_bytes, size_t *dense_bytes)
{
    pod_layout ly;
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    if (n < 0) return pod_fail(POD_ERR_INVALID_ARG, "n must be >= 0");
    const size_t row = (size_t)ly.D * 2; // one head
    const size_t n_prox = (size_t)(n < ly.P ? n : ly.P);
    const size_t n_dist = (size_t)(n > ly.P ? n - ly.P : 0);
    // per kv head: K and V of the proximal tokens and V of the distant ones at every layer; distant K once per block
    if (pod_bytes) *pod_bytes = row * ((size_t)ly.L * ly.Hkv * (2 * n_prox + n_dist) + (size_t)ly.nslots * n_dist);
    if (dense_bytes) *dense_bytes = row * ly.Hkv * 2 * (size_t)ly.L * (size_t)n;
    return POD_OK;
}

extern "C" int pod_workspace_bytes(const pod_config *cfg, size_t *bytes)
{
    pod_layout ly;
    if (!bytes) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL");
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    *bytes = pod_decode_workspace_bytes(ly);
    return POD_OK;
}

extern "C" int pod_cache_init(const pod_config *cfg, void *dev_buf, size_t bytes, void *stream, pod_cache **out)
{
    pod_layout ly;
    if (!out) return pod_fail(POD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    if (!dev_buf) return pod_fail(POD_ERR_INVALID_ARG, "dev_buf is NULL");
    if ((uintptr_t)dev_buf % 256) return pod_fail(POD_ERR_INVALID_ARG, "dev_buf must be 256-byte aligned");
    if (bytes < ly.total_bytes)
        return pod_fail(POD_ERR_CAPACITY, "buffer has %zu bytes, cache needs %zu", bytes, ly.total_bytes);
    pod_cache *c = new (std::nothrow) pod_cache;
    if (!c) return pod_fail(POD_ERR_CAPACITY, "out of host memory");
    c->ly = ly;
    c->base = (char *)dev_buf;
    c->host_len = (int64_t *)calloc((size_t)ly.L * ly.B, sizeof(int64_t));
    c->lowest = nullptr; c->kslot = nullptr; c->uniform = true;
    {
        int nslots = 0;
        rc = make_tables(cfg, &c->lowest, &c->kslot, &nslots, &c->uniform);
        if (rc) { free(c->host_len); delete c; return rc; }
    }
    c->device = -1;
    {   // tuning overrides: read here, once, so that the environment cannot change launch geometry between calls
        const char *e1 = getenv("POD_DECODE_CHUNK"), *e2 = getenv("POD_DECODE_CHUNK_PROX");
        c->tune_chunk = e1 && atoi(e1) > 0 ? atoi(e1) : 0;
        c->tune_chunk_prox = e2 && atoi(e2) > 0 ? atoi(e2) : 0;
        const char *e3 = getenv("POD_DECODE_FUSED");
        c->fused_merge = !(e3 && atoi(e3) == 0);
        const char *e4 = getenv("POD_DECODE_XCD_LOCAL");
        c->xcd_local = !(e4 && atoi(e4) == 0);
        c->nxcd = 0;
        c->device_lengths = false;
        const char *e7 = getenv("POD_DECODE_WALK_TURNS");
        c->walk_turns = !(e7 && atoi(e7) == 0);
        const char *e6 = getenv("POD_DECODE_EVEN");
        c->even_split = !(e6 && atoi(e6) == 0);
        const char *e5 = getenv("POD_CHUNK_IN_PLACE");
        c->chunk_in_place = !(e5 && atoi(e5) == 0);
    }
    c->prof_ev = nullptr; c->prof_cap = 0; c->prof_n = 0;
    c->trace = nullptr; c->trace_cap = 0;
    if (!c->host_len) { free(c->lowest); free(c->kslot); delete c; return pod_fail(POD_ERR_CAPACITY, "out of host memory"); }
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { free(c->host_len); free(c->lowest); free(c->kslot); delete c; return pod_hip_fail(e, "hipGetDevice"); }
    rc = pod_decode_static_scratch(&c->static_scratch, &c->static_scratch_bytes); // this device's copy of the array
    if (rc == POD_OK) rc = pod_probe_xcds(&c->nxcd);
    if (rc == POD_OK) rc = pod_launch_clear_header(c, (hipStream_t)stream);
    if (rc) { free(c->host_len); free(c->lowest); free(c->kslot); delete c; return rc; }
    *out = c;
    return POD_OK;
}

extern "C" int pod_cache_destroy(pod_cache *cache)
{
    if (!cache) return POD_OK;
    pod_profile_disable(cache);
    free(cache->host_len);
    free(cache->lowest);
    free(cache->kslot);
    delete cache;
    return POD_OK;
}

extern "C" int pod_profile_disable(pod_cache *cache)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    for (int i = 0; i < 2 * cache->prof_cap; ++i) (void)hipEventDestroy(cache->prof_ev[i]);
    free(cache->prof_ev);
    cache->prof_ev = nullptr; cache->prof_cap = 0; cache->prof_n = 0;
    return POD_OK;
}

extern "C" int pod_profile_enable(pod_cache *cache, int max_records)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    if (max_records < 1 || max_records > (1 << 20)) return pod_fail(POD_ERR_INVALID_ARG, "max_records out of range");
    pod_profile_disable(cache);
    cache->prof_ev = (hipEvent_t *)calloc((size_t)2 * max_records, sizeof(hipEvent_t));
    if (!cache->prof_ev) return pod_fail(POD_ERR_CAPACITY, "out of host memory");
    for (int i = 0; i < 2 * max_records; ++i) {
        // timing only: no system-scope fence when the event is reached (that fence is part of what an event pair
        // around a short kernel otherwise measures)
        hipError_t e = hipEventCreateWithFlags(&cache->prof_ev[i], hipEventDisableSystemFence);
        if (e != hipSuccess) {
            for (int k = 0; k < i; ++k) (void)hipEventDestroy(cache->prof_ev[k]);
            free(cache->prof_ev); cache->prof_ev = nullptr;
            return pod_hip_fail(e, "hipEventCreate");
        }
    }
    cache->prof_cap = max_records; cache->prof_n = 0;
    return POD_OK;
}

extern "C" int pod_profile_read(pod_cache *cache, double *total_ms, int *launches)
{
    if (!cache || !total_ms || !launches) return pod_fail(POD_ERR_INVALID_ARG, "NULL argument");
    double sum = 0.0;
    for (int i = 0; i < cache->prof_n; ++i) {
        POD_HIP_TRY(hipEventSynchronize(cache->prof_ev[2 * i + 1]));
        float ms = 0.f;
        POD_HIP_TRY(hipEventElapsedTime(&ms, cache->prof_ev[2 * i], cache->prof_ev[2 * i + 1]));
        sum += ms;
    }
    *total_ms = sum; *launches = cache->prof_n;
    cache->prof_n = 0;
    return POD_OK;
}

extern "C" int pod_profile_read_each(pod_cache *cache, float *ms_each, int capacity, int *launches)
{
    if (!cache || !ms_each || !launches || capacity < 0) return pod_fail(POD_ERR_INVALID_ARG, "NULL argument or negative capacity");
    const int n = cache->prof_n < capacity ? cache->prof_n : capacity;
    for (int i = 0; i < n; ++i) {
        POD_HIP_TRY(hipEventSynchronize(cache->prof_ev[2 * i + 1]));
        POD_HIP_TRY(hipEventElapsedTime(&ms_each[i], cache->prof_ev[2 * i], cache->prof_ev[2 * i + 1]));
    }
    *launches = n;
    cache->prof_n = 0;
    return POD_OK;
}

extern "C" int pod_profile_mfma_feed(int variant, int iters, void *dev_out, size_t out_bytes, void *stream)
{
    if (!dev_out || iters < 1 || iters > (1 << 24)) return pod_fail(POD_ERR_INVALID_ARG, "dev_out is NULL or iters outside [1, 2^24]");
    return pod_launch_mfma_feed(variant, iters, (float *)dev_out, out_bytes, (hipStream_t)stream);
}

extern "C" int pod_decode_plan(int num_cus, int batch, int num_kv_heads, int proximal_rows, int max_context_len, int32_t plan[6])
{
    if (!plan) return pod_fail(POD_ERR_INVALID_ARG, "plan is NULL");
    if (num_cus < 1 || batch < 1 || num_kv_heads < 1 || proximal_rows < 1 || max_context_len < 1)
        return pod_fail(POD_ERR_INVALID_ARG, "num_cus, batch, num_kv_heads, proximal_rows and max_context_len must be positive");
    if ((long long)batch * num_kv_heads > 0x7fffffffLL || (long long)batch * num_kv_heads * max_context_len > (1LL << 50))
        return pod_fail(POD_ERR_INVALID_ARG, "shape too large");
    const pod_decode_plan_t pl = pod_plan_decode(num_cus, batch, num_kv_heads, proximal_rows, max_context_len, 0, 0, false, false, true);
    plan[0] = pl.waves; plan[1] = pl.chunk; plan[2] = pl.chunk_p; plan[3] = pl.max_nd; plan[4] = pl.nc; plan[5] = pl.merge_inside ? 1 : 0;
    return POD_OK;
}

extern "C" int pod_decode_even_plan(int num_cus, int batch, int num_kv_heads, int proximal_rows, int distant_unit_tokens,
                                    const int32_t *context_lens, int32_t plan[4], int32_t *unit_cum)
{
    if (!plan || !context_lens || !unit_cum) return pod_fail(POD_ERR_INVALID_ARG, "plan, context_lens and unit_cum must not be NULL");
    if (num_cus < 1 || batch < 1 || batch > 256 || num_kv_heads < 1 || proximal_rows < 1)
        return pod_fail(POD_ERR_INVALID_ARG, "num_cus, num_kv_heads and proximal_rows must be positive, batch in [1, 256]");
    if (distant_unit_tokens != 128 && distant_unit_tokens != 256)
        return pod_fail(POD_ERR_INVALID_ARG, "distant_unit_tokens must be 128 or 256");
    pod_even_plan_t ev = {0, 0, 0, 0};
    if (!pod_plan_even(2 * num_cus, batch, num_kv_heads, proximal_rows, distant_unit_tokens, context_lens, unit_cum, &ev))
        ev = pod_even_plan_t{0, 0, 0, 0};
    plan[0] = ev.q; plan[1] = ev.nwg; plan[2] = ev.total; plan[3] = ev.most;
    return POD_OK;
}

extern "C" int pod_profile_set_trace(pod_cache *cache, void *dev_buf, size_t bytes)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    if (dev_buf && ((uintptr_t)dev_buf % 8)) return pod_fail(POD_ERR_INVALID_ARG, "dev_buf must be 8-byte aligned");
    cache->trace = dev_buf;
    cache->trace_cap = dev_buf ? (int)(bytes / 64 > 0x7fffffff ? 0x7fffffff : bytes / 64) : 0;
    return POD_OK;
}

extern "C" int pod_profile_stream_read(pod_cache *cache, const void *dev_buf, size_t bytes, void *stream)
{
    if (!dev_buf || ((uintptr_t)dev_buf % 16) || bytes < 16 || bytes % 16)
        return pod_fail(POD_ERR_INVALID_ARG, "dev_buf must be 16-byte aligned and bytes a positive multiple of 16");
    return pod_launch_stream_read(cache, dev_buf, bytes, (hipStream_t)stream);
}

static int check_cache_layer(const pod_cache *c, int layer)
{
    if (!c) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    if (layer < 0 || layer >= c->ly.L)
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d outside [0, %d)", layer, c->ly.L);
    return POD_OK;
}

extern "C" int pod_cache_reset(pod_cache *cache, int seq_slot, void *stream)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    if (seq_slot >= cache->ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, cache->ly.B);
    int rc = pod_launch_reset(cache, seq_slot, (hipStream_t)stream);
    if (rc) return rc;
    for (int l = 0; l < cache->ly.L; ++l)
        for (int b = 0; b < cache->ly.B; ++b)
            if (seq_slot < 0 || b == seq_slot) cache->host_len[(size_t)l * cache->ly.B + b] = 0;
    return POD_OK;
}

extern "C" int pod_cache_seq_len(const pod_cache *cache, int layer, int seq_slot, int64_t *n)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    if (seq_slot < 0 || seq_slot >= cache->ly.B || !n)
        return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d) or n is NULL", seq_slot, cache->ly.B);
    *n = cache->host_len[(size_t)layer * cache->ly.B + seq_slot];
    return POD_OK;
}

extern "C" int pod_cache_region_counts(const pod_cache *cache, int layer, int seq_slot, int64_t counts[3], int *has_distant_keys)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (seq_slot < 0 || seq_slot >= ly.B || !counts)
        return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d) or counts is NULL", seq_slot, ly.B);
    const int64_t n = cache->host_len[(size_t)layer * ly.B + seq_slot];
    counts[0] = n < ly.S ? n : ly.S;                         // sink
    counts[1] = n - counts[0] < ly.W ? n - counts[0] : ly.W; // recent window
    counts[2] = n - counts[0] - counts[1];                   // distant
    if (has_distant_keys) *has_distant_keys = layer_lowest_any(cache, layer) ? 1 : 0;
    return POD_OK;
}

extern "C" int pod_cache_check(pod_cache *cache, void *stream)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    int32_t flag = 0;
    hipStream_t st = (hipStream_t)stream;
    POD_HIP_TRY(hipMemcpyAsync(&flag, cache->base + cache->ly.off_flag, sizeof flag, hipMemcpyDeviceToHost, st));
    POD_HIP_TRY(hipStreamSynchronize(st));
    if (flag) {
        int32_t zero = 0;
        POD_HIP_TRY(hipMemcpyAsync(cache->base + cache->ly.off_flag, &zero, sizeof zero, hipMemcpyHostToDevice, st));
        POD_HIP_TRY(hipStreamSynchronize(st));
        return pod_fail(POD_ERR_STATE, "a kernel skipped at least one entry: device-side contract violated (flag %d)", flag);
    }
    return POD_OK;
}

extern "C" int pod_cache_sync_lengths(pod_cache *cache, void *stream)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    const size_t count = (size_t)cache->ly.L * cache->ly.B;
    int32_t *tmp = (int32_t *)malloc(count * sizeof(int32_t));
    if (!tmp) return pod_fail(POD_ERR_CAPACITY, "out of host memory");
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(tmp, cache->base + cache->ly.off_lens, count * sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { free(tmp); return pod_hip_fail(e, "copying the lengths to the host"); }
    for (size_t i = 0; i < count; ++i) cache->host_len[i] = tmp[i];
    free(tmp);
    return POD_OK;
}

extern "C" int pod_cache_append(pod_cache *cache, int layer, const void *k_new, const void *v_new,
                                const int32_t *positions, int B, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!k_new || !v_new || !positions) return pod_fail(POD_ERR_INVALID_ARG, "k_new, v_new and positions must not be NULL");
    if (B < 1 || B > ly.B) return pod_fail(POD_ERR_INVALID_ARG, "B = %d outside [1, max_batch = %d]", B, ly.B);
    int64_t *len = cache->host_len + (size_t)layer * ly.B;
    for (int b = 0; b < B; ++b)
        if (len[b] >= ly.maxctx)
            return pod_fail(POD_ERR_CAPACITY, "slot %d at layer %d already holds max_context = %d tokens", b, layer, ly.maxctx);
    rc = pod_launch_append(cache, layer, k_new, v_new, positions, B, (hipStream_t)stream);
    if (rc) return rc;
    for (int b = 0; b < B; ++b) len[b] += 1;
    return POD_OK;
}

extern "C" int pod_cache_fill(pod_cache *cache, int layer, int seq_slot, int n, const void *k, const void *v,
                              void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
    if (!k || !v) return pod_fail(POD_ERR_INVALID_ARG, "k and v must not be NULL");
    if (n < 1) return pod_fail(POD_ERR_INVALID_ARG, "n must be >= 1");
    if (n > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "n = %d exceeds max_context = %d", n, ly.maxctx);
    int64_t *len = cache->host_len + (size_t)layer * ly.B + seq_slot;
    if (*len != 0) return pod_fail(POD_ERR_STATE, "slot %d at layer %d is not empty (%lld tokens)", seq_slot, layer, (long long)*len);
    rc = pod_launch_fill(cache, layer, seq_slot, n, k, v, (hipStream_t)stream);
    if (rc) return rc;
    *len = n;
    return POD_OK;
}

static int decode_common(pod_cache *cache, int layer, const void *q, const void *q_shared,
                         const int32_t *context_lens, int B, int max_context_len, float scale, void *workspace,
                         size_t workspace_bytes, void *scores, float tau, void *out, void *stream, bool own_scratch = false);

extern "C" int pod_decode_attention_static(pod_cache *cache, int layer, const void *q, const void *q_shared,
                                           const int32_t *context_lens, int B, int max_context_len, float scale,
                                           void *out, void *stream)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    int dev = -1;
    POD_HIP_TRY(hipGetDevice(&dev));
    if (dev != cache->device)
        return pod_fail(POD_ERR_INVALID_ARG, "current device %d is not the cache's device %d", dev, cache->device);
    return decode_common(cache, layer, q, q_shared, context_lens, B, max_context_len, scale, cache->static_scratch,
                         cache->static_scratch_bytes, nullptr, -1.f, out, stream, true);
}

extern "C" int pod_decode_attention(pod_cache *cache, int layer, const void *q, const void *q_shared,
                                    const int32_t *context_lens, int B, int max_context_len, float scale,
                                    void *workspace, size_t workspace_bytes, void *out, void *stream)
{
    return decode_common(cache, layer, q, q_shared, context_lens, B, max_context_len, scale, workspace,
                         workspace_bytes, nullptr, -1.f, out, stream);
}

extern "C" int pod_score_buffer_bytes(const pod_config *cfg, size_t *bytes)
{
    pod_layout ly;
    if (!bytes) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL");
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    *bytes = pod_score_header_bytes(ly) + (size_t)ly.B * ly.Hq * pod_score_stride(ly) * sizeof(float);
    return POD_OK;
}

static int decode_with_scores(pod_cache *cache, int layer, const void *q, const int32_t *context_lens, int B,
                              int max_context_len, float scale, void *workspace, size_t workspace_bytes,
                              void *scores, size_t scores_bytes, float tau, void *out, void *stream);

extern "C" int pod_decode_attention_reuse(pod_cache *cache, int layer, const void *q, const int32_t *context_lens,
                                          int B, int max_context_len, float scale, void *workspace,
                                          size_t workspace_bytes, void *scores, size_t scores_bytes, void *out,
                                          void *stream)
{
    return decode_with_scores(cache, layer, q, context_lens, B, max_context_len, scale, workspace, workspace_bytes,
                              scores, scores_bytes, -1.f, out, stream);
}

extern "C" int pod_decode_attention_gated(pod_cache *cache, int layer, const void *q, const int32_t *context_lens,
                                          int B, int max_context_len, float scale, float tau, void *workspace,
                                          size_t workspace_bytes, void *scores, size_t scores_bytes, void *out,
                                          void *stream)
{
    if (!(tau >= 0.f && tau <= 1.f)) return pod_fail(POD_ERR_INVALID_ARG, "tau = %g outside [0, 1]", (double)tau);
    return decode_with_scores(cache, layer, q, context_lens, B, max_context_len, scale, workspace, workspace_bytes,
                              scores, scores_bytes, tau, out, stream);
}

extern "C" int pod_score_skip_offset(const pod_config *cfg, size_t *offset)
{
    pod_layout ly;
    if (!offset) return pod_fail(POD_ERR_INVALID_ARG, "offset is NULL");
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    *offset = pod_score_skip_offset_bytes(ly);
    return POD_OK;
}

static int decode_with_scores(pod_cache *cache, int layer, const void *q, const int32_t *context_lens, int B,
                              int max_context_len, float scale, void *workspace, size_t workspace_bytes,
                              void *scores, size_t scores_bytes, float tau, void *out, void *stream)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    if (!scores) return pod_fail(POD_ERR_INVALID_ARG, "scores is NULL");
    if ((uintptr_t)scores % 256) return pod_fail(POD_ERR_INVALID_ARG, "scores must be 256-byte aligned");
    const pod_layout &ly = cache->ly;
    const size_t need = pod_score_header_bytes(ly) + (size_t)ly.B * ly.Hq * pod_score_stride(ly) * sizeof(float);
    if (scores_bytes < need) return pod_fail(POD_ERR_CAPACITY, "score buffer has %zu bytes, needs %zu", scores_bytes, need);
    // upper layers take the distant logits from the buffer: q doubles as the (unused) shared query
    return decode_common(cache, layer, q, q, context_lens, B, max_context_len, scale, workspace, workspace_bytes,
                         scores, tau, out, stream);
}

static int decode_common(pod_cache *cache, int layer, const void *q, const void *q_shared,
                         const int32_t *context_lens, int B, int max_context_len, float scale, void *workspace,
                         size_t workspace_bytes, void *scores, float tau, void *out, void *stream, bool own_scratch)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!q || !context_lens || !out || !workspace)
        return pod_fail(POD_ERR_INVALID_ARG, "q, context_lens, workspace and out must not be NULL");
    if (B < 1 || B > ly.B) return pod_fail(POD_ERR_INVALID_ARG, "B = %d outside [1, max_batch = %d]", B, ly.B);
    // (a caller's workspace is held to the configuration's worst case; the library's own fixed array to what this
    // call's launch really needs, checked by the launcher)
    if (!own_scratch && workspace_bytes < pod_decode_workspace_bytes(ly))
        return pod_fail(POD_ERR_CAPACITY, "workspace has %zu bytes, needs %zu", workspace_bytes, pod_decode_workspace_bytes(ly));
    if (max_context_len < 0 || max_context_len > ly.maxctx)
        return pod_fail(POD_ERR_INVALID_ARG, "max_context_len %d outside [0, %d]", max_context_len, ly.maxctx);
    const int64_t *len = cache->host_len + (size_t)layer * ly.B;
    int64_t longest = 0;
    for (int b = 0; b < B; ++b) longest = len[b] > longest ? len[b] : longest;
    const bool lowest = layer_lowest_all(cache, layer);
    if (cache->device_lengths) {
        // the mirror is not consulted: the launch bound must come from the caller, and an upper layer always names its shared query
        if (max_context_len < 1) return pod_fail(POD_ERR_INVALID_ARG, "with lengths taken from the device, max_context_len must be given");
        if (!lowest && !q_shared) return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block: q_shared is required", layer);
        return pod_launch_decode(cache, layer, q, lowest ? nullptr : q_shared, context_lens, B, max_context_len, scale,
                                 workspace, workspace_bytes, scores, tau, out, (hipStream_t)stream);
    }
    if (!lowest && !q_shared && longest > ly.P)
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block and holds distant tokens: q_shared is required", layer);
    // every head's lowest layer must hold the same tokens as this layer (the device checks this layer's own lengths)
    for (int h = 0; h < ly.Hkv; ++h) {
        const int64_t *low = cache->host_len + (size_t)cache->lowest[(size_t)layer * ly.Hkv + h] * ly.B;
        for (int b = 0; b < B; ++b)
            if (len[b] > ly.P && low[b] != len[b])
                return pod_fail(POD_ERR_STATE, "slot %d: layer %d holds %lld tokens but layer %d, the lowest of kv head %d's block, holds %lld",
                                b, layer, (long long)len[b], cache->lowest[(size_t)layer * ly.Hkv + h], h, (long long)low[b]);
    }
    if (max_context_len == 0) max_context_len = (int)longest;
    if (max_context_len == 0) max_context_len = 1;
    return pod_launch_decode(cache, layer, q, lowest ? nullptr : q_shared, context_lens, B, max_context_len, scale,
                             workspace, workspace_bytes, scores, tau, out, (hipStream_t)stream);
}

extern "C" int pod_cache_launch_info(const pod_cache *cache, int32_t info[4])
{
    if (!cache || !info) return pod_fail(POD_ERR_INVALID_ARG, "NULL argument");
    info[0] = cache->nxcd;
    info[1] = cache->xcd_local && cache->nxcd >= 1;
    info[2] = cache->fused_merge;
    info[3] = cache->device_lengths;
    return POD_OK;
}

extern "C" int pod_cache_set_length_source(pod_cache *cache, int from_device)
{
    if (!cache) return pod_fail(POD_ERR_INVALID_ARG, "cache is NULL");
    cache->device_lengths = from_device != 0;
    return POD_OK;
}

extern "C" int pod_decode_step(pod_cache *cache, int layer, const void *k_new, const void *v_new, const void *q,
                               const void *q_shared, const int32_t *positions, int B, int max_context_len, float scale,
                               void *workspace, size_t workspace_bytes, void *out, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!k_new || !v_new || !q || !positions || !out || !workspace)
        return pod_fail(POD_ERR_INVALID_ARG, "k_new, v_new, q, positions, workspace and out must not be NULL");
    if (B < 1 || B > ly.B) return pod_fail(POD_ERR_INVALID_ARG, "B = %d outside [1, max_batch = %d]", B, ly.B);
    if (workspace_bytes < pod_decode_workspace_bytes(ly))
        return pod_fail(POD_ERR_CAPACITY, "workspace has %zu bytes, needs %zu", workspace_bytes, pod_decode_workspace_bytes(ly));
    if (max_context_len < 0 || max_context_len > ly.maxctx)
        return pod_fail(POD_ERR_INVALID_ARG, "max_context_len %d outside [0, %d]", max_context_len, ly.maxctx);
    const bool lowest = layer_lowest_all(cache, layer);
    const pod_step_args step = {k_new, v_new, positions};
    int64_t *len = cache->host_len + (size_t)layer * ly.B;
    if (cache->device_lengths) {
        if (max_context_len < 1) return pod_fail(POD_ERR_INVALID_ARG, "with lengths taken from the device, max_context_len must be given");
        if (!lowest && !q_shared) return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block: q_shared is required", layer);
    } else {
        int64_t longest = 0;
        for (int b = 0; b < B; ++b) {
            if (len[b] >= ly.maxctx)
                return pod_fail(POD_ERR_CAPACITY, "slot %d at layer %d already holds max_context = %d tokens", b, layer, ly.maxctx);
            longest = len[b] + 1 > longest ? len[b] + 1 : longest;
        }
        if (!lowest && !q_shared && longest > ly.P)
            return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block and holds distant tokens: q_shared is required", layer);
        // the lowest layer of every head's block must have taken this token already once distant tokens exist
        for (int h = 0; h < ly.Hkv; ++h) {
            const int la = cache->lowest[(size_t)layer * ly.Hkv + h];
            const int64_t *low = cache->host_len + (size_t)la * ly.B;
            for (int b = 0; b < B && la != layer; ++b)
                if (len[b] + 1 > ly.P && low[b] != len[b] + 1)
                    return pod_fail(POD_ERR_STATE, "slot %d: layer %d would hold %lld tokens but layer %d, the lowest of kv head %d's block, holds %lld",
                                    b, layer, (long long)len[b] + 1, la, h, (long long)low[b]);
        }
        if (max_context_len == 0) max_context_len = (int)longest;
    }
    rc = pod_launch_decode(cache, layer, q, lowest ? nullptr : q_shared, nullptr, B, max_context_len, scale, workspace,
                           workspace_bytes, nullptr, -1.f, out, (hipStream_t)stream, &step);
    if (rc) return rc;
    for (int b = 0; b < B; ++b) len[b] += 1;
    return POD_OK;
}

extern "C" int pod_decode_step_reuse(pod_cache *cache, int layer, const void *k_new, const void *v_new, const void *q,
                                     const int32_t *positions, int B, int max_context_len, float scale, void *workspace,
                                     size_t workspace_bytes, void *scores, size_t scores_bytes, void *out, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!k_new || !v_new || !q || !positions || !out || !workspace || !scores)
        return pod_fail(POD_ERR_INVALID_ARG, "k_new, v_new, q, positions, workspace, scores and out must not be NULL");
    if ((uintptr_t)scores % 256) return pod_fail(POD_ERR_INVALID_ARG, "scores must be 256-byte aligned");
    if (B < 1 || B > ly.B) return pod_fail(POD_ERR_INVALID_ARG, "B = %d outside [1, max_batch = %d]", B, ly.B);
    if (workspace_bytes < pod_decode_workspace_bytes(ly))
        return pod_fail(POD_ERR_CAPACITY, "workspace has %zu bytes, needs %zu", workspace_bytes, pod_decode_workspace_bytes(ly));
    const size_t need = pod_score_header_bytes(ly) + (size_t)ly.B * ly.Hq * pod_score_stride(ly) * sizeof(float);
    if (scores_bytes < need) return pod_fail(POD_ERR_CAPACITY, "score buffer has %zu bytes, needs %zu", scores_bytes, need);
    if (max_context_len < 0 || max_context_len > ly.maxctx)
        return pod_fail(POD_ERR_INVALID_ARG, "max_context_len %d outside [0, %d]", max_context_len, ly.maxctx);
    const pod_step_args step = {k_new, v_new, positions};
    int64_t *len = cache->host_len + (size_t)layer * ly.B;
    if (cache->device_lengths) {
        if (max_context_len < 1) return pod_fail(POD_ERR_INVALID_ARG, "with lengths taken from the device, max_context_len must be given");
    } else {
        int64_t longest = 0;
        for (int b = 0; b < B; ++b) {
            if (len[b] >= ly.maxctx)
                return pod_fail(POD_ERR_CAPACITY, "slot %d at layer %d already holds max_context = %d tokens", b, layer, ly.maxctx);
            longest = len[b] + 1 > longest ? len[b] + 1 : longest;
        }
        // the lowest layer of every head's block must have taken this token (and written its logits) already
        for (int h = 0; h < ly.Hkv; ++h) {
            const int la = cache->lowest[(size_t)layer * ly.Hkv + h];
            const int64_t *low = cache->host_len + (size_t)la * ly.B;
            for (int b = 0; b < B && la != layer; ++b)
                if (len[b] + 1 > ly.P && low[b] != len[b] + 1)
                    return pod_fail(POD_ERR_STATE, "slot %d: layer %d would hold %lld tokens but layer %d, the lowest of kv head %d's block, holds %lld",
                                    b, layer, (long long)len[b] + 1, la, h, (long long)low[b]);
        }
        if (max_context_len == 0) max_context_len = (int)longest;
    }
    rc = pod_launch_decode(cache, layer, q, nullptr, nullptr, B, max_context_len, scale, workspace, workspace_bytes, scores, -1.f, out,
                           (hipStream_t)stream, &step);
    if (rc) return rc;
    for (int b = 0; b < B; ++b) len[b] += 1;
    return POD_OK;
}

extern "C" int pod_layer_similarity(const float *att, int num_layers, int num_heads, int rows, int n, float *sim,
                                    void *stream)
{
    if (!att || !sim) return pod_fail(POD_ERR_INVALID_ARG, "att and sim must not be NULL");
    if (num_layers < 1 || num_heads < 1 || rows < 1 || n < 1)
        return pod_fail(POD_ERR_INVALID_ARG, "num_layers, num_heads, rows and n must be >= 1");
    if (num_heads > 65535 || (int64_t)num_layers * (num_layers - 1) / 2 > INT32_MAX)
        return pod_fail(POD_ERR_INVALID_ARG, "too many heads or layer pairs for one launch");
    if (((uintptr_t)att % 16) || ((size_t)rows * n) % 4)
        return pod_fail(POD_ERR_INVALID_ARG, "att must be 16-byte aligned and rows * n a multiple of 4");
    return pod_launch_similarity(att, num_layers, num_heads, rows, n, sim, (hipStream_t)stream);
}

extern "C" int pod_group_layers(const float *sim, int num_layers, int num_q_heads, int num_kv_heads, float threshold,
                                int32_t *lowest_out)
{
    if (!sim || !lowest_out) return pod_fail(POD_ERR_INVALID_ARG, "sim and lowest_out must not be NULL");
    if (num_layers < 1 || num_kv_heads < 1 || num_q_heads < 1 || num_q_heads % num_kv_heads)
        return pod_fail(POD_ERR_INVALID_ARG, "need num_layers >= 1 and num_q_heads a positive multiple of num_kv_heads");
    const int L = num_layers, rep = num_q_heads / num_kv_heads;
    // similar(a, b) for kv head g: more than half of its query heads have sim >= threshold
    auto similar = [&](int g, int a, int b) {
        int votes = 0;
        for (int h = g * rep; h < (g + 1) * rep; ++h) votes += sim[((size_t)h * L + a) * L + b] >= threshold;
        return 2 * votes > rep;
    };
    for (int g = 0; g < num_kv_heads; ++g) {
        int block_start = 0; // the current block is [block_start, l)
        lowest_out[g] = 0;
        for (int l = 1; l < L; ++l) {
            bool joins = true;
            for (int m = block_start; m < l && joins; ++m) joins = similar(g, l, m);
            if (!joins) block_start = l;
            lowest_out[(size_t)l * num_kv_heads + g] = block_start;
        }
    }
    return POD_OK;
}

extern "C" int pod_prefill_attention(pod_cache *cache, int layer, int seq_slot, int n, const void *q, const void *k,
                                     const void *v, const void *q_shared, const void *k_shared, float scale,
                                     void *out, int write_cache, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!q || !k || !v || !out) return pod_fail(POD_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
    if (n < 1) return pod_fail(POD_ERR_INVALID_ARG, "n must be >= 1");
    const bool lowest = layer_lowest_all(cache, layer);
    if ((q_shared == nullptr) != (k_shared == nullptr))
        return pod_fail(POD_ERR_INVALID_ARG, "q_shared and k_shared must be given together");
    if (!lowest && !q_shared && n > ly.P)
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block and the prompt has distant tokens: q_shared and k_shared are required", layer);
    if (write_cache) {
        if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
        if (n > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "n = %d exceeds max_context = %d", n, ly.maxctx);
        if (cache->host_len[(size_t)layer * ly.B + seq_slot] != 0)
            return pod_fail(POD_ERR_STATE, "slot %d at layer %d is not empty", seq_slot, layer);
    }
    if (lowest) { q_shared = nullptr; k_shared = nullptr; }
    rc = pod_launch_prefill(ly, layer, n, 0, q, k, v, q_shared, k_shared, pod_make_headmap(cache, layer).lowest_mask, scale, out,
                            (hipStream_t)stream);
    if (rc) return rc;
    if (write_cache) return pod_cache_fill(cache, layer, seq_slot, n, k, v, stream);
    return POD_OK;
}

extern "C" int pod_cache_append_many(pod_cache *cache, int layer, const void *k_new, const void *v_new,
                                     const int32_t *positions, const int32_t *counts, int T, int B, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!k_new || !v_new || !positions) return pod_fail(POD_ERR_INVALID_ARG, "k_new, v_new and positions must not be NULL");
    if (B < 1 || B > ly.B) return pod_fail(POD_ERR_INVALID_ARG, "B = %d outside [1, max_batch = %d]", B, ly.B);
    if (T < 1) return pod_fail(POD_ERR_INVALID_ARG, "T must be >= 1");
    int64_t *len = cache->host_len + (size_t)layer * ly.B;
    int32_t *cnt = (int32_t *)malloc((size_t)B * sizeof(int32_t));
    if (!cnt) return pod_fail(POD_ERR_CAPACITY, "out of host memory");
    for (int b = 0; b < B; ++b) {
        cnt[b] = counts ? counts[b] : T;
        if (cnt[b] < 0 || cnt[b] > T) { free(cnt); return pod_fail(POD_ERR_INVALID_ARG, "counts[%d] = %d outside [0, T = %d]", b, counts[b], T); }
        if (len[b] + cnt[b] > ly.maxctx) {
            free(cnt);
            return pod_fail(POD_ERR_CAPACITY, "slot %d at layer %d would exceed max_context = %d", b, layer, ly.maxctx);
        }
    }
    rc = pod_launch_append_many(cache, layer, k_new, v_new, positions, cnt, T, 0, B, (hipStream_t)stream);
    if (rc == POD_OK)
        for (int b = 0; b < B; ++b) len[b] += cnt[b];
    free(cnt);
    return rc;
}

static size_t chunk_rows_bytes(const pod_layout &ly, int64_t n) { return align_up((size_t)n * ly.Hkv * ly.D * 2, 256); }

extern "C" int pod_prefill_chunk_workspace_bytes(const pod_config *cfg, int64_t n_total, size_t *bytes)
{
    pod_layout ly;
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    if (!bytes || n_total < 1) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL or n_total < 1");
    if (n_total > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "n_total = %lld exceeds max_context = %d", (long long)n_total, ly.maxctx);
    const size_t copies = 3 * chunk_rows_bytes(ly, n_total), in_place = pod_chunk_direct_bytes(ly, n_total, 0);
    *bytes = copies > in_place ? copies : in_place;
    return POD_OK;
}

extern "C" int pod_prefill_chunk_in_place_bytes(const pod_config *cfg, int64_t n_total, int64_t T, size_t *bytes)
{
    pod_layout ly;
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    if (!bytes || n_total < 1 || T < 1 || T > n_total) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL, or not 1 <= T <= n_total");
    if (n_total > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "n_total = %lld exceeds max_context = %d", (long long)n_total, ly.maxctx);
    *bytes = pod_chunk_direct_bytes(ly, n_total, T);
    return POD_OK;
}

extern "C" int pod_prefill_attention_chunk(pod_cache *cache, int layer, int seq_slot, int T, const void *q, const void *k,
                                           const void *v, const void *q_shared, const void *k_shared, float scale,
                                           void *workspace, size_t workspace_bytes, void *out, int write_cache, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (!q || !k || !v || !out || !workspace) return pod_fail(POD_ERR_INVALID_ARG, "q, k, v, out and workspace must not be NULL");
    if (T < 1) return pod_fail(POD_ERR_INVALID_ARG, "T must be >= 1");
    if (scale <= 0.f) return pod_fail(POD_ERR_INVALID_ARG, "scale must be positive");
    if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
    if ((q_shared == nullptr) != (k_shared == nullptr))
        return pod_fail(POD_ERR_INVALID_ARG, "q_shared and k_shared must be given together");
    const int64_t p0 = cache->host_len[(size_t)layer * ly.B + seq_slot];
    const int64_t n = p0 + T;
    if (n > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "slot %d at layer %d would exceed max_context = %d", seq_slot, layer, ly.maxctx);
    const bool lowest = layer_lowest_all(cache, layer);
    if (!lowest && !q_shared && n > ly.P)
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest of its block and there are distant tokens: q_shared and k_shared are required", layer);
    for (int h = 0; h < ly.Hkv; ++h) {
        const int la = cache->lowest[(size_t)layer * ly.Hkv + h];
        const int64_t na = cache->host_len[(size_t)la * ly.B + seq_slot];
        if (la != layer && na != p0 && na != n)
            return pod_fail(POD_ERR_STATE, "layer %d (lowest of kv head %d's block) holds %lld tokens of slot %d; layer %d holds %lld and the chunk has %d",
                            la, h, (long long)na, seq_slot, layer, (long long)p0, T);
    }
    if (lowest) { q_shared = nullptr; k_shared = nullptr; }
    hipStream_t st = (hipStream_t)stream;
    // Usual case: the chunk is stored first and the attention kernel takes keys and values straight from the cache.
    // That needs the block's lowest layers to hold the chunk already (their keys are read where they lie) and the
    // caller's leave to store it here.
    bool in_place = write_cache && cache->chunk_in_place;
    for (int h = 0; h < ly.Hkv && in_place; ++h) {
        const int la = cache->lowest[(size_t)layer * ly.Hkv + h];
        if (la != layer && cache->host_len[(size_t)la * ly.B + seq_slot] != n) in_place = false;
    }
    if (in_place) {
        const unsigned long long *tab = nullptr;
        int ntiles = 0;
        rc = pod_launch_chunk_update(cache, layer, seq_slot, (int)p0, T, k, v, workspace, workspace_bytes, &tab, &ntiles, st);
        if (rc) return rc;
        cache->host_len[(size_t)layer * ly.B + seq_slot] = n;
        return pod_launch_prefill_tiles(ly, (int)n, (int)p0, q, q_shared, tab, ntiles,
                                        (int *)(cache->base + ly.off_lens) + (size_t)layer * ly.B + seq_slot, (int *)(cache->base + ly.off_flag),
                                        pod_make_headmap(cache, layer).lowest_mask, scale, out, st);
    }
    const size_t part = chunk_rows_bytes(ly, n);
    if (workspace_bytes < 3 * part) return pod_fail(POD_ERR_CAPACITY, "chunk workspace too small: %zu < %zu", workspace_bytes, 3 * part);
    char *k_all = (char *)workspace, *v_all = k_all + part, *ks_all = q_shared ? v_all + part : nullptr;
    rc = pod_launch_gather(cache, layer, seq_slot, (int)p0, T, k, v, k_shared, k_all, v_all, ks_all, st);
    if (rc) return rc;
    rc = pod_launch_prefill(ly, layer, (int)n, (int)p0, q, k_all, v_all, q_shared, ks_all, pod_make_headmap(cache, layer).lowest_mask,
                            scale, out, st);
    if (rc) return rc;
    if (write_cache) {
        const int32_t cnt = T;
        rc = pod_launch_append_many(cache, layer, k, v, nullptr, &cnt, T, seq_slot, 1, st);
        if (rc) return rc;
        cache->host_len[(size_t)layer * ly.B + seq_slot] = n;
    }
    return POD_OK;
}

// ---- token selection on the distant store (pod_select.hip) ----
constexpr int kMaxSelectRows = 4096; // query rows per kv head (observation window x query heads of a group)

static int check_select_shape(const pod_layout &ly, int64_t n, int obs, int keep)
{
    if (n > ly.maxctx) return pod_fail(POD_ERR_CAPACITY, "n = %lld exceeds max_context = %d", (long long)n, ly.maxctx);
    if (n < (int64_t)ly.S + ly.W + 1) return pod_fail(POD_ERR_INVALID_ARG, "n = %lld leaves no distant token (S + W = %d)", (long long)n, ly.P);
    if (obs < 1 || obs > ly.W || obs * ly.rep > kMaxSelectRows)
        return pod_fail(POD_ERR_INVALID_ARG, "obs = %d outside [1, min(W = %d, %d / %d query heads per kv head)]", obs, ly.W, kMaxSelectRows, ly.rep);
    if (keep < 1 || keep > n - ly.S - ly.W)
        return pod_fail(POD_ERR_INVALID_ARG, "keep = %d outside [1, n - S - W = %lld]", keep, (long long)(n - ly.S - ly.W));
    return POD_OK;
}

extern "C" int pod_select_workspace_bytes(const pod_config *cfg, int64_t n, int obs, int keep, size_t *bytes)
{
    pod_layout ly;
    int rc = make_layout(cfg, &ly);
    if (rc) return rc;
    if (!bytes) return pod_fail(POD_ERR_INVALID_ARG, "bytes is NULL");
    rc = check_select_shape(ly, n, obs, keep);
    if (rc) return rc;
    size_t b = pod_select_votes_bytes(ly, n, obs);
    if (pod_select_top_bytes(ly, n) > b) b = pod_select_top_bytes(ly, n);
    if (pod_compact_bytes(ly, keep) > b) b = pod_compact_bytes(ly, keep);
    *bytes = b;
    return POD_OK;
}

extern "C" int pod_select_votes(pod_cache *cache, int layer, int seq_slot, int n, const void *q_obs, int obs, const void *k,
                                float scale, float *votes, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
    rc = check_select_shape(ly, n, obs, 1);
    if (rc) return rc;
    if (!layer_lowest_any(cache, layer))
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest layer of any head's block: the block's votes are taken at its lowest layer", layer);
    if (!q_obs || !votes || !workspace) return pod_fail(POD_ERR_INVALID_ARG, "q_obs, votes and workspace must not be NULL");
    if (((uintptr_t)q_obs | (uintptr_t)k) % 16 || (uintptr_t)votes % 4 || (uintptr_t)workspace % 256)
        return pod_fail(POD_ERR_INVALID_ARG, "q_obs and k must be 16-byte aligned, workspace 256-byte aligned");
    if (!(scale > 0.f)) return pod_fail(POD_ERR_INVALID_ARG, "scale must be positive");
    if (!k && cache->host_len[(size_t)layer * ly.B + seq_slot] != n)
        return pod_fail(POD_ERR_STATE, "k is NULL (keys from the cache) but slot %d at layer %d holds %lld tokens, not n = %d", seq_slot,
                        layer, (long long)cache->host_len[(size_t)layer * ly.B + seq_slot], n);
    const size_t need = pod_select_votes_bytes(ly, n, obs);
    if (workspace_bytes < need) return pod_fail(POD_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
    return pod_launch_select_votes(cache, layer, seq_slot, pod_make_headmap(cache, layer).lowest_mask, n, q_obs, obs, k, scale, votes,
                                   workspace, (hipStream_t)stream);
}

extern "C" int pod_select_top(pod_cache *cache, int layer, int n, const float *votes, int pool_width, int pool_kind, int keep,
                              int32_t *sel, void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    rc = check_select_shape(ly, n, 1, keep);
    if (rc) return rc;
    if (!layer_lowest_any(cache, layer))
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d is not the lowest layer of any head's block", layer);
    if (!votes || !sel || !workspace) return pod_fail(POD_ERR_INVALID_ARG, "votes, sel and workspace must not be NULL");
    if (pool_width < 1 || pool_width % 2 == 0 || pool_width > 255 || (pool_kind != POD_POOL_AVG && pool_kind != POD_POOL_MAX))
        return pod_fail(POD_ERR_INVALID_ARG, "pool_width must be odd and in [1, 255], pool_kind POD_POOL_AVG or POD_POOL_MAX");
    if ((uintptr_t)votes % 4 || (uintptr_t)sel % 4 || (uintptr_t)workspace % 256)
        return pod_fail(POD_ERR_INVALID_ARG, "votes and sel must be 4-byte aligned, workspace 256-byte aligned");
    const size_t need = pod_select_top_bytes(ly, n);
    if (workspace_bytes < need) return pod_fail(POD_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
    return pod_launch_select_top(ly.Hkv, pod_make_headmap(cache, layer).lowest_mask, votes, n - ly.S - ly.W, pool_width,
                                 pool_kind == POD_POOL_MAX, keep, (float *)workspace, sel + (size_t)layer * ly.Hkv * keep, keep,
                                 (hipStream_t)stream);
}

extern "C" int pod_cache_compact(pod_cache *cache, int layer, int seq_slot, const int32_t *sel, int keep, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
    int64_t *len = cache->host_len + (size_t)layer * ly.B + seq_slot;
    if (*len < (int64_t)ly.S + ly.W + 1)
        return pod_fail(POD_ERR_STATE, "slot %d at layer %d holds %lld tokens: no distant token to select from", seq_slot, layer, (long long)*len);
    rc = check_select_shape(ly, *len, 1, keep);
    if (rc) return rc;
    if (!sel || !workspace) return pod_fail(POD_ERR_INVALID_ARG, "sel and workspace must not be NULL");
    if ((uintptr_t)sel % 4 || (uintptr_t)workspace % 256)
        return pod_fail(POD_ERR_INVALID_ARG, "sel must be 4-byte aligned, workspace 256-byte aligned");
    const size_t need = pod_compact_bytes(ly, keep);
    if (workspace_bytes < need) return pod_fail(POD_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
    rc = pod_launch_compact(cache, layer, seq_slot, (int)*len, sel, keep, workspace, (hipStream_t)stream);
    if (rc) return rc;
    *len = (int64_t)ly.S + keep + ly.W;
    return POD_OK;
}

extern "C" int pod_cache_export_logical(pod_cache *cache, int layer, int seq_slot, void *sinkK, void *sinkV,
                                        void *recentK, void *recentV, void *distK, void *distV, void *stream)
{
    int rc = check_cache_layer(cache, layer);
    if (rc) return rc;
    const pod_layout &ly = cache->ly;
    if (seq_slot < 0 || seq_slot >= ly.B) return pod_fail(POD_ERR_INVALID_ARG, "seq_slot %d outside [0, %d)", seq_slot, ly.B);
    if (distK && !layer_lowest_any(cache, layer))
        return pod_fail(POD_ERR_INVALID_ARG, "layer %d keeps no distant keys (not the lowest layer of any head's block)", layer);
    const int64_t n = cache->host_len[(size_t)layer * ly.B + seq_slot];
    if (n == 0) return POD_OK;
    return pod_launch_export(cache, layer, seq_slot, n, sinkK, sinkV, recentK, recentV, distK, distV, (hipStream_t)stream);
}
