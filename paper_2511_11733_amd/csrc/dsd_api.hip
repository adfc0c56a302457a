// Host side of libdsd: handles, validation, dispatch.  Every entry point of include/dsd.h
// is defined here; kernels live in the other translation units.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>

#include "dsd_internal.h"

static thread_local char g_err[512] = "";

void dsd_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* dsd_last_error(void) { return g_err; }

// ----------------------------------------------------------------------------- context
static void prof_drop(dsd_ctx* ctx);

extern "C" int dsd_create(int device, void* hip_stream, dsd_ctx** out) {
    if (!out) DSD_FAIL(DSD_EINVAL, "dsd_create: out is NULL");
    int n = 0;
    DSD_HIP(hipGetDeviceCount(&n));
    if (device < 0 || device >= n) DSD_FAIL(DSD_EINVAL, "dsd_create: device %d of %d", device, n);
    DSD_HIP(hipSetDevice(device));
    hipDeviceProp_t prop;
    DSD_HIP(hipGetDeviceProperties(&prop, device));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        DSD_FAIL(DSD_EUNSUPPORTED, "dsd_create: device is %s, this library is built for gfx950 only",
                 prop.gcnArchName);
    DSD_TRY(accept_static_scratch_init(device));         // address of this device's copy of the fixed scratch array
    dsd_ctx* c = new (std::nothrow) dsd_ctx();
    if (!c) DSD_FAIL(DSD_ENOMEM, "dsd_create: host allocation");
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->ws = nullptr;
    c->ws_bytes = 0;
    const char* p = getenv("DSD_PATH");
    c->force_simple = p && strcmp(p, "simple") == 0;
    c->prof_on = false;
    c->no_tiled = getenv("DSD_NO_TILED") != nullptr;
    c->n_cu = prop.multiProcessorCount;
    c->sat_dev = nullptr;
    if (hipMalloc((void**)&c->sat_dev, 256) != hipSuccess || hipMemset(c->sat_dev, 0, 256) != hipSuccess) {
        if (c->sat_dev) hipFree(c->sat_dev);
        delete c;
        DSD_FAIL(DSD_ENOMEM, "dsd_create: device allocation");
    }
    *out = c;
    return DSD_OK;
}

extern "C" int dsd_destroy(dsd_ctx* ctx) {
    if (!ctx) return DSD_OK;
    hipSetDevice(ctx->device);
    hipStreamSynchronize(ctx->stream);
    prof_drop(ctx);
    if (ctx->ws) hipFree(ctx->ws);
    if (ctx->sat_dev) hipFree(ctx->sat_dev);
    delete ctx;
    return DSD_OK;
}

static void prof_drop(dsd_ctx* ctx) {
    for (auto& r : ctx->prof) {
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    ctx->prof.clear();
}

extern "C" int dsd_profile_enable(dsd_ctx* ctx, int on) {
    if (!ctx) DSD_FAIL(DSD_EINVAL, "dsd_profile_enable: ctx is NULL");
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    prof_drop(ctx);
    ctx->prof_on = on != 0;
    return DSD_OK;
}

extern "C" int dsd_profile_read(dsd_ctx* ctx, double* ms_total, int64_t* launches) {
    if (!ctx || !ms_total || !launches) DSD_FAIL(DSD_EINVAL, "dsd_profile_read: NULL argument");
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    for (int i = 0; i < DSD_KC_COUNT; ++i) {
        ms_total[i] = 0.0;
        launches[i] = 0;
    }
    for (auto& r : ctx->prof) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess && r.cls >= 0 && r.cls < DSD_KC_COUNT) {
            ms_total[r.cls] += ms;
            launches[r.cls] += 1;
        }
    }
    prof_drop(ctx);
    return DSD_OK;
}

// ----------------------------------------------------------------------------- stream probe
// What a bare stream over device memory reaches on this chip: the yardstick the weight-streaming
// kernels are measured against besides the published peak.  Every thread keeps U 16-byte loads in
// flight over a grid-stride walk; the read kernel folds what it loads into a word that it stores only
// for a value that does not occur, so the loads cannot be dropped.
template <int U, bool NT>
__global__ void __launch_bounds__(256) stream_read_kernel(const uint4* __restrict__ p, size_t n, unsigned* __restrict__ sink) {
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t* q = (const u32x4_t*)p;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_t a = {0u, 0u, 0u, 0u};
    for (; i + (U - 1) * stride < n; i += U * stride) {
        u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(q + i + u * stride) : q[i + u * stride];
#pragma unroll
        for (int u = 0; u < U; ++u) a ^= v[u];
    }
    for (; i < n; i += stride) a ^= NT ? __builtin_nontemporal_load(q + i) : q[i];
    if ((a.x ^ a.y ^ a.z ^ a.w) == 0x9E3779B9u && a.x == 0x7F4A7C15u) *sink = a.y;
}
// The access pattern of the weight-streaming kernels: every wave walks a contiguous stream of its own,
// 1 KiB per load instruction, U of them in flight (8 waves per compute unit)
template <int U>
__global__ void __launch_bounds__(256) stream_tiles_kernel(const uint4* __restrict__ p, size_t per_stream, unsigned* __restrict__ sink) {
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint4* q = p + wave * per_stream + (threadIdx.x & 63);
    uint4 a = make_uint4(0, 0, 0, 0);
    for (size_t i = 0; i + U * 64 <= per_stream; i += U * 64) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = q[i + u * 64];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            a.x ^= v[u].x; a.y ^= v[u].y; a.z ^= v[u].z; a.w ^= v[u].w;
        }
    }
    if ((a.x ^ a.y ^ a.z ^ a.w) == 0x9E3779B9u && a.x == 0x7F4A7C15u) *sink = a.y;
}
__global__ void __launch_bounds__(256) stream_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        dst[i] = v0; dst[i + stride] = v1; dst[i + 2 * stride] = v2; dst[i + 3 * stride] = v3;
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

extern "C" int dsd_stream_probe(dsd_ctx* ctx, void* buf, size_t bytes, int mode, int iters, double* ms_avg) {
    if (!ctx || !buf || !ms_avg) DSD_FAIL(DSD_EINVAL, "dsd_stream_probe: NULL argument");
    if (bytes < (1u << 20) || (bytes & 31) || ((size_t)buf & 15)) DSD_FAIL(DSD_ESHAPE, "dsd_stream_probe: bytes=%zu", bytes);
    if (mode < 0 || mode > 3) DSD_FAIL(DSD_EINVAL, "dsd_stream_probe: mode=%d", mode);
    if (iters < 1 || iters > 1000) DSD_FAIL(DSD_EINVAL, "dsd_stream_probe: iters=%d", iters);
    DSD_HIP(hipSetDevice(ctx->device));
    DSD_TRY(dsd_ws_reserve(ctx, 256));
    const size_t n = mode == 1 ? bytes / 32 : bytes / 16;      // mode 1: first half -> second half
    // two workgroups of 256 threads per compute unit, four 16-byte loads per thread in flight (32 KiB per compute
    // unit): the fastest of the grids and depths tried on 1 GiB (6.4 TB/s; 8 workgroups per unit: 5.3, 16 loads: 4.8)
    const int grid = ctx->n_cu * 2;
    hipEvent_t e0, e1;
    DSD_HIP(hipEventCreate(&e0));
    DSD_HIP(hipEventCreate(&e1));
    for (int it = -2; it < iters; ++it) {
        if (it == 0) DSD_HIP(hipEventRecord(e0, ctx->stream));
        if (mode == 2) {
            const size_t per_stream = (bytes / 16 / ((size_t)grid * 4)) & ~(size_t)1023;
            stream_tiles_kernel<8><<<grid, 256, 0, ctx->stream>>>((const uint4*)buf, per_stream, (unsigned*)ctx->ws);
        } else if (mode == 0) stream_read_kernel<4, false><<<grid, 256, 0, ctx->stream>>>((const uint4*)buf, n, (unsigned*)ctx->ws);
        else if (mode == 3) stream_read_kernel<4, true><<<grid, 256, 0, ctx->stream>>>((const uint4*)buf, n, (unsigned*)ctx->ws);
        else stream_copy_kernel<<<grid, 256, 0, ctx->stream>>>((uint4*)buf + n, (const uint4*)buf, n);
    }
    DSD_HIP(hipEventRecord(e1, ctx->stream));
    DSD_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    DSD_HIP(hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    DSD_HIP(hipGetLastError());
    *ms_avg = (double)ms / iters;
    return DSD_OK;
}

extern "C" int dsd_set_stream(dsd_ctx* ctx, void* hip_stream) {
    if (!ctx) DSD_FAIL(DSD_EINVAL, "dsd_set_stream: ctx is NULL");
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    ctx->stream = (hipStream_t)hip_stream;
    return DSD_OK;
}

int dsd_ws_reserve(dsd_ctx* ctx, size_t bytes) {
    if (bytes <= ctx->ws_bytes) return DSD_OK;
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    if (ctx->ws) DSD_HIP(hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
    size_t want = (bytes + (size_t)(1 << 20)) & ~(size_t)((1 << 20) - 1);
    void* p = nullptr;
    if (hipMalloc(&p, want) != hipSuccess) DSD_FAIL(DSD_ENOMEM, "workspace of %zu bytes", want);
    ctx->ws = (char*)p;
    ctx->ws_bytes = want;
    return DSD_OK;
}

// ----------------------------------------------------------------------------- model checks
static int check_desc(const dsd_model_desc* d, const char* who) {
    if (!d) DSD_FAIL(DSD_EINVAL, "%s: desc is NULL", who);
    if (d->n_layers < 1 || d->d_model < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->d_ffn < 1)
        DSD_FAIL(DSD_ESHAPE, "%s: non-positive model size", who);
    if (d->n_q_heads % d->n_kv_heads) DSD_FAIL(DSD_ESHAPE, "%s: n_kv_heads must divide n_q_heads", who);
    if (d->head_dim != 64 && d->head_dim != 128) DSD_FAIL(DSD_ESHAPE, "%s: head_dim must be 64 or 128", who);
    if (d->dtype != DSD_F32 && d->dtype != DSD_BF16) DSD_FAIL(DSD_EINVAL, "%s: dtype", who);
    if ((d->has_embed || d->has_head) && d->vocab < 1) DSD_FAIL(DSD_ESHAPE, "%s: vocab", who);
    if (!(d->rope_theta > 1.0f) || !(d->rms_eps > 0.0f)) DSD_FAIL(DSD_EINVAL, "%s: rope_theta / rms_eps", who);
    return DSD_OK;
}

static bool same_geometry(const dsd_model_desc& a, const dsd_model_desc& b) {
    return a.n_layers == b.n_layers && a.n_kv_heads == b.n_kv_heads && a.head_dim == b.head_dim &&
           a.dtype == b.dtype;
}

// ----------------------------------------------------------------------------- weights
static int dev_copy(dsd_ctx* ctx, dsd_weights* w, const void* src, size_t bytes, void** out) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) DSD_FAIL(DSD_ENOMEM, "weight buffer of %zu bytes", bytes);
    w->allocs.push_back(p);
    DSD_HIP(hipMemcpyAsync(p, src, bytes, hipMemcpyDeviceToDevice, ctx->stream));
    *out = p;
    return DSD_OK;
}

extern "C" int dsd_weights_destroy(dsd_ctx* ctx, dsd_weights* w) {
    if (!w) return DSD_OK;
    if (ctx) {
        hipSetDevice(ctx->device);
        hipStreamSynchronize(ctx->stream);
    }
    for (void* p : w->allocs) hipFree(p);
    delete w;
    return DSD_OK;
}

extern "C" int dsd_weights_create(dsd_ctx* ctx, const dsd_model_desc* desc, const void* const* tensors,
                                  int n_tensors, dsd_weights** out) {
    if (!ctx || !tensors || !out) DSD_FAIL(DSD_EINVAL, "dsd_weights_create: NULL argument");
    DSD_TRY(check_desc(desc, "dsd_weights_create"));
    const int want = (desc->has_embed ? 1 : 0) + 9 * desc->n_layers + (desc->has_head ? 2 : 0);
    if (n_tensors != want) DSD_FAIL(DSD_ESHAPE, "dsd_weights_create: %d tensors given, %d expected", n_tensors, want);
    for (int i = 0; i < n_tensors; ++i)
        if (!tensors[i]) DSD_FAIL(DSD_EINVAL, "dsd_weights_create: tensor %d is NULL", i);
    DSD_HIP(hipSetDevice(ctx->device));
    dsd_weights* w = new (std::nothrow) dsd_weights();
    if (!w) DSD_FAIL(DSD_ENOMEM, "dsd_weights_create: host allocation");
    w->desc = *desc;
    w->embed = w->gf = w->lm = w->lm_t = nullptr;
    w->layers.resize(desc->n_layers);
    for (auto& l : w->layers) memset(&l, 0, sizeof(l));
    w->tiled = desc->dtype == DSD_BF16 && !ctx->force_simple && mfma_supported(desc);

    const size_t es = dsd_elem_size(desc->dtype);
    const size_t d = desc->d_model, qd = (size_t)desc->n_q_heads * desc->head_dim,
                 kd = (size_t)desc->n_kv_heads * desc->head_dim, F = desc->d_ffn, V = desc->vocab;
    int rc = DSD_OK;
    int t = 0;
    if (desc->has_embed) rc = dev_copy(ctx, w, tensors[t++], V * d * es, &w->embed);
    if (rc == DSD_OK && w->tiled) {
        rc = mfma_weights_tile(ctx, w, tensors);
    } else if (rc == DSD_OK) {
        for (int l = 0; l < desc->n_layers && rc == DSD_OK; ++l) {
            LayerW& L = w->layers[l];
            const size_t sizes[9] = {d, qd * d, kd * d, kd * d, d * qd, d, F * d, F * d, d * F};
            void** dst[9] = {&L.g1, &L.wq, &L.wk, &L.wv, &L.wo, &L.g2, &L.wg, &L.wu, &L.wd};
            for (int j = 0; j < 9 && rc == DSD_OK; ++j) rc = dev_copy(ctx, w, tensors[t++], sizes[j] * es, dst[j]);
        }
        if (rc == DSD_OK && desc->has_head) {
            rc = dev_copy(ctx, w, tensors[t++], d * es, &w->gf);
            if (rc == DSD_OK) rc = dev_copy(ctx, w, tensors[t++], V * d * es, &w->lm);
        }
    }
    if (rc == DSD_OK && hipStreamSynchronize(ctx->stream) != hipSuccess) {
        dsd_set_error("dsd_weights_create: synchronise failed");
        rc = DSD_EHIP;
    }
    if (rc != DSD_OK) {
        for (void* p : w->allocs) hipFree(p);
        delete w;
        return rc;
    }
    *out = w;
    return DSD_OK;
}

// ----------------------------------------------------------------------------- KV cache
extern "C" int dsd_kv_create(dsd_ctx* ctx, const dsd_model_desc* desc, int max_batch, int max_slots, dsd_kv** out) {
    if (!ctx || !out) DSD_FAIL(DSD_EINVAL, "dsd_kv_create: NULL argument");
    DSD_TRY(check_desc(desc, "dsd_kv_create"));
    if (max_batch < 1 || max_slots < 1) DSD_FAIL(DSD_ESHAPE, "dsd_kv_create: max_batch / max_slots");
    DSD_HIP(hipSetDevice(ctx->device));
    dsd_kv* kv = new (std::nothrow) dsd_kv();
    if (!kv) DSD_FAIL(DSD_ENOMEM, "dsd_kv_create: host allocation");
    kv->desc = *desc;
    KvGeom& g = kv->geom;
    g.Hkv = desc->n_kv_heads;
    g.hd = desc->head_dim;
    g.S = (max_slots + 63) / 64 * 64;
    g.Bmax = max_batch;
    g.layer_elems = (size_t)g.Bmax * g.Hkv * g.S * g.hd;
    const size_t bytes = g.layer_elems * desc->n_layers * dsd_elem_size(desc->dtype);
    kv->k = kv->v = nullptr;
    kv->len_dev = nullptr;
    kv->last_k = 0;
    kv->cap = max_slots;
    if (hipMalloc(&kv->k, bytes) != hipSuccess || hipMalloc(&kv->v, bytes) != hipSuccess ||
        hipMalloc((void**)&kv->len_dev, sizeof(int32_t) * max_batch) != hipSuccess) {
        if (kv->k) hipFree(kv->k);
        if (kv->v) hipFree(kv->v);
        if (kv->len_dev) hipFree(kv->len_dev);
        delete kv;
        DSD_FAIL(DSD_ENOMEM, "dsd_kv_create: 2 x %zu bytes", bytes);
    }
    // Unused slots are read (and masked) by the attention kernels in whole tiles: keep them finite.
    hipMemsetAsync(kv->k, 0, bytes, ctx->stream);
    hipMemsetAsync(kv->v, 0, bytes, ctx->stream);
    hipMemsetAsync(kv->len_dev, 0, sizeof(int32_t) * max_batch, ctx->stream);
    kv->len_bound.assign(max_batch, 0);
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    *out = kv;
    return DSD_OK;
}

extern "C" int dsd_kv_destroy(dsd_ctx* ctx, dsd_kv* kv) {
    if (!kv) return DSD_OK;
    if (ctx) {
        hipSetDevice(ctx->device);
        hipStreamSynchronize(ctx->stream);
    }
    hipFree(kv->k);
    hipFree(kv->v);
    hipFree(kv->len_dev);
    delete kv;
    return DSD_OK;
}

extern "C" int dsd_kv_set_len(dsd_ctx* ctx, dsd_kv* kv, const int32_t* host_len, int B) {
    if (!ctx || !kv || !host_len) DSD_FAIL(DSD_EINVAL, "dsd_kv_set_len: NULL argument");
    if (B < 1 || B > kv->geom.Bmax) DSD_FAIL(DSD_ESHAPE, "dsd_kv_set_len: B=%d, cache holds %d", B, kv->geom.Bmax);
    for (int b = 0; b < B; ++b)
        if (host_len[b] < 0 || host_len[b] > kv->cap)
            DSD_FAIL(DSD_ESHAPE, "dsd_kv_set_len: len[%d]=%d, cache holds %d slots", b, host_len[b], kv->cap);
    // the host array may go away after the call: copy synchronously
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    DSD_HIP(hipMemcpy(kv->len_dev, host_len, sizeof(int32_t) * B, hipMemcpyHostToDevice));
    for (int b = 0; b < B; ++b) kv->len_bound[b] = host_len[b];
    return DSD_OK;
}

extern "C" int dsd_kv_get_len(dsd_ctx* ctx, const dsd_kv* kv, int32_t* host_len, int B) {
    if (!ctx || !kv || !host_len) DSD_FAIL(DSD_EINVAL, "dsd_kv_get_len: NULL argument");
    if (B < 1 || B > kv->geom.Bmax) DSD_FAIL(DSD_ESHAPE, "dsd_kv_get_len: B=%d, cache holds %d", B, kv->geom.Bmax);
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    DSD_HIP(hipMemcpy(host_len, kv->len_dev, sizeof(int32_t) * B, hipMemcpyDeviceToHost));
    // a read-back is exact: tighten the bounds used for validation and grid sizes
    dsd_kv* m = const_cast<dsd_kv*>(kv);
    for (int b = 0; b < B; ++b) m->len_bound[b] = host_len[b];
    return DSD_OK;
}

extern "C" int dsd_kv_import(dsd_ctx* ctx, dsd_kv* kv, int layer, const void* k, const void* v, int B, int n_slots) {
    if (!ctx || !kv || !k || !v) DSD_FAIL(DSD_EINVAL, "dsd_kv_import: NULL argument");
    if (layer < 0 || layer >= kv->desc.n_layers) DSD_FAIL(DSD_EINVAL, "dsd_kv_import: layer %d", layer);
    if (B < 1 || B > kv->geom.Bmax || n_slots < 1 || n_slots > kv->cap)
        DSD_FAIL(DSD_ESHAPE, "dsd_kv_import: B=%d n_slots=%d vs cache %d x %d", B, n_slots, kv->geom.Bmax, kv->cap);
    DSD_HIP(hipSetDevice(ctx->device));
    return kv_import_launch(ctx, kv, layer, k, v, B, n_slots);
}

extern "C" int dsd_kv_export(dsd_ctx* ctx, const dsd_kv* kv, int layer, int first_slot, int n_slots, int B,
                             void* k_out, void* v_out) {
    if (!ctx || !kv || !k_out || !v_out) DSD_FAIL(DSD_EINVAL, "dsd_kv_export: NULL argument");
    if (layer < 0 || layer >= kv->desc.n_layers) DSD_FAIL(DSD_EINVAL, "dsd_kv_export: layer %d", layer);
    if (B < 1 || B > kv->geom.Bmax || first_slot < 0 || n_slots < 1 || first_slot + n_slots > kv->cap)
        DSD_FAIL(DSD_ESHAPE, "dsd_kv_export: B=%d slots [%d,%d) vs cache %d x %d", B, first_slot,
                 first_slot + n_slots, kv->geom.Bmax, kv->cap);
    DSD_HIP(hipSetDevice(ctx->device));
    return kv_export_launch(ctx, kv, layer, first_slot, n_slots, B, k_out, v_out);
}

extern "C" int dsd_kv_commit(dsd_ctx* ctx, dsd_kv* kv, const int32_t* accepted_len, const int32_t* accepted_path,
                             int B, int k) {
    if (!ctx || !kv || !accepted_len) DSD_FAIL(DSD_EINVAL, "dsd_kv_commit: NULL argument");
    if (B < 1 || B > kv->geom.Bmax || k < 1 || k > DSD_MAX_K) DSD_FAIL(DSD_ESHAPE, "dsd_kv_commit: B=%d k=%d", B, k);
    if (k != kv->last_k) DSD_FAIL(DSD_ESHAPE, "dsd_kv_commit: k=%d but the last verify wrote %d rows", k, kv->last_k);
    DSD_HIP(hipSetDevice(ctx->device));
    DSD_TRY(kv_commit_launch(ctx, kv, accepted_len, accepted_path, B, k));
    for (int b = 0; b < B; ++b) kv->len_bound[b] = std::min(kv->len_bound[b] + k, kv->cap);
    kv->last_k = 0;
    return DSD_OK;
}

// ----------------------------------------------------------------------------- verify
extern "C" int dsd_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                                const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth,
                                int B, int k, void* hidden_out, float* logits, int64_t logits_seq_stride) {
    if (!ctx || !w || !kv) DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: NULL handle");
    if (!same_geometry(w->desc, kv->desc)) DSD_FAIL(DSD_ESHAPE, "dsd_stage_verify: cache and weights differ in geometry");
    if (B < 1 || B > kv->geom.Bmax) DSD_FAIL(DSD_ESHAPE, "dsd_stage_verify: B=%d, cache holds %d", B, kv->geom.Bmax);
    if (k < 1 || k > DSD_MAX_K) DSD_FAIL(DSD_ESHAPE, "dsd_stage_verify: k=%d, limit %d", k, DSD_MAX_K);
    if ((tree_mask == nullptr) != (depth == nullptr))
        DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: tree_mask and depth go together");
    if (!hidden_in && !w->desc.has_embed) DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: hidden_in is NULL and the block has no embedding");
    if (!hidden_in && !draft_tokens) DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: draft_tokens is NULL");
    if (logits && !w->desc.has_head) DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: logits asked of a block without LM head");
    if (!logits && !hidden_out) DSD_FAIL(DSD_EINVAL, "dsd_stage_verify: no output requested");
    if (logits_seq_stride == 0) logits_seq_stride = (int64_t)k * w->desc.vocab;
    if (logits && logits_seq_stride < (int64_t)k * w->desc.vocab)
        DSD_FAIL(DSD_ESHAPE, "dsd_stage_verify: logits_seq_stride smaller than k*V");
    for (int b = 0; b < B; ++b)
        if (kv->len_bound[b] + k > kv->cap)
            DSD_FAIL(DSD_ESHAPE, "dsd_stage_verify: sequence %d: %d + %d rows exceed %d slots", b, kv->len_bound[b], k,
                     kv->cap);
    DSD_HIP(hipSetDevice(ctx->device));
    int rc;
    if (w->tiled)
        rc = mfma_stage_verify(ctx, w, kv, hidden_in, draft_tokens, tree_mask, depth, B, k, hidden_out, logits,
                               logits_seq_stride);
    else
        rc = simple_stage_verify(ctx, w, kv, hidden_in, draft_tokens, tree_mask, depth, B, k, hidden_out, logits,
                                 logits_seq_stride);
    if (rc == DSD_OK) kv->last_k = k;
    return rc;
}

extern "C" int dsd_stage_status(dsd_ctx* ctx, int64_t* saturated) {
    if (!ctx) DSD_FAIL(DSD_EINVAL, "dsd_stage_status: ctx is NULL");
    DSD_HIP(hipSetDevice(ctx->device));
    int n = 0;
    DSD_HIP(hipMemcpyAsync(&n, ctx->sat_dev, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    if (saturated) *saturated = n;
    if (n == 0) return DSD_OK;
    DSD_HIP(hipMemsetAsync(ctx->sat_dev, 0, sizeof(int), ctx->stream));
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    DSD_FAIL(DSD_EUNSUPPORTED, "%d conversion(s) of activations to fp16 matrix-core operands met magnitudes beyond 65504 (or NaN) "
             "since the last check: the results of those dsd_stage_verify calls are not valid", n);
}

// ----------------------------------------------------------------------------- accept
static int accept_check(const char* who, dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                        const float* uniforms, const dsd_accept_params* p, int B, int k, int V, int32_t* accepted_len,
                        int32_t* next_token) {
    const bool greedy = p && p->temperature == 0.0;      // draft_probs and uniforms are not read then
    if (!ctx || !logits || (!draft_probs && !greedy) || !draft_tokens || (!uniforms && !greedy) || !p || !accepted_len ||
        !next_token)
        DSD_FAIL(DSD_EINVAL, "%s: NULL argument", who);
    if (B < 1 || k < 1 || k > DSD_MAX_K || V < 1) DSD_FAIL(DSD_ESHAPE, "%s: B=%d k=%d V=%d", who, B, k, V);
    if (p->top_m < 1 || p->top_m > DSD_MAX_TOP_M || p->top_m > V)
        DSD_FAIL(DSD_ESHAPE, "%s: top_m=%d (limit %d, V=%d)", who, p->top_m, DSD_MAX_TOP_M, V);
    if (!(p->tau >= 0.0 && p->tau <= 1.0)) DSD_FAIL(DSD_EINVAL, "%s: tau=%g outside [0,1]", who, p->tau);
    if ((p->norm_match_kind != DSD_NM_TOP_M && p->norm_match_kind != DSD_NM_OVERLAP) ||
        (p->entropy_kind != DSD_H_TOKEN && p->entropy_kind != DSD_H_ROW))
        DSD_FAIL(DSD_EINVAL, "%s: norm_match_kind=%d entropy_kind=%d", who, p->norm_match_kind, p->entropy_kind);
    if (!(p->temperature >= 0.0)) DSD_FAIL(DSD_EINVAL, "%s: temperature=%g", who, p->temperature);
    if (p->tree_mode != DSD_TREE_LONGEST && p->tree_mode != DSD_TREE_FIRST_ACCEPTED && p->tree_mode != DSD_TREE_LOSSLESS)
        DSD_FAIL(DSD_EINVAL, "%s: tree_mode=%d", who, p->tree_mode);
    return DSD_OK;
}

extern "C" int dsd_accept(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                          const int32_t* parent, const float* uniforms, const dsd_accept_params* p, int B, int k,
                          int V, int32_t* accepted_len, int32_t* next_token, int32_t* accepted_path,
                          const dsd_accept_stats* stats) {
    DSD_TRY(accept_check("dsd_accept", ctx, logits, draft_probs, draft_tokens, uniforms, p, B, k, V, accepted_len, next_token));
    DSD_HIP(hipSetDevice(ctx->device));
    DSD_TRY(dsd_ws_reserve(ctx, accept_scratch_bytes(B, k, V, p->top_m)));
    return accept_launch(ctx, logits, draft_probs, draft_tokens, parent, uniforms, p, B, k, V, accepted_len,
                         next_token, accepted_path, stats, ctx->ws);
}

extern "C" int dsd_accept_noalloc(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                                  const int32_t* parent, const float* uniforms, const dsd_accept_params* p, int B, int k,
                                  int V, int32_t* accepted_len, int32_t* next_token, int32_t* accepted_path,
                                  const dsd_accept_stats* stats) {
    DSD_TRY(accept_check("dsd_accept_noalloc", ctx, logits, draft_probs, draft_tokens, uniforms, p, B, k, V, accepted_len,
                         next_token));
    size_t have = 0;
    char* scratch_dev = accept_static_scratch(ctx->device, &have);
    if (!scratch_dev) DSD_FAIL(DSD_EUNSUPPORTED, "dsd_accept_noalloc: device %d has no static scratch", ctx->device);
    const size_t need = accept_scratch_bytes(B, k, V, p->top_m);
    if (need > have)
        DSD_FAIL(DSD_ESHAPE, "dsd_accept_noalloc: B=%d k=%d V=%d top_m=%d need %zu bytes of scratch, the fixed array holds %zu; "
                 "use dsd_accept", B, k, V, p->top_m, need, have);
    DSD_HIP(hipSetDevice(ctx->device));
    // per-kernel timing creates events: not on this path
    const bool prof = ctx->prof_on;
    ctx->prof_on = false;
    const int rc = accept_launch(ctx, logits, draft_probs, draft_tokens, parent, uniforms, p, B, k, V, accepted_len,
                                 next_token, accepted_path, stats, scratch_dev);
    ctx->prof_on = prof;
    return rc;
}
