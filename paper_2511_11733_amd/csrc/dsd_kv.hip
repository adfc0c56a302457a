// KV cache import / export / commit kernels (layout: see KvGeom in dsd_internal.h).
#include "dsd_internal.h"

template <typename T>
__global__ void kv_import_kernel(T* __restrict__ kc, T* __restrict__ vc, const T* __restrict__ k,
                                 const T* __restrict__ v, KvGeom g, int n_slots) {
    const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const size_t src = (((size_t)b * g.Hkv + h) * n_slots + slot) * g.hd;
    for (int e = threadIdx.x; e < g.hd; e += blockDim.x) {
        kc[kv_k_off(g, b, h, slot, e)] = k[src + e];
        vc[kv_v_off(g, b, h, slot, e)] = v[src + e];
    }
}

template <typename T>
__global__ void kv_export_kernel(const T* __restrict__ kc, const T* __restrict__ vc, T* __restrict__ k,
                                 T* __restrict__ v, KvGeom g, int first, int n_slots) {
    const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const size_t dst = (((size_t)b * g.Hkv + h) * n_slots + s) * g.hd;
    for (int e = threadIdx.x; e < g.hd; e += blockDim.x) {
        k[dst + e] = kc[kv_k_off(g, b, h, first + s, e)];
        v[dst + e] = vc[kv_v_off(g, b, h, first + s, e)];
    }
}

// One thread owns feature e of one (layer, sequence, head) and moves it for every path node in
// path order.  Node ids grow along a path and node j of the path has id >= j+1, so a destination
// slot is never a source that is still needed.
template <typename T>
__global__ void kv_commit_kernel(T* __restrict__ kc, T* __restrict__ vc, KvGeom g, const int32_t* __restrict__ len,
                                 const int32_t* __restrict__ acc_len, const int32_t* __restrict__ acc_path, int k) {
    const int h = blockIdx.x, b = blockIdx.y, l = blockIdx.z;
    const int e = threadIdx.x;
    T* kl = kc + (size_t)l * g.layer_elems;
    T* vl = vc + (size_t)l * g.layer_elems;
    const int base = len[b];
    int a = acc_len[b];
    a = a < 0 ? 0 : (a > k ? k : a);
    for (int j = 0; j < a; ++j) {
        const int node = acc_path[(size_t)b * k + j];
        if (node < 1 || node > k) break;
        const int src = base + node - 1, dst = base + j;
        if (src == dst || src >= g.S) continue;
        kl[kv_k_off(g, b, h, dst, e)] = kl[kv_k_off(g, b, h, src, e)];
        vl[kv_v_off(g, b, h, dst, e)] = vl[kv_v_off(g, b, h, src, e)];
    }
}

__global__ void kv_advance_kernel(int32_t* __restrict__ len, const int32_t* __restrict__ acc_len, int B, int k, int S) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int a = acc_len[b];
    a = a < 0 ? 0 : (a > k ? k : a);
    int n = len[b] + a;
    len[b] = n > S ? S : n;
}

int kv_import_launch(dsd_ctx* ctx, dsd_kv* kv, int layer, const void* k, const void* v, int B, int n_slots) {
    const KvGeom& g = kv->geom;
    dim3 grid(n_slots, g.Hkv, B);
    const size_t off = (size_t)layer * g.layer_elems;
    if (kv->desc.dtype == DSD_BF16)
        kv_import_kernel<bf16_t><<<grid, 64, 0, ctx->stream>>>((bf16_t*)kv->k + off, (bf16_t*)kv->v + off,
                                                              (const bf16_t*)k, (const bf16_t*)v, g, n_slots);
    else
        kv_import_kernel<float><<<grid, 64, 0, ctx->stream>>>((float*)kv->k + off, (float*)kv->v + off,
                                                             (const float*)k, (const float*)v, g, n_slots);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}

int kv_export_launch(dsd_ctx* ctx, const dsd_kv* kv, int layer, int first, int n, int B, void* k, void* v) {
    const KvGeom& g = kv->geom;
    dim3 grid(n, g.Hkv, B);
    const size_t off = (size_t)layer * g.layer_elems;
    if (kv->desc.dtype == DSD_BF16)
        kv_export_kernel<bf16_t><<<grid, 64, 0, ctx->stream>>>((const bf16_t*)kv->k + off, (const bf16_t*)kv->v + off,
                                                              (bf16_t*)k, (bf16_t*)v, g, first, n);
    else
        kv_export_kernel<float><<<grid, 64, 0, ctx->stream>>>((const float*)kv->k + off, (const float*)kv->v + off,
                                                             (float*)k, (float*)v, g, first, n);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}

int kv_commit_launch(dsd_ctx* ctx, dsd_kv* kv, const int32_t* acc_len, const int32_t* acc_path, int B, int k) {
    const KvGeom& g = kv->geom;
    if (acc_path) {
        dim3 grid(g.Hkv, B, kv->desc.n_layers);
        if (kv->desc.dtype == DSD_BF16)
            kv_commit_kernel<bf16_t><<<grid, g.hd, 0, ctx->stream>>>((bf16_t*)kv->k, (bf16_t*)kv->v, g, kv->len_dev,
                                                                    acc_len, acc_path, k);
        else
            kv_commit_kernel<float><<<grid, g.hd, 0, ctx->stream>>>((float*)kv->k, (float*)kv->v, g, kv->len_dev,
                                                                   acc_len, acc_path, k);
        DSD_HIP(hipGetLastError());
    }
    kv_advance_kernel<<<(B + 63) / 64, 64, 0, ctx->stream>>>(kv->len_dev, acc_len, B, k, g.S);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}
