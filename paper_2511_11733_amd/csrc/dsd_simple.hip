// Generic kernels for the verification pass: any shape, fp32 or bf16 storage, fp32 arithmetic,
// no matrix cores.  This is the path of fp32 models (the tiny decoder configuration) and, with
// DSD_PATH=simple, a second GPU implementation to hold the bf16 MFMA path against.
//
// Steps per layer (section 2.1's single forward pass over the window, Llama decoder block):
//   a = rmsnorm(x; g1);  q,k,v = a W^T;  rotate q,k;  write k,v to the cache;
//   o = attention(q over cache + masked drafted rows);  x += o Wo^T;
//   b = rmsnorm(x; g2);  x += (silu(b Wg^T) * (b Wu^T)) Wd^T
#include "dsd_internal.h"

#define WAVE 64

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// block-wide reductions for blocks of up to 16 waves; `sh` holds 16 floats
__device__ inline float block_sum(float v, float* sh) {
    v = wave_sum(v);
    const int w = threadIdx.x / WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sh[w] = v;
    __syncthreads();
    float r = 0.f;
    for (int i = 0; i < nw; ++i) r += sh[i];
    return r;
}
__device__ inline float block_max(float v, float* sh) {
    v = wave_max(v);
    const int w = threadIdx.x / WAVE, nw = (blockDim.x + WAVE - 1) / WAVE;
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sh[w] = v;
    __syncthreads();
    float r = -INFINITY;
    for (int i = 0; i < nw; ++i) r = fmaxf(r, sh[i]);
    return r;
}

// x[m,:] = E[token[m],:]  or  x[m,:] = hidden_in[m,:]
template <typename T>
__global__ void load_rows_kernel(float* __restrict__ x, const T* __restrict__ hidden_in, const T* __restrict__ embed,
                                 const int32_t* __restrict__ tokens, int d, int vocab) {
    const int m = blockIdx.x;
    const T* src;
    if (hidden_in) {
        src = hidden_in + (size_t)m * d;
    } else {
        int t = tokens[m];
        t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
        src = embed + (size_t)t * d;
    }
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = ld_f32(src + i);
}

template <typename T>
__global__ void store_rows_kernel(T* __restrict__ out, const float* __restrict__ x, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) st_f32(out + i, x[i]);
}

template <typename T>
__global__ void rmsnorm_kernel(float* __restrict__ a, const float* __restrict__ x, const T* __restrict__ g, int d,
                               float eps) {
    __shared__ float sh[16];
    const int m = blockIdx.x;
    const float* xr = x + (size_t)m * d;
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) s += xr[i] * xr[i];
    s = block_sum(s, sh);
    const float r = 1.0f / sqrtf(s / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += blockDim.x) a[(size_t)m * d + i] = xr[i] * r * ld_f32(g + i);
}

// y[m,n] (+)= sum_k a[m,k] W[n,k].  One wave per output column, 8 rows at a time.
// Output row m lives at out + (m / rows_per_seq) * seq_stride + (m % rows_per_seq) * N.
template <typename T, bool ADD>
__global__ void gemm_rowdot_kernel(float* __restrict__ out, const float* __restrict__ a, const T* __restrict__ W,
                                   int M, int N, int K, int rows_per_seq, int64_t seq_stride) {
    const int n = blockIdx.x * (blockDim.x / WAVE) + threadIdx.x / WAVE;
    const int lane = threadIdx.x & (WAVE - 1);
    if (n >= N) return;
    const T* wr = W + (size_t)n * K;
    for (int m0 = 0; m0 < M; m0 += 8) {
        float acc[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = 0.f;
        for (int kk = lane; kk < K; kk += WAVE) {
            const float wv = ld_f32(wr + kk);
#pragma unroll
            for (int r = 0; r < 8; ++r)
                if (m0 + r < M) acc[r] += a[(size_t)(m0 + r) * K + kk] * wv;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float s = wave_sum(acc[r]);
            if (lane == 0 && m0 + r < M) {
                const int m = m0 + r;
                float* o = out + (size_t)(m / rows_per_seq) * seq_stride + (size_t)(m % rows_per_seq) * N + n;
                if (ADD) *o += s; else *o = s;
            }
        }
    }
}

// Rotates q in place (fp32), rotates k and writes k, v into the cache slots len[b] + t.
template <typename T>
__global__ void rope_append_kernel(float* __restrict__ q, const float* __restrict__ kx, const float* __restrict__ vx,
                                   T* __restrict__ kc, T* __restrict__ vc, KvGeom g, const int32_t* __restrict__ len,
                                   const int32_t* __restrict__ depth, int k, int Hq, float theta) {
    const int m = blockIdx.x;          // row = b*k + t
    const int b = m / k, t = m % k;
    const int hd = g.hd, half = hd / 2;
    const int L = len[b];
    const double pos = (double)(L + (depth ? depth[t] : t));
    const int slot = L + t;
    const int nheads = Hq + g.Hkv;
    for (int i = threadIdx.x; i < nheads * half; i += blockDim.x) {
        const int h = i / half, e = i % half;
        // the angle in fp64: at position 8192 an fp32 product is off by about 5e-4 rad
        const double inv = pow((double)theta, -2.0 * (double)e / (double)hd);
        double snd, csd;
        sincos(pos * inv, &snd, &csd);
        const float sn = (float)snd, cs = (float)csd;
        if (h < Hq) {
            float* p = q + ((size_t)m * Hq + h) * hd;
            const float a = p[e], c = p[e + half];
            p[e] = a * cs - c * sn;
            p[e + half] = c * cs + a * sn;
        } else {
            const int hk = h - Hq;
            const float* p = kx + ((size_t)m * g.Hkv + hk) * hd;
            const float a = p[e], c = p[e + half];
            if (slot < g.S) {
                st_f32(kc + kv_k_off(g, b, hk, slot, e), a * cs - c * sn);
                st_f32(kc + kv_k_off(g, b, hk, slot, e + half), c * cs + a * sn);
            }
        }
    }
    if (slot < g.S)
        for (int i = threadIdx.x; i < g.Hkv * hd; i += blockDim.x) {
            const int hk = i / hd, e = i % hd;
            st_f32(vc + kv_v_off(g, b, hk, slot, e), vx[((size_t)m * g.Hkv + hk) * hd + e]);
        }
}

// One block per (row, query head): scores over the visible slots in LDS, softmax, weighted sum.
template <typename T>
__global__ void attn_rowhead_kernel(float* __restrict__ out, const float* __restrict__ q, const T* __restrict__ kc,
                                    const T* __restrict__ vc, KvGeom g, const int32_t* __restrict__ len,
                                    const uint64_t* __restrict__ mask, int k, int Hq) {
    extern __shared__ float sc[];      // [n_keys] scores, then 16 floats of reduction scratch
    const int m = blockIdx.x, h = blockIdx.y;
    const int b = m / k, t = m % k;
    const int hk = h / (Hq / g.Hkv);
    const int hd = g.hd;
    const int L = len[b];
    const int nk = min(L + k, g.S);
    float* red = sc + nk;
    const uint64_t vis = mask ? mask[t] : ((t >= 63) ? ~0ull : ((1ull << (t + 1)) - 1ull));
    const float* qr = q + ((size_t)m * Hq + h) * hd;
    const float scale = 1.0f / sqrtf((float)hd);
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < nk; j += blockDim.x) {
        float s = -INFINITY;
        if (j < L || ((vis >> (j - L)) & 1ull)) {
            s = 0.f;
            for (int e = 0; e < hd; ++e) s += qr[e] * ld_f32(kc + kv_k_off(g, b, hk, j, e));
            s *= scale;
        }
        sc[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = block_max(mx, red);
    float sum = 0.f;
    for (int j = threadIdx.x; j < nk; j += blockDim.x) {
        const float p = (sc[j] == -INFINITY) ? 0.f : expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = block_sum(sum, red);
    __syncthreads();
    for (int e = threadIdx.x; e < hd; e += blockDim.x) {
        float acc = 0.f;
        for (int j = 0; j < nk; ++j) acc += sc[j] * ld_f32(vc + kv_v_off(g, b, hk, j, e));
        out[((size_t)m * Hq + h) * hd + e] = acc / sum;
    }
}

__global__ void swiglu_kernel(float* __restrict__ gate, const float* __restrict__ up, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const float gv = gate[i];
        gate[i] = gv / (1.0f + expf(-gv)) * up[i];
    }
}

template <typename T>
static void gemm(hipStream_t s, float* out, const float* a, const void* W, int M, int N, int K, bool add,
                 int rows_per_seq = 0, int64_t seq_stride = 0) {
    if (rows_per_seq == 0) {
        rows_per_seq = M;
        seq_stride = 0;
    }
    const int cols_per_block = 4;
    dim3 grid((N + cols_per_block - 1) / cols_per_block);
    if (add)
        gemm_rowdot_kernel<T, true><<<grid, cols_per_block * WAVE, 0, s>>>(out, a, (const T*)W, M, N, K, rows_per_seq, seq_stride);
    else
        gemm_rowdot_kernel<T, false><<<grid, cols_per_block * WAVE, 0, s>>>(out, a, (const T*)W, M, N, K, rows_per_seq, seq_stride);
}

template <typename T>
static int run_simple(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                      const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth, int B, int k,
                      void* hidden_out, float* logits, int64_t logits_seq_stride) {
    const dsd_model_desc& D = w->desc;
    const KvGeom& g = kv->geom;
    const int M = B * k, d = D.d_model, Hq = D.n_q_heads, Hkv = D.n_kv_heads, hd = D.head_dim, F = D.d_ffn;
    const size_t qd = (size_t)Hq * hd, kd = (size_t)Hkv * hd;
    const size_t wide = std::max((size_t)d, qd);
    size_t need = ((size_t)M * d + (size_t)M * wide + (size_t)M * qd + 2 * (size_t)M * kd + (size_t)M * qd +
                   2 * (size_t)M * F) * sizeof(float) + 16 * 256;
    DSD_TRY(dsd_ws_reserve(ctx, need));
    WsBump ws{ctx->ws, 0};
    float* x = ws.take<float>((size_t)M * d);
    float* a = ws.take<float>((size_t)M * wide);
    float* q = ws.take<float>((size_t)M * qd);
    float* kx = ws.take<float>((size_t)M * kd);
    float* vx = ws.take<float>((size_t)M * kd);
    float* att = ws.take<float>((size_t)M * qd);
    float* gate = ws.take<float>((size_t)M * F);
    float* up = ws.take<float>((size_t)M * F);
    hipStream_t s = ctx->stream;

    int max_len = 0;
    for (int b = 0; b < B; ++b) max_len = std::max(max_len, kv->len_bound[b]);
    const size_t attn_lds = ((size_t)max_len + k + 16) * sizeof(float);
    if (attn_lds > 160 * 1024 - 256) DSD_FAIL(DSD_EUNSUPPORTED, "generic attention: %d slots exceed LDS", max_len + k);
    if (attn_lds > 64 * 1024) {
        DSD_HIP(hipFuncSetAttribute((const void*)attn_rowhead_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)attn_lds));
    }

    load_rows_kernel<T><<<M, 256, 0, s>>>(x, (const T*)hidden_in, (const T*)w->embed, draft_tokens, d, D.vocab);
    for (int l = 0; l < D.n_layers; ++l) {
        const LayerW& W = w->layers[l];
        T* kc = (T*)kv->k + (size_t)l * g.layer_elems;
        T* vc = (T*)kv->v + (size_t)l * g.layer_elems;
        rmsnorm_kernel<T><<<M, 256, 0, s>>>(a, x, (const T*)W.g1, d, D.rms_eps);
        gemm<T>(s, q, a, W.wq, M, (int)qd, d, false);
        gemm<T>(s, kx, a, W.wk, M, (int)kd, d, false);
        gemm<T>(s, vx, a, W.wv, M, (int)kd, d, false);
        rope_append_kernel<T><<<M, 256, 0, s>>>(q, kx, vx, kc, vc, g, kv->len_dev, depth, k, Hq, D.rope_theta);
        attn_rowhead_kernel<T><<<dim3(M, Hq), 256, attn_lds, s>>>(att, q, kc, vc, g, kv->len_dev, tree_mask, k, Hq);
        gemm<T>(s, x, att, W.wo, M, d, (int)qd, true);
        rmsnorm_kernel<T><<<M, 256, 0, s>>>(a, x, (const T*)W.g2, d, D.rms_eps);
        gemm<T>(s, gate, a, W.wg, M, F, d, false);
        gemm<T>(s, up, a, W.wu, M, F, d, false);
        const size_t n = (size_t)M * F;
        swiglu_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(gate, up, n);
        gemm<T>(s, x, gate, W.wd, M, d, F, true);
    }
    if (hidden_out) {
        const size_t n = (size_t)M * d;
        store_rows_kernel<T><<<(unsigned)((n + 255) / 256), 256, 0, s>>>((T*)hidden_out, x, n);
    }
    if (logits) {
        rmsnorm_kernel<T><<<M, 256, 0, s>>>(a, x, (const T*)w->gf, d, D.rms_eps);
        gemm<T>(s, logits, a, w->lm, M, D.vocab, d, false, k, logits_seq_stride);
    }
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}

int simple_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                        const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth, int B, int k,
                        void* hidden_out, float* logits, int64_t logits_seq_stride) {
    if (w->desc.dtype == DSD_BF16)
        return run_simple<bf16_t>(ctx, w, kv, hidden_in, draft_tokens, tree_mask, depth, B, k, hidden_out, logits,
                                  logits_seq_stride);
    return run_simple<float>(ctx, w, kv, hidden_in, draft_tokens, tree_mask, depth, B, k, hidden_out, logits,
                             logits_seq_stride);
}
