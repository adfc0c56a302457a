// bf16 path of the verification pass (section 2.1: one forward pass over the k drafted rows, on
// this node's block of layers, section 2.2), written for gfx950 matrix cores.
//
// The pass is bound by streaming the block's weights and the KV cache from HBM once; the k*B
// activation rows are tiny.  Hence:
//   * weights are re-tiled once (dsd_weights_create) into the exact operand order of
//     v_mfma_f32_16x16x32_f16, converted to fp16 (exact for bf16 magnitudes 2^-17 .. 65504), so that
//     every wavefront load is one contiguous KiB;
//   * a GEMM workgroup owns one (or a pair of) 16-column tiles and splits K over its waves,
//     partial tiles meet in LDS, and the epilogue is fused: RMSNorm scale, rotary embedding +
//     KV-cache append, SiLU*up, residual add, or fp32 logits;
//   * RMSNorm never makes a pass of its own: x*g is applied while the A operand is loaded, the
//     sum of squares is accumulated from those same loads, and 1/rms scales the output rows;
//   * in these kernels activations enter the matrix cores as a sum of two fp16 terms (hi + lo, two
//     MFMAs per weight fragment, ~22 significant bits; the extra MFMA work is free while the pass is
//     bandwidth bound); on the panel path (dsd_gemm_tiled.hip: most row counts) as one fp16 term
//     (11 bits).  Queries and attention weights meet the bf16 cache as hi + lo bf16;
//   * attention computes S^T = K Q^T so that the scores a lane holds are exactly the P^T operand
//     of O^T = V^T P^T; V is cached transposed for that product (see KvGeom).
#include <stdlib.h>

#include "dsd_bf16_dev.h"

// ============================================================================ weight tiling
// dst fragment (nt, ks): lane l holds W[nt*16 + l%16][ks*32 + (l/16)*8 .. +8], converted to fp16.
// Fragments are stored k-step major: fragment (nt, ks) of a buffer of NTA column tiles sits at
// (ks*NTA + nt)*64 + lane.  All workgroups of a GEMM walk their k-steps at about the same pace, so at
// any moment the chip reads one narrow, advancing band of the buffer instead of one stream per wave;
// a bare read kernel was measured about a tenth faster in that pattern.
// The conversion is exact for every bf16 value of magnitude 2^-17 .. 65504 (8 significant bits fit
// into fp16's 11, and into its subnormals down to 2^-24 granularity); smaller ones round to the
// nearest multiple of 2^-24.  A weight beyond the fp16 range (or not finite) is counted in *bad.
__global__ void tile_weights_kernel(uint4* __restrict__ dst, const bf16_t* __restrict__ src, int N, int K,
                                    size_t dst_tile_off, size_t NTA, int* __restrict__ bad) {
    const int KS = K / 32;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t total = (size_t)(N / 16) * KS * 64;
    if (idx >= total) return;
    const int l = (int)(idx & 63);
    const size_t f = idx >> 6;
    const int ks = (int)(f % KS);
    const size_t nt = f / KS;
    const size_t s = (nt * 16 + (l & 15)) * (size_t)K + (size_t)ks * 32 + (l >> 4) * 8;
    float v[8];
    unpack_gain(*(const uint4*)(src + s), v);
    bool ok = true;
#pragma unroll
    for (int i = 0; i < 8; ++i) ok = ok && fabsf(v[i]) <= F16_MAX;      // false for NaN too
    if (!ok) atomicAdd(bad, 1);
    dst[((size_t)ks * NTA + dst_tile_off + nt) * 64 + l] = __builtin_bit_cast(uint4, pack8h(v));
}

int mfma_supported(const dsd_model_desc* d) {
    return d->dtype == DSD_BF16 && d->head_dim == 128 && d->d_model % 32 == 0 && d->d_ffn % 32 == 0 &&
           d->d_model % 16 == 0 && d->d_ffn % 16 == 0 && (!d->has_head || d->vocab % 16 == 0);
}

static int tile_into(dsd_ctx* ctx, int* bad, void* dst, size_t dst_tile_off, size_t NTA, const void* src, int N, int K) {
    const size_t total = (size_t)(N / 16) * (K / 32) * 64;
    tile_weights_kernel<<<(unsigned)((total + 255) / 256), 256, 0, ctx->stream>>>((uint4*)dst, (const bf16_t*)src, N, K,
                                                                              dst_tile_off, NTA, bad);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}

static int dev_alloc(dsd_weights* w, size_t bytes, void** out) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes) != hipSuccess) DSD_FAIL(DSD_ENOMEM, "weight buffer of %zu bytes", bytes);
    w->allocs.push_back(p);
    *out = p;
    return DSD_OK;
}

int mfma_weights_tile(dsd_ctx* ctx, dsd_weights* w, const void* const* tensors) {
    const dsd_model_desc& D = w->desc;
    const int d = D.d_model, qd = D.n_q_heads * D.head_dim, kd = D.n_kv_heads * D.head_dim, F = D.d_ffn;
    int t = D.has_embed ? 1 : 0;
    int* bad = nullptr;                               // weights that fp16 cannot hold
    DSD_TRY(dev_alloc(w, 256, (void**)&bad));
    DSD_HIP(hipMemsetAsync(bad, 0, 4, ctx->stream));
    for (int l = 0; l < D.n_layers; ++l) {
        LayerW& L = w->layers[l];
        const void* const* T = tensors + t;
        t += 9;
        DSD_TRY(dev_alloc(w, (size_t)d * 2, &L.g1));
        DSD_HIP(hipMemcpyAsync(L.g1, T[0], (size_t)d * 2, hipMemcpyDeviceToDevice, ctx->stream));
        DSD_TRY(dev_alloc(w, (size_t)d * 2, &L.g2));
        DSD_HIP(hipMemcpyAsync(L.g2, T[5], (size_t)d * 2, hipMemcpyDeviceToDevice, ctx->stream));
        DSD_TRY(dev_alloc(w, (size_t)(qd + 2 * kd) * d * 2, &L.qkv_t));
        DSD_TRY(tile_into(ctx, bad, L.qkv_t, 0, (qd + 2 * kd) / 16, T[1], qd, d));
        DSD_TRY(tile_into(ctx, bad, L.qkv_t, qd / 16, (qd + 2 * kd) / 16, T[2], kd, d));
        DSD_TRY(tile_into(ctx, bad, L.qkv_t, (qd + kd) / 16, (qd + 2 * kd) / 16, T[3], kd, d));
        DSD_TRY(dev_alloc(w, (size_t)d * qd * 2, &L.wo_t));
        DSD_TRY(tile_into(ctx, bad, L.wo_t, 0, d / 16, T[4], d, qd));
        DSD_TRY(dev_alloc(w, (size_t)2 * F * d * 2, &L.gu_t));
        DSD_TRY(tile_into(ctx, bad, L.gu_t, 0, 2 * F / 16, T[6], F, d));
        DSD_TRY(tile_into(ctx, bad, L.gu_t, F / 16, 2 * F / 16, T[7], F, d));
        DSD_TRY(dev_alloc(w, (size_t)d * F * 2, &L.wd_t));
        DSD_TRY(tile_into(ctx, bad, L.wd_t, 0, d / 16, T[8], d, F));
    }
    if (D.has_head) {
        DSD_TRY(dev_alloc(w, (size_t)d * 2, &w->gf));
        DSD_HIP(hipMemcpyAsync(w->gf, tensors[t], (size_t)d * 2, hipMemcpyDeviceToDevice, ctx->stream));
        DSD_TRY(dev_alloc(w, (size_t)D.vocab * d * 2, &w->lm_t));
        DSD_TRY(tile_into(ctx, bad, w->lm_t, 0, D.vocab / 16, tensors[t + 1], D.vocab, d));
    }
    int n_bad = 0;
    DSD_HIP(hipMemcpyAsync(&n_bad, bad, 4, hipMemcpyDeviceToHost, ctx->stream));
    DSD_HIP(hipStreamSynchronize(ctx->stream));
    if (n_bad) DSD_FAIL(DSD_EUNSUPPORTED, "%d weight fragments hold values that are not finite or exceed 65504 in magnitude", n_bad);
    return DSD_OK;
}

// ============================================================================ skinny GEMM
template <int MT, int NT, int AMODE, int EPI, int NW>
__global__ void __launch_bounds__(NW * 64) gemm_skinny_kernel(GemmArgs p) {
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = NW;
    const int c = lane & 15, g = lane >> 4;
    int tile[NT];
    unit_tiles<NT, EPI>(p, blockIdx.x, tile);
    const int K = p.KS * 32;
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float ssq[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) ssq[mt] = 0.f;
    float worst = 0.f;                                // largest |activation| this thread turned into an operand

    const uint4* wt[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wt[nt] = p.Wt + (size_t)tile[nt] * 64 + lane;

    // One k-step per turn: a wave has only its own 1-2 KiB of weights and 2 KiB of activations in
    // flight, and it is the 8 waves per SIMD (35-85 registers) that keep the memory system busy.
    // Issuing the loads of four k-steps before the first use was measured slower (gate/up at 5 rows
    // 50.0 against 45.4 us): twice the registers, half the waves.
    for (int ks = wave; ks < p.KS; ks += nw) {
        f16x8 bfrag[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {             // weights are read once: non-temporal
            typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
            bfrag[nt] = __builtin_bit_cast(f16x8, __builtin_nontemporal_load((const u32x4_t*)(wt[nt] + (size_t)ks * p.NTA * 64)));
        }
        const int kb = ks * 32 + g * 8;
        f16x8 ahi[MT], alo[MT];
        float gf[8];
        if (AMODE == A_F32_GAIN) {
            const uint4 gu = *(const uint4*)(p.gain + kb);
            const unsigned gw[4] = {gu.x, gu.y, gu.z, gu.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                gf[2 * i] = __uint_as_float(gw[i] << 16);
                gf[2 * i + 1] = __uint_as_float(gw[i] & 0xFFFF0000u);
            }
        }
        const float* asrc = (AMODE == A_F32_GAIN) ? p.x : p.a;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int row = mt * 16 + c;
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (row < p.M) {
                const float4 v0 = *(const float4*)(asrc + (size_t)row * K + kb);
                const float4 v1 = *(const float4*)(asrc + (size_t)row * K + kb + 4);
                v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w;
                v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
            }
            if (AMODE == A_F32_GAIN) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    ssq[mt] += v[i] * v[i];
                    v[i] *= gf[i];
                }
            }
            worst = absmax8(v, worst);
            split8h(v, &ahi[mt], &alo[mt]);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[mt][nt] = mfma16h(ahi[mt], bfrag[nt], acc[mt][nt]);
                acc[mt][nt] = mfma16h(alo[mt], bfrag[nt], acc[mt][nt]);
            }
    }

    report_saturation(p.sat, worst);
    // partial tiles (and partial sums of squares) of all waves meet in LDS
    f32x4* red = (f32x4*)lds;                              // [nw][MT][NT][64]
    float* ssr = lds + (size_t)nw * MT * NT * 64 * 4;      // [nw][MT][16]
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) red[((wave * MT + mt) * NT + nt) * 64 + lane] = acc[mt][nt];
        if (AMODE == A_F32_GAIN) {
            float s = ssq[mt];
            s += __shfl_xor(s, 16, WAVE);
            s += __shfl_xor(s, 32, WAVE);
            if (lane < 16) ssr[(wave * MT + mt) * 16 + lane] = s;
        }
    }
    __syncthreads();

    for (int mt = wave; mt < MT; mt += nw) {
        f32x4 o[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            o[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
            for (int w = 0; w < nw; ++w) o[nt] += red[((w * MT + mt) * NT + nt) * 64 + lane];
        }
        float rstd[4] = {1.f, 1.f, 1.f, 1.f};
        if (AMODE == A_F32_GAIN) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = 0.f;
                for (int w = 0; w < nw; ++w) s += ssr[(w * MT + mt) * 16 + g * 4 + i];
                rstd[i] = 1.0f / sqrtf(s / (float)K + p.eps);
            }
        }
        gemm_epilogue<NT, EPI>(p, tile, o, rstd, mt, c, g);
    }
}

template <int MT, int NT, int AMODE, int EPI, int NW>
static int launch_gemm(hipStream_t s, const GemmArgs& p, int n_blocks) {
    const int nw = NW;
    const size_t lds = (size_t)nw * MT * NT * 64 * 16 + (size_t)nw * MT * 16 * 4;
    auto kern = gemm_skinny_kernel<MT, NT, AMODE, EPI, NW>;
    // once per instantiation and process: the limit is a property of the function, and setting it
    // again on every call would put a non-stream call into a caller's graph capture
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
        DSD_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    kern<<<n_blocks, nw * 64, lds, s>>>(p);
    return DSD_OK;
}

template <int NT, int AMODE, int EPI>
static int gemm_dispatch(hipStream_t s, const GemmArgs& p, int n_blocks, int n_cu) {
    const int mt = (p.M + 15) / 16;
    switch (mt) {
        case 1:
            // The waves of a workgroup split K.  As many of them as keep the whole grid resident at once
            // (32 waves per compute unit): every wave has one k-step of loads in flight, so it is the
            // number of resident waves that feeds the memory system, and a grid that does not fit runs
            // in rounds.  16 for the narrow matrices (QKV, O, down; down at d_model 8192 with 4 waves:
            // 147 us, with 16: 105), 4 for gate/up (8 was measured at d_model 4096: 47.0 against 45.3 us).
            {
                const long resident = 32L * n_cu;
                if ((long)n_blocks * 16 <= resident) return launch_gemm<1, NT, AMODE, EPI, 16>(s, p, n_blocks);
                return launch_gemm<1, NT, AMODE, EPI, 4>(s, p, n_blocks);
            }
        case 2: return launch_gemm<2, NT, AMODE, EPI, 16>(s, p, n_blocks);
        case 3: return launch_gemm<3, NT, AMODE, EPI, 8>(s, p, n_blocks);
        case 4: return launch_gemm<4, NT, AMODE, EPI, 8>(s, p, n_blocks);
        case 5: case 6: return launch_gemm<6, NT, AMODE, EPI, 4>(s, p, n_blocks);
        case 7: case 8: return launch_gemm<8, NT, AMODE, EPI, 4>(s, p, n_blocks);
        default: DSD_FAIL(DSD_EUNSUPPORTED, "bf16 path: B*k = %d rows exceed 128", p.M);
    }
}

// ============================================================================ attention
// A run of keys of one (sequence, kv head) is walked in steps of 32 keys by n_rg wavefronts at once,
// each holding RT tiles of 16 of the k*G query rows (a row group); the partial (max, sum, O) of every
// (run, row group) goes to scratch and attn_combine_kernel merges the runs.  K and V never pass
// through registers on their way in: each step (8 KiB of K, 8 KiB of V, already in MFMA operand order
// per lane) is fetched global -> LDS directly into one of two stages that the run's waves share,
// one step ahead of the arithmetic, every wave bringing its share of the step's 16 fragments; one
// workgroup barrier per step hands a stage over.  So K and V of a run come from memory once however
// many query rows there are, and small row groups mean several waves per SIMD, whose matrix, vector
// and LDS instructions overlap (one wave alone issues them one after the other).  The caches are
// stored in operand order, so a step is two contiguous 8 KiB pieces.  Stage layout: 16 fragments of
// 1 KiB (lane l at 16*l): K tile 0 features 0..31, 32..63, 64..95, 96..127, K tile 1 likewise, then V
// features 16h..16h+15.  A workgroup holds rpw runs: wave w = (run in the workgroup) * n_rg + row group.
#define ATT_STAGE_BYTES 16384

// this wave's share of the fragments of the step at key j0: fragment f for f = rg, rg + n_rg, ...
__device__ __forceinline__ void attn_fetch(const bf16_t* __restrict__ kbase, const bf16_t* __restrict__ vbase, int j0,
                                           size_t block_stride, unsigned stage, int lane, int rg, int n_rg) {
    const bf16_t* kt = kbase + (size_t)(j0 >> 5) * block_stride + lane * 8;   // two tiles of 16 keys, 4 fragments each
    const bf16_t* vb = vbase + (size_t)(j0 >> 5) * block_stride + lane * 8;
    for (int f = rg; f < 16; f += n_rg) {
        if (f < 8) gload16_lds_stream(stage + f * 1024, kt + f * 512);
        else gload16_lds_stream(stage + f * 1024, vb + (f - 8) * 512);
    }
}

template <int RT>
__global__ void __launch_bounds__(512, 2) attn_stream_kernel(AttnArgs p, int n_rg, int rpw) {
    extern __shared__ uint4 att_lds[];                // per run of the workgroup: 2 stages of ATT_STAGE_BYTES
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 15, g = lane >> 4;
    const int hk = blockIdx.y, b = blockIdx.z;
    const int rg = wave % n_rg, rloc = wave / n_rg;
    const int run = blockIdx.x * rpw + rloc;
    const int row0 = p.row_base + rg * RT * 16;
    const int L = p.len[b];
    const int nkeys = min(L + p.k, p.g.S);
    const int rows = p.k * p.G;
    const bool in_grid = run < p.n_runs;
    // Steps of 32 keys are dealt out to the runs in turn: run r takes steps r, r + n_runs, ...  The runs of a
    // (sequence, kv head) advance side by side, so what the chip reads at any moment is one contiguous piece
    // per head rather than a stream per run.  (The online softmax does not care which keys a run holds.)
    const int n_chunks = (nkeys + 31) >> 5;
    // every wave of the workgroup makes as many turns (one barrier each) as the workgroup's first run has steps
    const int run0 = blockIdx.x * rpw;
    const int n_steps = run0 < n_chunks ? (n_chunks - run0 + p.n_runs - 1) / p.n_runs : 0;
    const int my_steps = (in_grid && run < n_chunks) ? (n_chunks - run + p.n_runs - 1) / p.n_runs : 0;
    const size_t unit = ((size_t)(b * p.g.Hkv + hk) * p.n_runs + run) * p.rows_pad + row0;
    const bf16_t* kbase = p.kc + kv_block_off(p.g, b, hk, 0);
    const bf16_t* vbase = p.vc + kv_block_off(p.g, b, hk, 0);
    const size_t block_stride = (size_t)p.g.Bmax * p.g.Hkv * (32 * 128);      // from a block of 32 keys to the next
    const uint4* stage_ptr = att_lds + (size_t)rloc * (2 * ATT_STAGE_BYTES / 16);
    const unsigned stage_addr = (unsigned)(size_t)stage_ptr;      // low half of a flat LDS pointer = LDS address

    // The first step is requested before anything else: its way from memory overlaps the queries'.  (The
    // compiler counts only its own loads when it waits for a query; vector loads come back in order, so the
    // older stage fetches it does not know about can only make such a wait longer than needed.)
    if (my_steps > 0) attn_fetch(kbase, vbase, run * 32, block_stride, stage_addr, lane, rg, n_rg);
    bf16x8 qh[RT][4], ql[RT][4];
    uint64_t vis[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int r = row0 + rt * 16 + c;
        const int t = r / p.G, hq = hk * p.G + r % p.G;
        vis[rt] = 0;
        if (r < rows) vis[rt] = p.mask ? p.mask[t] : (t >= 63 ? ~0ull : ((1ull << (t + 1)) - 1ull));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (r < rows) {
                const float* src = p.q + ((size_t)(b * p.k + t) * p.Hq + hq) * 128 + j * 32 + g * 8;
                const float4 v0 = *(const float4*)src, v1 = *(const float4*)(src + 4);
                v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w;
                v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
            }
            // the queries carry the softmax scale and log2(e): scores come out of the matrix
            // instructions ready for exp2
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] *= p.scale_log2e;
            split8(v, &qh[rt][j], &ql[rt][j]);
        }
    }
    f32x4 o[8][RT];
#pragma unroll
    for (int h = 0; h < 8; ++h)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) o[h][rt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float mrow[RT], lrow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        mrow[rt] = -INFINITY;
        lrow[rt] = 0.f;
    }
    for (int step = 0; step < n_steps; ++step) {
        const int j0 = (step * p.n_runs + run) * 32, st = step & 1;
        vm_wait_all<0>();                             // this wave's share of the step has landed
        __syncthreads();                              // so has everybody's; and the other stage is read no more
        if (step + 1 < my_steps) attn_fetch(kbase, vbase, j0 + p.n_runs * 32, block_stride, stage_addr + (st ^ 1) * ATT_STAGE_BYTES, lane, rg, n_rg);
        if (step >= my_steps) continue;               // a shorter run of the same workgroup: barriers only
        const uint4* sp = stage_ptr + st * (ATT_STAGE_BYTES / 16) + lane;
        f32x4 s[2][RT];
#pragma unroll
        for (int tl = 0; tl < 2; ++tl) {
            bf16x8 kf[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) kf[j] = __builtin_bit_cast(bf16x8, sp[(tl * 4 + j) * 64]);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    a = mfma16(kf[j], qh[rt][j], a);
                    a = mfma16(kf[j], ql[rt][j], a);
                }
                s[tl][rt] = a;
            }
        }
        bf16x8 vf[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) vf[h] = __builtin_bit_cast(bf16x8, sp[(8 + h) * 64]);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            float mx = -INFINITY;
            if (j0 + 32 <= L) {
                // a step of committed keys only (all but the last one or two of a run): every key is
                // visible to every row, no mask arithmetic
#pragma unroll
                for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[tl][rt][i]);
            } else {
#pragma unroll
                for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int key = j0 + tl * 16 + g * 4 + i;
                        bool ok = key < L;
                        if (!ok && key < nkeys) ok = (vis[rt] >> (key - L)) & 1ull;
                        const float v = ok ? s[tl][rt][i] : -INFINITY;
                        s[tl][rt][i] = v;
                        mx = fmaxf(mx, v);
                    }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, WAVE));
            mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
            // The reference exponent of a row moves only when a score exceeds it by more than 2^8 (any
            // reference gives the same softmax as long as nothing overflows; weights up to 256 are far
            // from that), so after a row's first few steps the rescaling of its sums and outputs is
            // skipped: one uniform branch instead of 34 multiplications.
            if (__builtin_amdgcn_ballot_w64(mx > mrow[rt] + 8.0f) != 0) {
                const float mnew = fmaxf(mrow[rt], mx);
                const float alpha = __builtin_amdgcn_exp2f(mrow[rt] - ((mnew == -INFINITY) ? 0.f : mnew));   // 0 when mrow was -inf
                mrow[rt] = mnew;
                lrow[rt] *= alpha;
#pragma unroll
                for (int h = 0; h < 8; ++h) o[h][rt] *= alpha;
            }
            const float muse = (mrow[rt] == -INFINITY) ? 0.f : mrow[rt];
            float pv[8];
            float ps = 0.f;
#pragma unroll
            for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // the bare instruction: results below 2^-126 become 0, which is what a weight that small is
                    const float e = __builtin_amdgcn_exp2f(s[tl][rt][i] - muse);
                    pv[tl * 4 + i] = e;
                    ps += e;
                }
            lrow[rt] += ps;
            bf16x8 ph, pl;
            split8(pv, &ph, &pl);
#pragma unroll
            for (int h = 0; h < 8; ++h) {
                o[h][rt] = mfma16(vf[h], ph, o[h][rt]);
                o[h][rt] = mfma16(vf[h], pl, o[h][rt]);
            }
        }
    }
    if (!in_grid) return;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float l = lrow[rt];
        l += __shfl_xor(l, 16, WAVE);
        l += __shfl_xor(l, 32, WAVE);
        const int r = rt * 16 + c;
        if (g == 0) {
            p.part_ml[(unit + r) * 2] = mrow[rt];
            p.part_ml[(unit + r) * 2 + 1] = l;
        }
        // the run's output goes out normalised (a weighted mean of value rows: bounded by the values
        // themselves) and as fp16; (max, sum) stay fp32 and carry the run's weight
        const float inv_l = l > 0.f ? 1.0f / l : 0.f;
        unsigned short* po = (unsigned short*)p.part_o + (unit + r) * 128 + g * 4;
        float worst = 0.f;
#pragma unroll
        for (int h = 0; h < 8; ++h) {
            const f32x4 v = o[h][rt] * inv_l;
            worst = fmaxf(fmaxf(worst, fmaxf(fabsf(v[0]), fabsf(v[1]))), fmaxf(fabsf(v[2]), fabsf(v[3])));
            *(uint2*)(po + h * 16) = make_uint2(pack_f16(v[0], v[1]), pack_f16(v[2], v[3]));
        }
        report_saturation(p.sat, worst);
    }
}

template <int RT>
static int attn_launch(hipStream_t s, const AttnArgs& t, int n_rg, int rpw, int Hkv, int B) {
    const size_t lds = (size_t)rpw * 2 * ATT_STAGE_BYTES;
    auto kern = attn_stream_kernel<RT>;
    // once per instantiation and process: the limit is a property of the function, and setting it
    // again on every call would put a non-stream call into a caller's graph capture
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
        DSD_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    const int n_wg = (t.n_runs + rpw - 1) / rpw;
    kern<<<dim3(n_wg, Hkv, B), n_rg * rpw * 64, lds, s>>>(t, n_rg, rpw);
    return DSD_OK;
}

__global__ void __launch_bounds__(128) attn_combine_kernel(float* __restrict__ out, const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml, int n_runs, int rows_pad,
                                                          int k, int G, int Hq, int Hkv,
                                                          unsigned short* __restrict__ panel, int panel_mt, int* __restrict__ sat) {
    __shared__ float wgt[MAX_RUNS];
    __shared__ float red[4];
    attn_combine_row<true>(out, part_o, part_ml, n_runs, rows_pad, k, G, Hq, Hkv, blockIdx.x, blockIdx.y, blockIdx.z, wgt,
                           red, panel, panel_mt, sat);
}

// ============================================================================ small kernels
// (cos, sin) of every row's 64 rotation angles, once per call: the angles are the same in every layer
// and for every head, and working them out in fp64 (pow + sincos) inside a GEMM epilogue kept one
// wave of every workgroup busy for microseconds after its last weight had arrived.  64 threads per row.
struct RopeArgs {
    float2* rope;            // [M][64]
    const int32_t* len;
    const int32_t* depth;    // NULL = chain
    int k, M;
    float theta;
};
__device__ __forceinline__ void rope_rows(const RopeArgs& r, int m, int e) {
    if (m >= r.M) return;
    const int b = m / r.k, t = m % r.k;
    const double pos = (double)(r.len[b] + (r.depth ? r.depth[t] : t));
    const double inv = pow((double)r.theta, -2.0 * (double)e / 128.0);
    double sn, cs;
    sincos(pos * inv, &sn, &cs);
    r.rope[m * 64 + e] = make_float2((float)cs, (float)sn);
}
__global__ void __launch_bounds__(64) rope_table_kernel(RopeArgs r) { rope_rows(r, blockIdx.x, threadIdx.x); }
void rope_table_launch(dsd_ctx* ctx, float2* rope, const int32_t* len, const int32_t* depth, int M, int k, float theta) {
    const RopeArgs r = {rope, len, depth, k, M, theta};
    rope_table_kernel<<<M, 64, 0, ctx->stream>>>(r);
}

// The call's first launch: the input rows into the fp32 residual stream (blocks below n_row_blocks) and
// the rotation table (the blocks after them, 4 rows each).
__global__ void __launch_bounds__(256) rows_in_kernel(float* __restrict__ x, const bf16_t* __restrict__ h, size_t n,
                                                      int n_row_blocks, RopeArgs r) {
    if ((int)blockIdx.x >= n_row_blocks) {
        rope_rows(r, ((int)blockIdx.x - n_row_blocks) * 4 + (threadIdx.x >> 6), threadIdx.x & 63);
        return;
    }
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) x[i] = bf16_to_f32(h[i]);
}
// first node of the pipeline: x[m,:] = E[token[m],:]  (ids clamped into the table); blocks M .. do the table
__global__ void __launch_bounds__(256) embed_rows_kernel(float* __restrict__ x, const bf16_t* __restrict__ embed,
                                                         const int32_t* __restrict__ tokens, int d, int vocab, RopeArgs r) {
    const int m = blockIdx.x;
    if (m >= r.M) {
        rope_rows(r, (m - r.M) * 4 + (threadIdx.x >> 6), threadIdx.x & 63);
        return;
    }
    int t = tokens[m];
    t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)m * d + i] = bf16_to_f32(embed[(size_t)t * d + i]);
}

// ============================================================================ orchestration
int mfma_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                      const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth, int B, int k,
                      void* hidden_out, float* logits, int64_t logits_seq_stride) {
    const dsd_model_desc& D = w->desc;
    const KvGeom& g = kv->geom;
    const int M = B * k, d = D.d_model, Hq = D.n_q_heads, Hkv = D.n_kv_heads, hd = D.head_dim, F = D.d_ffn;
    const int G = Hq / Hkv, qd = Hq * hd;
    if (M > 128) {
        // More rows than the GEMM tiles take.  Sequences are independent (own cache rows, own
        // positions), so they go through in groups of up to 128 rows; every group streams the
        // weights once more, which at this many rows per weight byte is no longer the only cost.
        const int per = 128 / k;
        const size_t seq_cache_bytes = (size_t)g.Hkv * 32 * g.hd * sizeof(bf16_t);     // a sequence's share of a block of 32 slots
        const int64_t lstride = logits_seq_stride ? logits_seq_stride : (int64_t)k * D.vocab;
        for (int b0 = 0; b0 < B; b0 += per) {
            const int nb = std::min(per, B - b0);
            dsd_kv view;
            view.desc = kv->desc;
            view.geom = kv->geom;
            view.k = (char*)kv->k + b0 * seq_cache_bytes;
            view.v = (char*)kv->v + b0 * seq_cache_bytes;
            view.len_dev = kv->len_dev + b0;
            view.len_bound.assign(kv->len_bound.begin() + b0, kv->len_bound.begin() + b0 + nb);
            view.last_k = kv->last_k;
            view.cap = kv->cap;
            const size_t row0 = (size_t)b0 * k;
            DSD_TRY(mfma_stage_verify(ctx, w, &view, hidden_in ? (const bf16_t*)hidden_in + row0 * d : nullptr,
                                      draft_tokens ? draft_tokens + row0 : nullptr, tree_mask, depth, nb, k,
                                      hidden_out ? (bf16_t*)hidden_out + row0 * d : nullptr,
                                      logits ? logits + b0 * lstride : nullptr, logits_seq_stride));
        }
        return DSD_OK;
    }
    if (!hidden_in && (!D.has_embed || !draft_tokens))
        DSD_FAIL(DSD_EINVAL, "bf16 path: neither hidden_in nor (embedding table, draft_tokens)");
    const int rows = k * G;
    const int n_rt = (rows + 15) / 16;       // 16-row tiles of query rows per kv head
    if (n_rt > 32) DSD_FAIL(DSD_EUNSUPPORTED, "bf16 path: k*G = %d query rows per kv head exceed 512", rows);
    // Row tiles per wave: one, so that a run's query rows spread over as many waves as possible (several waves
    // per SIMD, the run's K/V staged once for all of them); up to 8 waves share a run.  Measured against two
    // tiles per wave, attention per layer: 31.5 against 34.4 us (32-node tree, 128 rows per kv head), 54.5
    // against 63.4 (batch 16, k = 8), 9.5 against 11.3 (batch 1, k = 5), 64.8 against 65.7 (70B shape, k = 6).
    // Beyond 8 tiles (128 rows per kv head) two tiles per wave; beyond 16 the rows go through in groups of 16
    // tiles, one launch each (each streams K/V again: such windows, k*G > 256, are rare).
    const int tiles_per_launch = std::min(n_rt, 16);
    const int RT = tiles_per_launch > 8 ? 2 : 1;
    const int n_rg = (tiles_per_launch + RT - 1) / RT;
    // Which GEMM path.  The panel path (dsd_gemm_tiled.hip) at every row count for every shape it takes; one
    // workgroup per column tile converting the activations itself (gemm_skinny_kernel) for the others, and
    // with DSD_NO_TILED for tests.  Measured at d_model 4096, ms per step of 8 layers, panel path against
    // the other: 0.795 / 0.838 at 4 rows, 0.795 / 0.837 at 5; the other path's 1 to 3 rows take 0.817 to 0.829,
    // more than the panel path's 4.  (Before the weights were read with non-temporal loads the other kernel
    // won up to 3 rows, where d_model / 16 = 256 tiles are exactly one workgroup per compute unit.)  Wider
    // models were always faster on the panel path: per layer at 5 rows 136.9 against 149.0 us (d_model 5120),
    // 166.8 against 182.4 (6144), 333.7 against 353.2 (8192).
    const bool tiled = tiled_supported(&D) && !ctx->no_tiled;
    // The LM head takes the panel path at every row count: a vocabulary is a gigabyte of weights, and 256-column
    // workgroups stream it faster than one workgroup per 16 columns (207 against 228 us at 5 rows, V = 128256).
    const bool tiled_head = logits && tiled_supported(&D) && !ctx->no_tiled;

    int max_len = 0;
    for (int b = 0; b < B; ++b) max_len = std::max(max_len, kv->len_bound[b]);
    const int max_keys = std::min(max_len + k, g.S);
    // Runs of keys.  A workgroup is one run (its n_rg waves; two runs in a workgroup share its barrier and were
    // measured 13 % slower), as many workgroups per compute unit as give at most 8 waves there, and a number of
    // runs per (sequence, head) that makes the grid whole rounds of that: 8 runs at B = 16 (1024 workgroups of 2
    // waves), at the 70B shape with B = 8 (512 of 3) and for a 32-node tree at B = 4 (256 of 8) -- with 6, 10 or 12
    // runs each of the three is 5-25 % slower.  Small problems take shorter runs, of at least 64 keys.
    const long units = (long)B * Hkv;
    const long wg_per_cu = std::max(1, 8 / n_rg);
    long runs_wanted = std::max(1L, wg_per_cu * ctx->n_cu / units);
    int n_runs = (int)std::min(runs_wanted, (long)std::max(1, max_keys / 64));
    const int rpw = 1;
    if (n_runs > MAX_RUNS) DSD_FAIL(DSD_EUNSUPPORTED, "bf16 path: %d key runs", n_runs);
    const int rows_pad = (n_rt + RT - 1) / RT * RT * 16;      // whole row groups

    const int n_qkv = (Hq + 2 * Hkv) * hd;
    const size_t kmax = (size_t)std::max(std::max(d, qd), F);
    // tiled path: K slices of one GEMM's result (up to TILED_MAX_KSPLIT of them), and per-chunk sums of squares
    const size_t n_part = tiled ? (size_t)TILED_MAX_KSPLIT * M * std::max(d, n_qkv) : 0;
    const size_t n_ssq = (size_t)128 * (d / 128 + 1);
    // the workspace is carved twice with the same code: once to add up the sizes, once for the pointers
    float *x, *q, *att, *h, *part_o, *part_ml, *part, *ssq;
    float2* rope;
    void* panel;
    auto carve = [&](WsBump& ws) {
        x = ws.take<float>((size_t)M * d);
        q = ws.take<float>((size_t)M * qd);
        att = ws.take<float>(tiled ? 0 : (size_t)M * qd);          // on the tiled path the combine writes the O panel
        // on the tiled path: the down projection's panel, 16 * row tiles rows of fp16
        h = ws.take<float>(tiled ? std::max((size_t)M * F, (size_t)8 * tiled_row_tiles(M) * F) : (size_t)M * F);
        part_o = ws.take<float>((size_t)units * n_runs * rows_pad * 64);     // fp16 [unit][run][row][128]
        part_ml = ws.take<float>((size_t)units * n_runs * rows_pad * 2);
        rope = ws.take<float2>((size_t)M * 64);
        part = ws.take<float>(n_part);
        ssq = ws.take<float>(n_ssq);                               // [d/128][128]: sums of squares of the rows, per chunk of 128 columns
        panel = ws.take<float>(tiled || tiled_head ? 64 * kmax : 0);             // up to 128 rows of activations as fp16 in A-operand order
    };
    WsBump sizing{nullptr, 0};
    carve(sizing);
    DSD_TRY(dsd_ws_reserve(ctx, sizing.off));
    WsBump ws{ctx->ws, 0};
    carve(ws);
    void* panel_h = h;                                // SiLU*up goes straight into the operand panel of the down projection
    hipStream_t s = ctx->stream;
    int x_pending = 0;                                // K slices in `part` that the residual stream has not taken yet
    const size_t nx = (size_t)M * d;
    {
        ProfScope ps(ctx, DSD_KC_OTHER);
        const RopeArgs ra = {rope, kv->len_dev, depth, k, M, D.rope_theta};
        const int n_row_blocks = (int)((nx + 255) / 256), n_rope_blocks = (M + 3) / 4;
        if (hidden_in)
            rows_in_kernel<<<n_row_blocks + n_rope_blocks, 256, 0, s>>>(x, (const bf16_t*)hidden_in, nx, n_row_blocks, ra);
        else
            embed_rows_kernel<<<M + n_rope_blocks, 256, 0, s>>>(x, (const bf16_t*)w->embed, draft_tokens, d, D.vocab, ra);
    }

    for (int l = 0; l < D.n_layers; ++l) {
        const LayerW& W = w->layers[l];
        bf16_t* kc = (bf16_t*)kv->k + (size_t)l * g.layer_elems;
        bf16_t* vc = (bf16_t*)kv->v + (size_t)l * g.layer_elems;
        GemmArgs a = GemmArgs();
        a.sat = ctx->sat_dev;
        a.M = M;
        a.eps = D.rms_eps;
        // q, k, v = rmsnorm(x; g1) Wqkv^T, rotary, cache append
        a.Wt = (const uint4*)W.qkv_t; a.NTA = n_qkv / 16; a.KS = d / 32; a.x = x; a.gain = (const bf16_t*)W.g1;
        a.q = q; a.kc = kc; a.vc = vc; a.g = g; a.len = kv->len_dev; a.k = k; a.Hq = Hq;
        a.rope = rope;
        {
            ProfScope ps(ctx, DSD_KC_QKV);
            if (tiled) {
                DSD_TRY(tiled_gemm_qkv(ctx, W.qkv_t, x, (const bf16_t*)W.g1, part, x_pending, M, n_qkv, d, q, kc, vc, g,
                                       kv->len_dev, k, Hq, D.rms_eps, rope, panel, ssq));
                x_pending = 0;
            } else
                DSD_TRY((gemm_dispatch<2, A_F32_GAIN, EPI_QKV>(s, a, (Hq + 2 * Hkv) * 4, ctx->n_cu)));
        }
        // attention
        AttnArgs t;
        t.q = q; t.kc = kc; t.vc = vc; t.g = g; t.len = kv->len_dev; t.mask = tree_mask; t.k = k; t.Hq = Hq; t.G = G;
        t.n_runs = n_runs; t.part_o = part_o; t.part_ml = part_ml;
        t.sat = ctx->sat_dev; t.rows_pad = rows_pad; t.scale_log2e = 1.4426950408889634f / sqrtf((float)hd);
        {
            ProfScope ps(ctx, DSD_KC_ATTN);
            for (int tile0 = 0; tile0 < n_rt; tile0 += tiles_per_launch) {
                t.row_base = tile0 * 16;
                const int rg_here = (std::min(tiles_per_launch, n_rt - tile0) + RT - 1) / RT;
                if (RT == 1) DSD_TRY(attn_launch<1>(s, t, rg_here, rpw, Hkv, B));
                else DSD_TRY(attn_launch<2>(s, t, rg_here, rpw, Hkv, B));
            }
        }
        {
        ProfScope ps(ctx, DSD_KC_ATTN_COMBINE);
        // tiled path: straight into the operand panel of the output projection
        attn_combine_kernel<<<dim3(rows, Hkv, B), 128, 0, s>>>(att, part_o, part_ml, n_runs, t.rows_pad, k, G, Hq, Hkv,
                                                               tiled ? (unsigned short*)panel : nullptr,
                                                               tiled ? tiled_row_tiles(M) : 0, ctx->sat_dev);
        }
        // x += attn Wo^T
        a = GemmArgs();
        a.sat = ctx->sat_dev;
        a.M = M; a.Wt = (const uint4*)W.wo_t; a.NTA = d / 16; a.KS = qd / 32; a.a = att; a.xout = x; a.N = d;
        {
            ProfScope ps(ctx, DSD_KC_OPROJ);
            if (tiled) DSD_TRY(tiled_gemm_resid(ctx, W.wo_t, part, &x_pending, M, d, qd, panel));
            else DSD_TRY((gemm_dispatch<1, A_F32, EPI_RESID>(s, a, d / 16, ctx->n_cu)));
        }
        // h = silu(b Wg^T) * (b Wu^T),  b = rmsnorm(x; g2)
        a = GemmArgs();
        a.sat = ctx->sat_dev;
        a.M = M; a.eps = D.rms_eps; a.Wt = (const uint4*)W.gu_t; a.NTA = 2 * F / 16; a.KS = d / 32; a.x = x; a.gain = (const bf16_t*)W.g2;
        a.hout = h; a.N = F; a.up_tile_off = F / 16;
        {
            ProfScope ps(ctx, DSD_KC_GATEUP);
            if (tiled) {
                DSD_TRY(tiled_gemm_swiglu(ctx, W.gu_t, x, (const bf16_t*)W.g2, part, x_pending, panel_h, M, F, d, D.rms_eps,
                                          panel, ssq));
                x_pending = 0;
            } else DSD_TRY((gemm_dispatch<2, A_F32_GAIN, EPI_SWIGLU>(s, a, F / 16, ctx->n_cu)));
        }
        // x += h Wd^T
        a = GemmArgs();
        a.sat = ctx->sat_dev;
        a.M = M; a.Wt = (const uint4*)W.wd_t; a.NTA = d / 16; a.KS = F / 32; a.a = h; a.xout = x; a.N = d;
        if (l == D.n_layers - 1) a.hidden_out = (bf16_t*)hidden_out;     // the block's output leaves with the last residual update
        {
            ProfScope ps(ctx, DSD_KC_DOWN);
            if (tiled) DSD_TRY(tiled_gemm_resid(ctx, W.wd_t, part, &x_pending, M, d, F, panel_h));
            else DSD_TRY((gemm_dispatch<1, A_F32, EPI_RESID>(s, a, d / 16, ctx->n_cu)));
        }
    }
    // the block's output rows: off the panel path the last down projection's epilogue has written them; on the
    // panel path they leave with the sum of that projection's K slices
    if (hidden_out && tiled) {
        ProfScope ps(ctx, DSD_KC_OTHER);
        DSD_TRY(tiled_resid_reduce(ctx, x, part, x_pending, M, d, hidden_out));
        x_pending = 0;
    }
    if (logits) {
        GemmArgs a = GemmArgs();
        a.sat = ctx->sat_dev;
        a.M = M; a.eps = D.rms_eps; a.Wt = (const uint4*)w->lm_t; a.NTA = D.vocab / 16; a.KS = d / 32; a.x = x; a.gain = (const bf16_t*)w->gf;
        a.logits = logits; a.N = D.vocab; a.rows_per_seq = k; a.seq_stride = logits_seq_stride;
        ProfScope ps(ctx, DSD_KC_HEAD);
        if (tiled_head)
            DSD_TRY(tiled_gemm_logits(ctx, w->lm_t, x, (const bf16_t*)w->gf, part, x_pending, logits, M, D.vocab, d,
                                      D.rms_eps, k, logits_seq_stride, panel, ssq));
        else
            DSD_TRY((gemm_dispatch<1, A_F32_GAIN, EPI_LOGITS>(s, a, D.vocab / 16, ctx->n_cu)));
    }
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}
