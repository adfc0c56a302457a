// Weight-streaming GEMM for 17..128 rows (B*k of the batched verification pass, section 2.1).
//
// With this many rows the pass is still bound by streaming the weights once, but the activation
// operand is no longer negligible: every weight fragment meets 2*MT activation fragments (hi + lo
// bf16 of MT 16-row tiles).  So the activations are shared through LDS and only the weights come
// straight from HBM into registers:
//   * a workgroup of 4 waves owns 128 output columns (each wave two 16-column tiles) over one
//     contiguous slice of K (grid.y splits K when a matrix has too few column blocks to fill the
//     chip; partial results are then added atomically into an fp32 buffer);
//   * the slice is walked in chunks of 128 columns of K: the 256 threads convert the chunk of the
//     activation rows (gain, hi/lo split) into an LDS panel laid out in A-operand order, double
//     buffered, one chunk ahead;
//   * every wave keeps its next 32 weight fragments in flight in a register FIFO, issued by hand
//     (inline asm + explicit s_waitcnt counts, see gload16 / vm_wait) so that neither the panel
//     prefetch nor the workgroup barriers ever drain the weight stream.
#include "dsd_bf16_dev.h"

#define TW 4
#define TCH 128          // K per panel chunk: 4 k-steps
#define TFIFO 32         // fragments in flight per wave: 16 k-steps x 2 tiles

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void gload16(u32x4& dst, const void* ptr) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(ptr));
}
// count = loads of ours issued after the one needed (vector memory returns in order; a smaller
// count than the true number only waits longer)
template <int N>
__device__ __forceinline__ void vm_wait(u32x4& r) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N));
}
// The same pair for values parked in accumulation registers (the panel prefetch: it is only
// looked at after its wait, and the arch VGPRs are needed for the weight FIFO).  The compiler must
// never have a reason to copy a register whose load is still in flight, so register pressure is
// kept away from these values rather than left to the allocator.
__device__ __forceinline__ void gload16_acc(u32x4& dst, const void* ptr) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(dst) : "v"(ptr));
}
template <int N>
__device__ __forceinline__ void vm_wait_acc(u32x4& r) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+a"(r) : "n"(N));
}

enum { TE_ATOMIC = 0, TE_SWIGLU = 1, TE_LOGITS = 2 };

struct TArgs {
    const uint4* Wt;     // tiled weights
    int KS;              // K / 32
    int ks_per_split;    // k-steps per workgroup, multiple of 16
    int M;
    const float* a;      // [M][K] fp32 activations
    const bf16_t* gain;  // [K] RMSNorm gain applied to the activations, or NULL
    float eps;
    float* out;          // TE_ATOMIC: [M][N] fp32, += ;  TE_SWIGLU: h [M][N];  TE_LOGITS: logits
    int N;
    int up_tile_off;     // TE_SWIGLU: F/16
    int rows_per_seq;    // TE_LOGITS
    int64_t seq_stride;
};

template <int MT>
__device__ __forceinline__ void tpanel_load(u32x4 (&P)[2 * MT], u32x4& G, const TArgs& p, int K, int k0) {
    // thread t: k-group q8 = t%16 (8 values) of rows t/16 + 16*i
    const int q8 = threadIdx.x & 15, r0 = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        int r = r0 + 16 * i;
        r = r < p.M ? r : p.M - 1;                 // a fixed number of loads; rows >= M are never stored
        const float* src = p.a + (size_t)r * K + k0 + q8 * 8;
        gload16_acc(P[2 * i], src);
        gload16_acc(P[2 * i + 1], src + 4);
    }
    gload16_acc(G, p.gain ? (const void*)(p.gain + k0 + q8 * 8) : (const void*)(p.a + k0 + q8 * 8));
}

// YOUNGER: loads of ours issued after the panel loads
template <int MT, int YOUNGER>
__device__ __forceinline__ void tpanel_store(u32x4 (&P)[2 * MT], u32x4& G, const TArgs& p, uint4* __restrict__ buf,
                                             float (&ssq)[MT]) {
    vm_wait_acc<YOUNGER>(G);
#pragma unroll
    for (int r = 0; r < 2 * MT; ++r) asm volatile("" : "+a"(P[r]));
    float gf[8];
    if (p.gain) unpack_gain(make_uint4(G.x, G.y, G.z, G.w), gf);
    const int q8 = threadIdx.x & 15, c = threadIdx.x >> 4;      // row r0 + 16 i = tile i, row-in-tile c
    const int ks = q8 >> 2, g = q8 & 3;
    // planes: hi at [0], lo at [4*MT*64]; entry (ks*MT + mt)*64 + g*16 + c
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = __uint_as_float(P[2 * i][j]);
            v[4 + j] = __uint_as_float(P[2 * i + 1][j]);
        }
        if (p.gain) {
            float q = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                q += v[j] * v[j];
                v[j] *= gf[j];
            }
            ssq[i] += q;
        }
        bf16x8 hi, lo;
        split8(v, &hi, &lo);
        const int e = (ks * MT + i) * 64 + g * 16 + c;
        buf[e] = __builtin_bit_cast(uint4, hi);
        buf[4 * MT * 64 + e] = __builtin_bit_cast(uint4, lo);
    }
}

// one chunk (4 k-steps) against FIFO slots S0 .. S0+7
template <int MT, int S0>
__device__ __forceinline__ void tconsume(u32x4 (&fifo)[TFIFO], const uint4* __restrict__ panel, f32x4 (&acc)[MT][2],
                                         const uint4*& w0, const uint4*& w1, int& left, int lane) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 ahi[MT], alo[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            ahi[mt] = __builtin_bit_cast(bf16x8, panel[(ks * MT + mt) * 64 + lane]);
            alo[mt] = __builtin_bit_cast(bf16x8, panel[4 * MT * 64 + (ks * MT + mt) * 64 + lane]);
        }
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int slot = S0 + ks * 2 + nt;
            vm_wait<TFIFO - 1>(fifo[slot]);
            const bf16x8 b = __builtin_bit_cast(bf16x8, fifo[slot]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[mt][nt] = mfma16(ahi[mt], b, acc[mt][nt]);
                acc[mt][nt] = mfma16(alo[mt], b, acc[mt][nt]);
            }
            // refill 16 k-steps ahead; past the end of the slice keep re-reading the last fragment
            const uint4* src = nt ? w1 : w0;
            gload16(fifo[slot], src);
            if (nt) {
                if (left > 0) {
                    w0 += 64;
                    w1 += 64;
                }
                --left;
            }
        }
    }
}

template <int MT, int EPI>
__global__ void __launch_bounds__(TW * 64) gemm_tiled_kernel(TArgs p) {
    extern __shared__ uint4 lds[];                    // 2 panel buffers of 2 * 4*MT*64 uint4
    __shared__ float lds_ssq[MT * 16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int K = p.KS * 32;
    const int ks0 = blockIdx.y * p.ks_per_split;
    const int nchunk = p.ks_per_split / 4;
    int tile0, tile1;
    if (EPI == TE_SWIGLU) {                           // gate tile and its up tile
        tile0 = blockIdx.x * TW + wave;
        tile1 = tile0 + p.up_tile_off;
    } else {
        tile0 = blockIdx.x * (2 * TW) + wave * 2;
        tile1 = tile0 + 1;
    }
    const int n_tiles = (EPI == TE_SWIGLU) ? p.up_tile_off : p.N / 16;
    const bool live0 = tile0 < n_tiles, live1 = (EPI == TE_SWIGLU) ? live0 : tile1 < n_tiles;
    // dead tiles (ragged last column block) stream a valid tile and are not stored
    const uint4* w0 = p.Wt + ((size_t)(live0 ? tile0 : 0) * p.KS + ks0) * 64 + lane;
    const uint4* w1 = p.Wt + ((size_t)(live1 ? tile1 : 0) * p.KS + ks0) * 64 + lane;

    u32x4 fifo[TFIFO];
    int left = p.ks_per_split - 1;                    // k-steps the stream may still advance
#pragma unroll
    for (int i = 0; i < TFIFO / 2; ++i) {
        gload16(fifo[2 * i], w0);
        gload16(fifo[2 * i + 1], w1);
        if (left > 0) {
            w0 += 64;
            w1 += 64;
        }
        --left;
    }
    f32x4 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt][0] = acc[mt][1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float ssq[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) ssq[i] = 0.f;

    const size_t pbuf = (size_t)2 * 4 * MT * 64;
    u32x4 P[2 * MT], G;
    tpanel_load<MT>(P, G, p, K, ks0 * 32);
    tpanel_store<MT, 0>(P, G, p, lds, ssq);
    __syncthreads();
    for (int ch = 0; ch < nchunk; ch += 4) {          // 4 chunks = 16 k-steps = one turn of the FIFO
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool more = ch + q + 1 < nchunk;
            if (more) tpanel_load<MT>(P, G, p, K, (ks0 + (ch + q + 1) * 4) * 32);
            const uint4* panel = lds + ((ch + q) & 1) * pbuf;
            switch (q) {
                case 0: tconsume<MT, 0>(fifo, panel, acc, w0, w1, left, lane); break;
                case 1: tconsume<MT, 8>(fifo, panel, acc, w0, w1, left, lane); break;
                case 2: tconsume<MT, 16>(fifo, panel, acc, w0, w1, left, lane); break;
                default: tconsume<MT, 24>(fifo, panel, acc, w0, w1, left, lane); break;
            }
            if (more) tpanel_store<MT, 8>(P, G, p, lds + (((ch + q) & 1) ^ 1) * pbuf, ssq);
            __syncthreads();
        }
    }
    // drain what is still in flight before the registers die
    vm_wait<0>(fifo[0]);

    float rstd[MT][4];
    if (EPI != TE_ATOMIC && p.gain) {
        // thread t summed k-groups t%16 of rows t/16 + 16*i: reduce over the 16 threads of a row
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            float q = ssq[i];
            q += __shfl_xor(q, 1, WAVE);
            q += __shfl_xor(q, 2, WAVE);
            q += __shfl_xor(q, 4, WAVE);
            q += __shfl_xor(q, 8, WAVE);
            if ((threadIdx.x & 15) == 0) lds_ssq[i * 16 + (threadIdx.x >> 4)] = q;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) rstd[mt][i] = 1.0f / sqrtf(lds_ssq[mt * 16 + g * 4 + i] / (float)K + p.eps);
    } else {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) rstd[mt][i] = 1.f;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + g * 4 + i;
            if (m >= p.M) continue;
            if (EPI == TE_ATOMIC) {
                if (live0) unsafeAtomicAdd(p.out + (size_t)m * p.N + tile0 * 16 + c, acc[mt][0][i]);
                if (live1) unsafeAtomicAdd(p.out + (size_t)m * p.N + tile1 * 16 + c, acc[mt][1][i]);
            } else if (EPI == TE_SWIGLU) {
                if (live0) {
                    const float gate = acc[mt][0][i] * rstd[mt][i], up = acc[mt][1][i] * rstd[mt][i];
                    p.out[(size_t)m * p.N + tile0 * 16 + c] = gate / (1.0f + __expf(-gate)) * up;
                }
            } else {
                float* row = p.out + (size_t)(m / p.rows_per_seq) * p.seq_stride + (size_t)(m % p.rows_per_seq) * p.N;
                if (live0) row[tile0 * 16 + c] = acc[mt][0][i] * rstd[mt][i];
                if (live1) row[tile1 * 16 + c] = acc[mt][1][i] * rstd[mt][i];
            }
        }
}

// q, k, v rows accumulated by the split-K QKV GEMM -> RMSNorm scale, rotary embedding, cache append.
// One block per row; the accumulator row is cleared for the next layer.
__global__ void __launch_bounds__(256) qkv_finish_kernel(float* __restrict__ acc, const float* __restrict__ x,
                                                         float* __restrict__ q, bf16_t* __restrict__ kc,
                                                         bf16_t* __restrict__ vc, KvGeom g,
                                                         const int32_t* __restrict__ len,
                                                         const int32_t* __restrict__ depth, int k, int Hq, int d,
                                                         float eps, float theta) {
    __shared__ float red[4];
    const int m = blockIdx.x, b = m / k, t = m % k;
    float s = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
        const float v = x[(size_t)m * d + i];
        s += v * v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, WAVE);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    const int L = len[b];
    const int slot = L + t;
    const double pos = (double)(L + (depth ? depth[t] : t));
    const int heads = Hq + 2 * g.Hkv;
    float* row = acc + (size_t)m * heads * 128;
    for (int i = threadIdx.x; i < heads * 64; i += 256) {
        const int head = i >> 6, e = i & 63;
        const float lo = row[head * 128 + e] * rstd, hi = row[head * 128 + e + 64] * rstd;
        row[head * 128 + e] = 0.f;
        row[head * 128 + e + 64] = 0.f;
        if (head < Hq + g.Hkv) {
            const double inv = pow((double)theta, -2.0 * (double)e / 128.0);
            double sn, cs;
            sincos(pos * inv, &sn, &cs);
            const float r0 = lo * (float)cs - hi * (float)sn, r1 = hi * (float)cs + lo * (float)sn;
            if (head < Hq) {
                q[((size_t)m * Hq + head) * 128 + e] = r0;
                q[((size_t)m * Hq + head) * 128 + e + 64] = r1;
            } else if (slot < g.S) {
                kc[kv_k_off(g, b, head - Hq, slot, e)] = f32_to_bf16(r0);
                kc[kv_k_off(g, b, head - Hq, slot, e + 64)] = f32_to_bf16(r1);
            }
        } else if (slot < g.S) {
            vc[kv_v_off(g, b, head - Hq - g.Hkv, slot, e)] = f32_to_bf16(lo);
            vc[kv_v_off(g, b, head - Hq - g.Hkv, slot, e + 64)] = f32_to_bf16(hi);
        }
    }
}

// ---------------------------------------------------------------------------- host side
template <int MT, int EPI>
static int tiled_launch(hipStream_t s, const TArgs& p, int n_blocks, int ksplit) {
    const size_t lds = (size_t)2 * 2 * 4 * MT * 64 * 16;
    auto kern = gemm_tiled_kernel<MT, EPI>;
    if (lds > 64 * 1024) DSD_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<dim3(n_blocks, ksplit), TW * 64, lds, s>>>(p);
    return DSD_OK;
}

template <int EPI>
static int tiled_dispatch(hipStream_t s, const TArgs& p, int n_blocks, int ksplit) {
    switch ((p.M + 15) / 16) {
        case 2: return tiled_launch<2, EPI>(s, p, n_blocks, ksplit);
        case 3: return tiled_launch<3, EPI>(s, p, n_blocks, ksplit);
        case 4: return tiled_launch<4, EPI>(s, p, n_blocks, ksplit);
        case 5: case 6: return tiled_launch<6, EPI>(s, p, n_blocks, ksplit);
        case 7: case 8: return tiled_launch<8, EPI>(s, p, n_blocks, ksplit);
        default: DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: %d rows", p.M);
    }
}

// K split so that a matrix with few column blocks still fills the chip; every slice a multiple of
// 16 k-steps.  Returns 0 if K cannot be cut that way.
static int choose_ksplit(int KS, int n_blocks, int n_cu) {
    if (KS % 16) return 0;
    const int units = KS / 16;
    int best = 1;
    for (int sp = 1; sp <= units; ++sp) {
        if (units % sp) continue;
        best = sp;
        if ((long)n_blocks * sp >= n_cu) break;
    }
    return best;
}

int tiled_supported(const dsd_model_desc* d) {
    return mfma_supported(d) && d->d_model % 512 == 0 && (d->n_q_heads * d->head_dim) % 512 == 0 && d->d_ffn % 512 == 0;
}

// x[M][N] += a[M][K] W^T   (atomic accumulation over the K slices)
int tiled_gemm_resid(dsd_ctx* ctx, const void* Wt, const float* a, float* x, int M, int N, int K) {
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.KS = K / 32; p.M = M; p.a = a; p.out = x; p.N = N;
    const int nb = (N / 16 + 2 * TW - 1) / (2 * TW);
    const int sp = choose_ksplit(p.KS, nb, ctx->n_cu);
    if (!sp) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    p.ks_per_split = p.KS / sp;
    return tiled_dispatch<TE_ATOMIC>(ctx->stream, p, nb, sp);
}

// acc[M][N] += (x*gain)[M][K] Wqkv^T, then finish (norm scale, rotary, append)
int tiled_gemm_qkv(dsd_ctx* ctx, const void* Wt, const float* x, const bf16_t* gain, float* acc, int M, int N, int K,
                   float* q, bf16_t* kc, bf16_t* vc, const KvGeom& g, const int32_t* len, const int32_t* depth, int k,
                   int Hq, float eps, float theta) {
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.KS = K / 32; p.M = M; p.a = x; p.gain = gain; p.out = acc; p.N = N;
    const int nb = (N / 16 + 2 * TW - 1) / (2 * TW);
    const int sp = choose_ksplit(p.KS, nb, ctx->n_cu);
    if (!sp) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    p.ks_per_split = p.KS / sp;
    DSD_TRY(tiled_dispatch<TE_ATOMIC>(ctx->stream, p, nb, sp));
    qkv_finish_kernel<<<M, 256, 0, ctx->stream>>>(acc, x, q, kc, vc, g, len, depth, k, Hq, K, eps, theta);
    return DSD_OK;
}

// h[M][F] = silu(rms(x) Wg^T) * (rms(x) Wu^T)
int tiled_gemm_swiglu(dsd_ctx* ctx, const void* Wt, const float* x, const bf16_t* gain, float* h, int M, int F, int K,
                      float eps) {
    if ((K / 32) % 16) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.KS = K / 32; p.ks_per_split = p.KS; p.M = M; p.a = x; p.gain = gain; p.eps = eps;
    p.out = h; p.N = F; p.up_tile_off = F / 16;
    return tiled_dispatch<TE_SWIGLU>(ctx->stream, p, (F / 16 + TW - 1) / TW, 1);
}

// logits = rms(x; gf) Wlm^T
int tiled_gemm_logits(dsd_ctx* ctx, const void* Wt, const float* x, const bf16_t* gain, float* logits, int M, int V,
                      int K, float eps, int rows_per_seq, int64_t seq_stride) {
    if ((K / 32) % 16) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.KS = K / 32; p.ks_per_split = p.KS; p.M = M; p.a = x; p.gain = gain; p.eps = eps;
    p.out = logits; p.N = V; p.rows_per_seq = rows_per_seq; p.seq_stride = seq_stride;
    return tiled_dispatch<TE_LOGITS>(ctx->stream, p, (V / 16 + 2 * TW - 1) / (2 * TW), 1);
}
