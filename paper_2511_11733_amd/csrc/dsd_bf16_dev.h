// Device-side building blocks of the bf16 verification pass, shared by its translation units
// (dsd_stage_bf16.hip, dsd_gemm_tiled.hip).
#pragma once

#include "dsd_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

#define WAVE 64
#define MAX_RUNS 512

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ bf16x8 pack8(const float* f) {
    uint4 u = {pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7])};
    return __builtin_bit_cast(bf16x8, u);
}
// v = hi + lo with both halves bf16 (lo carries the rounding remainder of hi)
__device__ __forceinline__ void split8(const float* v, bf16x8* hi, bf16x8* lo) {
    uint4 hu = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
    const unsigned hw[4] = {hu.x, hu.y, hu.z, hu.w};
    float r[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r[2 * i] = v[2 * i] - __uint_as_float(hw[i] << 16);
        r[2 * i + 1] = v[2 * i + 1] - __uint_as_float(hw[i] & 0xFFFF0000u);
    }
    *hi = __builtin_bit_cast(bf16x8, hu);
    *lo = pack8(r);
}
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    // D[4*(lane/16)+i][lane%16] += sum_k A[lane%16][8*(lane/16)+k] * B[8*(lane/16)+k][lane%16]
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
// The weight GEMMs run on the fp16 form of the same instruction: the weights are stored as fp16
// (exact for every bf16 value of magnitude 2^-17 .. 65504, see tile_weights_kernel) and the
// activations enter with fp16's 11 significant bits, which one operand plane of bf16 cannot give.
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
#define F16_MAX 65504.0f
// round to nearest; magnitudes beyond the fp16 range saturate instead of becoming infinite
__device__ __forceinline__ unsigned pack_f16(float a, float b) {
    f32x2 v = {__builtin_fminf(__builtin_fmaxf(a, -F16_MAX), F16_MAX), __builtin_fminf(__builtin_fmaxf(b, -F16_MAX), F16_MAX)};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, f16x2));
}
__device__ __forceinline__ f16x8 pack8h(const float* f) {
    uint4 u = {pack_f16(f[0], f[1]), pack_f16(f[2], f[3]), pack_f16(f[4], f[5]), pack_f16(f[6], f[7])};
    return __builtin_bit_cast(f16x8, u);
}
// v = hi + lo with both halves fp16, ~21 significant bits.  hi is v rounded toward zero, which maps
// magnitudes beyond the fp16 range to the largest finite value at no cost (no clamp); lo carries the
// remainder (less than one unit in hi's last place), so the direction of hi's rounding is immaterial.
__device__ __forceinline__ unsigned pack_f16_rtz(float a, float b) {
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, b));
}
__device__ __forceinline__ void split8h(const float* v, f16x8* hi, f16x8* lo) {
    const uint4 hu = {pack_f16_rtz(v[0], v[1]), pack_f16_rtz(v[2], v[3]), pack_f16_rtz(v[4], v[5]), pack_f16_rtz(v[6], v[7])};
    const f16x8 h = __builtin_bit_cast(f16x8, hu);
    float r[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = v[i] - (float)h[i];
    const uint4 lu = {pack_f16_rtz(r[0], r[1]), pack_f16_rtz(r[2], r[3]), pack_f16_rtz(r[4], r[5]), pack_f16_rtz(r[6], r[7])};
    *hi = h;
    *lo = __builtin_bit_cast(f16x8, lu);
}
__device__ __forceinline__ f32x4 mfma16h(f16x8 a, f16x8 b, f32x4 c) {
    // operand and result layout as mfma16
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// Saturation is never silent: whoever turns an activation into an fp16 operand reports magnitudes
// beyond the fp16 range (NaN too: !(x <= max)) into the context's counter, which dsd_stage_status reads.
// `worst` is the largest |value| a thread has converted.
__device__ __forceinline__ void report_saturation(int* __restrict__ sat, float worst) {
    if (!(worst <= F16_MAX)) atomicAdd(sat, 1);
}
__device__ __forceinline__ float absmax8(const float* v, float m) {
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(v[i]));
    return m;
}

// 8 bf16 gains (one 16-byte load) -> floats
__device__ __forceinline__ void unpack_gain(uint4 gu, float* gf) {
    const unsigned gw[4] = {gu.x, gu.y, gu.z, gu.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        gf[2 * i] = __uint_as_float(gw[i] << 16);
        gf[2 * i + 1] = __uint_as_float(gw[i] & 0xFFFF0000u);
    }
}

// ============================================================================ GEMM pieces
enum { A_F32_GAIN = 0, A_F32 = 1 };
enum { EPI_QKV = 0, EPI_SWIGLU = 1, EPI_RESID = 2, EPI_LOGITS = 3 };

struct GemmArgs {
    const uint4* Wt;      // tiled weights: fragment (tile nt, k-step ks) at (ks*NTA + nt)*64 + lane
    int NTA;              // column tiles in the whole weight buffer
    int KS;               // K / 32
    int M;                // rows in use
    // A operand
    const float* x;       // [M][K] fp32 residual stream          (A_F32_GAIN)
    const bf16_t* gain;   // [K]                                   (A_F32_GAIN)
    const float* a;       // [M][K] fp32 activations               (A_F32)
    float eps;
    // epilogues
    float* xout;          // EPI_RESID: [M][N] fp32, updated in place
    int N;
    bf16_t* hidden_out;   // EPI_RESID, optional: the updated rows also go out in the model dtype (last layer of a block)
    float* hout;          // EPI_SWIGLU: [M][F]
    int up_tile_off;      // EPI_SWIGLU: F/16
    int* sat;             // counter of activations that left the fp16 range on their way into an operand
    float* logits;        // EPI_LOGITS
    int rows_per_seq;
    int64_t seq_stride;
    // EPI_QKV
    float* q;             // [M][Hq*hd] rotated queries, fp32
    bf16_t* kc;           // this layer's K cache
    bf16_t* vc;           // this layer's V cache
    KvGeom g;
    const int32_t* len;
    const float2* rope;   // [M][64] (cos, sin) of every row's rotation angles (rope_table_kernel)
    int k;
    int Hq;
};

// column tiles a workgroup / unit owns
template <int NT, int EPI>
__device__ __forceinline__ void unit_tiles(const GemmArgs& p, int unit, int (&tile)[NT]) {
    if (EPI == EPI_QKV) {               // column tiles (t, t+4) of one head: the rotary pair
        tile[0] = (unit >> 2) * 8 + (unit & 3);
        if (NT > 1) tile[NT - 1] = tile[0] + 4;
    } else if (EPI == EPI_SWIGLU) {     // gate tile and the matching up tile
        tile[0] = unit;
        if (NT > 1) tile[NT - 1] = unit + p.up_tile_off;
    } else {
#pragma unroll
        for (int i = 0; i < NT; ++i) tile[i] = unit * NT + i;
    }
}

// Fused epilogue for one 16-row tile: lane (c = lane%16, g = lane/16) holds rows mt*16 + 4g + i,
// column tile*16 + c of every tile in o[]; rstd[i] = 1/rms of those rows (1 when unused).
template <int NT, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& p, const int (&tile)[NT], const f32x4 (&o)[NT],
                                              const float (&rstd)[4], int mt, int c, int g) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = mt * 16 + g * 4 + i;      // output row of element i
        if (m >= p.M) continue;
        if (EPI == EPI_RESID) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const size_t at = (size_t)m * p.N + tile[nt] * 16 + c;
                const float r = p.xout[at] + o[nt][i];
                p.xout[at] = r;
                if (p.hidden_out) p.hidden_out[at] = f32_to_bf16(r);
            }
        } else if (EPI == EPI_LOGITS) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                p.logits[(size_t)(m / p.rows_per_seq) * p.seq_stride + (size_t)(m % p.rows_per_seq) * p.N +
                         tile[nt] * 16 + c] = o[nt][i] * rstd[i];
        } else if (EPI == EPI_SWIGLU) {
            const float gate = o[0][i] * rstd[i], up = o[NT - 1][i] * rstd[i];
            const float h = gate / (1.0f + __expf(-gate)) * up;
            p.hout[(size_t)m * p.N + tile[0] * 16 + c] = h;
        } else {  // EPI_QKV
            const int hd = 128, half = 64;
            const int head = tile[0] >> 3;                 // 8 column tiles per head
            const int e = (tile[0] & 7) * 16 + c;          // < 64: first element of the rotary pair
            const float lo = o[0][i] * rstd[i], hi = o[NT - 1][i] * rstd[i];
            const int b = m / p.k, t = m % p.k;
            const int L = p.len[b];
            const int slot = L + t;
            if (head < p.Hq + p.g.Hkv) {
                const float2 cs = p.rope[m * 64 + e];
                const float r0 = lo * cs.x - hi * cs.y;
                const float r1 = hi * cs.x + lo * cs.y;
                if (head < p.Hq) {
                    float* dst = p.q + ((size_t)m * p.Hq + head) * hd;
                    dst[e] = r0;
                    dst[e + half] = r1;
                } else if (slot < p.g.S) {
                    const int hk = head - p.Hq;
                    p.kc[kv_k_off(p.g, b, hk, slot, e)] = f32_to_bf16(r0);
                    p.kc[kv_k_off(p.g, b, hk, slot, e + half)] = f32_to_bf16(r1);
                }
            } else if (slot < p.g.S) {
                const int hk = head - p.Hq - p.g.Hkv;
                p.vc[kv_v_off(p.g, b, hk, slot, e)] = f32_to_bf16(lo);
                p.vc[kv_v_off(p.g, b, hk, slot, e + half)] = f32_to_bf16(hi);
            }
        }
    }
}

// ============================================================================ attention pieces
// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_addr + 16*l (lds_addr
// is wave-uniform and goes through M0).  No register ever holds the data, so nothing the register
// allocator does can touch a value whose load is still in flight; completion is counted by vmcnt
// like any other load.
__device__ __forceinline__ void gload16_lds(unsigned lds_addr, const void* ptr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(ptr) : "memory");
}
// The same for data that is read once (the K/V stream): marked non-temporal, so that it does not push what
// is read again and again (queries, operand panels, partial results) out of the caches.
__device__ __forceinline__ void gload16_lds_stream(unsigned lds_addr, const void* ptr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(lds_addr), "v"(ptr) : "memory");
}
template <int N>
__device__ __forceinline__ void vm_wait_all() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

struct AttnArgs {
    const float* q;        // [M][Hq*hd] fp32
    const bf16_t* kc;
    const bf16_t* vc;
    KvGeom g;
    const int32_t* len;
    const uint64_t* mask;
    int k, Hq, G;
    int n_runs;            // runs per (sequence, kv head)
    int* sat;              // counter of values that left the fp16 range
    float* part_o;         // [B][Hkv][n_runs][rows_pad][128]
    float* part_ml;        // [B][Hkv][n_runs][rows_pad][2]
    int rows_pad;          // multiple of 16, >= k*G
    int row_base;          // first query row of this launch (a multiple of 16)
    float scale_log2e;
};

// Merge of the key runs of one query row r of (sequence b, kv head hk):
//   out[m][hq*128 + e] = sum_runs 2^(m_run - M) O_run[e] / sum_runs 2^(m_run - M) l_run
// Called by a whole workgroup of at least 128 threads (all of them reach the barriers); threads
// 0..127 each own one feature.  wgt: MAX_RUNS floats of LDS, red: 4 floats of LDS.
// With `panel` the result goes out as fp16 in the A-operand order of the tiled GEMM for panel_mt
// row tiles instead (element (row m, column kk) of entry ((kk/32)*MT + m/16)*64 + m%16 + 16*((kk/8)%4),
// halfword kk%8), ready for the output projection.
// NORM16: the runs' partial outputs come normalised (O_run / l_run) and as fp16 (attn_stream_kernel
// writes them so: half the bytes of the largest intermediate of the attention, and a bounded range);
// the weight of a run is then 2^(m_run - M) * l_run.
template <bool NORM16 = false>
__device__ __forceinline__ void attn_combine_row(float* __restrict__ out, const float* __restrict__ part_o,
                                                 const float* __restrict__ part_ml, int n_runs, int rows_pad, int k,
                                                 int G, int Hq, int Hkv, int r, int hk, int b, float* wgt, float* red,
                                                 unsigned short* __restrict__ panel = nullptr, int panel_mt = 0,
                                                 int* __restrict__ sat = nullptr) {
    const int e = threadIdx.x, lane = e & 63, wave = e >> 6;
    const bool on = e < 128;
    const size_t u0 = (size_t)(b * Hkv + hk) * n_runs;
    float mx = -INFINITY;
    if (on)
        for (int s = e; s < n_runs; s += 128) {
            const float m = part_ml[((u0 + s) * rows_pad + r) * 2];
            wgt[s] = m;
            mx = fmaxf(mx, m);
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, WAVE));
    if (on && lane == 0) red[wave] = mx;
    __syncthreads();
    const float M = fmaxf(red[0], red[1]);
    float den = 0.f;
    if (on)
        for (int s = e; s < n_runs; s += 128) {
            const float m = wgt[s];
            float w = (m == -INFINITY) ? 0.f : exp2f(m - M);
            const float wl = w * part_ml[((u0 + s) * rows_pad + r) * 2 + 1];
            if (NORM16) w = wl;
            wgt[s] = w;
            den += wl;
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) den += __shfl_xor(den, o, WAVE);
    if (on && lane == 0) red[2 + wave] = den;
    __syncthreads();
    if (on) {
        den = red[2] + red[3];
        float num = 0.f;
        const size_t stride = (size_t)rows_pad * 128;
        if (NORM16) {
            const _Float16* po = (const _Float16*)part_o + (u0 * rows_pad + r) * 128 + e;
#pragma unroll 8
            for (int s = 0; s < n_runs; ++s) num += wgt[s] * (float)po[s * stride];
        } else {
            const float* po = part_o + (u0 * rows_pad + r) * 128 + e;
#pragma unroll 8
            for (int s = 0; s < n_runs; ++s) num += wgt[s] * po[s * stride];
        }
        const int t = r / G, hq = hk * G + r % G;
        if (panel) {
            const int m = b * k + t, kk = hq * 128 + e;
            const size_t entry = ((size_t)(kk >> 5) * panel_mt + (m >> 4)) * 64 + (m & 15) + 16 * ((kk >> 3) & 3);
            if (sat) report_saturation(sat, fabsf(num / den));
            const float v = __builtin_fminf(__builtin_fmaxf(num / den, -F16_MAX), F16_MAX);
            panel[entry * 8 + (kk & 7)] = __builtin_bit_cast(unsigned short, (_Float16)v);
        } else {
            out[((size_t)(b * k + t) * Hq + hq) * 128 + e] = num / den;
        }
    }
    __syncthreads();   // wgt / red may be reused by the caller's next row
}
