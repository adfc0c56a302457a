// Weight-streaming GEMM for up to 128 rows (B*k of the batched verification pass, section 2.1).
//
// The pass is bound by streaming the weights once, but with many rows the activation operand is no
// longer negligible: every weight fragment meets MT activation fragments (one fp16 plane of MT
// 16-row tiles; two planes, as the one-workgroup-per-tile kernels use, would make the matrix cores
// the bound at 128 rows).  So the activations are shared through LDS and only the weights
// come straight from HBM into registers:
//   * a workgroup of 4 (or 8) computing waves owns 128 (256) output columns, each wave two
//     16-column tiles, over one contiguous slice of K (grid.y splits K when a matrix has too few
//     column blocks to fill the chip; every slice then stores its partial result with plain stores
//     into a buffer of its own and the kernel that reads the result next adds the slices up in a
//     fixed order: fp32 atomics run at about a quarter of the rate of plain stores on this chip, and
//     their order of arrival would make the last bits of the result differ from run to run);
//   * the activations are converted ONCE per GEMM by a small kernel of their own (sum of the
//     previous GEMM's K slices into the residual stream, gain, fp16, A-operand order, sums of
//     squares for the RMSNorm scale) into a panel in global memory;
//     doing that inside every workgroup cost more vector ALU time than the matrix cores had work;
//   * the slice is walked in chunks of 128 columns of K; the workgroup has 4 more waves that do
//     nothing but fetch the next chunk of the panel from global memory straight into LDS (double
//     buffered).  Vector memory loads of one wave complete in order, so a wave that fetched the
//     panel itself would have to drain its older weight loads at every chunk; as it is, the only
//     things a computing wave ever waits for are its own weight stream and the workgroup barrier;
//   * every computing wave keeps its next 8 or 16 weight fragments in flight in a register FIFO,
//     issued by hand (inline asm + explicit s_waitcnt counts, see gload16 / vm_wait); a read stream
//     of this kind saturates HBM with 16 KiB in flight per compute unit, so the depth is set by the
//     registers the row count leaves, not by latency.
#include <stdlib.h>

#include "dsd_bf16_dev.h"

#define TP 4             // panel-fetching waves per workgroup
#define NTW 2            // 16-column tiles per computing wave

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// A weight fragment on its way into a FIFO register.  Weights are read once per pass: the load is marked
// non-temporal, so that the stream does not push the operand panel, which every workgroup reads again and
// again, out of the caches (a bare read runs at 6.9-7.4 TB/s that way against 6.3-6.5 with plain loads; the
// gate/up GEMM at 48 rows went from 163 to 148 us).
__device__ __forceinline__ void gload16(u32x4& dst, const void* ptr) {
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(dst) : "v"(ptr));
}
// count = loads of ours issued after the one needed (vector memory returns in order; a smaller
// count than the true number only waits longer)
template <int N>
__device__ __forceinline__ void vm_wait(u32x4& r) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N));
}
enum { TE_PARTIAL = 0, TE_SWIGLU = 1, TE_LOGITS = 2 };

struct TArgs {
    const uint4* Wt;     // tiled weights: fragment (tile nt, k-step ks) at (ks*NTA + nt)*64 + lane
    int NTA;             // column tiles in the whole weight buffer
    int KS;              // K / 32
    int ks_per_split;    // k-steps per workgroup, multiple of 16
    int M;
    const uint4* panel;  // activations as fp16 in A-operand order: [KS][MT][64] (act_panel_kernel)
    const float* ssq;    // [n_ssq][128] partial sums of squares of every activation row (act_panel_kernel)
    int n_ssq;
    float eps;
    float* out;          // TE_PARTIAL: [gridDim.y][M][N] fp32;  TE_LOGITS: logits
    unsigned short* panel_out;   // TE_SWIGLU: SiLU(gate)*up as fp16 in A-operand order, [N/32][MT][64] entries
    int N;
    int up_tile_off;     // TE_SWIGLU: F/16
    int rows_per_seq;    // TE_LOGITS
    int64_t seq_stride;
    int* sat;            // TE_SWIGLU: counter of SiLU*up values that left the fp16 range
};

// fetching wave ks (0..3) brings k-step ks of a chunk into the panel buffer at LDS byte address buf:
// entry (ks*MT + mt)*64 + lane
template <int MT>
__device__ __forceinline__ void tpanel_fetch(const TArgs& p, int ks_abs, unsigned buf, int ks) {
    const int lane = threadIdx.x & 63;
    const uint4* src = p.panel + ((size_t)(ks_abs + ks) * MT) * 64 + lane;
#pragma unroll
    for (int i = 0; i < MT; ++i) gload16_lds(buf + ((ks * MT + i) * 64) * 16, src + i * 64);
}

// Next k-step of the weight stream; past the end of the slice (the last turn of refills, never
// consumed) it stays on the last fragment.
__device__ __forceinline__ void tadvance(const uint4* (&w)[NTW], int& left, size_t kstep) {
    if (left > 0) {
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) w[nt] += kstep;
    }
    --left;
}

// one chunk (4 k-steps) against FIFO slots S0 .. S0 + 4*NTW - 1
template <int MT, int NF, int S0>
__device__ __forceinline__ void tconsume(u32x4 (&fifo)[NF], const uint4* __restrict__ panel, f32x4 (&acc)[MT][NTW],
                                         const uint4* (&w)[NTW], int& left, size_t kstep, int lane) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        f16x8 a[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[mt] = __builtin_bit_cast(f16x8, panel[(ks * MT + mt) * 64 + lane]);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int slot = (S0 + ks * NTW + nt) % NF;
            vm_wait<NF - 1>(fifo[slot]);
            const f16x8 b = __builtin_bit_cast(f16x8, fifo[slot]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt][nt] = mfma16h(a[mt], b, acc[mt][nt]);
            // refill one FIFO turn ahead; past the end of the slice keep re-reading the last fragment
            gload16(fifo[slot], w[nt]);
        }
        tadvance(w, left, kstep);
    }
}

// The same for 6 or 8 row tiles, where one k-step is 12..16 matrix instructions behind 6..8 LDS
// reads: the row tiles are taken in two halves and the activation fragments of the next half are
// requested before the matrix instructions of the current one, so that LDS latency hides behind
// them (a computing wave has no partner on its SIMD to do that for it).  A weight fragment is used
// by both halves and its FIFO slot refilled after the second, so when slot (ks, nt) is waited for,
// the refills of (ks, 0..nt-1) have not been issued yet: NF - 1 - nt younger loads.
template <int MT, int NF, int S0>
__device__ __forceinline__ void tconsume_halves(u32x4 (&fifo)[NF], const uint4* __restrict__ panel,
                                                f32x4 (&acc)[MT][NTW], const uint4* (&w)[NTW], int& left, size_t kstep, int lane) {
    constexpr int H = MT / 2;
    f16x8 a[2][H];                                    // [buffer][row tile of the half]
    auto fetch = [&](int buf, int ks, int half) {
#pragma unroll
        for (int m = 0; m < H; ++m) a[buf][m] = __builtin_bit_cast(f16x8, panel[(ks * MT + half * H + m) * 64 + lane]);
    };
    fetch(0, 0, 0);
#pragma unroll
    for (int hs = 0; hs < 8; ++hs) {
        const int ks = hs >> 1, half = hs & 1;
        if (hs + 1 < 8) fetch((hs + 1) & 1, (hs + 1) >> 1, (hs + 1) & 1);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int slot = (S0 + ks * NTW + nt) % NF;
            if (half == 0) {
                if (nt == 0) vm_wait<NF - 1>(fifo[slot]);
                else vm_wait<NF - 2>(fifo[slot]);
            }
            const f16x8 b = __builtin_bit_cast(f16x8, fifo[slot]);
#pragma unroll
            for (int m = 0; m < H; ++m) acc[half * H + m][nt] = mfma16h(a[hs & 1][m], b, acc[half * H + m][nt]);
            if (half == 1) gload16(fifo[slot], w[nt]);
        }
        if (half == 1) tadvance(w, left, kstep);
    }
}

// TWC computing waves (4 or 8), each MT 16-row tiles x NTW 16-column tiles; waves TWC .. TWC+3 fetch
// the panel.  More computing waves per workgroup mean fewer workgroups fetching the same panel.  The
// second launch bound is waves per SIMD: two resident workgroups for the smallest tiles.
template <int MT, int TWC, int EPI>
__global__ void __launch_bounds__((TWC + TP) * 64, TWC > 4 ? 3 : (MT <= 3 ? 4 : 2)) gemm_tiled_kernel(TArgs p) {
    extern __shared__ uint4 lds[];                    // 2 panel buffers of 4*MT*64 uint4, a table of 128 floats
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 15, g = lane >> 4;
    const int ks0 = blockIdx.y * p.ks_per_split;
    const int nchunk = p.ks_per_split / 4;
    const size_t pbuf = (size_t)4 * MT * 64;
    if (wave >= TWC) {
        // low half of a flat pointer into LDS = its LDS byte address
        const unsigned lds_addr = (unsigned)(size_t)lds;
        const unsigned pbuf_bytes = 4 * MT * 64 * 16;
        // one barrier per chunk, matched by the computing waves below
        tpanel_fetch<MT>(p, ks0, lds_addr, wave - TWC);
        vm_wait_all<0>();
        __syncthreads();
        for (int ch = 0; ch < nchunk; ++ch) {
            if (ch + 1 < nchunk) {
                tpanel_fetch<MT>(p, ks0 + (ch + 1) * 4, lds_addr + ((ch & 1) ^ 1) * pbuf_bytes, wave - TWC);
            } else if (EPI != TE_PARTIAL) {
                // nothing left to fetch: while the computing waves work through the last chunk, add up
                // the rows' sums of squares (in a fixed order: two lanes per row, four running sums
                // each; n_ssq is a multiple of 4) into a table of 1/rms behind the panel buffers; the
                // last barrier hands it over
                float* rs = (float*)(lds + 2 * pbuf);
                const int t = threadIdx.x - TWC * 64, r = t >> 1;
                if (r < 16 * MT) {
                    float q[4] = {0.f, 0.f, 0.f, 0.f};
                    for (int j = (t & 1) * 4; j < p.n_ssq; j += 8) {
#pragma unroll
                        for (int u = 0; u < 4; ++u) q[u] += p.ssq[(j + u) * 128 + r];
                    }
                    float sq = (q[0] + q[1]) + (q[2] + q[3]);
                    sq += __shfl_xor(sq, 1, WAVE);
                    if (!(t & 1)) rs[r] = 1.0f / sqrtf(sq / (float)(p.KS * 32) + p.eps);
                }
            }
            vm_wait_all<0>();
            __syncthreads();
        }
        return;
    }
    int tile[NTW];
    bool live[NTW];
    const uint4* w[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        if (EPI == TE_SWIGLU) {                       // (gate, up) pairs of the same columns
            const int j = blockIdx.x * (TWC * NTW / 2) + wave * (NTW / 2) + i / 2;
            live[i] = j < p.up_tile_off;
            tile[i] = j + (i & 1) * p.up_tile_off;
        } else {
            tile[i] = blockIdx.x * (TWC * NTW) + wave * NTW + i;
            live[i] = tile[i] < p.N / 16;
        }
        // dead tiles (ragged last column block) stream a valid tile and are not stored
        w[i] = p.Wt + ((size_t)ks0 * p.NTA + (live[i] ? tile[i] : 0)) * 64 + lane;
    }

    // Weight fragments in flight per wave: as many as put about 32 KiB in flight per compute unit, where a bare
    // read stream is fastest too (24-32 KiB: 7.1-7.4 TB/s; 64 KiB: 6.5; 256 KiB: 5.0): 8 (4 k-steps) for up to
    // 5 computing waves, 4 from 6 waves on (LM head at 128 rows: 212 -> 186 us; with 4 for every workgroup
    // size gate/up with 4 waves went from 55.5 to 63.9 us).  Deeper was never faster: 16 measured 0.7 % slower.
    constexpr int NF = TWC >= 6 ? 4 : 8;
    u32x4 fifo[NF];
    int left = p.ks_per_split - 1;                    // k-steps the stream may still advance
    const size_t kstep = (size_t)p.NTA * 64;          // from one k-step's fragment to the next
#pragma unroll
    for (int i = 0; i < NF / NTW; ++i) {
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) gload16(fifo[i * NTW + nt], w[nt]);
        tadvance(w, left, kstep);
    }
    f32x4 acc[MT][NTW];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) acc[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    // a chunk consumes 4*NTW slots: the FIFO turns twice per chunk (NF = 4) or once (NF = 8), slot numbers are
    // taken modulo NF; ks_per_split is a multiple of 16 k-steps = 4 chunks
#define TILED_CHUNK(Q)                                                                          \
    {                                                                                           \
        if (MT >= 6) tconsume_halves<MT, NF, ((Q) * 4 * NTW) % NF>(fifo, lds + ((Q) & 1) * pbuf, acc, w, left, kstep, lane); \
        else tconsume<MT, NF, ((Q) * 4 * NTW) % NF>(fifo, lds + ((Q) & 1) * pbuf, acc, w, left, kstep, lane); \
        __syncthreads();                                                                        \
    }
    for (int ch = 0; ch < nchunk; ch += 4) {
        TILED_CHUNK(0)
        TILED_CHUNK(1)
        TILED_CHUNK(2)
        TILED_CHUNK(3)
    }
#undef TILED_CHUNK
    // Drain what is still in flight (the last turn's refills are never consumed).  Every FIFO
    // register stays live across the wait, so none can be handed to the epilogue while a load may
    // still land in it.
    vm_wait_all<0>();
#pragma unroll
    for (int i = 0; i < NF; ++i) asm volatile("" : "+v"(fifo[i]));

    // 1/rms of this lane's rows, from the table the fetching waves left behind the panel buffers
    f32x4 rstd[MT];
    if (EPI != TE_PARTIAL) {
        const float* rs = (const float*)(lds + 2 * pbuf);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) rstd[mt] = *(const f32x4*)(rs + mt * 16 + g * 4);
    }
    float* part = p.out + (size_t)blockIdx.y * p.M * p.N;      // TE_PARTIAL: this K slice's own buffer
    float worst = 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = mt * 16 + g * 4 + i;
            if (m >= p.M) continue;
            if (EPI == TE_PARTIAL) {
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt)
                    if (live[nt]) part[(size_t)m * p.N + tile[nt] * 16 + c] = acc[mt][nt][i];
            } else if (EPI == TE_SWIGLU) {
#pragma unroll
                for (int nt = 0; nt < NTW; nt += 2)
                    if (live[nt]) {
                        // the next GEMM's operand: row m, column kk of its K -> entry ((kk/32)*MT + m/16)*64 +
                        // m%16 + 16*((kk/8)%4), halfword kk%8
                        const float gate = acc[mt][nt][i] * rstd[mt][i], up = acc[mt][nt + 1][i] * rstd[mt][i];
                        const float hv = gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
                        worst = fmaxf(worst, fabsf(hv));
                        const int kk = tile[nt] * 16 + c;
                        const size_t entry = ((size_t)(kk >> 5) * MT + mt) * 64 + (g * 4 + i) + 16 * ((kk >> 3) & 3);
                        p.panel_out[entry * 8 + (kk & 7)] =
                            __builtin_bit_cast(unsigned short, (_Float16)__builtin_fminf(__builtin_fmaxf(hv, -F16_MAX), F16_MAX));
                    }
            } else {
                float* row = p.out + (size_t)(m / p.rows_per_seq) * p.seq_stride + (size_t)(m % p.rows_per_seq) * p.N;
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt)
                    // tens of megabytes written once: past the caches (LM head 210 -> 196 us at 128 rows)
                    if (live[nt]) __builtin_nontemporal_store(acc[mt][nt][i] * rstd[mt][i], &row[tile[nt] * 16 + c]);
            }
        }
    if (EPI == TE_SWIGLU) report_saturation(p.sat, worst);
}

// Activations -> panel.  Block (chunk, mt) of 4 waves: wave w handles k-step 4*chunk + w, lane
// (c = lane%16, g = lane/16) the 8 values k = 32ks + 8g .. +8 of row 16mt + c.  If the GEMM before
// left n_part K slices of a residual update behind (part[s][M][K]), they are added to the values
// first, slice 0 first, and the sum is stored back: that is the residual stream's update.  Then
// the values are multiplied by the gain (if any), rounded to fp16 (saturating) and stored at entry
// (ks*MT + mt)*64 + lane.  With a gain the block's share of every row's sum of squares goes to
// ssq[chunk][128]; whoever needs the RMSNorm scale adds the chunks up in order.
__global__ void __launch_bounds__(256) act_panel_kernel(uint4* __restrict__ panel, float* __restrict__ ssq,
                                                        float* __restrict__ a, const bf16_t* __restrict__ gain,
                                                        const float* __restrict__ part, int n_part, int M, int K,
                                                        int MT, int* __restrict__ sat) {
    __shared__ float s_q[4][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4, mt = blockIdx.y;
    const int ks = blockIdx.x * 4 + wave;
    const int row = mt * 16 + c, kb = ks * 32 + g * 8;
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (row < M) {
        float* src = a + (size_t)row * K + kb;
        float4 v0 = *(const float4*)src, v1 = *(const float4*)(src + 4);
        if (n_part > 0) {
            const float* ps = part + (size_t)row * K + kb;
            const size_t slice = (size_t)M * K;
            int sl = 0;
            // up to eight slices in flight (the usual counts, 4..8, then take one trip to memory), added in slice order
            if (n_part >= 5 && n_part <= 8) {
                float4 p0[8], p1[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (u < n_part) {
                        p0[u] = *(const float4*)(ps + u * slice);
                        p1[u] = *(const float4*)(ps + u * slice + 4);
                    }
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (u < n_part) {
                        v0.x += p0[u].x; v0.y += p0[u].y; v0.z += p0[u].z; v0.w += p0[u].w;
                        v1.x += p1[u].x; v1.y += p1[u].y; v1.z += p1[u].z; v1.w += p1[u].w;
                    }
                }
                sl = n_part;
            }
            for (; sl + 4 <= n_part; sl += 4, ps += 4 * slice) {
                float4 p0[4], p1[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    p0[u] = *(const float4*)(ps + u * slice);
                    p1[u] = *(const float4*)(ps + u * slice + 4);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    v0.x += p0[u].x; v0.y += p0[u].y; v0.z += p0[u].z; v0.w += p0[u].w;
                    v1.x += p1[u].x; v1.y += p1[u].y; v1.z += p1[u].z; v1.w += p1[u].w;
                }
            }
            for (; sl < n_part; ++sl, ps += slice) {
                const float4 q0 = *(const float4*)ps, q1 = *(const float4*)(ps + 4);
                v0.x += q0.x; v0.y += q0.y; v0.z += q0.z; v0.w += q0.w;
                v1.x += q1.x; v1.y += q1.y; v1.z += q1.z; v1.w += q1.w;
            }
            *(float4*)src = v0;
            *(float4*)(src + 4) = v1;
        }
        v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w;
        v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
    }
    if (gain) {
        float gf[8];
        unpack_gain(*(const uint4*)(gain + kb), gf);
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            q += v[i] * v[i];
            v[i] *= gf[i];
        }
        q += __shfl_xor(q, 16, WAVE);
        q += __shfl_xor(q, 32, WAVE);
        if (lane < 16) s_q[wave][lane] = q;
        __syncthreads();
        if (threadIdx.x < 16)
            ssq[blockIdx.x * 128 + mt * 16 + threadIdx.x] =
                ((s_q[0][threadIdx.x] + s_q[1][threadIdx.x]) + s_q[2][threadIdx.x]) + s_q[3][threadIdx.x];
    }
    report_saturation(sat, absmax8(v, 0.f));
    panel[((size_t)ks * MT + mt) * 64 + lane] = __builtin_bit_cast(uint4, pack8h(v));
}

// x[M][K] += sum of n_part K slices, in order (the residual update when no panel kernel follows);
// the block's output rows in the model dtype go out from here too
__global__ void __launch_bounds__(256) resid_reduce_kernel(float* __restrict__ x, const float* __restrict__ part,
                                                           int n_part, size_t n, bf16_t* __restrict__ out) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    float4 v = *(const float4*)(x + i);
    for (int sl = 0; sl < n_part; ++sl) {
        const float4 p4 = *(const float4*)(part + (size_t)sl * n + i);
        v.x += p4.x; v.y += p4.y; v.z += p4.z; v.w += p4.w;
    }
    *(float4*)(x + i) = v;
    if (out) {
        out[i] = f32_to_bf16(v.x);
        out[i + 1] = f32_to_bf16(v.y);
        out[i + 2] = f32_to_bf16(v.z);
        out[i + 3] = f32_to_bf16(v.w);
    }
}

// K slices of the q, k, v rows (part[s][M][heads*128]) -> their sum in slice order, RMSNorm scale,
// rotary embedding (cos, sin from the call's table), cache append.  Block (row, share): the heads are
// dealt out over gridDim.y blocks; the first wave adds up the row's sums of squares.
__global__ void __launch_bounds__(256) qkv_finish_kernel(const float* __restrict__ part, int n_part, int M,
                                                         const float* __restrict__ ssq, int n_ssq,
                                                         float* __restrict__ q, bf16_t* __restrict__ kc,
                                                         bf16_t* __restrict__ vc, KvGeom g,
                                                         const int32_t* __restrict__ len, int k, int Hq, int d,
                                                         float eps, const float2* __restrict__ rope) {
    __shared__ float s_rstd;
    const int m = blockIdx.x, b = m / k, t = m % k;
    const int slot = len[b] + t;
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        float sq = 0.f;
        for (int j = lane; j < n_ssq; j += 64) sq += ssq[j * 128 + m];
#pragma unroll
        for (int o = 32; o; o >>= 1) sq += __shfl_xor(sq, o, WAVE);
        if (lane == 0) s_rstd = 1.0f / sqrtf(sq / (float)d + eps);
    }
    __syncthreads();
    const float rstd = s_rstd;
    const int heads = Hq + 2 * g.Hkv;
    const int per = (heads + gridDim.y - 1) / gridDim.y;
    const int h0 = blockIdx.y * per, h1 = min(h0 + per, heads);
    const float* row = part + (size_t)m * heads * 128;
    const size_t slice = (size_t)M * heads * 128;
    for (int i = h0 * 64 + threadIdx.x; i < h1 * 64; i += 256) {
        const int head = i >> 6, e = i & 63;
        float lo = 0.f, hi = 0.f;
        const float* src = row + head * 128 + e;
        int sl = 0;
        for (; sl + 4 <= n_part; sl += 4) {            // four slices in flight, added in slice order
            float l4[4], h4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                l4[u] = src[(sl + u) * slice];
                h4[u] = src[(sl + u) * slice + 64];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo += l4[u];
                hi += h4[u];
            }
        }
        for (; sl < n_part; ++sl) {
            lo += src[sl * slice];
            hi += src[sl * slice + 64];
        }
        lo *= rstd;
        hi *= rstd;
        if (head < Hq + g.Hkv) {
            const float2 rot = rope[m * 64 + e];
            const float cs = rot.x, sn = rot.y;
            const float r0 = lo * cs - hi * sn, r1 = hi * cs + lo * sn;
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
template <int MT, int TWC, int EPI>
static int tiled_launch(hipStream_t s, const TArgs& p, int n_blocks, int ksplit) {
    const size_t lds = (size_t)2 * 4 * MT * 64 * 16 + 128 * 4;
    auto kern = gemm_tiled_kernel<MT, TWC, EPI>;
    // once per instantiation and process: the limit is a property of the function, and setting it
    // again on every call would put a non-stream call into a caller's graph capture
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
        DSD_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        raised = true;
    }
    kern<<<dim3(n_blocks, ksplit), (TWC + TP) * 64, lds, s>>>(p);
    return DSD_OK;
}

// twc = computing waves per workgroup: 4 to 8 for the K-sliced GEMMs and gate/up (see choose_partial,
// choose_twc_pairs), 4 or 8 for the LM head
template <int EPI>
static int tiled_dispatch(hipStream_t s, const TArgs& p, int twc, int n_blocks, int ksplit) {
    const int mt = (p.M + 15) / 16;
#define TILED_CASE(T)                                                                    \
    case T:                                                                              \
        switch (mt) {                                                                    \
            case 1: case 2: return tiled_launch<2, T, EPI>(s, p, n_blocks, ksplit);      \
            case 3: return tiled_launch<3, T, EPI>(s, p, n_blocks, ksplit);              \
            case 4: return tiled_launch<4, T, EPI>(s, p, n_blocks, ksplit);              \
            case 5: case 6: return tiled_launch<6, T, EPI>(s, p, n_blocks, ksplit);      \
            case 7: case 8: return tiled_launch<8, T, EPI>(s, p, n_blocks, ksplit);      \
            default: DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: %d rows", p.M);             \
        }
    if constexpr (EPI != TE_LOGITS) {
        switch (twc) {
            TILED_CASE(5)
            TILED_CASE(6)
            TILED_CASE(7)
        }
    }
    switch (twc) {
        TILED_CASE(4)
        TILED_CASE(8)
    }
#undef TILED_CASE
    DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: %d computing waves", twc);
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Computing waves of an LM-head workgroup (2 column tiles each): 8 when the vocabulary is wide enough to
// give about a workgroup per compute unit that way, else 4.  A vocabulary gives several rounds of
// workgroups, each paying its pipeline fill and its epilogue; 8 waves halve the number of rounds.
static int choose_twc_head(int n_tiles16, int n_cu) {
    return (long)ceil_div(n_tiles16, 8 * NTW) * 5 >= (long)n_cu * 4 ? 8 : 4;
}

// Computing waves per workgroup of the gate/up GEMM (a wave owns one (gate, up) pair of column tiles):
// the count from 4 to 8 that leaves the least work on the busiest compute unit; equal counts go to the larger workgroup (fewer fetches of
// the panel).  F = 28672 on 256 compute units: 1792 pairs = 7 per unit exactly, one round of 256
// workgroups of 7 (8 waves would leave 32 units idle: 179.9 against 174.8 us per layer at 48 rows).
static int choose_twc_pairs(int n_pairs, int n_cu) {
    int best = 4;
    long best_cost = -1;
    for (int twc = 4; twc <= 8; ++twc) {
        const long n_wg = ceil_div(n_pairs, twc);
        const long cost = ((n_wg + n_cu - 1) / n_cu) * twc;      // pairs on the busiest compute unit
        if (best_cost < 0 || cost <= best_cost) {
            best = twc;
            best_cost = cost;
        }
    }
    return best;
}

// K split of a matrix with too few column blocks to fill the chip: the number of slices (a divisor
// of K/512, every slice a multiple of 16 k-steps, at most TILED_MAX_KSPLIT) with the smallest
// estimated time.  The estimate walks the rounds in which `slots` resident workgroups take the
// n_blocks*slices work items: a round costs a fixed part (pipeline fill, epilogue) plus the
// slice's weight bytes at the rate a workgroup gets -- its share of the chip's read stream, but no
// more than its share of what one compute unit pulls -- and every slice adds a read of the M x N
// result for whoever sums the slices.  More slices than one round holds lose: the next round pays
// the fixed part again.  The four constants are fitted to measured sweeps of the slice count at
// 48 and 128 rows (d_model 4096 and 8192); the pick is within 1.5 us of the best there.
// Returns 0 if K cannot be cut that way.
static int choose_ksplit(int KS, int n_blocks, int slots, int n_cu, int cols_per_block, int M, int N, double* t_us) {
    if (KS % 16) return 0;
    const int units = KS / 16;
    const double fixed_us = 3.0, chip_bytes_per_us = 5.4e6, cu_bytes_per_us = 28e3, reduce_bytes_per_us = 3.0e6;
    int best = 1;
    double best_t = 1e30;
    for (int sp = 1; sp <= units && sp <= TILED_MAX_KSPLIT; ++sp) {
        if (units % sp) continue;
        const double wg_bytes = (double)(KS / sp) * 32 * cols_per_block * 2;
        double t = (double)sp * M * N * 4 / reduce_bytes_per_us;
        for (long left = (long)n_blocks * sp; left > 0; left -= slots) {
            const long active = left < slots ? left : slots;
            const long per_cu = (active + n_cu - 1) / n_cu;
            const double share = chip_bytes_per_us / active, cu_share = cu_bytes_per_us / per_cu;
            t += fixed_us + wg_bytes / (share < cu_share ? share : cu_share);
        }
        if (t < best_t) {
            best_t = t;
            best = sp;
        }
    }
    *t_us = best_t;
    return best;
}
// workgroups of the tiled kernel the chip holds at once: two per compute unit up to 3 row tiles
static int tiled_slots(int M, int twc, int n_cu) { return (twc == 4 && (M + 15) / 16 <= 3) ? 2 * n_cu : n_cu; }

int tiled_supported(const dsd_model_desc* d) {
    return mfma_supported(d) && d->d_model % 512 == 0 && (d->n_q_heads * d->head_dim) % 512 == 0 && d->d_ffn % 512 == 0;
}

static int mt_of(int M) {
    const int mt = (M + 15) / 16;
    return mt == 1 ? 2 : (mt == 5 ? 6 : (mt == 7 ? 8 : mt));      // tile counts the kernel is built for
}
int tiled_row_tiles(int M) { return mt_of(M); }

// x_pending > 0: that many K slices of a residual update wait in `part` and are folded into `a` first
static void make_panel(dsd_ctx* ctx, uint4* panel, float* ssq, float* a, const bf16_t* gain, const float* part,
                       int x_pending, int M, int K) {
    const int MT = mt_of(M);
    act_panel_kernel<<<dim3(K / 128, MT), 256, 0, ctx->stream>>>(panel, ssq, a, gain, part, x_pending, M, K, MT, ctx->sat_dev);
}

// K-sliced GEMM: part[s][M][N] = slice s of a[M][K] W^T; returns the number of slices in *n_part
static int tiled_gemm_partial(dsd_ctx* ctx, const void* Wt, int M, int N, int K, const void* panel, float* part,
                              int* n_part) {
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.NTA = N / 16; p.KS = K / 32; p.M = M; p.panel = (const uint4*)panel; p.out = part; p.N = N;
    if (p.KS % 16) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    // computing waves per workgroup and K slices together: the pair with the smallest estimated time
    // (ties go to the smaller workgroup).  E.g. 640 column tiles (QKV at d_model 8192) on 256 compute
    // units: 5 waves x 4 slices = 256 workgroups, where 4 waves give 160 or 320.
    int twc = 4, sp = 1;
    double best_t = 1e30;
    for (int t = 4; t <= 8; ++t) {
        double t_us = 0;
        const int sp_t = choose_ksplit(p.KS, ceil_div(N / 16, t * NTW), tiled_slots(M, t, ctx->n_cu), ctx->n_cu, t * NTW * 16, M, N, &t_us);
        if (t_us < best_t) {
            best_t = t_us;
            twc = t;
            sp = sp_t;
        }
    }
    const int nb = ceil_div(N / 16, twc * NTW);
    p.ks_per_split = p.KS / sp;
    *n_part = sp;
    return tiled_dispatch<TE_PARTIAL>(ctx->stream, p, twc, nb, sp);
}

// The K slices of a[M][K] W^T, a given as the operand panel its producer wrote (attention combine,
// SiLU*up), go to `part`; *n_part of them wait there to be added to the residual stream by the next
// kernel that reads it (make_panel or tiled_resid_reduce).
int tiled_gemm_resid(dsd_ctx* ctx, const void* Wt, float* part, int* n_part, int M, int N, int K, const void* panel) {
    return tiled_gemm_partial(ctx, Wt, M, N, K, panel, part, n_part);
}

// x += the slices waiting in part
int tiled_resid_reduce(dsd_ctx* ctx, float* x, const float* part, int n_part, int M, int N, void* hidden_out) {
    const size_t n = (size_t)M * N;
    resid_reduce_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, ctx->stream>>>(x, part, n_part, n, (bf16_t*)hidden_out);
    return DSD_OK;
}

// q, k, v = finish((x*gain)[M][K] Wqkv^T): norm scale, rotary, append.  x first takes the x_pending
// slices waiting in part; the same buffer then carries the slices of the projection.
int tiled_gemm_qkv(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, float* part, int x_pending, int M, int N,
                   int K, float* q, bf16_t* kc, bf16_t* vc, const KvGeom& g, const int32_t* len,
                   int k, int Hq, float eps, const float2* rope, void* panel, float* ssq) {
    make_panel(ctx, (uint4*)panel, ssq, x, gain, part, x_pending, M, K);
    int sp = 0;
    DSD_TRY(tiled_gemm_partial(ctx, Wt, M, N, K, panel, part, &sp));
    // four heads (256 rotation pairs) per block: one pass of the block's threads, all slice loads in flight at once
    const int heads = N / 128;
    qkv_finish_kernel<<<dim3(M, (heads + 3) / 4), 256, 0, ctx->stream>>>(part, sp, M, ssq, K / 128, q, kc, vc, g, len, k, Hq, K,
                                                          eps, rope);
    return DSD_OK;
}

// h[M][F] = silu(rms(x) Wg^T) * (rms(x) Wu^T)
int tiled_gemm_swiglu(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, const float* part, int x_pending,
                      void* panel_h, int M, int F, int K, float eps, void* panel, float* ssq) {
    if ((K / 32) % 16) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    make_panel(ctx, (uint4*)panel, ssq, x, gain, part, x_pending, M, K);
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.NTA = 2 * F / 16; p.KS = K / 32; p.ks_per_split = p.KS; p.M = M; p.panel = (const uint4*)panel; p.ssq = ssq;
    p.n_ssq = K / 128; p.eps = eps; p.panel_out = (unsigned short*)panel_h; p.N = F; p.up_tile_off = F / 16;
    p.sat = ctx->sat_dev;
    // fused SiLU*up needs the whole K in one workgroup: no K split
    const int twc = choose_twc_pairs(F / 16, ctx->n_cu);
    return tiled_dispatch<TE_SWIGLU>(ctx->stream, p, twc, ceil_div(F / 16, twc * NTW / 2), 1);
}

// logits = rms(x; gf) Wlm^T
int tiled_gemm_logits(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, const float* part, int x_pending,
                      float* logits, int M, int V, int K, float eps, int rows_per_seq, int64_t seq_stride, void* panel,
                      float* ssq) {
    if ((K / 32) % 16) DSD_FAIL(DSD_EUNSUPPORTED, "tiled GEMM: K=%d", K);
    make_panel(ctx, (uint4*)panel, ssq, x, gain, part, x_pending, M, K);
    TArgs p = TArgs();
    p.Wt = (const uint4*)Wt; p.NTA = V / 16; p.KS = K / 32; p.ks_per_split = p.KS; p.M = M; p.panel = (const uint4*)panel; p.ssq = ssq;
    p.n_ssq = K / 128; p.eps = eps; p.out = logits; p.N = V; p.rows_per_seq = rows_per_seq; p.seq_stride = seq_stride;
    // A vocabulary gives several rounds of workgroups, each paying its pipeline fill and its epilogue with
    // the compute unit idle; 256-column workgroups (8 computing waves, a shorter weight FIFO to fit
    // the registers) halve the number of rounds.  Measured at 128 rows, V = 128256: 254 -> 238 us.
    const int twc = choose_twc_head(V / 16, ctx->n_cu);
    return tiled_dispatch<TE_LOGITS>(ctx->stream, p, twc, ceil_div(V / 16, twc * NTW), 1);
}
