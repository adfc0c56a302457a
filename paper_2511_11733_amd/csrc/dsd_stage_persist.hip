// Persistent form of the bf16 verification pass for up to 16 rows (B*k <= 16): the whole
// block of layers runs as ONE cooperative kernel, one workgroup of 4 waves per compute unit.
//
// Why: with so few rows the pass is a pure stream of weights (section 2.1's single forward pass
// over the window is memory bound), and every kernel boundary drains that stream for several
// microseconds.  Here the stream never stops: the weights a wave will need form one fixed
// sequence of 1 KiB fragments across units, phases and layers (weights do not depend on
// activations), and every wave keeps the next 16 fragments of ITS sequence in flight in a
// register FIFO.  Phases (QKV -> attention -> merge -> O-proj -> gate/up -> down) are separated
// by grid barriers; while a workgroup waits at a barrier or runs an epilogue its next 64 KiB of
// weights are already on their way.
//
// Work split: a unit is one 16-column tile (or the pair an epilogue needs) over the full K; unit u
// of a phase belongs to workgroup u mod n_wg; the 4 waves of the workgroup take interleaved
// k-steps and meet in LDS.  Fragment order of a wave inside a unit: k-step major, tile minor.
#include <stdio.h>
#include <stdlib.h>

#include "dsd_bf16_dev.h"

#define PW 4            // waves per workgroup
#define PT (PW * 64)
#define FIFO 16         // fragments in flight per wave

// The weight stream and the activation-panel prefetch are software pipelined by hand: the loads
// are issued through inline asm (the compiler then neither reorders them nor waits for them) and
// every use is preceded by an explicit s_waitcnt whose count is the number of OUR loads issued
// after the one needed (vector memory returns in order, so a smaller count than the true number of
// younger loads only waits longer, never too short).
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void gload16(u32x4& dst, const void* ptr) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(ptr));
}
template <int N>
__device__ __forceinline__ void vm_wait(u32x4& r) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(N));
}

struct PLayer {
    const uint4 *qkv, *wo, *gu, *wd;
    const bf16_t *g1, *g2;
};

struct PArgs {
    const PLayer* layers;
    int L, M, B, k, d, qd, F, Hq, Hkv, G;
    float eps;
    const float2* rope;   // [M][64] (cos, sin), rope_table_launch
    const bf16_t* hidden_in;
    bf16_t* hidden_out;
    float *x, *q, *att, *h;
    bf16_t *kc0, *vc0;          // layer 0 of the cache; layer l at + l * g.layer_elems
    KvGeom g;
    const int32_t *len, *depth;
    const uint64_t* mask;
    int keys_per_wave, n_runs, n_rt, rows_pad;
    float *part_o, *part_ml;
    float scale_log2e;
    const uint4* lm;            // LM head (NULL: none)
    const bf16_t* gf;
    float* logits;
    int V;
    int64_t seq_stride;
    unsigned* flags;            // [n_wg] barrier number each workgroup has reached (monotonic)
    unsigned* abort_dev;        // device abort word
    unsigned bar_base;          // number of the last barrier of the previous launch
    int* abort_host;            // pinned host word, set when a barrier times out
    unsigned spin_limit;
    int n_wg;
    unsigned long long* trace;  // optional: wall-clock stamps of workgroup 0 at every phase boundary
};

enum { WP_QKV = 0, WP_OPROJ = 1, WP_GATEUP = 2, WP_DOWN = 3, WP_HEAD = 4, WP_DONE = 5 };

// ---------------------------------------------------------------------------- weight stream
// One unit's share of the stream for this wave: fragment s lives at
// (s odd and nt == 2 ? b1 : b0)[(nt == 2 ? s/2 : s) * stride].
struct WUnit {
    const uint4 *b0, *b1;
    int nt, fpu, stride;
};

// Position in the fixed schedule layer -> phase -> unit (units of a workgroup: wg, wg+n_wg, ...).
struct WPos {
    int l, ph, u;
};

__device__ __forceinline__ void wphase(const PArgs& p, const WPos& q, const uint4** wt, int* ks, int* nu, int* ntl) {
    if (q.ph == WP_HEAD) {
        *wt = p.lm; *ks = p.d / 32; *nu = p.V / 16; *ntl = 1;
        return;
    }
    const PLayer& ly = p.layers[q.l];
    switch (q.ph) {
        case WP_QKV: *wt = ly.qkv; *ks = p.d / 32; *nu = (p.Hq + 2 * p.Hkv) * 4; *ntl = 2; break;
        case WP_OPROJ: *wt = ly.wo; *ks = p.qd / 32; *nu = p.d / 16; *ntl = 1; break;
        case WP_GATEUP: *wt = ly.gu; *ks = p.d / 32; *nu = p.F / 16; *ntl = 2; break;
        default: *wt = ly.wd; *ks = p.F / 32; *nu = p.d / 16; *ntl = 1; break;
    }
}

// First existing unit at or after q (q is updated); fills `out`.  Past the end the stream keeps
// re-reading one valid fragment (stride 0), so that fetches need no test.
__device__ __forceinline__ void wseek(const PArgs& p, WPos& q, WUnit& out, int wg, int wave, int lane) {
    for (;;) {
        if (q.ph == WP_DONE) {
            out.b0 = out.b1 = p.layers[0].qkv + lane;
            out.nt = 1; out.fpu = 0x7FFFFFFF; out.stride = 0;
            return;
        }
        const uint4* wt;
        int ks, nu, ntl;
        wphase(p, q, &wt, &ks, &nu, &ntl);
        if (q.u < nu) {
            int t0 = q.u, t1 = q.u;
            if (q.ph == WP_QKV) {
                t0 = (q.u >> 2) * 8 + (q.u & 3);
                t1 = t0 + 4;
            } else if (q.ph == WP_GATEUP) {
                t1 = q.u + p.F / 16;
            }
            out.b0 = wt + ((size_t)t0 * ks + wave) * 64 + lane;
            out.b1 = wt + ((size_t)t1 * ks + wave) * 64 + lane;
            out.nt = ntl;
            out.fpu = (ks / PW) * ntl;
            out.stride = PW * 64;
            return;
        }
        q.u = wg;
        if (q.ph == WP_HEAD) {
            q.ph = WP_DONE;
        } else if (q.ph == WP_DOWN) {
            ++q.l;
            if (q.l < p.L) q.ph = WP_QKV;
            else q.ph = p.lm ? WP_HEAD : WP_DONE;
        } else {
            ++q.ph;
        }
    }
}

// The stream runs 16 fragments ahead of the consumer.  Every unit is a multiple of 16 fragments
// and at least 32 long, so the stream leaves the consumer's unit exactly once while that unit is
// consumed: `nxt` is looked up when the consumer starts the unit (prepare), the switch itself
// (roll, once per 16 fetches) is a handful of scalar moves.
struct WIter {
    WPos pos;       // position of nxt
    WUnit cur, nxt;
    int s;
    __device__ __forceinline__ void fetch(u32x4& dst) {
        const uint4* base = (cur.nt == 2 && (s & 1)) ? cur.b1 : cur.b0;
        const int ksl = (cur.nt == 2) ? (s >> 1) : s;
        ++s;
        gload16(dst, base + (size_t)ksl * cur.stride);
    }
    __device__ __forceinline__ void roll() {
        if (s >= cur.fpu) {
            cur = nxt;
            s = 0;
        }
    }
    __device__ __forceinline__ void prepare(const PArgs& p, int wg, int wave, int lane) {
        pos.u += p.n_wg;
        wseek(p, pos, nxt, wg, wave, lane);
    }
};

// ---------------------------------------------------------------------------- grid barrier
// All workgroups are co-resident (cooperative launch).  Every workgroup owns one flag word and
// publishes the number of the barrier it has reached; wave 0 of every workgroup then reads all
// flags (4 per lane) until none is behind.  No read-modify-write on a shared word: arrivals from
// the 8 XCDs do not serialise at the memory side.  Barrier numbers grow monotonically over the
// life of the context, so the flags are never reset.
// The wait is bounded: after spin_limit polls the workgroup raises the abort word, every later
// barrier falls through, and the host refuses further calls on the context.
__device__ __forceinline__ void grid_barrier(const PArgs& p, unsigned epoch) {
    __syncthreads();
    if (threadIdx.x < WAVE) {
        const int lane = threadIdx.x;
        if (lane == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // this workgroup's writes become visible device-wide
            __hip_atomic_store(&p.flags[blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        unsigned spins = 0;
        for (;;) {
            bool behind = false;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int w = lane * 4 + i;
                if (w < p.n_wg) {
                    const unsigned f = __hip_atomic_load(&p.flags[w], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    behind |= (int)(f - epoch) < 0;
                }
            }
            if (!__any(behind)) break;
            if (__hip_atomic_load(p.abort_dev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            __builtin_amdgcn_s_sleep(2);
            if (++spins > p.spin_limit) {
                if (lane == 0) {
                    __hip_atomic_store(p.abort_dev, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    *p.abort_host = 1;
                }
                break;
            }
        }
        if (lane == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // drop stale lines before reading what others wrote
    }
    __syncthreads();
}
__device__ __forceinline__ void stamp(const PArgs& p, int& n) {
    if (p.trace && blockIdx.x == 0 && threadIdx.x == 0) p.trace[n] = wall_clock64();
    ++n;
}

// ---------------------------------------------------------------------------- GEMM phase
// Activations reach the matrix cores through an LDS panel: 2048 columns of K at a time, for the
// M <= 8 rows in use, already multiplied by the RMSNorm gain, split into hi + lo fp16 and laid
// out in A-operand order (entry ((ks*4 + g)*M + r)*2 + {hi, lo}: the 8 values k = 32ks + 8g .. +8
// of row r).  Thread t of the workgroup owns k-group t of every chunk (ks = t/4, g = t%4): it
// loads the raw rows of the NEXT chunk into registers when a chunk starts (those loads are older
// than the chunk's weight refills, so waiting for them later never drains the weight stream) and
// converts them into the other panel buffer when the chunk ends.  The hot loop itself touches
// only LDS and the weight FIFO.
#define CHK 2048
#define CKS (CHK / 32)        // k-steps per chunk (64): 16 per wave
#define MAXM 8

template <int AMODE>
__device__ __forceinline__ void panel_load(u32x4 (&P)[2 * MAXM], u32x4& G, const float* __restrict__ asrc,
                                           const bf16_t* __restrict__ gain, int K, int M, int chunk) {
    const int k0 = chunk * CHK + threadIdx.x * 8;
    // rows >= M re-read row M-1 (a valid address) so that the number of loads is fixed
#pragma unroll
    for (int r = 0; r < MAXM; ++r) {
        const int rr = r < M ? r : M - 1;
        gload16(P[2 * r], asrc + (size_t)rr * K + k0);
        gload16(P[2 * r + 1], asrc + (size_t)rr * K + k0 + 4);
    }
    gload16(G, (AMODE == A_F32_GAIN) ? (const void*)(gain + k0) : (const void*)(asrc + k0));
}

// YOUNGER = loads of ours issued after the panel loads (the weight refills of the chunk)
template <int AMODE, int YOUNGER>
__device__ __forceinline__ void panel_store(u32x4 (&P)[2 * MAXM], u32x4& G, uint4* __restrict__ buf, int M,
                                            float (&ssq)[MAXM], bool count) {
    vm_wait<YOUNGER>(G);      // G was the last panel load: everything in P has arrived as well
#pragma unroll
    for (int r = 0; r < 2 * MAXM; ++r) asm volatile("" : "+v"(P[r]));   // uses of P stay below the wait
    float gf[8];
    if (AMODE == A_F32_GAIN) unpack_gain(make_uint4(G.x, G.y, G.z, G.w), gf);
    uint4* dst = buf + (size_t)threadIdx.x * M * 2;      // ((ks*4 + g)*M + r)*2 with ks*4 + g == thread
#pragma unroll
    for (int r = 0; r < MAXM; ++r)
        if (r < M) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = __uint_as_float(P[2 * r][i]);
                v[4 + i] = __uint_as_float(P[2 * r + 1][i]);
            }
            if (AMODE == A_F32_GAIN) {
                float q = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    q += v[i] * v[i];
                    v[i] *= gf[i];
                }
                if (count) ssq[r] += q;
            }
            f16x8 hi, lo;
            split8h(v, &hi, &lo);
            dst[2 * r] = __builtin_bit_cast(uint4, hi);
            dst[2 * r + 1] = __builtin_bit_cast(uint4, lo);
        }
}

// 8 k-steps of this wave (j0 .. j0+7 of its 16 in the chunk) against FIFO slots S0 ...
template <int NT, int S0>
__device__ __forceinline__ void consume8(u32x4 (&fifo)[FIFO], WIter& it, const uint4* __restrict__ panel, int M,
                                         int j0, f32x4 (&acc)[NT], int wave, int c, int g) {
    const int r = c < M ? c : M - 1;      // rows >= M of the A tile are never stored: any valid data will do
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int ks = wave + PW * (j0 + j);
        const uint4* src = panel + ((size_t)(ks * 4 + g) * M + r) * 2;
        const f16x8 hi = __builtin_bit_cast(f16x8, src[0]);
        const f16x8 lo = __builtin_bit_cast(f16x8, src[1]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int slot = S0 + j * NT + nt;
            vm_wait<FIFO - 1>(fifo[slot]);      // at most the 15 younger refills may still be in flight
            const f16x8 b = __builtin_bit_cast(f16x8, fifo[slot]);
            acc[nt] = mfma16h(hi, b, acc[nt]);
            acc[nt] = mfma16h(lo, b, acc[nt]);
            asm volatile("" : "+v"(acc[nt]) : "v"(fifo[slot]));   // the refill below must not overtake the reads
            it.fetch(fifo[slot]);
        }
    }
}

template <int NT, int AMODE, int EPI>
__device__ __forceinline__ void gemm_phase(const PArgs& p, const GemmArgs& ga, int n_units, u32x4 (&fifo)[FIFO],
                                           WIter& it, uint4* lds_panel, f32x4* lds_red, float* lds_ssq, int& parity,
                                           int wg, int wave, int lane) {
    if (wg >= n_units) return;
    const int c = lane & 15, g = lane >> 4;
    const int K = ga.KS * 32;
    const int M = ga.M;
    const int nchunk = K / CHK;
    const size_t pbuf = (size_t)CKS * 4 * M * 2;      // uint4 per panel buffer
    const float* asrc = (AMODE == A_F32_GAIN) ? ga.x : ga.a;
    u32x4 P[2 * MAXM];
    u32x4 G;
    float ssq[MAXM];
#pragma unroll
    for (int r = 0; r < MAXM; ++r) ssq[r] = 0.f;
    int cur = 0;
    // first chunk of the phase: nothing to overlap it with but the weights already in flight
    panel_load<AMODE>(P, G, asrc, ga.gain, K, M, 0);
    panel_store<AMODE, 0>(P, G, lds_panel, M, ssq, true);
    __syncthreads();
    bool first = true;
    for (int u = wg; u < n_units; u += p.n_wg) {
        const bool last_unit = u + p.n_wg >= n_units;
        it.prepare(p, wg, wave, lane);     // the stream is inside this unit now; look up the one after it
        f32x4 acc[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int ch = 0; ch < nchunk; ++ch) {
            const int nxt = (ch + 1 == nchunk) ? 0 : ch + 1;
            const bool has_next = !(last_unit && ch + 1 == nchunk);
            if (has_next) panel_load<AMODE>(P, G, asrc, ga.gain, K, M, nxt);
            const uint4* panel = lds_panel + cur * pbuf;
            it.roll();
            consume8<NT, 0>(fifo, it, panel, M, 0, acc, wave, c, g);
            if (NT == 2) it.roll();
            consume8<NT, (NT == 1 ? 8 : 0)>(fifo, it, panel, M, 8, acc, wave, c, g);
            if (has_next) panel_store<AMODE, 16 * NT>(P, G, lds_panel + (cur ^ 1) * pbuf, M, ssq, first && nxt != 0);
            __syncthreads();
            cur ^= 1;
        }
        if (AMODE == A_F32_GAIN && first) {
            // every row's sum of squares: threads hold disjoint k-groups -> wave shuffles, then LDS
#pragma unroll
            for (int r = 0; r < MAXM; ++r) {
                float q = ssq[r];
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, WAVE);
                if (lane == 0) lds_ssq[wave * MAXM + r] = q;
            }
        }
        first = false;
        // the 4 waves' partial tiles meet in LDS (two regions, used alternately, so that only one
        // workgroup barrier per unit is needed); wave 0 runs the fused epilogue
        f32x4* red = lds_red + parity * (PW * 2 * 64);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) red[(wave * NT + nt) * 64 + lane] = acc[nt];
        __syncthreads();
        if (wave == 0) {
            f32x4 o[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                o[nt] = red[nt * 64 + lane];
#pragma unroll
                for (int w = 1; w < PW; ++w) o[nt] += red[(w * NT + nt) * 64 + lane];
            }
            float rstd[4] = {1.f, 1.f, 1.f, 1.f};
            if (AMODE == A_F32_GAIN) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = g * 4 + i;
                    if (row < M) {
                        float q = 0.f;
#pragma unroll
                        for (int w = 0; w < PW; ++w) q += lds_ssq[w * MAXM + row];
                        rstd[i] = 1.0f / sqrtf(q / (float)K + ga.eps);
                    }
                }
            }
            int tile[NT];
            unit_tiles<NT, EPI>(ga, u, tile);
            gemm_epilogue<NT, EPI>(ga, tile, o, rstd, 0, c, g);
        }
        parity ^= 1;
    }
    __syncthreads();      // lds_ssq and the panel are free again for the next phase
}

// ---------------------------------------------------------------------------- the kernel
__global__ void __launch_bounds__(PT) stage_persist_kernel(PArgs p) {
    extern __shared__ uint4 lds_panel[];          // 2 buffers of CKS*4*M*2 uint4
    __shared__ f32x4 lds_red[2 * PW * 2 * 64];
    __shared__ float lds_ssq[PW * MAXM];
    __shared__ float lds_wgt[MAX_RUNS];
    __shared__ float lds_r4[4];
    const int wg = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int parity = 0;
    int nst = 0;
    unsigned target = p.bar_base;
    stamp(p, nst);

    // start the weight stream
    WIter it;
    it.pos.l = 0; it.pos.ph = WP_QKV; it.pos.u = wg;
    it.s = 0;
    wseek(p, it.pos, it.cur, wg, wave, lane);
    it.nxt = it.cur;
    u32x4 fifo[FIFO];
#pragma unroll
    for (int i = 0; i < FIFO; ++i) it.fetch(fifo[i]);

    // rows handed over by the previous node -> fp32 residual stream
    const size_t nx = (size_t)p.M * p.d;
    for (size_t i = (size_t)wg * PT + threadIdx.x; i < nx; i += (size_t)p.n_wg * PT) p.x[i] = bf16_to_f32(p.hidden_in[i]);
    target += 1u;
    stamp(p, nst);
    grid_barrier(p, target);
    stamp(p, nst);

    GemmArgs ga;
    for (int l = 0; l < p.L; ++l) {
        const PLayer ly = p.layers[l];
        bf16_t* kc = p.kc0 + (size_t)l * p.g.layer_elems;
        bf16_t* vc = p.vc0 + (size_t)l * p.g.layer_elems;
        // q, k, v = rmsnorm(x; g1) Wqkv^T, rotary, cache append
        ga = GemmArgs();
        ga.KS = p.d / 32; ga.M = p.M; ga.x = p.x; ga.gain = ly.g1; ga.eps = p.eps;
        ga.q = p.q; ga.kc = kc; ga.vc = vc; ga.g = p.g; ga.len = p.len; ga.rope = p.rope; ga.k = p.k; ga.Hq = p.Hq;
        gemm_phase<2, A_F32_GAIN, EPI_QKV>(p, ga, (p.Hq + 2 * p.Hkv) * 4, fifo, it, lds_panel, lds_red, lds_ssq, parity, wg, wave, lane);
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);

        // attention: one wave per (sequence, kv head, key run, 16-row tile)
        {
            AttnArgs t;
            t.q = p.q; t.kc = kc; t.vc = vc; t.g = p.g; t.len = p.len; t.mask = p.mask; t.k = p.k; t.Hq = p.Hq; t.G = p.G;
            t.keys_per_wave = p.keys_per_wave; t.n_runs = p.n_runs; t.part_o = p.part_o; t.part_ml = p.part_ml;
            t.rows_pad = p.rows_pad; t.scale_log2e = p.scale_log2e;
            const int total = p.B * p.Hkv * p.n_runs * p.n_rt;
            for (int wu = wave * p.n_wg + wg; wu < total; wu += PW * p.n_wg) {
                const int rt = wu % p.n_rt;
                int r = wu / p.n_rt;
                const int run = r % p.n_runs;
                r /= p.n_runs;
                attn_run<1>(t, r / p.Hkv, r % p.Hkv, run, rt * 16, lane);
            }
        }
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);
        {
            const int rows = p.k * p.G;
            const int items = p.B * p.Hkv * rows;
            for (int item = wg; item < items; item += p.n_wg) {
                const int r = item % rows;
                const int bh = item / rows;
                attn_combine_row(p.att, p.part_o, p.part_ml, p.n_runs, p.rows_pad, p.k, p.G, p.Hq, p.Hkv, r,
                                 bh % p.Hkv, bh / p.Hkv, lds_wgt, lds_r4);
            }
        }
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);

        // x += attn Wo^T
        ga = GemmArgs();
        ga.KS = p.qd / 32; ga.M = p.M; ga.a = p.att; ga.xout = p.x; ga.N = p.d;
        gemm_phase<1, A_F32, EPI_RESID>(p, ga, p.d / 16, fifo, it, lds_panel, lds_red, lds_ssq, parity, wg, wave, lane);
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);

        // h = silu(b Wg^T) * (b Wu^T),  b = rmsnorm(x; g2)
        ga = GemmArgs();
        ga.KS = p.d / 32; ga.M = p.M; ga.x = p.x; ga.gain = ly.g2; ga.eps = p.eps; ga.hout = p.h; ga.N = p.F;
        ga.up_tile_off = p.F / 16;
        gemm_phase<2, A_F32_GAIN, EPI_SWIGLU>(p, ga, p.F / 16, fifo, it, lds_panel, lds_red, lds_ssq, parity, wg, wave, lane);
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);

        // x += h Wd^T
        ga = GemmArgs();
        ga.KS = p.F / 32; ga.M = p.M; ga.a = p.h; ga.xout = p.x; ga.N = p.d;
        gemm_phase<1, A_F32, EPI_RESID>(p, ga, p.d / 16, fifo, it, lds_panel, lds_red, lds_ssq, parity, wg, wave, lane);
        target += 1u;
        stamp(p, nst);
        grid_barrier(p, target);
        stamp(p, nst);
    }
    if (p.hidden_out)
        for (size_t i = (size_t)wg * PT + threadIdx.x; i < nx; i += (size_t)p.n_wg * PT) p.hidden_out[i] = f32_to_bf16(p.x[i]);
    if (p.lm) {
        ga = GemmArgs();
        ga.KS = p.d / 32; ga.M = p.M; ga.x = p.x; ga.gain = p.gf; ga.eps = p.eps; ga.logits = p.logits; ga.N = p.V;
        ga.rows_per_seq = p.k; ga.seq_stride = p.seq_stride;
        gemm_phase<1, A_F32_GAIN, EPI_LOGITS>(p, ga, p.V / 16, fifo, it, lds_panel, lds_red, lds_ssq, parity, wg, wave, lane);
    }
}

// ---------------------------------------------------------------------------- host side
int persist_supported(const dsd_model_desc* d) {
    return mfma_supported(d) && d->d_model % 2048 == 0 && (d->n_q_heads * d->head_dim) % 2048 == 0 &&
           d->d_ffn % 2048 == 0;
}

int persist_build_layer_table(dsd_weights* w) {
    std::vector<PLayer> t(w->desc.n_layers);
    for (int l = 0; l < w->desc.n_layers; ++l) {
        const LayerW& L = w->layers[l];
        t[l].qkv = (const uint4*)L.qkv_t; t[l].wo = (const uint4*)L.wo_t; t[l].gu = (const uint4*)L.gu_t;
        t[l].wd = (const uint4*)L.wd_t; t[l].g1 = (const bf16_t*)L.g1; t[l].g2 = (const bf16_t*)L.g2;
    }
    void* p = nullptr;
    if (hipMalloc(&p, t.size() * sizeof(PLayer)) != hipSuccess) DSD_FAIL(DSD_ENOMEM, "layer table");
    w->allocs.push_back(p);
    DSD_HIP(hipMemcpy(p, t.data(), t.size() * sizeof(PLayer), hipMemcpyHostToDevice));
    w->layer_table = p;
    return DSD_OK;
}

static int persist_init(dsd_ctx* ctx) {
    if (ctx->bar_dev) return DSD_OK;
    hipDeviceProp_t prop;
    DSD_HIP(hipGetDeviceProperties(&prop, ctx->device));
    if (!prop.cooperativeLaunch) DSD_FAIL(DSD_EUNSUPPORTED, "device has no cooperative launch");
    int per_cu = 0;
    const int max_dyn = 2 * CKS * 4 * MAXM * 2 * 16;
    DSD_HIP(hipFuncSetAttribute((const void*)stage_persist_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, max_dyn));
    DSD_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stage_persist_kernel, PT, max_dyn));
    if (per_cu < 1) DSD_FAIL(DSD_EUNSUPPORTED, "persistent stage kernel does not fit a compute unit");
    ctx->n_cu = prop.multiProcessorCount;
    void* p = nullptr;
    if (ctx->n_cu > 256) DSD_FAIL(DSD_EUNSUPPORTED, "persistent stage kernel: more than 256 compute units");
    if (hipMalloc(&p, 260 * sizeof(unsigned)) != hipSuccess) DSD_FAIL(DSD_ENOMEM, "barrier words");
    DSD_HIP(hipMemset(p, 0, 260 * sizeof(unsigned)));
    void* h = nullptr;
    if (hipHostMalloc(&h, sizeof(int), hipHostMallocDefault) != hipSuccess) {
        (void)hipFree(p);
        DSD_FAIL(DSD_ENOMEM, "abort word");
    }
    *(int*)h = 0;
    ctx->bar_dev = (unsigned*)p;
    ctx->abort_host = (int*)h;
    ctx->bar_base = 0;
    return DSD_OK;
}

int persist_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                         const uint64_t* tree_mask, const int32_t* depth, int B, int k, void* hidden_out,
                         float* logits, int64_t logits_seq_stride) {
    const dsd_model_desc& D = w->desc;
    const KvGeom& g = kv->geom;
    DSD_TRY(persist_init(ctx));
    if (*ctx->abort_host) DSD_FAIL(DSD_EHIP, "a grid barrier of an earlier verify step timed out; the context is unusable");
    PArgs p = PArgs();
    p.layers = (const PLayer*)w->layer_table;
    p.L = D.n_layers; p.M = B * k; p.B = B; p.k = k; p.d = D.d_model; p.Hq = D.n_q_heads; p.Hkv = D.n_kv_heads;
    p.G = p.Hq / p.Hkv; p.qd = p.Hq * D.head_dim; p.F = D.d_ffn; p.eps = D.rms_eps;
    p.n_wg = ctx->n_cu;

    int max_len = 0;
    for (int b = 0; b < B; ++b) max_len = std::max(max_len, kv->len_bound[b]);
    const int max_keys = std::min(max_len + k, g.S);
    const int rows = k * p.G;
    p.n_rt = (rows + 15) / 16;
    p.rows_pad = p.n_rt * 16;
    // key runs: about one (run, row tile) per wave of the grid
    const long units = (long)B * p.Hkv * p.n_rt;
    long kpw = ((long)max_keys * units + (long)p.n_wg * PW - 1) / ((long)p.n_wg * PW);
    kpw = std::max(32L, (kpw + 31) / 32 * 32);
    p.keys_per_wave = (int)kpw;
    p.n_runs = (max_keys + p.keys_per_wave - 1) / p.keys_per_wave;
    if (p.n_runs > MAX_RUNS) DSD_FAIL(DSD_EUNSUPPORTED, "bf16 path: %d key runs", p.n_runs);
    p.scale_log2e = 1.4426950408889634f / sqrtf((float)D.head_dim);

    const size_t M = p.M;
    const size_t nunit = (size_t)B * p.Hkv * p.n_runs * p.rows_pad;
    size_t need = M * p.d * 4 + M * p.qd * 4 * 2 + M * p.F * 4 + nunit * 130 * 4 + M * 64 * 8 + 9 * 256;
    DSD_TRY(dsd_ws_reserve(ctx, need));
    WsBump ws{ctx->ws, 0};
    p.x = ws.take<float>(M * p.d);
    p.q = ws.take<float>(M * p.qd);
    p.att = ws.take<float>(M * p.qd);
    p.h = ws.take<float>(M * p.F);
    p.part_o = ws.take<float>(nunit * 128);
    p.part_ml = ws.take<float>(nunit * 2);
    float2* rope = ws.take<float2>(M * 64);
    p.rope = rope;
    rope_table_launch(ctx, rope, kv->len_dev, depth, (int)M, k, D.rope_theta);
    p.hidden_in = (const bf16_t*)hidden_in;
    p.hidden_out = (bf16_t*)hidden_out;
    p.kc0 = (bf16_t*)kv->k; p.vc0 = (bf16_t*)kv->v; p.g = g;
    p.len = kv->len_dev; p.depth = depth; p.mask = tree_mask;
    if (logits) {
        p.lm = (const uint4*)w->lm_t; p.gf = (const bf16_t*)w->gf; p.logits = logits; p.V = D.vocab;
        p.seq_stride = logits_seq_stride;
    }
    p.flags = ctx->bar_dev;
    p.abort_dev = ctx->bar_dev + 256;
    p.bar_base = ctx->bar_base;
    p.abort_host = ctx->abort_host;
    p.spin_limit = 4000000u;       // polls of >= 64 cycles each: seconds, not forever
    const int n_barriers = 1 + 6 * p.L;
    ctx->bar_base += (unsigned)n_barriers;

    static const bool want_trace = getenv("DSD_PERSIST_TRACE") != nullptr;
    unsigned long long* trace_dev = nullptr;
    const int n_stamps = 2 * n_barriers + 1;
    if (want_trace) {
        if (hipMalloc((void**)&trace_dev, n_stamps * 8) != hipSuccess) trace_dev = nullptr;
        p.trace = trace_dev;
    }
    {
        ProfScope ps(ctx, DSD_KC_STAGE);
        void* args[] = {&p};
        const size_t dyn = (size_t)2 * CKS * 4 * p.M * 2 * 16;
        DSD_HIP(hipLaunchCooperativeKernel((const void*)stage_persist_kernel, dim3(p.n_wg), dim3(PT), args, dyn, ctx->stream));
    }
    if (trace_dev) {   // diagnostic only: synchronises and prints the phase times of the first layer
        std::vector<unsigned long long> t(n_stamps);
        DSD_HIP(hipStreamSynchronize(ctx->stream));
        DSD_HIP(hipMemcpy(t.data(), trace_dev, n_stamps * 8, hipMemcpyDeviceToHost));
        (void)hipFree(trace_dev);
        static int calls = 0;
        if (++calls == 20) {
            const char* names[7] = {"rows_in", "qkv", "attn", "merge", "oproj", "gateup", "down"};
            double tick = 0.01;  // wall_clock64 ticks at 100 MHz -> microseconds
            fprintf(stderr, "[persist trace] total %.1f us\n", (t[n_stamps - 1] - t[0]) * tick);
            for (int i = 0; i < 7 + 6 && 2 * i + 2 < n_stamps; ++i)
                fprintf(stderr, "  %-8s work %.2f us  barrier wait %.2f us\n", names[i == 0 ? 0 : 1 + (i - 1) % 6],
                        (t[2 * i + 1] - t[2 * i]) * tick, (t[2 * i + 2] - t[2 * i + 1]) * tick);
        }
    }
    return DSD_OK;
}
