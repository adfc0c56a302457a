// Acceptance loop of Algorithm 1 (lines 2-16) with the key-token rule and the softened target
// of section 2.3, for B sequences at once.
//
// The logits rows and the draft rows are read ONCE, by slice_pass_kernel: one wavefront per slice of
// SLICE ids of one row reduces everything the rule needs from the vocabulary to a few numbers --
// the slice's share of the log-sum-exp, of Z~ = sum_v P_t(v)^(1-tau) q(v)^tau (the call has one tau;
// a key token only chooses between Z~ and 1), and the slice's top-M candidates of both rows (NormMatch).
// Only those partials reach memory: no probability row is materialised.  seq_kernel (one workgroup
// per sequence) merges them per row, applies the key rule and the test u*q(y) < P(y) to every node,
// walks the tree for the accepted path and says what the extra token is drawn from; that row is
// then read a second time by draw_parts / draw_pick (inverse CDF in token-id order).
//
// Precision.  Every quantity that decides something by itself (a drafted token's own probabilities,
// the accept test, all sums over slices and cumulative sums) is fp64.  The per-id terms of the
// vocabulary-wide sums are fp32: the exponent (l/T - reference) log2(e) is formed with a two-float
// constant so that its error is one rounding of the exponent itself (about 6e-8 of its magnitude,
// independent between ids), the terms of a lane are added in four short fp32 chains and everything
// above that in fp64; a sum over thousands of ids is then good to about 1e-8.  The integer outputs
// therefore follow an fp64 reference except within the near-tie bands the tests state.
//
//   slice_pass  per (sequence, row, slice): max, sum-exp and Z~ share, top-M candidates of both rows
//   seq         per sequence: rows' log-sum-exp, Z~, NormMatch; key test and accept test of every
//               node; accepted path; what to draw from
//   node_z      only with tau_override (a tau per node): per (sequence, node, slice) share of that node's Z~
//   draw_parts  per (sequence, slice): partial mass of the distribution the extra token comes from
//   draw_pick   per sequence: inverse CDF in token-id order
#include "dsd_internal.h"

#define WAVE 64
#define SLICE 2048
#define TPB 256
#define EPT (SLICE / TPB)
#define MAXM DSD_MAX_TOP_M
#define LCAP 32           // candidate keys a slice may hand to the row merge (top_m <= 16 of them matter)

typedef unsigned long long u64;

// order-preserving key: larger value first, then lower id
__device__ inline u64 rank_key(float v, int id) {
    unsigned u = __float_as_uint(v);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((u64)u << 32) | (u64)(0xFFFFFFFFu - (unsigned)id);
}
__device__ inline int key_id(u64 key) { return (int)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull)); }

__device__ inline double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline double wave_max_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ inline u64 wave_max_u(u64 v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        u64 t = __shfl_xor(v, o, WAVE);
        v = t > v ? t : v;
    }
    return v;
}
// block reductions over TPB threads; sh has TPB/WAVE entries; result broadcast to all threads
__device__ inline double block_sum_d(double v, double* sh) {
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sh[threadIdx.x / WAVE] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int i = 0; i < TPB / WAVE; ++i) r += sh[i];
    return r;
}
__device__ inline double block_max_d(double v, double* sh) {
    v = wave_max_d(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sh[threadIdx.x / WAVE] = v;
    __syncthreads();
    double r = sh[0];
#pragma unroll
    for (int i = 1; i < TPB / WAVE; ++i) r = fmax(r, sh[i]);
    return r;
}
__device__ inline u64 block_max_u(u64 v, u64* sh) {
    v = wave_max_u(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == 0) sh[threadIdx.x / WAVE] = v;
    __syncthreads();
    u64 r = sh[0];
#pragma unroll
    for (int i = 1; i < TPB / WAVE; ++i) r = sh[i] > r ? sh[i] : r;
    return r;
}

// P_t(v)^(1-tau) * q(v)^tau from ln P_t(v) and q(v), with x^0 = 1 for every x
__device__ inline double soft_weight(double ln_pt, double q, double tau) {
    const double a = 1.0 - tau;
    double e = (a == 0.0) ? 0.0 : a * ln_pt;
    if (tau != 0.0) {
        if (q <= 0.0) return 0.0;
        e += tau * log(q);
    }
    return exp(e);
}

// the same weight for one id of a vocabulary-wide sum: fp32 terms (see the header)
__device__ inline float soft_weight_f(float ln_pt, float q, float tau) {
    const float a = 1.0f - tau;
    float e = (a == 0.0f) ? 0.0f : a * ln_pt;
    if (tau != 0.0f) {
        if (q <= 0.0f) return 0.0f;
        e += tau * logf(q);
    }
    return expf(e);
}

__device__ inline unsigned order_u32(float v) {
    const unsigned u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---------------------------------------------------------------------------- wave-level tools
__device__ inline float wave_max_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
__device__ __forceinline__ u64 readlane_u64(u64 v, int l) {      // l wave-uniform
    const unsigned lo = __builtin_amdgcn_readlane((int)(unsigned)v, l), hi = __builtin_amdgcn_readlane((int)(unsigned)(v >> 32), l);
    return ((u64)hi << 32) | (u64)lo;
}
// The top_m-th largest of the 64 / GL group maxima of v (a group = GL neighbouring lanes), equal
// values counted separately: a lower bound of the top_m-th largest of all the values the lanes'
// v stand for, as long as every v is the maximum of a set of ids of its own.  top_m <= 64 / GL.
// All lanes get the result.  T = float or u64 (anything ordered by > and ==).
__device__ __forceinline__ float rd_lane(float v, int l) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l)); }
__device__ __forceinline__ u64 rd_lane(u64 v, int l) { return readlane_u64(v, l); }
template <int GL, typename T>
__device__ inline T group_threshold(T v, int lane, int top_m) {
#pragma unroll
    for (int o = 1; o < GL; o <<= 1) {
        const T t = __shfl_xor(v, o, WAVE);
        v = t > v ? t : v;
    }
    int rank = 0;                                         // of this lane's group among the 64 / GL groups
    const int mine = lane / GL;
#pragma unroll
    for (int g = 0; g < WAVE / GL; ++g) {
        const T o = rd_lane(v, g * GL);
        rank += (o > v || (o == v && g < mine)) ? 1 : 0;
    }
    const unsigned long long holder = __ballot(rank == top_m - 1);      // the lanes of exactly one group
    return rd_lane(v, __ffsll((long long)holder) - 1);
}

// Between a wave's LDS writes and its own lanes' reads of them: LDS operations of one wave complete in
// order; this keeps the compiler from moving them and waits for the writes.
__device__ __forceinline__ void wave_lds_sync() { __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup"); }

// cnt <= 64 distinct keys sit in cand[0..cnt) (LDS of this wave): the top_m largest go to out[0..top_m),
// best first, 0 where the keys run out.  Every lane counts the keys above its own.
__device__ inline void rank_out(const u64* __restrict__ cand, int cnt, int top_m, int lane, u64* __restrict__ out) {
    const u64 c = lane < cnt ? cand[lane] : 0ull;
    int rank = 0;
    for (int i = 0; i < cnt; ++i) rank += readlane_u64(c, i) > c ? 1 : 0;
    if (lane < cnt) {
        if (rank < top_m) out[rank] = c;
    } else if (lane < top_m) {
        out[lane] = 0ull;                                 // cnt <= lane < top_m: fewer keys than top_m
    }
}

struct AcceptWs {
    float* part_m;      // [B][R][S]   reference exponent of the slice: (max logit / T) log2 e, as one float
    double* part_s;     // [B][R][S]   sum_v 2^(x_v - part_m),  x_v = (l_v / T) log2 e
    double* part_zs;    // [B][R][S]   sum_v 2^((1-tau)(x_v - part_m)) q_v^tau   (rows with children, call-wide tau > 0)
    u64* part_top_t;    // [B][R][S][LCAP]  (value, id) keys of the slice's candidates for the row's top_m, logits row, unordered
    u64* part_top_q;    // [B][R][S][LCAP]  the same of the draft row
    int32_t* part_cnt;  // [B][R][S][2]     how many of them (logits row, draft row)
    double* row_lse;    // [B][R]  natural-log log-sum-exp of logits / T
    double* row_z;      // [B][R]  Z~ of the row under the call-wide tau
    double* row_nm;     // [B][R]
    double* row_ht;     // [B][R]  Shannon entropy of the target row   (DSD_H_ROW)
    double* row_hd;     // [B][R]  Shannon entropy of the draft row    (DSD_H_ROW)
    double* part_x;     // [B][R][S][3] per-slice sum min(P_t, q), -sum P_t ln P_t, -sum q ln q
    int32_t* node_key;  // [B][k]
    double* part_z;     // [B][k][S]  per-node Z~ shares (tau_override only)
    int32_t* draw_row;  // [B]
    int32_t* draw_mode; // [B] 0 = target row (bonus), 1 = positive part of P - q
    double* draw_tau;   // [B]
    double* draw_z;     // [B]   Z~ of the softened target used for the draw
    double* part_res;   // [B][S]
    double* part_fb;    // [B][S]  mass of P itself (used when the positive part is all zero)
};

// What one pass over the rows has to know about the call.
struct SliceArgs {
    const float* logits;
    const float* qp;
    const int32_t* parent;   // [k] or NULL
    int k, V, S, top_m;
    float c_hi, c_lo;        // log2(e) / T as a two-float sum
    float a_hi, a_lo;        // 1 - tau as a two-float sum
    float t_hi, t_lo;        // tau as a two-float sum
    int soft;                // 1: accumulate the Z~ share (call-wide tau in (0, 1], no per-node override)
    int tau_is_one;          // the Z~ share is sum q
    int want_top;            // 1: top_m candidates wanted (the top-M reading of NormMatch)
};

#define EPL (SLICE / WAVE)       // ids per lane of a slice
// id of element j of a lane: with 16-byte loads a lane takes 4 consecutive ids of each 256-id piece
template <bool VEC>
__device__ __forceinline__ int slice_id(int base, int lane, int j) {
    return VEC ? base + (j >> 2) * (4 * WAVE) + lane * 4 + (j & 3) : base + j * WAVE + lane;
}
template <bool VEC>
__device__ __forceinline__ void slice_load(const float* __restrict__ row, int base, int V, int lane, float (&v)[EPL], float fill) {
    if (VEC) {      // row start and V are multiples of 4 ids: a 16-byte piece lies inside the row or outside
#pragma unroll
        for (int jj = 0; jj < EPL / 4; ++jj) {
            const int id0 = base + jj * (4 * WAVE) + lane * 4;
            float4 x = make_float4(fill, fill, fill, fill);
            if (id0 < V) x = *(const float4*)(row + id0);
            v[jj * 4] = x.x; v[jj * 4 + 1] = x.y; v[jj * 4 + 2] = x.z; v[jj * 4 + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int id = base + j * WAVE + lane;
            v[j] = id < V ? row[id] : fill;
        }
    }
}

// The slice's candidates for the row's top_m of one row kind: every id at or above a threshold that is
// known not to exceed the slice's own top_m-th largest value -- the top_m-th largest of the maxima of
// 16 (32 from top_m = 9 on) groups of lanes (those maxima are that many different ids at least that
// large).  Usually a dozen ids pass; they go out as (value, id) keys in no particular order, the row
// merge ranks them.  The comparisons leave wave-wide lane masks in scalar registers, so counting,
// positions and skipping the ids nobody passes cost no vector work.  If more than LCAP ids pass (many
// equal values), the slice's exact top_m instead, by rounds of a wave-wide maximum, equal values to
// the lower id.  Returns the number of keys written to out[].
template <bool VEC, bool FULL>
__device__ __forceinline__ int slice_candidates(const float (&v)[EPL], float lm, int base, int V, int lane, int top_m,
                                                u64* __restrict__ out) {
    // lm: the largest of this lane's values (ids inside the row only)
    const float thr = top_m <= 8 ? group_threshold<4, float>(lm, lane, top_m) : group_threshold<2, float>(lm, lane, top_m);
    int cnt = 0;                                          // wave-uniform
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
        const int id = slice_id<VEC>(base, lane, j);
        const unsigned long long m = __builtin_amdgcn_ballot_w64((FULL || id < V) && v[j] >= thr);
        if (m) {
            const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
            if (((m >> lane) & 1ull) && pos < LCAP) out[pos] = rank_key(v[j], id);
            cnt += __popcll(m);
        }
    }
    if (cnt <= LCAP) return cnt;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");    // the stores above land before the ones below
    u64 last = ~0ull;
    int n = 0;
    for (int round = 0; round < top_m; ++round) {
        u64 best = 0ull;
#pragma unroll
        for (int j = 0; j < EPL; ++j) {
            const int id = slice_id<VEC>(base, lane, j);
            const u64 key = (FULL || id < V) ? rank_key(v[j], id) : 0ull;
            best = (key < last && key > best) ? key : best;
        }
        last = wave_max_u(best);
        if (last == 0ull) break;                          // the slice ran out of ids
        if (lane == 0) out[round] = last;
        ++n;
    }
    return n;
}

// FULL: every id of the slice lies inside the row (all slices of a row but the last)
template <bool VEC, bool FULL>
__device__ __forceinline__ void slice_pass_body(const SliceArgs& p, const AcceptWs& ws, bool has_child) {
    const int s = blockIdx.x, r = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int R = p.k + 1;
    const size_t row = ((size_t)b * R + r) * p.V;
    const int base = s * SLICE;
    const size_t pidx = ((size_t)b * R + r) * p.S + s;
    float lv[EPL], qv[EPL];
    slice_load<VEC>(p.logits + row, base, p.V, lane, lv, -INFINITY);
    if (has_child) slice_load<VEC>(p.qp + row, base, p.V, lane, qv, 0.f);
    float lane_max = -INFINITY;                           // ids past V hold -inf
#pragma unroll
    for (int j = 0; j < EPL; ++j) lane_max = fmaxf(lane_max, lv[j]);
    const float lmax = wave_max_f(lane_max);
    const bool live = lmax > -INFINITY && lmax < INFINITY;
    const float ref = live ? lmax * p.c_hi : 0.f;         // the slice's reference exponent: one rounding; the merge uses this very float
    // x_v - ref = l c_hi - ref + l c_lo.  c_lo > 0, so a logit of -inf (a masked id, an id past V)
    // gives -inf, weight 0, without a test.
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    float x[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
        x[j] = fmaf(lv[j], p.c_lo, fmaf(lv[j], p.c_hi, -ref));
        acc[j & 3] += __builtin_amdgcn_exp2f(x[j]);
    }
    double sum = ((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]);
    sum = wave_sum_d(sum);
    if (lane == 0) {
        ws.part_m[pidx] = live ? ref : -INFINITY;
        ws.part_s[pidx] = live ? sum : 0.0;
    }
    if (!has_child) return;                               // a leaf's draft row is never read
    if (p.soft) {
        float zacc[4] = {0.f, 0.f, 0.f, 0.f};
        if (p.tau_is_one) {
#pragma unroll
            for (int j = 0; j < EPL; ++j) zacc[j & 3] += fmaxf(qv[j], 0.f);      // P_t^0 = 1 for every id; ids past V hold 0
        } else {
            // (1-tau) x + tau log2 q = x + tau (log2 q - x), x short for x_v - ref.  q = 0 gives -inf, weight 0
            // (t_lo > 0); so does a logit of -inf.  The hardware logarithm takes subnormal q for 0: if the
            // slice holds any (next to never), the library's logarithm does the pass again.
            bool subnormal = false;
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                subnormal = subnormal || __builtin_amdgcn_ballot_w64(__builtin_amdgcn_class(qv[j], 0x010 | 0x080)) != 0ull;
                const float lq = __builtin_amdgcn_logf(qv[j]);
                const float d = lq - fmaxf(x[j], -1.0e30f);       // finite also for a logit of -inf: no inf - inf below
                const float e = fmaf(p.t_hi, d, fmaf(p.t_lo, d, x[j]));
                zacc[j & 3] += __builtin_amdgcn_exp2f(e);
            }
            if (subnormal) {                              // wave-uniform
                zacc[0] = zacc[1] = zacc[2] = zacc[3] = 0.f;
#pragma unroll
                for (int j = 0; j < EPL; ++j) {
                    const float d = log2f(qv[j]) - fmaxf(x[j], -1.0e30f);
                    zacc[j & 3] += __builtin_amdgcn_exp2f(fmaf(p.t_hi, d, fmaf(p.t_lo, d, x[j])));
                }
            }
        }
        double z = ((double)zacc[0] + (double)zacc[1]) + ((double)zacc[2] + (double)zacc[3]);
        z = wave_sum_d(z);
        if (lane == 0) ws.part_zs[pidx] = live ? z : 0.0;
    }
    if (p.want_top) {
        float q_max = -INFINITY;
#pragma unroll
        for (int j = 0; j < EPL; ++j)
            if (FULL || slice_id<VEC>(base, lane, j) < p.V) q_max = fmaxf(q_max, qv[j]);
        const int n_t = slice_candidates<VEC, FULL>(lv, lane_max, base, p.V, lane, p.top_m, ws.part_top_t + pidx * LCAP);
        const int n_q = slice_candidates<VEC, FULL>(qv, q_max, base, p.V, lane, p.top_m, ws.part_top_q + pidx * LCAP);
        if (lane == 0) *(int2*)(ws.part_cnt + pidx * 2) = make_int2(n_t, n_q);
    }
}

// Does any node hang under row r?  One load per lane instead of a walk over the parent array.
__device__ __forceinline__ bool row_has_child(const int32_t* __restrict__ parent, int k, int r, int lane) {
    if (!parent) return r < k;                            // chain
    bool mine = false;
    for (int c = lane + 1; c <= k; c += WAVE) {
        int par = parent[c - 1];
        par = par < 0 ? 0 : (par > c - 1 ? c - 1 : par);
        mine = mine || par == r;
    }
    return __builtin_amdgcn_ballot_w64(mine) != 0ull;
}

// One wavefront per (slice, row, sequence).
template <bool VEC>
__global__ void __launch_bounds__(WAVE, 4) slice_pass_kernel(SliceArgs p, AcceptWs ws) {
    const bool has_child = row_has_child(p.parent, p.k, blockIdx.y, threadIdx.x);
    if ((blockIdx.x + 1) * SLICE <= p.V) slice_pass_body<VEC, true>(p, ws, has_child);
    else slice_pass_body<VEC, false>(p, ws, has_child);
}

// Row quantities of the other readings of the key rule (only launched when one is selected; needs
// the rows' log-sum-exp): per slice sum min(P_t, q), -sum P_t ln P_t, -sum q ln q (fp32 terms, fp64
// sums), then per row their totals: NormMatch := the overlap if asked for, and the two entropies.
__global__ void __launch_bounds__(TPB)
row_extra_kernel(const float* __restrict__ logits, const float* __restrict__ qp, AcceptWs ws, int R, int V, int S,
                 double inv_temp) {
    __shared__ double shd[TPB / WAVE];
    const int s = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
    const size_t row = ((size_t)b * R + r) * V;
    const double lse = ws.row_lse[(size_t)b * R + r];
    float ov = 0.f, ht = 0.f, hd = 0.f;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = s * SLICE + threadIdx.x + j * TPB;
        if (i < V) {
            const float ln_p = (float)((double)logits[row + i] * inv_temp - lse);
            const float p = expf(ln_p), q = qp[row + i];
            ov += fminf(p, q);
            if (p > 0.f) ht -= p * ln_p;
            if (q > 0.f) hd -= q * logf(q);
        }
    }
    const double sov = block_sum_d((double)ov, shd), sht = block_sum_d((double)ht, shd), shd_ = block_sum_d((double)hd, shd);
    if (threadIdx.x == 0) {
        double* o = ws.part_x + (((size_t)b * R + r) * S + s) * 3;
        o[0] = sov;
        o[1] = sht;
        o[2] = shd_;
    }
}
__global__ void __launch_bounds__(WAVE)
row_extra_merge_kernel(AcceptWs ws, int R, int S, int overlap_is_norm_match) {
    const int r = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const size_t ridx = (size_t)b * R + r;
    double ov = 0.0, ht = 0.0, hd = 0.0;
    for (int s = lane; s < S; s += WAVE) {
        const double* o = ws.part_x + (ridx * S + s) * 3;
        ov += o[0];
        ht += o[1];
        hd += o[2];
    }
    ov = wave_sum_d(ov);
    ht = wave_sum_d(ht);
    hd = wave_sum_d(hd);
    if (lane == 0) {
        if (overlap_is_norm_match) ws.row_nm[ridx] = ov;
        ws.row_ht[ridx] = ht;
        ws.row_hd[ridx] = hd;
    }
}

// Only with tau_override: node i's own Z~ = sum_v P_t(v)^(1-tau_i) q(v)^tau_i, per slice (skipped for tau_i = 0).
__global__ void __launch_bounds__(TPB)
node_z_kernel(const float* __restrict__ logits, const float* __restrict__ qp, const int32_t* __restrict__ parent,
              const float* __restrict__ tau_override, AcceptWs ws, int k, int V, int S, double inv_temp) {
    __shared__ double shd[TPB / WAVE];
    const int s = blockIdx.x, node = blockIdx.y + 1, b = blockIdx.z;
    const int R = k + 1;
    int p = parent ? parent[node - 1] : node - 1;
    p = p < 0 ? 0 : (p > node - 1 ? node - 1 : p);
    const size_t nidx = (size_t)b * k + node - 1;
    double tau = (double)tau_override[nidx];
    tau = tau < 0.0 ? 0.0 : (tau > 1.0 ? 1.0 : tau);
    if (tau == 0.0) return;     // P~ = P_t, Z~ = 1
    const size_t row = ((size_t)b * R + p) * V;
    const double lse = ws.row_lse[(size_t)b * R + p];
    float fz = 0.f;
    const int base = s * SLICE;
    const float ftau = (float)tau;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        if (i < V) fz += soft_weight_f((float)((double)logits[row + i] * inv_temp - lse), qp[row + i], ftau);
    }
    const double z = block_sum_d((double)fz, shd);
    if (threadIdx.x == 0) ws.part_z[nidx * S + s] = z;
}

// The top_m best keys of a row from its slices' candidate lists (LCAP slots each, cnt[2*l + kind] of
// them in use), by one wave, to out[0..top_m) (LDS), best first, 0 where the keys run out.  Same
// scheme as inside a slice: a lane's head is the best key of the lists it owns, the top_m-th largest
// group maximum of the heads bounds the answer from below, the few keys at or above it are ranked
// (every lane counts the keys above its own).  More than 64 such keys (few lists, many equal
// values): rounds of a wave-wide maximum.  A lane's lists are fetched whole, all loads in flight at once.
__device__ inline void merge_top_lists(const u64* __restrict__ lists, const int32_t* __restrict__ cnts, int kind, int n_lists,
                                       int top_m, int lane, u64* __restrict__ cand, u64* __restrict__ out) {
    u64 h = 0ull;
    for (int l = lane; l < n_lists; l += WAVE) {
        const int n = cnts[2 * l + kind];
        const ulonglong2* src = (const ulonglong2*)(lists + (size_t)l * LCAP);
        ulonglong2 kk[LCAP / 2];
#pragma unroll
        for (int i = 0; i < LCAP / 2; ++i) kk[i] = src[i];
#pragma unroll
        for (int i = 0; i < LCAP / 2; ++i) {
            const u64 a = 2 * i < n ? kk[i].x : 0ull, c = 2 * i + 1 < n ? kk[i].y : 0ull;
            h = a > h ? a : h;
            h = c > h ? c : h;
        }
    }
    const u64 thr = top_m <= 8 ? group_threshold<4, u64>(h, lane, top_m) : group_threshold<2, u64>(h, lane, top_m);
    int cnt = 0;
    for (int l0 = 0; l0 < n_lists; l0 += WAVE) {
        const int l = l0 + lane;
        const int n = l < n_lists ? cnts[2 * l + kind] : 0;
        const ulonglong2* src = (const ulonglong2*)(lists + (size_t)(l < n_lists ? l : 0) * LCAP);
        ulonglong2 kk[LCAP / 2];
#pragma unroll
        for (int i = 0; i < LCAP / 2; ++i) kk[i] = src[i];
#pragma unroll
        for (int i = 0; i < LCAP; ++i) {
            const u64 key = i < n ? ((i & 1) ? kk[i / 2].y : kk[i / 2].x) : 0ull;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(key != 0ull && key >= thr);
            if (m) {
                const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                if (((m >> lane) & 1ull) && pos < WAVE) cand[pos] = key;
                cnt += __popcll(m);
            }
        }
    }
    wave_lds_sync();
    if (cnt <= WAVE) {
        rank_out(cand, cnt, top_m, lane, out);
    } else {
        u64 last = ~0ull;
        for (int round = 0; round < top_m; ++round) {
            u64 best = 0ull;
            for (int l = lane; l < n_lists; l += WAVE) {
                const int n = cnts[2 * l + kind];
                for (int i = 0; i < n; ++i) {
                    const u64 key = lists[(size_t)l * LCAP + i];
                    best = (key < last && key > best) ? key : best;
                }
            }
            last = wave_max_u(best);
            if (lane == 0) out[round] = last;
            if (last == 0ull) last = 1ull;
        }
    }
    __syncthreads();
}

struct SeqArgs {
    const float* logits;
    const float* qp;
    const int32_t* tokens;
    const int32_t* parent;
    const float* uniforms;
    dsd_accept_params prm;
    int k, V, S;
    double c;                // log2(e) / T exactly as slice_pass used it: (double)c_hi + (double)c_lo
    int walk;                // 0: lossless mode -- key flags only; the walk kernel does the rest
    int32_t* accepted_len;
    int32_t* accepted_path;
    dsd_accept_stats st;
};

// Sequence b by one workgroup of nt threads (all of them call; nt >= 64): thread i takes node i
// (0 = the root): key rule, tau_i, P(y), the test u q(y) < P(y), statistics; then every node walks
// up to the root for its depth and for whether it and all its ancestors passed; thread 0 picks the
// accepted path and what the extra token is drawn from.  The tree lives in LDS.
struct SeqLds {
    int par[DSD_MAX_K + 1], acc[DSD_MAX_K + 1], dep[DSD_MAX_K + 1], ok[DSD_MAX_K + 1];
    double tau[DSD_MAX_K + 1], z[DSD_MAX_K + 1];
};
__device__ inline void seq_body(const SeqArgs& p, const AcceptWs& ws, SeqLds& L, int b, int tid, int nt) {
    const int k = p.k, R = k + 1, S = p.S;
    for (int i = tid; i <= k; i += nt) {
        int pr = 0;
        if (i > 0) {
            pr = p.parent ? p.parent[i - 1] : i - 1;
            pr = pr < 0 ? 0 : (pr > i - 1 ? i - 1 : pr);
        }
        L.par[i] = pr;
    }
    __syncthreads();
    for (int i = tid; i <= k; i += nt) {
        if (i == 0) {
            L.acc[0] = 1;
            continue;
        }
        const int pr = L.par[i];
        const size_t nidx = (size_t)b * k + i - 1, ridx = (size_t)b * R + pr;
        int y = p.tokens[nidx];
        y = y < 0 ? 0 : (y >= p.V ? p.V - 1 : y);
        const size_t row = ridx * p.V;
        const double lse = ws.row_lse[ridx];
        const double ln_pt = (double)p.logits[row + y] * p.c * 0.6931471805599453094 - lse;
        const double pt_y = exp(ln_pt);
        const double q_y = (double)p.qp[row + y];
        const double nm = ws.row_nm[ridx];
        // key-token rule: any of the three criteria
        double h_t = -ln_pt, h_d = -log(q_y);
        if (p.prm.entropy_kind == DSD_H_ROW) {
            h_t = ws.row_ht[ridx];
            h_d = ws.row_hd[ridx];
        }
        const bool key = (h_d > p.prm.lambda1 * h_t) || (fabs(pt_y - q_y) > p.prm.lambda2) || (nm < p.prm.lambda3);
        double tau = key ? 0.0 : p.prm.tau;
        double z = (tau == 0.0) ? 1.0 : ws.row_z[ridx];
        if (p.prm.tau_override) {
            tau = (double)p.prm.tau_override[nidx];
            tau = tau < 0.0 ? 0.0 : (tau > 1.0 ? 1.0 : tau);
            z = 1.0;
            if (tau != 0.0) {
                z = 0.0;
                for (int s = 0; s < S; ++s) z += ws.part_z[nidx * S + s];
            }
        }
        ws.node_key[nidx] = key ? 1 : 0;
        if (p.walk) {
            const double p_y = soft_weight(ln_pt, q_y, tau) / z;
            const double u = (double)p.uniforms[(size_t)b * R + i];
            const bool a = u * q_y < p_y;
            L.acc[i] = a ? 1 : 0;
            L.tau[i] = tau;
            L.z[i] = z;
            if (p.st.key_flags) p.st.key_flags[nidx] = key ? 1 : 0;
            if (p.st.node_accept) p.st.node_accept[nidx] = a ? 1 : 0;
            if (p.st.ratio) p.st.ratio[nidx] = q_y > 0.0 ? p_y / q_y : (p_y > 0.0 ? INFINITY : 0.0);
            if (p.st.norm_match) p.st.norm_match[nidx] = nm;
        }
    }
    if (!p.walk) return;
    if (p.accepted_path)
        for (int i = tid; i < k; i += nt) p.accepted_path[(size_t)b * k + i] = -1;
    __syncthreads();
    for (int i = tid; i <= k; i += nt) {
        int d = 0, good = L.acc[i];
        for (int n = i; n != 0; n = L.par[n]) {        // parents precede children: at most k steps
            ++d;
            good &= L.acc[L.par[n]];
        }
        L.dep[i] = d;
        L.ok[i] = good;
    }
    __syncthreads();
    if (tid != 0) return;
    int vstar = 0;
    if (p.prm.tree_mode == DSD_TREE_FIRST_ACCEPTED) {
        for (;;) {
            int nxt = 0;
            for (int c = vstar + 1; c <= k; ++c)
                if (L.par[c] == vstar && L.acc[c]) { nxt = c; break; }
            if (!nxt) break;
            vstar = nxt;
        }
    } else {
        for (int c = 1; c <= k; ++c)
            if (L.ok[c] && L.dep[c] > L.dep[vstar]) vstar = c;
    }
    const int a = L.dep[vstar];
    p.accepted_len[b] = a;
    if (p.accepted_path)
        for (int n = vstar, j = a - 1; n != 0; n = L.par[n], --j) p.accepted_path[(size_t)b * k + j] = n;
    int child = 0;
    for (int c = vstar + 1; c <= k; ++c)
        if (L.par[c] == vstar) { child = c; break; }
    ws.draw_row[b] = vstar;
    if (!child) {
        ws.draw_mode[b] = 0;
        ws.draw_tau[b] = 0.0;
        ws.draw_z[b] = 1.0;
    } else {
        ws.draw_mode[b] = 1;
        ws.draw_tau[b] = L.tau[child];
        ws.draw_z[b] = L.z[child];
    }
}

#define SEQ_TPB 128
#define DECIDE_TPB 128
__global__ void __launch_bounds__(SEQ_TPB) seq_kernel(SeqArgs p, AcceptWs ws) {
    __shared__ SeqLds L;
    seq_body(p, ws, L, blockIdx.x, threadIdx.x, SEQ_TPB);
}

struct RowArgs {
    const int32_t* parent;
    int k, S, top_m;
    double a;                // 1 - tau of the call
    int soft, want_top;
};

// The same for a row of at most 64 slices whose lists already sit in registers, lane l holding the
// n keys kk[] of slice l (0 beyond its list).
__device__ inline void merge_top_regs(const u64 (&key)[LCAP], int top_m, int lane, u64* __restrict__ cand, u64* __restrict__ out) {
    u64 h = 0ull;
#pragma unroll
    for (int i = 0; i < LCAP; ++i) h = key[i] > h ? key[i] : h;
    const u64 thr = top_m <= 8 ? group_threshold<4, u64>(h, lane, top_m) : group_threshold<2, u64>(h, lane, top_m);
    int cnt = 0;
#pragma unroll
    for (int i = 0; i < LCAP; ++i) {
        const unsigned long long m = __builtin_amdgcn_ballot_w64(key[i] != 0ull && key[i] >= thr);
        if (m) {
            const int pos = cnt + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
            if (((m >> lane) & 1ull) && pos < WAVE) cand[pos] = key[i];
            cnt += __popcll(m);
        }
    }
    wave_lds_sync();
    if (cnt <= WAVE) {
        rank_out(cand, cnt, top_m, lane, out);
    } else {
        u64 last = ~0ull;
        for (int round = 0; round < top_m; ++round) {
            u64 best = 0ull;
#pragma unroll
            for (int i = 0; i < LCAP; ++i) best = (key[i] < last && key[i] > best) ? key[i] : best;
            last = wave_max_u(best);
            if (lane == 0) out[round] = last;
            if (last == 0ull) last = 1ull;
        }
    }
    wave_lds_sync();
}

// One workgroup of three wavefronts per (row, sequence): wave 0 forms the log-sum-exp from the slice
// partials and Z~ of the row under the call-wide tau, waves 1 and 2 the row's top_m of the logits and of
// the draft row from the slices' candidate lists (NormMatch).  With at most 64 slices (a vocabulary of
// up to 131072 ids) lane l takes slice l and everything a wave needs is requested before anything is
// waited for: one round trip to memory and a few microseconds of arithmetic, the three side by side.
#define ROW_TPB (3 * WAVE)
__global__ void __launch_bounds__(ROW_TPB) row_merge_kernel(RowArgs p, AcceptWs ws) {
    __shared__ u64 cand[2][WAVE], top[2][MAXM];
    const int r = blockIdx.x, b = blockIdx.y, lane = threadIdx.x & (WAVE - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int R = p.k + 1, S = p.S;
    const size_t ridx = (size_t)b * R + r;
    const bool one = S <= WAVE;
    const int sl = lane < S ? lane : 0;
    double lse2 = 0.0, z = 1.0;
    if (wave == 0) {
        float ms1 = -INFINITY;
        double ss1 = 0.0, zs1 = 0.0;
        if (one) {                                        // requests first
            ms1 = ws.part_m[ridx * S + sl];
            ss1 = ws.part_s[ridx * S + sl];
            if (p.soft) zs1 = ws.part_zs[ridx * S + sl];
            if (lane >= S) ms1 = -INFINITY;
        }
        const bool has_child = row_has_child(p.parent, p.k, r, lane);
        float mf = -INFINITY;
        if (one) mf = ms1;
        else
            for (int s = lane; s < S; s += WAVE) mf = fmaxf(mf, ws.part_m[ridx * S + s]);
        mf = wave_max_f(mf);
        const double m = (double)mf;
        double sum = 0.0;
        if (one) {
            if (ms1 > -INFINITY) sum = ss1 * exp2((double)ms1 - m);
        } else {
            for (int s = lane; s < S; s += WAVE) {
                const float ms = ws.part_m[ridx * S + s];
                if (ms > -INFINITY) sum += ws.part_s[ridx * S + s] * exp2((double)ms - m);
            }
        }
        sum = wave_sum_d(sum);
        lse2 = m + log2(sum);                             // log2 of sum_v 2^(x_v)
        if (has_child && p.soft) {
            z = 0.0;
            if (one) {
                if (ms1 > -INFINITY) z = zs1 * (p.a == 0.0 ? 1.0 : exp2(p.a * ((double)ms1 - lse2)));
            } else {
                for (int s = lane; s < S; s += WAVE) {
                    const float ms = ws.part_m[ridx * S + s];
                    if (ms > -INFINITY) z += ws.part_zs[ridx * S + s] * (p.a == 0.0 ? 1.0 : exp2(p.a * ((double)ms - lse2)));
                }
            }
            z = wave_sum_d(z);
        }
    } else if (p.want_top) {
        const int kind = wave - 1;
        const u64* lists = (kind ? ws.part_top_q : ws.part_top_t) + ridx * S * LCAP;
        const int32_t* cnts = ws.part_cnt + ridx * S * 2;
        int n1 = 0;
        ulonglong2 kk[LCAP / 2];
        if (one) {                                        // requests first
            n1 = cnts[2 * sl + kind];
            const ulonglong2* src = (const ulonglong2*)(lists + (size_t)sl * LCAP);
#pragma unroll
            for (int i = 0; i < LCAP / 2; ++i) kk[i] = src[i];
        }
        if (row_has_child(p.parent, p.k, r, lane)) {      // wave-uniform
            if (one) {
                u64 key[LCAP];
                const int n = lane < S ? n1 : 0;
#pragma unroll
                for (int i = 0; i < LCAP; ++i) key[i] = i < n ? ((i & 1) ? kk[i / 2].y : kk[i / 2].x) : 0ull;
                merge_top_regs(key, p.top_m, lane, cand[kind], top[kind]);
            } else {
                merge_top_lists(lists, cnts, kind, S, p.top_m, lane, cand[kind], top[kind]);
            }
        } else if (lane < MAXM) {
            top[kind][lane] = 0ull;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    double nm = 0.0;
    if (p.want_top) {
        const u64 mine = lane < p.top_m ? top[0][lane] : 0ull;
        bool hit = false;
        for (int j = 0; j < p.top_m; ++j) {
            const u64 o = top[1][j];
            hit = hit || (mine != 0ull && o != 0ull && key_id(o) == key_id(mine));
        }
        nm = (double)__popcll(__ballot(hit)) / (double)p.top_m;
    }
    if (lane == 0) {
        ws.row_lse[ridx] = lse2 * 0.6931471805599453094;          // natural log
        ws.row_z[ridx] = z;
        if (p.want_top) ws.row_nm[ridx] = nm;
    }
}

// weight of id i in the distribution the extra token is drawn from; also P itself
__device__ inline void draw_weight(const float* __restrict__ logits, const float* __restrict__ qp, size_t row, int i,
                                   double inv_temp, double lse, int mode, double tau, double inv_z, double* w,
                                   double* p) {
    const float ln_pt = (float)((double)logits[row + i] * inv_temp - lse);
    if (mode == 0) {
        *p = (double)expf(ln_pt);
        *w = *p;
    } else {
        const float q = qp[row + i];
        *p = (double)soft_weight_f(ln_pt, q, (float)tau) * inv_z;
        *w = fmax(*p - (double)q, 0.0);
    }
}

// Workgroup (slice, sequence): the slice's mass under the distribution the extra token is drawn from.
__global__ void __launch_bounds__(TPB)
draw_parts_kernel(const float* __restrict__ logits, const float* __restrict__ qp, AcceptWs ws, int R, int V, int S,
                  double inv_temp) {
    __shared__ double shd[TPB / WAVE];
    const int s = blockIdx.x, b = blockIdx.y;
    const int r = ws.draw_row[b], mode = ws.draw_mode[b];
    const double tau = ws.draw_tau[b], inv_z = 1.0 / ws.draw_z[b];   // one division per thread, a product per id
    const size_t row = ((size_t)b * R + r) * V;
    const double lse = ws.row_lse[(size_t)b * R + r];
    double sw = 0.0, sp = 0.0;
    const int base = s * SLICE;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        if (i < V) {
            double w, p;
            draw_weight(logits, qp, row, i, inv_temp, lse, mode, tau, inv_z, &w, &p);
            sw += w;
            sp += p;
        }
    }
    sw = block_sum_d(sw, shd);
    sp = block_sum_d(sp, shd);
    if (threadIdx.x == 0) {
        ws.part_res[(size_t)b * S + s] = sw;
        ws.part_fb[(size_t)b * S + s] = sp;
    }
}

// One workgroup per sequence: the extra token from the slice masses: the slice whose cumulative mass
// crosses u_0 * total, then the id inside it (that slice's weights once more).
__global__ void __launch_bounds__(TPB)
draw_pick_kernel(const float* __restrict__ logits, const float* __restrict__ qp, const float* __restrict__ uniforms,
                 AcceptWs ws, int R, int V, int S, double inv_temp, int32_t* __restrict__ next_token) {
    __shared__ double pre[TPB / WAVE];
    __shared__ int sh_slice, sh_fallback, sh_best[TPB / WAVE], sh_last[TPB / WAVE];
    __shared__ double sh_before, sh_target;
    const int b = blockIdx.x;
    const int r = ws.draw_row[b], mode = ws.draw_mode[b];
    const double tau = ws.draw_tau[b], inv_z = 1.0 / ws.draw_z[b];   // one division per thread, a product per id
    const size_t row = ((size_t)b * R + r) * V;
    const double lse = ws.row_lse[(size_t)b * R + r];
    if (threadIdx.x < WAVE) {
        // wave 0: total mass, then the first slice whose inclusive cumulative mass exceeds u0 * total
        const int lane = threadIdx.x;
        const double* part = ws.part_res + (size_t)b * S;
        double total = 0.0;
        for (int s = lane; s < S; s += WAVE) total += part[s];
        total = wave_sum_d(total);
        int fb = 0;
        if (!(total > 0.0)) {      // positive part empty: draw from P itself
            fb = 1;
            part = ws.part_fb + (size_t)b * S;
            total = 0.0;
            for (int s = lane; s < S; s += WAVE) total += part[s];
            total = wave_sum_d(total);
        }
        const double target = (double)uniforms[(size_t)b * R] * total;
        double carry = 0.0;
        int pick = -1, last_pos = 0;
        double before = 0.0;
        for (int s0 = 0; s0 < S; s0 += WAVE) {
            const int s = s0 + lane;
            const double v = s < S ? part[s] : 0.0;
            double inc = v;                                   // inclusive scan over the 64 lanes
#pragma unroll
            for (int o = 1; o < WAVE; o <<= 1) {
                const double t = __shfl_up(inc, o, WAVE);
                if (lane >= o) inc += t;
            }
            inc += carry;
            const unsigned long long pos = __ballot(v > 0.0);
            if (pos) last_pos = s0 + 63 - __clzll(pos);
            const unsigned long long hit = __ballot(s < S && inc > target);
            if (pick < 0 && hit) {
                const int l = __ffsll((long long)hit) - 1;
                pick = s0 + l;
                before = __shfl(inc - v, l, WAVE);
            }
            carry = __shfl(inc, WAVE - 1, WAVE);
        }
        if (lane == 0) {
            if (pick < 0) {        // rounding left no crossing: last id with positive weight
                pick = last_pos;
                before = -1.0;     // marks "take the last positive id of the slice"
            }
            sh_slice = pick;
            sh_before = before;
            sh_fallback = fb;
            sh_target = target;
        }
    }
    __syncthreads();
    const int s = sh_slice, fb = sh_fallback;
    const double target = sh_target, before = sh_before;
    // thread t owns ids [base + t*EPT, base + (t+1)*EPT), in id order
    const int base = s * SLICE + threadIdx.x * EPT;
    double w[EPT], loc = 0.0;
    int lastpos = -1;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + j;
        w[j] = 0.0;
        if (i < V) {
            double ww, pp;
            draw_weight(logits, qp, row, i, inv_temp, lse, mode, tau, inv_z, &ww, &pp);
            w[j] = fb ? pp : ww;
            if (w[j] > 0.0) lastpos = i;
        }
        loc += w[j];
    }
    // mass before this thread's ids: scan over the lanes of a wave, then the waves before it, in thread order
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    double inc = loc;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
        const double t = __shfl_up(inc, o, WAVE);
        if (lane >= o) inc += t;
    }
    if (lane == WAVE - 1) pre[wave] = inc;
    __syncthreads();
    double start = before < 0.0 ? 0.0 : before;
    for (int i = 0; i < wave; ++i) start += pre[i];
    start += inc - loc;
    int found = 0x7FFFFFFF;
    if (before >= 0.0) {
        double c = start;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            c += w[j];
            if (c > target && base + j < V && found == 0x7FFFFFFF) found = base + j;
        }
    }
    // block minimum of `found`, block maximum of `lastpos`
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        found = min(found, __shfl_xor(found, o, WAVE));
        lastpos = max(lastpos, __shfl_xor(lastpos, o, WAVE));
    }
    if ((threadIdx.x & (WAVE - 1)) == 0) {
        sh_best[threadIdx.x / WAVE] = found;
        sh_last[threadIdx.x / WAVE] = lastpos;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int f = 0x7FFFFFFF, l = -1;
        for (int i = 0; i < TPB / WAVE; ++i) {
            f = min(f, sh_best[i]);
            l = max(l, sh_last[i]);
        }
        int tok = (f != 0x7FFFFFFF) ? f : l;
        if (tok < 0) tok = min(V - 1, s * SLICE);
        next_token[b] = tok;
    }
}

// ---------------------------------------------------------------------------- DSD_TREE_LOSSLESS
// Recursive rejection over siblings drawn without replacement (see dsd.h).  One workgroup per
// sequence walks down the tree; what it carries at a node after n rejected children is the chain
//     p_{j+1}(id) = max(0, p_j(id) - q_j(id)) / Z_j,   q_j(id) = [id not among y_0..y_{j-1}] q(id) / (1 - R_j)
// with Z_j the sum of the positive parts and R_j the draft mass of the removed tokens, so that any
// p_n(id) is a few operations on the two rows and 2n stored scalars.  A child's test evaluates the
// chain for its own token in fp64; a rejection costs one pass of the workgroup over the vocabulary
// (fp32 terms, fp64 sum) for the next Z; the additional token costs one pass for the per-thread
// masses of contiguous id ranges, a scan, and a rescan of one range.
#define WALK_TPB 1024
struct WalkChain {
    int n;                            // rejections so far at this node
    const int* y;                     // [n] removed tokens
    const float* inv_z;               // [n] 1/Z_j, 0 = "p_j equals q_j: keep p"
    const float* q_scale;             // [n+1] 1/(1 - R_j), 0 when the draft row is used up
};
__device__ inline float walk_p(const WalkChain& c, float p1, float q1, int id, float* q_n) {
    float p = p1;
    bool removed = false;
    for (int j = 0; j < c.n; ++j) {
        const float qj = removed ? 0.f : q1 * c.q_scale[j];
        if (c.inv_z[j] > 0.f) p = fmaxf(p - qj, 0.f) * c.inv_z[j];
        removed = removed || id == c.y[j];
    }
    *q_n = removed ? 0.f : q1 * c.q_scale[c.n];
    return p;
}

// sum over the WALK_TPB threads of the workgroup, to every thread (red: WALK_TPB / WAVE doubles of LDS)
__device__ inline double walk_block_sum(double v, double* red, int lane, int wave) {
    v = wave_sum_d(v);
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double tot = 0.0;
    for (int i = 0; i < WALK_TPB / WAVE; ++i) tot += red[i];
    return tot;
}
// the chain of walk_p in fp64
__device__ inline double walk_p_d(int n, const int* y, const double* inv_z, const double* q_scale, double p1, double q1, int id,
                                  double* q_n) {
    double p = p1;
    bool removed = false;
    for (int j = 0; j < n; ++j) {
        const double qj = removed ? 0.0 : q1 * q_scale[j];
        if (inv_z[j] > 0.0) p = fmax(p - qj, 0.0) * inv_z[j];
        removed = removed || id == y[j];
    }
    *q_n = removed ? 0.0 : q1 * q_scale[n];
    return p;
}

// A residual mass below this is summed again in fp64 (see the walk)
#define WALK_SMALL_Z 0.05

__global__ void __launch_bounds__(WALK_TPB)
lossless_walk_kernel(const float* __restrict__ logits, const float* __restrict__ qp, const int32_t* __restrict__ tokens,
                     const int32_t* __restrict__ parent, const float* __restrict__ uniforms, AcceptWs ws, int k, int V,
                     double inv_temp, int32_t* __restrict__ accepted_len, int32_t* __restrict__ next_token,
                     int32_t* __restrict__ accepted_path, dsd_accept_stats st) {
    __shared__ int s_par[DSD_MAX_K + 1], s_y[DSD_MAX_K];
    __shared__ float s_inv_z[DSD_MAX_K], s_q_scale[DSD_MAX_K + 1];
    __shared__ double s_inv_z_d[DSD_MAX_K], s_q_scale_d[DSD_MAX_K + 1];
    __shared__ double s_red[WALK_TPB / WAVE];
    __shared__ double s_wave_tot[WALK_TPB / WAVE];
    __shared__ int s_pick[2];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int R = k + 1;
    for (int i = tid; i <= k; i += WALK_TPB) {
        int p = 0;
        if (i > 0) {
            p = parent ? parent[i - 1] : i - 1;
            p = p < 0 ? 0 : (p > i - 1 ? i - 1 : p);
            const size_t nidx = (size_t)b * k + i - 1;
            if (st.key_flags) st.key_flags[nidx] = ws.node_key[nidx];
            if (st.norm_match) st.norm_match[nidx] = ws.row_nm[(size_t)b * R + p];
            if (st.node_accept) st.node_accept[nidx] = 0;
            if (st.ratio) st.ratio[nidx] = 0.0;
            if (accepted_path) accepted_path[nidx] = -1;
        }
        s_par[i] = p;
    }
    if (tid == 0) {
        s_q_scale[0] = 1.f;
        s_q_scale_d[0] = 1.0;
    }
    __syncthreads();

    int v = 0, a = 0, n = 0;
    size_t row = (size_t)b * R * V;
    double lse = ws.row_lse[(size_t)b * R];
    for (;;) {                                        // one turn per node on the path; all branches are uniform
        row = ((size_t)b * R + v) * V;
        lse = ws.row_lse[(size_t)b * R + v];
        n = 0;
        double removed_mass = 0.0;
        double norm = 1.0;                            // 1 / sum_v exp(l_v / T - lse) in fp64, once a small Z asks for it
        bool have_norm = false;
        int taken = 0;
        for (int c = v + 1; c <= k && !taken; ++c) {
            if (s_par[c] != v) continue;
            int y = tokens[(size_t)b * k + c - 1];
            y = y < 0 ? 0 : (y >= V ? V - 1 : y);
            // the child's own test, fp64, by every thread alike
            double p = exp((double)logits[row + y] * inv_temp - lse) * norm;
            const double q1 = (double)qp[row + y];
            bool removed = false;
            for (int j = 0; j < n; ++j) {
                const double qj = removed ? 0.0 : q1 * s_q_scale_d[j];
                if (s_inv_z_d[j] > 0.0) p = fmax(p - qj, 0.0) * s_inv_z_d[j];
                removed = removed || y == s_y[j];
            }
            const double qn = removed ? 0.0 : q1 * s_q_scale_d[n];
            const double u = (double)uniforms[(size_t)b * R + c];
            const bool acc = u * qn < p;
            if (tid == 0) {
                const size_t nidx = (size_t)b * k + c - 1;
                if (st.node_accept) st.node_accept[nidx] = acc ? 1 : 0;
                if (st.ratio) st.ratio[nidx] = qn > 0.0 ? p / qn : (p > 0.0 ? INFINITY : 0.0);
            }
            if (acc) {
                taken = c;
                break;
            }
            // rejected: Z_n = sum of the positive part of p_n - q_n
            double tot = 0.0;
            if (!have_norm) {                         // (after a small Z at this node every later one is summed in fp64)
                WalkChain ch{n, s_y, s_inv_z, s_q_scale};
                double z = 0.0;
                const bool vec = (V & 3) == 0 && (row & 3) == 0;      // rows start 16-byte aligned
                const int step = vec ? 4 : 1;
                for (int id = tid * step; id < V; id += WALK_TPB * step) {
                    float lv[4], qv[4];
                    if (vec) {
                        const float4 l4 = *(const float4*)(logits + row + id), q4 = *(const float4*)(qp + row + id);
                        lv[0] = l4.x; lv[1] = l4.y; lv[2] = l4.z; lv[3] = l4.w;
                        qv[0] = q4.x; qv[1] = q4.y; qv[2] = q4.z; qv[3] = q4.w;
                    } else {
                        lv[0] = logits[row + id];
                        qv[0] = qp[row + id];
                    }
                    float zf = 0.f;                                   // at most 4 terms: exact enough before the fp64 sum
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (e < step) {
                            const float p1 = expf((float)((double)lv[e] * inv_temp - lse));
                            float qn_id;
                            const float pn = walk_p(ch, p1, qv[e], id + e, &qn_id);
                            zf += fmaxf(pn - qn_id, 0.f);
                        }
                    }
                    z += (double)zf;
                }
                tot = walk_block_sum(z, s_red, lane, wave);
            }
            if (have_norm || tot < WALK_SMALL_Z) {    // workgroup-uniform
                // Target and draft nearly coincide here (a good draft on peaked rows): the next sibling's p is
                // the residual divided by this small Z, so the absolute error of the fp32 terms (1e-7 of p)
                // and of the row's log-sum-exp would show up 1/Z times larger, here and, through the differences
                // p - q inside the chain, in every later Z of this node.  In fp64, with the row renormalised by its
                // own fp64 sum.
                if (!have_norm) {
                    double s1 = 0.0;
                    for (int id = tid; id < V; id += WALK_TPB) s1 += exp((double)logits[row + id] * inv_temp - lse);
                    s1 = walk_block_sum(s1, s_red, lane, wave);
                    norm = s1 > 0.0 ? 1.0 / s1 : 1.0;
                    have_norm = true;
                }
                double z64 = 0.0;
                for (int id = tid; id < V; id += WALK_TPB) {
                    const double p1 = exp((double)logits[row + id] * inv_temp - lse) * norm;
                    double qn_id;
                    const double pn = walk_p_d(n, s_y, s_inv_z_d, s_q_scale_d, p1, (double)qp[row + id], id, &qn_id);
                    z64 += fmax(pn - qn_id, 0.0);
                }
                tot = walk_block_sum(z64, s_red, lane, wave);
            }
            __syncthreads();                          // everyone is done with the chain arrays
            if (tid == 0) {
                const double iz = tot > 0.0 ? 1.0 / tot : 0.0;
                if (!removed) removed_mass += q1;
                const double left = 1.0 - removed_mass;
                const double qs = left > 0.0 ? 1.0 / left : 0.0;
                s_y[n] = y;
                s_inv_z_d[n] = iz;
                s_inv_z[n] = (float)iz;
                s_q_scale_d[n + 1] = qs;
                s_q_scale[n + 1] = (float)qs;
            }
            // removed_mass lives in thread 0 only; the others never read it
            ++n;
            __syncthreads();
        }
        if (!taken) break;
        if (tid == 0 && accepted_path) accepted_path[(size_t)b * k + a] = taken;
        ++a;
        v = taken;
    }

    // The additional token: inverse CDF over p_n of row v in token-id order with u_0.  Wave w owns
    // the contiguous ids [w*span, (w+1)*span), read 64 at a time in lane order (coalesced): first the
    // mass of every wave's range, then the wave holding the crossing walks its range again in groups
    // of 64 ids, and the crossing group is resolved by a scan over its lanes.
    WalkChain ch{n, s_y, s_inv_z, s_q_scale};
    const int span = ((V + WALK_TPB / WAVE - 1) / (WALK_TPB / WAVE) + WAVE - 1) / WAVE * WAVE;
    const int w0 = wave * span, w1 = min(w0 + span, V);
    auto weight = [&](int id) -> float {
        const float p1 = expf((float)((double)logits[row + id] * inv_temp - lse));
        float qn_id;
        return walk_p(ch, p1, qp[row + id], id, &qn_id);
    };
    double mass = 0.0;
    int lastpos = -1;
    for (int id = w0 + lane; id < w1; id += WAVE) {
        const float pn = weight(id);
        mass += (double)pn;
        if (pn > 0.f) lastpos = id;
    }
    mass = wave_sum_d(mass);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, o, WAVE));
    if (lane == 0) s_wave_tot[wave] = mass;
    if (tid == 0) {
        s_pick[0] = 0x7FFFFFFF;
        s_pick[1] = -1;
    }
    __syncthreads();
    double before = 0.0, total = 0.0;
    for (int i = 0; i < WALK_TPB / WAVE; ++i) {
        if (i < wave) before += s_wave_tot[i];
        total += s_wave_tot[i];
    }
    const double target = (double)uniforms[(size_t)b * R] * total;
    if (lane == 0 && lastpos >= 0) atomicMax(&s_pick[1], lastpos);
    if (before <= target && target < before + mass) {     // the crossing lies in this wave's range (at most one wave)
        double c = before;
        int found = -1;
        for (int g0 = w0; g0 < w1 && found < 0; g0 += WAVE) {
            const int id = g0 + lane;
            const double wgt = id < w1 ? (double)weight(id) : 0.0;
            const double gsum = wave_sum_d(wgt);
            if (c + gsum > target) {
                double inc = wgt;                             // inclusive scan over the lanes
#pragma unroll
                for (int o = 1; o < WAVE; o <<= 1) {
                    const double t = __shfl_up(inc, o, WAVE);
                    if (lane >= o) inc += t;
                }
                const unsigned long long hit = __ballot(id < w1 && c + inc > target);
                if (hit) found = g0 + __ffsll((long long)hit) - 1;
            }
            c += gsum;
        }
        if (lane == 0 && found >= 0) atomicMin(&s_pick[0], found);
    }
    __syncthreads();
    if (tid == 0) {
        int tok = s_pick[0];
        if (tok == 0x7FFFFFFF) tok = s_pick[1] >= 0 ? s_pick[1] : 0;   // rounding left no crossing: last id with mass
        next_token[b] = tok;
        accepted_len[b] = a;
    }
}

// ---------------------------------------------------------------------------- temperature 0
// Greedy verification: the target is the one-hot on arg max logits (ties to the lower id).
// row_argmax: per (sequence, row, slice) the best (value, id) key; greedy_decide: per sequence the
// arg max of every row, the nodes whose token equals their parent's arg max, the path (as decide_kernel)
// and the arg max of the last node's row as the additional token.
__global__ void __launch_bounds__(TPB)
row_argmax_kernel(const float* __restrict__ logits, u64* __restrict__ part, int R, int V, int S) {
    __shared__ u64 shu[TPB / WAVE];
    const int s = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
    const size_t row = ((size_t)b * R + r) * V;
    u64 best = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = s * SLICE + threadIdx.x + j * TPB;
        if (i < V) {
            const u64 key = rank_key(logits[row + i], i);
            best = key > best ? key : best;
        }
    }
    best = block_max_u(best, shu);
    if (threadIdx.x == 0) part[((size_t)b * R + r) * S + s] = best;
}

__global__ void __launch_bounds__(DECIDE_TPB)
greedy_decide_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ parent, const u64* __restrict__ part,
                     int tree_mode, int k, int S, int32_t* __restrict__ accepted_len, int32_t* __restrict__ next_token,
                     int32_t* __restrict__ accepted_path, dsd_accept_stats st) {
    __shared__ int par[DSD_MAX_K + 1], acc[DSD_MAX_K + 1], dep[DSD_MAX_K + 1], ok[DSD_MAX_K + 1], amax[DSD_MAX_K + 1];
    const int b = blockIdx.x, i = threadIdx.x, R = k + 1;
    if (i <= k) {
        u64 best = 0;
        for (int s = 0; s < S; ++s) {
            const u64 key = part[((size_t)b * R + i) * S + s];
            best = key > best ? key : best;
        }
        amax[i] = key_id(best);
        int p = 0;
        if (i > 0) {
            p = parent ? parent[i - 1] : i - 1;
            p = p < 0 ? 0 : (p > i - 1 ? i - 1 : p);
        }
        par[i] = p;
    }
    if (accepted_path && i < k) accepted_path[(size_t)b * k + i] = -1;
    __syncthreads();
    if (i <= k) {
        const int a = i == 0 ? 1 : (tokens[(size_t)b * k + i - 1] == amax[par[i]] ? 1 : 0);
        acc[i] = a;
        if (i > 0) {
            const size_t nidx = (size_t)b * k + i - 1;
            if (st.node_accept) st.node_accept[nidx] = a;
            if (st.ratio) st.ratio[nidx] = a ? 1.0 : 0.0;
            if (st.key_flags) st.key_flags[nidx] = 0;
            if (st.norm_match) st.norm_match[nidx] = 0.0;
        }
    }
    __syncthreads();
    if (i <= k) {
        int d = 0, good = acc[i];
        for (int n = i; n != 0; n = par[n]) {
            ++d;
            good &= acc[par[n]];
        }
        dep[i] = d;
        ok[i] = good;
    }
    __syncthreads();
    if (i != 0) return;
    int vstar = 0;
    if (tree_mode == DSD_TREE_LONGEST) {
        for (int c = 1; c <= k; ++c)
            if (ok[c] && dep[c] > dep[vstar]) vstar = c;
    } else {
        for (;;) {
            int nxt = 0;
            for (int c = vstar + 1; c <= k; ++c)
                if (par[c] == vstar && acc[c]) { nxt = c; break; }
            if (!nxt) break;
            vstar = nxt;
        }
    }
    const int a = dep[vstar];
    accepted_len[b] = a;
    if (accepted_path)
        for (int n = vstar, j = a - 1; n != 0; n = par[n], --j) accepted_path[(size_t)b * k + j] = n;
    next_token[b] = amax[vstar];
}

// v > 0 as hi + lo with lo > 0 (hi rounded down): products of a -inf exponent with both parts then stay -inf
static void split_down(double v, float* hi, float* lo) {
    float h = (float)v;
    if (v > 0.0 && (double)h >= v) h = nextafterf(h, 0.0f);
    *hi = h;
    *lo = (float)(v - (double)h);
}

// Carves the scratch memory of one call out of [base, ...); returns the bytes used (base may be NULL to size it).
static size_t accept_carve(AcceptWs& ws, char* base, size_t B, size_t k, size_t S, size_t top_m) {
    const size_t BR = B * (k + 1), BK = B * k;
    WsBump bump{base, 0};
    ws.part_m = bump.take<float>(BR * S);
    ws.part_s = bump.take<double>(BR * S);
    ws.part_zs = bump.take<double>(BR * S);
    ws.part_top_t = bump.take<u64>(BR * S * LCAP);
    ws.part_top_q = bump.take<u64>(BR * S * LCAP);
    ws.part_cnt = bump.take<int32_t>(BR * S * 2);
    ws.row_lse = bump.take<double>(BR);
    ws.row_z = bump.take<double>(BR);
    ws.row_nm = bump.take<double>(BR);
    ws.row_ht = bump.take<double>(BR);
    ws.row_hd = bump.take<double>(BR);
    ws.part_x = bump.take<double>(BR * S * 3);
    ws.node_key = bump.take<int32_t>(BK);
    ws.part_z = bump.take<double>(BK * S);
    ws.draw_row = bump.take<int32_t>(B);
    ws.draw_mode = bump.take<int32_t>(B);
    ws.draw_tau = bump.take<double>(B);
    ws.draw_z = bump.take<double>(B);
    ws.part_res = bump.take<double>(B * S);
    ws.part_fb = bump.take<double>(B * S);
    return bump.off;
}

size_t accept_scratch_bytes(int B, int k, int V, int top_m) {
    AcceptWs ws;
    const size_t S = ((size_t)V + SLICE - 1) / SLICE;
    const size_t greedy = (size_t)B * (k + 1) * S * 8 + 256;
    const size_t full = accept_carve(ws, nullptr, B, k, S, top_m);
    return full > greedy ? full : greedy;
}

// ---------------------------------------------------------------------------- scratch that nobody allocates
// For callers that must not allocate (dsd_accept_noalloc): the partials of one call live in a fixed
// array in the library's device image.  Every GPU the library runs on holds its own copy, at its own
// address, until the process ends; the host-side name is only a handle, the address a kernel can use
// comes from hipGetSymbolAddress, once per device, when a context is created there.
#define ACCEPT_STATIC_SCRATCH_BYTES (8u << 20)
#define ACCEPT_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[ACCEPT_STATIC_SCRATCH_BYTES];
static char* g_static_scratch[ACCEPT_MAX_DEVICES];        // per device: device address of its copy of scratch[]

// Called by dsd_create with `device` current.
int accept_static_scratch_init(int device) {
    if (device < 0 || device >= ACCEPT_MAX_DEVICES) return DSD_OK;      // such a device simply has no static scratch
    if (g_static_scratch[device]) return DSD_OK;
    void* ptr = nullptr;
    DSD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) DSD_FAIL(DSD_EHIP, "hipGetSymbolAddress returned no address for the static scratch array");
    g_static_scratch[device] = (char*)ptr;
    return DSD_OK;
}
char* accept_static_scratch(int device, size_t* bytes) {
    *bytes = ACCEPT_STATIC_SCRATCH_BYTES;
    return (device >= 0 && device < ACCEPT_MAX_DEVICES) ? g_static_scratch[device] : nullptr;
}

// scratch_dev: device memory of at least accept_scratch_bytes(B, k, V, top_m) bytes, 256-byte aligned; its contents
// need not be cleared (every word read by a kernel was written by an earlier kernel of the same call)
int accept_launch(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                  const int32_t* parent, const float* uniforms, const dsd_accept_params* prm, int B, int k, int V,
                  int32_t* accepted_len, int32_t* next_token, int32_t* accepted_path, const dsd_accept_stats* stats,
                  char* scratch_dev) {
    const int R = k + 1;
    const int S = (V + SLICE - 1) / SLICE;
    hipStream_t s = ctx->stream;
    dsd_accept_stats st = {nullptr, nullptr, nullptr, nullptr};
    if (stats) st = *stats;
    if (B > 65535 || R > 65535) DSD_FAIL(DSD_ESHAPE, "dsd_accept: B=%d exceeds 65535", B);
    if (prm->temperature == 0.0) {
        u64* part = (u64*)scratch_dev;
        ProfScope ps(ctx, DSD_KC_ACCEPT);
        row_argmax_kernel<<<dim3(S, R, B), TPB, 0, s>>>(logits, part, R, V, S);
        greedy_decide_kernel<<<B, DECIDE_TPB, 0, s>>>(draft_tokens, parent, part, prm->tree_mode, k, S, accepted_len,
                                                     next_token, accepted_path, st);
        DSD_HIP(hipGetLastError());
        return DSD_OK;
    }
    AcceptWs ws;
    accept_carve(ws, scratch_dev, B, k, S, prm->top_m);
    const double inv_temp = 1.0 / prm->temperature;
    const bool lossless = prm->tree_mode == DSD_TREE_LOSSLESS;
    const bool variants = prm->norm_match_kind == DSD_NM_OVERLAP || prm->entropy_kind == DSD_H_ROW;
    const bool per_node_tau = prm->tau_override != nullptr && !lossless;

    SliceArgs sa;
    sa.logits = logits; sa.qp = draft_probs; sa.parent = parent; sa.k = k; sa.V = V; sa.S = S; sa.top_m = prm->top_m;
    const double tau = lossless ? 0.0 : prm->tau;         // no relaxation under the lossless tree rule
    split_down(1.4426950408889634074 * inv_temp, &sa.c_hi, &sa.c_lo);
    split_down(1.0 - tau, &sa.a_hi, &sa.a_lo);
    split_down(tau, &sa.t_hi, &sa.t_lo);
    sa.soft = (tau > 0.0 && !per_node_tau) ? 1 : 0;
    sa.tau_is_one = tau == 1.0 ? 1 : 0;
    sa.want_top = prm->norm_match_kind == DSD_NM_TOP_M ? 1 : 0;

    RowArgs ra;
    ra.parent = parent; ra.k = k; ra.S = S; ra.top_m = prm->top_m; ra.a = 1.0 - tau; ra.soft = sa.soft; ra.want_top = sa.want_top;

    SeqArgs q;
    q.logits = logits; q.qp = draft_probs; q.tokens = draft_tokens; q.parent = parent; q.uniforms = uniforms;
    q.prm = *prm;
    q.prm.tau = tau;
    if (lossless) q.prm.tau_override = nullptr;
    q.k = k; q.V = V; q.S = S; q.c = (double)sa.c_hi + (double)sa.c_lo;
    q.walk = lossless ? 0 : 1;
    q.accepted_len = accepted_len; q.accepted_path = accepted_path; q.st = st;

    const bool vec = (V & 3) == 0 && (((size_t)logits | (size_t)draft_probs) & 15) == 0;
    ProfScope ps(ctx, DSD_KC_ACCEPT);
    if (vec) slice_pass_kernel<true><<<dim3(S, R, B), WAVE, 0, s>>>(sa, ws);
    else slice_pass_kernel<false><<<dim3(S, R, B), WAVE, 0, s>>>(sa, ws);
    row_merge_kernel<<<dim3(R, B), ROW_TPB, 0, s>>>(ra, ws);
    if (variants) {
        row_extra_kernel<<<dim3(S, R, B), TPB, 0, s>>>(logits, draft_probs, ws, R, V, S, inv_temp);
        row_extra_merge_kernel<<<dim3(R, B), WAVE, 0, s>>>(ws, R, S, prm->norm_match_kind == DSD_NM_OVERLAP ? 1 : 0);
    }
    if (per_node_tau)
        node_z_kernel<<<dim3(S, k, B), TPB, 0, s>>>(logits, draft_probs, parent, prm->tau_override, ws, k, V, S, inv_temp);
    seq_kernel<<<B, SEQ_TPB, 0, s>>>(q, ws);
    if (lossless) {
        lossless_walk_kernel<<<B, WALK_TPB, 0, s>>>(logits, draft_probs, draft_tokens, parent, uniforms, ws, k, V, inv_temp,
                                                      accepted_len, next_token, accepted_path, st);
        DSD_HIP(hipGetLastError());
        return DSD_OK;
    }
    draw_parts_kernel<<<dim3(S, B), TPB, 0, s>>>(logits, draft_probs, ws, R, V, S, inv_temp);
    draw_pick_kernel<<<B, TPB, 0, s>>>(logits, draft_probs, uniforms, ws, R, V, S, inv_temp, next_token);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}
