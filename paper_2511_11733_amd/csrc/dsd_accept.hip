// Acceptance loop of Algorithm 1 (lines 2-16) with the key-token rule and the softened target
// of section 2.3, for B sequences at once.
//
// The vocabulary is cut into slices of SLICE ids; every vocabulary-wide quantity is reduced per
// slice by one workgroup (wavefront shuffles + one LDS hop), the few per-slice partials are
// merged by a small second kernel, and only those partials ever reach memory: no probability
// row is materialised.  Every quantity that decides something by itself (a drafted token's own
// probabilities, the accept test, all sums and cumulative sums) is fp64; the per-id terms of the
// vocabulary-wide sums are evaluated in fp32 (relative error below 1e-6, independent between ids,
// so that a sum over thousands of ids is good to about 1e-9) and accumulated in fp64.  The
// integer outputs therefore follow an fp64 reference except within the near-tie bands the tests
// state.
//
//   row_stats   per (sequence, row, slice): max and sum-exp of logits/T, top-M candidates of the
//               logits row and of the draft row
//   row_merge   per (sequence, row): log-sum-exp, NormMatch
//   node_soft   per (sequence, node, slice): key test -> tau_i; partial of
//               Z~ = sum_v P_t(v)^(1-tau_i) q(v)^tau_i   (skipped when tau_i = 0)
//   decide      per sequence: every node's test u*q(y) < P(y), accepted path, what to draw from
//   draw_parts  per (sequence, slice): partial mass of the distribution the extra token comes from
//   draw_pick   per sequence: inverse CDF in token-id order
#include "dsd_internal.h"

#define WAVE 64
#define SLICE 2048
#define TPB 256
#define EPT (SLICE / TPB)
#define MAXM DSD_MAX_TOP_M

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
// One selection round of a wave over o[j] = order_u32 of id base + threadIdx.x + j*TPB (0 = not a
// candidate): finds the largest value, the lowest id among its holders, clears it there and returns
// its rank_key to every lane (0 when nothing is left).
__device__ inline u64 select_round(unsigned (&o)[EPT], int base, int lane) {
    unsigned best = 0;
#pragma unroll
    for (int j = 0; j < EPT; ++j) best = o[j] > best ? o[j] : best;
    unsigned top = best;
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) {
        const unsigned t = __shfl_xor(top, s, WAVE);
        top = t > top ? t : top;
    }
    if (top == 0) return 0ull;                        // wave-uniform
    int my_j = EPT;
#pragma unroll
    for (int j = EPT - 1; j >= 0; --j) my_j = o[j] == top ? j : my_j;
    const unsigned long long holders = __ballot(my_j < EPT);
    int win = __ffsll((long long)holders) - 1;
    if (__popcll(holders) > 1) {                      // rare: equal values in several lanes
        int key = my_j < EPT ? (my_j << 6) | lane : 0x7FFFFFFF;
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) key = min(key, __shfl_xor(key, s, WAVE));
        win = key & 63;
    }
    const int win_j = __shfl(my_j, win, WAVE);
#pragma unroll
    for (int j = 0; j < EPT; ++j) o[j] = (lane == win && j == win_j) ? 0u : o[j];
    const int id = base + (int)(threadIdx.x - lane) + win + win_j * TPB;
    return ((u64)top << 32) | (u64)(0xFFFFFFFFu - (unsigned)id);
}

struct AcceptWs {
    double* part_m;     // [B][R][S]
    double* part_s;     // [B][R][S]
    u64* part_top_t;    // [B][R][S][MAXM]
    u64* part_top_q;    // [B][R][S][MAXM]
    double* row_lse;    // [B][R]
    double* row_nm;     // [B][R]
    double* row_ht;     // [B][R]  Shannon entropy of the target row   (DSD_H_ROW)
    double* row_hd;     // [B][R]  Shannon entropy of the draft row    (DSD_H_ROW)
    double* part_x;     // [B][R][S][3] per-slice sum min(P_t, q), -sum P_t ln P_t, -sum q ln q
    double* node_tau;   // [B][k]
    double* node_lnpt;  // [B][k]  ln P_t(y)
    double* node_q;     // [B][k]  q(y)
    int32_t* node_key;  // [B][k]
    int32_t* node_acc;  // [B][k]  the node's own test
    double* node_z;     // [B][k]  Z~ of the node's softened target
    double* part_z;     // [B][k][S]
    int32_t* draw_row;  // [B]
    int32_t* draw_mode; // [B] 0 = target row (bonus), 1 = positive part of P - q
    double* draw_tau;   // [B]
    double* draw_z;     // [B]   Z~ of the softened target used for the draw
    double* part_res;   // [B][S]
    double* part_fb;    // [B][S]  mass of P itself (used when the positive part is all zero)
};

__global__ void __launch_bounds__(TPB)
row_stats_kernel(const float* __restrict__ logits, const float* __restrict__ qp, AcceptWs ws, int R, int V, int S,
                 double inv_temp, int top_m) {
    __shared__ double shd[TPB / WAVE];
    __shared__ u64 sh_top[2][TPB / WAVE][MAXM];
    const int s = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
    const size_t row = ((size_t)b * R + r) * V;
    const int base = s * SLICE;
    float lv[EPT], qv[EPT];
    double mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        const bool in = i < V;
        lv[j] = in ? logits[row + i] : -INFINITY;
        qv[j] = in ? qp[row + i] : -INFINITY;
        if (in) mx = fmax(mx, (double)lv[j] * inv_temp);
    }
    mx = block_max_d(mx, shd);
    float fsum = 0.f;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        if (i < V) fsum += expf((float)((double)lv[j] * inv_temp - mx));
    }
    double sum = block_sum_d((double)fsum, shd);
    const size_t pidx = ((size_t)b * R + r) * S + s;
    if (threadIdx.x == 0) {
        ws.part_m[pidx] = mx;
        ws.part_s[pidx] = sum;
    }
    // top_m candidates of this slice, for the logits row (a = 0) and for the draft row (a = 1), on
    // the 32-bit order-preserving image of the values (0 = out of range), ties to the lowest id.
    // A threshold first: the slice is 16 groups of 16 lanes x 8 ids, and the top_m-th largest of
    // the 16 group maxima cannot exceed the slice's top_m-th largest value (the maxima are top_m
    // different ids at least that large), so everything that can be among the top_m lies at or
    // above it.  Usually a dozen ids pass; they go to a list in LDS and one wave per row kind picks
    // the top_m of them.  If more than 64 pass (many equal values), the slice falls back to
    // selection rounds over all ids.
    const int lane = threadIdx.x & (WAVE - 1), wave = threadIdx.x / WAVE;
    __shared__ unsigned sh_gm[2][16];
    __shared__ int sh_n[2];
    __shared__ u64 sh_cand[2][64];
    unsigned ot[EPT], oq[EPT];
    unsigned gt = 0u, gq = 0u;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        ot[j] = i < V ? order_u32(lv[j]) : 0u;
        oq[j] = i < V ? order_u32(qv[j]) : 0u;
        gt = ot[j] > gt ? ot[j] : gt;
        gq = oq[j] > gq ? oq[j] : gq;
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
        const unsigned t = __shfl_xor(gt, o, WAVE), q = __shfl_xor(gq, o, WAVE);
        gt = t > gt ? t : gt;
        gq = q > gq ? q : gq;
    }
    if ((lane & 15) == 0) {
        sh_gm[0][wave * 4 + (lane >> 4)] = gt;
        sh_gm[1][wave * 4 + (lane >> 4)] = gq;
    }
    if (threadIdx.x < 2) sh_n[threadIdx.x] = 0;
    __syncthreads();
    unsigned thr[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        // rank of group maximum (lane & 15) among the 16, equal values in index order
        const unsigned mine = sh_gm[a][lane & 15];
        int rank = 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const unsigned other = sh_gm[a][i];
            rank += (other > mine || (other == mine && i < (lane & 15))) ? 1 : 0;
        }
        const unsigned long long holder = __ballot(rank == top_m - 1);      // one lane in each group of 16
        thr[a] = __shfl(mine, __ffsll((long long)holder) - 1, WAVE);
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const unsigned (&o)[EPT] = a ? oq : ot;
        unsigned long long mask[EPT];
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            mask[j] = __ballot(o[j] != 0u && o[j] >= thr[a]);
            cnt += __popcll(mask[j]);
        }
        int at = 0;
        if (lane == 0) at = atomicAdd(&sh_n[a], cnt);
        at = __shfl(at, 0, WAVE);
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int pos = at + __popcll(mask[j] & ((1ull << lane) - 1ull));
            if (((mask[j] >> lane) & 1ull) && pos < 64) {
                const int id = base + threadIdx.x + j * TPB;
                sh_cand[a][pos] = ((u64)o[j] << 32) | (u64)(0xFFFFFFFFu - (unsigned)id);
            }
            at += __popcll(mask[j]);
        }
    }
    __syncthreads();
    const int n_t = sh_n[0], n_q = sh_n[1];
    u64* out_t = ws.part_top_t + pidx * MAXM;
    u64* out_q = ws.part_top_q + pidx * MAXM;
    if (wave < 2) {
        const int n = wave ? n_q : n_t;
        if (n <= 64) {
            u64 c = lane < n ? sh_cand[wave][lane] : 0ull;
            u64* out = wave ? out_q : out_t;
            for (int round = 0; round < top_m; ++round) {
                const u64 w = wave_max_u(c);                  // 0 when the slice ran out of ids
                c = c == w ? 0ull : c;
                if (lane == 0) out[round] = w;
            }
        }
    }
    if (n_t <= 64 && n_q <= 64) return;                        // block-uniform
    // Fallback.  Every wave selects among its own 512 ids, without barriers: top_m rounds of a
    // wave-wide maximum; among equal values the lowest id wins, which inside a wave is the lowest j,
    // then the lowest lane.  Wave 0 then merges the 4 lists (at most 64 candidates: one per lane) on
    // the full (value, id) keys.
    const bool redo_t = n_t > 64, redo_q = n_q > 64;
    for (int round = 0; round < top_m; ++round) {
        const u64 wt = redo_t ? select_round(ot, base, lane) : 0ull, wq = redo_q ? select_round(oq, base, lane) : 0ull;
        if (lane == 0) {
            sh_top[0][wave][round] = wt;
            sh_top[1][wave][round] = wq;
        }
    }
    __syncthreads();
    if (wave == 0) {
        const int w = lane / MAXM, r = lane % MAXM;          // TPB/WAVE * MAXM = 64 candidates
        u64 ct = r < top_m ? sh_top[0][w][r] : 0ull, cq = r < top_m ? sh_top[1][w][r] : 0ull;
        for (int round = 0; round < top_m; ++round) {
            const u64 wt = wave_max_u(ct), wq = wave_max_u(cq);   // 0 when the slice ran out of ids
            ct = ct == wt ? 0ull : ct;
            cq = cq == wq ? 0ull : cq;
            if (lane == 0) {
                if (redo_t) out_t[round] = wt;
                if (redo_q) out_q[round] = wq;
            }
        }
    }
}

// cand_lds = 1: the 2 * S * top_m candidates of the row fit the dynamic LDS and are read from memory once
__global__ void __launch_bounds__(WAVE)
row_merge_kernel(AcceptWs ws, int R, int S, int top_m, int cand_lds) {
    extern __shared__ u64 sh_cand[];                  // [2][S*top_m] when cand_lds
    const int r = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x;
    const size_t ridx = (size_t)b * R + r;
    double m = -INFINITY;
    for (int s = lane; s < S; s += WAVE) m = fmax(m, ws.part_m[ridx * S + s]);
    m = wave_max_d(m);
    double sum = 0.0;
    for (int s = lane; s < S; s += WAVE) sum += ws.part_s[ridx * S + s] * exp(ws.part_m[ridx * S + s] - m);
    sum = wave_sum_d(sum);
    // merge the per-slice candidate lists: top_m rounds of a wave-wide maximum; keys are distinct, so
    // each round selects strictly below the previous winner
    const u64* gt = ws.part_top_t + ridx * S * MAXM;
    const u64* gq = ws.part_top_q + ridx * S * MAXM;
    const int n = S * top_m;
    if (cand_lds) {
        for (int i = lane; i < n; i += WAVE) {
            const int src = (i / top_m) * MAXM + i % top_m;
            sh_cand[i] = gt[src];
            sh_cand[n + i] = gq[src];
        }
        __syncthreads();
    }
    int idt[MAXM], idq[MAXM];
    u64 last_t = ~0ull, last_q = ~0ull;
    for (int round = 0; round < top_m; ++round) {
        u64 bt = 0, bq = 0;
        for (int i = lane; i < n; i += WAVE) {
            u64 a, c;
            if (cand_lds) {
                a = sh_cand[i];
                c = sh_cand[n + i];
            } else {
                const int src = (i / top_m) * MAXM + i % top_m;
                a = gt[src];
                c = gq[src];
            }
            if (a < last_t && a > bt) bt = a;
            if (c < last_q && c > bq) bq = c;
        }
        last_t = wave_max_u(bt);
        last_q = wave_max_u(bq);
        idt[round] = key_id(last_t);
        idq[round] = key_id(last_q);
    }
    if (lane == 0) {
        int common = 0;
        for (int i = 0; i < top_m; ++i)
            for (int j = 0; j < top_m; ++j) common += (idt[i] == idq[j]) ? 1 : 0;
        ws.row_lse[ridx] = m + log(sum);
        ws.row_nm[ridx] = (double)common / (double)top_m;
    }
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

__global__ void __launch_bounds__(TPB)
node_soft_kernel(const float* __restrict__ logits, const float* __restrict__ qp, const int32_t* __restrict__ tokens,
                 const int32_t* __restrict__ parent, AcceptWs ws, dsd_accept_params prm, int k, int V, int S,
                 double inv_temp) {
    __shared__ double shd[TPB / WAVE];
    const int s = blockIdx.x, node = blockIdx.y + 1, b = blockIdx.z;
    const int R = k + 1;
    int p = parent ? parent[node - 1] : node - 1;
    p = p < 0 ? 0 : (p > node - 1 ? node - 1 : p);
    int y = tokens[(size_t)b * k + node - 1];
    y = y < 0 ? 0 : (y >= V ? V - 1 : y);
    const size_t row = ((size_t)b * R + p) * V;
    const double lse = ws.row_lse[(size_t)b * R + p];
    const double ln_pt = (double)logits[row + y] * inv_temp - lse;
    const double pt_y = exp(ln_pt);
    const double q_y = (double)qp[row + y];
    // key-token rule: any of the three criteria
    double h_t = -ln_pt, h_d = -log(q_y);
    if (prm.entropy_kind == DSD_H_ROW) {
        h_t = ws.row_ht[(size_t)b * R + p];
        h_d = ws.row_hd[(size_t)b * R + p];
    }
    const bool key = (h_d > prm.lambda1 * h_t) || (fabs(pt_y - q_y) > prm.lambda2) ||
                     (ws.row_nm[(size_t)b * R + p] < prm.lambda3);
    double tau = key ? 0.0 : prm.tau;
    if (prm.tau_override) tau = (double)prm.tau_override[(size_t)b * k + node - 1];
    tau = tau < 0.0 ? 0.0 : (tau > 1.0 ? 1.0 : tau);
    const size_t nidx = (size_t)b * k + node - 1;
    if (s == 0 && threadIdx.x == 0) {
        ws.node_tau[nidx] = tau;
        ws.node_lnpt[nidx] = ln_pt;
        ws.node_q[nidx] = q_y;
        ws.node_key[nidx] = key ? 1 : 0;
    }
    if (tau == 0.0) return;     // P~ = P_t, Z~ = 1
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

// One wavefront per (sequence, node): Z~ of the node's softened target from the slice partials, the
// node's test u * q(y) < P~(y), and the optional statistics.
__global__ void __launch_bounds__(WAVE)
node_accept_kernel(const int32_t* __restrict__ parent, const float* __restrict__ uniforms, AcceptWs ws, int k, int S,
                   dsd_accept_stats st) {
    const int i = blockIdx.x + 1, b = blockIdx.y;
    const int lane = threadIdx.x;
    const int R = k + 1;
    int p = parent ? parent[i - 1] : i - 1;
    p = p < 0 ? 0 : (p > i - 1 ? i - 1 : p);
    const size_t nidx = (size_t)b * k + i - 1;
    const double tau = ws.node_tau[nidx];
    double z = 1.0;
    if (tau != 0.0) {
        z = 0.0;
        for (int s = lane; s < S; s += WAVE) z += ws.part_z[nidx * S + s];
        z = wave_sum_d(z);
    }
    if (lane != 0) return;
    const double q_y = ws.node_q[nidx];
    const double p_y = soft_weight(ws.node_lnpt[nidx], q_y, tau) / z;
    const double u = (double)uniforms[(size_t)b * R + i];
    const bool acc = u * q_y < p_y;
    ws.node_z[nidx] = z;
    ws.node_acc[nidx] = acc ? 1 : 0;
    if (st.key_flags) st.key_flags[nidx] = ws.node_key[nidx];
    if (st.node_accept) st.node_accept[nidx] = acc ? 1 : 0;
    if (st.ratio) st.ratio[nidx] = q_y > 0.0 ? p_y / q_y : (p_y > 0.0 ? INFINITY : 0.0);
    if (st.norm_match) st.norm_match[nidx] = ws.row_nm[(size_t)b * R + p];
}

// One workgroup per sequence: thread i = node i (0 = the root) walks up to the root for its depth and
// for whether it and all its ancestors passed their tests; thread 0 then picks the accepted path and
// what the extra token is drawn from.  The tree lives in LDS.
#define DECIDE_TPB 128
__global__ void __launch_bounds__(DECIDE_TPB)
decide_kernel(const int32_t* __restrict__ parent, AcceptWs ws, dsd_accept_params prm, int k,
              int32_t* __restrict__ accepted_len, int32_t* __restrict__ accepted_path) {
    __shared__ int par[DSD_MAX_K + 1], acc[DSD_MAX_K + 1], dep[DSD_MAX_K + 1], ok[DSD_MAX_K + 1];
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    if (i <= k) {
        int p = 0, a = 1;
        if (i > 0) {
            p = parent ? parent[i - 1] : i - 1;
            p = p < 0 ? 0 : (p > i - 1 ? i - 1 : p);
            a = ws.node_acc[(size_t)b * k + i - 1] != 0;
        }
        par[i] = p;
        acc[i] = a;
    }
    if (accepted_path && i < k) accepted_path[(size_t)b * k + i] = -1;
    __syncthreads();
    if (i <= k) {
        int d = 0, good = acc[i];
        for (int n = i; n != 0; n = par[n]) {        // parents precede children: at most k steps
            ++d;
            good &= acc[par[n]];
        }
        dep[i] = d;
        ok[i] = good;
    }
    __syncthreads();
    if (i != 0) return;
    int vstar = 0;
    if (prm.tree_mode == DSD_TREE_FIRST_ACCEPTED) {
        for (;;) {
            int nxt = 0;
            for (int c = vstar + 1; c <= k; ++c)
                if (par[c] == vstar && acc[c]) { nxt = c; break; }
            if (!nxt) break;
            vstar = nxt;
        }
    } else {
        for (int c = 1; c <= k; ++c)
            if (ok[c] && dep[c] > dep[vstar]) vstar = c;
    }
    const int a = dep[vstar];
    accepted_len[b] = a;
    if (accepted_path)
        for (int n = vstar, j = a - 1; n != 0; n = par[n], --j) accepted_path[(size_t)b * k + j] = n;
    int child = 0;
    for (int c = vstar + 1; c <= k; ++c)
        if (par[c] == vstar) { child = c; break; }
    ws.draw_row[b] = vstar;
    if (!child) {
        ws.draw_mode[b] = 0;
        ws.draw_tau[b] = 0.0;
        ws.draw_z[b] = 1.0;
    } else {
        ws.draw_mode[b] = 1;
        ws.draw_tau[b] = ws.node_tau[(size_t)b * k + child - 1];
        ws.draw_z[b] = ws.node_z[(size_t)b * k + child - 1];
    }
}

// weight of id i in the distribution the extra token is drawn from; also P itself
__device__ inline void draw_weight(const float* __restrict__ logits, const float* __restrict__ qp, size_t row, int i,
                                   double inv_temp, double lse, int mode, double tau, double z, double* w,
                                   double* p) {
    const float ln_pt = (float)((double)logits[row + i] * inv_temp - lse);
    if (mode == 0) {
        *p = (double)expf(ln_pt);
        *w = *p;
    } else {
        const float q = qp[row + i];
        *p = (double)soft_weight_f(ln_pt, q, (float)tau) / z;
        *w = fmax(*p - (double)q, 0.0);
    }
}

__global__ void __launch_bounds__(TPB)
draw_parts_kernel(const float* __restrict__ logits, const float* __restrict__ qp, AcceptWs ws, int R, int V, int S,
                  double inv_temp) {
    __shared__ double shd[TPB / WAVE];
    const int s = blockIdx.x, b = blockIdx.y;
    const int r = ws.draw_row[b], mode = ws.draw_mode[b];
    const double tau = ws.draw_tau[b], z = ws.draw_z[b];
    const size_t row = ((size_t)b * R + r) * V;
    const double lse = ws.row_lse[(size_t)b * R + r];
    double sw = 0.0, sp = 0.0;
    const int base = s * SLICE;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = base + threadIdx.x + j * TPB;
        if (i < V) {
            double w, p;
            draw_weight(logits, qp, row, i, inv_temp, lse, mode, tau, z, &w, &p);
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

__global__ void __launch_bounds__(TPB)
draw_pick_kernel(const float* __restrict__ logits, const float* __restrict__ qp, const float* __restrict__ uniforms,
                 AcceptWs ws, int R, int V, int S, double inv_temp, int32_t* __restrict__ next_token) {
    __shared__ double pre[TPB + 1];
    __shared__ int sh_slice, sh_fallback, sh_best[TPB / WAVE], sh_last[TPB / WAVE];
    __shared__ double sh_before, sh_target;
    const int b = blockIdx.x;
    const int r = ws.draw_row[b], mode = ws.draw_mode[b];
    const double tau = ws.draw_tau[b], z = ws.draw_z[b];
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
            draw_weight(logits, qp, row, i, inv_temp, lse, mode, tau, z, &ww, &pp);
            w[j] = fb ? pp : ww;
            if (w[j] > 0.0) lastpos = i;
        }
        loc += w[j];
    }
    pre[threadIdx.x + 1] = loc;
    __syncthreads();
    if (threadIdx.x == 0) {
        pre[0] = before < 0.0 ? 0.0 : before;
        for (int t = 1; t <= TPB; ++t) pre[t] += pre[t - 1];
    }
    __syncthreads();
    int found = 0x7FFFFFFF;
    if (before >= 0.0) {
        double c = pre[threadIdx.x];
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
        int taken = 0;
        for (int c = v + 1; c <= k && !taken; ++c) {
            if (s_par[c] != v) continue;
            int y = tokens[(size_t)b * k + c - 1];
            y = y < 0 ? 0 : (y >= V ? V - 1 : y);
            // the child's own test, fp64, by every thread alike
            double p = exp((double)logits[row + y] * inv_temp - lse);
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
            z = wave_sum_d(z);
            __syncthreads();                          // everyone is done with the chain arrays and s_red
            if (lane == 0) s_red[wave] = z;
            __syncthreads();
            if (tid == 0) {
                double tot = 0.0;
                for (int i = 0; i < WALK_TPB / WAVE; ++i) tot += s_red[i];
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

int accept_launch(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                  const int32_t* parent, const float* uniforms, const dsd_accept_params* prm, int B, int k, int V,
                  int32_t* accepted_len, int32_t* next_token, int32_t* accepted_path, const dsd_accept_stats* stats) {
    const int R = k + 1;
    const int S = (V + SLICE - 1) / SLICE;
    const size_t BR = (size_t)B * R, BK = (size_t)B * k;
    if (prm->temperature == 0.0) {
        DSD_TRY(dsd_ws_reserve(ctx, BR * S * 8 + 256));
        u64* part = (u64*)ctx->ws;
        dsd_accept_stats st0 = {nullptr, nullptr, nullptr, nullptr};
        if (stats) st0 = *stats;
        if (B > 65535) DSD_FAIL(DSD_ESHAPE, "dsd_accept: B=%d exceeds 65535", B);
        ProfScope ps(ctx, DSD_KC_ACCEPT);
        row_argmax_kernel<<<dim3(S, R, B), TPB, 0, ctx->stream>>>(logits, part, R, V, S);
        greedy_decide_kernel<<<B, DECIDE_TPB, 0, ctx->stream>>>(draft_tokens, parent, part, prm->tree_mode, k, S, accepted_len,
                                                                 next_token, accepted_path, st0);
        DSD_HIP(hipGetLastError());
        return DSD_OK;
    }
    size_t need = (BR * S * 5 + BR * 4 + BK * 4 + BK * S + (size_t)B * 2 + (size_t)B * S * 2) * 8 +
                  BR * S * MAXM * 8 * 2 + (2 * BK + 2 * (size_t)B) * 4 + 32 * 256;
    DSD_TRY(dsd_ws_reserve(ctx, need));
    WsBump bump{ctx->ws, 0};
    AcceptWs ws;
    ws.part_m = bump.take<double>(BR * S);
    ws.part_s = bump.take<double>(BR * S);
    ws.part_top_t = bump.take<u64>(BR * S * MAXM);
    ws.part_top_q = bump.take<u64>(BR * S * MAXM);
    ws.row_lse = bump.take<double>(BR);
    ws.row_nm = bump.take<double>(BR);
    ws.row_ht = bump.take<double>(BR);
    ws.row_hd = bump.take<double>(BR);
    ws.part_x = bump.take<double>(BR * S * 3);
    ws.node_tau = bump.take<double>(BK);
    ws.node_lnpt = bump.take<double>(BK);
    ws.node_q = bump.take<double>(BK);
    ws.node_key = bump.take<int32_t>(BK);
    ws.node_acc = bump.take<int32_t>(BK);
    ws.node_z = bump.take<double>(BK);
    ws.part_z = bump.take<double>(BK * S);
    ws.draw_row = bump.take<int32_t>(B);
    ws.draw_mode = bump.take<int32_t>(B);
    ws.draw_tau = bump.take<double>(B);
    ws.draw_z = bump.take<double>(B);
    ws.part_res = bump.take<double>((size_t)B * S);
    ws.part_fb = bump.take<double>((size_t)B * S);
    if (bump.off > ctx->ws_bytes) DSD_FAIL(DSD_ENOMEM, "accept workspace estimate too small");
    hipStream_t s = ctx->stream;
    const double inv_temp = 1.0 / prm->temperature;
    dsd_accept_stats st = {nullptr, nullptr, nullptr, nullptr};
    if (stats) st = *stats;
    if (B > 65535) DSD_FAIL(DSD_ESHAPE, "dsd_accept: B=%d exceeds 65535", B);
    ProfScope ps(ctx, DSD_KC_ACCEPT);
    row_stats_kernel<<<dim3(S, R, B), TPB, 0, s>>>(logits, draft_probs, ws, R, V, S, inv_temp, prm->top_m);
    const size_t cand_bytes = (size_t)2 * S * prm->top_m * sizeof(u64);
    const int cand_lds = cand_bytes <= 48 * 1024;
    row_merge_kernel<<<dim3(R, B), WAVE, cand_lds ? cand_bytes : 0, s>>>(ws, R, S, prm->top_m, cand_lds);
    if (prm->norm_match_kind == DSD_NM_OVERLAP || prm->entropy_kind == DSD_H_ROW) {
        row_extra_kernel<<<dim3(S, R, B), TPB, 0, s>>>(logits, draft_probs, ws, R, V, S, inv_temp);
        row_extra_merge_kernel<<<dim3(R, B), WAVE, 0, s>>>(ws, R, S, prm->norm_match_kind == DSD_NM_OVERLAP ? 1 : 0);
    }
    if (prm->tree_mode == DSD_TREE_LOSSLESS) {
        // no relaxation in this mode: node_soft only evaluates the key rule (reported), then the walk
        dsd_accept_params strict = *prm;
        strict.tau = 0.0;
        strict.tau_override = nullptr;
        node_soft_kernel<<<dim3(S, k, B), TPB, 0, s>>>(logits, draft_probs, draft_tokens, parent, ws, strict, k, V, S, inv_temp);
        lossless_walk_kernel<<<B, WALK_TPB, 0, s>>>(logits, draft_probs, draft_tokens, parent, uniforms, ws, k, V, inv_temp,
                                                      accepted_len, next_token, accepted_path, st);
        DSD_HIP(hipGetLastError());
        return DSD_OK;
    }
    node_soft_kernel<<<dim3(S, k, B), TPB, 0, s>>>(logits, draft_probs, draft_tokens, parent, ws, *prm, k, V, S, inv_temp);
    node_accept_kernel<<<dim3(k, B), WAVE, 0, s>>>(parent, uniforms, ws, k, S, st);
    decide_kernel<<<B, DECIDE_TPB, 0, s>>>(parent, ws, *prm, k, accepted_len, accepted_path);
    draw_parts_kernel<<<dim3(S, B), TPB, 0, s>>>(logits, draft_probs, ws, R, V, S, inv_temp);
    draw_pick_kernel<<<B, TPB, 0, s>>>(logits, draft_probs, uniforms, ws, R, V, S, inv_temp, next_token);
    DSD_HIP(hipGetLastError());
    return DSD_OK;
}
