/*
 * libdsd -- the verification step of Decentralized Speculative Decoding on one MI355X.
 *
 * One node of a decentralized deployment hosts a contiguous block of the target model's
 * layers (paper section 2.2) and, once per round, scores all k drafted tokens in a single
 * forward pass (section 2.1).  The last node turns hidden states into logits and runs the
 * acceptance loop of Algorithm 1 with the key-token rule and the softened target of
 * section 2.3.  This header is the whole boundary of the library.
 *
 * Conventions
 *   - Plain C ABI.  Every call returns 0 (DSD_OK) or a negative dsd_status; the message of the
 *     last failure on the calling thread is available from dsd_last_error().  Nothing aborts or
 *     throws across the boundary.  A call that fails validation launches nothing.
 *   - "device" pointers are HIP device memory owned by the caller, on the device the context
 *     was created for; "host" pointers are ordinary host memory.  The library never frees or
 *     keeps a caller's pointer beyond the call, except where stated.
 *   - All work is enqueued on the context's HIP stream, in order.  Calls do not synchronise
 *     unless stated; outputs are valid once the caller has synchronised that stream.
 *   - Row-major everywhere.  B = sequences, k = drafted rows per sequence (nodes of the draft
 *     tree, numbered 1..k with parents before children; 0 is the root = committed context),
 *     d = d_model, V = vocabulary.
 */
#ifndef DSD_H
#define DSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dsd_ctx dsd_ctx;         /* device, stream, workspace            */
typedef struct dsd_weights dsd_weights; /* the node's layer block, library-owned */
typedef struct dsd_kv dsd_kv;           /* the node's KV cache, library-owned    */

enum dsd_status {
    DSD_OK = 0,
    DSD_EINVAL = -1,       /* NULL or out-of-range argument                     */
    DSD_ESHAPE = -2,       /* sizes that do not fit the model / cache / limits  */
    DSD_ENOMEM = -3,       /* device allocation failed                          */
    DSD_EHIP = -4,         /* a HIP runtime call failed                         */
    DSD_EUNSUPPORTED = -5  /* a combination this build has no kernel for        */
};

enum dsd_dtype { DSD_F32 = 0, DSD_BF16 = 1 };
/* Other readings of two loosely specified ingredients of the key rule (section 2.3):
 * DSD_NM_OVERLAP: NormMatch(p) = sum_v min(P_t(v), q_p(v)), the mass the rows share (1 - total variation);
 * DSD_H_ROW: H_d, H_t = Shannon entropies -sum_v P ln P of the draft row and of the target row. */
enum dsd_norm_match_kind { DSD_NM_TOP_M = 0, DSD_NM_OVERLAP = 1 };
enum dsd_entropy_kind { DSD_H_TOKEN = 0, DSD_H_ROW = 1 };
enum dsd_tree_mode { DSD_TREE_LONGEST = 0, DSD_TREE_FIRST_ACCEPTED = 1, DSD_TREE_LOSSLESS = 2 };

#define DSD_MAX_K 64      /* drafted rows per sequence (tree masks are 64-bit rows) */
#define DSD_MAX_TOP_M 16  /* support size of NormMatch                             */

/* The node's share of the target model: a block of Llama-style decoder layers (pre-norm
 * RMSNorm, rotary embedding pairing element i with i + head_dim/2, grouped-query attention,
 * SwiGLU FFN, no biases), optionally preceded by the token embedding (first node) and
 * followed by the final RMSNorm + LM head (last node).  The paper names the model families
 * only (section 3.1). */
typedef struct dsd_model_desc {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;   /* divides n_q_heads */
    int32_t head_dim;     /* 64 or 128 */
    int32_t d_ffn;
    int32_t vocab;        /* used when has_embed or has_head */
    int32_t dtype;        /* dsd_dtype of weights, hidden states and KV cache */
    int32_t has_embed;
    int32_t has_head;
    float rope_theta;
    float rms_eps;
} dsd_model_desc;

/* Thresholds of the key-token rule and the relaxation of section 2.3.
 * A drafted token y with parent row p is a key token when any of
 *     -ln q_p(y) > lambda1 * -ln P_t(y)      (cross-entropy contrast, product form)
 *     |P_t(y) - q_p(y)| > lambda2
 *     NormMatch(p) < lambda3                 (share of the top_m ids of P_t found in the top_m ids of q_p)
 * holds.  Key tokens are verified against P_t, the others against
 * P~ = P_t^(1-tau) q_p^tau renormalised over the vocabulary.  tau = 0 is the strict rule. */
typedef struct dsd_accept_params {
    double lambda1, lambda2, lambda3;
    double tau;          /* in [0,1] */
    double temperature;  /* > 0: P_t = softmax(logits / temperature); 0: greedy verification (see dsd_accept) */
    int32_t top_m;       /* 1..DSD_MAX_TOP_M */
    int32_t tree_mode;   /* dsd_tree_mode */
    const float* tau_override; /* device [B,k] or NULL: tau of node i whatever the key rule says */
    int32_t norm_match_kind;   /* dsd_norm_match_kind; 0 = the top_m overlap above */
    int32_t entropy_kind;      /* dsd_entropy_kind; 0 = the token cross entropies above */
} dsd_accept_params;

/* Optional per-node outputs of dsd_accept (device pointers, each may be NULL). */
typedef struct dsd_accept_stats {
    int32_t* key_flags;   /* [B,k] 1 if node i is a key token            */
    int32_t* node_accept; /* [B,k] 1 if node i passed its own test       */
    double* ratio;        /* [B,k] P~(y)/q(y) (inf when q(y)=0<P~(y))    */
    double* norm_match;   /* [B,k] NormMatch of node i's parent row      */
} dsd_accept_stats;

/* Message of the last failing call on this thread ("" if none).  Never NULL. */
const char* dsd_last_error(void);

/* Context for HIP device `device`; hip_stream is a hipStream_t (NULL = the default stream).
 * The context owns a workspace that grows on demand (allocation happens inside the first
 * call that needs more, which then synchronises).  dsd_destroy frees it.
 * Read from the environment here, for testing: DSD_PATH=simple (generic kernels also for bf16
 * models), DSD_NO_TILED (no activation panels: one workgroup per column tile at every row count). */
int dsd_create(int device, void* hip_stream, dsd_ctx** out);
int dsd_destroy(dsd_ctx* ctx);
int dsd_set_stream(dsd_ctx* ctx, void* hip_stream);

/* Takes the layer block a node hosts (section 2.2: each node holds a contiguous shard of the
 * target model's layers).  `tensors` is a host array of n_tensors device pointers in this order:
 *   [embed V x d]                                              if has_embed
 *   per layer: g1[d], Wq[Hq*hd x d], Wk[Hkv*hd x d], Wv[Hkv*hd x d], Wo[d x Hq*hd],
 *              g2[d], Wg[F x d], Wu[F x d], Wd[d x F]
 *   [gf[d], Wlm[V x d]]                                        if has_head
 * every matrix stored [out_features x in_features], all in desc->dtype.  The library copies
 * (and for bf16 re-tiles) them into buffers of its own and synchronises before returning;
 * the caller may free its tensors afterwards.
 * The matrix-core path holds bf16 projection weights as fp16, which is exact for every bf16
 * value of magnitude 2^-17 .. 65504 (smaller ones round to a multiple of 2^-24).
 * Errors: DSD_EUNSUPPORTED if a bf16 projection weight is not finite or exceeds 65504 in
 * magnitude; DSD_ENOMEM; DSD_EINVAL / DSD_ESHAPE for a bad description or tensor count. */
int dsd_weights_create(dsd_ctx* ctx, const dsd_model_desc* desc, const void* const* tensors,
                       int n_tensors, dsd_weights** out);
int dsd_weights_destroy(dsd_ctx* ctx, dsd_weights* w);

/* KV cache for max_batch sequences of up to max_slots positions (committed + drafted) in
 * every layer of the block: the state the single forward pass over the window of section 2.1
 * reads (committed context) and extends (the k drafted rows).  Lengths start at 0.  The storage
 * layout is the library's. */
int dsd_kv_create(dsd_ctx* ctx, const dsd_model_desc* desc, int max_batch, int max_slots, dsd_kv** out);
int dsd_kv_destroy(dsd_ctx* ctx, dsd_kv* kv);

/* Brings in the keys and values of an already processed context (the prompt, or a cache kept
 * elsewhere), which verification in section 2.1 presupposes: loads positions [0, n_slots) of one
 * layer from device arrays k, v of shape
 * [B, Hkv, n_slots, hd] (desc dtype; keys already rotated).  Does not change lengths. */
int dsd_kv_import(dsd_ctx* ctx, dsd_kv* kv, int layer, const void* k, const void* v, int B, int n_slots);
/* Reads positions [first_slot, first_slot + n_slots) of one layer back into device arrays of
 * shape [B, Hkv, n_slots, hd] (desc dtype). */
int dsd_kv_export(dsd_ctx* ctx, const dsd_kv* kv, int layer, int first_slot, int n_slots, int B,
                  void* k_out, void* v_out);
/* Sets / reads the committed length of sequences 0..B-1 (host arrays).  get synchronises. */
int dsd_kv_set_len(dsd_ctx* ctx, dsd_kv* kv, const int32_t* host_len, int B);
int dsd_kv_get_len(dsd_ctx* ctx, const dsd_kv* kv, int32_t* host_len, int B);

/* The verification pass of one node over k drafted rows per sequence (section 2.1: one
 * forward pass over the window; section 2.2: on this node's layer block).
 *   hidden_in    device [B,k,d] in desc dtype: rows handed over by the previous node;
 *                NULL on the first node, where rows are the embeddings of draft_tokens
 *   draft_tokens device int32 [B,k], read only when hidden_in is NULL
 *   tree_mask    device uint64 [k]: bit s-1 of row t-1 set iff node s is node t or an ancestor
 *                of node t; NULL = chain (row t sees rows 1..t)
 *   depth        device int32 [k]: position offset of each row (chain: 0..k-1); NULL = chain
 *   hidden_out   device [B,k,d] in desc dtype, rows after the last layer of the block
 *                (before the final norm); may be NULL when logits are requested
 *   logits       device float [B rows of k x V], sequence b starting at logits + b*logits_seq_stride
 *                elements (0 = k*V); only when has_head, else must be NULL.  A caller that keeps
 *                the root row in the same buffer passes logits + V and stride (k+1)*V.
 * Row t of sequence b sits at position len[b] + depth[t]; its rotated key and its value are
 * written to cache slot len[b] + t of every layer; it attends to slots [0, len[b]) and to the
 * drafted rows its mask allows.  Lengths are not advanced: see dsd_kv_commit.
 * Every sum is taken in a fixed order: the same call on the same inputs and cache contents
 * writes the same bits.  On the matrix-core path activations enter the projections as fp16
 * (11 significant bits or more); magnitudes beyond 65504 at those points saturate and are counted:
 * see dsd_stage_status.
 * Errors: DSD_ESHAPE if B > max_batch, k > DSD_MAX_K or max(len) + k > max_slots. */
int dsd_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                     const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth,
                     int B, int k, void* hidden_out, float* logits, int64_t logits_seq_stride);

/* Whether the dsd_stage_verify calls since the last check stayed inside the range of the matrix-core path.
 * That path (bf16 models) feeds the projections with fp16 operands: the normalised rows, the attention
 * output, SiLU(gate)*up and the attention's partial outputs are converted on the way, and a magnitude
 * beyond 65504 (or a NaN) saturates there.  Every such conversion is counted on the device.  This call
 * synchronises the context's stream, stores the count in *saturated (host, may be NULL), clears it, and
 * returns DSD_EUNSUPPORTED if it was not zero: the outputs of the calls in between are then not the model's.
 * (Section 2.1 asks of the verification pass that it scores the drafted window with the target model itself.)
 * A caller checks once per round, after it has synchronised anyway; fp32 models never count anything. */
int dsd_stage_status(dsd_ctx* ctx, int64_t* saturated);

/* Algorithm 1, lines 2-16, for B sequences.
 *   logits       device float [B,k+1,V]: row 0 follows the committed context, row i follows node i
 *   draft_probs  device float [B,k+1,V]: row p is the draft distribution the children of node p
 *                were drawn from (rows of leaves are not read); used as given
 *   draft_tokens device int32 [B,k]: token of node i
 *   parent       device int32 [k], values in 0..k with parent[i-1] < i; NULL = chain
 *   uniforms     device float [B,k+1] in [0,1): u_i decides node i, u_0 draws the extra token
 * Node i passes when u_i * q(y_i) < P(y_i), P being P_t for key tokens and P~ otherwise (the
 * min(1, p/q) rule of the speculative sampling work cited in section 2.1).  The accepted path
 * is the leading run of passes (chain), or per tree_mode the deepest fully passed root-to-node
 * path (ties to the lower node id) / the greedy descent through lowest-id passing children.
 * The additional token (Algorithm 1 line 16): if the path's last node has no children it is
 * drawn from P_t of that node's row; otherwise from the normalised positive part of P - q of
 * that row, P as used for its lowest-id child (if that is all zero, from P); drawn by inverse
 * CDF in token-id order with u_0.
 * DSD_TREE_LOSSLESS replaces the per-node test by recursive rejection over siblings that were
 * drawn WITHOUT replacement from their parent's draft row (the token-tree verification of the
 * SpecInfer line of work cited in section 1), which keeps the target distribution when a node
 * has several children: at node v, starting from p = P_t(. | v) and q = draft row v, the children
 * are tried in node order; child c with token y passes when u_c * q(y) < p(y); after a rejection
 * p becomes the normalised positive part of p - q and q loses y and is renormalised.  The first
 * passing child becomes v (its own rows are used from there); when no child passes, or v is a
 * leaf, the additional token is drawn from the p that is left.  The relaxation (tau) is not
 * applied in this mode; key flags and NormMatch are still reported, node_accept and ratio only
 * for the nodes the walk tried (0 elsewhere).  A chain gives the same result as the strict rule.
 * temperature = 0 is greedy verification (the t = 0.0 rows of Table 1): node i passes iff its
 * token is the arg max of its parent's logits row (ties to the lower id), the additional token is
 * the arg max of the row of the path's last node; draft_probs and uniforms are not read (may be
 * NULL), nothing is relaxed, key flags and NormMatch are reported as 0, ratio as 1 / 0.
 *   accepted_len  device int32 [B]
 *   next_token    device int32 [B]
 *   accepted_path device int32 [B,k] node ids of the path, -1 padded; may be NULL
 *   stats         optional, may be NULL
 * Sums over the vocabulary are accumulated in fp64 from fp32 per-id terms; every quantity that
 * decides something by itself is fp64; no probability row is written to memory.  Under DSD_TREE_LOSSLESS
 * a later sibling is tested against the residual max(0, p - q) / Z; a Z below 0.05 (target and draft
 * nearly coincide) is summed in fp64 with the row renormalised in fp64, as is every later Z of the same
 * node, so the reported ratios keep 1e-6 relative accuracy down to Z of about 1e-6; above 0.05 the fp32 terms bound
 * the error of Z by 1e-7 / Z. */
int dsd_accept(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
               const int32_t* parent, const float* uniforms, const dsd_accept_params* params,
               int B, int k, int V, int32_t* accepted_len, int32_t* next_token,
               int32_t* accepted_path, const dsd_accept_stats* stats);

/* dsd_accept for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same results (bit for bit: the same kernels run),
 * but the per-slice partials of the call live in a fixed 8 MiB array in the library's device image instead
 * of the context's growing workspace, and the call issues nothing but kernel launches on the context's
 * stream: no hipMalloc, hipFree, memset or event.  Per-kernel timing (dsd_profile_enable) does not see it.
 * Errors: DSD_ESHAPE when the call needs more scratch than the array holds -- about
 * B*(k+1)*ceil(V/2048)*560 bytes; B=16, k=8 and B=4, k=32 at V=128256 fit, use dsd_accept beyond;
 * DSD_EUNSUPPORTED on a device index above 63.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads,
 * two contexts) race and must be serialised by the caller.  Nothing in the array has to be cleared
 * between calls: every word a kernel reads was written by an earlier kernel of the same call. */
int dsd_accept_noalloc(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                       const int32_t* parent, const float* uniforms, const dsd_accept_params* params,
                       int B, int k, int V, int32_t* accepted_len, int32_t* next_token,
                       int32_t* accepted_path, const dsd_accept_stats* stats);

/* Advances every sequence by its accepted tokens (section 2.1: x_{1:i+k} = x_{1:i} (+) y_{i+1:i+k}):
 * in every layer the K/V rows that the last dsd_stage_verify wrote for the path's nodes become
 * slots len[b] .. len[b]+a-1, and len[b] += a.  accepted_len / accepted_path are device arrays
 * as written by dsd_accept ([B], [B,k]); accepted_path NULL = chain (first a rows, nothing moves).
 * Does not synchronise: the lengths live on the device, and the host only keeps an upper bound
 * (+k per commit) for validation and grid sizes.  dsd_kv_get_len reads the true lengths back and
 * tightens that bound; a caller that never does loses k - a slots of usable capacity per round.
 * Errors: DSD_ESHAPE if k differs from the last dsd_stage_verify on this cache. */
int dsd_kv_commit(dsd_ctx* ctx, dsd_kv* kv, const int32_t* accepted_len, const int32_t* accepted_path,
                  int B, int k);

/* Diagnostics: time per kernel class.  While enabled, every kernel launch of dsd_stage_verify and
 * dsd_accept is bracketed by a pair of HIP events on the context's stream (this serialises
 * nothing but costs a little per launch, so leave it off when timing whole calls).
 * dsd_profile_read synchronises the stream, adds up the event pairs recorded since the last
 * read into ms_total[DSD_KC_COUNT] / launches[DSD_KC_COUNT] (host arrays) and forgets them. */
enum dsd_kernel_class {
    DSD_KC_QKV = 0,      /* RMSNorm + QKV projection + rotary + cache append */
    DSD_KC_ATTN,         /* k-query attention over the cache                 */
    DSD_KC_ATTN_COMBINE, /* merge of the key runs                            */
    DSD_KC_OPROJ,        /* output projection + residual                     */
    DSD_KC_GATEUP,       /* RMSNorm + gate/up projection + SiLU*up           */
    DSD_KC_DOWN,         /* down projection + residual                       */
    DSD_KC_HEAD,         /* final RMSNorm + LM head                          */
    DSD_KC_ACCEPT,       /* all kernels of dsd_accept                        */
    DSD_KC_OTHER,        /* row load / store                                 */
    DSD_KC_COUNT
};
int dsd_profile_enable(dsd_ctx* ctx, int on);
int dsd_profile_read(dsd_ctx* ctx, double* ms_total, int64_t* launches);

/* Diagnostics: what a bare stream over device memory reaches on this device, the yardstick for a pass that
 * the paper's own argument (section 2.1, Fig. 1) makes memory bound.  buf: device, `bytes` long (a multiple
 * of 32, at least 1 MiB, 16-byte aligned), contents irrelevant.  mode 0: one kernel reads all of it, the
 * whole grid sweeping one contiguous front; mode 1: one kernel copies its first half onto its second half
 * (bytes/2 read + bytes/2 written); mode 2: one kernel reads it with every wave walking a contiguous
 * stream of its own (bytes rounded down to whole streams of 16 KiB steps); mode 3: as mode 0 with
 * non-temporal loads, which is how the library's kernels read what they read once (weights, K/V).
 * Runs 2 untimed + `iters` timed launches on the context's stream, synchronises, and returns the
 * average time of a launch in *ms_avg (host). */
int dsd_stream_probe(dsd_ctx* ctx, void* buf, size_t bytes, int mode, int iters, double* ms_avg);

#ifdef __cplusplus
}
#endif
#endif /* DSD_H */
