// Internal declarations shared by the translation units of libdsd (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "dsd.h"

// ----------------------------------------------------------------------------- errors
void dsd_set_error(const char* fmt, ...);
#define DSD_FAIL(code, ...)          \
    do {                             \
        dsd_set_error(__VA_ARGS__);  \
        return (code);               \
    } while (0)
#define DSD_HIP(expr)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (expr);                                                            \
        if (e_ != hipSuccess) DSD_FAIL(DSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_));  \
    } while (0)
#define DSD_TRY(expr)          \
    do {                       \
        int rc_ = (expr);      \
        if (rc_ != DSD_OK) return rc_; \
    } while (0)

// ----------------------------------------------------------------------------- bf16 bits
typedef unsigned short bf16_t;  // storage only

__host__ __device__ inline float bf16_to_f32(bf16_t b) {
    union { unsigned u; float f; } c;
    c.u = ((unsigned)b) << 16;
    return c.f;
}
__host__ __device__ inline bf16_t f32_to_bf16(float f) {  // round to nearest even
    union { unsigned u; float f; } c;
    c.f = f;
    unsigned u = c.u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
template <typename T> __device__ inline float ld_f32(const T* p);
template <> __device__ inline float ld_f32<float>(const float* p) { return *p; }
template <> __device__ inline float ld_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void st_f32(T* p, float v);
template <> __device__ inline void st_f32<float>(float* p, float v) { *p = v; }
template <> __device__ inline void st_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ----------------------------------------------------------------------------- KV cache layout
// Both caches are kept in the order in which the attention kernel's matrix instructions take their
// operands, so that a wavefront fetches every operand fragment as one contiguous 1 KiB (hd = 128)
// piece, lane l taking bytes 16l .. 16l+15.  Per layer the order is block of 32 slots, sequence, kv
// head: [S/32][Bmax][Hkv][block], and inside a block
//   K : [2][hd/8][16][8]             tile of 16 slots; inside it feature group e/8, slot, feature e%8
//   V : [hd/16][4][16][8]            feature tile e/16, then the slot's place p = v_slot_perm(slot % 32)
//                                    in the P*V product as p/8, feature e%16, p%8
// Slot blocks come first because every (sequence, head) is walked from its first key on at about the
// same pace: what the chip reads at any moment is then one advancing band of each cache, not a band
// per head a whole sequence's cache apart (the same reason the weights are stored k-step major).
// v_slot_perm is the order in which the score tiles of S^T = K Q^T hand their keys to the P*V
// product: key 16*tile + 4g + i sits at reduction index 8g + 4*tile + i.
// S (slots per sequence) is a multiple of 64.
struct KvGeom {
    int Hkv, hd, S, Bmax;
    size_t layer_elems;  // Bmax * Hkv * S * hd
};
__host__ __device__ inline int v_slot_perm(int s32) {
    const int tile = s32 >> 4, r = s32 & 15;
    return ((r >> 2) << 3) + (r & 3) + (tile << 2);
}
__host__ __device__ inline size_t kv_block_off(const KvGeom& g, int b, int h, int slot) {
    return ((size_t)(slot >> 5) * (g.Bmax * g.Hkv) + (size_t)(b * g.Hkv + h)) * (size_t)(32 * g.hd);
}
__host__ __device__ inline size_t kv_k_off(const KvGeom& g, int b, int h, int slot, int e) {
    return kv_block_off(g, b, h, slot) + (size_t)(slot & 16) * g.hd + (size_t)(e >> 3) * 128 + (slot & 15) * 8 + (e & 7);
}
__host__ __device__ inline size_t kv_v_off(const KvGeom& g, int b, int h, int slot, int e) {
    const int p = v_slot_perm(slot & 31);
    return kv_block_off(g, b, h, slot) + (size_t)(e >> 4) * 512 + (p >> 3) * 128 + (e & 15) * 8 + (p & 7);
}

// ----------------------------------------------------------------------------- handles
struct ProfRec {
    int cls;
    hipEvent_t e0, e1;
};

struct dsd_ctx {
    int device;
    hipStream_t stream;
    char* ws;
    size_t ws_bytes;
    bool force_simple;  // DSD_PATH=simple: run the generic kernels also for bf16 models
    bool prof_on;
    std::vector<ProfRec> prof;
    int* sat_dev;                  // activations that left the fp16 range on their way into a matrix-core operand (dsd_stage_status)
    bool no_tiled;                 // DSD_NO_TILED set: the one-workgroup-per-tile GEMMs at every row count (testing)
    int n_cu;
};

// Brackets the launches of one scope with a pair of events when profiling is on.
struct ProfScope {
    dsd_ctx* c;
    ProfRec r;
    ProfScope(dsd_ctx* ctx, int cls) : c(ctx) {
        r.cls = cls;
        r.e0 = r.e1 = nullptr;
        if (c->prof_on && hipEventCreate(&r.e0) == hipSuccess && hipEventCreate(&r.e1) == hipSuccess)
            (void)hipEventRecord(r.e0, c->stream);
    }
    ~ProfScope() {
        if (c->prof_on && r.e0 && r.e1) {
            (void)hipEventRecord(r.e1, c->stream);
            c->prof.push_back(r);
        }
    }
};

struct LayerW {
    // plain copies (generic path), in the model dtype
    void *g1, *wq, *wk, *wv, *wo, *g2, *wg, *wu, *wd;
    // MFMA-tiled copies (bf16 fast path)
    void *qkv_t, *wo_t, *gu_t, *wd_t;
};

struct dsd_weights {
    dsd_model_desc desc;
    bool tiled;  // true: *_t members valid (bf16 fast path); false: plain members valid
    void* embed;
    void* gf;
    void* lm;
    void* lm_t;
    std::vector<LayerW> layers;
    std::vector<void*> allocs;
};

struct dsd_kv {
    dsd_model_desc desc;
    KvGeom geom;
    void* k;           // [L] layers of geom.layer_elems
    void* v;
    int32_t* len_dev;  // [Bmax] committed lengths (the truth)
    std::vector<int32_t> len_bound;  // host upper bounds, used to size grids and validate
    int last_k;        // rows written by the last dsd_stage_verify
    int cap;           // slots per sequence the caller asked for (<= geom.S)
};

inline size_t dsd_elem_size(int dtype) { return dtype == DSD_BF16 ? 2 : 4; }
int dsd_ws_reserve(dsd_ctx* ctx, size_t bytes);

// A bump allocator over the context workspace (256-byte aligned pieces).
struct WsBump {
    char* base;
    size_t off;
    template <typename T> T* take(size_t n) {
        T* p = (T*)(base + off);
        off += (n * sizeof(T) + 255) & ~(size_t)255;
        return p;
    }
};

// ----------------------------------------------------------------------------- launchers
// generic path (dsd_simple.hip)
int simple_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                        const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth, int B,
                        int k, void* hidden_out, float* logits, int64_t logits_seq_stride);
// bf16 MFMA path (dsd_stage_bf16.hip)
int mfma_supported(const dsd_model_desc* d);
int mfma_weights_tile(dsd_ctx* ctx, dsd_weights* w, const void* const* tensors);
int mfma_stage_verify(dsd_ctx* ctx, const dsd_weights* w, dsd_kv* kv, const void* hidden_in,
                      const int32_t* draft_tokens, const uint64_t* tree_mask, const int32_t* depth, int B,
                      int k, void* hidden_out, float* logits, int64_t logits_seq_stride);
// weight-streaming GEMMs for up to 128 rows (dsd_gemm_tiled.hip)
int tiled_supported(const dsd_model_desc* d);
// rope[m][e] = (cos, sin) of (len[m/k] + depth[m%k]) * theta^(-2e/128), e < 64, worked out in fp64
void rope_table_launch(dsd_ctx* ctx, float2* rope, const int32_t* len, const int32_t* depth, int M, int k, float theta);
#define TILED_MAX_KSPLIT 16
int tiled_row_tiles(int M);
int tiled_gemm_resid(dsd_ctx* ctx, const void* Wt, float* part, int* n_part, int M, int N, int K, const void* panel);
int tiled_resid_reduce(dsd_ctx* ctx, float* x, const float* part, int n_part, int M, int N, void* hidden_out);
int tiled_gemm_qkv(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, float* part, int x_pending, int M, int N,
                   int K, float* q, bf16_t* kc, bf16_t* vc, const KvGeom& g, const int32_t* len,
                   int k, int Hq, float eps, const float2* rope, void* panel, float* ssq);
int tiled_gemm_swiglu(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, const float* part, int x_pending,
                      void* panel_h, int M, int F, int K, float eps, void* panel, float* ssq);
int tiled_gemm_logits(dsd_ctx* ctx, const void* Wt, float* x, const bf16_t* gain, const float* part, int x_pending,
                      float* logits, int M, int V, int K, float eps, int rows_per_seq, int64_t seq_stride, void* panel,
                      float* ssq);
// KV utilities (dsd_kv.hip)
int kv_import_launch(dsd_ctx* ctx, dsd_kv* kv, int layer, const void* k, const void* v, int B, int n_slots);
int kv_export_launch(dsd_ctx* ctx, const dsd_kv* kv, int layer, int first, int n, int B, void* k, void* v);
int kv_commit_launch(dsd_ctx* ctx, dsd_kv* kv, const int32_t* acc_len, const int32_t* acc_path, int B, int k);
// accept (dsd_accept.hip)
size_t accept_scratch_bytes(int B, int k, int V, int top_m);
int accept_static_scratch_init(int device);                  // with `device` current; once per device
char* accept_static_scratch(int device, size_t* bytes);      // device address of this device's static scratch (NULL if none)
int accept_launch(dsd_ctx* ctx, const float* logits, const float* draft_probs, const int32_t* draft_tokens,
                  const int32_t* parent, const float* uniforms, const dsd_accept_params* prm, int B, int k,
                  int V, int32_t* accepted_len, int32_t* next_token, int32_t* accepted_path,
                  const dsd_accept_stats* stats, char* scratch);
