// ee_internal.h -- host-side structures and kernel launchers shared by the
// translation units of libee.  Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <string>
#include <vector>

#include "ee.h"

struct ExitWeights {
    const float* gain = nullptr;
    const void*  w = nullptr;
    bool set = false;
};

struct ee_model {
    ee_model_config cfg;
    std::vector<ee_layer_weights> layers;   // index 0 = layer 1
    std::vector<char> resident;
    ExitWeights exits[EE_MAX_EXITS];
    const void* emb = nullptr;
    float* d_rope = nullptr;                // [max_pos][hd/2][2] (cos, sin), device
    const void**  d_wqkv_tab = nullptr;     // device [n_layers]: w_qkv of each layer (null if not resident)
    const float** d_gattn_tab = nullptr;    // device [n_layers]: g_attn of each layer
    int device = 0;
};

struct ee_kv {
    char*    pool = nullptr;
    size_t   bytes = 0;
    int      n_layers = 0;
    int      B = 0;
    int64_t  T = 0;                         // total positions over all rows
    int32_t* d_cap = nullptr;               // device [B]
    int64_t* d_off = nullptr;               // device [B]: T_b
    std::vector<int32_t> h_cap;
    std::vector<int64_t> h_off;
};

// byte offsets inside the workspace
struct WsLayout {
    size_t x, qkv, q_hi, q_lo, ao, act, part_max, part_sum, part_arg, logits, fill_x, fill_kv, total;
    size_t gemm_part, gemm_part_bytes;                            // K-slice partial planes
    size_t attn_part, attn_part_bytes;                            // attention position shares
    size_t attn_order;                                            // int32 [Mpad]: list entries, longest context first
    size_t kv_seq;                                                // int32 [Mpad]: cache row of each entry (context pass)
    size_t gone_idx, n_gone;                                      // int32 [Mpad], int32: rows that left at any exit of the running step
};

struct ee_batch {
    const ee_model* m = nullptr;
    int B = 0;
    int Mpad = 0;                           // B rounded up to 32
    char* state = nullptr;
    char* ws = nullptr;
    ee_batch_layout L;
    WsLayout W;
    const int32_t* kv_seq = nullptr;        // device [Mpad], set only while a context pass runs: entry -> cache row
    template <class T> T* st(size_t off) const { return reinterpret_cast<T*>(state + off); }
    template <class T> T* wsp(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

// ----------------------------------------------------------------- errors
void ee_set_error(const std::string& msg);
int  ee_fail(int code, const std::string& msg);
#define EE_HIP_CHECK(expr)                                                              \
    do {                                                                                \
        hipError_t _e = (expr);                                                         \
        if (_e != hipSuccess)                                                           \
            return ee_fail(EE_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(_e)); \
    } while (0)
#define EE_LAUNCH_CHECK()  EE_HIP_CHECK(hipGetLastError())

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ----------------------------------------------------------------- kernel timing (opt-in)
// Every launch of a kernel class whose bit is set in the mask is bracketed by a pair of
// HIP events on the launch stream; ee_timing_read adds up the elapsed times.
void ee_timing_mark(int kind, hipStream_t s, bool begin);
extern unsigned g_ee_timing_mask;
struct TimedScope {
    int kind; hipStream_t s; bool on;
    TimedScope(int k, hipStream_t st) : kind(k), s(st), on((g_ee_timing_mask >> k) & 1u) { if (on) ee_timing_mark(kind, s, true); }
    ~TimedScope() { if (on) ee_timing_mark(kind, s, false); }
};

// Per-(layer,row,head) addressing of the key/value pool, passed by value to kernels.
struct KvView {
    char*          pool;
    const int32_t* cap;      // device [B]
    const int64_t* off;      // device [B]
    int64_t        T;
    int32_t        n_kv_heads;
    int32_t        head_dim;
    int32_t        layer0;   // layer - 1
    const int32_t* seq;      // device: cache row of a batch row, or null when batch row b owns cache row b
};

// ----------------------------------------------------------------- launchers
// common (ee_kernels_common.hip)
int launch_rope_table(float* d_table, int max_pos, int hd, double theta, hipStream_t s);
int launch_begin_step(const ee_model* m, ee_batch* b, hipStream_t s);
int launch_end_step(ee_batch* b, hipStream_t s);
int launch_reset(ee_batch* b, const int32_t* tok, const int32_t* pos, const float* scale, hipStream_t s);
int launch_set_scale(ee_batch* b, const float* scale, hipStream_t s);
int launch_compact(ee_batch* b, int exit_idx, int exit_layer, hipStream_t s);
int launch_exit_decide(ee_batch* b, int n_part, float th, int force, hipStream_t s);
int launch_prefill_begin(const ee_model* m, const ee_kv* kv, ee_batch* b, const int32_t* tok, const int32_t* pos,
                         const int32_t* seq, int n, hipStream_t s);
int launch_set_layer_ptrs(ee_model* m, int layer, const void* w_qkv, const float* g_attn, hipStream_t s);
int launch_hstore_put(const ee_model* m, const ee_kv* kv, const ee_batch* b, int n, bool entries, float* store,
                      hipStream_t s);
int launch_backfill_begin(const ee_model* m, const ee_kv* kv, ee_batch* b, const float* store, const int32_t* pos,
                          const int32_t* seq, int n, hipStream_t s);
int launch_verify_begin(const ee_model* m, const ee_kv* kv, const ee_batch* b, ee_batch* vb, int k, const float* store,
                        hipStream_t s);
int launch_accept_drafts(ee_batch* b, const ee_batch* vb, int k, const int32_t* drafts, int32_t* n_emit, int32_t* emit,
                         hipStream_t s);
int launch_cbc_init(void* st, int window, int cbc_max, hipStream_t s);
int launch_cbc_push(void* st, const uint8_t* flags, int n, hipStream_t s);
int launch_pht_init(void* row, hipStream_t s);
int launch_pht_push(void* row, const ee_model* m, const ee_batch* b, hipStream_t s);
int launch_pack_weight(const void* src, int n_out, int n_in, void* dst, int row_off, int row_stride,
                       int dst_rows, hipStream_t s);
int launch_kv_copy_context(const ee_model* m, const ee_kv* kv, int layer, int row, int pos0, int n_pos,
                           void* k, void* v, bool to_pool, hipStream_t s);

// fp32 path (ee_kernels_f32.hip)
int f32_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, hipStream_t s);
int f32_exit_head(const ee_model* m, int e, float th, int force, ee_batch* b, float* dbg, hipStream_t s);
int f32_fill_kv(const ee_model* m, int from_excl, int to_incl, ee_kv* kv, ee_batch* b, hipStream_t s);

// bf16 path (ee_kernels_bf16.hip)
int bf16_layer_forward(const ee_model* m, int layer, ee_kv* kv, ee_batch* b, hipStream_t s, bool x_ready = false,
                       const float* tail_gain = nullptr, bool* x_done = nullptr);
int bf16_exit_head(const ee_model* m, int e, float th, int force, ee_batch* b, float* dbg, hipStream_t s,
                   bool x_ready = false);
// rows: the batch's exited_idx / n_exited unless another device list (idx, n_ptr) is given
int bf16_fill_kv(const ee_model* m, int from_excl, int to_incl, ee_kv* kv, ee_batch* b, hipStream_t s,
                 const int32_t* idx = nullptr, const int32_t* n_ptr = nullptr);
