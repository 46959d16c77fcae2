// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "la.h"

namespace la {

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);

#define LA_HIP(call)                                   \
  do {                                                 \
    hipError_t e__ = (call);                           \
    if (e__ != hipSuccess) return la::hip_fail(e__, #call); \
  } while (0)

#define LA_REQUIRE(cond, status, ...) \
  do {                                \
    if (!(cond)) {                    \
      la::set_error(__VA_ARGS__);     \
      return (status);                \
    }                                 \
  } while (0)

// ---- profiling: every launch goes through Launch so it can be bracketed by events ----
struct ProfScope {
  hipStream_t s;
  int slot;
  ProfScope(const char *name, hipStream_t s);
  ~ProfScope();
};

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Device-side layer record of the generic (any shape, any dtype) path.
struct GenericLayer {
  void *wqkv = nullptr;   // [d, (Hq+2Hkv)*dh]  q | k | v columns
  void *wo = nullptr;     // [Hq*dh, d]
  void *wgu = nullptr;    // [d, 2F]  gate | up columns
  void *wdown = nullptr;  // [F, d]
  float *g_attn = nullptr, *g_mlp = nullptr;
  bool set = false;
};

struct MfmaModel;  // packed bf16 weights + plans of the MFMA path (la_mfma.hip)

}  // namespace la

struct la_model {
  la_model_desc d;
  int device = 0;
  bool use_mfma = false;
  size_t esize = 4;  // bytes per stored weight / cache element
  std::vector<la::GenericLayer> layers;
  void *embed = nullptr, *unembed = nullptr;
  float *g_final = nullptr;
  // scratch of the generic path, sized for LA_MAX_ROWS rows
  float *h = nullptr, *qkv = nullptr, *attn = nullptr, *gu = nullptr, *act = nullptr, *logits = nullptr;
  float *rope_cs = nullptr;  // [LA_MAX_ROWS][dh/2][2] cos, sin at each row's position
  // la_prefill's chunk: residual stream [LA_MAX_ROWS, d], positions and causal masks of its rows
  float *pf_hidden = nullptr;
  int32_t *pf_pos = nullptr;
  uint64_t *pf_vis = nullptr;
  la::MfmaModel *mf = nullptr;
  // Errors raised by kernels (a block that does not fit the cache: 1; a grid barrier that gave up: 4).  err_dev is the
  // device word the kernels OR into (the caches of this model alias it); err_host is one word of mapped pinned host
  // memory (device alias err_map) that a kernel stores its code to when it raises one, so that the next entry point
  // on this model or one of its caches can report the error without synchronising.
  int32_t *err_dev = nullptr;
  int32_t *err_host = nullptr, *err_map = nullptr;
  bool recover = false;          // an error was reported: the next launch clears err_dev and the barrier words first
  unsigned barrier_spins = 0;    // polls of the grid barrier's release word before a workgroup gives up (0: the default)
  int nqkv() const { return (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim; }
  int qdim() const { return d.n_q_heads * d.head_dim; }
  int kvdim() const { return d.n_kv_heads * d.head_dim; }
};

struct la_kv {
  const la_model *m = nullptr;
  int max_len = 0;     // rows the caller may use
  int rows_alloc = 0;  // rows allocated per layer (max_len rounded up to a multiple of 32)
  int n_layers = 0;
  bool v_blocked = false;  // V stored in the MFMA path's key-blocked layout
  void *K = nullptr, *V = nullptr;  // [n_layers][max_len][Hkv][dh] (V: see v_blocked)
  int32_t *L_dev = nullptr;         // committed length, on the device
  int32_t *err_dev = nullptr;       // the model's device error word (not owned)
  int L_bound = 0;                  // host-side upper bound on L
  size_t layer_elems() const { return (size_t)rows_alloc * m->d.n_kv_heads * m->d.head_dim; }
};

struct la_pool {
  int vocab = 0, N = 0, G = 0;
  uint32_t *stamp = nullptr;    // [vocab][G], 0 = empty
  int32_t *toks = nullptr;      // [vocab][G][N-1]
  uint32_t *counter = nullptr;  // global insert counter
};

namespace la {
// Non-blocking: reports (once) an error that a kernel of an earlier launch on this model stored to its host word.
int pending_error(const la_model *m);
// Clears the error word and the barrier words on `s` after an error was reported, so that the next launch starts clean.
int recover_if_needed(la_model *m, hipStream_t s);
#define LA_PENDING(m)                     \
  do {                                    \
    int rc__ = la::pending_error(m);      \
    if (rc__) return rc__;                \
  } while (0)

// generic path (la_generic.hip)
int generic_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos,
                    const uint64_t *vis, la_kv *kv, hipStream_t s);
int generic_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2,
                           hipStream_t s);
int launch_rope_table(la_model *m, const int32_t *pos, int Bp, hipStream_t s);
int launch_argmax_rows(const float *logits, int Bp, int V, int32_t *ids, float *top2, hipStream_t s);

// MFMA path (la_mfma.hip)
int mfma_supported(const la_model_desc *d);
int mfma_create(la_model *m);
void mfma_destroy(la_model *m);
int mfma_set_layer(la_model *m, int layer, const la_layer_weights *w, hipStream_t s);
int mfma_set_head(la_model *m, const void *unembed, hipStream_t s);
int mfma_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos,
                 const uint64_t *vis, la_kv *kv, hipStream_t s);
int mfma_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2,
                        hipStream_t s);
void mfma_reset_sync(la_model *m, hipStream_t s);
int mfma_prefill_rows(const la_model *m);  // rows of one large-M prompt chunk; 0: this model has no large-M path
int mfma_prefill_min();                    // prompts shorter than this go through the block kernel
int mfma_prefill_chunk(la_model *m, la_kv *kv, const int32_t *tok, int M, int L0, hipStream_t s);
int mfma_unembed_argmax_noalloc(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2,
                                hipStream_t s);
}  // namespace la
