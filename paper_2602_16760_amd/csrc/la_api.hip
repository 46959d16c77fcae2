// C-ABI entry points: argument checks, handle lifetime, dispatch to the kernel paths.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>

#include "la_device.h"
#include "la_internal.h"

namespace la {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char *what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return LA_EHIP;
}

// ---- profiling ------------------------------------------------------------------------
struct ProfRec {
  const char *name;
  hipEvent_t a, b;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;
static char g_prof_only[48] = "";

ProfScope::ProfScope(const char *name, hipStream_t s_) : s(s_), slot(-1) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_prof_only[0] && strcmp(g_prof_only, name) != 0) return;
  ProfRec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, s);
  g_prof.push_back(r);
  slot = (int)g_prof.size() - 1;
}
ProfScope::~ProfScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  (void)hipEventRecord(g_prof[slot].b, s);
}

template <typename T>
__global__ void embed_kernel(const T *E, const int32_t *tok, int V, int d, float *hidden) {
  int t = tok[blockIdx.x];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  for (int i = threadIdx.x; i < d; i += blockDim.x)
    hidden[(size_t)blockIdx.x * d + i] = load_as_float<T>(E + (size_t)t * d + i);
}

// rows [row0, row0+n) of one layer <-> row-major [n, Hkv, dh] buffers
template <typename T>
__global__ void kv_copy_kernel(T *Kl, T *Vl, T *k, T *v, int row0, int n, int Hkv, int dh, int v_blocked,
                               int to_cache) {
  int r = blockIdx.x;
  int w = Hkv * dh;
  for (int i = threadIdx.x; i < w; i += blockDim.x) {
    size_t ko = (size_t)(row0 + r) * w + i;
    size_t vo = v_index(v_blocked, row0 + r, i / dh, i % dh, Hkv, dh);
    if (to_cache) {
      Kl[ko] = k[(size_t)r * w + i];
      Vl[vo] = v[(size_t)r * w + i];
    } else {
      k[(size_t)r * w + i] = Kl[ko];
      v[(size_t)r * w + i] = Vl[vo];
    }
  }
}

__global__ void set_i32_kernel(int32_t *p, int32_t v) { *p = v; }

// positions t, t+1, ... and the plain causal masks of a chunk of n rows
__global__ void causal_layout_kernel(int32_t *pos, uint64_t *vis, int t, int n) {
  int i = threadIdx.x;
  if (i < n) {
    pos[i] = t + i;
    vis[i] = i == 63 ? ~0ull : ((1ull << (i + 1)) - 1ull);
  }
}

__global__ void calib_copy_kernel(uint4 *dst, const uint4 *src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

}  // namespace la

using namespace la;

extern "C" const char *la_last_error(void) { return g_err; }

extern "C" int la_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
  return LA_OK;
}

extern "C" int la_profile_select(const char *name) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_only[0] = 0;
  if (name) strncpy(g_prof_only, name, sizeof(g_prof_only) - 1);
  g_prof_only[sizeof(g_prof_only) - 1] = 0;
  return LA_OK;
}

extern "C" int la_profile_read(la_profile_entry *out, int cap) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int n = 0;
  for (auto &r : g_prof) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) == hipSuccess) (void)hipEventElapsedTime(&ms, r.a, r.b);
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
    int j = 0;
    for (; j < n && j < cap; ++j)
      if (strcmp(out[j].name, r.name) == 0) break;
    if (j >= cap) continue;
    if (j == n) {
      memset(&out[j], 0, sizeof(out[j]));
      strncpy(out[j].name, r.name, sizeof(out[j].name) - 1);
      ++n;
    }
    out[j].launches += 1;
    out[j].total_ms += ms;
  }
  g_prof.clear();
  return n;
}

extern "C" int la_profile_copy(void *dst, const void *src, size_t bytes, void *stream) {
  LA_REQUIRE(dst && src && bytes % 16 == 0 && ((uintptr_t)dst | (uintptr_t)src) % 16 == 0, LA_EINVAL,
             "la_profile_copy needs 16-byte aligned pointers and a multiple of 16 bytes");
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps("calib_copy", s);
  calib_copy_kernel<<<2048, 256, 0, s>>>((uint4 *)dst, (const uint4 *)src, bytes / 16);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

namespace la {
int pending_error(const la_model *m) {
  if (!m || !m->err_host) return LA_OK;
  volatile int32_t *w = m->err_host;
  int32_t v = *w;
  if (v == 0) return LA_OK;
  *w = 0;
  const_cast<la_model *>(m)->recover = true;
  if (v & 4) {
    set_error("an earlier launch on this model gave up waiting at a grid barrier (every workgroup of the persistent kernel "
              "must be resident at once); its results are invalid");
    return LA_EHIP;
  }
  set_error("an earlier block did not fit the cache (L + Bp > max_len) and was skipped");
  return LA_ERANGE;
}

int recover_if_needed(la_model *m, hipStream_t s) {
  if (!m->recover) return LA_OK;
  set_i32_kernel<<<1, 1, 0, s>>>(m->err_dev, 0);
  LA_HIP(hipGetLastError());
  if (m->mf) mfma_reset_sync(m, s);
  m->recover = false;
  return LA_OK;
}
}  // namespace la

static void *dev_alloc(size_t bytes) {
  void *p = nullptr;
  if (hipMalloc(&p, bytes ? bytes : 1) != hipSuccess) return nullptr;
  return p;
}

extern "C" void la_free_model(la_model *m) {
  if (!m) return;
  if (m->mf) mfma_destroy(m);
  for (auto &l : m->layers) {
    void *ps[] = {l.wqkv, l.wo, l.wgu, l.wdown, l.g_attn, l.g_mlp};
    for (void *p : ps)
      if (p) (void)hipFree(p);
  }
  void *ps[] = {m->embed, m->unembed, m->g_final, m->h, m->qkv, m->attn, m->gu, m->act, m->logits, m->rope_cs, m->err_dev,
                m->pf_hidden, m->pf_pos, m->pf_vis};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  if (m->err_host) (void)hipHostFree(m->err_host);
  delete m;
}

extern "C" int la_init_model(const la_model_desc *desc, const la_layer_weights *layers, const void *embed,
                             const float *g_final, const void *unembed, void *stream, la_model **out) {
  LA_REQUIRE(out != nullptr, LA_EINVAL, "out is NULL");
  *out = nullptr;
  LA_REQUIRE(desc != nullptr, LA_EINVAL, "desc is NULL");
  const la_model_desc &d = *desc;
  LA_REQUIRE(d.n_layers > 0 && d.d_model > 0 && d.n_q_heads > 0 && d.n_kv_heads > 0 && d.head_dim > 0 &&
                 d.d_ffn > 0 && d.vocab > 0,
             LA_EINVAL, "model dimensions must be positive");
  LA_REQUIRE(d.n_q_heads % d.n_kv_heads == 0, LA_EINVAL, "n_q_heads %d is not a multiple of n_kv_heads %d",
             d.n_q_heads, d.n_kv_heads);
  LA_REQUIRE(d.head_dim % 2 == 0 && d.head_dim <= 256, LA_EINVAL, "head_dim %d must be even and <= 256", d.head_dim);
  LA_REQUIRE(d.dtype == LA_F32 || d.dtype == LA_BF16 || d.dtype == LA_F16, LA_EINVAL, "unknown dtype %d", d.dtype);
  LA_REQUIRE(d.rms_eps >= 0.f && d.rope_theta > 1.f, LA_EINVAL, "bad rms_eps / rope_theta");
  hipStream_t s = (hipStream_t)stream;
  la_model *m = new (std::nothrow) la_model();
  LA_REQUIRE(m != nullptr, LA_ENOMEM, "out of host memory");
  m->d = d;
  m->esize = d.dtype == LA_F32 ? 4 : 2;
  (void)hipGetDevice(&m->device);
  m->layers.resize(d.n_layers);
  const char *force = getenv("LA_FORCE_GENERIC");
  m->use_mfma = (d.dtype == LA_BF16 || d.dtype == LA_F16) && mfma_supported(&d) && !(force && force[0] == '1');
  size_t R = LA_MAX_ROWS;
  bool ok = true;
  ok = ok && (m->rope_cs = (float *)dev_alloc(R * d.head_dim * sizeof(float)));
  ok = ok && (m->err_dev = (int32_t *)dev_alloc(4)) && hipMemset(m->err_dev, 0, 4) == hipSuccess;
  ok = ok && (m->pf_hidden = (float *)dev_alloc(R * d.d_model * 4));
  ok = ok && (m->pf_pos = (int32_t *)dev_alloc(R * 4)) && (m->pf_vis = (uint64_t *)dev_alloc(R * 8));
  ok = ok && hipHostMalloc((void **)&m->err_host, 64, hipHostMallocMapped) == hipSuccess;
  if (ok) {
    memset(m->err_host, 0, 64);
    ok = hipHostGetDevicePointer((void **)&m->err_map, m->err_host, 0) == hipSuccess;
  }
  if (!m->use_mfma) {
    ok = ok && (m->h = (float *)dev_alloc(R * d.d_model * 4));
    ok = ok && (m->qkv = (float *)dev_alloc(R * m->nqkv() * 4));
    ok = ok && (m->attn = (float *)dev_alloc(R * m->qdim() * 4));
    ok = ok && (m->gu = (float *)dev_alloc(R * 2 * (size_t)d.d_ffn * 4));
    ok = ok && (m->act = (float *)dev_alloc(R * (size_t)d.d_ffn * 4));
    if (unembed) ok = ok && (m->logits = (float *)dev_alloc(R * (size_t)d.vocab * 4));
  }
  if (embed) ok = ok && (m->embed = dev_alloc((size_t)d.vocab * d.d_model * m->esize));
  if (g_final) ok = ok && (m->g_final = (float *)dev_alloc((size_t)d.d_model * 4));
  if (unembed && !m->use_mfma) ok = ok && (m->unembed = dev_alloc((size_t)d.vocab * d.d_model * m->esize));
  if (!ok) {
    la_free_model(m);
    set_error("device allocation failed in la_init_model");
    return LA_ENOMEM;
  }
  int rc = LA_OK;
  if (m->use_mfma) rc = mfma_create(m);
  auto fail = [&](int code) {
    la_free_model(m);
    return code;
  };
  if (rc) return fail(rc);
  hipError_t e = hipSuccess;
  if (embed) e = hipMemcpyAsync(m->embed, embed, (size_t)d.vocab * d.d_model * m->esize, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && g_final) e = hipMemcpyAsync(m->g_final, g_final, (size_t)d.d_model * 4, hipMemcpyDeviceToDevice, s);
  if (e == hipSuccess && unembed) {
    if (m->use_mfma) {
      rc = mfma_set_head(m, unembed, s);
      if (rc) return fail(rc);
    } else {
      e = hipMemcpyAsync(m->unembed, unembed, (size_t)d.vocab * d.d_model * m->esize, hipMemcpyDeviceToDevice, s);
    }
  }
  if (e != hipSuccess) return fail(hip_fail(e, "copy of head weights"));
  if (layers)
    for (int l = 0; l < d.n_layers; ++l) {
      rc = la_model_set_layer(m, l, &layers[l], stream);
      if (rc) return fail(rc);
    }
  *out = m;
  return LA_OK;
}

extern "C" int la_model_set_layer(la_model *m, int layer, const la_layer_weights *w, void *stream) {
  LA_REQUIRE(m && w, LA_EINVAL, "NULL argument");
  LA_PENDING(m);
  LA_REQUIRE(layer >= 0 && layer < m->d.n_layers, LA_ERANGE, "layer %d outside [0, %d)", layer, m->d.n_layers);
  LA_REQUIRE(w->wq && w->wk && w->wv && w->wo && w->wgate && w->wup && w->wdown && w->g_attn && w->g_mlp, LA_EINVAL,
             "layer %d: NULL weight pointer", layer);
  hipStream_t s = (hipStream_t)stream;
  const la_model_desc &d = m->d;
  GenericLayer &g = m->layers[layer];
  size_t es = m->esize;
  if (!g.g_attn) g.g_attn = (float *)dev_alloc((size_t)d.d_model * 4);
  if (!g.g_mlp) g.g_mlp = (float *)dev_alloc((size_t)d.d_model * 4);
  LA_REQUIRE(g.g_attn && g.g_mlp, LA_ENOMEM, "device allocation failed");
  LA_HIP(hipMemcpyAsync(g.g_attn, w->g_attn, (size_t)d.d_model * 4, hipMemcpyDeviceToDevice, s));
  LA_HIP(hipMemcpyAsync(g.g_mlp, w->g_mlp, (size_t)d.d_model * 4, hipMemcpyDeviceToDevice, s));
  if (m->use_mfma) {
    int rc = mfma_set_layer(m, layer, w, s);
    if (rc) return rc;
    g.set = true;
    return LA_OK;
  }
  int nqkv = m->nqkv(), qd = m->qdim(), kvd = m->kvdim(), F = d.d_ffn, dm = d.d_model;
  if (!g.wqkv) g.wqkv = dev_alloc((size_t)dm * nqkv * es);
  if (!g.wo) g.wo = dev_alloc((size_t)qd * dm * es);
  if (!g.wgu) g.wgu = dev_alloc((size_t)dm * 2 * F * es);
  if (!g.wdown) g.wdown = dev_alloc((size_t)F * dm * es);
  LA_REQUIRE(g.wqkv && g.wo && g.wgu && g.wdown, LA_ENOMEM, "device allocation failed");
  auto cols = [&](void *dst, int dst_ld, int col0, const void *src, int n_cols, int rows) {
    return hipMemcpy2DAsync((char *)dst + (size_t)col0 * es, (size_t)dst_ld * es, src, (size_t)n_cols * es,
                            (size_t)n_cols * es, rows, hipMemcpyDeviceToDevice, s);
  };
  LA_HIP(cols(g.wqkv, nqkv, 0, w->wq, qd, dm));
  LA_HIP(cols(g.wqkv, nqkv, qd, w->wk, kvd, dm));
  LA_HIP(cols(g.wqkv, nqkv, qd + kvd, w->wv, kvd, dm));
  LA_HIP(cols(g.wgu, 2 * F, 0, w->wgate, F, dm));
  LA_HIP(cols(g.wgu, 2 * F, F, w->wup, F, dm));
  LA_HIP(hipMemcpyAsync(g.wo, w->wo, (size_t)qd * dm * es, hipMemcpyDeviceToDevice, s));
  LA_HIP(hipMemcpyAsync(g.wdown, w->wdown, (size_t)F * dm * es, hipMemcpyDeviceToDevice, s));
  g.set = true;
  return LA_OK;
}

// ---- KV cache -----------------------------------------------------------------------------
extern "C" void la_free_kv(la_kv *kv) {
  if (!kv) return;
  void *ps[] = {kv->K, kv->V, kv->L_dev};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  delete kv;
}

extern "C" int la_kv_alloc(const la_model *m, int max_len, la_kv **out) {
  LA_REQUIRE(out != nullptr, LA_EINVAL, "out is NULL");
  *out = nullptr;
  LA_REQUIRE(m != nullptr && max_len > 0, LA_EINVAL, "bad arguments to la_kv_alloc");
  // the matrix-core path addresses a layer's K (and V) through 32-bit byte offsets
  LA_REQUIRE(!m->use_mfma || ((size_t)max_len + 31) / 32 * 32 * m->d.n_kv_heads * m->d.head_dim * 2 < ((size_t)1 << 31), LA_EINVAL,
             "max_len=%d: one layer's K rows would reach 2 GiB (limit %zu rows for this model)", max_len,
             (((size_t)1 << 31) / ((size_t)m->d.n_kv_heads * m->d.head_dim * 2) - 1) / 32 * 32);
  la_kv *kv = new (std::nothrow) la_kv();
  LA_REQUIRE(kv != nullptr, LA_ENOMEM, "out of host memory");
  kv->m = m;
  kv->max_len = max_len;
  kv->rows_alloc = (max_len + 31) / 32 * 32;
  kv->n_layers = m->d.n_layers;
  kv->v_blocked = m->use_mfma;
  size_t bytes = kv->layer_elems() * kv->n_layers * m->esize;
  kv->K = dev_alloc(bytes);
  kv->V = dev_alloc(bytes);
  kv->L_dev = (int32_t *)dev_alloc(4);
  kv->err_dev = m->err_dev;
  if (!kv->K || !kv->V || !kv->L_dev) {
    la_free_kv(kv);
    set_error("KV cache allocation of 2 x %zu bytes failed", bytes);
    return LA_ENOMEM;
  }
  // zero everything once: rows of the key-blocked V layout are read in blocks of 32
  if (hipMemset(kv->K, 0, bytes) != hipSuccess || hipMemset(kv->V, 0, bytes) != hipSuccess ||
      hipMemset(kv->L_dev, 0, 4) != hipSuccess) {
    la_free_kv(kv);
    set_error("KV cache clear failed");
    return LA_EHIP;
  }
  *out = kv;
  return LA_OK;
}

extern "C" int la_kv_set_len(la_kv *kv, int L, void *stream) {
  LA_REQUIRE(kv != nullptr, LA_EINVAL, "kv is NULL");
  LA_PENDING(kv->m);
  LA_REQUIRE(L >= 0 && L <= kv->max_len, LA_ERANGE, "L=%d outside [0, %d]", L, kv->max_len);
  set_i32_kernel<<<1, 1, 0, (hipStream_t)stream>>>(kv->L_dev, L);
  LA_HIP(hipGetLastError());
  kv->L_bound = L;
  return LA_OK;
}

extern "C" int la_kv_get_len(la_kv *kv, int *L_host, void *stream) {
  LA_REQUIRE(kv && L_host, LA_EINVAL, "NULL argument");
  int32_t v[2] = {0, 0};
  LA_HIP(hipMemcpyAsync(&v[0], kv->L_dev, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
  LA_HIP(hipMemcpyAsync(&v[1], kv->err_dev, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
  LA_HIP(hipStreamSynchronize((hipStream_t)stream));
  *L_host = v[0];
  kv->L_bound = v[0];
  if (v[1] != 0) {  // the stream has drained: the device word is final; report it once and start clean
    la_model *mm = const_cast<la_model *>(kv->m);
    *(volatile int32_t *)mm->err_host = 0;
    mm->recover = true;
  }
  LA_REQUIRE((v[1] & 4) == 0, LA_EHIP, "a grid barrier timed out: the persistent kernel needs every workgroup resident at once");
  LA_REQUIRE(v[1] == 0, LA_ERANGE, "a block did not fit the cache (L + Bp > max_len) and was skipped");
  LA_PENDING(kv->m);
  return LA_OK;
}

static int kv_copy(la_kv *kv, int layer, int row0, void *k, void *v, int n, int to_cache, hipStream_t s) {
  LA_REQUIRE(kv != nullptr, LA_EINVAL, "kv is NULL");
  LA_PENDING(kv->m);
  if (n == 0) return LA_OK;
  LA_REQUIRE(k && v, LA_EINVAL, "NULL argument");
  LA_REQUIRE(layer >= 0 && layer < kv->n_layers, LA_ERANGE, "layer %d outside [0, %d)", layer, kv->n_layers);
  LA_REQUIRE(n >= 0 && row0 >= 0 && row0 + n <= kv->max_len, LA_ERANGE, "rows [%d, %d) outside the cache (max_len %d)",
             row0, row0 + n, kv->max_len);
  if (n == 0) return LA_OK;
  const la_model_desc &d = kv->m->d;
  size_t off = (size_t)layer * kv->layer_elems();
  ProfScope ps("kv_copy", s);
  if (d.dtype == LA_F32)
    kv_copy_kernel<float><<<n, 256, 0, s>>>((float *)kv->K + off, (float *)kv->V + off, (float *)k, (float *)v, row0, n,
                                            d.n_kv_heads, d.head_dim, kv->v_blocked, to_cache);
  else
    kv_copy_kernel<uint16_t><<<n, 256, 0, s>>>((uint16_t *)kv->K + off, (uint16_t *)kv->V + off, (uint16_t *)k,
                                               (uint16_t *)v, row0, n, d.n_kv_heads, d.head_dim, kv->v_blocked, to_cache);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

extern "C" int la_kv_fill(la_kv *kv, int layer, int row0, const void *k, const void *v, int n, void *stream) {
  return kv_copy(kv, layer, row0, (void *)k, (void *)v, n, 1, (hipStream_t)stream);
}
extern "C" int la_kv_read(la_kv *kv, int layer, int row0, int n, void *k, void *v, void *stream) {
  return kv_copy(kv, layer, row0, k, v, n, 0, (hipStream_t)stream);
}

// ---- the step -----------------------------------------------------------------------------
extern "C" int la_embed(la_model *m, const int32_t *tok, int Bp, float *hidden, void *stream) {
  LA_REQUIRE(m && tok && hidden, LA_EINVAL, "NULL argument");
  LA_PENDING(m);
  LA_REQUIRE(Bp >= 1 && Bp <= LA_MAX_ROWS, LA_EINVAL, "Bp=%d outside [1, %d]", Bp, LA_MAX_ROWS);
  LA_REQUIRE(m->embed != nullptr, LA_EINVAL, "model was created without an embedding table");
  hipStream_t s = (hipStream_t)stream;
  ProfScope ps("embed", s);
  if (m->d.dtype == LA_F32)
    embed_kernel<float><<<Bp, 256, 0, s>>>((const float *)m->embed, tok, m->d.vocab, m->d.d_model, hidden);
  else if (m->d.dtype == LA_F16)
    embed_kernel<_Float16><<<Bp, 256, 0, s>>>((const _Float16 *)m->embed, tok, m->d.vocab, m->d.d_model, hidden);
  else
    embed_kernel<uint16_t><<<Bp, 256, 0, s>>>((const uint16_t *)m->embed, tok, m->d.vocab, m->d.d_model, hidden);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

extern "C" int la_forward_layers(la_model *m, int layer_begin, int layer_end, float *hidden, int Bp,
                                 const int32_t *pos, const uint64_t *vis, la_kv *kv, void *stream) {
  LA_REQUIRE(m && hidden && pos && vis && kv, LA_EINVAL, "NULL argument");
  LA_REQUIRE(kv->m == m, LA_EINVAL, "the cache belongs to another model");
  LA_PENDING(m);
  LA_REQUIRE(Bp >= 1 && Bp <= LA_MAX_ROWS, LA_EINVAL, "Bp=%d outside [1, %d]", Bp, LA_MAX_ROWS);
  LA_REQUIRE(layer_begin >= 0 && layer_begin <= layer_end && layer_end <= m->d.n_layers, LA_ERANGE,
             "layers [%d, %d) outside the model's %d layers", layer_begin, layer_end, m->d.n_layers);
  hipStream_t s = (hipStream_t)stream;
  if (kv->L_bound + Bp > kv->max_len) {  // the bound is loose after accepts: get the exact length
    int L = 0;
    int rc = la_kv_get_len(kv, &L, stream);
    if (rc) return rc;
    LA_REQUIRE(L + Bp <= kv->max_len, LA_ERANGE, "block of %d rows at L=%d exceeds max_len %d", Bp, L, kv->max_len);
  }
  for (int l = layer_begin; l < layer_end; ++l)
    LA_REQUIRE(m->layers[l].set, LA_EINVAL, "layer %d has no weights", l);
  {
    int rc = recover_if_needed(m, s);
    if (rc) return rc;
  }
  if (m->use_mfma) return mfma_forward(m, layer_begin, layer_end, hidden, Bp, pos, vis, kv, s);
  return generic_forward(m, layer_begin, layer_end, hidden, Bp, pos, vis, kv, s);
}

extern "C" int la_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, void *stream) {
  LA_REQUIRE(m && hidden && ids, LA_EINVAL, "NULL argument");
  LA_REQUIRE(Bp >= 1 && Bp <= LA_MAX_ROWS, LA_EINVAL, "Bp=%d outside [1, %d]", Bp, LA_MAX_ROWS);
  LA_REQUIRE(m->g_final && (m->unembed || m->use_mfma), LA_EINVAL, "model was created without final norm / unembedding");
  LA_PENDING(m);
  hipStream_t s = (hipStream_t)stream;
  {
    int rc = recover_if_needed(m, s);
    if (rc) return rc;
  }
  if (m->use_mfma) return mfma_unembed_argmax(m, hidden, Bp, ids, top2, s);
  return generic_unembed_argmax(m, hidden, Bp, ids, top2, s);
}

extern "C" int la_unembed_argmax_noalloc(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, void *stream) {
  LA_REQUIRE(m && hidden && ids, LA_EINVAL, "NULL argument");
  LA_REQUIRE(Bp >= 1 && Bp <= LA_MAX_ROWS, LA_EINVAL, "Bp=%d outside [1, %d]", Bp, LA_MAX_ROWS);
  LA_REQUIRE(m->use_mfma, LA_EINVAL, "only models on the matrix-core path (LA_BF16 or LA_F16, supported shape) have this entry point");
  LA_REQUIRE(m->g_final, LA_EINVAL, "model was created without final norm / unembedding");
  LA_PENDING(m);
  {
    int rc = recover_if_needed(m, (hipStream_t)stream);
    if (rc) return rc;
  }
  return mfma_unembed_argmax_noalloc(m, hidden, Bp, ids, top2, (hipStream_t)stream);
}

extern "C" int la_set_barrier_timeout(la_model *m, unsigned polls) {
  LA_REQUIRE(m != nullptr, LA_EINVAL, "NULL argument");
  m->barrier_spins = polls;
  return LA_OK;
}

extern "C" int la_causal_layout(int t, int n, int32_t *pos_host, uint64_t *vis_host) {
  LA_REQUIRE(pos_host && vis_host, LA_EINVAL, "NULL output");
  LA_REQUIRE(n >= 1 && n <= LA_MAX_ROWS && t >= 0, LA_EINVAL, "n=%d outside [1, %d] or t=%d negative", n, LA_MAX_ROWS, t);
  for (int i = 0; i < n; ++i) {
    pos_host[i] = t + i;
    vis_host[i] = i == 63 ? ~0ull : ((1ull << (i + 1)) - 1ull);
  }
  return LA_OK;
}

// ---- latency model of the split deployment (host arithmetic, double) ------------------------------
extern "C" int la_rtt_fixed_overhead(double per_step_ms, double rtt_ms, double *fixed_ms) {
  LA_REQUIRE(fixed_ms != nullptr, LA_EINVAL, "NULL output");
  LA_REQUIRE(rtt_ms >= 0.0 && per_step_ms >= rtt_ms, LA_EINVAL, "a step of %g ms cannot contain a round trip of %g ms", per_step_ms, rtt_ms);
  *fixed_ms = per_step_ms - rtt_ms;
  return LA_OK;
}

extern "C" int la_rtt_project(double tokens_per_step, double rtt_ms, double fixed_ms, double *tok_per_s) {
  LA_REQUIRE(tok_per_s != nullptr, LA_EINVAL, "NULL output");
  LA_REQUIRE(tokens_per_step > 0.0 && rtt_ms >= 0.0 && fixed_ms >= 0.0 && rtt_ms + fixed_ms > 0.0, LA_EINVAL,
             "need tokens_per_step > 0 and a positive step time (rtt %g ms + fixed %g ms)", rtt_ms, fixed_ms);
  *tok_per_s = tokens_per_step / ((rtt_ms + fixed_ms) / 1000.0);
  return LA_OK;
}

extern "C" int la_jacobi_project(int k, double iterations, double rtt_ms, double *tok_per_s) {
  LA_REQUIRE(tok_per_s != nullptr, LA_EINVAL, "NULL output");
  LA_REQUIRE(k >= 1 && iterations > 0.0 && rtt_ms > 0.0, LA_EINVAL, "need k >= 1, iterations > 0 and rtt > 0");
  *tok_per_s = (double)k / (iterations * rtt_ms / 1000.0);
  return LA_OK;
}

extern "C" int la_prefill(la_model *m, la_kv *kv, const int32_t *tok, int n, int L0, void *stream) {
  LA_REQUIRE(m && kv && (tok || n == 0), LA_EINVAL, "NULL argument");
  LA_REQUIRE(kv->m == m, LA_EINVAL, "the cache belongs to another model");
  LA_REQUIRE(m->embed != nullptr, LA_EINVAL, "model was created without an embedding table");
  LA_REQUIRE(n >= 0 && L0 >= 0 && (long long)L0 + n <= kv->max_len, LA_ERANGE, "rows [%d, %d) outside the cache (max_len %d)", L0,
             L0 + n, kv->max_len);
  hipStream_t s = (hipStream_t)stream;
  int rc = la_kv_set_len(kv, L0, stream);
  if (!rc && m->use_mfma && mfma_prefill_rows(m) > 0 && n >= mfma_prefill_min()) {
    // the large-M pass: one matrix product per weight matrix and prompt chunk
    for (int l = 0; l < m->d.n_layers; ++l) LA_REQUIRE(m->layers[l].set, LA_EINVAL, "layer %d has no weights", l);
    if ((rc = recover_if_needed(m, s))) return rc;
    const int rows = mfma_prefill_rows(m);
    for (int done = 0; !rc && done < n; done += rows) {
      const int M = n - done < rows ? n - done : rows;
      rc = mfma_prefill_chunk(m, kv, tok + done, M, L0 + done, s);
      if (!rc) rc = la_kv_set_len(kv, L0 + done + M, stream);
    }
    return rc;
  }
  for (int done = 0; !rc && done < n; done += LA_MAX_ROWS) {
    const int rows = n - done < LA_MAX_ROWS ? n - done : LA_MAX_ROWS;
    rc = la_embed(m, tok + done, rows, m->pf_hidden, stream);
    if (rc) break;
    causal_layout_kernel<<<1, 64, 0, s>>>(m->pf_pos, m->pf_vis, L0 + done, rows);
    LA_HIP(hipGetLastError());
    rc = la_forward_layers(m, 0, m->d.n_layers, m->pf_hidden, rows, m->pf_pos, m->pf_vis, kv, stream);
    if (rc) break;
    rc = la_kv_set_len(kv, L0 + done + rows, stream);
  }
  return rc;
}
