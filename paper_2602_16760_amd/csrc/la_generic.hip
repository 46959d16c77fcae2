// Any-shape kernels in fp32 arithmetic: the LA_F32 model's compute path, and the path of
// LA_BF16 models whose shape the MFMA kernels do not cover.  Plain, one op per kernel:
// these shapes are small (the tiny decoder of the test configuration), so clarity wins.
#include "la_device.h"
#include "la_internal.h"

namespace la {

// cos/sin of pos[b] * theta^(-2i/dh), evaluated in double so that the float result is
// correctly rounded for every position the cache can hold.
__global__ void rope_table_kernel(const int32_t *pos, int Bp, int half, double theta, float *cs) {
  int b = blockIdx.x;
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    double inv = exp2(-(double)i / (double)half * log2(theta));
    double phi = (double)pos[b] * inv;
    double s, c;
    sincos(phi, &s, &c);
    cs[((size_t)b * half + i) * 2 + 0] = (float)c;
    cs[((size_t)b * half + i) * 2 + 1] = (float)s;
  }
}

__device__ __forceinline__ float block_sum(float v, float *red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

__device__ __forceinline__ float block_max(float v, float *red) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// out[b,:] = x[b,:] * rsqrt(mean(x[b,:]^2) + eps) * g
__global__ void rmsnorm_kernel(const float *x, const float *g, float eps, int d, float *out) {
  __shared__ float red[8];
  const float *xr = x + (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) ss += xr[i] * xr[i];
  ss = block_sum(ss, red);
  float r = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[(size_t)blockIdx.x * d + i] = xr[i] * r * g[i];
}

// C[M,N] (=|+=) A[M,K] W[K,N].  One thread owns one column for 8 rows.
template <typename T>
__global__ void gemm_generic_kernel(const float *A, int lda, const T *W, int ldw, float *C, int ldc, int M,
                                    int K, int N, int accumulate) {
  constexpr int KT = 128, MR = 8;
  __shared__ float As[MR][KT];
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  int m0 = blockIdx.y * MR;
  float acc[MR];
#pragma unroll
  for (int i = 0; i < MR; ++i) acc[i] = 0.f;
  for (int k0 = 0; k0 < K; k0 += KT) {
    __syncthreads();
    for (int e = threadIdx.x; e < MR * KT; e += blockDim.x) {
      int i = e / KT, kk = e % KT;
      As[i][kk] = (m0 + i < M && k0 + kk < K) ? A[(size_t)(m0 + i) * lda + k0 + kk] : 0.f;
    }
    __syncthreads();
    if (n < N) {
      int kmax = min(KT, K - k0);
      for (int kk = 0; kk < kmax; ++kk) {
        float w = load_as_float<T>(W + (size_t)(k0 + kk) * ldw + n);
#pragma unroll
        for (int i = 0; i < MR; ++i) acc[i] = fmaf(As[i][kk], w, acc[i]);
      }
    }
  }
  if (n < N) {
#pragma unroll
    for (int i = 0; i < MR; ++i)
      if (m0 + i < M) {
        float *c = C + (size_t)(m0 + i) * ldc + n;
        *c = accumulate ? (*c + acc[i]) : acc[i];
      }
  }
}

// Rotates q (in place) and k by the row's position and writes k, v to cache rows L+b.
template <typename T>
__global__ void rope_kvwrite_kernel(float *qkv, int Hq, int Hkv, int dh, const float *cs, T *Kc, T *Vc,
                                    const int32_t *L_dev, int max_len, int Bp, int32_t *err, int32_t *err_map) {
  int b = blockIdx.x;
  int L = *L_dev;
  if (L < 0 || L + Bp > max_len) {
    if (threadIdx.x == 0) {  // the device word, and the host's mapped word (read without synchronising)
      *err = 1;
      __hip_atomic_store(err_map, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    return;
  }
  int half = dh / 2;
  int nq = Hq * dh, nkv = Hkv * dh;
  float *row = qkv + (size_t)b * (nq + 2 * nkv);
  for (int e = threadIdx.x; e < (Hq + Hkv) * half; e += blockDim.x) {
    int hd = e / half, i = e % half;
    float c = cs[((size_t)b * half + i) * 2], s = cs[((size_t)b * half + i) * 2 + 1];
    float *u = row + hd * dh;  // q heads then k heads are contiguous
    float x0 = u[i], x1 = u[i + half];
    float y0 = x0 * c - x1 * s, y1 = x1 * c + x0 * s;
    if (hd < Hq) {
      u[i] = y0;
      u[i + half] = y1;
    } else {
      int h = hd - Hq;
      size_t o = ((size_t)(L + b) * Hkv + h) * dh;
      store_from_float<T>(Kc + o + i, y0);
      store_from_float<T>(Kc + o + i + half, y1);
    }
  }
  for (int e = threadIdx.x; e < nkv; e += blockDim.x)
    store_from_float<T>(Vc + (size_t)(L + b) * nkv + e, row[nq + nkv + e]);
}

// One workgroup per (row b, query head): online softmax over the visible keys in chunks
// of blockDim.x keys.  Scores and probabilities in float.
template <typename T>
__global__ void attention_generic_kernel(const float *qkv, int Hq, int Hkv, int dh, const T *Kc, const T *Vc,
                                         const int32_t *L_dev, int max_len, int Bp, const uint64_t *vis,
                                         float *out) {
  extern __shared__ float sm[];
  float *qs = sm;            // [dh]
  float *ps = sm + dh;       // [blockDim.x]
  float *red = ps + blockDim.x;  // [8]
  int b = blockIdx.x, hq = blockIdx.y;
  int L = *L_dev;
  if (L < 0 || L + Bp > max_len) return;
  int kvh = hq / (Hq / Hkv);
  int nq = Hq * dh, nkv = Hkv * dh;
  const float *q = qkv + (size_t)b * (nq + 2 * nkv) + hq * dh;
  for (int i = threadIdx.x; i < dh; i += blockDim.x) qs[i] = q[i];
  __syncthreads();
  uint64_t vb = vis[b];
  float scale = 1.0f / sqrtf((float)dh);
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;  // acc: output channel threadIdx.x (< dh)
  int total = L + Bp;
  for (int k0 = 0; k0 < total; k0 += blockDim.x) {
    int key = k0 + threadIdx.x;
    bool ok = key < total && (key < L || ((vb >> (key - L)) & 1ull));
    float s = -INFINITY;
    if (ok) {
      const T *kr = Kc + ((size_t)key * Hkv + kvh) * dh;
      float d = 0.f;
      for (int i = 0; i < dh; ++i) d = fmaf(qs[i], load_as_float<T>(kr + i), d);
      s = d * scale;
    }
    float m_new = fmaxf(m_run, block_max(s, red));
    float p = ok ? expf(s - m_new) : 0.f;
    float corr = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    __syncthreads();
    ps[threadIdx.x] = p;
    float psum = block_sum(p, red);  // contains the barriers that publish ps
    l_run = l_run * corr + psum;
    m_run = m_new;
    if ((int)threadIdx.x < dh) {
      acc *= corr;
      int kmax = min((int)blockDim.x, total - k0);
      for (int j = 0; j < kmax; ++j) {
        float pj = ps[j];
        if (pj != 0.f) acc = fmaf(pj, load_as_float<T>(Vc + ((size_t)(k0 + j) * Hkv + kvh) * dh + threadIdx.x), acc);
      }
    }
    __syncthreads();
  }
  if ((int)threadIdx.x < dh) out[(size_t)b * nq + hq * dh + threadIdx.x] = acc / l_run;
}

__global__ void swiglu_kernel(const float *gu, int F, float *act) {
  int b = blockIdx.y;
  int f = blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= F) return;
  float g = gu[(size_t)b * 2 * F + f], u = gu[(size_t)b * 2 * F + F + f];
  act[(size_t)b * F + f] = g / (1.0f + expf(-g)) * u;
}

// Greedy choice per row with ties to the lowest index, plus the two largest values.
struct Top {
  float v1;
  int i1;
  float v2;
};
__device__ __forceinline__ Top top_merge(Top a, Top b) {
  bool b_wins = (b.v1 > a.v1) || (b.v1 == a.v1 && b.i1 < a.i1);
  Top r;
  if (b_wins) {
    r.v1 = b.v1; r.i1 = b.i1; r.v2 = fmaxf(a.v1, fmaxf(a.v2, b.v2));
  } else {
    r.v1 = a.v1; r.i1 = a.i1; r.v2 = fmaxf(b.v1, fmaxf(a.v2, b.v2));
  }
  return r;
}

__global__ void argmax_rows_kernel(const float *logits, int V, int32_t *ids, float *top2) {
  __shared__ Top red[256];
  const float *r = logits + (size_t)blockIdx.x * V;
  Top t{-INFINITY, 0x7fffffff, -INFINITY};
  for (int i = threadIdx.x; i < V; i += blockDim.x) {
    float v = r[i];
    if (v > t.v1) { t.v2 = t.v1; t.v1 = v; t.i1 = i; }
    else if (v > t.v2) t.v2 = v;
  }
  red[threadIdx.x] = t;
  __syncthreads();
  for (int o = blockDim.x / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] = top_merge(red[threadIdx.x], red[threadIdx.x + o]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    ids[blockIdx.x] = red[0].i1;
    if (top2) { top2[blockIdx.x * 2] = red[0].v1; top2[blockIdx.x * 2 + 1] = red[0].v2; }
  }
}

int launch_rope_table(la_model *m, const int32_t *pos, int Bp, hipStream_t s) {
  ProfScope p("rope_table", s);
  rope_table_kernel<<<Bp, 64, 0, s>>>(pos, Bp, m->d.head_dim / 2, (double)m->d.rope_theta, m->rope_cs);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int launch_argmax_rows(const float *logits, int Bp, int V, int32_t *ids, float *top2, hipStream_t s) {
  ProfScope p("argmax_rows", s);
  argmax_rows_kernel<<<Bp, 256, 0, s>>>(logits, V, ids, top2);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

template <typename T>
static int gemm(const char *name, const float *A, int lda, const void *W, int ldw, float *C, int ldc, int M, int K,
                int N, int accumulate, hipStream_t s) {
  ProfScope p(name, s);
  dim3 grid(ceil_div(N, 256), ceil_div(M, 8));
  gemm_generic_kernel<T><<<grid, 256, 0, s>>>(A, lda, (const T *)W, ldw, C, ldc, M, K, N, accumulate);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

template <typename T>
static int forward_t(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos, const uint64_t *vis,
                     la_kv *kv, hipStream_t s) {
  const la_model_desc &d = m->d;
  int nqkv = m->nqkv(), qd = m->qdim(), F = d.d_ffn, dm = d.d_model;
  int rc = launch_rope_table(m, pos, Bp, s);
  if (rc) return rc;
  for (int l = lb; l < le; ++l) {
    const GenericLayer &w = m->layers[l];
    LA_REQUIRE(w.set, LA_EINVAL, "layer %d has no weights", l);
    T *Kc = (T *)kv->K + (size_t)l * kv->layer_elems();
    T *Vc = (T *)kv->V + (size_t)l * kv->layer_elems();
    {
      ProfScope p("rmsnorm", s);
      rmsnorm_kernel<<<Bp, 256, 0, s>>>(hidden, w.g_attn, d.rms_eps, dm, m->h);
    }
    if ((rc = gemm<T>("gemm_qkv", m->h, dm, w.wqkv, nqkv, m->qkv, nqkv, Bp, dm, nqkv, 0, s))) return rc;
    {
      ProfScope p("rope_kvwrite", s);
      rope_kvwrite_kernel<T><<<Bp, 256, 0, s>>>(m->qkv, d.n_q_heads, d.n_kv_heads, d.head_dim, m->rope_cs, Kc, Vc,
                                                 kv->L_dev, kv->max_len, Bp, kv->err_dev, m->err_map);
    }
    {
      ProfScope p("attention", s);
      int threads = 256;
      size_t sh = (d.head_dim + threads + 8) * sizeof(float);
      attention_generic_kernel<T><<<dim3(Bp, d.n_q_heads), threads, sh, s>>>(
          m->qkv, d.n_q_heads, d.n_kv_heads, d.head_dim, Kc, Vc, kv->L_dev, kv->max_len, Bp, vis, m->attn);
    }
    if ((rc = gemm<T>("gemm_o", m->attn, qd, w.wo, dm, hidden, dm, Bp, qd, dm, 1, s))) return rc;
    {
      ProfScope p("rmsnorm", s);
      rmsnorm_kernel<<<Bp, 256, 0, s>>>(hidden, w.g_mlp, d.rms_eps, dm, m->h);
    }
    if ((rc = gemm<T>("gemm_gateup", m->h, dm, w.wgu, 2 * F, m->gu, 2 * F, Bp, dm, 2 * F, 0, s))) return rc;
    {
      ProfScope p("swiglu", s);
      swiglu_kernel<<<dim3(ceil_div(F, 256), Bp), 256, 0, s>>>(m->gu, F, m->act);
    }
    if ((rc = gemm<T>("gemm_down", m->act, F, w.wdown, dm, hidden, dm, Bp, F, dm, 1, s))) return rc;
    LA_HIP(hipGetLastError());
  }
  return LA_OK;
}

int generic_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos, const uint64_t *vis,
                    la_kv *kv, hipStream_t s) {
  if (m->d.dtype == LA_F32) return forward_t<float>(m, lb, le, hidden, Bp, pos, vis, kv, s);
  if (m->d.dtype == LA_F16) return forward_t<_Float16>(m, lb, le, hidden, Bp, pos, vis, kv, s);
  return forward_t<uint16_t>(m, lb, le, hidden, Bp, pos, vis, kv, s);
}

int generic_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, hipStream_t s) {
  const la_model_desc &d = m->d;
  {
    ProfScope p("rmsnorm", s);
    rmsnorm_kernel<<<Bp, 256, 0, s>>>(hidden, m->g_final, d.rms_eps, d.d_model, m->h);
  }
  int rc;
  if (d.dtype == LA_F32)
    rc = gemm<float>("gemm_unembed", m->h, d.d_model, m->unembed, d.vocab, m->logits, d.vocab, Bp, d.d_model, d.vocab, 0, s);
  else if (d.dtype == LA_F16)
    rc = gemm<_Float16>("gemm_unembed", m->h, d.d_model, m->unembed, d.vocab, m->logits, d.vocab, Bp, d.d_model, d.vocab, 0, s);
  else
    rc = gemm<uint16_t>("gemm_unembed", m->h, d.d_model, m->unembed, d.vocab, m->logits, d.vocab, Bp, d.d_model, d.vocab, 0, s);
  if (rc) return rc;
  return launch_argmax_rows(m->logits, Bp, d.vocab, ids, top2, s);
}

}  // namespace la
