// Lookahead controller on the device (Section 4.3 of the paper; Section 3.3 for the cache
// crop / relocation): block layout, n-gram pool, verification, acceptance, KV commit.
// All integer work.  One small workgroup runs the controller so that a step never needs
// the host; the cache rows of accepted verification rows are moved by a second kernel.
#include "la_device.h"
#include "la_internal.h"

namespace la {

struct PoolView {
  uint32_t *stamp;
  int32_t *toks;
  uint32_t *counter;
  int vocab, N, G;
};

__host__ __device__ inline int la_row_index(int W, int r, int c) { return 1 + r * W + c; }
__host__ __device__ inline int v_row_index(int W, int N, int k, int j) { return 1 + W * (N - 1) + k * (N - 1) + (j - 1); }

// Token-free part of the block: position and visibility of every row.  Row 0 is the real
// next-token row at position t.  Window entry (r, c) sits at t+1+c+r and sees row 0, the
// level-0 entries of columns <= c and the entries above it in its own column.  Verification
// row (k, j) sits at t+j and sees row 0 and the earlier tokens of candidate k.  Rows that
// carry nothing (candidates absent, padding) sit at t and see only themselves.
__host__ __device__ inline void block_layout(int W, int N, int G, int n_cand, int t, int Bp, int32_t *pos,
                                             uint64_t *vis) {
  for (int i = 0; i < Bp; ++i) {
    pos[i] = t;
    vis[i] = 1ull << i;
  }
  for (int r = 0; r < N - 1; ++r)
    for (int c = 0; c < W; ++c) {
      int i = la_row_index(W, r, c);
      uint64_t m = 1ull;
      for (int c2 = 0; c2 <= c; ++c2) m |= 1ull << la_row_index(W, 0, c2);
      for (int r2 = 1; r2 <= r; ++r2) m |= 1ull << la_row_index(W, r2, c);
      pos[i] = t + 1 + c + r;
      vis[i] = m;
    }
  for (int k = 0; k < n_cand && k < G; ++k)
    for (int j = 1; j <= N - 1; ++j) {
      int i = v_row_index(W, N, k, j);
      uint64_t m = 1ull;
      for (int j2 = 1; j2 <= j; ++j2) m |= 1ull << v_row_index(W, N, k, j2);
      pos[i] = t + j;
      vis[i] = m;
    }
}

__device__ void build_block(la_step_state *st, int W, int N, int G) {
  int Bp = st->Bp;
  block_layout(W, N, G, st->n_cand, st->L, Bp, st->pos, st->vis);
  for (int i = 0; i < Bp; ++i) st->tok[i] = st->c0;
  for (int r = 0; r < N - 1; ++r)
    for (int c = 0; c < W; ++c) st->tok[la_row_index(W, r, c)] = st->win[r * W + c];
  for (int k = 0; k < st->n_cand; ++k)
    for (int j = 1; j <= N - 1; ++j) st->tok[v_row_index(W, N, k, j)] = st->cand[k * (N - 1) + j - 1];
}

// Insert (key -> tup[0..N-2]).  Present: refresh its stamp.  Else take a free slot, else
// replace the slot with the smallest stamp.
__device__ void pool_insert(const PoolView &p, int key, const int32_t *tup) {
  uint32_t now = *p.counter + 1u;
  *p.counter = now;
  if (p.G == 0 || key < 0 || key >= p.vocab) return;
  int n1 = p.N - 1;
  uint32_t *st = p.stamp + (size_t)key * p.G;
  int32_t *tk = p.toks + (size_t)key * p.G * n1;
  int free_slot = -1, old_slot = 0;
  uint32_t old_stamp = 0xffffffffu;
  for (int s = 0; s < p.G; ++s) {
    uint32_t sv = st[s];
    if (sv == 0u) {
      if (free_slot < 0) free_slot = s;
      continue;
    }
    bool same = true;
    for (int j = 0; j < n1; ++j) same = same && (tk[s * n1 + j] == tup[j]);
    if (same) {
      st[s] = now;
      return;
    }
    if (sv < old_stamp) {
      old_stamp = sv;
      old_slot = s;
    }
  }
  int s = free_slot >= 0 ? free_slot : old_slot;
  for (int j = 0; j < n1; ++j) tk[s * n1 + j] = tup[j];
  st[s] = now;
}

// Candidates of `key`, most recently inserted first, into cand[k*(N-1)+j]; returns the count.
__device__ int pool_lookup(const PoolView &p, int key, int32_t *cand) {
  if (p.G == 0 || key < 0 || key >= p.vocab) return 0;
  int n1 = p.N - 1;
  const uint32_t *st = p.stamp + (size_t)key * p.G;
  const int32_t *tk = p.toks + (size_t)key * p.G * n1;
  int n = 0;
  uint32_t below = 0xffffffffu;  // stamps are distinct: walk them in descending order
  for (;;) {
    int best = -1;
    uint32_t bs = 0u;
    for (int s = 0; s < p.G; ++s) {
      uint32_t sv = st[s];
      if (sv != 0u && sv < below && sv > bs) {
        bs = sv;
        best = s;
      }
    }
    if (best < 0) break;
    for (int j = 0; j < n1; ++j) cand[n * n1 + j] = tk[best * n1 + j];
    below = bs;
    ++n;
  }
  return n;
}

__global__ void fill_u32_kernel(uint32_t *p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void state_init_kernel(PoolView p, la_step_state *st, const int32_t *prompt, int P, int W, int N, int G,
                                  int Bp, int seed_pool, int32_t *kv_L) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  *p.counter = 0u;
  if (seed_pool)
    for (int i = 0; i + N <= P; ++i) pool_insert(p, prompt[i], prompt + i + 1);
  for (int r = 0; r < N - 1; ++r)
    for (int c = 0; c < W; ++c) st->win[r * W + c] = prompt[(r + c) % P];
  st->L = P - 1;
  st->c0 = prompt[P - 1];
  st->Bp = Bp;
  st->steps = st->matched_steps = st->n_emitted = st->last_emitted = st->last_k = st->last_m = 0;
  st->error = st->reserved = 0;
  st->n_cand = (N >= 2) ? pool_lookup(p, st->c0, st->cand) : 0;
  build_block(st, W, N, G);
  *kv_L = P - 1;
}

__global__ void accept_kernel(PoolView p, la_step_state *st, const int32_t *ids, int32_t *emitted, int max_total,
                              int W, int N, int G, int32_t *kv_L, const int32_t *err) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->error = *err;  // what the launches before this one on the model raised (0: nothing)
  int remaining = max_total - st->n_emitted;
  if (remaining <= 0) {  // budget spent: the step is a no-op
    st->last_emitted = 0;
    return;
  }
  int n1 = N - 1;
  int y0 = ids[0];
  int best_k = 0, best_m = 0;
  for (int k = 0; k < st->n_cand; ++k) {
    const int32_t *cd = st->cand + k * n1;
    int m = 0;
    if (cd[0] == y0) {
      m = 1;
      while (m < n1 && cd[m] == ids[v_row_index(W, N, k, m)]) ++m;
    }
    if (m > best_m) {
      best_m = m;
      best_k = k;
    }
  }
  int e = best_m + 1;
  if (e > remaining) e = remaining;
  int base = st->n_emitted;
  int last = y0;
  emitted[base] = y0;
  for (int j = 1; j < e; ++j) {
    last = ids[v_row_index(W, N, best_k, j)];
    emitted[base + j] = last;
  }
  st->n_emitted = base + e;
  st->last_emitted = e;
  st->last_k = best_k;
  st->last_m = best_m;
  st->steps += 1;
  st->matched_steps += (best_m >= 1) ? 1 : 0;
  // harvest: each window column yields one n-gram ending in the model's newest guess
  if (N >= 2) {
    int32_t tup[LA_MAX_ROWS];
    for (int c = 0; c < W; ++c) {
      int nl = ids[la_row_index(W, N - 2, c)];
      for (int r = 1; r < n1; ++r) tup[r - 1] = st->win[r * W + c];
      tup[n1 - 1] = nl;
      pool_insert(p, st->win[c], tup);
    }
    for (int c = 0; c < W; ++c) {
      int nl = ids[la_row_index(W, N - 2, c)];
      for (int r = 0; r + 1 < n1; ++r) st->win[r * W + c] = st->win[(r + 1) * W + c];
      st->win[(n1 - 1) * W + c] = nl;
    }
  }
  st->L += e;
  *kv_L = st->L;
  st->c0 = last;
  st->n_cand = (N >= 2) ? pool_lookup(p, last, st->cand) : 0;
  build_block(st, W, N, G);
}

// ---- Jacobi decoding (Section 4.2) --------------------------------------------------------------
// The block's rows: row 0 = c0 at position L, row i = guess y_i at L + i (i < k) under the plain
// causal mask; rows k.. carry nothing.  The guesses live in st->cand[0..k-1].
__device__ void jacobi_build(la_step_state *st, int k) {
  const int Bp = st->Bp, t = st->L;
  for (int i = 0; i < Bp; ++i) {
    if (i < k) {
      st->tok[i] = i == 0 ? st->c0 : st->cand[i - 1];
      st->pos[i] = t + i;
      st->vis[i] = i == 63 ? ~0ull : ((1ull << (i + 1)) - 1ull);
    } else {
      st->tok[i] = 0;
      st->pos[i] = t + k - 1;
      st->vis[i] = 1ull << i;
    }
  }
}

__global__ void jacobi_init_kernel(la_step_state *st, const int32_t *prompt, int P, int k, int Bp, int32_t *kv_L) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->L = P - 1;
  st->c0 = prompt[P - 1];
  st->Bp = Bp;
  st->n_cand = k;
  st->steps = st->matched_steps = st->n_emitted = st->last_emitted = st->last_k = st->last_m = 0;
  st->error = st->reserved = 0;
  for (int i = 0; i < k; ++i) st->cand[i] = st->c0;  // every position starts from the last committed token
  jacobi_build(st, k);
  *kv_L = P - 1;
}

// One pass's greedy ids become the new guesses (ids[i] is the prediction for position L + i + 1).  The block has
// converged when the pass returned its own input, and after k passes at the latest (pass j fixes guess j for good);
// it then commits: the pass's cache rows L.. were computed from the final tokens, so they stay and L advances.
__global__ void jacobi_accept_kernel(la_step_state *st, const int32_t *ids, int32_t *emitted, int max_total, int k,
                                     int32_t *kv_L, const int32_t *err) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->error = *err;
  int remaining = max_total - st->n_emitted;
  if (remaining <= 0) {
    st->last_emitted = 0;
    return;
  }
  bool same = true;
  for (int i = 0; i < k; ++i) {
    same = same && (ids[i] == st->cand[i]);
    st->cand[i] = ids[i];
  }
  st->steps += 1;
  st->last_k += 1;
  if (!same && st->last_k < k) {
    st->last_emitted = 0;
    jacobi_build(st, k);
    return;
  }
  int e = k < remaining ? k : remaining;
  for (int i = 0; i < e; ++i) emitted[st->n_emitted + i] = st->cand[i];
  st->n_emitted += e;
  st->last_emitted = e;
  st->last_m = st->last_k;
  st->last_k = 0;
  st->matched_steps += 1;
  st->L += e;
  *kv_L = st->L;
  st->c0 = st->cand[e - 1];
  for (int i = 0; i < k; ++i) st->cand[i] = st->c0;
  jacobi_build(st, k);
}

// Cache relocation: the accepted verification rows of candidate last_k move from block rows
// v(k, j) to cache rows L0 + j, j = 1..e-1, in every layer (L0 = cache length before the step).
template <typename T>
__global__ void kv_commit_kernel(const la_step_state *st, T *K, T *V, size_t layer_elems, int Hkv, int dh,
                                 int v_blocked, int W, int N, int max_len) {
  int e = st->last_emitted;
  int j = blockIdx.y + 1;
  if (j >= e) return;
  int L0 = st->L - e;
  int src = L0 + v_row_index(W, N, st->last_k, j), dst = L0 + j;
  if (src >= max_len || dst >= max_len || L0 < 0) return;
  T *Kl = K + (size_t)blockIdx.x * layer_elems;
  T *Vl = V + (size_t)blockIdx.x * layer_elems;
  int n = Hkv * dh;
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    Kl[(size_t)dst * n + i] = Kl[(size_t)src * n + i];
    int h = i / dh, c = i % dh;
    Vl[v_index(v_blocked, dst, h, c, Hkv, dh)] = Vl[v_index(v_blocked, src, h, c, Hkv, dh)];
  }
}

}  // namespace la

using namespace la;

static int check_la(const la_lookahead_desc *d, int Bp) {
  LA_REQUIRE(d != nullptr, LA_EINVAL, "lookahead desc is NULL");
  LA_REQUIRE(d->N >= 1 && d->W >= 0 && d->G >= 0, LA_EINVAL, "bad lookahead parameters W=%d N=%d G=%d", d->W, d->N, d->G);
  LA_REQUIRE(d->N >= 2 || (d->G == 0), LA_EINVAL, "N=1 (sequential decoding) needs G=0");
  int rows = 1 + (d->W + d->G) * (d->N - 1);
  LA_REQUIRE(rows <= LA_MAX_ROWS, LA_EINVAL, "block of %d rows exceeds %d", rows, LA_MAX_ROWS);
  LA_REQUIRE(Bp >= rows && Bp <= LA_MAX_ROWS, LA_EINVAL, "Bp=%d must be in [%d, %d]", Bp, rows, LA_MAX_ROWS);
  return LA_OK;
}

extern "C" int la_lookahead_layout(const la_lookahead_desc *d, int t, int n_cand, int Bp, int32_t *pos_host,
                                   uint64_t *vis_host) {
  int rc = check_la(d, Bp);
  if (rc) return rc;
  LA_REQUIRE(pos_host && vis_host, LA_EINVAL, "NULL output");
  LA_REQUIRE(n_cand >= 0 && n_cand <= d->G, LA_EINVAL, "n_cand=%d outside [0, G=%d]", n_cand, d->G);
  block_layout(d->W, d->N, d->G, n_cand, t, Bp, pos_host, vis_host);
  return LA_OK;
}

extern "C" int la_pool_alloc(int vocab, int N, int G, la_pool **out) {
  LA_REQUIRE(out != nullptr, LA_EINVAL, "out is NULL");
  *out = nullptr;
  LA_REQUIRE(vocab > 0 && N >= 1 && G >= 0 && N <= LA_MAX_ROWS, LA_EINVAL, "bad pool shape vocab=%d N=%d G=%d", vocab, N, G);
  la_pool *p = new (std::nothrow) la_pool();
  LA_REQUIRE(p != nullptr, LA_ENOMEM, "out of host memory");
  p->vocab = vocab; p->N = N; p->G = G;
  size_t slots = (size_t)vocab * (G > 0 ? G : 1);
  size_t n1 = N > 1 ? N - 1 : 1;
  if (hipMalloc(&p->stamp, slots * sizeof(uint32_t)) != hipSuccess ||
      hipMalloc(&p->toks, slots * n1 * sizeof(int32_t)) != hipSuccess ||
      hipMalloc(&p->counter, sizeof(uint32_t)) != hipSuccess) {
    la_free_pool(p);
    set_error("pool allocation failed");
    return LA_ENOMEM;
  }
  *out = p;
  return LA_OK;
}

extern "C" void la_free_pool(la_pool *p) {
  if (!p) return;
  if (p->stamp) (void)hipFree(p->stamp);
  if (p->toks) (void)hipFree(p->toks);
  if (p->counter) (void)hipFree(p->counter);
  delete p;
}

static PoolView view(la_pool *p) { return PoolView{p->stamp, p->toks, p->counter, p->vocab, p->N, p->G}; }

extern "C" int la_state_init(la_pool *p, la_kv *kv, const la_lookahead_desc *d, const int32_t *prompt, int P, int Bp,
                             int seed_pool, la_step_state *state, void *stream) {
  LA_REQUIRE(p && kv && prompt && state, LA_EINVAL, "NULL argument");
  LA_PENDING(kv->m);
  int rc = check_la(d, Bp);
  if (rc) return rc;
  LA_REQUIRE(P >= 1, LA_EINVAL, "prompt must have at least one token");
  LA_REQUIRE(p->N == d->N && p->G == d->G, LA_EINVAL, "pool was allocated for N=%d G=%d", p->N, p->G);
  LA_REQUIRE(P - 1 + Bp <= kv->max_len, LA_ERANGE, "prompt of %d tokens + block of %d rows exceeds max_len %d", P, Bp, kv->max_len);
  hipStream_t s = (hipStream_t)stream;
  size_t slots = (size_t)p->vocab * (p->G > 0 ? p->G : 1);
  {
    ProfScope ps("pool_clear", s);
    fill_u32_kernel<<<1024, 256, 0, s>>>(p->stamp, slots, 0u);
  }
  {
    ProfScope ps("state_init", s);
    state_init_kernel<<<1, 64, 0, s>>>(view(p), state, prompt, P, d->W, d->N, d->G, Bp, seed_pool, kv->L_dev);
  }
  LA_HIP(hipGetLastError());
  kv->L_bound = P - 1;
  return LA_OK;
}

extern "C" int la_ngram_accept(la_pool *p, la_kv *kv, const la_lookahead_desc *d, const int32_t *ids,
                               la_step_state *state, int32_t *emitted, int max_total, void *stream) {
  LA_REQUIRE(p && kv && ids && state && emitted, LA_EINVAL, "NULL argument");
  LA_PENDING(kv->m);
  int rc = check_la(d, 1 + (d ? (d->W + d->G) * (d->N - 1) : 0));
  if (rc) return rc;
  LA_REQUIRE(p->N == d->N && p->G == d->G, LA_EINVAL, "pool was allocated for N=%d G=%d", p->N, p->G);
  LA_REQUIRE(max_total >= 0, LA_EINVAL, "max_total < 0");
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps("ngram_accept", s);
    accept_kernel<<<1, 64, 0, s>>>(view(p), state, ids, emitted, max_total, d->W, d->N, d->G, kv->L_dev, kv->err_dev);
  }
  if (d->N >= 2) {
    ProfScope ps("kv_commit", s);
    const la_model_desc &md = kv->m->d;
    dim3 grid(kv->n_layers, d->N - 1);
    if (md.dtype == LA_F32)
      kv_commit_kernel<float><<<grid, 256, 0, s>>>(state, (float *)kv->K, (float *)kv->V, kv->layer_elems(),
                                                    md.n_kv_heads, md.head_dim, kv->v_blocked, d->W, d->N, kv->max_len);
    else
      kv_commit_kernel<uint16_t><<<grid, 256, 0, s>>>(state, (uint16_t *)kv->K, (uint16_t *)kv->V, kv->layer_elems(),
                                                       md.n_kv_heads, md.head_dim, kv->v_blocked, d->W, d->N, kv->max_len);
  }
  LA_HIP(hipGetLastError());
  kv->L_bound += d->N;
  return LA_OK;
}

extern "C" int la_jacobi_init(la_kv *kv, int k, const int32_t *prompt, int P, int Bp, la_step_state *state, void *stream) {
  LA_REQUIRE(kv && prompt && state, LA_EINVAL, "NULL argument");
  LA_PENDING(kv->m);
  LA_REQUIRE(k >= 1 && k <= Bp && Bp <= LA_MAX_ROWS, LA_EINVAL, "need 1 <= k=%d <= Bp=%d <= %d", k, Bp, LA_MAX_ROWS);
  LA_REQUIRE(P >= 1, LA_EINVAL, "prompt must have at least one token");
  LA_REQUIRE(P - 1 + Bp <= kv->max_len, LA_ERANGE, "prompt of %d tokens + block of %d rows exceeds max_len %d", P, Bp, kv->max_len);
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps("jacobi_init", s);
    jacobi_init_kernel<<<1, 64, 0, s>>>(state, prompt, P, k, Bp, kv->L_dev);
  }
  LA_HIP(hipGetLastError());
  kv->L_bound = P - 1;
  return LA_OK;
}

extern "C" int la_jacobi_accept(la_kv *kv, int k, const int32_t *ids, la_step_state *state, int32_t *emitted, int max_total,
                                void *stream) {
  LA_REQUIRE(kv && ids && state && emitted, LA_EINVAL, "NULL argument");
  LA_PENDING(kv->m);
  LA_REQUIRE(k >= 1 && k <= LA_MAX_ROWS, LA_EINVAL, "k=%d outside [1, %d]", k, LA_MAX_ROWS);
  LA_REQUIRE(max_total >= 0, LA_EINVAL, "max_total < 0");
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope ps("jacobi_accept", s);
    jacobi_accept_kernel<<<1, 64, 0, s>>>(state, ids, emitted, max_total, k, kv->L_dev, kv->err_dev);
  }
  LA_HIP(hipGetLastError());
  kv->L_bound += k;
  return LA_OK;
}
