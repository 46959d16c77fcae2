// Host side of the bf16 MFMA path: weight packing into the per-CU streams, scratch buffers,
// launch of the persistent kernel (la_stack.h).
#include <stdio.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "la_rstack.h"

namespace la {

namespace rs {
extern template int launch_rstack_kernel<1, 4>(const StackArgs &, int, hipStream_t);
extern template int launch_rstack_kernel<2, 4>(const StackArgs &, int, hipStream_t);
extern template int launch_rstack_kernel<3, 4>(const StackArgs &, int, hipStream_t);
extern template int launch_rstack_kernel<4, 4>(const StackArgs &, int, hipStream_t);
extern template int prepare_rstack_kernel<1, 4>(int, int);
extern template int prepare_rstack_kernel<2, 4>(int, int);
extern template int prepare_rstack_kernel<3, 4>(int, int);
extern template int prepare_rstack_kernel<4, 4>(int, int);
}  // namespace rs
constexpr int R_NW = 4;  // MFMA waves of the register-streaming kernel

extern template int launch_stack_kernel<1>(const StackArgs &, int, hipStream_t);
extern template int launch_stack_kernel<2>(const StackArgs &, int, hipStream_t);
extern template int launch_stack_kernel<3>(const StackArgs &, int, hipStream_t);
extern template int launch_stack_kernel<4>(const StackArgs &, int, hipStream_t);
extern template int prepare_stack_kernel<1>(int, int);
extern template int prepare_stack_kernel<2>(int, int);
extern template int prepare_stack_kernel<3>(int, int);
extern template int prepare_stack_kernel<4>(int, int);

// ---- weight packing (once, at model set-up) -----------------------------------------------------
// Destination: the per-CU streams.  Source column of packed column pc of a GEMM:
//   kind 0: one source [K, N];
//   kind 1: q | k | v heads; each 16-column tile holds channels 8j..8j+7 and dh/2+8j.. of one
//           head, i.e. both members of eight RoPE pairs;
//   kind 2: per tile, 8 gate channels followed by the same 8 channels of up.
struct PackSrc {
  const uint16_t *s0, *s1, *s2;
  int n0, n1, n2;
  int kind, F, dh;
  int half;  // the source already is IEEE half (LA_F16): copied as stored
};
__device__ __forceinline__ const uint16_t *pack_col(const PackSrc &p, int pc, int &ld) {
  if (p.kind == 0) {
    ld = p.n0;
    return p.s0 + pc;
  }
  if (p.kind == 1) {
    int tile = pc >> 4, w = pc & 15, spj = p.dh >> 4;
    int hs = tile / spj, j = tile - hs * spj;
    pc = hs * p.dh + (w < 8 ? 8 * j + w : (p.dh >> 1) + 8 * j + (w - 8));
    if (pc < p.n0) { ld = p.n0; return p.s0 + pc; }
    pc -= p.n0;
    if (pc < p.n1) { ld = p.n1; return p.s1 + pc; }
    ld = p.n2;
    return p.s2 + (pc - p.n1);
  }
  int tile = pc >> 4, w = pc & 15;
  ld = p.F;
  return (w < 8 ? p.s0 : p.s1) + tile * 8 + (w & 7);
}

// dst_frag0: fragment index (inside a CU's region) of the GEMM's first fragment is
// seg_base + off_c where off_c depends on the CU: passed as the four per-GEMM tile counts that
// precede this GEMM in a layer (ntiles, KT pairs), so the kernel can recompute it.
struct PackDst {
  uint8_t *wstream;
  size_t cu_bytes;
  unsigned seg_base;      // fragment offset of the layer inside a CU's region
  int G;
  int prev_ntiles[3], prev_KT[3], n_prev;
  int ntiles, KT, ntp;
  int r_nw;  // 0: layout of the LDS-ring kernel (la_stack.h); else the register-streaming kernel's, for that many MFMA waves
};

__global__ void pack_weights_kernel(PackSrc p, PackDst d) {
  size_t total = (size_t)d.ntiles * d.KT * 64;
  for (size_t fi = (size_t)blockIdx.x * blockDim.x + threadIdx.x; fi < total; fi += (size_t)gridDim.x * blockDim.x) {
    int lane = fi & 63;
    size_t r = fi >> 6;
    int kt = r % d.KT;
    int tile = r / d.KT;
    int c = tile % d.G, lt = tile / d.G;            // owner CU, local tile
    int nt = (d.ntiles - c + d.G - 1) / d.G;        // tiles of that CU
    int pass = lt / d.ntp, tp = lt - pass * d.ntp;  // pass and position in it
    int n_pass = nt - pass * d.ntp < d.ntp ? nt - pass * d.ntp : d.ntp;
    size_t off = 0;
    for (int i = 0; i < d.n_prev; ++i) {
      int pn = d.prev_ntiles[i] > c ? (d.prev_ntiles[i] - c + d.G - 1) / d.G : 0;
      off += (size_t)pn * d.prev_KT[i];
    }
    if (d.r_nw) {
      // per MFMA wave w: [its k-tiles w, w + NW, ...][all column tiles of this CU]
      int w = kt % d.r_nw, i = kt / d.r_nw;
      size_t before = 0;  // k-tiles of the waves in front of w
      for (int v = 0; v < w; ++v) before += d.KT > v ? (d.KT - v + d.r_nw - 1) / d.r_nw : 0;
      off += (before + i) * nt + lt;
    } else {
      off += (size_t)pass * d.ntp * d.KT + (size_t)kt * n_pass + tp;
    }
    int pc = tile * 16 + (lane & 15);
    int k0 = kt * 32 + 8 * (lane >> 4);
    int ld;
    const uint16_t *src = pack_col(p, pc, ld);
    // bf16 -> half precision: exact for every weight of magnitude 2^-14 or more (8 significant
    // bits fit in 11); smaller ones land on the subnormal grid, at most 2^-25 away
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint16_t bits = src[(size_t)(k0 + i) * ld];
      const float w = __uint_as_float((uint32_t)bits << 16);
      const float lim = 65504.0f;
      v[i] = p.half ? bits : __builtin_bit_cast(uint16_t, (_Float16)fminf(fmaxf(w, -lim), lim));
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    uint8_t *dst = d.wstream + (size_t)c * d.cu_bytes + ((size_t)d.seg_base + off) * 1024 + (size_t)lane * 16;
    *reinterpret_cast<uint4 *>(dst) = o;
  }
}

__global__ void zero_u32_kernel(unsigned *p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---- host side --------------------------------------------------------------------------------------
struct GemmPlan {
  int N = 0, K = 0, KT = 0, ntiles = 0, ntp = 1, nt_max = 0;
};

struct PfBuffers {  // the large-M prompt pass (la_prefill.h), allocated at its first use
  float *x = nullptr, *rs = nullptr, *cs = nullptr;
  uint16_t *A = nullptr, *Q = nullptr, *attn = nullptr, *act = nullptr;
};

struct MfmaModel {
  int n_wgs = 256;
  bool use_r = true;  // the register-streaming kernel (la_rstack.h); false: the LDS-ring kernel (la_stack.h)
  GemmPlan p_qkv, p_o, p_gu, p_down, p_un;
  uint8_t *wstream = nullptr;   // [CU][layer][seg_frags][1 KB]
  size_t cu_bytes = 0;
  unsigned seg_frags = 0;
  uint8_t *ustream = nullptr;   // unembedding: [CU][un_frags][1 KB]
  size_t ucu_bytes = 0;
  std::vector<LayerGains> host_gains;
  LayerGains *dev_gains = nullptr;
  bool gains_dirty = true;
  uint16_t *xa = nullptr, *attn_a = nullptr, *act_a = nullptr, *qf = nullptr;  // per layer (and use)
  uint16_t *xa_u = nullptr;                                                    // unembedding input
  float *rsq = nullptr, *rsq_u = nullptr;
  Top *un_part = nullptr;
  int un_parts_per_cu = 0;
  float *att_part = nullptr;    // attention with the keys split over workgroups: one partial record per workgroup
  unsigned *att_cnt = nullptr;  // ... and per unit the number of records delivered
  unsigned *sync = nullptr;
  unsigned *sched[3][2] = {};  // register-streaming kernel: schedule tables per ring depth (32, 24, 16 slots) and mode (stack, unembedding)
  int32_t *zero_len = nullptr;  // a cache length of 0: the unembedding has no cache to overflow
  unsigned epoch = 0;
  unsigned long long *trace = nullptr;  // LA_TRACE=1: per-phase timestamps, printed after each launch
  int trace_phases = 0;
  PfBuffers pf;
};

static int env_int(const char *name, int dflt) {
  const char *v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

static GemmPlan make_plan(int N, int K, int n_wgs) {
  GemmPlan p;
  p.N = N; p.K = K; p.KT = K / 32; p.ntiles = N / 16;
  p.nt_max = ceil_div(p.ntiles, n_wgs);
  int passes = ceil_div(p.nt_max, MAX_NT);
  p.ntp = ceil_div(p.nt_max, passes);
  return p;
}

int mfma_supported(const la_model_desc *d) {
  int qd = d->n_q_heads * d->head_dim, nqkv = (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim;
  if (d->d_model % 64 || qd % 32 || d->d_ffn % 32 || nqkv % 16 || d->vocab % 16) return 0;
  if (d->head_dim != 64 && d->head_dim != 128) return 0;
  if (d->n_q_heads / d->n_kv_heads > 8) return 0;
  if (d->d_model / 16 > 512) return 0;  // the row statistics are read as two 128-bit vectors per lane
  // operand buffers are addressed through 32-bit buffer offsets
  size_t lim = (size_t)1 << 31;
  if ((size_t)LA_MAX_ROWS * d->d_ffn * 2 >= lim) return 0;
  return 1;
}

static void *dalloc(size_t bytes) {
  void *p = nullptr;
  if (hipMalloc(&p, bytes ? bytes : 1) != hipSuccess) return nullptr;
  return p;
}

void mfma_destroy(la_model *m) {
  MfmaModel *f = m->mf;
  if (!f) return;
  void *ps[] = {f->wstream, f->ustream, f->xa, f->attn_a, f->act_a, f->qf, f->xa_u, f->rsq_u, f->rsq, f->un_part,
                f->sync, f->dev_gains, f->zero_len, f->trace, f->att_part, f->att_cnt,
                f->sched[0][0], f->sched[0][1], f->sched[1][0], f->sched[1][1], f->sched[2][0], f->sched[2][1],
                f->pf.x, f->pf.rs, f->pf.cs, f->pf.A, f->pf.Q, f->pf.attn, f->pf.act};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  delete f;
  m->mf = nullptr;
}

void mfma_reset_sync(la_model *m, hipStream_t s) {
  MfmaModel *f = m->mf;
  zero_u32_kernel<<<ceil_div(SYNC_STRIDE * 66, 256), 256, 0, s>>>(f->sync, SYNC_STRIDE * 66);
  f->epoch = 0;
}

static int na_setup(int device);  // address of the static scratch array on this device (defined with its entry point below)
static GemmDev dev_plan(const GemmPlan &p);

int mfma_create(la_model *m) {
  const la_model_desc &d = m->d;
  MfmaModel *f = new (std::nothrow) MfmaModel();
  LA_REQUIRE(f != nullptr, LA_ENOMEM, "out of host memory");
  m->mf = f;
  {
    int rc = na_setup(m->device);
    if (rc) return rc;
  }
  hipDeviceProp_t prop;
  LA_HIP(hipGetDeviceProperties(&prop, m->device));
  int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  f->n_wgs = std::max(1, std::min(env_int("LA_WGS", cus), cus));  // one resident workgroup per CU: the barrier needs co-residency
  f->use_r = env_int("LA_LDS_RING", 0) == 0;
  LA_REQUIRE(f->use_r || d.dtype != LA_F16, LA_EINVAL, "LA_F16 models run on the register-streaming kernel only (unset LA_LDS_RING)");
  LA_REQUIRE((size_t)prop.sharedMemPerBlockOptin >= (size_t)LDS_BYTES || (size_t)prop.maxSharedMemoryPerMultiProcessor >= (size_t)LDS_BYTES,
             LA_EINVAL, "the device offers less LDS per workgroup than the %d bytes the kernel needs", LDS_BYTES);
  {  // co-residency of the grid: the barrier would otherwise wait for workgroups that cannot start
    int rc = f->use_r ? rs::prepare_rstack_kernel<1, R_NW>(f->n_wgs, cus) : prepare_stack_kernel<1>(f->n_wgs, cus);
    if (!rc) rc = f->use_r ? rs::prepare_rstack_kernel<2, R_NW>(f->n_wgs, cus) : prepare_stack_kernel<2>(f->n_wgs, cus);
    if (!rc) rc = f->use_r ? rs::prepare_rstack_kernel<3, R_NW>(f->n_wgs, cus) : prepare_stack_kernel<3>(f->n_wgs, cus);
    if (!rc) rc = f->use_r ? rs::prepare_rstack_kernel<4, R_NW>(f->n_wgs, cus) : prepare_stack_kernel<4>(f->n_wgs, cus);
    if (rc) return rc;
  }
  int qd = m->qdim(), nqkv = m->nqkv(), g = d.n_q_heads / d.n_kv_heads;
  f->p_qkv = make_plan(nqkv, d.d_model, f->n_wgs);
  f->p_o = make_plan(d.d_model, qd, f->n_wgs);
  f->p_gu = make_plan(2 * d.d_ffn, d.d_model, f->n_wgs);
  f->p_down = make_plan(d.d_model, d.d_ffn, f->n_wgs);
  f->p_un = make_plan(d.vocab, d.d_model, f->n_wgs);
  if (f->use_r)  // the MFMA waves' schedule tables hold a fixed number of entries per layer (and for the unembedding)
    for (int ring : {rs::Geo<2>::RING, rs::Geo<3>::RING, rs::Geo<4>::RING}) {
      auto nb = [&](const GemmPlan &p) { return rs::schedule_bodies(p.KT, p.nt_max, p.ntp, rs::Geo<1>::NTMAX, ring, R_NW); };
      const int layer = nb(f->p_qkv) + nb(f->p_o) + nb(f->p_gu) + nb(f->p_down), un = nb(f->p_un);
      LA_REQUIRE(layer <= rs::TAB_MAX && un <= rs::TAB_MAX, LA_EINVAL,
                 "the register-streaming kernel's schedule has %d entries per layer and %d for the unembedding; it holds %d (LA_LDS_RING=1 "
                 "selects the other kernel)", layer, un, rs::TAB_MAX);
    }
  f->seg_frags = (unsigned)(f->p_qkv.nt_max * f->p_qkv.KT + f->p_o.nt_max * f->p_o.KT + f->p_gu.nt_max * f->p_gu.KT +
                            f->p_down.nt_max * f->p_down.KT);
  f->seg_frags = (f->seg_frags + CHUNK - 1) / CHUNK * CHUNK;  // the producer moves whole chunks
  f->cu_bytes = (size_t)d.n_layers * f->seg_frags * 1024;
  LA_REQUIRE(f->cu_bytes < ((size_t)1 << 31), LA_EINVAL, "one CU's weight stream exceeds 2 GiB");
  f->ucu_bytes = (size_t)(((size_t)f->p_un.nt_max * f->p_un.KT + CHUNK - 1) / CHUNK * CHUNK) * 1024;
  LA_REQUIRE(f->ucu_bytes < ((size_t)1 << 31), LA_EINVAL, "one CU's unembedding stream exceeds 2 GiB");
  f->host_gains.resize(d.n_layers);
  size_t R = LA_MAX_ROWS, nl = d.n_layers;
  size_t QR = (size_t)g * MAX_MT * 16;
  int n_sync = SYNC_STRIDE * 66;
  size_t ncg = d.d_model / 16;
  bool ok = true;
  ok = ok && (f->wstream = (uint8_t *)dalloc((size_t)f->n_wgs * f->cu_bytes));
  ok = ok && (f->xa = (uint16_t *)dalloc(2 * (nl + 1) * R * d.d_model * 2));
  ok = ok && (f->attn_a = (uint16_t *)dalloc(nl * R * qd * 2));
  ok = ok && (f->act_a = (uint16_t *)dalloc(nl * R * (size_t)d.d_ffn * 2));
  ok = ok && (f->xa_u = (uint16_t *)dalloc(R * d.d_model * 2));
  ok = ok && (f->qf = (uint16_t *)dalloc((size_t)d.n_kv_heads * QR * d.head_dim * 2));
  ok = ok && (f->rsq = (float *)dalloc(2 * (nl + 1) * R * ncg * 4));
  ok = ok && (f->rsq_u = (float *)dalloc(R * ncg * 4));
  ok = ok && (f->sync = (unsigned *)dalloc((size_t)n_sync * 4));
  ok = ok && (f->dev_gains = (LayerGains *)dalloc((size_t)d.n_layers * sizeof(LayerGains)));
  ok = ok && (f->zero_len = (int32_t *)dalloc(8));
  ok = ok && (f->att_part = (float *)dalloc((size_t)f->n_wgs * (8 * 1024 + 512)));
  ok = ok && (f->att_cnt = (unsigned *)dalloc((size_t)d.n_q_heads * MAX_MT * 4));
  LA_REQUIRE(ok, LA_ENOMEM, "device allocation failed in the MFMA path");
  LA_HIP(hipMemset(f->wstream, 0, (size_t)f->n_wgs * f->cu_bytes));  // padding fragments are streamed too
  // pad rows of the operand buffers are read by the MFMAs: keep them finite
  LA_HIP(hipMemset(f->xa, 0, 2 * (nl + 1) * R * d.d_model * 2));
  LA_HIP(hipMemset(f->attn_a, 0, nl * R * qd * 2));
  LA_HIP(hipMemset(f->act_a, 0, nl * R * (size_t)d.d_ffn * 2));
  LA_HIP(hipMemset(f->xa_u, 0, R * d.d_model * 2));
  LA_HIP(hipMemset(f->qf, 0, (size_t)d.n_kv_heads * QR * d.head_dim * 2));
  LA_HIP(hipMemset(f->sync, 0, (size_t)n_sync * 4));
  LA_HIP(hipMemset(f->zero_len, 0, 8));
  if (f->use_r) {  // the MFMA waves' schedules, once per model: per ring depth (row-tile counts 1-2, 3, 4) and mode
    const int rings[3] = {rs::Geo<2>::RING, rs::Geo<3>::RING, rs::Geo<4>::RING};
    const size_t bytes = (size_t)f->n_wgs * R_NW * rs::TAB_BYTES;
    for (int c = 0; c < 3; ++c)
      for (int mode = 0; mode < 2; ++mode) {
        f->sched[c][mode] = (unsigned *)dalloc(bytes);
        LA_REQUIRE(f->sched[c][mode] != nullptr, LA_ENOMEM, "device allocation failed in the MFMA path");
        StackArgs a{};
        a.mode = mode;
        a.lb = 0;
        a.le = 1;
        a.qkv = dev_plan(f->p_qkv);
        a.o = dev_plan(f->p_o);
        a.gu = dev_plan(f->p_gu);
        a.down = dev_plan(f->p_down);
        a.un = dev_plan(f->p_un);
        a.seg_frags = mode == 0 ? f->seg_frags : (unsigned)(f->ucu_bytes / 1024);
        int rc = rs::write_schedule_tables<R_NW>(a, rings[c], f->sched[c][mode], f->n_wgs, nullptr);
        if (rc) return rc;
      }
    LA_HIP(hipDeviceSynchronize());
  }
#ifdef LA_EXPERIMENTS
  if (env_int("LA_TRACE", 0)) {
    f->trace_phases = 2 + 5 * d.n_layers;
    f->trace = (unsigned long long *)dalloc(((size_t)TRACE_SLOTS * f->trace_phases + TRACE_WG * f->n_wgs) * 8);
    LA_REQUIRE(f->trace != nullptr, LA_ENOMEM, "device allocation failed");
    LA_HIP(hipMemset(f->trace, 0, ((size_t)TRACE_SLOTS * f->trace_phases + TRACE_WG * f->n_wgs) * 8));
  }
#endif
  return LA_OK;
}

static int pack(const PackSrc &src, const PackDst &dst, hipStream_t s) {
  ProfScope ps("pack_weights", s);
  pack_weights_kernel<<<2048, 256, 0, s>>>(src, dst);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int mfma_set_layer(la_model *m, int layer, const la_layer_weights *w, hipStream_t s) {
  MfmaModel *f = m->mf;
  int qd = m->qdim(), kvd = m->kvdim();
  const la_model_desc &d = m->d;
  const GemmPlan *plans[4] = {&f->p_qkv, &f->p_o, &f->p_gu, &f->p_down};
  PackSrc srcs[4] = {
      {(const uint16_t *)w->wq, (const uint16_t *)w->wk, (const uint16_t *)w->wv, qd, kvd, kvd, 1, 0, d.head_dim},
      {(const uint16_t *)w->wo, nullptr, nullptr, d.d_model, 0, 0, 0, 0, 0},
      {(const uint16_t *)w->wgate, (const uint16_t *)w->wup, nullptr, d.d_ffn, d.d_ffn, 0, 2, d.d_ffn, 0},
      {(const uint16_t *)w->wdown, nullptr, nullptr, d.d_model, 0, 0, 0, 0, 0},
  };
  for (int gi = 0; gi < 4; ++gi) {
    srcs[gi].half = d.dtype == LA_F16;
    PackDst dst{};
    dst.wstream = f->wstream;
    dst.cu_bytes = f->cu_bytes;
    dst.seg_base = (unsigned)layer * f->seg_frags;
    dst.G = f->n_wgs;
    dst.n_prev = gi;
    for (int i = 0; i < gi; ++i) {
      dst.prev_ntiles[i] = plans[i]->ntiles;
      dst.prev_KT[i] = plans[i]->KT;
    }
    dst.ntiles = plans[gi]->ntiles;
    dst.KT = plans[gi]->KT;
    dst.ntp = plans[gi]->ntp;
    dst.r_nw = f->use_r ? R_NW : 0;
    int rc = pack(srcs[gi], dst, s);
    if (rc) return rc;
  }
  f->host_gains[layer] = LayerGains{m->layers[layer].g_attn, m->layers[layer].g_mlp};
  f->gains_dirty = true;
  return LA_OK;
}

int mfma_set_head(la_model *m, const void *unembed, hipStream_t s) {
  MfmaModel *f = m->mf;
  if (!f->ustream) f->ustream = (uint8_t *)dalloc((size_t)f->n_wgs * f->ucu_bytes);
  LA_REQUIRE(f->ustream != nullptr, LA_ENOMEM, "device allocation of the unembedding stream failed");
  LA_HIP(hipMemsetAsync(f->ustream, 0, (size_t)f->n_wgs * f->ucu_bytes, s));
  PackSrc u{(const uint16_t *)unembed, nullptr, nullptr, m->d.vocab, 0, 0, 0, 0, 0, m->d.dtype == LA_F16};
  PackDst dst{};
  dst.wstream = f->ustream;
  dst.cu_bytes = f->ucu_bytes;
  dst.seg_base = 0;
  dst.G = f->n_wgs;
  dst.n_prev = 0;
  dst.ntiles = f->p_un.ntiles;
  dst.KT = f->p_un.KT;
  dst.ntp = f->p_un.ntp;
  dst.r_nw = f->use_r ? R_NW : 0;
  int rc = pack(u, dst, s);
  if (rc) return rc;
  // partial arg-max records per CU: one per reduction chunk of every pass, at any row count
  int passes = ceil_div(f->p_un.nt_max, f->p_un.ntp);
  f->un_parts_per_cu = passes * f->p_un.ntp;  // an upper bound (chunks hold at least one tile)
  if (!f->un_part) f->un_part = (Top *)dalloc((size_t)f->n_wgs * f->un_parts_per_cu * 64 * sizeof(Top));
  LA_REQUIRE(f->un_part != nullptr, LA_ENOMEM, "device allocation failed");
  return LA_OK;
}

static GemmDev dev_plan(const GemmPlan &p) { return GemmDev{p.KT, p.ntiles, p.ntp}; }

// fresh_sync: a.sync was cleared on `s` just before and does not belong to the model, so the launch starts at barrier
// epoch 0 and leaves the model's epoch alone; such launches are not traced.
static int launch_stack(const char *name, MfmaModel *f, StackArgs a, int n_barriers, hipStream_t s, bool fresh_sync = false) {
  if (fresh_sync) {
    a.epoch0 = 0;
  } else {
    if (f->epoch > (1u << 26)) {  // keep the monotonic counters far from wrapping
      zero_u32_kernel<<<ceil_div(SYNC_STRIDE * 66, 256), 256, 0, s>>>(f->sync, SYNC_STRIDE * 66);
      f->epoch = 0;
    }
    a.epoch0 = f->epoch;
    f->epoch += (unsigned)n_barriers;
  }
  a.n_groups = (unsigned)ceil_div(f->n_wgs, SYNC_GROUP);
  a.sched = f->sched[a.MT <= 2 ? 0 : a.MT == 3 ? 1 : 2][a.mode];
  a.trace = fresh_sync ? nullptr : f->trace;
  a.trace_phases = f->trace_phases;
  a.trace_sel = env_int("LA_TRACE_SEL", 6);
  a.trace_seg = env_int("LA_TRACE_SEG", 2);
  int rc;
  {
    ProfScope ps(name, s);
    if (f->use_r) {
      switch (a.MT) {
      case 1: rc = rs::launch_rstack_kernel<1, R_NW>(a, f->n_wgs, s); break;
      case 2: rc = rs::launch_rstack_kernel<2, R_NW>(a, f->n_wgs, s); break;
      case 3: rc = rs::launch_rstack_kernel<3, R_NW>(a, f->n_wgs, s); break;
      default: rc = rs::launch_rstack_kernel<4, R_NW>(a, f->n_wgs, s); break;
      }
    } else {
      switch (a.MT) {
      case 1: rc = launch_stack_kernel<1>(a, f->n_wgs, s); break;
      case 2: rc = launch_stack_kernel<2>(a, f->n_wgs, s); break;
      case 3: rc = launch_stack_kernel<3>(a, f->n_wgs, s); break;
      default: rc = launch_stack_kernel<4>(a, f->n_wgs, s); break;
      }
    }
  }
  if (rc) return rc;
#ifdef LA_EXPERIMENTS
  if (a.trace) {  // debugging aid: timeline of workgroup 0 (100 MHz clock) and producer statistics
    int np = n_barriers + 1;
    std::vector<unsigned long long> h((size_t)TRACE_SLOTS * f->trace_phases + TRACE_WG * f->n_wgs);
    LA_HIP(hipStreamSynchronize(s));
    LA_HIP(hipMemcpy(h.data(), f->trace, h.size() * 8, hipMemcpyDeviceToHost));
    const int S = TRACE_SLOTS;
    fprintf(stderr, "[la trace] %s: %d phases, total %.1f us (times below: us after the phase's start, workgroup 0 wave 0)\n", name, np,
            (h[S * (np - 1) + 2] - h[0]) * 0.01);
    for (int q = 0; q < np; ++q) {
      if (q >= 12 && !(env_int("LA_TRACE", 0) > 2 && q >= np - 6)) continue;
      const unsigned long long t0 = h[S * q];
      auto rel = [&](int k) { return h[S * q + k] > t0 ? (h[S * q + k] - t0) * 0.01 : -1.0; };
      double since_prev = q > 0 ? (t0 - h[S * (q - 1) + 2]) * 0.01 : 0.0;
      fprintf(stderr, "[la trace]   phase %2d: +%5.2f | k-loop end %6.2f (waited for weights %6.2f) tile %6.2f epilogue %6.2f | pass entry %6.2f first operand %6.2f next pass %6.2f | "
              "work end %6.2f | barrier: stores %6.2f waves %6.2f released %6.2f\n", q, since_prev, rel(1), h[S * q + 1] > t0 ? h[S * q + 3] * 0.01 : -1.0,
              rel(4), rel(5), rel(10), rel(9), rel(11), rel(2), rel(6), rel(7), rel(8));
      if (h[S * q + 14]) {
        fprintf(stderr, "[la trace]             attention per wave (loads issued / first block landed / blocks done):");
        for (int w = 0; w < NCW; ++w) fprintf(stderr, " %.2f/%.2f/%.2f", rel(16 + w), rel(24 + w), rel(32 + w));
        fprintf(stderr, "\n");
      }
      if (h[S * q + 14])
        fprintf(stderr, "[la trace]             attention loop of wave 0: %d key blocks in %.2f us, of which %.2f us waiting for them\n",
                (int)h[S * q + 14], h[S * q + 15] * 0.01, h[S * q + 13] * 0.01);
    }
    if (f->use_r) fprintf(stderr, "[la trace]   kernel entry %.1f us, schedules written %.1f us before the first phase\n", (double)(long long)(h[0] - h[13]) * 0.01, (double)(long long)(h[0] - h[14]) * 0.01);
    if (f->use_r) {
      fprintf(stderr, "[la trace]   waves end, us after the first phase (workgroup 0, then workgroup 200):");
      for (int k = 0; k < 16; ++k) fprintf(stderr, " %.1f", (double)(long long)(h[16 + k] - h[0]) * 0.01);
      fprintf(stderr, "\n");
    }
    if (f->use_r) {
      unsigned long long hi = 0; int who = -1, wv = -1;
      for (int g = 3; g < f->n_wgs; ++g)
        for (int k = 0; k < 8; ++k) {
          unsigned long long t = h[(size_t)TRACE_SLOTS * f->trace_phases + (size_t)TRACE_WG * g + k];
          if (t > hi) { hi = t; who = g; wv = k; }
        }
      fprintf(stderr, "[la trace]   last wave to end: workgroup %d wave %d, %.1f us after the first phase; ends of the last workgroups' waves:", who, wv, (double)(long long)(hi - h[0]) * 0.01);
      for (int g = std::max(1, f->n_wgs - 3); g < f->n_wgs; ++g)
        for (int k = 0; k < 8; ++k) fprintf(stderr, " %.0f", (double)(long long)(h[(size_t)TRACE_SLOTS * f->trace_phases + (size_t)TRACE_WG * g + k] - h[0]) * 0.01);
      fprintf(stderr, "\n");
    }
    if (f->use_r && np > 11) {  // register-streaming kernel: when the MFMA waves of workgroup 0 started each body of the second layer
      const unsigned long long *mw = &h[(size_t)TRACE_SLOTS * f->trace_phases + TRACE_WG];
      const unsigned t0 = (unsigned)h[(size_t)TRACE_SLOTS * 6];  // (start of the second layer's first phase)
      for (int w = 0; w < 4; ++w) {
        fprintf(stderr, "[la trace]   MFMA wave %d, second layer, start of its bodies, us after the layer's first phase began (of which waiting for operand):", w);
        for (int e = 0; e < 16; ++e)
          fprintf(stderr, " %.1f(%.1f)", (double)(short)(unsigned short)(((unsigned)mw[16 * w + e] & 0xffffu) - (t0 & 0xffffu)) * 0.01,
                  (double)((unsigned)mw[16 * w + e] >> 16) * 0.01);
        fprintf(stderr, "\n");
      }
    }
    if (np > 1 && h[S * (np - 1)] > h[0])
      fprintf(stderr, "[la trace]   shader clock over the launch: %.0f MHz\n",
              (double)(h[S * (np - 1) + 12] - h[12]) / ((h[S * (np - 1)] - h[0]) * 0.01));
    if (np > 11 && (np - 1) % 5 == 0) {  // layer_stack: five phases a layer after the first one
      fprintf(stderr, "[la trace]   per layer, us (shader clock, MHz):");
      for (int l = 0; 5 * l + 6 < np; ++l) {
        const unsigned long long *p0 = &h[(size_t)S * (5 * l + 1)], *p1 = &h[(size_t)S * (5 * l + 6)];
        fprintf(stderr, " %.1f (%.0f)", (p1[0] - p0[0]) * 0.01, p1[0] > p0[0] ? (double)(p1[12] - p0[12]) / ((p1[0] - p0[0]) * 0.01) : 0.0);
      }
      fprintf(stderr, "\n");
    }
    if (env_int("LA_TRACE", 0) > 2) {  // every phase: start after the launch's first mark, duration up to its last mark
      fprintf(stderr, "[la trace]   every phase, start (us):");
      for (int q = 0; q < np; ++q) fprintf(stderr, " %.1f", (h[S * q] - h[0]) * 0.01);
      fprintf(stderr, "\n");
    }
    double st[6] = {0, 0, 0, 0, 0, 0};
    for (int g = 0; g < f->n_wgs; ++g)
      for (int k = 0; k < 6; ++k) st[k] += (double)h[(size_t)TRACE_SLOTS * f->trace_phases + TRACE_WG * g + k] / f->n_wgs;
    fprintf(stderr, "[la trace]   producer (mean per workgroup): ring full %.1f times, %.1f polls; of %.1f us: draining before a poll %.1f us, "
            "polling for space %.1f us, waiting for the oldest chunk %.1f us\n", st[1], st[0], st[5] * 0.01, st[2] * 0.01, st[3] * 0.01, st[4] * 0.01);
    {  // the producers at eight positions of one stretch of the stream (layer_stack: the gate / up weights of the second layer)
      for (int g : {0, 1, 130, env_int("LA_TRACE_WG", 130)}) {
        if (g >= f->n_wgs) continue;
        const unsigned long long *sa = &h[(size_t)TRACE_SLOTS * f->trace_phases + (size_t)TRACE_WG * g + 16];
        if (!sa[7] || sa[7] <= sa[0]) continue;
        fprintf(stderr, "[la trace]   producer of workgroup %d over one weight matrix of the second layer (LA_TRACE_SEG: 0 QKV, 1 O, 2 gate/up, 3 down), per eighth: us (waiting oldest / polling / pacing):", g);
        for (int k = 1; k < 8; ++k) {
          auto w = [&](int i) { return (double)(sa[8 + i] & 0xffffffu); };
          auto pl = [&](int i) { return (double)((sa[8 + i] >> 24) & 0xffffffu); };
          auto pc = [&](int i) { return (double)((sa[8 + i] >> 48) & 0xffffu); };
          fprintf(stderr, " %.1f (%.1f/%.1f/%.1f)", (sa[k] - sa[k - 1]) * 0.01, (w(k) - w(k - 1)) * 0.01, (pl(k) - pl(k - 1)) * 0.01,
                  (pc(k) - pc(k - 1)) * 0.01);
        }
        fprintf(stderr, "\n");
      }
    }
    if (env_int("LA_TRACE", 0) > 1) {  // every producer: when it reached the traced matrix's end, and how long the matrix took it
      unsigned long long lo = ~0ull;
      for (int g = 0; g < f->n_wgs; ++g) lo = std::min(lo, h[(size_t)TRACE_SLOTS * f->trace_phases + (size_t)TRACE_WG * g + 16 + 7]);
      for (int x = 0; x < 8; ++x) {
        fprintf(stderr, "[la trace]     producers %d (end after the first / duration of the last three quarters, us):", x);
        for (int g = x; g < f->n_wgs; g += 8) {
          const unsigned long long *sa = &h[(size_t)TRACE_SLOTS * f->trace_phases + (size_t)TRACE_WG * g + 16];
          fprintf(stderr, " %.1f/%.1f", (sa[7] - lo) * 0.01, (sa[7] - sa[2]) * 0.01);
        }
        fprintf(stderr, "\n");
      }
    }
    // when each workgroup reached the barrier that ends a phase, relative to the first one there
    for (int k = 0; k < 8 && a.trace_sel + k < np - 1; ++k) {
      const size_t base = (size_t)TRACE_SLOTS * f->trace_phases + 8 + k;
      unsigned long long lo = ~0ull, hi = 0;
      auto counted = [&](int g) { return !(f->use_r && (g == 1 || g == 2)); };  // (their words hold the MFMA waves' timeline)
      for (int g = 0; g < f->n_wgs; ++g) {
        if (!counted(g)) continue;
        lo = std::min(lo, h[base + (size_t)TRACE_WG * g]);
        hi = std::max(hi, h[base + (size_t)TRACE_WG * g]);
      }
      double mean = 0, xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, half[2] = {0, 0};
      int nx[8] = {0, 0, 0, 0, 0, 0, 0, 0}, nh[2] = {0, 0};
      for (int g = 0; g < f->n_wgs; ++g) {
        if (!counted(g)) continue;
        double t = (h[base + (size_t)TRACE_WG * g] - lo) * 0.01;
        mean += t / f->n_wgs;
        xcd[g % 8] += t; ++nx[g % 8];
        half[g * 2 / f->n_wgs] += t; ++nh[g * 2 / f->n_wgs];
      }
      fprintf(stderr, "[la trace]   arrivals at the barrier after phase %d: mean %.2f last %.2f us after the first (workgroup 0: %.2f); "
              "by workgroup %% 8:", a.trace_sel + k, mean, (hi - lo) * 0.01, (h[base] - lo) * 0.01);
      for (int x = 0; x < 8; ++x) fprintf(stderr, " %.2f", nx[x] ? xcd[x] / nx[x] : 0.0);
      fprintf(stderr, "; first / second half of the grid: %.2f / %.2f\n", nh[0] ? half[0] / nh[0] : 0.0, nh[1] ? half[1] / nh[1] : 0.0);
      if (env_int("LA_TRACE", 0) > 1) {  // every workgroup, one line per (workgroup % 8)
        for (int x = 0; x < 8; ++x) {
          fprintf(stderr, "[la trace]     %d:", x);
          for (int g = x; g < f->n_wgs; g += 8) fprintf(stderr, " %.1f", counted(g) ? (h[base + (size_t)TRACE_WG * g] - lo) * 0.01 : -1.0);
          fprintf(stderr, "\n");
        }
      }
    }
  }
#endif
  return LA_OK;
}

static int sync_gains(MfmaModel *f, hipStream_t s) {
  if (!f->gains_dirty) return LA_OK;
  LA_HIP(hipMemcpyAsync(f->dev_gains, f->host_gains.data(), f->host_gains.size() * sizeof(LayerGains), hipMemcpyHostToDevice, s));
  LA_HIP(hipStreamSynchronize(s));  // host_gains is pageable memory
  f->gains_dirty = false;
  return LA_OK;
}

static StackArgs base_stack_args(la_model *m, int Bp) {
  MfmaModel *f = m->mf;
  const la_model_desc &d = m->d;
  StackArgs a{};
  a.gains = f->dev_gains;
  a.Bp = Bp;
  a.MT = ceil_div(Bp, 16);
  a.d = d.d_model;
  a.Hq = d.n_q_heads;
  a.Hkv = d.n_kv_heads;
  a.dh = d.head_dim;
  a.F = d.d_ffn;
  a.ncg = d.d_model / 16;
  a.eps = d.rms_eps;
  a.inv_d = 1.0f / (float)d.d_model;
  a.theta = (double)d.rope_theta;
  a.xa = f->xa;
  a.attn_a = f->attn_a;
  a.act_a = f->act_a;
  a.qf = f->qf;
  a.xa_stride = (size_t)LA_MAX_ROWS * d.d_model;
  a.attn_stride = (size_t)LA_MAX_ROWS * m->qdim();
  a.act_stride = (size_t)LA_MAX_ROWS * d.d_ffn;
  a.rsq_stride = (size_t)LA_MAX_ROWS * (d.d_model / 16);
  a.rsq = f->rsq;
  a.cs = m->rope_cs;
  a.sync = f->sync;
  a.att_part = f->att_part;
  a.att_cnt = f->att_cnt;
  a.err = m->err_dev;
  a.err_map = m->err_map;
  a.spin_global = m->barrier_spins ? m->barrier_spins : SPIN_GLOBAL;
#ifdef LA_EXPERIMENTS
  a.dbg = env_int("LA_DBG", 0);
#endif
  a.pace = (unsigned)env_int("LA_PACE", 700);
  a.qkv = dev_plan(f->p_qkv);
  a.o = dev_plan(f->p_o);
  a.gu = dev_plan(f->p_gu);
  a.down = dev_plan(f->p_down);
  a.un = dev_plan(f->p_un);
  return a;
}

int mfma_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos, const uint64_t *vis,
                 la_kv *kv, hipStream_t s) {
  MfmaModel *f = m->mf;
  if (lb == le) return LA_OK;
  int rc = sync_gains(f, s);
  if (rc) return rc;
  StackArgs a = base_stack_args(m, Bp);
  a.mode = 0;
  a.f16 = m->d.dtype == LA_F16;
  a.lb = lb;
  a.le = le;
  a.wstream = f->wstream;
  a.cu_bytes = f->cu_bytes;
  a.seg_frags = f->seg_frags;
  a.x = hidden;
  a.pos = pos;
  a.vis = vis;
  a.K = (uint16_t *)kv->K;
  a.V = (uint16_t *)kv->V;
  a.layer_elems = kv->layer_elems();
  a.L_dev = kv->L_dev;
  a.max_len = kv->max_len;
  return launch_stack("layer_stack", f, a, 5 * (le - lb), s);
}

int mfma_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, hipStream_t s) {
  MfmaModel *f = m->mf;
  LA_REQUIRE(f->ustream != nullptr, LA_EINVAL, "model was created without an unembedding matrix");
  StackArgs a = base_stack_args(m, Bp);
  a.mode = 1;
  a.wstream = f->ustream;
  a.cu_bytes = f->ucu_bytes;
  a.seg_frags = (unsigned)(f->ucu_bytes / 1024);
  a.xa = f->xa_u;
  a.rsq = f->rsq_u;
  a.x = const_cast<float *>(hidden);
  a.g_final = m->g_final;
  a.un_part = f->un_part;
  a.un_parts_per_cu = f->un_parts_per_cu;
  a.ids = ids;
  a.top2 = top2;
  a.L_dev = f->zero_len;
  a.max_len = LA_MAX_ROWS;
  return launch_stack("unembed_argmax", f, a, 2, s);
}

}  // namespace la
#include "la_prefill.h"
namespace la {

// ---- the unembedding for callers that cannot allocate ------------------------------------------------
// Everything the unembedding kernel needs beyond the caller's buffers and the packed weights sits in one static array per
// GPU: the barrier words and the {cache length 0, error word} pair (cleared by every call), the f16 operand fragments of
// the normalised rows, the row statistics and the partial arg-max records (each fully rewritten, for the rows in use,
// before it is read).  Calls that overlap on one GPU would share these words and race.
constexpr size_t NA_SYNC_BYTES = (size_t)SYNC_STRIDE * 66 * 4;
constexpr size_t NA_ZERO_BYTES = NA_SYNC_BYTES + 256;  // barrier words, then the length / error pair
constexpr int NA_MAX_D = 8192;                         // d_model
constexpr int NA_MAX_PARTS = 4096;                     // workgroups x partial records per workgroup
constexpr size_t NA_OFF_XA = NA_ZERO_BYTES;
constexpr size_t NA_OFF_RSQ = NA_OFF_XA + (size_t)LA_MAX_ROWS * NA_MAX_D * 2;
constexpr size_t NA_OFF_TOP = NA_OFF_RSQ + (size_t)LA_MAX_ROWS * (NA_MAX_D / 16) * 4;
constexpr size_t NA_BYTES = NA_OFF_TOP + (size_t)NA_MAX_PARTS * 64 * sizeof(Top);  // 4.1 MiB
static_assert(NA_OFF_XA % 256 == 0 && NA_OFF_RSQ % 256 == 0 && NA_OFF_TOP % 256 == 0, "256-byte aligned parts");
static __device__ __align__(256) unsigned char scratch[NA_BYTES];

constexpr int NA_MAX_DEVICES = 64;
static unsigned char *na_ptr[NA_MAX_DEVICES] = {};  // this GPU's copy of `scratch`, looked up once per device
static std::mutex na_mutex;

// Called at model creation with the model's device current.
static int na_setup(int device) {
  if (device < 0 || device >= NA_MAX_DEVICES) return LA_OK;  // the entry point reports the missing address
  std::lock_guard<std::mutex> lock(na_mutex);
  if (na_ptr[device]) return LA_OK;
  unsigned char *p = nullptr;
  LA_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
  LA_REQUIRE(p != nullptr, LA_EHIP, "no device address for the static scratch array");
  LA_HIP(hipMemset(p, 0, NA_BYTES));
  na_ptr[device] = p;
  return LA_OK;
}

int mfma_unembed_argmax_noalloc(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, hipStream_t s) {
  MfmaModel *f = m->mf;
  LA_REQUIRE(f->ustream != nullptr, LA_EINVAL, "model was created without an unembedding matrix");
  LA_REQUIRE(m->d.d_model <= NA_MAX_D, LA_ERANGE, "d_model=%d exceeds the %d the static scratch array holds", m->d.d_model, NA_MAX_D);
  LA_REQUIRE((long long)f->n_wgs * f->un_parts_per_cu <= NA_MAX_PARTS, LA_ERANGE,
             "vocab=%d needs %lld partial arg-max records, the static scratch array holds %d", m->d.vocab,
             (long long)f->n_wgs * f->un_parts_per_cu, NA_MAX_PARTS);
  unsigned char *base = (m->device >= 0 && m->device < NA_MAX_DEVICES) ? na_ptr[m->device] : nullptr;
  LA_REQUIRE(base != nullptr, LA_EHIP, "the static scratch array has no address on device %d", m->device);
  zero_u32_kernel<<<ceil_div((int)(NA_ZERO_BYTES / 4), 256), 256, 0, s>>>((unsigned *)base, (int)(NA_ZERO_BYTES / 4));
  LA_HIP(hipGetLastError());
  StackArgs a = base_stack_args(m, Bp);
  a.mode = 1;
  a.wstream = f->ustream;
  a.cu_bytes = f->ucu_bytes;
  a.seg_frags = (unsigned)(f->ucu_bytes / 1024);
  a.sync = (unsigned *)base;
  a.xa = (uint16_t *)(base + NA_OFF_XA);
  a.rsq = (float *)(base + NA_OFF_RSQ);
  a.x = const_cast<float *>(hidden);
  a.g_final = m->g_final;
  a.un_part = (Top *)(base + NA_OFF_TOP);
  a.un_parts_per_cu = f->un_parts_per_cu;
  a.ids = ids;
  a.top2 = top2;
  a.L_dev = (int32_t *)(base + NA_SYNC_BYTES);
  a.max_len = LA_MAX_ROWS;
  a.err = (int32_t *)(base + NA_SYNC_BYTES) + 1;
  return launch_stack("unembed_argmax", f, a, 2, s, true);
}

}  // namespace la
