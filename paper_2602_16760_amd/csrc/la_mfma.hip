// bf16 MFMA path for gfx950: the whole layer stack of a verification step as ONE persistent
// kernel -- weight-streaming skinny GEMMs, masked-block GQA attention, fused norm / RoPE /
// SwiGLU / residual epilogues -- and a second one for the unembedding with fused arg-max.
//
// Why one kernel.  A step reads every weight once (13 GB at the 30-layer Mistral-7B shape) and
// computes almost nothing per byte, so it is bound by HBM; a layer is ~55 us of streaming
// split over four GEMMs with an attention and several small reductions in between.  Separate
// kernels drain the memory pipeline at each of those ~270 boundaries.  Here one workgroup per
// CU stays resident and walks a list of phases; phases are separated by a grid barrier, and
// the weights of the next GEMM are already in flight (loaded into registers) while the
// barrier is being waited for.
//
// Data movement
//   weights      [slab][k-tile][tile-in-slab][lane][8] bf16; a slab is T 16-column tiles.
//                HBM -> registers -> MFMA, no LDS: each 1 KB fragment is used exactly once.
//   activations  [k-tile][row-tile][lane][8] bf16, the MFMA operand fragment, written by the
//                producing phase.  A fragment: lane l holds index (l & 15) of the 16-wide
//                dimension and contraction indices 8*(l >> 4) .. +7 of a 32-wide k-tile, so
//                every load a wave issues is one contiguous 1 KB segment (64 lanes x 128 bit).
//   Everything one workgroup writes for another to read in a later phase (operand fragments,
//   fp32 partials, norm statistics, the block's K/V rows, attention partials) is stored and
//   loaded with the device-scope cache policy (sc1) so that no cache flush or invalidate is
//   needed at a barrier: the barrier is a wait for the stores plus relaxed atomics.
//
// GEMM tasks.  A task is one slab with the whole contraction, so every task yields finished
// outputs and its epilogue can apply what follows the product: the QKV epilogue scales by the
// norm factor, rotates q and k (the packed column order puts channel i and i + dh/2 of a head
// in the same slab), writes q as operand fragments and K, V into the cache; the O and down
// epilogues add to the residual stream, emit the sum of squares of their columns and the
// operand fragments of the next GEMM; the gate/up epilogue applies SwiGLU.  Seven waves split
// the contraction, accumulate in registers and are summed through LDS in a fixed tree; the
// eighth wave runs the grid barrier so that its polling never queues behind prefetched weights.
// RMSNorm is applied as ((x * g) W) * rsqrt(mean(x^2) + eps), the row factor after the
// contraction.  All reductions have a fixed order: results are run-to-run identical.
//
// Operand fragments and norm statistics live in buffers that are written once per launch
// (one per layer and use), so a reader can never find a stale copy in its L2 and may load
// them through the cache; only data read once (attention partials, q fragments, the block's
// K/V rows) is loaded with sc1.
#include <stdio.h>

#include <algorithm>
#include <new>

#include "la_device.h"
#include "la_internal.h"

namespace la {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

constexpr int WG_THREADS = 512;
constexpr int NCW = 7;             // compute waves of a GEMM phase; wave 7 runs the grid barrier
constexpr int MAX_T = 8;           // 16-column tiles per slab
constexpr int MAX_MT = LA_MAX_ROWS / 16;
constexpr unsigned OOB = 0x80000000u;   // voffset beyond every buffer (all are < 2 GiB)
constexpr unsigned RSRC_BYTES = 0x7fffffffu;
constexpr int DEV = 16;            // cache policy sc1: device-scope coherent load / store
constexpr int SYNC_GROUP = 16;     // workgroups per arrival counter of the grid barrier
constexpr int SYNC_STRIDE = 64;    // 32-bit words between barrier variables (256 B)
constexpr unsigned SPIN_LIMIT = 1u << 19;  // polls (~1 us each) before a barrier gives up

struct Top {  // running arg-max of one row: best value, its index, runner-up value
  float v1;
  int i1;
  float v2;
};

__device__ __forceinline__ Top top_merge2(Top a, Top b) {
  bool bw = (b.v1 > a.v1) || (b.v1 == a.v1 && b.i1 < a.i1);
  Top r;
  r.v1 = bw ? b.v1 : a.v1;
  r.i1 = bw ? b.i1 : a.i1;
  r.v2 = fmaxf(bw ? a.v1 : b.v1, fmaxf(a.v2, b.v2));
  return r;
}

enum Phase {
  PH_PREP = 0,  // x -> operand fragments of the first QKV GEMM, norm statistics, RoPE table
  PH_QKV,       // QKV GEMM; epilogue: norm factor, RoPE, q fragments, K/V rows into the cache
  PH_ATT,       // masked-block attention per (kv head, key split)
  PH_COMB,      // merge key splits -> operand fragments of the O GEMM
  PH_O,         // output projection; epilogue: x +=, statistics, fragments for gate/up
  PH_GU,        // gate/up GEMM + SwiGLU -> fragments for down
  PH_DOWN,      // down projection; epilogue: x +=, statistics, fragments for the next layer
  PH_UPREP,     // final norm operand fragments
  PH_UGEMM,     // unembedding with per-slab arg-max
  PH_UFINAL     // arg-max over slabs
};
constexpr int PHASES_PER_LAYER = 6;

enum GemmMode { MODE_QKV = 0, MODE_RESID = 1, MODE_GATEUP = 2, MODE_UNEMBED = 3 };

struct GemmDev {
  int KT, T, n_slabs, N;
};

struct LayerPtrs {
  const uint16_t *wqkv, *wo, *wgu, *wdown;
  const float *g_attn, *g_mlp;
};

struct StackArgs {
  const LayerPtrs *layers;
  int mode;  // 0: layer stack, 1: unembedding
  int lb, le, p_begin, p_end;
  int Bp, MT, d, Hq, Hkv, dh, F, ncg, ns;
  float eps, inv_d;
  double theta;
  GemmDev qkv, o, gu, down, un;
  float *x;
  const int32_t *pos;
  const uint64_t *vis;
  // write-once operand / statistics buffers, indexed by absolute layer (see frag_of)
  uint16_t *xa, *attn_a, *act_a, *qf;
  size_t xa_stride, attn_stride, act_stride, rsq_stride;  // elements per (layer, use)
  float *rsq, *o_part, *ml_part, *cs;
  uint16_t *K, *V;
  size_t layer_elems;
  const int32_t *L_dev;
  int max_len;
  int32_t *err;
  const uint16_t *un_w;
  const float *g_final;
  Top *un_part;
  int32_t *ids;
  float *top2;
  unsigned *sync;
  unsigned epoch0, n_groups;
  unsigned long long *trace;  // optional: 3 timestamps per phase from workgroup 0 (entry, after barrier, end)
  size_t trace_wg_off;        // then per barrier and workgroup: arrival and release time
};

__device__ __forceinline__ void trace_mark(const StackArgs &a, int slot) {
  if (a.trace && blockIdx.x == 0 && threadIdx.x == 0) a.trace[slot] = wall_clock64();
}

// ---- device-scope accessors ------------------------------------------------------------------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void *p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, RSRC_BYTES, 0x00020000);
}
__device__ __forceinline__ u32x4 ld128(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, DEV);
}
__device__ __forceinline__ void st128(__amdgpu_buffer_rsrc_t r, unsigned byte_off, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, DEV);
}
__device__ __forceinline__ float ld32f(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, DEV));
}
__device__ __forceinline__ void st32f(__amdgpu_buffer_rsrc_t r, unsigned byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, byte_off, 0, DEV);
}
__device__ __forceinline__ void st16(__amdgpu_buffer_rsrc_t r, unsigned byte_off, uint16_t v) {
  __builtin_amdgcn_raw_buffer_store_b16(v, r, byte_off, 0, DEV);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return (uint32_t)float_to_bf16(lo) | ((uint32_t)float_to_bf16(hi) << 16);
}

// ---- grid barrier -----------------------------------------------------------------------------
// Arrival counters per group of SYNC_GROUP workgroups, one top counter, one release word; all
// monotonic (epoch e is complete when a counter reaches e * members).  Only relaxed device-scope
// atomics: the data exchanged between workgroups travels with sc1 accesses.  The spin is
// bounded: on a timeout the error flag is raised, this workgroup leaves the kernel (the others
// then time out at the same barrier and leave too) and the host reports the failure.
__device__ __forceinline__ void grid_arrive_wait(const StackArgs &a, unsigned epoch, int *dead) {
  if ((threadIdx.x & 63) == 0) {
    unsigned n = gridDim.x;
    unsigned g = blockIdx.x / SYNC_GROUP;
    unsigned gsize = (g + 1) * SYNC_GROUP <= n ? SYNC_GROUP : n - g * SYNC_GROUP;
    unsigned *gc = a.sync + SYNC_STRIDE * g, *top = a.sync + SYNC_STRIDE * 64, *rel = a.sync + SYNC_STRIDE * 65;
    unsigned long long *tr = a.trace ? a.trace + a.trace_wg_off + ((size_t)(epoch - a.epoch0) * gridDim.x + blockIdx.x) * 2 : nullptr;
    if (tr) tr[0] = wall_clock64();
    unsigned old = __hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == epoch * gsize) {
      unsigned t = __hip_atomic_fetch_add(top, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (t + 1 == epoch * a.n_groups) __hip_atomic_store(rel, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    unsigned spins = 0;
    while (__hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > SPIN_LIMIT) {
        __hip_atomic_fetch_or(a.err, 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *dead = 1;
        break;
      }
    }
    if (tr) tr[1] = wall_clock64();
  }
}

// Workgroup barrier that the compiler may not move memory operations across, without the
// implicit wait for outstanding loads that __syncthreads() carries.
__device__ __forceinline__ void wg_barrier_raw() {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_barrier();
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

// All of this wave's stores have been acknowledged; then the whole workgroup's.
__device__ __forceinline__ void wg_stores_done() {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);
  wg_barrier_raw();
}

// Entry barrier of a phase that has nothing to prefetch.  Returns false after a timeout.
__device__ __forceinline__ bool grid_barrier(const StackArgs &a, unsigned epoch, int *dead) {
  wg_stores_done();
  if ((threadIdx.x >> 6) == NCW) grid_arrive_wait(a, epoch, dead);
  wg_barrier_raw();
  return *dead == 0;
}

// ---- GEMM phase -------------------------------------------------------------------------------
template <int MT, int T>
struct Depth {  // k-tiles in flight per wave, bounded by the register file
  static constexpr int raw = (184 - 4 * MT * T) / (4 * (MT + T));
  static constexpr int value = raw < 2 ? 2 : (raw > 10 ? 10 : raw);
};

struct GemmIo {
  const uint16_t *W;
  const uint16_t *A;      // operand fragments (a write-once buffer: loaded through the cache)
  int mode;
  const float *rsq_in;    // MODE_QKV, MODE_GATEUP: sums of squares of the input rows [64][ncg]
  uint16_t *Kc, *Vc;      // MODE_QKV: this layer's cache
  int L;
  const float *gain;      // MODE_RESID: gain of the next norm (nullptr: no fragments wanted)
  uint16_t *xa_out;       // MODE_RESID: fragments of x * gain for the next GEMM
  float *rsq_out;         // MODE_RESID: sums of squares of the new x
  uint16_t *act_a;        // MODE_GATEUP: fragments for the down projection
  Top *un_part;           // MODE_UNEMBED
};

// One GEMM phase of this workgroup.  `epoch` != 0: run the grid barrier first, with the
// weights of the first task already requested before the wait.
template <int MT, int T>
__device__ __forceinline__ bool gemm_phase(const StackArgs &a, const GemmDev &g, const GemmIo &io, unsigned epoch,
                                           f32x4 *lds, int *dead) {
  constexpr int D = Depth<MT, T>::value;
  constexpr int LDT = 16 * T + 4;  // padded row length of the result tile in LDS
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int n_tasks = g.n_slabs;
  __amdgpu_buffer_rsrc_t rw = rsrc_of(io.W), ra = rsrc_of(io.A);
  float *tile = (float *)lds;                         // [16 MT][LDT] after the tree
  float *rs_lds = (float *)(lds + 3 * MT * T * 64);   // [64] row factors (MODE_GATEUP)
  const unsigned voff = lane * 16;

  if (epoch) wg_stores_done();
  bool first = true;
  for (int task = blockIdx.x; task < n_tasks || first; task += gridDim.x) {
    const bool live = task < n_tasks;
    const int slab = live ? task : 0;
    const int cw = wave < NCW ? wave : 0;
    const int wk0 = g.KT * cw / NCW, wk1 = g.KT * (cw + 1) / NCW;
    const int n = (live && wave < NCW) ? wk1 - wk0 : 0;
    const unsigned w_base = (unsigned)(((size_t)slab * g.KT + wk0) * T * 1024);
    const unsigned a_base = (unsigned)wk0 * MT * 1024;

    u32x4 rA[D][MT], rW[D][T];
    auto load_w = [&](int slot, int i) {
      unsigned vo = (i < n) ? voff : OOB;  // out of range: zeros come back, no memory traffic
#pragma unroll
      for (int t = 0; t < T; ++t)
        rW[slot][t] = __builtin_amdgcn_raw_buffer_load_b128(rw, vo, w_base + (unsigned)(i * T + t) * 1024, 0);
    };
    auto load_a = [&](int slot, int i) {
      unsigned vo = (i < n) ? voff : OOB;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        rA[slot][mt] = __builtin_amdgcn_raw_buffer_load_b128(ra, vo, a_base + (unsigned)(i * MT + mt) * 1024, 0);
    };
    // weights do not depend on the previous phase: request them before waiting at the barrier
#pragma unroll
    for (int s = 0; s < D; ++s) {
      load_w(s, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (first && epoch) {
      if (wave == NCW) grid_arrive_wait(a, epoch, dead);
      wg_barrier_raw();
      if (*dead) return false;
    }
    if (first) trace_mark(a, 3 * (int)(epoch - a.epoch0) + 1);
    first = false;
    if (!live) break;
#pragma unroll
    for (int s = 0; s < D; ++s) {
      load_a(s, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    if ((io.mode == MODE_GATEUP || io.mode == MODE_QKV) && wave == NCW) {
      // row factors rsqrt(mean(x^2) + eps) from the per-slab sums of squares: one row per
      // lane, all loads independent of each other (ncg is a multiple of 4)
      float s = 0.f;
      if (lane < a.Bp) {
        const f32x4 *rq = reinterpret_cast<const f32x4 *>(io.rsq_in + (size_t)lane * a.ncg);
        for (int c4 = 0; c4 < a.ncg / 4; ++c4) {
          f32x4 v = rq[c4];
          s += (v[0] + v[1]) + (v[2] + v[3]);
        }
      }
      rs_lds[lane] = 1.0f / sqrtf(s * a.inv_d + a.eps);
    }

    f32x4 acc[MT][T];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int t = 0; t < T; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 < n; i0 += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < T; ++t)
            acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, rA[s][mt]),
                                                                  __builtin_bit_cast(bf16x8, rW[s][t]), acc[mt][t], 0, 0, 0);
        load_w(s, i0 + s + D);
        load_a(s, i0 + s + D);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // fixed-order tree over the 7 compute waves: (0+4, 1+5, 2+6), (0+2, 1+3), (0+1)
    __syncthreads();
#pragma unroll
    for (int half = 4; half >= 1; half >>= 1) {
      if (wave >= half && wave < 2 * half && wave < NCW) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < T; ++t) lds[((wave - half) * MT * T + mt * T + t) * 64 + lane] = acc[mt][t];
      }
      __syncthreads();
      if (wave < half && wave + half < NCW) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < T; ++t) acc[mt][t] += lds[(wave * MT * T + mt * T + t) * 64 + lane];
      }
      __syncthreads();
    }
    // wave 0 lays the finished tile out row-major in LDS; acc[mt][t][i] is the element
    // (row 16 mt + 4 (lane >> 4) + i, column 16 t + (lane & 15)) of the slab
    if (wave == 0) {
      const int q4 = lane >> 4, c16 = lane & 15;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) tile[(16 * mt + 4 * q4 + i) * LDT + 16 * t + c16] = acc[mt][t][i];
    }
    __syncthreads();

    if (io.mode == MODE_QKV) {
      // The slab holds channels 8j..8j+7 (columns 0..7) and dh/2 + 8j.. (columns 8..15) of one
      // head: both members of every RoPE pair.  One thread per row.
      const int b = threadIdx.x;
      if (b < a.Bp) {
        const int half = a.dh >> 1, spj = a.dh >> 4, grp = a.Hq / a.Hkv;
        const int hs = slab / spj, j = slab - hs * spj;
        const float rs = rs_lds[b];
        const float *tr = tile + b * LDT;
        const float qscale = hs < a.Hq ? 1.0f / sqrtf((float)a.dh) : 1.0f;
        float y0[8], y1[8];
#pragma unroll
        for (int w = 0; w < 8; ++w) {
          float x0 = tr[w] * rs, x1 = tr[8 + w] * rs;
          if (hs < a.Hq + a.Hkv) {
            float c = a.cs[((size_t)b * half + 8 * j + w) * 2], sn = a.cs[((size_t)b * half + 8 * j + w) * 2 + 1];
            y0[w] = (x0 * c - x1 * sn) * qscale;
            y1[w] = (x1 * c + x0 * sn) * qscale;
          } else {
            y0[w] = x0;
            y1[w] = x1;
          }
        }
        u32x4 lo = {pack_bf16(y0[0], y0[1]), pack_bf16(y0[2], y0[3]), pack_bf16(y0[4], y0[5]), pack_bf16(y0[6], y0[7])};
        u32x4 hi = {pack_bf16(y1[0], y1[1]), pack_bf16(y1[2], y1[3]), pack_bf16(y1[4], y1[5]), pack_bf16(y1[6], y1[7])};
        const int o_lo = j, o_hi = (half >> 3) + j;  // channel octets of the two pieces
        if (hs < a.Hq) {
          __amdgpu_buffer_rsrc_t rqf = rsrc_of(a.qf);
          int kvh = hs / grp, jq = hs - kvh * grp, rt = jq * MT + (b >> 4);
          size_t fb = ((size_t)kvh * (grp * MT) + rt) * (a.dh >> 5);
          st128(rqf, (unsigned)(((fb + (o_lo >> 2)) * 64 + (b & 15) + 16 * (o_lo & 3)) * 16), lo);
          st128(rqf, (unsigned)(((fb + (o_hi >> 2)) * 64 + (b & 15) + 16 * (o_hi & 3)) * 16), hi);
        } else if (hs < a.Hq + a.Hkv) {
          __amdgpu_buffer_rsrc_t rk = rsrc_of(io.Kc);
          size_t rb = ((size_t)(io.L + b) * a.Hkv + (hs - a.Hq)) * a.dh;
          st128(rk, (unsigned)((rb + 8 * o_lo) * 2), lo);
          st128(rk, (unsigned)((rb + 8 * o_hi) * 2), hi);
        } else {
          __amdgpu_buffer_rsrc_t rv = rsrc_of(io.Vc);
          int h = hs - a.Hq - a.Hkv;
#pragma unroll
          for (int w = 0; w < 8; ++w) {
            st16(rv, (unsigned)(v_index(true, io.L + b, h, 8 * j + w, a.Hkv, a.dh) * 2), float_to_bf16(y0[w]));
            st16(rv, (unsigned)(v_index(true, io.L + b, h, half + 8 * j + w, a.Hkv, a.dh) * 2), float_to_bf16(y1[w]));
          }
        }
      }
    } else if (io.mode == MODE_RESID) {
      // x[:, slab columns] += tile; sum of squares of the new values; fragments of x * gain.
      // Two threads per row, eight columns each.  This workgroup owns these columns of x in
      // every layer, so x needs no device-scope accesses.
      const int b = threadIdx.x >> 1, oct = threadIdx.x & 1;
      if (b < a.Bp) {
        const int col = 16 * slab + 8 * oct;
        f32x4 *xp = reinterpret_cast<f32x4 *>(a.x + (size_t)b * a.d + col);
        const float *tr = tile + b * LDT + 8 * oct;
        f32x4 x0 = xp[0], x1 = xp[1];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          x0[i] += tr[i];
          x1[i] += tr[4 + i];
        }
        xp[0] = x0;
        xp[1] = x1;
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
        sq += __shfl_xor(sq, 1, 64);
        if (io.gain) {
          if (oct == 0) st32f(rsrc_of(io.rsq_out), (unsigned)(b * a.ncg + slab) * 4, sq);
          const float *gp = io.gain + col;
          u32x4 w = {pack_bf16(x0[0] * gp[0], x0[1] * gp[1]), pack_bf16(x0[2] * gp[2], x0[3] * gp[3]),
                     pack_bf16(x1[0] * gp[4], x1[1] * gp[5]), pack_bf16(x1[2] * gp[6], x1[3] * gp[7])};
          st128(rsrc_of(io.xa_out), (unsigned)((((size_t)(col >> 5) * MT + (b >> 4)) * 64 + (b & 15) + 16 * ((col & 31) >> 3)) * 16), w);
        }
      }
    } else if (io.mode == MODE_GATEUP) {
      // slab columns: 8T gate channels, then the same 8T channels of up
      __amdgpu_buffer_rsrc_t rp = rsrc_of(io.act_a);
      const int chunks = a.Bp * T;
      for (int c = threadIdx.x; c < chunks; c += WG_THREADS) {
        int row = c / T, oct = c - row * T;
        float rs = rs_lds[row];
        const float *gp = tile + row * LDT + 8 * oct, *up = gp + 8 * T;
        float act[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float gt = gp[i] * rs, u = up[i] * rs;
          act[i] = gt / (1.0f + __expf(-gt)) * u;
        }
        int f = slab * 8 * T + 8 * oct;
        unsigned o = (unsigned)((((size_t)(f >> 5) * MT + (row >> 4)) * 64 + (row & 15) + 16 * ((f & 31) >> 3)) * 16);
        st128(rp, o, u32x4{pack_bf16(act[0], act[1]), pack_bf16(act[2], act[3]), pack_bf16(act[4], act[5]),
                           pack_bf16(act[6], act[7])});
      }
    } else {  // MODE_UNEMBED: arg-max of each row over this slab's columns
      int row = threadIdx.x >> 3, j = threadIdx.x & 7;
      Top best{-INFINITY, 0x7fffffff, -INFINITY};
      if (row < a.Bp)
        for (int c = j; c < 16 * T; c += 8) best = top_merge2(best, Top{tile[row * LDT + c], slab * 16 * T + c, -INFINITY});
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) {
        Top other;
        other.v1 = __shfl_xor(best.v1, o, 64);
        other.i1 = __shfl_xor(best.i1, o, 64);
        other.v2 = __shfl_xor(best.v2, o, 64);
        best = top_merge2(best, other);
      }
      if (j == 0 && row < a.Bp) {
        __amdgpu_buffer_rsrc_t rp = rsrc_of(io.un_part);
        unsigned o = (unsigned)(((size_t)slab * 64 + row) * sizeof(Top));
        st32f(rp, o, best.v1);
        __builtin_amdgcn_raw_buffer_store_b32((unsigned)best.i1, rp, o + 4, 0, DEV);
        st32f(rp, o + 8, best.v2);
      }
    }
    __syncthreads();
  }
  return true;
}

template <int MT>
__device__ __forceinline__ bool gemm_dispatch(const StackArgs &a, const GemmDev &g, const GemmIo &io, unsigned epoch,
                                              f32x4 *lds, int *dead) {
  switch (g.T) {
    case 1: return gemm_phase<MT, 1>(a, g, io, epoch, lds, dead);
    case 2: return gemm_phase<MT, 2>(a, g, io, epoch, lds, dead);
    case 3: return gemm_phase<MT, 3>(a, g, io, epoch, lds, dead);
    case 4: return gemm_phase<MT, 4>(a, g, io, epoch, lds, dead);
    case 5: return gemm_phase<MT, 5>(a, g, io, epoch, lds, dead);
    case 6: return gemm_phase<MT, 6>(a, g, io, epoch, lds, dead);
    case 7: return gemm_phase<MT, 7>(a, g, io, epoch, lds, dead);
    default: return gemm_phase<MT, 8>(a, g, io, epoch, lds, dead);
  }
}

// ---- first operand of a launch: norm statistics and fragments of x * gain ----------------------
// Task = two groups of 32 columns (one per half of the workgroup).  Sums of squares are kept per
// 16 columns, the granularity of the GEMM epilogues that produce them in later phases.
__device__ __forceinline__ void prep_phase(const StackArgs &a, const float *gain, uint16_t *xa_out, float *rsq_out) {
  __amdgpu_buffer_rsrc_t rq = rsrc_of(rsq_out), rx = rsrc_of(xa_out);
  const int sub = threadIdx.x >> 8, r = (threadIdx.x & 255) >> 2, oct = threadIdx.x & 3;
  const int n_cg = a.d / 32;
  for (int task = blockIdx.x; task * 2 < n_cg; task += gridDim.x) {
    int cg = task * 2 + sub;
    if (cg >= n_cg || r >= a.Bp) continue;
    int c0 = cg * 32 + oct * 8;
    const f32x4 *xp = reinterpret_cast<const f32x4 *>(a.x + (size_t)r * a.d + c0);
    f32x4 x0 = xp[0], x1 = xp[1];
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
    sq += __shfl_xor(sq, 1, 64);
    if ((oct & 1) == 0) st32f(rq, (unsigned)(r * a.ncg + 2 * cg + (oct >> 1)) * 4, sq);
    const float *gp = gain + c0;
    u32x4 w = {pack_bf16(x0[0] * gp[0], x0[1] * gp[1]), pack_bf16(x0[2] * gp[2], x0[3] * gp[3]),
               pack_bf16(x1[0] * gp[4], x1[1] * gp[5]), pack_bf16(x1[2] * gp[6], x1[3] * gp[7])};
    st128(rx, (unsigned)((((size_t)cg * a.MT + (r >> 4)) * 64 + (r & 15) + 16 * oct) * 16), w);
  }
}

// cos/sin of pos[b] * theta^(-2i/dh) in double (exact to float rounding at any cache position)
__device__ __forceinline__ void rope_table_phase(const StackArgs &a) {
  __amdgpu_buffer_rsrc_t rc = rsrc_of(a.cs);
  int half = a.dh >> 1, total = a.Bp * half;
  for (int e = blockIdx.x * WG_THREADS + threadIdx.x; e < total; e += gridDim.x * WG_THREADS) {
    int b = e / half, i = e - b * half;
    double inv = exp2(-(double)i / (double)half * log2(a.theta));
    double s, c;
    sincos((double)a.pos[b] * inv, &s, &c);
    st32f(rc, (unsigned)e * 8, (float)c);
    st32f(rc, (unsigned)e * 8 + 4, (float)s);
  }
}

// ---- masked-block GQA attention ------------------------------------------------------------------
// Task = (kv head, key split); each wave takes q-row tiles of the head's group.  Scores are
// computed transposed (keys x q-rows) so that the probabilities leave the MFMA in the operand
// layout of the second product:
//   S^T = K Q^T      A = K tile [16 keys x 32 dh],   B = q fragment        -> lane: 4 keys of one q-row
//   O^T = V^T P^T    A = V^T tile [16 dh x 32 keys], B = p of 2 key tiles  -> lane: 4 channels of one q-row
// V is stored key-blocked (v_index) so that the V^T tile is one 128-bit load per lane.
// Output per split: O^T unnormalised, running max and sum per q-row.
template <int DH>
__device__ __forceinline__ void attention_phase(const StackArgs &a, const uint16_t *Kc, const uint16_t *Vc, int L) {
  constexpr int KT = DH / 32, DT = DH / 16;
  __amdgpu_buffer_rsrc_t rk = rsrc_of(Kc), rv = rsrc_of(Vc), rqf = rsrc_of(a.qf), ro = rsrc_of(a.o_part),
                         rm = rsrc_of(a.ml_part);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, q4 = lane >> 4,
            c16 = lane & 15;
  const int g = a.Hq / a.Hkv, n_rt = g * a.MT, QR = n_rt * 16;
  const int total = L + a.Bp, nkb = (total + 31) >> 5;
  for (int task = blockIdx.x; task < a.Hkv * a.ns; task += gridDim.x) {
    const int kvh = task / a.ns, split = task - kvh * a.ns;
    const int kb0 = (int)((long long)nkb * split / a.ns), kb1 = (int)((long long)nkb * (split + 1) / a.ns);
    for (int rt = wave; rt < n_rt; rt += 8) {
      const int b = (rt % a.MT) * 16 + c16;  // block row of this lane's q-row
      const uint64_t vb = b < a.Bp ? a.vis[b] : 0ull;
      bf16x8 q[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
        q[kt] = __builtin_bit_cast(bf16x8, ld128(rqf, (unsigned)(((((size_t)kvh * n_rt + rt) * KT + kt) * 64 + lane) * 16)));
      f32x4 o[DT];
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
      float m_run = -1e30f, l_run = 0.f;
      u32x4 ka[KT], kbv[KT], vt[DT], nka[KT], nkbv[KT], nvt[DT];
      auto load_kv = [&](int kb, u32x4 *pa, u32x4 *pb, u32x4 *pv) {
        const unsigned k_off = kb < kb1 ? (unsigned)((((size_t)(kb * 32 + c16) * a.Hkv + kvh) * DH + 8 * q4) * 2) : OOB;
        const unsigned v_off = kb < kb1 ? (unsigned)(((((size_t)kb * a.Hkv + kvh) * DH + c16) * 32 + 8 * q4) * 2) : OOB;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          pa[kt] = ld128(rk, k_off + kt * 64);
          pb[kt] = ld128(rk, k_off + (unsigned)(16 * a.Hkv * DH * 2) + kt * 64);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) pv[dt] = ld128(rv, v_off + dt * 16 * 32 * 2);
      };
      load_kv(kb0, nka, nkbv, nvt);
      for (int kb = kb0; kb < kb1; ++kb) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          ka[kt] = nka[kt];
          kbv[kt] = nkbv[kt];
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vt[dt] = nvt[dt];
        load_kv(kb + 1, nka, nkbv, nvt);  // the next block's tiles travel while this one is used
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kt]), q[kt], sa, 0, 0, 0);
          sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kbv[kt]), q[kt], sb, 0, 0, 0);
        }
        // lane holds keys kb*32 + 4 q4 + i (sa) and kb*32 + 16 + 4 q4 + i (sb) of q-row c16
        float sv[8];
        bool ok[8];
        float mx = -1e30f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          int key = kb * 32 + (i >> 2) * 16 + 4 * q4 + (i & 3);
          sv[i] = i < 4 ? sa[i] : sb[i - 4];
          ok[i] = key < L || (key < total && ((vb >> (key - L)) & 1ull));
          if (ok[i]) mx = fmaxf(mx, sv[i]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float m_new = fmaxf(m_run, mx);
        float corr = __expf(m_run - m_new);
        float p[8], ps = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          p[i] = ok[i] ? __expf(sv[i] - m_new) : 0.f;
          ps += p[i];
        }
        ps += __shfl_xor(ps, 16, 64);
        ps += __shfl_xor(ps, 32, 64);
        l_run = l_run * corr + ps;
        m_run = m_new;
        u32x4 pw = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
        bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          o[dt] *= corr;
          o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[dt]), pb, o[dt], 0, 0, 0);
        }
      }
      // o[dt][i] = O^T[channel 16 dt + 4 q4 + i][q-row rt*16 + c16]; partials are stored
      // [kv head][split][q-row][channel]: 16 bytes per lane and store
      size_t base = (((size_t)kvh * a.ns + split) * QR + rt * 16 + c16) * DH;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) st128(ro, (unsigned)((base + 16 * dt + 4 * q4) * 4), __builtin_bit_cast(u32x4, o[dt]));
      if (q4 == 0) {
        unsigned mo = (unsigned)(((((size_t)kvh * a.ns + split) * QR + rt * 16 + c16) * 2) * 4);
        st32f(rm, mo, m_run);
        st32f(rm, mo + 4, l_run);
      }
    }
  }
}

// Merge the key splits; write the attention output as operand fragments of the O GEMM.
// Task = (kv head, q-row tile) per half workgroup: 16 q-rows x DH/8 channel octets.
template <int DH>
__device__ __forceinline__ void combine_phase(const StackArgs &a, uint16_t *attn_out) {
  __amdgpu_buffer_rsrc_t ro = rsrc_of(a.o_part), rm = rsrc_of(a.ml_part), ra = rsrc_of(attn_out);
  const int g = a.Hq / a.Hkv, n_rt = g * a.MT, QR = n_rt * 16, n_units = a.Hkv * n_rt;
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255, rr = t & 15, oct = t >> 4;
  for (int task = blockIdx.x; task * 2 < n_units; task += gridDim.x) {
    int u = task * 2 + sub;
    if (u >= n_units || oct >= DH / 8) continue;
    int kvh = u / n_rt, rt = u - kvh * n_rt;
    int r = rt * 16 + rr, b = (rt % a.MT) * 16 + rr, j = rt / a.MT;
    if (b >= a.Bp) continue;
    // online merge in split order; loads of eight splits are issued together
    float M = -1e30f, lsum = 0.f;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < a.ns; s0 += 8) {
      float ms[8], ls[8];
      f32x4 lo[8], hi[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        int sp = min(s0 + k, a.ns - 1);
        size_t row = ((size_t)kvh * a.ns + sp) * QR + r;
        ms[k] = ld32f(rm, (unsigned)(row * 8));
        ls[k] = ld32f(rm, (unsigned)(row * 8 + 4));
        lo[k] = __builtin_bit_cast(f32x4, ld128(ro, (unsigned)((row * DH + oct * 8) * 4)));
        hi[k] = __builtin_bit_cast(f32x4, ld128(ro, (unsigned)((row * DH + oct * 8 + 4) * 4)));
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if (s0 + k < a.ns) {
          float m_new = fmaxf(M, ms[k]);
          float c_old = __expf(M - m_new), c_new = __expf(ms[k] - m_new);
          lsum = lsum * c_old + ls[k] * c_new;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[i] = acc[i] * c_old + lo[k][i] * c_new;
            acc[4 + i] = acc[4 + i] * c_old + hi[k][i] * c_new;
          }
          M = m_new;
        }
      }
    }
    float inv = 1.0f / lsum;
    int col = (kvh * g + j) * DH + oct * 8;
    unsigned o = (unsigned)((((size_t)(col >> 5) * a.MT + (b >> 4)) * 64 + (b & 15) + 16 * ((col & 31) >> 3)) * 16);
    st128(ra, o, u32x4{pack_bf16(acc[0] * inv, acc[1] * inv), pack_bf16(acc[2] * inv, acc[3] * inv),
                       pack_bf16(acc[4] * inv, acc[5] * inv), pack_bf16(acc[6] * inv, acc[7] * inv)});
  }
}

// Arg-max over the slabs' partial results; logits carry the row's norm factor from here on.
__device__ __forceinline__ void unembed_final_phase(const StackArgs &a, Top *red) {
  __amdgpu_buffer_rsrc_t ru = rsrc_of(a.un_part);
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255;
  for (int task = blockIdx.x; task * 2 < a.Bp; task += gridDim.x) {
    int b = task * 2 + sub;
    Top best{-INFINITY, 0x7fffffff, -INFINITY};
    if (b < a.Bp)
      for (int s = t; s < a.un.n_slabs; s += 256) {
        unsigned o = (unsigned)(((size_t)s * 64 + b) * sizeof(Top));
        Top c{ld32f(ru, o), (int)__builtin_amdgcn_raw_buffer_load_b32(ru, o + 4, 0, DEV), ld32f(ru, o + 8)};
        best = top_merge2(best, c);
      }
    red[threadIdx.x] = best;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if (t < o) red[threadIdx.x] = top_merge2(red[threadIdx.x], red[threadIdx.x + o]);
      __syncthreads();
    }
    if (t < 64 && b < a.Bp) {
      float s = 0.f;
      for (int c = t; c < a.ncg; c += 64) s += a.rsq[(size_t)b * a.ncg + c];
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (t == 0) {
        float rs = 1.0f / sqrtf(s * a.inv_d + a.eps);
        Top w = red[sub * 256];
        a.ids[b] = w.i1;
        if (a.top2) {
          a.top2[b * 2] = w.v1 * rs;
          a.top2[b * 2 + 1] = w.v2 * rs;
        }
      }
    }
    __syncthreads();
  }
}

// ---- the persistent kernel ------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(WG_THREADS) void stack_kernel(StackArgs a) {
  extern __shared__ f32x4 lds[];
  __shared__ int dead;  // set when a grid barrier timed out: the workgroup leaves the kernel
  const int L = *a.L_dev;
  if (L < 0 || L + a.Bp > a.max_len) {  // every workgroup takes the same exit: no barrier is left waiting
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.err = 1;
    return;
  }
  if (threadIdx.x == 0) dead = 0;
  __syncthreads();
  for (int p = a.p_begin; p < a.p_end; ++p) {
    const unsigned epoch = p > a.p_begin ? a.epoch0 + (unsigned)(p - a.p_begin) : 0u;
    int ph, layer = a.lb;
    if (a.mode == 1) {
      ph = PH_UPREP + p;
    } else if (p == 0) {
      ph = PH_PREP;
    } else {
      layer = a.lb + (p - 1) / PHASES_PER_LAYER;
      ph = PH_QKV + (p - 1) % PHASES_PER_LAYER;
    }
    uint16_t *Kc = a.K + (size_t)layer * a.layer_elems, *Vc = a.V + (size_t)layer * a.layer_elems;
    // write-once buffers of this layer: fragments of the attn-norm and mlp-norm inputs with
    // their statistics, the attention output, the SwiGLU output
    uint16_t *xa0 = a.xa + (size_t)(2 * layer) * a.xa_stride, *xa1 = xa0 + a.xa_stride;
    float *rsq0 = a.rsq + (size_t)(2 * layer) * a.rsq_stride, *rsq1 = rsq0 + a.rsq_stride;
    uint16_t *attn_l = a.attn_a + (size_t)layer * a.attn_stride, *act_l = a.act_a + (size_t)layer * a.act_stride;
    const bool is_gemm = ph == PH_QKV || ph == PH_O || ph == PH_GU || ph == PH_DOWN || ph == PH_UGEMM;
    trace_mark(a, 3 * (p - a.p_begin));
    if (epoch && !is_gemm && !grid_barrier(a, epoch, &dead)) return;
    if (!is_gemm) trace_mark(a, 3 * (p - a.p_begin) + 1);
    GemmIo io{};
    switch (ph) {
      case PH_PREP:
        prep_phase(a, a.layers[layer].g_attn, xa0, rsq0);
        rope_table_phase(a);
        break;
      case PH_QKV:
        io.W = a.layers[layer].wqkv; io.A = xa0; io.mode = MODE_QKV; io.rsq_in = rsq0; io.Kc = Kc; io.Vc = Vc; io.L = L;
        if (!gemm_dispatch<MT>(a, a.qkv, io, epoch, lds, &dead)) return;
        break;
      case PH_ATT:
        if (a.dh == 128) attention_phase<128>(a, Kc, Vc, L);
        else attention_phase<64>(a, Kc, Vc, L);
        break;
      case PH_COMB:
        if (a.dh == 128) combine_phase<128>(a, attn_l);
        else combine_phase<64>(a, attn_l);
        break;
      case PH_O:
        io.W = a.layers[layer].wo; io.A = attn_l; io.mode = MODE_RESID; io.gain = a.layers[layer].g_mlp; io.xa_out = xa1; io.rsq_out = rsq1;
        if (!gemm_dispatch<MT>(a, a.o, io, epoch, lds, &dead)) return;
        break;
      case PH_GU:
        io.W = a.layers[layer].wgu; io.A = xa1; io.mode = MODE_GATEUP; io.rsq_in = rsq1; io.act_a = act_l;
        if (!gemm_dispatch<MT>(a, a.gu, io, epoch, lds, &dead)) return;
        break;
      case PH_DOWN:
        // the fragments feed the next layer's QKV GEMM; the last layer of the call needs none
        io.W = a.layers[layer].wdown; io.A = act_l; io.mode = MODE_RESID;
        io.gain = layer + 1 < a.le ? a.layers[layer + 1].g_attn : nullptr;
        io.xa_out = xa0 + 2 * a.xa_stride; io.rsq_out = rsq0 + 2 * a.rsq_stride;
        if (!gemm_dispatch<MT>(a, a.down, io, epoch, lds, &dead)) return;
        break;
      case PH_UPREP:
        prep_phase(a, a.g_final, a.xa, a.rsq);
        break;
      case PH_UGEMM:
        io.W = a.un_w; io.A = a.xa; io.mode = MODE_UNEMBED; io.un_part = a.un_part;
        if (!gemm_dispatch<MT>(a, a.un, io, epoch, lds, &dead)) return;
        break;
      case PH_UFINAL:
        unembed_final_phase(a, (Top *)lds);
        break;
    }
    trace_mark(a, 3 * (p - a.p_begin) + 2);
  }
}

// ---- weight packing (once, at model set-up) -----------------------------------------------------
// Packed column pc of the destination -> (source matrix, source column).
//   kind 0: one source [K, N];
//   kind 1: q | k | v heads; each 16-column slab holds channels 8j..8j+7 and dh/2+8j.. of one
//           head, i.e. both members of eight RoPE pairs (slabs are one tile wide);
//   kind 2: per slab, 8T gate channels followed by the same 8T channels of up.
struct PackSrc {
  const uint16_t *s0, *s1, *s2;
  int n0, n1, n2;
  int kind, T, F, dh;
};
__device__ __forceinline__ const uint16_t *pack_col(const PackSrc &p, int pc, int &ld) {
  if (p.kind == 0) {
    ld = p.n0;
    return p.s0 + pc;
  }
  if (p.kind == 1) {
    int slab = pc >> 4, w = pc & 15, spj = p.dh >> 4;
    int hs = slab / spj, j = slab - hs * spj;
    pc = hs * p.dh + (w < 8 ? 8 * j + w : (p.dh >> 1) + 8 * j + (w - 8));
    if (pc < p.n0) { ld = p.n0; return p.s0 + pc; }
    pc -= p.n0;
    if (pc < p.n1) { ld = p.n1; return p.s1 + pc; }
    ld = p.n2;
    return p.s2 + (pc - p.n1);
  }
  int slab = pc / (16 * p.T), w = pc - slab * 16 * p.T, Fg = 8 * p.T;
  ld = p.F;
  return (w < Fg ? p.s0 : p.s1) + slab * Fg + (w < Fg ? w : w - Fg);
}

__global__ void pack_weights_kernel(PackSrc p, int KT, int T, int n_slabs, uint16_t *dst) {
  size_t total = (size_t)n_slabs * KT * T * 64;
  for (size_t fi = (size_t)blockIdx.x * blockDim.x + threadIdx.x; fi < total; fi += (size_t)gridDim.x * blockDim.x) {
    int lane = fi & 63;
    size_t r = fi >> 6;
    int t = r % T;
    r /= T;
    int kt = r % KT;
    int slab = r / KT;
    int pc = (slab * T + t) * 16 + (lane & 15);
    int k0 = kt * 32 + 8 * (lane >> 4);
    int ld;
    const uint16_t *src = pack_col(p, pc, ld);
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(size_t)(k0 + i) * ld];
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16);
    o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16);
    o.w = v[6] | ((uint32_t)v[7] << 16);
    *reinterpret_cast<uint4 *>(dst + fi * 8) = o;
  }
}

__global__ void zero_u32_kernel(unsigned *p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---- host side --------------------------------------------------------------------------------------
struct GemmPlan {
  int N = 0, K = 0, KT = 0, T = 1, n_slabs = 0;
  size_t bytes = 0;
};

struct MfmaLayer {
  uint16_t *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wdown = nullptr;
};

struct MfmaModel {
  int n_wgs = 256;
  bool persistent = true;
  GemmPlan p_qkv, p_o, p_gu, p_down, p_un;
  std::vector<MfmaLayer> layers;
  std::vector<LayerPtrs> host_ptrs;
  LayerPtrs *dev_ptrs = nullptr;
  bool ptrs_dirty = true;
  uint16_t *un = nullptr;
  uint16_t *xa = nullptr, *attn_a = nullptr, *act_a = nullptr, *qf = nullptr;  // per layer (and use)
  uint16_t *xa_u = nullptr;                                                    // unembedding input
  float *rsq = nullptr, *rsq_u = nullptr, *o_part = nullptr, *ml_part = nullptr;
  Top *un_part = nullptr;
  unsigned *sync = nullptr;
  int32_t *zero_len = nullptr;  // {0, scratch error word}: the unembedding has no cache to overflow
  unsigned epoch = 0;
  int max_ns = 32;
  unsigned long long *trace = nullptr;  // LA_TRACE=1: per-phase timestamps, printed after each launch
};

static int env_int(const char *name, int dflt) {
  const char *v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

// Tiles per slab for the gate/up and unembedding GEMMs: the slab count should fill the CUs in
// whole rounds, and wide slabs are preferred (fewer operand re-reads per weight byte).
static GemmPlan make_plan(int N, int K, int n_wgs, bool gateup, int F, const char *env) {
  GemmPlan p;
  p.N = N; p.K = K; p.KT = K / 32;
  int tiles = N / 16;
  double best = 1e300;
  for (int T = MAX_T; T >= 1; --T) {
    if (gateup ? (F % (8 * T) != 0) : (tiles % T != 0)) continue;
    int rounds = ceil_div(tiles / T, n_wgs);
    double cost = (double)rounds * (T + 2.0);  // per k-tile: T weight fragments + ~2 operand fragments
    if (cost < best) { best = cost; p.T = T; }
  }
  int forced = env_int(env, 0);
  if (forced >= 1 && forced <= MAX_T && (gateup ? (F % (8 * forced) == 0) : (tiles % forced == 0))) p.T = forced;
  p.n_slabs = tiles / p.T;
  p.bytes = (size_t)N * K * 2;
  return p;
}

static GemmPlan slab1_plan(int N, int K) {  // one 16-column tile per slab: the epilogue-fused GEMMs
  GemmPlan p;
  p.N = N; p.K = K; p.KT = K / 32; p.T = 1; p.n_slabs = N / 16;
  p.bytes = (size_t)N * K * 2;
  return p;
}

int mfma_supported(const la_model_desc *d) {
  int qd = d->n_q_heads * d->head_dim, nqkv = (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim;
  if (d->d_model % 128 || qd % 32 || d->d_ffn % 32 || nqkv % 16 || d->vocab % 16) return 0;
  if (d->head_dim != 64 && d->head_dim != 128) return 0;
  if (d->n_q_heads / d->n_kv_heads > 8) return 0;
  // packed matrices and scratch are addressed through 32-bit buffer offsets
  size_t lim = (size_t)1 << 31;
  if ((size_t)d->d_model * 2 * d->d_ffn * 2 >= lim || (size_t)d->d_model * d->vocab * 2 >= lim) return 0;
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
  for (auto &l : f->layers) {
    void *ps[] = {l.wqkv, l.wo, l.wgu, l.wdown};
    for (void *p : ps)
      if (p) (void)hipFree(p);
  }
  void *ps[] = {f->un, f->xa, f->attn_a, f->act_a, f->qf, f->xa_u, f->rsq_u, f->rsq, f->o_part, f->ml_part, f->un_part,
                f->sync, f->dev_ptrs, f->zero_len, f->trace};
  for (void *p : ps)
    if (p) (void)hipFree(p);
  delete f;
  m->mf = nullptr;
}

int mfma_create(la_model *m) {
  const la_model_desc &d = m->d;
  MfmaModel *f = new (std::nothrow) MfmaModel();
  LA_REQUIRE(f != nullptr, LA_ENOMEM, "out of host memory");
  m->mf = f;
  hipDeviceProp_t prop;
  LA_HIP(hipGetDeviceProperties(&prop, m->device));
  int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  f->n_wgs = std::min(env_int("LA_WGS", cus), cus);  // one resident workgroup per CU: the barrier needs co-residency
  f->persistent = env_int("LA_PERSISTENT", 1) != 0;
  int qd = m->qdim(), nqkv = m->nqkv(), g = d.n_q_heads / d.n_kv_heads;
  f->p_qkv = slab1_plan(nqkv, d.d_model);
  f->p_o = slab1_plan(d.d_model, qd);
  f->p_gu = make_plan(2 * d.d_ffn, d.d_model, f->n_wgs, true, d.d_ffn, "LA_T_GU");
  f->p_down = slab1_plan(d.d_model, d.d_ffn);
  f->p_un = make_plan(d.vocab, d.d_model, f->n_wgs, false, 0, "LA_T_UN");
  f->layers.resize(d.n_layers);
  f->host_ptrs.resize(d.n_layers);
  size_t R = LA_MAX_ROWS, nl = d.n_layers;
  f->max_ns = std::max(1, std::min(64, f->n_wgs / d.n_kv_heads));
  size_t QR = (size_t)g * MAX_MT * 16;
  int n_sync = SYNC_STRIDE * 66;
  size_t ncg = d.d_model / 16;
  bool ok = true;
  ok = ok && (f->xa = (uint16_t *)dalloc(2 * nl * R * d.d_model * 2));
  ok = ok && (f->attn_a = (uint16_t *)dalloc(nl * R * qd * 2));
  ok = ok && (f->act_a = (uint16_t *)dalloc(nl * R * (size_t)d.d_ffn * 2));
  ok = ok && (f->xa_u = (uint16_t *)dalloc(R * d.d_model * 2));
  ok = ok && (f->qf = (uint16_t *)dalloc((size_t)d.n_kv_heads * QR * d.head_dim * 2));
  ok = ok && (f->rsq = (float *)dalloc(2 * nl * R * ncg * 4));
  ok = ok && (f->rsq_u = (float *)dalloc(R * ncg * 4));
  ok = ok && (f->o_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * d.head_dim * 4));
  ok = ok && (f->ml_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * 2 * 4));
  ok = ok && (f->sync = (unsigned *)dalloc((size_t)n_sync * 4));
  ok = ok && (f->dev_ptrs = (LayerPtrs *)dalloc((size_t)d.n_layers * sizeof(LayerPtrs)));
  ok = ok && (f->zero_len = (int32_t *)dalloc(8));
  LA_REQUIRE(ok, LA_ENOMEM, "device allocation failed in the MFMA path");
  // pad rows of the operand buffers are read by the MFMAs: keep them finite
  LA_HIP(hipMemset(f->xa, 0, 2 * nl * R * d.d_model * 2));
  LA_HIP(hipMemset(f->attn_a, 0, nl * R * qd * 2));
  LA_HIP(hipMemset(f->act_a, 0, nl * R * (size_t)d.d_ffn * 2));
  LA_HIP(hipMemset(f->xa_u, 0, R * d.d_model * 2));
  LA_HIP(hipMemset(f->qf, 0, (size_t)d.n_kv_heads * QR * d.head_dim * 2));
  LA_HIP(hipMemset(f->sync, 0, (size_t)n_sync * 4));
  LA_HIP(hipMemset(f->zero_len, 0, 8));
  if (env_int("LA_TRACE", 0)) {
    size_t np = 2 + PHASES_PER_LAYER * d.n_layers;
    f->trace = (unsigned long long *)dalloc((3 * np + 2 * np * f->n_wgs) * 8);
    LA_REQUIRE(f->trace != nullptr, LA_ENOMEM, "device allocation failed");
  }
  return LA_OK;
}

static int pack(const PackSrc &src, const GemmPlan &p, uint16_t **dst, hipStream_t s) {
  if (!*dst) *dst = (uint16_t *)dalloc(p.bytes);
  LA_REQUIRE(*dst != nullptr, LA_ENOMEM, "device allocation of %zu bytes failed", p.bytes);
  ProfScope ps("pack_weights", s);
  pack_weights_kernel<<<2048, 256, 0, s>>>(src, p.KT, p.T, p.n_slabs, *dst);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int mfma_set_layer(la_model *m, int layer, const la_layer_weights *w, hipStream_t s) {
  MfmaModel *f = m->mf;
  MfmaLayer &l = f->layers[layer];
  int qd = m->qdim(), kvd = m->kvdim();
  const la_model_desc &d = m->d;
  int rc;
  PackSrc q{(const uint16_t *)w->wq, (const uint16_t *)w->wk, (const uint16_t *)w->wv, qd, kvd, kvd, 1, f->p_qkv.T, 0, d.head_dim};
  if ((rc = pack(q, f->p_qkv, &l.wqkv, s))) return rc;
  PackSrc o{(const uint16_t *)w->wo, nullptr, nullptr, d.d_model, 0, 0, 0, f->p_o.T, 0, 0};
  if ((rc = pack(o, f->p_o, &l.wo, s))) return rc;
  PackSrc gu{(const uint16_t *)w->wgate, (const uint16_t *)w->wup, nullptr, d.d_ffn, d.d_ffn, 0, 2, f->p_gu.T, d.d_ffn, 0};
  if ((rc = pack(gu, f->p_gu, &l.wgu, s))) return rc;
  PackSrc dn{(const uint16_t *)w->wdown, nullptr, nullptr, d.d_model, 0, 0, 0, f->p_down.T, 0, 0};
  if ((rc = pack(dn, f->p_down, &l.wdown, s))) return rc;
  f->host_ptrs[layer] = LayerPtrs{l.wqkv, l.wo, l.wgu, l.wdown, m->layers[layer].g_attn, m->layers[layer].g_mlp};
  f->ptrs_dirty = true;
  return LA_OK;
}

int mfma_set_head(la_model *m, const void *unembed, hipStream_t s) {
  MfmaModel *f = m->mf;
  PackSrc u{(const uint16_t *)unembed, nullptr, nullptr, m->d.vocab, 0, 0, 0, f->p_un.T, 0, 0};
  int rc = pack(u, f->p_un, &f->un, s);
  if (rc) return rc;
  if (!f->un_part) f->un_part = (Top *)dalloc((size_t)f->p_un.n_slabs * 64 * sizeof(Top));
  LA_REQUIRE(f->un_part != nullptr, LA_ENOMEM, "device allocation failed");
  return LA_OK;
}

static GemmDev dev_plan(const GemmPlan &p) { return GemmDev{p.KT, p.T, p.n_slabs, p.N}; }

static size_t stack_lds_bytes(int MT) {
  // GEMM: tree buffers 3 MT T KB (the row-major tile reuses them) + row factors; the other
  // phases need less (8 x 512 B staging, 512 arg-max records)
  size_t gemm = (size_t)3 * MT * MAX_T * 64 * sizeof(f32x4) + 64 * sizeof(float) + 1024;
  size_t tile = (size_t)16 * MT * (16 * MAX_T + 4) * sizeof(float);
  return std::max(std::max(gemm, tile), (size_t)WG_THREADS * sizeof(Top));
}

template <int MT>
static int launch_stack_mt(const char *name, const StackArgs &a, int n_wgs, hipStream_t s) {
  size_t lds = stack_lds_bytes(MT);
  static bool attr_set = false;
  if (!attr_set) {
    LA_HIP(hipFuncSetAttribute((const void *)stack_kernel<MT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  ProfScope ps(name, s);
  stack_kernel<MT><<<n_wgs, WG_THREADS, lds, s>>>(a);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

static int launch_stack(const char *name, MfmaModel *f, StackArgs a, hipStream_t s) {
  // persistent: one launch walks all phases with grid barriers in between;
  // otherwise (LA_PERSISTENT=0) one launch per phase, ordered by the stream
  int p0 = a.p_begin, p1 = a.p_end;
  int step = f->persistent ? (p1 - p0) : 1;
  for (int p = p0; p < p1; p += step) {
    a.p_begin = p;
    a.p_end = std::min(p1, p + step);
    int n_bar = a.p_end - a.p_begin - 1;
    if (f->epoch > (1u << 26)) {  // keep the monotonic counters far from wrapping
      zero_u32_kernel<<<ceil_div(SYNC_STRIDE * 66, 256), 256, 0, s>>>(f->sync, SYNC_STRIDE * 66);
      f->epoch = 0;
    }
    a.epoch0 = f->epoch;
    f->epoch += (unsigned)n_bar;
    a.n_groups = (unsigned)ceil_div(f->n_wgs, SYNC_GROUP);
    int rc;
    switch (a.MT) {
      case 1: rc = launch_stack_mt<1>(name, a, f->n_wgs, s); break;
      case 2: rc = launch_stack_mt<2>(name, a, f->n_wgs, s); break;
      case 3: rc = launch_stack_mt<3>(name, a, f->n_wgs, s); break;
      default: rc = launch_stack_mt<4>(name, a, f->n_wgs, s); break;
    }
    if (rc) return rc;
    if (f->trace && f->persistent) {  // debugging aid: per-phase timeline of workgroup 0 (100 MHz clock)
      int np = a.p_end - a.p_begin;
      std::vector<unsigned long long> h(3 * np);
      LA_HIP(hipStreamSynchronize(s));
      LA_HIP(hipMemcpy(h.data(), f->trace, h.size() * 8, hipMemcpyDeviceToHost));
      fprintf(stderr, "[la trace] %s: %d phases, total %.1f us\n", name, np, (h[3 * np - 1] - h[0]) * 0.01);
      std::vector<unsigned long long> w((size_t)2 * np * f->n_wgs);
      LA_HIP(hipMemcpy(w.data(), f->trace + a.trace_wg_off, w.size() * 8, hipMemcpyDeviceToHost));
      for (int q = 0; q < np && q < 1 + 2 * PHASES_PER_LAYER; ++q) {
        fprintf(stderr, "[la trace]   phase %2d: barrier %6.2f us  work %7.2f us", q, (h[3 * q + 1] - h[3 * q]) * 0.01,
                (h[3 * q + 2] - h[3 * q + 1]) * 0.01);
        if (q > 0) {  // barrier q: spread of arrivals, and release latency after the last arrival
          unsigned long long a0 = ~0ull, a1 = 0, r0 = ~0ull, r1 = 0;
          for (int g = 0; g < f->n_wgs; ++g) {
            unsigned long long ta = w[((size_t)q * f->n_wgs + g) * 2], trl = w[((size_t)q * f->n_wgs + g) * 2 + 1];
            a0 = std::min(a0, ta); a1 = std::max(a1, ta); r0 = std::min(r0, trl); r1 = std::max(r1, trl);
          }
          fprintf(stderr, "   | arrivals spread %6.2f us, first release %5.2f us after last arrival, releases spread %5.2f us",
                  (a1 - a0) * 0.01, ((double)r0 - (double)a1) * 0.01, (r1 - r0) * 0.01);
        }
        fprintf(stderr, "\n");
      }
    }
  }
  return LA_OK;
}

static int sync_layer_ptrs(MfmaModel *f, hipStream_t s) {
  if (!f->ptrs_dirty) return LA_OK;
  LA_HIP(hipMemcpyAsync(f->dev_ptrs, f->host_ptrs.data(), f->host_ptrs.size() * sizeof(LayerPtrs), hipMemcpyHostToDevice, s));
  LA_HIP(hipStreamSynchronize(s));  // host_ptrs is pageable memory
  f->ptrs_dirty = false;
  return LA_OK;
}

static StackArgs base_stack_args(la_model *m, int Bp) {
  MfmaModel *f = m->mf;
  const la_model_desc &d = m->d;
  StackArgs a{};
  a.layers = f->dev_ptrs;
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
  a.o_part = f->o_part;
  a.ml_part = f->ml_part;
  a.cs = m->rope_cs;
  a.sync = f->sync;
  a.trace = f->trace;
  a.trace_wg_off = (size_t)3 * (2 + PHASES_PER_LAYER * d.n_layers);
  return a;
}

int mfma_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos, const uint64_t *vis,
                 la_kv *kv, hipStream_t s) {
  MfmaModel *f = m->mf;
  if (lb == le) return LA_OK;
  int rc = sync_layer_ptrs(f, s);
  if (rc) return rc;
  StackArgs a = base_stack_args(m, Bp);
  a.mode = 0;
  a.lb = lb;
  a.le = le;
  a.p_begin = 0;
  a.p_end = 1 + PHASES_PER_LAYER * (le - lb);
  a.qkv = dev_plan(f->p_qkv);
  a.o = dev_plan(f->p_o);
  a.gu = dev_plan(f->p_gu);
  a.down = dev_plan(f->p_down);
  // key splits: a few blocks of 32 keys per workgroup, within the scratch sized at set-up
  int nkb = ceil_div(kv->L_bound + Bp, 32);
  a.ns = std::max(1, std::min(f->max_ns, ceil_div(nkb, env_int("LA_ATTN_KB", 2))));
  a.x = hidden;
  a.pos = pos;
  a.vis = vis;
  a.K = (uint16_t *)kv->K;
  a.V = (uint16_t *)kv->V;
  a.layer_elems = kv->layer_elems();
  a.L_dev = kv->L_dev;
  a.max_len = kv->max_len;
  a.err = kv->err_dev;
  return launch_stack("layer_stack", f, a, s);
}

int mfma_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, hipStream_t s) {
  MfmaModel *f = m->mf;
  LA_REQUIRE(f->un != nullptr, LA_EINVAL, "model was created without an unembedding matrix");
  StackArgs a = base_stack_args(m, Bp);
  a.mode = 1;
  a.p_begin = 0;
  a.p_end = 3;
  a.un = dev_plan(f->p_un);
  a.xa = f->xa_u;
  a.rsq = f->rsq_u;
  a.x = const_cast<float *>(hidden);
  a.un_w = f->un;
  a.g_final = m->g_final;
  a.un_part = f->un_part;
  a.ids = ids;
  a.top2 = top2;
  a.L_dev = f->zero_len;
  a.max_len = LA_MAX_ROWS;
  a.err = f->zero_len + 1;
  return launch_stack("unembed_argmax", f, a, s);
}

}  // namespace la
