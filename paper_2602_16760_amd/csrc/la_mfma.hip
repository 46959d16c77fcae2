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
// GEMM tasks.  A task is (slab, k-range).  Seven waves split the k-range, accumulate in
// registers, and are summed through LDS in a fixed tree; the eighth wave runs the grid barrier
// so that its polling loads never queue behind prefetched weights.  Tasks whose k-range is a
// fraction of K write fp32 partials which the next small phase adds in a fixed order together
// with the residual stream; it also emits the RMSNorm statistics and the operand fragments of
// the next GEMM.  RMSNorm is applied as ((x * g) W) * rsqrt(mean(x^2) + eps), the row factor
// after the contraction.  All reductions have a fixed order: results are run-to-run identical.
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
constexpr int MAX_S = 8;           // k-splits across workgroups
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
  PH_QKV,       // [q|k|v] partials
  PH_QKVF,      // reduce partials, norm factor, RoPE, q fragments, K/V rows into the cache
  PH_ATT,       // masked-block attention per (kv head, key split)
  PH_COMB,      // merge key splits -> operand fragments of the O GEMM
  PH_O,         // attention output projection partials
  PH_FO,        // x += partials; statistics; fragments for gate/up
  PH_GU,        // gate/up GEMM + SwiGLU -> fragments for down
  PH_DOWN,      // down projection partials
  PH_FD,        // x += partials; statistics; fragments for the next layer's QKV
  PH_UPREP,     // final norm operand fragments
  PH_UGEMM,     // unembedding with per-slab arg-max
  PH_UFINAL     // arg-max over slabs
};
constexpr int PHASES_PER_LAYER = 9;

enum GemmMode { MODE_PARTIAL = 0, MODE_GATEUP = 1, MODE_UNEMBED = 2 };

struct GemmDev {
  int KT, T, n_slabs, S, N;
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
  uint16_t *xa, *attn_a, *act_a, *qf;
  float *part, *rsq, *o_part, *ml_part, *cs;
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
};

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
  static constexpr int value = raw < 2 ? 2 : (raw > 6 ? 6 : raw);
};

struct GemmIo {
  const uint16_t *W;
  const uint16_t *A;
  int mode;
  float *part;      // MODE_PARTIAL
  uint16_t *act_a;  // MODE_GATEUP
  Top *un_part;     // MODE_UNEMBED
};

// One GEMM phase of this workgroup.  `epoch` != 0: run the grid barrier first, with the
// weights of the first task already requested before the wait.
template <int MT, int T>
__device__ __forceinline__ bool gemm_phase(const StackArgs &a, const GemmDev &g, const GemmIo &io, unsigned epoch,
                                           f32x4 *lds, int *dead) {
  constexpr int D = Depth<MT, T>::value;
  constexpr int LDT = 16 * T + 4;  // padded row length of the result tile in LDS
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int n_tasks = g.n_slabs * g.S;
  __amdgpu_buffer_rsrc_t rw = rsrc_of(io.W), ra = rsrc_of(io.A);
  float *tile = (float *)lds;                         // [16 MT][LDT] after the tree
  float *rs_lds = (float *)(lds + 3 * MT * T * 64);   // [64] row factors (MODE_GATEUP)
  const unsigned voff = lane * 16;

  if (epoch) wg_stores_done();
  bool first = true;
  for (int task = blockIdx.x; task < n_tasks || first; task += gridDim.x) {
    const bool live = task < n_tasks;
    const int slab = live ? task / g.S : 0, ks = live ? task - slab * g.S : 0;
    const int kt0 = (int)((long long)g.KT * ks / g.S), kt1 = (int)((long long)g.KT * (ks + 1) / g.S);
    const int nk = kt1 - kt0;
    const int cw = wave < NCW ? wave : 0;
    const int wk0 = kt0 + nk * cw / NCW, wk1 = kt0 + nk * (cw + 1) / NCW;
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
        rA[slot][mt] = __builtin_amdgcn_raw_buffer_load_b128(ra, vo, a_base + (unsigned)(i * MT + mt) * 1024, DEV);
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
    first = false;
    if (!live) break;
#pragma unroll
    for (int s = 0; s < D; ++s) {
      load_a(s, s);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (io.mode == MODE_GATEUP && wave == NCW) {
      // row factors rsqrt(mean(x^2) + eps) from the per-column-group partial sums
      __amdgpu_buffer_rsrc_t rq = rsrc_of(a.rsq);
      for (int r = 0; r < a.Bp; ++r) {
        float s = 0.f;
        for (int c = lane; c < a.ncg; c += 64) s += ld32f(rq, (unsigned)(r * a.ncg + c) * 4);
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (lane == 0) rs_lds[r] = 1.0f / sqrtf(s * a.inv_d + a.eps);
      }
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

    if (io.mode == MODE_PARTIAL) {
      __amdgpu_buffer_rsrc_t rp = rsrc_of(io.part);
      const int chunks = a.Bp * 4 * T;  // 16-byte pieces of the tile's live rows
      for (int c = threadIdx.x; c < chunks; c += WG_THREADS) {
        int row = c / (4 * T), c4 = c - row * 4 * T;
        f32x4 v = *reinterpret_cast<const f32x4 *>(tile + row * LDT + 4 * c4);
        st128(rp, (unsigned)((((size_t)ks * 64 + row) * g.N + (size_t)slab * 16 * T + 4 * c4) * 4),
              __builtin_bit_cast(u32x4, v));
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

// ---- residual update, norm statistics, operand fragments -------------------------------------
// Task = two groups of 32 columns (one per half of the workgroup): x += sum_s part[s] in a
// fixed order; partial sum of squares per row over the group; bf16(x * gain) as fragments.
__device__ __forceinline__ void finish_phase(const StackArgs &a, int S, int N, const float *gain, bool update_x) {
  __amdgpu_buffer_rsrc_t rp = rsrc_of(a.part), rq = rsrc_of(a.rsq), rx = rsrc_of(a.xa);
  const int sub = threadIdx.x >> 8, r = (threadIdx.x & 255) >> 2, oct = threadIdx.x & 3;
  for (int task = blockIdx.x; task * 2 < a.ncg; task += gridDim.x) {
    int cg = task * 2 + sub;
    if (cg >= a.ncg || r >= a.Bp) continue;
    int c0 = cg * 32 + oct * 8;
    float v[8];
    const f32x4 *xp = reinterpret_cast<const f32x4 *>(a.x + (size_t)r * a.d + c0);
    f32x4 x0 = xp[0], x1 = xp[1];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] = x0[i];
      v[4 + i] = x1[i];
    }
    for (int s = 0; s < S; ++s) {
      unsigned o = (unsigned)((((size_t)s * 64 + r) * N + c0) * 4);
      f32x4 p0 = __builtin_bit_cast(f32x4, ld128(rp, o)), p1 = __builtin_bit_cast(f32x4, ld128(rp, o + 16));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] += p0[i];
        v[4 + i] += p1[i];
      }
    }
    if (update_x) {
      f32x4 *xo = reinterpret_cast<f32x4 *>(a.x + (size_t)r * a.d + c0);
      xo[0] = f32x4{v[0], v[1], v[2], v[3]};
      xo[1] = f32x4{v[4], v[5], v[6], v[7]};
    }
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) sq += v[i] * v[i];
    sq += __shfl_xor(sq, 1, 64);
    sq += __shfl_xor(sq, 2, 64);
    if (oct == 0) st32f(rq, (unsigned)(r * a.ncg + cg) * 4, sq);
    if (gain) {
      u32x4 w;
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = pack_bf16(v[2 * i] * gain[c0 + 2 * i], v[2 * i + 1] * gain[c0 + 2 * i + 1]);
      st128(rx, (unsigned)((((size_t)cg * a.MT + (r >> 4)) * 64 + (r & 15) + 16 * oct) * 16), w);
    }
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

// ---- QKV epilogue: one wave per (row, head slot) ------------------------------------------------
// q fragments: [kv head][q-row tile][dh k-tile][lane][8], q-row = j * 16 MT + b for the j-th
// query head of the group, pre-multiplied by 1/sqrt(dh).  Keys are cached after rotation.
__device__ __forceinline__ void qkvf_phase(const StackArgs &a, int S, uint16_t *Kc, uint16_t *Vc, int L,
                                           uint16_t *stage_all) {
  __amdgpu_buffer_rsrc_t rp = rsrc_of(a.part), rq = rsrc_of(a.rsq), rc = rsrc_of(a.cs), rqf = rsrc_of(a.qf),
                         rk = rsrc_of(Kc), rv = rsrc_of(Vc);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  uint16_t *stage = stage_all + wave * 256;
  const int nh = a.Hq + 2 * a.Hkv, n_units = a.Bp * nh, half = a.dh >> 1, g = a.Hq / a.Hkv;
  const int N = a.qkv.N;
  for (int u = blockIdx.x * 8 + wave; u < n_units; u += gridDim.x * 8) {
    int b = u / nh, hs = u - b * nh;
    float s = 0.f;
    for (int c = lane; c < a.ncg; c += 64) s += ld32f(rq, (unsigned)(b * a.ncg + c) * 4);
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    float rs = 1.0f / sqrtf(s * a.inv_d + a.eps);
    int col0 = hs * a.dh;
    auto val = [&](int c) {
      float t = 0.f;
      for (int k = 0; k < S; ++k) t += ld32f(rp, (unsigned)((((size_t)k * 64 + b) * N + col0 + c) * 4));
      return t * rs;
    };
    if (hs < a.Hq + a.Hkv) {
      float qscale = hs < a.Hq ? 1.0f / sqrtf((float)a.dh) : 1.0f;
      if (lane < half) {
        float c = ld32f(rc, (unsigned)(b * half + lane) * 8), sn = ld32f(rc, (unsigned)(b * half + lane) * 8 + 4);
        float x0 = val(lane), x1 = val(lane + half);
        stage[lane] = float_to_bf16((x0 * c - x1 * sn) * qscale);
        stage[lane + half] = float_to_bf16((x1 * c + x0 * sn) * qscale);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (lane < a.dh / 8) {  // one 16-byte piece of 8 channels per lane
        u32x4 w = *reinterpret_cast<const u32x4 *>(stage + 8 * lane);
        if (hs < a.Hq) {
          int kvh = hs / g, j = hs - kvh * g;
          int rt = j * a.MT + (b >> 4);
          unsigned o = (unsigned)(((((size_t)kvh * (g * a.MT) + rt) * (a.dh >> 5) + (lane >> 2)) * 64 + (b & 15) + 16 * (lane & 3)) * 16);
          st128(rqf, o, w);
        } else {
          st128(rk, (unsigned)((((size_t)(L + b) * a.Hkv + (hs - a.Hq)) * a.dh + 8 * lane) * 2), w);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
      int h = hs - a.Hq - a.Hkv;
      for (int c = lane; c < a.dh; c += 64)
        st16(rv, (unsigned)(v_index(true, L + b, h, c, a.Hkv, a.dh) * 2), float_to_bf16(val(c)));
    }
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
      for (int kb = kb0; kb < kb1; ++kb) {
        const unsigned k_off = (unsigned)((((size_t)(kb * 32 + c16) * a.Hkv + kvh) * DH + 8 * q4) * 2);
        const unsigned v_off = (unsigned)(((((size_t)kb * a.Hkv + kvh) * DH + c16) * 32 + 8 * q4) * 2);
        u32x4 ka[KT], kbv[KT], vt[DT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          ka[kt] = ld128(rk, k_off + kt * 64);
          kbv[kt] = ld128(rk, k_off + (unsigned)(16 * a.Hkv * DH * 2) + kt * 64);
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vt[dt] = ld128(rv, v_off + dt * 16 * 32 * 2);
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
      // o[dt][i] = O^T[channel 16 dt + 4 q4 + i][q-row rt*16 + c16]
      size_t base = ((size_t)kvh * a.ns + split) * DH * QR;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          st32f(ro, (unsigned)((base + (size_t)(16 * dt + 4 * q4 + i) * QR + rt * 16 + c16) * 4), o[dt][i]);
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
__device__ __forceinline__ void combine_phase(const StackArgs &a) {
  __amdgpu_buffer_rsrc_t ro = rsrc_of(a.o_part), rm = rsrc_of(a.ml_part), ra = rsrc_of(a.attn_a);
  const int g = a.Hq / a.Hkv, n_rt = g * a.MT, QR = n_rt * 16, n_units = a.Hkv * n_rt;
  const int sub = threadIdx.x >> 8, t = threadIdx.x & 255, rr = t & 15, oct = t >> 4;
  for (int task = blockIdx.x; task * 2 < n_units; task += gridDim.x) {
    int u = task * 2 + sub;
    if (u >= n_units || oct >= DH / 8) continue;
    int kvh = u / n_rt, rt = u - kvh * n_rt;
    int r = rt * 16 + rr, b = (rt % a.MT) * 16 + rr, j = rt / a.MT;
    if (b >= a.Bp) continue;
    float M = -1e30f;
    for (int s = 0; s < a.ns; ++s) M = fmaxf(M, ld32f(rm, (unsigned)(((((size_t)kvh * a.ns + s) * QR + r) * 2) * 4)));
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, lsum = 0.f;
    for (int s = 0; s < a.ns; ++s) {
      unsigned mo = (unsigned)(((((size_t)kvh * a.ns + s) * QR + r) * 2) * 4);
      float w = __expf(ld32f(rm, mo) - M);
      lsum += w * ld32f(rm, mo + 4);
      size_t ob = ((size_t)kvh * a.ns + s) * DH * QR + (size_t)(oct * 8) * QR + r;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += w * ld32f(ro, (unsigned)((ob + (size_t)i * QR) * 4));
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
  __amdgpu_buffer_rsrc_t ru = rsrc_of(a.un_part), rq = rsrc_of(a.rsq);
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
      for (int c = t; c < a.ncg; c += 64) s += ld32f(rq, (unsigned)(b * a.ncg + c) * 4);
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
    const bool is_gemm = ph == PH_QKV || ph == PH_O || ph == PH_GU || ph == PH_DOWN || ph == PH_UGEMM;
    if (epoch && !is_gemm && !grid_barrier(a, epoch, &dead)) return;
    switch (ph) {
      case PH_PREP:
        finish_phase(a, 0, 0, a.layers[layer].g_attn, false);
        rope_table_phase(a);
        break;
      case PH_QKV:
        if (!gemm_dispatch<MT>(a, a.qkv, GemmIo{a.layers[layer].wqkv, a.xa, MODE_PARTIAL, a.part, nullptr, nullptr}, epoch, lds, &dead)) return;
        break;
      case PH_QKVF:
        qkvf_phase(a, a.qkv.S, Kc, Vc, L, (uint16_t *)lds);
        break;
      case PH_ATT:
        if (a.dh == 128) attention_phase<128>(a, Kc, Vc, L);
        else attention_phase<64>(a, Kc, Vc, L);
        break;
      case PH_COMB:
        if (a.dh == 128) combine_phase<128>(a);
        else combine_phase<64>(a);
        break;
      case PH_O:
        if (!gemm_dispatch<MT>(a, a.o, GemmIo{a.layers[layer].wo, a.attn_a, MODE_PARTIAL, a.part, nullptr, nullptr}, epoch, lds, &dead)) return;
        break;
      case PH_FO:
        finish_phase(a, a.o.S, a.o.N, a.layers[layer].g_mlp, true);
        break;
      case PH_GU:
        if (!gemm_dispatch<MT>(a, a.gu, GemmIo{a.layers[layer].wgu, a.xa, MODE_GATEUP, nullptr, a.act_a, nullptr}, epoch, lds, &dead)) return;
        break;
      case PH_DOWN:
        if (!gemm_dispatch<MT>(a, a.down, GemmIo{a.layers[layer].wdown, a.act_a, MODE_PARTIAL, a.part, nullptr, nullptr}, epoch, lds, &dead)) return;
        break;
      case PH_FD:
        // the fragments feed the next layer's QKV GEMM; the last layer of the call needs none
        finish_phase(a, a.down.S, a.down.N, layer + 1 < a.le ? a.layers[layer + 1].g_attn : nullptr, true);
        break;
      case PH_UPREP:
        finish_phase(a, 0, 0, a.g_final, false);
        break;
      case PH_UGEMM:
        if (!gemm_dispatch<MT>(a, a.un, GemmIo{a.un_w, a.xa, MODE_UNEMBED, nullptr, nullptr, a.un_part}, epoch, lds, &dead)) return;
        break;
      case PH_UFINAL:
        unembed_final_phase(a, (Top *)lds);
        break;
    }
  }
}

// ---- weight packing (once, at model set-up) -----------------------------------------------------
// Packed column pc of the destination -> (source matrix, source column).
//   kind 0: one source [K, N];  kind 1: q | k | v concatenation;
//   kind 2: per slab, 8T gate channels followed by the same 8T channels of up.
struct PackSrc {
  const uint16_t *s0, *s1, *s2;
  int n0, n1, n2;
  int kind, T, F;
};
__device__ __forceinline__ const uint16_t *pack_col(const PackSrc &p, int pc, int &ld) {
  if (p.kind == 0) {
    ld = p.n0;
    return p.s0 + pc;
  }
  if (p.kind == 1) {
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
  uint16_t *xa = nullptr, *attn_a = nullptr, *act_a = nullptr, *qf = nullptr;
  float *part = nullptr, *rsq = nullptr, *o_part = nullptr, *ml_part = nullptr;
  Top *un_part = nullptr;
  unsigned *sync = nullptr;
  int32_t *zero_len = nullptr;  // {0, scratch error word}: the unembedding has no cache to overflow
  unsigned epoch = 0;
  int max_ns = 32;
};

static int env_int(const char *name, int dflt) {
  const char *v = getenv(name);
  return (v && *v) ? atoi(v) : dflt;
}

// Tiles per slab: the slab count times a k-split of 1, 2, 4 or 8 should fill the CUs in whole
// rounds, and wide slabs are preferred (fewer activation re-reads per weight byte).
static GemmPlan make_plan(int N, int K, int n_wgs, bool gateup, int F, const char *env) {
  GemmPlan p;
  p.N = N; p.K = K; p.KT = K / 32;
  int tiles = N / 16;
  double best = 1e300;
  for (int T = MAX_T; T >= 1; --T) {
    if (gateup ? (F % (8 * T) != 0) : (tiles % T != 0)) continue;
    int slabs = tiles / T;
    for (int S = 1; S <= MAX_S; S *= 2) {
      if (p.KT / S < NCW && S > 1) continue;
      int rounds = ceil_div(slabs * S, n_wgs);
      double cost = (double)rounds * ceil_div(p.KT, S) * (T + 2.0) + 6.0 * S;
      if (cost < best) { best = cost; p.T = T; }
    }
  }
  int forced = env_int(env, 0);
  if (forced >= 1 && forced <= MAX_T && (gateup ? (F % (8 * forced) == 0) : (tiles % forced == 0))) p.T = forced;
  p.n_slabs = tiles / p.T;
  p.bytes = (size_t)N * K * 2;
  return p;
}

static int choose_split(const GemmPlan &p, int n_wgs, int MT, const char *env) {
  int best_S = 1;
  double best = 1e300;
  for (int S = 1; S <= MAX_S; S *= 2) {
    if (p.KT / S < NCW && S > 1) continue;
    int rounds = ceil_div(p.n_slabs * S, n_wgs);
    double cost = (double)rounds * ceil_div(p.KT, S) * (p.T + MT) + 6.0 * S;
    if (cost < best) { best = cost; best_S = S; }
  }
  int forced = env_int(env, 0);
  if (forced >= 1 && forced <= MAX_S && p.KT / forced >= 1) best_S = forced;
  return best_S;
}

int mfma_supported(const la_model_desc *d) {
  int qd = d->n_q_heads * d->head_dim, nqkv = (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim;
  if (d->d_model % 32 || qd % 32 || d->d_ffn % 32 || nqkv % 16 || d->vocab % 16) return 0;
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
  void *ps[] = {f->un, f->xa, f->attn_a, f->act_a, f->qf, f->part, f->rsq, f->o_part, f->ml_part, f->un_part,
                f->sync, f->dev_ptrs, f->zero_len};
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
  f->p_qkv = make_plan(nqkv, d.d_model, f->n_wgs, false, 0, "LA_T_QKV");
  f->p_o = make_plan(d.d_model, qd, f->n_wgs, false, 0, "LA_T_O");
  f->p_gu = make_plan(2 * d.d_ffn, d.d_model, f->n_wgs, true, d.d_ffn, "LA_T_GU");
  f->p_down = make_plan(d.d_model, d.d_ffn, f->n_wgs, false, 0, "LA_T_DOWN");
  f->p_un = make_plan(d.vocab, d.d_model, f->n_wgs, false, 0, "LA_T_UN");
  f->layers.resize(d.n_layers);
  f->host_ptrs.resize(d.n_layers);
  size_t R = LA_MAX_ROWS;
  int n_max = std::max(nqkv, d.d_model);
  f->max_ns = std::max(1, std::min(64, f->n_wgs / d.n_kv_heads));
  size_t QR = (size_t)g * MAX_MT * 16;
  int n_sync = SYNC_STRIDE * 66;
  bool ok = true;
  ok = ok && (f->xa = (uint16_t *)dalloc(R * d.d_model * 2));
  ok = ok && (f->attn_a = (uint16_t *)dalloc(R * qd * 2));
  ok = ok && (f->act_a = (uint16_t *)dalloc(R * (size_t)d.d_ffn * 2));
  ok = ok && (f->qf = (uint16_t *)dalloc((size_t)d.n_kv_heads * QR * d.head_dim * 2));
  ok = ok && (f->part = (float *)dalloc((size_t)MAX_S * R * n_max * 4));
  ok = ok && (f->rsq = (float *)dalloc((size_t)(d.d_model / 32) * 64 * 4));
  ok = ok && (f->o_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * d.head_dim * 4));
  ok = ok && (f->ml_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * 2 * 4));
  ok = ok && (f->sync = (unsigned *)dalloc((size_t)n_sync * 4));
  ok = ok && (f->dev_ptrs = (LayerPtrs *)dalloc((size_t)d.n_layers * sizeof(LayerPtrs)));
  ok = ok && (f->zero_len = (int32_t *)dalloc(8));
  LA_REQUIRE(ok, LA_ENOMEM, "device allocation failed in the MFMA path");
  // pad rows of the operand buffers are read by the MFMAs: keep them finite
  LA_HIP(hipMemset(f->xa, 0, R * d.d_model * 2));
  LA_HIP(hipMemset(f->attn_a, 0, R * qd * 2));
  LA_HIP(hipMemset(f->act_a, 0, R * (size_t)d.d_ffn * 2));
  LA_HIP(hipMemset(f->qf, 0, (size_t)d.n_kv_heads * QR * d.head_dim * 2));
  LA_HIP(hipMemset(f->sync, 0, (size_t)n_sync * 4));
  LA_HIP(hipMemset(f->zero_len, 0, 8));
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
  PackSrc q{(const uint16_t *)w->wq, (const uint16_t *)w->wk, (const uint16_t *)w->wv, qd, kvd, kvd, 1, f->p_qkv.T, 0};
  if ((rc = pack(q, f->p_qkv, &l.wqkv, s))) return rc;
  PackSrc o{(const uint16_t *)w->wo, nullptr, nullptr, d.d_model, 0, 0, 0, f->p_o.T, 0};
  if ((rc = pack(o, f->p_o, &l.wo, s))) return rc;
  PackSrc gu{(const uint16_t *)w->wgate, (const uint16_t *)w->wup, nullptr, d.d_ffn, d.d_ffn, 0, 2, f->p_gu.T, d.d_ffn};
  if ((rc = pack(gu, f->p_gu, &l.wgu, s))) return rc;
  PackSrc dn{(const uint16_t *)w->wdown, nullptr, nullptr, d.d_model, 0, 0, 0, f->p_down.T, 0};
  if ((rc = pack(dn, f->p_down, &l.wdown, s))) return rc;
  f->host_ptrs[layer] = LayerPtrs{l.wqkv, l.wo, l.wgu, l.wdown, m->layers[layer].g_attn, m->layers[layer].g_mlp};
  f->ptrs_dirty = true;
  return LA_OK;
}

int mfma_set_head(la_model *m, const void *unembed, hipStream_t s) {
  MfmaModel *f = m->mf;
  PackSrc u{(const uint16_t *)unembed, nullptr, nullptr, m->d.vocab, 0, 0, 0, f->p_un.T, 0};
  int rc = pack(u, f->p_un, &f->un, s);
  if (rc) return rc;
  if (!f->un_part) f->un_part = (Top *)dalloc((size_t)f->p_un.n_slabs * 64 * sizeof(Top));
  LA_REQUIRE(f->un_part != nullptr, LA_ENOMEM, "device allocation failed");
  return LA_OK;
}

static GemmDev dev_plan(const GemmPlan &p, int S) { return GemmDev{p.KT, p.T, p.n_slabs, S, p.N}; }

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
  a.ncg = d.d_model / 32;
  a.eps = d.rms_eps;
  a.inv_d = 1.0f / (float)d.d_model;
  a.theta = (double)d.rope_theta;
  a.xa = f->xa;
  a.attn_a = f->attn_a;
  a.act_a = f->act_a;
  a.qf = f->qf;
  a.part = f->part;
  a.rsq = f->rsq;
  a.o_part = f->o_part;
  a.ml_part = f->ml_part;
  a.cs = m->rope_cs;
  a.sync = f->sync;
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
  a.qkv = dev_plan(f->p_qkv, choose_split(f->p_qkv, f->n_wgs, a.MT, "LA_S_QKV"));
  a.o = dev_plan(f->p_o, choose_split(f->p_o, f->n_wgs, a.MT, "LA_S_O"));
  a.gu = dev_plan(f->p_gu, 1);
  a.down = dev_plan(f->p_down, choose_split(f->p_down, f->n_wgs, a.MT, "LA_S_DOWN"));
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
  a.un = dev_plan(f->p_un, 1);
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
