// MFMA path for gfx950 (bf16 models): the whole layer stack of a verification step as ONE persistent
// kernel, and a second launch of the same kernel for the unembedding with fused arg-max.
//
// A step reads every weight once (13 GB at the 30-layer Mistral-7B shape) and computes almost
// nothing per byte, so it is bound by HBM.  The kernel is built so that the weight stream
// never has to stop for the arithmetic that depends on it:
//
//   * One workgroup of 8 waves per CU stays resident for the whole launch.  Wave 7 is the
//     PRODUCER: it walks this CU's share of the weights (one contiguous, pre-packed stream per
//     CU, in the order the GEMMs will use it) and copies it HBM -> LDS with direct-to-LDS
//     128-bit loads into a ring of 1 KB slots.  It knows nothing of phases or barriers: it
//     runs ahead of the arithmetic by up to the size of the ring, across every grid barrier.
//   * Waves 0..6 are CONSUMERS.  In a GEMM phase each takes every 7th k-tile of the CU's
//     column tiles, reads the weight fragments from the ring (ds_read_b128), the activation
//     fragments from L2, multiplies (MFMA 16x16x32 f16, fp32 accumulate); the seven partial
//     sums are added in a fixed tree through LDS and the epilogue of the GEMM runs on the
//     finished tile.  The other phases (attention, operand preparation, arg-max) also run on
//     the consumer waves.
//   * Producer and consumers talk through monotonic counters in LDS (fragments landed; per
//     consumer wave the first fragment it still needs).  The consumer waves synchronise among
//     themselves with LDS counters too: the hardware workgroup barrier is not used after
//     start-up, because the producer could not take part in it without stopping the stream.
//   * Phases are separated by a grid barrier (relaxed device-scope atomics).  Everything one
//     workgroup writes for another to read in a later phase is stored with the device-scope
//     cache policy (sc1), so the barrier needs no cache flush or invalidate.
//
// Data layout
//   weights      per CU c, per layer: [GEMM][pass][k-tile][tile-in-pass][lane][8] halves (the bf16
//                weights convert to IEEE half precision without loss, see pack_f16).  Column
//                tile t (16 columns) of a GEMM belongs to CU t mod G.  A fragment is the MFMA B
//                operand of one k-tile (32 deep) x 16 columns: lane l holds column (l & 15),
//                contraction indices 8 (l >> 4) .. +7; the direct-to-LDS load writes lane l's
//                16 bytes at slot + 16 l, which is where the ds_read_b128 of lane l finds them.
//   activations  [k-tile][row-tile][lane][8] halves, the MFMA A operand, written by the epilogue
//                that produces them, in buffers written once per launch (one per layer and
//                use), so a reader can never find a stale copy in its L2.
//   attention    q, K, V and the probabilities are bf16 (the KV cache is), on bf16 MFMA.
//   RMSNorm      is applied as ((x * g) W) * rsqrt(mean(x^2) + eps): the row factor after the
//                contraction, from per-tile sums of squares the O / down epilogues emit.
// All reductions have a fixed order: results are run-to-run identical, and a row's result
// does not depend on how many rows the block has (except for the key split of attention).
#pragma once
#include <type_traits>

#include "la_device.h"
#include "la_internal.h"

namespace la {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef _Float16 __attribute__((ext_vector_type(8))) f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2;

#define LDS_AS __attribute__((address_space(3)))
typedef LDS_AS uint8_t *lds_t;

constexpr int WG_THREADS = 512;
constexpr int NCW = 7;                     // consumer waves 0..6; wave 7 streams the weights
constexpr int CONS_THREADS = NCW * 64;
constexpr int NSLOT = 128;                 // ring slots of 1 KB (a power of two)
constexpr int CHUNK = 8;                   // fragments the producer issues back to back
constexpr int FLIGHT = 7;                  // chunks in flight: 56 loads, the counter holds 63
constexpr int RED_TILES = 8;               // 1 KB accumulator tiles per tree-reduction buffer
constexpr int MAX_NT = 8;                  // column tiles of one pass
constexpr int MAX_MT = LA_MAX_ROWS / 16;
constexpr unsigned OOB = 0x80000000u;      // voffset beyond every buffer (all are < 2 GiB)
constexpr unsigned RSRC_BYTES = 0x7fffffffu;
constexpr int DEV = 16;                    // cache policy sc1: device-scope coherent load / store
constexpr int TRACE_SLOTS = 40;            // timestamps per phase of the optional timeline
constexpr int TRACE_WG = 32;               // words per workgroup after the phases: 8 of the producer, 8 barrier arrival times, 2 x 8 producer snapshots
constexpr int NT_HINT = 2;                 // cache policy nt: streamed once
constexpr int SYNC_GROUP = 16;             // workgroups per arrival counter of the grid barrier
constexpr int SYNC_STRIDE = 64;            // 32-bit words between barrier variables (256 B)
constexpr unsigned SPIN_LDS = 1u << 24;    // polls of an LDS word (~0.1 us each) before giving up
constexpr unsigned SPIN_GLOBAL = 1u << 21; // polls of a global word (~1 us each) before giving up

// LDS map (bytes)
constexpr int LDS_RING = 0;
constexpr int LDS_RED = NSLOT * 1024;                 // 3 buffers of RED_TILES KB; also the result tile
constexpr int LDS_ML = LDS_RED + 3 * RED_TILES * 1024;  // attention: running max / sum per wave and lane
constexpr int LDS_RS = LDS_ML + 4 * 512;              // [64] row factors of the norm
constexpr int LDS_CTL = LDS_RS + 256;                 // control words
constexpr int LDS_CONST = LDS_CTL + 256;                // per-launch constants (LaunchConst)
constexpr int LDS_ARGS = LDS_CONST + 128;               // per consumer wave: arguments of the GEMM pass it calls (PassArgs)
constexpr int LDS_SINK = LDS_ARGS + NCW * 128;             // 256 B that cache-warming loads land in; never read
constexpr int X_TILES = 2;                                 // 1 KB tiles of the residual stream a workgroup can keep in LDS
constexpr int LDS_X = LDS_SINK + 256;                      // this workgroup's columns of x: [column tile][row][16] floats
constexpr int LDS_GAIN = LDS_X + X_TILES * 1024;           // the norm gains of those columns for the running phase: [column tile][16]
constexpr int LDS_BYTES = LDS_GAIN + 256;                  // (a whole wave's 4-byte loads land there: 256 B)
static_assert(X_TILES * 16 <= 64, "one load instruction stages the gains");
static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
// control words
constexpr int C_LANDED = 0;   // fragments of this workgroup's stream that have landed in the ring
constexpr int C_DEAD = 1;     // a wait timed out: every wave leaves the kernel
constexpr int C_CBAR = 2;     // arrivals at the consumer-wave barrier
constexpr int C_GPASS = 3;    // last grid-barrier epoch seen released
constexpr int C_PROG = 8;     // [8..14] per consumer wave: first stream fragment it still needs
constexpr int C_SPARE = 7;   // written, never read
constexpr int C_TREE = 16;    // [16..22] per consumer wave: hand-off sequence number

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

enum GemmMode { MODE_QKV = 0, MODE_RESID = 1, MODE_GATEUP = 2, MODE_UNEMBED = 3 };

// Timelines (StackArgs::trace) and timing experiments (StackArgs::dbg, which make results wrong) exist only in a build
// with -DLA_EXPERIMENTS; in the default build every test of them is a compile-time constant and the code is dropped.
#ifdef LA_EXPERIMENTS
#define LA_TRACE_PTR(a) ((a).trace)
#define LA_DBG_BITS(x) (x)
#else
#define LA_TRACE_PTR(a) ((unsigned long long *)nullptr)
#define LA_DBG_BITS(x) 0
#endif

struct GemmDev {
  int KT;      // k-tiles (32 deep)
  int ntiles;  // 16-column tiles of the whole matrix
  int ntp;     // tiles per pass
};

struct LayerGains {
  const float *g_attn, *g_mlp;
};

struct StackArgs {
  const LayerGains *gains;
  int mode;  // 0: layer stack, 1: unembedding
  int f16;   // the cache, q and the attention's probabilities are IEEE half instead of bfloat16 (register-streaming kernel only)
  int dbg;   // timing experiments (results are wrong when set): 1 producer moves nothing, 2 one operand k-tile, 4 no operand loads, 8 no epilogue, 16 no K/V cache warming, 32 attention on the first workgroups, 64 every workgroup calls the attention, 128 x stays in memory
  int lb, le;
  int Bp, MT, d, Hq, Hkv, dh, F, ncg;
  float eps, inv_d;
  double theta;
  GemmDev qkv, o, gu, down, un;
  // weight stream: CU c reads wstream + c * cu_bytes; per layer seg_frags fragments apart
  const uint8_t *wstream;
  size_t cu_bytes;
  unsigned seg_frags;
  unsigned pace;  // shader-clock cycles a producer lets pass between two chunks (0: as fast as it can).
                  // About the memory's share per CU (8 KB per 700 cycles at 2.4 GHz is 28 GB/s, times
                  // 256 CUs 7.2 TB/s): 650-750 measure the same, 600 and none 1.5-2 % longer (the
                  // producers' bursts after every stall fill the memory queues unevenly), 800 4 % longer.
  float *x;
  const int32_t *pos;
  const uint64_t *vis;
  // write-once operand / statistics buffers, indexed by absolute layer
  uint16_t *xa, *attn_a, *act_a, *qf;
  size_t xa_stride, attn_stride, act_stride, rsq_stride;  // elements per (layer, use)
  float *rsq, *cs;
  uint16_t *K, *V;
  size_t layer_elems;
  const int32_t *L_dev;
  int max_len;
  int32_t *err;      // device error word: 1 the block does not fit the cache, 4 a grid barrier gave up
  int32_t *err_map;  // mapped host word that receives the same code (plain store), read by the host without synchronising
  unsigned spin_global;  // polls of the barrier's release word before a workgroup gives up
  // attention with the keys split over workgroups (register-streaming kernel): partial (o, m, l) records per
  // split unit, and per unit a counter of the records delivered
  float *att_part;
  unsigned *att_cnt;
  const float *g_final;
  Top *un_part;
  int un_parts_per_cu;
  int32_t *ids;
  float *top2;
  unsigned *sync;
  const unsigned *sched;  // register-streaming kernel: the MFMA waves' schedule tables of every workgroup (written once per model)
  unsigned epoch0, n_groups;
  unsigned long long *trace;  // optional: per phase TRACE_SLOTS timestamps of workgroup 0, then TRACE_WG words per workgroup
  int trace_phases;
  int trace_seg;              // which weight matrix of the second layer the producer's eight snapshots cover (0 QKV, 1 O, 2 gate / up, 3 down)
  int trace_sel;              // every workgroup records when it reaches the barriers that end phases trace_sel .. trace_sel + 7
};

// Raises an error: ORs the code into the device word and stores it to the host's mapped word.
__device__ __forceinline__ void raise_error(const StackArgs &a, int code) {
  __hip_atomic_fetch_or(a.err, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(a.err_map, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Values that are the same in every lane, moved to scalar registers.  The compiler cannot see
// that words read from LDS or memory are wave-uniform; without this it guards loads with
// per-lane loops and keeps loop control in vector registers.
__device__ __forceinline__ unsigned uni(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T *uni_ptr(T *p) {
  uint64_t u = (uint64_t)p;
  uint32_t lo = uni((unsigned)u), hi = uni((unsigned)(u >> 32));
  return (T *)(((uint64_t)hi << 32) | lo);
}

// Per-launch constants every phase function needs, kept in LDS so that they need not travel as
// arguments (a function's arguments beyond 32 registers go through memory).
struct LaunchConst {
  int Bp, MT, d, ncg, Hq, Hkv, dh, L, dbg;
  int x_lds;  // this workgroup keeps its columns of the residual stream in LDS (LDS_X)
  float inv_d, eps;
  float *x;
  const float *cs;
  uint16_t *qf;
};
static_assert(sizeof(LaunchConst) <= 128, "LDS_CONST region");
__device__ __forceinline__ LaunchConst launch_const(unsigned lds0) {
  LDS_AS const LaunchConst *p = (LDS_AS const LaunchConst *)(uintptr_t)(lds0 + LDS_CONST);
  LaunchConst c;
  c.Bp = uni(p->Bp); c.MT = uni(p->MT); c.d = uni(p->d); c.ncg = uni(p->ncg); c.Hq = uni(p->Hq); c.Hkv = uni(p->Hkv);
  c.dh = uni(p->dh); c.L = uni(p->L); c.dbg = uni(p->dbg); c.x_lds = uni(p->x_lds);
  c.inv_d = __uint_as_float(uni(__float_as_uint(p->inv_d)));
  c.eps = __uint_as_float(uni(__float_as_uint(p->eps)));
  c.x = uni_ptr(p->x); c.cs = uni_ptr(p->cs); c.qf = uni_ptr(p->qf);
  return c;
}

// Plain structs to and from LDS, word by word (a struct cannot be copied across address spaces).
template <typename T>
__device__ __forceinline__ T lds_get(unsigned addr) {
  static_assert(sizeof(T) % 4 == 0, "whole words");
  T v;
  LDS_AS const unsigned *src = (LDS_AS const unsigned *)(uintptr_t)addr;
  unsigned *dst = reinterpret_cast<unsigned *>(&v);
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) dst[i] = src[i];
  return v;
}
template <typename T>
__device__ __forceinline__ void lds_put(unsigned addr, const T &v) {
  static_assert(sizeof(T) % 4 == 0, "whole words");
  LDS_AS unsigned *dst = (LDS_AS unsigned *)(uintptr_t)addr;
  const unsigned *src = reinterpret_cast<const unsigned *>(&v);
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) dst[i] = src[i];
}

// ---- LDS control words: inline assembly, so that the compiler neither caches them nor puts
// waits for the producer's outstanding direct-to-LDS loads in front of them --------------------
__device__ __forceinline__ unsigned ctl_read(unsigned addr) {
  unsigned v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
  return uni(v);
}
__device__ __forceinline__ unsigned ctl_read_lanes(unsigned addr) {  // a different word per lane
  unsigned v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void ctl_write(unsigned addr, unsigned v) {
  asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void ctl_add(unsigned addr, unsigned v) {
  asm volatile("ds_add_u32 %0, %1" : : "v"(addr), "v"(v) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {  // at most N vector-memory operations outstanding
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

// Sequence numbers a consumer wave carries from phase to phase (all waves hold the same
// values), passed by value into and out of the phase functions.
struct WaveState {
  unsigned cbar_seq;   // consumer barrier: arrivals expected so far
  unsigned tree_seq;   // hand-off sequence of the reduction tree
  unsigned seen;       // cached copy of C_LANDED
  int ok;              // 0 after a wait timed out: the wave leaves the kernel
};

struct Wave {          // a wave's view inside one function
  unsigned ctl;        // LDS byte address of the control words
  int w, lane;
  WaveState st;
};

// Spin until the control word reaches `want`.  Returns false (and raises C_DEAD) on a timeout
// or when another wave has raised C_DEAD.
__device__ __forceinline__ bool ctl_wait_ge(Wave &wv, int word, unsigned want) {
  unsigned spins = 0;
  for (;;) {
    unsigned v = ctl_read(wv.ctl + 4 * word);
    if ((int)(v - want) >= 0) return true;
    __builtin_amdgcn_s_sleep(1);
    ++spins;
    if ((spins & 255u) == 0) {
      if (ctl_read(wv.ctl + 4 * C_DEAD) != 0 || spins > SPIN_LDS) {
        ctl_write(wv.ctl + 4 * C_DEAD, 1u);
        wv.st.ok = 0;
        return false;
      }
    }
  }
}

// Barrier of the seven consumer waves.  LDS executes one wave's operations in order, so the
// data a wave wrote before arriving is visible to every wave that has seen the arrival.
__device__ __forceinline__ bool cons_barrier(Wave &wv) {
  wv.st.cbar_seq += NCW;
  if (wv.lane == 0) ctl_add(wv.ctl + 4 * C_CBAR, 1u);
  return ctl_wait_ge(wv, C_CBAR, wv.st.cbar_seq);
}

// Timeline of workgroup 0, wave 0 (tracing only): tr is null everywhere else.
__device__ __forceinline__ void tr_mark(unsigned long long *tr, const Wave &wv, int k) {
  if (tr && wv.w == 0 && wv.lane == 0) tr[k] = wall_clock64();
}
__device__ __forceinline__ void tr_mark_wave(unsigned long long *tr, const Wave &wv, int k) {  // slot k + wave
  if (tr && wv.lane == 0) tr[k + wv.w] = wall_clock64();
}

// ---- device-scope accessors ------------------------------------------------------------------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const void *p) {
  return __builtin_amdgcn_make_buffer_rsrc(uni_ptr(const_cast<void *>(p)), 0, RSRC_BYTES, 0x00020000);
}
template <int POLICY>
__device__ __forceinline__ u32x4 ld128p(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, POLICY));
}
__device__ __forceinline__ u32x4 ld128(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, DEV);
}
__device__ __forceinline__ void st128(__amdgpu_buffer_rsrc_t r, unsigned byte_off, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_off, 0, DEV);
}
__device__ __forceinline__ void st64(__amdgpu_buffer_rsrc_t r, unsigned byte_off, u32x2 v) {
  __builtin_amdgcn_raw_buffer_store_b64(v, r, byte_off, 0, DEV);
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
// Two activations as IEEE half precision (round to nearest even; beyond the format's range: the
// largest finite value).  The weight GEMMs take their operands in this format: the bf16 weights
// convert to it without loss (see pack_weights_kernel), and an activation keeps 11 significant
// bits instead of 8, which removes most of the rounding noise of a deep stack.
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi);
// two values in the cache's 16-bit type
__device__ __forceinline__ uint32_t pack_kv(bool half, float lo, float hi) { return half ? pack_f16(lo, hi) : pack_bf16(lo, hi); }
__device__ __forceinline__ uint16_t kv_bits(bool half, float v) { return (uint16_t)(pack_kv(half, v, 0.f) & 0xffffu); }
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  const float lim = 65504.0f;
  const _Float16 a = (_Float16)fminf(fmaxf(lo, -lim), lim), b = (_Float16)fminf(fmaxf(hi, -lim), lim);
  return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}
// byte offset of the 16-byte piece (row b, columns col..col+7, col a multiple of 8) of an
// operand-fragment buffer with MT row tiles
__device__ __forceinline__ unsigned frag_piece(int col, int b, int MT) {
  return (unsigned)((((size_t)(col >> 5) * MT + (b >> 4)) * 64 + (b & 15) + 16 * ((col & 31) >> 3)) * 16);
}

// tiles of a matrix that belong to this CU (tile t -> CU t mod G)
__device__ __forceinline__ int my_tiles(int ntiles) {
  int c = blockIdx.x, G = gridDim.x;
  return ntiles > c ? (ntiles - c + G - 1) / G : 0;
}

// ---- grid barrier (consumer waves) -----------------------------------------------------------
// Arrival counters per group of SYNC_GROUP workgroups, one top counter, one release word; all
// monotonic (epoch e is complete when a counter reaches e * members).  Only relaxed device-scope
// atomics: the data exchanged between workgroups travels with sc1 accesses, and each wave waits
// for its own stores before the workgroup arrives.  Every spin is bounded: on a timeout the
// error flag is raised and the workgroup leaves the kernel (the others then time out too).
__device__ __forceinline__ bool grid_sync(const StackArgs &a, Wave &wv, unsigned epoch, unsigned long long *tr) {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  wait_vmcnt<0>();  // this wave's stores are acknowledged
  tr_mark(tr, wv, 6);
  if (!cons_barrier(wv)) return false;
  tr_mark(tr, wv, 7);
  if (wv.w == 0) {
    if (wv.lane == 0) {
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
      bool ok = true;
      while ((int)(__hip_atomic_load(rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) < 0) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > a.spin_global) {
          raise_error(a, 4);
          ok = false;
          break;
        }
      }
      if (ok) ctl_write(wv.ctl + 4 * C_GPASS, epoch);
      else ctl_write(wv.ctl + 4 * C_DEAD, 1u);
    }
  }
  const bool ok = ctl_wait_ge(wv, C_GPASS, epoch);
  tr_mark(tr, wv, 8);
  return ok;
}

// ---- producer ----------------------------------------------------------------------------------
// Streams n_seg segments of seg_used fragments each (a layer's share of this CU, padded to whole
// chunks; seg_stride fragments apart in memory) into the ring, in order.  Keeps FLIGHT chunks in flight, publishes
// C_LANDED as chunks land, and never overwrites a slot before every consumer wave has moved
// past the fragment it held.
template <bool TR>  // TR: with the timeline's clock reads and counters (the untraced loop holds none of them)
__device__ __forceinline__ void producer(const StackArgs &a, unsigned ctl, LDS_AS uint8_t *ring, unsigned first_seg, unsigned n_seg,
                                         unsigned seg_used, unsigned seg_stride, unsigned long long *stats, unsigned snap_a,
                                         unsigned snap_b) {
  const int lane = threadIdx.x & 63;
  const uint8_t *base = uni_ptr(a.wstream + (size_t)blockIdx.x * a.cu_bytes);
  __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base), 0, uni((unsigned)a.cu_bytes), 0x00020000);
  first_seg = uni(first_seg);
  n_seg = uni(n_seg);
  seg_used = uni(seg_used);
  seg_stride = uni(seg_stride);
  ctl = uni(ctl);
  const unsigned total = n_seg * seg_used;
  unsigned next = 0, landed = 0, inflight = 0, free_until = NSLOT;
  unsigned seg_off = first_seg * seg_stride, f_in_seg = 0;  // memory position of fragment `next`
  unsigned polls = 0, full_events = 0;
  unsigned long long t_wait = 0, t_poll = 0;
  constexpr bool tr = TR;
  const unsigned long long t_begin = tr ? wall_clock64() : 0ull;
  if (LA_DBG_BITS(a.dbg) & 1) {
    ctl_write(ctl + 4 * C_LANDED, total);
    return;
  }
  // the oldest chunk in flight has landed once at most (inflight - 1) chunks are outstanding
  auto retire_oldest = [&]() {
    switch (inflight) {
      case 1: wait_vmcnt<0 * CHUNK>(); break;
      case 2: wait_vmcnt<1 * CHUNK>(); break;
      case 3: wait_vmcnt<2 * CHUNK>(); break;
      case 4: wait_vmcnt<3 * CHUNK>(); break;
      case 5: wait_vmcnt<4 * CHUNK>(); break;
      case 6: wait_vmcnt<5 * CHUNK>(); break;
      default: wait_vmcnt<6 * CHUNK>(); break;
    }
    static_assert(FLIGHT == 7 && FLIGHT * CHUNK <= 63, "one case per number of chunks in flight");
    landed += CHUNK;
    ctl_write(ctl + 4 * C_LANDED, landed < total ? landed : total);
    --inflight;
  };
  auto read_space = [&]() {
    const unsigned c = ctl_read_lanes(ctl + 4 * (C_PROG + (lane < NCW ? lane : 0)));
    // minimum of lanes 0..7 (lane 7 holds wave 0's word again) in three steps within the row:
    // after the shifts by 1, 2 and 4 lanes, lane 7 has seen lanes 0..7
    unsigned m = c;
    m = min(m, (unsigned)__builtin_amdgcn_update_dpp((int)m, (int)m, 0x111, 0xf, 0xf, false));
    m = min(m, (unsigned)__builtin_amdgcn_update_dpp((int)m, (int)m, 0x112, 0xf, 0xf, false));
    m = min(m, (unsigned)__builtin_amdgcn_update_dpp((int)m, (int)m, 0x114, 0xf, 0xf, false));
    static_assert(NCW == 7, "eight lanes: seven waves and one repeat");
    free_until = (unsigned)__builtin_amdgcn_readlane((int)m, 7) + NSLOT;
  };
  unsigned idle_spins = 0;
  const unsigned pace = uni(a.pace);
  unsigned long long t_pace = 0;
  unsigned t_next = (unsigned)clock64();  // (the clock's low word: differences are taken modulo 2^32)
  snap_a = uni(snap_a);
  snap_b = uni(snap_b);
  int snaps = 0;
  while (next < total) {
    if (tr && snaps < 8 && next >= snap_a + (unsigned)snaps * ((snap_b - snap_a) / 7)) {  // (timeline only) eight stream positions
      if (lane == 0) {
        stats[16 + snaps] = wall_clock64();
        stats[24 + snaps] = ((unsigned long long)(t_wait & 0xffffffu)) | ((unsigned long long)(t_poll & 0xffffffu) << 24) | ((unsigned long long)(t_pace & 0xffffu) << 48);
      }
      ++snaps;
    }
    if (next + CHUNK > free_until) {
      read_space();
      if (next + CHUNK > free_until) {
        // Ring full.  Chunks in flight keep landing meanwhile: retire them one at a time (the
        // consumers may be waiting for exactly those), and look for space again after each.
        if (inflight) {
          const unsigned long long t0 = tr ? wall_clock64() : 0ull;
          retire_oldest();
          if (tr) t_wait += wall_clock64() - t0;
          continue;
        }
        const unsigned long long t0 = tr ? wall_clock64() : 0ull;
        ++full_events;
        for (;;) {
          __builtin_amdgcn_s_sleep(1);
          ++polls;
          read_space();
          if (next + CHUNK <= free_until) break;
          if ((++idle_spins & 255u) == 0 && (ctl_read(ctl + 4 * C_DEAD) != 0 || idle_spins > SPIN_LDS)) {
            ctl_write(ctl + 4 * C_DEAD, 1u);
            return;
          }
        }
        idle_spins = 0;
        if (tr) t_poll += wall_clock64() - t0;
      }
    }
    if (pace) {
      const unsigned long long t0 = tr ? wall_clock64() : 0ull;
      unsigned now = (unsigned)clock64();
      while ((int)(now - t_next) < 0) {
        __builtin_amdgcn_s_sleep(1);
        now = (unsigned)clock64();
      }
      t_next = now + pace;
      if (tr) t_pace += wall_clock64() - t0;
    }
    {
      // a chunk is contiguous in memory and in the ring (segments are padded to whole chunks):
      // one scalar offset, one LDS base, the instruction offset steps through both
      LDS_AS void *dst = (LDS_AS void *)(ring + (next & (NSLOT - 1)) * 1024);
      const unsigned soff = (seg_off + f_in_seg) * 1024u;
      const unsigned vo = (unsigned)lane * 16u;
      static_assert(CHUNK == 8, "the chunk is unrolled by hand");
      // (the instruction offset reaches 4095: two groups of four)
      LDS_AS void *dst2 = (LDS_AS void *)(ring + (next & (NSLOT - 1)) * 1024 + 4096);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vo, soff, 0, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vo, soff, 1024, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vo, soff, 2048, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst, 16, vo, soff, 3072, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst2, 16, vo, soff + 4096u, 0, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst2, 16, vo, soff + 4096u, 1024, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst2, 16, vo, soff + 4096u, 2048, NT_HINT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r, dst2, 16, vo, soff + 4096u, 3072, NT_HINT);
      f_in_seg += CHUNK;
      if (f_in_seg == seg_used) {
        f_in_seg = 0;
        seg_off += seg_stride;
      }
    }
    next += CHUNK;
    if (++inflight == FLIGHT) {
      const unsigned long long t0 = tr ? wall_clock64() : 0ull;
      retire_oldest();
      if (tr) t_wait += wall_clock64() - t0;
    }
  }
  while (inflight) retire_oldest();
  ctl_write(ctl + 4 * C_LANDED, total);
  if (stats && lane == 0) {
    stats[0] = polls;
    stats[1] = full_events;
    stats[2] = 0;
    stats[3] = t_poll;
    stats[4] = t_wait;
    stats[5] = wall_clock64() - t_begin;
  }
}

// ---- GEMM pass (consumer waves) --------------------------------------------------------------
template <int MT, int NT>
struct Depth {  // k-tiles per batch of a wave = depth of its activation-operand prefetch
  // A wave waits for the weights of its whole batch before it starts, which keeps (DA - 1) 7 NT
  // ring slots from being refilled meanwhile: deep batches only where the k-tiles are small and
  // the operand latency (about six k-tiles of a wave at full stream rate) would show otherwise.
  static constexpr int value = NT == 1 ? 6 : NT == 2 ? 4 : NT == 3 ? 3 : NT == 4 ? 2 : 1;
  static_assert((NCW - 1 + NCW * (value - 1) + 1) * NT <= NSLOT - CHUNK, "the last wave's batch must fit the ring");
};

// Row factors rsqrt(mean(x^2) + eps) of the block's rows into LDS: wave w takes rows w, w+7, ...
// Loads first, fixed-order reduction after: the caller puts the k-loop in between.
template <int MT>
struct RowStat {
  static constexpr int NR = (16 * MT + NCW - 1) / NCW;
  f32x4 v[NR][2];
};
template <int MT>
__device__ __forceinline__ void rowstat_load(int Bp, int ncg, const Wave &wv, const float *rsq_in, RowStat<MT> &rs) {
  // ncg / 4 <= 128 vectors per row: two per lane, no branches (beyond the row or the block:
  // out-of-range loads that move nothing and return zeros)
  __amdgpu_buffer_rsrc_t rr = rsrc_of(rsq_in);
#pragma unroll
  for (int i = 0; i < RowStat<MT>::NR; ++i) {
    const int row = wv.w + NCW * i;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c4 = wv.lane + 64 * j;
      const unsigned vo = (row < Bp && c4 < (ncg >> 2)) ? (unsigned)c4 * 16u : OOB;
      rs.v[i][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, vo, (unsigned)(row * ncg) * 4u, 0));
    }
  }
}
template <int MT>
__device__ __forceinline__ void rowstat_finish(int Bp, float inv_d, float eps, const Wave &wv, const RowStat<MT> &rs,
                                               LDS_AS float *rs_lds) {
#pragma unroll
  for (int i = 0; i < RowStat<MT>::NR; ++i) {
    int row = wv.w + NCW * i;
    f32x4 t = rs.v[i][0] + rs.v[i][1];
    float s = (t[0] + t[1]) + (t[2] + t[3]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (row < 16 * MT && wv.lane == 0) rs_lds[row] = row < Bp ? 1.0f / sqrtf(s * inv_d + eps) : 0.f;
  }
}

// ---- GEMM epilogues ----------------------------------------------------------------------------
// Run by all consumer waves on a finished chunk of the result (rows x ntc column tiles, row-major
// in LDS).  A function of its own, with everything it needs passed by value: it runs once per
// chunk, and keeping it out of the GEMM loops keeps their register allocation free of it.
// (Two structs: an aggregate of more than 64 bytes is passed through memory.)
struct EpiPtrs {
  uint16_t *Kc, *Vc;
  const float *gain;
  uint16_t *xa_out;
  float *rsq_out;
  uint16_t *act_a;
  Top *un_part;
};
struct EpiInts {
  int mode, tile_first, ntc, LDT, part, tid;
  unsigned lds0;  // LDS byte address of the kernel's dynamic LDS
};
static_assert(sizeof(EpiPtrs) <= 64 && sizeof(EpiInts) <= 64, "passed in registers");

// Everything one GEMM pass needs.  The pass is a function of its own (one per number of column
// tiles), so that its loops get registers of their own and nothing of the rest of the kernel is
// kept alive, or spilled, across them.  The caller leaves the arguments in the wave's slot of
// LDS_ARGS: arguments beyond 32 registers would travel through scratch memory, whose latency is
// that of a global load.
struct alignas(16) PassArgs {
  EpiPtrs q;               // epilogue outputs
  int mode;                // epilogue (GemmMode)
  const uint16_t *A;       // operand fragments (a write-once buffer: loaded through the cache)
  const float *rsq_in;     // sums of squares of the input rows [64][ncg], or null: no row factors
  int KT, tile0, part0;
  unsigned sbase;          // index in the workgroup's stream of the pass's first fragment
  unsigned long long *tr;  // timeline slots of this phase (workgroup 0 only) or null
};

// One pass: NT column tiles of this CU (local tiles tile0 .. tile0+NT-1), the whole contraction.
static_assert(sizeof(PassArgs) <= 128, "LDS_ARGS slot");

__device__ __attribute__((noinline)) void gemm_epilogue(EpiInts e) {
  const unsigned lds0 = uni(e.lds0);
  const EpiPtrs q = lds_get<EpiPtrs>(lds0 + LDS_ARGS + 128 * uni(e.tid >> 6));  // first member of the wave's PassArgs
  const LaunchConst lc = launch_const(lds0);
  const int mode = uni(e.mode), Bp = lc.Bp, MT = lc.MT, d = lc.d, ncg = lc.ncg, Hq = lc.Hq, Hkv = lc.Hkv, dh = lc.dh, L = lc.L,
            tile_first = uni(e.tile_first), ntc = uni(e.ntc), LDT = uni(e.LDT), part = uni(e.part);
  const int tid = e.tid;
  const float *cs = lc.cs;
  LDS_AS const float *tile = (LDS_AS const float *)(uintptr_t)(lds0 + LDS_RED);
  LDS_AS const float *rs_lds = (LDS_AS const float *)(uintptr_t)(lds0 + LDS_RS);
  const int G = gridDim.x, cu = blockIdx.x;
  if (mode == MODE_QKV) {
    // A tile holds channels 8j..8j+7 (columns 0..7) and dh/2 + 8j.. (columns 8..15) of one
    // head: both members of eight RoPE pairs.  One thread per (row, tile).
    for (int it = tid; it < Bp * ntc; it += CONS_THREADS) {
      const int b = it / ntc, tt = it - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const int half = dh >> 1, spj = dh >> 4, grp = Hq / Hkv;
      const int hs = gt / spj, j = gt - hs * spj;
      const float rsf = rs_lds[b];
      LDS_AS const float *tr = tile + b * LDT + 16 * tt;
      const float qscale = hs < Hq ? 1.0f / sqrtf((float)dh) : 1.0f;
      float y0[8], y1[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float x0 = tr[k] * rsf, x1 = tr[8 + k] * rsf;
        if (hs < Hq + Hkv) {
          float c = cs[((size_t)b * half + 8 * j + k) * 2], sn = cs[((size_t)b * half + 8 * j + k) * 2 + 1];
          y0[k] = (x0 * c - x1 * sn) * qscale;
          y1[k] = (x1 * c + x0 * sn) * qscale;
        } else {
          y0[k] = x0;
          y1[k] = x1;
        }
      }
      u32x4 lo = {pack_bf16(y0[0], y0[1]), pack_bf16(y0[2], y0[3]), pack_bf16(y0[4], y0[5]), pack_bf16(y0[6], y0[7])};
      u32x4 hi = {pack_bf16(y1[0], y1[1]), pack_bf16(y1[2], y1[3]), pack_bf16(y1[4], y1[5]), pack_bf16(y1[6], y1[7])};
      const int o_lo = j, o_hi = (half >> 3) + j;  // channel octets of the two pieces
      if (hs < Hq) {
        __amdgpu_buffer_rsrc_t rqf = rsrc_of(lc.qf);
        int kvh = hs / grp, jq = hs - kvh * grp, rt = jq * MT + (b >> 4);
        size_t fb = ((size_t)kvh * (grp * MT) + rt) * (dh >> 5);
        st128(rqf, (unsigned)(((fb + (o_lo >> 2)) * 64 + (b & 15) + 16 * (o_lo & 3)) * 16), lo);
        st128(rqf, (unsigned)(((fb + (o_hi >> 2)) * 64 + (b & 15) + 16 * (o_hi & 3)) * 16), hi);
      } else if (hs < Hq + Hkv) {
        __amdgpu_buffer_rsrc_t rk = rsrc_of(q.Kc);
        size_t rb = ((size_t)(L + b) * Hkv + (hs - Hq)) * dh;
        st128(rk, (unsigned)((rb + 8 * o_lo) * 2), lo);
        st128(rk, (unsigned)((rb + 8 * o_hi) * 2), hi);
      } else {
        __amdgpu_buffer_rsrc_t rv = rsrc_of(q.Vc);
        int h = hs - Hq - Hkv;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          st16(rv, (unsigned)(v_index(true, L + b, h, 8 * j + k, Hkv, dh) * 2), float_to_bf16(y0[k]));
          st16(rv, (unsigned)(v_index(true, L + b, h, half + 8 * j + k, Hkv, dh) * 2), float_to_bf16(y1[k]));
        }
      }
    }
  } else if (mode == MODE_RESID) {
    // x[:, tile columns] += tile; sum of squares of the new values; fragments of x * gain.
    // Two threads per (row, tile), eight columns each.  This workgroup owns these columns of
    // x in every layer, so x needs no device-scope accesses.
    for (int it = tid; it < Bp * ntc * 2; it += CONS_THREADS) {
      const int oct = it & 1, bt = it >> 1;
      const int b = bt / ntc, tt = bt - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const int col = 16 * gt + 8 * oct;
      f32x4 *xp = reinterpret_cast<f32x4 *>(lc.x + (size_t)b * d + col);
      LDS_AS const float *tr = tile + b * LDT + 16 * tt + 8 * oct;
      // (x in LDS: no load from memory stands between the reduction and the stores)
      LDS_AS f32x4 *xs = (LDS_AS f32x4 *)(uintptr_t)(lds0 + LDS_X + (((tile_first + tt) * 16 * MT + b) * 16 + 8 * oct) * 4);
      f32x4 x0, x1;
      if (lc.x_lds) {
        x0 = xs[0];
        x1 = xs[1];
      } else {
        x0 = xp[0];
        x1 = xp[1];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x0[i] += tr[i];
        x1[i] += tr[4 + i];
      }
      if (lc.x_lds) {
        xs[0] = x0;
        xs[1] = x1;
      }
      xp[0] = x0;
      xp[1] = x1;
      float sq = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
      sq += __shfl_xor(sq, 1, 64);
      if (q.gain) {
        if (oct == 0) st32f(rsrc_of(q.rsq_out), (unsigned)(b * ncg + gt) * 4, sq);
        float gp[8];
        if (lc.x_lds) {  // staged at the start of the phase (gain_stage)
          LDS_AS const f32x4 *gs = (LDS_AS const f32x4 *)(uintptr_t)(lds0 + LDS_GAIN + ((tile_first + tt) * 16 + 8 * oct) * 4);
          const f32x4 g0 = gs[0], g1 = gs[1];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            gp[i] = g0[i];
            gp[4 + i] = g1[i];
          }
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) gp[i] = q.gain[col + i];
        }
        u32x4 v = {pack_f16(x0[0] * gp[0], x0[1] * gp[1]), pack_f16(x0[2] * gp[2], x0[3] * gp[3]),
                   pack_f16(x1[0] * gp[4], x1[1] * gp[5]), pack_f16(x1[2] * gp[6], x1[3] * gp[7])};
        st128(rsrc_of(q.xa_out), frag_piece(col, b, MT), v);
      }
    }
  } else if (mode == MODE_GATEUP) {
    // tile columns: 8 gate channels, then the same 8 channels of up
    __amdgpu_buffer_rsrc_t rp = rsrc_of(q.act_a);
    for (int it = tid; it < Bp * ntc; it += CONS_THREADS) {
      const int b = it / ntc, tt = it - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const float rsf = rs_lds[b];
      LDS_AS const float *gp = tile + b * LDT + 16 * tt, *up = gp + 8;
      float act[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float g = gp[i] * rsf, u = up[i] * rsf;
        act[i] = g / (1.0f + __expf(-g)) * u;
      }
      st128(rp, frag_piece(8 * gt, b, MT),
            u32x4{pack_f16(act[0], act[1]), pack_f16(act[2], act[3]), pack_f16(act[4], act[5]), pack_f16(act[6], act[7])});
    }
  } else {  // MODE_UNEMBED: arg-max of each row over this chunk's columns, 4 threads per row
    const int row = tid >> 2, j = tid & 3;
    Top best{-INFINITY, 0x7fffffff, -INFINITY};
    if (row < Bp)
      for (int c = j; c < 16 * ntc; c += 4) {
        int gt = cu + G * (tile_first + (c >> 4));
        best = top_merge2(best, Top{tile[row * LDT + c], 16 * gt + (c & 15), -INFINITY});
      }
#pragma unroll
    for (int o = 1; o < 4; o <<= 1) {
      Top other;
      other.v1 = __shfl_xor(best.v1, o, 64);
      other.i1 = __shfl_xor(best.i1, o, 64);
      other.v2 = __shfl_xor(best.v2, o, 64);
      best = top_merge2(best, other);
    }
    if (j == 0 && row < Bp) {
      __amdgpu_buffer_rsrc_t rp = rsrc_of(q.un_part);
      unsigned o = (unsigned)(((size_t)part * 64 + row) * sizeof(Top));
      st32f(rp, o, best.v1);
      __builtin_amdgcn_raw_buffer_store_b32((unsigned)best.i1, rp, o + 4, 0, DEV);
      st32f(rp, o + 8, best.v2);
    }
  }
}


template <int MT, int NT>
__device__ __attribute__((noinline)) WaveState gemm_pass(unsigned lds0_in, WaveState st_in) {
  constexpr int DA = Depth<MT, NT>::value;
  constexpr int TPC = (RED_TILES / MT) < NT ? (RED_TILES / MT) : NT;  // column tiles per reduction chunk
  constexpr int LDT = 16 * TPC + 4;                                  // padded row length of the result tile
  Wave wv;
  wv.w = uni((int)(threadIdx.x >> 6));
  wv.lane = threadIdx.x & 63;
  const unsigned lds0 = uni(lds0_in);
  const PassArgs p = lds_get<PassArgs>(lds0 + LDS_ARGS + 128 * wv.w);
  const LaunchConst lc = launch_const(lds0);
  wv.ctl = lds0 + LDS_CTL;
  wv.st.cbar_seq = uni(st_in.cbar_seq);
  wv.st.tree_seq = uni(st_in.tree_seq);
  wv.st.seen = uni(st_in.seen);
  wv.st.ok = 1;
  const int w = wv.w, lane = wv.lane;
  const int KT = uni(p.KT), tile0 = uni(p.tile0), Bp = lc.Bp, ncg = lc.ncg;
  const unsigned sbase = uni(p.sbase);
  unsigned long long *tr = uni_ptr(p.tr);
  const float *rsq_in = uni_ptr(p.rsq_in);
  const bool need_rs = rsq_in != nullptr;
  LDS_AS const u32x4 *ring = (LDS_AS const u32x4 *)(uintptr_t)(lds0 + LDS_RING);
  LDS_AS f32x4 *red = (LDS_AS f32x4 *)(uintptr_t)(lds0 + LDS_RED);
  LDS_AS float *tile = (LDS_AS float *)(uintptr_t)(lds0 + LDS_RED);
  LDS_AS float *rs_lds = (LDS_AS float *)(uintptr_t)(lds0 + LDS_RS);
  __amdgpu_buffer_rsrc_t ra = rsrc_of(p.A);
  const unsigned voff = lane * 16;
  const int nk = KT > w ? (KT - w + NCW - 1) / NCW : 0;  // this wave's k-tiles: w, w + 7, ...
  unsigned long long wait_ticks = 0;
  // (no timeline marks between here and the end of the k-loop: a conditional store among the
  // operand loads makes the number of outstanding memory operations path-dependent, and the
  // compiler then waits for all of them at every use)

  u32x4 rA[DA][MT];
  auto load_a = [&](int slot, int i) {
    unsigned vo = (i < nk && !(LA_DBG_BITS(lc.dbg) & 4)) ? voff : OOB;  // out of range: zeros come back, no memory traffic
    unsigned kt = (LA_DBG_BITS(lc.dbg) & 2) ? 0u : (unsigned)(w + NCW * i);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) rA[slot][mt] = __builtin_amdgcn_raw_buffer_load_b128(ra, vo, (kt * MT + mt) * 1024u, 0);
  };
#pragma unroll
  for (int s = 0; s < DA; ++s) load_a(s, s);
  RowStat<MT> rs;
  if (need_rs) rowstat_load<MT>(Bp, ncg, wv, rsq_in, rs);

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The wave's k-tiles are taken DA at a time.  One wait per batch (for the weights of its last
  // k-tile), then straight-line code: every slot reads its weights from the ring, multiplies and
  // requests the operand of the slot's next turn, so the operand prefetch is a full batch deep.
  // A slot beyond the wave's last k-tile multiplies zeros and loads out of range (nothing moves).
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  for (int i0 = 0; i0 < nk; i0 += DA) {
    const int last = (i0 + DA < nk ? i0 + DA : nk) - 1;  // the batch's last valid k-tile of this wave
    const unsigned need = sbase + (unsigned)(w + NCW * last + 1) * NT;
    if ((int)(wv.st.seen - need) < 0) {
      unsigned spins = 0;
      const unsigned long long t0 = tr ? wall_clock64() : 0ull;
      for (;;) {
        wv.st.seen = ctl_read(wv.ctl + 4 * C_LANDED);
        if ((int)(wv.st.seen - need) >= 0) break;
        __builtin_amdgcn_s_sleep(1);
        if ((++spins & 255u) == 0 && (ctl_read(wv.ctl + 4 * C_DEAD) != 0 || spins > SPIN_LDS)) {
          ctl_write(wv.ctl + 4 * C_DEAD, 1u);
          wv.st.ok = 0;
          return wv.st;
        }
      }
      if (tr) wait_ticks += wall_clock64() - t0;
    }
#pragma unroll
    for (int s = 0; s < DA; ++s) {
      const int i = i0 + s;
      const bool valid = i < nk;
      const unsigned kt = valid ? (unsigned)(w + NCW * i) : 0u;
      const unsigned first = sbase + kt * NT;
      u32x4 rW[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        u32x4 v = ring[((first + t) & (NSLOT - 1)) * 64 + lane];
        rW[t] = valid ? v : zero4;
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, rA[s][mt]),
                                                               __builtin_bit_cast(f16x8, rW[t]), acc[mt][t], 0, 0, 0);
      // this k-tile's reads are in the LDS queue before the write below: when the producer sees
      // the new value, the slots have been read (LDS traffic does not disturb the load counting)
      // Written by every lane, and to a spare word for a slot beyond the last k-tile: a branch
      // here would split the batch into blocks and cost the precise load counting.
      {
        const unsigned nxt = i + 1 < nk ? kt + NCW : (unsigned)KT;
        // (a plain volatile store between compiler fences rather than the inline-assembly
        // accessor: inline assembly inside the batch also costs the precise load counting)
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        *(volatile LDS_AS unsigned *)(uintptr_t)(wv.ctl + 4 * (valid ? C_PROG + w : C_SPARE)) = sbase + nxt * NT;
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
      }
      load_a(s, i + DA);
    }
  }
  // nothing of this pass is needed any more (also covers a wave that had no k-tile)
  if (lane == 0) ctl_write(wv.ctl + 4 * (C_PROG + w), sbase + (unsigned)KT * NT);
  if (need_rs) rowstat_finish<MT>(Bp, lc.inv_d, lc.eps, wv, rs, rs_lds);
  if (tr && w == 0 && lane == 0 && tile0 == 0) {
    tr[1] = wall_clock64();
    tr[3] = wait_ticks;
  }

  // ---- reduction over the seven waves and epilogue, TPC column tiles at a time ----
#pragma unroll
  for (int c0 = 0; c0 < NT; c0 += TPC) {
    auto put = [&](int buf) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tt = 0; tt < TPC; ++tt)
          if (c0 + tt < NT) red[(buf * RED_TILES + mt * TPC + tt) * 64 + lane] = acc[mt][c0 + tt];
    };
    auto add = [&](int buf) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tt = 0; tt < TPC; ++tt)
          if (c0 + tt < NT) acc[mt][c0 + tt] += red[(buf * RED_TILES + mt * TPC + tt) * 64 + lane];
    };
    const unsigned q = wv.st.tree_seq;
    auto signal = [&](unsigned v) {
      if (lane == 0) ctl_write(wv.ctl + 4 * (C_TREE + w), v);
    };
    // ((w0 + w4) + (w2 + w6)) + (w3 + (w1 + w5)); a wave only ever overwrites a buffer it has
    // itself finished reading
    if (w >= 4) { put(w - 4); signal(q + 1); }
    if (w < 3) { if (!ctl_wait_ge(wv, C_TREE + w + 4, q + 1)) return wv.st; add(w); }
    if (w == 2) { put(2); signal(q + 2); }
    if (w == 1) { put(1); signal(q + 2); }
    if (w == 0) { if (!ctl_wait_ge(wv, C_TREE + 2, q + 2)) return wv.st; add(2); }
    if (w == 3) { if (!ctl_wait_ge(wv, C_TREE + 1, q + 2)) return wv.st; add(1); put(1); signal(q + 3); }
    if (w == 0) {
      if (!ctl_wait_ge(wv, C_TREE + 3, q + 3)) return wv.st;
      add(1);
      // finished tile, row-major: acc[mt][t][i] is (row 16 mt + 4 (lane >> 4) + i, column 16 t + (lane & 15))
      const int q4 = lane >> 4, c16 = lane & 15;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tt = 0; tt < TPC; ++tt)
          if (c0 + tt < NT)
#pragma unroll
            for (int i = 0; i < 4; ++i) tile[(16 * mt + 4 * q4 + i) * LDT + 16 * tt + c16] = acc[mt][c0 + tt][i];
      signal(q + 4);
    }
    wv.st.tree_seq = q + 4;
    if (!ctl_wait_ge(wv, C_TREE + 0, q + 4)) return wv.st;
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    if (c0 == 0 && tile0 == 0) tr_mark(tr, wv, 4);
    {
      EpiInts e;
      e.lds0 = lds0;
      e.mode = uni(p.mode);
      e.tile_first = tile0 + c0;
      e.ntc = (NT - c0) < TPC ? (NT - c0) : TPC;
      e.LDT = LDT;
      e.part = p.part0 + c0 / TPC;
      e.tid = w * 64 + lane;
      if (!(LA_DBG_BITS(lc.dbg) & 8)) gemm_epilogue(e);
    }
    // everyone has finished reading the tile before the buffers are written again
    if (c0 == 0 && tile0 == 0) tr_mark(tr, wv, 5);
    if (!cons_barrier(wv)) return wv.st;
  }
  return wv.st;
}

// All passes of one GEMM for this CU.  p.sbase: stream index of the GEMM's first fragment.
template <int MT>
__device__ __forceinline__ WaveState gemm_phase(PassArgs p, WaveState st, const GemmDev &g, unsigned lds0, int w) {
  const int nt = uni(my_tiles(g.ntiles));
  p.KT = g.KT;
  int part = 0;
  for (int t0 = 0; t0 < nt; t0 += g.ntp) {
    const int n = nt - t0 < g.ntp ? nt - t0 : g.ntp;
    p.part0 = part;
    p.tile0 = t0;
    lds_put(lds0 + LDS_ARGS + 128 * w, p);  // every lane stores the same values
    switch (n) {
      case 1: st = gemm_pass<MT, 1>(lds0, st); break;
      case 2: st = gemm_pass<MT, 2>(lds0, st); break;
      case 3: st = gemm_pass<MT, 3>(lds0, st); break;
      case 4: st = gemm_pass<MT, 4>(lds0, st); break;
      case 5: st = gemm_pass<MT, 5>(lds0, st); break;
      case 6: st = gemm_pass<MT, 6>(lds0, st); break;
      case 7: st = gemm_pass<MT, 7>(lds0, st); break;
      default: st = gemm_pass<MT, 8>(lds0, st); break;
    }
    st.ok = uni(st.ok);
    if (!st.ok) return st;
    p.sbase += (unsigned)(n * g.KT);
    constexpr int tpc_max = RED_TILES / MT;
    part += (n + tpc_max - 1) / tpc_max;
  }
  return st;
}

// ---- first operand of a launch: norm statistics and fragments of x * gain ----------------------
// One thread per (row, 8 columns).  Sums of squares are kept per 16 columns, the granularity of
// the GEMM epilogues that produce them in later phases.
// This workgroup's columns of x (column tiles blockIdx.x, blockIdx.x + G, ...) into LDS_X.
__device__ __forceinline__ void x_stage(const StackArgs &a, const Wave &wv, unsigned lds0, int nt_x) {
  const int rows = 16 * a.MT;
  for (int it = wv.w * 64 + wv.lane; it < nt_x * a.Bp * 4; it += CONS_THREADS) {
    const int part = it & 3, bt = it >> 2, tt = bt / a.Bp, b = bt - tt * a.Bp;
    const int col = 16 * ((int)blockIdx.x + (int)gridDim.x * tt) + 4 * part;
    *(LDS_AS f32x4 *)(uintptr_t)(lds0 + LDS_X + ((tt * rows + b) * 16 + 4 * part) * 4) =
        *reinterpret_cast<const f32x4 *>(a.x + (size_t)b * a.d + col);
  }
}

// The gains of this workgroup's x columns into LDS_GAIN, straight from memory into LDS: issued by
// wave 0 before its GEMM pass, landed long before the epilogue reads them (a wave's loads return
// in order, and wave 0 has waited for its operand loads by then).
__device__ __forceinline__ void gain_stage(const float *gain, const Wave &wv, unsigned lds0, int nt_x) {
  if (wv.w != 0 || gain == nullptr) return;
  const int tt = wv.lane >> 4;
  const unsigned vo = tt < nt_x ? (unsigned)((16 * ((int)blockIdx.x + (int)gridDim.x * tt) + (wv.lane & 15)) * 4) : OOB;
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_of(gain), (LDS_AS void *)(uintptr_t)(lds0 + LDS_GAIN), 4, vo, 0, 0, 0);
}

__device__ __forceinline__ void prep_phase(const StackArgs &a, const Wave &wv, const float *gain, uint16_t *xa_out, float *rsq_out) {
  __amdgpu_buffer_rsrc_t rq = rsrc_of(rsq_out), rx = rsrc_of(xa_out);
  const int octs = a.d >> 3, total = a.Bp * octs;
  for (int it = blockIdx.x * CONS_THREADS + wv.w * 64 + wv.lane; it < total; it += gridDim.x * CONS_THREADS) {
    const int r = it / octs, oct = it - r * octs, c0 = oct * 8;
    const f32x4 *xp = reinterpret_cast<const f32x4 *>(a.x + (size_t)r * a.d + c0);
    f32x4 x0 = xp[0], x1 = xp[1];
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
    sq += __shfl_xor(sq, 1, 64);  // octs is even: both octets of a 16-column group sit in one wave
    if ((oct & 1) == 0) st32f(rq, (unsigned)(r * a.ncg + (oct >> 1)) * 4, sq);
    const float *gp = gain + c0;
    u32x4 v = {pack_f16(x0[0] * gp[0], x0[1] * gp[1]), pack_f16(x0[2] * gp[2], x0[3] * gp[3]),
               pack_f16(x1[0] * gp[4], x1[1] * gp[5]), pack_f16(x1[2] * gp[6], x1[3] * gp[7])};
    st128(rx, frag_piece(c0, r, a.MT), v);
  }
}

// cos/sin of pos[b] * theta^(-2i/dh) in double (exact to float rounding at any cache position)
__device__ __forceinline__ void rope_table_phase(const StackArgs &a, const Wave &wv) {
  __amdgpu_buffer_rsrc_t rc = rsrc_of(a.cs);
  int half = a.dh >> 1, total = a.Bp * half;
  for (int e = blockIdx.x * CONS_THREADS + wv.w * 64 + wv.lane; e < total; e += gridDim.x * CONS_THREADS) {
    int b = e / half, i = e - b * half;
    double inv = exp2(-(double)i / (double)half * log2(a.theta));
    double s, c;
    sincos((double)a.pos[b] * inv, &s, &c);
    st32f(rc, (unsigned)e * 8, (float)c);
    st32f(rc, (unsigned)e * 8 + 4, (float)s);
  }
}

// ---- masked-block GQA attention ------------------------------------------------------------------
// Unit = (kv head, tile of 16 q-rows of the head's group); one workgroup per unit.  The seven
// consumer waves split the key blocks (of 32 keys) round-robin, each keeps a running max / sum
// and an unnormalised output, and the seven are merged in the same fixed tree as the GEMMs.
// Scores are computed transposed (keys x q-rows) so that the probabilities leave the MFMA in the
// operand layout of the second product:
//   S^T = K Q^T      A = K tile [16 keys x 32 dh],   B = q fragment        -> lane: 4 keys of one q-row
//   O^T = V^T P^T    A = V^T tile [16 dh x 32 keys], B = p of 2 key tiles  -> lane: 4 channels of one q-row
// V is stored key-blocked (v_index) so that the V^T tile is one 128-bit load per lane.
struct AttArgs {
  const uint16_t *Kc, *Vc;
  uint16_t *attn_out;
  const uint64_t *vis;
  unsigned lds0;
  int u0;  // this workgroup's first unit (the next ones follow at gridDim.x)
  unsigned long long *tr;
};

// Which workgroups run the attention units.  When the QKV tiles do not divide evenly, the
// workgroups behind the first (ntiles mod G) have one tile fewer and reach the end of the QKV
// phase early: if there are enough of them they take the units (and warm the cache for them
// meanwhile, see kv_touch).  Returns the workgroup of unit 0.
__device__ __forceinline__ int att_first_wg(int qkv_tiles, int n_units) {
  const int G = gridDim.x, heavy = qkv_tiles % G;
  return G - heavy >= n_units ? heavy : 0;
}

// Requests the cache lines of the committed K, V rows of one kv head that this unit's share
// covers: key blocks that end at or before row L, which the attention then reads with ordinary
// loads and finds in the XCD's L2 (all units of a kv head sit on one XCD).  Issued when the
// workgroup has finished its QKV tiles; the lines travel while it waits at the barrier.  One
// 4-byte load per 128-byte line into a sink in LDS: nothing is kept.
__device__ __forceinline__ void kv_touch(const uint16_t *Kc, const uint16_t *Vc, int u, int n_rt, int Hkv, int dh, int L, const Wave &wv,
                                         unsigned lds0) {
  const int rt = u / Hkv, kvh = u - rt * Hkv;
  const int kb_split = L >> 5;
  const int k_lines_row = dh >> 6, v_lines_blk = dh >> 1;  // 128-byte lines per K row of a head / per V key block of a head
  if (k_lines_row == 0) return;                            // (head_dim 64 and 128 only reach here)
  const int nlk = kb_split * 32 * k_lines_row, nl = nlk + kb_split * v_lines_blk;
  __amdgpu_buffer_rsrc_t rk = rsrc_of(Kc), rv = rsrc_of(Vc);
  LDS_AS void *sink = (LDS_AS void *)(uintptr_t)(lds0 + LDS_SINK);
  for (int t0 = (rt * NCW + wv.w) * 64; t0 < nl; t0 += n_rt * NCW * 64) {
    const int t = t0 + wv.lane;
    unsigned ko = OOB, vo = OOB;
    if (t < nlk) {
      const int row = t / k_lines_row, part = t - row * k_lines_row;
      ko = (unsigned)((((size_t)row * Hkv + kvh) * dh) * 2 + part * 128);
    } else if (t < nl) {
      const int j = t - nlk, kb = j / v_lines_blk, l = j - kb * v_lines_blk;
      vo = (unsigned)((((size_t)kb * Hkv + kvh) * dh * 32) * 2 + l * 128);
    }
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, sink, 4, ko, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, sink, 4, vo, 0, 0, 0);
  }
}

template <int DH>
__device__ __attribute__((noinline)) WaveState attention_phase(AttArgs p, WaveState st_in) {
  constexpr int KT = DH / 32, DT = DH / 16;
  static_assert(DT <= RED_TILES, "one wave's output must fit a reduction buffer");
  struct {
    int Bp, MT, Hq, Hkv;
    const uint64_t *vis;
  } a;
  const unsigned lds0 = uni(p.lds0);
  const LaunchConst lc = launch_const(lds0);
  a.Bp = lc.Bp; a.MT = lc.MT; a.Hq = lc.Hq; a.Hkv = lc.Hkv; a.vis = uni_ptr(p.vis);
  const int L = lc.L;
  unsigned long long *tr = uni_ptr(p.tr);
  Wave wv;
  wv.w = uni((int)(threadIdx.x >> 6));
  wv.lane = threadIdx.x & 63;
  wv.ctl = lds0 + LDS_CTL;
  wv.st.cbar_seq = uni(st_in.cbar_seq);
  wv.st.tree_seq = uni(st_in.tree_seq);
  wv.st.seen = uni(st_in.seen);
  wv.st.ok = 1;
  __amdgpu_buffer_rsrc_t rk = rsrc_of(p.Kc), rv = rsrc_of(p.Vc), rqf = rsrc_of(lc.qf), ra = rsrc_of(p.attn_out);
  LDS_AS f32x4 *red = (LDS_AS f32x4 *)(uintptr_t)(lds0 + LDS_RED);
  LDS_AS float *mlb = (LDS_AS float *)(uintptr_t)(lds0 + LDS_ML);
  const int w = wv.w, lane = wv.lane, q4 = lane >> 4, c16 = lane & 15;
  const int g = a.Hq / a.Hkv, n_rt = g * a.MT;
  const int total = L + a.Bp, nkb = (total + 31) >> 5;
  for (int u = uni(p.u0); u < a.Hkv * n_rt; u += gridDim.x) {
    // kv head = unit mod Hkv: consecutive workgroups sit on different XCDs, so with eight kv heads
    // all units of a head share one XCD's L2 and its K, V are fetched from memory once
    const int kvh = u / n_rt, rt = u - kvh * n_rt;
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
    // Key blocks that end at or before row L ("early") were written by earlier launches:
    // ordinary cached loads (they hit in L2 when warmed, see kv_touch), and every key is visible.
    // A block that holds rows of this step ("late") was written by other workgroups in the phase
    // before: device-scope loads, and the mask applies.  A wave takes its late block first (there
    // are at most three, dealt to the waves from the last one down), then its early blocks
    // w, w + 7, ...  One register set for K and one for V: the next block's K is requested as soon
    // as the scores are out of the matrix unit and travels during the softmax and P V; the next V
    // follows P V and travels during the next scores.  Every load in the loop is of the same kind
    // and unconditional (a block beyond the last is requested out of range: nothing moves), so
    // the count of outstanding loads stays exact; and the function stays within the registers
    // that a callee may use without saving them.
    u32x4 ka[KT], kb2[KT], vt[DT];
    auto load_k = [&](auto policy, int kb, bool valid) {
      constexpr int POL = decltype(policy)::value;
      const unsigned k_off = valid ? (unsigned)((((size_t)(kb * 32 + c16) * a.Hkv + kvh) * DH + 8 * q4) * 2) : OOB;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        ka[kt] = ld128p<POL>(rk, k_off + kt * 64);
        kb2[kt] = ld128p<POL>(rk, k_off + (unsigned)(16 * a.Hkv * DH * 2) + kt * 64);
      }
    };
    auto load_v = [&](auto policy, int kb, bool valid) {
      constexpr int POL = decltype(policy)::value;
      const unsigned v_off = valid ? (unsigned)(((((size_t)kb * a.Hkv + kvh) * DH + c16) * 32 + 8 * q4) * 2) : OOB;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) vt[dt] = ld128p<POL>(rv, v_off + dt * 16 * 32 * 2);
    };
    // scores of the block in ka / kb2: lane holds keys kb*32 + 4 q4 + i (sv[0..3]) and
    // kb*32 + 16 + 4 q4 + i (sv[4..7]) of q-row c16
    auto scores = [&](float *sv) {
      f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kt]), q[kt], sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb2[kt]), q[kt], sb, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) sv[i] = i < 4 ? sa[i] : sb[i - 4];
    };
    // running softmax over the block's scores; returns the probabilities as a matrix operand
    auto softmax = [&](auto masked, const float *sv, int kb, float &corr) {
      constexpr bool MASKED = decltype(masked)::value;
      bool ok[8];
      float mx = -1e30f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (MASKED) {
          const int key = kb * 32 + (i >> 2) * 16 + 4 * q4 + (i & 3);
          ok[i] = key < L || (key < total && ((vb >> (key - L)) & 1ull));
          if (ok[i]) mx = fmaxf(mx, sv[i]);
        } else {
          ok[i] = true;
          mx = fmaxf(mx, sv[i]);
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      corr = __expf(m_run - m_new);
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
      const u32x4 pw = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
      return __builtin_bit_cast(bf16x8, pw);
    };
    auto pv = [&](bf16x8 pb, float corr) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        o[dt] *= corr;
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[dt]), pb, o[dt], 0, 0, 0);
      }
    };
    static_assert(LA_MAX_ROWS <= 64, "at most three late key blocks: one per wave");
    const std::integral_constant<int, 0> plain{};
    const std::integral_constant<int, DEV> coherent{};
    const int kb_split = L >> 5;                // early blocks: 0 .. kb_split - 1
    const int late = kb_split + (NCW - 1 - w);  // this wave's late block, if it exists
    const bool has_late = late < nkb;
    const bool any = has_late || w < kb_split;
    int kb = has_late ? late : w;               // the block in the registers
    int ne = has_late ? w : w + NCW;            // the next early block to request
    if (has_late) {
      load_k(coherent, late, true);
      load_v(coherent, late, true);
    } else {
      load_k(plain, w, w < kb_split);
      load_v(plain, w, w < kb_split);
    }
    tr_mark_wave(tr, wv, 16);  // loads issued
    if (tr) {
      wait_vmcnt<DT>();
      tr_mark(tr, wv, 9);
      tr_mark_wave(tr, wv, 24);  // first K tiles (and q) landed
    }
    unsigned long long n_iter = 0;
    const unsigned long long t_loop = tr ? wall_clock64() : 0ull;
    if (any) {
      float sv[8], corr;
      scores(sv);
      load_k(plain, ne, ne < kb_split);
      const bf16x8 pb = has_late ? softmax(std::true_type{}, sv, kb, corr) : softmax(std::false_type{}, sv, kb, corr);
      pv(pb, corr);
      load_v(plain, ne, ne < kb_split);
      ++n_iter;
      while (ne < kb_split) {
        kb = ne;
        ne += NCW;
        scores(sv);
        load_k(plain, ne, ne < kb_split);
        const bf16x8 pb2 = softmax(std::false_type{}, sv, kb, corr);
        pv(pb2, corr);
        load_v(plain, ne, ne < kb_split);
        ++n_iter;
      }
    }
    tr_mark(tr, wv, 10);
    tr_mark_wave(tr, wv, 32);  // key blocks done
    if (tr && w == 0 && lane == 0) {
      tr[13] = 0;
      tr[14] = n_iter;
      tr[15] = wall_clock64() - t_loop;
    }
    // merge the seven partial results: ((w0 + w4) + (w2 + w6)) + (w3 + (w1 + w5))
    auto put = [&](int buf) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) red[(buf * RED_TILES + dt) * 64 + lane] = o[dt];
      mlb[(buf * 64 + lane) * 2] = m_run;
      mlb[(buf * 64 + lane) * 2 + 1] = l_run;
    };
    auto merge = [&](int buf) {
      float mo = mlb[(buf * 64 + lane) * 2], lo = mlb[(buf * 64 + lane) * 2 + 1];
      float m_new = fmaxf(m_run, mo);
      float ca = __expf(m_run - m_new), cb = __expf(mo - m_new);
      l_run = l_run * ca + lo * cb;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = o[dt] * ca + red[(buf * RED_TILES + dt) * 64 + lane] * cb;
      m_run = m_new;
    };
    const unsigned qs = wv.st.tree_seq;
    auto signal = [&](unsigned v) {
      if (lane == 0) ctl_write(wv.ctl + 4 * (C_TREE + w), v);
    };
    if (w >= 4) { put(w - 4); signal(qs + 1); }
    if (w < 3) { if (!ctl_wait_ge(wv, C_TREE + w + 4, qs + 1)) return wv.st; merge(w); }
    if (w == 2) { put(2); signal(qs + 2); }
    if (w == 1) { put(1); signal(qs + 2); }
    if (w == 0) { if (!ctl_wait_ge(wv, C_TREE + 2, qs + 2)) return wv.st; merge(2); }
    if (w == 3) { if (!ctl_wait_ge(wv, C_TREE + 1, qs + 2)) return wv.st; merge(1); put(1); signal(qs + 3); }
    if (w == 0) {
      if (!ctl_wait_ge(wv, C_TREE + 3, qs + 3)) return wv.st;
      merge(1);
      tr_mark(tr, wv, 11);
      // o[dt][i] = O^T[channel 16 dt + 4 q4 + i][q-row c16]: four channels = half a 16-byte piece
      if (b < a.Bp) {
        const float inv = 1.0f / l_run;
        const int j = rt / a.MT;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          int col = (kvh * g + j) * DH + 16 * dt + 8 * (q4 >> 1);
          st64(ra, frag_piece(col, b, a.MT) + 8 * (q4 & 1),
               u32x2{pack_f16(o[dt][0] * inv, o[dt][1] * inv), pack_f16(o[dt][2] * inv, o[dt][3] * inv)});
        }
      }
      signal(qs + 4);
    }
    wv.st.tree_seq = qs + 4;
    // the buffers are free again once wave 0 has read the last of them
    if (!ctl_wait_ge(wv, C_TREE + 0, qs + 4)) return wv.st;
  }
  return wv.st;
}

// Arg-max over the partial records; logits carry the row's norm factor from here on.
// One wave per row.
__device__ __forceinline__ void unembed_final_phase(const StackArgs &a, const Wave &wv) {
  __amdgpu_buffer_rsrc_t ru = rsrc_of(a.un_part);
  const int n_part = gridDim.x * a.un_parts_per_cu;
  for (int b = blockIdx.x * NCW + wv.w; b < a.Bp; b += gridDim.x * NCW) {
    Top best{-INFINITY, 0x7fffffff, -INFINITY};
    // eight records per lane and turn, all requested before the first is merged (a record beyond
    // the last is requested out of range and reads as zeros: it is skipped)
    for (int s0 = wv.lane; s0 < n_part; s0 += 64 * 8) {
      Top c[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int s = s0 + 64 * j;
        const unsigned o = s < n_part ? (unsigned)(((size_t)s * 64 + b) * sizeof(Top)) : OOB;
        c[j] = Top{ld32f(ru, o), (int)__builtin_amdgcn_raw_buffer_load_b32(ru, o + 4, 0, DEV), ld32f(ru, o + 8)};
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (s0 + 64 * j < n_part) best = top_merge2(best, c[j]);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      Top other;
      other.v1 = __shfl_xor(best.v1, o, 64);
      other.i1 = __shfl_xor(best.i1, o, 64);
      other.v2 = __shfl_xor(best.v2, o, 64);
      best = top_merge2(best, other);
    }
    float s = 0.f;
    for (int c = wv.lane; c < a.ncg; c += 64) s += ld32f(rsrc_of(a.rsq), (unsigned)((size_t)b * a.ncg + c) * 4);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (wv.lane == 0) {
      float rsf = 1.0f / sqrtf(s * a.inv_d + a.eps);
      a.ids[b] = best.i1;
      if (a.top2) {
        a.top2[b * 2] = best.v1 * rsf;
        a.top2[b * 2 + 1] = best.v2 * rsf;
      }
    }
  }
}

// ---- the persistent kernel ------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(WG_THREADS) void stack_kernel(StackArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds_generic[];
  const lds_t lds = (lds_t)lds_generic;
  const int L = uni(*a.L_dev);
  if (L < 0 || L + a.Bp > a.max_len) {  // every workgroup takes the same exit: no barrier is left waiting
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_error(a, 1);
    return;
  }
  if (threadIdx.x < 64) ((LDS_AS unsigned *)(lds + LDS_CTL))[threadIdx.x] = 0u;
  if (threadIdx.x == 64) {
    LDS_AS LaunchConst *c = (LDS_AS LaunchConst *)(lds + LDS_CONST);
    c->Bp = a.Bp; c->MT = MT; c->d = a.d; c->ncg = a.ncg; c->Hq = a.Hq; c->Hkv = a.Hkv; c->dh = a.dh; c->L = L; c->dbg = LA_DBG_BITS(a.dbg);
    c->x_lds = (a.mode == 0 && my_tiles(a.o.ntiles) * MT <= X_TILES && !(LA_DBG_BITS(a.dbg) & 128)) ? 1 : 0;
    c->inv_d = a.inv_d; c->eps = a.eps; c->x = a.x; c->cs = a.cs; c->qf = a.qf;
  }
  __syncthreads();  // the only hardware barrier: from here on the waves run decoupled
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned ctl = (unsigned)(uintptr_t)(lds + LDS_CTL);

  // this CU's share of each GEMM, in fragments
  const unsigned f_qkv = (unsigned)(my_tiles(a.qkv.ntiles) * a.qkv.KT), f_o = (unsigned)(my_tiles(a.o.ntiles) * a.o.KT);
  const unsigned f_gu = (unsigned)(my_tiles(a.gu.ntiles) * a.gu.KT), f_down = (unsigned)(my_tiles(a.down.ntiles) * a.down.KT);
  const unsigned f_layer = (f_qkv + f_o + f_gu + f_down + CHUNK - 1) / CHUNK * CHUNK;  // padded to whole chunks
  const unsigned f_un = ((unsigned)(my_tiles(a.un.ntiles) * a.un.KT) + CHUNK - 1) / CHUNK * CHUNK;

  if (wave == NCW) {
    __builtin_amdgcn_s_setprio(3);  // the producer's few instructions go first on its SIMD (4 % on a one-row step)
    unsigned long long *st = LA_TRACE_PTR(a) ? LA_TRACE_PTR(a) + TRACE_SLOTS * a.trace_phases + TRACE_WG * blockIdx.x : nullptr;
    // (timeline: producer snapshots at the start and the end of the second layer's gate / up weights)
    // (timeline: which of the second layer's four weight matrices the snapshots cover: 0 QKV, 1 O, 2 gate / up, 3 down)
    const unsigned seg0 = a.trace_seg == 0 ? 0u : a.trace_seg == 1 ? f_qkv : a.trace_seg == 3 ? f_qkv + f_o + f_gu : f_qkv + f_o;
    const unsigned seg_n = a.trace_seg == 0 ? f_qkv : a.trace_seg == 1 ? f_o : a.trace_seg == 3 ? f_down : f_gu;
    const unsigned gu0 = f_layer + seg0;
    const unsigned first_seg = a.mode == 0 ? (unsigned)a.lb : 0u, n_seg = a.mode == 0 ? (unsigned)(a.le - a.lb) : 1u;
    const unsigned seg_used = a.mode == 0 ? f_layer : f_un;
    if (st) producer<true>(a, ctl, lds + LDS_RING, first_seg, n_seg, seg_used, a.seg_frags, st, a.mode == 0 ? gu0 : ~0u, a.mode == 0 ? gu0 + seg_n : ~0u);
    else producer<false>(a, ctl, lds + LDS_RING, first_seg, n_seg, seg_used, a.seg_frags, nullptr, ~0u, ~0u);
    return;
  }

  Wave wv;
  wv.ctl = ctl;
  wv.w = wave;
  wv.lane = threadIdx.x & 63;
  wv.st.cbar_seq = 0;
  wv.st.tree_seq = 0;
  wv.st.seen = 0;
  wv.st.ok = 1;
  unsigned epoch = a.epoch0;
  const unsigned lds0 = (unsigned)(uintptr_t)lds;

  // Phase list.  Layer stack: PREP, then per layer QKV, ATT, O, GU, DOWN.  Unembedding: PREP,
  // GEMM, FINAL.  The GEMM passes and the attention are functions of their own; this loop only
  // sets up their arguments and runs the grid barrier between phases.
  const int n_phases = a.mode == 1 ? 3 : 1 + 5 * (a.le - a.lb);
  const bool x_lds = launch_const(lds0).x_lds != 0;
  const int n_rt = a.Hq / a.Hkv * MT, n_units = a.Hkv * n_rt;
  const int att_first = (LA_DBG_BITS(a.dbg) & 32) ? 0 : att_first_wg(a.qkv.ntiles, n_units);
  const int att_u0 = (int)blockIdx.x >= att_first ? (int)blockIdx.x - att_first : n_units;  // no unit: n_units
  unsigned sbase = 0;
  unsigned long long *tr = nullptr;  // timeline slots of the current phase (workgroup 0 only)
  for (int ph = 0; ph < n_phases; ++ph) {
    if (ph > 0) {
      const int k = ph - 1 - a.trace_sel;
      if (LA_TRACE_PTR(a) && k >= 0 && k < 8 && wv.w == 0 && wv.lane == 0)
        LA_TRACE_PTR(a)[(size_t)TRACE_SLOTS * a.trace_phases + TRACE_WG * blockIdx.x + 8 + k] = wall_clock64();
      if (!grid_sync(a, wv, ++epoch, tr)) return;
    }
    tr = (LA_TRACE_PTR(a) && blockIdx.x == 0 && ph < a.trace_phases) ? LA_TRACE_PTR(a) + TRACE_SLOTS * ph : nullptr;
    tr_mark(tr, wv, 0);
    if (tr && wv.w == 0 && wv.lane == 0) tr[12] = clock64();  // shader clock, to report the running frequency
    const int sub = a.mode == 1 ? (ph == 0 ? 0 : ph == 1 ? 6 : 7) : (ph == 0 ? 0 : 1 + (ph - 1) % 5);
    const int layer = a.mode == 1 ? 0 : (ph == 0 ? a.lb : a.lb + (ph - 1) / 5);
    uint16_t *Kc = a.K + (size_t)layer * a.layer_elems, *Vc = a.V + (size_t)layer * a.layer_elems;
    // write-once buffers of this layer: fragments of the attn-norm and mlp-norm inputs with
    // their statistics, the attention output, the SwiGLU output
    uint16_t *xa0 = a.xa + (size_t)(2 * layer) * a.xa_stride, *xa1 = xa0 + a.xa_stride;
    float *rsq0 = a.rsq + (size_t)(2 * layer) * a.rsq_stride, *rsq1 = rsq0 + a.rsq_stride;
    uint16_t *attn_l = a.attn_a + (size_t)layer * a.attn_stride, *act_l = a.act_a + (size_t)layer * a.act_stride;
    PassArgs p{};
    p.tr = tr;

    GemmDev g{};
    bool have_g = false;
    unsigned frags = 0;
    switch (sub) {
      case 0:  // first operand of the launch
        if (a.mode == 1) {
          prep_phase(a, wv, a.g_final, a.xa, a.rsq);
        } else {
          prep_phase(a, wv, a.gains[layer].g_attn, xa0, rsq0);
          rope_table_phase(a, wv);
          if (x_lds) x_stage(a, wv, lds0, my_tiles(a.o.ntiles));
        }
        break;
      case 1:
        p.A = xa0; p.mode = MODE_QKV; p.rsq_in = rsq0; p.q.Kc = Kc; p.q.Vc = Vc;
        g = a.qkv; have_g = true; frags = f_qkv;
        break;
      case 2:
        if (att_u0 < n_units || (LA_DBG_BITS(a.dbg) & 64)) {  // (a call costs the callee's register saves: only where there is work)
          AttArgs t;
          t.Kc = Kc; t.Vc = Vc; t.attn_out = attn_l; t.vis = a.vis; t.lds0 = lds0; t.u0 = att_u0;
          // (the timeline shows the attention of the workgroup that runs unit 0)
          t.tr = (LA_TRACE_PTR(a) && att_u0 == 0 && ph < a.trace_phases) ? LA_TRACE_PTR(a) + TRACE_SLOTS * ph : nullptr;
          wv.st = a.dh == 128 ? attention_phase<128>(t, wv.st) : attention_phase<64>(t, wv.st);
          wv.st.ok = uni(wv.st.ok);
          if (!wv.st.ok) return;
        }
        break;
      case 3:
        p.A = attn_l; p.mode = MODE_RESID; p.q.gain = a.gains[layer].g_mlp; p.q.xa_out = xa1; p.q.rsq_out = rsq1;
        g = a.o; have_g = true; frags = f_o;
        if (x_lds) gain_stage(p.q.gain, wv, lds0, my_tiles(a.o.ntiles));
        break;
      case 4:
        p.A = xa1; p.mode = MODE_GATEUP; p.rsq_in = rsq1; p.q.act_a = act_l;
        g = a.gu; have_g = true; frags = f_gu;
        break;
      case 5:
        // the fragments feed the next layer's QKV GEMM; the last layer of the call needs none
        p.A = act_l; p.mode = MODE_RESID;
        p.q.gain = layer + 1 < a.le ? a.gains[layer + 1].g_attn : nullptr;
        p.q.xa_out = xa0 + 2 * a.xa_stride; p.q.rsq_out = rsq0 + 2 * a.rsq_stride;
        g = a.down; have_g = true; frags = f_layer - f_qkv - f_o - f_gu;  // with the layer's padding
        if (x_lds) gain_stage(p.q.gain, wv, lds0, my_tiles(a.o.ntiles));
        break;
      case 6: {
        // every CU writes all of its partial records: the ones it has no tiles for stay empty
        __amdgpu_buffer_rsrc_t rp = rsrc_of(a.un_part);
        constexpr int tpc_max = RED_TILES / MT;
        int nt = my_tiles(a.un.ntiles), used = 0;
        for (int t0 = 0; t0 < nt; t0 += a.un.ntp) used += ((nt - t0 < a.un.ntp ? nt - t0 : a.un.ntp) + tpc_max - 1) / tpc_max;
        for (int it = wv.w * 64 + wv.lane; it < (a.un_parts_per_cu - used) * 64; it += CONS_THREADS) {
          unsigned o = (unsigned)(((size_t)(blockIdx.x * a.un_parts_per_cu + used + (it >> 6)) * 64 + (it & 63)) * sizeof(Top));
          st32f(rp, o, -INFINITY);
          __builtin_amdgcn_raw_buffer_store_b32(0x7fffffffu, rp, o + 4, 0, DEV);
          st32f(rp, o + 8, -INFINITY);
        }
        p.A = a.xa; p.mode = MODE_UNEMBED; p.q.un_part = a.un_part + (size_t)blockIdx.x * a.un_parts_per_cu * 64;
        g = a.un; have_g = true; frags = f_un;
        break;
      }
      default:
        unembed_final_phase(a, wv);
        break;
    }
    if (have_g) {
      p.sbase = sbase;
      wv.st = gemm_phase<MT>(p, wv.st, g, lds0, wv.w);
      if (!wv.st.ok) return;
      sbase += frags;
      if (sub == 1 && !(LA_DBG_BITS(a.dbg) & 16))
        for (int u = att_u0; u < n_units; u += gridDim.x) kv_touch(Kc, Vc, u, n_rt, a.Hkv, a.dh, L, wv, lds0);
    }
    tr_mark(tr, wv, 2);
  }
}

// Launches the persistent kernel for MT row tiles (explicitly instantiated in la_stack_mt*.hip,
// one translation unit per MT so that they compile in parallel).
// Run once per model: raises the kernel's LDS limit and checks that n_wgs workgroups can be resident at once.
template <int MT>
int prepare_stack_kernel(int n_wgs, int cus) {
  LA_HIP(hipFuncSetAttribute((const void *)stack_kernel<MT>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
  int per_cu = 0;
  LA_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stack_kernel<MT>, WG_THREADS, LDS_BYTES));
  LA_REQUIRE(per_cu >= 1 && n_wgs <= per_cu * cus, LA_EINVAL,
             "the persistent kernel for %d row tiles cannot keep %d workgroups resident (%d per compute unit on %d units)", MT, n_wgs,
             per_cu, cus);
  return LA_OK;
}

template <int MT>
int launch_stack_kernel(const StackArgs &a, int n_wgs, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    LA_HIP(hipFuncSetAttribute((const void *)stack_kernel<MT>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
    attr_set = true;
  }
  stack_kernel<MT><<<n_wgs, WG_THREADS, LDS_BYTES, s>>>(a);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

}  // namespace la
