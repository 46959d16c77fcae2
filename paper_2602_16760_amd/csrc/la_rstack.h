// MFMA path for gfx950 (bf16 models), second generation: the whole layer stack of a verification
// step as ONE persistent kernel whose weight stream lives in REGISTERS.
//
// A step reads every weight once and computes almost nothing per byte, so it is bound by HBM --
// if the memory never has to wait for the chain of small dependent steps (load the activations,
// multiply, reduce, epilogue, publish, grid barrier) that separates one GEMM from the next.
// The design keeps that chain short and the weights decoupled from it:
//
//   * One workgroup of 8 waves per CU stays resident.  Waves 0..NW-1 are MFMA WAVES.  Each owns a
//     private, contiguous stream of weight fragments (every NW-th k-tile of the CU's column
//     tiles, in the order it will use them, across GEMMs and layers) and keeps the next D = 32
//     fragments of it (24 and 16 for blocks of 48 and 64 rows, whose accumulators need the
//     registers) in flight or landed in its own registers (buffer_load_dwordx4 ... nt, one
//     s_waitcnt vmcnt(D-1) per use: the wave touches memory for nothing else, so the counter
//     counts weight fragments only).  A fragment is re-requested the moment the matrix unit has
//     read it, whatever GEMM the next fragment belongs to: the streams run ahead across every
//     epilogue and grid barrier by NW x 32 KB per CU.
//   * Waves NW..7 are IO WAVES.  They own everything that depends on other workgroups: the grid
//     barrier, the activation operand (copied L2 -> LDS with direct-to-LDS loads, k-tile by
//     k-tile, into a small ring per MFMA wave), the reduction of the MFMA waves' partial tiles,
//     the epilogues (RoPE + KV write, residual + statistics, SwiGLU, arg-max), the attention.
//   * An MFMA wave never waits for memory latency of activations: it polls an LDS counter for its
//     next k-tile of operand, reads it with ds_read_b128 and multiplies.  When its k-tiles of a
//     pass are done it leaves its partial tile in LDS (in the space of its idle operand ring)
//     and goes on to the next pass, where it blocks until the IO waves have been through the
//     barrier and deliver the first operand k-tile -- with its registers full of the next
//     weights.
//
// Data layout
//   weights      per CU, per layer, per GEMM, per MFMA wave w: [k-tile w, w+NW, ...][this CU's column
//                tiles][lane][8] halves (a pass takes a run of <= NTMAX tiles out of every k-tile's
//                row; with one pass per GEMM, the usual case, the wave's stream is contiguous).
//                Column tile t (16 columns) of a GEMM belongs to CU t mod G.  A fragment (1 KB) is the MFMA B operand of one
//                k-tile (32 deep) x 16 columns: lane l holds column (l & 15), contraction indices
//                8 (l >> 4) .. +7.
//   activations  as in la_stack.h: [k-tile][row tile][lane][8] halves, the MFMA A operand, in
//                write-once buffers; RMSNorm applied as a row factor after the contraction.
// All reductions have a fixed order (partials of wave 0, 1, ... are added in that order).
#pragma once
#include "la_stack.h"

namespace la {
namespace rs {

constexpr int RING_MAX = 32;  // most weight fragments per MFMA wave in flight or landed (4 VGPRs each; Geo<MT>::RING)

template <int MT>
struct Geo {
  static constexpr int NTMAX = 8;                                     // column tiles per pass
  // Weight fragments per MFMA wave in flight or landed.  Up to 32 rows a wave's registers hold 32 of them beside the
  // accumulators of eight column tiles; with 48 and 64 rows they hold 24 and 16 (the depth matters little: 16 instead
  // of 32 cost 0.9 % at 32 rows), so that gate/up (seven tiles per workgroup at the 7B shape) stays one pass.
  static constexpr int RING = MT <= 2 ? 32 : MT == 3 ? 24 : 16;
  static constexpr int LDTMAX = 16 * NTMAX + 4;                       // padded row length of a partial tile (floats)
  static constexpr int PART_BYTES = 16 * MT * LDTMAX * 4;             // one wave's partial tile
};
// One MFMA wave's LDS region: its operand ring (RS k-tiles, a multiple of the loader's batch), which
// is also where it leaves its partial tile.  Sized so that NW regions fit beside the rest.
template <int MT, int NW>
struct Lay {
  static constexpr int RS = NW <= 4 ? (MT == 1 ? 32 : MT == 2 ? 16 : 8) : (MT == 1 ? 16 : MT == 2 ? 8 : 4);
  static constexpr int RING_BYTES = RS * MT * 1024;
  static constexpr int REG = ((Geo<MT>::PART_BYTES > RING_BYTES ? Geo<MT>::PART_BYTES : RING_BYTES) + 1023) / 1024 * 1024;
};

// LDS map: NW regions (operand ring / partial tile of each MFMA wave), then the small stuff.
constexpr int M_RS = 0;        // [64] row factors of the norm
constexpr int M_CTL = 256;     // control words
constexpr int M_CONST = 512;   // LaunchConst
constexpr int M_EPI = 640;     // EpiPtrs of the running pass
constexpr int M_SINK = 768;    // (spare)
constexpr int M_GAIN = 1024;   // norm gains of this workgroup's x columns
constexpr int M_X = 1280;      // this workgroup's columns of x: [column tile][row][16] floats
constexpr int X_BYTES = 4096;
constexpr int M_BYTES = M_X + X_BYTES;
template <int MT, int NW>
constexpr int lds_bytes() { return NW * Lay<MT, NW>::REG + M_BYTES + NW * (16 + 128 * 20) + 256; }    // (regions, small stuff, schedule tables, timeline of MFMA wave 0)

// control words (32-bit, at M_CTL)
constexpr int K_DEAD = 0;      // a wait timed out: every wave leaves the kernel
constexpr int K_IOBAR = 1;     // arrivals at the IO-wave barrier
constexpr int K_GPASS = 2;     // last grid-barrier epoch seen released
constexpr int K_SPARE = 3;
constexpr int K_ALAND = 8;     // [8..15] per MFMA wave: operand k-tiles landed in its ring (monotonic over the launch)
constexpr int K_ADONE = 16;    // [16..23] per MFMA wave: operand k-tiles it has read
constexpr int K_PDONE = 24;    // [24..31] per MFMA wave: passes whose partial tile is in LDS
constexpr int K_ATT = 32;      // [32..39] per IO wave: hand-off sequence of the attention merge

// One pass of one GEMM on this CU, as both kinds of waves see it.
struct Pass {
  int gemm;        // 0 QKV, 1 O, 2 gate / up, 3 down, 4 unembedding
  int layer;
  int KT, NT, NTS;  // k-tiles, column tiles, ring slots per k-tile (1, 2, 4 or 8 >= NT)
  int tile0, pidx;  // first local column tile, index of the pass in its GEMM
  int nt_all;       // column tiles of this CU in the GEMM (all passes)
  unsigned wbase;   // fragment index in this CU's stream of the GEMM's first fragment
};

__device__ __forceinline__ int slots_for(int nt) { return nt <= 1 ? 1 : nt <= 2 ? 2 : nt <= 4 ? 4 : 8; }
// k-tiles of one body of a pass with NTS slots per k-tile
__device__ __forceinline__ int body_rows(int NTS, int ring) { return ring / NTS; }

// Walks the passes of a launch in order (uniform values only; plain integers, picked by
// comparisons: an indexed array or a selected struct would live in scratch memory, and an MFMA
// wave must not touch memory for anything but its weights).
struct PassWalk {
  int mode, lb, le, G, cu, ntmax;
  int kt0, kt1, kt2, kt3, kt4;  // k-tiles of the five GEMMs
  int n0, n1, n2, n3, n4;       // their column tiles
  int c0, c1, c2, c3, c4;       // ... of which this CU's (computed once: a division each)
  int p0, p1, p2, p3, p4;       // tiles per pass (plan)
  unsigned seg_frags;
  // state
  int layer, gemm, t0, nt, pidx;
  unsigned gbase;  // fragment index of the current GEMM's first fragment
  bool done;
  Pass cur;

  __device__ __forceinline__ int kt_of(int gi) const { return gi == 0 ? kt0 : gi == 1 ? kt1 : gi == 2 ? kt2 : gi == 3 ? kt3 : kt4; }
  __device__ __forceinline__ int ntiles_of(int gi) const { return gi == 0 ? n0 : gi == 1 ? n1 : gi == 2 ? n2 : gi == 3 ? n3 : n4; }
  __device__ __forceinline__ int ntp_of(int gi) const {
    const int p = gi == 0 ? p0 : gi == 1 ? p1 : gi == 2 ? p2 : gi == 3 ? p3 : p4;
    return p < ntmax ? p : ntmax;
  }
  __device__ __forceinline__ int tiles_calc(int gi) const {
    const int n = ntiles_of(gi);
    return n > cu ? (n - cu + G - 1) / G : 0;
  }
  __device__ __forceinline__ int tiles_of(int gi) const { return gi == 0 ? c0 : gi == 1 ? c1 : gi == 2 ? c2 : gi == 3 ? c3 : c4; }
  __device__ __forceinline__ void init(const StackArgs &a, int ntmax_, bool one_layer = false) {
    mode = uni(a.mode); lb = uni(a.lb); le = one_layer ? lb + 1 : uni(a.le); G = uni((int)gridDim.x); cu = uni((int)blockIdx.x); ntmax = ntmax_;
    kt0 = uni(a.qkv.KT); kt1 = uni(a.o.KT); kt2 = uni(a.gu.KT); kt3 = uni(a.down.KT); kt4 = uni(a.un.KT);
    n0 = uni(a.qkv.ntiles); n1 = uni(a.o.ntiles); n2 = uni(a.gu.ntiles); n3 = uni(a.down.ntiles); n4 = uni(a.un.ntiles);
    p0 = uni(a.qkv.ntp); p1 = uni(a.o.ntp); p2 = uni(a.gu.ntp); p3 = uni(a.down.ntp); p4 = uni(a.un.ntp);
    seg_frags = uni(a.seg_frags);
    c0 = tiles_calc(0); c1 = tiles_calc(1); c2 = tiles_calc(2); c3 = tiles_calc(3); c4 = tiles_calc(4);
    layer = mode == 0 ? lb : 0;
    gemm = mode == 0 ? 0 : 4;
    done = false;
    gbase = mode == 0 ? (unsigned)layer * seg_frags : 0u;
    enter_gemm();
  }
  // positions on the first pass at or after (layer, gemm); sets done when there is none
  __device__ __forceinline__ void enter_gemm() {
    for (;;) {
      if (mode == 0 ? layer >= le : gemm > 4) { done = true; return; }
      nt = tiles_of(gemm);
      if (nt > 0) break;
      skip_gemm();
    }
    t0 = 0; pidx = 0;
    fill();
  }
  __device__ __forceinline__ void skip_gemm() {
    gbase += (unsigned)(tiles_of(gemm) * kt_of(gemm));
    if (mode != 0) { gemm = 5; return; }
    if (++gemm == 4) { gemm = 0; ++layer; gbase = (unsigned)layer * seg_frags; }
  }
  __device__ __forceinline__ void fill() {
    const int ntp = ntp_of(gemm);
    cur.gemm = gemm; cur.layer = layer; cur.KT = kt_of(gemm);
    cur.NT = nt - t0 < ntp ? nt - t0 : ntp;
    cur.NTS = slots_for(cur.NT);
    cur.tile0 = t0; cur.pidx = pidx; cur.nt_all = nt;
    cur.wbase = gbase;
  }
  __device__ __forceinline__ void next() {
    t0 += ntp_of(gemm); ++pidx;
    if (t0 < nt) { fill(); return; }
    skip_gemm();
    enter_gemm();
  }
};

// k-tiles of a GEMM with KT k-tiles that belong to MFMA wave w of NW: w, w + NW, ...
__device__ __forceinline__ int nk_of(int KT, int w, int NW) { return KT > w ? (KT - w + NW - 1) / NW : 0; }
// fragments of a GEMM that precede wave w's share: waves before it hold NT fragments per k-tile
__device__ __forceinline__ unsigned wave_off(int KT, int NT, int w, int NW) {
  unsigned n = 0;
  for (int v = 0; v < w; ++v) n += (unsigned)nk_of(KT, v, NW);
  return n * (unsigned)NT;
}

// ---- MFMA waves ----------------------------------------------------------------------------------
// The ring registers are loaded and waited for in inline assembly: the compiler neither counts
// these loads nor moves the registers (each statement reads and writes the ring register in
// place), and the one wait per use is exact: every ring slot is (re-)requested exactly once per
// turn, in slot order, so when slot j is due, the D - 1 younger requests may still be out.
__device__ __forceinline__ void ring_load(u32x4 &slot, u32x4 rsrc, unsigned voff, unsigned soff) {
  asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen nt" : "+v"(slot) : "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
template <int N>
__device__ __forceinline__ void ring_wait(u32x4 &slot) {
  asm volatile("s_waitcnt vmcnt(%1)" : "+v"(slot) : "n"(N) : "memory");
}

// Per-wave cursor over the bodies (RING_D ring slots each) of the wave's stream.
template <int NW>
struct BodyCursor {
  PassWalk pw;
  int w, ring;         // MFMA wave; slots per body
  int nk, i0;          // this wave's k-tiles of the current pass; first k-tile (of its own) of the current body
  unsigned frag0;      // stream fragment index of (this wave's first k-tile, the pass's first tile)
  unsigned a_seq0;     // operand k-tiles of this wave before the current pass
  unsigned pseq;       // passes before the current one
  __device__ __forceinline__ void init(const StackArgs &a, int ntmax, int ring_, int w_, bool one_layer = false) {
    pw.init(a, ntmax, one_layer);
    w = w_; ring = ring_; a_seq0 = 0; pseq = 0;
    enter();
  }
  __device__ __forceinline__ void enter() {
    if (pw.done) { nk = 0; i0 = 0; return; }
    nk = nk_of(pw.cur.KT, w, NW);
    i0 = 0;
    frag0 = pw.cur.wbase + wave_off(pw.cur.KT, pw.cur.nt_all, w, NW) + (unsigned)pw.cur.tile0;
  }
  // stream fragment index of slot 0 of the current body; slot j is (j / NTS) * nt_all + j % NTS further
  __device__ __forceinline__ unsigned frag() const { return pw.done ? 0u : frag0 + (unsigned)(i0 * pw.cur.nt_all); }
  __device__ __forceinline__ unsigned row_stride() const { return pw.done ? 0u : (unsigned)pw.cur.nt_all; }
  __device__ __forceinline__ int lg_slots() const {  // log2 of the ring slots per k-tile
    const int n = pw.done ? 1 : pw.cur.NTS;
    return n == 8 ? 3 : n == 4 ? 2 : n == 2 ? 1 : 0;
  }
  __device__ __forceinline__ bool done() const { return pw.done; }
  __device__ __forceinline__ bool pass_finished() const { return i0 >= nk; }
  // real slots of the current body: slot j <-> (k-tile i0 + j / NTS, tile j % NTS)
  __device__ __forceinline__ unsigned mask() const {
    if (pw.done) return 0u;
    const int NTS = pw.cur.NTS, DK = body_rows(NTS, ring);
    const int left = nk - i0;
    const int rows = left < DK ? (left > 0 ? left : 0) : DK;
    const unsigned rowmask = (1u << pw.cur.NT) - 1u;
    unsigned m = 0;
    for (int r = 0; r < rows; ++r) m |= rowmask << (r * NTS);
    return m;
  }
  __device__ __forceinline__ void next_body() {  // (only while !pass_finished())
    i0 += body_rows(pw.cur.NTS, ring);
  }
  __device__ __forceinline__ void next_pass() {
    a_seq0 += (unsigned)nk;
    ++pseq;
    pw.next();
    enter();
  }
};

// ---- the MFMA waves' schedule -----------------------------------------------------------------------
// What an MFMA wave does is the same in every layer of a launch, and in every launch of a model
// with the same row-tile count.  It is written down once per model (schedule_tables_kernel, one
// thread per MFMA wave of every workgroup) as a table of bodies (offsets relative to the layer)
// that every launch copies into LDS; the wave's own loop then only reads the table, so that it
// holds little state besides its ring and accumulators and never touches scratch memory.
struct BodyEnt {
  unsigned mask;    // real slots of the body
  unsigned frag;    // fragment index, relative to the layer's segment, of slot 0
  unsigned a_off;   // operand k-tile sequence number of the body's first k-tile, relative to the layer
  uint16_t stride;  // fragments from one k-tile's row to the next
  uint8_t lg, rows; // log2 of the slots per k-tile; k-tiles of the body that exist
  uint8_t last;     // the body ends a pass: the partial tile is due
  uint8_t nts_pad;
  uint16_t pseq;    // pass number, relative to the layer
};
static_assert(sizeof(BodyEnt) == 20, "five words");
constexpr int TAB_MAX = 128;       // bodies of one MFMA wave per layer
constexpr int TAB_HDR = 16;        // per wave: {bodies, operand k-tiles per layer, passes per layer, 0}
constexpr int TAB_BYTES = TAB_HDR + TAB_MAX * 20;

// Host: bodies of one GEMM in an MFMA wave's schedule, at most (the workgroup with the most column tiles, the wave
// with the most k-tiles), for passes of up to ntmax tiles.  The tables hold TAB_MAX bodies per layer.
inline int schedule_bodies(int KT, int nt_max, int ntp, int ntmax, int ring, int NW) {
  const int step = ntp < ntmax ? ntp : ntmax;
  const int nk = (KT + NW - 1) / NW;
  int n = 0;
  for (int t0 = 0; t0 < nt_max; t0 += step) {
    const int NT = nt_max - t0 < step ? nt_max - t0 : step;
    const int NTS = NT <= 1 ? 1 : NT <= 2 ? 2 : NT <= 4 ? 4 : 8;
    const int b = (nk * NTS + ring - 1) / ring;
    n += b > 1 ? b : 1;
  }
  return n;
}

template <int NW>
__device__ __forceinline__ void build_schedule(const StackArgs &a, int ntmax, int ring, int w, unsigned tab) {
  // one layer's worth: layers lb .. lb + 1 of a stack launch, or the unembedding
  BodyCursor<NW> c;
  c.init(a, ntmax, ring, w, true);
  const unsigned seg0 = a.mode == 0 ? (unsigned)a.lb * a.seg_frags : 0u;
  LDS_AS unsigned *hdr = (LDS_AS unsigned *)(uintptr_t)tab;
  int n = 0;
  while (!c.done()) {
    if (c.pass_finished()) {  // (a pass in which this wave has no k-tile: an empty body that only delivers zeros)
      if (n < TAB_MAX) {
        LDS_AS unsigned *e = (LDS_AS unsigned *)(uintptr_t)(tab + TAB_HDR + n * 20);
        e[0] = 0u; e[1] = 0u; e[2] = c.a_seq0;
        e[3] = (unsigned)c.pw.cur.nt_all | ((unsigned)c.lg_slots() << 16) | (0u << 24);
        e[4] = 1u | ((unsigned)c.pseq << 16);
      }
      ++n;
      c.next_pass();
      continue;
    }
    const int DK = body_rows(c.pw.cur.NTS, ring);
    const int rows = c.nk - c.i0 < DK ? c.nk - c.i0 : DK;
    const bool last = c.i0 + DK >= c.nk;
    if (n < TAB_MAX) {
      LDS_AS unsigned *e = (LDS_AS unsigned *)(uintptr_t)(tab + TAB_HDR + n * 20);
      e[0] = c.mask();
      e[1] = c.frag() - seg0;
      e[2] = c.a_seq0 + (unsigned)c.i0;
      e[3] = (unsigned)c.pw.cur.nt_all | ((unsigned)c.lg_slots() << 16) | ((unsigned)rows << 24);
      e[4] = (last ? 1u : 0u) | ((unsigned)c.pseq << 16);
    }
    ++n;
    c.next_body();
    if (c.pass_finished()) c.next_pass();
  }
  hdr[0] = (unsigned)n;      // (more than TAB_MAX: the host refuses such a shape when the model is created)
  hdr[1] = c.a_seq0;         // operand k-tiles of this wave per layer
  hdr[2] = c.pseq;           // passes per layer
  hdr[3] = 0u;
}

// Bounded spin on an LDS counter (MFMA waves): on a timeout, or when another wave has given up, the
// dead flag is raised and the wait ends -- the wave runs on with whatever it finds, every later
// wait ends at once, the kernel drains, and the IO waves report the error.  Returns the counter.
__device__ __forceinline__ unsigned m_wait_ge(unsigned ctl, int word, unsigned want) {
  unsigned spins = 0;
  for (;;) {
    const unsigned v = ctl_read(ctl + 4 * word);
    if ((int)(v - want) >= 0) return v;
    __builtin_amdgcn_s_sleep(1);
    if ((++spins & 15u) == 0 && (ctl_read(ctl + 4 * K_DEAD) != 0 || spins > SPIN_LDS)) {
      ctl_write(ctl + 4 * K_DEAD, 1u);
      return want;
    }
  }
}

// One body: RING_D ring slots.  Slot j holds the weights of (k-tile j >> lg of the body, column
// tile j & (2^lg - 1) of the pass) and is multiplied into accumulator j & (NTMAX - 1), whatever lg is: the
// same straight-line code serves every pass.  With fewer than NTMAX slots per k-tile an
// accumulator therefore holds the sum over every (NTMAX >> lg)-th k-tile of one column tile, and the
// partial tile is the sum of the accumulators of a tile (dump_partial).
// The operand is read from LDS for GQ slots at a time (one fragment set per slot, the same one
// several times when the slots share a k-tile): one look at the landing counter and one LDS
// latency per GQ slots.
// A wave issues an instruction every four to six cycles, and the weights of a 16-column tile are
// through the matrix unit in 16 MT cycles: what a slot costs is its instruction count.  So
// everything that depends on the slot number alone is worked out once per body, ALL SLOTS AT ONCE,
// lane j for slot j (where the next occupant of the slot lies in the stream, where the slot's
// operand k-tile lies in LDS, and per group of GQ slots whether it fetches the operand, which
// landing count it needs and which count it acknowledges); a slot then takes its values out of
// these vectors with one v_readlane each.
template <int MT, int NW>
__device__ __forceinline__ void mfma_body(u32x4 (&ring)[Geo<MT>::RING], f32x4 (&acc)[MT][Geo<MT>::NTMAX], u32x4 rsrc, int lane, bool no_weights, unsigned mask,
                                          int lg, unsigned a_seq, unsigned ctl, unsigned region, int w, unsigned next_mask, unsigned next_frag,
                                          unsigned next_stride, int next_lg, unsigned &seen, bool timed, unsigned &op_wait) {
  constexpr int RS = Lay<MT, NW>::RS, AM = Geo<MT>::NTMAX - 1;
  constexpr int GQ = MT <= 2 ? 4 : 2;  // slots per operand fetch (GQ x MT fragments in registers)
  constexpr int RING_D = Geo<MT>::RING, NG = RING_D / GQ;
  static_assert((RS & (RS - 1)) == 0 && RING_D <= RING_MAX && RING_D % GQ == 0 && RING_D % Geo<MT>::NTMAX == 0,
                "ring slot by masking; one slot per lane of a half wave; whole groups and whole k-tiles per body");
  const unsigned lane16 = (unsigned)lane * 16u;
  // -- per slot (lane j) --
  const unsigned j_l = (unsigned)lane & 31u;
  // byte offset in this CU's stream of the slot's next occupant (slot j of the body one turn ahead), or out of range (no
  // traffic, zeros come back)
  const unsigned v_w = (((next_mask >> j_l) & 1u) && !no_weights)
                           ? (next_frag + (j_l >> next_lg) * next_stride + (j_l & ((1u << next_lg) - 1u))) * 1024u
                           : OOB;
  // LDS address of the slot's operand k-tile
  const unsigned v_a = region + ((a_seq + (j_l >> lg)) & (unsigned)(RS - 1)) * (unsigned)(MT * 1024);
  // -- per group (lane q) --
  const unsigned q_l = ((unsigned)lane & 31u) < (unsigned)NG ? ((unsigned)lane & 31u) : 0u;  // (lanes beyond the groups are never read)
  const unsigned g0 = (unsigned)GQ * q_l;
  const unsigned qm_l = (mask >> g0) & ((1u << GQ) - 1u);
  // (a group that lies inside the k-tile of the group before it keeps that group's fragments)
  const bool same_kt = q_l > 0 && (((g0 - 1u) >> lg) == ((g0 + (unsigned)GQ - 1u) >> lg)) && ((mask >> (g0 - 1u)) & 1u);
  const unsigned pos = g0 + (unsigned)(31 - __builtin_clz(qm_l ? qm_l : 1u));  // the group's last real slot
  // k-tiles of this body that no later slot needs once the group has its operand: everything in front of the next real
  // slot's k-tile
  const unsigned rest = pos + 1u < 32u ? mask >> (pos + 1u) : 0u;
  const unsigned fin = rest ? ((pos + 1u + (unsigned)__builtin_ctz(rest)) >> lg) : ((pos >> lg) + 1u);
  const unsigned v_need = (qm_l != 0 && !same_kt) ? a_seq + (pos >> lg) + 1u : 0u;  // 0: no fetch (sequence numbers + 1 are never 0)
  const unsigned v_fin = a_seq + fin;

  u32x4 av[GQ][MT];
#pragma unroll
  for (int i = 0; i < GQ; ++i)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) av[i][mt] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int q = 0; q < NG; ++q) {
    const unsigned need = (unsigned)__builtin_amdgcn_readlane((int)v_need, q);
    if (need != 0) {
      if ((int)(seen - need) < 0) {
        const unsigned long long t0 = timed ? wall_clock64() : 0ull;
        seen = m_wait_ge(ctl, K_ALAND + w, need);
        if (timed) op_wait += (unsigned)(wall_clock64() - t0);  // (timeline: how long this body waited for its operand)
      }
#pragma unroll
      for (int i = 0; i < GQ; ++i) {
        const unsigned ad = (unsigned)__builtin_amdgcn_readlane((int)v_a, GQ * q + i) + lane16;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) av[i][mt] = *(LDS_AS const u32x4 *)(uintptr_t)(ad + (unsigned)mt * 1024u);
      }
      // (the reads above are in the LDS queue before this write, so when the IO wave sees it, the operand slots have
      // been read)
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      *(volatile LDS_AS unsigned *)(uintptr_t)(ctl + 4 * (K_ADONE + w)) = (unsigned)__builtin_amdgcn_readlane((int)v_fin, q);
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
    }
#pragma unroll
    for (int i = 0; i < GQ; ++i) {
      const int j = GQ * q + i;
      ring_wait<RING_D - 1>(ring[j]);
      if ((mask >> j) & 1u) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[mt][j & AM] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, av[i][mt]), __builtin_bit_cast(f16x8, ring[j]),
                                                                    acc[mt][j & AM], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      ring_load(ring[j], rsrc, (unsigned)__builtin_amdgcn_readlane((int)v_w, j) + lane16, 0u);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// A wave's finished partial tile into its LDS region, row-major [row][LDT], LDT = 16 * 2^lg + 4:
// column tile t is the sum of accumulators t, t + 2^lg, ... (in that order).
template <int MT>
__device__ __forceinline__ void dump_partial(const f32x4 (&acc)[MT][Geo<MT>::NTMAX], int lg, unsigned region, int lane) {
  constexpr int NA = Geo<MT>::NTMAX;
  const int q4 = lane >> 4, c16 = lane & 15;
  LDS_AS float *tile = (LDS_AS float *)(uintptr_t)region;
  auto put = [&](auto nts_c) {
    constexpr int NTS = decltype(nts_c)::value;
    constexpr int LDT = 16 * NTS + 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int t = 0; t < NTS; ++t) {
        f32x4 s = acc[mt][t];
#pragma unroll
        for (int k = t + NTS; k < NA; k += NTS) s += acc[mt][k];
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[(16 * mt + 4 * q4 + i) * LDT + 16 * t + c16] = s[i];
      }
  };
  if constexpr (NA == 8) {
    if (lg == 3) {
      put(std::integral_constant<int, 8>{});
      return;
    }
  }
  if (lg == 2) put(std::integral_constant<int, 4>{});
  else if (lg == 1) put(std::integral_constant<int, 2>{});
  else put(std::integral_constant<int, 1>{});
}

template <int MT, int NW>
__device__ __forceinline__ void mfma_wave_main(const StackArgs &a, unsigned lds0, int w, int lane) {
  constexpr int NTMAX = Geo<MT>::NTMAX, RING_D = Geo<MT>::RING;
  const unsigned misc = lds0 + NW * Lay<MT, NW>::REG;
  const unsigned ctl = misc + M_CTL;
  const unsigned tab = misc + M_BYTES + (unsigned)w * TAB_BYTES;
  const unsigned region = lds0 + (unsigned)w * Lay<MT, NW>::REG;
  const unsigned lane16 = (unsigned)lane * 16u;
  const bool no_weights = (LA_DBG_BITS(a.dbg) & 1) != 0;  // (timing experiment: no weight traffic)
  // buffer resource over this CU's stream
  const uint64_t base = (uint64_t)(a.wstream + (size_t)blockIdx.x * a.cu_bytes);
  u32x4 rsrc;
  rsrc[0] = uni((unsigned)base);
  rsrc[1] = uni((unsigned)(base >> 32));
  rsrc[2] = uni((unsigned)a.cu_bytes);
  rsrc[3] = 0x00020000u;
  const int n_tab = uni((int)ctl_read(tab)), n_ent = n_tab < TAB_MAX ? n_tab : TAB_MAX, n_layers = a.mode == 0 ? uni(a.le - a.lb) : 1;
  const unsigned a_per_layer = ctl_read(tab + 4), p_per_layer = ctl_read(tab + 8);
  const unsigned seg_stride = uni(a.seg_frags);
  const unsigned seg_first = a.mode == 0 ? uni((unsigned)a.lb * a.seg_frags) : 0u;
  // entry e of layer l (both uniform): mask, absolute fragment of slot 0, row stride, log2 slots
  auto ent_word = [&](int e, int k) { return ctl_read(tab + TAB_HDR + (unsigned)e * 20u + 4u * (unsigned)k); };

  u32x4 ring[RING_D];
#pragma unroll
  for (int j = 0; j < RING_D; ++j) ring[j] = u32x4{0u, 0u, 0u, 0u};
  if (n_ent > 0 && n_layers > 0) {
    const unsigned m = ent_word(0, 0), f0 = seg_first + ent_word(0, 1), w3 = ent_word(0, 3);
    const unsigned st = w3 & 0xffffu;
    const int lg = (int)((w3 >> 16) & 0xffu);
#pragma unroll
    for (int j = 0; j < RING_D; ++j) {
      const bool real = (m >> j) & 1u;
      ring_load(ring[j], rsrc, (real && !no_weights) ? lane16 : OOB, uni((f0 + (unsigned)(j >> lg) * st + (unsigned)(j & ((1 << lg) - 1))) * 1024u));
    }
  }
  f32x4 acc[MT][NTMAX];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NTMAX; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  unsigned seen = 0;  // operand k-tiles known to have landed (sequence number + 1)
  for (int l = 0; l < n_layers; ++l) {
    const unsigned seg = seg_first + (unsigned)l * seg_stride;
    for (int e = 0; e < n_ent; ++e) {
      const bool timed = LA_TRACE_PTR(a) && l == 1 && e < 16 && w < 4;  // (timeline: when each of the first four MFMA waves starts each body of the second layer)
      const unsigned t_body = timed ? (unsigned)wall_clock64() : 0u;
      unsigned op_wait = 0;
      const unsigned a_seq = (unsigned)l * a_per_layer + ent_word(e, 2);
      const unsigned w3 = ent_word(e, 3), w4 = ent_word(e, 4);
      const int lg = (int)((w3 >> 16) & 0xffu);
      // the body one turn ahead: the next entry, or the first one of the next layer, or nothing
      const bool wrap = e + 1 == n_ent;
      const bool none = wrap && l + 1 == n_layers;
      const int ne = wrap ? 0 : e + 1;
      const unsigned nseg = wrap ? seg + seg_stride : seg;
      const unsigned nm = none ? 0u : ent_word(ne, 0);
      const unsigned nf = nseg + ent_word(ne, 1);
      const unsigned nw3 = ent_word(ne, 3);
      const unsigned nst = nw3 & 0xffffu;
      const int nlg = (int)((nw3 >> 16) & 0xffu);
      const bool last = (w4 & 1u) != 0;
      const unsigned pseq = (unsigned)l * p_per_layer + (w4 >> 16);
      mfma_body<MT, NW>(ring, acc, rsrc, lane, no_weights, uni(ent_word(e, 0)), lg, a_seq, ctl, region, w, nm, nf, nst, nlg, seen, timed, op_wait);
      // (low 16 bits of the clock at the body's start, and the time it waited for operand, in 10 ns)
      if (timed && lane == 0) ctl_write(misc + M_BYTES + NW * TAB_BYTES + 4u * (unsigned)(16 * w + e), (t_body & 0xffffu) | ((op_wait > 0xffffu ? 0xffffu : op_wait) << 16));
      if (last) {
        // the pass is done for this wave: partial tile to LDS (its operand ring is idle now), tell the IO waves
        dump_partial<MT>(acc, lg, region, lane);
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        *(volatile LDS_AS unsigned *)(uintptr_t)(ctl + 4 * (K_PDONE + w)) = pseq + 1u;
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < NTMAX; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }
  // the out-of-range requests of the last turn are still counted: let them retire
  wait_vmcnt<0>();
}

// ---- IO waves -----------------------------------------------------------------------------------
struct Io {
  unsigned ctl;     // LDS byte address of the control words
  unsigned lds0;    // LDS byte address of the kernel's LDS
  unsigned misc;    // LDS byte address of the small stuff (M_*)
  int v, lane, tid; // IO wave index, lane, thread index among the IO threads
  unsigned bar_seq;
  int ok;
  unsigned long long *tr;  // timeline slots of the running phase (workgroup 0, IO wave 0, lane 0) or null
  int ph;                  // phase number (timeline)
};
__device__ __forceinline__ void io_mark(const Io &io, int k) {
  if (io.tr && io.v == 0 && io.lane == 0) io.tr[k] = wall_clock64();
}

__device__ __forceinline__ bool io_wait_ge(Io &io, int word, unsigned want) {
  unsigned spins = 0;
  for (;;) {
    unsigned x = ctl_read(io.ctl + 4 * word);
    if ((int)(x - want) >= 0) return true;
    __builtin_amdgcn_s_sleep(1);
    if ((++spins & 255u) == 0 && (ctl_read(io.ctl + 4 * K_DEAD) != 0 || spins > SPIN_LDS)) {
      ctl_write(io.ctl + 4 * K_DEAD, 1u);
      io.ok = 0;
      return false;
    }
  }
}

template <int NIO>
__device__ __forceinline__ bool io_barrier(Io &io) {
  io.bar_seq += NIO;
  if (io.lane == 0) ctl_add(io.ctl + 4 * K_IOBAR, 1u);
  return io_wait_ge(io, K_IOBAR, io.bar_seq);
}

// Grid barrier, run by the IO waves (same counters and protocol as la_stack.h's grid_sync).
template <int NIO>
__device__ __forceinline__ bool io_grid_sync(const StackArgs &a, Io &io, unsigned epoch) {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  io_mark(io, 2);
  if (LA_TRACE_PTR(a) && io.v == 0 && io.lane == 0 && (blockIdx.x == 0 || blockIdx.x > 2)) {  // (timeline: when each workgroup ends a phase)
    const int k = io.ph - a.trace_sel;
    if (k >= 0 && k < 8) LA_TRACE_PTR(a)[(size_t)TRACE_SLOTS * a.trace_phases + TRACE_WG * blockIdx.x + 8 + k] = wall_clock64();
  }
  wait_vmcnt<0>();  // this wave's stores are acknowledged
  io_mark(io, 6);
  if (!io_barrier<NIO>(io)) return false;
  io_mark(io, 7);
  if (io.v == 0 && io.lane == 0) {
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
    if (ok) ctl_write(io.ctl + 4 * K_GPASS, epoch);
    else ctl_write(io.ctl + 4 * K_DEAD, 1u);
  }
  const bool ok = io_wait_ge(io, K_GPASS, epoch);
  io_mark(io, 8);
  return ok;
}

// The operand of one pass into the rings of the MFMA waves this IO wave serves (w = v, v + NIO,
// ...), in batches of GB k-tiles per served wave (GB x SV x MT loads of 1 KB; a missing k-tile is
// requested out of range, so every batch counts the same).  Up to RS / GB batches in flight,
// retired one at a time, which publishes their k-tiles.  (Batches, because one turn of this
// loop costs about half a microsecond of scalar code whatever it moves.)
// The MT fragments of one operand k-tile (contiguous in memory and in the ring) with one LDS address and one offset.
template <int MT, int I = 0>
__device__ __forceinline__ void operand_ktile(__amdgpu_buffer_rsrc_t ra, unsigned dst, unsigned voff, unsigned soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (LDS_AS void *)(uintptr_t)dst, 16, voff, soff, I * 1024, 0);
  if constexpr (I + 1 < MT) operand_ktile<MT, I + 1>(ra, dst, voff, soff);
}

// The usual case, one MFMA wave per IO wave, with the loop's cost per k-tile cut down: a whole batch that does not wrap
// in the ring is requested with constant offsets from one LDS address and one stream offset (three scalar
// instructions and MT loads per k-tile; with the slot, the validity and the addresses worked out per load it was
// nineteen, and the down projection waited for its operand), and the ring space is looked up only when the space
// known from the last look does not cover the batch.
template <int MT, int NW>
__device__ __forceinline__ bool load_operand_1(Io &io, const uint16_t *A, int KT, unsigned &a_seq, int dbg) {
  constexpr int RS = Lay<MT, NW>::RS, GB = RS >= 16 ? 8 : 4, LPB = GB * MT;
  constexpr int FL0 = RS / GB < 63 / LPB + 1 ? RS / GB : 63 / LPB + 1;  // batches in flight: (FL - 1) LPB loads must fit the counter
  constexpr int FL = FL0 < 4 ? FL0 : 4;
  static_assert(RS % GB == 0 && FL >= 1 && (FL - 1) * LPB <= 63 && (RS & (RS - 1)) == 0, "ring and load counter");
  __amdgpu_buffer_rsrc_t ra = rsrc_of(A);
  const unsigned voff = (dbg & 4) ? OOB : (unsigned)io.lane * 16u;
  const int w = io.v;
  const int nk = nk_of(KT, w, NW), n_batches = (nk + GB - 1) / GB;
  const unsigned region = io.lds0 + (unsigned)w * Lay<MT, NW>::REG;
  const unsigned ctl_done = io.ctl + 4 * (K_ADONE + w), ctl_land = io.ctl + 4 * (K_ALAND + w);
  int issued = 0, retired = 0;  // batches
  unsigned landed = a_seq;
  unsigned done = ctl_read(ctl_done);  // operand k-tiles the MFMA wave has read, as last seen
  auto retire_oldest = [&]() {
    switch (issued - retired) {
      case 1: wait_vmcnt<0>(); break;
      case 2: wait_vmcnt<(1 * LPB > 63 ? 63 : 1 * LPB)>(); break;
      case 3: wait_vmcnt<(2 * LPB > 63 ? 63 : 2 * LPB)>(); break;
      default: wait_vmcnt<(3 * LPB > 63 ? 63 : 3 * LPB)>(); break;
    }
    const int left = nk - retired * GB;
    landed += (unsigned)(left > GB ? GB : left);
    if (io.lane == 0) ctl_write(ctl_land, landed);
    ++retired;
    if (retired == 1) io_mark(io, 9);
  };
  unsigned idle = 0;
  while (issued < n_batches) {
    const int i0 = issued * GB;
    const int nv = nk - i0 < GB ? nk - i0 : GB;
    // ring space: a slot is free once its wave has read the k-tile that was there RS before
    bool room = (int)(a_seq + (unsigned)nv - done) <= RS;
    if (!room) {
      done = ctl_read(ctl_done);
      room = (int)(a_seq + (unsigned)nv - done) <= RS;
    }
    if (!room || issued - retired == FL) {  // (the first batches go out together: waiting for the first one alone cost 0.3 % at 32 rows and 1.7 % at one row)
      if (issued > retired) {
        retire_oldest();
        continue;
      }
      __builtin_amdgcn_s_sleep(1);
      if ((++idle & 255u) == 0 && (ctl_read(io.ctl + 4 * K_DEAD) != 0 || idle > SPIN_LDS)) {
        ctl_write(io.ctl + 4 * K_DEAD, 1u);
        io.ok = 0;
        return false;
      }
      continue;
    }
    idle = 0;
    const unsigned slot0 = a_seq & (unsigned)(RS - 1);
    const unsigned so = (unsigned)(w + NW * i0) * (unsigned)(MT * 1024);
    if (nv == GB && slot0 + GB <= (unsigned)RS) {
      const unsigned dst = region + slot0 * (unsigned)(MT * 1024);
#pragma unroll
      for (int g = 0; g < GB; ++g) operand_ktile<MT>(ra, dst + (unsigned)(g * MT * 1024), voff, so + (unsigned)(g * NW * MT * 1024));
    } else {
#pragma unroll
      for (int g = 0; g < GB; ++g) {  // (a missing k-tile is requested out of range, so every batch counts the same)
        const unsigned dst = region + ((slot0 + (unsigned)g) & (unsigned)(RS - 1)) * (unsigned)(MT * 1024);
        operand_ktile<MT>(ra, dst, g < nv ? voff : OOB, g < nv ? so + (unsigned)(g * NW * MT * 1024) : 0u);
      }
    }
    a_seq += (unsigned)nv;
    ++issued;
  }
  while (retired < issued) retire_oldest();
  return true;
}

template <int MT, int NW>
__device__ __forceinline__ bool load_operand(Io &io, const uint16_t *A, int KT, unsigned (&a_seq)[NW / (8 - NW)], int dbg) {
  if constexpr (NW == 8 - NW) return load_operand_1<MT, NW>(io, A, KT, a_seq[0], dbg);
  constexpr int NIO = 8 - NW, SV = NW / NIO, RS = Lay<MT, NW>::RS, GB = 4, LPB = GB * SV * MT;
  constexpr int FL0 = RS / GB < 63 / LPB + 1 ? RS / GB : 63 / LPB + 1;  // batches in flight: (FL - 1) LPB loads must fit the counter
  constexpr int FL = FL0 < 8 ? FL0 : 8;
  static_assert(RS % GB == 0 && FL >= 1 && (FL - 1) * LPB <= 63, "ring and load counter");
  __amdgpu_buffer_rsrc_t ra = rsrc_of(A);
  const unsigned voff = (unsigned)io.lane * 16u;
  int nk[SV], n_batches = 0;
#pragma unroll
  for (int s = 0; s < SV; ++s) {
    nk[s] = nk_of(KT, io.v + NIO * s, NW);
    const int nb = (nk[s] + GB - 1) / GB;
    n_batches = nb > n_batches ? nb : n_batches;
  }
  auto valid_in = [&](int s, int batch) {  // k-tiles of served wave s in a batch
    const int left = nk[s] - batch * GB;
    return left < 0 ? 0 : left > GB ? GB : left;
  };
  int issued = 0, retired = 0;  // batches
  unsigned landed[SV];
#pragma unroll
  for (int s = 0; s < SV; ++s) landed[s] = a_seq[s];
  auto retire_oldest = [&]() {
    switch (issued - retired) {
      case 1: wait_vmcnt<0>(); break;
      case 2: wait_vmcnt<(1 * LPB > 63 ? 63 : 1 * LPB)>(); break;
      case 3: wait_vmcnt<(2 * LPB > 63 ? 63 : 2 * LPB)>(); break;
      case 4: wait_vmcnt<(3 * LPB > 63 ? 63 : 3 * LPB)>(); break;
      case 5: wait_vmcnt<(4 * LPB > 63 ? 63 : 4 * LPB)>(); break;
      case 6: wait_vmcnt<(5 * LPB > 63 ? 63 : 5 * LPB)>(); break;
      case 7: wait_vmcnt<(6 * LPB > 63 ? 63 : 6 * LPB)>(); break;
      default: wait_vmcnt<(7 * LPB > 63 ? 63 : 7 * LPB)>(); break;
    }
#pragma unroll
    for (int s = 0; s < SV; ++s) {
      const int nv = valid_in(s, retired);
      if (nv > 0) {
        landed[s] += (unsigned)nv;
        if (io.lane == 0) ctl_write(io.ctl + 4 * (K_ALAND + io.v + NIO * s), landed[s]);
      }
    }
    ++retired;
    if (retired == 1) io_mark(io, 9);
  };
  unsigned idle = 0;
  while (issued < n_batches) {
    // ring space: a slot is free once its wave has read the k-tile that was there RS before
    bool room = true;
#pragma unroll
    for (int s = 0; s < SV; ++s) {
      const int nv = valid_in(s, issued);
      if (nv > 0) {
        const unsigned done = ctl_read(io.ctl + 4 * (K_ADONE + io.v + NIO * s));
        if ((int)(a_seq[s] + (unsigned)nv - done) > RS) room = false;
      }
    }
    if (!room || issued - retired == FL || (retired == 0 && issued == 1)) {  // (the first batch is waited for alone: the MFMA waves start on it)
      if (issued > retired) {
        retire_oldest();
        continue;
      }
      __builtin_amdgcn_s_sleep(1);
      if ((++idle & 255u) == 0 && (ctl_read(io.ctl + 4 * K_DEAD) != 0 || idle > SPIN_LDS)) {
        ctl_write(io.ctl + 4 * K_DEAD, 1u);
        io.ok = 0;
        return false;
      }
      continue;
    }
    idle = 0;
#pragma unroll
    for (int s = 0; s < SV; ++s) {
      const int w = io.v + NIO * s;
#pragma unroll
      for (int g = 0; g < GB; ++g) {
        const int i = issued * GB + g;
        const bool valid = i < nk[s];
        const int kt = w + NW * i;
        const unsigned slot = (a_seq[s] + (unsigned)g) % (unsigned)RS;
        const unsigned dst = uni(io.lds0 + (unsigned)w * Lay<MT, NW>::REG + slot * (MT * 1024u));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (LDS_AS void *)(uintptr_t)(dst + mt * 1024u), 16, (valid && !(dbg & 4)) ? voff : OOB,
                                                   (unsigned)(valid ? kt * MT + mt : 0) * 1024u, 0, 0);
      }
      a_seq[s] += (unsigned)valid_in(s, issued);
    }
    ++issued;
  }
  while (retired < issued) retire_oldest();
  return true;
}

// Row factors rsqrt(mean(x^2) + eps) of the block's rows into LDS (M_RS), from the per-column-tile
// sums of squares the residual epilogues leave.  IO wave v takes rows v, v + NIO, ...: a row's ncg
// values are at most two 16-byte vectors per lane (whole cache lines per request), added per
// lane and then across the lanes in a fixed tree.
// In two steps: the loads are requested before the operand (anything requested later waits
// behind the operand in the memory pipeline), the sums are formed after it.
template <int MT, int NIO>
struct RowStat {
  static constexpr int NR = (16 * MT + NIO - 1) / NIO;
  f32x4 t[NR][2];
};
template <int MT, int NIO>
__device__ __forceinline__ void row_factors_load(const Io &io, const float *rsq_in, int Bp, int ncg, RowStat<MT, NIO> &rs) {
  __amdgpu_buffer_rsrc_t rr = rsrc_of(rsq_in);
  const int nv = ncg >> 2;
#pragma unroll
  for (int i = 0; i < RowStat<MT, NIO>::NR; ++i) {
    const int row = io.v + NIO * i;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c4 = io.lane + 64 * j;
      const unsigned vo = (row < Bp && c4 < nv) ? (unsigned)c4 * 16u : OOB;
      rs.t[i][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rr, vo, (unsigned)(row * ncg) * 4u, 0));
    }
  }
}
template <int MT, int NIO>
__device__ __forceinline__ void row_factors_finish(const Io &io, int Bp, float inv_d, float eps, const RowStat<MT, NIO> &rs) {
  LDS_AS float *rs_lds = (LDS_AS float *)(uintptr_t)(io.misc + M_RS);
#pragma unroll
  for (int i = 0; i < RowStat<MT, NIO>::NR; ++i) {
    const int row = io.v + NIO * i;
    const f32x4 t = rs.t[i][0] + rs.t[i][1];
    float s = (t[0] + t[1]) + (t[2] + t[3]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (row < 16 * MT && io.lane == 0) rs_lds[row] = row < Bp ? 1.0f / sqrtf(s * inv_d + eps) : 0.f;
  }
}

// What one pass's epilogue needs (uniform values).
struct Epi {
  int mode;  // GemmMode
  uint16_t *Kc, *Vc;
  const float *gain;
  uint16_t *xa_out;
  float *rsq_out;
  uint16_t *act_a;
  Top *un_part;
  int part;
  bool keep_x;  // residual epilogue: x may stay in LDS alone (a later epilogue of the launch writes it to memory)
};

// The rotation factors of a thread's item of the QKV epilogue (16 floats: cos, sin of eight pairs), requested before
// the wait for the partial tiles: they do not depend on the product, and read inside the epilogue their latency stood
// between the reduction and the stores of every layer.  Covers the first item of each thread (there is no second one
// unless a workgroup has more than 256 / rows column tiles in the pass; later items read theirs in place).
struct QkvPre {
  f32x4 c[4];
  bool have;
};
template <int NIO>
__device__ __forceinline__ void qkv_prefetch(const StackArgs &a, const Io &io, int tile_first, int ntc, QkvPre &pre) {
  const int it = io.tid, dh = a.dh, half = dh >> 1, spj = dh >> 4;
  pre.have = false;
#pragma unroll
  for (int i = 0; i < 4; ++i) pre.c[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (it >= a.Bp * ntc) return;
  const int b = it / ntc, tt = it - b * ntc;
  const int gt = (int)blockIdx.x + (int)gridDim.x * (tile_first + tt);
  const int hs = gt / spj, j = gt - hs * spj;
  if (hs >= a.Hq + a.Hkv) return;
  const f32x4 *cp = reinterpret_cast<const f32x4 *>(a.cs + ((size_t)b * half + 8 * j) * 2);
#pragma unroll
  for (int i = 0; i < 4; ++i) pre.c[i] = cp[i];
  pre.have = true;
}

// Eight consecutive floats of the pass's tile: the MFMA waves' partial tiles, at the
// same place in each wave's region, added in wave order.
template <int NW, int REG>
__device__ __forceinline__ void tile8(unsigned lds0, unsigned byte_off, float (&out)[8]) {
  f32x4 s0 = *(LDS_AS const f32x4 *)(uintptr_t)(lds0 + byte_off), s1 = *(LDS_AS const f32x4 *)(uintptr_t)(lds0 + byte_off + 16u);
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    s0 += *(LDS_AS const f32x4 *)(uintptr_t)(lds0 + (unsigned)(w * REG) + byte_off);
    s1 += *(LDS_AS const f32x4 *)(uintptr_t)(lds0 + (unsigned)(w * REG) + byte_off + 16u);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[i] = s0[i];
    out[4 + i] = s1[i];
  }
}
// The epilogue of a pass (rows x NT column tiles; every MFMA wave's partial tile row-major [row][LDT] at the start of
// its region), by all IO threads: each thread adds the partial tiles of the elements it works on (a pass over the whole
// tile first, with a barrier behind it, took 0.5 - 1 us more per phase).  Same arithmetic as la_stack.h's gemm_epilogue.
template <int MT, int NIO>
__device__ __forceinline__ void pass_epilogue(const StackArgs &a, const Io &io, const Epi &q, int L, int x_lds, int tile_first, int ntc,
                                              int LDT, const QkvPre &pre) {
  constexpr int NT_IO = NIO * 64;
  const int Bp = a.Bp, d = a.d, ncg = a.ncg, Hq = a.Hq, Hkv = a.Hkv, dh = a.dh;
  const int tid = io.tid;
  const float *cs = a.cs;
  constexpr int NW = 8 - NIO, REG = Lay<MT, 8 - NIO>::REG;
  LDS_AS const float *rs_lds = (LDS_AS const float *)(uintptr_t)(io.misc + M_RS);
  const int G = gridDim.x, cu = blockIdx.x;
  if (q.mode == MODE_QKV) {
    for (int it = tid; it < Bp * ntc; it += NT_IO) {
      const int b = it / ntc, tt = it - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const int half = dh >> 1, spj = dh >> 4, grp = Hq / Hkv;
      const int hs = gt / spj, j = gt - hs * spj;
      const float rsf = rs_lds[b];
      float tr[16];
      {
        float lo8[8], hi8[8];
        tile8<NW, REG>(io.lds0, (unsigned)(b * LDT + 16 * tt) * 4u, lo8);
        tile8<NW, REG>(io.lds0, (unsigned)(b * LDT + 16 * tt + 8) * 4u, hi8);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          tr[k] = lo8[k];
          tr[8 + k] = hi8[k];
        }
      }
      const float qscale = hs < Hq ? 1.0f / sqrtf((float)dh) : 1.0f;
      float y0[8], y1[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        float x0 = tr[k] * rsf, x1 = tr[8 + k] * rsf;
        if (hs < Hq + Hkv) {
          float c, sn;
          if (it == tid && pre.have) {
            c = pre.c[k >> 1][(k & 1) * 2];
            sn = pre.c[k >> 1][(k & 1) * 2 + 1];
          } else {
            c = cs[((size_t)b * half + 8 * j + k) * 2];
            sn = cs[((size_t)b * half + 8 * j + k) * 2 + 1];
          }
          y0[k] = (x0 * c - x1 * sn) * qscale;
          y1[k] = (x1 * c + x0 * sn) * qscale;
        } else {
          y0[k] = x0;
          y1[k] = x1;
        }
      }
      const bool h16 = a.f16 != 0;
      u32x4 lo = {pack_kv(h16, y0[0], y0[1]), pack_kv(h16, y0[2], y0[3]), pack_kv(h16, y0[4], y0[5]), pack_kv(h16, y0[6], y0[7])};
      u32x4 hi = {pack_kv(h16, y1[0], y1[1]), pack_kv(h16, y1[2], y1[3]), pack_kv(h16, y1[4], y1[5]), pack_kv(h16, y1[6], y1[7])};
      const int o_lo = j, o_hi = (half >> 3) + j;
      if (hs < Hq) {
        __amdgpu_buffer_rsrc_t rqf = rsrc_of(a.qf);
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
          st16(rv, (unsigned)(v_index(true, L + b, h, 8 * j + k, Hkv, dh) * 2), kv_bits(h16, y0[k]));
          st16(rv, (unsigned)(v_index(true, L + b, h, half + 8 * j + k, Hkv, dh) * 2), kv_bits(h16, y1[k]));
        }
      }
    }
  } else if (q.mode == MODE_RESID) {
    for (int it = tid; it < Bp * ntc * 2; it += NT_IO) {
      const int oct = it & 1, bt = it >> 1;
      const int b = bt / ntc, tt = bt - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const int col = 16 * gt + 8 * oct;
      f32x4 *xp = reinterpret_cast<f32x4 *>(a.x + (size_t)b * d + col);
      float tr[8];
      tile8<NW, REG>(io.lds0, (unsigned)(b * LDT + 16 * tt + 8 * oct) * 4u, tr);
      LDS_AS f32x4 *xs = (LDS_AS f32x4 *)(uintptr_t)(io.misc + M_X + (((tile_first + tt) * 16 * MT + b) * 16 + 8 * oct) * 4);
      f32x4 x0, x1;
      if (x_lds) {
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
      if (x_lds) {
        xs[0] = x0;
        xs[1] = x1;
      }
      // (x goes to memory when the launch ends, or when it is not kept in LDS: these 32-byte pieces of rows 4 d bytes
      // apart are partial cache lines, and storing them in every residual epilogue cost 1.5 us per phase)
      if (!(x_lds && q.keep_x)) {
        xp[0] = x0;
        xp[1] = x1;
      }
      float sq = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
      sq += __shfl_xor(sq, 1, 64);
      if (q.gain) {
        if (oct == 0) st32f(rsrc_of(q.rsq_out), (unsigned)(b * ncg + gt) * 4, sq);
        float gp[8];
        if (x_lds) {
          LDS_AS const f32x4 *gs = (LDS_AS const f32x4 *)(uintptr_t)(io.misc + M_GAIN + ((tile_first + tt) * 16 + 8 * oct) * 4);
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
  } else if (q.mode == MODE_GATEUP) {
    __amdgpu_buffer_rsrc_t rp = rsrc_of(q.act_a);
    for (int it = tid; it < Bp * ntc; it += NT_IO) {
      const int b = it / ntc, tt = it - b * ntc;
      const int gt = cu + G * (tile_first + tt);
      const float rsf = rs_lds[b];
      float gp[8], up[8];
      tile8<NW, REG>(io.lds0, (unsigned)(b * LDT + 16 * tt) * 4u, gp);
      tile8<NW, REG>(io.lds0, (unsigned)(b * LDT + 16 * tt + 8) * 4u, up);
      float act[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float g = gp[i] * rsf, u = up[i] * rsf;
        act[i] = g / (1.0f + __expf(-g)) * u;
      }
      st128(rp, frag_piece(8 * gt, b, MT),
            u32x4{pack_f16(act[0], act[1]), pack_f16(act[2], act[3]), pack_f16(act[4], act[5]), pack_f16(act[6], act[7])});
    }
  } else {  // MODE_UNEMBED: arg-max of each row over this pass's columns, 4 threads per row (rows beyond the threads: in turns)
    for (int r0 = 0; r0 < 16 * MT; r0 += NT_IO / 4) {
      const int row = r0 + (tid >> 2), j = tid & 3;
      Top best{-INFINITY, 0x7fffffff, -INFINITY};
      if (row < Bp)
        for (int c8 = j; c8 < 2 * ntc; c8 += 4) {  // eight columns at a time
          float v[8];
          tile8<NW, REG>(io.lds0, (unsigned)(row * LDT + 8 * c8) * 4u, v);
          const int col0 = 16 * (cu + G * (tile_first + (c8 >> 1))) + 8 * (c8 & 1);
#pragma unroll
          for (int k = 0; k < 8; ++k) best = top_merge2(best, Top{v[k], col0 + k, -INFINITY});
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
        unsigned o = (unsigned)(((size_t)q.part * 64 + row) * sizeof(Top));
        st32f(rp, o, best.v1);
        __builtin_amdgcn_raw_buffer_store_b32((unsigned)best.i1, rp, o + 4, 0, DEV);
        st32f(rp, o + 8, best.v2);
      }
    }
  }
}

// One pass on the IO side: operand in, wait for the partial tiles, add them (wave 0, 1, ... in
// that order), epilogue.
template <int MT, int NW, typename Between>
__device__ __forceinline__ bool io_pass(const StackArgs &a, Io &io, const Pass &p, unsigned pseq, const uint16_t *A, const float *rsq_in,
                                        const Epi &q, int L, int x_lds, unsigned (&a_seq)[NW / (8 - NW)], Between between) {
  constexpr int NIO = 8 - NW, NT_IO = NIO * 64;
  const unsigned long long t_a = io.tr ? wall_clock64() : 0ull;
  if (p.pidx == 0) io_mark(io, 10);
  RowStat<MT, NIO> rs;
  if (rsq_in) row_factors_load<MT, NIO>(io, rsq_in, a.Bp, a.ncg, rs);
  if (!load_operand<MT, NW>(io, A, p.KT, a_seq, LA_DBG_BITS(a.dbg))) return false;
  if (io.tr && io.v == 0 && io.lane == 0 && p.pidx == 0) io.tr[3] = wall_clock64() - t_a;  // (reported as "waited for weights": the operand's way in)
  if (rsq_in) row_factors_finish<MT, NIO>(io, a.Bp, a.inv_d, a.eps, rs);
  QkvPre pre;
  pre.have = false;
  if (q.mode == MODE_QKV) qkv_prefetch<NIO>(a, io, p.tile0, p.NT, pre);
  between();  // (bookkeeping of the caller that needs no result of this pass: it runs while the MFMA waves finish)
  if (!io_barrier<NIO>(io)) return false;  // (the row factors, gains and x tiles the IO waves staged for each other)
  for (int w = 0; w < NW; ++w)
    if (!io_wait_ge(io, K_PDONE + w, pseq + 1u)) return false;
  if (p.pidx == 0) io_mark(io, 1);
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  const int LDT = 16 * p.NTS + 4;
  if (p.pidx == 0) io_mark(io, 4);
  pass_epilogue<MT, NIO>(a, io, q, L, x_lds, p.tile0, p.NT, LDT, pre);
  if (p.pidx == 0) io_mark(io, 5);
  return true;
}

// ---- first operand of a launch, RoPE table, staging (IO threads of all workgroups) ----------------
template <int NIO>
__device__ __forceinline__ void r_prep(const StackArgs &a, const Io &io, const float *gain, uint16_t *xa_out, float *rsq_out) {
  constexpr int NT_IO = NIO * 64;
  __amdgpu_buffer_rsrc_t rq = rsrc_of(rsq_out), rx = rsrc_of(xa_out);
  const int octs = a.d >> 3, total = a.Bp * octs;
  for (int it = blockIdx.x * NT_IO + io.tid; it < total; it += gridDim.x * NT_IO) {
    const int r = it / octs, oct = it - r * octs, c0 = oct * 8;
    const f32x4 *xp = reinterpret_cast<const f32x4 *>(a.x + (size_t)r * a.d + c0);
    f32x4 x0 = xp[0], x1 = xp[1];
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) sq += x0[i] * x0[i] + x1[i] * x1[i];
    sq += __shfl_xor(sq, 1, 64);
    if ((oct & 1) == 0) st32f(rq, (unsigned)(r * a.ncg + (oct >> 1)) * 4, sq);
    const float *gp = gain + c0;
    u32x4 v = {pack_f16(x0[0] * gp[0], x0[1] * gp[1]), pack_f16(x0[2] * gp[2], x0[3] * gp[3]),
               pack_f16(x1[0] * gp[4], x1[1] * gp[5]), pack_f16(x1[2] * gp[6], x1[3] * gp[7])};
    st128(rx, frag_piece(c0, r, a.MT), v);
  }
}

template <int NIO>
__device__ __forceinline__ void r_rope_table(const StackArgs &a, const Io &io) {
  constexpr int NT_IO = NIO * 64;
  __amdgpu_buffer_rsrc_t rc = rsrc_of(a.cs);
  int half = a.dh >> 1, total = a.Bp * half;
  for (int e = blockIdx.x * NT_IO + io.tid; e < total; e += gridDim.x * NT_IO) {
    int b = e / half, i = e - b * half;
    double inv = exp2(-(double)i / (double)half * log2(a.theta));
    double s, c;
    sincos((double)a.pos[b] * inv, &s, &c);
    st32f(rc, (unsigned)e * 8, (float)c);
    st32f(rc, (unsigned)e * 8 + 4, (float)s);
  }
}

template <int MT, int NIO>
__device__ __forceinline__ void r_x_stage(const StackArgs &a, const Io &io, int nt_x) {
  constexpr int NT_IO = NIO * 64;
  const int rows = 16 * MT;
  for (int it = io.tid; it < nt_x * a.Bp * 4; it += NT_IO) {
    const int part = it & 3, bt = it >> 2, tt = bt / a.Bp, b = bt - tt * a.Bp;
    const int col = 16 * ((int)blockIdx.x + (int)gridDim.x * tt) + 4 * part;
    *(LDS_AS f32x4 *)(uintptr_t)(io.misc + M_X + ((tt * rows + b) * 16 + 4 * part) * 4) =
        *reinterpret_cast<const f32x4 *>(a.x + (size_t)b * a.d + col);
  }
}

__device__ __forceinline__ void r_gain_stage(const float *gain, const Io &io, int nt_x) {
  if (io.v != 0 || gain == nullptr) return;
  const int tt = io.lane >> 4;
  const unsigned vo = tt < nt_x ? (unsigned)((16 * ((int)blockIdx.x + (int)gridDim.x * tt) + (io.lane & 15)) * 4) : OOB;
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_of(gain), (LDS_AS void *)(uintptr_t)(io.misc + M_GAIN), 4, vo, 0, 0, 0);
}

// ---- masked-block GQA attention on the IO waves -----------------------------------------------------
// Same unit, same products and the same running softmax as la_stack.h's attention_phase; the NIO
// waves of a unit's workgroup split the 32-key blocks, and wave 0 merges the others' partial
// results in wave order.  The merge buffers sit in the MFMA waves' LDS regions, which are idle
// between the QKV pass and the O pass.
template <int DH, int MT, int NIO, bool F16>
__device__ __forceinline__ bool r_attention(const StackArgs &a, Io &io, const uint16_t *Kc, const uint16_t *Vc, uint16_t *attn_out, int L,
                                            int su0, int S, unsigned &att_seq) {
  constexpr int KT = DH / 32, DT = DH / 16;
  using v8 = std::conditional_t<F16, f16x8, bf16x8>;  // q, K, V and the probabilities: the cache's 16-bit type
  auto mma = [](v8 x, v8 y, f32x4 c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(x, y, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, c, 0, 0, 0);
  };
  __amdgpu_buffer_rsrc_t rk = rsrc_of(Kc), rv = rsrc_of(Vc), rqf = rsrc_of(a.qf), ra = rsrc_of(attn_out);
  // per merging wave: DT KB of output tiles, then 512 B of (max, sum) per lane
  constexpr unsigned BUF = DT * 1024u + 512u;
  const int v = io.v, lane = io.lane, q4 = lane >> 4, c16 = lane & 15;
  const int g = a.Hq / a.Hkv, n_rt = g * MT;
  const int total = L + a.Bp, nkb = (total + 31) >> 5;
  // Split units: unit u = su % n_units, key slice ks = su / n_units of S.  With S > 1 the committed key blocks are cut
  // into S contiguous runs (the blocks holding this step's rows go with the last run); every split unit leaves its
  // (o, m, l) in memory, and the one that delivers last adds all S records in slice order and writes the result, so the
  // sum has one order whoever forms it.
  const int n_units = a.Hkv * n_rt;
  constexpr unsigned PART = DT * 1024u + 512u;  // bytes of a record: DT output tiles (16 B per lane each), then (m, l) per lane
  for (int su = su0; su < n_units * S; su += gridDim.x) {
    const int u = su % n_units, ks = su / n_units;
    // unit u = kvh + Hkv * rt sits on workgroup att_first + u: with 8 kv heads (and the first unit on a multiple of 8)
    // all units of a kv head run on one XCD and share its K, V lines in that XCD's L2 (requesting those lines ahead, during
    // the QKV phase, as the earlier kernel does, was measured here and costs 0.5 - 2.4 %: it is not done)
    const int rt = u / a.Hkv, kvh = u - rt * a.Hkv;
    const int b = (rt % MT) * 16 + c16;
    io_mark(io, 10);  // (timeline of a unit: entry, late blocks done, early blocks done, merged, stored)
    const uint64_t vb = b < a.Bp ? a.vis[b] : 0ull;
    v8 q[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
      q[kt] = __builtin_bit_cast(v8, ld128(rqf, (unsigned)(((((size_t)kvh * n_rt + rt) * KT + kt) * 64 + lane) * 16)));
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -1e30f, l_run = 0.f;
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
    auto scores = [&](float *sv) {
      f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        sa = mma(__builtin_bit_cast(v8, ka[kt]), q[kt], sa);
        sb = mma(__builtin_bit_cast(v8, kb2[kt]), q[kt], sb);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) sv[i] = i < 4 ? sa[i] : sb[i - 4];
    };
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
      const u32x4 pw = {pack_kv(F16, p[0], p[1]), pack_kv(F16, p[2], p[3]), pack_kv(F16, p[4], p[5]), pack_kv(F16, p[6], p[7])};
      return __builtin_bit_cast(v8, pw);
    };
    auto pv = [&](v8 pb, float corr) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        o[dt] *= corr;
        o[dt] = mma(__builtin_bit_cast(v8, vt[dt]), pb, o[dt]);
      }
    };
    const std::integral_constant<int, 0> plain{};
    const std::integral_constant<int, DEV> coherent{};
    const int kb_split = L >> 5;  // key blocks 0 .. kb_split - 1 end at or before row L ("early")
    const int e_lo = kb_split * ks / S, e_hi = kb_split * (ks + 1) / S;  // this slice's early blocks
    // The blocks that hold rows of this step ("late": at most three, written by other workgroups in
    // the phase before, so device-scope loads and the mask) are dealt to the waves round-robin and
    // taken first, one at a time; the early blocks (ordinary loads, every key visible) follow in
    // the wave's pipeline: the next block's K is requested as soon as the scores are out of the
    // matrix unit, the next V after P V.
    for (int kb = kb_split + v; kb < nkb && ks == S - 1; kb += NIO) {
      float sv[8], corr;
      load_k(coherent, kb, true);
      load_v(coherent, kb, true);
      scores(sv);
      const v8 pb = softmax(std::true_type{}, sv, kb, corr);
      pv(pb, corr);
    }
    io_mark(io, 9);
    if (e_lo + v < e_hi) {
      int kb = e_lo + v, ne = kb + NIO;
      float sv[8], corr;
      load_k(plain, kb, true);
      load_v(plain, kb, true);
      for (;;) {
        scores(sv);
        load_k(plain, ne, ne < e_hi);
        const v8 pb = softmax(std::false_type{}, sv, kb, corr);
        pv(pb, corr);
        load_v(plain, ne, ne < e_hi);
        if (ne >= e_hi) break;
        kb = ne;
        ne += NIO;
      }
    }
    io_mark(io, 1);
    // merge: waves 1 .. NIO-1 leave (o, m, l) in LDS, wave 0 adds them in wave order
    const unsigned qs = att_seq;
    if (v > 0) {
      LDS_AS f32x4 *red = (LDS_AS f32x4 *)(uintptr_t)(io.lds0 + (unsigned)(v - 1) * BUF);
      LDS_AS float *ml = (LDS_AS float *)(uintptr_t)(io.lds0 + (unsigned)(v - 1) * BUF + DT * 1024u);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) red[dt * 64 + lane] = o[dt];
      ml[lane * 2] = m_run;
      ml[lane * 2 + 1] = l_run;
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      if (lane == 0) ctl_write(io.ctl + 4 * (K_ATT + v), qs + 1u);
    } else {
#pragma unroll
      for (int ov = 1; ov < NIO; ++ov) {
        if (!io_wait_ge(io, K_ATT + ov, qs + 1u)) return false;
        LDS_AS const f32x4 *red = (LDS_AS const f32x4 *)(uintptr_t)(io.lds0 + (unsigned)(ov - 1) * BUF);
        LDS_AS const float *ml = (LDS_AS const float *)(uintptr_t)(io.lds0 + (unsigned)(ov - 1) * BUF + DT * 1024u);
        const float mo = ml[lane * 2], lo = ml[lane * 2 + 1];
        const float m_new = fmaxf(m_run, mo);
        const float ca = __expf(m_run - m_new), cb = __expf(mo - m_new);
        l_run = l_run * ca + lo * cb;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = o[dt] * ca + red[dt * 64 + lane] * cb;
        m_run = m_new;
      }
      io_mark(io, 4);
      bool writer = true;
      if (S > 1) {
        __amdgpu_buffer_rsrc_t rp = rsrc_of(a.att_part);
        const unsigned mine = (unsigned)su * PART;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) st128(rp, mine + (unsigned)(dt * 64 + lane) * 16u, __builtin_bit_cast(u32x4, o[dt]));
        st64(rp, mine + DT * 1024u + (unsigned)lane * 8u, u32x2{__float_as_uint(m_run), __float_as_uint(l_run)});
        wait_vmcnt<0>();  // the record is acknowledged before it is counted
        unsigned last = 0;
        if (lane == 0) {
          const unsigned old = __hip_atomic_fetch_add(a.att_cnt + u, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          last = ((old + 1u) % (unsigned)S) == 0u ? 1u : 0u;
        }
        writer = uni(last) != 0u;
        if (writer) {
          m_run = -1e30f;
          l_run = 0.f;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
          for (int k = 0; k < S; ++k) {
            const unsigned rec = (unsigned)(u + n_units * k) * PART;
            const u32x2 ml2 = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rp, rec + DT * 1024u + (unsigned)lane * 8u, 0, DEV));
            const float mo = __uint_as_float(ml2[0]), lo = __uint_as_float(ml2[1]);
            const float m_new = fmaxf(m_run, mo);
            const float ca = __expf(m_run - m_new), cb = __expf(mo - m_new);
            l_run = l_run * ca + lo * cb;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
              o[dt] = o[dt] * ca + __builtin_bit_cast(f32x4, ld128(rp, rec + (unsigned)(dt * 64 + lane) * 16u)) * cb;
            m_run = m_new;
          }
        }
      }
      if (writer && b < a.Bp) {
        const float inv = 1.0f / l_run;
        const int j = rt / MT;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          int col = (kvh * g + j) * DH + 16 * dt + 8 * (q4 >> 1);
          st64(ra, frag_piece(col, b, MT) + 8 * (q4 & 1),
               u32x2{pack_f16(o[dt][0] * inv, o[dt][1] * inv), pack_f16(o[dt][2] * inv, o[dt][3] * inv)});
        }
      }
      io_mark(io, 5);
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      if (lane == 0) ctl_write(io.ctl + 4 * (K_ATT + 0), qs + 1u);
    }
    att_seq = qs + 1u;
    // the buffers are free again once wave 0 has read them
    if (!io_wait_ge(io, K_ATT + 0, qs + 1u)) return false;
  }
  return true;
}

template <int NIO>
__device__ __forceinline__ void r_unembed_final(const StackArgs &a, const Io &io) {
  __amdgpu_buffer_rsrc_t ru = rsrc_of(a.un_part);
  const int n_part = gridDim.x * a.un_parts_per_cu;
  for (int b = blockIdx.x * NIO + io.v; b < a.Bp; b += gridDim.x * NIO) {
    Top best{-INFINITY, 0x7fffffff, -INFINITY};
    for (int s0 = io.lane; s0 < n_part; s0 += 64 * 8) {
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
    for (int c = io.lane; c < a.ncg; c += 64) s += ld32f(rsrc_of(a.rsq), (unsigned)((size_t)b * a.ncg + c) * 4);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (io.lane == 0) {
      float rsf = 1.0f / sqrtf(s * a.inv_d + a.eps);
      a.ids[b] = best.i1;
      if (a.top2) {
        a.top2[b * 2] = best.v1 * rsf;
        a.top2[b * 2 + 1] = best.v2 * rsf;
      }
    }
  }
}

template <int MT, int NW>
__device__ __forceinline__ void io_wave_main(const StackArgs &a, unsigned lds0, int v, int lane, int L) {
  constexpr int NIO = 8 - NW, SV = NW / NIO;
  static_assert(NW % NIO == 0, "every IO wave serves the same number of MFMA waves");
  Io io;
  io.lds0 = lds0;
  io.misc = lds0 + NW * Lay<MT, NW>::REG;
  io.ctl = io.misc + M_CTL;
  io.v = v; io.lane = lane; io.tid = v * 64 + lane;
  io.bar_seq = 0; io.ok = 1;
  io.tr = nullptr;
  io.ph = 0;
  int ph = 0;  // phase number as in la_stack.h: first operand, then five per layer
  auto set_phase = [&](int k) {
    ph = k;
    io.ph = k;
    io.tr = (LA_TRACE_PTR(a) && blockIdx.x == 0 && k < a.trace_phases) ? LA_TRACE_PTR(a) + TRACE_SLOTS * k : nullptr;
    io_mark(io, 0);
    if (io.tr && io.v == 0 && io.lane == 0) io.tr[12] = (unsigned long long)clock64();  // (shader clock, for its rate over the launch)
  };
  set_phase(0);
  unsigned epoch = a.epoch0;
  unsigned a_seq[SV];
#pragma unroll
  for (int s = 0; s < SV; ++s) a_seq[s] = 0;
  unsigned pseq = 0, att_seq = 0;
  PassWalk pw;
  pw.init(a, Geo<MT>::NTMAX);

  if (a.mode == 1) {  // unembedding: operand, GEMM passes with arg-max records, final arg-max
    r_prep<NIO>(a, io, a.g_final, a.xa, a.rsq);
    {
      // every CU writes all of its partial records: the ones it has no pass for stay empty
      __amdgpu_buffer_rsrc_t rp = rsrc_of(a.un_part);
      const int nt = pw.tiles_of(4), ntp = a.un.ntp < Geo<MT>::NTMAX ? a.un.ntp : Geo<MT>::NTMAX;
      const int used = (nt + ntp - 1) / ntp;
      for (int it = io.tid; it < (a.un_parts_per_cu - used) * 64; it += NIO * 64) {
        unsigned o = (unsigned)(((size_t)(blockIdx.x * a.un_parts_per_cu + used + (it >> 6)) * 64 + (it & 63)) * sizeof(Top));
        st32f(rp, o, -INFINITY);
        __builtin_amdgcn_raw_buffer_store_b32(0x7fffffffu, rp, o + 4, 0, DEV);
        st32f(rp, o + 8, -INFINITY);
      }
    }
    if (!io_grid_sync<NIO>(a, io, ++epoch)) return;
    set_phase(1);
    bool first = true;
    while (!pw.done) {
      if (!first) {  // (the first region is read by every IO wave's epilogue: all done before it is loaded again)
        if (!io_barrier<NIO>(io)) return;
      }
      first = false;
      Epi q{};
      q.mode = MODE_UNEMBED;
      q.un_part = a.un_part + (size_t)blockIdx.x * a.un_parts_per_cu * 64;
      q.part = pw.cur.pidx;
      const Pass cur = pw.cur;
      if (!io_pass<MT, NW>(a, io, cur, pseq, a.xa, nullptr, q, L, 0, a_seq, [&]() { pw.next(); })) return;
      ++pseq;
    }
    if (!io_grid_sync<NIO>(a, io, ++epoch)) return;
    set_phase(2);
    r_unembed_final<NIO>(a, io);
    io_mark(io, 2);
    return;
  }

  const int nt_x = pw.tiles_of(1);
  const int x_lds = (nt_x * MT * 1024 <= X_BYTES && nt_x <= 4) ? 1 : 0;  // (one load instruction stages the gains of four tiles)
  const int n_rt = a.Hq / a.Hkv * MT, n_units = a.Hkv * n_rt;
  // Key split of the attention: S slices per unit while every split unit still gets a workgroup of its own and a wave
  // keeps four or more key blocks (short contexts gain nothing from more workgroups: the merge costs what they save).
  int S = 1;
  {
    const int nkb = (L + a.Bp + 31) >> 5;
    while (S < 8 && n_units * 2 * S <= (int)gridDim.x && nkb >= 16 * 2 * S) S *= 2;
  }
  const int n_su = n_units * S;
  const int att_first = (LA_DBG_BITS(a.dbg) & 32) ? 0 : att_first_wg(a.qkv.ntiles, n_su);  // (timing experiment: the traced workgroup runs a unit)
  const int att_u0 = (int)blockIdx.x >= att_first ? (int)blockIdx.x - att_first : n_su;
  if (blockIdx.x == 0)  // the delivery counters start every launch at zero (visible after the first grid barrier)
    for (int i = io.tid; i < n_units; i += NIO * 64) __builtin_amdgcn_raw_buffer_store_b32(0u, rsrc_of(a.att_cnt), (unsigned)i * 4u, 0, DEV);
  r_prep<NIO>(a, io, a.gains[a.lb].g_attn, a.xa + (size_t)(2 * a.lb) * a.xa_stride, a.rsq + (size_t)(2 * a.lb) * a.rsq_stride);
  r_rope_table<NIO>(a, io);
  if (x_lds) r_x_stage<MT, NIO>(a, io, nt_x);

  for (int layer = a.lb; layer < a.le; ++layer) {
    uint16_t *Kc = a.K + (size_t)layer * a.layer_elems, *Vc = a.V + (size_t)layer * a.layer_elems;
    uint16_t *xa0 = a.xa + (size_t)(2 * layer) * a.xa_stride, *xa1 = xa0 + a.xa_stride;
    float *rsq0 = a.rsq + (size_t)(2 * layer) * a.rsq_stride, *rsq1 = rsq0 + a.rsq_stride;
    uint16_t *attn_l = a.attn_a + (size_t)layer * a.attn_stride, *act_l = a.act_a + (size_t)layer * a.act_stride;
    for (int gemm = 0; gemm < 4; ++gemm) {
      if (!io_grid_sync<NIO>(a, io, ++epoch)) return;
      set_phase(1 + 5 * (layer - a.lb) + (gemm <= 1 ? gemm : gemm + 1));
      if (gemm == 1) {
        if (att_u0 < n_su) {
          bool ok;
          if (a.f16)
            ok = a.dh == 128 ? r_attention<128, MT, NIO, true>(a, io, Kc, Vc, attn_l, L, att_u0, S, att_seq)
                             : r_attention<64, MT, NIO, true>(a, io, Kc, Vc, attn_l, L, att_u0, S, att_seq);
          else
            ok = a.dh == 128 ? r_attention<128, MT, NIO, false>(a, io, Kc, Vc, attn_l, L, att_u0, S, att_seq)
                             : r_attention<64, MT, NIO, false>(a, io, Kc, Vc, attn_l, L, att_u0, S, att_seq);
          if (!ok) return;
        }
        if (!io_grid_sync<NIO>(a, io, ++epoch)) return;
        set_phase(1 + 5 * (layer - a.lb) + 2);
      }
      const uint16_t *A = nullptr;
      const float *rsq_in = nullptr;
      Epi q{};
      switch (gemm) {
        case 0:
          A = xa0; rsq_in = rsq0; q.mode = MODE_QKV; q.Kc = Kc; q.Vc = Vc;
          break;
        case 1:
          A = attn_l; q.mode = MODE_RESID; q.gain = a.gains[layer].g_mlp; q.xa_out = xa1; q.rsq_out = rsq1; q.keep_x = true;
          break;
        case 2:
          A = xa1; rsq_in = rsq1; q.mode = MODE_GATEUP; q.act_a = act_l;
          break;
        default:
          A = act_l; q.mode = MODE_RESID;
          q.gain = layer + 1 < a.le ? a.gains[layer + 1].g_attn : nullptr;
          q.xa_out = xa0 + 2 * a.xa_stride; q.rsq_out = rsq0 + 2 * a.rsq_stride; q.keep_x = layer + 1 < a.le;
          break;
      }
      if (q.mode == MODE_RESID && x_lds) r_gain_stage(q.gain, io, nt_x);
      bool first = true;
      while (!pw.done && pw.cur.layer == layer && pw.cur.gemm == gemm) {
        if (!first) {
          wait_vmcnt<0>();
          if (!io_barrier<NIO>(io)) return;
        }
        first = false;
        const Pass cur = pw.cur;
        if (!io_pass<MT, NW>(a, io, cur, pseq, A, rsq_in, q, L, x_lds, a_seq, [&]() { pw.next(); })) return;
        ++pseq;
        io_mark(io, 11);
      }
    }
  }
  io_mark(io, 2);
}

// ---- the persistent kernel ------------------------------------------------------------------------
template <int MT, int NW>
__global__ __launch_bounds__(WG_THREADS) void rstack_kernel(StackArgs a) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds_generic[];
  const lds_t lds = (lds_t)lds_generic;
  if (LA_TRACE_PTR(a) && blockIdx.x == 0 && threadIdx.x == 0) LA_TRACE_PTR(a)[13] = wall_clock64();  // (timeline: kernel entry)
  const int L = uni(*a.L_dev);
  if (L < 0 || L + a.Bp > a.max_len) {  // every workgroup takes the same exit: no barrier is left waiting
    if (blockIdx.x == 0 && threadIdx.x == 0) raise_error(a, 1);
    return;
  }
  if (threadIdx.x < 64) ((LDS_AS unsigned *)(lds + NW * Lay<MT, NW>::REG + M_CTL))[threadIdx.x] = 0u;
  const unsigned lds0 = (unsigned)(uintptr_t)lds;
  // The MFMA waves' schedules: the same for every launch of a model with this row-tile count, so they are worked out
  // once, when the model is created (schedule_tables_kernel), and every launch copies its workgroup's tables into LDS
  // (built here by one thread per MFMA wave they took 10 - 15 us at the start of every launch).
  {
    constexpr int N16 = NW * TAB_BYTES / 16;
    static_assert(NW * TAB_BYTES % 16 == 0, "whole 16-byte pieces");
    const u32x4 *src = reinterpret_cast<const u32x4 *>(a.sched) + (size_t)blockIdx.x * N16;
    LDS_AS u32x4 *dst = (LDS_AS u32x4 *)(lds + NW * Lay<MT, NW>::REG + M_BYTES);
    for (int i = threadIdx.x; i < N16; i += WG_THREADS) dst[i] = src[i];
  }
  __syncthreads();  // the only hardware barrier: from here on the waves run decoupled
  if (LA_TRACE_PTR(a) && blockIdx.x == 0 && threadIdx.x == 0) LA_TRACE_PTR(a)[14] = wall_clock64();  // (timeline: schedules written)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (wave < NW) {
    mfma_wave_main<MT, NW>(a, lds0, wave, lane);
    if (LA_TRACE_PTR(a) && lane == 0 && (blockIdx.x == 0 || blockIdx.x == 200)) LA_TRACE_PTR(a)[16 + (blockIdx.x ? 8 : 0) + wave] = wall_clock64();
    if (LA_TRACE_PTR(a) && lane == 0 && blockIdx.x > 2) LA_TRACE_PTR(a)[(size_t)TRACE_SLOTS * a.trace_phases + TRACE_WG * blockIdx.x + wave] = wall_clock64();
  } else {
    __builtin_amdgcn_s_setprio(3);  // (the IO waves' short bursts go first: measured neutral at 32 rows, 1.6 % on the one-row step; the other way round costs 0.8 %)
    io_wave_main<MT, NW>(a, lds0, wave - NW, lane, L);
    // a wait that gave up anywhere in the workgroup: tell the host
    if (lane == 0 && ctl_read(lds0 + NW * Lay<MT, NW>::REG + M_CTL + 4 * K_DEAD) != 0)
      raise_error(a, 4);
    if (LA_TRACE_PTR(a) && lane == 0 && (blockIdx.x == 0 || blockIdx.x == 200)) LA_TRACE_PTR(a)[16 + (blockIdx.x ? 8 : 0) + wave] = wall_clock64();  // (timeline: when each wave ends)
    if (LA_TRACE_PTR(a) && lane == 0 && blockIdx.x > 2) LA_TRACE_PTR(a)[(size_t)TRACE_SLOTS * a.trace_phases + TRACE_WG * blockIdx.x + wave] = wall_clock64();
    if (LA_TRACE_PTR(a) && wave == 7 && blockIdx.x == 0) {  // (timeline of MFMA wave 0: LDS -> the workgroup's trace words; the MFMA waves finish before the last epilogue)
      const unsigned v = ctl_read_lanes(lds0 + NW * Lay<MT, NW>::REG + M_BYTES + NW * TAB_BYTES + 4u * (unsigned)lane);
      LA_TRACE_PTR(a)[(size_t)TRACE_SLOTS * a.trace_phases + TRACE_WG + lane] = v;  // (the words of workgroups 1 and 2, which leave theirs alone)
    }
  }
}

// Writes the schedule tables of every workgroup of a launch shape (a.mode, the plans and a.seg_frags; ring slots per
// body as for the row-tile count that will use them) into out[workgroup][MFMA wave][TAB_BYTES].  Launched with the grid
// of the persistent kernel (the tables depend on the workgroup's index and the grid's size) and NW threads.
template <int NW>
__global__ void schedule_tables_kernel(StackArgs a, int ntmax, int ring, unsigned *out) {
  __shared__ __attribute__((aligned(16))) uint8_t tabs[NW * TAB_BYTES];
  const unsigned base = (unsigned)(uintptr_t)(lds_t)tabs;
  if (threadIdx.x < NW) {
    LDS_AS unsigned *mine = (LDS_AS unsigned *)(uintptr_t)(base + threadIdx.x * TAB_BYTES);
    for (int i = 0; i < TAB_BYTES / 4; ++i) mine[i] = 0u;
    build_schedule<NW>(a, ntmax, ring, (int)threadIdx.x, base + threadIdx.x * TAB_BYTES);
    unsigned *dst = out + ((size_t)blockIdx.x * NW + threadIdx.x) * (TAB_BYTES / 4);
    for (int i = 0; i < TAB_BYTES / 4; ++i) dst[i] = mine[i];
  }
}
template <int NW>
int write_schedule_tables(const StackArgs &a, int ring, unsigned *out, int n_wgs, hipStream_t s) {
  schedule_tables_kernel<NW><<<n_wgs, 64, 0, s>>>(a, Geo<1>::NTMAX, ring, out);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

// Run once per model: raises the kernel's LDS limit and checks that n_wgs workgroups can be resident at once on `cus`
// compute units (the grid barrier waits for all of them; what other work shares the GPU is the caller's concern).
template <int MT, int NW>
int prepare_rstack_kernel(int n_wgs, int cus) {
  constexpr int bytes = lds_bytes<MT, NW>();
  LA_HIP(hipFuncSetAttribute((const void *)rstack_kernel<MT, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  int per_cu = 0;
  LA_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, rstack_kernel<MT, NW>, WG_THREADS, bytes));
  LA_REQUIRE(per_cu >= 1 && n_wgs <= per_cu * cus, LA_EINVAL,
             "the persistent kernel for %d row tiles cannot keep %d workgroups resident (%d per compute unit on %d units)", MT, n_wgs,
             per_cu, cus);
  return LA_OK;
}

template <int MT, int NW>
int launch_rstack_kernel(const StackArgs &a, int n_wgs, hipStream_t s) {
  static bool attr_set = false;
  constexpr int bytes = lds_bytes<MT, NW>();
  static_assert(bytes <= 160 * 1024, "LDS of one CU");
  if (!attr_set) {
    LA_HIP(hipFuncSetAttribute((const void *)rstack_kernel<MT, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    attr_set = true;
  }
  rstack_kernel<MT, NW><<<n_wgs, WG_THREADS, bytes, s>>>(a);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

}  // namespace rs
}  // namespace la
