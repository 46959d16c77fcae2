// bf16 MFMA path for gfx950: weight-streaming skinny GEMMs, masked-block GQA attention,
// fused norm / RoPE / SwiGLU / residual epilogues, unembedding with fused arg-max.
//
// A verification step is bound by reading every weight once from HBM.  The block has at
// most 64 rows, so each 16-column x 32-k weight fragment (1 KB) feeds one or a few
// v_mfma_f32_16x16x32_bf16 and is never reused: weights go HBM -> registers -> MFMA with
// no LDS staging.  Layouts are chosen so that every load a wave issues is one contiguous
// 1 KB segment (64 lanes x 128 bit):
//
//   weights      [slab][k-tile][tile-in-slab][lane][8]   a slab is T 16-column tiles
//   activations  [k-tile][row-tile][lane][8]             bf16, the MFMA operand fragment
//   fragment     lane l holds index (l & 15) of the 16-wide dimension and the eight
//                contraction indices 8*(l >> 4) .. 8*(l >> 4)+7 of a 32-wide k-tile
//
// One GEMM workgroup (8 waves) owns a (slab, k-range) task; its waves split the k-range,
// accumulate in registers and are summed through LDS in a fixed tree, so results do not
// depend on timing.  Tasks whose k-range is a fraction of K write fp32 partials that the
// next (small) kernel adds in a fixed order, together with the residual stream, the
// RMSNorm statistics and the bf16 operand fragments of the following GEMM.
// RMSNorm is applied as (x * g) W scaled per row by rsqrt(mean(x^2) + eps) afterwards.
#include <algorithm>
#include <new>

#include "la_device.h"
#include "la_internal.h"

namespace la {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

constexpr int NW = 8;              // waves per GEMM workgroup
constexpr int GEMM_THREADS = NW * 64;
constexpr int MAX_T = 8;           // 16-column tiles per slab
constexpr int MAX_MT = LA_MAX_ROWS / 16;
constexpr int MAX_S = 8;           // k-splits across workgroups
constexpr unsigned OOB = 0x80000000u;  // voffset that no buffer of < 2 GiB contains

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

struct GemmPlan {
  int N = 0, K = 0, KT = 0;  // KT = K / 32
  int T = 1, n_slabs = 0;
  size_t bytes = 0;
};

enum GemmMode { MODE_PARTIAL = 0, MODE_GATEUP = 1, MODE_UNEMBED = 2 };

struct GemmArgs {
  const void *W;
  unsigned w_bytes;
  const void *A;
  unsigned a_bytes;
  int KT, S, n_tasks, Bp, N, mode;
  float *part;  // MODE_PARTIAL: [S][64][N]
  const float *rsq;  // [ncg][64] partial sums of squares of the residual stream
  int ncg;
  float inv_d, eps;
  uint16_t *act_a;  // MODE_GATEUP: activation fragments of the down projection
  Top *un_part;     // MODE_UNEMBED: [n_slabs][64]
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}

template <int MT, int T>
struct Depth {  // k-tiles in flight per wave, bounded by the register file
  static constexpr int raw = (200 - 4 * MT * T) / (4 * (MT + T));
  static constexpr int value = raw < 2 ? 2 : (raw > 6 ? 6 : raw);
};

// Sum over column groups of the partial sums of squares -> rsqrt(mean + eps) for rows < Bp.
__device__ __forceinline__ void row_scales_to_lds(const float *rsq, int ncg, float inv_d, float eps, int Bp,
                                                  float *rs_lds) {
  if ((int)threadIdx.x < Bp) {
    float s = 0.f;
    for (int c = 0; c < ncg; ++c) s += rsq[c * 64 + threadIdx.x];
    rs_lds[threadIdx.x] = 1.0f / sqrtf(s * inv_d + eps);
  }
}

template <int MT, int T>
__device__ __forceinline__ void gemm_task(const GemmArgs &g, int task, f32x4 *red, const float *rs_lds) {
  constexpr int D = Depth<MT, T>::value;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int slab = task / g.S, ks = task - slab * g.S;
  const int kt0 = (int)((long long)g.KT * ks / g.S), kt1 = (int)((long long)g.KT * (ks + 1) / g.S);
  const int nk = kt1 - kt0;
  const int wk0 = kt0 + nk * wave / NW, wk1 = kt0 + nk * (wave + 1) / NW;
  const int n = wk1 - wk0;
  __amdgpu_buffer_rsrc_t rw = make_rsrc(g.W, g.w_bytes), ra = make_rsrc(g.A, g.a_bytes);
  const unsigned w_base = (unsigned)(((size_t)slab * g.KT + wk0) * T * 1024);
  const unsigned a_base = (unsigned)wk0 * MT * 1024;
  const unsigned voff = lane * 16;

  f32x4 acc[MT][T];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < T; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  u32x4 rA[D][MT], rW[D][T];
  // Loads past the wave's k-range carry an out-of-range offset: the buffer unit returns
  // zeros without touching memory, and the MFMAs on them add nothing.  No branches.
  auto load = [&](int slot, int i) {
    unsigned vo = (i < n) ? voff : OOB;
#pragma unroll
    for (int t = 0; t < T; ++t)
      rW[slot][t] = __builtin_amdgcn_raw_buffer_load_b128(rw, vo, w_base + (unsigned)(i * T + t) * 1024, 0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      rA[slot][mt] = __builtin_amdgcn_raw_buffer_load_b128(ra, vo, a_base + (unsigned)(i * MT + mt) * 1024, 0);
  };
#pragma unroll
  for (int s = 0; s < D; ++s) load(s, s);
  for (int i0 = 0; i0 < n; i0 += D) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t)
          acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, rA[s][mt]),
                                                                __builtin_bit_cast(bf16x8, rW[s][t]), acc[mt][t], 0, 0, 0);
      load(s, i0 + s + D);
    }
  }

  // fixed-order tree over the 8 waves: (w, w+4), then (w, w+2), then (0, 1)
#pragma unroll
  for (int half = NW / 2; half >= 1; half >>= 1) {
    if (wave >= half && wave < 2 * half) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) red[((wave - half) * MT * T + mt * T + t) * 64 + lane] = acc[mt][t];
    }
    __syncthreads();
    if (wave < half) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < T; ++t) acc[mt][t] += red[(wave * MT * T + mt * T + t) * 64 + lane];
    }
    __syncthreads();
  }
  if (wave != 0) return;

  // acc[mt][t][i] is the element (row 16 mt + 4 (lane>>4) + i, packed column 16 (slab T + t) + (lane&15))
  const int q4 = lane >> 4, c16 = lane & 15;
  if (g.mode == MODE_PARTIAL) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int row = 16 * mt + 4 * q4 + i;
        if (row < g.Bp) {
          float *dst = g.part + ((size_t)ks * 64 + row) * g.N + (size_t)(slab * T) * 16 + c16;
#pragma unroll
          for (int t = 0; t < T; ++t) dst[t * 16] = acc[mt][t][i];
        }
      }
  } else if (g.mode == MODE_GATEUP) {
    // Slab columns: tile pairs (2p, 2p+1) hold gate and up of the same 16 FFN channels; with
    // T odd the last tile holds gate in columns 0..7 and up in columns 8..15 of 8 channels.
    const int Fg = 8 * T;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int p = 0; p < (T + 1) / 2; ++p) {
        const bool split_tile = (2 * p + 1 == T);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int row = 16 * mt + 4 * q4 + i;
          float gt, up;
          if (!split_tile) {
            gt = acc[mt][2 * p][i];
            up = acc[mt][(2 * p + 1 < T) ? 2 * p + 1 : 2 * p][i];
          } else {
            gt = acc[mt][2 * p][i];
            up = __shfl_xor(gt, 8, 64);
          }
          bool active = row < g.Bp && (!split_tile || c16 < 8);
          if (active) {
            float rs = rs_lds[row];
            gt *= rs;
            up *= rs;
            float a = gt / (1.0f + __expf(-gt)) * up;
            int f = slab * Fg + 16 * p + c16;
            size_t o = (((size_t)(f >> 5) * MT + mt) * 64 + (row & 15) + 16 * ((f & 31) >> 3)) * 8 + (f & 7);
            g.act_a[o] = float_to_bf16(a);
          }
        }
      }
    }
  } else {  // MODE_UNEMBED: arg-max over this slab's columns, per row
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Top best{-INFINITY, 0x7fffffff, -INFINITY};
#pragma unroll
        for (int t = 0; t < T; ++t) {
          Top c{acc[mt][t][i], (slab * T + t) * 16 + c16, -INFINITY};
          best = top_merge2(best, c);
        }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
          Top other;
          other.v1 = __shfl_xor(best.v1, o, 64);
          other.i1 = __shfl_xor(best.i1, o, 64);
          other.v2 = __shfl_xor(best.v2, o, 64);
          best = top_merge2(best, other);
        }
        int row = 16 * mt + 4 * q4 + i;
        if (c16 == 0 && row < g.Bp) g.un_part[(size_t)slab * 64 + row] = best;
      }
  }
}

template <int MT, int T>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(GemmArgs g) {
  extern __shared__ f32x4 lds[];
  float *rs_lds = (float *)(lds + (NW / 2) * MT * T * 64);
  if (g.mode == MODE_GATEUP) row_scales_to_lds(g.rsq, g.ncg, g.inv_d, g.eps, g.Bp, rs_lds);
  for (int task = blockIdx.x; task < g.n_tasks; task += gridDim.x) {
    gemm_task<MT, T>(g, task, lds, rs_lds);
    __syncthreads();
  }
}

// ---- weight packing (once, at model set-up) -----------------------------------------------
// Packed column pc of the destination -> (source matrix, source column).
//   kind 0: one source [K, N];  kind 1: q | k | v concatenation;  kind 2: gate/up interleave.
struct PackSrc {
  const uint16_t *s0, *s1, *s2;
  int n0, n1, n2;  // columns of each source
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
  int slab = pc / (16 * p.T), w = pc % (16 * p.T), t = w >> 4, c = w & 15;
  int Fg = 8 * p.T, f;
  bool up;
  if ((p.T & 1) && t == p.T - 1) {
    up = c >= 8;
    f = slab * Fg + (p.T / 2) * 16 + (c & 7);
  } else {
    up = t & 1;
    f = slab * Fg + (t >> 1) * 16 + c;
  }
  ld = p.F;
  return (up ? p.s1 : p.s0) + f;
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

// ---- residual update, norm statistics, operand fragments -----------------------------------
// One workgroup per group of 32 columns: x += sum_s part[s] (fixed order); writes the partial
// sum of squares of each row over these columns, and bf16(x * gain) in fragment layout.
__global__ void finish_kernel(float *x, int d, int Bp, const float *part, int S, int N, const float *gain,
                              uint16_t *xa, int MT, float *rsq) {
  int cg = blockIdx.x;
  int r = threadIdx.x >> 2, oct = threadIdx.x & 3;
  if (r >= Bp) return;
  int c0 = cg * 32 + oct * 8;
  float v[8];
  const float4 *xp = reinterpret_cast<const float4 *>(x + (size_t)r * d + c0);
  float4 a = xp[0], b = xp[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  for (int s = 0; s < S; ++s) {
    const float4 *pp = reinterpret_cast<const float4 *>(part + ((size_t)s * 64 + r) * N + c0);
    float4 pa = pp[0], pb = pp[1];
    v[0] += pa.x; v[1] += pa.y; v[2] += pa.z; v[3] += pa.w; v[4] += pb.x; v[5] += pb.y; v[6] += pb.z; v[7] += pb.w;
  }
  if (S > 0) {
    float4 *xo = reinterpret_cast<float4 *>(x + (size_t)r * d + c0);
    xo[0] = float4{v[0], v[1], v[2], v[3]};
    xo[1] = float4{v[4], v[5], v[6], v[7]};
  }
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) sq += v[i] * v[i];
  sq += __shfl_xor(sq, 1, 64);
  sq += __shfl_xor(sq, 2, 64);
  if (oct == 0) rsq[cg * 64 + r] = sq;
  if (gain) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t lo = float_to_bf16(v[2 * i] * gain[c0 + 2 * i]);
      uint32_t hi = float_to_bf16(v[2 * i + 1] * gain[c0 + 2 * i + 1]);
      w[i] = lo | (hi << 16);
    }
    size_t o = (((size_t)cg * MT + (r >> 4)) * 64 + (r & 15) + 16 * oct) * 8;
    *reinterpret_cast<uint4 *>(xa + o) = uint4{w[0], w[1], w[2], w[3]};
  }
}

// ---- QKV epilogue: reduce partials, norm scale, RoPE, q fragments, cache write --------------
// grid (Bp, Hq + 2 Hkv), 64 threads.  q is pre-multiplied by 1/sqrt(dh).
// q fragments: [kv head][q-row tile][dh k-tile][lane][8], q-row = j * 16 MT + b for the j-th
// query head of the group.
__global__ void qkv_finish_kernel(const float *part, int S, int N, const float *rsq, int ncg, float inv_d, float eps,
                                  const float *cs, int Hq, int Hkv, int dh, int MT, uint16_t *qf, uint16_t *Kc,
                                  uint16_t *Vc, const int32_t *L_dev, int max_len, int Bp, int32_t *err) {
  int b = blockIdx.x, hs = blockIdx.y;
  int L = *L_dev;
  if (L < 0 || L + Bp > max_len) {
    if (threadIdx.x == 0 && hs == 0) *err = 1;
    return;
  }
  float s = 0.f;
  for (int c = threadIdx.x; c < ncg; c += 64) s += rsq[c * 64 + b];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  float rs = 1.0f / sqrtf(s * inv_d + eps);
  int half = dh >> 1, g = Hq / Hkv;
  int col0 = hs * dh;
  auto val = [&](int c) {
    float a = 0.f;
    for (int k = 0; k < S; ++k) a += part[((size_t)k * 64 + b) * N + col0 + c];
    return a * rs;
  };
  if (hs < Hq + Hkv) {
    float qscale = hs < Hq ? 1.0f / sqrtf((float)dh) : 1.0f;
    for (int i = threadIdx.x; i < half; i += 64) {
      float c = cs[((size_t)b * half + i) * 2], sn = cs[((size_t)b * half + i) * 2 + 1];
      float x0 = val(i), x1 = val(i + half);
      float y0 = (x0 * c - x1 * sn) * qscale, y1 = (x1 * c + x0 * sn) * qscale;
      if (hs < Hq) {
        int kvh = hs / g, j = hs % g;
        int rt = j * MT + (b >> 4);
        auto qo = [&](int ch) {
          return ((((size_t)kvh * (g * MT) + rt) * (dh >> 5) + (ch >> 5)) * 64 + (b & 15) + 16 * ((ch & 31) >> 3)) * 8 + (ch & 7);
        };
        qf[qo(i)] = float_to_bf16(y0);
        qf[qo(i + half)] = float_to_bf16(y1);
      } else {
        size_t o = ((size_t)(L + b) * Hkv + (hs - Hq)) * dh;
        Kc[o + i] = float_to_bf16(y0);
        Kc[o + i + half] = float_to_bf16(y1);
      }
    }
  } else {
    int h = hs - Hq - Hkv;
    for (int c = threadIdx.x; c < dh; c += 64) Vc[v_index(true, L + b, h, c, Hkv, dh)] = float_to_bf16(val(c));
  }
}

// ---- masked-block GQA attention -----------------------------------------------------------
// One workgroup per (kv head, key split); its 4 waves take the q-row tiles of the head's
// group in turn.  Scores are computed transposed (keys x q-rows) so that the probabilities
// come out of the MFMA already in the operand layout of the second product:
//   S^T = K Q^T      A = K tile [16 keys x 32 dh],   B = q fragment        -> lane holds 4 keys of one q-row
//   O^T = V^T P^T    A = V^T tile [16 dh x 32 keys], B = (p of 2 key tiles) -> lane holds 4 channels of one q-row
// V is stored key-blocked (see v_index) to make the V^T tile a 128-bit load per lane.
// Partial results per split: O^T unnormalised, running max m and sum l per q-row.
template <int DH>
__global__ __launch_bounds__(256) void attention_kernel(const uint16_t *qf, const uint16_t *Kc, const uint16_t *Vc,
                                                        const int32_t *L_dev, int max_len, int Bp, int MT, int Hkv,
                                                        int g, const uint64_t *vis, int ns, float *o_part,
                                                        float *ml_part) {
  constexpr int KT = DH / 32, DT = DH / 16;
  const int kvh = blockIdx.x / ns, split = blockIdx.x % ns;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, q4 = lane >> 4, c16 = lane & 15;
  const int L = *L_dev;
  if (L < 0 || L + Bp > max_len) return;
  const int total = L + Bp;
  const int nkb = (total + 31) >> 5;
  const int kb0 = (int)((long long)nkb * split / ns), kb1 = (int)((long long)nkb * (split + 1) / ns);
  const int n_rt = g * MT, QR = n_rt * 16;
  for (int rt = wave; rt < n_rt; rt += 4) {
    const int b = (rt % MT) * 16 + c16;  // block row of this lane's q-row
    const uint64_t vb = b < Bp ? vis[b] : 0ull;
    bf16x8 q[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
      q[kt] = *reinterpret_cast<const bf16x8 *>(qf + ((((size_t)kvh * n_rt + rt) * KT + kt) * 64 + lane) * 8);
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -1e30f, l_run = 0.f;
    for (int kb = kb0; kb < kb1; ++kb) {
      f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
      const uint16_t *kr = Kc + ((size_t)(kb * 32 + c16) * Hkv + kvh) * DH + 8 * q4;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(kr + kt * 32);
        bf16x8 kbv = *reinterpret_cast<const bf16x8 *>(kr + (size_t)16 * Hkv * DH + kt * 32);
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, q[kt], sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kbv, q[kt], sb, 0, 0, 0);
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
      u32x4 pw;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        pw[i] = (uint32_t)float_to_bf16(p[2 * i]) | ((uint32_t)float_to_bf16(p[2 * i + 1]) << 16);
      bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
      const uint16_t *vr = Vc + (((size_t)kb * Hkv + kvh) * DH + c16) * 32 + 8 * q4;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        bf16x8 vt = *reinterpret_cast<const bf16x8 *>(vr + (size_t)dt * 16 * 32);
        o[dt] *= corr;
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pb, o[dt], 0, 0, 0);
      }
    }
    // o[dt][i] = O^T[channel 16 dt + 4 q4 + i][q-row rt*16 + c16]
    size_t base = ((size_t)kvh * ns + split) * DH * QR;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) o_part[base + (size_t)(16 * dt + 4 * q4 + i) * QR + rt * 16 + c16] = o[dt][i];
    if (q4 == 0) {
      size_t mo = (((size_t)kvh * ns + split) * QR + rt * 16 + c16) * 2;
      ml_part[mo] = m_run;
      ml_part[mo + 1] = l_run;
    }
  }
}

// Merge the key splits and write the attention output as operand fragments of the O GEMM.
// grid (Hkv, g*MT), 16 q-rows x (DH/8) channel octets per workgroup.
template <int DH>
__global__ void attn_combine_kernel(const float *o_part, const float *ml_part, int ns, int Hkv, int g, int MT, int Bp,
                                    uint16_t *attn_a) {
  int kvh = blockIdx.x, rt = blockIdx.y;
  int rr = threadIdx.x & 15, oct = threadIdx.x >> 4;
  if (oct >= DH / 8) return;
  int QR = g * MT * 16, r = rt * 16 + rr;
  int b = (rt % MT) * 16 + rr, j = rt / MT;
  if (b >= Bp) return;
  float M = -1e30f;
  for (int s = 0; s < ns; ++s) M = fmaxf(M, ml_part[(((size_t)kvh * ns + s) * QR + r) * 2]);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, lsum = 0.f;
  for (int s = 0; s < ns; ++s) {
    size_t mo = (((size_t)kvh * ns + s) * QR + r) * 2;
    float w = __expf(ml_part[mo] - M);
    lsum += w * ml_part[mo + 1];
    const float *op = o_part + ((size_t)kvh * ns + s) * DH * QR + (size_t)(oct * 8) * QR + r;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += w * op[(size_t)i * QR];
  }
  float inv = 1.0f / lsum;
  uint32_t w4[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w4[i] = (uint32_t)float_to_bf16(acc[2 * i] * inv) | ((uint32_t)float_to_bf16(acc[2 * i + 1] * inv) << 16);
  int col = (kvh * g + j) * DH + oct * 8;
  size_t o = (((size_t)(col >> 5) * MT + (b >> 4)) * 64 + (b & 15) + 16 * ((col & 31) >> 3)) * 8;
  *reinterpret_cast<uint4 *>(attn_a + o) = uint4{w4[0], w4[1], w4[2], w4[3]};
}

// Final arg-max over the slabs' partial results; logits are scaled by the row's norm factor.
__global__ void unembed_final_kernel(const Top *un_part, int n_slabs, const float *rsq, int ncg, float inv_d, float eps,
                                     int32_t *ids, float *top2) {
  __shared__ Top red[256];
  __shared__ float rs_s;
  int b = blockIdx.x;
  if (threadIdx.x < 64) {
    float s = 0.f;
    for (int c = threadIdx.x; c < ncg; c += 64) s += rsq[c * 64 + b];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (threadIdx.x == 0) rs_s = 1.0f / sqrtf(s * inv_d + eps);
  }
  Top t{-INFINITY, 0x7fffffff, -INFINITY};
  for (int s = threadIdx.x; s < n_slabs; s += blockDim.x) t = top_merge2(t, un_part[(size_t)s * 64 + b]);
  red[threadIdx.x] = t;
  __syncthreads();
  for (int o = blockDim.x / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] = top_merge2(red[threadIdx.x], red[threadIdx.x + o]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    ids[b] = red[0].i1;
    if (top2) {
      top2[b * 2] = red[0].v1 * rs_s;
      top2[b * 2 + 1] = red[0].v2 * rs_s;
    }
  }
}

// ---- host side ----------------------------------------------------------------------------
struct MfmaLayer {
  uint16_t *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wdown = nullptr;
};

struct MfmaModel {
  int n_wgs = 256;
  GemmPlan p_qkv, p_o, p_gu, p_down, p_un;
  std::vector<MfmaLayer> layers;
  uint16_t *un = nullptr;
  uint16_t *xa = nullptr, *attn_a = nullptr, *act_a = nullptr, *qf = nullptr;
  float *part = nullptr, *rsq = nullptr, *o_part = nullptr, *ml_part = nullptr;
  Top *un_part = nullptr;
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
      if (p.KT / S < NW && S > 1) continue;
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
    if (p.KT / S < NW && S > 1) continue;
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
  // packed matrices are addressed through 32-bit buffer offsets
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
  void *ps[] = {f->un, f->xa, f->attn_a, f->act_a, f->qf, f->part, f->rsq, f->o_part, f->ml_part, f->un_part};
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
  f->n_wgs = env_int("LA_WGS", prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256);
  int qd = m->qdim(), nqkv = m->nqkv(), g = d.n_q_heads / d.n_kv_heads;
  f->p_qkv = make_plan(nqkv, d.d_model, f->n_wgs, false, 0, "LA_T_QKV");
  f->p_o = make_plan(d.d_model, qd, f->n_wgs, false, 0, "LA_T_O");
  f->p_gu = make_plan(2 * d.d_ffn, d.d_model, f->n_wgs, true, d.d_ffn, "LA_T_GU");
  f->p_down = make_plan(d.d_model, d.d_ffn, f->n_wgs, false, 0, "LA_T_DOWN");
  f->p_un = make_plan(d.vocab, d.d_model, f->n_wgs, false, 0, "LA_T_UN");
  f->layers.resize(d.n_layers);
  size_t R = LA_MAX_ROWS;
  int n_max = std::max(nqkv, d.d_model);
  f->max_ns = std::max(1, std::min(64, f->n_wgs / d.n_kv_heads));
  size_t QR = (size_t)g * MAX_MT * 16;
  bool ok = true;
  ok = ok && (f->xa = (uint16_t *)dalloc(R * d.d_model * 2));
  ok = ok && (f->attn_a = (uint16_t *)dalloc(R * qd * 2));
  ok = ok && (f->act_a = (uint16_t *)dalloc(R * (size_t)d.d_ffn * 2));
  ok = ok && (f->qf = (uint16_t *)dalloc((size_t)d.n_kv_heads * QR * d.head_dim * 2));
  ok = ok && (f->part = (float *)dalloc((size_t)MAX_S * R * n_max * 4));
  ok = ok && (f->rsq = (float *)dalloc((size_t)(d.d_model / 32) * 64 * 4));
  ok = ok && (f->o_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * d.head_dim * 4));
  ok = ok && (f->ml_part = (float *)dalloc((size_t)d.n_kv_heads * f->max_ns * QR * 2 * 4));
  LA_REQUIRE(ok, LA_ENOMEM, "device allocation failed in the MFMA path");
  // pad rows of the operand buffers are read by the MFMAs: keep them finite
  LA_HIP(hipMemset(f->xa, 0, R * d.d_model * 2));
  LA_HIP(hipMemset(f->attn_a, 0, R * qd * 2));
  LA_HIP(hipMemset(f->act_a, 0, R * (size_t)d.d_ffn * 2));
  LA_HIP(hipMemset(f->qf, 0, (size_t)d.n_kv_heads * QR * d.head_dim * 2));
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

template <int MT, int T>
static int launch_gemm_t(const char *name, const GemmArgs &a, int n_wgs, hipStream_t s) {
  size_t lds = (size_t)(NW / 2) * MT * T * 64 * sizeof(f32x4) + 64 * sizeof(float);
  static bool attr_set = false;
  if (!attr_set) {
    LA_HIP(hipFuncSetAttribute((const void *)gemm_kernel<MT, T>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  ProfScope ps(name, s);
  int grid = std::min(a.n_tasks, n_wgs);
  gemm_kernel<MT, T><<<grid, GEMM_THREADS, lds, s>>>(a);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

template <int MT>
static int launch_gemm_mt(const char *name, int T, const GemmArgs &a, int n_wgs, hipStream_t s) {
  switch (T) {
    case 1: return launch_gemm_t<MT, 1>(name, a, n_wgs, s);
    case 2: return launch_gemm_t<MT, 2>(name, a, n_wgs, s);
    case 3: return launch_gemm_t<MT, 3>(name, a, n_wgs, s);
    case 4: return launch_gemm_t<MT, 4>(name, a, n_wgs, s);
    case 5: return launch_gemm_t<MT, 5>(name, a, n_wgs, s);
    case 6: return launch_gemm_t<MT, 6>(name, a, n_wgs, s);
    case 7: return launch_gemm_t<MT, 7>(name, a, n_wgs, s);
    case 8: return launch_gemm_t<MT, 8>(name, a, n_wgs, s);
  }
  set_error("unsupported tiles-per-slab %d", T);
  return LA_EINVAL;
}

static int launch_gemm(const char *name, int MT, int T, const GemmArgs &a, int n_wgs, hipStream_t s) {
  switch (MT) {
    case 1: return launch_gemm_mt<1>(name, T, a, n_wgs, s);
    case 2: return launch_gemm_mt<2>(name, T, a, n_wgs, s);
    case 3: return launch_gemm_mt<3>(name, T, a, n_wgs, s);
    case 4: return launch_gemm_mt<4>(name, T, a, n_wgs, s);
  }
  set_error("unsupported row-tile count %d", MT);
  return LA_EINVAL;
}

static GemmArgs base_args(const GemmPlan &p, const uint16_t *W, const uint16_t *A, int MT, int Bp, int S, int mode) {
  GemmArgs a{};
  a.W = W;
  a.w_bytes = (unsigned)p.bytes;
  a.A = A;
  a.a_bytes = (unsigned)((size_t)p.KT * MT * 1024);
  a.KT = p.KT;
  a.S = S;
  a.n_tasks = p.n_slabs * S;
  a.Bp = Bp;
  a.N = p.N;
  a.mode = mode;
  return a;
}

static int launch_finish(const char *name, float *x, int d, int Bp, const float *part, int S, int N, const float *gain,
                         uint16_t *xa, int MT, float *rsq, hipStream_t s) {
  ProfScope ps(name, s);
  finish_kernel<<<d / 32, 256, 0, s>>>(x, d, Bp, part, S, N, gain, xa, MT, rsq);
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int mfma_forward(la_model *m, int lb, int le, float *hidden, int Bp, const int32_t *pos, const uint64_t *vis,
                 la_kv *kv, hipStream_t s) {
  MfmaModel *f = m->mf;
  const la_model_desc &d = m->d;
  const int MT = ceil_div(Bp, 16), dm = d.d_model, g = d.n_q_heads / d.n_kv_heads;
  const int ncg = dm / 32;
  const float inv_d = 1.0f / (float)dm;
  int rc;
  if (lb == le) return LA_OK;
  if ((rc = launch_rope_table(m, pos, Bp, s))) return rc;
  const int S_qkv = choose_split(f->p_qkv, f->n_wgs, MT, "LA_S_QKV");
  const int S_o = choose_split(f->p_o, f->n_wgs, MT, "LA_S_O");
  const int S_down = choose_split(f->p_down, f->n_wgs, MT, "LA_S_DOWN");
  // key splits: about 4 blocks of 32 keys per workgroup, within the scratch that was sized at set-up
  int nkb = ceil_div(kv->L_bound + Bp, 32);
  int ns = std::max(1, std::min(f->max_ns, ceil_div(nkb, env_int("LA_ATTN_KB", 4))));
  if ((rc = launch_finish("prep_x", hidden, dm, Bp, nullptr, 0, 0, m->layers[lb].g_attn, f->xa, MT, f->rsq, s))) return rc;
  for (int l = lb; l < le; ++l) {
    const MfmaLayer &w = f->layers[l];
    uint16_t *Kc = (uint16_t *)kv->K + (size_t)l * kv->layer_elems();
    uint16_t *Vc = (uint16_t *)kv->V + (size_t)l * kv->layer_elems();
    {
      GemmArgs a = base_args(f->p_qkv, w.wqkv, f->xa, MT, Bp, S_qkv, MODE_PARTIAL);
      a.part = f->part;
      if ((rc = launch_gemm("gemm_qkv", MT, f->p_qkv.T, a, f->n_wgs, s))) return rc;
    }
    {
      ProfScope ps("qkv_finish", s);
      qkv_finish_kernel<<<dim3(Bp, d.n_q_heads + 2 * d.n_kv_heads), 64, 0, s>>>(
          f->part, S_qkv, f->p_qkv.N, f->rsq, ncg, inv_d, d.rms_eps, m->rope_cs, d.n_q_heads, d.n_kv_heads, d.head_dim,
          MT, f->qf, Kc, Vc, kv->L_dev, kv->max_len, Bp, kv->err_dev);
    }
    {
      ProfScope ps("attention", s);
      if (d.head_dim == 128)
        attention_kernel<128><<<d.n_kv_heads * ns, 256, 0, s>>>(f->qf, Kc, Vc, kv->L_dev, kv->max_len, Bp, MT,
                                                                 d.n_kv_heads, g, vis, ns, f->o_part, f->ml_part);
      else
        attention_kernel<64><<<d.n_kv_heads * ns, 256, 0, s>>>(f->qf, Kc, Vc, kv->L_dev, kv->max_len, Bp, MT,
                                                                d.n_kv_heads, g, vis, ns, f->o_part, f->ml_part);
    }
    {
      ProfScope ps("attn_combine", s);
      if (d.head_dim == 128)
        attn_combine_kernel<128><<<dim3(d.n_kv_heads, g * MT), 256, 0, s>>>(f->o_part, f->ml_part, ns, d.n_kv_heads, g,
                                                                             MT, Bp, f->attn_a);
      else
        attn_combine_kernel<64><<<dim3(d.n_kv_heads, g * MT), 128, 0, s>>>(f->o_part, f->ml_part, ns, d.n_kv_heads, g,
                                                                            MT, Bp, f->attn_a);
    }
    {
      GemmArgs a = base_args(f->p_o, w.wo, f->attn_a, MT, Bp, S_o, MODE_PARTIAL);
      a.part = f->part;
      if ((rc = launch_gemm("gemm_o", MT, f->p_o.T, a, f->n_wgs, s))) return rc;
    }
    if ((rc = launch_finish("finish_o", hidden, dm, Bp, f->part, S_o, dm, m->layers[l].g_mlp, f->xa, MT, f->rsq, s)))
      return rc;
    {
      GemmArgs a = base_args(f->p_gu, w.wgu, f->xa, MT, Bp, 1, MODE_GATEUP);
      a.rsq = f->rsq;
      a.ncg = ncg;
      a.inv_d = inv_d;
      a.eps = d.rms_eps;
      a.act_a = f->act_a;
      if ((rc = launch_gemm("gemm_gateup", MT, f->p_gu.T, a, f->n_wgs, s))) return rc;
    }
    {
      GemmArgs a = base_args(f->p_down, w.wdown, f->act_a, MT, Bp, S_down, MODE_PARTIAL);
      a.part = f->part;
      if ((rc = launch_gemm("gemm_down", MT, f->p_down.T, a, f->n_wgs, s))) return rc;
    }
    const float *next_gain = (l + 1 < le) ? m->layers[l + 1].g_attn : nullptr;
    if ((rc = launch_finish("finish_down", hidden, dm, Bp, f->part, S_down, dm, next_gain, f->xa, MT, f->rsq, s)))
      return rc;
  }
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int mfma_unembed_argmax(la_model *m, const float *hidden, int Bp, int32_t *ids, float *top2, hipStream_t s) {
  MfmaModel *f = m->mf;
  const la_model_desc &d = m->d;
  LA_REQUIRE(f->un != nullptr, LA_EINVAL, "model was created without an unembedding matrix");
  const int MT = ceil_div(Bp, 16), dm = d.d_model, ncg = dm / 32;
  int rc;
  if ((rc = launch_finish("prep_x", const_cast<float *>(hidden), dm, Bp, nullptr, 0, 0, m->g_final, f->xa, MT, f->rsq, s)))
    return rc;
  GemmArgs a = base_args(f->p_un, f->un, f->xa, MT, Bp, 1, MODE_UNEMBED);
  a.un_part = f->un_part;
  if ((rc = launch_gemm("gemm_unembed", MT, f->p_un.T, a, f->n_wgs, s))) return rc;
  {
    ProfScope ps("unembed_final", s);
    unembed_final_kernel<<<Bp, 256, 0, s>>>(f->un_part, f->p_un.n_slabs, f->rsq, ncg, 1.0f / (float)dm, d.rms_eps, ids,
                                            top2);
  }
  LA_HIP(hipGetLastError());
  return LA_OK;
}

}  // namespace la
