// Large-M prompt pass (Section 4.1 step 1, Section 6.3 "Prefill"; chunked prefill is the paper's named future work,
// Section 8): the whole prompt, up to PF_ROWS tokens at a time, goes through each layer as ONE matrix product per weight
// matrix, so the weights are read once per prompt chunk instead of once per 64 rows.  Included by la_mfma.hip (it needs
// the model's packed weight streams).
//
// Per layer: pf_prep (row factors of the norm, x * gain as half-precision MFMA operand fragments) -> pf_gemm QKV
// (epilogue: row factor, RoPE, K and V rows into the cache, q as operand fragments) -> pf_attn (causal flash attention
// of every 16-row tile over the cache) -> pf_gemm O (x += ...) -> pf_prep -> pf_gemm gate/up (epilogue: SwiGLU into operand
// fragments) -> pf_gemm down (x += ...).  The arithmetic is the block kernel's (half-precision operands, f32
// accumulation, the cache's 16-bit type in the attention); only the order of the sums differs.
//
// pf_gemm: one wave computes 64 rows x 128 columns (4 x 8 MFMA tiles, 128 accumulator registers) straight from
// memory: the activation operand is stored as MFMA fragments [k-tile][row tile][lane][8 halves] by its producer and a
// weight fragment is the 1 KB block of the per-CU streams the block kernel reads, so both operands are single 16-byte
// loads per lane and there is no LDS stage; the four waves of a workgroup share their rows (the A fragments hit L1) and
// take adjacent column groups.  Next k-tile's twelve fragments are requested before the current ones are multiplied.
#pragma once

namespace la {

constexpr int PF_ROWS = 1024;  // rows of one prompt chunk (buffers are sized for it)
constexpr int PF_MIN = 128;    // shorter prompts go through the block kernel
constexpr int PF_NS = 4;       // k-tiles a wave of the matrix product keeps in flight: all operands in registers
constexpr int PF_NS_LDS = 4;   // ... weight fragments through LDS (a step takes half the memory latency at four, measured)

enum PfMode { PF_QKV = 0, PF_RESID = 1, PF_GATEUP = 2 };

struct PfGemm {
  const uint8_t *wstream;
  size_t cu_bytes;
  unsigned frag0;  // fragment index of the layer inside a CU's region
  int G, NW;       // workgroups and MFMA waves the streams were packed for
  int n_prev, prev_ntiles[3], prev_KT[3];
  int ntiles, KT;
  const uint16_t *A;  // operand fragments [KT][RT][64][8]
  int RT, M;          // row tiles of the chunk (buffers hold RT4 = RT rounded up to 4), rows
  // epilogues
  float *x;           // RESID: residual stream [M][d], updated in place
  int d;
  const float *rs;    // QKV, GATEUP: row factors of the norm
  const float *cs;    // QKV: cos, sin [M][dh/2][2]
  uint16_t *Kc, *Vc;  // QKV: this layer's cache
  uint16_t *Q;        // QKV: q fragments [Hq][RT][dh/32][64][8]
  int L0, Hq, Hkv, dh, f16;
  uint16_t *act;      // GATEUP: operand fragments of the down projection [F/32][RT][64][8]
};

// The epilogue of a wave's tile.  The products are formed with the weight fragment as the MFMA's first operand, so
// a lane holds FOUR CONSECUTIVE COLUMNS of one row: acc[m][j][i] is row 16 (r0 + m) + c16, column 4 q4 + i of column
// tile t0 + j.  Every store is then an 8- or 16-byte vector (the cache's V layout aside), and the partner of a RoPE
// pair or of a gate channel (8 columns further) sits 32 lanes further.
template <int MODE, int NTW>
__device__ __forceinline__ void pf_epilogue(const PfGemm &p, const f32x4 (&acc)[4][NTW], int r0, int t0, int lane) {
  const int q4 = lane >> 4, c16 = lane & 15;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    const int t = t0 + j;
    if (t >= p.ntiles) continue;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int row = 16 * (r0 + m) + c16;
      const f32x4 v = acc[m][j];
      if (MODE == PF_RESID) {
        if (row < p.M) {
          f32x4 *xp = reinterpret_cast<f32x4 *>(p.x + (size_t)row * p.d + 16 * t + 4 * q4);
          *xp = *xp + v;
        }
      } else {
        const float rsf = row < p.M ? p.rs[row] : 0.f;
        f32x4 other;
#pragma unroll
        for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(v[i], 32, 64);
        if (row >= p.M) continue;
        if (MODE == PF_GATEUP) {
          // tile columns: 8 gate channels (lanes q4 = 0, 1), then the same 8 channels of up (q4 = 2, 3)
          if (q4 < 2) {
            float y[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float g = v[i] * rsf, u = other[i] * rsf;
              y[i] = g / (1.0f + __expf(-g)) * u;
            }
            const int ch = 8 * t + 4 * q4;
            *(u32x2 *)((uint8_t *)p.act + frag_piece(ch & ~7, row, p.RT) + 8 * (q4 & 1)) = u32x2{pack_f16(y[0], y[1]), pack_f16(y[2], y[3])};
          }
        } else {
          // tile columns: channels 8 jj .. 8 jj + 7 (q4 = 0, 1) and dh/2 + 8 jj .. (q4 = 2, 3) of head hs: eight RoPE pairs
          const int spj = p.dh >> 4, half = p.dh >> 1;
          const int hs = t / spj, jj = t - hs * spj;
          const int pr = 8 * jj + 4 * (q4 & 1);  // first of this lane's four pairs
          const int ch = q4 < 2 ? pr : half + pr;
          const bool h16 = p.f16 != 0;
          float y[4];
          if (hs < p.Hq + p.Hkv) {
            const float qscale = hs < p.Hq ? 1.0f / sqrtf((float)p.dh) : 1.0f;
            const f32x4 *csp = reinterpret_cast<const f32x4 *>(p.cs + ((size_t)row * half + pr) * 2);
            const f32x4 cs0 = csp[0], cs1 = csp[1];  // (cos, sin) of pairs pr .. pr + 3
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float c = i < 2 ? cs0[2 * i] : cs1[2 * (i - 2)], sn = i < 2 ? cs0[2 * i + 1] : cs1[2 * (i - 2) + 1];
              const float mine = v[i] * rsf, oth = other[i] * rsf;
              y[i] = (q4 < 2 ? mine * c - oth * sn : mine * c + oth * sn) * qscale;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) y[i] = v[i] * rsf;
          }
          if (hs < p.Hq) {
            const int KTq = p.dh >> 5;
            const size_t frag = ((size_t)hs * p.RT + (row >> 4)) * KTq + (ch >> 5);
            *(u32x2 *)(p.Q + (frag * 64 + (row & 15) + 16 * ((ch & 31) >> 3)) * 8 + (ch & 7)) = u32x2{pack_kv(h16, y[0], y[1]), pack_kv(h16, y[2], y[3])};
          } else if (hs < p.Hq + p.Hkv) {
            *(u32x2 *)(p.Kc + ((size_t)(p.L0 + row) * p.Hkv + (hs - p.Hq)) * p.dh + ch) = u32x2{pack_kv(h16, y[0], y[1]), pack_kv(h16, y[2], y[3])};
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) p.Vc[v_index(true, p.L0 + row, hs - p.Hq - p.Hkv, ch + i, p.Hkv, p.dh)] = kv_bits(h16, y[i]);
          }
        }
      }
    }
  }
}

// NTW: column tiles per wave (8: 128 columns, for the wide matrices; 4: 64 columns, so that the 4096-column matrices
// still give every CU a workgroup); NS: k-tiles in flight per wave (NS - 1 requested ahead of the one being multiplied).
template <int MODE, int NTW, int NS>
__global__ __launch_bounds__(256) void pf_gemm_kernel(PfGemm p) {
  const int wave = uni((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int q4 = lane >> 4, c16 = lane & 15;
  // Workgroup -> (row group, column group): workgroup b runs on XCD b % 8; all row groups of a column group get the same
  // XCD and consecutive turns there, so a weight fragment comes from memory once and the other row groups find it in that
  // XCD's L2 (the other order read every weight once per row group: 16 times for a 1024-token prompt).
  const int n_cg = (p.ntiles + NTW - 1) / NTW, n_cg4 = (n_cg + 3) / 4, RG = p.RT / 4;
  const int xcd = (int)blockIdx.x % 8, turn = (int)blockIdx.x / 8;
  const int rb = turn % RG, cg4 = (turn / RG) * 8 + xcd;
  const int cg = cg4 * 4 + wave;
  if (cg >= n_cg) return;
  const int r0 = rb * 4;  // first row tile
  // weight fragments of column tile t0 + j, k-tile kt: base_j + (before[kt % NW] + kt / NW) * nt_j KB
  const uint8_t *wb[NTW];
  unsigned wnt[NTW];
  const int t0 = cg * NTW;
#pragma unroll
  for (int j = 0; j < NTW; ++j) {
    const int t = t0 + j < p.ntiles ? t0 + j : p.ntiles - 1;  // (a group past the last tile repeats it; its result is dropped)
    const int c = t % p.G, lt = t / p.G;
    unsigned off = p.frag0;
    for (int i = 0; i < p.n_prev; ++i) off += (unsigned)((p.prev_ntiles[i] > c ? (p.prev_ntiles[i] - c + p.G - 1) / p.G : 0) * p.prev_KT[i]);
    wnt[j] = (unsigned)((p.ntiles - c + p.G - 1) / p.G);
    wb[j] = p.wstream + (size_t)c * p.cu_bytes + ((size_t)off + (unsigned)lt) * 1024u + (unsigned)lane * 16u;
  }
  const int nk_q = p.KT / p.NW, nk_r = p.KT % p.NW;  // wave w of the packing holds nk_q (+1 if w < nk_r) k-tiles
  const uint8_t *ab = (const uint8_t *)p.A + ((size_t)r0 * 64 + (unsigned)lane) * 16u;
  const size_t a_kt = (size_t)p.RT * 1024u;  // bytes from one k-tile's fragments to the next
  auto load = [&](int kt, u32x4 (&a)[4], u32x4 (&b)[NTW]) {
    const int w = kt % p.NW, i = kt / p.NW;
    const unsigned row = (unsigned)(w * nk_q + (w < nk_r ? w : nk_r) + i);  // k-tiles of the waves in front of w, then its own
#pragma unroll
    for (int m = 0; m < 4; ++m) a[m] = *(const u32x4 *)(ab + (size_t)kt * a_kt + (unsigned)m * 1024u);
#pragma unroll
    for (int j = 0; j < NTW; ++j) b[j] = *(const u32x4 *)(wb[j] + (size_t)row * wnt[j] * 1024u);
  };
  f32x4 acc[4][NTW];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto mul = [&](const u32x4 (&a)[4], const u32x4 (&b)[NTW]) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int j = 0; j < NTW; ++j)
        acc[m][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, b[j]), __builtin_bit_cast(f16x8, a[m]), acc[m][j], 0, 0, 0);
  };
  // A window of NS k-tiles: stage s holds k-tile kt with kt % NS == s (all indices are constants after unrolling).
  // The loop body has no branch (requests past the last k-tile repeat it and are never used): with a branch around a
  // request the compiler cannot count the requests in flight and waits for all of them at every use.
  u32x4 sa[NS][4], sb[NS][NTW];
  const int last_kt = p.KT - 1, n_full = p.KT / NS * NS;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) load(s < last_kt ? s : last_kt, sa[s], sb[s]);
  for (int kt0 = 0; kt0 < n_full; kt0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int nx = kt0 + s + NS - 1;
      load(nx < last_kt ? nx : last_kt, sa[(s + NS - 1) % NS], sb[(s + NS - 1) % NS]);
      __builtin_amdgcn_sched_barrier(0);  // (the requests stay in front of the products: the scheduler would sink them to their uses)
      mul(sa[s], sb[s]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  for (int kt = n_full; kt < p.KT; ++kt) {  // fewer than NS k-tiles left: one at a time
    load(kt, sa[0], sb[0]);
    mul(sa[0], sb[0]);
  }
  pf_epilogue<MODE, NTW>(p, acc, r0, t0, lane);
}

// The same product with the weight fragments shared through LDS: a workgroup's four waves take four consecutive 64-row
// groups of ONE column group, so the NTW weight fragments of a k-tile are fetched once per workgroup (each wave brings
// NTW / 4 of them with direct-to-LDS loads into a ring of NS stages) instead of once per wave; the activation fragments
// stay per wave in registers.  What a CU takes in per k-tile drops from 4 x (4 + NTW) KB to 16 + NTW KB, which is what
// bounded the first kernel.  One workgroup barrier per k-tile: past it every wave's part of the stage has landed and
// every wave is done reading the stage that the next requests overwrite.  Needs KT to be a multiple of NS.
template <int MODE, int NTW, int NS>
__device__ __forceinline__ void pf_gemm_lds_body(const PfGemm &p, LDS_AS uint8_t *pf_lds) {  // (device-only types: not in the kernel's own body, which the host pass instantiates too)
  static_assert(NTW % 4 == 0, "every wave brings the same number of weight fragments");
  constexpr int BW = NTW / 4;       // weight fragments a wave brings per k-tile
  constexpr int LPS = 4 + BW;       // this wave's requests per stage
  const int wave = uni((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int n_cg = (p.ntiles + NTW - 1) / NTW, RB = (p.RT / 4 + 3) / 4;
  const int xcd = (int)blockIdx.x % 8, turn = (int)blockIdx.x / 8;
  const int rb = turn % RB, cg = (turn / RB) * 8 + xcd;
  if (cg >= n_cg) return;  // (the whole workgroup)
  const int rg = rb * 4 + wave;                       // this wave's 64-row group
  const bool active = rg * 4 < p.RT;
  const int r0 = active ? rg * 4 : p.RT - 4;          // (a wave without rows runs along on the last group and drops the result)
  const int t0 = cg * NTW;
  const unsigned lds0 = (unsigned)(uintptr_t)pf_lds;
  // the weight fragments this wave brings: column tiles t0 + BW wave .. + BW - 1
  __amdgpu_buffer_rsrc_t wr[BW];
  unsigned wof[BW], wnt[BW];
#pragma unroll
  for (int jj = 0; jj < BW; ++jj) {
    const int tj = t0 + BW * wave + jj;
    const int t = tj < p.ntiles ? tj : p.ntiles - 1;
    const int c = uni(t % p.G), lt = uni(t / p.G);
    unsigned off = p.frag0;
    for (int i = 0; i < p.n_prev; ++i) off += (unsigned)((p.prev_ntiles[i] > c ? (p.prev_ntiles[i] - c + p.G - 1) / p.G : 0) * p.prev_KT[i]);
    wr[jj] = rsrc_of(p.wstream + (size_t)c * p.cu_bytes);
    wof[jj] = uni((off + (unsigned)lt) * 1024u);
    wnt[jj] = uni((unsigned)((p.ntiles - c + p.G - 1) / p.G) * 1024u);
  }
  const int nk_q = p.KT / p.NW, nk_r = p.KT % p.NW;
  const uint8_t *ab = (const uint8_t *)p.A + ((size_t)r0 * 64 + (unsigned)lane) * 16u;
  const size_t a_kt = (size_t)p.RT * 1024u;
  const unsigned voff = (unsigned)lane * 16u;
  auto request = [&](int kt, int slot, u32x4 (&a)[4]) {
    const int w = kt % p.NW, i = kt / p.NW;
    const unsigned row = (unsigned)(w * nk_q + (w < nk_r ? w : nk_r) + i);
#pragma unroll
    for (int jj = 0; jj < BW; ++jj)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(wr[jj], (LDS_AS void *)(uintptr_t)(lds0 + (unsigned)((slot * NTW + BW * wave + jj) * 1024)), 16, voff,
                                               uni(wof[jj] + row * wnt[jj]), 0, 0);
#pragma unroll
    for (int m = 0; m < 4; ++m) a[m] = *(const u32x4 *)(ab + (size_t)kt * a_kt + (unsigned)m * 1024u);
  };
  f32x4 acc[4][NTW];
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int j = 0; j < NTW; ++j) acc[m][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  u32x4 sa[NS][4];
  const int last_kt = p.KT - 1;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) request(s < last_kt ? s : last_kt, s, sa[s]);
  for (int kt0 = 0; kt0 < p.KT; kt0 += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      wait_vmcnt<(NS - 2) * LPS>();        // this wave's requests of stage s are in (the NS - 2 younger stages may be out)
      __atomic_signal_fence(__ATOMIC_SEQ_CST);
      __builtin_amdgcn_s_barrier();        // ... and everybody's; the stage before is read by nobody any more
      __atomic_signal_fence(__ATOMIC_SEQ_CST);  // (compiler fences: no LDS read moves across the barrier; no hardware wait for memory is wanted here)
      const int nx = kt0 + s + NS - 1;
      request(nx < last_kt ? nx : last_kt, (s + NS - 1) % NS, sa[(s + NS - 1) % NS]);
      __builtin_amdgcn_sched_barrier(0);
      u32x4 b[NTW];
#pragma unroll
      for (int j = 0; j < NTW; ++j) b[j] = *(LDS_AS const u32x4 *)(uintptr_t)(lds0 + (unsigned)((s * NTW + j) * 1024) + voff);
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
          acc[m][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, b[j]), __builtin_bit_cast(f16x8, sa[s][m]), acc[m][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  wait_vmcnt<0>();  // (the requests past the last k-tile land before the LDS is given back)
  if (active) pf_epilogue<MODE, NTW>(p, acc, r0, t0, lane);
}

template <int MODE, int NTW, int NS>
__global__ __launch_bounds__(256) void pf_gemm_lds_kernel(PfGemm p) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t pf_lds[];
  pf_gemm_lds_body<MODE, NTW, NS>(p, (LDS_AS uint8_t *)pf_lds);
}

// Row factors rsqrt(mean x^2 + eps) and the operand fragments of x * gain; one workgroup per row.  Rows M .. 16 RT4 - 1
// of the fragments are written as zeros (the matrix products read whole 64-row groups).
__global__ __launch_bounds__(256) void pf_prep_kernel(const float *x, const float *gain, int M, int d, int RT, float eps, float *rs, uint16_t *A) {
  const int row = blockIdx.x;
  __shared__ float red[4];
  float sq = 0.f;
  for (int c0 = threadIdx.x * 8; c0 < d; c0 += 256 * 8) {
    u32x4 out = {0u, 0u, 0u, 0u};
    if (row < M) {
      const float *xp = x + (size_t)row * d + c0;
      float y[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float v = xp[i];
        sq += v * v;
        y[i] = v * gain[c0 + i];
      }
      out = u32x4{pack_f16(y[0], y[1]), pack_f16(y[2], y[3]), pack_f16(y[4], y[5]), pack_f16(y[6], y[7])};
    }
    *(u32x4 *)((uint8_t *)A + frag_piece(c0, row, RT)) = out;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
  __syncthreads();
  if (threadIdx.x == 0 && row < M) rs[row] = 1.0f / sqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)d + eps);
}

// cos, sin of position L0 + row for every RoPE pair (double precision angles, as the block kernel's table)
__global__ void pf_rope_kernel(float *cs, int M, int half, int L0, double theta) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= M * half) return;
  const int row = e / half, i = e - row * half;
  const double inv = exp2(-(double)i / (double)half * log2(theta));
  double s, c;
  sincos((double)(L0 + row) * inv, &s, &c);
  cs[(size_t)e * 2] = (float)c;
  cs[(size_t)e * 2 + 1] = (float)s;
}

// Causal attention of one 16-row tile of one q head per wave over cache rows 0 .. L0 + row (Section 4.4's plain causal
// mask); the same products and running softmax as the block kernel's attention, one key block of 32 at a time, the next
// block's K requested when the scores are out of the matrix unit and its V after P V.  Output: operand fragments of the
// O projection.
template <int DH, bool F16>
__global__ __launch_bounds__(256) void pf_attn_kernel(const uint16_t *Q, const uint16_t *Kc, const uint16_t *Vc, uint16_t *out, int M, int RT, int RTr,
                                                      int L0, int Hq, int Hkv) {  // RT: row tiles the fragment buffers are laid out for; RTr: tiles that hold rows
  constexpr int KT = DH / 32, DT = DH / 16;
  using v8 = std::conditional_t<F16, f16x8, bf16x8>;
  auto mma = [](v8 x, v8 y, f32x4 c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(x, y, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, c, 0, 0, 0);
  };
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, q4 = lane >> 4, c16 = lane & 15;
  // the longest rows first: tiles are dealt from the end of the chunk
  const int task = blockIdx.x * 4 + wave;
  if (task >= RTr * Hq) return;
  const int rt = RTr - 1 - task / Hq, h = task % Hq, kvh = h / (Hq / Hkv);
  const int row = 16 * rt + c16;          // this lane's query row (as a column of the transposed scores)
  const int last = L0 + (row < M ? row : M - 1);  // last visible cache row
  v8 q[KT];
#pragma unroll
  for (int kt = 0; kt < KT; ++kt) q[kt] = *(const v8 *)(Q + ((((size_t)h * RT + rt) * KT + kt) * 64 + lane) * 8);
  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -1e30f, l_run = 0.f;
  u32x4 ka[KT], kb2[KT], vt[DT];
  auto load_k = [&](int kb) {
    const uint16_t *kp = Kc + (((size_t)(kb * 32 + c16) * Hkv + kvh) * DH + 8 * q4);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      ka[kt] = *(const u32x4 *)(kp + kt * 32);
      kb2[kt] = *(const u32x4 *)(kp + (size_t)16 * Hkv * DH + kt * 32);
    }
  };
  auto load_v = [&](int kb) {
    const uint16_t *vp = Vc + ((((size_t)kb * Hkv + kvh) * DH + c16) * 32 + 8 * q4);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) vt[dt] = *(const u32x4 *)(vp + dt * 16 * 32);
  };
  const int nkb = ((L0 + 16 * rt + 15 < L0 + M - 1 ? L0 + 16 * rt + 15 : L0 + M - 1) >> 5) + 1;  // blocks that hold a visible key of the tile
  load_k(0);
  load_v(0);
  for (int kb = 0; kb < nkb; ++kb) {
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      sa = mma(__builtin_bit_cast(v8, ka[kt]), q[kt], sa);
      sb = mma(__builtin_bit_cast(v8, kb2[kt]), q[kt], sb);
    }
    if (kb + 1 < nkb) load_k(kb + 1);
    float sv[8], p[8], mx = -1e30f;
    bool ok[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      sv[i] = i < 4 ? sa[i] : sb[i - 4];
      const int key = kb * 32 + (i >> 2) * 16 + 4 * q4 + (i & 3);
      ok[i] = key <= last;
      if (ok[i]) mx = fmaxf(mx, sv[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float corr = __expf(m_run - m_new);
    float ps = 0.f;
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
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      o[dt] *= corr;
      o[dt] = mma(__builtin_bit_cast(v8, vt[dt]), __builtin_bit_cast(v8, pw), o[dt]);
    }
    if (kb + 1 < nkb) load_v(kb + 1);
  }
  if (row < M) {
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int col = h * DH + 16 * dt + 8 * (q4 >> 1);
      *(u32x2 *)((uint8_t *)out + frag_piece(col, row, RT) + 8 * (q4 & 1)) =
          u32x2{pack_f16(o[dt][0] * inv, o[dt][1] * inv), pack_f16(o[dt][2] * inv, o[dt][3] * inv)};
    }
  }
}

__global__ void pf_embed_kernel(const uint16_t *E, const int32_t *tok, int V, int d, int half, float *x) {
  int t = tok[blockIdx.x];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const uint16_t b = E[(size_t)t * d + i];
    x[(size_t)blockIdx.x * d + i] = half ? (float)__builtin_bit_cast(_Float16, b) : __uint_as_float((uint32_t)b << 16);
  }
}

// ---- host side ----------------------------------------------------------------------------------------
static int pf_alloc(la_model *m, PfBuffers &b) {
  const la_model_desc &d = m->d;
  const size_t R = PF_ROWS;
  bool ok = true;
  ok = ok && (b.x = (float *)dalloc(R * d.d_model * 4));
  ok = ok && (b.rs = (float *)dalloc(R * 4));
  ok = ok && (b.cs = (float *)dalloc(R * d.head_dim * 4));
  ok = ok && (b.A = (uint16_t *)dalloc(R * d.d_model * 2));
  ok = ok && (b.Q = (uint16_t *)dalloc(R * (size_t)m->qdim() * 2));
  ok = ok && (b.attn = (uint16_t *)dalloc(R * (size_t)m->qdim() * 2));
  ok = ok && (b.act = (uint16_t *)dalloc(R * (size_t)d.d_ffn * 2));
  LA_REQUIRE(ok, LA_ENOMEM, "device allocation of the prefill buffers failed");
  // the fragments of rows past the prompt's end are read by the matrix products: keep them finite
  LA_HIP(hipMemset(b.Q, 0, R * (size_t)m->qdim() * 2));
  LA_HIP(hipMemset(b.attn, 0, R * (size_t)m->qdim() * 2));
  LA_HIP(hipMemset(b.act, 0, R * (size_t)d.d_ffn * 2));
  return LA_OK;
}


template <int MODE, int NTW>
static int pf_launch_gemm(const PfGemm &p, hipStream_t s, const char *name) {
  const int n_cg = (p.ntiles + NTW - 1) / NTW;
  ProfScope ps(name, s);
  if (p.KT % PF_NS_LDS == 0) {  // weight fragments shared through LDS
    const int RB = (p.RT / 4 + 3) / 4;
    pf_gemm_lds_kernel<MODE, NTW, PF_NS_LDS><<<RB * ((n_cg + 7) / 8 * 8), 256, PF_NS_LDS * NTW * 1024, s>>>(p);
  } else {
    const int n_cg4 = (n_cg + 3) / 4, row_groups = p.RT / 4;
    pf_gemm_kernel<MODE, NTW, PF_NS><<<row_groups * ((n_cg4 + 7) / 8 * 8), 256, 0, s>>>(p);
  }
  LA_HIP(hipGetLastError());
  return LA_OK;
}

int mfma_prefill_rows(const la_model *m) { return m->mf && m->mf->use_r && m->embed ? PF_ROWS : 0; }
int mfma_prefill_min() { return PF_MIN; }

// One prompt chunk of M <= PF_ROWS tokens at positions L0 .. L0 + M - 1 through every layer (the caller sets the cache
// length afterwards).
int mfma_prefill_chunk(la_model *m, la_kv *kv, const int32_t *tok, int M, int L0, hipStream_t s) {
  MfmaModel *f = m->mf;
  const la_model_desc &d = m->d;
  LA_REQUIRE(f->use_r, LA_EINVAL, "the large-M prompt pass reads the register-streaming kernel's weight layout");
  if (!f->pf.x) {
    int rc = pf_alloc(m, f->pf);
    if (rc) return rc;
  }
  PfBuffers &b = f->pf;
  const int RT = (M + 63) / 64 * 4, RTr = (M + 15) / 16, half = d.head_dim / 2, f16 = d.dtype == LA_F16;
  {
    ProfScope ps("pf_embed", s);
    pf_embed_kernel<<<M, 256, 0, s>>>((const uint16_t *)m->embed, tok, d.vocab, d.d_model, f16, b.x);
    pf_rope_kernel<<<ceil_div(M * half, 256), 256, 0, s>>>(b.cs, M, half, L0, (double)d.rope_theta);
  }
  LA_HIP(hipGetLastError());
  const GemmPlan *plans[4] = {&f->p_qkv, &f->p_o, &f->p_gu, &f->p_down};
  for (int l = 0; l < d.n_layers; ++l) {
    auto gemm_args = [&](int gi) {
      PfGemm p{};
      p.wstream = f->wstream;
      p.cu_bytes = f->cu_bytes;
      p.frag0 = (unsigned)l * f->seg_frags;
      p.G = f->n_wgs;
      p.NW = R_NW;
      p.n_prev = gi;
      for (int i = 0; i < gi; ++i) {
        p.prev_ntiles[i] = plans[i]->ntiles;
        p.prev_KT[i] = plans[i]->KT;
      }
      p.ntiles = plans[gi]->ntiles;
      p.KT = plans[gi]->KT;
      p.RT = RT;
      p.M = M;
      p.x = b.x;
      p.d = d.d_model;
      p.rs = b.rs;
      p.cs = b.cs;
      p.Kc = (uint16_t *)kv->K + (size_t)l * kv->layer_elems();
      p.Vc = (uint16_t *)kv->V + (size_t)l * kv->layer_elems();
      p.Q = b.Q;
      p.L0 = L0;
      p.Hq = d.n_q_heads;
      p.Hkv = d.n_kv_heads;
      p.dh = d.head_dim;
      p.f16 = f16;
      p.act = b.act;
      return p;
    };
    int rc;
    {
      ProfScope ps("pf_prep", s);
      pf_prep_kernel<<<16 * RT, 256, 0, s>>>(b.x, m->layers[l].g_attn, M, d.d_model, RT, d.rms_eps, b.rs, b.A);
    }
    PfGemm p = gemm_args(0);
    p.A = b.A;
    if ((rc = pf_launch_gemm<PF_QKV, 4>(p, s, "pf_gemm_qkv"))) return rc;
    {
      ProfScope ps("pf_attn", s);
      const int grid = ceil_div(RTr * d.n_q_heads, 4);
      const uint16_t *Kc = p.Kc, *Vc = p.Vc;
      if (d.head_dim == 128) {
        if (f16) pf_attn_kernel<128, true><<<grid, 256, 0, s>>>(b.Q, Kc, Vc, b.attn, M, RT, RTr, L0, d.n_q_heads, d.n_kv_heads);
        else pf_attn_kernel<128, false><<<grid, 256, 0, s>>>(b.Q, Kc, Vc, b.attn, M, RT, RTr, L0, d.n_q_heads, d.n_kv_heads);
      } else {
        if (f16) pf_attn_kernel<64, true><<<grid, 256, 0, s>>>(b.Q, Kc, Vc, b.attn, M, RT, RTr, L0, d.n_q_heads, d.n_kv_heads);
        else pf_attn_kernel<64, false><<<grid, 256, 0, s>>>(b.Q, Kc, Vc, b.attn, M, RT, RTr, L0, d.n_q_heads, d.n_kv_heads);
      }
    }
    p = gemm_args(1);
    p.A = b.attn;
    if ((rc = pf_launch_gemm<PF_RESID, 4>(p, s, "pf_gemm_o"))) return rc;
    {
      ProfScope ps("pf_prep", s);
      pf_prep_kernel<<<16 * RT, 256, 0, s>>>(b.x, m->layers[l].g_mlp, M, d.d_model, RT, d.rms_eps, b.rs, b.A);
    }
    p = gemm_args(2);
    p.A = b.A;
    if ((rc = pf_launch_gemm<PF_GATEUP, 4>(p, s, "pf_gemm_gateup"))) return rc;
    p = gemm_args(3);
    p.A = b.act;
    if ((rc = pf_launch_gemm<PF_RESID, 4>(p, s, "pf_gemm_down"))) return rc;
  }
  LA_HIP(hipGetLastError());
  return LA_OK;
}

}  // namespace la
