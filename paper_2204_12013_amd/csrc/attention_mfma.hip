// Tiled softmax attention on the gfx950 matrix cores (bf16 in, fp32 softmax and
// accumulation), head size 64 or 128, any sequence length.
//
// Forward: a wavefront owns 32 queries and streams 64-key tiles through LDS.  It
// computes the TRANSPOSED score tile S^T = K Q^T, so a lane owns one query and
// its registers run over keys: the row maximum and row sum of the online
// softmax are then plain per-lane reductions (one exchange with the other
// half-wave), and the rescaling of the running output is a per-lane scalar.
// The probabilities never leave registers: in the MFMA accumulator layout a
// lane's 16 values of a 32x32 tile are 16 keys of its query, which is exactly an
// operand fragment of O^T = V^T P^T once V is read from LDS with the transposing
// load (ds_read_b64_tr_b16) in the matching key order.  Only the per-row
// log-sum-exp is kept for the backward.
//
// Backward recomputes the probabilities from the log-sum-exp and uses no
// atomics: one kernel owns query rows (dQ), one owns key rows (dK, dV), so the
// result is bitwise reproducible.
#include "common.h"

namespace bamboo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMasked = -1.0e30f;
constexpr int TILE = 64;   // rows streamed through LDS per step

// Workgroup -> (row block, batch*head).  The grid is one-dimensional and ordered by row block
// first, all (batch, head) pairs of a row block being consecutive; with a causal mask the row
// blocks with the most key tiles to visit come first (HEAVY_LAST: the highest row block is the
// heaviest, as for query owners; otherwise the lowest, as for key owners), so the dispatcher
// hands out long workgroups first and the short ones fill the tail of the launch.
template <bool CAUSAL, bool HEAVY_LAST>
__device__ __forceinline__ void block_of(int nblk, int nbh, int* blk, int* bh) {
  const int i = blockIdx.x / nbh;
  *bh = blockIdx.x % nbh;
  *blk = (CAUSAL && HEAVY_LAST) ? nblk - 1 - i : i;
}

// ---- cooperative copy of 64 rows x D (bf16) global -> registers -> LDS -------------
// Rows at or beyond row_lim are read from row row_lim - 1 (finite values that the consumers' masks turn
// into exact zeros), so no load sits behind a branch.  A thread's byte offsets inside a tile and their
// upper limits (the same chunk in the last valid row) are computed once; per tile and chunk an add and a
// min remain.  Offsets are 32-bit: the launcher checks that a sequence stays below 4 GiB.
template <int D>
struct TileAddr {
  static constexpr int N = TILE * D / 8 / 256;   // 16-byte chunks per thread
  unsigned ofs[N], last[N];
  unsigned tile_bytes;                           // 64 rows
  __device__ __forceinline__ void init(long row_stride, int row_lim) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const unsigned col = (unsigned)((c % (D / 8)) * 8) * 2u;
      ofs[i] = (unsigned)(c / (D / 8)) * (unsigned)row_stride * 2u + col;
      last[i] = (unsigned)(row_lim - 1) * (unsigned)row_stride * 2u + col;
    }
    tile_bytes = (unsigned)TILE * (unsigned)row_stride * 2u;
  }
};
template <int D>
struct RowTile {
  static constexpr int N = TileAddr<D>::N;
  bf16x8 v[N];
  // tile: index of the 64-row tile counted from g (uniform)
  __device__ __forceinline__ void fetch(const bf16_t* g, const TileAddr<D>& ta, int tile) {
    const unsigned t0 = (unsigned)tile * ta.tile_bytes;
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = *(const bf16x8*)((const char*)g + min(t0 + ta.ofs[i], ta.last[i]));
  }
  __device__ __forceinline__ void stash(bf16_t* s, int ld) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      *(bf16x8*)(s + (c / (D / 8)) * ld + (c % (D / 8)) * 8) = v[i];
    }
  }
};

// Operand fragment with the contraction index contiguous in LDS: lane l holds
// row row_base + l%32, contraction elements 16*ks + 8*(l/32) .. +7.
__device__ __forceinline__ bf16x8 frag_k(const bf16_t* s, int ld, int row_base, int ks) {
  const int l = threadIdx.x & 63;
  return *(const bf16x8*)(s + (row_base + (l & 31)) * ld + ks * 16 + (l >> 5) * 8);
}
// Operand fragment with the contraction index running over LDS rows (transposing
// load): lane l holds column col_base + l%32; its 8 contraction slots are rows
// kbase + 4*(l/32) + {0..3} and kbase + 8 + 4*(l/32) + {0..3} -- the order in
// which a 32x32 accumulator tile hands 8 of a lane's 16 values to the next MFMA.
__device__ __forceinline__ bf16x8 frag_tr(const bf16_t* s, int ld, int col_base, int kbase) {
  const int l = threadIdx.x & 63, i = l & 15;
  const bf16_t* p = s + (kbase + 4 * (l >> 5) + (i >> 2)) * ld + col_base + ((l >> 4) & 1) * 16 + (i & 3) * 4;
  typedef __attribute__((address_space(3))) short4_t* lds_ptr;
  union { short4_t s4[2]; bf16x8 b; } u;
  u.s4[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  u.s4[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * ld));
  return u.b;
}
// registers 8*half .. 8*half+7 of an accumulator tile as a bf16 operand fragment
__device__ __forceinline__ bf16x8 pack8(const f32x16& t, int half) {
  bf16x8 o;
#pragma unroll
  for (int j = 0; j < 8; ++j) o[j] = (bf16_t)t[8 * half + j];
  return o;
}
// the value the lane 32 places away holds (v_permlane32_swap: no trip through LDS)
__device__ __forceinline__ float other_half(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0]: lanes 0..31 keep theirs, lanes 32..63 receive the lower half's; r[1]: the other way round
  const unsigned lo = r[0], hi = r[1];
  return __builtin_bit_cast(float, (threadIdx.x & 32) ? lo : hi);
}
// row index inside a 32x32 accumulator tile of register r for this lane
__device__ __forceinline__ int acc_row(int r) { return 8 * (r >> 2) + 4 * ((threadIdx.x & 63) >> 5) + (r & 3); }

// Per-lane operand fragments of 32 rows taken straight from global memory
// (lane l: row row0 + l%32, elements 16*ks + 8*(l/32) .. +7), zero beyond row_lim.
template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[D / 16], const bf16_t* g, long row_stride, int row0,
                                               int row_lim) {
  const int l = threadIdx.x & 63;
  const int row = row0 + (l & 31);
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    bf16x8 t = {};
    if (row < row_lim) t = *(const bf16x8*)(g + (long)row * row_stride + ks * 16 + (l >> 5) * 8);
    f[ks] = t;
  }
}

// Write a wavefront's transposed result (lane = output row, accumulator rows =
// feature index) through its private LDS area to global rows of D features.
// cs (optional): the lane's running sums of the 8 columns it stores (every pass meets the same 8, as 64 is a
// multiple of the chunks per row), over the rows it stores.
template <int D, bool SUM>
__device__ __forceinline__ void store_rows_impl(const f32x16 (&acc)[D / 32], float mul, bf16_t* stage, bf16_t* g,
                                                long row_stride, int row0, int row_lim, float (&cs)[8]) {
  constexpr int LD = D + 8;
  const int l = threadIdx.x & 63;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      bf16x4 o;
#pragma unroll
      for (int c = 0; c < 4; ++c) o[c] = (bf16_t)(acc[dt][4 * a + c] * mul);
      *(bf16x4*)(stage + (l & 31) * LD + dt * 32 + 8 * a + 4 * (l >> 5)) = o;
    }
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 32 * (D / 8) / 64; ++it) {
    const int idx = l + it * 64;
    const int row = idx / (D / 8), ch = (idx % (D / 8)) * 8;
    const bf16x8 t = *(const bf16x8*)(stage + row * LD + ch);
    if (row0 + row < row_lim) {
      *(bf16x8*)(g + (long)(row0 + row) * row_stride + ch) = t;
      if (SUM) {
#pragma unroll
        for (int j = 0; j < 8; ++j) cs[j] += (float)t[j];
      }
    }
  }
  __builtin_amdgcn_wave_barrier();
}

template <int D>
__device__ __forceinline__ void store_rows(const f32x16 (&acc)[D / 32], float mul, bf16_t* stage, bf16_t* g,
                                           long row_stride, int row0, int row_lim) {
  float unused[8];
  store_rows_impl<D, false>(acc, mul, stage, g, row_stride, row0, row_lim, unused);
}
template <int D>
__device__ __forceinline__ void store_rows_sum(const f32x16 (&acc)[D / 32], float mul, bf16_t* stage, bf16_t* g,
                                               long row_stride, int row0, int row_lim, float (&cs)[8]) {
  store_rows_impl<D, true>(acc, mul, stage, g, row_stride, row0, row_lim, cs);
}

// Column sums of what the workgroup's four wavefronts stored with store_rows (D columns, 128 rows): lanes that
// share a chunk first, then the wavefronts, both in a fixed order; written to dst[0..D).  xch: 4 * D floats of
// LDS that nobody else uses between the two barriers.  Must be reached by the whole workgroup.
template <int D>
__device__ __forceinline__ void block_colsum_write(float (&cs)[8], float* xch, float* dst) {
  constexpr int CH = D / 8;
  static_assert(64 % CH == 0, "a lane must keep its columns across passes");
  const int wave = threadIdx.x >> 6, l = threadIdx.x & 63;
#pragma unroll
  for (int o = CH; o < 64; o <<= 1)
#pragma unroll
    for (int j = 0; j < 8; ++j) cs[j] += __shfl_xor(cs[j], o, 64);
  __syncthreads();
  if (l < CH)
#pragma unroll
    for (int j = 0; j < 8; ++j) xch[wave * D + l * 8 + j] = cs[j];
  __syncthreads();
  if (wave == 0 && l < CH)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int c = l * 8 + j;
      dst[c] = ((xch[c] + xch[D + c]) + xch[2 * D + c]) + xch[3 * D + c];
    }
}

// =============================================================== forward
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(AttnDesc a) {
  constexpr int LDK = D + 8, LDV = D + 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* Ks = (bf16_t*)smem_raw;                 // [2][64][LDK]
  bf16_t* Vs = Ks + 2 * TILE * LDK;               // [2][64][LDV]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 5;
  const int H = a.heads * D, S = a.S;
  int qblk, bh;
  block_of<CAUSAL, true>((S + 127) / 128, a.B * a.heads, &qblk, &bh);
  const int b = bh / a.heads, h = bh % a.heads;
  const int q0 = qblk * 128, qw0 = q0 + wave * 32;
  const long rs = 3L * H;
  const bf16_t* base = (const bf16_t*)a.qkv + (long)b * S * rs + h * D;
  const float c = rsqrtf((float)D) * kLog2e;

  bf16x8 qf[D / 16];
  load_row_frags<D>(qf, base, rs, qw0, S);
  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
  float m_i = kMasked, l_i = 0.f;
  const int query = qw0 + (lane & 31);

  const int kend = CAUSAL ? min(S, q0 + 128) : S;
  const int nt = (kend + TILE - 1) / TILE;
  RowTile<D> kt_regs, vt_regs;
  TileAddr<D> ta;
  ta.init(rs, S);
  kt_regs.fetch(base + H, ta, 0);
  vt_regs.fetch(base + 2 * H, ta, 0);
  kt_regs.stash(Ks, LDK);
  vt_regs.stash(Vs, LDV);
  __syncthreads();
  for (int t = 0; t < nt; ++t) {
    const bf16_t* ks_ = Ks + (t & 1) * TILE * LDK;
    const bf16_t* vs_ = Vs + (t & 1) * TILE * LDV;
    const int k0 = t * TILE;
    if (t + 1 < nt) {
      kt_regs.fetch(base + H, ta, t + 1);
      vt_regs.fetch(base + 2 * H, ta, t + 1);
    }
    if (!CAUSAL || k0 <= qw0 + 31) {              // wave-uniform: tile not entirely above the diagonal
      f32x16 s[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[u][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int u = 0; u < 2; ++u)
          s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_k(ks_, LDK, u * 32, ks), qf[ks], s[u], 0, 0, 0);
      // Online softmax in the log2 domain.  The running maximum m_i is only raised when some row's
      // maximum has grown by more than 8 (a factor 256, harmless in fp32 and bf16): softmax is
      // invariant to the shift, and the rescaling of the running output then happens on a few
      // tiles instead of on every one.  Tiles that need no masking take a path without the
      // per-element index arithmetic (the choice is uniform over the wavefront).
      const bool need_mask = (k0 + TILE > S) || (CAUSAL && k0 + TILE - 1 > qw0);
      float mx = kMasked;
      if (need_mask) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = k0 + u * 32 + acc_row(r);
            const float v = (key >= S || (CAUSAL && key > query)) ? kMasked : s[u][r] * c;
            s[u][r] = v;
            mx = fmaxf(mx, v);
          }
      } else {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[u][r]);
        mx *= c;
      }
      mx = fmaxf(mx, other_half(mx));
      const bool grow = mx > m_i + 8.f;
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float m_new = grow ? mx : m_i;
        const float alpha = __builtin_amdgcn_exp2f(m_i - m_new);
        l_i *= alpha;
        m_i = m_new;
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      }
      if (need_mask) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[u][r] = __builtin_amdgcn_exp2f(s[u][r] - m_i);
      } else {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[u][r] = __builtin_amdgcn_exp2f(fmaf(s[u][r], c, -m_i));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 pb = pack8(s[u >> 1], u & 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) l_i += s[u >> 1][8 * (u & 1) + j];
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(vs_, LDV, dt * 32, 16 * u), pb, o[dt], 0, 0, 0);
      }
    }
    if (t + 1 < nt) {
      kt_regs.stash(Ks + ((t + 1) & 1) * TILE * LDK, LDK);
      vt_regs.stash(Vs + ((t + 1) & 1) * TILE * LDV, LDV);
    }
    __syncthreads();
  }
  const float l_tot = l_i + __shfl_xor(l_i, 32, 64);
  const float inv = 1.f / l_tot;
  bf16_t* stage = (bf16_t*)smem_raw + wave * 32 * (D + 8);
  store_rows<D>(o, inv, stage, (bf16_t*)a.ctx + (long)b * S * H + h * D, H, qw0, S);
  if (g == 0 && query < S) a.lse[((long)b * a.heads + h) * S + query] = (m_i + __builtin_amdgcn_logf(l_tot)) * kLn2;
}

// =============================================================== backward
// dQ: a wavefront owns 32 queries (lane = query) and streams 64-key tiles.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(AttnDesc a) {
  constexpr int LD = D + 8;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* Ks = (bf16_t*)smem_raw;                 // [2][64][LD]
  bf16_t* Vs = Ks + 2 * TILE * LD;                // [2][64][LD]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int H = a.heads * D, S = a.S;
  int qblk, bh;
  block_of<CAUSAL, true>((S + 127) / 128, a.B * a.heads, &qblk, &bh);
  const int b = bh / a.heads, h = bh % a.heads;
  const int q0 = qblk * 128, qw0 = q0 + wave * 32;
  const long rs = 3L * H;
  const bf16_t* base = (const bf16_t*)a.qkv + (long)b * S * rs + h * D;
  const bf16_t* dbase = (const bf16_t*)a.dctx + (long)b * S * H + h * D;
  const float scale = rsqrtf((float)D), c = scale * kLog2e;

  bf16x8 qf[D / 16], dof[D / 16];
  load_row_frags<D>(qf, base, rs, qw0, S);
  load_row_frags<D>(dof, dbase, H, qw0, S);
  const int query = qw0 + (lane & 31);
  const long sidx = ((long)b * a.heads + h) * S + min(query, S - 1);
  const float lse2 = a.lse[sidx] * kLog2e;
  // delta[q] = sum over the head's features of ctx * dctx: the two lanes of a query hold the two halves of
  // every 16-feature group of dctx already; the same pieces of ctx are read once.  The dK/dV kernel, which
  // runs after this one, takes delta from memory.
  float delta = 0.f;
  {
    bf16x8 of[D / 16];
    load_row_frags<D>(of, (const bf16_t*)a.ctx + (long)b * S * H + h * D, H, qw0, S);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
      for (int j = 0; j < 8; ++j) delta += (float)of[ks][j] * (float)dof[ks][j];
    delta += __shfl_xor(delta, 32, 64);
    if (lane < 32 && query < S) a.delta[sidx] = delta;
  }
  f32x16 dq[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  // the dP MFMAs start from -delta (a per-lane constant here: a lane owns a query), so their accumulator
  // comes out as dP - delta
  f32x16 neg_delta, zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    neg_delta[r] = -delta;
    zero16[r] = 0.f;
  }

  const int kend = CAUSAL ? min(S, q0 + 128) : S;
  const int nt = (kend + TILE - 1) / TILE;
  RowTile<D> kt_regs, vt_regs;
  TileAddr<D> ta;
  ta.init(rs, S);
  kt_regs.fetch(base + H, ta, 0);
  vt_regs.fetch(base + 2 * H, ta, 0);
  kt_regs.stash(Ks, LD);
  vt_regs.stash(Vs, LD);
  __syncthreads();
  for (int t = 0; t < nt; ++t) {
    const bf16_t* ks_ = Ks + (t & 1) * TILE * LD;
    const bf16_t* vs_ = Vs + (t & 1) * TILE * LD;
    const int k0 = t * TILE;
    if (t + 1 < nt) {
      kt_regs.fetch(base + H, ta, t + 1);
      vt_regs.fetch(base + 2 * H, ta, t + 1);
    }
    if (!CAUSAL || k0 <= qw0 + 31) {
      f32x16 s[2], dp[2];
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_k(ks_, LD, u * 32, ks), qf[ks], ks == 0 ? zero16 : s[u], 0, 0, 0);
          dp[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_k(vs_, LD, u * 32, ks), dof[ks], ks == 0 ? neg_delta : dp[u], 0,
                                                          0, 0);
        }
      const bool need_mask = (k0 + TILE > S) || (CAUSAL && k0 + TILE - 1 > qw0);
      if (need_mask) {                            // uniform over the wavefront
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = __builtin_amdgcn_exp2f(fmaf(s[u][r], c, -lse2));
            const int key = k0 + u * 32 + acc_row(r);
            if (key >= S || (CAUSAL && key > query)) p = 0.f;
            s[u][r] = p * dp[u][r];               // dS^T
          }
      } else {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[u][r] = __builtin_amdgcn_exp2f(fmaf(s[u][r], c, -lse2)) * dp[u][r];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 dsb = pack8(s[u >> 1], u & 1);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(ks_, LD, dt * 32, 16 * u), dsb, dq[dt], 0, 0, 0);
      }
    }
    if (t + 1 < nt) {
      kt_regs.stash(Ks + ((t + 1) & 1) * TILE * LD, LD);
      vt_regs.stash(Vs + ((t + 1) & 1) * TILE * LD, LD);
    }
    __syncthreads();
  }
  bf16_t* stage = (bf16_t*)smem_raw + wave * 32 * (D + 8);
  float* xch = (float*)((bf16_t*)smem_raw + 4 * 32 * (D + 8));     // behind the four staging areas
  if (a.dqkv_colsum != nullptr) {                                  // uniform over the grid
    float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_rows_sum<D>(dq, scale, stage, (bf16_t*)a.dqkv + (long)b * S * rs + h * D, rs, qw0, S, cs);
    float* part = a.dqkv_colsum + ((long)b * ((S + 127) / 128) + qblk) * rs;
    block_colsum_write<D>(cs, xch, part + h * D);
  } else {
    store_rows<D>(dq, scale, stage, (bf16_t*)a.dqkv + (long)b * S * rs + h * D, rs, qw0, S);
  }
}

// dK, dV: a wavefront owns 32 keys (lane = key) and streams 64-query tiles.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(AttnDesc a) {
  constexpr int LD = D + 8;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* Qs = (bf16_t*)smem_raw;                 // [2][64][LD]
  bf16_t* dOs = Qs + 2 * TILE * LD;               // [2][64][LD]
  float* lse_s = (float*)(dOs + 2 * TILE * LD);   // [2][64]  (log2 domain)
  float* del_s = lse_s + 2 * TILE;                // [2][64]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 5;
  const int H = a.heads * D, S = a.S;
  int kblk, bh;
  block_of<CAUSAL, false>((S + 127) / 128, a.B * a.heads, &kblk, &bh);
  const int b = bh / a.heads, h = bh % a.heads;
  const int kb0 = kblk * 128, kw0 = kb0 + wave * 32;
  const long rs = 3L * H;
  const bf16_t* base = (const bf16_t*)a.qkv + (long)b * S * rs + h * D;
  const bf16_t* dbase = (const bf16_t*)a.dctx + (long)b * S * H + h * D;
  const float* lse_g = a.lse + ((long)b * a.heads + h) * S;
  const float* del_g = a.delta + ((long)b * a.heads + h) * S;
  const float scale = rsqrtf((float)D), c = scale * kLog2e;

  bf16x8 kf[D / 16], vf[D / 16];
  load_row_frags<D>(kf, base + H, rs, kw0, S);
  load_row_frags<D>(vf, base + 2 * H, rs, kw0, S);
  const int key = kw0 + (lane & 31);
  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }

  const int qbeg = CAUSAL ? (kb0 / TILE) * TILE : 0;
  const int nt = (S - qbeg + TILE - 1) / TILE;
  RowTile<D> q_regs, do_regs;
  float lse_r = 0.f, del_r = 0.f;
  auto fetch_stats = [&](int q0t) {
    if (threadIdx.x < TILE) {
      const int q = q0t + threadIdx.x;
      lse_r = q < S ? lse_g[q] * kLog2e : 0.f;
      del_r = q < S ? -del_g[q] : 0.f;             // negated: the dP accumulators start from it
    }
  };
  auto stash_stats = [&](int buf) {
    if (threadIdx.x < TILE) {
      lse_s[buf * TILE + threadIdx.x] = lse_r;
      del_s[buf * TILE + threadIdx.x] = del_r;
    }
  };
  TileAddr<D> ta_q, ta_do;
  ta_q.init(rs, S);
  ta_do.init(H, S);
  q_regs.fetch(base, ta_q, qbeg / TILE);
  do_regs.fetch(dbase, ta_do, qbeg / TILE);
  fetch_stats(qbeg);
  q_regs.stash(Qs, LD);
  do_regs.stash(dOs, LD);
  stash_stats(0);
  __syncthreads();
  for (int t = 0; t < nt; ++t) {
    const int buf = t & 1;
    const bf16_t* qs_ = Qs + buf * TILE * LD;
    const bf16_t* dos_ = dOs + buf * TILE * LD;
    const int q0t = qbeg + t * TILE;
    if (t + 1 < nt) {
      q_regs.fetch(base, ta_q, qbeg / TILE + t + 1);
      do_regs.fetch(dbase, ta_do, qbeg / TILE + t + 1);
      fetch_stats(q0t + TILE);
    }
    if (!CAUSAL || q0t + TILE - 1 >= kw0) {       // wave-uniform: some query at or after the wave's first key
      // the queries' -delta runs along the accumulator registers here and comes from LDS with the tile: the
      // dP accumulators start from it and come out as dP - delta
      f32x16 s[2], dp[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
          const f32x4 d4 = *(const f32x4*)(del_s + buf * TILE + u * 32 + 8 * a4 + 4 * g);
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) dp[u][4 * a4 + cc] = d4[cc];
        }
      const f32x16 zero16 = {};
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_k(qs_, LD, u * 32, ks), kf[ks], ks == 0 ? zero16 : s[u], 0, 0, 0);
          dp[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_k(dos_, LD, u * 32, ks), vf[ks], dp[u], 0, 0, 0);
        }
      const bool need_mask = (q0t + TILE > S) || (kw0 + 32 > S) || (CAUSAL && q0t < kw0 + 31);
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
          const int row = u * 32 + 8 * a4 + 4 * g;   // first of 4 consecutive query rows of this lane
          const f32x4 l4 = *(const f32x4*)(lse_s + buf * TILE + row);
          if (need_mask) {                        // uniform over the wavefront
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
              const int r = 4 * a4 + cc;
              float p = __builtin_amdgcn_exp2f(fmaf(s[u][r], c, -l4[cc]));
              const int query = q0t + row + cc;
              if (query >= S || key >= S || (CAUSAL && key > query)) p = 0.f;
              s[u][r] = p;
              dp[u][r] *= p;                      // dS
            }
          } else {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
              const int r = 4 * a4 + cc;
              const float p = __builtin_amdgcn_exp2f(fmaf(s[u][r], c, -l4[cc]));
              s[u][r] = p;
              dp[u][r] *= p;                      // dS
            }
          }
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bf16x8 pb = pack8(s[u >> 1], u & 1);
        const bf16x8 dsb = pack8(dp[u >> 1], u & 1);
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(dos_, LD, dt * 32, 16 * u), pb, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(qs_, LD, dt * 32, 16 * u), dsb, dk[dt], 0, 0, 0);
        }
      }
    }
    if (t + 1 < nt) {
      q_regs.stash(Qs + (buf ^ 1) * TILE * LD, LD);
      do_regs.stash(dOs + (buf ^ 1) * TILE * LD, LD);
      stash_stats(buf ^ 1);
    }
    __syncthreads();
  }
  bf16_t* stage = (bf16_t*)smem_raw + wave * 32 * (D + 8);
  bf16_t* out = (bf16_t*)a.dqkv + (long)b * S * rs + h * D;
  float* xch = (float*)((bf16_t*)smem_raw + 4 * 32 * (D + 8));     // behind the four staging areas
  if (a.dqkv_colsum != nullptr) {                                  // uniform over the grid
    float* part = a.dqkv_colsum + ((long)b * ((S + 127) / 128) + kblk) * rs;
    float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_rows_sum<D>(dk, scale, stage, out + H, rs, kw0, S, cs);
    block_colsum_write<D>(cs, xch, part + H + h * D);
    float cv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    store_rows_sum<D>(dv, 1.f, stage, out + 2 * H, rs, kw0, S, cv);
    block_colsum_write<D>(cv, xch, part + 2 * H + h * D);
  } else {
    store_rows<D>(dk, scale, stage, out + H, rs, kw0, S);
    store_rows<D>(dv, 1.f, stage, out + 2 * H, rs, kw0, S);
  }
}

// ------------------------------------------------------------------ launchers
static bool covered(const AttnDesc& a) {
  if (a.d != 64 && a.d != 128) return false;
  // 32-bit byte offsets inside one sequence, the rows of a last, partial tile included (they are clamped after the add)
  if ((long)(a.S + TILE) * 3 * a.heads * a.d * 2 >= (1L << 32)) return false;
  auto misaligned = [](const void* p) { return p != nullptr && ((uintptr_t)p & 15) != 0; };
  return !(misaligned(a.qkv) || misaligned(a.ctx) || misaligned(a.dctx) || misaligned(a.dqkv));
}

template <int D, bool CAUSAL>
static hipError_t fwd_launch(hipStream_t s, const AttnDesc& a) {
  constexpr int BYTES = 2 * TILE * (D + 8) * 2 + 2 * TILE * (D + 16) * 2;
  constexpr auto kern = attn_fwd_mfma_kernel<D, CAUSAL>;
  const hipError_t e = ensure_lds_attribute<kern, BYTES>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(((a.S + 127) / 128) * a.B * a.heads), dim3(256), BYTES, s, a);
  return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t bwd_launch(hipStream_t s, const AttnDesc& a) {
  constexpr int BYTES_DQ = 4 * TILE * (D + 8) * 2;
  constexpr int BYTES_DKV = 4 * TILE * (D + 8) * 2 + 4 * TILE * 4;
  constexpr auto kq = attn_bwd_dq_mfma_kernel<D, CAUSAL>;
  constexpr auto kkv = attn_bwd_dkv_mfma_kernel<D, CAUSAL>;
  hipError_t e = ensure_lds_attribute<kq, BYTES_DQ>();
  if (e == hipSuccess) e = ensure_lds_attribute<kkv, BYTES_DKV>();
  if (e != hipSuccess) return e;
  dim3 grid(((a.S + 127) / 128) * a.B * a.heads);
  hipLaunchKernelGGL(kq, grid, dim3(256), BYTES_DQ, s, a);
  hipLaunchKernelGGL(kkv, grid, dim3(256), BYTES_DKV, s, a);
  if (a.dqkv_colsum != nullptr && a.dqkv_colsum_parts != nullptr) *a.dqkv_colsum_parts = a.B * ((a.S + 127) / 128);
  return hipGetLastError();
}

hipError_t launch_attention_fwd_mfma(hipStream_t s, const AttnDesc& a) {
  if (!covered(a)) return hipErrorNotSupported;
  if (a.d == 64) return a.causal ? fwd_launch<64, true>(s, a) : fwd_launch<64, false>(s, a);
  return a.causal ? fwd_launch<128, true>(s, a) : fwd_launch<128, false>(s, a);
}

hipError_t launch_attention_bwd_mfma(hipStream_t s, const AttnDesc& a) {
  if (!covered(a)) return hipErrorNotSupported;
  if (a.d == 64) return a.causal ? bwd_launch<64, true>(s, a) : bwd_launch<64, false>(s, a);
  return a.causal ? bwd_launch<128, true>(s, a) : bwd_launch<128, false>(s, a);
}

}  // namespace bamboo
