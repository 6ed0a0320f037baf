// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32
// accumulation, fused epilogues.  One kernel template covers the three forms
// the layer needs:
//   forward          Y  = X W      A K-contiguous,  B N-contiguous
//   input gradient   dX = dY W^T   A K-contiguous,  B K-contiguous
//   weight gradient  dW += X^T dY  A M-contiguous,  B N-contiguous
//
// A workgroup of 4 wavefronts (2 x 2) owns a (64*WM) x (64*WN) output tile and
// walks K in slices of 64, double-buffered in LDS.  The main kernel streams the
// slices global -> LDS directly and runs a hand-ordered, software-pipelined loop
// (see gemm_mfma_pl_kernel); a register-staged variant covers K that is not a
// multiple of 64.  Operands whose contraction index is contiguous
// in memory are kept as [row][k] in LDS and read with ds_read_b128; operands
// whose contraction index is strided are kept in their memory order [k][row]
// and read with the transposing LDS load (ds_read_b64_tr_b16), which hands each
// lane four consecutive k of its row, so no operand is ever transposed in
// registers or re-laid-out in HBM.  The accumulators leave through a
// wavefront-private LDS staging area so that bias / residual / GELU inputs are
// read and results written with 16-byte row-contiguous accesses.
#include <stdlib.h>

#include <atomic>
#include <type_traits>

#include <string.h>

#include "common.h"
#include "reduce_device.h"

namespace bamboo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---- GELU table -------------------------------------------------------------------------------
// The forward epilogue of the first FFN GEMM needs GELU(h) and GELU'(h) for 16.8 M values per call at
// the BERT-large stage; evaluated with exp and rcp that is ~28 vector instructions per value and as
// long as the GEMM's main loop.  Both results are stored as bf16, so it is enough to know
// Phi(h) = GELU(h) / h and GELU'(h) at the bf16 value nearest to h: a table over the bf16 values with
// 2^-11 <= |h| < 16 (15 exponents x 128 mantissas x 2 signs, fp32 pairs, 30 KB, kept in LDS) replaces
// the arithmetic by one LDS read.  Below 2^-11 Phi and GELU' are 0.5 to within 4e-4, above 16 they
// are 0 or 1 to fp32 precision, so clamping the index is exact enough at both ends.
constexpr int kGeluExpLo = 116, kGeluExpHi = 131;          // biased bf16 exponents covered
constexpr int kGeluN = (kGeluExpHi - kGeluExpLo) * 128;    // entries per sign
constexpr int kGeluBytes = 2 * kGeluN * 8;
__device__ float2 g_gelu_table[2 * kGeluN];

__global__ void gelu_table_init_kernel() {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 2 * kGeluN) return;
  const unsigned bits = ((unsigned)(i / kGeluN) << 15) | (unsigned)((kGeluExpLo << 7) + i % kGeluN);
  const float h = __uint_as_float(bits << 16);
  const float phi = 0.5f * (1.0f + erff(h * 0.70710678118654752f));
  g_gelu_table[i] = make_float2(phi, phi + h * expf(-0.5f * h * h) * 0.39894228040143268f);
}

// Fills the table once per device and waits for the fill: done by prepare_gemm_tables at set-up
// (stage_init); a GEMM with a GELU epilogue that finds it missing (the kernel used on its own, without a
// stage) does it on its first launch, the one launcher call that waits for the device.  A failed fill
// is tried again by the next caller.
static hipError_t ensure_gelu_table(hipStream_t s) {
  static std::mutex lock;
  static bool ready[kMaxDevices];
  const int dev = current_device_index();
  std::lock_guard<std::mutex> hold(lock);
  if (ready[dev]) return hipSuccess;
  hipLaunchKernelGGL(gelu_table_init_kernel, dim3((2 * kGeluN + 255) / 256), dim3(256), 0, s);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess) ready[dev] = true;
  return e;
}

// Set-up hook: fill the table now (and wait), so that no later launch has to.
hipError_t prepare_gemm_tables(hipStream_t s) { return ensure_gelu_table(s); }

// (GELU(h), GELU'(h)) from the table in LDS at byte address `tab`
__device__ __forceinline__ void gelu_pair_lookup(float h, unsigned tab, float* g, float* dg) {
  const bf16_t hb = (bf16_t)h;
  const unsigned b = __builtin_bit_cast(unsigned short, hb);
  int rel = (int)(b & 0x7fffu) - (kGeluExpLo << 7);
  rel = min(max(rel, 0), kGeluN - 1);
  const unsigned addr = tab + ((b & 0x8000u) ? kGeluN * 8 : 0) + rel * 8;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  const f32x2 t = *(__attribute__((address_space(3))) const f32x2*)(uintptr_t)addr;
  *g = h * t[0];
  *dg = t[1];
}

constexpr int BK = 64;          // k-slice
constexpr int KROW = BK + 8;    // LDS row length (elements) of a k-contiguous operand: 144 B, conflict-free b128 reads

template <int ROWS>
struct MnMajor {                 // LDS row length (elements) of an operand stored [k][row]
  static constexpr int LD = ROWS + 32;   // +64 B: the 4 k-rows x 64 B of a transposing read fall in distinct banks
};

template <int WM, int WN, bool A_K, bool B_K, bool GELU = false>
struct Smem {
  static constexpr int BM = 64 * WM, BN = 64 * WN;
  static constexpr int A_ELEMS = A_K ? BM * KROW : BK * MnMajor<BM>::LD;
  static constexpr int B_ELEMS = B_K ? BN * KROW : BK * MnMajor<BN>::LD;
  static constexpr int STAGE = A_ELEMS + B_ELEMS;                       // elements per pipeline stage
  static constexpr int EPI_LD = 32 * WN + 4;                             // floats per staged output row
  static constexpr int EPI_BYTES = 4 * 32 * EPI_LD * 4;                  // 4 waves x 32 rows
  static constexpr int MAIN_BYTES = 2 * STAGE * 2;
  static constexpr int TABLE_OFF = (MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES);   // GELU table behind the rest
  static constexpr int BYTES = TABLE_OFF + (GELU ? kGeluBytes : 0);
};

// ---- global -> register -> LDS copies of one operand slice --------------------
// K-contiguous operand: ROWS rows x 64 k.  Element (row, k) at g[row*ld + k].
template <int ROWS>
struct LoadK {
  static constexpr int N = ROWS / 32;    // 16-byte chunks per thread
  bf16x8 v[N];
  __device__ __forceinline__ void fetch(const bf16_t* g, long ld, int row0, int row_lim, int k0, int K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int row = c >> 3, kc = (c & 7) * 8;
      bf16x8 t = {};
      if (row0 + row < row_lim && k0 + kc < K) t = *(const bf16x8*)(g + (long)(row0 + row) * ld + k0 + kc);
      v[i] = t;
    }
  }
  __device__ __forceinline__ void stash(bf16_t* s) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      *(bf16x8*)(s + (c >> 3) * KROW + (c & 7) * 8) = v[i];
    }
  }
};
// Row-contiguous operand: 64 k-rows x ROWS.  Element (row, k) at g[k*ld + row].
template <int ROWS>
struct LoadMN {
  static constexpr int N = ROWS / 32;
  static constexpr int CPR = ROWS / 8;   // chunks per k-row
  bf16x8 v[N];
  __device__ __forceinline__ void fetch(const bf16_t* g, long ld, int row0, int row_lim, int k0, int K) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      const int kr = c / CPR, rc = (c % CPR) * 8;
      bf16x8 t = {};
      if (k0 + kr < K && row0 + rc < row_lim) t = *(const bf16x8*)(g + (long)(k0 + kr) * ld + row0 + rc);
      v[i] = t;
    }
  }
  __device__ __forceinline__ void stash(bf16_t* s) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = threadIdx.x + i * 256;
      *(bf16x8*)(s + (c / CPR) * MnMajor<ROWS>::LD + (c % CPR) * 8) = v[i];
    }
  }
};

// ---- LDS -> MFMA operand fragments ------------------------------------------------
// Fragment of a 32-row block for k-step ks (16 k): lane l holds row l%32,
// k = 8*(l/32) .. +7.
__device__ __forceinline__ bf16x8 frag_k(const bf16_t* s, int row_base, int ks) {
  const int l = threadIdx.x & 63;
  return *(const bf16x8*)(s + (row_base + (l & 31)) * KROW + ks * 16 + (l >> 5) * 8);
}
template <int ROWS>
__device__ __forceinline__ bf16x8 frag_mn(const bf16_t* s, int row_base, int ks) {
  // transposing read: within 16 lanes, lane i addresses k-row i/4, columns 4*(i%4)..+3,
  // and receives rows k..k+3 of column i
  const int l = threadIdx.x & 63, i = l & 15;
  const int col = row_base + ((l >> 4) & 1) * 16 + (i & 3) * 4;
  const int k = ks * 16 + (l >> 5) * 8 + (i >> 2);
  const bf16_t* p = s + k * MnMajor<ROWS>::LD + col;
  typedef __attribute__((address_space(3))) short4_t* lds_ptr;
  const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * MnMajor<ROWS>::LD));
  union { short4_t s4[2]; bf16x8 b; } u;
  u.s4[0] = lo;
  u.s4[1] = hi;
  return u.b;
}


// ---- direct global -> LDS copies (global_load_lds_dwordx4) -----------------------
// The load writes 16 bytes per lane to consecutive LDS addresses starting at a
// wavefront-uniform base, so a slice cannot be padded per row.  Bank conflicts
// are avoided instead by choosing WHICH 16-byte chunk of global memory each
// lane fetches: chunks are XOR-swizzled inside their LDS row, and the fragment
// readers apply the same XOR.  Out-of-range rows are clamped to a valid row (they
// only feed output rows/columns that are never stored); K must be a multiple of
// the 64-wide slice.
// The load is inline assembly so that the compiler's wait-count insertion does
// not see an LDS write that "may alias" every later LDS read and serialise the
// copy with the MFMAs; the kernel waits on vmcnt itself before the barrier
// that publishes a slice.  M0 carries the wavefront-uniform LDS base.

// ---- epilogue ---------------------------------------------------------------------------
// The accumulators leave through a wavefront-private LDS staging area, one 32-row block of the
// wave's sub-tile at a time; afterwards lane l owns, for pass `it`, the 8 consecutive outputs of
// chunk idx = l + 64 * it of the staged 32 x (32 * WN) block (row idx / CHUNKS, columns
// 8 * (idx % CHUNKS) ..).  What the epilogue has to read from memory for those outputs (residual,
// stored activation derivative, fp32 gradient to add to) is known long before the accumulators are
// final: EpiOperands::issue requests one row block's worth.  The kernel calls it for row block 0
// ahead of the last slices of the main loop, so the latency is covered by MFMAs, and write_tile
// requests row block i + 1 before it works on row block i.
template <int WM, int WN, int EPI>
struct EpiOperands {
  static constexpr int CHUNKS = 4 * WN, ITS = 32 * CHUNKS / 64;
  static constexpr bool BF = EPI == EPI_BIAS_RES || EPI == EPI_RES || EPI == EPI_MUL;
  static constexpr bool F32 = EPI == EPI_ACC_F32;
  static constexpr bool PRE = BF || F32;
  static constexpr bool HASB = EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU;
  static constexpr int NLOADS = BF ? ITS : (F32 ? 2 * ITS : 0);   // load instructions per lane and row block
  bf16x8 b[BF ? ITS : 1];
  f32x4 f[F32 ? ITS : 1][2];
  // The bias of a lane's columns is the same for every row block: fetched once per tile, at its start
  // (a load inside the row-block loop would put its latency on every block).
  bf16x8 bias[HASB ? ITS : 1];
  __device__ __forceinline__ void issue_bias(const GemmDesc& d, int n0) {
    if (!HASB) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wn = wave & 1;
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      const int n = min(n0 + wn * 32 * WN + ((lane + it * 64) % CHUNKS) * 8, d.N - 8);
      bias[it] = *(const bf16x8*)((const bf16_t*)d.bias + n);
    }
  }
  // Rows / columns past the edge are clamped to the last valid ones (their values are never used), so
  // that every lane issues exactly NLOADS loads: the main loop counts them in its vmcnt waits.
  __device__ __forceinline__ void issue(const GemmDesc& d, int m0, int n0, int i) {
    if (!PRE) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const void* src = EPI == EPI_MUL ? d.aux_in : (F32 ? (const void*)d.C : d.res);
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
      const int idx = lane + it * 64;
      const int m = min(m0 + wm * 32 * WM + i * 32 + idx / CHUNKS, d.M - 1);
      const int n = min(n0 + wn * 32 * WN + (idx % CHUNKS) * 8, d.N - 8);
      const long e = (long)m * d.N + n;
      if (BF) b[it] = *(const bf16x8*)((const bf16_t*)src + e);
      if (F32) {
        f[it][0] = *(const f32x4*)((const float*)src + e);
        f[it][1] = *(const f32x4*)((const float*)src + e + 4);
      }
    }
  }
};

// epilogue on 8 consecutive outputs of one row; `pb` / `pf` are the operands fetched ahead
template <int EPI>
__device__ __forceinline__ void epilogue8(const GemmDesc& d, int m, int n, const float (&acc)[8], const bf16x8& pb,
                                          const f32x4 (&pf)[2], const bf16x8& pbias, unsigned gelu_tab,
                                          float* stored = nullptr) {
  const long i = (long)m * d.N + n;
  if (EPI == EPI_ACC_F32) {
    float* c = (float*)d.C + i;
    f32x4 a = pf[0], b = pf[1];
#pragma unroll
    for (int j = 0; j < 4; ++j) { a[j] += acc[j]; b[j] += acc[4 + j]; }
    *(f32x4*)c = a;
    *(f32x4*)(c + 4) = b;
    return;
  }
  float v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = acc[j];
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += (float)pbias[j];
  }
  if (EPI == EPI_BIAS_RES || EPI == EPI_RES) {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += (float)pb[j];
  }
  bf16x8 o;
  if (EPI == EPI_MUL) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      o[j] = (bf16_t)(v[j] * (float)pb[j]);
      if (stored != nullptr) stored[j] = (float)o[j];
    }
  } else if (EPI == EPI_BIAS_GELU) {
    bf16x8 g;
#pragma unroll
    for (int j = 0; j < 8; ++j) {   // activation and its derivative, looked up at the nearest bf16 value
      float gv, dgv;
      gelu_pair_lookup(v[j], gelu_tab, &gv, &dgv);
      g[j] = (bf16_t)gv;
      o[j] = (bf16_t)dgv;
    }
    *(bf16x8*)((bf16_t*)d.aux_out + i) = g;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (bf16_t)v[j];
  }
  *(bf16x8*)((bf16_t*)d.C + i) = o;
}

// Accumulators -> wavefront-private LDS rows -> 16-byte global accesses.  `first` holds the operands
// of row block 0 (requested by the caller).
template <int WM, int WN, int EPI, int EPI_LD>
__device__ __forceinline__ void write_tile(const GemmDesc& d, f32x16 (&acc)[WM][WN], float* stage_all, int m0, int n0,
                                           const EpiOperands<WM, WN, EPI>& first, unsigned gelu_tab) {
  typedef EpiOperands<WM, WN, EPI> Ops;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 1, wn = wave & 1;
  float* stage = stage_all + wave * 32 * EPI_LD;
  Ops ops[2];
  ops[0] = first;
  // Column sums of the stored outputs (EPI_MUL with d.tile_colsum): where 64 is a multiple of the chunks per
  // staged row, a lane meets the same 8 columns in every pass, so it keeps 8 running sums over its rows.
  constexpr bool CAN_SUM = EPI == EPI_MUL && 64 % Ops::CHUNKS == 0;
  const bool sum_cols = CAN_SUM && d.tile_colsum != nullptr;
  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    if (i + 1 < WM) ops[(i + 1) & 1].issue(d, m0, n0, i + 1);
    const Ops& cur = ops[i & 1];
    // D[row][col]: lane holds col = lane%32, rows 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        stage[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * EPI_LD + j * 32 + (lane & 31)] = acc[i][j][r];
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the wave's own LDS writes have landed
    __builtin_amdgcn_wave_barrier();
    constexpr int CHUNKS = Ops::CHUNKS;   // 8-float chunks per staged row
#pragma unroll
    for (int it = 0; it < Ops::ITS; ++it) {
      const int idx = lane + it * 64;
      const int row = idx / CHUNKS, ch = idx % CHUNKS;
      const int m = m0 + wm * 32 * WM + i * 32 + row;
      const int n = n0 + wn * 32 * WN + ch * 8;
      const f32x4 lo = *(const f32x4*)(stage + row * EPI_LD + ch * 8);
      const f32x4 hi = *(const f32x4*)(stage + row * EPI_LD + ch * 8 + 4);
      if (m < d.M && n < d.N) {
        const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        if (CAN_SUM) {
          float st8[8];
          epilogue8<EPI>(d, m, n, v, cur.b[Ops::BF ? it : 0], cur.f[Ops::F32 ? it : 0], first.bias[Ops::HASB ? it : 0],
                         gelu_tab, st8);
#pragma unroll
          for (int j = 0; j < 8; ++j) cs[j] += st8[j];
        } else {
          epilogue8<EPI>(d, m, n, v, cur.b[Ops::BF ? it : 0], cur.f[Ops::F32 ? it : 0], first.bias[Ops::HASB ? it : 0],
                         gelu_tab);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();      // reads done before the next row block overwrites the stage
  }
  if (CAN_SUM) {
    if (sum_cols) {     // uniform over the workgroup
      // lanes that share a chunk (same lane % CHUNKS), in a fixed order; then the two wavefronts that share
      // the columns (wm = 0, 1), again in a fixed order
#pragma unroll
      for (int o = Ops::CHUNKS; o < 64; o <<= 1)
#pragma unroll
        for (int j = 0; j < 8; ++j) cs[j] += __shfl_xor(cs[j], o, 64);
      float* xch = stage_all;               // [2 wn][CHUNKS][8]: the staging area is free now
      __syncthreads();
      if (wm == 1 && lane < Ops::CHUNKS)
#pragma unroll
        for (int j = 0; j < 8; ++j) xch[(wn * Ops::CHUNKS + lane) * 8 + j] = cs[j];
      __syncthreads();
      if (wm == 0 && lane < Ops::CHUNKS) {
        const int n = n0 + wn * 32 * WN + lane * 8;
        if (n < d.N) {
          float* dst = d.tile_colsum + (long)(m0 / (64 * WM)) * d.N + n;
#pragma unroll
          for (int j = 0; j < 8; ++j) dst[j] = cs[j] + xch[(wn * Ops::CHUNKS + lane) * 8 + j];
        }
      }
    }
  }
}

// Tile order: consecutive workgroup ids are spread round-robin over the 8 XCDs,
// each with its own L2.  Give every XCD a contiguous range of tiles (xcd_range), and inside
// the range walk down GROUP rows of tiles before moving to the next column (tile_walk), so
// that the tiles an XCD works on at one time share operand slices in its L2.
__device__ __forceinline__ int xcd_range(int pid, int total) {
  const int per = total / 8;
  return pid < per * 8 ? (pid % 8) * per + pid / 8 : pid;
}
__device__ __forceinline__ void tile_walk(int pid, int tiles_m, int tiles_n, int* tm, int* tn) {
  constexpr int GROUP = 8;
  const int width = GROUP * tiles_n;
  const int group = pid / width;
  const int first_m = group * GROUP;
  const int rows = min(tiles_m - first_m, GROUP);
  *tm = first_m + (pid % width) % rows;
  *tn = (pid % width) / rows;
}

template <int WM, int WN, bool A_K, bool B_K, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmDesc d) {
  typedef Smem<WM, WN, A_K, B_K, EPI == EPI_BIAS_GELU> SM;
  constexpr int BM = SM::BM, BN = SM::BN;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = (bf16_t*)smem_raw;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;       // 2 x 2 wavefronts
  int tile_m, tile_n;
  {
    const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
    tile_walk(xcd_range(blockIdx.x, tiles_m * tiles_n), tiles_m, tiles_n, &tile_m, &tile_n);
  }
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const bf16_t* A = (const bf16_t*)d.A;
  const bf16_t* B = (const bf16_t*)d.B;
  const long lda = A_K ? d.a_sm : d.a_sk;
  const long ldb = B_K ? d.b_sn : d.b_sk;

  typename std::conditional<A_K, LoadK<BM>, LoadMN<BM>>::type la;
  typename std::conditional<B_K, LoadK<BN>, LoadMN<BN>>::type lb;

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Pipeline: while slice kt feeds the MFMAs from one LDS buffer, slice kt+1
  // (fetched during the previous iteration) is written to the other buffer and
  // the global loads of slice kt+2 are issued, so a load has a whole iteration
  // to land before anything waits for it.
  const int nk = (d.K + BK - 1) / BK;
  la.fetch(A, lda, m0, d.M, 0, d.K);
  lb.fetch(B, ldb, n0, d.N, 0, d.K);
  la.stash(smem);
  lb.stash(smem + SM::A_ELEMS);
  if (nk > 1) {
    la.fetch(A, lda, m0, d.M, BK, d.K);
    lb.fetch(B, ldb, n0, d.N, BK, d.K);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const bf16_t* sa = smem + (kt & 1) * SM::STAGE;
    const bf16_t* sb = sa + SM::A_ELEMS;
    if (kt + 1 < nk) {
      bf16_t* na = smem + ((kt + 1) & 1) * SM::STAGE;
      la.stash(na);
      lb.stash(na + SM::A_ELEMS);
    }
    if (kt + 2 < nk) {
      la.fetch(A, lda, m0, d.M, (kt + 2) * BK, d.K);
      lb.fetch(B, ldb, n0, d.N, (kt + 2) * BK, d.K);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[WM], fb[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        fa[i] = A_K ? frag_k(sa, wm * 32 * WM + i * 32, ks) : frag_mn<BM>(sa, wm * 32 * WM + i * 32, ks);
#pragma unroll
      for (int j = 0; j < WN; ++j)
        fb[j] = B_K ? frag_k(sb, wn * 32 * WN + j * 32, ks) : frag_mn<BN>(sb, wn * 32 * WN + j * 32, ks);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  const unsigned gelu_tab = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)smem_raw + SM::TABLE_OFF;
  if (EPI == EPI_BIAS_GELU) {     // the table region lies behind everything else: no barrier needed before writing it
    for (int c = threadIdx.x; c < kGeluBytes / 16; c += 256)
      ((f32x4*)(smem_raw + SM::TABLE_OFF))[c] = ((const f32x4*)g_gelu_table)[c];
    __syncthreads();
  }
  EpiOperands<WM, WN, EPI> ops;
  ops.issue_bias(d, n0);
  ops.issue(d, m0, n0, 0);
  write_tile<WM, WN, EPI, SM::EPI_LD>(d, acc, (float*)smem_raw, m0, n0, ops, gelu_tab);
}

// ---- software-pipelined kernel with direct global -> LDS loads (K a multiple of 64) ------
// Per-thread address tables are set up once; inside the K loop a slice costs
// one scalar pointer bump per operand.  The instruction order of the loop body
// is fixed by hand (scheduling barriers between the groups):
//   k-step s of a slice issues its MFMAs interleaved with the LDS reads of the
//   fragments of k-step s+1 (two fragment register sets), so no MFMA waits on LDS;
//   all LDS reads of a slice are complete after k-step 2, where the one
//   workgroup barrier of the slice sits; k-step 3 then runs its MFMAs
//   interleaved with the fragment reads of the next slice (other buffer) and
//   with the global -> LDS loads of the slice after that (into the buffer just
//   vacated), which therefore have a whole slice of MFMA time to land.
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(3))) const bf16x8* lds_bf16x8_ptr;
typedef __attribute__((address_space(3))) short4_t* lds_short4_ptr;

__device__ __forceinline__ void gload_lds16(unsigned voff, const void* sbase, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(sbase), "s"(lds_addr)
               : "memory", "m0");
}

// K-contiguous operand, ROWS x 64 per slice; LDS row r = 128 bytes, 16-byte chunk c at position
// c ^ ((r / 2) % 8).  The LDS has 64 four-byte banks and serves a 16-byte read for 16 lanes per
// cycle: 16 consecutive rows then cover every bank exactly once (rows 2j and 2j+1 share a position
// in the two 128-byte halves of the 256-byte bank line).
template <int ROWS>
struct PlK {
  static constexpr int NLOAD = ROWS / 32;
  static constexpr int BYTES = ROWS * BK * 2;
  // byte offsets of this thread's chunks relative to row row0, k 0 of the slice
  __device__ static __forceinline__ void load_offsets(unsigned (&off)[NLOAD], long ld, int row0, int row_lim) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int r = i * 32 + (tid >> 3), p = tid & 7;
      const int row = min(row0 + r, row_lim - 1) - row0;
      off[i] = (unsigned)((long)row * ld * 2 + ((p ^ ((r >> 1) & 7)) << 4));
    }
  }
  __device__ static __forceinline__ const char* base(const bf16_t* g, long ld, int row0) {
    return (const char*)(g + (long)row0 * ld);
  }
  __device__ static __forceinline__ long slice_bytes(long ld) { return BK * 2; }
  // fragment address table: entry ks = address (within the operand's LDS area) of block 0 for k-step ks
  __device__ static __forceinline__ void frag_table(unsigned (&t)[4], int wave_row0) {
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      t[ks] = (unsigned)((wave_row0 + (l & 31)) * (BK * 2) + (((2 * ks + (l >> 5)) ^ ((l >> 1) & 7)) << 4));
  }
  __device__ static __forceinline__ bf16x8 frag(const unsigned (&t)[4], unsigned lds_base, int blk, int ks) {
    return *(lds_bf16x8_ptr)(lds_base + t[ks] + blk * 32 * BK * 2);
  }
};
// Row-contiguous operand, 64 k-rows x ROWS per slice; the 16-byte chunk g of k-row k sits at chunk position
// place(g, k) of that row.  A transposing 8-byte read is served for 32 lanes per cycle, which address 4
// consecutive k-rows x 64 bytes: the placement moves those four 64-byte pieces to distinct quarters of the
// 256-byte bank line.  Rows of 128 or 256 bytes and more: XOR with a k-dependent chunk offset.  Rows of 384
// bytes (ROWS = 192) already alternate between the two halves of the bank line from one k-row to the
// next; rotating every second pair of k-rows by 64 bytes (modulo the row) separates the rest.
template <int ROWS>
struct PlMN {
  static constexpr int NLOAD = ROWS / 32;
  static constexpr int BYTES = ROWS * BK * 2;
  static constexpr int CPR = ROWS / 8;
  static constexpr bool ROTATE = (CPR & (CPR - 1)) != 0;
  static_assert(!ROTATE || ROWS == 192, "placement derived for rows of 384 bytes only");
  __device__ static __forceinline__ int swz(int k) {
    return ROTATE ? 4 * ((k >> 1) & 1) : (ROWS >= 128 ? 4 * (k & 3) : 4 * ((k >> 1) & 1));
  }
  // position of chunk g in k-row k, and the chunk found at position p
  __device__ static __forceinline__ int place(int g, int k) {
    if (!ROTATE) return g ^ swz(k);
    const int p = g + swz(k);
    return p >= CPR ? p - CPR : p;
  }
  __device__ static __forceinline__ int chunk_at(int p, int k) {
    if (!ROTATE) return p ^ swz(k);
    const int g = p - swz(k);
    return g < 0 ? g + CPR : g;
  }
  __device__ static __forceinline__ void load_offsets(unsigned (&off)[NLOAD], long ld, int row0, int row_lim) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int c = i * 256 + tid;
      const int kr = c / CPR, p = c % CPR;
      const int col = min(row0 + (chunk_at(p, kr) << 3), row_lim - 8) - row0;
      off[i] = (unsigned)((long)kr * ld * 2 + col * 2);
    }
  }
  __device__ static __forceinline__ const char* base(const bf16_t* g, long ld, int row0) {
    return (const char*)(g + row0);
  }
  __device__ static __forceinline__ long slice_bytes(long ld) { return BK * ld * 2; }
  // entry blk = address of k-step 0 for 32-row block blk
  __device__ static __forceinline__ void frag_table(unsigned (&t)[4], int wave_row0) {
    const int l = threadIdx.x & 63, i = l & 15;
    const int k = (l >> 5) * 8 + (i >> 2);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int col = wave_row0 + b * 32 + ((l >> 4) & 1) * 16 + (i & 3) * 4;
      t[b] = (unsigned)(k * ROWS * 2 + (place(col >> 3, k) << 4) + (col & 7) * 2);
    }
  }
  __device__ static __forceinline__ bf16x8 frag(const unsigned (&t)[4], unsigned lds_base, int blk, int ks) {
    const unsigned a = lds_base + t[blk] + ks * 16 * ROWS * 2;
    union { short4_t s4[2]; bf16x8 b; } u;
    u.s4[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(a));
    u.s4[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(a + 4 * ROWS * 2));
    return u.b;
  }
};

template <int WM, int WN, int NS, bool GELU = false>
struct SmemPl {
  static constexpr int BM = 64 * WM, BN = 64 * WN;
  static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int EPI_LD = 32 * WN + 4;
  static constexpr int EPI_BYTES = 4 * 32 * EPI_LD * 4;
  static constexpr int MAIN_BYTES = NS * STAGE_BYTES;
  static constexpr int TABLE_OFF = (MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES);   // GELU table behind the rest
  static constexpr int BYTES = TABLE_OFF + (GELU ? kGeluBytes : 0);
};

#define BAMBOO_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int WM, int WN, bool A_K, bool B_K>
struct PlLoop {
  typedef SmemPl<WM, WN, 2> SM;
  typedef typename std::conditional<A_K, PlK<SM::BM>, PlMN<SM::BM>>::type OpA;
  typedef typename std::conditional<B_K, PlK<SM::BN>, PlMN<SM::BN>>::type OpB;
  static constexpr int NLA = OpA::NLOAD, NLB = OpB::NLOAD, NL = NLA + NLB;

  unsigned offA[NLA], offB[NLB];      // per-thread global byte offsets
  unsigned tabA[4], tabB[4];          // per-thread LDS fragment addresses
  const char* gA;                     // wavefront-uniform slice pointers
  const char* gB;
  long stepA, stepB;
  unsigned lds0;                      // LDS address of stage 0
  unsigned wave_lds;                  // wave * 1024: where this wave's lanes of a 256-chunk group land

  __device__ __forceinline__ void issue_one(int n, unsigned stage) const {
    // n-th load of a slice: A chunks first, then B chunks
    if (n < NLA) gload_lds16(offA[n], gA, lds0 + stage + n * 4096 + wave_lds);
    else gload_lds16(offB[n - NLA], gB, lds0 + stage + SM::A_BYTES + (n - NLA) * 4096 + wave_lds);
  }
  __device__ __forceinline__ void issue_slice(unsigned stage) {
#pragma unroll
    for (int n = 0; n < NL; ++n) issue_one(n, stage);
    gA += stepA;
    gB += stepB;
  }
  __device__ __forceinline__ void read_one(int n, unsigned stage, int ks, bf16x8 (&fa)[WM], bf16x8 (&fb)[WN]) const {
    if (n < WM) fa[n] = OpA::frag(tabA, lds0 + stage, n, ks);
    else fb[n - WM] = OpB::frag(tabB, lds0 + stage + SM::A_BYTES, n - WM, ks);
  }
  // One k-step: MFMAs on (ca, cb); if READ, the fragments (na, nb) of k-step ks_next of the slice
  // in `rstage` are fetched meanwhile, all of them behind the first MFMAs so that they have the
  // rest of this k-step and all of the next one to return; LOADPART 1 / 2 issues the first / second
  // half of the global loads of a slice into `lstage`, spread over the MFMAs.
  template <bool READ, int LOADPART>
  __device__ __forceinline__ void kstep(f32x16 (&acc)[WM][WN], const bf16x8 (&ca)[WM], const bf16x8 (&cb)[WN],
                                        bf16x8 (&na)[WM], bf16x8 (&nb)[WN], unsigned rstage, int ks_next,
                                        unsigned lstage) {
    constexpr int NMFMA = WM * WN, NR = WM + WN;
    constexpr int RSPAN = NMFMA >= 4 ? NMFMA / 2 : 1;           // MFMAs that carry the reads
    constexpr int RPM = (NR + RSPAN - 1) / RSPAN;               // reads per MFMA
    constexpr int NLH = (NL + 1) / 2;                           // loads per half
    constexpr int LPM = (NLH + NMFMA - 1) / NMFMA;              // loads per MFMA
    constexpr int L0 = LOADPART == 2 ? NLH : 0, L1 = LOADPART == 1 ? NLH : NL;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const int n = i * WN + j;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[i], cb[j], acc[i][j], 0, 0, 0);
        if (READ) {
#pragma unroll
          for (int q = 0; q < RPM; ++q)
            if (n < RSPAN && n * RPM + q < NR) read_one(n * RPM + q, rstage, ks_next, na, nb);
        }
        if (LOADPART != 0) {
#pragma unroll
          for (int q = 0; q < LPM; ++q)
            if (L0 + n * LPM + q < L1) issue_one(L0 + n * LPM + q, lstage);
        }
        BAMBOO_SCHED_FENCE();
      }
    if (LOADPART == 2) {
      gA += stepA;
      gB += stepB;
    }
  }
};

// vmcnt(n) lgkmcnt(0): at most n of this wave's global loads still in flight, every LDS read returned
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at its maximum, lgkmcnt 11:8)
template <int N>
__device__ __forceinline__ void wait_loads_and_lds() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// Slices are kept in NS LDS buffers used round-robin; the global -> LDS loads of slice kt + NS - 1 ... are
// in flight while slice kt feeds the MFMAs, i.e. a load has NS - 1 slices of MFMA time to land.
// pid: position of this workgroup's tile in the tile sequence of problem d (the caller has applied xcd_range)
template <int WM, int WN, bool A_K, bool B_K, int EPI, int NS>
__device__ __forceinline__ void gemm_pl_body(const GemmDesc& d, int pid) {
  typedef SmemPl<WM, WN, NS, EPI == EPI_BIAS_GELU> SM;
  typedef PlLoop<WM, WN, A_K, B_K> Loop;
  constexpr int BM = SM::BM, BN = SM::BN, NL = Loop::NL;
  constexpr unsigned STAGE = SM::STAGE_BYTES, RING = NS * STAGE;
  static_assert((NS - 1) * NL + (WM * WN <= 8 ? EpiOperands<WM, WN, EPI>::NLOADS : 0) < 64,
                "too many loads in flight for the vmcnt counter");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  tile_walk(pid, (d.M + BM - 1) / BM, (d.N + BN - 1) / BN, &tile_m, &tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const long lda = A_K ? d.a_sm : d.a_sk;
  const long ldb = B_K ? d.b_sn : d.b_sk;

  Loop L;
  Loop::OpA::load_offsets(L.offA, lda, m0, d.M);
  Loop::OpB::load_offsets(L.offB, ldb, n0, d.N);
  Loop::OpA::frag_table(L.tabA, wm * 32 * WM);
  Loop::OpB::frag_table(L.tabB, wn * 32 * WN);
  L.gA = Loop::OpA::base((const bf16_t*)d.A, lda, m0);
  L.gB = Loop::OpB::base((const bf16_t*)d.B, ldb, n0);
  L.stepA = Loop::OpA::slice_bytes(lda);
  L.stepB = Loop::OpB::slice_bytes(ldb);
  L.lds0 = (unsigned)(uintptr_t)(lds_void_ptr)smem_raw;
  L.wave_lds = wave * 1024;

  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = d.K / BK;                 // nk >= NS (checked by the launcher)
  if (EPI == EPI_BIAS_GELU) {
    // GELU table -> its own LDS region, by the same direct loads as the slices and ahead of them: the
    // wait for slice 0 below covers these older loads too.  A wavefront copies 1 KB per load.
#pragma unroll
    for (int it = 0; it < (kGeluBytes / 16 + 255) / 256; ++it) {
      const int c0 = it * 256 + wave * 64;            // first chunk of this wavefront, uniform
      if (c0 < kGeluBytes / 16)
        gload_lds16((unsigned)(((threadIdx.x & 63)) << 4), (const char*)g_gelu_table + (long)c0 * 16,
                    L.lds0 + SM::TABLE_OFF + c0 * 16);
    }
  }
  // The bias is requested before any slice load: the waits below count the loads that are YOUNGER than
  // the slice they wait for, so however many bias loads the compiler keeps (the columns of a lane often
  // repeat) and wherever it puts them before this point, they can never stand in for a slice load there.
  EpiOperands<WM, WN, EPI> ops;
  ops.issue_bias(d, n0);
  BAMBOO_SCHED_FENCE();
  // four fragment register sets: k-step s of a slice computes from set s while set (s + 2) % 4 is
  // filled for the k-step after the next one, so an LDS read has more than a whole k-step to return
  bf16x8 fa[4][WM], fb[4][WN];
#pragma unroll
  for (int j = 0; j < NS; ++j) L.issue_slice(j * STAGE);
  wait_loads_and_lds<(NS - 1) * NL>();     // slice 0 has landed
  __syncthreads();
#pragma unroll
  for (int n = 0; n < WM + WN; ++n) L.read_one(n, 0, 0, fa[0], fb[0]);
#pragma unroll
  for (int n = 0; n < WM + WN; ++n) L.read_one(n, 0, 1, fa[1], fb[1]);

  // Steady state: slice kt computes from buffer cur.  During its first two k-steps the fragments of
  // its last two are read, so after them every LDS read of cur has been issued; once they have
  // returned and slice kt+1 has landed for every wave, the barrier frees cur for the loads of slice
  // kt+NS (issued between the MFMAs of the last two k-steps) and opens buffer nxt for reading.
  unsigned cur = 0;
  for (int kt = 0; kt < nk - NS; ++kt) {
    const unsigned nxt = cur + STAGE == RING ? 0 : cur + STAGE;
    L.template kstep<true, 0>(acc, fa[0], fb[0], fa[2], fb[2], cur, 2, 0);
    L.template kstep<true, 0>(acc, fa[1], fb[1], fa[3], fb[3], cur, 3, 0);
    wait_loads_and_lds<(NS - 2) * NL>();
    __syncthreads();
    BAMBOO_SCHED_FENCE();
    L.template kstep<true, 1>(acc, fa[2], fb[2], fa[0], fb[0], nxt, 0, cur);
    L.template kstep<true, 2>(acc, fa[3], fb[3], fa[1], fb[1], nxt, 1, cur);
    cur = nxt;
  }
  // The last NS slices issue no slice loads; instead the epilogue's operands for the first row block
  // are requested now, so that they arrive under the remaining MFMAs.  They are younger than every
  // slice load, hence simply add to the number of loads that may still be in flight at the waits below.
  // (256 x 256 tiles have no registers to spare for them until the fragments are dead.)
  constexpr bool EARLY = WM * WN <= 8;
  if (EARLY) ops.issue(d, m0, n0, 0);
  constexpr int NEPI = EARLY ? EpiOperands<WM, WN, EPI>::NLOADS : 0;
  // the waits below assume these NEPI loads are in flight from here on: keep the compiler from moving them
  asm volatile("" ::: "memory");
  BAMBOO_SCHED_FENCE();
  // slice nk-1-J still has J slices after it, J-1 of which may be in flight
  auto tail = [&](auto jc) __attribute__((always_inline)) {
    constexpr int J = decltype(jc)::value;
    const unsigned nxt = cur + STAGE == RING ? 0 : cur + STAGE;
    L.template kstep<true, 0>(acc, fa[0], fb[0], fa[2], fb[2], cur, 2, 0);
    L.template kstep<true, 0>(acc, fa[1], fb[1], fa[3], fb[3], cur, 3, 0);
    if (J > 0) {
      wait_loads_and_lds<(J > 1 ? J - 1 : 0) * NL + NEPI>();
      __syncthreads();
      BAMBOO_SCHED_FENCE();
    }
    L.template kstep<(J > 0), 0>(acc, fa[2], fb[2], fa[0], fb[0], nxt, 0, 0);
    L.template kstep<(J > 0), 0>(acc, fa[3], fb[3], fa[1], fb[1], nxt, 1, 0);
    cur = nxt;
  };
  if constexpr (NS >= 4) tail(std::integral_constant<int, 3>());
  if constexpr (NS >= 3) tail(std::integral_constant<int, 2>());
  tail(std::integral_constant<int, 1>());
  tail(std::integral_constant<int, 0>());
  // every wave is done with the slice buffers before the staging area reuses them
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __syncthreads();
  BAMBOO_SCHED_FENCE();
  if (!EARLY) ops.issue(d, m0, n0, 0);
  write_tile<WM, WN, EPI, SM::EPI_LD>(d, acc, (float*)smem_raw, m0, n0, ops, L.lds0 + SM::TABLE_OFF);
}

template <int WM, int WN, bool A_K, bool B_K, int EPI, int NS, int MINB>
__global__ __launch_bounds__(256, MINB) void gemm_mfma_pl_kernel(GemmDesc d) {
  constexpr int BM = 64 * WM, BN = 64 * WN;
  gemm_pl_body<WM, WN, A_K, B_K, EPI, NS>(d, xcd_range(blockIdx.x, ((d.M + BM - 1) / BM) * ((d.N + BN - 1) / BN)));
}

// Several weight-gradient problems in one launch: workgroup b works on problem p where
// first[p] <= b < first[p+1].  The problems of a layer's backward are independent of each other and
// most of them do not fill a whole number of rounds of the 256 CUs on their own (1024 x 1024 outputs
// are 64 tiles of 128 x 128); launched together their tiles pack, and a CU goes from one problem's
// tile to the next one's without the chip draining in between.
template <int WM, int WN, int NS, int MINB>
__global__ __launch_bounds__(256, MINB) void gemm_mfma_pl_group_kernel(GemmGroup g) {
  const int total = g.first[GemmGroup::MAX];
  if ((int)blockIdx.x >= total) {                  // behind the GEMM tiles: the reductions riding along
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    colreduce_batch_block(g.tail, (int)blockIdx.x - total, (float*)smem_raw);
    return;
  }
  // g.whole_launch_ranges: every XCD takes one contiguous range of the CONCATENATED tile sequences, so that
  // a problem's operands go to the L2s of the two or three XCDs its range spans instead of to all eight
  // (launches of one round); otherwise each problem is spread over all XCDs, a range per XCD inside it.
  const int b = g.whole_launch_ranges ? xcd_range(blockIdx.x, total) : (int)blockIdx.x;
  int p = 0;
#pragma unroll
  for (int q = 1; q < GemmGroup::MAX; ++q)
    if (q < g.n && b >= g.first[q]) p = q;
  int local = b - g.first[p];
  if (!g.whole_launch_ranges) {
    int end = total;
#pragma unroll
    for (int q = GemmGroup::MAX - 1; q >= 1; --q)
      if (q > p && q < g.n) end = g.first[q];
    local = xcd_range(local, end - g.first[p]);
  }
  gemm_pl_body<WM, WN, false, false, EPI_ACC_F32, NS>(g.d[p], local);
}

template <int WM, int WN, bool A_K, bool B_K, int EPI, int NS>
static hipError_t launch_pl(hipStream_t s, const GemmDesc& d, int tiles) {
  typedef SmemPl<WM, WN, NS, EPI == EPI_BIAS_GELU> SM;
  constexpr auto kern = gemm_mfma_pl_kernel<WM, WN, A_K, B_K, EPI, NS, (2 * SM::BYTES <= 160 * 1024 ? 2 : 1)>;
  const hipError_t e = ensure_lds_attribute<kern, SM::BYTES>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), SM::BYTES, s, d);
  return hipGetLastError();
}

static std::atomic<int> g_forced_stages{0};      // test / tuning knob, process-wide
int set_gemm_stages(int n) { return g_forced_stages.exchange(n); }

template <int WM, int WN, bool A_K, bool B_K, int EPI>
static hipError_t launch_cfg(hipStream_t s, const GemmDesc& d, int ns) {
  const int tiles = ((d.M + 64 * WM - 1) / (64 * WM)) * ((d.N + 64 * WN - 1) / (64 * WN));
  static const bool no_direct = getenv("BAMBOO_GEMM_NO_DIRECT") != nullptr;   // tuning knob
  if (d.K % BK == 0 && d.K >= 2 * BK && !no_direct) {
    const int nk = d.K / BK;
    if (g_forced_stages) ns = g_forced_stages;
    if (ns > nk) ns = nk >= 3 ? 3 : 2;
    constexpr bool G = EPI == EPI_BIAS_GELU;
    if constexpr (SmemPl<WM, WN, 4, G>::BYTES <= 160 * 1024) {
      if (ns == 4) return launch_pl<WM, WN, A_K, B_K, EPI, 4>(s, d, tiles);
    }
    if constexpr (SmemPl<WM, WN, 3, G>::BYTES <= 160 * 1024) {
      if (ns >= 3) return launch_pl<WM, WN, A_K, B_K, EPI, 3>(s, d, tiles);
    }
    return launch_pl<WM, WN, A_K, B_K, EPI, 2>(s, d, tiles);
  }
  typedef Smem<WM, WN, A_K, B_K, EPI == EPI_BIAS_GELU> SM;
  constexpr auto kern = gemm_mfma_kernel<WM, WN, A_K, B_K, EPI>;
  const hipError_t e = ensure_lds_attribute<kern, SM::BYTES>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), SM::BYTES, s, d);
  return hipGetLastError();
}

static std::atomic<int> g_forced_tile{0};        // test / tuning knob, process-wide
bool gemm_tile_code_valid(int code) {
  return code == 0 || code == 44 || code == 43 || code == 42 || code == 24 || code == 22 || code == 11;
}
int set_gemm_tile(int code) { return g_forced_tile.exchange(code); }

// Tile and pipeline-depth choice.  Each candidate's run time is estimated as
//   rounds * (a + b * slices) + c   [microseconds]
// where rounds = ceil(tiles / (256 CUs * workgroups that fit a CU)) and slices = K / 64; a is the
// per-tile fill and epilogue cost, b the time of one 64-deep slice, c a launch constant.  The
// coefficients are least-squares fits to timings of the BERT-large- and GPT-2-shaped stage GEMMs
// on an MI355X with operands that are not cache-resident (as inside a training iteration): big
// tiles have the best MFMA : LDS ratio but need enough of them to fill the chip; two buffers leave
// room for two workgroups per CU, which hide each other's stalls; when a CU gets one workgroup
// anyway, a deeper ring hides the load latency instead.
struct TileCost { int code, ns; float a, b, c; };
static const TileCost kCostStore[] = {     // bf16 output (forward and input-gradient forms)
    {11, 2, 1.96f, 0.377f, 3.94f}, {11, 4, 1.48f, 0.396f, 5.05f}, {22, 2, 5.04f, 0.949f, 0.35f},
    {22, 3, 4.52f, 0.545f, 1.60f}, {24, 2, 4.93f, 1.068f, 5.59f}, {24, 3, 7.76f, 0.816f, 1.45f},
    {42, 2, 1.85f, 1.107f, 8.18f}, {42, 3, 5.44f, 0.874f, 2.50f}, {44, 2, 14.98f, 1.281f, 0.58f},
    // 256 x 192 (offered for the bias-only forward form: N = 3 H of the QKV projection is 16 x 192 when
    // H = 1024, i.e. with 4096 tokens exactly 256 tiles); coefficients scaled from the 256 x 256 tile's
    {43, 2, 11.6f, 0.98f, 0.58f}};
static const TileCost kCostAcc[] = {       // fp32 read-modify-write output (weight-gradient form)
    {11, 2, 0.f, 0.487f, 1.98f}, {11, 4, 0.f, 0.504f, 0.f}, {22, 2, 0.f, 0.983f, 0.f},
    {22, 3, 0.f, 0.616f, 2.88f}, {24, 2, 0.f, 1.216f, 6.12f}, {24, 3, 0.f, 1.072f, 1.03f},
    {42, 2, 0.f, 1.102f, 11.56f}, {42, 3, 0.f, 0.997f, 4.55f}, {44, 2, 0.f, 1.737f, 0.f}};

static void choose_tile(const GemmDesc& d, bool acc_form, long extra_lds, int* code, int* ns, bool offer_43 = false) {
  const bool by_work = d.shared_chip != 0;
  const int nk = d.K / BK;
  const TileCost* tab = acc_form ? kCostAcc : kCostStore;
  const int ntab = acc_form ? (int)(sizeof(kCostAcc) / sizeof(kCostAcc[0])) : (int)(sizeof(kCostStore) / sizeof(kCostStore[0]));
  float best = 0.f;
  bool found = false;
  *code = 22;
  *ns = 2;
  for (int i = 0; i < ntab; ++i) {
    const TileCost& t = tab[i];
    if (t.ns > nk && t.ns > 2) continue;
    if (t.code == 43 && !offer_43) continue;
    const int wm = t.code / 10, wn = t.code % 10;
    const long tiles = (long)((d.M + 64 * wm - 1) / (64 * wm)) * ((d.N + 64 * wn - 1) / (64 * wn));
    const long stage = (long)(wm + wn) * 64 * BK * 2, epi = 4L * 32 * (32 * wn + 4) * 4;
    const long lds = (t.ns * stage > epi ? t.ns * stage : epi) + extra_lds;
    if (lds > 160 * 1024) continue;
    const long slots = 256 * (2 * lds <= 160 * 1024 ? 2 : 1);
    const long rounds = (tiles + slots - 1) / slots;
    // alone on the chip: rounds of tiles.  Beside another stream's kernels: CU time summed over the tiles, but
    // no shape that leaves fewer than 128 tiles where another offers more -- the launch still has to finish
    // (measured: with 64-tile launches on the second lane that lane becomes the critical path).
    const float cost = by_work ? (float)(tiles < 128 ? 4 * 256 : tiles) * (t.a + t.b * nk) : rounds * (t.a + t.b * nk) + t.c;
    if (!found || cost < best) {
      found = true;
      best = cost;
      *code = t.code;
      *ns = t.ns;
    }
  }
}

template <bool A_K, bool B_K, int EPI>
static hipError_t launch_form(hipStream_t s, const GemmDesc& d) {
  int pick, ns;
  // the 256 x 192 tile exists in the pipelined kernel only (K a multiple of the slice depth)
  constexpr bool HAS_43 = A_K && !B_K && EPI == EPI_BIAS;
  choose_tile(d, EPI == EPI_ACC_F32, EPI == EPI_BIAS_GELU ? kGeluBytes : 0, &pick, &ns,
              HAS_43 && d.K % BK == 0 && d.K >= 2 * BK && !g_forced_stages);
  if (EPI == EPI_BIAS_GELU) {
    const hipError_t e = ensure_gelu_table(s);
    if (e != hipSuccess) return e;
  }
  if (g_forced_tile) {
    pick = g_forced_tile;
    ns = 2;
    // 256 x 192 where this form and shape have it, the next larger tile otherwise
    if (pick == 43 && !(HAS_43 && d.K % BK == 0 && d.K >= 2 * BK)) pick = 44;
  }
  if (EPI == EPI_MUL && d.tile_colsum != nullptr && d.tile_colsum_parts != nullptr)
    *d.tile_colsum_parts = (d.M + 64 * (pick / 10) - 1) / (64 * (pick / 10));   // one row of column sums per tile row
  if constexpr (HAS_43) {
    if (pick == 43) {
      if (d.K % BK != 0 || d.K < 2 * BK) return hipErrorNotSupported;
      const int tiles = ((d.M + 255) / 256) * ((d.N + 191) / 192);
      return launch_pl<4, 3, A_K, B_K, EPI, 2>(s, d, tiles);
    }
  }
  switch (pick) {
    case 44: return launch_cfg<4, 4, A_K, B_K, EPI>(s, d, ns);
    case 42: return launch_cfg<4, 2, A_K, B_K, EPI>(s, d, ns);
    case 24: return launch_cfg<2, 4, A_K, B_K, EPI>(s, d, ns);
    case 22: return launch_cfg<2, 2, A_K, B_K, EPI>(s, d, ns);
    case 11: return launch_cfg<1, 1, A_K, B_K, EPI>(s, d, ns);
    default: return hipErrorInvalidValue;
  }
}

template <int WM, int WN, int NS>
static hipError_t launch_group_cfg(hipStream_t s, GemmGroup& g) {
  typedef SmemPl<WM, WN, NS, false> SM;
  constexpr auto kern = gemm_mfma_pl_group_kernel<WM, WN, NS, (2 * SM::BYTES <= 160 * 1024 ? 2 : 1)>;
  const hipError_t e = ensure_lds_attribute<kern, SM::BYTES>();
  if (e != hipSuccess) return e;
  int total = 0;
  for (int i = 0; i < g.n; ++i) {
    g.first[i] = total;
    total += ((g.d[i].M + 64 * WM - 1) / (64 * WM)) * ((g.d[i].N + 64 * WN - 1) / (64 * WN));
  }
  for (int i = g.n; i <= GemmGroup::MAX; ++i) g.first[i] = total;
  // One round of tiles: XCD ranges over the whole launch halve what the L2s fetch (measured at the
  // BERT-large-shaped stage: 231 instead of 440 MiB per launch, 1.3 x the operands) at the same run time.
  // Over several rounds the per-problem ranges are faster (GPT-2-shaped stage: 288 against 302 us), so
  // they stay there.
  g.whole_launch_ranges = total <= 256 * (2 * SM::BYTES <= 160 * 1024 ? 2 : 1) ? 1 : 0;
  static_assert(SM::BYTES >= kReduceLdsFloats * 4, "the tail workgroups use the front of the tile ring");
  total += grad_reduce_blocks(g.tail);
  hipLaunchKernelGGL(kern, dim3(total), dim3(256), SM::BYTES, s, g);
  return hipGetLastError();
}

static bool wgrad_form_ok(const GemmDesc& d) {
  if (d.epi != EPI_ACC_F32 || d.a_sk == 1 || d.b_sk == 1 || d.a_sm != 1 || d.b_sn != 1) return false;
  if (d.M % 8 || d.N % 8 || d.K % BK || d.a_sk % 8 || d.b_sk % 8) return false;
  if (((uintptr_t)d.A | (uintptr_t)d.B | (uintptr_t)d.C) & 15) return false;
  return d.M > 0 && d.N > 0;
}

// n <= GemmGroup::MAX weight-gradient GEMMs (dW += X^T dY) as one launch where the pipelined MFMA kernel
// covers all of them with one tile shape; hipErrorNotSupported otherwise (the caller launches them singly).
hipError_t launch_gemm_group_mfma(hipStream_t s, const GemmDesc* d, int n, const GradReduceBatch* tail) {
  if (n < 1 || n > GemmGroup::MAX) return hipErrorNotSupported;
  GemmGroup g;
  memset(&g, 0, sizeof(g));
  g.n = n;
  if (tail != nullptr) g.tail = *tail;
  int nk_min = 1 << 30;
  for (int i = 0; i < n; ++i) {
    if (!wgrad_form_ok(d[i])) return hipErrorNotSupported;
    g.d[i] = d[i];
    nk_min = d[i].K / BK < nk_min ? d[i].K / BK : nk_min;
  }
  if (nk_min < 3) return hipErrorNotSupported;
  // Tile shape for the whole group: 128 x 128, 128 x 256 or 256 x 128 with a ring of three, or 256 x 256
  // with a ring of two -- the cheapest by the cost model of the single launches, with all tiles of the
  // group sharing the rounds.
  const int codes[4] = {22, 44, 24, 42}, nss[4] = {3, 2, 3, 3};
  int pick = 0;
  float best = 0.f;
  for (int c = 0; c < 4; ++c) {
    const TileCost* t = nullptr;
    for (const TileCost& e : kCostAcc)
      if (e.code == codes[c] && e.ns == nss[c]) t = &e;
    if (!t) continue;
    const int wm = codes[c] / 10, wn = codes[c] % 10;
    long tiles = 0;
    double slices = 0;
    for (int i = 0; i < n; ++i) {
      const long ti = (long)((d[i].M + 64 * wm - 1) / (64 * wm)) * ((d[i].N + 64 * wn - 1) / (64 * wn));
      tiles += ti;
      slices += (double)ti * (d[i].K / BK);
    }
    const long rounds = (tiles + 255) / 256;
    const float cost = rounds * (t->a + t->b * (float)(slices / tiles)) + t->c;
    if (pick == 0 || cost < best) {
      pick = codes[c];
      best = cost;
    }
  }
  if (g_forced_tile == 22 || g_forced_tile == 44 || g_forced_tile == 24 || g_forced_tile == 42) pick = g_forced_tile;
  else if (g_forced_tile || g_forced_stages) return hipErrorNotSupported;   // a forced shape this launch does not offer
  switch (pick) {
    case 44: return launch_group_cfg<4, 4, 2>(s, g);
    case 24: return launch_group_cfg<2, 4, 3>(s, g);
    case 42: return launch_group_cfg<4, 2, 3>(s, g);
    default: return launch_group_cfg<2, 2, 3>(s, g);
  }
}

hipError_t launch_gemm_mfma(hipStream_t s, const GemmDesc& d) {
  const bool a_k = d.a_sk == 1, b_k = d.b_sk == 1;
  if (!a_k && d.a_sm != 1) return hipErrorNotSupported;
  if (!b_k && d.b_sn != 1) return hipErrorNotSupported;
  // 16-byte accesses everywhere: dimensions and leading dimensions in multiples of 8
  const long lda = a_k ? d.a_sm : d.a_sk, ldb = b_k ? d.b_sn : d.b_sk;
  if (d.M % 8 || d.N % 8 || d.K % 8 || lda % 8 || ldb % 8) return hipErrorNotSupported;
  auto misaligned = [](const void* p) { return p != nullptr && ((uintptr_t)p & 15) != 0; };
  if (misaligned(d.A) || misaligned(d.B) || misaligned(d.C) || misaligned(d.bias) || misaligned(d.res) ||
      misaligned(d.aux_in) || misaligned(d.aux_out))
    return hipErrorNotSupported;
  if (a_k && !b_k) {           // forward
    switch (d.epi) {
      case EPI_STORE: return launch_form<true, false, EPI_STORE>(s, d);   // the LM head has no bias
      case EPI_BIAS: return launch_form<true, false, EPI_BIAS>(s, d);
      case EPI_BIAS_RES: return launch_form<true, false, EPI_BIAS_RES>(s, d);
      case EPI_BIAS_GELU: return launch_form<true, false, EPI_BIAS_GELU>(s, d);
      default: return hipErrorNotSupported;
    }
  }
  if (a_k && b_k) {            // input gradient
    switch (d.epi) {
      case EPI_STORE: return launch_form<true, true, EPI_STORE>(s, d);
      case EPI_RES: return launch_form<true, true, EPI_RES>(s, d);
      case EPI_MUL: return launch_form<true, true, EPI_MUL>(s, d);
      default: return hipErrorNotSupported;
    }
  }
  if (!a_k && !b_k && d.epi == EPI_ACC_F32) return launch_form<false, false, EPI_ACC_F32>(s, d);
  return hipErrorNotSupported;
}

}  // namespace bamboo
