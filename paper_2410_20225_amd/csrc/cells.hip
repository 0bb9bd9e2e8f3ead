// Node bodies of the vector operators, fired over all tags of a dependency level at once:
// leaf rows (EMBED), the tree cells as gathered-operand MFMA GEMMs with fused epilogues,
// the classification head, and their gradient operators (Section 4: op^grad takes the
// forward inputs and the output gradient).  Parameter gradients are sums over all tags,
// formed without floating-point atomics: one split GEMM over the tag dimension with an
// ordered reduction of the partial tiles, and a segmented sum over leaves sorted by token.
#include <stdlib.h>

#include <algorithm>
#include <type_traits>

#include "bucket.h"
#include "die_sync.h"
#include "engine.h"

namespace tdf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;   // one 16-byte chunk
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

// ---- element traits --------------------------------------------------------------------
template <typename T> struct El;
template <> struct El<__bf16> {
  static constexpr int BK = 64;      // k extent of one LDS tile
  static constexpr int PAD = 8;      // row padding in elements
  static constexpr int MK = 16;      // k extent of one MFMA
  static constexpr int CH = 8;       // elements per 16-byte chunk
  typedef bf16x8 Frag;
  static __device__ __forceinline__ Frag frag(const __bf16* row, int ks, int lane) {
    return *reinterpret_cast<const Frag*>(row + ks * MK + (lane >> 5) * 8);
  }
  static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct El<float> {
  static constexpr int BK = 32;
  static constexpr int PAD = 4;
  static constexpr int MK = 2;
  static constexpr int CH = 4;
  typedef float Frag;
  static __device__ __forceinline__ Frag frag(const float* row, int ks, int lane) {
    return row[ks * MK + (lane >> 5)];
  }
  static __device__ __forceinline__ f32x16 mma(Frag a, Frag b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
};

// Kernels are instantiated on the tdf_dtype value (readable names in profiles), not on the type.
template <int DT> struct TypeOf;
template <> struct TypeOf<TDF_F32> { typedef float type; };
template <> struct TypeOf<TDF_BF16> { typedef __bf16 type; };
template <typename T> struct DtOf;
template <> struct DtOf<float> { static constexpr int value = TDF_F32; };
template <> struct DtOf<__bf16> { static constexpr int value = TDF_BF16; };

__device__ __forceinline__ float to_f(float x) { return x; }
__device__ __forceinline__ float to_f(__bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f(float x) { return (T)x; }

// Activations.  The fp32 path uses the accurate library functions; the bf16 path, whose
// results are rounded to 8 bits of mantissa anyway, uses the hardware exponential.
// sigmoid_b / tanh_b take the accumulator and a bias prepared by pre_sigmoid / pre_tanh: the bf16
// path folds the bias and the exponent's scale into one multiply-add.
template <typename T> struct Act {
  static __device__ __forceinline__ float sigmoid(float x) { return 1.0f / (1.0f + expf(-x)); }
  static __device__ __forceinline__ float tanh(float x) { return tanhf(x); }
  static __device__ __forceinline__ float pre_sigmoid(float b) { return b; }
  static __device__ __forceinline__ float pre_tanh(float b) { return b; }
  static __device__ __forceinline__ float sigmoid_b(float acc, float pb) { return sigmoid(acc + pb); }
  static __device__ __forceinline__ float tanh_b(float acc, float pb) { return tanh(acc + pb); }
};
template <> struct Act<__bf16> {
  static constexpr float LOG2E = 1.4426950408889634f;
  static __device__ __forceinline__ float sigmoid(float x) {
    return __builtin_amdgcn_rcpf(1.0f + __expf(-x));
  }
  static __device__ __forceinline__ float tanh(float x) {
    const float xc = fminf(fmaxf(x, -15.f), 15.f);
    const float e = __expf(2.0f * xc);
    return (e - 1.0f) * __builtin_amdgcn_rcpf(e + 1.0f);
  }
  static __device__ __forceinline__ float pre_sigmoid(float b) { return -LOG2E * b; }
  static __device__ __forceinline__ float pre_tanh(float b) { return 2.0f * LOG2E * b; }
  // 1 / (1 + 2^(-log2e (acc + b)))
  static __device__ __forceinline__ float sigmoid_b(float acc, float pb) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(fmaf(acc, -LOG2E, pb)));
  }
  // 1 - 2 / (1 + 2^(2 log2e (acc + b))): the exponential's overflow and underflow give exactly 1 and -1
  static __device__ __forceinline__ float tanh_b(float acc, float pb) {
    return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(fmaf(acc, 2.0f * LOG2E, pb))), 1.0f);
  }
};

// ---- GEMM  C[M x N] = A[M x K] * B[N x K]^T, both operands k-contiguous ----------------------
enum GemmMode { RNN_FWD = 0, LSTM_FWD = 1, DX_BWD = 2, DW_SPLIT = 3 };

struct GemmArgs {
  int M, N, K;               // N, K multiples of 32
  const void* A;             // dense A (DX_BWD: Dz + q0 rows; DW_SPLIT: DzT)
  size_t lda;
  const void* B;
  size_t ldb;
  const void* Bf;            // B in operand order (frag_offset), for the small-level kernel
  // gathered A rows for the forward cells: row m = [Hs[l[m]]; Hs[r[m]]]
  const void* Hs;
  int Hp;
  uint32_t out0;             // state row of the level's first cell: cell m of the level writes row out0 + m
  const uint32_t *l, *r;     // children's rows, already offset to the level's first cell
  const float* bias;
  void* Hs_out;              // state rows written by the forward cells
  float* Cs;                 // LSTM cell state rows
  uint32_t leaf_rows;        // rows below this one are leaves: their cell state is zero and is not stored
  void* gates;               // LSTM activations, row m of this level
  size_t ldg;
  float* C;                  // fp32 output (DX_BWD: dH; DW_SPLIT: partial tiles)
  size_t ldc;
  int k_per_split;           // DW_SPLIT: k range of one split
  int n_splits;
  int n_tiles_n;             // column tiles of the launch
  int save_gates;
  int narrow;                // LSTM_FWD: state rows and this level's gate rows end below 4 GiB
};

constexpr int BM_FULL = 128;   // rows of a workgroup tile; half of it for levels that would not fill the GPU

// Workgroup tile BM x BN, NW waves as (NW/WNS) x WNS, each wave BM*WNS/NW rows x WN column blocks
// of 32.  One LDS stage of BK columns; the next stage travels global -> registers while the current
// one is multiplied.  With eight waves a wave's accumulators fit half the register file, two
// waves share a SIMD, and one multiplies while the other waits for LDS or memory.  LSTM_FWD
// gives every wave the five gate blocks of the same 32 hidden units, so the gate epilogue needs
// no exchange between lanes; its workgroups are one such block wide (WNS = 1).
template <int DT, int MODE, int NW, int BM, int WNS, bool NARROW = false>
__global__ void __launch_bounds__(NW * 64, WNS == 1 ? 3 : 1) k_gemm(GemmArgs g) {
  constexpr int GEMM_THREADS = NW * 64;
  constexpr int MB = BM * WNS / (32 * NW);       // 32-row blocks per wave (waves as NW/WNS x WNS)
  typedef typename TypeOf<DT>::type T;
  typedef El<T> E;
  constexpr int WN = MODE == LSTM_FWD ? 5 : 2;   // 32-wide column blocks per wave
  constexpr int BN = WNS * WN * 32;              // columns per workgroup
  constexpr int LDT = E::BK + E::PAD;            // LDS row stride
  constexpr int CPR = E::BK / E::CH;             // 16-byte chunks per tile row
  constexpr int A_CHUNKS = BM * CPR / GEMM_THREADS;
  constexpr int B_CHUNKS = BN * CPR / GEMM_THREADS;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  T* sA = reinterpret_cast<T*>(smem);            // [BM][LDT]
  T* sB = sA + BM * LDT;                         // [BN][LDT]

  // tile coordinates: the column tiles of one row tile run back to back on one XCD
  // (workgroups are dealt round-robin to the 8 XCDs), so the gathered rows are shared in its L2
  const int n_mt = (g.M + BM - 1) / BM;
  const int xcd = blockIdx.x & 7, u = blockIdx.x >> 3;
  int nt, mt, split = 0;
  if (MODE == DW_SPLIT) {
    // all tiles of one split of the reduction run on one XCD, side by side: they walk the same
    // slices of both operands in step, so each slice comes from HBM once
    const int tiles = n_mt * g.n_tiles_n;
    split = (u / tiles) * 8 + xcd;
    if (split >= g.n_splits) return;
    mt = (u % tiles) / g.n_tiles_n;
    nt = (u % tiles) % g.n_tiles_n;
  } else {
    nt = u % g.n_tiles_n;
    mt = (u / g.n_tiles_n) * 8 + xcd;
    if (mt >= n_mt) return;
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WNS, wn = wave % WNS;
  const int wrow = wm * MB * 32;                 // the wave's first row in the tile
  const int m0 = mt * BM;
  int k_begin = 0, k_end = g.K;
  if (MODE == DW_SPLIT) {
    k_begin = split * g.k_per_split;
    k_end = min(g.K, k_begin + g.k_per_split);
  }

  // element offsets of the 16-byte chunks this thread copies in every k-tile
  uint32_t a_off[A_CHUNKS], a_off2[A_CHUNKS], b_off[B_CHUNKS];
#pragma unroll
  for (int c = 0; c < A_CHUNKS; ++c) {
    const int id = tid + c * GEMM_THREADS, row = id / CPR, ch = id % CPR;
    const int m = min(m0 + row, g.M - 1);
    if (MODE == RNN_FWD || MODE == LSTM_FWD) {
      a_off[c] = g.l[m] * (uint32_t)g.Hp + ch * E::CH;
      a_off2[c] = g.r[m] * (uint32_t)g.Hp + ch * E::CH;
    } else {
      a_off[c] = a_off2[c] = (uint32_t)m * (uint32_t)g.lda + ch * E::CH;
    }
  }
#pragma unroll
  for (int c = 0; c < B_CHUNKS; ++c) {
    const int id = tid + c * GEMM_THREADS, row = id / CPR, ch = id % CPR;
    int brow;
    if (MODE == LSTM_FWD) {
      const int w = row / 160, gate = (row % 160) / 32, jj = row % 32;
      brow = gate * g.Hp + min(nt * WNS + w, g.Hp / 32 - 1) * 32 + jj;
    } else {
      brow = min(nt * BN + row, g.N - 1);
    }
    b_off[c] = (uint32_t)brow * (uint32_t)g.ldb + ch * E::CH;
  }
  const T* Abase = reinterpret_cast<const T*>((MODE == RNN_FWD || MODE == LSTM_FWD) ? g.Hs : g.A);
  const T* Bbase = reinterpret_cast<const T*>(g.B);

  // staging registers of the next k-tile (global -> registers -> LDS)
  u32x4 ra[A_CHUNKS], rb[B_CHUNKS];
#define TDF_LOAD_TILE(K0)                                                                        \
  _Pragma("unroll") for (int c = 0; c < A_CHUNKS; ++c) {                                         \
    uint32_t off;                                                                                \
    if (MODE == RNN_FWD || MODE == LSTM_FWD)                                                     \
      off = (K0) < g.Hp ? a_off[c] + (K0) : a_off2[c] + ((K0) - g.Hp);                           \
    else                                                                                         \
      off = a_off[c] + (K0);                                                                     \
    ra[c] = *reinterpret_cast<const u32x4*>(Abase + off);                                        \
  }                                                                                              \
  _Pragma("unroll") for (int c = 0; c < B_CHUNKS; ++c)                                           \
    rb[c] = *reinterpret_cast<const u32x4*>(Bbase + b_off[c] + (K0));

  f32x16 acc[MB][WN];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const T* tA = sA + (wrow + (lane & 31)) * LDT;
  const T* tB = sB + (wn * WN * 32 + (lane & 31)) * LDT;
  if (k_begin < k_end) {
    TDF_LOAD_TILE(k_begin)
  }
  for (int k0 = k_begin; k0 < k_end; k0 += E::BK) {
#pragma unroll
    for (int c = 0; c < A_CHUNKS; ++c) {
      const int id = tid + c * GEMM_THREADS;
      *reinterpret_cast<u32x4*>(sA + (id / CPR) * LDT + (id % CPR) * E::CH) = ra[c];
    }
#pragma unroll
    for (int c = 0; c < B_CHUNKS; ++c) {
      const int id = tid + c * GEMM_THREADS;
      *reinterpret_cast<u32x4*>(sB + (id / CPR) * LDT + (id % CPR) * E::CH) = rb[c];
    }
    __syncthreads();
    if (k0 + E::BK < k_end) {
      TDF_LOAD_TILE(k0 + E::BK)
    }
#pragma unroll
    for (int ks = 0; ks < E::BK / E::MK; ++ks) {
      typename E::Frag fa[MB], fb[WN];
#pragma unroll
      for (int i = 0; i < MB; ++i) fa[i] = E::frag(tA + i * 32 * LDT, ks, lane);
#pragma unroll
      for (int j = 0; j < WN; ++j) fb[j] = E::frag(tB + j * 32 * LDT, ks, lane);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = E::mma(fa[i], fb[j], acc[i][j]);
    }
    __syncthreads();
  }
#undef TDF_LOAD_TILE

  // ---- epilogue.  acc[i][j][r]: row = i*32 + (r/4)*8 + (lane/32)*4 + r%4, column = lane%32
  // The element offsets of the tile's rows (row index x Hp: below 2^32, the host checks) go through
  // LDS, so that no store waits on an index load and no lane multiplies.  LSTM_FWD: a child that is
  // a leaf has no stored cell state; it reads row 0 of Cs instead, a leaf's row that k_embed zeroes.
  uint32_t* sOut = reinterpret_cast<uint32_t*>(smem);
  uint32_t* sL = sOut + BM;
  uint32_t* sR = sL + BM;
  if (MODE != DW_SPLIT && tid < BM) {
    const int m = min(m0 + tid, g.M - 1);
    if (MODE == RNN_FWD) sOut[tid] = (g.out0 + (uint32_t)m) * (uint32_t)g.Hp;
    const uint32_t l = g.l[m], r = g.r[m];
    sL[tid] = MODE == LSTM_FWD && l < g.leaf_rows ? 0u : l * (uint32_t)g.Hp;
    sR[tid] = MODE == LSTM_FWD && r < g.leaf_rows ? 0u : r * (uint32_t)g.Hp;
  }
  __syncthreads();
  const int col = lane & 31;
  auto row_of = [&](int i, int r) { return wrow + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); };
  if constexpr (MODE == LSTM_FWD) {
    // Byte offsets: 32 bits wide where every array of the launch ends below 4 GiB (NARROW, checked by
    // the host: an address is then a uniform base plus one 32-bit register), else 64.
    typedef typename std::conditional<NARROW, uint32_t, size_t>::type Off;
    const int jb = nt * WNS + wn;
    if (jb * 32 < g.Hp) {
      const int n = jb * 32 + col;   // hidden unit
      const float bi = Act<T>::pre_sigmoid(g.bias[n]), bfl = Act<T>::pre_sigmoid(g.bias[g.Hp + n]);
      const float bfr = Act<T>::pre_sigmoid(g.bias[2 * g.Hp + n]), bo = Act<T>::pre_sigmoid(g.bias[3 * g.Hp + n]);
      const float bu = Act<T>::pre_tanh(g.bias[4 * g.Hp + n]);
      const char* const cs_in = reinterpret_cast<const char*>(g.Cs);
      char* const cs = reinterpret_cast<char*>(g.Cs);
      char* const hs = reinterpret_cast<char*>(g.Hs_out);
      // the five gate blocks of a row lie Hp elements apart: five uniform bases, one lane offset
      char* gt[5];
#pragma unroll
      for (int k = 0; k < 5; ++k) gt[k] = reinterpret_cast<char*>(g.gates) + (size_t)k * g.Hp * sizeof(T);
      // The lane's first row of the tile; its other rows lie whole multiples of a row further on, and
      // those multiples are uniform values (kept apart from the lane's own offset: one add per access).
      const int row0 = wrow + (lane >> 5) * 4;
      const Off out_b = ((Off)(g.out0 + (uint32_t)(m0 + row0)) * (Off)g.Hp + (Off)n) * (Off)4;   // bytes into Cs
      const Off gate_b = ((Off)(m0 + row0) * (Off)g.ldg + (Off)n) * (Off)sizeof(T);              // bytes into gates
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        float cl[16], cr[16];   // children's cell states: all loads in flight before any store
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_of(i, r);
          cl[r] = *reinterpret_cast<const float*>(cs_in + (Off)(sL[row] + (uint32_t)n) * (Off)4);
          cr[r] = *reinterpret_cast<const float*>(cs_in + (Off)(sR[row] + (uint32_t)n) * (Off)4);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int d = i * 32 + (r >> 2) * 8 + (r & 3);   // row of the tile = row0 + d
          if (m0 + row0 + d >= g.M) continue;
          const float gi = Act<T>::sigmoid_b(acc[i][0][r], bi);
          const float gfl = Act<T>::sigmoid_b(acc[i][1][r], bfl);
          const float gfr = Act<T>::sigmoid_b(acc[i][2][r], bfr);
          const float go = Act<T>::sigmoid_b(acc[i][3][r], bo);
          const float gu = Act<T>::tanh_b(acc[i][4][r], bu);
          const float c = gi * gu + gfl * cl[r] + gfr * cr[r];
          const Off o = out_b + (Off)(uint32_t)__builtin_amdgcn_readfirstlane(d * g.Hp * 4);
          *reinterpret_cast<float*>(cs + o) = c;
          *reinterpret_cast<T*>(hs + o / (Off)(4 / sizeof(T))) = from_f<T>(go * Act<T>::tanh_b(c, 0.f));
          if (g.save_gates) {
            const Off go_b = gate_b + (Off)(uint32_t)__builtin_amdgcn_readfirstlane(d * (int)g.ldg * (int)sizeof(T));
            *reinterpret_cast<T*>(gt[0] + go_b) = from_f<T>(gi);
            *reinterpret_cast<T*>(gt[1] + go_b) = from_f<T>(gfl);
            *reinterpret_cast<T*>(gt[2] + go_b) = from_f<T>(gfr);
            *reinterpret_cast<T*>(gt[3] + go_b) = from_f<T>(go);
            *reinterpret_cast<T*>(gt[4] + go_b) = from_f<T>(gu);
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int n = nt * BN + (wn * WN + j) * 32 + col;
      if (n >= g.N) continue;
      float bias = 0.f;
      if (MODE == RNN_FWD) bias = g.bias[n];
#pragma unroll
      for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_of(i, r), m = m0 + row;
          if (m >= g.M) continue;
          if constexpr (MODE == RNN_FWD) {
            reinterpret_cast<T*>(g.Hs_out)[sOut[row] + (uint32_t)n] = from_f<T>(Act<T>::tanh(acc[i][j][r] + bias));
          } else if constexpr (MODE == DX_BWD) {
            // column n of [dh_l; dh_r]: each child row has exactly one consumer, plain store
            if (n < g.Hp) g.C[sL[row] + (uint32_t)n] = acc[i][j][r];
            else g.C[sR[row] + (uint32_t)(n - g.Hp)] = acc[i][j][r];
          } else {
            g.C[(size_t)split * g.M * g.ldc + (size_t)m * g.ldc + n] = acc[i][j][r];
          }
        }
      }
    }
  }
}

template <typename T, int MODE, int BM, int WNS> size_t gemm_lds_bytes() {
  constexpr int WN = MODE == LSTM_FWD ? 5 : 2;
  return (size_t)(BM + WNS * WN * 32) * (El<T>::BK + El<T>::PAD) * sizeof(T);
}

// Waves per workgroup of the tiled GEMM: 8 where a level's rows are gathered or scattered (two waves
// per SIMD hide each other's waits), 4 for the dense split GEMM of the weight gradients (fewer LDS
// reads per MFMA).
static int gemm_waves(int mode) { return mode == DW_SPLIT ? 4 : 8; }

template <typename T, int MODE, int NW, int BM, int WNS = 2, bool NARROW = false>
void launch_gemm_nw(GemmArgs g, int n_tiles_n, int splits, hipStream_t s) {
  if (g.M <= 0) return;
  g.n_tiles_n = n_tiles_n;
  const int n_mt = (g.M + BM - 1) / BM;
  g.n_splits = splits;
  dim3 grid(MODE == DW_SPLIT ? 8 * n_mt * n_tiles_n * ((splits + 7) / 8) : (n_mt + 7) / 8 * 8 * n_tiles_n);
  static bool lds_opt_in = false;   // tiles above 64 KiB of LDS need an explicit opt-in
  if (!lds_opt_in) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<DtOf<T>::value, MODE, NW, BM, WNS, NARROW>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)gemm_lds_bytes<T, MODE, BM, WNS>());
    lds_opt_in = true;
  }
  const size_t lds = gemm_lds_bytes<T, MODE, BM, WNS>();
  hipLaunchKernelGGL((k_gemm<DtOf<T>::value, MODE, NW, BM, WNS, NARROW>), grid, dim3(NW * 64), lds, s, g);
}

template <typename T, int MODE> void launch_gemm(GemmArgs g, int n_tiles_n, int splits, hipStream_t s) {
  // a level whose full tiles would leave compute units without a workgroup gets tiles of half the rows
  const bool half = MODE != DW_SPLIT && ((g.M + BM_FULL - 1) / BM_FULL) * n_tiles_n < 256;
  // LSTM cells: one block of 32 hidden units (x 5 gates) per workgroup, four waves of 32 rows: the
  // accumulators fit a third of the register file and three workgroups share a compute unit, each
  // in another phase of its k loop
  if (MODE == LSTM_FWD && g.narrow) launch_gemm_nw<T, MODE, 4, 128, 1, true>(g, n_tiles_n * 2, splits, s);
  else if (MODE == LSTM_FWD) launch_gemm_nw<T, MODE, 4, 128, 1>(g, n_tiles_n * 2, splits, s);
  else if (half) launch_gemm_nw<T, MODE, 4, 64>(g, n_tiles_n, splits, s);
  else if (gemm_waves(MODE) == 4) launch_gemm_nw<T, MODE, 4, 128>(g, n_tiles_n, splits, s);
  else launch_gemm_nw<T, MODE, 8, 128>(g, n_tiles_n, splits, s);
}

// ---- small levels ----------------------------------------------------------------------
// Deep in the recursion a dependency level holds few cells, and a level costs the latency of
// one kernel.  This variant keeps that chain short: a workgroup owns 32 cells x 32 hidden units
// (x gates), its four waves split the reduction four ways and load their MFMA operands
// straight from global memory (the weights come from L2, no LDS staging, few dependent round
// trips), and the partial tiles meet in LDS; wave w then finishes rows 8w..8w+7 of the tile.
// Operands are fetched as 16-byte chunks: for bf16 one chunk is one 32x32x16 operand; for fp32
// a chunk of four k-values feeds four 32x32x2 products, component j of both operands in
// product j (a fixed permutation of the reduction index).
// Operand order of a k-contiguous matrix [rows x K] for 32-row MFMA operands: the 16-byte chunks
// that the 64 lanes of a wave feed into one product step are stored one after the other (lane l
// holds row 32 rt + l % 32, reduction indices s * KC + (l / 32) * EPC ...), so a wave fetches an
// operand with one fully coalesced 1 KB load instead of touching 32 rows.
template <typename T> __host__ __device__ inline size_t frag_offset(int row, int k, int K) {
  constexpr int EPC = 16 / (int)sizeof(T), KC = 2 * EPC;
  const int rt = row >> 5, r = row & 31, st = k / KC, kk = k % KC, half = kk / EPC, el = kk % EPC;
  return (((size_t)rt * (K / KC) + st) * 64 + half * 32 + r) * EPC + el;
}

template <typename T> struct Chunk;
template <> struct Chunk<__bf16> {
  static constexpr int KC = 16;   // reduction indices covered by one chunk step of a wave
  static __device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Chunk<float> {
  static constexpr int KC = 8;
  static __device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    const f32x4 x = __builtin_bit_cast(f32x4, a), y = __builtin_bit_cast(f32x4, b);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.x, y.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.y, y.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.z, y.z, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.w, y.w, c, 0, 0, 0);
    return c;
  }
};

// One tile: rows 32 rt .. 32 rt + 31 of the level, hidden units (output columns) 32 ct .. 32 ct + 31.
// Called by all NW * 64 threads of a workgroup (NW = 4 or 8 waves split the reduction); `part` is
// its LDS scratch [wave][G][16][64].
// Weight operands of a wave for one column tile, kept in registers across tiles by the tail
// kernels (a workgroup there always works on the same column tile): RES chunk steps.
template <int MODE, int RES> struct ResidentB {
  static constexpr int G = MODE == LSTM_FWD ? 5 : 1;
  u32x4 f[RES > 0 ? RES : 1][G];
};

template <int DT, int MODE, int NW>
__device__ __forceinline__ const typename TypeOf<DT>::type* tile_b_base(const GemmArgs& g, int ct, int j) {
  typedef typename TypeOf<DT>::type T;
  constexpr int EPC = 16 / (int)sizeof(T);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int brt = (MODE == LSTM_FWD ? j * (g.Hp / 32) : 0) + ct;
  // operand order: chunk step st of this wave is 64 * EPC elements further on
  return reinterpret_cast<const T*>(g.Bf) + (((size_t)brt * (g.K / Chunk<T>::KC) + wave * (g.K / NW / Chunk<T>::KC)) * 64 + lane) * EPC;
}

template <int DT, int MODE, int NW, int RES>
__device__ __forceinline__ void load_resident_b(const GemmArgs& g, int ct, ResidentB<MODE, RES>& rb) {
  typedef typename TypeOf<DT>::type T;
  constexpr int EPC = 16 / (int)sizeof(T);
  const int steps = g.K / NW / Chunk<T>::KC;
#pragma unroll
  for (int j = 0; j < ResidentB<MODE, RES>::G; ++j) {
    const T* bp = tile_b_base<DT, MODE, NW>(g, ct, j);
#pragma unroll
    for (int st = 0; st < RES; ++st) rb.f[st][j] = *reinterpret_cast<const u32x4*>(bp + (size_t)min(st, steps - 1) * 64 * EPC);
  }
}

// RES > 0: the weight operands come from `rb` (which holds all chunk steps of this wave: the
// caller checked steps <= RES); RES == 0: they are fetched here.
// DX_BWD tiles of the tail launches also form the pre-activation gradients of the children they
// have just given their dh: a child has one parent, so once the parent's tile has produced dh of
// (child, unit) everything that dz of (child, unit) needs is final (dc came from the parent's own
// dz, the rest is forward state).  The separate dz pass over a level, and the barrier after it,
// are not needed then.  Only children inside the tail are handled (cq >= q_first): the cells of
// the wide levels get their dz from k_dz as before.
struct DzFuse {
  const VecArgs* v;
  const uint32_t *q_l, *q_r;     // children rows of every cell of the sorted log
  uint32_t row0;                 // first cell row: a child row below it is a leaf, else it is cell (row - row0)
  uint32_t q_first;              // first cell of the tail in the sorted log
};

template <int DT, int MODE, int NW, int RES = 0>
__device__ __forceinline__ void cell_small_tile(const GemmArgs& g, int rt, int ct, float* part,
                                                const ResidentB<MODE, RES>* rb = nullptr, const DzFuse* fz = nullptr) {
  typedef typename TypeOf<DT>::type T;
  typedef Chunk<T> C;
  constexpr int G = MODE == LSTM_FWD ? 5 : 1;      // 32-wide column blocks per tile
  constexpr int BATCH = 8;                          // chunk steps in flight
  constexpr int EPC = 16 / (int)sizeof(T);         // elements per chunk
  constexpr int RPW = 16 / NW;                     // accumulator registers (rows of a lane) a wave finishes
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = rt * 32;
  const int mA = min(m0 + (lane & 31), g.M - 1);   // operand row of this lane
  const int kw = g.K / NW;                         // reduction range of this wave: [wave * kw, +kw)

  // rows this lane finishes: accumulator register r = RPW * wave + rr holds row (r / 4) * 8 + (lane / 32) * 4 + r % 4
  auto row_of = [&](int rr) {
    const int r = RPW * wave + rr;
    return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
  };
  uint32_t o_out[RPW], o_l[RPW], o_r[RPW];
#pragma unroll
  for (int rr = 0; rr < RPW; ++rr) {
    const int m = min(m0 + row_of(rr), g.M - 1);
    if (MODE != DX_BWD) o_out[rr] = g.out0 + (uint32_t)m;
    if (MODE != RNN_FWD) { o_l[rr] = g.l[m]; o_r[rr] = g.r[m]; }
  }
  // operand bases (elements)
  const T* Ap;
  if (MODE == DX_BWD) {
    Ap = reinterpret_cast<const T*>(g.A) + (size_t)mA * g.lda + wave * kw;
  } else {
    const uint32_t child = wave < NW / 2 ? g.l[mA] : g.r[mA];   // first half of the waves: h_l of [h_l; h_r]
    Ap = reinterpret_cast<const T*>(g.Hs) + (size_t)child * g.Hp + (wave % (NW / 2)) * kw;
  }
  Ap += (lane >> 5) * EPC;
  const T* Bp[G];
#pragma unroll
  for (int j = 0; j < G; ++j) Bp[j] = tile_b_base<DT, MODE, NW>(g, ct, j);
  // children's cell states for the epilogue, requested before the products start
  float cl[RPW], cr[RPW];
  const int unit = ct * 32 + (lane & 31);
  if (MODE == LSTM_FWD) {
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      // (a leaf child has no stored cell state: it reads row 0, a leaf's row that k_embed keeps zero)
      cl[rr] = g.Cs[(o_l[rr] >= g.leaf_rows ? o_l[rr] : 0u) * (uint32_t)g.Hp + (uint32_t)unit];
      cr[rr] = g.Cs[(o_r[rr] >= g.leaf_rows ? o_r[rr] : 0u) * (uint32_t)g.Hp + (uint32_t)unit];
    }
  }

  // fused dz (DX_BWD in the tail): which child cell, and what its dz needs, requested early
  uint32_t z_q[RPW], z_row[RPW], z_gl[RPW], z_gr[RPW];
  float z_gate[RPW][5], z_c[RPW], z_dc[RPW], z_h[RPW], z_own[RPW];
  const bool z_on = MODE == DX_BWD && fz != nullptr;
  const bool z_left = unit < g.Hp;
  const int z_n = z_left ? unit : unit - g.Hp;
  if (MODE == DX_BWD && z_on) {
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int m = min(m0 + row_of(rr), g.M - 1);
      z_row[rr] = z_left ? o_l[rr] : o_r[rr];
      z_q[rr] = z_row[rr] >= fz->row0 ? z_row[rr] - fz->row0 : 0xFFFFFFFFu;   // a leaf has no cell
    }
  }

  f32x16 acc[G];
#pragma unroll
  for (int j = 0; j < G; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  const int steps = kw / C::KC;
  if (MODE == DX_BWD && z_on) {
    const VecArgs& v = *fz->v;
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const bool ok = z_q[rr] != 0xFFFFFFFFu && z_q[rr] >= fz->q_first;
      if (!ok) z_q[rr] = 0xFFFFFFFFu;
      const uint32_t qc = ok ? z_q[rr] : 0u;   // (cell 0 exists whenever a level has cells: a safe address)
      const size_t o = (size_t)z_row[rr] * v.Hp + z_n;
      z_own[rr] = v.dHn ? v.dHn[o] : 0.f;   // gradient of the child's own loss term
      if (v.cell_kind == 1) {
        z_h[rr] = to_f(reinterpret_cast<const T*>(v.Hs)[o]);
      } else {
        const T* g5 = reinterpret_cast<const T*>(v.gates) + (size_t)qc * v.Np + z_n;
#pragma unroll
        for (int k = 0; k < 5; ++k) z_gate[rr][k] = to_f(g5[k * v.Hp]);
        z_c[rr] = v.Cs[o];
        z_dc[rr] = v.dC[o];
        z_gl[rr] = fz->q_l[qc];
        z_gr[rr] = fz->q_r[qc];
      }
    }
  }
  if constexpr (RES > 0) {
    u32x4 fa[RES];
#pragma unroll
    for (int st = 0; st < RES; ++st) fa[st] = *reinterpret_cast<const u32x4*>(Ap + min(st, steps - 1) * C::KC);
#pragma unroll
    for (int st = 0; st < RES; ++st) {
      if (st < steps) {
#pragma unroll
        for (int j = 0; j < G; ++j) acc[j] = C::mma(fa[st], rb->f[st][j], acc[j]);
      }
    }
  } else
  for (int s0 = 0; s0 < steps; s0 += BATCH) {
    u32x4 fa[BATCH], fb[BATCH][G];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      const int st = min(s0 + b, steps - 1);       // a short last batch repeats its final chunk ...
#pragma unroll
      for (int j = 0; j < G; ++j) fb[b][j] = *reinterpret_cast<const u32x4*>(Bp[j] + (size_t)st * 64 * EPC);
      fa[b] = *reinterpret_cast<const u32x4*>(Ap + st * C::KC);
    }
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
      if (s0 + b < steps) {                        // ... and leaves it out of the sum
#pragma unroll
        for (int j = 0; j < G; ++j) acc[j] = C::mma(fa[b], fb[b][j], acc[j]);
      }
    }
  }

  // partial tiles -> LDS; wave w sums and finishes r = 4w .. 4w+3
#pragma unroll
  for (int j = 0; j < G; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) part[((wave * G + j) * 16 + r) * 64 + lane] = acc[j][r];
  __syncthreads();
  float z[G][RPW];
#pragma unroll
  for (int j = 0; j < G; ++j)
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) t += part[((w * G + j) * 16 + RPW * wave + rr) * 64 + lane];
      z[j][rr] = t;
    }

  if constexpr (MODE == LSTM_FWD) {
    const float bi = Act<T>::pre_sigmoid(g.bias[unit]), bfl = Act<T>::pre_sigmoid(g.bias[g.Hp + unit]);
    const float bfr = Act<T>::pre_sigmoid(g.bias[2 * g.Hp + unit]), bo = Act<T>::pre_sigmoid(g.bias[3 * g.Hp + unit]);
    const float bu = Act<T>::pre_tanh(g.bias[4 * g.Hp + unit]);
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int m = m0 + row_of(rr);
      if (m >= g.M) continue;
      const float gi = Act<T>::sigmoid_b(z[0][rr], bi);
      const float gfl = Act<T>::sigmoid_b(z[1][rr], bfl);
      const float gfr = Act<T>::sigmoid_b(z[2][rr], bfr);
      const float go = Act<T>::sigmoid_b(z[3][rr], bo);
      const float gu = Act<T>::tanh_b(z[4][rr], bu);
      const float c = gi * gu + gfl * cl[rr] + gfr * cr[rr];
      const size_t o = (size_t)o_out[rr] * g.Hp + unit;
      g.Cs[o] = c;
      reinterpret_cast<T*>(g.Hs_out)[o] = from_f<T>(go * Act<T>::tanh_b(c, 0.f));
      if (g.save_gates) {
        T* gr = reinterpret_cast<T*>(g.gates) + (size_t)m * g.ldg;
        gr[unit] = from_f<T>(gi);
        gr[g.Hp + unit] = from_f<T>(gfl);
        gr[2 * g.Hp + unit] = from_f<T>(gfr);
        gr[3 * g.Hp + unit] = from_f<T>(go);
        gr[4 * g.Hp + unit] = from_f<T>(gu);
      }
    }
  } else if constexpr (MODE == RNN_FWD) {
    const float bias = g.bias[unit];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int m = m0 + row_of(rr);
      if (m >= g.M) continue;
      reinterpret_cast<T*>(g.Hs_out)[(size_t)o_out[rr] * g.Hp + unit] = from_f<T>(Act<T>::tanh(z[0][rr] + bias));
    }
  } else {   // DX_BWD: column `unit` of [dh_l; dh_r]; each child row has exactly one consumer
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
      const int m = m0 + row_of(rr);
      if (m >= g.M) continue;
      if (unit < g.Hp) g.C[(size_t)o_l[rr] * g.Hp + unit] = z[0][rr];
      else g.C[(size_t)o_r[rr] * g.Hp + (unit - g.Hp)] = z[0][rr];
    }
    if (z_on) {
      const VecArgs& v = *fz->v;
      float z_cl[RPW], z_cr[RPW];
      if (v.cell_kind == 2) {
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
          z_cl[rr] = z_gl[rr] >= fz->row0 ? v.Cs[(size_t)z_gl[rr] * v.Hp + z_n] : 0.f;   // (a leaf's cell state is zero)
          z_cr[rr] = z_gr[rr] >= fz->row0 ? v.Cs[(size_t)z_gr[rr] * v.Hp + z_n] : 0.f;
        }
      }
#pragma unroll
      for (int rr = 0; rr < RPW; ++rr) {
        const int m = m0 + row_of(rr);
        if (m >= g.M || z_q[rr] == 0xFFFFFFFFu) continue;
        const float dh = z[0][rr] + z_own[rr];
        if (z_n == 0) atomicAdd(&v.gmark[z_row[rr]], 1u);   // one lane per child cell: its gradient body fires here
        T* dz = reinterpret_cast<T*>(v.Dz) + (size_t)z_q[rr] * v.Np + z_n;
        if (v.cell_kind == 1) {
          dz[0] = from_f<T>(dh * (1.f - z_h[rr] * z_h[rr]));
        } else {
          const float gi = z_gate[rr][0], gfl = z_gate[rr][1], gfr = z_gate[rr][2], go = z_gate[rr][3], gu = z_gate[rr][4];
          const float tc = Act<T>::tanh(z_c[rr]);
          const float dc = z_dc[rr] + dh * go * (1.f - tc * tc);
          dz[0] = from_f<T>(dc * gu * gi * (1.f - gi));
          dz[v.Hp] = from_f<T>(dc * z_cl[rr] * gfl * (1.f - gfl));
          dz[2 * v.Hp] = from_f<T>(dc * z_cr[rr] * gfr * (1.f - gfr));
          dz[3 * v.Hp] = from_f<T>(dh * tc * go * (1.f - go));
          dz[4 * v.Hp] = from_f<T>(dc * gi * (1.f - gu * gu));
          if (z_gl[rr] >= fz->row0) v.dC[(size_t)z_gl[rr] * v.Hp + z_n] = dc * gfl;   // (a leaf has no use for dc)
          if (z_gr[rr] >= fz->row0) v.dC[(size_t)z_gr[rr] * v.Hp + z_n] = dc * gfr;
        }
      }
    }
  }
  __syncthreads();   // `part` is free for the workgroup's next tile
}

template <int DT, int MODE, int NW>
__global__ void __launch_bounds__(NW * 64) k_cell_small(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int n_ct = g.n_tiles_n;                    // column tiles of 32
  cell_small_tile<DT, MODE, NW>(g, blockIdx.x / n_ct, blockIdx.x % n_ct, reinterpret_cast<float*>(smem));
}

// Levels of at most this many cells take the small-level kernel (TDF_SMALL_LEVEL overrides).
static uint32_t small_level() {
  const char* e = getenv("TDF_SMALL_LEVEL");
  return e ? (uint32_t)atoll(e) : 1024u;
}

// Waves that split the reduction of a small-level tile: eight where the tile has one column
// block (RNN forward, input gradient) and the reduction divides evenly, else four.
template <typename T, int MODE> int small_tile_waves(int K) {
  return MODE != LSTM_FWD && (K / 8) % Chunk<T>::KC == 0 && K / 8 >= Chunk<T>::KC ? 8 : 4;
}

template <typename T, int MODE, int NW> void launch_cell_small_nw(GemmArgs g, int n_col_tiles, hipStream_t s) {
  constexpr int G = MODE == LSTM_FWD ? 5 : 1;
  const size_t lds = (size_t)NW * G * 16 * 64 * sizeof(float);
  static bool lds_opt_in = false;
  if (!lds_opt_in && lds > 48 * 1024) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_cell_small<DtOf<T>::value, MODE, NW>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    lds_opt_in = true;
  }
  g.n_tiles_n = n_col_tiles;
  const int n_rt = (g.M + 31) / 32;
  hipLaunchKernelGGL((k_cell_small<DtOf<T>::value, MODE, NW>), dim3(n_rt * n_col_tiles), dim3(NW * 64), lds, s, g);
}
template <typename T, int MODE> void launch_cell_small(GemmArgs g, int n_col_tiles, hipStream_t s) {
  if (g.M <= 0) return;
  if constexpr (MODE != LSTM_FWD) {
    if (small_tile_waves<T, MODE>(g.K) == 8) return launch_cell_small_nw<T, MODE, 8>(g, n_col_tiles, s);
  }
  launch_cell_small_nw<T, MODE, 4>(g, n_col_tiles, s);
}

// ---- packing of W: padded, k-contiguous [Np x Kp], and its transpose [Kp x Np] ---------------
template <int DT>
__global__ void k_pack_w(VecArgs v) {
  typedef typename TypeOf<DT>::type T;
  const int total = v.Np * v.Kp;
  for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
    const int np = idx / v.Kp, kp = idx % v.Kp;
    const int gate = np / v.Hp, j = np % v.Hp, half = kp / v.Hp, i = kp % v.Hp;
    T w = from_f<T>(0.f);
    if (j < v.H && i < v.H)
      w = reinterpret_cast<const T*>(v.W)[(size_t)(gate * v.H + j) * (2 * v.H) + half * v.H + i];
    reinterpret_cast<T*>(v.Wp)[idx] = w;
    reinterpret_cast<T*>(v.Wf)[frag_offset<T>(np, kp, v.Kp)] = w;
    if (v.WpT) {
      reinterpret_cast<T*>(v.WpT)[(size_t)kp * v.Np + np] = w;
      reinterpret_cast<T*>(v.WfT)[frag_offset<T>(kp, np, v.Np)] = w;
    }
    if (kp == 0) v.bp[np] = j < v.H ? v.b[gate * v.H + j] : 0.f;
  }
}

// ---- leaves: state row = E[token], zero padding; no cell state (row 0 of Cs is kept zero in its place) ----
// A group of `lpl` lanes (a power of two, at least the row's 16-byte chunks up to 64) copies one leaf's row
// in 16-byte chunks where the rows of E are aligned for that (H a multiple of the chunk), else element by
// element.
template <int DT>
__global__ void k_embed(VecArgs v, Engine e, uint32_t n_leaf, int lpl) {
  typedef typename TypeOf<DT>::type T;
  constexpr int EPC = 16 / (int)sizeof(T);
  const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x, n_threads = gridDim.x * blockDim.x;
  if (v.cell_kind == 2 && tid < (uint32_t)v.Hp) v.Cs[tid] = 0.f;   // (Hp <= 8192 <= threads of the launch: see vec_embed)
  const uint32_t group = tid / (uint32_t)lpl, n_groups = n_threads / (uint32_t)lpl;
  const int gl = (int)(tid % (uint32_t)lpl);
  const bool chunks = v.H % EPC == 0 && reinterpret_cast<uintptr_t>(v.E) % 16 == 0;
  for (uint32_t i = group; i < n_leaf; i += n_groups) {
    const uint32_t tok = e.leaf_tok[i];   // (token ids were checked when the leaf fired)
    const T* src = reinterpret_cast<const T*>(v.E) + (size_t)(tok < (uint32_t)v.vocab ? tok : 0) * v.H;
    T* dst = reinterpret_cast<T*>(v.Hs) + (size_t)i * v.Hp;   // leaf i has row i
    if (chunks) {
      for (int n = gl * EPC; n < v.Hp; n += lpl * EPC) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4*>(dst + n) = n < v.H ? *reinterpret_cast<const u32x4*>(src + n) : zero;
      }
    } else {
      for (int n = gl; n < v.Hp; n += lpl) dst[n] = n < v.H ? src[n] : from_f<T>(0.f);
    }
  }
}

// ---- classification head: loss_b = -log softmax(U h + u0)[label]; dh = U^T (p - onehot) dloss ---
template <int DT>
__global__ void k_head(VecArgs v, Engine e, const float* dy, int with_grad, int cls) {
  typedef typename TypeOf<DT>::type T;
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (wave >= (int)e.n_inst) return;
  if (cls >= 0 && (int)e.inst_class[wave] != cls) return;   // only the instances of one class
  const uint32_t row = e.head_row[wave];
  const int label = (int)e.head_label[wave];
  const T* h = reinterpret_cast<const T*>(v.Hs) + (size_t)row * v.Hp;
  float logit[16];
  float mx = -3.0e38f;
  for (int c = 0; c < v.n_classes; ++c) {
    float s = 0.f;
    for (int n = lane; n < v.H; n += 64) s += v.U[c * v.H + n] * to_f(h[n]);
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    logit[c] = s + v.u0[c];
    mx = fmaxf(mx, logit[c]);
  }
  float z = 0.f;
  for (int c = 0; c < v.n_classes; ++c) z += expf(logit[c] - mx);
  const float lse = mx + logf(z);
  if (lane == 0) v.loss[wave] = lse - logit[label < v.n_classes ? label : 0];
  if (with_grad) {
    const float d = dy[wave];
    for (int n = lane; n < v.Hp; n += 64) {
      float s = 0.f;
      if (n < v.H)
        for (int c = 0; c < v.n_classes; ++c)
          s += (expf(logit[c] - lse) - (c == label ? 1.f : 0.f)) * v.U[c * v.H + n];
      v.dH[(size_t)row * v.Hp + n] = s * d;
      if (v.cell_kind == 2) v.dC[(size_t)row * v.Hp + n] = 0.f;
    }
  }
}

// Loss terms of the nodes (CE_NODE): sixteen lanes per state row, four rows per wave, U in LDS
// (padded to the row stride) where it fits.  A row that was marked with a tree node v whose
// label is a class gets loss[v] = -log softmax(U h + u0)[label]; in a gradient run the row of
// dHn becomes dnode[v] U^T (p - onehot), 0 for rows without a term.
template <int DT>
__global__ void __launch_bounds__(256) k_node_ce(VecArgs v, Engine e, uint32_t n_leaf, uint32_t n_cell, const int32_t* node_label,
                                                 float* out_loss, const float* dnode, int with_grad, int u_in_lds) {
  typedef typename TypeOf<DT>::type T;
  constexpr int CH = 16 / (int)sizeof(T);   // elements of a 16-byte chunk of a state row
  extern __shared__ __attribute__((aligned(16))) float sU[];
  if (u_in_lds) {
    for (int i = threadIdx.x; i < v.n_classes * v.Hp; i += blockDim.x) {
      const int c = i / v.Hp, n = i % v.Hp;
      sU[i] = n < v.H ? v.U[c * v.H + n] : 0.f;
    }
    __syncthreads();
  }
  auto u_at4 = [&](int c, int n) -> float4 {   // U[c][n .. n+3], zero beyond H
    if (u_in_lds) return *reinterpret_cast<const float4*>(sU + c * v.Hp + n);
    const float* u = v.U + (size_t)c * v.H;
    return make_float4(n < v.H ? u[n] : 0.f, n + 1 < v.H ? u[n + 1] : 0.f, n + 2 < v.H ? u[n + 2] : 0.f, n + 3 < v.H ? u[n + 3] : 0.f);
  };
  const int sub = threadIdx.x & 15;
  const uint32_t grp = (blockIdx.x * blockDim.x + threadIdx.x) >> 4, n_grp = (gridDim.x * blockDim.x) >> 4;
  for (uint32_t i = grp; i < n_leaf + n_cell; i += n_grp) {
    const uint32_t row = i;
    const uint32_t node = e.node_of_row[row];
    int label = -1;
    if (node != 0xFFFFFFFFu) label = node_label[node];
    if (label >= v.n_classes) label = -1;
    float* dh = with_grad ? v.dHn + (size_t)row * v.Hp : nullptr;
    if (label < 0) {   // (the sixteen lanes of a row take this branch together)
      if (with_grad)
        for (int n = sub * 4; n < v.Hp; n += 64) *reinterpret_cast<float4*>(dh + n) = make_float4(0.f, 0.f, 0.f, 0.f);
      continue;
    }
    const T* h = reinterpret_cast<const T*>(v.Hs) + (size_t)row * v.Hp;
    float logit[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) logit[c] = 0.f;
    for (int n0 = sub * CH; n0 < v.Hp; n0 += 16 * CH) {
      union { u32x4 raw; T t[CH]; } x;
      x.raw = *reinterpret_cast<const u32x4*>(h + n0);
      float xf[CH];
#pragma unroll
      for (int j = 0; j < CH; ++j) xf[j] = to_f(x.t[j]);
#pragma unroll
      for (int c = 0; c < 16; ++c)
        if (c < v.n_classes) {
#pragma unroll
          for (int j = 0; j < CH; j += 4) {
            const float4 u = u_at4(c, n0 + j);
            logit[c] += u.x * xf[j] + u.y * xf[j + 1] + u.z * xf[j + 2] + u.w * xf[j + 3];
          }
        }
    }
    float mx = -3.0e38f;
#pragma unroll
    for (int c = 0; c < 16; ++c)
      if (c < v.n_classes) {
        float s = logit[c];
        for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off);
        logit[c] = s + v.u0[c];
        mx = fmaxf(mx, logit[c]);
      }
    float z = 0.f, own = 0.f;
#pragma unroll
    for (int c = 0; c < 16; ++c)
      if (c < v.n_classes) {
        z += expf(logit[c] - mx);
        own = c == label ? logit[c] : own;
      }
    const float lse = mx + logf(z);
    if (sub == 0) out_loss[node] = lse - own;
    if (with_grad) {
      const float d = dnode[node];
#pragma unroll
      for (int c = 0; c < 16; ++c)   // logit becomes d (p - onehot)
        if (c < v.n_classes) logit[c] = d * (expf(logit[c] - lse) - (c == label ? 1.f : 0.f));
      for (int n0 = sub * CH; n0 < v.Hp; n0 += 16 * CH) {
        float g[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) g[j] = 0.f;
#pragma unroll
        for (int c = 0; c < 16; ++c)
          if (c < v.n_classes) {
#pragma unroll
            for (int j = 0; j < CH; j += 4) {
              const float4 u = u_at4(c, n0 + j);
              g[j] += logit[c] * u.x; g[j + 1] += logit[c] * u.y; g[j + 2] += logit[c] * u.z; g[j + 3] += logit[c] * u.w;
            }
          }
#pragma unroll
        for (int j = 0; j < CH; j += 4) *reinterpret_cast<float4*>(dh + n0 + j) = make_float4(g[j], g[j + 1], g[j + 2], g[j + 3]);
      }
    }
  }
}

// vector result: seed dH of each root row with the caller's dy (none: zero); copy the root rows out
__global__ void k_seed_dy(VecArgs v, Engine e, const float* dy) {
  const int b = blockIdx.x;
  const uint32_t row = e.root_ref[b];
  for (int n = threadIdx.x; n < v.Hp; n += blockDim.x) {
    v.dH[(size_t)row * v.Hp + n] = dy && n < v.H ? dy[(size_t)b * v.H + n] : 0.f;
    if (v.cell_kind == 2) v.dC[(size_t)row * v.Hp + n] = 0.f;
  }
}

template <int DT>
__global__ void k_out_rows(VecArgs v, Engine e, float* out_h, float* out_c) {
  typedef typename TypeOf<DT>::type T;
  const int b = blockIdx.x;
  const uint32_t row = e.root_ref[b];
  for (int n = threadIdx.x; n < v.H; n += blockDim.x) {
    if (out_h) out_h[(size_t)b * v.H + n] = to_f(reinterpret_cast<const T*>(v.Hs)[(size_t)row * v.Hp + n]);
    if (out_c && v.cell_kind == 2) out_c[(size_t)b * v.H + n] = row >= e.row0 ? v.Cs[(size_t)row * v.Hp + n] : 0.f;
  }
}

// ---- pre-activation gradients of one level ------------------------------------------------------
// TreeRNN: delta = dh * (1 - h^2).  TreeLSTM: the gate gradients (i, f_l, f_r, o, u) and the
// cell-state gradients handed to the two children.
template <int DT>
__device__ __forceinline__ void dz_row(const VecArgs& v, const Engine& e, uint32_t q) {
  typedef typename TypeOf<DT>::type T;
  const size_t o = (size_t)(e.row0 + q) * v.Hp;
  T* dz = reinterpret_cast<T*>(v.Dz) + (size_t)q * v.Np;
  if (threadIdx.x == 0) atomicAdd(&v.gmark[e.row0 + q], 1u);   // the gradient body of this tag fires
  if (v.cell_kind == 1) {
    for (int n = threadIdx.x; n < v.Hp; n += blockDim.x) {
      const float h = to_f(reinterpret_cast<const T*>(v.Hs)[o + n]);
      dz[n] = from_f<T>((v.dH[o + n] + (v.dHn ? v.dHn[o + n] : 0.f)) * (1.f - h * h));
    }
  } else {
    const bool cell_l = e.q_l[q] >= e.row0, cell_r = e.q_r[q] >= e.row0;   // a leaf child: c = 0, no use for dc
    const size_t ol = (size_t)e.q_l[q] * v.Hp, orr = (size_t)e.q_r[q] * v.Hp;
    const T* gt = reinterpret_cast<const T*>(v.gates) + (size_t)q * v.Np;
    for (int n = threadIdx.x; n < v.Hp; n += blockDim.x) {
      const float gi = to_f(gt[n]), gfl = to_f(gt[v.Hp + n]), gfr = to_f(gt[2 * v.Hp + n]);
      const float go = to_f(gt[3 * v.Hp + n]), gu = to_f(gt[4 * v.Hp + n]);
      const float tc = Act<T>::tanh(v.Cs[o + n]);
      const float dh = v.dH[o + n] + (v.dHn ? v.dHn[o + n] : 0.f);
      const float dc = v.dC[o + n] + dh * go * (1.f - tc * tc);
      const float cl = cell_l ? v.Cs[ol + n] : 0.f, cr = cell_r ? v.Cs[orr + n] : 0.f;
      dz[n] = from_f<T>(dc * gu * gi * (1.f - gi));
      dz[v.Hp + n] = from_f<T>(dc * cl * gfl * (1.f - gfl));
      dz[2 * v.Hp + n] = from_f<T>(dc * cr * gfr * (1.f - gfr));
      dz[3 * v.Hp + n] = from_f<T>(dh * tc * go * (1.f - go));
      dz[4 * v.Hp + n] = from_f<T>(dc * gi * (1.f - gu * gu));
      if (cell_l) v.dC[ol + n] = dc * gfl;
      if (cell_r) v.dC[orr + n] = dc * gfr;
    }
  }
}
// The same for a whole level, four hidden units per lane (8- and 16-byte accesses; the padded width is a
// multiple of 64): a group of Hp / 4 lanes (at most 256) per cell, 256 / group cells per workgroup.
template <typename T> __device__ __forceinline__ f32x4 load4(const T* p);
template <> __device__ __forceinline__ f32x4 load4<float>(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
template <> __device__ __forceinline__ f32x4 load4<__bf16>(const __bf16* p) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
  const bf16x4 w = *reinterpret_cast<const bf16x4*>(p);
  return f32x4{(float)w[0], (float)w[1], (float)w[2], (float)w[3]};
}
template <typename T> __device__ __forceinline__ void store4(T* p, f32x4 x);
template <> __device__ __forceinline__ void store4<float>(float* p, f32x4 x) { *reinterpret_cast<f32x4*>(p) = x; }
template <> __device__ __forceinline__ void store4<__bf16>(__bf16* p, f32x4 x) {
  typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
  bf16x4 w;
  w[0] = (__bf16)x[0]; w[1] = (__bf16)x[1]; w[2] = (__bf16)x[2]; w[3] = (__bf16)x[3];
  *reinterpret_cast<bf16x4*>(p) = w;
}
template <int DT>
__global__ void __launch_bounds__(256) k_dz(VecArgs v, Engine e, uint32_t q0, uint32_t count) {
  typedef typename TypeOf<DT>::type T;
  const int group = min(256, v.Hp / 4), per_block = 256 / group;
  const int gi = threadIdx.x / group, gl = threadIdx.x % group;
  const uint32_t k = blockIdx.x * per_block + gi;
  if (gi >= per_block || k >= count) return;
  const uint32_t q = q0 + k;
  const size_t o = (size_t)(e.row0 + q) * v.Hp;
  T* dz = reinterpret_cast<T*>(v.Dz) + (size_t)q * v.Np;
  if (gl == 0) atomicAdd(&v.gmark[e.row0 + q], 1u);   // the gradient body of this tag fires
  if (v.cell_kind == 1) {
    for (int n = gl * 4; n < v.Hp; n += group * 4) {
      const f32x4 h = load4<T>(reinterpret_cast<const T*>(v.Hs) + o + n);
      f32x4 dh = load4<float>(v.dH + o + n);
      if (v.dHn) dh += load4<float>(v.dHn + o + n);
      store4<T>(dz + n, dh * (1.f - h * h));
    }
  } else {
    const bool cell_l = e.q_l[q] >= e.row0, cell_r = e.q_r[q] >= e.row0;   // a leaf child: c = 0, no use for dc
    const size_t ol = (size_t)e.q_l[q] * v.Hp, orr = (size_t)e.q_r[q] * v.Hp;
    const T* gt = reinterpret_cast<const T*>(v.gates) + (size_t)q * v.Np;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (int n = gl * 4; n < v.Hp; n += group * 4) {
      const f32x4 gi4 = load4<T>(gt + n), gfl = load4<T>(gt + v.Hp + n), gfr = load4<T>(gt + 2 * v.Hp + n);
      const f32x4 go = load4<T>(gt + 3 * v.Hp + n), gu = load4<T>(gt + 4 * v.Hp + n);
      const f32x4 c = load4<float>(v.Cs + o + n);
      f32x4 dh = load4<float>(v.dH + o + n);
      if (v.dHn) dh += load4<float>(v.dHn + o + n);
      const f32x4 dc_in = load4<float>(v.dC + o + n);
      const f32x4 cl = cell_l ? load4<float>(v.Cs + ol + n) : zero, cr = cell_r ? load4<float>(v.Cs + orr + n) : zero;
      f32x4 tc;
#pragma unroll
      for (int t = 0; t < 4; ++t) tc[t] = Act<T>::tanh(c[t]);
      const f32x4 dc = dc_in + dh * go * (1.f - tc * tc);
      store4<T>(dz + n, dc * gu * gi4 * (1.f - gi4));
      store4<T>(dz + v.Hp + n, dc * cl * gfl * (1.f - gfl));
      store4<T>(dz + 2 * v.Hp + n, dc * cr * gfr * (1.f - gfr));
      store4<T>(dz + 3 * v.Hp + n, dh * tc * go * (1.f - go));
      store4<T>(dz + 4 * v.Hp + n, dc * gi4 * (1.f - gu * gu));
      if (cell_l) store4<float>(v.dC + ol + n, dc * gfl);
      if (cell_r) store4<float>(v.dC + orr + n, dc * gfr);
    }
  }
}

// ---- the tail of the level schedule in one launch ------------------------------------------------
// The cells of a level are sorted by the tag machine (= die) their instance was dealt to, and a
// cell depends only on cells of its own instance.  So each die can walk the levels on its own:
// workgroups i, i + 8, ... of the launch take the tiles of machine i % 8's cells, level after
// level, with a barrier among themselves (die_sync.h) where a launch boundary would be.  Used
// for the deep levels, where a level is a few tiles per die and costs one barrier (~2 us)
// instead of one launch (~10 us).
struct TailArgs {
  const uint32_t* level_off;   // first cell of (level, machine) in the sorted log, by sort key
  uint32_t lvl_first, lvl_last;
  uint32_t n_dies;
  DieSync* sync;               // [8], zero on entry
  long long spin_ticks;
  uint32_t q_first;            // first cell of the tail in the sorted log
};

template <int DT, int MODE, int NW>
__global__ void __launch_bounds__(NW * 64) k_tail_fwd(GemmArgs g, TailArgs t) {
  typedef typename TypeOf<DT>::type T;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ uint32_t sh_ok;
  float* part = reinterpret_cast<float*>(smem);
  const uint32_t die = blockIdx.x % XCDS, rank = blockIdx.x / XCDS, G = gridDim.x / XCDS;
  if (die >= t.n_dies) return;
  // A level here is one link of a dependency chain: these waves are bound by latency, and other
  // kernels (the wide levels of other instances) may share the compute unit: issue before them.
  __builtin_amdgcn_s_setprio(3);
  DieSync* sy = t.sync + die;
  if (threadIdx.x == 0) atomicOr(&sy->xcc_mask, 1u << xcc_id());
  const int n_ct = g.n_tiles_n;
  // A workgroup keeps to one column tile where the tiles divide evenly among the workgroups,
  // and then holds that tile's weight operands in registers for the whole launch.
  constexpr int RES = 8;
  const bool resident = G % (uint32_t)n_ct == 0 && g.K / NW / Chunk<T>::KC <= RES;
  ResidentB<MODE, RES> rb;
  if (resident) load_resident_b<DT, MODE, NW, RES>(g, (int)(rank % n_ct), rb);
  uint32_t gen = 0;
  for (uint32_t lvl = t.lvl_first; lvl <= t.lvl_last; ++lvl) {
    const uint32_t q0 = t.level_off[lvl * LEVEL_KEY_DIES + die];
    const uint32_t cnt = t.level_off[lvl * LEVEL_KEY_DIES + die + 1] - q0;
    GemmArgs gl = g;
    gl.M = (int)cnt;
    gl.out0 = g.out0 + q0; gl.l = g.l + q0; gl.r = g.r + q0;
    gl.gates = g.gates ? reinterpret_cast<T*>(g.gates) + (size_t)q0 * g.ldg : nullptr;
    const uint32_t n_rt = (cnt + 31) / 32;
    if (resident) {
      for (uint32_t rt = rank / n_ct; rt < n_rt; rt += G / n_ct)
        cell_small_tile<DT, MODE, NW, RES>(gl, (int)rt, (int)(rank % n_ct), part, &rb);
    } else {
      for (uint32_t tile = rank; tile < n_rt * n_ct; tile += G)
        cell_small_tile<DT, MODE, NW>(gl, (int)(tile / n_ct), (int)(tile % n_ct), part);
    }
    if (!die_barrier(sy, G, gen++, t.spin_ticks, &sh_ok)) return;
  }
}

// Gradient pass over the same levels, deepest first: dz of the die's cells of a level, barrier,
// their input gradients, barrier.
template <int DT, int NW>
__global__ void __launch_bounds__(NW * 64) k_tail_bwd(GemmArgs g, VecArgs v, Engine e, TailArgs t) {
  typedef typename TypeOf<DT>::type T;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  __shared__ uint32_t sh_ok;
  float* part = reinterpret_cast<float*>(smem);
  const uint32_t die = blockIdx.x % XCDS, rank = blockIdx.x / XCDS, G = gridDim.x / XCDS;
  if (die >= t.n_dies) return;
  // A level here is one link of a dependency chain: these waves are bound by latency, and other
  // kernels (the wide levels of other instances) may share the compute unit: issue before them.
  __builtin_amdgcn_s_setprio(3);
  DieSync* sy = t.sync + die;
  if (threadIdx.x == 0) atomicOr(&sy->xcc_mask, 1u << xcc_id());
  const int n_ct = g.n_tiles_n;
  constexpr int RES = 10;
  const bool resident = G % (uint32_t)n_ct == 0 && g.K / NW / Chunk<T>::KC <= RES;
  ResidentB<DX_BWD, RES> rb;
  if (resident) load_resident_b<DT, DX_BWD, NW, RES>(g, (int)(rank % n_ct), rb);
  uint32_t gen = 0;
  for (uint32_t lvl = t.lvl_last; lvl >= t.lvl_first; --lvl) {
    const uint32_t q0 = t.level_off[lvl * LEVEL_KEY_DIES + die];
    const uint32_t cnt = t.level_off[lvl * LEVEL_KEY_DIES + die + 1] - q0;
    // (dz of this level's cells: from their parents' tiles, or, for the roots, from k_dz_tail_roots)
    GemmArgs gl = g;
    DzFuse fz{&v, e.q_l, e.q_r, e.row0, t.q_first};
    gl.M = (int)cnt;
    gl.A = reinterpret_cast<const T*>(g.A) + (size_t)q0 * g.lda;
    gl.l = g.l + q0; gl.r = g.r + q0;
    const uint32_t n_rt = (cnt + 31) / 32;
    if (resident) {
      for (uint32_t rt = rank / n_ct; rt < n_rt; rt += G / n_ct)
        cell_small_tile<DT, DX_BWD, NW, RES>(gl, (int)rt, (int)(rank % n_ct), part, &rb, &fz);
    } else {
      for (uint32_t tile = rank; tile < n_rt * n_ct; tile += G)
        cell_small_tile<DT, DX_BWD, NW, 0>(gl, (int)(tile / n_ct), (int)(tile % n_ct), part,
                                           (const ResidentB<DX_BWD, 0>*)nullptr, &fz);
    }
    if (!die_barrier(sy, G, gen++, t.spin_ticks, &sh_ok)) return;
  }
}

// ---- numbering of the state rows by the sorted schedule ------------------------------------------
// Leaf i of the leaf log gets row i, the cell at position q of the level-sorted log row n_leaf + q;
// then every reference to a producing frame (children of the cells, roots, head rows, loss-term
// marks) is translated to rows once.
__global__ void k_number_rows(Engine e, uint32_t n_leaf, uint32_t n_cell) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_leaf + n_cell; i += gridDim.x * blockDim.x) {
    const uint32_t f = i < n_leaf ? e.leaf_row[i] : e.q_out[i - n_leaf];
    e.row_of[f] = i;
    if (e.node_of_row) e.node_of_row[i] = e.row_node[f];
  }
}
__global__ void k_translate_rows(Engine e, uint32_t n_cell, int has_head, int has_root) {
  const uint32_t n = n_cell > e.n_inst ? n_cell : e.n_inst;
  for (uint32_t q = blockIdx.x * blockDim.x + threadIdx.x; q < n; q += gridDim.x * blockDim.x) {
    if (q < n_cell) {
      e.q_l[q] = e.row_of[e.q_l[q]];
      e.q_r[q] = e.row_of[e.q_r[q]];
    }
    if (q < e.n_inst) {
      if (has_head) e.head_row[q] = e.row_of[e.head_row[q]];
      if (has_root) e.root_ref[q] = e.row_of[e.root_ref[q]];
    }
  }
}
// dz of the cells of the tail that have no parent: the roots, whose dh came from the head (or the caller)
template <int DT>
__global__ void k_dz_tail_roots(VecArgs v, Engine e, const uint32_t* root_rows, uint32_t q_first) {
  const uint32_t row = root_rows[blockIdx.x];
  if (row >= e.row0 && row - e.row0 >= q_first) dz_row<DT>(v, e, row - e.row0);
}

// Gradient-body firings counted on the device: the marks of all leaf and cell rows, summed, and the
// number of rows whose mark is not exactly one.  out[0] += sum, out[1] += rows fired other than once.
__global__ void k_count_grad(VecArgs v, Engine e, uint32_t n_leaf, uint32_t n_cell, unsigned long long* out) {
  unsigned long long sum = 0, odd = 0;
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_leaf + n_cell; i += gridDim.x * blockDim.x) {
    const uint32_t m = v.gmark[i];
    sum += m;
    odd += m != 1u;
  }
  for (int off = 32; off > 0; off >>= 1) {
    sum += __shfl_xor(sum, off);
    odd += __shfl_xor(odd, off);
  }
  if ((threadIdx.x & 63) == 0) {
    if (sum) atomicAdd(&out[0], sum);
    if (odd) atomicAdd(&out[1], odd);
  }
}

// ---- transposes feeding the weight-gradient GEMM (reduction over tags must be k-contiguous) -----
// out[c][q] = in_row(q)[c] for q < n_q, 0 for n_q <= q < q_stride.  GATHER: in_row(q) is
// [Hs[l[q]]; Hs[r[q]]], else row q of Dz.
template <int DT, bool GATHER>
__global__ void __launch_bounds__(256) k_transpose(VecArgs v, Engine e, uint32_t n_q, int n_cols, void* out_, float* col_sums) {
  typedef typename TypeOf<DT>::type T;
  constexpr int CH = El<T>::CH;          // elements per 16-byte chunk
  constexpr int TQ = 64, TC = 64;        // tile: 64 tags x 64 columns
  constexpr int CPR = TC / CH;           // chunks per tile row
  T* out = reinterpret_cast<T*>(out_);
  __shared__ T tile[TQ][TC + 2];
  const uint32_t q0 = blockIdx.x * TQ;
  const int c0 = blockIdx.y * TC;
  // in: 16 bytes per thread along the columns (rows of 128 B / 256 B, coalesced)
  for (int id = threadIdx.x; id < TQ * CPR; id += blockDim.x) {
    const int r = id / CPR, cc = (id % CPR) * CH;
    const uint32_t q = q0 + r;
    const int c = c0 + cc;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (q < n_q && c < n_cols) {
      if (GATHER) {
        const uint32_t row = c < v.Hp ? e.q_l[q] : e.q_r[q];
        raw = *reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(v.Hs) + (size_t)row * v.Hp + (c < v.Hp ? c : c - v.Hp));
      } else {
        raw = *reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(v.Dz) + (size_t)q * v.Np + c);
      }
    }
    const T* x = reinterpret_cast<const T*>(&raw);
#pragma unroll
    for (int i = 0; i < CH; ++i) tile[r][cc + i] = x[i];
  }
  __syncthreads();
  // column sums of the tile (db = sum over tags of Dz: one partial per 64 tags, summed in tag order)
  if (!GATHER && col_sums && threadIdx.x < TC && c0 + (int)threadIdx.x < n_cols) {
    float sum = 0.f;
    for (int r = 0; r < TQ; ++r) sum += to_f(tile[r][threadIdx.x]);
    col_sums[(size_t)blockIdx.x * v.Np + c0 + threadIdx.x] = sum;
  }
  // out: 16 bytes per thread along the tags
  constexpr int QPR = TQ / CH;           // chunks per output row
  for (int id = threadIdx.x; id < TC * QPR; id += blockDim.x) {
    const int c = id / QPR, qq = (id % QPR) * CH;
    if (c0 + c >= n_cols || q0 + qq >= v.q_stride) continue;
    u32x4 raw;
    T* x = reinterpret_cast<T*>(&raw);
#pragma unroll
    for (int i = 0; i < CH; ++i) x[i] = tile[qq + i][c];
    *reinterpret_cast<u32x4*>(out + (size_t)(c0 + c) * v.q_stride + q0 + qq) = raw;
  }
}

// ---- weight gradients without transposed copies (16-bit state) ------------------------------
// dW[n][k] = sum over the tags q of Dz[q][n] * X[q][k], X[q] = [h_l ; h_r] of cell q.  Both
// operands are stored with the reduction index q as the slow one, which is the wrong way round for
// an MFMA operand (a lane wants eight consecutive q of one n).  The LDS transpose load of CDNA4
// (ds_read_b64_tr_b16) turns a 4 x 16 block [q][n] into lanes-by-n with four q each, so the tiles
// go into LDS exactly as they lie in memory, Dz rows and gathered h rows, and the transposed copies
// and their kernels are not needed.  MFMA 16x16x32: lane l holds row (column) l % 16 and k = 8 (l /
// 16) .. + 7, i.e. two transpose loads; both operands use the same k order.  db[n] = sum_q Dz[q][n]
// rides along as a product with a block of ones in the workgroups of the first column tile.
// Tile 128 (n) x 128 (k) per workgroup, four waves as 2 x 2, 64 tags per LDS stage; the split of
// the reduction and its placement on the dies are those of k_gemm<DW_SPLIT>.
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
constexpr int DWT = 128;        // tile edge
constexpr int DWQ = 64;         // tags per stage
constexpr int DWLD = DWT + 16;  // LDS row stride in elements: rows 288 bytes apart

// One MFMA operand from a tile stored as it lies in memory ([tag][column], DWLD elements per row), read
// transposed: `p` is the lane's own place in the block [8 g .. 8 g + 7][16 columns] (g = lane / 16; source
// lane s of a group points at tag 8 g + 4 t + s / 4, columns 4 (s % 4) .. + 3, and receives column s of
// the tags 8 g + 4 t + 0 .. 3), the same for every block of the tile up to a constant offset.
__device__ __forceinline__ bf16x8 tr_frag(const __bf16* p) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 4 * DWLD));
  s16x8 v;
  v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
  v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
  return __builtin_bit_cast(bf16x8, v);
}

struct DwArgs {
  const __bf16* Dz;      // [n_q][Np]
  const __bf16* Hs;      // state rows
  const uint32_t *q_l, *q_r;
  uint32_t n_q;
  int Np, Kp, Hp;
  int k_per_split, n_splits, n_tiles_n;
  float* dW_part;        // [splits][Np][Kp]
  float* db_part;        // [splits][Np]
};

__global__ void __launch_bounds__(256, 3) k_dw_direct(DwArgs g) {
  __shared__ __attribute__((aligned(16))) __bf16 sA[DWQ * DWLD];
  __shared__ __attribute__((aligned(16))) __bf16 sB[DWQ * DWLD];
  const int n_mt = (g.Np + DWT - 1) / DWT;
  const int xcd = blockIdx.x & 7, u = blockIdx.x >> 3;
  const int tiles = n_mt * g.n_tiles_n;
  const int split = (u / tiles) * 8 + xcd;
  if (split >= g.n_splits) return;
  const int mt = (u % tiles) / g.n_tiles_n, nt = (u % tiles) % g.n_tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const uint32_t q_begin = (uint32_t)split * (uint32_t)g.k_per_split;
  const uint32_t q_end = min(g.n_q, q_begin + (uint32_t)g.k_per_split);

  // This thread's four 16-byte chunks of each tile: rows r0 + 16 c, chunk column ch.  A chunk whose
  // columns lie beyond the matrix reads the last valid columns instead (its products are never stored),
  // so the loads of a whole stage need no predicate; only the last, partial stage of a split checks
  // its tags.  The addresses advance by one stage per pass (no multiplication per chunk).
  const int r0 = tid >> 4, ch = (tid & 15) * 8;
  // Rows are 72 banks apart, so the rows of two neighbouring groups of 16 lanes (8 tags apart) would start
  // in the same bank: the tile is stored with column bit 6 flipped in every other block of eight tags, which
  // sends those groups to different halves of the banks.  A wave's 64 columns keep to one half of the tile's
  // 128, so the flip is part of the lane's base address and costs the reads nothing.
  const int ch_lds = ch ^ (((r0 >> 3) & 1) << 6);
  const int fg = lane >> 4, fs = lane & 15;
  const __bf16* const a_lane = sA + (8 * fg + (fs >> 2)) * DWLD + 4 * (fs & 3) + (((wm ^ fg) & 1) << 6);
  const __bf16* const b_lane = sB + (8 * fg + (fs >> 2)) * DWLD + 4 * (fs & 3) + (((wn ^ fg) & 1) << 6);
  const int a_col = min(mt * DWT + ch, g.Np - 8), b_col = min(nt * DWT + ch, g.Kp - 8);
  const bool b_left = b_col < g.Hp;
  const uint32_t b_off = (uint32_t)(b_left ? b_col : b_col - g.Hp);
  const uint32_t* const b_rows = b_left ? g.q_l : g.q_r;
  u32x4 ra[4], rb[4];
  uint32_t row_next[4];   // gathered rows of the stage after the one in ra / rb
  const __bf16* pa = g.Dz + (size_t)(q_begin + r0) * g.Np + a_col;   // chunk c = 0 of the stage to be loaded next
  const size_t a_step = (size_t)16 * g.Np;
  auto load_rows = [&](uint32_t q0, bool full) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t q = q0 + r0 + 16 * c;
      row_next[c] = (full || q < q_end) ? b_rows[q] : 0u;
    }
  };
  auto load_tile = [&](uint32_t q0, bool full) {   // uses row_next, which must hold the rows of q0
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t q = q0 + r0 + 16 * c;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const uint32_t hs_off = row_next[c] * (uint32_t)g.Hp + b_off;   // (rows x Hp stays below 2^32: the host checks)
      if (full) {
        ra[c] = *reinterpret_cast<const u32x4*>(pa + c * a_step);
        rb[c] = *reinterpret_cast<const u32x4*>(g.Hs + hs_off);
      } else {
        ra[c] = q < q_end ? *reinterpret_cast<const u32x4*>(pa + c * a_step) : zero;
        rb[c] = q < q_end ? *reinterpret_cast<const u32x4*>(g.Hs + hs_off) : zero;
      }
    }
    pa += 4 * a_step;
  };

  f32x4 acc[4][4], accdb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    accdb[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  s16x8 ones_bits;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones_bits[i] = (short)0x3F80;   // bf16 1.0
  const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
  const bool with_db = nt == 0 && wn == 0;

  // a stage is full if all its DWQ tags belong to the split (uniform for the workgroup)
  auto is_full = [&](uint32_t q0) { return q0 + DWQ <= q_end; };
  if (q_begin < q_end) {
    load_rows(q_begin, is_full(q_begin));
    load_tile(q_begin, is_full(q_begin));
    if (q_begin + DWQ < q_end) load_rows(q_begin + DWQ, is_full(q_begin + DWQ));
  }
  for (uint32_t q0 = q_begin; q0 < q_end; q0 += DWQ) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      *reinterpret_cast<u32x4*>(sA + (r0 + 16 * c) * DWLD + ch_lds) = ra[c];
      *reinterpret_cast<u32x4*>(sB + (r0 + 16 * c) * DWLD + ch_lds) = rb[c];
    }
    __syncthreads();
    if (q0 + DWQ < q_end) {
      load_tile(q0 + DWQ, is_full(q0 + DWQ));
      if (q0 + 2 * DWQ < q_end) load_rows(q0 + 2 * DWQ, is_full(q0 + 2 * DWQ));
    }
#pragma unroll
    for (int ks = 0; ks < DWQ / 32; ++ks) {
      bf16x8 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = tr_frag(a_lane + ks * 32 * DWLD + i * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[j] = tr_frag(b_lane + ks * 32 * DWLD + j * 16);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        if (with_db) accdb[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], ones, accdb[i], 0, 0, 0);
      }
    }
    __syncthreads();
  }
  // acc[i][j][r]: n = 4 (lane / 16) + r of block i, k = lane % 16 of block j
  float* C = g.dW_part + (size_t)split * g.Np * g.Kp;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n = mt * DWT + wm * 64 + i * 16 + 4 * (lane >> 4) + r;
      if (n >= g.Np) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = nt * DWT + wn * 64 + j * 16 + (lane & 15);
        if (k < g.Kp) C[(size_t)n * g.Kp + k] = acc[i][j][r];
      }
      if (with_db && (lane & 15) == 0) g.db_part[(size_t)split * g.Np + n] = accdb[i][r];
    }
}

// dW[n][k] = sum over splits, in split order; written in the caller's unpadded layout
__global__ void k_reduce_dw(VecArgs v, float* dW, int splits) {
  const int R = v.N, K2 = 2 * v.H;
  for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < R * K2; idx += gridDim.x * blockDim.x) {
    const int n = idx / K2, k = idx % K2;
    const int np = (n / v.H) * v.Hp + n % v.H, kp = (k / v.H) * v.Hp + k % v.H;
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += v.dW_part[((size_t)z * v.Np + np) * v.Kp + kp];
    dW[idx] = s;
  }
}

// db[n] = sum_q Dz[q][n]: partial sums over 64 tags each come from the transpose of Dz.  First
// every run of DB_RUN partials is summed into its first row (64 columns per block, rows of 256
// bytes, four groups of rows that meet in LDS in a fixed order), then the rows left are summed.
constexpr int DB_RUN = 64;
__global__ void __launch_bounds__(256) k_db_runs(VecArgs v, float* part, int n_parts) {
  __shared__ float red[4][64];
  const int c = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int np = blockIdx.x * 64 + c;
  const int p0 = blockIdx.y * DB_RUN, p1 = min(n_parts, p0 + DB_RUN);
  float s = 0.f;
  if (np < v.Np)
    for (int p = p0 + grp; p < p1; p += 4) s += part[(size_t)p * v.Np + np];
  red[grp][c] = s;
  __syncthreads();   // every row of the run has been read before its first row is overwritten
  if (grp == 0 && np < v.Np) part[(size_t)p0 * v.Np + np] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
}
// 16 columns per block; 16 groups of partials (every `stride`-th row), each summed in order, meet in LDS
__global__ void k_db_final(VecArgs v, const float* part, int n_parts, int stride, float* db) {
  __shared__ float red[16][17];
  const int c = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int np = blockIdx.x * 16 + c;
  float s = 0.f;
  if (np < v.Np)
    for (int p = grp; p < n_parts; p += 16) s += part[(size_t)p * stride * v.Np + np];
  red[grp][c] = s;
  __syncthreads();
  if (grp == 0 && np < v.Np) {
    float t = 0.f;
    for (int g2 = 0; g2 < 16; ++g2) t += red[g2][c];
    const int gate = np / v.Hp, j = np % v.Hp;
    if (j < v.H) db[gate * v.H + j] = t;
  }
}

// ---- embedding gradient: leaves grouped by token, segments summed without atomics ---------------
__global__ void k_tok_hist(Engine e, uint32_t n_leaf, uint32_t* count, int vocab) {
  for (uint32_t base = blockIdx.x * blockDim.x; base < n_leaf; base += gridDim.x * blockDim.x) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t t = i < n_leaf ? e.leaf_tok[i] : 0xFFFFFFFFu;
    (void)wave_alloc_keyed(t < (uint32_t)vocab, t, count);
  }
}
// single block: exclusive scans of the per-token leaf counts and chunk counts
__global__ void __launch_bounds__(1024) k_tok_scan(const uint32_t* count, uint32_t* seg_off, uint32_t* chunk_off, int vocab,
                                                   uint32_t chunk) {
  // entries 0 .. vocab (one past the end holds the totals); every thread owns a run of consecutive
  // entries, the runs' sums are scanned over the block (waves by shuffles, wave totals in LDS)
  __shared__ uint32_t wsum[2][16];
  const int per = (vocab + 1 + 1023) / 1024;
  const int lo = threadIdx.x * per, hi = min(lo + per, vocab + 1);
  uint32_t sa = 0, sb = 0;
  for (int i = lo; i < hi; ++i) {
    const uint32_t a = i < vocab ? count[i] : 0;
    sa += a;
    sb += (a + chunk - 1) / chunk;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t ia = sa, ib = sb;   // inclusive scan inside the wave
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t ta = __shfl_up(ia, off), tb = __shfl_up(ib, off);
    if (lane >= off) {
      ia += ta;
      ib += tb;
    }
  }
  if (lane == 63) {
    wsum[0][wave] = ia;
    wsum[1][wave] = ib;
  }
  __syncthreads();
  uint32_t ba = ia - sa, bb = ib - sb;   // exclusive prefix of this thread's run
  for (int w = 0; w < wave; ++w) {
    ba += wsum[0][w];
    bb += wsum[1][w];
  }
  for (int i = lo; i < hi; ++i) {
    const uint32_t a = i < vocab ? count[i] : 0;
    seg_off[i] = ba;
    chunk_off[i] = bb;
    ba += a;
    bb += (a + chunk - 1) / chunk;
  }
}
__global__ void k_tok_scatter(Engine e, uint32_t n_leaf, const uint32_t* seg_off, uint32_t* fill,
                              uint32_t* sorted_row, int vocab) {
  for (uint32_t base = blockIdx.x * blockDim.x; base < n_leaf; base += gridDim.x * blockDim.x) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t t = i < n_leaf ? e.leaf_tok[i] : 0xFFFFFFFFu;
    const bool on = t < (uint32_t)vocab;
    const uint32_t rank = wave_alloc_keyed(on, t, fill);
    if (on) sorted_row[seg_off[t] + rank] = i;   // leaf i has row i
  }
}
struct TokenSink {   // leaf rows grouped by token (leaf i has row i)
  uint32_t* sorted_row;
  __device__ void operator()(uint32_t i, uint32_t pos) const { sorted_row[pos] = i; }
};
// one wave per chunk of at most `chunk` leaves of one token: partial[chunk] = sum of their dH rows
__global__ void k_de_partial(VecArgs v, const uint32_t* seg_off, const uint32_t* chunk_off,
                             const uint32_t* sorted_row, uint32_t chunk, float* part) {
  const uint32_t n_chunks = chunk_off[v.vocab];
  const uint32_t wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  const uint32_t n_waves = (gridDim.x * blockDim.x) >> 6;
  for (uint32_t c = wave; c < n_chunks; c += n_waves) {
    // token owning chunk c: the last t with chunk_off[t] <= c
    uint32_t lo = 0, hi = (uint32_t)v.vocab;
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (chunk_off[mid] <= c) lo = mid; else hi = mid;
    }
    const uint32_t p_lo = seg_off[lo] + (c - chunk_off[lo]) * chunk;
    const uint32_t p_hi = min(seg_off[lo + 1], p_lo + chunk);
    for (int n = lane * 4; n < v.Hp; n += 256) {
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      for (uint32_t p = p_lo; p < p_hi; p += 8) {   // eight rows in flight, added in leaf order
        uint32_t row[8];
        float4 x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) row[j] = sorted_row[min(p + j, p_hi - 1)];
        if (n == 0)   // (lane 0, first column group) the gradient body of a leaf's tag is its term of dE
          for (int j = 0; j < 8; ++j)
            if (p + j < p_hi) atomicAdd(&v.gmark[row[j]], 1u);
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = *reinterpret_cast<const float4*>(v.dH + (size_t)row[j] * v.Hp + n);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (p + j < p_hi) {
            s.x += x[j].x; s.y += x[j].y; s.z += x[j].z; s.w += x[j].w;
          }
        if (v.dHn) {   // the leaves' own loss terms
#pragma unroll
          for (int j = 0; j < 8; ++j) x[j] = *reinterpret_cast<const float4*>(v.dHn + (size_t)row[j] * v.Hp + n);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (p + j < p_hi) {
              s.x += x[j].x; s.y += x[j].y; s.z += x[j].z; s.w += x[j].w;
            }
        }
      }
      *reinterpret_cast<float4*>(part + (size_t)c * v.Hp + n) = s;
    }
  }
}
// one wave per token: the token's chunk sums, added in chunk order; rows of tokens without a
// leaf are written as zeros
__global__ void __launch_bounds__(256) k_de_final(VecArgs v, const uint32_t* chunk_off, const float* part, float* dE) {
  const int tok = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (tok >= v.vocab) return;
  const uint32_t c_lo = chunk_off[tok], c_hi = chunk_off[tok + 1];
  if ((v.H & 3) == 0) {
    for (int n = lane * 4; n < v.H; n += 256) {
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      for (uint32_t c = c_lo; c < c_hi; ++c) {
        const float4 x = *reinterpret_cast<const float4*>(part + (size_t)c * v.Hp + n);
        s.x += x.x; s.y += x.y; s.z += x.z; s.w += x.w;
      }
      *reinterpret_cast<float4*>(dE + (size_t)tok * v.H + n) = s;
    }
  } else {
    for (int n = lane; n < v.H; n += 64) {
      float s = 0.f;
      for (uint32_t c = c_lo; c < c_hi; ++c) s += part[(size_t)c * v.Hp + n];
      dE[(size_t)tok * v.H + n] = s;
    }
  }
}

}  // namespace

// ---- host entry points used by eval.hip ------------------------------------------------------
template <typename T> static void pack_w_t(const VecArgs& v, hipStream_t s) {
  hipLaunchKernelGGL(k_pack_w<DtOf<T>::value>, dim3(1024), dim3(256), 0, s, v);
}
void vec_pack_w(const VecArgs& v, hipStream_t s) {
  if (v.dtype == TDF_BF16) pack_w_t<__bf16>(v, s); else pack_w_t<float>(v, s);
}

void vec_embed(const VecArgs& v, const Engine& e, uint32_t n_leaf, hipStream_t s) {
  if (!n_leaf) return;
  const int epc = v.dtype == TDF_BF16 ? 8 : 4;
  int lpl = 1;   // lanes per leaf: the row's 16-byte chunks rounded up to a power of two, at most 64
  while (lpl < 64 && lpl * epc < v.Hp) lpl *= 2;
  const uint32_t per_block = 256u / (uint32_t)lpl;
  // at least 8192 threads, so that the first Hp of them can clear row 0 of Cs
  const int blocks = (int)std::min<uint32_t>(std::max<uint32_t>((n_leaf + per_block - 1) / per_block, 32u), 8192u);
  if (v.dtype == TDF_BF16) hipLaunchKernelGGL(k_embed<TDF_BF16>, dim3(blocks), dim3(256), 0, s, v, e, n_leaf, lpl);
  else hipLaunchKernelGGL(k_embed<TDF_F32>, dim3(blocks), dim3(256), 0, s, v, e, n_leaf, lpl);
}

template <typename T> static void cell_fwd_t(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count,
                                             int save_gates, hipStream_t s) {
  GemmArgs g{};
  g.M = (int)count; g.N = v.Np; g.K = v.Kp;
  g.B = v.Wp; g.ldb = v.Kp; g.Bf = v.Wf;
  g.Hs = v.Hs; g.Hp = v.Hp;
  g.out0 = e.row0 + q0; g.l = e.q_l + q0; g.r = e.q_r + q0;
  g.bias = v.bp; g.Hs_out = v.Hs; g.Cs = v.Cs; g.leaf_rows = e.row0;
  g.gates = v.gates ? reinterpret_cast<T*>(v.gates) + (size_t)q0 * v.Np : nullptr;
  g.ldg = v.Np; g.save_gates = save_gates && v.gates;
  g.narrow = !v.wide_offsets && (uint64_t)(e.row0 + q0 + count) * (uint64_t)v.Hp * 4u < (1ull << 32) &&
             (uint64_t)count * (uint64_t)v.Np * sizeof(T) < (1ull << 32);
  if (count <= small_level()) {
    if (v.cell_kind == 2) launch_cell_small<T, LSTM_FWD>(g, v.Hp / 32, s);
    else launch_cell_small<T, RNN_FWD>(g, v.Hp / 32, s);
  } else if (v.cell_kind == 2) {
    launch_gemm<T, LSTM_FWD>(g, (v.Hp / 32 + 1) / 2, 1, s);
  } else {
    launch_gemm<T, RNN_FWD>(g, (v.Np + 127) / 128, 1, s);
  }
}
void vec_cell_fwd(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count, int save_gates, hipStream_t s) {
  if (v.dtype == TDF_BF16) cell_fwd_t<__bf16>(v, e, q0, count, save_gates, s);
  else cell_fwd_t<float>(v, e, q0, count, save_gates, s);
}

template <typename T> static void cell_bwd_t(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count, hipStream_t s) {
  if (!count) return;
  const int per_block = 256 / std::min(256, v.Hp / 4);
  hipLaunchKernelGGL(k_dz<DtOf<T>::value>, dim3((count + per_block - 1) / per_block), dim3(256), 0, s, v, e, q0, count);
  GemmArgs g{};
  g.M = (int)count; g.N = v.Kp; g.K = v.Np;
  g.A = reinterpret_cast<const T*>(v.Dz) + (size_t)q0 * v.Np; g.lda = v.Np;
  g.B = v.WpT; g.ldb = v.Np; g.Bf = v.WfT;
  g.Hp = v.Hp; g.l = e.q_l + q0; g.r = e.q_r + q0;
  g.C = v.dH;
  if (count <= small_level()) launch_cell_small<T, DX_BWD>(g, v.Kp / 32, s);
  else launch_gemm<T, DX_BWD>(g, (v.Kp + 127) / 128, 1, s);
}
void vec_cell_bwd(const VecArgs& v, const Engine& e, uint32_t q0, uint32_t count, hipStream_t s) {
  if (v.dtype == TDF_BF16) cell_bwd_t<__bf16>(v, e, q0, count, s); else cell_bwd_t<float>(v, e, q0, count, s);
}

uint32_t vec_small_level() { return small_level(); }

// The levels lvl_first .. lvl_last in one launch, every die walking its own cells (k_tail_fwd).
// level_off: device array of first cells by sort key; sync: eight zeroed DieSync records.
template <typename T> static void tail_fwd_t(const VecArgs& v, const Engine& e, const TailArgs& t, int per_die, int save_gates,
                                             hipStream_t s) {
  GemmArgs g{};
  g.N = v.Np; g.K = v.Kp;
  g.B = v.Wp; g.ldb = v.Kp; g.Bf = v.Wf;
  g.Hs = v.Hs; g.Hp = v.Hp;
  g.out0 = e.row0; g.l = e.q_l; g.r = e.q_r;
  g.bias = v.bp; g.Hs_out = v.Hs; g.Cs = v.Cs; g.leaf_rows = e.row0;
  g.gates = v.gates; g.ldg = v.Np; g.save_gates = save_gates && v.gates;
  g.n_tiles_n = v.Hp / 32;
  const int grid = std::max(per_die, 1) * (int)XCDS;
  if (v.cell_kind == 2) {
    const size_t lds = (size_t)4 * 5 * 16 * 64 * sizeof(float);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tail_fwd<DtOf<T>::value, LSTM_FWD, 4>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL((k_tail_fwd<DtOf<T>::value, LSTM_FWD, 4>), dim3(grid), dim3(256), lds, s, g, t);
  } else if (small_tile_waves<T, RNN_FWD>(g.K) == 8) {
    const size_t lds = (size_t)8 * 16 * 64 * sizeof(float);
    hipLaunchKernelGGL((k_tail_fwd<DtOf<T>::value, RNN_FWD, 8>), dim3(grid), dim3(512), lds, s, g, t);
  } else {
    const size_t lds = (size_t)4 * 16 * 64 * sizeof(float);
    hipLaunchKernelGGL((k_tail_fwd<DtOf<T>::value, RNN_FWD, 4>), dim3(grid), dim3(256), lds, s, g, t);
  }
}
// per_die: workgroups per accelerator die (all of one launch must be resident together)
void vec_tail_fwd(const VecArgs& v, const Engine& e, const uint32_t* level_off, uint32_t lvl_first, uint32_t lvl_last,
                  uint32_t n_dies, void* sync, long long spin_ticks, int per_die, int save_gates, hipStream_t s) {
  TailArgs t{level_off, lvl_first, lvl_last, n_dies, (DieSync*)sync, spin_ticks};
  if (v.dtype == TDF_BF16) tail_fwd_t<__bf16>(v, e, t, per_die, save_gates, s); else tail_fwd_t<float>(v, e, t, per_die, save_gates, s);
}

template <typename T> static void tail_bwd_t(const VecArgs& v, const Engine& e, const TailArgs& t, int per_die, hipStream_t s) {
  GemmArgs g{};
  g.N = v.Kp; g.K = v.Np;
  g.A = v.Dz; g.lda = v.Np;
  g.B = v.WpT; g.ldb = v.Np; g.Bf = v.WfT;
  g.Hp = v.Hp; g.l = e.q_l; g.r = e.q_r;
  g.C = v.dH;
  g.n_tiles_n = v.Kp / 32;
  const int grid = std::max(per_die, 1) * (int)XCDS;
  if (small_tile_waves<T, DX_BWD>(g.K) == 8) {
    const size_t lds = (size_t)8 * 16 * 64 * sizeof(float);
    hipLaunchKernelGGL((k_tail_bwd<DtOf<T>::value, 8>), dim3(grid), dim3(512), lds, s, g, v, e, t);
  } else {
    const size_t lds = (size_t)4 * 16 * 64 * sizeof(float);
    hipLaunchKernelGGL((k_tail_bwd<DtOf<T>::value, 4>), dim3(grid), dim3(256), lds, s, g, v, e, t);
  }
}
// After the level sort: rows numbered by the sorted schedule, references translated.
void vec_number_rows(const Engine& e, uint32_t n_leaf, uint32_t n_cell, int has_head, int has_root, hipStream_t s) {
  const int g1 = (int)std::min<uint32_t>((n_leaf + n_cell + 255) / 256, 2048u);
  hipLaunchKernelGGL(k_number_rows, dim3(std::max(g1, 1)), dim3(256), 0, s, e, n_leaf, n_cell);
  const int g2 = (int)std::min<uint32_t>((std::max(n_cell, e.n_inst) + 255) / 256, 2048u);
  hipLaunchKernelGGL(k_translate_rows, dim3(std::max(g2, 1)), dim3(256), 0, s, e, n_cell, has_head, has_root);
}

void vec_tail_bwd(const VecArgs& v, const Engine& e, const uint32_t* level_off, uint32_t lvl_first, uint32_t lvl_last,
                  uint32_t n_dies, void* sync, long long spin_ticks, int per_die, uint32_t q_first, const uint32_t* root_rows,
                  hipStream_t s) {
  TailArgs t{level_off, lvl_first, lvl_last, n_dies, (DieSync*)sync, spin_ticks, q_first};
  if (v.dtype == TDF_BF16) hipLaunchKernelGGL(k_dz_tail_roots<TDF_BF16>, dim3(e.n_inst), dim3(256), 0, s, v, e, root_rows, q_first);
  else hipLaunchKernelGGL(k_dz_tail_roots<TDF_F32>, dim3(e.n_inst), dim3(256), 0, s, v, e, root_rows, q_first);
  if (v.dtype == TDF_BF16) tail_bwd_t<__bf16>(v, e, t, per_die, s); else tail_bwd_t<float>(v, e, t, per_die, s);
}

// cls < 0: every instance; else only the instances of that class (Engine::inst_class)
void vec_head(const VecArgs& v, const Engine& e, const float* dy, int with_grad, int cls, hipStream_t s) {
  int blocks = ((int)e.n_inst + 3) / 4;
  if (v.dtype == TDF_BF16) hipLaunchKernelGGL(k_head<TDF_BF16>, dim3(blocks), dim3(256), 0, s, v, e, dy, with_grad, cls);
  else hipLaunchKernelGGL(k_head<TDF_F32>, dim3(blocks), dim3(256), 0, s, v, e, dy, with_grad, cls);
}
void vec_node_loss(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t n_cell, const int32_t* node_label,
                   float* out_node_loss, const float* dnode, int with_grad, hipStream_t s) {
  const uint32_t rows = n_leaf + n_cell;
  if (!rows) return;
  const int blocks = (int)std::min<uint32_t>((rows + 15) / 16, 2048u);
  const size_t u_bytes = (size_t)v.n_classes * v.Hp * sizeof(float);
  const int u_in_lds = u_bytes <= 48 * 1024;
  const size_t lds = u_in_lds ? u_bytes : 0;
  if (v.dtype == TDF_BF16)
    hipLaunchKernelGGL(k_node_ce<TDF_BF16>, dim3(blocks), dim3(256), lds, s, v, e, n_leaf, n_cell, node_label, out_node_loss, dnode,
                       with_grad, u_in_lds);
  else
    hipLaunchKernelGGL(k_node_ce<TDF_F32>, dim3(blocks), dim3(256), lds, s, v, e, n_leaf, n_cell, node_label, out_node_loss, dnode,
                       with_grad, u_in_lds);
}
void vec_count_grad(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t n_cell, unsigned long long* out, hipStream_t s) {
  const uint32_t n = n_leaf + n_cell;
  if (!n) return;
  hipLaunchKernelGGL(k_count_grad, dim3(std::min<uint32_t>((n + 255) / 256, 1024u)), dim3(256), 0, s, v, e, n_leaf, n_cell, out);
}
void vec_seed_dy(const VecArgs& v, const Engine& e, const float* dy, hipStream_t s) {
  hipLaunchKernelGGL(k_seed_dy, dim3(e.n_inst), dim3(128), 0, s, v, e, dy);
}
void vec_out_rows(const VecArgs& v, const Engine& e, float* out_h, float* out_c, hipStream_t s) {
  if (v.dtype == TDF_BF16) hipLaunchKernelGGL(k_out_rows<TDF_BF16>, dim3(e.n_inst), dim3(128), 0, s, v, e, out_h, out_c);
  else hipLaunchKernelGGL(k_out_rows<TDF_F32>, dim3(e.n_inst), dim3(128), 0, s, v, e, out_h, out_c);
}

// Splits of the reduction over the tags in the weight-gradient GEMM: enough for about 640
// workgroups, at least 1024 tags each, at most 64 (every split writes a partial dW that the
// ordered reduction reads again).
int vec_dw_splits(uint32_t q_stride, int Np, int Kp) {
  const int tiles = ((Np + BM_FULL - 1) / BM_FULL) * ((Kp + 127) / 128);
  const int want = (640 + tiles - 1) / tiles;
  const int most = (int)std::min<uint32_t>(64u, q_stride / 1024u);
  return std::max(1, std::min(want, most));
}

static void weight_grads_direct(const VecArgs& v, const Engine& e, uint32_t n_q, float* dW, float* db, float* db_part,
                                hipStream_t s) {
  const int splits = vec_dw_splits(v.q_stride, v.Np, v.Kp);
  DwArgs g{};
  g.Dz = reinterpret_cast<const __bf16*>(v.Dz);
  g.Hs = reinterpret_cast<const __bf16*>(v.Hs);
  g.q_l = e.q_l; g.q_r = e.q_r;
  g.n_q = n_q;
  g.Np = v.Np; g.Kp = v.Kp; g.Hp = v.Hp;
  g.k_per_split = (int)((v.q_stride / 64 + splits - 1) / splits) * 64;
  g.n_splits = splits;
  g.n_tiles_n = (v.Kp + DWT - 1) / DWT;
  g.dW_part = v.dW_part;
  g.db_part = db_part;
  const int n_mt = (v.Np + DWT - 1) / DWT;
  hipLaunchKernelGGL(k_dw_direct, dim3(8 * n_mt * g.n_tiles_n * ((splits + 7) / 8)), dim3(256), 0, s, g);
  hipLaunchKernelGGL(k_reduce_dw, dim3(512), dim3(256), 0, s, v, dW, splits);
  hipLaunchKernelGGL(k_db_final, dim3((v.Np + 15) / 16), dim3(256), 0, s, v, db_part, splits, 1, db);
}

template <typename T> static void weight_grads_t(const VecArgs& v, const Engine& e, uint32_t n_q, float* dW, float* db,
                                                 float* db_part, hipStream_t s) {
  // transposed copies so that the reduction over tags is k-contiguous for both operands
  dim3 tb(256);
  hipLaunchKernelGGL((k_transpose<DtOf<T>::value, false>), dim3(v.q_stride / 64, v.Np / 64), tb, 0, s, v, e, n_q, v.Np,
                     v.DzT, db_part);
  hipLaunchKernelGGL((k_transpose<DtOf<T>::value, true>), dim3(v.q_stride / 64, v.Kp / 64), tb, 0, s, v, e, n_q, v.Kp,
                     v.XT, (float*)nullptr);
  const int splits = vec_dw_splits(v.q_stride, v.Np, v.Kp);
  int kps = (int)((v.q_stride / 64 + splits - 1) / splits) * 64;
  GemmArgs g{};
  g.M = v.Np; g.N = v.Kp; g.K = (int)v.q_stride;
  g.A = v.DzT; g.lda = v.q_stride;
  g.B = v.XT; g.ldb = v.q_stride;
  g.C = v.dW_part; g.ldc = v.Kp;
  g.k_per_split = kps;
  launch_gemm<T, DW_SPLIT>(g, (v.Kp + 127) / 128, splits, s);
  hipLaunchKernelGGL(k_reduce_dw, dim3(512), dim3(256), 0, s, v, dW, splits);
  const int parts = (int)(v.q_stride / 64);   // written by the transpose of Dz above
  hipLaunchKernelGGL(k_db_runs, dim3((v.Np + 63) / 64, (parts + DB_RUN - 1) / DB_RUN), dim3(256), 0, s, v, db_part, parts);
  hipLaunchKernelGGL(k_db_final, dim3((v.Np + 15) / 16), dim3(256), 0, s, v, db_part, (parts + DB_RUN - 1) / DB_RUN, DB_RUN, db);
}
// 16-bit state: operands as they lie in memory, transposed by the LDS transpose loads; fp32 (which has
// no such load): transposed copies first.
void vec_weight_grads(const VecArgs& v, const Engine& e, uint32_t n_q, float* dW, float* db, float* db_part, hipStream_t s) {
  if (v.dtype == TDF_BF16) weight_grads_direct(v, e, n_q, dW, db, db_part, s);
  else weight_grads_t<float>(v, e, n_q, dW, db, db_part, s);
}

// The embedding gradient in two steps.  vec_embed_sort orders the leaves by token (a counting
// sort of the leaf log): it needs the leaf log only, so it can run beside the cells.  vec_embed_sums
// adds the leaves' state gradients token by token in that order, once the gradient pass is done.
void vec_embed_sort(const VecArgs& v, const Engine& e, uint32_t n_leaf, uint32_t* count, uint32_t* seg_off,
                    uint32_t* chunk_off, uint32_t* fill, uint32_t* sorted_row, uint32_t chunk, hipStream_t s) {
  int g = (int)std::min<uint32_t>((n_leaf + 255) / 256, 2048u);
  if (g < 1) g = 1;
  if (bucket_fits((uint32_t)v.vocab)) {
    const uint32_t n_keys = (uint32_t)v.vocab;
    const size_t lds = (size_t)n_keys * 4;
    bucket_lds_opt_in(reinterpret_cast<const void*>(&k_bucket_count), n_keys);
    bucket_lds_opt_in(reinterpret_cast<const void*>(&k_bucket_place<TokenSink>), n_keys);
    hipLaunchKernelGGL(k_bucket_count, dim3(BUCKET_BLOCKS), dim3(BUCKET_THREADS), lds, s, e.leaf_tok, n_leaf, n_keys, count);
    hipLaunchKernelGGL(k_tok_scan, dim3(1), dim3(1024), 0, s, count, seg_off, chunk_off, v.vocab, chunk);
    hipLaunchKernelGGL(k_bucket_place<TokenSink>, dim3(BUCKET_BLOCKS), dim3(BUCKET_THREADS), lds, s, e.leaf_tok, n_leaf, n_keys,
                       seg_off, fill, TokenSink{sorted_row});
  } else {
    hipLaunchKernelGGL(k_tok_hist, dim3(g), dim3(256), 0, s, e, n_leaf, count, v.vocab);
    hipLaunchKernelGGL(k_tok_scan, dim3(1), dim3(1024), 0, s, count, seg_off, chunk_off, v.vocab, chunk);
    hipLaunchKernelGGL(k_tok_scatter, dim3(g), dim3(256), 0, s, e, n_leaf, seg_off, fill, sorted_row, v.vocab);
  }
}
void vec_embed_sums(const VecArgs& v, uint32_t n_leaf, const uint32_t* seg_off, const uint32_t* chunk_off,
                    const uint32_t* sorted_row, float* part, float* dE, uint32_t chunk, hipStream_t s) {
  const uint32_t max_chunks = n_leaf / chunk + std::min<uint32_t>((uint32_t)v.vocab, n_leaf) + 1;
  hipLaunchKernelGGL(k_de_partial, dim3(std::min<uint32_t>((max_chunks + 3) / 4, 16384u)), dim3(256), 0, s, v, seg_off,
                     chunk_off, sorted_row, chunk, part);
  hipLaunchKernelGGL(k_de_final, dim3((v.vocab + 3) / 4), dim3(256), 0, s, v, chunk_off, part, dE);
}

}  // namespace tdf
