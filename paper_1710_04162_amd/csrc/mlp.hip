// The sliced gradient function (Sec. 3.3 step 1 evaluated as Sec. 3.2 / 5.1
// describe) for a ReLU MLP with softmax cross-entropy.
//
// One call covers every worker and every slice.  The parameters are read-only
// for the whole call, so all slices see the same values (Sec. 5.1).  A slice's
// rows carry the weight that the aggregation op gives that slice, so the
// accumulators of the dW GEMM, which run over a worker's rows in slice order,
// ARE the in-place aggregation of the slice results; each worker's gradient is
// written once, to that worker's own flat array.
//
// Dense contractions run on the matrix cores (MFMA 32x32x16 bf16 or 32x32x2
// fp32, fp32 accumulators), staged through LDS:
//   forward   H_l   = act(H_{l-1} W_l + b_l)         per worker rows
//   dX        dZ_{l-1} = (dZ_l W_l^T) * [H_{l-1} > 0]  per worker rows
//   dW        dW_l = H_{l-1}^T dZ_l , db_l = colsum(dZ_l)  per worker
// Every operand is used in the layout it has in memory; an operand whose
// contraction index is strided in memory is transposed on its way into LDS.
#include <math.h>

#include "common.h"

namespace synk {

typedef uint16_t bf16_t;                                       // raw bfloat16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));     // MFMA operand type

constexpr int kMBlock = 256;   // 4 wavefronts, arranged 2 x 2 over the tile

enum GemmMode { MODE_FWD = 0, MODE_DX = 1, MODE_DW = 2 };
enum OperandLayout { KC = 0 /* contraction index contiguous */, XC = 1 /* row/col index contiguous */ };

template <typename T> struct ET;
template <> struct ET<float> {
  static constexpr int V = 4;    // elements per 16-byte vector
  static constexpr int KM = 2;   // contraction depth of one MFMA
  static constexpr int BK = 16;  // contraction depth of one LDS tile
};
template <> struct ET<bf16_t> {
  static constexpr int V = 8;
  static constexpr int KM = 16;
  static constexpr int BK = 32;
};

// LDS footprint of one operand tile, in 4-byte words.
template <typename T, int LAYOUT, int X>
__host__ __device__ constexpr int tile_words() {
  if (sizeof(T) == 2) return LAYOUT == KC ? X * (ET<T>::BK + 8) / 2 : (ET<T>::BK / 2) * X;
  return LAYOUT == KC ? X * (ET<T>::BK + 1) : ET<T>::BK * X;
}

// V elements along the contiguous dimension starting at (rr, cc) of a matrix
// with RR x CC valid elements; anything outside reads as zero.
template <typename T>
__device__ __forceinline__ u32x4 load_vec(const T* __restrict__ base, int64_t ld, int64_t rr,
                                          int64_t cc, int64_t RR, int64_t CC, bool vec_ok) {
  constexpr int V = ET<T>::V;
  u32x4 out = {0u, 0u, 0u, 0u};
  if (rr < RR && cc < CC) {
    const T* p = base + rr * ld + cc;
    if (vec_ok && cc + V <= CC) {
      out = *reinterpret_cast<const u32x4*>(p);
    } else {
      __attribute__((aligned(16))) T tmp[V];
#pragma unroll
      for (int e = 0; e < V; ++e) tmp[e] = (cc + e < CC) ? p[e] : (T)0;
      out = *reinterpret_cast<u32x4*>(tmp);
    }
  }
  return out;
}

// This thread's share of one operand tile: global -> registers -> LDS.
// The tile covers X rows/cols (index x) by BK contraction steps (index k).
//   KC: element (x, k) is base[x*ld + k]     LDS: rows of k, padded
//   XC: element (x, k) is base[k*ld + x]     LDS: bf16: words (k pair, x); fp32: words (k, x)
template <typename T, int LAYOUT, int X>
struct TileStage {
  static constexpr int V = ET<T>::V, BK = ET<T>::BK;
  static constexpr bool HALF = sizeof(T) == 2;
  static constexpr int UNITS = LAYOUT == KC ? X * (BK / V) : (HALF ? (BK / 2) * (X / V) : BK * (X / V));
  static constexpr int PER_T = (UNITS + kMBlock - 1) / kMBlock;
  static constexpr int NV = (LAYOUT == XC && HALF) ? 2 : 1;
  u32x4 r[PER_T][NV];

  __device__ __forceinline__ void load(const T* __restrict__ base, int64_t ld, int64_t x0,
                                       int64_t xlim, int64_t k0, int64_t klim, bool vec_ok, int tid) {
#pragma unroll
    for (int it = 0; it < PER_T; ++it) {
      const int id = it * kMBlock + tid;
      if (UNITS % kMBlock != 0 && id >= UNITS) {
#pragma unroll
        for (int q = 0; q < NV; ++q) r[it][q] = u32x4{0u, 0u, 0u, 0u};
        continue;
      }
      if (LAYOUT == KC) {
        const int xl = id / (BK / V), kl = (id % (BK / V)) * V;
        r[it][0] = load_vec<T>(base, ld, x0 + xl, k0 + kl, xlim, klim, vec_ok);
      } else if (HALF) {
        const int kp = id / (X / V), xl = (id % (X / V)) * V;
        r[it][0] = load_vec<T>(base, ld, k0 + 2 * kp, x0 + xl, klim, xlim, vec_ok);
        r[it][NV - 1] = load_vec<T>(base, ld, k0 + 2 * kp + 1, x0 + xl, klim, xlim, vec_ok);
      } else {
        const int kl = id / (X / V), xl = (id % (X / V)) * V;
        r[it][0] = load_vec<T>(base, ld, k0 + kl, x0 + xl, klim, xlim, vec_ok);
      }
    }
  }

  __device__ __forceinline__ void store(uint32_t* __restrict__ lds, int tid) const {
#pragma unroll
    for (int it = 0; it < PER_T; ++it) {
      const int id = it * kMBlock + tid;
      if (UNITS % kMBlock != 0 && id >= UNITS) continue;
      if (LAYOUT == KC && HALF) {
        const int xl = id / (BK / V), kl = (id % (BK / V)) * V;
        *reinterpret_cast<u32x4*>(lds + (xl * (BK + 8) + kl) / 2) = r[it][0];
      } else if (LAYOUT == KC) {
        const int xl = id / (BK / V), kl = (id % (BK / V)) * V;
        uint32_t* d = lds + xl * (BK + 1) + kl;
        d[0] = r[it][0].x; d[1] = r[it][0].y; d[2] = r[it][0].z; d[3] = r[it][0].w;
      } else if (HALF) {
        // interleave rows k and k+1: word j = (row_k[x_j], row_k1[x_j])
        const int kp = id / (X / V), xl = (id % (X / V)) * V;
        const u32x4 a = r[it][0], b = r[it][NV - 1];
        u32x4 lo, hi;
        lo.x = (a.x & 0xffffu) | (b.x << 16); lo.y = (a.x >> 16) | (b.x & 0xffff0000u);
        lo.z = (a.y & 0xffffu) | (b.y << 16); lo.w = (a.y >> 16) | (b.y & 0xffff0000u);
        hi.x = (a.z & 0xffffu) | (b.z << 16); hi.y = (a.z >> 16) | (b.z & 0xffff0000u);
        hi.z = (a.w & 0xffffu) | (b.w << 16); hi.w = (a.w >> 16) | (b.w & 0xffff0000u);
        u32x4* d = reinterpret_cast<u32x4*>(lds + kp * X + xl);
        d[0] = lo;
        d[1] = hi;
      } else {
        const int kl = id / (X / V), xl = (id % (X / V)) * V;
        *reinterpret_cast<u32x4*>(lds + kl * X + xl) = r[it][0];
      }
    }
  }
};

// MFMA operand of lane (xi = lane % 32, g = lane / 32) for contraction step ks
// of the tile: bf16: k = ks*16 + g*8 + [0,8); fp32: k = ks*2 + g.
template <typename T, int LAYOUT, int X> struct Frag;

template <int LAYOUT, int X>
struct Frag<bf16_t, LAYOUT, X> {
  typedef bf16x8 type;
  static __device__ __forceinline__ type read(const uint32_t* __restrict__ lds, int x, int ks, int g) {
    constexpr int BK = ET<bf16_t>::BK;
    u32x4 v;
    if (LAYOUT == KC) {
      v = *reinterpret_cast<const u32x4*>(lds + (x * (BK + 8) + ks * 16 + g * 8) / 2);
    } else {
      const uint32_t* p = lds + (ks * 8 + g * 4) * X + x;
      v.x = p[0]; v.y = p[X]; v.z = p[2 * X]; v.w = p[3 * X];
    }
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int LAYOUT, int X>
struct Frag<float, LAYOUT, X> {
  typedef float type;
  static __device__ __forceinline__ type read(const uint32_t* __restrict__ lds, int x, int ks, int g) {
    constexpr int BK = ET<float>::BK;
    const uint32_t w = LAYOUT == KC ? lds[x * (BK + 1) + ks * 2 + g] : lds[(ks * 2 + g) * X + x];
    return __uint_as_float(w);
  }
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }
__device__ __forceinline__ void store_as(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_as(bf16_t* p, float v) { *p = f32_to_bf16(v); }

struct GemmArgs {
  const void* a[SYNK_MAX_WORKERS];   // A operand base per worker
  void* c[SYNK_MAX_WORKERS];         // output base per worker
  int64_t row_off[SYNK_MAX_WORKERS + 1];  // first row of each worker in the packed activations
  const void* b;        // B operand base (row_off[w]*ldb is added in MODE_DW)
  const void* mask;     // MODE_DX: activations of the layer below (row_off[w]*ldmask added)
  const float* bias;    // MODE_FWD
  int64_t m_fixed;      // MODE_DW: rows of the output (= fan-in)
  int64_t n;            // columns of the output
  int64_t k_fixed;      // MODE_FWD/DX: contraction length
  int64_t lda, ldb, ldc, ldmask;
  int64_t colsum_off;   // MODE_DW: element offset from c[w] to the bias gradient, or -1
  int relu;             // MODE_FWD: apply relu
  int out_f32;          // MODE_FWD: store fp32 (logits) instead of T
  int a_vec, b_vec;     // operands may be read with 16-byte loads
};

// C[M x N] = A * B on one (worker, m-tile, n-tile).  grid = (n tiles, m tiles,
// workers); 256 threads; wave (wm, wn) of the 2 x 2 arrangement owns a
// (BM/2) x (BN/2) block made of TM x TN MFMA tiles of 32 x 32.
template <typename T, int MODE, int BM, int BN>
__global__ __launch_bounds__(kMBlock) void mlp_gemm_kernel(GemmArgs g) {
  constexpr int LA = MODE == MODE_DW ? XC : KC;
  constexpr int LB = MODE == MODE_DX ? KC : XC;
  constexpr int BK = ET<T>::BK, KM = ET<T>::KM;
  constexpr int TM = BM / 64, TN = BN / 64;
  __shared__ __attribute__((aligned(16))) uint32_t sA[tile_words<T, LA, BM>()];
  __shared__ __attribute__((aligned(16))) uint32_t sB[tile_words<T, LB, BN>()];

  const int w = blockIdx.z;
  const int64_t rows_w = g.row_off[w + 1] - g.row_off[w];
  const int64_t M = MODE == MODE_DW ? g.m_fixed : rows_w;
  const int64_t N = g.n;
  const int64_t Kc = MODE == MODE_DW ? rows_w : g.k_fixed;
  const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
  if (m0 >= M) return;   // uniform for the block

  const T* A = reinterpret_cast<const T*>(g.a[w]);
  const T* B = reinterpret_cast<const T*>(g.b) + (MODE == MODE_DW ? g.row_off[w] * g.ldb : 0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int xi = lane & 31, gk = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const bool want_colsum = MODE == MODE_DW && g.colsum_off >= 0 && blockIdx.y == 0;
  float colsum = 0.0f;

  TileStage<T, LA, BM> stA;
  TileStage<T, LB, BN> stB;
  const int64_t n_tiles = (Kc + BK - 1) / BK;
  if (n_tiles > 0) {
    stA.load(A, g.lda, m0, M, 0, Kc, g.a_vec != 0, tid);
    stB.load(B, g.ldb, n0, N, 0, Kc, g.b_vec != 0, tid);
  }
  for (int64_t t = 0; t < n_tiles; ++t) {
    __syncthreads();   // everyone is done reading the previous tile
    stA.store(sA, tid);
    stB.store(sB, tid);
    __syncthreads();
    if (t + 1 < n_tiles) {   // next tile's global loads fly during the MFMAs
      stA.load(A, g.lda, m0, M, (t + 1) * BK, Kc, g.a_vec != 0, tid);
      stB.load(B, g.ldb, n0, N, (t + 1) * BK, Kc, g.b_vec != 0, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK / KM; ++ks) {
      typename Frag<T, LA, BM>::type fa[TM];
      typename Frag<T, LB, BN>::type fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[i] = Frag<T, LA, BM>::read(sA, wm * (BM / 2) + i * 32 + xi, ks, gk);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[j] = Frag<T, LB, BN>::read(sB, wn * (BN / 2) + j * 32 + xi, ks, gk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
    }
    if (MODE == MODE_DW) {
      if (want_colsum && tid < BN) {   // column sums of the dZ tile, in row order
        if (sizeof(T) == 2) {
#pragma unroll
          for (int kp = 0; kp < BK / 2; ++kp) {
            const uint32_t wd = sB[kp * BN + tid];
            colsum += bf16_to_f32((uint16_t)(wd & 0xffffu));
            colsum += bf16_to_f32((uint16_t)(wd >> 16));
          }
        } else {
#pragma unroll
          for (int k = 0; k < BK; ++k) colsum += __uint_as_float(sB[k * BN + tid]);
        }
      }
    }
  }

  // epilogue: lane holds column (xi) of 16 rows per MFMA tile
  char* Cw = reinterpret_cast<char*>(g.c[w]);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t col = n0 + wn * (BN / 2) + j * 32 + xi;
      if (col >= N) continue;
      float bias = 0.0f;
      if (MODE == MODE_FWD) bias = g.bias[col];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t row = m0 + wm * (BM / 2) + i * 32 + (v >> 2) * 8 + gk * 4 + (v & 3);
        if (row >= M) continue;
        float val = acc[i][j][v];
        if (MODE == MODE_FWD) {
          val += bias;
          if (g.relu) val = fmaxf(val, 0.0f);
          if (g.out_f32) reinterpret_cast<float*>(Cw)[row * g.ldc + col] = val;
          else store_as(reinterpret_cast<T*>(Cw) + row * g.ldc + col, val);
        } else if (MODE == MODE_DX) {
          const T h = reinterpret_cast<const T*>(g.mask)[(g.row_off[w] + row) * g.ldmask + col];
          if (!(to_f32(h) > 0.0f)) val = 0.0f;
          store_as(reinterpret_cast<T*>(Cw) + row * g.ldc + col, val);
        } else {
          reinterpret_cast<float*>(Cw)[row * g.ldc + col] = val;
        }
      }
    }
  }
  if (MODE == MODE_DW) {
    if (want_colsum && tid < BN && n0 + tid < N)
      reinterpret_cast<float*>(Cw)[g.colsum_off + n0 + tid] = colsum;
  }
}

// ---------------------------------------------------------------- softmax CE
struct CeArgs {
  const int32_t* y[SYNK_MAX_WORKERS];
  int64_t row_off[SYNK_MAX_WORKERS + 1];
  const float* logits;   // [R x C]
  void* dz;              // [R x C] in T
  float* row_loss;       // [R]
  int64_t classes;
  int n_slices;
  int grad_op;
};

constexpr int kCeRowsPerBlock = 4;   // one wavefront per row

// Per row: loss_i = logsumexp - logit[y]; dZ = (softmax - onehot) * weight,
// weight = 1/|R_w| (MEAN over slices) or 1/|R_ws| (SUM over slices).
template <typename T>
__global__ __launch_bounds__(kMBlock) void softmax_ce_kernel(CeArgs a) {
  const int w = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t rows_w = a.row_off[w + 1] - a.row_off[w];
  const int64_t r = (int64_t)blockIdx.x * kCeRowsPerBlock + wave;
  if (r >= rows_w) return;
  const int64_t row = a.row_off[w] + r;
  const int64_t C = a.classes;
  const float* x = a.logits + row * C;
  const int y = a.y[w][r];

  float weight;
  if (a.grad_op == SYNK_MEAN) {
    weight = 1.0f / (float)rows_w;
  } else {
    int s;
    int64_t start;
    share_of(rows_w, a.n_slices, r, &s, &start);
    const int64_t n_ws = rows_w / a.n_slices + (s < rows_w % a.n_slices ? 1 : 0);
    weight = 1.0f / (float)n_ws;
  }

  float m = -INFINITY, ssum = 0.0f, xy = 0.0f;
  for (int64_t c = lane; c < C; c += 64) {
    const float v = x[c];
    if (v > m) {
      ssum = ssum * expf(m - v) + 1.0f;
      m = v;
    } else {
      ssum += expf(v - m);
    }
    if (c == y) xy = v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float om = __shfl_xor(m, off), os = __shfl_xor(ssum, off), oxy = __shfl_xor(xy, off);
    const float nm = fmaxf(m, om);
    const float sa = (m == nm) ? ssum : ssum * expf(m - nm);
    const float sb = (om == nm) ? os : os * expf(om - nm);
    ssum = sa + sb;
    m = nm;
    xy += oxy;
  }
  if (lane == 0) a.row_loss[row] = (logf(ssum) + m) - xy;
  const float inv = 1.0f / ssum;
  T* dz = reinterpret_cast<T*>(a.dz) + row * C;
  for (int64_t c = lane; c < C; c += 64) {
    const float p = expf(x[c] - m) * inv;
    store_as(dz + c, (p - (c == y ? 1.0f : 0.0f)) * weight);
  }
}

// loss[w] = aggregate over the worker's slices of the slice mean losses.
__global__ __launch_bounds__(kMBlock) void slice_loss_kernel(const float* __restrict__ row_loss,
                                                             CeArgs a, float* __restrict__ loss) {
  __shared__ float s_part[kMBlock];
  const int w = blockIdx.x;
  const int64_t rows_w = a.row_off[w + 1] - a.row_off[w];
  const float* rl = row_loss + a.row_off[w];
  float total = 0.0f;
  for (int s = 0; s < a.n_slices; ++s) {
    const int64_t base = rows_w / a.n_slices, extra = rows_w % a.n_slices;
    const int64_t n_ws = base + (s < extra ? 1 : 0);
    const int64_t start = base * s + (s < extra ? s : extra);
    float part = 0.0f;
    for (int64_t i = threadIdx.x; i < n_ws; i += kMBlock) part += rl[start + i];
    s_part[threadIdx.x] = part;
    __syncthreads();
    for (int off = kMBlock / 2; off > 0; off >>= 1) {
      if (threadIdx.x < off) s_part[threadIdx.x] += s_part[threadIdx.x + off];
      __syncthreads();
    }
    if (n_ws > 0) {
      const float slice_mean = s_part[0] / (float)n_ws;
      total += (a.grad_op == SYNK_MEAN) ? slice_mean * ((float)n_ws / (float)rows_w) : slice_mean;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[w] = total;
}

// ------------------------------------------------------------ host side
struct MlpPlan {
  int L;
  int64_t d[SYNK_MAX_LAYERS + 1];
  int64_t offW[SYNK_MAX_LAYERS], offB[SYNK_MAX_LAYERS];
  int64_t P;
  int64_t R;                                   // total rows
  int64_t row_off[SYNK_MAX_WORKERS + 1];
  int64_t max_rows;
  size_t elem;                                 // bytes of T
  // workspace offsets (bytes)
  size_t h[SYNK_MAX_LAYERS];                   // h[l], l = 1..L-1: activations of hidden layer l
  size_t dz[SYNK_MAX_LAYERS + 1];              // dz[l], l = 1..L
  size_t logits, row_loss, total;
};

static int make_plan(const synk_mlp_desc* m, const int64_t* rows, int n_workers, MlpPlan* p) {
  if (!m || !m->dims) return SYNK_ERR_NULL;
  if (m->n_layers < 1 || m->n_layers > SYNK_MAX_LAYERS) return SYNK_ERR_SHAPE;
  if (m->compute_dtype != SYNK_F32 && m->compute_dtype != SYNK_BF16) return SYNK_ERR_DTYPE;
  p->L = m->n_layers;
  p->elem = m->compute_dtype == SYNK_F32 ? 4 : 2;
  int64_t at = 0;
  for (int l = 0; l <= p->L; ++l) {
    if (m->dims[l] <= 0 || m->dims[l] > (1LL << 21)) return SYNK_ERR_SHAPE;   // grid.y limit
    p->d[l] = m->dims[l];
  }
  for (int l = 0; l < p->L; ++l) {
    p->offW[l] = at;
    at += p->d[l] * p->d[l + 1];
    p->offB[l] = at;
    at += p->d[l + 1];
  }
  p->P = at;
  p->R = 0;
  p->max_rows = 0;
  if (rows) {
    if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS) return SYNK_ERR_SHAPE;
    for (int w = 0; w < n_workers; ++w) {
      if (rows[w] < 0 || rows[w] > (1LL << 21)) return SYNK_ERR_SHAPE;     // grid.y limit
      p->row_off[w] = p->R;
      p->R += rows[w];
      if (rows[w] > p->max_rows) p->max_rows = rows[w];
    }
    p->row_off[n_workers] = p->R;
    if (p->R == 0) return SYNK_ERR_SHAPE;
    size_t o = 0;
    for (int l = 1; l < p->L; ++l) {
      p->h[l] = o;
      o += round_up((size_t)p->R * p->d[l] * p->elem, 256);
    }
    for (int l = 1; l <= p->L; ++l) {
      p->dz[l] = o;
      o += round_up((size_t)p->R * p->d[l] * p->elem, 256);
    }
    p->logits = o;
    o += round_up((size_t)p->R * p->d[p->L] * 4, 256);
    p->row_loss = o;
    o += round_up((size_t)p->R * 4, 256);
    p->total = o;
  }
  return SYNK_OK;
}

template <typename T, int MODE>
static int launch_gemm(const GemmArgs& g, int64_t m_max, int n_workers, hipStream_t s) {
  // large tiles when they alone fill the chip, small ones otherwise
  const int64_t big = ((m_max + 127) / 128) * ((g.n + 127) / 128) * n_workers;
  if (big >= 2 * kNumCU) {
    const dim3 grid((unsigned)((g.n + 127) / 128), (unsigned)((m_max + 127) / 128), n_workers);
    hipLaunchKernelGGL((mlp_gemm_kernel<T, MODE, 128, 128>), grid, dim3(kMBlock), 0, s, g);
  } else {
    const dim3 grid((unsigned)((g.n + 63) / 64), (unsigned)((m_max + 63) / 64), n_workers);
    hipLaunchKernelGGL((mlp_gemm_kernel<T, MODE, 64, 64>), grid, dim3(kMBlock), 0, s, g);
  }
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

template <typename T>
static int run_sliced_grad(const MlpPlan& p, const float* params, const void* params_lp,
                           const void* const* x, const int32_t* const* y, const int64_t* rows,
                           int n_workers, int n_slices, int grad_op, float* const* grad,
                           float* loss, char* ws, hipStream_t s) {
  constexpr int V = ET<T>::V;
  const T* wts = sizeof(T) == 4 ? reinterpret_cast<const T*>(params)
                                : reinterpret_cast<const T*>(params_lp);
  const int L = p.L;
  auto act = [&](int l) { return reinterpret_cast<T*>(ws + p.h[l]); };   // l = 1..L-1
  auto dzp = [&](int l) { return reinterpret_cast<T*>(ws + p.dz[l]); };  // l = 1..L
  float* logits = reinterpret_cast<float*>(ws + p.logits);
  float* row_loss = reinterpret_cast<float*>(ws + p.row_loss);

  bool x_vec = true, grad_al = true;
  for (int w = 0; w < n_workers; ++w) {
    if (rows[w] > 0) x_vec = x_vec && aligned_to(x[w], 16);
    grad_al = grad_al && aligned_to(grad[w], 16);
  }
  (void)grad_al;

  GemmArgs g;
  for (int w = 0; w <= n_workers; ++w) g.row_off[w] = p.row_off[w];
  for (int w = n_workers + 1; w <= SYNK_MAX_WORKERS; ++w) g.row_off[w] = p.R;

  // ---- forward (layer index l = 1..L, weights W_l = [d_{l-1} x d_l])
  for (int l = 1; l <= L; ++l) {
    const int64_t K = p.d[l - 1], N = p.d[l];
    const T* W = wts + p.offW[l - 1];
    for (int w = 0; w < n_workers; ++w) {
      g.a[w] = l == 1 ? x[w] : (const void*)(act(l - 1) + p.row_off[w] * K);
      g.c[w] = l == L ? (void*)(logits + p.row_off[w] * N) : (void*)(act(l) + p.row_off[w] * N);
    }
    g.b = W;
    g.mask = nullptr;
    g.bias = params + p.offB[l - 1];
    g.m_fixed = 0;
    g.n = N;
    g.k_fixed = K;
    g.lda = K; g.ldb = N; g.ldc = N; g.ldmask = 0;
    g.colsum_off = -1;
    g.relu = l < L;
    g.out_f32 = l == L;
    g.a_vec = (K % V == 0) && (l == 1 ? x_vec : true);
    g.b_vec = (N % V == 0) && aligned_to(W, 16);
    if (int rc = launch_gemm<T, MODE_FWD>(g, p.max_rows, n_workers, s)) return rc;
  }

  // ---- loss and dZ_L
  CeArgs ce;
  for (int w = 0; w < n_workers; ++w) ce.y[w] = y[w];
  for (int w = 0; w <= SYNK_MAX_WORKERS; ++w) ce.row_off[w] = g.row_off[w];
  ce.logits = logits;
  ce.dz = dzp(L);
  ce.row_loss = row_loss;
  ce.classes = p.d[L];
  ce.n_slices = n_slices;
  ce.grad_op = grad_op;
  {
    const dim3 grid((unsigned)((p.max_rows + kCeRowsPerBlock - 1) / kCeRowsPerBlock), n_workers);
    hipLaunchKernelGGL((softmax_ce_kernel<T>), grid, dim3(kMBlock), 0, s, ce);
    SYNK_LAUNCH_CHECK();
    hipLaunchKernelGGL(slice_loss_kernel, dim3(n_workers), dim3(kMBlock), 0, s, row_loss, ce, loss);
    SYNK_LAUNCH_CHECK();
  }

  // ---- backward
  for (int l = L; l >= 1; --l) {
    const int64_t K = p.d[l - 1], N = p.d[l];
    // dW_l[w] = H_{l-1}[w]^T dZ_l[w]; db_l[w] = column sums of dZ_l[w]
    for (int w = 0; w < n_workers; ++w) {
      g.a[w] = l == 1 ? x[w] : (const void*)(act(l - 1) + p.row_off[w] * K);
      g.c[w] = grad[w] + p.offW[l - 1];
    }
    g.b = dzp(l);
    g.mask = nullptr;
    g.bias = nullptr;
    g.m_fixed = K;
    g.n = N;
    g.k_fixed = 0;
    g.lda = K; g.ldb = N; g.ldc = N; g.ldmask = 0;
    g.colsum_off = p.offB[l - 1] - p.offW[l - 1];
    g.relu = 0;
    g.out_f32 = 1;
    g.a_vec = (K % V == 0) && (l == 1 ? x_vec : true);
    g.b_vec = (N % V == 0);
    if (int rc = launch_gemm<T, MODE_DW>(g, K, n_workers, s)) return rc;

    if (l > 1) {
      // dZ_{l-1} = (dZ_l W_l^T) * [H_{l-1} > 0]
      const T* W = wts + p.offW[l - 1];
      for (int w = 0; w < n_workers; ++w) {
        g.a[w] = dzp(l) + p.row_off[w] * N;
        g.c[w] = dzp(l - 1) + p.row_off[w] * K;
      }
      g.b = W;
      g.mask = act(l - 1);
      g.m_fixed = 0;
      g.n = K;          // output columns = fan-in of layer l
      g.k_fixed = N;    // contraction over the layer's outputs
      g.lda = N; g.ldb = N; g.ldc = K; g.ldmask = K;
      g.colsum_off = -1;
      g.a_vec = (N % V == 0);
      g.b_vec = (N % V == 0) && aligned_to(W, 16);
      if (int rc = launch_gemm<T, MODE_DX>(g, p.max_rows, n_workers, s)) return rc;
    }
  }
  return SYNK_OK;
}

}  // namespace synk

using namespace synk;

extern "C" int synk_mlp_param_count(const synk_mlp_desc* m, int64_t* count) {
  if (!count) return SYNK_ERR_NULL;
  MlpPlan p;
  if (int rc = make_plan(m, nullptr, 0, &p)) return rc;
  *count = p.P;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_workspace_bytes(const synk_mlp_desc* m, const int64_t* rows,
                                                int n_workers, size_t* bytes) {
  if (!rows || !bytes) return SYNK_ERR_NULL;
  MlpPlan p;
  if (int rc = make_plan(m, rows, n_workers, &p)) return rc;
  *bytes = p.total;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad(const synk_mlp_desc* m, const float* params, const void* params_lp,
                                const void* const* x, const int32_t* const* y, const int64_t* rows,
                                int n_workers, int n_slices, int grad_op, float* const* grad,
                                float* loss, void* ws, size_t ws_bytes, void* stream) {
  if (!m || !params || !x || !y || !rows || !grad || !loss) return SYNK_ERR_NULL;
  MlpPlan p;
  if (int rc = make_plan(m, rows, n_workers, &p)) return rc;
  if (n_slices < 1) return SYNK_ERR_SHAPE;
  if (grad_op != SYNK_SUM && grad_op != SYNK_MEAN) return SYNK_ERR_OP;
  if (m->compute_dtype == SYNK_BF16 && !params_lp) return SYNK_ERR_NULL;
  if (!aligned_to(params, 4) || !aligned_to(loss, 4)) return SYNK_ERR_ALIGN;
  if (m->compute_dtype == SYNK_BF16 && !aligned_to(params_lp, 2)) return SYNK_ERR_ALIGN;
  for (int w = 0; w < n_workers; ++w) {
    if (!grad[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grad[w], 4)) return SYNK_ERR_ALIGN;
    if (rows[w] > 0) {
      if (!x[w] || !y[w]) return SYNK_ERR_NULL;
      if (!aligned_to(x[w], p.elem) || !aligned_to(y[w], 4)) return SYNK_ERR_ALIGN;
    }
  }
  if (!ws || !aligned_to(ws, 256) || ws_bytes < p.total) return SYNK_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (m->compute_dtype == SYNK_F32)
    return run_sliced_grad<float>(p, params, params_lp, x, y, rows, n_workers, n_slices, grad_op,
                                  grad, loss, reinterpret_cast<char*>(ws), s);
  return run_sliced_grad<bf16_t>(p, params, params_lp, x, y, rows, n_workers, n_slices, grad_op,
                                 grad, loss, reinterpret_cast<char*>(ws), s);
}
