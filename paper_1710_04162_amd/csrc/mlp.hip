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

#include <type_traits>

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
};
template <> struct ET<bf16_t> {
  static constexpr int V = 8;
  static constexpr int KM = 16;
};

// LDS footprint of one operand tile (X rows/cols by BK contraction steps), in
// 4-byte words.
template <typename T, int LAYOUT, int X, int BK>
__host__ __device__ constexpr int tile_words() {
  if (sizeof(T) == 2) return LAYOUT == KC ? X * (BK + 8) / 2 : (BK / 2) * X;
  return LAYOUT == KC ? X * (BK + 1) : BK * X;
}

// V elements along the contiguous dimension starting at (rr, cc) of a matrix
// with RR x CC valid elements; anything outside reads as zero.  Element-wise
// and branchy: only for operands that cannot be read with 16-byte loads.
template <typename T>
__device__ __forceinline__ u32x4 load_vec_slow(const T* __restrict__ base, int64_t ld, int64_t rr,
                                               int64_t cc, int64_t RR, int64_t CC) {
  constexpr int V = ET<T>::V;
  u32x4 out = {0u, 0u, 0u, 0u};
  if (rr < RR && cc < CC) {
    const T* p = base + rr * ld + cc;
    __attribute__((aligned(16))) T tmp[V];
#pragma unroll
    for (int e = 0; e < V; ++e) tmp[e] = (cc + e < CC) ? p[e] : (T)0;
    out = *reinterpret_cast<u32x4*>(tmp);
  }
  return out;
}

// This thread's share of one operand tile: global -> registers -> LDS.
// The tile covers X rows/cols (index x) by BK contraction steps (index k).
//   KC: element (x, k) is base[x*ld + k]     LDS: rows of k, padded
//   XC: element (x, k) is base[k*ld + x]     LDS: bf16: words (k pair, x); fp32: words (k, x)
// ALIGNED: every vector is wholly inside or wholly outside the matrix.  Loads
// are then issued unconditionally (an outside vector reads the matrix origin
// and is zeroed when it goes to LDS), so that nothing but the data dependence
// orders them against the MFMAs of the tile before.
//
// TileAddr holds what does not change along the contraction: one pointer per
// unit (64-bit address arithmetic done once, before the loop) and whether the
// unit's x is inside the matrix.  Per tile only a wave-uniform offset is added.
template <typename T, int LAYOUT, int X, int BK>
struct TileGeom {
  static constexpr int V = ET<T>::V;
  static constexpr bool HALF = sizeof(T) == 2;
  static constexpr int UNITS = LAYOUT == KC ? X * (BK / V) : (HALF ? (BK / 2) * (X / V) : BK * (X / V));
  static constexpr int PER_T = (UNITS + kMBlock - 1) / kMBlock;
  static constexpr int NV = (LAYOUT == XC && HALF) ? 2 : 1;
  // position of unit `id` inside the tile: x offset and k offset
  static __device__ __forceinline__ void unit_pos(int id, int* xl, int* kl) {
    if (LAYOUT == KC) {
      *xl = id / (BK / V);
      *kl = (id % (BK / V)) * V;
    } else if (HALF) {
      *kl = 2 * (id / (X / V));
      *xl = (id % (X / V)) * V;
    } else {
      *kl = id / (X / V);
      *xl = (id % (X / V)) * V;
    }
  }
};

template <typename T, int LAYOUT, int X, int BK>
struct TileAddr {
  typedef TileGeom<T, LAYOUT, X, BK> G;
  const T* ptr[G::PER_T];   // unit's first vector in the tile that starts at k = 0
  const T* base;
  int64_t ld;
  int x0, xlim;
  uint32_t xok;
  // Fast path (tile wholly inside the matrix): address = wave-uniform tile
  // origin (scalar registers) + a 32-bit per-thread byte offset that never
  // changes, so a load costs no vector address arithmetic at all.
  const char* origin;       // element (x0, k = 0)
  uint32_t off[G::PER_T];   // bytes from the tile origin to the unit's first vector
  bool interior;            // x0 + X <= xlim: every unit is inside along x

  __device__ __forceinline__ void init(const T* b, int64_t ld_, int64_t x0_, int64_t xlim_, int tid) {
    base = b;
    ld = ld_;
    x0 = (int)x0_;
    xlim = (int)xlim_;
    xok = 0u;
    interior = x0_ + X <= xlim_;
    origin = reinterpret_cast<const char*>(b + (LAYOUT == KC ? x0_ * ld_ : x0_));
#pragma unroll
    for (int it = 0; it < G::PER_T; ++it) {
      const int id = it * kMBlock + tid;
      int xl, kl;
      G::unit_pos(id, &xl, &kl);
      const bool unit = (G::UNITS % kMBlock == 0) || id < G::UNITS;
      const bool live = unit && x0 + xl < xlim;
      const int64_t off64 = LAYOUT == KC ? (int64_t)(x0 + xl) * ld + kl : (int64_t)kl * ld + (x0 + xl);
      ptr[it] = b + (live ? off64 : 0);
      xok |= (live ? 1u : 0u) << it;
      const int64_t rel = LAYOUT == KC ? (int64_t)xl * ld + kl : (int64_t)kl * ld + xl;
      off[it] = unit ? (uint32_t)(rel * (int64_t)sizeof(T)) : 0u;
    }
  }
};

template <typename T, int LAYOUT, int X, int BK, bool ALIGNED>
struct TileStage {
  typedef TileGeom<T, LAYOUT, X, BK> G;
  static constexpr int V = G::V, PER_T = G::PER_T, NV = G::NV, UNITS = G::UNITS;
  static constexpr bool HALF = G::HALF;
  u32x4 r[PER_T][NV];
  uint32_t ok;   // bit (it*NV + q): vector is inside the matrix
  bool whole;    // wave-uniform: loaded by load_whole(), nothing to zero

  // all units this thread owns, all their vectors
  static constexpr uint32_t kAllOk = (PER_T * NV >= 32) ? 0xffffffffu : ((1u << (PER_T * NV)) - 1u);

  // A tile wholly inside the matrix (ALIGNED, ta.interior, k0 + BK <= klim).
  __device__ __forceinline__ void load_whole(const TileAddr<T, LAYOUT, X, BK>& ta, int k0) {
    const int64_t ldb = ta.ld * (int64_t)sizeof(T);
    load_at(ta, ta.origin + (LAYOUT == KC ? (int64_t)k0 * (int64_t)sizeof(T) : (int64_t)k0 * ldb));
  }
  // tb: the tile's origin (wave-uniform); offmask 0 sends every lane to tb itself
  __device__ __forceinline__ void load_at(const TileAddr<T, LAYOUT, X, BK>& ta, const char* tb,
                                          uint32_t offmask = 0xffffffffu) {
    const int64_t ldb = offmask ? ta.ld * (int64_t)sizeof(T) : 0;
#pragma unroll
    for (int it = 0; it < PER_T; ++it) {
#pragma unroll
      for (int q = 0; q < NV; ++q)
        r[it][q] = *reinterpret_cast<const u32x4*>(tb + (q ? ldb : 0) + (ta.off[it] & offmask));
    }
    ok = kAllOk;
    whole = true;
  }

  __device__ __forceinline__ void load(const TileAddr<T, LAYOUT, X, BK>& ta, int k0, int klim, int tid) {
    whole = false;
    const int64_t koff = LAYOUT == KC ? (int64_t)k0 : (int64_t)k0 * ta.ld;   // wave-uniform
    if (ALIGNED && k0 + BK <= klim) {
      // a tile wholly inside along the contraction: one 64-bit add per vector
      ok = 0u;
#pragma unroll
      for (int it = 0; it < PER_T; ++it) {
#pragma unroll
        for (int q = 0; q < NV; ++q)
          r[it][q] = *reinterpret_cast<const u32x4*>(ta.ptr[it] + koff + (q ? ta.ld : 0));
        ok |= (((ta.xok >> it) & 1u) ? ((1u << NV) - 1u) : 0u) << (it * NV);
      }
      return;
    }
    ok = 0u;
#pragma unroll
    for (int it = 0; it < PER_T; ++it) {
      const int id = it * kMBlock + tid;
      int xl, kl;
      G::unit_pos(id, &xl, &kl);
      if (ALIGNED) {
#pragma unroll
        for (int q = 0; q < NV; ++q) {
          const bool in = ((ta.xok >> it) & 1u) && (k0 + kl + q < klim);
          const T* p = ta.ptr[it] + koff + (q ? ta.ld : 0);
          r[it][q] = *reinterpret_cast<const u32x4*>(in ? p : ta.base);
          ok |= (in ? 1u : 0u) << (it * NV + q);
        }
      } else {
        const bool live = (UNITS % kMBlock == 0) || id < UNITS;
#pragma unroll
        for (int q = 0; q < NV; ++q) {
          if (!live) r[it][q] = u32x4{0u, 0u, 0u, 0u};
          else if (LAYOUT == KC)
            r[it][q] = load_vec_slow<T>(ta.base, ta.ld, ta.x0 + xl, k0 + kl, ta.xlim, klim);
          else
            r[it][q] = load_vec_slow<T>(ta.base, ta.ld, k0 + kl + q, ta.x0 + xl, klim, ta.xlim);
        }
        ok = kAllOk;
      }
    }
  }

  template <bool CHECK>
  __device__ __forceinline__ void store_impl(uint32_t* __restrict__ lds, int tid) const {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < PER_T; ++it) {
      const int id = it * kMBlock + tid;
      if (UNITS % kMBlock != 0 && id >= UNITS) continue;
      int xl, kl;
      G::unit_pos(id, &xl, &kl);
      const u32x4 a = (!CHECK || ((ok >> (it * NV)) & 1u)) ? r[it][0] : zero;
      if (LAYOUT == KC && HALF) {
        *reinterpret_cast<u32x4*>(lds + (xl * (BK + 8) + kl) / 2) = a;
      } else if (LAYOUT == KC) {
        uint32_t* d = lds + xl * (BK + 1) + kl;
        d[0] = a.x; d[1] = a.y; d[2] = a.z; d[3] = a.w;
      } else if (HALF) {
        // interleave rows k and k+1: word j = (row_k[x_j], row_k1[x_j]); one byte permute each
        const u32x4 b = (!CHECK || ((ok >> (it * NV + NV - 1)) & 1u)) ? r[it][NV - 1] : zero;
        u32x4 lo, hi;
        lo.x = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u); lo.y = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
        lo.z = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u); lo.w = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
        hi.x = __builtin_amdgcn_perm(b.z, a.z, 0x05040100u); hi.y = __builtin_amdgcn_perm(b.z, a.z, 0x07060302u);
        hi.z = __builtin_amdgcn_perm(b.w, a.w, 0x05040100u); hi.w = __builtin_amdgcn_perm(b.w, a.w, 0x07060302u);
        // A 16-byte LDS store goes out eight lanes at a time; the lanes' first
        // halves would sit eight words apart and meet in four banks twice.  Lanes
        // in the upper 32 words of a row store their halves in the other order.
        u32x4* d = reinterpret_cast<u32x4*>(lds + (kl / 2) * X + xl);
        const bool sw = (xl & 32) != 0;
        const u32x4 first = sw ? hi : lo, second = sw ? lo : hi;
        d[sw ? 1 : 0] = first;
        d[sw ? 0 : 1] = second;
      } else {
        *reinterpret_cast<u32x4*>(lds + kl * X + xl) = a;
      }
    }
  }

  __device__ __forceinline__ void store(uint32_t* __restrict__ lds, int tid) const {
    if (whole) store_impl<false>(lds, tid);   // nothing to zero: the common case (a scalar branch)
    else store_impl<true>(lds, tid);
  }
};

// MFMA operand of lane (xi = lane % 32, g = lane / 32) for contraction step ks
// of the tile: bf16: k = ks*16 + g*8 + [0,8); fp32: k = ks*2 + g.
template <typename T, int LAYOUT, int X, int BK> struct Frag;

template <int LAYOUT, int X, int BK>
struct Frag<bf16_t, LAYOUT, X, BK> {
  typedef bf16x8 type;
  static __device__ __forceinline__ type read(const uint32_t* __restrict__ lds, int x, int ks, int g) {
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

template <int LAYOUT, int X, int BK>
struct Frag<float, LAYOUT, X, BK> {
  typedef float type;
  static __device__ __forceinline__ type read(const uint32_t* __restrict__ lds, int x, int ks, int g) {
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

// loss[w] = aggregate over the worker's slices of the slice mean losses.  One
// wavefront per slice: lanes stride over the slice's rows, a fixed shuffle tree
// adds the 64 partial sums; thread 0 then folds the slices in slice order.
// Called by a whole workgroup of NW wavefronts; s_mean: NW floats of LDS.
template <int NW>
__device__ __forceinline__ void slice_loss_worker(const float* __restrict__ row_loss,
                                                  const int64_t* row_off, int n_slices, int grad_op,
                                                  int w, float* __restrict__ loss, float* s_mean) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t rows_w = row_off[w + 1] - row_off[w];
  const float* rl = row_loss + row_off[w];
  const int64_t base = rows_w / n_slices, extra = rows_w % n_slices;
  float total = 0.0f;
  for (int s0 = 0; s0 < n_slices; s0 += NW) {
    const int s = s0 + wave;
    float contrib = 0.0f;
    if (s < n_slices) {
      const int64_t n_ws = base + (s < extra ? 1 : 0);
      const int64_t start = base * s + (s < extra ? s : extra);
      float part = 0.0f;
      for (int64_t i = lane; i < n_ws; i += 64) part += rl[start + i];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
      if (n_ws > 0) {
        const float slice_mean = part / (float)n_ws;
        contrib = (grad_op == SYNK_MEAN) ? slice_mean * ((float)n_ws / (float)rows_w) : slice_mean;
      }
    }
    if (lane == 0) s_mean[wave] = contrib;
    __syncthreads();
    if (threadIdx.x == 0)
      for (int k = 0; k < NW; ++k) total += s_mean[k];   // slice order: s0, s0+1, ...
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[w] = total;
}

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
  int c_vec;            // output rows may be written with 16-byte stores
  // MODE_DW only: the workgroups of grid slice z == task_z do no GEMM; the first
  // of them turns the row losses of the kernel before into the workers' slice-
  // aggregated losses (a launch saved).  task_z < 0: no such slice.
  int task_z, task_workers, task_slices, task_op;
  const float* task_row_loss;
  float* task_loss;
  // Input indexing folded into the first forward product (gather_src == nullptr: a[w] holds the
  // rows already).  Row r of the packed batch is row gather_idx[r] of gather_src ([gather_rows x K]
  // of T, pitch lda); the forward kernel also leaves the rows in a[w] and, if gather_labels is
  // given, their labels in gather_y (packed: entry r for packed row r), for the kernels after it.
  const void* gather_src;
  const int32_t* gather_idx;
  const int32_t* gather_labels;
  int64_t gather_rows;
  int32_t* gather_y;
};

}  // namespace synk
#include "gemm_dma.h"
namespace synk {

// The whole-tile bf16 core as a kernel of its own (forward and dX products).
template <int MODE, int BM, int BN, int NS, bool GATHER = false>
__global__ __launch_bounds__(gdma::kThreads) void mlp_gemm_dma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(1024))) unsigned char smem[gdma::lds_bytes<BM, BN, NS>()];
  gdma::tile<MODE, BM, BN, NS, GemmArgs, GATHER>(g, blockIdx.x, tiles_m, tiles_n, smem);
}

// Workgroups are dealt to the 8 XCDs round-robin by launch order.  Re-deal so
// that each XCD (each L2) owns a contiguous run of tiles with the n-tile index
// running fastest: tiles that differ only in their row range keep hitting the
// same few L2 channels (rows are a multiple of 2 KiB apart), while neighbouring
// n-tiles spread over all of them.
// (lin: the workgroup's launch-order index in a gx x gy x gz grid whose first
// workgroup sits on XCD 0; a kernel that holds several grids passes each one's
// own index and extent.)
__device__ __forceinline__ void xcd_tile(unsigned lin, unsigned gx, unsigned gy, unsigned gz, int* bx,
                                         int* by, int* bz) {
  const unsigned total = gx * gy * gz;
  const unsigned logical = (total & 7u) == 0u ? (lin & 7u) * (total >> 3) + (lin >> 3) : lin;
  *bx = logical % gx;
  *by = (logical / gx) % gy;
  *bz = logical / (gx * gy);
}
constexpr int kGemmThreads = 2 * kMBlock;

// LDS words one workgroup of the kernel below needs (two operand tile pairs).
template <typename T, int MODE, int BM, int BN, int BK>
__host__ __device__ constexpr int gemm_lds_words() {
  return 2 * ((tile_words<T, MODE == MODE_DW ? XC : KC, BM, BK>() + tile_words<T, MODE == MODE_DX ? KC : XC, BN, BK>() + 3) / 4 * 4);
}

// The body of the kernel as a function of the workgroup's place (lin) in a
// gx x gy x gz grid and of its LDS, so that one launch can hold several grids.
template <typename T, int MODE, int BM, int BN, int BK, bool AL_A, bool AL_B>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, unsigned lin, unsigned gx, unsigned gy, unsigned gz,
                                          uint32_t* __restrict__ smem) {
  constexpr int LA = MODE == MODE_DW ? XC : KC;
  constexpr int LB = MODE == MODE_DX ? KC : XC;
  constexpr int KM = ET<T>::KM;
  constexpr int KSTEPS = BK / KM;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int WA = tile_words<T, LA, BM, BK>(), WB = tile_words<T, LB, BN, BK>();
  constexpr int WT = (WA + WB + 3) / 4 * 4;      // one tile pair, 16-byte multiple
  static_assert(2 * WT == gemm_lds_words<T, MODE, BM, BN, BK>(), "LDS size helper out of step");
  static_assert(64 * BN <= 2 * WT, "output staging (64 rows of fp32) must fit in the operand LDS");

  int bx, by, bz;
  xcd_tile(lin, gx, gy, gz, &bx, &by, &bz);
  if (MODE == MODE_DW && g.task_z >= 0 && bz == g.task_z) {   // uniform for the block
    if (bx == 0 && by == 0) {
      __shared__ float s_mean[kGemmThreads / 64];
      for (int ww = 0; ww < g.task_workers; ++ww)
        slice_loss_worker<kGemmThreads / 64>(g.task_row_loss, g.row_off, g.task_slices, g.task_op, ww, g.task_loss,
                                             s_mean);
    }
    return;
  }
  const int w = bz;
  const int64_t rows_w = g.row_off[w + 1] - g.row_off[w];
  const int64_t M = MODE == MODE_DW ? g.m_fixed : rows_w;
  const int64_t N = g.n;
  const int kc = (int)(MODE == MODE_DW ? rows_w : g.k_fixed);
  const int64_t m0 = (int64_t)by * BM, n0 = (int64_t)bx * BN;
  if (m0 >= M) return;   // uniform for the block
  const int n_tiles = (kc + BK - 1) / BK;
  const bool producer = threadIdx.x >= kMBlock;
  const int tid = threadIdx.x & (kMBlock - 1);
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int xi = lane & 31, gk = lane >> 5;
  const int m_rows = (int)M;

  f32x16 acc[TM][TN];
  float bias[TN];
  T hmask[MODE == MODE_DX ? TM : 1][MODE == MODE_DX ? TN : 1][16];
  float colsum = 0.0f;
  const bool want_colsum = MODE == MODE_DW && g.colsum_off >= 0 && by == 0;

  if (producer) {
    const T* A = reinterpret_cast<const T*>(g.a[w]);
    const T* B = reinterpret_cast<const T*>(g.b) + (MODE == MODE_DW ? g.row_off[w] * g.ldb : 0);
    TileAddr<T, LA, BM, BK> adA;
    TileAddr<T, LB, BN, BK> adB;
    adA.init(A, g.lda, m0, M, tid);
    adB.init(B, g.ldb, n0, N, tid);
    // A ring of four register stages: while tile t is multiplied, the loads of
    // tiles t+2 .. t+5 are in flight.  Loads, stores and barriers are issued on
    // every path (the loop runs a multiple of four steps), so that the number
    // of loads outstanding at each wait is known exactly.
    TileStage<T, LA, BM, BK, AL_A> stA[4];
    TileStage<T, LB, BN, BK, AL_B> stB[4];
    const int n_whole = kc / BK;                     // tiles wholly inside along the contraction
    const bool fastA = AL_A && adA.interior, fastB = AL_B && adB.interior;
    auto load_tile = [&](auto& sa, auto& sb, int j) {
      // (a tile past the end has every vector masked and lands in a half nobody reads)
      if (fastA && j < n_whole) sa.load_whole(adA, j * BK);
      else sa.load(adA, j * BK, kc, tid);
      if (fastB && j < n_whole) sb.load_whole(adB, j * BK);
      else sb.load(adB, j * BK, kc, tid);
    };
#pragma unroll
    for (int u = 0; u < 4; ++u) load_tile(stA[u], stB[u], u);
    stA[0].store(smem, tid);
    stB[0].store(smem + WA, tid);
    load_tile(stA[0], stB[0], 4);
    __syncthreads();                               // tile 0 is in slot 0
    int t = 0;
    if (fastA && fastB) {
      // Steady state: every tile stored (t+1 .. t+4) or loaded (t+5 .. t+8) in
      // the round is wholly inside both operands, or past the end (then what is
      // stored goes to a half nobody reads).  Straight-line code: four loads,
      // the LDS stores and one barrier per tile, with the two tile origins
      // advanced in scalar registers until they reach the last whole tile.
      const int64_t stepA = (LA == KC ? (int64_t)BK : (int64_t)BK * g.lda) * (int64_t)sizeof(T);
      const int64_t stepB = (LB == KC ? (int64_t)BK : (int64_t)BK * g.ldb) * (int64_t)sizeof(T);
      const char* nextA = adA.origin + 5 * stepA;     // used only while tile 5, 6, ... exist
      const char* nextB = adB.origin + 5 * stepB;
      // TAIL: some tile loaded in the round is past the end; every lane then
      // reads the first vector of the operand's first tile (one cache line).
      auto fast_round = [&](int t0, auto tail) {
        constexpr bool TAIL = decltype(tail)::value;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          uint32_t* half = smem + ((u + 1) & 1) * WT;
          stA[(u + 1) & 3].template store_impl<false>(half, tid);
          stB[(u + 1) & 3].template store_impl<false>(half + WA, tid);
          const bool in = !TAIL || t0 + u + 5 < n_whole;
          stA[(u + 1) & 3].load_at(adA, in ? nextA : adA.origin, in ? 0xffffffffu : 0u);
          stB[(u + 1) & 3].load_at(adB, in ? nextB : adB.origin, in ? 0xffffffffu : 0u);
          nextA += in ? stepA : 0;
          nextB += in ? stepB : 0;
          __syncthreads();
          // Keep every step's work in its step: hoisted into an earlier step,
          // the byte permutes of a later stage wait for that stage's loads,
          // the youngest in flight, and the ring drains.
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      for (; t + 8 < n_whole; t += 4) fast_round(t, std::false_type());
      if (n_whole == n_tiles)                        // no partial tile: the tail rounds are fast too
        for (; t < n_tiles; t += 4) fast_round(t, std::true_type());
    }
    for (; t < n_tiles; t += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        // tile t+u+1 -> the half that tile t+u (read before the last barrier) does not use
        uint32_t* half = smem + ((u + 1) & 1) * WT;
        stA[(u + 1) & 3].store(half, tid);
        stB[(u + 1) & 3].store(half + WA, tid);
        load_tile(stA[(u + 1) & 3], stB[(u + 1) & 3], t + u + 5);
        __syncthreads();
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // What the epilogue needs from memory (bias, relu mask of the layer below)
    // is requested now, so that its latency hides behind the contraction.
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int64_t col = n0 + wn * (BN / 2) + j * 32 + xi;
      bias[j] = 0.0f;
      if (MODE == MODE_FWD) bias[j] = g.bias[col < N ? col : 0];
      if (MODE == MODE_DX) {
        const T* mk = reinterpret_cast<const T*>(g.mask) + g.row_off[w] * g.ldmask;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int row0 = (int)m0 + wm * (BM / 2) + i * 32 + gk * 4;
          const T* mk0 = mk + (int64_t)row0 * g.ldmask + col;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int dr = (v >> 2) * 8 + (v & 3);
            hmask[i][j][v] = (col < N && row0 + dr < m_rows) ? mk0[dr * g.ldmask] : mk[0];
          }
        }
      }
    }

    // A wavefront that owns one MFMA tile (WHOLE) asks for every fragment of an
    // operand tile at once, one tile ahead: the LDS reads of tile t+1 are in
    // flight while tile t is multiplied out of registers, and the LDS latency
    // is paid once per tile.  A wavefront that owns several MFMA tiles reads
    // the fragments of k-step s+1 while step s is multiplied, inside the tile.
    constexpr bool WHOLE = TM * TN == 1;
    constexpr int FK = WHOLE ? KSTEPS : 1;
    static_assert(WHOLE || KSTEPS % 2 == 0, "fragment parity must not depend on the tile");
    typename Frag<T, LA, BM, BK>::type fa[2][FK][TM];
    typename Frag<T, LB, BN, BK>::type fb[2][FK][TN];
    auto read_frags = [&](const uint32_t* sA, const uint32_t* sB, int ks, auto& da, auto& db) {
#pragma unroll
      for (int i = 0; i < TM; ++i) da[i] = Frag<T, LA, BM, BK>::read(sA, wm * (BM / 2) + i * 32 + xi, ks, gk);
#pragma unroll
      for (int j = 0; j < TN; ++j) db[j] = Frag<T, LB, BN, BK>::read(sB, wn * (BN / 2) + j * 32 + xi, ks, gk);
    };
    auto read_tile = [&](const uint32_t* sA, const uint32_t* sB, int buf) {
#pragma unroll
      for (int ks = 0; ks < FK; ++ks) read_frags(sA, sB, ks, fa[buf][ks], fb[buf][ks]);
    };
    auto mfma_step = [&](int buf, int ks) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma(fa[buf][ks][i], fb[buf][ks][j], acc[i][j]);
    };
    auto column_sums = [&](const uint32_t* sB) {
      if (MODE == MODE_DW) {
        if (want_colsum && tid < BN) {   // column sums of the dZ tile, in row order
          if (sizeof(T) == 2) {
#pragma unroll 8
            for (int kp = 0; kp < BK / 2; ++kp) {
              const uint32_t wd = sB[kp * BN + tid];
              colsum += bf16_to_f32((uint16_t)(wd & 0xffffu));
              colsum += bf16_to_f32((uint16_t)(wd >> 16));
            }
          } else {
#pragma unroll 8
            for (int k = 0; k < BK; ++k) colsum += __uint_as_float(sB[k * BN + tid]);
          }
        }
      }
    };

    __syncthreads();                                 // tile 0 is in half 0
    if (WHOLE) {
      read_tile(smem, smem + WA, 0);
      column_sums(smem + WA);
    }
    // One round of the loop; ALL: tiles t .. t+4 exist (no tests in the round).
    auto round = [&](int t, auto all) {
      constexpr bool ALL = decltype(all)::value;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t* cur = smem + (u & 1) * WT;
        const uint32_t* nxt = smem + ((u + 1) & 1) * WT;
        const bool live = ALL || t + u < n_tiles, more = ALL || t + u + 1 < n_tiles;
        if (WHOLE) {
          __syncthreads();                           // tile t+u+1 is in its half
          // Left alone, the scheduler pulls the products of tile t+u+1 up behind
          // its fragment reads to shorten live ranges, which puts an LDS
          // latency in front of every MFMA.
          __builtin_amdgcn_sched_barrier(0);
          if (more) {
            read_tile(nxt, nxt + WA, (u + 1) & 1);
            column_sums(nxt + WA);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (live) {
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) mfma_step(u & 1, ks);
          }
          __builtin_amdgcn_sched_barrier(0);
        } else {
          if (live) {
            column_sums(cur + WA);
            read_frags(cur, cur + WA, 0, fa[0][0], fb[0][0]);
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
              if (ks + 1 < KSTEPS) read_frags(cur, cur + WA, ks + 1, fa[(ks + 1) & 1][0], fb[(ks + 1) & 1][0]);
              mfma_step(ks & 1, 0);
            }
          }
          __syncthreads();                           // tile t+u+1 is in its half
        }
      }
    };
    int t = 0;
    for (; t + 5 <= n_tiles; t += 4) round(t, std::true_type());
    for (; t < n_tiles; t += 4) round(t, std::false_type());   // same number of barriers as the producers

    // bias / relu / mask applied in registers
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float val = acc[i][j][v];
          if (MODE == MODE_FWD) {
            val += bias[j];
            if (g.relu) val = fmaxf(val, 0.0f);
          } else if (MODE == MODE_DX) {
            if (!(to_f32(hmask[MODE == MODE_DX ? i : 0][MODE == MODE_DX ? j : 0][v]) > 0.0f)) val = 0.0f;
          }
          acc[i][j][v] = val;
        }
  }

  // ---------------------------------------------------------------- output
  __syncthreads();   // every LDS read of the contraction is over before the output is staged
  const bool out_f32 = MODE == MODE_DW || sizeof(T) == 4 || (MODE == MODE_FWD && g.out_f32);
  char* Cw = reinterpret_cast<char*>(g.c[w]);
  if (g.c_vec) {
    constexpr int PASSES = BM / 64;
    for (int ps = 0; ps < PASSES; ++ps) {
      if (!producer) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int tile_row = wm * (BM / 2) + i * 32;     // first row of the MFMA tile in the block tile
          if (tile_row / 64 != ps) continue;
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            // one base address per MFMA tile; the 16 results sit at compile-time offsets from it
            const int base = ((tile_row & 63) + gk * 4) * BN + wn * (BN / 2) + j * 32 + xi;
            if (out_f32) {
              float* sp = reinterpret_cast<float*>(smem) + base;
#pragma unroll
              for (int v = 0; v < 16; ++v) sp[((v >> 2) * 8 + (v & 3)) * BN] = acc[i][j][v];
            } else {
              uint16_t* sp = reinterpret_cast<uint16_t*>(smem) + base;
#pragma unroll
              for (int v = 0; v < 16; ++v) sp[((v >> 2) * 8 + (v & 3)) * BN] = f32_to_bf16(acc[i][j][v]);
            }
            // keep the tiles apart in the schedule: interleaving them only lengthens live ranges
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __syncthreads();
      const int elem_b = out_f32 ? 4 : 2;
      const int cpr = BN * elem_b / 16;                      // 16-byte chunks per row
      for (int c = threadIdx.x; c < 64 * cpr; c += kGemmThreads) {
        const int rl = c / cpr, ch = c - rl * cpr;
        const int64_t row = m0 + ps * 64 + rl;
        const int64_t col = n0 + ch * (16 / elem_b);
        if (row < M && col < N) {
          const u32x4 q = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(smem) +
                                                          ((int64_t)rl * BN * elem_b + ch * 16));
          *reinterpret_cast<u32x4*>(Cw + (row * g.ldc + col) * elem_b) = q;
        }
      }
      if (ps + 1 < PASSES) __syncthreads();
    }
  } else if (!producer) {
    // element-wise stores straight from the MFMA layout
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int64_t col = n0 + wn * (BN / 2) + j * 32 + xi;
        const int row0 = (int)m0 + wm * (BM / 2) + i * 32 + gk * 4;   // row of v: row0 + (v>>2)*8 + (v&3)
        const int64_t e0 = (int64_t)row0 * g.ldc + col;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int dr = (v >> 2) * 8 + (v & 3);
          if (col >= N || row0 + dr >= m_rows) continue;
          const int64_t e = e0 + dr * g.ldc;
          if (out_f32) reinterpret_cast<float*>(Cw)[e] = acc[i][j][v];
          else reinterpret_cast<uint16_t*>(Cw)[e] = f32_to_bf16(acc[i][j][v]);
        }
      }
    }
  }
  if (MODE == MODE_DW) {
    if (!producer && want_colsum && tid < BN && n0 + tid < N)
      reinterpret_cast<float*>(Cw)[g.colsum_off + n0 + tid] = colsum;
  }
}

template <typename T, int MODE, int BM, int BN, int BK, bool AL_A, bool AL_B>
__global__ __launch_bounds__(kGemmThreads, (BM == 128 && MODE != MODE_DX) ? 4 : 2) void mlp_gemm_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[gemm_lds_words<T, MODE, BM, BN, BK>()];
  gemm_tile<T, MODE, BM, BN, BK, AL_A, AL_B>(g, blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z),
                                             gridDim.x, gridDim.y, gridDim.z, smem);
}

// ------------------------------------------------------- persistent dW
// dW_l[w] = H_{l-1}[w]^T dZ_l[w] when a worker has few rows: the contraction is
// then a handful of k-tiles and a workgroup per output tile spends its life in
// the first loads and in the write-out.  Here a workgroup walks a list of
// output tiles and the producers' tile stream runs straight across tile
// boundaries: while the consumers write tile i out (through a staging area of
// its own in LDS, as whole 512-byte row segments: 32-byte pieces straight from
// the accumulators measured slower), the operand tiles of tile i+1 are already
// on their way.
// Preconditions (checked on the host): both operands and the output take
// 16-byte accesses, the output is a whole number of 128 x 128 tiles, and every
// worker's row count is a multiple of four k-tiles (zero rows allowed).
template <typename T>
__host__ __device__ constexpr int dw_persistent_lds_words() {
  constexpr int BK = sizeof(T) == 2 ? 32 : 16;
  return 2 * ((tile_words<T, XC, 128, BK>() + tile_words<T, XC, 128, BK>() + 3) / 4 * 4) + 64 * 128;
}

// vblock of vgrid: this workgroup's place among the workgroups that share the tile list
template <typename T>
__device__ __forceinline__ void dw_persistent_body(const GemmArgs& g, int tiles_m, int tiles_n, int n_workers,
                                                   unsigned vblock, unsigned vgrid, uint32_t* __restrict__ smem) {
  constexpr int BM = 128, BN = 128, BK = sizeof(T) == 2 ? 32 : 16;
  constexpr int KM = ET<T>::KM;
  constexpr int KSTEPS = BK / KM;
  constexpr int TM = 2, TN = 2;
  constexpr int WA = tile_words<T, XC, BM, BK>(), WB = tile_words<T, XC, BN, BK>();
  constexpr int WT = (WA + WB + 3) / 4 * 4;
  static_assert(2 * WT + 64 * BN == dw_persistent_lds_words<T>(), "LDS size helper out of step");
  float* stage = reinterpret_cast<float*>(smem + 2 * WT);       // two buffers of 32 rows of the fp32 output tile

  const bool producer = threadIdx.x >= kMBlock;
  const int tid = threadIdx.x & (kMBlock - 1);
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int xi = lane & 31, gk = lane >> 5;
  const int tiles_w = tiles_m * tiles_n;
  const int total = tiles_w * n_workers;
  const int64_t lda = g.lda, ldb = g.ldb;

  // j-th tile of this workgroup.  Workgroups are dealt to the 8 XCDs round-robin;
  // each XCD (each L2) gets a contiguous run of tiles with the n-tile running fastest.
  auto tile_of = [&](int j, int* w, int* m0, int* n0) -> bool {
    int lin;
    if ((total & 7) == 0 && (vgrid & 7u) == 0u) {
      const int per = total >> 3, idx = (int)(vblock >> 3) + j * (int)(vgrid >> 3);
      if (idx >= per) return false;
      lin = (int)(vblock & 7u) * per + idx;
    } else {
      lin = (int)vblock + j * (int)vgrid;
      if (lin >= total) return false;
    }
    *w = lin / tiles_w;
    const int r = lin - *w * tiles_w;
    *m0 = (r / tiles_n) * BM;
    *n0 = (r % tiles_n) * BN;
    return true;
  };
  auto k_tiles = [&](int w) { return (int)((g.row_off[w + 1] - g.row_off[w]) / BK); };
  // Write-out in four passes of 32 rows: two consumer wavefronts put their MFMA
  // row block into one of two staging buffers, and after the barrier all 512
  // threads (the producers have nothing else to do here) copy it out as whole
  // 512-byte row segments while the next pass is written into the other buffer.
  auto read_out = [&](int ps, float* Cw, int m0, int n0) {
    constexpr int CPR = BN * 4 / 16;                           // 16-byte chunks per row
    const float* buf = stage + (ps & 1) * 32 * BN;
    for (int c = threadIdx.x; c < 32 * CPR; c += kGemmThreads) {
      const int rl = c / CPR, ch = c - rl * CPR;
      const f32x4 q = *reinterpret_cast<const f32x4*>(buf + rl * BN + ch * 4);
      *reinterpret_cast<f32x4*>(Cw + (int64_t)(m0 + ps * 32 + rl) * g.ldc + n0 + ch * 4) = q;
    }
  };

  if (producer) {
    // per-thread byte offsets inside a tile do not depend on the tile
    TileAddr<T, XC, BM, BK> adA;
    TileAddr<T, XC, BN, BK> adB;
    adA.init(reinterpret_cast<const T*>(g.a[0]), lda, 0, BM, tid);
    adB.init(reinterpret_cast<const T*>(g.b), ldb, 0, BN, tid);
    const int64_t stepA = (int64_t)BK * lda * (int64_t)sizeof(T), stepB = (int64_t)BK * ldb * (int64_t)sizeof(T);
    // load cursor: the next k-tile of the stream (tiles without rows contribute none)
    int lj = -1, lk = 0, lnk = 0;
    const char* la = reinterpret_cast<const char*>(g.a[0]);
    const char* lb = reinterpret_cast<const char*>(g.b);
    bool lvalid = true;
    auto next_tile = [&]() {
      while (lvalid) {
        ++lj;
        int w, m0, n0;
        if (!tile_of(lj, &w, &m0, &n0)) { lvalid = false; break; }
        lnk = k_tiles(w);
        if (lnk == 0) continue;
        lk = 0;
        la = reinterpret_cast<const char*>(reinterpret_cast<const T*>(g.a[w]) + m0);
        lb = reinterpret_cast<const char*>(reinterpret_cast<const T*>(g.b) + g.row_off[w] * ldb + n0);
        break;
      }
    };
    next_tile();
    TileStage<T, XC, BM, BK, true> stA[4];
    TileStage<T, XC, BN, BK, true> stB[4];
    auto load_next = [&](auto& sa, auto& sb) {
      // past the end of the stream every lane reads the first vector of the first operand (one line)
      sa.load_at(adA, lvalid ? la : reinterpret_cast<const char*>(g.a[0]), lvalid ? 0xffffffffu : 0u);
      sb.load_at(adB, lvalid ? lb : reinterpret_cast<const char*>(g.b), lvalid ? 0xffffffffu : 0u);
      if (lvalid) {
        la += stepA;
        lb += stepB;
        if (++lk == lnk) next_tile();
      }
    };
#pragma unroll
    for (int u = 0; u < 4; ++u) load_next(stA[u], stB[u]);
    stA[0].template store_impl<false>(smem, tid);
    stB[0].template store_impl<false>(smem + WA, tid);
    load_next(stA[0], stB[0]);
    __syncthreads();                               // stream step 0 is in half 0
    for (int j = 0;; ++j) {
      int w, m0, n0;
      if (!tile_of(j, &w, &m0, &n0)) break;
      const int nk = k_tiles(w);
      for (int k = 0; k < nk; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          uint32_t* half = smem + ((u + 1) & 1) * WT;
          stA[(u + 1) & 3].template store_impl<false>(half, tid);
          stB[(u + 1) & 3].template store_impl<false>(half + WA, tid);
          load_next(stA[(u + 1) & 3], stB[(u + 1) & 3]);
          __syncthreads();
        }
      }
      float* Cw = reinterpret_cast<float*>(g.c[w]);
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        __syncthreads();
        read_out(ps, Cw, m0, n0);
      }
    }
  } else {
    __syncthreads();                               // stream step 0 is in half 0
    for (int j = 0;; ++j) {
      int w, m0, n0;
      if (!tile_of(j, &w, &m0, &n0)) break;
      const int nk = k_tiles(w);
      f32x16 acc[TM][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jj = 0; jj < TN; ++jj)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.0f;
      float colsum = 0.0f;
      const bool want_colsum = g.colsum_off >= 0 && m0 == 0;
      for (int k = 0; k < nk; k += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t* sA = smem + (u & 1) * WT;
          const uint32_t* sB = sA + WA;
          if (want_colsum && tid < BN) {   // column sums of the dZ tile, in row order
            if (sizeof(T) == 2) {
#pragma unroll 8
              for (int kp = 0; kp < BK / 2; ++kp) {
                const uint32_t wd = sB[kp * BN + tid];
                colsum += bf16_to_f32((uint16_t)(wd & 0xffffu));
                colsum += bf16_to_f32((uint16_t)(wd >> 16));
              }
            } else {
#pragma unroll 8
              for (int kk = 0; kk < BK; ++kk) colsum += __uint_as_float(sB[kk * BN + tid]);
            }
          }
          typename Frag<T, XC, BM, BK>::type fa[2][TM];
          typename Frag<T, XC, BN, BK>::type fb[2][TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) fa[0][i] = Frag<T, XC, BM, BK>::read(sA, wm * 64 + i * 32 + xi, 0, gk);
#pragma unroll
          for (int jj = 0; jj < TN; ++jj) fb[0][jj] = Frag<T, XC, BN, BK>::read(sB, wn * 64 + jj * 32 + xi, 0, gk);
#pragma unroll
          for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks + 1 < KSTEPS) {
#pragma unroll
              for (int i = 0; i < TM; ++i)
                fa[(ks + 1) & 1][i] = Frag<T, XC, BM, BK>::read(sA, wm * 64 + i * 32 + xi, ks + 1, gk);
#pragma unroll
              for (int jj = 0; jj < TN; ++jj)
                fb[(ks + 1) & 1][jj] = Frag<T, XC, BN, BK>::read(sB, wn * 64 + jj * 32 + xi, ks + 1, gk);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int jj = 0; jj < TN; ++jj) acc[i][jj] = mfma(fa[ks & 1][i], fb[ks & 1][jj], acc[i][jj]);
          }
          __syncthreads();
        }
      }
      // write-out, 64 rows at a time through the staging area (the producers keep
      // filling the operand halves meanwhile)
      float* Cw = reinterpret_cast<float*>(g.c[w]);
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        if (wm == (ps >> 1)) {
          float* buf = stage + (ps & 1) * 32 * BN;
#pragma unroll
          for (int jj = 0; jj < TN; ++jj) {
            float* sp = buf + (gk * 4) * BN + wn * 64 + jj * 32 + xi;
#pragma unroll
            for (int v = 0; v < 16; ++v) sp[((v >> 2) * 8 + (v & 3)) * BN] = acc[ps & 1][jj][v];
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        __syncthreads();
        read_out(ps, Cw, m0, n0);
      }
      if (want_colsum && tid < BN) Cw[g.colsum_off + n0 + tid] = colsum;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kGemmThreads, 4) void mlp_dw_persistent_kernel(GemmArgs g, int tiles_m,
                                                                            int tiles_n, int n_workers) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[dw_persistent_lds_words<T>()];
  dw_persistent_body<T>(g, tiles_m, tiles_n, n_workers, blockIdx.x, gridDim.x, smem);
}

// ------------------------------------------------------- small forward (fp32)
// H = act(X W + b) when the rows are so few that 64 x 64 tiles leave most of the chip idle and a
// workgroup walks the whole contraction alone (the tiny configuration: 16 tiles, 25 serial k-steps
// of 64-cycle fp32 MFMAs).  Plain multiply-adds instead, arranged so that a workgroup pays few memory
// latencies: 16 wavefronts own 8 rows x 64 columns; the 8 x rows go into LDS once; wavefront q takes
// the q-th sixteenth of the contraction, a lane one column, and asks for all its weights (one
// coalesced 256-byte row segment per k) before the first multiply-add, in batches of 48; an x value
// is an LDS read at one address for the whole wavefront.  The 16 partial sums meet in LDS and are
// added in wavefront order (bit-reproducible).
constexpr int kSmallRows = 8, kSmallCols = 64, kSmallWaves = 16, kSmallBatch = 56;
constexpr int kSmallMaxK = 2048;   // the x tile (8 rows) stays within 64 KB of LDS

template <int ROWS>
__global__ __launch_bounds__(64 * kSmallWaves) void mlp_fwd_small_kernel(GemmArgs g, int row_tiles, int col_tiles) {
  extern __shared__ __attribute__((aligned(16))) float small_lds[];
  const int K = (int)g.k_fixed;
  const int Kp = (K + 3) & ~3;                                 // x tile row pitch in LDS: [k][8 rows] is used instead
  float* xs = small_lds;                                       // [Kp][8]
  float* part = small_lds + (size_t)Kp * ROWS;           // [16][8][64]
  const int w = blockIdx.y;
  const int rt = blockIdx.x / col_tiles, ct = blockIdx.x % col_tiles;
  const int64_t rows_w = g.row_off[w + 1] - g.row_off[w];
  const int64_t r0 = (int64_t)rt * ROWS;
  if (r0 >= rows_w) return;                                    // uniform for the workgroup
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int64_t N = g.n;
  const int64_t n = (int64_t)ct * kSmallCols + lane;
  const bool col_ok = n < N;
  const float* X = reinterpret_cast<const float*>(g.a[w]);
  const float* W = reinterpret_cast<const float*>(g.b) + (col_ok ? n : 0);
  // input indexing folded in: the 8 rows come from the resident data through the index
  const bool gather = g.gather_src != nullptr;
  const float* xrow[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    const int64_t rr = r0 + r < rows_w ? r0 + r : r0;          // a row past the end repeats row r0
    if (gather) {
      int64_t src = g.gather_idx[g.row_off[w] + rr];
      if (src < 0 || src >= g.gather_rows) src = 0;
      xrow[r] = reinterpret_cast<const float*>(g.gather_src) + src * g.lda;
      if (ct == 0 && g.gather_labels && threadIdx.x == r && r0 + r < rows_w) g.gather_y[g.row_off[w] + rr] = g.gather_labels[src];
    } else {
      xrow[r] = X + rr * g.lda;
    }
  }
  // this wavefront's part of the contraction
  const int kc = (K + kSmallWaves - 1) / kSmallWaves;
  const int kb = q * kc, ke = kb + kc < K ? kb + kc : K;
  // its first batch of weights is asked for before the x tile is staged
  float wv[kSmallBatch];
#pragma unroll
  for (int u = 0; u < kSmallBatch; ++u) wv[u] = W[(int64_t)(kb + u < ke ? kb + u : (kb < K ? kb : 0)) * g.ldb];
  for (int k = threadIdx.x; k < K; k += 64 * kSmallWaves) {
    float xv[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) xv[r] = xrow[r][k];
    *reinterpret_cast<f32x4*>(xs + k * ROWS) = f32x4{xv[0], xv[1], xv[2], xv[3]};
    if (ROWS == 8) *reinterpret_cast<f32x4*>(xs + k * ROWS + 4) = f32x4{xv[ROWS - 4], xv[ROWS - 3], xv[ROWS - 2], xv[ROWS - 1]};
    // the rows are left in a[w] for the weight gradient: of a row tile's workgroups, column tile ct
    // copies the 64-wide column blocks ct, ct + col_tiles, ...
    if (gather && (k >> 6) % col_tiles == ct) {
      float* Xo = const_cast<float*>(X);
#pragma unroll
      for (int r = 0; r < ROWS; ++r)
        if (r0 + r < rows_w) Xo[(r0 + r) * g.lda + k] = xv[r];
    }
  }
  __syncthreads();
  float acc[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) acc[r] = 0.0f;
  for (int k0 = kb; k0 < ke; k0 += kSmallBatch) {
    if (k0 > kb) {
#pragma unroll
      for (int u = 0; u < kSmallBatch; ++u) wv[u] = W[(int64_t)(k0 + u < ke ? k0 + u : k0) * g.ldb];
    }
#pragma unroll
    for (int u = 0; u < kSmallBatch; ++u) {
      if (k0 + u < ke) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(xs + (k0 + u) * ROWS);
        acc[0] = fmaf(lo.x, wv[u], acc[0]); acc[1] = fmaf(lo.y, wv[u], acc[1]);
        acc[2] = fmaf(lo.z, wv[u], acc[2]); acc[3] = fmaf(lo.w, wv[u], acc[3]);
        if (ROWS == 8) {
          const f32x4 hi = *reinterpret_cast<const f32x4*>(xs + (k0 + u) * ROWS + 4);
          acc[ROWS - 4] = fmaf(hi.x, wv[u], acc[ROWS - 4]); acc[ROWS - 3] = fmaf(hi.y, wv[u], acc[ROWS - 3]);
          acc[ROWS - 2] = fmaf(hi.z, wv[u], acc[ROWS - 2]); acc[ROWS - 1] = fmaf(hi.w, wv[u], acc[ROWS - 1]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < ROWS; ++r) part[(q * ROWS + r) * kSmallCols + lane] = acc[r];
  __syncthreads();
  // wavefront r (< 8) finishes row r: the 16 partial sums in wavefront order
  if (q < ROWS && col_ok && r0 + q < rows_w) {
    float pv[kSmallWaves];
#pragma unroll
    for (int qq = 0; qq < kSmallWaves; ++qq) pv[qq] = part[(qq * ROWS + q) * kSmallCols + lane];
    float v = pv[0];
#pragma unroll
    for (int qq = 1; qq < kSmallWaves; ++qq) v += pv[qq];
    v += g.bias[n];
    if (g.relu) v = fmaxf(v, 0.0f);
    reinterpret_cast<float*>(g.c[w])[(r0 + q) * g.ldc + n] = v;
  }
}

static inline size_t fwd_small_lds_bytes(int64_t K, int rows) {
  return ((size_t)((K + 3) & ~(int64_t)3) * rows + (size_t)kSmallWaves * rows * kSmallCols) * 4;
}

// ------------------------------------------------------- narrow last layer dW
// dW_L[w] = H_{L-1}[w]^T dZ_L[w] and db_L[w] for a last layer of at most 16 outputs: a 10-column
// product leaves the matrix cores nothing to do and its rows (20 bytes) take no vector loads, so it is
// plain multiply-adds.  A workgroup of 512 threads owns one worker and KB = 128 (or 32) of the K inputs:
// thread (kk, rg) walks the rows rg, rg + RG, ... of the worker for input kk (RG = 512 / KB row groups),
// the row's dZ_L (padded to 16 floats) read from LDS at one address for all threads; the row groups
// are then added in a fixed order.
// The workgroup after the last one turns the row losses into the workers' slice-aggregated losses.
constexpr int kNarrowMaxC = 16, kNarrowKB = 128, kNarrowRows = 256;
constexpr int64_t kNarrowMaxRows = 1024;   // rows a worker may have: one workgroup walks them all for its 128 inputs
__host__ __device__ constexpr int dw_narrow_lds_words() { return kNarrowRows * 16 + 4 * 16 * kNarrowKB; }

// KB: inputs a workgroup owns, 128 or 32 (with few workers and inputs, 32: four times the workgroups,
// sixteen row groups instead of four)
static inline int dw_narrow_kb(int64_t K, int n_workers) {
  return n_workers * ((K + kNarrowKB - 1) / kNarrowKB) < 64 ? 32 : kNarrowKB;
}
static inline unsigned dw_narrow_blocks(int64_t K, int n_workers, int KB) {
  return (unsigned)(n_workers * ((K + KB - 1) / KB) + 1);
}

template <typename T>
__device__ __forceinline__ void dw_narrow_body(const GemmArgs& g, unsigned b, int n_workers, int KB,
                                               uint32_t* __restrict__ smem) {
  const int K = (int)g.m_fixed, C = (int)g.n;
  const int kb = (K + KB - 1) / KB;
  if (b >= (unsigned)(n_workers * kb)) {
    if (b == (unsigned)(n_workers * kb) && g.task_z >= 0) {
      float* s_mean = reinterpret_cast<float*>(smem);
      for (int ww = 0; ww < g.task_workers; ++ww)
        slice_loss_worker<kGemmThreads / 64>(g.task_row_loss, g.row_off, g.task_slices, g.task_op, ww, g.task_loss,
                                             s_mean);
    }
    return;
  }
  const int w = b / kb, k0 = (b % kb) * KB;
  const int RG = kGemmThreads / KB;                       // row groups: 4 or 16
  const int64_t rows_w = g.row_off[w + 1] - g.row_off[w];
  float* sdz = reinterpret_cast<float*>(smem);          // [kNarrowRows][16]: a chunk of the worker's dZ_L rows
  float* sred = sdz + kNarrowRows * 16;                 // [row groups][16][KB]
  const int t = threadIdx.x, kk = t % KB, rg = t / KB;
  const bool live = k0 + kk < K;
  const T* H = reinterpret_cast<const T*>(g.a[w]) + k0 + (live ? kk : 0);   // a dead thread reads input k0, unused
  const T* dZ = reinterpret_cast<const T*>(g.b) + g.row_off[w] * g.ldb;
  const bool want_colsum = g.colsum_off >= 0 && k0 == 0;
  float acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = 0.0f;
  float bsum = 0.0f;
  for (int64_t r0 = 0; r0 < rows_w; r0 += kNarrowRows) {
    const int nr = (int)(rows_w - r0 < kNarrowRows ? rows_w - r0 : kNarrowRows);
    __syncthreads();                                    // the chunk before has been used
    for (int e = t; e < nr * 16; e += kGemmThreads) {
      const int r = e >> 4, c = e & 15;
      sdz[e] = c < C ? to_f32(dZ[(r0 + r) * g.ldb + c]) : 0.0f;
    }
    // eight of this thread's rows at a time: the loads first, then the multiply-adds, in row order; the
    // first batch is asked for before the barrier that publishes the dZ chunk (rows past the end are
    // clamped into the chunk and not used)
    float h[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int r = rg + RG * u;
      h[u] = to_f32(H[(r0 + (r < nr ? r : nr - 1)) * g.lda]);
    }
    __syncthreads();                                    // the dZ chunk is in LDS
    for (int rb = rg; rb < nr; rb += 8 * RG) {
      if (rb != rg) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int r = rb + RG * u;
          h[u] = to_f32(H[(r0 + (r < nr ? r : nr - 1)) * g.lda]);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = rb + RG * u;
        if (r < nr) {
          const float* d = sdz + r * 16;
#pragma unroll
          for (int c = 0; c < 16; ++c) acc[c] = fmaf(h[u], d[c], acc[c]);
        }
      }
    }
    if (want_colsum && t < 16)
      for (int r = 0; r < nr; ++r) bsum += sdz[r * 16 + t];
  }
#pragma unroll
  for (int c = 0; c < 16; ++c) sred[(rg * 16 + c) * KB + kk] = acc[c];
  __syncthreads();
  float* Cw = reinterpret_cast<float*>(g.c[w]);
  if (rg == 0 && live) {
    for (int c = 0; c < C; ++c) {
      float v = sred[c * KB + kk];
      for (int q = 1; q < RG; ++q) v += sred[(q * 16 + c) * KB + kk];
      Cw[(int64_t)(k0 + kk) * g.ldc + c] = v;
    }
  }
  if (want_colsum && t < C) Cw[g.colsum_off + t] = bsum;
}

template <typename T>
__global__ __launch_bounds__(kGemmThreads) void mlp_dw_narrow_kernel(GemmArgs g, int n_workers, int KB) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[dw_narrow_lds_words()];
  dw_narrow_body<T>(g, blockIdx.x, n_workers, KB, smem);
}

// ------------------------------------------------------- backward group
// After the last-layer kernel both dZ_L and dZ_{L-1} exist, so dW_L, dW_{L-1}
// and dZ_{L-2} = (dZ_{L-1} W_{L-1}^T) * [H_{L-2} > 0] do not depend on one
// another: one launch holds the three grids (every kernel boundary costs a few
// microseconds of dispatch and drain, and none of the three fills the chip
// alone).  Each grid starts at a multiple of eight workgroups so that its
// workgroups keep their XCD phase.
struct GroupArgs {
  GemmArgs dwp;   // dW_{L-1}: the tile-walking kernel
  GemmArgs dx;    // dZ_{L-2}: 64 x 64 tiles
  GemmArgs dwl;   // dW_L (+ the slice losses): 64 x 64 tiles
  unsigned n_dwp, n_dx, n_dwl;          // workgroups of each grid (all but the last one multiples of 8)
  int dwl_narrow;                       // dW_L by the multiply-add kernel for narrow last layers
  unsigned dx_gx, dx_gy, dx_gz, dwl_gx, dwl_gy, dwl_gz;
  int tiles_m, tiles_n, n_workers;
  int dx_whole;                         // dZ_{L-2} by the whole-tile core: dx_gx x dx_gy tiles of 64 x 64 over all rows
};

constexpr int kGroupDxStages = 4;   // LDS ring of the whole-tile dX core inside the group: 64 KB, what the dW walker takes

template <typename T>
__host__ __device__ constexpr int group_lds_words() {
  constexpr int BKS = sizeof(T) == 2 ? 64 : 32;
  int m = dw_persistent_lds_words<T>();
  if (gemm_lds_words<T, MODE_DX, 64, 64, BKS>() > m) m = gemm_lds_words<T, MODE_DX, 64, 64, BKS>();
  if (gemm_lds_words<T, MODE_DW, 64, 64, BKS>() > m) m = gemm_lds_words<T, MODE_DW, 64, 64, BKS>();
  if (dw_narrow_lds_words() > m) m = dw_narrow_lds_words();
  if (sizeof(T) == 2 && gdma::lds_bytes<64, 64, kGroupDxStages>() / 4 > m) m = gdma::lds_bytes<64, 64, kGroupDxStages>() / 4;
  return m;
}

template <typename T, bool AL_B_LAST>
__global__ __launch_bounds__(kGemmThreads, 4) void mlp_backward_group_kernel(GroupArgs ga) {
  constexpr int BKS = sizeof(T) == 2 ? 64 : 32;
  __shared__ __attribute__((aligned(16))) uint32_t smem[group_lds_words<T>()];
  // Order of the parts = order in which workgroups get their place on the chip: the short ones first
  // (dW_L of a narrow last layer with the slice losses, then the dZ_{L-2} product the next launch waits
  // for), the tile walkers of dW_{L-1} beside and behind them.
  unsigned b = blockIdx.x;
  if (ga.dwl_narrow) {
    if (b < ga.n_dwl) {
      dw_narrow_body<T>(ga.dwl, b, ga.n_workers, kNarrowKB, smem);
      return;
    }
    b -= ga.n_dwl;
  }
  if (b < ga.n_dx) {
    if (sizeof(T) == 2 && ga.dx_whole) {
      if (b < ga.dx_gx * ga.dx_gy)
        gdma::tile<gdma::DX, 64, 64, kGroupDxStages>(ga.dx, b, (int)ga.dx_gy, (int)ga.dx_gx,
                                                     reinterpret_cast<unsigned char*>(smem));
    } else if (b < ga.dx_gx * ga.dx_gy * ga.dx_gz) {
      gemm_tile<T, MODE_DX, 64, 64, BKS, true, true>(ga.dx, b, ga.dx_gx, ga.dx_gy, ga.dx_gz, smem);
    }
    return;
  }
  b -= ga.n_dx;
  if (b < ga.n_dwp) {
    dw_persistent_body<T>(ga.dwp, ga.tiles_m, ga.tiles_n, ga.n_workers, b, ga.n_dwp, smem);
    return;
  }
  b -= ga.n_dwp;
  if (!ga.dwl_narrow && b < ga.dwl_gx * ga.dwl_gy * ga.dwl_gz)
    gemm_tile<T, MODE_DW, 64, 64, BKS, true, AL_B_LAST>(ga.dwl, b, ga.dwl_gx, ga.dwl_gy, ga.dwl_gz, smem);
}

// dW_L of a narrow last layer and dW_{L-1} in one launch (two-layer networks, where no dX lies between
// them: the last-layer kernel has already produced dZ_{L-1}).
struct PairArgs {
  GemmArgs narrow;   // dW_L (+ the slice losses)
  GemmArgs dw;       // dW_{L-1}: 64 x 64 tiles
  unsigned n_narrow; // workgroups of the first part, a multiple of 8
  unsigned gx, gy, gz;
  int n_workers, kb;
};

template <typename T>
__host__ __device__ constexpr int pair_lds_words() {
  constexpr int BKS = sizeof(T) == 2 ? 64 : 32;
  return dw_narrow_lds_words() > gemm_lds_words<T, MODE_DW, 64, 64, BKS>() ? dw_narrow_lds_words()
                                                                           : gemm_lds_words<T, MODE_DW, 64, 64, BKS>();
}

template <typename T>
__global__ __launch_bounds__(kGemmThreads, 2) void mlp_dw_pair_kernel(PairArgs pa) {
  constexpr int BKS = sizeof(T) == 2 ? 64 : 32;
  __shared__ __attribute__((aligned(16))) uint32_t smem[pair_lds_words<T>()];
  unsigned b = blockIdx.x;
  if (b < pa.n_narrow) {
    dw_narrow_body<T>(pa.narrow, b, pa.n_workers, pa.kb, smem);
    return;
  }
  b -= pa.n_narrow;
  if (b < pa.gx * pa.gy * pa.gz) gemm_tile<T, MODE_DW, 64, 64, BKS, true, true>(pa.dw, b, pa.gx, pa.gy, pa.gz, smem);
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

// ------------------------------------------------------------------ head
// Narrow last layer (at most kHeadMaxC classes), all in one kernel, one
// wavefront per row: logits = h W_L + b_L, softmax cross-entropy, dZ_L, and
// the back-propagated dZ_{L-1} = (dZ_L W_L^T) * [h > 0].  A 10-column GEMM
// would leave the matrix cores idle.  Each lane owns 8 consecutive features of
// the row; the 8 x C block of W_L that goes with them is contiguous in memory
// (W_L is [K x C] row-major), so it is read with 16-byte loads straight into
// registers and serves the forward and the backward product: no LDS, no
// barrier.
constexpr int kHeadMaxC = 16;
constexpr int kHeadRowsPerBlock = 4;
constexpr int kHeadCached = 2;   // 512-feature blocks of a row the last-layer kernel keeps in registers

struct HeadArgs {
  const int32_t* y[SYNK_MAX_WORKERS];
  int64_t row_off[SYNK_MAX_WORKERS + 1];
  const void* h;        // [R x K] activations below the last layer, in T
  const void* w;        // [K x C] in T, 16-byte aligned
  const float* bias;    // [C]
  void* dz;             // [R x C] in T
  void* dz_below;       // [R x K] in T
  float* row_loss;      // [R]
  int K;
  int n_slices, grad_op;
};

template <typename T> struct Vec8;   // 8 consecutive elements as floats
template <> struct Vec8<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
    const u32x4 q = *reinterpret_cast<const u32x4*>(p);
    v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
    v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
    v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
    u32x4 q;
    q.x = pack_bf16x2(v[0], v[1]); q.y = pack_bf16x2(v[2], v[3]);
    q.z = pack_bf16x2(v[4], v[5]); q.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<u32x4*>(p) = q;
  }
};
template <> struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float* v) {
    const f32x4 a = reinterpret_cast<const f32x4*>(p)[0], b = reinterpret_cast<const f32x4*>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    reinterpret_cast<f32x4*>(p)[0] = f32x4{v[0], v[1], v[2], v[3]};
    reinterpret_cast<f32x4*>(p)[1] = f32x4{v[4], v[5], v[6], v[7]};
  }
};
__device__ __forceinline__ float round_like(float v, float) { return v; }
__device__ __forceinline__ float round_like(float v, bf16_t) { return bf16_to_f32(f32_to_bf16(v)); }

// the 8 x C block of W_L for features [k0, k0+8): wv[j*C + c]
template <typename T, int C>
__device__ __forceinline__ void load_w_block(const T* __restrict__ W, int k0, float* wv) {
#pragma unroll
  for (int q = 0; q < C; ++q) Vec8<T>::load(W + (int64_t)k0 * C + q * 8, wv + q * 8);
}

template <typename T, int C>
__global__ __launch_bounds__(kMBlock) void mlp_head_kernel(HeadArgs a) {
  const int K = a.K;
  const T* Wg = reinterpret_cast<const T*>(a.w);
  const int w = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t rows_w = a.row_off[w + 1] - a.row_off[w];
  const int64_t r = (int64_t)blockIdx.x * kHeadRowsPerBlock + wave;
  if (r >= rows_w) return;
  const int64_t row = a.row_off[w] + r;
  const T* h = reinterpret_cast<const T*>(a.h) + row * K;
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

  // Up to kHeadCached * 512 features, a lane's features and weight blocks are
  // loaded once, all of them before the first use, and stay in registers for
  // the backward half (the kernel is a chain of memory round trips: this takes
  // two of the four out).  A lane's block past the end is read at the row's
  // last block and its features zeroed.
  constexpr int NIT = kHeadCached;
  const bool cached = K <= NIT * 512 && K >= 8;
  float hc[NIT][8], wc[NIT][8 * C];

  // forward: each lane accumulates its features' share of every logit
  float acc[C];
#pragma unroll
  for (int c = 0; c < C; ++c) acc[c] = 0.0f;
  if (cached) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int k0 = lane * 8 + it * 512;
      const int kc = k0 < K ? k0 : K - 8;
      Vec8<T>::load(h + kc, hc[it]);
      load_w_block<T, C>(Wg, kc, wc[it]);
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const bool in = lane * 8 + it * 512 < K;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        hc[it][j] = in ? hc[it][j] : 0.0f;
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = fmaf(hc[it][j], wc[it][j * C + c], acc[c]);
      }
    }
  } else {
    for (int k0 = lane * 8; k0 < K; k0 += 64 * 8) {
      float hv[8], wv[8 * C];
      Vec8<T>::load(h + k0, hv);
      load_w_block<T, C>(Wg, k0, wv);
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int c = 0; c < C; ++c) acc[c] = fmaf(hv[j], wv[j * C + c], acc[c]);
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int c = 0; c < C; ++c) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc[c] += __shfl_xor(acc[c], off);
    acc[c] += a.bias[c];
    m = fmaxf(m, acc[c]);
  }
  float ssum = 0.0f, xy = 0.0f;
#pragma unroll
  for (int c = 0; c < C; ++c) {
    ssum += expf(acc[c] - m);
    if (c == y) xy = acc[c];
  }
  if (lane == 0) a.row_loss[row] = (logf(ssum) + m) - xy;
  const float inv = 1.0f / ssum;
  T* dz = reinterpret_cast<T*>(a.dz) + row * C;
  float dzq[C];   // dZ_L as the GEMMs will read it back (rounded to T)
#pragma unroll
  for (int c = 0; c < C; ++c) {
    const float p = expf(acc[c] - m) * inv;
    dzq[c] = round_like((p - (c == y ? 1.0f : 0.0f)) * weight, T());
    if (lane == c) store_as(dz + c, dzq[c]);
  }
  if (a.dz_below == nullptr) return;

  // backward through the last layer, masked by the relu below
  T* dzb = reinterpret_cast<T*>(a.dz_below) + row * K;
  if (cached) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int k0 = lane * 8 + it * 512;
      if (k0 < K) {
        float dh[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float d = 0.0f;
#pragma unroll
          for (int c = 0; c < C; ++c) d = fmaf(dzq[c], wc[it][j * C + c], d);
          dh[j] = (hc[it][j] > 0.0f) ? d : 0.0f;
        }
        Vec8<T>::store(dzb + k0, dh);
      }
    }
    return;
  }
  for (int k0 = lane * 8; k0 < K; k0 += 64 * 8) {
    float hv[8], wv[8 * C], dh[8];
    Vec8<T>::load(h + k0, hv);
    load_w_block<T, C>(Wg, k0, wv);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float d = 0.0f;
#pragma unroll
      for (int c = 0; c < C; ++c) d = fmaf(dzq[c], wv[j * C + c], d);
      dh[j] = (hv[j] > 0.0f) ? d : 0.0f;
    }
    Vec8<T>::store(dzb + k0, dh);
  }
}

template <typename T>
static int launch_head(const HeadArgs& ha, int C, dim3 grid, hipStream_t s) {
#define SYNK_HEAD(CC) \
  case CC: SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_HEAD, (mlp_head_kernel<T, CC>), grid, dim3(kMBlock), 0, s, ha); break
  switch (C) {
    SYNK_HEAD(1); SYNK_HEAD(2); SYNK_HEAD(3); SYNK_HEAD(4); SYNK_HEAD(5); SYNK_HEAD(6); SYNK_HEAD(7);
    SYNK_HEAD(8); SYNK_HEAD(9); SYNK_HEAD(10); SYNK_HEAD(11); SYNK_HEAD(12); SYNK_HEAD(13); SYNK_HEAD(14);
    SYNK_HEAD(15); SYNK_HEAD(16);
    default: return SYNK_ERR_UNSUPPORTED;
  }
#undef SYNK_HEAD
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
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
  // the indexed call keeps the gathered rows (packed [R x d0] of T) and labels in the workspace too
  size_t xin, ylab, total_indexed;
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
    p->xin = o;
    o += round_up((size_t)p->R * p->d[0] * p->elem, 256);
    p->ylab = o;
    o += round_up((size_t)p->R * 4, 256);
    p->total_indexed = o;
  }
  return SYNK_OK;
}

template <typename T>
struct GemmTiling {
  static constexpr int BK_BIG = sizeof(T) == 2 ? 32 : 16, BK_SMALL = sizeof(T) == 2 ? 64 : 32;
};

// 128 x 128 tiles when they alone fill the chip, 64 x 64 otherwise
static inline int64_t big_tiles(const GemmArgs& g, int64_t m_max, int grid_z) {
  return ((m_max + 127) / 128) * ((g.n + 127) / 128) * grid_z;
}

// vector loads per operand: both (2), only A (1: e.g. a narrow last layer's dZ as B), or neither (0)
static inline int gemm_alignment(const GemmArgs& g) { return (g.a_vec && g.b_vec) ? 2 : (g.a_vec ? 1 : 0); }

// The tile-walking weight-gradient kernel applies: few rows per worker, in whole rounds of k-tiles.
template <typename T>
static bool dw_persistent_ok(const GemmArgs& g, int64_t m_max, int n_workers) {
  constexpr int BK = GemmTiling<T>::BK_BIG;
  if (!(big_tiles(g, m_max, n_workers) >= 2 * kNumCU && gemm_alignment(g) == 2 && g.c_vec && g.task_z < 0 &&
        m_max % 128 == 0 && g.n % 128 == 0))
    return false;
  for (int w = 0; w < n_workers; ++w) {
    const int64_t r = g.row_off[w + 1] - g.row_off[w];
    if (r % (4 * BK) != 0 || r > 16 * BK) return false;
  }
  return true;
}

static inline unsigned dw_persistent_blocks(const GemmArgs& g, int64_t m_max, int n_workers) {
  const int64_t big = big_tiles(g, m_max, n_workers);
  int64_t blocks = big < 2 * kNumCU ? big : 2 * kNumCU;
  if (big % 8 == 0) blocks = blocks / 8 * 8;
  return (unsigned)blocks;
}

// The whole-tile bf16 core applies (forward and dX): every worker holds whole tiles of rows, the
// contraction is whole 64-deep tiles, everything takes 16-byte accesses, bf16 in and out.
template <typename T, int MODE>
static bool gemm_dma_ok(const GemmArgs& g, int n_workers, int bm, int bn) {
  if (sizeof(T) != 2 || MODE == MODE_DW) return false;
  if (gemm_alignment(g) != 2 || !g.c_vec) return false;
  if (MODE == MODE_FWD && g.out_f32) return false;
  if (g.k_fixed < 64 || g.k_fixed % 64 != 0 || g.n % bn != 0) return false;
  if (g.lda % 8 != 0 || g.ldb % 8 != 0 || g.ldc % 8 != 0 || (MODE == MODE_DX && g.ldmask % 8 != 0)) return false;
  if (g.row_off[n_workers] > (1 << 30) / 64) return false;      // tile indexes stay small integers
  for (int w = 0; w < n_workers; ++w) {
    const int64_t r = g.row_off[w + 1] - g.row_off[w];
    if (r % bm != 0) return false;
    if (r > 0 && (!aligned_to(g.a[w], 16) || !aligned_to(g.c[w], 16))) return false;
  }
  return true;
}

// Which whole-tile kernel a forward or dX product takes: 0 none, else 1 = 256 x 128, 2 = 128 x 128,
// 3 = 64 x 64.  Large products: the operand fetch rate of a CU bounds them, so the tile with the most
// flops per fetched byte that still fills the chip: 256 x 128 (36 % of the bf16 peak at 65,536 x 1024
// x 3072 against 31 % for 128 x 128).
template <typename T, int MODE>
static int gemm_dma_choice(const GemmArgs& g, int n_workers) {
  if (MODE == MODE_DW) return 0;
  const int64_t R = g.row_off[n_workers];
  if (gemm_dma_ok<T, MODE>(g, n_workers, 256, 128) && (R / 256) * (g.n / 128) >= 4 * kNumCU) return 1;
  if (gemm_dma_ok<T, MODE>(g, n_workers, 128, 128) && (R / 128) * (g.n / 128) >= 2 * kNumCU) return 2;
  if (gemm_dma_ok<T, MODE>(g, n_workers, 64, 64)) return 3;
  return 0;
}

template <typename T, int MODE>
static int launch_gemm(const GemmArgs& g, int64_t m_max, int n_workers, hipStream_t s, int prof_id) {
  constexpr int BK_BIG = GemmTiling<T>::BK_BIG, BK_SMALL = GemmTiling<T>::BK_SMALL;
  const int64_t big = big_tiles(g, m_max, n_workers);
  const int al = gemm_alignment(g);
  if (MODE != MODE_DW) {
    constexpr int GM = MODE == MODE_FWD ? gdma::FWD : gdma::DX;
    constexpr bool CAN_GATHER = MODE == MODE_FWD;
    const int64_t R = g.row_off[n_workers];
    const int choice = gemm_dma_choice<T, MODE>(g, n_workers);
    const bool gather = g.gather_src != nullptr;
    if (gather && (!CAN_GATHER || choice == 0)) return SYNK_ERR_UNSUPPORTED;   // the caller gathers first in that case
#define SYNK_GEMM_DMA(BM_, BN_, NS_)                                                                         \
  do {                                                                                                       \
    const int tm = (int)(R / BM_), tn = (int)(g.n / BN_);                                                    \
    if (CAN_GATHER && gather)                                                                                \
      SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_gemm_dma_kernel<GM, BM_, BN_, NS_, CAN_GATHER>),                    \
                           dim3((unsigned)(tm * tn)), dim3(gdma::kThreads), 0, s, g, tm, tn);                \
    else                                                                                                     \
      SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_gemm_dma_kernel<GM, BM_, BN_, NS_>), dim3((unsigned)(tm * tn)),     \
                           dim3(gdma::kThreads), 0, s, g, tm, tn);                                           \
    SYNK_LAUNCH_CHECK();                                                                                     \
    return SYNK_OK;                                                                                          \
  } while (0)
    if (choice == 1) SYNK_GEMM_DMA(256, 128, 3);
    if (choice == 2) SYNK_GEMM_DMA(128, 128, 3);
    if (choice == 3) SYNK_GEMM_DMA(64, 64, 6);
#undef SYNK_GEMM_DMA
  }
  if (g.gather_src != nullptr) return SYNK_ERR_UNSUPPORTED;
#define SYNK_GEMM(BM_, BN_, BK_)                                                                              \
  do {                                                                                                       \
    if (al == 2)                                                                                             \
      SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_gemm_kernel<T, MODE, BM_, BN_, BK_, true, true>), grid,             \
                           dim3(kGemmThreads), 0, s, g);                                                     \
    else if (al == 1)                                                                                        \
      SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_gemm_kernel<T, MODE, BM_, BN_, BK_, true, false>), grid,            \
                           dim3(kGemmThreads), 0, s, g);                                                     \
    else                                                                                                     \
      SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_gemm_kernel<T, MODE, BM_, BN_, BK_, false, false>), grid,           \
                           dim3(kGemmThreads), 0, s, g);                                                     \
  } while (0)
  if (MODE == MODE_DW && dw_persistent_ok<T>(g, m_max, n_workers)) {
    SYNK_LAUNCH_TIMED_AS(prof_id, (mlp_dw_persistent_kernel<T>), dim3(dw_persistent_blocks(g, m_max, n_workers)),
                         dim3(kGemmThreads), 0, s, g, (int)(m_max / 128), (int)(g.n / 128), n_workers);
    SYNK_LAUNCH_CHECK();
    return SYNK_OK;
  }
  if (big >= 2 * kNumCU) {
    const dim3 grid((unsigned)((g.n + 127) / 128), (unsigned)((m_max + 127) / 128), n_workers);
    SYNK_GEMM(128, 128, BK_BIG);
  } else {
    const dim3 grid((unsigned)((g.n + 63) / 64), (unsigned)((m_max + 63) / 64), n_workers);
    SYNK_GEMM(64, 64, BK_SMALL);
  }
#undef SYNK_GEMM
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

// The resident dataset and the index list of the indexed call (Sec. 5.2).
struct GatherIn {
  const void* data;        // [n_data x d0] of T
  const int32_t* labels;   // [n_data]
  int64_t n_data;
  const int32_t* idx;      // [R]
};

// gin == nullptr: x[w], y[w] hold the workers' rows and labels.  Otherwise they are buffers the call
// fills from the dataset first (the first forward product does it on its way where its kernel can,
// else a gather launch of its own).
template <typename T>
static int run_sliced_grad(const MlpPlan& p, const float* params, const void* params_lp,
                           const void* const* x, const int32_t* const* y, const int64_t* rows,
                           int n_workers, int n_slices, int grad_op, float* const* grad,
                           float* loss, char* ws, hipStream_t s, const GatherIn* gin = nullptr) {
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

  GemmArgs g;
  g.gather_src = nullptr;
  g.gather_idx = g.gather_labels = nullptr;
  g.gather_rows = 0;
  g.gather_y = nullptr;
  g.task_z = -1;
  g.task_workers = g.task_slices = g.task_op = 0;
  g.task_row_loss = nullptr;
  g.task_loss = nullptr;
  for (int w = 0; w <= n_workers; ++w) g.row_off[w] = p.row_off[w];
  for (int w = n_workers + 1; w <= SYNK_MAX_WORKERS; ++w) g.row_off[w] = p.R;

  // The narrow-last-layer kernel replaces the last forward GEMM, the softmax
  // kernel and the last dX GEMM when the layer fits it.
  const bool use_head = L >= 2 && p.d[L] <= kHeadMaxC && p.d[L - 1] % 8 == 0 &&
                        aligned_to(wts + p.offW[L - 1], 16);

  const int n_fwd = use_head ? L - 1 : L;

  // ---- forward (layer index l = 1..L, weights W_l = [d_{l-1} x d_l])
  for (int l = 1; l <= n_fwd; ++l) {
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
    g.c_vec = N % 8 == 0;     // workspace rows: 256-byte aligned base, rows a multiple of 16 bytes
    const int fwd_id = l == 1 ? SYNK_KERNEL_MAIN : SYNK_KERNEL_MLP_FORWARD(l);
    // fp32 with so few rows that 64 x 64 tiles would occupy under a quarter of the CUs: multiply-add kernel
    const bool small = sizeof(T) == 4 && K <= kSmallMaxK &&
                       ((p.max_rows + 63) / 64) * ((N + 63) / 64) * n_workers < kNumCU / 4;
    if (l == 1 && gin) {
      // input indexing: on the way into this product where its kernel reads rows through the index,
      // else gathered by a launch of its own
      const bool fused = small || (aligned_to(gin->data, 16) && gemm_dma_choice<T, MODE_FWD>(g, n_workers) != 0);
      if (fused) {
        g.gather_src = gin->data;
        g.gather_idx = gin->idx;
        g.gather_labels = gin->labels;
        g.gather_rows = gin->n_data;
        g.gather_y = const_cast<int32_t*>(y[0]);   // packed labels: y[w] = y[0] + row_off[w] in the indexed call
      } else {
        const int dt = sizeof(T) == 4 ? SYNK_F32 : SYNK_BF16;
        ProfileHold hold;   // a pending event pair is for the forward product, not for the gather
        if (int rc = synk_gather_rows(gin->data, gin->n_data, K, dt, gin->idx, p.R, const_cast<void* const*>(x), n_workers,
                                      dt, nullptr, 0, gin->labels, const_cast<int32_t* const*>(y), 0, nullptr, 0, s))
          return rc;
      }
    }
    if (small) {
      // 8 rows a workgroup, or 4 when that leaves most CUs without one (a row's sum is the same either way)
      const int col_tiles = (int)((N + kSmallCols - 1) / kSmallCols);
      const bool four = ((p.max_rows + 7) / 8) * col_tiles * n_workers < kNumCU;
      const int rows_wg = four ? 4 : kSmallRows;
      const int row_tiles = (int)((p.max_rows + rows_wg - 1) / rows_wg);
      if (four)
        SYNK_LAUNCH_TIMED_AS(fwd_id, mlp_fwd_small_kernel<4>, dim3((unsigned)(row_tiles * col_tiles), n_workers),
                             dim3(64 * kSmallWaves), fwd_small_lds_bytes(K, 4), s, g, row_tiles, col_tiles);
      else
        SYNK_LAUNCH_TIMED_AS(fwd_id, mlp_fwd_small_kernel<8>, dim3((unsigned)(row_tiles * col_tiles), n_workers),
                             dim3(64 * kSmallWaves), fwd_small_lds_bytes(K, 8), s, g, row_tiles, col_tiles);
      SYNK_LAUNCH_CHECK();
      g.gather_src = nullptr;
      continue;
    }
    if (int rc = launch_gemm<T, MODE_FWD>(g, p.max_rows, n_workers, s, fwd_id)) return rc;
    g.gather_src = nullptr;
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
  if (use_head) {
    HeadArgs ha;
    for (int w = 0; w < n_workers; ++w) ha.y[w] = y[w];
    for (int w = 0; w <= SYNK_MAX_WORKERS; ++w) ha.row_off[w] = g.row_off[w];
    ha.h = act(L - 1);
    ha.w = wts + p.offW[L - 1];
    ha.bias = params + p.offB[L - 1];
    ha.dz = dzp(L);
    ha.dz_below = dzp(L - 1);
    ha.row_loss = row_loss;
    ha.K = (int)p.d[L - 1];
    ha.n_slices = n_slices;
    ha.grad_op = grad_op;
    const dim3 grid((unsigned)((p.max_rows + kHeadRowsPerBlock - 1) / kHeadRowsPerBlock), n_workers);
    if (int rc = launch_head<T>(ha, (int)p.d[L], grid, s)) return rc;
  } else {
    const dim3 grid((unsigned)((p.max_rows + kCeRowsPerBlock - 1) / kCeRowsPerBlock), n_workers);
    SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_HEAD, (softmax_ce_kernel<T>), grid, dim3(kMBlock), 0, s, ce);
    SYNK_LAUNCH_CHECK();
  }

  // ---- backward
  // dW_l[w] = H_{l-1}[w]^T dZ_l[w]; db_l[w] = column sums of dZ_l[w]
  auto fill_dw = [&](GemmArgs& q, int l, bool with_loss) {
    const int64_t K = p.d[l - 1], N = p.d[l];
    for (int w = 0; w < n_workers; ++w) {
      // a worker without rows still gets a block (it writes the zero gradient); its
      // operand pointer must be readable because loads are issued unconditionally
      q.a[w] = l == 1 ? (rows[w] > 0 ? x[w] : (const void*)ws)
                      : (const void*)(act(l - 1) + p.row_off[w] * K);
      q.c[w] = grad[w] + p.offW[l - 1];
    }
    q.b = dzp(l);
    q.mask = nullptr;
    q.bias = nullptr;
    q.m_fixed = K;
    q.n = N;
    q.k_fixed = 0;
    q.lda = K; q.ldb = N; q.ldc = N; q.ldmask = 0;
    q.colsum_off = p.offB[l - 1] - p.offW[l - 1];
    q.relu = 0;
    q.out_f32 = 1;
    q.a_vec = (K % V == 0) && (l == 1 ? x_vec : true);
    q.b_vec = (N % V == 0);
    q.c_vec = grad_al && N % 4 == 0 && p.offW[l - 1] % 4 == 0;
    // the first kernel after the row losses exist also aggregates them over slices (one more grid slice)
    q.task_z = with_loss ? n_workers : -1;
    q.task_workers = n_workers;
    q.task_slices = n_slices;
    q.task_op = grad_op;
    q.task_row_loss = row_loss;
    q.task_loss = loss;
  };
  // dZ_{l-1} = (dZ_l W_l^T) * [H_{l-1} > 0]
  auto fill_dx = [&](GemmArgs& q, int l) {
    const int64_t K = p.d[l - 1], N = p.d[l];
    const T* W = wts + p.offW[l - 1];
    for (int w = 0; w < n_workers; ++w) {
      q.a[w] = dzp(l) + p.row_off[w] * N;
      q.c[w] = dzp(l - 1) + p.row_off[w] * K;
    }
    q.b = W;
    q.mask = act(l - 1);
    q.bias = nullptr;
    q.m_fixed = 0;
    q.n = K;          // output columns = fan-in of layer l
    q.k_fixed = N;    // contraction over the layer's outputs
    q.lda = N; q.ldb = N; q.ldc = K; q.ldmask = K;
    q.colsum_off = -1;
    q.relu = 0;
    q.a_vec = (N % V == 0);
    q.b_vec = (N % V == 0) && aligned_to(W, 16);
    q.c_vec = K % 8 == 0;
    q.out_f32 = 0;
    q.task_z = -1;
  };

  int l = L;
  if (use_head && L >= 3) {
    // dZ_L and dZ_{L-1} both exist: dW_L, dW_{L-1} and dZ_{L-2} in one launch when each takes the
    // tiling the group kernel holds
    GroupArgs ga;
    ga.dwl = g; ga.dwp = g; ga.dx = g;
    fill_dw(ga.dwl, L, true);
    fill_dw(ga.dwp, L - 1, false);
    fill_dx(ga.dx, L - 1);
    const int al_last = gemm_alignment(ga.dwl);
    ga.dwl_narrow = (p.d[L] <= kNarrowMaxC && p.max_rows <= kNarrowMaxRows) ? 1 : 0;
    const bool ok = (ga.dwl_narrow || (al_last >= 1 && big_tiles(ga.dwl, p.d[L - 1], n_workers + 1) < 2 * kNumCU)) &&
                    dw_persistent_ok<T>(ga.dwp, p.d[L - 2], n_workers) && gemm_alignment(ga.dx) == 2 &&
                    big_tiles(ga.dx, p.max_rows, n_workers) < 2 * kNumCU;
    if (ok) {
      ga.n_dwp = dw_persistent_blocks(ga.dwp, p.d[L - 2], n_workers);
      ga.tiles_m = (int)(p.d[L - 2] / 128);
      ga.tiles_n = (int)(p.d[L - 1] / 128);
      ga.n_workers = n_workers;
      ga.dx_whole = gemm_dma_ok<T, MODE_DX>(ga.dx, n_workers, 64, 64) ? 1 : 0;
      ga.dx_gx = (unsigned)((ga.dx.n + 63) / 64);
      if (ga.dx_whole) {
        ga.dx_gy = (unsigned)(p.R / 64);           // row tiles over all workers' packed rows
        ga.dx_gz = 1u;
      } else {
        ga.dx_gy = (unsigned)((p.max_rows + 63) / 64);
        ga.dx_gz = (unsigned)n_workers;
      }
      ga.n_dx = (ga.dx_gx * ga.dx_gy * ga.dx_gz + 7u) / 8u * 8u;
      ga.dwl_gx = (unsigned)((ga.dwl.n + 63) / 64);
      ga.dwl_gy = (unsigned)((p.d[L - 1] + 63) / 64);
      ga.dwl_gz = (unsigned)(n_workers + 1);
      ga.n_dwl = ga.dwl_narrow ? (dw_narrow_blocks(p.d[L - 1], n_workers, kNarrowKB) + 7u) / 8u * 8u
                               : ga.dwl_gx * ga.dwl_gy * ga.dwl_gz;
      const dim3 grid(ga.n_dx + ga.n_dwp + ga.n_dwl);
      if (al_last == 2)
        SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_BACKWARD_GROUP, (mlp_backward_group_kernel<T, true>), grid,
                             dim3(kGemmThreads), 0, s, ga);
      else
        SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_BACKWARD_GROUP, (mlp_backward_group_kernel<T, false>), grid,
                             dim3(kGemmThreads), 0, s, ga);
      SYNK_LAUNCH_CHECK();
      l = L - 2;
    }
  }
  for (; l >= 1; --l) {
    fill_dw(g, l, l == L);
    if (l == L && p.d[L] <= kNarrowMaxC && p.max_rows <= kNarrowMaxRows) {
      const int KB = dw_narrow_kb(p.d[L - 1], n_workers);
      if (use_head && l >= 2) {
        // no dX of layer L is needed (the last-layer kernel made dZ_{L-1}): dW_{L-1} shares the launch when it
        // takes 64 x 64 tiles with vector loads
        PairArgs pa;
        pa.narrow = g;
        pa.dw = g;
        fill_dw(pa.dw, l - 1, false);
        if (gemm_alignment(pa.dw) == 2 && !dw_persistent_ok<T>(pa.dw, p.d[l - 2], n_workers) &&
            big_tiles(pa.dw, p.d[l - 2], n_workers) < 2 * kNumCU) {
          pa.n_narrow = (dw_narrow_blocks(p.d[L - 1], n_workers, KB) + 7u) / 8u * 8u;
          pa.gx = (unsigned)((pa.dw.n + 63) / 64);
          pa.gy = (unsigned)((p.d[l - 2] + 63) / 64);
          pa.gz = (unsigned)n_workers;
          pa.n_workers = n_workers;
          pa.kb = KB;
          SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_BACKWARD_GROUP, (mlp_dw_pair_kernel<T>),
                               dim3(pa.n_narrow + pa.gx * pa.gy * pa.gz), dim3(kGemmThreads), 0, s, pa);
          SYNK_LAUNCH_CHECK();
          g.task_z = -1;
          if (l - 1 > 1) {
            fill_dx(g, l - 1);
            if (int rc = launch_gemm<T, MODE_DX>(g, p.max_rows, n_workers, s, SYNK_KERNEL_MLP_DX(l - 1))) return rc;
          }
          --l;          // layer l-1 is done too
          continue;
        }
      }
      SYNK_LAUNCH_TIMED_AS(SYNK_KERNEL_MLP_DW(l), (mlp_dw_narrow_kernel<T>), dim3(dw_narrow_blocks(p.d[L - 1], n_workers, KB)),
                           dim3(kGemmThreads), 0, s, g, n_workers, KB);
      SYNK_LAUNCH_CHECK();
      g.task_z = -1;
      if (l > 1 && !use_head) {
        fill_dx(g, l);
        if (int rc = launch_gemm<T, MODE_DX>(g, p.max_rows, n_workers, s, SYNK_KERNEL_MLP_DX(l))) return rc;
      }
      continue;
    }
    if (int rc = launch_gemm<T, MODE_DW>(g, p.d[l - 1], n_workers + (l == L ? 1 : 0), s, SYNK_KERNEL_MLP_DW(l)))
      return rc;
    g.task_z = -1;
    if (l > 1 && !(use_head && l == L)) {
      fill_dx(g, l);
      if (int rc = launch_gemm<T, MODE_DX>(g, p.max_rows, n_workers, s, SYNK_KERNEL_MLP_DX(l))) return rc;
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

extern "C" int synk_sliced_grad_indexed_workspace_bytes(const synk_mlp_desc* m, int64_t n_idx, int n_workers,
                                                        size_t* bytes) {
  if (!bytes) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_idx < 1) return SYNK_ERR_SHAPE;
  int64_t rows[SYNK_MAX_WORKERS];
  for (int w = 0; w < n_workers; ++w) {
    int64_t start;
    share(n_idx, n_workers, w, &start, &rows[w]);
  }
  MlpPlan p;
  if (int rc = make_plan(m, rows, n_workers, &p)) return rc;
  *bytes = p.total_indexed;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_indexed(const synk_mlp_desc* m, const float* params, const void* params_lp,
                                        const void* data, const int32_t* labels, int64_t n_data,
                                        const int32_t* idx, int64_t n_idx, int n_workers, int n_slices,
                                        int grad_op, float* const* grad, float* loss, void* ws,
                                        size_t ws_bytes, void* stream) {
  if (!m || !params || !data || !labels || !idx || !grad || !loss) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_idx < 1 || n_data < 1) return SYNK_ERR_SHAPE;
  int64_t rows[SYNK_MAX_WORKERS];
  for (int w = 0; w < n_workers; ++w) {
    int64_t start;
    share(n_idx, n_workers, w, &start, &rows[w]);
  }
  MlpPlan p;
  if (int rc = make_plan(m, rows, n_workers, &p)) return rc;
  if (n_slices < 1) return SYNK_ERR_SHAPE;
  if (grad_op != SYNK_SUM && grad_op != SYNK_MEAN) return SYNK_ERR_OP;
  if (m->compute_dtype == SYNK_BF16 && !params_lp) return SYNK_ERR_NULL;
  if (!aligned_to(params, 4) || !aligned_to(loss, 4) || !aligned_to(data, p.elem) || !aligned_to(labels, 4) ||
      !aligned_to(idx, 4))
    return SYNK_ERR_ALIGN;
  if (m->compute_dtype == SYNK_BF16 && !aligned_to(params_lp, 2)) return SYNK_ERR_ALIGN;
  for (int w = 0; w < n_workers; ++w) {
    if (!grad[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grad[w], 4)) return SYNK_ERR_ALIGN;
  }
  if (!ws || !aligned_to(ws, 256) || ws_bytes < p.total_indexed) return SYNK_ERR_WORKSPACE;
  // the workers' gathered rows and labels live in the workspace, packed in worker order
  char* wsb = reinterpret_cast<char*>(ws);
  const void* x[SYNK_MAX_WORKERS];
  const int32_t* y[SYNK_MAX_WORKERS];
  for (int w = 0; w < n_workers; ++w) {
    x[w] = wsb + p.xin + (size_t)p.row_off[w] * p.d[0] * p.elem;
    y[w] = reinterpret_cast<const int32_t*>(wsb + p.ylab) + p.row_off[w];
  }
  const GatherIn gin{data, labels, n_data, idx};
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (m->compute_dtype == SYNK_F32)
    return run_sliced_grad<float>(p, params, params_lp, x, y, rows, n_workers, n_slices, grad_op, grad, loss, wsb,
                                  s, &gin);
  return run_sliced_grad<bf16_t>(p, params, params_lp, x, y, rows, n_workers, n_slices, grad_op, grad, loss, wsb, s,
                                 &gin);
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
