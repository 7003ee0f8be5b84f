// bf16 GEMM core for the forward (H W) and input-gradient (dZ W^T) contractions
// of the MLP (Sec. 3.3 step 1) at shapes that are whole tiles.
//
// Operand tiles go from global memory straight into LDS (global_load_lds, 16
// bytes a lane, no registers and no LDS store instructions), in the layout they
// have in memory; which 16-byte piece a lane fetches is chosen so that the
// fragment reads below meet no bank conflict (an XOR swizzle of the piece index
// with the row).  A wavefront's MFMA fragment of an operand whose contraction
// index is contiguous in memory is one 16-byte LDS read; of an operand whose
// contraction index is strided (the weights in the forward product) it is two
// LDS transpose reads (ds_read_b64_tr_b16: a 16-lane group reads 4 rows x 16
// columns and every lane receives one column).
//
// Eight wavefronts: wavefront (q, h) owns quadrant q of the BM x BN tile for
// half h of every 64-deep k tile; the two halves' partial sums meet in LDS once,
// at the end, always added in the same order (results are bit-reproducible).
// A ring of NS stages in LDS keeps NS-1 tiles in flight; one barrier a tile.
#pragma once
#include "common.h"

namespace synk {
namespace gdma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int kBK = 64;        // contraction depth of a tile
constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;

enum { FWD = 0, DX = 1 };

// 16 bytes a lane from global memory straight into LDS at lds_addr + lane*16
// (lds_addr wave-uniform).  Assembly, so that the compiler does not order later
// LDS reads behind it: completion is waited for by hand (vmcnt).  The instruction
// takes the LDS address from M0, a register the compiler manages: its value is
// put back before the statement ends.
__device__ __forceinline__ void load_to_lds16(const void* gptr, unsigned lds_addr) {
  unsigned saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %2\n\t"
      "global_load_lds_dwordx4 %1, off\n\t"
      "s_nop 0\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "v"(gptr), "s"(lds_addr)
      : "memory");
}

// swizzle of a row whose contraction index is contiguous (rows of 128 bytes, 8 pieces)
__device__ __forceinline__ int swz_kc(int r) { return (r & 7) ^ ((r >> 3) & 1); }
// swizzle of a row of the strided operand: rows of BN*2 bytes
template <int BN>
__device__ __forceinline__ int swz_xc(int r) {
  if (BN == 64) return 2 * (r & 3);
  const int t = r & 3;
  return t == 0 ? 0 : (t == 1 ? 4 : (t == 2 ? 10 : 14));
}

template <int BM, int BN, int NS>
__host__ __device__ constexpr int lds_bytes() { return NS * (BM + BN) * 128; }

// The argument block (ArgsT below) is the caller's: it has, per worker w, the A operand base a[w]
// ([rows_w x K] bf16, row pitch lda) and the output base c[w] ([rows_w x N] bf16, pitch ldc);
// row_off[0..SYNK_MAX_WORKERS] (first packed row of each worker, entries past the last worker
// equal to the total); b (FWD: W [K x N], n contiguous; DX: W [N x K], k contiguous; pitch ldb);
// mask (DX: activations of the layer below, packed [R x N] bf16, pitch ldmask); bias (FWD:
// float[N]); n (output columns); k_fixed (contraction length); relu (FWD).
// With GATHER (FWD only) the A rows are not in a[w] yet: row r of the packed batch is row
// gather_idx[r] of gather_src ([gather_rows x K] bf16, pitch lda; an index outside
// [0, gather_rows) reads row 0), and the kernel leaves the rows in a[w] for the kernels after it
// (of a row tile's workgroups, the one in tile column bn copies the k tiles t with
// t % tiles_n == bn, from its own LDS pieces while they are there) and their labels
// gather_labels[gather_idx[r]] in gather_y[r] (tile column 0; gather_labels may be null).
// Measured at 1024 x 3072 -> 1024 (forward product 16.9 us with the rows already in a[w]):
// 19.1 us this way; 20.5 with the copy after the main loop (loads before the k halves meet,
// stores after the output); 25-27 with copy workgroups appended to the launch (they need
// the product's LDS allocation too, so they run after it instead of beside it); a gather
// launch of its own takes 7.4.

// Workgroup `lin` of a grid of tiles_m x tiles_n tiles whose first workgroup sits
// on XCD 0 (workgroups go to the 8 XCDs round-robin): each XCD, i.e. each L2,
// gets a compact block of tiles.  The 8 XCDs are arranged xr x xc over the tile
// grid (xr * xc = 8, both dividing the grid) so that the operand rows an XCD
// fetches, (tiles_m / xr) * BM of A plus (tiles_n / xc) * BN of B, are fewest.
template <int BM, int BN>
__device__ __forceinline__ void tile_of(unsigned lin, int tiles_m, int tiles_n, int* bm, int* bn) {
  int best_xr = 0;
  long best = -1;
#pragma unroll
  for (int xr = 1; xr <= 8; xr *= 2) {
    const int xc = 8 / xr;
    if (tiles_m % xr == 0 && tiles_n % xc == 0) {
      const long cost = (long)(tiles_m / xr) * BM + (long)(tiles_n / xc) * BN;
      if (best < 0 || cost < best) { best = cost; best_xr = xr; }
    }
  }
  if (best_xr == 0) {            // the grid does not divide over 8 XCDs: plain order
    *bm = lin / tiles_n;
    *bn = lin % tiles_n;
    return;
  }
  const int xr = best_xr, xc = 8 / xr;
  const int xcd = lin & 7, idx = lin >> 3;
  const int bh = tiles_m / xr, bw = tiles_n / xc;
  *bm = (xcd / xc) * bh + idx / bw;
  *bn = (xcd % xc) * bw + idx % bw;
}

// One BM x BN output tile.  Preconditions (checked on the host): K % 64 == 0,
// N % BN == 0, every worker's row count a multiple of BM, all bases 16-byte
// aligned and all pitches multiples of 8 elements.  smem: lds_bytes<BM,BN,NS>()
// bytes, 1024-byte aligned.  Called by all kThreads threads of a workgroup.
template <int MODE, int BM, int BN, int NS, typename ArgsT, bool GATHER = false>
__device__ __forceinline__ void tile(const ArgsT& g, unsigned lin, int tiles_m, int tiles_n,
                                     unsigned char* __restrict__ smem) {
  static_assert(!GATHER || MODE == FWD, "input indexing belongs to the forward product");
  constexpr int TM = BM / 64, TN = BN / 64;            // MFMA tiles of a quadrant
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  constexpr int A_INSTR = A_BYTES / 1024 / kWaves, B_INSTR = B_BYTES / 1024 / kWaves;
  constexpr int PER_TILE = A_INSTR + B_INSTR;          // direct loads a wavefront issues per tile
  static_assert(A_INSTR >= 1 && B_INSTR >= 1, "tile too small for eight wavefronts");
  static_assert(NS >= 3 && NS * STAGE >= BM * BN * 4, "partial sums of one k half must fit in LDS");
  static_assert(NS * STAGE >= 64 * BN * 2, "output staging must fit");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wq = wave & 3, kh = wave >> 2;             // quadrant, k half
  const int wm = wq >> 1, wn = wq & 1;
  const int x = lane & 31, gk = lane >> 5;
  int bm, bn;
  tile_of<BM, BN>(lin, tiles_m, tiles_n, &bm, &bn);
  const int64_t row0 = (int64_t)bm * BM;               // first packed row of the tile
  const int n0 = bn * BN;
  int w = 0;
  while (w + 1 < SYNK_MAX_WORKERS && g.row_off[w + 1] <= row0) ++w;   // uniform: the worker that holds these rows
  const int64_t rw = row0 - g.row_off[w];              // first row inside the worker's arrays
  const int T = (int)(g.k_fixed / kBK);

  // ---- producer side: this lane's global address in tile 0; a constant step per tile
  const char* pa[A_INSTR];
  const char* pb[B_INSTR];
  char* pd[A_INSTR];                                   // GATHER: where this lane's piece of tile 0 is left in a[w]
  const char* Ab = reinterpret_cast<const char*>(g.a[w]);
  const char* Bb = reinterpret_cast<const char*>(g.b);
#pragma unroll
  for (int j = 0; j < A_INSTR; ++j) {
    const int row = 8 * (wave + kWaves * j) + (lane >> 3), phys = lane & 7;
    const int64_t piece = (phys ^ swz_kc(row)) * 16;
    if constexpr (GATHER) {
      int64_t src = g.gather_idx[row0 + row];
      if (src < 0 || src >= g.gather_rows) src = 0;
      pa[j] = reinterpret_cast<const char*>(g.gather_src) + (src * g.lda) * 2 + piece;
      pd[j] = const_cast<char*>(Ab) + ((rw + row) * g.lda) * 2 + piece;
    } else {
      pa[j] = Ab + ((rw + row) * g.lda) * 2 + piece;
      pd[j] = nullptr;
    }
  }
  if constexpr (GATHER) {
    if (bn == 0 && g.gather_labels && tid < BM) {
      int64_t src = g.gather_idx[row0 + tid];
      if (src < 0 || src >= g.gather_rows) src = 0;
      g.gather_y[row0 + tid] = g.gather_labels[src];
    }
  }
  int64_t step_b;
  if (MODE == FWD) {
    constexpr int SPR = BN / 8, RPI = 64 / SPR;        // 16-byte pieces a row; rows an instruction covers
#pragma unroll
    for (int j = 0; j < B_INSTR; ++j) {
      const int row = RPI * (wave + kWaves * j) + lane / SPR, phys = lane % SPR;
      pb[j] = Bb + ((int64_t)row * g.ldb + n0) * 2 + (phys ^ swz_xc<BN>(row)) * 16;
    }
    step_b = (int64_t)kBK * g.ldb * 2;
  } else {
#pragma unroll
    for (int j = 0; j < B_INSTR; ++j) {
      const int row = 8 * (wave + kWaves * j) + (lane >> 3), phys = lane & 7;
      pb[j] = Bb + ((int64_t)(n0 + row) * g.ldb) * 2 + (phys ^ swz_kc(row)) * 16;
    }
    step_b = kBK * 2;
  }
  const unsigned lds0 = __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)((__attribute__((address_space(3))) void*)(smem)) + wave * 1024);
  auto issue = [&](int stage) {
    const unsigned sa = lds0 + stage * STAGE, sb = sa + A_BYTES;
#pragma unroll
    for (int j = 0; j < A_INSTR; ++j) {
      load_to_lds16(pa[j], sa + kWaves * j * 1024);
      pa[j] += kBK * 2;
    }
#pragma unroll
    for (int j = 0; j < B_INSTR; ++j) {
      load_to_lds16(pb[j], sb + kWaves * j * 1024);
      pb[j] += step_b;
    }
  };

  // ---- consumer side: this lane's byte offsets inside a stage, for its two k-steps of a tile
  int offA[TM][2], offB[TN][2][2];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int r = wm * (BM / 2) + i * 32 + x;
#pragma unroll
    for (int kq = 0; kq < 2; ++kq) offA[i][kq] = r * 128 + ((((kh * 2 + kq) * 2 + gk) ^ swz_kc(r)) << 4);
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if (MODE == FWD) {
      // lane (group q of 16, i16) gives the address of 4 columns of one row; after the transpose it
      // holds column (q&1)*16 + i16 of the MFMA tile for k = (q>>1)*8 + h*4 + 0..3
      const int q = lane >> 4, i16 = lane & 15;
      const int col = wn * (BN / 2) + j * 32 + (q & 1) * 16 + (i16 & 3) * 4;
#pragma unroll
      for (int kq = 0; kq < 2; ++kq)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int row = (kh * 2 + kq) * 16 + (q >> 1) * 8 + h * 4 + (i16 >> 2);
          offB[j][kq][h] = A_BYTES + row * (BN * 2) + (((col >> 3) ^ swz_xc<BN>(row)) << 4) + (col & 7) * 2;
        }
    } else {
      const int r = wn * (BN / 2) + j * 32 + x;
#pragma unroll
      for (int kq = 0; kq < 2; ++kq) {
        offB[j][kq][0] = A_BYTES + r * 128 + ((((kh * 2 + kq) * 2 + gk) ^ swz_kc(r)) << 4);
        offB[j][kq][1] = 0;
      }
    }
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // what the output pass needs from memory is asked for now
  float bias[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) bias[j] = MODE == FWD ? g.bias[n0 + wn * (BN / 2) + j * 32 + x] : 0.0f;

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < T) issue(s);

  auto compute = [&](int stage) {
    const unsigned char* st = smem + stage * STAGE;
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int kq = 0; kq < 2; ++kq) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[kq][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(st + offA[i][kq]));
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (MODE == FWD) {
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(st + offB[j][kq][0]));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(st + offB[j][kq][1]));
          const s16x8 both = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          fb[kq][j] = __builtin_bit_cast(bf16x8, both);
        } else {
          fb[kq][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(st + offB[j][kq][0]));
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // all fragment reads of the tile are issued before its products
#pragma unroll
    for (int kq = 0; kq < 2; ++kq)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kq][i], fb[kq][j], acc[i][j], 0, 0, 0);
  };

  // ---- main loop, NS tiles a trip so that the stage of every access is a compile-time constant
  for (int t0 = 0; t0 < T; t0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int t = t0 + u;
      if (t < T) {
        // this wavefront's loads of tile t have landed once only the younger tiles' loads are pending
        const int younger = (T - 1 - t) < (NS - 2) ? (T - 1 - t) : (NS - 2);
        if (younger >= NS - 2 && NS >= 4) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * PER_TILE) : "memory");
        else if (younger == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (younger == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_TILE) : "memory");
        else if (younger == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * PER_TILE) : "memory");
        else if (younger == 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(3 * PER_TILE) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // deeper rings than this code lists: wait for all
        __syncthreads();                 // every wavefront's part of tile t is in LDS; tile t-1 has been consumed
        if (t + NS - 1 < T) issue((u + NS - 1) % NS);           // into the stage tile t-1 used
        if constexpr (GATHER) {
          if (t % tiles_n == bn) {       // this workgroup's share of the rows' columns: its own pieces, LDS -> a[w]
#pragma unroll
            for (int j = 0; j < A_INSTR; ++j) {
              const u32x4 q = *reinterpret_cast<const u32x4*>(smem + u * STAGE + (kWaves * j + wave) * 1024 + lane * 16);
              *reinterpret_cast<u32x4*>(pd[j] + (int64_t)t * (kBK * 2)) = q;
            }
          }
        }
        compute(u);
      }
    }
  }

  // ---- the two k halves meet: half 1 hands its sums over (lane-major: no bank conflict), half 0 adds
  __syncthreads();
  {
    float* red = reinterpret_cast<float*>(smem) + wq * (TM * TN * 16 * 64) + lane;
    if (kh == 1) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) red[((i * TN + j) * 16 + v) * 64] = acc[i][j][v];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float val = acc[i][j][v] + red[((i * TN + j) * 16 + v) * 64];
            if (MODE == FWD) {
              val += bias[j];
              if (g.relu) val = fmaxf(val, 0.0f);
            }
            acc[i][j][v] = val;
          }
    }
    __syncthreads();
  }

  // ---- output: bf16, staged through LDS in passes of 64 rows, written as 16-byte pieces of whole rows;
  //      the relu mask of the layer below (DX) is applied to the pieces on their way out
  uint16_t* so = reinterpret_cast<uint16_t*>(smem);
  char* Cw = reinterpret_cast<char*>(g.c[w]);
  const char* Mk = MODE == DX ? reinterpret_cast<const char*>(g.mask) : nullptr;
  constexpr int CPR = BN * 2 / 16;                     // 16-byte pieces a row
  constexpr int PIECES = 64 * CPR / kThreads;          // per thread and pass
  static_assert(64 * CPR % kThreads == 0, "output pieces divide over the threads");
#pragma unroll
  for (int ps = 0; ps < BM / 64; ++ps) {
    u32x4 mk[PIECES];
    if (MODE == DX) {
#pragma unroll
      for (int e = 0; e < PIECES; ++e) {
        const int c = tid + e * kThreads, rl = c / CPR, ch = c % CPR;
        mk[e] = *reinterpret_cast<const u32x4*>(Mk + ((row0 + ps * 64 + rl) * g.ldmask + n0) * 2 + ch * 16);
      }
    }
    if (kh == 0) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int tile_row = wm * (BM / 2) + i * 32;
        if (tile_row / 64 != ps) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int base = ((tile_row & 63) + gk * 4) * BN + wn * (BN / 2) + j * 32 + x;
#pragma unroll
          for (int v = 0; v < 16; ++v) so[base + ((v >> 2) * 8 + (v & 3)) * BN] = f32_to_bf16(acc[i][j][v]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PIECES; ++e) {
      const int c = tid + e * kThreads, rl = c / CPR, ch = c % CPR;
      u32x4 q = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(so) + rl * BN * 2 + ch * 16);
      if (MODE == DX) {
        // keep an element where the activation below is positive (bf16: sign bit clear and not zero)
        auto keep = [](uint32_t h) -> uint32_t {
          const uint32_t lo = ((h & 0x8000u) == 0u && (h & 0x7fffu) != 0u) ? 0x0000ffffu : 0u;
          const uint32_t hi = ((h & 0x80000000u) == 0u && (h & 0x7fff0000u) != 0u) ? 0xffff0000u : 0u;
          return lo | hi;
        };
        q.x &= keep(mk[e].x); q.y &= keep(mk[e].y); q.z &= keep(mk[e].z); q.w &= keep(mk[e].w);
      }
      *reinterpret_cast<u32x4*>(Cw + ((rw + ps * 64 + rl) * g.ldc + n0) * 2 + ch * 16) = q;
    }
    if (ps + 1 < BM / 64) __syncthreads();
  }
}

}  // namespace gdma
}  // namespace synk
