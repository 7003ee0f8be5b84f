// A second sliced gradient function (Sec. 3.3 step 1 evaluated as Sec. 3.2 /
// 5.1 describe): one 3x3 convolution + batch-normalisation + ReLU block of the
// kind the scaling study's network is built from (Sec. 6), closed by global
// average pooling, one affine layer and softmax cross-entropy.
//
// One call covers every worker and every slice.  A slice is one call of the
// function (Sec. 5.1), so the batch statistics are per slice; a slice's images
// carry the weight that the aggregation op gives the slice, which makes every
// sum over a worker's images the in-place aggregation of its slice results.
//
// Images are channels-last (a gathered row is H*W*C_in values), so the
// convolution is a product [pixels x 9 C_in] . [9 C_in x C_out] whose left
// operand is never built: for one tap, the row of a pixel is the C_in vector
// of its shifted neighbour (or zero outside the image), which is one
// wave-uniform offset away from the pixel's own address.  Both contractions
// (forward, weight gradient) run on the matrix cores (MFMA 32x32x16 bf16 or
// 32x32x2 fp32, fp32 accumulators) out of LDS; everything between them is
// streaming work over z (kept in the compute type) in fp32 arithmetic.
//
// No floating-point atomics: every sum has a fixed order.
#include <math.h>

#include <algorithm>

#include "common.h"

namespace synk {

typedef uint16_t bf16_t;                                     // raw bfloat16 bits
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));   // MFMA operand type

namespace {

template <typename T> struct EL;
template <> struct EL<float> { static constexpr int V = 4; };    // elements per 16-byte vector
template <> struct EL<bf16_t> { static constexpr int V = 8; };

constexpr int kThreads = 256;
constexpr int kChunkRows = 256;     // pixels of one image handled by one workgroup of the streaming kernels
constexpr int kMaxCout = 512;
constexpr int kMaxClasses = 4096;

struct ConvShape {
  int H, W, cin, cout, classes, HW;
  int n_workers, n_slices, grad_op;
  int n_chunks;      // ceil(HW / kChunkRows)
  int total_images;
  float eps;
};

struct WorkerTable {
  const void* x[SYNK_MAX_WORKERS];
  const int32_t* y[SYNK_MAX_WORKERS];
  float* grad[SYNK_MAX_WORKERS];
  int32_t rows[SYNK_MAX_WORKERS];
  int32_t row_off[SYNK_MAX_WORKERS + 1];   // images held by the workers before w
  // Input indexing folded into the call (gsrc == nullptr: x[w], y[w] hold the workers' images and
  // labels): packed image i is row gidx[i] of the dataset gsrc ([grows x H*W*C_in] in the compute
  // type), its label glabels[gidx[i]]; an index outside [0, grows) reads row 0.
  const void* gsrc;
  const int32_t* gidx;
  const int32_t* glabels;
  int32_t grows;
};

// Dataset row of packed image i under input indexing.
__device__ __forceinline__ int64_t gathered_row(const WorkerTable& tab, int i) {
  int64_t s = tab.gidx[i];
  if (s < 0 || s >= tab.grows) s = 0;
  return s;
}

// Offsets into the flat parameter / gradient array.
struct ParamOff {
  int64_t wc, gamma, beta, wf, bf, total;
};
__host__ __device__ inline ParamOff param_off(int cin, int cout, int classes) {
  ParamOff o;
  o.wc = 0;
  o.gamma = (int64_t)9 * cin * cout;
  o.beta = o.gamma + cout;
  o.wf = o.beta + cout;
  o.bf = o.wf + (int64_t)cout * classes;
  o.total = o.bf + classes;
  return o;
}

__device__ __forceinline__ void slice_bounds(int rows, int parts, int s, int* start, int* size) {
  const int base = rows / parts, extra = rows % parts;
  *size = base + (s < extra ? 1 : 0);
  *start = base * s + (s < extra ? s : extra);
}

__device__ __forceinline__ f32x16 zero16() {
  f32x16 a;
#pragma unroll
  for (int v = 0; v < 16; ++v) a[v] = 0.0f;
  return a;
}

// 16 bytes at base + byte_off if ok, else zeros.  The load itself is unconditional (a refused
// vector reads `base`, which must be a valid address) and the zeroing is a bit mask: a select
// would let the compiler fold the pair into a branch around the load, and a load inside a
// branch is waited for before the next one is issued.
__device__ __forceinline__ u32x4 load_or_zero(const void* base, int64_t byte_off, bool ok) {
  const int64_t m = -(int64_t)ok;
  const u32x4 v = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(base) + (byte_off & m));
  const uint32_t k = (uint32_t)m;
  return u32x4{v.x & k, v.y & k, v.z & k, v.w & k};
}

// z (the convolution's output) is kept in the compute type.  Four consecutive channels as
// floats, and one value.
__device__ __forceinline__ f32x4 load_z4(const float* z, int64_t i) { return *reinterpret_cast<const f32x4*>(z + i); }
__device__ __forceinline__ f32x4 load_z4(const bf16_t* z, int64_t i) {
  const u32x2 q = *reinterpret_cast<const u32x2*>(z + i);
  return f32x4{__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xffff0000u), __uint_as_float(q.y << 16),
               __uint_as_float(q.y & 0xffff0000u)};
}
__device__ __forceinline__ float load_z1(const float* z, int64_t i) { return z[i]; }
__device__ __forceinline__ float load_z1(const bf16_t* z, int64_t i) { return bf16_to_f32(z[i]); }
__device__ __forceinline__ void store_z1(float* z, int64_t i, float v) { z[i] = v; }
__device__ __forceinline__ void store_z1(bf16_t* z, int64_t i, float v) { z[i] = f32_to_bf16(v); }

// One 16-byte operand pair -> the MFMAs it feeds.  bf16: 8 contraction steps in
// one instruction.  fp32: lane group g holds steps 4g..4g+3 of an 8-step run;
// instruction j takes element j of both operands (any pairing of steps works
// as long as both operands use the same one).
__device__ __forceinline__ f32x16 mma(bf16_t, u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(float, u32x4 a, u32x4 b, f32x16 c) {
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
  return c;
}

// ------------------------------------------------------------ weight layout
// wmat[o][k] = (T) Wc[k][o], k = tap*C_in + c: the convolution's right operand
// with its contraction index contiguous, rounded to the compute type.
template <typename T>
__global__ __launch_bounds__(kThreads) void conv_weight_kernel(const float* __restrict__ params, T* __restrict__ wmat,
                                                               int K, int cout) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= (int64_t)K * cout) return;
  const int o = (int)(i / K), k = (int)(i - (int64_t)o * K);
  const float v = params[(int64_t)k * cout + o];
  if (sizeof(T) == 2) reinterpret_cast<uint16_t*>(wmat)[i] = f32_to_bf16(v);
  else reinterpret_cast<float*>(wmat)[i] = v;
}

// The same operand in the order the padded-patch kernel's wavefronts read it:
// one 1 KB block per (tap, 64-channel input chunk, 32-wide output tile, step
// kk): lane (xi, gk) owns the 8 values Wc[tap*C_in + chunk*64 + kk*16 + gk*8 +
// e][tile*32 + xi], so that a wavefront's operand load is one contiguous KB.
// Output channels past C_out read as zero.
__global__ __launch_bounds__(kThreads) void conv_weight_frag_kernel(const float* __restrict__ params,
                                                                    uint16_t* __restrict__ wfrag, int cin,
                                                                    int cout, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;   // one bf16 value
  if (i >= total) return;
  const int e = (int)(i & 7), lane = (int)((i >> 3) & 63), kk = (int)((i >> 9) & 3);
  const int64_t blk = i >> 11;                 // (tap * chunks + chunk) * tiles + tile
  const int tiles = (cout + 31) / 32, chunks = cin / 64;
  const int tile = (int)(blk % tiles);
  const int64_t tc = blk / tiles;
  const int chunk = (int)(tc % chunks), tap = (int)(tc / chunks);
  const int k = tap * cin + chunk * 64 + kk * 16 + (lane >> 5) * 8 + e, o = tile * 32 + (lane & 31);
  wfrag[i] = o < cout ? f32_to_bf16(params[(int64_t)k * cout + o]) : (uint16_t)0;
}

// ------------------------------------------------------------ forward conv
// z[pixel][o] for a 128-pixel x 64-channel tile of one (worker, slice) unit.
// LDS rows are 8 vectors of 16 bytes (64 bf16 or 32 fp32 contraction steps of
// one tap) plus 16 bytes of padding; two buffers, one barrier per k-tile.
constexpr int kFwdBM = 128, kFwdBN = 64, kLdsRow = 144;

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_fwd_kernel(WorkerTable tab, ConvShape sh,
                                                                  const T* __restrict__ wmat,
                                                                  T* __restrict__ z) {
  constexpr int V = EL<T>::V, BK = 8 * V;
  __shared__ __attribute__((aligned(16))) char smem[2][(kFwdBM + kFwdBN) * kLdsRow];

  const int unit = blockIdx.z;
  const int w = unit / sh.n_slices, s = unit - w * sh.n_slices;
  int img0, nimg;
  slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
  const int M = nimg * sh.HW;
  const int m0 = blockIdx.x * kFwdBM;
  if (m0 >= M) return;
  const int n0 = blockIdx.y * kFwdBN;
  const T* __restrict__ xw = reinterpret_cast<const T*>(tab.x[w]) + (int64_t)img0 * sh.HW * sh.cin;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, wm = wv >> 1, wn = wv & 1;
  const int kv = tid & 7, ur = tid >> 3;   // this thread's vector in a row, and its row within a group of 32

  // left operand: 4 pixel rows per thread; bit 4 = row exists, bits 0..3 = it
  // has a neighbour above / below / left / right
  const T* arow[4];
  uint32_t amask[4];
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int q = m0 + it * 32 + ur;
    arow[it] = xw;
    amask[it] = 0u;
    if (q < M) {
      const int rem = q % sh.HW;
      const int h = rem / sh.W, ww = rem - h * sh.W;
      arow[it] = xw + (int64_t)q * sh.cin;
      amask[it] = 16u | (h > 0 ? 1u : 0u) | (h < sh.H - 1 ? 2u : 0u) | (ww > 0 ? 4u : 0u) | (ww < sh.W - 1 ? 8u : 0u);
    }
  }
  const int K = 9 * sh.cin;
  const T* brow[2];
  bool bok[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int o = n0 + it * 32 + ur;
    bok[it] = o < sh.cout;
    brow[it] = wmat + (int64_t)(bok[it] ? o : 0) * K;
  }

  const int cpt = (sh.cin + BK - 1) / BK;   // k-tiles per tap
  const int n_kt = 9 * cpt;
  u32x4 ra[4], rb[2];

  auto gload = [&](int t) {
    const int tap = t / cpt;
    const int c = (t - tap * cpt) * BK + kv * V;
    const int kh = tap / 3, kw = tap - kh * 3;
    const bool cok = c < sh.cin;
    const uint32_t need = 16u | (kh == 0 ? 1u : 0u) | (kh == 2 ? 2u : 0u) | (kw == 0 ? 4u : 0u) | (kw == 2 ? 8u : 0u);
    const int delta = ((kh - 1) * sh.W + (kw - 1)) * sh.cin + c;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const bool ok = cok && ((amask[it] & need) == need);
      ra[it] = load_or_zero(xw, ((arow[it] - xw) + delta) * (int64_t)sizeof(T), ok);
    }
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const bool ok = cok && bok[it];
      rb[it] = load_or_zero(wmat, ((brow[it] - wmat) + tap * sh.cin + c) * (int64_t)sizeof(T), ok);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int it = 0; it < 4; ++it)
      *reinterpret_cast<u32x4*>(&smem[buf][(it * 32 + ur) * kLdsRow + kv * 16]) = ra[it];
#pragma unroll
    for (int it = 0; it < 2; ++it)
      *reinterpret_cast<u32x4*>(&smem[buf][(kFwdBM + it * 32 + ur) * kLdsRow + kv * 16]) = rb[it];
  };

  f32x16 acc[2] = {zero16(), zero16()};
  gload(0);
  lstore(0);
  __syncthreads();
  for (int t = 0; t < n_kt; ++t) {
    if (t + 1 < n_kt) gload(t + 1);
    const char* A = smem[t & 1] + (wm * 64 + xi) * kLdsRow + gk * 16;
    const char* B = smem[t & 1] + (kFwdBM + wn * 32 + xi) * kLdsRow + gk * 16;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const u32x4 a0 = *reinterpret_cast<const u32x4*>(A + kk * 32);
      const u32x4 a1 = *reinterpret_cast<const u32x4*>(A + 32 * kLdsRow + kk * 32);
      const u32x4 b = *reinterpret_cast<const u32x4*>(B + kk * 32);
      acc[0] = mma(T(), a0, b, acc[0]);
      acc[1] = mma(T(), a1, b, acc[1]);
    }
    if (t + 1 < n_kt) lstore((t + 1) & 1);
    __syncthreads();
  }

  // accumulator v of lane (xi, gk) is row gk*4 + (v>>2)*8 + (v&3), column xi
  T* __restrict__ zu = z + ((int64_t)(tab.row_off[w] + img0) * sh.HW) * sh.cout;
  const int col = n0 + wn * 32 + xi;
  if (col < sh.cout) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r0 = m0 + wm * 64 + i * 32 + gk * 4;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = r0 + (v >> 2) * 8 + (v & 3);
        if (row < M) store_z1(zu, (int64_t)row * sh.cout + col, acc[i][v]);
      }
    }
  }
}

// The same contraction for bf16 with C_in a multiple of 64 and rows of at most
// 61 pixels, in the coordinates of the zero-padded image: position u = hp * Wp +
// wp on the (H+2) x (W+2) grid, Wp = W + 2.  There a tap is the plain shift
// (kh-1) * Wp + (kw-1) of the position index, with no case distinction at the
// border.  A workgroup takes TILE consecutive positions of one image (from the
// first real pixel on; border positions in between are computed and dropped)
// and lays the positions it can reach, one 64-channel chunk at a time, into LDS
// once, zeros included; the nine taps then read shifted rows of that patch.
// Wave (row half, column tile) owns TILE/2 positions x 32 channels; its slice of
// the weights comes straight from memory in operand order
// (conv_weight_frag_kernel), a few taps ahead, so the tap loop has no barrier.
template <int TILE, int MINB, int AHEAD>
__global__ __launch_bounds__(kThreads, MINB) void conv3x3_fwd_patch_kernel(WorkerTable tab, ConvShape sh,
                                                                        const bf16_t* __restrict__ wmat,
                                                                        bf16_t* __restrict__ z,
                                                                        int tiles_per_image, int n_tiles) {
  constexpr int kPatchTile = TILE, kPatchMaxRows = TILE + 2 * 64;
  constexpr int RT = TILE / 64;                  // 32-row MFMA tiles per wavefront (it owns TILE/2 positions)
  __shared__ __attribute__((aligned(16))) char patch[kPatchMaxRows * kLdsRow];
  __shared__ int zrow[kPatchTile];

  // Workgroups go to the 8 XCDs round-robin in launch order.  XCD k takes the k-th eighth of the
  // (image, tile) list in order, so that tiles next to each other, which share their halo, run on
  // one XCD at about the same time and the second fetch of the halo hits that XCD's L2.
  const int per_xcd = (n_tiles + 7) / 8;
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (item >= n_tiles) return;
  const int img = item / tiles_per_image, tile = item - img * tiles_per_image, n0 = blockIdx.y * 64;
  int w = 0;
  while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= img) ++w;
  const bf16_t* __restrict__ xi_ =
      tab.gsrc ? reinterpret_cast<const bf16_t*>(tab.gsrc) + gathered_row(tab, img) * sh.HW * sh.cin
               : reinterpret_cast<const bf16_t*>(tab.x[w]) + (int64_t)(img - tab.row_off[w]) * sh.HW * sh.cin;
  const int Wp = sh.W + 2;
  const int first = Wp + 1;                       // position of pixel (0, 0)
  const int n_out = sh.H * Wp - 2;                // positions from the first to the last real pixel
  const int prow = kPatchTile + 2 * Wp + 2;       // patch rows: the tile and Wp + 1 positions either side

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, rh = wv >> 1, ct = wv & 1;
  const int kv = tid & 7, ur = tid >> 3;

  // output row of every position of the tile (-1: border position or past the image)
  if (tid < kPatchTile) {
    const int r = tile * kPatchTile + tid;
    const int u = first + r;
    const int hp = u / Wp, wp = u - hp * Wp;
    zrow[tid] = (r < n_out && wp >= 1 && wp <= sh.W) ? (hp - 1) * sh.W + (wp - 1) : -1;
  }

  // this wave's operand blocks: tile index fixed, (tap, chunk) advance by `wstep` vectors
  const int tiles32 = (sh.cout + 31) / 32;
  const int my_tile = min(blockIdx.y * 2 + ct, tiles32 - 1);
  const u32x4* __restrict__ wfrag = reinterpret_cast<const u32x4*>(wmat) + (int64_t)my_tile * 256 + lane;
  const int wstep = tiles32 * 256;                 // vectors from one (tap, chunk) to the next
  const int chunks = sh.cin / 64;

  f32x16 acc[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) acc[rt] = zero16();
  constexpr int kAhead = AHEAD;      // taps whose weights are in flight ahead of the one in use
  for (int cc = 0; cc < sh.cin; cc += 64) {
    if (cc > 0) __syncthreads();     // every wave is done with the previous chunk's patch
    u32x4 b[kAhead + 1][4];
#pragma unroll
    for (int tp = 0; tp < kAhead; ++tp)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) b[tp][kk] = wfrag[(int64_t)(tp * chunks + cc / 64) * wstep + kk * 64];
    // patch row j holds position tile*TILE + j (that is first + tile*TILE + j - (Wp+1)); all of a
    // thread's loads are issued before the first of them is stored
    {
      constexpr int NIT = kPatchMaxRows / 32;
      int up = tile * kPatchTile + ur;
      int hp = up / Wp, wp = up - hp * Wp;
      const int adv_h = 32 / Wp, adv_w = 32 - adv_h * Wp;
      u32x4 rv[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const bool real = ur + it * 32 < prow && hp >= 1 && hp <= sh.H && wp >= 1 && wp <= sh.W;
        rv[it] = load_or_zero(xi_, (((int64_t)(hp - 1) * sh.W + (wp - 1)) * sh.cin + cc + kv * 8) * 2, real);
        wp += adv_w;
        hp += adv_h;
        if (wp >= Wp) { wp -= Wp; ++hp; }
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int j = ur + it * 32;
        if (j < prow) *reinterpret_cast<u32x4*>(&patch[j * kLdsRow + kv * 16]) = rv[it];
      }
    }
    __syncthreads();
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (tap + kAhead < 9) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          b[(tap + kAhead) % (kAhead + 1)][kk] = wfrag[(int64_t)((tap + kAhead) * chunks + cc / 64) * wstep + kk * 64];
      }
      const int d = (tap / 3 - 1) * Wp + (tap % 3 - 1);
      const char* A = patch + (rh * (TILE / 2) + xi + first + d) * kLdsRow + gk * 16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          const u32x4 a = *reinterpret_cast<const u32x4*>(A + rt * 32 * kLdsRow + kk * 32);
          acc[rt] = mma(bf16_t(), a, b[tap % (kAhead + 1)][kk], acc[rt]);
        }
      }
    }
  }

  // Output through LDS, 128 positions x 64 channels fp32 at a time, so that z is written in whole
  // 128-byte rows of bf16.  Row pitch 72 floats: the two lane groups of a wavefront (rows 4
  // apart) land in different banks.
  constexpr int kPitch = 72;
  float* stage = reinterpret_cast<float*>(patch);
  bf16_t* __restrict__ zi = z + (int64_t)img * sh.HW * sh.cout;
  for (int h = 0; h < TILE / 128; ++h) {
    __syncthreads();       // the patch (h = 0) or the pass before has been read
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int row0 = rh * (TILE / 2) + rt * 32;          // first position of this MFMA tile
      if (row0 / 128 == h) {
        float* sp = stage + (row0 % 128 + gk * 4) * kPitch + ct * 32 + xi;
#pragma unroll
        for (int v = 0; v < 16; ++v) sp[((v >> 2) * 8 + (v & 3)) * kPitch] = acc[rt][v];
      }
    }
    __syncthreads();
    const int c8 = tid & 7, rr = tid >> 3;
    if (n0 + c8 * 8 < sh.cout) {
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int r = it * 32 + rr;
        const int row = zrow[h * 128 + r];
        if (row >= 0) {
          const f32x4 a = *reinterpret_cast<const f32x4*>(stage + r * kPitch + c8 * 8);
          const f32x4 b = *reinterpret_cast<const f32x4*>(stage + r * kPitch + c8 * 8 + 4);
          const u32x4 q = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]),
                           pack_bf16x2(b[2], b[3])};
          *reinterpret_cast<u32x4*>(zi + (int64_t)row * sh.cout + n0 + c8 * 8) = q;
        }
      }
    }
  }
}

// The same contraction for bf16 with 64 input channels and at most 64 output
// channels: the whole right operand is 9 * 64 * 64 values, so a wavefront keeps
// all of it in registers (72 operand vectors, most of them in the accumulation
// registers, which the MFMA reads directly) for the life of the workgroup, and
// the tap loop reads only positions from LDS: one 16-byte read per lane feeds
// two MFMAs.  One workgroup per CU (one wavefront per SIMD, 512 registers)
// takes units of work, a unit being a run of consecutive 128-position tiles of
// one image.  The padded positions of the image slide through a ring of four
// blocks of 128 positions: tile t needs blocks t and t + 1 (its taps reach at
// most 2 (W + 3) <= 128 positions past its first); block t + 3 is asked for
// during tile t and goes from registers to the ring during tile t + 1; one
// barrier per tile.
//
// With one wavefront per SIMD nothing else hides the work around the MFMAs, so
// it is cut into slices that sit between them (a slot = the two MFMAs of one
// contraction step and what follows them): the ring stores and block loads, and
// the output of the tile BEFORE this one, whose sums wait in a second set of
// registers: pack to bf16 (the channels are the MFMA's M side, a lane holds four
// consecutive channels of one position), through a staging area of the
// wavefront's own (no barrier) into whole 128-byte rows, and out.  The stores
// are buffer stores whose offset is out of range for a border position, so that
// the tile body has no branch.
constexpr int kHoldTile = 128, kHoldRing = 4 * kHoldTile;
constexpr int kHoldStageRow = 144;     // bytes: 64 channels bf16 + 16, as kLdsRow
constexpr uint32_t kHoldDrop = 0x80000000u;     // a store offset past every image

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1)))
void conv3x3_fwd_hold_kernel(WorkerTable tab, ConvShape sh, const float* __restrict__ params, bf16_t* __restrict__ z,
                             int tiles_per_image, int per_img, int n_units) {
  __shared__ __attribute__((aligned(16))) char ring[kHoldRing * kLdsRow];
  __shared__ __attribute__((aligned(16))) char stage[(kThreads / 64) * 32 * kHoldStageRow];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5;
  const int kv = tid & 7, ur = tid >> 3, c8 = lane & 7;
  const int H = sh.H, W = sh.W, Wp = W + 2, cout = sh.cout;
  const int z_image_bytes = sh.HW * cout * 2;

  // steps of a padded position by 8, 32 and 128: rows and columns of the (H+2) x (W+2) grid
  const int a8h = 8 / Wp, a8w = 8 - a8h * Wp, a32h = 32 / Wp, a32w = 32 - a32h * Wp;
  const int a128h = 128 / Wp, a128w = 128 - a128h * Wp;
  auto adv = [&](int& hp, int& wp, int ah, int aw) {
    wp += aw;
    hp += ah;
    if (wp >= Wp) { wp -= Wp; ++hp; }
  };

  // A block of 128 positions: thread (ur, kv) holds vector kv of positions ur + 32 it.  The loads
  // carry no condition (a position outside the image reads the image's first vector) and the
  // zeroing waits until the store, so that nothing waits for a load where it is issued.
  struct Block { u32x4 v[4]; uint32_t keep[4]; };
  const char* ximg = nullptr;
  int lhp = 0, lwp = 0;                 // padded position of row ur of the next block to ask for
  auto load_row = [&](int it, Block& blk, int hp, int wp) {
    const uint32_t m = -(uint32_t)((unsigned)(hp - 1) < (unsigned)H & (unsigned)(wp - 1) < (unsigned)W);
    const uint32_t off = (uint32_t)(((hp - 1) * W + (wp - 1)) * 128 + kv * 16) & m;
    blk.v[it] = *reinterpret_cast<const u32x4*>(ximg + off);
    blk.keep[it] = m;
  };
  auto load_block = [&](Block& blk) {   // the block at (lhp, lwp); moves on to the next block
    int hp = lhp, wp = lwp;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      load_row(it, blk, hp, wp);
      adv(hp, wp, a32h, a32w);
    }
    adv(lhp, lwp, a128h, a128w);
  };
  auto store_row = [&](int b, int it, const Block& blk) {
    const uint32_t k = blk.keep[it];
    const u32x4 q = {blk.v[it].x & k, blk.v[it].y & k, blk.v[it].z & k, blk.v[it].w & k};
    *reinterpret_cast<u32x4*>(&ring[(((b & 3) * kHoldTile) + ur + it * 32) * kLdsRow + kv * 16]) = q;
  };

  // z of one image as a buffer: an offset of kHoldDrop or more is dropped by the range check.  The
  // address is wave-uniform; said explicitly, so that the descriptor sits in scalar registers.
  auto z_rsrc = [&](int img) {
    const uint64_t a = reinterpret_cast<uint64_t>(z + (int64_t)img * sh.HW * cout);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((uint64_t)hi << 32) | (uint64_t)lo), 0,
                                             z_image_bytes, 0x00020000);
  };
  char* my_stage = stage + wv * 32 * kHoldStageRow;
  // the tile before: its sums, where its four rows per lane go, its image
  auto stage_chunk = [&](const f32x16 (&accp)[2], int c) {   // chunk c: channels ct*32 + j*8 + gk*4 .. +4
    const int ct = c >> 2, j = c & 3;
    const u32x2 q = {pack_bf16x2(accp[ct][4 * j], accp[ct][4 * j + 1]),
                     pack_bf16x2(accp[ct][4 * j + 2], accp[ct][4 * j + 3])};
    *reinterpret_cast<u32x2*>(my_stage + xi * kHoldStageRow + (ct * 32 + j * 8 + gk * 4) * 2) = q;
  };
  auto stage_row = [&](int it) {
    return *reinterpret_cast<const u32x4*>(my_stage + (it * 8 + (lane >> 3)) * kHoldStageRow + c8 * 16);
  };

  u32x4 wr[9][4][2];
  f32x16 accp[2] = {zero16(), zero16()};
  uint32_t poff[4] = {kHoldDrop, kHoldDrop, kHoldDrop, kHoldDrop};
  int pimg = 0;
  bool have_weights = false;

  for (int unit = blockIdx.x; unit < n_units; unit += gridDim.x) {
    const int img = unit / per_img, part = unit - img * per_img;
    const int t0 = part * tiles_per_image / per_img, t1 = (part + 1) * tiles_per_image / per_img;
    if (t0 >= t1) continue;
    {
      int w = 0;
      while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= img) ++w;
      ximg = tab.gsrc ? reinterpret_cast<const char*>(tab.gsrc) + gathered_row(tab, img) * sh.HW * 128
                      : reinterpret_cast<const char*>(tab.x[w]) + (int64_t)(img - tab.row_off[w]) * sh.HW * 128;
      const int up = t0 * kHoldTile + ur;
      lhp = up / Wp;
      lwp = up - lhp * Wp;
    }
    // rows of tile t: position r = t*128 + wv*32 + it*8 + lane/8 counted from the first real pixel,
    // which is padded position Wp + 1 + r
    int shp, swp;
    {
      const int u = Wp + 1 + t0 * kHoldTile + wv * 32 + (lane >> 3);
      shp = u / Wp;
      swp = u - shp * Wp;
    }
    Block rn;
    {
      Block r0, r1;
      load_block(r0);
      load_block(r1);
      load_block(rn);
      if (!have_weights) {
        have_weights = true;
        // The right operand, while the first blocks travel: the workgroup rounds Wc (fp32 in
        // params, [9 * 64][C_out]) to bf16 into the ring's memory in operand order, vector
        // ((tap * 2 + ct) * 4 + kk) * 64 + lane = the 8 values Wc[tap*64 + kk*16 + gk*8 + e][ct*32 + xi]
        // (zero past C_out), and every wavefront takes its 72 vectors from there.  A launch that
        // prepares this for all workgroups costs more than they spend here.
        {
          const int o = tid & 63;
#pragma unroll 9
          for (int it = 0; it < 18; ++it) {
            const int q = it * 4 + (tid >> 6);                    // (tap, kk, gk)
            const int tap = q >> 3, kk = (q >> 1) & 3, g = q & 1;
            const float* src = params + (int64_t)(tap * 64 + kk * 16 + g * 8) * cout + min(o, cout - 1);
            float f[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = src[e * cout];
            u32x4 v = {pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7])};
            if (o >= cout) v = u32x4{0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(&ring[(((tap * 2 + (o >> 5)) * 4 + kk) * 64 + g * 32 + (o & 31)) * 16]) = v;
          }
        }
        __syncthreads();
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
              wr[tap][kk][ct] = *reinterpret_cast<const u32x4*>(&ring[(((tap * 2 + ct) * 4 + kk) * 64 + lane) * 16]);
        // Every vector is named in an empty asm statement: that fixes its register file (64 of the
        // 72 in the accumulation registers), and it puts the wait for these reads here.
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            if (tap < 8) {
              asm volatile("" : "+a"(wr[tap][kk][0]));
              asm volatile("" : "+a"(wr[tap][kk][1]));
            } else {
              asm volatile("" : "+v"(wr[tap][kk][0]));
              asm volatile("" : "+v"(wr[tap][kk][1]));
            }
          }
        __syncthreads();               // the ring's memory is free for the blocks
      }
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        store_row(t0, it, r0);
        store_row(t0 + 1, it, r1);
      }
      __syncthreads();
    }

    for (int t = t0; t < t1; ++t) {
      f32x16 acc[2] = {zero16(), zero16()};
      uint32_t coff[4];
      u32x4 qv[4];
      const __amdgpu_buffer_rsrc_t prs = z_rsrc(pimg);
      const int p0 = t * kHoldTile + wv * 32 + xi;      // this lane's position; tap (kh, kw) reads p0 + kh Wp + kw
      auto read_tap = [&](int tap, u32x4 (&a)[4]) {
        const int row = (p0 + (tap / 3) * Wp + tap % 3) & (kHoldRing - 1);
        const char* P = ring + row * kLdsRow + gk * 16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) a[kk] = *reinterpret_cast<const u32x4*>(P + kk * 32);
      };
      int hp_l = lhp, wp_l = lwp, hp_s = shp, wp_s = swp;
      auto side = [&](int s) {
        if (s < 8) {
          const int it = s >> 1;
          if (!(s & 1)) {
            store_row(t + 2, it, rn);          // block t+2, asked for one tile ago
          } else {
            load_row(it, rn, hp_l, wp_l);      // block t+3
            adv(hp_l, wp_l, a32h, a32w);
          }
        } else if (s < 24) {
          const int c = (s - 8) >> 1;
          if (!(s & 1)) {
            stage_chunk(accp, c);
          } else if (c < 4) {                  // where this tile's rows go
            const uint32_t bad = (uint32_t)!((unsigned)(hp_s - 1) < (unsigned)H & (unsigned)(wp_s - 1) < (unsigned)W &
                                             c8 * 8 < cout);
            coff[c] = (uint32_t)(((hp_s - 1) * W + (wp_s - 1)) * cout * 2 + c8 * 16) | (bad << 31);
            adv(hp_s, wp_s, a8h, a8w);
          }
        } else if (s < 28) {
          qv[s - 24] = stage_row(s - 24);
        } else if (!(s & 1)) {
          const int it = (s - 28) >> 1;
          __builtin_amdgcn_raw_buffer_store_b128(qv[it], prs, poff[it], 0, 0);
        }
      };
      // the positions of a tap are read while the tap before it is multiplied
      u32x4 a[2][4];
      read_tap(0, a[0]);
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        if (tap + 1 < 9) read_tap(tap + 1, a[(tap + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);       // the reads stay ahead of the MFMAs that hide them
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          acc[0] = mma(bf16_t(), wr[tap][kk][0], a[tap & 1][kk], acc[0]);
          acc[1] = mma(bf16_t(), wr[tap][kk][1], a[tap & 1][kk], acc[1]);
          side(tap * 4 + kk);
          __builtin_amdgcn_sched_barrier(0);     // and every slice stays in its slot
        }
      }
      adv(lhp, lwp, a128h, a128w);
      adv(shp, swp, a128h, a128w);
      accp[0] = acc[0];
      accp[1] = acc[1];
#pragma unroll
      for (int it = 0; it < 4; ++it) poff[it] = coff[it];
      pimg = img;
      __syncthreads();
    }
  }

  // the last tile's rows
  const __amdgpu_buffer_rsrc_t prs = z_rsrc(pimg);
#pragma unroll
  for (int c = 0; c < 8; ++c) stage_chunk(accp, c);
#pragma unroll
  for (int it = 0; it < 4; ++it) __builtin_amdgcn_raw_buffer_store_b128(stage_row(it), prs, poff[it], 0, 0);
}

// -------------------------------------------------- streaming passes over z
// A workgroup takes up to kChunkRows pixels of one image and all channels:
// thread = (4 consecutive channels, row group); row groups are folded through
// LDS in a fixed order.
struct Chunk {
  int w, unit, img, chunk, nrows, cnt_unit;
  int64_t row0;        // first pixel row in the packed z / dz arrays
  int c4, rg, n_rg;    // this thread's channel quad and row group; number of row groups
  bool active;
};

__device__ __forceinline__ Chunk chunk_of(const WorkerTable& tab, const ConvShape& sh, int bid = blockIdx.x) {
  Chunk c;
  c.img = bid / sh.n_chunks;
  c.chunk = bid - c.img * sh.n_chunks;
  int w = 0;
  while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= c.img) ++w;
  c.w = w;
  int s;
  int64_t start;
  share_of(tab.rows[w], sh.n_slices, c.img - tab.row_off[w], &s, &start);
  c.unit = w * sh.n_slices + s;
  int s0, sn;
  slice_bounds(tab.rows[w], sh.n_slices, s, &s0, &sn);
  c.cnt_unit = sn * sh.HW;
  const int r0 = c.chunk * kChunkRows;
  c.nrows = min(kChunkRows, sh.HW - r0);
  c.row0 = (int64_t)c.img * sh.HW + r0;
  const int C4 = sh.cout / 4;
  c.n_rg = kThreads / C4;
  c.c4 = threadIdx.x % C4;
  c.rg = threadIdx.x / C4;
  c.active = c.rg < c.n_rg;
  return c;
}

// Sum over row groups of one float4 per thread, for NQ quantities at once:
// red[q][rg][channel].  Returns, for channel ch (ch < cout, called by threads
// ch = tid, tid + 256, ...), the sums in fixed row-group order.
template <int NQ>
__device__ __forceinline__ void fold_store(float* red, const Chunk& c, int cout, const f32x4 (&v)[NQ]) {
  if (c.active) {
#pragma unroll
    for (int q = 0; q < NQ; ++q)
      *reinterpret_cast<f32x4*>(red + ((q * c.n_rg + c.rg) * cout + c.c4 * 4)) = v[q];
  }
}
__device__ __forceinline__ float fold_sum(const float* red, int q, int n_rg, int cout, int ch) {
  float s = 0.0f;
  for (int r = 0; r < n_rg; ++r) s += red[(q * n_rg + r) * cout + ch];
  return s;
}

// f(r, four channels of row r) for this thread's rows r = rg, rg + n_rg, ... of the chunk, eight
// loads at a time: a row past the end re-reads the last row and is dropped, so that the loads
// carry no condition and are all in flight together.
template <typename Tz, typename F>
__device__ __forceinline__ void for_rows(const Chunk& c, const Tz* __restrict__ z, int64_t base, int cout, F f) {
  for (int r0 = c.rg; r0 < c.nrows; r0 += 8 * c.n_rg) {
    f32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = load_z4(z, base + (int64_t)min(r0 + u * c.n_rg, c.nrows - 1) * cout);
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (r0 + u * c.n_rg < c.nrows) f(r0 + u * c.n_rg, v[u]);
  }
}

// Per (image, chunk, channel): mean and centred sum of squares of z, computed
// about the chunk's first row so that nothing cancels.
template <typename Tz>
__global__ __launch_bounds__(kThreads) void bn_stats_chunk_kernel(WorkerTable tab, ConvShape sh,
                                                                  const Tz* __restrict__ z,
                                                                  float* __restrict__ statp) {
  __shared__ __attribute__((aligned(16))) float red[2 * kThreads * 4];
  const Chunk c = chunk_of(tab, sh);
  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    const int64_t p = c.row0 * sh.cout + c.c4 * 4;
    const f32x4 k = load_z4(z, p);
    for_rows(c, z, p, sh.cout, [&](int, const f32x4& zz) {
      const f32x4 d = zz - k;
      acc[0] += d;
      acc[1] += d * d;
    });
  }
  fold_store<2>(red, c, sh.cout, acc);
  __syncthreads();
  const float n = (float)c.nrows;
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    const float s1 = fold_sum(red, 0, c.n_rg, sh.cout, ch), s2 = fold_sum(red, 1, c.n_rg, sh.cout, ch);
    const float k = load_z1(z, c.row0 * sh.cout + ch);
    float* o = statp + ((int64_t)blockIdx.x * sh.cout + ch) * 2;
    o[0] = k + s1 / n;
    o[1] = fmaxf(s2 - s1 * s1 / n, 0.0f);
  }
}

// Merge of two (count, mean, centred sum of squares) summaries.
__device__ __forceinline__ void merge_stats(float& na, float& mean, float& m2, float nb, float mb, float m2b) {
  const float nn = na + nb;
  if (nn > 0.0f) {
    const float d = mb - mean;
    mean += d * (nb / nn);
    m2 += m2b + d * d * (na * nb / nn);
    na = nn;
  }
}

// Per (unit, channel), one wavefront: lane l merges the chunk summaries l,
// l + 64, ... in that order, then the 64 lanes merge over a fixed butterfly ->
// mu and 1 / sqrt(var + eps).
__global__ __launch_bounds__(kThreads) void bn_stats_unit_kernel(WorkerTable tab, ConvShape sh,
                                                                 const float* __restrict__ statp,
                                                                 float* __restrict__ mu, float* __restrict__ rstd) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (item >= sh.n_workers * sh.n_slices * sh.cout) return;
  const int unit = item / sh.cout, ch = item - unit * sh.cout;
  const int w = unit / sh.n_slices, s = unit - w * sh.n_slices;
  int img0, nimg;
  slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
  img0 += tab.row_off[w];
  const int n_ent = nimg * sh.n_chunks;
  float na = 0.0f, mean = 0.0f, m2 = 0.0f;
  for (int e = lane; e < n_ent; e += 64) {
    const int k = e % sh.n_chunks;
    const float* p = statp + (((int64_t)img0 * sh.n_chunks + e) * sh.cout + ch) * 2;
    merge_stats(na, mean, m2, (float)min(kChunkRows, sh.HW - k * kChunkRows), p[0], p[1]);
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const float nb = __shfl_xor(na, off), mb = __shfl_xor(mean, off), m2b = __shfl_xor(m2, off);
    // both partners must compute the same merge: order the pair by lane
    if (lane & off) {
      float n0 = nb, me0 = mb, q0 = m2b;
      merge_stats(n0, me0, q0, na, mean, m2);
      na = n0; mean = me0; m2 = q0;
    } else {
      merge_stats(na, mean, m2, nb, mb, m2b);
    }
  }
  if (lane == 0) {
    mu[(int64_t)unit * sh.cout + ch] = mean;
    rstd[(int64_t)unit * sh.cout + ch] = nimg > 0 ? 1.0f / sqrtf(m2 / na + sh.eps) : 0.0f;
  }
}

// Per (image, chunk, channel): sum over the chunk's pixels of
// relu(gamma * xhat + beta).
template <typename Tz>
__global__ __launch_bounds__(kThreads) void bn_relu_pool_kernel(WorkerTable tab, ConvShape sh,
                                                                const float* __restrict__ params,
                                                                const Tz* __restrict__ z,
                                                                const float* __restrict__ mu,
                                                                const float* __restrict__ rstd,
                                                                float* __restrict__ poolp) {
  __shared__ __attribute__((aligned(16))) float red[kThreads * 4];
  const Chunk c = chunk_of(tab, sh);
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 acc[1] = {{0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    f32x4 g, b, m, rs;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      g[e] = params[po.gamma + c.c4 * 4 + e];
      b[e] = params[po.beta + c.c4 * 4 + e];
    }
    m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
    rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
    const int64_t p = c.row0 * sh.cout + c.c4 * 4;
    for_rows(c, z, p, sh.cout, [&](int, const f32x4& zz) {
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[0][e] += fmaxf(g[e] * ((zz[e] - m[e]) * rs[e]) + b[e], 0.0f);
    });
  }
  fold_store<1>(red, c, sh.cout, acc);
  __syncthreads();
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads)
    poolp[(int64_t)blockIdx.x * sh.cout + ch] = fold_sum(red, 0, c.n_rg, sh.cout, ch);
}

// ------------------------------------------------------------------- head
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// One workgroup of 1024 threads per image: pooled features, logits (a thread
// owns a class and walks its column of Wf, eight loads in flight), loss and
// d loss / d logits, both scaled by the image's weight in its worker's
// aggregate (1/|R_w| for MEAN: slice weight |R_s|/|R_w| times the slice mean's
// 1/|R_s|; 1/|R_s| for SUM), and d loss / d p (a wavefront owns a channel and
// walks its row of Wf).
// HOLD (at most 64 channels and 1024 classes): a thread asks for its class's column of Wf before
// anything else and keeps it in registers: the loads run beside the pooling and the first barrier
// instead of behind them (eight at a time before), and d loss / d p uses the same registers (every
// thread multiplies its class's d logit into its column, the 16 wavefronts are summed over lanes and
// then in wavefront order) instead of reading Wf again.  Only 64 workgroups run (one per image), so
// this kernel is a chain of about ten latencies: 13.5 -> 12.7 us at 64 images of 64 channels and 1000 classes.
constexpr int kHeadThreads = 1024;
constexpr int kHeadHold = 64;
template <bool HOLD>
__global__ __launch_bounds__(kHeadThreads) void head_image_kernel(WorkerTable tab, ConvShape sh,
                                                                  const float* __restrict__ params,
                                                                  const float* __restrict__ poolp,
                                                                  float* __restrict__ pooled,
                                                                  float* __restrict__ dlogits,
                                                                  float* __restrict__ dpooled,
                                                                  float* __restrict__ row_loss) {
  __shared__ float sp[kMaxCout];
  __shared__ float sl[kMaxClasses];
  __shared__ float sred[2 * kHeadThreads / 64];
  constexpr int NW = kHeadThreads / 64, PER = kMaxClasses / kHeadThreads;
  const int img = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int w = 0;
  while (w + 1 < sh.n_workers && tab.row_off[w + 1] <= img) ++w;
  const int j = img - tab.row_off[w];
  int s;
  int64_t start;
  share_of(tab.rows[w], sh.n_slices, j, &s, &start);
  int s0, sn;
  slice_bounds(tab.rows[w], sh.n_slices, s, &s0, &sn);
  const float scale = sh.grad_op == SYNK_MEAN ? 1.0f / (float)tab.rows[w] : 1.0f / (float)sn;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  const float* __restrict__ Wf = params + po.wf;

  float wreg[HOLD ? kHeadHold : 1];
  if (HOLD) {
    // unconditional loads (addresses clamped into the matrix), zeroed where the entry does not exist
    const int kc = min(tid, sh.classes - 1);
#pragma unroll
    for (int ch = 0; ch < kHeadHold; ++ch) wreg[ch] = Wf[(int64_t)min(ch, sh.cout - 1) * sh.classes + kc];
#pragma unroll
    for (int ch = 0; ch < kHeadHold; ++ch) wreg[ch] = (tid < sh.classes && ch < sh.cout) ? wreg[ch] : 0.0f;
  }

  for (int ch = tid; ch < sh.cout; ch += kHeadThreads) {
    float a = 0.0f;
#pragma unroll 8
    for (int c = 0; c < sh.n_chunks; ++c) a += poolp[((int64_t)img * sh.n_chunks + c) * sh.cout + ch];
    a /= (float)sh.HW;
    sp[ch] = a;
    pooled[(int64_t)img * sh.cout + ch] = a;
  }
  __syncthreads();

  float l[PER];
  float mx = -INFINITY;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int k = q * kHeadThreads + tid;
    l[q] = -INFINITY;
    if (k < sh.classes) {
      float a = params[po.bf + k];
      if (HOLD) {
#pragma unroll
        for (int ch = 0; ch < kHeadHold; ++ch) a = fmaf(ch < sh.cout ? sp[ch] : 0.0f, wreg[ch], a);
      } else {
#pragma unroll 8
        for (int ch = 0; ch < sh.cout; ++ch) a = fmaf(sp[ch], Wf[(int64_t)ch * sh.classes + k], a);
      }
      l[q] = a;
      sl[k] = a;
    }
    mx = fmaxf(mx, l[q]);
  }
  mx = wave_max(mx);
  if (lane == 0) sred[wv] = mx;
  __syncthreads();
  mx = sred[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) mx = fmaxf(mx, sred[i]);
  float se = 0.0f;
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    l[q] = expf(l[q] - mx);   // exp(-inf) = 0 for the classes that do not exist
    se += l[q];
  }
  se = wave_sum(se);
  if (lane == 0) sred[NW + wv] = se;
  __syncthreads();
  se = 0.0f;
#pragma unroll
  for (int i = 0; i < NW; ++i) se += sred[NW + i];
  const int y = tab.gsrc ? tab.glabels[gathered_row(tab, tab.row_off[w] + j)] : tab.y[w][j];
  const bool yok = y >= 0 && y < sh.classes;
  if (tid == 0) row_loss[img] = (mx + logf(se) - (yok ? sl[y] : 0.0f)) * scale;
  __syncthreads();   // sl[y] is read before sl is overwritten
  const float inv = 1.0f / se;
  float d0 = 0.0f;   // this thread's d logit (HOLD: classes <= threads, so q = 0 is the only one)
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int k = q * kHeadThreads + tid;
    if (k < sh.classes) {
      const float d = (l[q] * inv - ((yok && k == y) ? 1.0f : 0.0f)) * scale;
      sl[k] = d;
      dlogits[(int64_t)img * sh.classes + k] = d;
      if (q == 0) d0 = d;
    }
  }
  __syncthreads();
  if (HOLD) {
    // d p[ch] = sum over classes of d logit * Wf[ch][class]: lanes, then wavefronts in order
    float* part = sl;                    // [NW][kHeadHold]; the d logits in sl are no longer needed
    // 64 sums over the 64 lanes at once: at every halving a lane hands the half of its values that
    // its partner keeps, so lane l ends with channel l's sum after 63 exchanges (one butterfly per
    // channel would be 384: the kernel took 29.6 us that way)
    float v[kHeadHold];
#pragma unroll
    for (int ch = 0; ch < kHeadHold; ++ch) v[ch] = d0 * wreg[ch];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const bool upper = (lane & off) != 0;
#pragma unroll
      for (int i = 0; i < off; ++i) {
        const float give = upper ? v[i] : v[i + off];
        const float keep = upper ? v[i + off] : v[i];
        v[i] = keep + __shfl_xor(give, off);
      }
    }
    part[wv * kHeadHold + lane] = v[0];
    __syncthreads();
    if (tid < sh.cout) {
      float a = 0.0f;
#pragma unroll
      for (int i = 0; i < NW; ++i) a += part[i * kHeadHold + tid];
      dpooled[(int64_t)img * sh.cout + tid] = a;
    }
    return;
  }
  for (int ch = wv; ch < sh.cout; ch += NW) {
    const float* __restrict__ wr = Wf + (int64_t)ch * sh.classes;
    float a = 0.0f;
#pragma unroll 4
    for (int k = lane; k < sh.classes; k += 64) a = fmaf(sl[k], wr[k], a);
    a = wave_sum(a);
    if (lane == 0) dpooled[(int64_t)img * sh.cout + ch] = a;
  }
}

constexpr int kImgTile = 8;   // images held in registers at a time by head_worker_body
constexpr int kWorkerChans = 64;

// Per worker w, class k (block bx of 256 classes) and group bz of kWorkerChans channels:
// dWf[group, k] over the worker's images in image order, kImgTile images at a time held in
// registers; group 0 also writes dbf[k], and its block (0, w) folds the image losses into
// loss[w].  Runs as the first workgroups of bn_bwd_chunk_kernel's launch.
__device__ __forceinline__ void head_worker_body(const WorkerTable& tab, const ConvShape& sh,
                                                 const float* __restrict__ pooled,
                                                 const float* __restrict__ dlogits,
                                                 const float* __restrict__ row_loss, float* __restrict__ loss,
                                                 int bx, int w, int bz) {
  __shared__ float sp[kImgTile][kWorkerChans];
  const int k = bx * kThreads + threadIdx.x;
  const int ch0 = bz * kWorkerChans, nch = min(kWorkerChans, sh.cout - ch0);
  const int i0 = tab.row_off[w], n = tab.rows[w];
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  float* __restrict__ g = tab.grad[w];
  if (bz == 0 && bx == 0 && threadIdx.x == 0) {
    float a = 0.0f;
    for (int i = 0; i < n; ++i) a += row_loss[i0 + i];
    loss[w] = a;
  }
  const bool live = k < sh.classes;
  float b = 0.0f;
  for (int t0 = 0; t0 < n || t0 == 0; t0 += kImgTile) {
    const int nt = min(kImgTile, n - t0);
    __syncthreads();
    for (int e = threadIdx.x; e < kImgTile * nch; e += kThreads) {
      const int i = e / nch, ch = e - i * nch;
      sp[i][ch] = i < nt ? pooled[(int64_t)(i0 + t0 + i) * sh.cout + ch0 + ch] : 0.0f;
    }
    __syncthreads();
    if (live) {
      float d[kImgTile];
#pragma unroll
      for (int i = 0; i < kImgTile; ++i) {
        d[i] = i < nt ? dlogits[(int64_t)(i0 + t0 + i) * sh.classes + k] : 0.0f;
        b += d[i];
      }
      for (int ch = 0; ch < nch; ++ch) {
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < kImgTile; ++i) a = fmaf(sp[i][ch], d[i], a);
        float* o = g + po.wf + (int64_t)(ch0 + ch) * sh.classes + k;
        *o = t0 == 0 ? a : *o + a;
      }
    }
  }
  if (live && bz == 0) g[po.bf + k] = b;
}

// ------------------------------------------------------ batch-norm backward
// dy = (dp / HW) [gamma*xhat + beta > 0].  Per (image, chunk, channel): sum of
// dy and of dy * xhat.
// The first head_blocks workgroups of the launch do the head's per-worker sums instead
// (head_worker_body; block = (class block, worker, channel group), class block fastest): both need
// only what head_image_kernel left, nothing after this launch but the update reads those sums, and
// a launch of their own would be one more latency-bound link in the chain (9 us at 8 workers, 64
// channels and 1000 classes); here they run beside the pass over z.
template <typename Tz>
__global__ __launch_bounds__(kThreads) void bn_bwd_chunk_kernel(WorkerTable tab, ConvShape sh,
                                                                const float* __restrict__ params,
                                                                const Tz* __restrict__ z,
                                                                const float* __restrict__ mu,
                                                                const float* __restrict__ rstd,
                                                                const float* __restrict__ dpooled,
                                                                float* __restrict__ bwdp,
                                                                const float* __restrict__ pooled,
                                                                const float* __restrict__ dlogits,
                                                                const float* __restrict__ row_loss,
                                                                float* __restrict__ loss, int head_blocks,
                                                                int class_blocks) {
  if ((int)blockIdx.x < head_blocks) {
    const int bx = blockIdx.x % class_blocks, r = blockIdx.x / class_blocks;
    head_worker_body(tab, sh, pooled, dlogits, row_loss, loss, bx, r % sh.n_workers, r / sh.n_workers);
    return;
  }
  const int bid = blockIdx.x - head_blocks;
  __shared__ __attribute__((aligned(16))) float red[2 * kThreads * 4];
  const Chunk c = chunk_of(tab, sh, bid);
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  if (c.active) {
    f32x4 g, b, m, rs, da;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      g[e] = params[po.gamma + c.c4 * 4 + e];
      b[e] = params[po.beta + c.c4 * 4 + e];
      da[e] = dpooled[(int64_t)c.img * sh.cout + c.c4 * 4 + e] / (float)sh.HW;
    }
    m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
    rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
    const int64_t p = c.row0 * sh.cout + c.c4 * 4;
    for_rows(c, z, p, sh.cout, [&](int, const f32x4& zz) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float xh = (zz[e] - m[e]) * rs[e];
        const float dy = (g[e] * xh + b[e] > 0.0f) ? da[e] : 0.0f;
        acc[0][e] += dy;
        acc[1][e] += dy * xh;
      }
    });
  }
  fold_store<2>(red, c, sh.cout, acc);
  __syncthreads();
  for (int ch = threadIdx.x; ch < sh.cout; ch += kThreads) {
    float* o = bwdp + ((int64_t)bid * sh.cout + ch) * 2;
    o[0] = fold_sum(red, 0, c.n_rg, sh.cout, ch);
    o[1] = fold_sum(red, 1, c.n_rg, sh.cout, ch);
  }
}

// Per (worker, channel), one wavefront: for every slice the lanes add the chunk
// sums l, l + 64, ... and a fixed butterfly adds the lanes -> the slice's means
// (for dz); the slices add up in slice order to the worker's d gamma, d beta.
__global__ __launch_bounds__(kThreads) void bn_bwd_worker_kernel(WorkerTable tab, ConvShape sh,
                                                                 const float* __restrict__ bwdp,
                                                                 float* __restrict__ bmean) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (item >= sh.n_workers * sh.cout) return;
  const int w = item / sh.cout, ch = item - w * sh.cout;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  float gb = 0.0f, gg = 0.0f;
  for (int s = 0; s < sh.n_slices; ++s) {
    int img0, nimg;
    slice_bounds(tab.rows[w], sh.n_slices, s, &img0, &nimg);
    img0 += tab.row_off[w];
    const int n_ent = nimg * sh.n_chunks;
    float sb = 0.0f, sg = 0.0f;
    for (int e = lane; e < n_ent; e += 64) {
      const float* p = bwdp + (((int64_t)img0 * sh.n_chunks + e) * sh.cout + ch) * 2;
      sb += p[0];
      sg += p[1];
    }
    sb = wave_sum(sb);
    sg = wave_sum(sg);
    const float cnt = (float)(nimg * sh.HW);
    if (lane == 0) {
      float* o = bmean + ((int64_t)(w * sh.n_slices + s) * sh.cout + ch) * 2;
      o[0] = nimg > 0 ? sb / cnt : 0.0f;
      o[1] = nimg > 0 ? sg / cnt : 0.0f;
    }
    gb += sb;
    gg += sg;
  }
  if (lane == 0) {
    tab.grad[w][po.beta + ch] = gb;
    tab.grad[w][po.gamma + ch] = gg;
  }
}

// dz = gamma * rstd * (dy - mean(dy) - xhat * mean(dy * xhat)), stored in the
// compute type for the weight-gradient contraction.
template <typename T>
__global__ __launch_bounds__(kThreads) void bn_bwd_dz_kernel(WorkerTable tab, ConvShape sh,
                                                             const float* __restrict__ params,
                                                             const T* __restrict__ z,
                                                             const float* __restrict__ mu,
                                                             const float* __restrict__ rstd,
                                                             const float* __restrict__ dpooled,
                                                             const float* __restrict__ bmean,
                                                             T* __restrict__ dz) {
  const Chunk c = chunk_of(tab, sh);
  if (!c.active) return;
  const ParamOff po = param_off(sh.cin, sh.cout, sh.classes);
  f32x4 g, b, m, rs, da, mb, mg;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    g[e] = params[po.gamma + c.c4 * 4 + e];
    b[e] = params[po.beta + c.c4 * 4 + e];
    da[e] = dpooled[(int64_t)c.img * sh.cout + c.c4 * 4 + e] / (float)sh.HW;
    mb[e] = bmean[((int64_t)c.unit * sh.cout + c.c4 * 4 + e) * 2];
    mg[e] = bmean[((int64_t)c.unit * sh.cout + c.c4 * 4 + e) * 2 + 1];
  }
  m = *reinterpret_cast<const f32x4*>(mu + (int64_t)c.unit * sh.cout + c.c4 * 4);
  rs = *reinterpret_cast<const f32x4*>(rstd + (int64_t)c.unit * sh.cout + c.c4 * 4);
  const int64_t e0 = c.row0 * sh.cout + c.c4 * 4;
  for_rows(c, z, e0, sh.cout, [&](int r, const f32x4& zz) {
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xh = (zz[e] - m[e]) * rs[e];
      const float dy = (g[e] * xh + b[e] > 0.0f) ? da[e] : 0.0f;
      o[e] = g[e] * rs[e] * (dy - mb[e] - xh * mg[e]);
    }
    if (sizeof(T) == 2) {
      u32x2 q = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
      *reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(dz) + e0 + (int64_t)r * sh.cout) = q;
    } else {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(dz) + e0 + (int64_t)r * sh.cout) = o;
    }
  });
}

// -------------------------------------------------------- weight gradient
// dWc[tap*C_in + c][o] = sum over a worker's pixels r of X[r shifted by tap][c]
// dz[r][o].  A workgroup owns one tap, a 64 x 64 (c, o) tile and one run of
// pixels; its sum goes to a partial array that conv_dw_fold_kernel adds up in
// run order.  Both operands have the contraction index (the pixel) strided in
// memory: they are laid into LDS pixel-major as loaded (bf16: two pixels
// interleaved per 32-bit word), which is the form the MFMA operands gather
// from.
template <typename T> struct DwGeom;
template <> struct DwGeom<bf16_t> { static constexpr int BR = 64, LROWS = 32; };
template <> struct DwGeom<float> { static constexpr int BR = 32, LROWS = 32; };

template <typename T>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_dw_kernel(WorkerTable tab, ConvShape sh,
                                                                 const T* __restrict__ dz,
                                                                 float* __restrict__ dwp, int n_runs,
                                                                 int run_rows) {
  constexpr bool HALF = sizeof(T) == 2;
  constexpr int BR = DwGeom<T>::BR, LROWS = DwGeom<T>::LROWS;
  __shared__ __attribute__((aligned(16))) uint32_t smem[2][2][LROWS * 64];   // [buffer][X | dz][pixel (pair)][64]

  const int w = blockIdx.z, run = blockIdx.y;
  const int ct = (sh.cin + 63) / 64, ot = (sh.cout + 63) / 64;
  const int tap = blockIdx.x / (ct * ot);
  const int rest = blockIdx.x - tap * (ct * ot);
  const int c0 = (rest / ot) * 64, n0 = (rest % ot) * 64;
  const int kh = tap / 3, kw = tap - kh * 3;
  const int M = tab.rows[w] * sh.HW;
  const int r_begin = min(run * run_rows, M), r_end = min(r_begin + run_rows, M);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, wm = wv >> 1, wn = wv & 1;

  const T* __restrict__ xw = reinterpret_cast<const T*>(tab.x[w]);
  const T* __restrict__ dw_ = dz + (int64_t)tab.row_off[w] * sh.HW * sh.cout;
  const int delta = ((kh - 1) * sh.W + (kw - 1)) * sh.cin;

  // this thread's vector: bf16: pixel pair tid/8, channels 8*(tid%8); fp32:
  // pixels tid/16 and 16 + tid/16, channels 4*(tid%16)
  constexpr int VPR = HALF ? 8 : 16;            // vectors per 64-channel row
  constexpr int V = EL<T>::V;
  const int uv = tid % VPR, ur = tid / VPR;
  const int rl0 = HALF ? 2 * ur : ur, rl1 = HALF ? 2 * ur + 1 : 16 + ur;   // rows within a step
  const bool xcok = c0 + uv * V < sh.cin, dcok = n0 + uv * V < sh.cout;
  // position (h, w) of the two pixels at the first step, advanced step by step
  int ph[2], pw[2];
  {
    const int q0 = r_begin + rl0, q1 = r_begin + rl1;
    const int e0 = q0 % sh.HW, e1 = q1 % sh.HW;
    ph[0] = e0 / sh.W; pw[0] = e0 - ph[0] * sh.W;
    ph[1] = e1 / sh.W; pw[1] = e1 - ph[1] * sh.W;
  }
  const int adv_h = BR / sh.W, adv_w = BR - adv_h * sh.W;
  const int rl[2] = {rl0, rl1};
  u32x4 rx[2], rd[2];

  auto gload = [&](int r0) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int q = r0 + rl[e];
      const bool in = q < r_end;
      const bool nb = (kh != 0 || ph[e] > 0) && (kh != 2 || ph[e] < sh.H - 1) && (kw != 0 || pw[e] > 0) &&
                      (kw != 2 || pw[e] < sh.W - 1);
      const bool okx = in && nb && xcok, okd = in && dcok;
      rx[e] = load_or_zero(xw, ((int64_t)q * sh.cin + delta + c0 + uv * V) * (int64_t)sizeof(T), okx);
      rd[e] = load_or_zero(dw_, ((int64_t)q * sh.cout + n0 + uv * V) * (int64_t)sizeof(T), okd);
      // next step's position
      pw[e] += adv_w;
      ph[e] += adv_h;
      if (pw[e] >= sh.W) { pw[e] -= sh.W; ++ph[e]; }
      while (ph[e] >= sh.H) ph[e] -= sh.H;
    }
  };
  auto interleave = [](const u32x4& a, const u32x4& b, u32x4* lo, u32x4* hi) {
    // word j = (a[j], b[j]) as (low half, high half)
    lo->x = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u); lo->y = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
    lo->z = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u); lo->w = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
    hi->x = __builtin_amdgcn_perm(b.z, a.z, 0x05040100u); hi->y = __builtin_amdgcn_perm(b.z, a.z, 0x07060302u);
    hi->z = __builtin_amdgcn_perm(b.w, a.w, 0x05040100u); hi->w = __builtin_amdgcn_perm(b.w, a.w, 0x07060302u);
  };
  auto lstore = [&](int buf) {
    if (HALF) {
      u32x4 lo, hi;
      interleave(rx[0], rx[1], &lo, &hi);
      u32x4* d = reinterpret_cast<u32x4*>(&smem[buf][0][ur * 64 + uv * 8]);
      d[0] = lo; d[1] = hi;
      interleave(rd[0], rd[1], &lo, &hi);
      d = reinterpret_cast<u32x4*>(&smem[buf][1][ur * 64 + uv * 8]);
      d[0] = lo; d[1] = hi;
    } else {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        *reinterpret_cast<u32x4*>(&smem[buf][0][rl[e] * 64 + uv * 4]) = rx[e];
        *reinterpret_cast<u32x4*>(&smem[buf][1][rl[e] * 64 + uv * 4]) = rd[e];
      }
    }
  };

  f32x16 acc = zero16();
  const int n_steps = (r_end - r_begin + BR - 1) / BR;
  if (n_steps > 0) {
    gload(r_begin);
    lstore(0);
  }
  __syncthreads();
  for (int t = 0; t < n_steps; ++t) {
    if (t + 1 < n_steps) gload(r_begin + (t + 1) * BR);
    const uint32_t* Xs = smem[t & 1][0] + wm * 32 + xi;
    const uint32_t* Ds = smem[t & 1][1] + wn * 32 + xi;
    if (HALF) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint32_t* pa = Xs + (ks * 8 + gk * 4) * 64;
        const uint32_t* pb = Ds + (ks * 8 + gk * 4) * 64;
        const u32x4 a = {pa[0], pa[64], pa[128], pa[192]};
        const u32x4 b = {pb[0], pb[64], pb[128], pb[192]};
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const float a = __uint_as_float(Xs[(ks * 2 + gk) * 64]);
        const float b = __uint_as_float(Ds[(ks * 2 + gk) * 64]);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
      }
    }
    if (t + 1 < n_steps) lstore((t + 1) & 1);
    __syncthreads();
  }

  const int K = 9 * sh.cin;
  float* __restrict__ out = dwp + ((int64_t)(w * n_runs + run) * K + (int64_t)tap * sh.cin) * sh.cout;
  const int col = n0 + wn * 32 + xi;
  if (col < sh.cout) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int c = c0 + wm * 32 + gk * 4 + (v >> 2) * 8 + (v & 3);
      if (c < sh.cin) out[(int64_t)c * sh.cout + col] = acc[v];
    }
  }
}

// The weight gradient for bf16 with C_in a multiple of 64, in padded
// coordinates: a worker's positions form one stream s = image * H*Wp + (hp-1) *
// Wp + wp over the rows hp = 1..H of the padded images (Wp = W + 2; dz is zero
// at the border columns), and the three taps of one kernel row kh are the
// shifts -1, 0, +1 of s in X taken one image row up / level / down.  A
// workgroup owns (kh, 64 x 64 tile of (c, o), run of the stream).  Per step of
// 64 positions it lays into LDS, pixel pairs interleaved per 32-bit word: dz,
// X paired as (2q, 2q+1) [taps -1 and +1 start on such a pair] and X paired as
// (2q+1, 2q+2) [tap 0].  Wave (c half, position half) holds the 3 taps x 2
// output-channel halves of its 32 input channels; the two position halves are
// added through LDS at the end.
constexpr int kRowsBR = 64;
constexpr int kRowsPitch = 72;   // words per pixel-pair row: 64 + 8, so that the two lane groups (4 rows apart) use different banks
constexpr int kRowsLdsWords = (33 + 32 + 32) * kRowsPitch;

__global__ __launch_bounds__(kThreads, 2) void conv3x3_dw_rows_kernel(WorkerTable tab, ConvShape sh,
                                                                      const bf16_t* __restrict__ dz,
                                                                      float* __restrict__ dwp, int n_runs,
                                                                      int run_len) {
  __shared__ __attribute__((aligned(16))) uint32_t smem[2][kRowsLdsWords];
  // Workgroups go to the 8 XCDs round-robin in launch order.  The three kernel rows of one
  // (tile, run, worker) read the same X and dz: they sit 8 apart in launch order, i.e. on one
  // XCD at about the same time, so that two of the three find the data in that XCD's L2.
  const int ct = (sh.cin + 63) / 64, ot = (sh.cout + 63) / 64;
  const int groups = ct * ot * n_runs * sh.n_workers;
  const int slot = blockIdx.x >> 3;
  const int grp = (slot / 3) * 8 + (blockIdx.x & 7);
  if (grp >= groups) return;
  const int kh = slot % 3;
  const int w = grp / (ct * ot * n_runs);
  const int run = (grp / (ct * ot)) % n_runs;
  const int rest = grp % (ct * ot);
  const int c0 = (rest / ot) * 64, n0 = (rest % ot) * 64;
  const int Wp = sh.W + 2, PI = sh.H * Wp;
  const int S = tab.rows[w] * PI;
  const int s_begin = min(run * run_len, S), s_end = min(s_begin + run_len, S);
  const int n_steps = (s_end - s_begin + kRowsBR - 1) / kRowsBR;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5, cti = wv & 1, uh = wv >> 1;
  const int kv = tid & 7, pr = tid >> 3;       // this thread's 8 channels and its pixel pair

  const bf16_t* __restrict__ xw = reinterpret_cast<const bf16_t*>(tab.x[w]);
  const bf16_t* __restrict__ dzw = dz + (int64_t)tab.row_off[w] * sh.HW * sh.cout;
  const bool xcok = c0 + kv * 8 < sh.cin, dcok = n0 + kv * 8 < sh.cout;

  // state of X row l = 2*pr of the current step: stream position s, and its (image pixel base,
  // hp, wp).  Decoded one image ahead so that s = -1 (a border position) needs no special case.
  int ps = s_begin - 1 + 2 * pr;
  int pimg, php, pwp;
  {
    const int sp = ps + PI;
    const int i = sp / PI, rem = sp - i * PI;
    php = rem / Wp;
    pwp = rem - php * Wp;
    php += 1;
    pimg = (i - 1) * sh.HW;
  }
  const int adv_h = kRowsBR / Wp, adv_w = kRowsBR - adv_h * Wp;
  // one step's loads: X rows l .. l+2 (and, for pair 0, rows 64, 65); dz at the positions of rows l+1, l+2
  struct Set { u32x4 rx[5], rd[2]; };
  Set setA, setB;

  // (unsigned compares fold the two-sided range checks; pixel indexes are 32-bit, the byte offset
  // is one 32 x 32 -> 64-bit multiply-add)
  const int xrow_b = sh.cin * 2, drow_b = sh.cout * 2;
  const int xoff_b = (c0 + kv * 8) * 2, doff_b = (n0 + kv * 8) * 2;
  auto x_load = [&](int s, int img, int hp, int wp) -> u32x4 {
    const int hx = hp + kh - 2;                       // image row of the tap, 0-based
    const bool ok = xcok && (unsigned)s < (unsigned)S && (unsigned)(wp - 1) < (unsigned)sh.W &&
                    (unsigned)hx < (unsigned)sh.H;
    const int pix = img + hx * sh.W + (wp - 1);
    return load_or_zero(xw, (int64_t)pix * (int64_t)xrow_b + xoff_b, ok);
  };
  auto d_load = [&](int s, int img, int hp, int wp) -> u32x4 {
    const bool ok = dcok && (unsigned)(s - s_begin) < (unsigned)(s_end - s_begin) &&
                    (unsigned)(wp - 1) < (unsigned)sh.W;
    const int pix = img + (hp - 1) * sh.W + (wp - 1);
    return load_or_zero(dzw, (int64_t)pix * (int64_t)drow_b + doff_b, ok);
  };
  auto next_pos = [&](int& img, int& hp, int& wp) {   // one position on
    if (++wp >= Wp) {
      wp = 0;
      if (++hp > sh.H) { hp = 1; img += sh.HW; }
    }
  };
  auto gload = [&](Set& st) {
    u32x4 (&rx)[5] = st.rx;
    u32x4 (&rd)[2] = st.rd;
    int img = pimg, hp = php, wp = pwp;
    rx[0] = x_load(ps, img, hp, wp);
    next_pos(img, hp, wp);
    rx[1] = x_load(ps + 1, img, hp, wp);
    rd[0] = d_load(ps + 1, img, hp, wp);
    next_pos(img, hp, wp);
    rx[2] = x_load(ps + 2, img, hp, wp);
    rd[1] = d_load(ps + 2, img, hp, wp);
    // advance the state by one step; for pair 0 the new state is row 64 of this step
    ps += kRowsBR;
    pwp += adv_w;
    php += adv_h;
    if (pwp >= Wp) { pwp -= Wp; ++php; }
    while (php > sh.H) { php -= sh.H; pimg += sh.HW; }
    if (pr == 0) {
      img = pimg; hp = php; wp = pwp;
      rx[3] = x_load(ps, img, hp, wp);
      next_pos(img, hp, wp);
      rx[4] = x_load(ps + 1, img, hp, wp);
    }
  };
  auto interleave = [](const u32x4& a, const u32x4& b, u32x4* lo, u32x4* hi) {
    // word j = (a[j], b[j]) as (low half, high half)
    lo->x = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u); lo->y = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
    lo->z = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u); lo->w = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
    hi->x = __builtin_amdgcn_perm(b.z, a.z, 0x05040100u); hi->y = __builtin_amdgcn_perm(b.z, a.z, 0x07060302u);
    hi->z = __builtin_amdgcn_perm(b.w, a.w, 0x05040100u); hi->w = __builtin_amdgcn_perm(b.w, a.w, 0x07060302u);
  };
  auto put = [&](uint32_t* base, int row, const u32x4& a, const u32x4& b) {
    u32x4 lo, hi;
    interleave(a, b, &lo, &hi);
    u32x4* d = reinterpret_cast<u32x4*>(base + row * kRowsPitch + kv * 8);
    d[0] = lo;
    d[1] = hi;
  };
  auto lstore = [&](int buf, const Set& st) {
    const u32x4 (&rx)[5] = st.rx;
    const u32x4 (&rd)[2] = st.rd;
    uint32_t* E = smem[buf];
    put(E, pr, rx[0], rx[1]);
    put(E + 33 * kRowsPitch, pr, rx[1], rx[2]);
    put(E + 65 * kRowsPitch, pr, rd[0], rd[1]);
    if (pr == 0) put(E, 32, rx[3], rx[4]);
  };

  f32x16 acc[3][2];
#pragma unroll
  for (int a = 0; a < 3; ++a) { acc[a][0] = zero16(); acc[a][1] = zero16(); }

  auto compute = [&](int buf) {
    constexpr int P = kRowsPitch;
    const uint32_t* E = smem[buf] + cti * 32 + xi;
    const uint32_t* O = E + 33 * P;
    const uint32_t* D = smem[buf] + 65 * P + xi;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int r = ((uh * 2 + q) * 8 + gk * 4) * P;       // first pair row of this lane's 8 positions
      const u32x4 d0 = {D[r], D[r + P], D[r + 2 * P], D[r + 3 * P]};
      const u32x4 d1 = {D[r + 32], D[r + P + 32], D[r + 2 * P + 32], D[r + 3 * P + 32]};
      const uint32_t e4 = E[r + 4 * P];
      const u32x4 xa = {E[r], E[r + P], E[r + 2 * P], E[r + 3 * P]};     // tap -1
      const u32x4 xc = {xa.y, xa.z, xa.w, e4};                            // tap +1: one pair further
      const u32x4 xb = {O[r], O[r + P], O[r + 2 * P], O[r + 3 * P]};     // tap 0
      acc[0][0] = mma(bf16_t(), xa, d0, acc[0][0]);
      acc[0][1] = mma(bf16_t(), xa, d1, acc[0][1]);
      acc[1][0] = mma(bf16_t(), xb, d0, acc[1][0]);
      acc[1][1] = mma(bf16_t(), xb, d1, acc[1][1]);
      acc[2][0] = mma(bf16_t(), xc, d0, acc[2][0]);
      acc[2][1] = mma(bf16_t(), xc, d1, acc[2][1]);
    }
  };

  // Loads run two steps ahead of the MFMAs: step t+1 sits in one register set, step t+2 in the
  // other, while step t is computed out of LDS.  A set is stored to LDS one step before its
  // use and refilled at once with the step after next.
  if (n_steps > 0) {
    gload(setA);
    lstore(0, setA);
    if (n_steps > 1) gload(setA);
    if (n_steps > 2) gload(setB);
  }
  __syncthreads();
  for (int t = 0; t < n_steps; t += 2) {
    compute(0);
    if (t + 1 < n_steps) lstore(1, setA);
    if (t + 3 < n_steps) gload(setA);
    __syncthreads();
    if (t + 1 < n_steps) {
      compute(1);
      if (t + 2 < n_steps) lstore(0, setB);
      if (t + 4 < n_steps) gload(setB);
      __syncthreads();
    }
  }

  // add the two position halves: waves 2, 3 hand their sums to waves 0, 1
  float* red = reinterpret_cast<float*>(&smem[0][0]);     // 2 waves x 6 tiles x 16 x 64 floats = 48 KB
  if (uh == 1) {
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[((cti * 6 + a * 2 + b) * 16 + v) * 64 + lane] = acc[a][b][v];
  }
  __syncthreads();
  if (uh == 0) {
    const int K = 9 * sh.cin;
    float* __restrict__ out = dwp + ((int64_t)(w * n_runs + run) * K + (int64_t)kh * 3 * sh.cin) * sh.cout;
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int col = n0 + b * 32 + xi;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int c = c0 + cti * 32 + gk * 4 + (v >> 2) * 8 + (v & 3);
          const float sum = acc[a][b][v] + red[((cti * 6 + a * 2 + b) * 16 + v) * 64 + lane];
          if (c < sh.cin && col < sh.cout) out[((int64_t)a * sh.cin + c) * sh.cout + col] = sum;
        }
      }
  }
}

// The weight gradient for bf16, C_in a multiple of 64 and image rows of 31..61
// pixels: all nine taps in one workgroup of twelve wavefronts, one padded image
// row per step.  A worker's padded rows g = image * (H+2) + hx (hx = 0 and H+1
// are the zero rows) slide through a ring in LDS: a step with dz row g needs X
// rows g-1, g, g+1, each laid out once as 66 entries b = wp + 1 (pixel pairs
// interleaved per 32-bit word, zeros at the border), so that tap kw of dz entry
// j = wp is X entry j + kw: taps 0 and 2 start on a word, tap 1 is the funnel
// shift of two neighbouring words.  X and dz are read from memory once.  Wave
// (kernel row kh, c half, o half) holds the three taps of its kernel row for a
// 32 x 32 tile; per step it reads one X row and the dz row.  Threads 0..255
// bring in the X row that enters the ring, threads 256..511 the dz row, two
// 16-byte vectors each, three steps ahead of their use (three register sets
// that take turns); the row decode is wave-uniform.
constexpr int kRingThreads = 768;
constexpr int kRingP = 72;                      // words per pixel-pair row (64 + 8: see kRowsPitch)
constexpr int kRingXWords = 33 * kRingP, kRingDWords = 32 * kRingP;

__global__ __launch_bounds__(kRingThreads, 1) void conv3x3_dw_ring_kernel(WorkerTable tab, ConvShape sh,
                                                                         const bf16_t* __restrict__ dz,
                                                                         float* __restrict__ dwp, int n_runs,
                                                                         int run_rows) {
  __shared__ __attribute__((aligned(16))) uint32_t xs[4][kRingXWords];   // X row r in slot (r + 4) & 3
  __shared__ __attribute__((aligned(16))) uint32_t ds[2][kRingDWords];   // dz row r in slot r & 1
  const int w = blockIdx.z, run = blockIdx.y;
  const int ot = (sh.cout + 63) / 64;
  const int c0 = (blockIdx.x / ot) * 64, n0 = (blockIdx.x % ot) * 64;
  const int HP = sh.H + 2;
  const int G = tab.rows[w] * HP;
  const int g0 = min(run * run_rows, G), g1 = min(g0 + run_rows, G);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int xi = lane & 31, gk = lane >> 5;
  const int kh = wv >> 2, cti = wv & 1, coti = (wv >> 1) & 1;
  // loaders: unit = (pixel pair pr, 8 channels kv) of the X row (role 0) or the dz row (role 1)
  const int role = tid >> 8, kv = tid & 7, pr = (tid >> 3) & 31;

  // with input indexing the X rows come from the dataset: an image's first byte is looked up when
  // the row counter enters the image (wave-uniform, once per H + 2 steps)
  const bool gathered = tab.gsrc != nullptr;
  const bf16_t* __restrict__ xw = reinterpret_cast<const bf16_t*>(gathered ? tab.gsrc : tab.x[w]);
  const bf16_t* __restrict__ dzw = dz + (int64_t)tab.row_off[w] * sh.HW * sh.cout;
  // the unit's two pixels: X entries b = 2pr, 2pr+1 are w = 2pr-2, 2pr-1; dz entries j = 2pr,
  // 2pr+1 are w = 2pr-1, 2pr
  const bool isx = role == 0;
  const int wpx = 2 * pr - (isx ? 2 : 1);
  const int chn = (isx ? c0 : n0) + kv * 8, nch = isx ? sh.cin : sh.cout;
  const bool v0 = role < 2 && chn < nch && wpx >= 0 && wpx < sh.W;
  const bool v1 = role < 2 && chn < nch && wpx + 1 >= 0 && wpx + 1 < sh.W;
  const int64_t off0 = ((int64_t)wpx * nch + chn) * 2, off1 = off0 + (int64_t)nch * 2;
  const int64_t row_bytes = (int64_t)sh.W * nch * 2;
  const bf16_t* __restrict__ src = isx ? xw : dzw;
  const int64_t image_bytes = (int64_t)sh.H * row_bytes;

  struct Row { int g, i, h; int64_t ib; };     // padded row g = i * (H+2) + h (wave-uniform); ib: first byte of image i in src
  auto image_base = [&](int i) -> int64_t {
    if (!(gathered && isx)) return (int64_t)i * image_bytes;
    return (i >= 0 && i < tab.rows[w]) ? gathered_row(tab, tab.row_off[w] + i) * image_bytes : 0;
  };
  auto row_at = [&](int g) {
    Row r;
    r.g = g;
    r.i = (g + HP) / HP - 1;
    r.h = g - r.i * HP;
    r.ib = image_base(r.i);
    return r;
  };
  auto next_row = [&](Row& r) {
    ++r.g;
    if (++r.h == HP) { r.h = 0; ++r.i; r.ib = image_base(r.i); }
  };
  struct Set { u32x4 a, b; };
  // the X loaders take row xr, the dz loaders row dr (a dz row outside the run reads as zeros)
  auto gload = [&](Set& s, const Row& xr, const Row& dr) {
    const Row& r = isx ? xr : dr;
    const bool ok = r.h >= 1 && r.h <= sh.H && (isx ? (r.g >= 0 && r.g < G) : (r.g >= g0 && r.g < g1));
    const int64_t base = r.ib + (int64_t)(r.h - 1) * row_bytes;
    s.a = load_or_zero(src, base + off0, ok && v0);
    s.b = load_or_zero(src, base + off1, ok && v1);
  };
  auto lstore = [&](const Set& s, int xg, int dg) {
    if (role < 2) {
      // word j = (a[j], b[j]) as (low half, high half): entries 2pr and 2pr+1 of 8 channels
      const u32x4& a = s.a;
      const u32x4& b = s.b;
      u32x4 lo, hi;
      lo.x = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u); lo.y = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
      lo.z = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u); lo.w = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
      hi.x = __builtin_amdgcn_perm(b.z, a.z, 0x05040100u); hi.y = __builtin_amdgcn_perm(b.z, a.z, 0x07060302u);
      hi.z = __builtin_amdgcn_perm(b.w, a.w, 0x05040100u); hi.w = __builtin_amdgcn_perm(b.w, a.w, 0x07060302u);
      uint32_t* base = isx ? xs[(xg + 4) & 3] : ds[dg & 1];
      u32x4* d = reinterpret_cast<u32x4*>(base + pr * kRingP + kv * 8);
      d[0] = lo;
      d[1] = hi;
    }
  };

  f32x16 acc[3] = {zero16(), zero16(), zero16()};
  auto compute = [&](int g) {
    const uint32_t* D = ds[g & 1] + coti * 32 + xi;
    const uint32_t* X = xs[(g + kh + 3) & 3] + cti * 32 + xi;     // X row g + kh - 1
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int r = (ks * 8 + gk * 4) * kRingP;
      const u32x4 d = {D[r], D[r + kRingP], D[r + 2 * kRingP], D[r + 3 * kRingP]};
      const uint32_t w0 = X[r], w1 = X[r + kRingP], w2 = X[r + 2 * kRingP], w3 = X[r + 3 * kRingP],
                     w4 = X[r + 4 * kRingP];
      const u32x4 t0 = {w0, w1, w2, w3};
      const u32x4 t1 = {__builtin_amdgcn_alignbit(w1, w0, 16), __builtin_amdgcn_alignbit(w2, w1, 16),
                        __builtin_amdgcn_alignbit(w3, w2, 16), __builtin_amdgcn_alignbit(w4, w3, 16)};
      const u32x4 t2 = {w1, w2, w3, w4};
      acc[0] = mma(bf16_t(), t0, d, acc[0]);
      acc[1] = mma(bf16_t(), t1, d, acc[1]);
      acc[2] = mma(bf16_t(), t2, d, acc[2]);
    }
  };

  const int n_steps = g1 - g0;
  if (n_steps > 0) {
    // entries 64, 65 (pair row 32) of every X slot stay zero: rows are at most 61 pixels wide
    for (int e = tid; e < 4 * 64; e += kRingThreads) xs[e >> 6][32 * kRingP + (e & 63)] = 0u;
    // rows g0-1, g0, g0+1 of X and row g0 of dz go straight to LDS; the rows of the next two
    // steps wait in registers
    Set s0, s1, s2;
    {
      Set a, b;
      Row q = row_at(g0 - 1);
      const Row none = row_at(-1);     // no dz row: -1 is outside every run
      gload(s0, q, row_at(g0));        // X g0-1, dz g0
      next_row(q);
      gload(a, q, none);               // X g0
      next_row(q);
      gload(b, q, none);               // X g0+1
      lstore(s0, g0 - 1, g0);
      if (isx) {
        lstore(a, g0, 0);
        lstore(b, g0 + 1, 0);
      }
    }
    // xr, dr: the rows the next gload brings in.  Before the loop: (X g0+2, dz g0+1) -> s1,
    // (X g0+3, dz g0+2) -> s2; step t then loads (X g0+t+4, dz g0+t+3).
    Row xr = row_at(g0 + 2), dr = row_at(g0 + 1);
    gload(s1, xr, dr);
    next_row(xr); next_row(dr);
    gload(s2, xr, dr);
    next_row(xr); next_row(dr);
    __syncthreads();

    Row cur = row_at(g0);          // only g and h of it are used
    // step: issue the loads of the rows three steps on, compute row cur, store the rows of the
    // next step (loaded two steps ago), barrier.  Every step issues its loads and stores its
    // set, also past the end of the run (rows outside it load as zeros and land in slots nobody
    // reads), and the loop always does three steps per trip: each register set is back in its
    // own registers at the back edge, so no loaded value is ever copied (a copy would force a
    // wait for its load) and the wait before a store is for that set only.
    auto step = [&](Set& issue, const Set& store) {
      gload(issue, xr, dr);
      next_row(xr); next_row(dr);
      if (cur.g < g1 && cur.h >= 1 && cur.h <= sh.H) compute(cur.g);
      lstore(store, cur.g + 2, cur.g + 1);
      next_row(cur);
      __syncthreads();
    };
    for (int t = 0; t < n_steps; t += 3) {
      step(s0, s1);
      step(s1, s2);
      step(s2, s0);
    }
  }

  const int K = 9 * sh.cin;
  float* __restrict__ out = dwp + ((int64_t)(w * n_runs + run) * K + (int64_t)kh * 3 * sh.cin) * sh.cout;
  const int col = n0 + coti * 32 + xi;
  if (col < sh.cout) {
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int c = c0 + cti * 32 + gk * 4 + (v >> 2) * 8 + (v & 3);
        if (c < sh.cin) out[((int64_t)a * sh.cin + c) * sh.cout + col] = acc[a][v];
      }
    }
  }
}

// A wavefront owns 64 consecutive 16-byte vectors of the gradient; the four wavefronts of a
// workgroup take a quarter of the runs each (up to eight loads in flight per thread; a run past
// the quarter's last re-reads it and is dropped), added in run order, and the quarters are added
// in order through LDS.  With one thread adding all runs of its vector the launch was four
// dependent rounds of loads in 288 workgroups.
constexpr int kFoldParts = 4;
__global__ __launch_bounds__(64 * kFoldParts) void conv_dw_fold_kernel(WorkerTable tab, const float* __restrict__ dwp,
                                                                int n_runs, int64_t len) {
  __shared__ __attribute__((aligned(16))) f32x4 part[kFoldParts][64];
  const int w = blockIdx.y, lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int64_t i = ((int64_t)blockIdx.x * 64 + lane) * 4;
  const bool live = i < len;
  const int per = (n_runs + kFoldParts - 1) / kFoldParts;
  const int r_begin = min(q * per, n_runs), r_end = min(r_begin + per, n_runs);
  f32x4 a = {0.f, 0.f, 0.f, 0.f};
  if (live && r_begin < r_end) {
    const float* p = dwp + (int64_t)w * n_runs * len + i;
    for (int r0 = r_begin; r0 < r_end; r0 += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(p + (int64_t)min(r0 + u, r_end - 1) * len);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (r0 + u < r_end) a += v[u];
    }
  }
  part[q][lane] = a;
  __syncthreads();
  if (q == 0 && live) {
    f32x4 t = part[0][lane];
#pragma unroll
    for (int j = 1; j < kFoldParts; ++j) t += part[j][lane];
    *reinterpret_cast<f32x4*>(tab.grad[w] + i) = t;
  }
}

// ------------------------------------------------------------------- host
struct Plan {
  ConvShape sh;
  WorkerTable tab;
  int64_t K, P;
  int max_unit_images, max_rows, n_units, n_runs, run_rows, n_runs_rows, run_len_rows, n_runs_ring, run_rows_ring;
  size_t elem;
  // workspace offsets in bytes
  size_t o_wmat, o_z, o_dz, o_statp, o_mu, o_rstd, o_poolp, o_pooled, o_dpooled, o_dlogits, o_row_loss, o_bwdp,
      o_bmean, o_dwp, total;
  // the indexed call: room for the gathered images and labels (used when its kernels cannot read
  // through the index list and the call gathers first)
  size_t o_xin, o_ylab, total_indexed;
};

// Which convolution kernels a shape takes (both read the images through the index list).
static inline bool patch_kernels_ok(const ConvShape& sh, size_t elem) {
  return elem == 2 && sh.cin % 64 == 0 && sh.W + 2 <= 63;
}
static inline bool hold_kernel_ok(const ConvShape& sh, size_t elem) {
  return patch_kernels_ok(sh, elem) && sh.cin == 64 && sh.cout <= 64;
}
static inline bool ring_kernel_ok(const ConvShape& sh, size_t elem) {
  return patch_kernels_ok(sh, elem) && sh.W >= 31;     // rows wide enough to fill most of a 64-position step
}

int make_plan(const synk_convblock_desc* d, const int64_t* rows, int n_workers, int n_slices, Plan* p) {
  if (!d || !rows) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_slices < 1) return SYNK_ERR_SHAPE;
  if (d->height < 1 || d->width < 1 || d->c_in < 8 || d->c_out < 8 || d->classes < 1) return SYNK_ERR_SHAPE;
  if (d->c_in % 8 || d->c_out % 8 || d->c_out > kMaxCout || d->classes > kMaxClasses) return SYNK_ERR_SHAPE;
  if (d->height > 4096 || d->width > 4096 || d->c_in > 4096) return SYNK_ERR_SHAPE;
  if (!(d->eps >= 0.0f)) return SYNK_ERR_SHAPE;
  if (d->compute_dtype != SYNK_F32 && d->compute_dtype != SYNK_BF16) return SYNK_ERR_DTYPE;
  if ((int64_t)n_workers * n_slices > 65535) return SYNK_ERR_SHAPE;
  ConvShape& sh = p->sh;
  sh.H = d->height; sh.W = d->width; sh.cin = d->c_in; sh.cout = d->c_out; sh.classes = d->classes;
  sh.HW = d->height * d->width;
  sh.n_workers = n_workers; sh.n_slices = n_slices; sh.grad_op = 0;
  sh.n_chunks = (sh.HW + kChunkRows - 1) / kChunkRows;
  sh.eps = d->eps;
  int64_t total = 0;
  p->max_rows = 0;
  p->max_unit_images = 0;
  for (int w = 0; w < n_workers; ++w) {
    if (rows[w] < 0) return SYNK_ERR_SHAPE;
    if (total + rows[w] > (int64_t)1 << 30) return SYNK_ERR_SHAPE;
    p->tab.rows[w] = (int32_t)rows[w];
    p->tab.row_off[w] = (int32_t)total;
    total += rows[w];
    if (rows[w] > p->max_rows) p->max_rows = (int)rows[w];
    const int64_t u = (rows[w] + n_slices - 1) / n_slices;
    if (u > p->max_unit_images) p->max_unit_images = (int)u;
  }
  p->tab.row_off[n_workers] = (int32_t)total;
  if (total == 0) return SYNK_ERR_SHAPE;
  // pixel rows, and every element index derived from them, stay below 2^31 per array dimension
  if (total * sh.HW >= ((int64_t)1 << 31) / 4 || total * sh.n_chunks >= ((int64_t)1 << 31)) return SYNK_ERR_SHAPE;
  sh.total_images = (int)total;
  p->n_units = n_workers * n_slices;
  p->K = (int64_t)9 * sh.cin;
  p->P = param_off(sh.cin, sh.cout, sh.classes).total;
  p->elem = d->compute_dtype == SYNK_BF16 ? 2 : 4;

  // runs of the weight gradient: enough workgroups to fill the chip, few enough to keep the partials small
  const int BR = d->compute_dtype == SYNK_BF16 ? DwGeom<bf16_t>::BR : DwGeom<float>::BR;
  const int64_t tiles = (int64_t)9 * ((sh.cin + 63) / 64) * ((sh.cout + 63) / 64);
  const int64_t max_px = (int64_t)p->max_rows * sh.HW;
  int64_t runs = (1024 + tiles * n_workers - 1) / (tiles * n_workers);
  const int64_t max_runs = (max_px + 4 * BR - 1) / (4 * BR);   // at least four steps per run
  if (runs > max_runs) runs = max_runs;
  if (runs > 64) runs = 64;
  if (runs < 1) runs = 1;
  int64_t rr = (max_px + runs - 1) / runs;
  rr = (rr + BR - 1) / BR * BR;
  p->n_runs = (int)runs;
  p->run_rows = (int)rr;
  {
    // the padded-stream kernel: one workgroup per (kernel row, tile, run, worker), about two per CU
    const int64_t t3 = tiles / 3 * n_workers;
    const int64_t max_s = (int64_t)p->max_rows * sh.H * (sh.W + 2);
    int64_t r2 = (2 * kNumCU) / t3;               // at most two workgroups per CU: one round
    const int64_t cap = (max_s + 4 * kRowsBR - 1) / (4 * kRowsBR);
    if (r2 > cap) r2 = cap;
    if (r2 > 64) r2 = 64;
    if (r2 < 1) r2 = 1;
    int64_t rl = (max_s + r2 - 1) / r2;
    rl = (rl + kRowsBR - 1) / kRowsBR * kRowsBR;
    p->n_runs_rows = (int)r2;
    p->run_len_rows = (int)rl;
    // the ring kernel: one workgroup per (tile, run, worker), about one per CU, a dozen padded
    // image rows or more per run
    const int64_t t9 = tiles / 9 * n_workers;
    const int64_t max_g = (int64_t)p->max_rows * (sh.H + 2);
    int64_t r3 = (kNumCU + t9 - 1) / t9;
    const int64_t cap3 = max_g / 12;
    if (r3 > cap3) r3 = cap3;
    if (r3 > 64) r3 = 64;
    if (r3 < 1) r3 = 1;
    p->n_runs_ring = (int)r3;
    p->run_rows_ring = (int)((max_g + r3 - 1) / r3);
  }

  const int64_t R = total, px = total * sh.HW;
  size_t at = 0;
  auto take = [&](size_t bytes) {
    const size_t o = at;
    at += round_up(bytes, 256);
    return o;
  };
  p->o_wmat = take((size_t)p->K * round_up((size_t)sh.cout, 32) * p->elem);
  p->o_z = take((size_t)px * sh.cout * p->elem);
  p->o_dz = take((size_t)px * sh.cout * p->elem);
  p->o_statp = take((size_t)R * sh.n_chunks * sh.cout * 2 * 4);
  p->o_mu = take((size_t)p->n_units * sh.cout * 4);
  p->o_rstd = take((size_t)p->n_units * sh.cout * 4);
  p->o_poolp = take((size_t)R * sh.n_chunks * sh.cout * 4);
  p->o_pooled = take((size_t)R * sh.cout * 4);
  p->o_dpooled = take((size_t)R * sh.cout * 4);
  p->o_dlogits = take((size_t)R * sh.classes * 4);
  p->o_row_loss = take((size_t)R * 4);
  p->o_bwdp = take((size_t)R * sh.n_chunks * sh.cout * 2 * 4);
  p->o_bmean = take((size_t)p->n_units * sh.cout * 2 * 4);
  const int runs_max = std::max(p->n_runs, std::max(p->n_runs_rows, p->n_runs_ring));
  p->o_dwp = take((size_t)n_workers * runs_max * p->K * sh.cout * 4);
  p->total = at;
  p->o_xin = take((size_t)px * sh.cin * p->elem);
  p->o_ylab = take((size_t)R * 4);
  p->total_indexed = at;
  p->tab.gsrc = nullptr;
  p->tab.gidx = nullptr;
  p->tab.glabels = nullptr;
  p->tab.grows = 0;
  return SYNK_OK;
}

template <typename T>
int run(const Plan& p, const float* params, float* loss, char* ws, hipStream_t st) {
  const ConvShape& sh = p.sh;
  const WorkerTable& tab = p.tab;
  T* wmat = reinterpret_cast<T*>(ws + p.o_wmat);
  T* z = reinterpret_cast<T*>(ws + p.o_z);
  T* dz = reinterpret_cast<T*>(ws + p.o_dz);
  float* statp = reinterpret_cast<float*>(ws + p.o_statp);
  float* mu = reinterpret_cast<float*>(ws + p.o_mu);
  float* rstd = reinterpret_cast<float*>(ws + p.o_rstd);
  float* poolp = reinterpret_cast<float*>(ws + p.o_poolp);
  float* pooled = reinterpret_cast<float*>(ws + p.o_pooled);
  float* dpooled = reinterpret_cast<float*>(ws + p.o_dpooled);
  float* dlogits = reinterpret_cast<float*>(ws + p.o_dlogits);
  float* row_loss = reinterpret_cast<float*>(ws + p.o_row_loss);
  float* bwdp = reinterpret_cast<float*>(ws + p.o_bwdp);
  float* bmean = reinterpret_cast<float*>(ws + p.o_bmean);
  float* dwp = reinterpret_cast<float*>(ws + p.o_dwp);

  const int64_t wn = p.K * sh.cout;
  const bool patch_ok = patch_kernels_ok(sh, sizeof(T)), hold_ok = hold_kernel_ok(sh, sizeof(T));
  if (hold_ok) {
    // the forward kernel lays the weights out itself
  } else if (patch_ok) {
    const int64_t total = p.K * (int64_t)round_up((size_t)sh.cout, 32);
    hipLaunchKernelGGL(conv_weight_frag_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads),
                       0, st, params, reinterpret_cast<uint16_t*>(wmat), sh.cin, sh.cout, total);
  } else {
    hipLaunchKernelGGL(conv_weight_kernel<T>, dim3((unsigned)((wn + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       st, params, wmat, (int)p.K, sh.cout);
  }
  SYNK_LAUNCH_CHECK();
  const dim3 gf((unsigned)(((int64_t)p.max_unit_images * sh.HW + kFwdBM - 1) / kFwdBM),
                (unsigned)((sh.cout + kFwdBN - 1) / kFwdBN), (unsigned)p.n_units);
  if (hold_ok) {
    // units: an image's tiles in per_img runs; per_img so that the rounds of units over the CUs,
    // times a unit's tiles plus one for its start, come out smallest
    const int tiles_per_image = (sh.H * (sh.W + 2) - 2 + kHoldTile - 1) / kHoldTile;
    int per_img = 1;
    int64_t best = -1;
    for (int g = 1; g <= std::min(tiles_per_image, 16); ++g) {
      const int64_t rounds = ((int64_t)sh.total_images * g + kNumCU - 1) / kNumCU;
      const int64_t cost = rounds * ((tiles_per_image + g - 1) / g + 1);
      if (best < 0 || cost < best) { best = cost; per_img = g; }
    }
    const int64_t n_units = (int64_t)sh.total_images * per_img;
    SYNK_LAUNCH_TIMED(conv3x3_fwd_hold_kernel, dim3((unsigned)std::min<int64_t>(kNumCU, n_units)), dim3(kThreads), 0,
                      st, tab, sh, params, reinterpret_cast<bf16_t*>(z), tiles_per_image, per_img, (int)n_units);
  } else if (patch_ok) {
    // 128 positions per workgroup, three workgroups per CU, weights two taps ahead: measured against
    // 256 / two / four (30.7 vs 32.1 us at 64 images of 56 x 56 x 64)
    constexpr int kTile = 128;
    const int tiles_per_image = (sh.H * (sh.W + 2) - 2 + kTile - 1) / kTile;
    const int64_t n_tiles = (int64_t)tiles_per_image * sh.total_images;
    const dim3 gp((unsigned)((n_tiles + 7) / 8 * 8), (unsigned)((sh.cout + 63) / 64));
    SYNK_LAUNCH_TIMED((conv3x3_fwd_patch_kernel<kTile, 3, 2>), gp, dim3(kThreads), 0, st, tab, sh,
                      reinterpret_cast<const bf16_t*>(wmat), reinterpret_cast<bf16_t*>(z), tiles_per_image,
                      (int)n_tiles);
  } else {
    SYNK_LAUNCH_TIMED(conv3x3_fwd_kernel<T>, gf, dim3(kThreads), 0, st, tab, sh, (const T*)wmat, z);
  }
  SYNK_LAUNCH_CHECK();
  const dim3 gc((unsigned)((int64_t)sh.total_images * sh.n_chunks));
  hipLaunchKernelGGL(bn_stats_chunk_kernel<T>, gc, dim3(kThreads), 0, st, tab, sh, (const T*)z, statp);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_stats_unit_kernel, dim3((unsigned)(((int64_t)p.n_units * sh.cout + 3) / 4)), dim3(kThreads), 0,
                     st, tab, sh,
                     (const float*)statp, mu, rstd);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_relu_pool_kernel<T>, gc, dim3(kThreads), 0, st, tab, sh, params, (const T*)z,
                     (const float*)mu, (const float*)rstd, poolp);
  SYNK_LAUNCH_CHECK();
  if (sh.cout <= kHeadHold && sh.classes <= kHeadThreads)
    hipLaunchKernelGGL(head_image_kernel<true>, dim3((unsigned)sh.total_images), dim3(kHeadThreads), 0, st, tab, sh,
                       params, (const float*)poolp, pooled, dlogits, dpooled, row_loss);
  else
    hipLaunchKernelGGL(head_image_kernel<false>, dim3((unsigned)sh.total_images), dim3(kHeadThreads), 0, st, tab, sh,
                       params, (const float*)poolp, pooled, dlogits, dpooled, row_loss);
  SYNK_LAUNCH_CHECK();
  const int class_blocks = (sh.classes + kThreads - 1) / kThreads;
  const int head_blocks = class_blocks * sh.n_workers * ((sh.cout + kWorkerChans - 1) / kWorkerChans);
  hipLaunchKernelGGL(bn_bwd_chunk_kernel<T>, dim3(gc.x + (unsigned)head_blocks), dim3(kThreads), 0, st, tab, sh, params,
                     (const T*)z, (const float*)mu, (const float*)rstd, (const float*)dpooled, bwdp,
                     (const float*)pooled, (const float*)dlogits, (const float*)row_loss, loss, head_blocks,
                     class_blocks);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_bwd_worker_kernel, dim3((unsigned)((sh.n_workers * sh.cout + 3) / 4)), dim3(kThreads), 0, st,
                     tab, sh,
                     (const float*)bwdp, bmean);
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(bn_bwd_dz_kernel<T>, gc, dim3(kThreads), 0, st, tab, sh, params, (const T*)z,
                     (const float*)mu, (const float*)rstd, (const float*)dpooled, (const float*)bmean, dz);
  SYNK_LAUNCH_CHECK();
  const dim3 gd((unsigned)(9 * ((sh.cin + 63) / 64) * ((sh.cout + 63) / 64)), (unsigned)p.n_runs,
                (unsigned)sh.n_workers);
  const bool ring_ok = ring_kernel_ok(sh, sizeof(T));
  int fold_runs = p.n_runs;
  if (ring_ok) {
    fold_runs = p.n_runs_ring;
    const dim3 gg((unsigned)((sh.cin / 64) * ((sh.cout + 63) / 64)), (unsigned)p.n_runs_ring, (unsigned)sh.n_workers);
    hipLaunchKernelGGL(conv3x3_dw_ring_kernel, gg, dim3(kRingThreads), 0, st, tab, sh,
                       reinterpret_cast<const bf16_t*>(dz), dwp, p.n_runs_ring, p.run_rows_ring);
  } else if (patch_ok) {
    fold_runs = p.n_runs_rows;
    const int64_t groups = (int64_t)((sh.cin + 63) / 64) * ((sh.cout + 63) / 64) * p.n_runs_rows * sh.n_workers;
    const dim3 gr((unsigned)(3 * ((groups + 7) / 8) * 8));
    hipLaunchKernelGGL(conv3x3_dw_rows_kernel, gr, dim3(kThreads), 0, st, tab, sh,
                       reinterpret_cast<const bf16_t*>(dz), dwp, p.n_runs_rows, p.run_len_rows);
  } else {
    hipLaunchKernelGGL(conv3x3_dw_kernel<T>, gd, dim3(kThreads), 0, st, tab, sh, (const T*)dz, dwp, p.n_runs,
                       p.run_rows);
  }
  SYNK_LAUNCH_CHECK();
  hipLaunchKernelGGL(conv_dw_fold_kernel, dim3((unsigned)((wn / 4 + 63) / 64), (unsigned)sh.n_workers),
                     dim3(64 * kFoldParts), 0, st, tab, (const float*)dwp, fold_runs, wn);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

}  // namespace
}  // namespace synk

using namespace synk;

extern "C" int synk_convblock_param_count(const synk_convblock_desc* d, int64_t* count) {
  if (!d || !count) return SYNK_ERR_NULL;
  const int64_t one = 1;
  Plan p;
  const int st = make_plan(d, &one, 1, 1, &p);
  if (st != SYNK_OK) return st;
  *count = p.P;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_conv_workspace_bytes(const synk_convblock_desc* d, const int64_t* rows,
                                                     int n_workers, int n_slices, size_t* bytes) {
  if (!bytes) return SYNK_ERR_NULL;
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  *bytes = p.total;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_conv(const synk_convblock_desc* d, const float* params, const void* const* x,
                                     const int32_t* const* y, const int64_t* rows, int n_workers, int n_slices,
                                     int grad_op, float* const* grad, float* loss, void* ws, size_t ws_bytes,
                                     void* stream) {
  if (!d || !params || !x || !y || !rows || !grad || !loss) return SYNK_ERR_NULL;
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  if (grad_op != SYNK_SUM && grad_op != SYNK_MEAN) return SYNK_ERR_OP;
  p.sh.grad_op = grad_op;
  if (!aligned_to(params, 16)) return SYNK_ERR_ALIGN;
  for (int w = 0; w < n_workers; ++w) {
    if (!grad[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grad[w], 16)) return SYNK_ERR_ALIGN;
    if (rows[w] > 0) {
      if (!x[w] || !y[w]) return SYNK_ERR_NULL;
      if (!aligned_to(x[w], 16)) return SYNK_ERR_ALIGN;
    }
    p.tab.x[w] = x[w];
    p.tab.y[w] = y[w];
    p.tab.grad[w] = grad[w];
  }
  for (int w = n_workers; w < SYNK_MAX_WORKERS; ++w) {
    p.tab.x[w] = nullptr; p.tab.y[w] = nullptr; p.tab.grad[w] = nullptr;
    p.tab.rows[w] = 0; p.tab.row_off[w + 1] = p.tab.row_off[n_workers];
  }
  if (!ws || !aligned_to(ws, 256) || ws_bytes < p.total) return SYNK_ERR_WORKSPACE;
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  if (d->compute_dtype == SYNK_BF16) return run<bf16_t>(p, params, loss, reinterpret_cast<char*>(ws), s);
  return run<float>(p, params, loss, reinterpret_cast<char*>(ws), s);
}

extern "C" int synk_sliced_grad_conv_indexed_workspace_bytes(const synk_convblock_desc* d, int64_t n_idx,
                                                             int n_workers, int n_slices, size_t* bytes) {
  if (!bytes) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_idx < 1) return SYNK_ERR_SHAPE;
  int64_t rows[SYNK_MAX_WORKERS];
  for (int w = 0; w < n_workers; ++w) {
    int64_t start;
    share(n_idx, n_workers, w, &start, &rows[w]);
  }
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  *bytes = p.total_indexed;
  return SYNK_OK;
}

extern "C" int synk_sliced_grad_conv_indexed(const synk_convblock_desc* d, const float* params, const void* data,
                                             const int32_t* labels, int64_t n_data, const int32_t* idx,
                                             int64_t n_idx, int n_workers, int n_slices, int grad_op,
                                             float* const* grad, float* loss, void* ws, size_t ws_bytes,
                                             void* stream) {
  if (!d || !params || !data || !labels || !idx || !grad || !loss) return SYNK_ERR_NULL;
  if (n_workers < 1 || n_workers > SYNK_MAX_WORKERS || n_idx < 1 || n_data < 1 || n_data > 0x7fffffff)
    return SYNK_ERR_SHAPE;
  int64_t rows[SYNK_MAX_WORKERS];
  for (int w = 0; w < n_workers; ++w) {
    int64_t start;
    share(n_idx, n_workers, w, &start, &rows[w]);
  }
  Plan p;
  const int st = make_plan(d, rows, n_workers, n_slices, &p);
  if (st != SYNK_OK) return st;
  if (grad_op != SYNK_SUM && grad_op != SYNK_MEAN) return SYNK_ERR_OP;
  p.sh.grad_op = grad_op;
  if (!aligned_to(params, 16) || !aligned_to(data, 16) || !aligned_to(labels, 4) || !aligned_to(idx, 4))
    return SYNK_ERR_ALIGN;
  for (int w = 0; w < n_workers; ++w) {
    if (!grad[w]) return SYNK_ERR_NULL;
    if (!aligned_to(grad[w], 16)) return SYNK_ERR_ALIGN;
  }
  if (!ws || !aligned_to(ws, 256) || ws_bytes < p.total_indexed) return SYNK_ERR_WORKSPACE;
  char* wsb = reinterpret_cast<char*>(ws);
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const int64_t row_elems = (int64_t)p.sh.HW * p.sh.cin;
  const bool through_index = ring_kernel_ok(p.sh, p.elem);   // both convolution kernels read through the list
  void* xw[SYNK_MAX_WORKERS];
  int32_t* yw[SYNK_MAX_WORKERS];
  for (int w = 0; w < SYNK_MAX_WORKERS; ++w) {
    const bool live = w < n_workers;
    xw[w] = live ? wsb + p.o_xin + (size_t)p.tab.row_off[w] * row_elems * p.elem : nullptr;
    yw[w] = live ? reinterpret_cast<int32_t*>(wsb + p.o_ylab) + p.tab.row_off[w] : nullptr;
    p.tab.x[w] = through_index ? nullptr : xw[w];
    p.tab.y[w] = through_index ? nullptr : yw[w];
    p.tab.grad[w] = live ? grad[w] : nullptr;
    if (!live) { p.tab.rows[w] = 0; p.tab.row_off[w + 1] = p.tab.row_off[n_workers]; }
  }
  if (through_index) {
    p.tab.gsrc = data;
    p.tab.gidx = idx;
    p.tab.glabels = labels;
    p.tab.grows = (int32_t)n_data;
  } else {
    const int dt = d->compute_dtype;
    ProfileHold hold;   // a pending event pair is for the forward convolution, not for the gather
    if (int rc = synk_gather_rows(data, n_data, row_elems, dt, idx, n_idx, xw, n_workers, dt, nullptr, 0, labels, yw,
                                  0, nullptr, 0, stream))
      return rc;
  }
  if (d->compute_dtype == SYNK_BF16) return run<bf16_t>(p, params, loss, wsb, s);
  return run<float>(p, params, loss, wsb, s);
}
