// Six-output evaluation over slices with on-GPU aggregation (Sec. 3.1: one
// reduce/gather op per output; Sec. 5.1: slice results aggregated in place).
//
// Stage 1 (one pass over the logits, bound by HBM bandwidth): a group of 16,
// 32 or 64 lanes holds a row in registers and computes arg-max, max, min and
// the log-sum-exp, merged across the group with shuffles; a workgroup covers a
// run of rows of ONE slice and leaves per-(slice, chunk) partial results and
// the rows' arg-max classes.
// Stage 2 folds chunk partials into slice results and slice results into the
// outputs with each output's op, in a fixed order (no float atomics), and
// counts the arg-max classes (integer atomics: exact in any order).
#include <math.h>

#include <mutex>

#include "common.h"

namespace synk {

constexpr int kEBlock = 256;
constexpr int kEWaves = kEBlock / kWave;
constexpr int kRowsPerBlock = 32;
// Rows of a workgroup of the branch-free kernel: 32 lanes a row, one row pair a wavefront.
constexpr int kRegularG = 32, kRegularUPL = 8;
constexpr int kRegularRows = kEWaves * (kWave / kRegularG);
constexpr int kMaxClasses = 4096;

// One workgroup's partial results: cross-entropy sum, max, min and (as bits) the
// count of correct rows, in one 16-byte record so that stage 1 leaves them with one
// store and stage 2 fetches them with one load.
struct EvalWs {
  f32x4* part;           // [S x CH] {ce, max, min, correct}
};

__device__ __forceinline__ f32x4 pack_partial(float ce, float mx, float mn, int correct) {
  return f32x4{ce, mx, mn, __int_as_float(correct)};
}

// Workgroups (= partial results) a slice takes at rows_per_block rows each.
static inline size_t eval_chunks(int64_t rows, int n_slices, int rows_per_block) {
  const int64_t longest = (rows + n_slices - 1) / n_slices;
  int64_t ch = (longest + rows_per_block - 1) / rows_per_block;
  return (size_t)(ch < 1 ? 1 : ch);
}

static inline size_t eval_ws_layout(int64_t rows, int64_t classes, int n_slices, void* ws,
                                    EvalWs* out) {
  const size_t ch = eval_chunks(rows, n_slices, kRegularRows);   // the finest split any kernel uses
  if (out) out->part = reinterpret_cast<f32x4*>(ws);
  return round_up((size_t)n_slices * ch * sizeof(f32x4), 1024);
}

// The first workgroup of stage 1 clears the class counts that stage 2 adds into
// (a launch of its own for that costs more than the whole of stage 2).
__device__ __forceinline__ void clear_counts(int32_t* __restrict__ class_counts, int classes) {
  if (blockIdx.x == 0 && blockIdx.y == 0)
    for (int c = threadIdx.x; c < classes; c += kEBlock) class_counts[c] = 0;
}

// A row without a largest element has no arg-max: whatever the scan left is brought into range (class 0).
__device__ __forceinline__ int in_range(int arg, int classes) {
  return (unsigned)arg < (unsigned)classes ? arg : 0;
}

struct RowStat {
  float m;     // running max (also the row max)
  float s;     // sum of exp(x - m)
  float mn;    // row min
  int arg;     // index of the first maximum
  float xy;    // logit of the label class (0 if the label is out of range)
};

__device__ __forceinline__ void take(RowStat& st, float x, int c, int y) {
  if (x > st.m) {
    st.s = st.s * __expf(st.m - x) + 1.0f;
    st.m = x;
    st.arg = c;
  } else {
    st.s += __expf(x - st.m);
  }
  st.mn = fminf(st.mn, x);
  if (c == y) st.xy = x;
}

// Generic stage 1 (any class count, any alignment): one wavefront per row,
// scalar loads, running (max, sum) pair merged over the 64 lanes.
__global__ __launch_bounds__(kEBlock) void eval_stage1_generic_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ labels, int64_t rows, int classes,
    int n_slices, int chunks, EvalWs ws, int32_t* __restrict__ argmax_out, int32_t* __restrict__ class_counts) {
  clear_counts(class_counts, classes);
  const int slice = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t base = rows / n_slices, extra = rows % n_slices;
  const int64_t s_rows = base + (slice < extra ? 1 : 0);
  const int64_t s_start = base * slice + (slice < extra ? slice : extra);
  const int64_t r0 = (int64_t)chunk * kRowsPerBlock;
  int64_t r1 = r0 + kRowsPerBlock;
  if (r1 > s_rows) r1 = s_rows;

  float w_ce = 0.0f, w_max = -INFINITY, w_min = INFINITY;
  int w_correct = 0;
  for (int64_t r = r0 + wave; r < r1; r += kEWaves) {
    const int64_t row = s_start + r;
    const float* x = logits + row * classes;
    const int y = labels[row];
    RowStat st{-INFINITY, 0.0f, INFINITY, 0x7fffffff, 0.0f};
    for (int c = lane; c < classes; c += kWave) take(st, x[c], c, y);
    // merge the 64 lanes: larger max wins, equal maxima keep the lower index
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      const float om = __shfl_xor(st.m, off);
      const float os = __shfl_xor(st.s, off);
      const float omn = __shfl_xor(st.mn, off);
      const int oarg = __shfl_xor(st.arg, off);
      const float oxy = __shfl_xor(st.xy, off);
      const float nm = fmaxf(st.m, om);
      // lanes that saw no element have m = -inf and s = 0
      const float sa = (st.m == nm) ? st.s : st.s * __expf(st.m - nm);
      const float sb = (om == nm) ? os : os * __expf(om - nm);
      if (om > st.m || (om == st.m && oarg < st.arg)) st.arg = oarg;
      st.s = sa + sb;
      st.m = nm;
      st.mn = fminf(st.mn, omn);
      st.xy += oxy;   // exactly one lane holds a non-zero value
    }
    if (lane == 0) {
      w_ce += (__logf(st.s) + st.m) - st.xy;
      w_max = fmaxf(w_max, st.m);
      w_min = fminf(w_min, st.mn);
      const int arg = in_range(st.arg, classes);
      w_correct += (arg == y) ? 1 : 0;
      argmax_out[row] = arg;
    }
  }
  __shared__ float s_ce[kEWaves], s_max[kEWaves], s_min[kEWaves];
  __shared__ int s_cor[kEWaves];
  if (lane == 0) {
    s_ce[wave] = w_ce;
    s_max[wave] = w_max;
    s_min[wave] = w_min;
    s_cor[wave] = w_correct;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float ce = s_ce[0], mx = s_max[0], mn = s_min[0];
    int cor = s_cor[0];
    for (int w = 1; w < kEWaves; ++w) {
      ce += s_ce[w];
      mx = fmaxf(mx, s_max[w]);
      mn = fminf(mn, s_min[w]);
      cor += s_cor[w];
    }
    const int64_t o = (int64_t)slice * chunks + chunk;
    ws.part[o] = pack_partial(ce, mx, mn, cor);
  }
}

// Fast stage 1 (class count a multiple of 4, 16-byte aligned rows): G lanes
// share a row, so a wavefront works on 64/G rows at once and the cross-lane
// merges span only G lanes.  The whole row sits in registers (UPL 16-byte
// vectors per lane): one HBM read, the maximum is reduced first and the
// exponentials are taken against the final maximum.
template <int G, int UPL>
__global__ __launch_bounds__(kEBlock) void eval_stage1_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ labels, int64_t rows, int classes,
    int n_slices, int chunks, EvalWs ws, int32_t* __restrict__ argmax_out, int32_t* __restrict__ class_counts) {
  constexpr int RW = kWave / G;            // rows a wavefront handles at once
  constexpr int NACC = kEWaves * RW;       // per-block accumulators
  constexpr float kLog2e = 1.4426950408889634f;
  clear_counts(class_counts, classes);
  const int slice = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane % G, grp = lane / G;
  const int units = classes >> 2;
  const int64_t base = rows / n_slices, extra = rows % n_slices;
  const int64_t s_rows = base + (slice < extra ? 1 : 0);
  const int64_t s_start = base * slice + (slice < extra ? slice : extra);
  const int64_t r0 = (int64_t)chunk * kRowsPerBlock;
  int64_t r1 = r0 + kRowsPerBlock;
  if (r1 > s_rows) r1 = s_rows;

  float w_ce = 0.0f, w_max = -INFINITY, w_min = INFINITY;
  int w_correct = 0;
  for (int64_t rb = r0 + (int64_t)wave * RW; rb < r1; rb += (int64_t)kEWaves * RW) {
    const int64_t r = rb + grp;
    const bool valid = r < r1;
    const int64_t row = s_start + (valid ? r : r0);
    const f32x4* x = reinterpret_cast<const f32x4*>(logits + row * classes);
    f32x4 q[UPL];
#pragma unroll
    for (int k = 0; k < UPL; ++k) {
      const int u = k * G + sub;
      if (valid && u < units) q[k] = __builtin_nontemporal_load(x + u);
      else q[k] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    }
    const int y = valid ? labels[row] : -1;
    // label logit: one extra load of a line this wavefront has just requested
    const float xy = (valid && y >= 0 && y < classes) ? logits[row * classes + y] : 0.0f;

    // lane-local maximum and minimum; padding is -inf, so the minimum skips it
    float m = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int k = 0; k < UPL; ++k) {
      m = fmaxf(m, fmaxf(fmaxf(q[k].x, q[k].y), fmaxf(q[k].z, q[k].w)));
      const float lo = fminf(fminf(q[k].x, q[k].y), fminf(q[k].z, q[k].w));
      if (k * G + sub < units) mn = fminf(mn, lo);
    }
    // first position of the lane-local maximum (scan downwards, keep the last hit)
    int arg = 0x7fffffff;
#pragma unroll
    for (int k = UPL - 1; k >= 0; --k) {
      const int c = (k * G + sub) << 2;
      if (q[k].w == m) arg = c + 3;
      if (q[k].z == m) arg = c + 2;
      if (q[k].y == m) arg = c + 1;
      if (q[k].x == m) arg = c;
    }
    if (m == -INFINITY) arg = 0x7fffffff;   // lane holds padding only
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) {
      const float om = __shfl_xor(m, off);
      const int oarg = __shfl_xor(arg, off);
      if (om > m || (om == m && oarg < arg)) arg = oarg;
      m = fmaxf(m, om);
    }
    const float mb = m * kLog2e;
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < UPL; ++k) {
      // arguments are <= 0: the raw hardware exp2 (no denormal fix-up) is exact enough
      s += __builtin_amdgcn_exp2f(fmaf(q[k].x, kLog2e, -mb)) + __builtin_amdgcn_exp2f(fmaf(q[k].y, kLog2e, -mb)) +
           __builtin_amdgcn_exp2f(fmaf(q[k].z, kLog2e, -mb)) + __builtin_amdgcn_exp2f(fmaf(q[k].w, kLog2e, -mb));
    }
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) {
      s += __shfl_xor(s, off);
      mn = fminf(mn, __shfl_xor(mn, off));
    }
    if (sub == 0 && valid) {
      w_ce += (__logf(s) + m) - xy;
      w_max = fmaxf(w_max, m);
      w_min = fminf(w_min, mn);
      arg = in_range(arg, classes);
      w_correct += (arg == y) ? 1 : 0;
      argmax_out[row] = arg;
    }
  }
  __shared__ float s_ce[NACC], s_max[NACC], s_min[NACC];
  __shared__ int s_cor[NACC];
  if (sub == 0) {
    s_ce[wave * RW + grp] = w_ce;
    s_max[wave * RW + grp] = w_max;
    s_min[wave * RW + grp] = w_min;
    s_cor[wave * RW + grp] = w_correct;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float ce = s_ce[0], mx = s_max[0], mn = s_min[0];
    int cor = s_cor[0];
    for (int w = 1; w < NACC; ++w) {
      ce += s_ce[w];
      mx = fmaxf(mx, s_max[w]);
      mn = fminf(mn, s_min[w]);
      cor += s_cor[w];
    }
    const int64_t o = (int64_t)slice * chunks + chunk;
    ws.part[o] = pack_partial(ce, mx, mn, cor);
  }
}

// The same stage 1 without a branch in the load path, for the regular case:
// every slice is a whole number of row sets (kEWaves * 64/G rows, one set per
// workgroup) and a row needs all UPL vectors of its lane group ((UPL-1)*G <
// classes/4 <= UPL*G).  Every load is issued unconditionally before the first
// use (the last vector's address is clamped into the row, its padding applied
// when it is used), so nothing waits behind a condition.  Measured on 65,536
// rows of 1,000 classes: many short-lived workgroups of one set each stream
// faster than longer ones that pipeline several sets through two register
// buffers (G = 32, one set: 43.5 us; G = 16, one / two / four / eight sets:
// 47.1 / 48.3 / 49.7 / 52.5 us), and 32 lanes a row beat 16 and 64.  The register
// budget is set for five wavefronts per SIMD: whole call 45.1 us against 46.0 at the
// seven the compiler picks by itself, 45.4 at six, 46.5 at four and 48.1 at eight
// (16 rows per 512-thread workgroup: 45.1 as well).
template <int G, int UPL>
__global__ __launch_bounds__(kEBlock) __attribute__((amdgpu_waves_per_eu(1, 5))) void eval_stage1_regular_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ labels, int64_t rows, int classes,
    int n_slices, int chunks, EvalWs ws, int32_t* __restrict__ argmax_out, int32_t* __restrict__ class_counts) {
  constexpr int RW = kWave / G;            // rows a wavefront handles at once
  constexpr int NACC = kEWaves * RW;       // rows of the workgroup = per-block accumulators
  constexpr float kLog2e = 1.4426950408889634f;
  clear_counts(class_counts, classes);
  const int slice = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane % G, grp = lane / G;
  const int units = classes >> 2;
  const int64_t s_rows = rows / n_slices;                     // the same for every slice here
  const int64_t row = s_rows * slice + (int64_t)chunk * NACC + wave * RW + grp;

  const int u_last = (UPL - 1) * G + sub;                     // this lane's last vector
  const bool last_in = u_last < units;
  const int u_last_c = last_in ? u_last : units - 1;
  const float pad_ub = last_in ? INFINITY : -INFINITY;

  const int y = labels[row];
  const f32x4* x = reinterpret_cast<const f32x4*>(logits + row * classes);
  f32x4 q[UPL];
#pragma unroll
  for (int k = 0; k < UPL - 1; ++k) q[k] = __builtin_nontemporal_load(x + k * G + sub);
  q[UPL - 1] = __builtin_nontemporal_load(x + u_last_c);
  float m = -INFINITY, mn = INFINITY;
#pragma unroll
  for (int k = 0; k < UPL - 1; ++k) {
    m = fmaxf(m, fmaxf(fmaxf(q[k].x, q[k].y), fmaxf(q[k].z, q[k].w)));
    mn = fminf(mn, fminf(fminf(q[k].x, q[k].y), fminf(q[k].z, q[k].w)));
  }
  {
    // padding by arithmetic, not by a branch: the load above must stay unconditional
    f32x4& v = q[UPL - 1];
    const float lo = fminf(fminf(v.x, v.y), fminf(v.z, v.w));
    mn = fminf(mn, fmaxf(lo, -pad_ub));                      // +inf where the lane holds padding
    v = f32x4{fminf(v.x, pad_ub), fminf(v.y, pad_ub), fminf(v.z, pad_ub), fminf(v.w, pad_ub)};   // -inf there
    m = fmaxf(m, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
  }
  // first position of the lane-local maximum (scan downwards, keep the last hit)
  int arg = 0x7fffffff;
#pragma unroll
  for (int k = UPL - 1; k >= 0; --k) {
    const int c = (k * G + sub) << 2;
    if (q[k].w == m) arg = c + 3;
    if (q[k].z == m) arg = c + 2;
    if (q[k].y == m) arg = c + 1;
    if (q[k].x == m) arg = c;
  }
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) {
    const float om = __shfl_xor(m, off);
    const int oarg = __shfl_xor(arg, off);
    if (om > m || (om == m && oarg < arg)) arg = oarg;
    m = fmaxf(m, om);
  }
  const float mb = m * kLog2e;
  float sum = 0.0f;
#pragma unroll
  for (int k = 0; k < UPL; ++k) {
    // arguments are <= 0: the raw hardware exp2 (no denormal fix-up) is exact enough
    sum += __builtin_amdgcn_exp2f(fmaf(q[k].x, kLog2e, -mb)) + __builtin_amdgcn_exp2f(fmaf(q[k].y, kLog2e, -mb)) +
           __builtin_amdgcn_exp2f(fmaf(q[k].z, kLog2e, -mb)) + __builtin_amdgcn_exp2f(fmaf(q[k].w, kLog2e, -mb));
  }
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) {
    sum += __shfl_xor(sum, off);
    mn = fminf(mn, __shfl_xor(mn, off));
  }

  __shared__ float s_ce[NACC], s_max[NACC], s_min[NACC];
  __shared__ int s_cor[NACC];
  // The logit of the label's class out of the row in registers (vector k of lane sub holds classes
  // 4*(k*G+sub) .. +3): the lane that holds it picks it, the others contribute 0, and a G-lane shuffle
  // sum hands it to every lane; 0 for a label outside [0, classes); a padding vector (index >=
  // classes / 4) is never the one picked.  A load of logits[row*classes + y] instead depends on the
  // label load: one more memory round trip per workgroup (0.2 us over the call's 8,192 workgroups).
  float label_logit;
  {
    const int uy = y >> 2, ky = uy / G, sy = uy % G, ey = y & 3;
    f32x4 v = q[0];
#pragma unroll
    for (int k = 1; k < UPL; ++k)
      if (ky == k) v = q[k];
    float t = ey == 0 ? v.x : (ey == 1 ? v.y : (ey == 2 ? v.z : v.w));
    t = (sub == sy && (unsigned)y < (unsigned)classes) ? t : 0.0f;
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) t += __shfl_xor(t, off);
    label_logit = t;
  }
  if (sub == 0) {
    s_ce[wave * RW + grp] = (__logf(sum) + m) - label_logit;
    s_max[wave * RW + grp] = m;
    s_min[wave * RW + grp] = mn;
    arg = in_range(arg, classes);
    s_cor[wave * RW + grp] = (arg == y) ? 1 : 0;
    argmax_out[row] = arg;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float ce = s_ce[0], mx = s_max[0], mnb = s_min[0];
    int cor = s_cor[0];
    for (int w = 1; w < NACC; ++w) {
      ce += s_ce[w];
      mx = fmaxf(mx, s_max[w]);
      mnb = fminf(mnb, s_min[w]);
      cor += s_cor[w];
    }
    const int64_t o = (int64_t)slice * chunks + chunk;
    ws.part[o] = pack_partial(ce, mx, mnb, cor);
  }
}

// Stage 2.  Block 0 (dispatched first: it is the longer path) folds the partial
// results: 16 lanes share a slice, every lane fetches its chunks' records in one
// batch of 16-byte loads (eight at a time), a fixed 16-lane shuffle tree gives the
// slice result, and the slice results are folded with each output's op in slice
// order (per lane group, then over the 64 lane groups in order).  The other blocks
// meanwhile: a histogram of the rows' arg-max classes, built in LDS over the
// block's share of the rows and added into class_counts (integer sums: any order
// gives the same counts; summed over slices, the counts do not depend on where
// the slices are cut).  Measured on 65,536 rows in 64 slices (8,192 records),
// time of the call beyond stage 1: an empty second launch 0.8 us, the histogram
// blocks alone 2.2, a fold with one wavefront per slice and four 4-byte loads
// per record 6.8, this fold 4.6 with 4-byte loads and 3.4 with 16-byte records.
constexpr int kE2Block = 1024;
constexpr int kE2RowsPerBlock = 2048;
constexpr int kFoldLanes = 16;                       // lanes that share a slice
constexpr int kFoldPerWave = kWave / kFoldLanes;     // slices a wavefront folds at once
constexpr int kFoldBatch = 8;                        // records a lane fetches before it uses the first

__global__ __launch_bounds__(kE2Block) void eval_stage2_kernel(
    EvalWs ws, int64_t rows, int n_slices, int chunks, int classes,
    const int32_t* __restrict__ argmax, float* __restrict__ ce_sum,
    int32_t* __restrict__ class_counts, float* __restrict__ max_logit,
    float* __restrict__ min_logit, int32_t* __restrict__ n_correct) {
  if (blockIdx.x != 0) {
    __shared__ int32_t hist[kMaxClasses];
    for (int c = threadIdx.x; c < classes; c += kE2Block) hist[c] = 0;
    __syncthreads();
    const int64_t stride = (int64_t)(gridDim.x - 1) * kE2Block;
    for (int64_t r = (int64_t)(blockIdx.x - 1) * kE2Block + threadIdx.x; r < rows; r += stride) {
      const int a = argmax[r];
      if ((unsigned)a < (unsigned)classes) atomicAdd(&hist[a], 1);
    }
    __syncthreads();
    for (int c = threadIdx.x; c < classes; c += kE2Block) {
      const int32_t v = hist[c];
      if (v != 0) atomicAdd(class_counts + c, v);
    }
    return;
  }
  constexpr int NW = kE2Block / kWave;
  constexpr int NACC = NW * kFoldPerWave;            // lane groups of the block
  __shared__ float s_ce[NACC], s_max[NACC], s_min[NACC];
  __shared__ int s_cor[NACC];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane % kFoldLanes, grp = lane / kFoldLanes;
  float ce = 0.0f, mx = -INFINITY, mn = INFINITY;   // this lane group's slices, in slice order
  int cor = 0;
  for (int s0 = 0; s0 < n_slices; s0 += NACC) {
    const int s = s0 + wave * kFoldPerWave + grp;
    float sce = 0.0f, smx = -INFINITY, smn = INFINITY;
    int scor = 0;
    if (s < n_slices) {
      const f32x4* rec = ws.part + (int64_t)s * chunks;
      for (int k0 = sub; k0 < chunks; k0 += kFoldLanes * kFoldBatch) {
        f32x4 q[kFoldBatch];
#pragma unroll
        for (int u = 0; u < kFoldBatch; ++u) {
          const int k = k0 + u * kFoldLanes;
          q[u] = k < chunks ? rec[k] : pack_partial(0.0f, -INFINITY, INFINITY, 0);
        }
#pragma unroll
        for (int u = 0; u < kFoldBatch; ++u) {
          sce += q[u].x;
          smx = fmaxf(smx, q[u].y);
          smn = fminf(smn, q[u].z);
          scor += __float_as_int(q[u].w);
        }
      }
    }
#pragma unroll
    for (int off = kFoldLanes / 2; off > 0; off >>= 1) {
      sce += __shfl_xor(sce, off);
      smx = fmaxf(smx, __shfl_xor(smx, off));
      smn = fminf(smn, __shfl_xor(smn, off));
      scor += __shfl_xor(scor, off);
    }
    ce += sce;              // op SUM over slices
    mx = fmaxf(mx, smx);    // op MAX
    mn = fminf(mn, smn);    // op MIN
    cor += scor;            // op SUM (int)
  }
  if (sub == 0) {
    s_ce[wave * kFoldPerWave + grp] = ce;
    s_max[wave * kFoldPerWave + grp] = mx;
    s_min[wave * kFoldPerWave + grp] = mn;
    s_cor[wave * kFoldPerWave + grp] = cor;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tce = s_ce[0], tmx = s_max[0], tmn = s_min[0];
    int tcor = s_cor[0];
    for (int k = 1; k < NACC; ++k) {
      tce += s_ce[k];
      tmx = fmaxf(tmx, s_max[k]);
      tmn = fminf(tmn, s_min[k]);
      tcor += s_cor[k];
    }
    ce_sum[0] = tce;
    max_logit[0] = tmx;
    min_logit[0] = tmn;
    n_correct[0] = tcor;
  }
}

}  // namespace synk

using namespace synk;

static int eval_check(int64_t rows, int64_t classes, int n_slices) {
  if (rows < 1 || classes < 1 || classes > kMaxClasses || n_slices < 1) return SYNK_ERR_SHAPE;
  if (n_slices > 65535) return SYNK_ERR_UNSUPPORTED;
  if (eval_chunks(rows, n_slices, kRegularRows) > 0x7fffffffULL) return SYNK_ERR_UNSUPPORTED;
  return SYNK_OK;
}

extern "C" int synk_sliced_eval_workspace_bytes(int64_t rows, int64_t classes, int n_slices,
                                                size_t* bytes) {
  if (!bytes) return SYNK_ERR_NULL;
  if (int rc = eval_check(rows, classes, n_slices)) return rc;
  *bytes = eval_ws_layout(rows, classes, n_slices, nullptr, nullptr);
  return SYNK_OK;
}

// Argument checks common to both entry points (no HIP call).
static int eval_args_check(const float* logits, const int32_t* labels, int64_t rows, int64_t classes,
                           int n_slices, float* ce_sum, int32_t* class_counts, float* max_logit,
                           float* min_logit, int32_t* n_correct, int32_t* argmax) {
  if (!logits || !labels || !ce_sum || !class_counts || !max_logit || !min_logit || !n_correct ||
      !argmax)
    return SYNK_ERR_NULL;
  if (int rc = eval_check(rows, classes, n_slices)) return rc;
  if (!aligned_to(logits, 4) || !aligned_to(labels, 4) || !aligned_to(argmax, 4) ||
      !aligned_to(class_counts, 4) || !aligned_to(ce_sum, 4) || !aligned_to(max_logit, 4) ||
      !aligned_to(min_logit, 4) || !aligned_to(n_correct, 4))
    return SYNK_ERR_ALIGN;
  return SYNK_OK;
}

// The two launches of a call, with the partial results in `w`.
static int eval_launch(const float* logits, const int32_t* labels, int64_t rows, int64_t classes,
                       int n_slices, float* ce_sum, int32_t* class_counts, float* max_logit,
                       float* min_logit, int32_t* n_correct, int32_t* argmax, const EvalWs& w,
                       hipStream_t s) {
  constexpr int kUnitsLo = (kRegularUPL - 1) * kRegularG, kUnitsHi = kRegularUPL * kRegularG;   // vectors a row
  const bool regular = classes % 4 == 0 && aligned_to(logits, 16) && rows % ((int64_t)n_slices * kRegularRows) == 0 &&
                       classes / 4 > kUnitsLo && classes / 4 <= kUnitsHi;
  const int chunks = (int)eval_chunks(rows, n_slices, regular ? kRegularRows : kRowsPerBlock);
  const dim3 grid(chunks, n_slices);
  if (regular)
    SYNK_LAUNCH_TIMED((eval_stage1_regular_kernel<kRegularG, kRegularUPL>), grid, dim3(kEBlock), 0, s, logits,
                      labels, rows, (int)classes, n_slices, chunks, w, argmax, class_counts);
  else if (classes % 4 == 0 && aligned_to(logits, 16) && classes <= 1024)
    SYNK_LAUNCH_TIMED((eval_stage1_kernel<16, 16>), grid, dim3(kEBlock), 0, s, logits, labels, rows,
                       (int)classes, n_slices, chunks, w, argmax, class_counts);
  else if (classes % 4 == 0 && aligned_to(logits, 16))
    SYNK_LAUNCH_TIMED((eval_stage1_kernel<64, 16>), grid, dim3(kEBlock), 0, s, logits, labels, rows,
                       (int)classes, n_slices, chunks, w, argmax, class_counts);
  else
    SYNK_LAUNCH_TIMED(eval_stage1_generic_kernel, grid, dim3(kEBlock), 0, s, logits, labels, rows,
                       (int)classes, n_slices, chunks, w, argmax, class_counts);
  SYNK_LAUNCH_CHECK();
  int64_t b2 = (rows + kE2RowsPerBlock - 1) / kE2RowsPerBlock;
  if (b2 > kNumCU) b2 = kNumCU;
  hipLaunchKernelGGL(eval_stage2_kernel, dim3((unsigned)b2 + 1), dim3(kE2Block), 0, s, w, rows, n_slices, chunks,
                     (int)classes, argmax, ce_sum, class_counts, max_logit, min_logit, n_correct);
  SYNK_LAUNCH_CHECK();
  return SYNK_OK;
}

extern "C" int synk_sliced_eval(const float* logits, const int32_t* labels, int64_t rows,
                                int64_t classes, int n_slices, float* ce_sum,
                                int32_t* class_counts, float* max_logit, float* min_logit,
                                int32_t* n_correct, int32_t* argmax, void* ws, size_t ws_bytes,
                                void* stream) {
  if (int rc = eval_args_check(logits, labels, rows, classes, n_slices, ce_sum, class_counts, max_logit,
                               min_logit, n_correct, argmax))
    return rc;
  EvalWs w;
  const size_t need = eval_ws_layout(rows, classes, n_slices, ws, &w);
  if (!ws || !aligned_to(ws, 256) || ws_bytes < need) return SYNK_ERR_WORKSPACE;
  return eval_launch(logits, labels, rows, classes, n_slices, ce_sum, class_counts, max_logit, min_logit,
                     n_correct, argmax, w, reinterpret_cast<hipStream_t>(stream));
}

// ------------------------------------------------ the entry point that allocates nothing
// Partial results live in a fixed array in the library's own device image instead
// of a caller's workspace.  Every GPU the library runs on holds its own copy at
// its own address; in host code the array's name is only a handle for
// hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[SYNK_SLICED_EVAL_STATIC_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];   // per device: where that device's copy of `scratch` lives

// The current device's copy of `scratch` (resolved once per device, with that device current).
int scratch_for_current_device(void** out) {
  int dev = -1;
  SYNK_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SYNK_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    SYNK_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return SYNK_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SYNK_OK;
}
}  // namespace

extern "C" int synk_static_scratch_init(void) {
  void* ptr;
  return scratch_for_current_device(&ptr);
}

extern "C" int synk_sliced_eval_static(const float* logits, const int32_t* labels, int64_t rows,
                                       int64_t classes, int n_slices, float* ce_sum,
                                       int32_t* class_counts, float* max_logit, float* min_logit,
                                       int32_t* n_correct, int32_t* argmax, void* stream) {
  if (int rc = eval_args_check(logits, labels, rows, classes, n_slices, ce_sum, class_counts, max_logit,
                               min_logit, n_correct, argmax))
    return rc;
  if (eval_ws_layout(rows, classes, n_slices, nullptr, nullptr) > (size_t)SYNK_SLICED_EVAL_STATIC_BYTES)
    return SYNK_ERR_WORKSPACE;   // more (slice, chunk) partial results than the fixed array holds
  void* base = nullptr;
  if (int rc = scratch_for_current_device(&base)) return rc;
  EvalWs w;
  eval_ws_layout(rows, classes, n_slices, base, &w);
  // Nothing in the array needs clearing: stage 1 writes every (slice, chunk) entry that stage 2
  // reads, whatever an earlier call left there.
  return eval_launch(logits, labels, rows, classes, n_slices, ce_sum, class_counts, max_logit, min_logit,
                     n_correct, argmax, w, reinterpret_cast<hipStream_t>(stream));
}
