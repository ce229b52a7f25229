// Depth-wise windows: every channel convolved with its own single-channel filter.
//
// In the paper's operators (Table 1, Table 2) this is the concat, along the channel dimension, of
// the 2D-convolution program of Fig. 2a applied to channel c of the activations and filter c of
// the weights (slice ... 1 c c+1 / slice ... 0 c c+1): C independent one-channel convolutions.
// No contraction over channels is left, so there is nothing for the matrix units: 2*Kh*Kw
// operations per 2-byte input element.  The kernel is bound by memory traffic and is built like the
// pooling kernel: every input byte leaves HBM once, however much the windows overlap.
//
// A task is a contiguous run of the input: G whole planes (small images) or a band of rows of one
// plane (large images).  Its workgroup copies the run into LDS with aligned 16-byte reads -- a plain
// linear copy that does not care how long a row is or where a plane starts -- and every thread
// then produces strips of 8 neighbouring outputs of one output row from LDS.  Cells outside the
// image are never read as data: rows outside are skipped, columns outside are replaced by zero in
// the (few) strips that touch the left or right border.  The 16-byte loads of the next task are in
// flight while the current one is computed.
#include "common.h"

#include <string.h>

namespace gs {

namespace {

constexpr int kVX = 8;             // outputs per strip
constexpr int kMaxVec = 8;         // 16-byte loads per thread and task
constexpr int kGuard = 64;         // bytes of LDS in front of the copy (reads of columns < 0 land here)

struct DwArgs {
  const void* in;
  const void* w;
  void* out;
  int out_dtype, relu;
  int C, H, W, Ho, Wo, Kh, Kw, Sh, Sw, Ph, Pw;
  int G;            // planes per task (1 when a plane is cut into bands)
  int HB, bands;    // output rows per band, bands per plane
  int XS;           // strips per output row
  int KKP;          // filter taps padded to a multiple of 4
  int64_t planes, groups, tasks, total;   // N*C, ceil(planes / G), groups * bands, elements of the input
  int vec_in, vec_out, pair_out;
  uint32_t lds_w;   // byte offset of the filters in LDS
  FastDiv dXS, dHo, dKK;
  int step_r, step_xs;   // 256 items further: step_r rows of strips and step_xs strips
};

template <typename T> struct DwElem;
template <> struct DwElem<uint16_t> {
  using acc = float;
  __device__ static inline float cvt(uint16_t v) { return bf16_bits_to_float(v); }
};
template <> struct DwElem<int8_t> {
  using acc = int32_t;
  __device__ static inline int32_t cvt(int8_t v) { return v; }
};

struct DwTask {
  int64_t plane0;
  int gcount, ho0, nho, R;   // planes, first output row, output rows, gcount * nho
  int64_t ebase;     // first element (16-byte aligned) of the copy
  int nvec;          // 16-byte vectors in the copy
  int shift;         // LDS element index of (g, ih, iw) is (g*H + ih)*W + iw - shift
};

__device__ __forceinline__ DwTask dw_task(const DwArgs& a, int64_t task, int epv) {
  DwTask t;
  const int64_t grp = task / a.bands;
  const int band = int(task - grp * a.bands);
  t.plane0 = grp * a.G;
  const int64_t left = a.planes - t.plane0;
  t.gcount = left < a.G ? int(left) : a.G;
  t.ho0 = band * a.HB;
  t.nho = a.Ho - t.ho0 < a.HB ? a.Ho - t.ho0 : a.HB;
  t.R = t.gcount * t.nho;
  int ih0 = t.ho0 * a.Sh - a.Ph;
  ih0 = ih0 < 0 ? 0 : ih0;
  int ih1 = (t.ho0 + t.nho - 1) * a.Sh - a.Ph + a.Kh;
  ih1 = ih1 > a.H ? a.H : ih1;
  ih1 = ih1 < ih0 ? ih0 : ih1;
  const int64_t e0 = (t.plane0 * a.H + ih0) * a.W;
  const int64_t e1 = ((t.plane0 + t.gcount - 1) * a.H + ih1) * a.W;
  t.ebase = e0 / epv * epv;
  t.nvec = int((e1 + epv - 1) / epv - e0 / epv);
  t.shift = int(t.ebase - t.plane0 * a.H * a.W);
  return t;
}

// KH, KW, SW > 0: window and horizontal stride fixed at compile time; 0: run-time loops.
template <typename T, int KH, int KW, int SW>
__global__ void __launch_bounds__(256)
depthwise_kernel(DwArgs a) {
  using A = typename DwElem<T>::acc;
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  constexpr bool FIXED = KH > 0;
  typedef T vec_t __attribute__((ext_vector_type(EPV)));
  extern __shared__ __attribute__((aligned(16))) uint8_t dw_lds[];
  T* const stage = reinterpret_cast<T*>(dw_lds + kGuard);
  A* const wl = reinterpret_cast<A*>(dw_lds + a.lds_w);
  const T* const in = static_cast<const T*>(a.in);
  const int tid = threadIdx.x;
  const int kh = FIXED ? KH : a.Kh, kw = FIXED ? KW : a.Kw, sw = FIXED ? SW : a.Sw;
  const int kk = kh * kw;

  vec_t val[kMaxVec];
  auto issue_loads = [&](const DwTask& t) {
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
      const int v = u * 256 + tid;
      const int64_t e = t.ebase + int64_t(v) * EPV;
#pragma unroll
      for (int i = 0; i < EPV; ++i) val[u][i] = 0;
      if (v < t.nvec) {
        if (a.vec_in && e + EPV <= a.total) {
          val[u] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(in + e));   // read once
        } else {
#pragma unroll
          for (int i = 0; i < EPV; ++i)
            if (e + i < a.total) val[u][i] = in[e + i];
        }
      }
    }
  };

  int64_t task = blockIdx.x;
  if (task >= a.tasks) return;
  DwTask cur = dw_task(a, task, EPV);
  issue_loads(cur);
  for (; task < a.tasks; task += gridDim.x) {
    __syncthreads();                                   // the previous task has been computed
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
      const int v = u * 256 + tid;
      if (v < cur.nvec) *reinterpret_cast<vec_t*>(stage + v * EPV) = val[u];
    }
    for (int id = tid; id < cur.gcount * kk; id += 256) {   // the filters of this task's planes
      uint32_t g, i;
      a.dKK.divmod(uint32_t(id), &g, &i);
      const int c = int((cur.plane0 + g) % a.C);
      wl[int(g) * a.KKP + int(i)] = DwElem<T>::cvt(static_cast<const T*>(a.w)[int64_t(c) * kk + int(i)]);
    }
    __syncthreads();
    const DwTask t = cur;
    if (task + gridDim.x < a.tasks) {
      cur = dw_task(a, task + gridDim.x, EPV);
      issue_loads(cur);
    }

    // Strips are numbered along the rows: neighbouring lanes read neighbouring 16 bytes of LDS
    // and write neighbouring 16 bytes of the result.
    const int items = a.XS * t.R;
    // (row of strips, strip) of this thread's item: divided once, then stepped by 256 items.
    uint32_t r, xs;
    a.dXS.divmod(uint32_t(tid), &r, &xs);
    const int64_t obase = t.plane0 * a.Ho * a.Wo;       // results of the task's first plane
    for (int id = tid; id < items; id += 256, r += a.step_r, xs += a.step_xs) {
      if (int(xs) >= a.XS) {
        xs -= a.XS;
        ++r;
      }
      uint32_t g = 0, yl = r;
      if (a.G > 1) a.dHo.divmod(r, &g, &yl);           // G > 1: whole planes, nho == Ho
      const int y = t.ho0 + int(yl);
      const int x0 = int(xs) * kVX;
      const int iw0 = x0 * sw - a.Pw;                   // column of the first element of the span
      const A* wg = wl + __mul24(int(g), a.KKP);
      A acc[kVX];
#pragma unroll
      for (int v = 0; v < kVX; ++v) acc[v] = 0;
      if constexpr (FIXED) {
        constexpr int SPAN = (kVX - 1) * SW + KW;
        constexpr int KKP = (KH * KW + 3) / 4 * 4;
        A wr[KKP];
#pragma unroll
        for (int q = 0; q < KKP / 4; ++q) {
          typedef A a4 __attribute__((ext_vector_type(4)));
          const a4 w4 = *reinterpret_cast<const a4*>(wg + 4 * q);
#pragma unroll
          for (int i = 0; i < 4; ++i) wr[4 * q + i] = w4[i];
        }
        // All LDS reads of the strip first (rows outside the image read nothing and count as
        // zeros), then straight-line arithmetic: the reads of the KH rows overlap.
        const int ih_first = __mul24(y, a.Sh) - a.Ph;
        // 24-bit multiplies: LDS indices are far below 2^23
        const T* row0 = stage + (__mul24(__mul24(int(g), a.H) + ih_first, a.W) + iw0 - t.shift);
        T raw[KH][SPAN];
#pragma unroll
        for (int ky = 0; ky < KH; ++ky) {
#pragma unroll
          for (int j = 0; j < SPAN; ++j) raw[ky][j] = 0;
          if (ih_first + ky >= 0 && ih_first + ky < a.H) {
            const T* row = row0 + ky * a.W;
#pragma unroll
            for (int j = 0; j < SPAN; ++j) raw[ky][j] = row[j];
          }
        }
        // Element j of a span sits in column iw0 + j: columns left of the image (only the first
        // KW - 1 elements can be) and right of it hold a neighbouring row's data and count as zero.
        const int lo_bad = -iw0, hi_ok = a.W - iw0;
#pragma unroll
        for (int ky = 0; ky < KH; ++ky) {
          A e[SPAN];
#pragma unroll
          for (int j = 0; j < SPAN; ++j) {
            e[j] = DwElem<T>::cvt(raw[ky][j]);
            if (j < KW - 1) e[j] = j >= lo_bad ? e[j] : A(0);
            e[j] = j < hi_ok ? e[j] : A(0);
          }
#pragma unroll
          for (int v = 0; v < kVX; ++v)
#pragma unroll
            for (int kx = 0; kx < KW; ++kx) acc[v] += e[v * SW + kx] * wr[ky * KW + kx];
        }
      } else {
        for (int ky = 0; ky < kh; ++ky) {
          const int ih = y * a.Sh - a.Ph + ky;
          if (ih < 0 || ih >= a.H) continue;
          const T* row = stage + ((int(g) * a.H + ih) * a.W - t.shift);
          for (int kx = 0; kx < kw; ++kx) {
            const A wv = wg[ky * kw + kx];
#pragma unroll
            for (int v = 0; v < kVX; ++v) {
              const int iw = iw0 + v * sw + kx;
              if (iw >= 0 && iw < a.W && x0 + v < a.Wo) acc[v] += DwElem<T>::cvt(row[iw]) * wv;
            }
          }
        }
      }
      if (a.relu) {
#pragma unroll
        for (int v = 0; v < kVX; ++v) acc[v] = acc[v] > A(0) ? acc[v] : A(0);
      }
      // within a task the results are fewer than 2^23 rows of fewer than 2^23 values
      const int64_t o = obase + (int64_t(__mul24(__mul24(int(g), a.Ho) + y, a.Wo)) + x0);
      if (a.vec_out && x0 + kVX <= a.Wo) {
        if (a.out_dtype == GS_BF16) {
          if constexpr (__is_same(A, float)) {
            typedef uint32_t u4 __attribute__((ext_vector_type(4)));
            u4 p;
#pragma unroll
            for (int q = 0; q < 4; ++q) p[q] = pack_bf16x2(acc[2 * q], acc[2 * q + 1]);
            __builtin_nontemporal_store(p, reinterpret_cast<u4*>(static_cast<uint16_t*>(a.out) + o));
          }
        } else {                                        // 32-bit results: two 16-byte stores
          typedef A a4 __attribute__((ext_vector_type(4)));
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const a4 p = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
            __builtin_nontemporal_store(p, reinterpret_cast<a4*>(static_cast<A*>(a.out) + o) + q);
          }
        }
      } else if (__is_same(A, float) && a.out_dtype == GS_BF16 && a.pair_out) {
        // rows of an even number of results: pairs never straddle the end of a row
        if constexpr (__is_same(A, float)) {
#pragma unroll
          for (int q = 0; q < kVX / 2; ++q)
            if (x0 + 2 * q < a.Wo)
              reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(a.out) + o)[q] = pack_bf16x2(acc[2 * q], acc[2 * q + 1]);
        }
      } else {
#pragma unroll
        for (int v = 0; v < kVX; ++v) {
          if (x0 + v < a.Wo) {
            if constexpr (__is_same(A, float)) {
              if (a.out_dtype == GS_BF16) static_cast<uint16_t*>(a.out)[o + v] = float_to_bf16_bits(acc[v]);
              else static_cast<float*>(a.out)[o + v] = acc[v];
            } else {
              static_cast<int32_t*>(a.out)[o + v] = acc[v];
            }
          }
        }
      }
    }
  }
}

int dw_num_cus() {
  static int n = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    return cus;
  }();
  return n;
}

template <typename T>
hipError_t launch_depthwise_t(const DepthwiseArgs& d, hipStream_t s) {
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  using A = typename DwElem<T>::acc;
  DwArgs a;
  memset(&a, 0, sizeof(a));
  a.in = d.in; a.w = d.w; a.out = d.out; a.out_dtype = d.out_dtype; a.relu = d.relu;
  a.C = d.C; a.H = d.H; a.W = d.W; a.Ho = d.Ho; a.Wo = d.Wo; a.Kh = d.Kh; a.Kw = d.Kw;
  a.Sh = d.Sh; a.Sw = d.Sw; a.Ph = d.Ph; a.Pw = d.Pw;
  a.planes = int64_t(d.N) * d.C;
  a.total = a.planes * d.H * d.W;
  if (a.planes == 0 || d.Ho <= 0 || d.Wo <= 0) return hipSuccess;
  if (a.total >= (int64_t(1) << 40)) return hipErrorInvalidValue;
  // positions inside a plane (of the input and of the result) are 32-bit in the kernel
  if ((int64_t(d.H) + 64) * (int64_t(d.W) + 64) >= (int64_t(1) << 31)) return hipErrorInvalidValue;
  // The copy of a task: at most kMaxVec * 256 vectors, two of them spent on the ragged ends.
  const int64_t cap = int64_t(kMaxVec * 256 - 2) * EPV;           // elements
  const int64_t plane = int64_t(d.H) * d.W;
  if (plane <= cap) {
    // Planes per task: the strips of a task are worked off 256 at a time, and the chip holds
    // `slots` tasks at once; take the G with the fewest (rounds + one round of fixed cost) x passes.
    int gmax = int(cap / plane);
    gmax = gmax > 64 ? 64 : gmax;
    const int64_t slots = int64_t(dw_num_cus()) * 4;
    const int64_t strips = ceil_div(d.Wo, kVX) * d.Ho;
    int64_t best = -1;
    a.G = 1;
    for (int g = 1; g <= gmax; ++g) {
      const int64_t cost = ceil_div(ceil_div(a.planes, g), slots) * (ceil_div(strips * g, 256) + 1);
      if (best < 0 || cost <= best) {
        best = cost;
        a.G = g;
      }
    }
    a.HB = d.Ho;
    a.bands = 1;
  } else {
    a.G = 1;
    const int64_t rows = cap / d.W;                                 // input rows that fit
    if (rows < d.Kh) return hipErrorInvalidValue;
    int64_t hb = (rows - d.Kh) / d.Sh + 1;
    hb = hb > d.Ho ? d.Ho : hb;
    a.bands = int(ceil_div(d.Ho, hb));
    a.HB = int(ceil_div(d.Ho, a.bands));
  }
  a.groups = ceil_div(a.planes, a.G);
  a.tasks = a.groups * a.bands;
  a.XS = int(ceil_div(d.Wo, kVX));
  a.KKP = int(round_up(int64_t(d.Kh) * d.Kw, 4));
  a.dXS = FastDiv::make(uint32_t(a.XS));
  a.step_r = 256 / a.XS;
  a.step_xs = 256 % a.XS;
  a.dHo = FastDiv::make(uint32_t(d.Ho));
  a.dKK = FastDiv::make(uint32_t(d.Kh * d.Kw));
  a.vec_in = reinterpret_cast<uintptr_t>(d.in) % 16 == 0;
  a.vec_out = d.Wo % kVX == 0 && reinterpret_cast<uintptr_t>(d.out) % 16 == 0;
  a.pair_out = d.Wo % 2 == 0 && reinterpret_cast<uintptr_t>(d.out) % 4 == 0;
  // LDS: guard, the copy, room for the last strip's reads past the end of a row, the filters.
  const int64_t span_max = int64_t(kVX) * d.Sw + d.Kw;
  const int64_t copy_bytes = int64_t(kMaxVec) * 256 * 16;
  a.lds_w = uint32_t(round_up(kGuard + copy_bytes + span_max * ESZ, 16));
  const size_t lds = a.lds_w + size_t(a.G) * a.KKP * sizeof(A);
  if (d.Pw * ESZ > kGuard || lds > 64 * 1024) return hipErrorInvalidValue;
  int per_cu = int((160 * 1024) / (lds + 512));
  per_cu = per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu;
  int64_t grid = int64_t(dw_num_cus()) * per_cu;
  if (grid > a.tasks) grid = a.tasks;
  grid = ceil_div(a.tasks, ceil_div(a.tasks, grid));     // the same number of tasks for everyone
  const dim3 g{unsigned(grid)}, b{256};
  if (d.Kh == 3 && d.Kw == 3 && d.Sw == 1)
    hipLaunchKernelGGL((depthwise_kernel<T, 3, 3, 1>), g, b, lds, s, a);
  else if (d.Kh == 3 && d.Kw == 3 && d.Sw == 2)
    hipLaunchKernelGGL((depthwise_kernel<T, 3, 3, 2>), g, b, lds, s, a);
  else if (d.Kh == 5 && d.Kw == 5 && d.Sw == 1)
    hipLaunchKernelGGL((depthwise_kernel<T, 5, 5, 1>), g, b, lds, s, a);
  else
    hipLaunchKernelGGL((depthwise_kernel<T, 0, 0, 0>), g, b, lds, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_depthwise(const DepthwiseArgs& d, hipStream_t s) {
  for (int v : {d.H, d.W, d.Ho, d.Wo})
    if (v > (1 << 20)) return hipErrorInvalidValue;
  for (int v : {d.Kh, d.Kw, d.Sh, d.Sw, d.Ph, d.Pw})
    if (v < 0 || v > 64) return hipErrorInvalidValue;
  if (d.Kh < 1 || d.Kw < 1 || d.Sh < 1 || d.Sw < 1) return hipErrorInvalidValue;
  // Padding is smaller than the window: no window lies wholly outside the image, and the reads of
  // the last strip of a row stay within the LDS reserved behind the copy.
  if (d.Ph >= d.Kh || d.Pw >= d.Kw) return hipErrorInvalidValue;
  return d.in_dtype == GS_I8 ? launch_depthwise_t<int8_t>(d, s) : launch_depthwise_t<uint16_t>(d, s);
}

}  // namespace gs
