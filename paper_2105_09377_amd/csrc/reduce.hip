// `compute reduceSum | reduceMax` (Table 2), the fused `compute reduce (windows ...)` used by
// pooling (Fig. 2c), and `compute reduce (pair a b)` (the element-wise sum idiom of Sec. 5.4).
//
// Row reductions pick a lane-group width G (power of two, 1..64) no smaller than the row length
// when it is short, so that the lanes of a wave read consecutive addresses and several rows are
// reduced per wave with cross-lane shuffles; long rows use one wave (or one workgroup) per row.
// Rows that are whole 16-byte vectors take a streaming vector kernel; 2D pooling is staged
// through LDS by persistent workgroups (pool2d_* below).
#include "common.h"

#include <float.h>
#include <limits.h>

namespace gs {

template <typename T> struct Elem;
template <> struct Elem<int8_t> {
  using acc = int32_t;
  __device__ static acc load(const int8_t* p, int64_t i) { return p[i]; }
  __device__ static acc cvt(int8_t v) { return v; }
};
template <> struct Elem<int32_t> {
  using acc = int32_t;
  __device__ static acc load(const int32_t* p, int64_t i) { return p[i]; }
  __device__ static acc cvt(int32_t v) { return v; }
};
template <> struct Elem<float> {
  using acc = float;
  __device__ static acc load(const float* p, int64_t i) { return p[i]; }
  __device__ static acc cvt(float v) { return v; }
};
template <> struct Elem<uint16_t> {  // bfloat16 bits
  using acc = float;
  __device__ static acc load(const uint16_t* p, int64_t i) { return bf16_bits_to_float(p[i]); }
  __device__ static acc cvt(uint16_t v) { return bf16_bits_to_float(v); }
};

template <typename A> __device__ inline A ident(int op);
template <> __device__ inline int32_t ident<int32_t>(int op) { return op == GS_MAX ? INT_MIN : 0; }
template <> __device__ inline float ident<float>(int op) { return op == GS_MAX ? -INFINITY : 0.0f; }

template <typename A> __device__ inline A combine(A a, A b, int op) {
  if (op == GS_MAX) return a > b ? a : b;
  return a + b;
}

template <typename A> __device__ inline void store_out(void* out, int out_dtype, int64_t i, A v) {
  if constexpr (__is_same(A, int32_t)) {
    if (out_dtype == GS_I8) static_cast<int8_t*>(out)[i] = int8_t(v);
    else static_cast<int32_t*>(out)[i] = v;
  } else {
    if (out_dtype == GS_BF16) static_cast<uint16_t*>(out)[i] = float_to_bf16_bits(v);
    else static_cast<float*>(out)[i] = v;
  }
}

template <typename A> __device__ inline A finish(A v, float scale) {
  if constexpr (__is_same(A, float)) return scale == 1.0f ? v : v * scale;
  else return v;
}

// G lanes per row, G a power of two <= 64; rows_per_block = 256 / G.
template <typename T, int G>
__global__ void __launch_bounds__(256)
reduce_rows_group_kernel(const T* __restrict__ in, void* __restrict__ out, int out_dtype, int op,
                         int64_t rows, int64_t cols, float scale) {
  using A = typename Elem<T>::acc;
  const int lane_in_group = threadIdx.x % G;
  const int64_t row = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) / G;
  A acc = ident<A>(op);
  if (row < rows) {
    for (int64_t c = lane_in_group; c < cols; c += G)
      acc = combine(acc, Elem<T>::load(in, row * cols + c), op);
  }
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) acc = combine(acc, __shfl_xor(acc, off, G), op);
  if (row < rows && lane_in_group == 0) store_out<A>(out, out_dtype, row, finish(acc, scale));
}

// Rows that are whole 16-byte vectors: G lanes per row load 16 bytes each per step (streaming
// loads: every byte is read once), fold the vector's elements, then combine across the group.
template <typename T, int G>
__global__ void __launch_bounds__(256)
reduce_rows_vec_kernel(const T* __restrict__ in, void* __restrict__ out, int out_dtype, int op,
                       int64_t rows, int64_t cols, float scale) {
  using A = typename Elem<T>::acc;
  constexpr int EPV = 16 / int(sizeof(T));
  typedef T vec_t __attribute__((ext_vector_type(EPV)));
  const int lane_in_group = threadIdx.x % G;
  const int64_t nv = cols / EPV;
  for (int64_t row = (int64_t(blockIdx.x) * blockDim.x + threadIdx.x) / G; row < rows;
       row += int64_t(gridDim.x) * blockDim.x / G) {
    const vec_t* src = reinterpret_cast<const vec_t*>(in + row * cols);
    A acc = ident<A>(op);
    for (int64_t v = lane_in_group; v < nv; v += G) {
      const vec_t x = __builtin_nontemporal_load(src + v);
#pragma unroll
      for (int i = 0; i < EPV; ++i) acc = combine(acc, Elem<T>::cvt(x[i]), op);
    }
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) acc = combine(acc, __shfl_xor(acc, off, G), op);
    if (lane_in_group == 0) store_out<A>(out, out_dtype, row, finish(acc, scale));
  }
}

// Short rows of any length and alignment (a 7x7 plane averaged to one value): the rows are
// contiguous in memory, so a workgroup copies its 128 rows to LDS with aligned 16-byte loads,
// whatever the row length, and two threads then fold each row from LDS.
constexpr int kShortRows = 128;   // rows per workgroup: 128 * cols * sizeof(T) is a multiple of 16
template <typename T>
__global__ void __launch_bounds__(256)
reduce_rows_short_kernel(const T* __restrict__ in, void* __restrict__ out, int out_dtype, int op,
                         int64_t rows, int cols, float scale) {
  using A = typename Elem<T>::acc;
  constexpr int EPV = 16 / int(sizeof(T));
  extern __shared__ __attribute__((aligned(16))) uint8_t short_lds[];
  T* buf = reinterpret_cast<T*>(short_lds);
  const int64_t row0 = int64_t(blockIdx.x) * kShortRows;
  const int nrows = int(rows - row0 < kShortRows ? rows - row0 : kShortRows);
  const int nelem = nrows * cols;
  const T* src = in + row0 * cols;                 // 16-byte aligned: row0 is a multiple of 128
  const int nvec = nelem / EPV;                    // whole vectors inside this workgroup's rows
  for (int v = threadIdx.x; v < nvec; v += 256)
    reinterpret_cast<i32x4*>(buf)[v] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src) + v);
  for (int e = nvec * EPV + threadIdx.x; e < nelem; e += 256) buf[e] = src[e];
  __syncthreads();
  const int r = threadIdx.x >> 1, half = threadIdx.x & 1;
  A acc = ident<A>(op);
  if (r < nrows)
    for (int c = half; c < cols; c += 2) acc = combine(acc, Elem<T>::load(buf, int64_t(r) * cols + c), op);
  acc = combine(acc, __shfl_xor(acc, 1, 2), op);
  if (r < nrows && half == 0) store_out<A>(out, out_dtype, row0 + r, finish(acc, scale));
}

// One workgroup of 256 threads per row, for long rows.
template <typename T>
__global__ void __launch_bounds__(256)
reduce_rows_block_kernel(const T* __restrict__ in, void* __restrict__ out, int out_dtype, int op,
                         int64_t rows, int64_t cols, float scale) {
  using A = typename Elem<T>::acc;
  __shared__ A part[4];
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
    A acc = ident<A>(op);
    for (int64_t c = threadIdx.x; c < cols; c += 256)
      acc = combine(acc, Elem<T>::load(in, row * cols + c), op);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc = combine(acc, __shfl_xor(acc, off, 64), op);
    if (threadIdx.x % 64 == 0) part[threadIdx.x / 64] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      A r = combine(combine(part[0], part[1], op), combine(part[2], part[3], op), op);
      store_out<A>(out, out_dtype, row, finish(r, scale));
    }
    __syncthreads();
  }
}

static int reduce_num_cus() {
  static int cus = 0;
  if (!cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

template <typename T>
static hipError_t launch_reduce_t(const ReduceArgs& a, hipStream_t s) {
  if (a.rows == 0) return hipSuccess;
  const T* in = static_cast<const T*>(a.in);
#define GS_LAUNCH_GROUP(G)                                                                       \
  hipLaunchKernelGGL((reduce_rows_group_kernel<T, G>), dim3(unsigned(ceil_div(a.rows * G, 256))), \
                     dim3(256), 0, s, in, a.out, a.out_dtype, a.op, a.rows, a.cols, a.scale)
  constexpr int EPV = 16 / int(sizeof(T));
  if (a.cols % EPV == 0 && a.cols >= 8 * EPV && reinterpret_cast<uintptr_t>(a.in) % 16 == 0 &&
      (a.cols <= 2048 || a.rows >= 1024) && a.cols <= (int64_t(1) << 24)) {
    const int64_t nv = a.cols / EPV;
    const int64_t cap = int64_t(reduce_num_cus()) * 32;     // workgroups: enough to fill the chip, rows looped
#define GS_LAUNCH_VEC(G)                                                                           \
  {                                                                                                \
    const int64_t want = ceil_div(a.rows * G, 256);                                                \
    hipLaunchKernelGGL((reduce_rows_vec_kernel<T, G>), dim3(unsigned(want < cap ? want : cap)),    \
                       dim3(256), 0, s, in, a.out, a.out_dtype, a.op, a.rows, a.cols, a.scale);    \
  }
    if (nv <= 8) GS_LAUNCH_VEC(8)
    else if (nv <= 16) GS_LAUNCH_VEC(16)
    else if (nv <= 32) GS_LAUNCH_VEC(32)
    else GS_LAUNCH_VEC(64)
#undef GS_LAUNCH_VEC
    return hipGetLastError();
  }
  if (a.cols > 8 && a.cols < 8 * EPV && a.rows >= 4 * kShortRows && reinterpret_cast<uintptr_t>(a.in) % 16 == 0) {
    const size_t lds = size_t(round_up(int64_t(kShortRows) * a.cols * int64_t(sizeof(T)), 16));
    hipLaunchKernelGGL((reduce_rows_short_kernel<T>), dim3(unsigned(ceil_div(a.rows, kShortRows))), dim3(256),
                       lds, s, in, a.out, a.out_dtype, a.op, a.rows, int(a.cols), a.scale);
    return hipGetLastError();
  }
  if (a.cols <= 1) GS_LAUNCH_GROUP(1);
  else if (a.cols <= 2) GS_LAUNCH_GROUP(2);
  else if (a.cols <= 4) GS_LAUNCH_GROUP(4);
  else if (a.cols <= 8) GS_LAUNCH_GROUP(8);
  else if (a.cols <= 16) GS_LAUNCH_GROUP(16);
  else if (a.cols <= 32) GS_LAUNCH_GROUP(32);
  else if (a.cols <= 2048) GS_LAUNCH_GROUP(64);
  else {
    const int64_t blocks = a.rows < 65536 ? a.rows : 65536;
    hipLaunchKernelGGL((reduce_rows_block_kernel<T>), dim3(unsigned(blocks)), dim3(256), 0, s, in,
                       a.out, a.out_dtype, a.op, a.rows, a.cols, a.scale);
  }
#undef GS_LAUNCH_GROUP
  return hipGetLastError();
}

hipError_t launch_reduce(const ReduceArgs& a, hipStream_t s) {
  switch (a.in_dtype) {
    case GS_I8: return launch_reduce_t<int8_t>(a, s);
    case GS_I32: return launch_reduce_t<int32_t>(a, s);
    case GS_BF16: return launch_reduce_t<uint16_t>(a, s);
    case GS_F32: return launch_reduce_t<float>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// ---------------------------------------------------------------------------------------------
// compute reduce (windows in w s): one output per thread, the window read straight from `in`.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
windows_reduce_kernel(const T* __restrict__ in, void* __restrict__ out, WindowsReduceArgs a,
                      int64_t total, int64_t out_pos) {
  using A = typename Elem<T>::acc;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    int64_t p = f % out_pos;
    const int64_t o = f / out_pos;
    int64_t base[3] = {0, 0, 0};
    for (int d = a.n_compute - 1; d >= 0; --d) {
      base[d] = (p % a.out_dim[d]) * a.stride[d] - a.pad_lo[d];
      p /= a.out_dim[d];
    }
    int64_t plane = 1;
    for (int d = 0; d < a.n_compute; ++d) plane *= a.in_dim[d];
    const T* src = in + o * plane;
    A acc = ident<A>(a.op);   // padded cells read the identity: lowest for max, zero for sum
    const int64_t w0 = a.n_compute > 2 ? a.win[a.n_compute - 3] : 1;
    const int64_t w1 = a.n_compute > 1 ? a.win[a.n_compute - 2] : 1;
    const int64_t w2 = a.win[a.n_compute - 1];
    for (int64_t q0 = 0; q0 < w0; ++q0)
      for (int64_t q1 = 0; q1 < w1; ++q1)
        for (int64_t q2 = 0; q2 < w2; ++q2) {
          const int64_t q[3] = {q0, q1, q2};
          int64_t off = 0;
          bool inside = true;
          for (int d = 0; d < a.n_compute; ++d) {
            const int64_t pos = base[d] + q[3 - a.n_compute + d];
            inside = inside && pos >= 0 && pos < a.in_dim[d];
            off = off * a.in_dim[d] + pos;
          }
          if (inside) acc = combine(acc, Elem<T>::load(src, off), a.op);
        }
    store_out<A>(out, a.out_dtype, f, finish(acc, a.scale));
  }
}

template <typename T>
static hipError_t launch_windows_reduce_t(const WindowsReduceArgs& a, hipStream_t s) {
  int64_t out_pos = 1;
  for (int d = 0; d < a.n_compute; ++d) out_pos *= a.out_dim[d];
  const int64_t total = a.outer * out_pos;
  if (total == 0) return hipSuccess;
  const int64_t b = ceil_div(total, 256);
  hipLaunchKernelGGL((windows_reduce_kernel<T>), dim3(unsigned(b < (1 << 20) ? b : (1 << 20))),
                     dim3(256), 0, s, static_cast<const T*>(a.in), a.out, a, total, out_pos);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// compute reduce (windows in w s) over the last two dims (pooling, Fig. 2c), staged through LDS.
// A workgroup owns a band of output rows of one plane: it copies the input rows the band needs
// into LDS with coalesced 16-byte reads (padding cells hold the operator's identity), then every
// thread folds whole windows out of LDS, so each input byte leaves HBM once however much the
// windows overlap.  KH / KW fix the window at compile time (0 = run-time loops).
// ---------------------------------------------------------------------------------------------
struct Pool2dArgs {
  const void* in;
  void* out;
  int out_dtype, op;
  int H, W, Ho, Wo, Kh, Kw, Sh, Sw, Ph, Pw;
  int HB;          // output rows per band
  int bands;       // bands per plane
  int rows;        // LDS rows per band: (HB - 1) * Sh + Kh
  int pitch, XO;   // LDS row pitch and first data column, in elements
  int64_t tasks;   // planes * bands
  float scale;
  int G;           // groups of VO outputs per output row (vector kernel)
  int rows_alloc;  // LDS rows allocated
  FastDiv dvpr, dW, dhalo, dWo, dG;
};

constexpr int kPoolLdsBudget = 32 * 1024;

template <typename T> __device__ inline T ident_elem(int op);
template <> __device__ inline int8_t ident_elem<int8_t>(int op) { return op == GS_MAX ? int8_t(-128) : int8_t(0); }
template <> __device__ inline int32_t ident_elem<int32_t>(int op) { return op == GS_MAX ? INT_MIN : 0; }
template <> __device__ inline float ident_elem<float>(int op) { return op == GS_MAX ? -INFINITY : 0.0f; }
template <> __device__ inline uint16_t ident_elem<uint16_t>(int op) { return op == GS_MAX ? uint16_t(0xff80) : uint16_t(0); }

// Copies the input rows of one band into LDS; cells outside the image hold the identity.
template <typename T>
__device__ __forceinline__ void pool2d_stage(const Pool2dArgs& a, T* stage, const T* src, int ih0,
                                             int nrows, int tid) {
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  typedef T vec_t __attribute__((ext_vector_type(EPV)));
  const T idv = ident_elem<T>(a.op);
  const bool vec_ok = (a.W * ESZ) % 16 == 0 && reinterpret_cast<uintptr_t>(a.in) % 16 == 0;
  const int vpr = a.W * ESZ / 16;
  const int halo = a.pitch - a.W;
  if (vec_ok) {
    // Loads are issued kBatch at a time before any is stored: one memory latency per batch.
    constexpr int kBatch = 8;
    vec_t idvec;
#pragma unroll
    for (int i = 0; i < EPV; ++i) idvec[i] = idv;
    const int nvec = nrows * vpr;
    for (int base = 0; base < nvec; base += 256 * kBatch) {
      vec_t val[kBatch];
      int dst[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int id = base + u * 256 + tid;
        uint32_t r, v;
        a.dvpr.divmod(uint32_t(id), &r, &v);
        const int ih = ih0 + int(r);
        dst[u] = id < nvec ? int(r) * a.pitch + a.XO + int(v) * EPV : -1;
        val[u] = idvec;
        if (id < nvec && ih >= 0 && ih < a.H)
          val[u] = *reinterpret_cast<const vec_t*>(src + int64_t(ih) * a.W + int(v) * EPV);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (dst[u] >= 0) *reinterpret_cast<vec_t*>(stage + dst[u]) = val[u];
    }
  } else {
    for (int id = tid; id < nrows * a.W; id += 256) {
      uint32_t r, x;
      a.dW.divmod(uint32_t(id), &r, &x);
      const int ih = ih0 + int(r);
      stage[int(r) * a.pitch + a.XO + int(x)] = (ih >= 0 && ih < a.H) ? src[int64_t(ih) * a.W + int(x)] : idv;
    }
  }
  for (int id = tid; id < nrows * halo; id += 256) {
    uint32_t r, h;
    a.dhalo.divmod(uint32_t(id), &r, &h);
    stage[int(r) * a.pitch + (int(h) < a.XO ? int(h) : a.W + int(h))] = idv;
  }
}

// Any window: one output per thread and step, run-time window loops.
template <typename T>
__global__ void __launch_bounds__(256)
pool2d_kernel(Pool2dArgs a) {
  using A = typename Elem<T>::acc;
  extern __shared__ __attribute__((aligned(16))) uint8_t pool_lds[];
  T* stage = reinterpret_cast<T*>(pool_lds);
  const int tid = threadIdx.x;
  for (int64_t task = blockIdx.x; task < a.tasks; task += gridDim.x) {
    const int64_t plane = task / a.bands;
    const int band = int(task - plane * a.bands);
    const int ho0 = band * a.HB;
    const int nho = a.Ho - ho0 < a.HB ? a.Ho - ho0 : a.HB;
    const int nrows = (nho - 1) * a.Sh + a.Kh;
    if (task != int64_t(blockIdx.x)) __syncthreads();
    pool2d_stage<T>(a, stage, static_cast<const T*>(a.in) + plane * a.H * a.W, ho0 * a.Sh - a.Ph, nrows, tid);
    __syncthreads();
    const int64_t obase = (plane * a.Ho + ho0) * a.Wo;
    const int items = nho * a.Wo;
    for (int id = tid; id < items; id += 256) {
      uint32_t hl, y;
      a.dWo.divmod(uint32_t(id), &hl, &y);
      const T* w0 = stage + int(hl) * a.Sh * a.pitch + a.XO - a.Pw + int(y) * a.Sw;
      A acc = ident<A>(a.op);
      for (int dx = 0; dx < a.Kh; ++dx)
        for (int dy = 0; dy < a.Kw; ++dy) acc = combine(acc, Elem<T>::load(w0, dx * a.pitch + dy), a.op);
      store_out<A>(a.out, a.out_dtype, obase + id, finish(acc, a.scale));
    }
  }
}

// Compile-time window, stride and left padding, input rows that are whole 16-byte vectors.
// Persistent workgroups walk over (plane, band) tasks; while one task is folded out of LDS the
// 16-byte loads of the next are in flight into registers.  A thread produces VO = EPV / SW
// neighbouring outputs of one output row from aligned 16-byte LDS reads (plus the PW elements in
// front of them): it converts each element once, folds the KH rows element-wise, then the KW
// neighbours of every output.
template <typename T, int KH, int KW, int SH, int SW, int PW, bool ISMAX, int B>
__global__ void __launch_bounds__(256)
pool2d_vec_kernel(Pool2dArgs a) {
  using A = typename Elem<T>::acc;
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  constexpr int VO = EPV / SW;                      // outputs per thread and step
  constexpr int NEED = (VO - 1) * SW + KW - PW;     // elements from the aligned boundary on
  constexpr int NVF = NEED / EPV, TAIL = NEED % EPV;
  constexpr int SPAN = PW + NEED;
  constexpr int OP = ISMAX ? GS_MAX : GS_SUM;
  typedef T vec_t __attribute__((ext_vector_type(EPV)));
  extern __shared__ __attribute__((aligned(16))) uint8_t pool_lds[];
  T* stage = reinterpret_cast<T*>(pool_lds);
  const int tid = threadIdx.x;
  const T idv = ident_elem<T>(OP);
  vec_t idvec;
#pragma unroll
  for (int i = 0; i < EPV; ++i) idvec[i] = idv;
  const int vpr = a.W * ESZ / 16;
  const int halo = a.pitch - a.W;
  const bool out_native = a.out_dtype == (__is_same(T, int8_t) ? GS_I8 : __is_same(T, int32_t) ? GS_I32
                                          : __is_same(T, uint16_t) ? GS_BF16 : GS_F32);
  const bool vec_store = out_native && a.Wo % VO == 0 &&
                         reinterpret_cast<uintptr_t>(a.out) % (VO * ESZ) == 0;

  vec_t val[B];
  auto issue_loads = [&](int64_t task) {
    const int64_t plane = task / a.bands;
    const int band = int(task - plane * a.bands);
    const int ho0 = band * a.HB;
    const int nho = a.Ho - ho0 < a.HB ? a.Ho - ho0 : a.HB;
    const int nvec = ((nho - 1) * SH + KH) * vpr;
    const int ih0 = ho0 * SH - a.Ph;
    const T* src = static_cast<const T*>(a.in) + plane * a.H * a.W;
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int id = u * 256 + tid;
      uint32_t r, v;
      a.dvpr.divmod(uint32_t(id), &r, &v);
      const int ih = ih0 + int(r);
      val[u] = idvec;
      if (id < nvec && ih >= 0 && ih < a.H)
        val[u] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(src + int64_t(ih) * a.W + int(v) * EPV));   // read once
    }
  };

  int64_t task = blockIdx.x;
  if (task >= a.tasks) return;
  for (int id = tid; id < a.rows_alloc * halo; id += 256) {   // padding cells, written once
    uint32_t r, h;
    a.dhalo.divmod(uint32_t(id), &r, &h);
    stage[int(r) * a.pitch + (int(h) < a.XO ? int(h) : a.W + int(h))] = idv;
  }
  issue_loads(task);
  for (; task < a.tasks; task += gridDim.x) {
    const int64_t plane = task / a.bands;
    const int band = int(task - plane * a.bands);
    const int ho0 = band * a.HB;
    const int nho = a.Ho - ho0 < a.HB ? a.Ho - ho0 : a.HB;
    const int nvec = ((nho - 1) * SH + KH) * vpr;
    __syncthreads();                                 // the previous task has been folded
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int id = u * 256 + tid;
      if (id < nvec) {
        uint32_t r, v;
        a.dvpr.divmod(uint32_t(id), &r, &v);
        *reinterpret_cast<vec_t*>(stage + int(r) * a.pitch + a.XO + int(v) * EPV) = val[u];
      }
    }
    __syncthreads();
    if (task + gridDim.x < a.tasks) issue_loads(task + gridDim.x);
    const int64_t obase = (plane * a.Ho + ho0) * a.Wo;
    const int items = nho * a.G;
    for (int id = tid; id < items; id += 256) {
      uint32_t hl, g;
      a.dG.divmod(uint32_t(id), &hl, &g);
      // element (dx, c) of the span: LDS row hl*SH + dx, column XO + g*EPV - PW + c
      const T* base = stage + int(hl) * SH * a.pitch + a.XO + int(g) * EPV;
      A col[SPAN];
      static_for<KH>([&](auto dx) {
        const T* row = base + dx * a.pitch;
        A e[SPAN];
        static_for<PW>([&](auto c) { e[c] = Elem<T>::load(row, int(c) - PW); });
        static_for<NVF>([&](auto q) {
          const vec_t v = *reinterpret_cast<const vec_t*>(row + q * EPV);
          static_for<EPV>([&](auto i) { e[PW + q * EPV + i] = Elem<T>::cvt(v[int(i)]); });
        });
        static_for<TAIL>([&](auto c) { e[PW + NVF * EPV + c] = Elem<T>::load(row, NVF * EPV + c); });
        static_for<SPAN>([&](auto c) {
          if constexpr (decltype(dx)::value == 0) col[c] = e[c];
          else col[c] = combine(col[c], e[c], OP);
        });
      });
      A res[VO];
      static_for<VO>([&](auto v) {
        A acc = col[v * SW];
        static_for<KW - 1>([&](auto dy) { acc = combine(acc, col[v * SW + dy + 1], OP); });
        res[v] = acc;
      });
      const int y0 = int(g) * VO;
      const int64_t o = obase + int64_t(hl) * a.Wo + y0;
      if (vec_store) {
        typedef T ovec_t __attribute__((ext_vector_type(VO)));
        ovec_t ov;
        static_for<VO>([&](auto v) {
          if constexpr (__is_same(T, uint16_t)) {
            // a maximum is one of the inputs: its bfloat16 bits are the high half, no rounding
            ov[int(v)] = ISMAX ? uint16_t(__float_as_uint(res[v]) >> 16) : float_to_bf16_bits(finish(res[v], a.scale));
          } else {
            ov[int(v)] = T(finish(res[v], a.scale));
          }
        });
        __builtin_nontemporal_store(ov, reinterpret_cast<ovec_t*>(static_cast<T*>(a.out) + o));   // written once
      } else {
        static_for<VO>([&](auto v) {
          if (y0 + v < a.Wo) store_out<A>(a.out, a.out_dtype, o + v, finish(res[v], a.scale));
        });
      }
    }
  }
}

template <typename T>
static hipError_t launch_pool2d_t(const WindowsReduceArgs& w, hipStream_t s) {
  constexpr int ESZ = int(sizeof(T));
  constexpr int EPV = 16 / ESZ;
  if (w.n_compute != 2) return hipErrorInvalidValue;
  for (int d = 0; d < 2; ++d)
    if (w.in_dim[d] > (1 << 20) || w.out_dim[d] > (1 << 20) || w.win[d] > (1 << 12) ||
        w.stride[d] > (1 << 12) || w.pad_lo[d] > (1 << 12) || w.out_dim[d] < 1)
      return hipErrorInvalidValue;
  Pool2dArgs a;
  a.in = w.in; a.out = w.out; a.out_dtype = w.out_dtype; a.op = w.op; a.scale = w.scale;
  a.H = int(w.in_dim[0]); a.W = int(w.in_dim[1]);
  a.Ho = int(w.out_dim[0]); a.Wo = int(w.out_dim[1]);
  a.Kh = int(w.win[0]); a.Kw = int(w.win[1]);
  a.Sh = int(w.stride[0]); a.Sw = int(w.stride[1]);
  a.Ph = int(w.pad_lo[0]); a.Pw = int(w.pad_lo[1]);
  a.XO = int(round_up(a.Pw, EPV));
  const int64_t reach = int64_t(a.XO) - a.Pw + int64_t(a.Wo - 1) * a.Sw + a.Kw;
  const int64_t width = reach > a.XO + a.W ? reach : a.XO + a.W;
  // one spare vector per row: the last group of outputs of a row may read past the last window
  a.pitch = int(round_up(width + EPV, EPV));
  const int64_t row_bytes = int64_t(a.pitch) * ESZ;
  const int64_t max_rows = kPoolLdsBudget / row_bytes;
  if (max_rows < a.Kh) return hipErrorInvalidValue;
  int64_t hb = (max_rows - a.Kh) / a.Sh + 1;
  if (hb > a.Ho) hb = a.Ho;
  a.bands = int(ceil_div(a.Ho, hb));
  a.HB = int(ceil_div(a.Ho, a.bands));
  a.rows = (a.HB - 1) * a.Sh + a.Kh;
  a.tasks = w.outer * a.bands;
  if (a.tasks == 0) return hipSuccess;
  if (int64_t(a.H) * a.W > (int64_t(1) << 40) / (w.outer > 0 ? w.outer : 1)) return hipErrorInvalidValue;
  a.dvpr = FastDiv::make(uint32_t(a.W * ESZ / 16 > 0 ? a.W * ESZ / 16 : 1));
  a.dW = FastDiv::make(uint32_t(a.W > 0 ? a.W : 1));
  a.dhalo = FastDiv::make(uint32_t(a.pitch - a.W > 0 ? a.pitch - a.W : 1));
  a.dWo = FastDiv::make(uint32_t(a.Wo));
  a.rows_alloc = a.rows;
  a.G = 1;
  a.dG = FastDiv::make(1);
  const size_t lds = size_t(a.rows) * row_bytes;
  if (lds > 60 * 1024) return hipErrorInvalidValue;
  const bool is_max = a.op == GS_MAX;
  const bool vec_in = (a.W * ESZ) % 16 == 0 && reinterpret_cast<uintptr_t>(a.in) % 16 == 0;
  const int64_t need = ceil_div(int64_t(a.rows) * (a.W * ESZ / 16), 256);
  // Persistent grid for the vector kernels: what the chip holds at once, by LDS.
  int per_cu = int((160 * 1024) / (lds + 512));
  per_cu = per_cu < 1 ? 1 : per_cu > 8 ? 8 : per_cu;
  int64_t pgrid = int64_t(reduce_num_cus()) * per_cu;
  if (pgrid > a.tasks) pgrid = a.tasks;
  // Every workgroup gets the same number of tasks: as few workgroups as finish in that many rounds.
  pgrid = ceil_div(a.tasks, ceil_div(a.tasks, pgrid));
#define GS_POOL_VEC(KH_, KW_, SH_, SW_, PW_)                                                        \
  if (vec_in && need <= 8 && a.Kh == KH_ && a.Kw == KW_ && a.Sh == SH_ && a.Sw == SW_ &&           \
      a.Pw == PW_ && EPV % SW_ == 0) {                                                             \
    constexpr int VO_ = EPV / SW_ > 0 ? EPV / SW_ : 1;                                             \
    constexpr int NEED_ = (VO_ - 1) * SW_ + KW_ - PW_;                                             \
    Pool2dArgs v = a;                                                                              \
    v.G = int(ceil_div(a.Wo, VO_));                                                                \
    v.dG = FastDiv::make(uint32_t(v.G));                                                           \
    const int64_t wide = int64_t(v.XO) + int64_t(v.G - 1) * EPV + NEED_;                           \
    if (wide <= a.pitch) {                                                                         \
      if (need <= 4) {                                                                             \
        if (is_max) hipLaunchKernelGGL((pool2d_vec_kernel<T, KH_, KW_, SH_, SW_, PW_, true, 4>),   \
                                       dim3(unsigned(pgrid)), dim3(256), lds, s, v);               \
        else hipLaunchKernelGGL((pool2d_vec_kernel<T, KH_, KW_, SH_, SW_, PW_, false, 4>),         \
                                dim3(unsigned(pgrid)), dim3(256), lds, s, v);                      \
      } else {                                                                                     \
        if (is_max) hipLaunchKernelGGL((pool2d_vec_kernel<T, KH_, KW_, SH_, SW_, PW_, true, 8>),   \
                                       dim3(unsigned(pgrid)), dim3(256), lds, s, v);               \
        else hipLaunchKernelGGL((pool2d_vec_kernel<T, KH_, KW_, SH_, SW_, PW_, false, 8>),         \
                                dim3(unsigned(pgrid)), dim3(256), lds, s, v);                      \
      }                                                                                            \
      return hipGetLastError();                                                                    \
    }                                                                                              \
  }
  GS_POOL_VEC(3, 3, 2, 2, 1)
  GS_POOL_VEC(2, 2, 2, 2, 0)
  GS_POOL_VEC(3, 3, 1, 1, 1)
#undef GS_POOL_VEC
  const unsigned grid = unsigned(a.tasks < (1 << 22) ? a.tasks : (1 << 22));
  hipLaunchKernelGGL((pool2d_kernel<T>), dim3(grid), dim3(256), lds, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_windows_reduce_any(const WindowsReduceArgs& a, hipStream_t s) {
  const hipError_t e = launch_pool2d_t<T>(a, s);
  if (e != hipErrorInvalidValue) return e;
  return launch_windows_reduce_t<T>(a, s);
}

hipError_t launch_windows_reduce(const WindowsReduceArgs& a, hipStream_t s) {
  switch (a.in_dtype) {
    case GS_I8: return launch_windows_reduce_any<int8_t>(a, s);
    case GS_I32: return launch_windows_reduce_any<int32_t>(a, s);
    case GS_BF16: return launch_windows_reduce_any<uint16_t>(a, s);
    case GS_F32: return launch_windows_reduce_any<float>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// ---------------------------------------------------------------------------------------------
// compute reduce (pair a b): element-wise sum or max of two tensors, optional ReLU.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
pair_reduce_kernel(const T* __restrict__ x, const T* __restrict__ y, void* __restrict__ out,
                   int dtype, int op, int relu, int64_t n) {
  using A = typename Elem<T>::acc;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
       i += int64_t(gridDim.x) * blockDim.x) {
    A v = combine(Elem<T>::load(x, i), Elem<T>::load(y, i), op);
    if (relu) v = v > A(0) ? v : A(0);
    store_out<A>(out, dtype, i, v);
  }
}

hipError_t launch_pair_reduce(const PairArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  const int64_t b = ceil_div(a.n, 256);
  const dim3 grid(unsigned(b < (1 << 18) ? b : (1 << 18)));
  switch (a.dtype) {
    case GS_I32:
      hipLaunchKernelGGL((pair_reduce_kernel<int32_t>), grid, dim3(256), 0, s,
                         static_cast<const int32_t*>(a.a), static_cast<const int32_t*>(a.b), a.out,
                         a.dtype, a.op, a.relu, a.n);
      break;
    case GS_BF16:
      hipLaunchKernelGGL((pair_reduce_kernel<uint16_t>), grid, dim3(256), 0, s,
                         static_cast<const uint16_t*>(a.a), static_cast<const uint16_t*>(a.b),
                         a.out, a.dtype, a.op, a.relu, a.n);
      break;
    case GS_F32:
      hipLaunchKernelGGL((pair_reduce_kernel<float>), grid, dim3(256), 0, s,
                         static_cast<const float*>(a.a), static_cast<const float*>(a.b), a.out,
                         a.dtype, a.op, a.relu, a.n);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace gs
