// `compute reduceSum | reduceMax` (Table 2), the fused `compute reduce (windows ...)` used by
// pooling (Fig. 2c), and `compute reduce (pair a b)` (the element-wise sum idiom of Sec. 5.4).
//
// Row reductions pick a lane-group width G (power of two, 1..64) no smaller than the row length
// when it is short, so that the lanes of a wave read consecutive addresses and several rows are
// reduced per wave with cross-lane shuffles; long rows use one wave (or one workgroup) per row.
#include "common.h"

#include <float.h>
#include <limits.h>

namespace gs {

template <typename T> struct Elem;
template <> struct Elem<int8_t> {
  using acc = int32_t;
  __device__ static acc load(const int8_t* p, int64_t i) { return p[i]; }
};
template <> struct Elem<int32_t> {
  using acc = int32_t;
  __device__ static acc load(const int32_t* p, int64_t i) { return p[i]; }
};
template <> struct Elem<float> {
  using acc = float;
  __device__ static acc load(const float* p, int64_t i) { return p[i]; }
};
template <> struct Elem<uint16_t> {  // bfloat16 bits
  using acc = float;
  __device__ static acc load(const uint16_t* p, int64_t i) { return bf16_bits_to_float(p[i]); }
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

template <typename T>
static hipError_t launch_reduce_t(const ReduceArgs& a, hipStream_t s) {
  if (a.rows == 0) return hipSuccess;
  const T* in = static_cast<const T*>(a.in);
#define GS_LAUNCH_GROUP(G)                                                                       \
  hipLaunchKernelGGL((reduce_rows_group_kernel<T, G>), dim3(unsigned(ceil_div(a.rows * G, 256))), \
                     dim3(256), 0, s, in, a.out, a.out_dtype, a.op, a.rows, a.cols, a.scale)
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

hipError_t launch_windows_reduce(const WindowsReduceArgs& a, hipStream_t s) {
  switch (a.in_dtype) {
    case GS_I8: return launch_windows_reduce_t<int8_t>(a, s);
    case GS_I32: return launch_windows_reduce_t<int32_t>(a, s);
    case GS_BF16: return launch_windows_reduce_t<uint16_t>(a, s);
    case GS_F32: return launch_windows_reduce_t<float>(a, s);
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
