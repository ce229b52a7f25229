// `windows` transformer (Table 1) as an explicit gather: out[a, p.., q..] = in[a, p_i*s_i+q_i-lo_i ..].
//
// windows_generic : any 1..4 compute dims, one output element per thread, consecutive threads
//                   write consecutive output elements (coalesced stores, cached gathers).
#include "common.h"

namespace gs {

template <typename T, typename IdxT>
__global__ void __launch_bounds__(256)
windows_generic_kernel(const T* __restrict__ in, T* __restrict__ out, WindowsArgs a, IdxT total,
                       IdxT win_elems, IdxT out_pos) {
  // total = outer * out_pos * win_elems logical output elements.
  for (IdxT f = IdxT(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += IdxT(gridDim.x) * blockDim.x) {
    IdxT q = f % win_elems;
    IdxT row = f / win_elems;          // (outer, p..) flattened
    IdxT p = row % out_pos;
    IdxT o = row / out_pos;
    int64_t src = o;
    bool inside = true;
    // Decode p and q from the innermost dim outwards, accumulating the source offset.
    int64_t off = 0, mul = 1;
    for (int d = a.n_compute - 1; d >= 0; --d) {
      IdxT qd = q % IdxT(a.win[d]);
      q /= IdxT(a.win[d]);
      IdxT pd = p % IdxT(a.out_dim[d]);
      p /= IdxT(a.out_dim[d]);
      int64_t pos = int64_t(pd) * a.stride[d] + int64_t(qd) - a.pad_lo[d];
      inside = inside && pos >= 0 && pos < a.in_dim[d];
      off += pos * mul;
      mul *= a.in_dim[d];
    }
    src = src * mul + off;
    T v;
    if (inside) {
      v = in[src];
    } else {
      uint32_t bits = a.fill_bits;
      v = *reinterpret_cast<const T*>(&bits);
    }
    out[int64_t(row) * a.out_row_stride + int64_t(f % win_elems)] = v;
  }
}

// Pad columns [K, out_row_stride) of every row with zeros (only used when the row stride is padded).
template <typename T>
__global__ void __launch_bounds__(256)
windows_pad_tail_kernel(T* __restrict__ out, int64_t rows, int64_t K, int64_t ld) {
  const int64_t tail = ld - K;
  const int64_t total = rows * tail;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    out[(f / tail) * ld + K + (f % tail)] = T(0);
  }
}

template <typename T>
static hipError_t launch_generic_t(const WindowsArgs& a, hipStream_t s) {
  int64_t win_elems = 1, out_pos = 1;
  for (int d = 0; d < a.n_compute; ++d) {
    win_elems *= a.win[d];
    out_pos *= a.out_dim[d];
  }
  const int64_t total = a.outer * out_pos * win_elems;
  if (total == 0) return hipSuccess;
  const int threads = 256;
  const int64_t blocks64 = ceil_div(total, threads);
  const int blocks = int(blocks64 < (1 << 20) ? blocks64 : (1 << 20));
  if (total < (int64_t(1) << 31)) {
    hipLaunchKernelGGL((windows_generic_kernel<T, uint32_t>), dim3(blocks), dim3(threads), 0, s,
                       static_cast<const T*>(a.in), static_cast<T*>(a.out), a, uint32_t(total),
                       uint32_t(win_elems), uint32_t(out_pos));
  } else {
    hipLaunchKernelGGL((windows_generic_kernel<T, int64_t>), dim3(blocks), dim3(threads), 0, s,
                       static_cast<const T*>(a.in), static_cast<T*>(a.out), a, total, win_elems,
                       out_pos);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (a.out_row_stride > win_elems) {
    const int64_t rows = a.outer * out_pos;
    const int64_t t2 = rows * (a.out_row_stride - win_elems);
    const int64_t b2 = ceil_div(t2, threads);
    hipLaunchKernelGGL((windows_pad_tail_kernel<T>), dim3(int(b2 < (1 << 20) ? b2 : (1 << 20))),
                       dim3(threads), 0, s, static_cast<T*>(a.out), rows, win_elems,
                       a.out_row_stride);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_windows(const WindowsArgs& a, hipStream_t s) {
  switch (a.esz) {
    case 1: return launch_generic_t<uint8_t>(a, s);
    case 2: return launch_generic_t<uint16_t>(a, s);
    case 4: return launch_generic_t<uint32_t>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace gs
