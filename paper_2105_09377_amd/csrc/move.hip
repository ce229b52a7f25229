// The Table 1 transformers that move data -- transpose, slice, concat, pair (and the padding
// extension) -- materialised as standalone kernels.  Every one of them is a copy between two
// strided views of dense row-major tensors:
//
//   out[out_off + sum_d i_d * os[d]] = in[in_off + sum_d i_d * is[d]]   for 0 <= i_d < dims[d]
//
// (transpose: `is` are the input's strides permuted; slice: an input offset; concat / pair: two
// copies into disjoint parts of the output; pad: a fill and a copy at an output offset.)  The
// work is pure HBM traffic: |in| + |out| bytes.  Three kernels:
//   * move_rows_kernel      the last dimension is contiguous on both sides: rows of 16-byte vectors;
//   * move_transpose_kernel the input's contiguous dimension is not the output's: 64 x 64 tiles
//                           through LDS, so that both the reads and the writes are coalesced
//                           (8 bytes per lane on both sides when everything is 8-byte aligned);
//   * move_generic_kernel   anything else, one element per thread.
#include "common.h"

namespace gs {

namespace {

constexpr int kMaxDims = 8;

struct MoveK {
  const uint8_t* in;
  uint8_t* out;
  int rank;                       // dims in use (after dropping extents of 1 and merging)
  int64_t dims[kMaxDims];
  int64_t is[kMaxDims], os[kMaxDims];   // element strides
  int64_t total;                  // product of dims
};

template <typename T>
__global__ void __launch_bounds__(256) move_generic_kernel(MoveK k) {
  const T* in = reinterpret_cast<const T*>(k.in);
  T* out = reinterpret_cast<T*>(k.out);
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < k.total;
       f += int64_t(gridDim.x) * blockDim.x) {
    int64_t r = f, io = 0, oo = 0;
    for (int d = k.rank - 1; d >= 0; --d) {
      const int64_t q = r / k.dims[d], i = r - q * k.dims[d];
      io += i * k.is[d];
      oo += i * k.os[d];
      r = q;
    }
    out[oo] = in[io];
  }
}

// Last dimension contiguous on both sides and a whole number of 16-byte vectors, every other
// stride and both bases multiples of 16 bytes.  A row is cut into segments of `seg` vectors; G
// threads (a power of two) share one (row, segment) unit.
struct RowsK {
  MoveK m;                        // m.dims[rank-1] is the row length in VECTORS; strides in vectors
  int64_t rows, nseg, seg;
  int G;
};
__global__ void __launch_bounds__(256) move_rows_kernel(RowsK k) {
  const i32x4* in = reinterpret_cast<const i32x4*>(k.m.in);
  i32x4* out = reinterpret_cast<i32x4*>(k.m.out);
  const int G = k.G, lane = threadIdx.x & (G - 1);
  const int64_t units_per_step = int64_t(gridDim.x) * (256 / G), units = k.rows * k.nseg;
  const int64_t nv = k.m.dims[k.m.rank - 1];
  for (int64_t unit = int64_t(blockIdx.x) * (256 / G) + threadIdx.x / G; unit < units; unit += units_per_step) {
    const int64_t row = unit / k.nseg, sg = unit - row * k.nseg;
    int64_t r = row, io = 0, oo = 0;
    for (int d = k.m.rank - 2; d >= 0; --d) {
      const int64_t q = r / k.m.dims[d], i = r - q * k.m.dims[d];
      io += i * k.m.is[d];
      oo += i * k.m.os[d];
      r = q;
    }
    const int64_t v0 = sg * k.seg, v1 = v0 + k.seg < nv ? v0 + k.seg : nv;
    for (int64_t v = v0 + lane; v < v1; v += G)
      __builtin_nontemporal_store(__builtin_nontemporal_load(in + io + v), out + oo + v);
  }
}

// Tiled transposition.  Dimension A is contiguous in the input (is = 1), dimension B in the
// output (os = 1); the remaining dimensions are a batch.  A workgroup moves a 64 (B) x 64 (A)
// tile: reads run along A, writes along B, the LDS tile is padded by one element per row.
struct TransK {
  const uint8_t* in;
  uint8_t* out;
  int64_t EA, EB;                 // extents of A and B
  int64_t sA_out, sB_in;          // out stride of A, in stride of B (elements)
  int nb;                         // batch dims
  int64_t bdims[kMaxDims], bis[kMaxDims], bos[kMaxDims];
  int64_t tilesA, tilesB;
};
template <typename T>
__global__ void __launch_bounds__(256) move_transpose_kernel(TransK k) {
  __shared__ T tile[64][64 + 4 / sizeof(T)];
  const T* in = reinterpret_cast<const T*>(k.in);
  T* out = reinterpret_cast<T*>(k.out);
  int64_t t = blockIdx.x;
  const int64_t ta = t % k.tilesA;
  t /= k.tilesA;
  const int64_t tb = t % k.tilesB;
  t /= k.tilesB;
  int64_t io = 0, oo = 0;
  for (int d = k.nb - 1; d >= 0; --d) {
    const int64_t q = t / k.bdims[d], i = t - q * k.bdims[d];
    io += i * k.bis[d];
    oo += i * k.bos[d];
    t = q;
  }
  const int64_t a0 = ta * 64, b0 = tb * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;     // 64 x 4 threads
#pragma unroll 4
  for (int j = ty; j < 64; j += 4) {                          // row j of the tile: B index b0 + j
    const int64_t a = a0 + tx, b = b0 + j;
    if (a < k.EA && b < k.EB) tile[j][tx] = in[io + b * k.sB_in + a];
  }
  __syncthreads();
#pragma unroll 4
  for (int j = ty; j < 64; j += 4) {                          // A index a0 + j, threads along B
    const int64_t a = a0 + j, b = b0 + tx;
    if (a < k.EA && b < k.EB) out[oo + a * k.sA_out + b] = tile[tx][j];
  }
}

// The same with 8 bytes per lane on both sides (extents, strides and bases whole numbers of
// 8-byte vectors): a thread reads NV = 8 / sizeof(T) elements along A, and writes NV along B that
// it collects from NV rows of the LDS tile.  The tile is 64 (A) x TB (B): TB = 256 puts sixteen
// loads per thread in flight before the barrier (large transpositions are bound by how many bytes
// a compute unit keeps in flight), TB = 64 keeps small ones spread over the chip.
template <typename T, int TB>
__global__ void __launch_bounds__(256) move_transpose_vec_kernel(TransK k) {
  constexpr int ESZ = int(sizeof(T)), NV = 8 / ESZ;
  constexpr int TPR = 64 / NV, RPP = 256 / TPR, NPL = TB / RPP;   // loads: threads per tile row, rows per pass, passes
  constexpr int TPS = TB / NV, RPS = 256 / TPS, NPS = 64 / RPS;   // stores: threads per result row, rows per pass, passes
  constexpr int PITCH = 64 + 4 / ESZ;                             // tile row: a whole number of dwords, odd in dwords
  __shared__ __attribute__((aligned(8))) T tile[TB * PITCH];
  const T* in = reinterpret_cast<const T*>(k.in);
  T* out = reinterpret_cast<T*>(k.out);
  int64_t t = blockIdx.x;
  const int64_t ta = t % k.tilesA;
  t /= k.tilesA;
  const int64_t tb = t % k.tilesB;
  t /= k.tilesB;
  int64_t io = 0, oo = 0;
  for (int d = k.nb - 1; d >= 0; --d) {
    const int64_t q = t / k.bdims[d], i = t - q * k.bdims[d];
    io += i * k.bis[d];
    oo += i * k.bos[d];
    t = q;
  }
  const int64_t a0 = ta * 64, b0 = tb * TB;
  {
    const int c = threadIdx.x % TPR, r = threadIdx.x / TPR;
    i32x2 v[NPL];
#pragma unroll
    for (int p = 0; p < NPL; ++p) {                    // every load is issued before the first LDS store
      const int64_t a = a0 + c * NV, b = b0 + p * RPP + r;
      v[p] = i32x2{0, 0};
      if (a < k.EA && b < k.EB)
        v[p] = __builtin_nontemporal_load(reinterpret_cast<const i32x2*>(in + io + b * k.sB_in + a));
    }
#pragma unroll
    for (int p = 0; p < NPL; ++p) {
      uint32_t* d = reinterpret_cast<uint32_t*>(&tile[(p * RPP + r) * PITCH + c * NV]);
      d[0] = uint32_t(v[p].x);
      d[1] = uint32_t(v[p].y);
    }
  }
  __syncthreads();
  const int c = threadIdx.x % TPS, r = threadIdx.x / TPS;
#pragma unroll
  for (int p = 0; p < NPS; ++p) {
    const int ja = p * RPS + r;
    const int64_t a = a0 + ja, b = b0 + c * NV;
    if (a < k.EA && b < k.EB) {
      union {
        T e[NV];
        i32x2 v;
      } u;
#pragma unroll
      for (int i = 0; i < NV; ++i) u.e[i] = tile[(c * NV + i) * PITCH + ja];
      __builtin_nontemporal_store(u.v, reinterpret_cast<i32x2*>(out + oo + a * k.sA_out + b));
    }
  }
}

__global__ void __launch_bounds__(256) fill_kernel(uint8_t* out, int esz, int64_t n, uint32_t bits) {
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < n;
       f += int64_t(gridDim.x) * blockDim.x) {
    if (esz == 1) out[f] = uint8_t(bits);
    else if (esz == 2) reinterpret_cast<uint16_t*>(out)[f] = uint16_t(bits);
    else reinterpret_cast<uint32_t*>(out)[f] = bits;
  }
}

unsigned blocks_for(int64_t items, int64_t cap) {
  const int64_t b = ceil_div(items, 256);
  return unsigned(b < 1 ? 1 : b < cap ? b : cap);
}

}  // namespace

hipError_t launch_fill(void* out, int esz, int64_t n, uint32_t bits, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3(blocks_for(n, 65536)), dim3(256), 0, s,
                     static_cast<uint8_t*>(out), esz, n, bits);
  return hipGetLastError();
}

hipError_t launch_move(const MoveArgs& a, hipStream_t s) {
  if (a.rank < 0 || a.rank > kMaxDims || (a.esz != 1 && a.esz != 2 && a.esz != 4)) return hipErrorInvalidValue;
  MoveK k;
  k.in = static_cast<const uint8_t*>(a.in) + a.in_off * a.esz;
  k.out = static_cast<uint8_t*>(a.out) + a.out_off * a.esz;
  k.rank = 0;
  k.total = 1;
  // Drop dimensions of extent 1; merge neighbours that are contiguous in both views.
  for (int d = 0; d < a.rank; ++d) {
    if (a.dims[d] == 0) return hipSuccess;
    if (a.dims[d] == 1) continue;
    k.total *= a.dims[d];
    if (k.rank > 0 && k.is[k.rank - 1] == a.is[d] * a.dims[d] && k.os[k.rank - 1] == a.os[d] * a.dims[d]) {
      k.dims[k.rank - 1] *= a.dims[d];
      k.is[k.rank - 1] = a.is[d];
      k.os[k.rank - 1] = a.os[d];
    } else {
      k.dims[k.rank] = a.dims[d];
      k.is[k.rank] = a.is[d];
      k.os[k.rank] = a.os[d];
      ++k.rank;
    }
  }
  if (k.rank == 0) {                 // a single element
    k.rank = 1;
    k.dims[0] = 1;
    k.is[0] = k.os[0] = 1;
  }
  const int last = k.rank - 1;
  const int esz = a.esz;

  // Rows of vectors.
  if (k.is[last] == 1 && k.os[last] == 1) {
    bool vec = (k.dims[last] * esz) % 16 == 0 && reinterpret_cast<uintptr_t>(k.in) % 16 == 0 &&
               reinterpret_cast<uintptr_t>(k.out) % 16 == 0;
    for (int d = 0; d < last && vec; ++d) vec = (k.is[d] * esz) % 16 == 0 && (k.os[d] * esz) % 16 == 0;
    if (vec) {
      RowsK r;
      r.m = k;
      const int epv = 16 / esz;
      r.m.dims[last] = k.dims[last] / epv;
      for (int d = 0; d < last; ++d) {
        r.m.is[d] = k.is[d] / epv;
        r.m.os[d] = k.os[d] / epv;
      }
      r.rows = k.total / k.dims[last];
      r.seg = 1024;                                   // 16 KB per unit
      r.nseg = ceil_div(r.m.dims[last], r.seg);
      const int64_t per_unit = r.m.dims[last] < r.seg ? r.m.dims[last] : r.seg;
      int G = 256;
      while (G > 1 && G / 2 >= per_unit) G /= 2;
      r.G = G;
      const int64_t want = ceil_div(r.rows * r.nseg, 256 / G);
      hipLaunchKernelGGL(move_rows_kernel, dim3(unsigned(want < 16384 ? want : 16384)), dim3(256), 0, s, r);
      return hipGetLastError();
    }
  }

  // Tiled transposition: the output's last dimension has a non-unit input stride and some other
  // dimension is the input's contiguous one.
  if (k.os[last] == 1 && k.is[last] != 1) {
    int pa = -1;
    for (int d = 0; d < last; ++d)
      if (k.is[d] == 1) pa = d;
    if (pa >= 0) {
      TransK t;
      t.in = k.in;
      t.out = k.out;
      t.EA = k.dims[pa];
      t.EB = k.dims[last];
      t.sA_out = k.os[pa];
      t.sB_in = k.is[last];
      t.nb = 0;
      int64_t batch = 1;
      for (int d = 0; d < last; ++d) {
        if (d == pa) continue;
        t.bdims[t.nb] = k.dims[d];
        t.bis[t.nb] = k.is[d];
        t.bos[t.nb] = k.os[d];
        batch *= k.dims[d];
        ++t.nb;
      }
      t.tilesA = ceil_div(t.EA, 64);
      t.tilesB = ceil_div(t.EB, 64);
      const int64_t blocks = t.tilesA * t.tilesB * batch;
      const int64_t nv = 8 / esz;
      bool vec8 = t.EA % nv == 0 && t.EB % nv == 0 && t.sA_out % nv == 0 && t.sB_in % nv == 0 &&
                  reinterpret_cast<uintptr_t>(t.in) % 8 == 0 && reinterpret_cast<uintptr_t>(t.out) % 8 == 0;
      for (int d = 0; d < t.nb && vec8; ++d) vec8 = t.bis[d] % nv == 0 && t.bos[d] % nv == 0;
      if (blocks <= 0x7fffffff && vec8) {
        // Tiles 256 long in B while that still leaves several workgroups per compute unit.
        TransK w = t;
        w.tilesB = ceil_div(t.EB, 256);
        const int64_t wide = w.tilesA * w.tilesB * batch;
        if (t.EB >= 256 && wide >= 512) {
          if (esz == 1) hipLaunchKernelGGL((move_transpose_vec_kernel<uint8_t, 256>), dim3(unsigned(wide)), dim3(256), 0, s, w);
          else if (esz == 2) hipLaunchKernelGGL((move_transpose_vec_kernel<uint16_t, 256>), dim3(unsigned(wide)), dim3(256), 0, s, w);
          else hipLaunchKernelGGL((move_transpose_vec_kernel<uint32_t, 256>), dim3(unsigned(wide)), dim3(256), 0, s, w);
          return hipGetLastError();
        }
        if (esz == 1) hipLaunchKernelGGL((move_transpose_vec_kernel<uint8_t, 64>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        else if (esz == 2) hipLaunchKernelGGL((move_transpose_vec_kernel<uint16_t, 64>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        else hipLaunchKernelGGL((move_transpose_vec_kernel<uint32_t, 64>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        return hipGetLastError();
      }
      if (blocks <= 0x7fffffff) {
        if (esz == 1) hipLaunchKernelGGL((move_transpose_kernel<uint8_t>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        else if (esz == 2) hipLaunchKernelGGL((move_transpose_kernel<uint16_t>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        else hipLaunchKernelGGL((move_transpose_kernel<uint32_t>), dim3(unsigned(blocks)), dim3(256), 0, s, t);
        return hipGetLastError();
      }
    }
  }

  const dim3 grid(blocks_for(k.total, 65536));
  if (esz == 1) hipLaunchKernelGGL((move_generic_kernel<uint8_t>), grid, dim3(256), 0, s, k);
  else if (esz == 2) hipLaunchKernelGGL((move_generic_kernel<uint16_t>), grid, dim3(256), 0, s, k);
  else hipLaunchKernelGGL((move_generic_kernel<uint32_t>), grid, dim3(256), 0, s, k);
  return hipGetLastError();
}

}  // namespace gs
