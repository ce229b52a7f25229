// Direct 2D convolution (Fig. 2a) for inputs with fewer channels than one 32-byte channel chunk
// (the 3-channel stem of a CNN).  With so few channels the contraction length K = C*Kh*Kw is
// short, so the whole im2col row of a position fits in LDS: a workgroup forms the rows of the
// im2col matrix of Fig. 5 for 128 positions *in LDS* -- never in memory -- and multiplies them
// with the weight matrix ((O),(K)), which already is K-contiguous in the listing's (C,Kh,Kw)
// order.
//
// A task is up to 128 consecutive positions of one output row (n, x).  Persistent workgroups
// (8 waves) stage the C*Kh input rows of a task in LDS (16-byte loads issued one task ahead into
// registers, padding cells zero), gather the task's [position][k] tile through a table
// k -> LDS offset, run the MFMAs (wave w: positions 32 (w % 4) .. + 31 against channels 32 (w / 4) .. + 31), and
// write the results through a per-wave LDS staging area as 8- or 16-byte stores with residual add
// and ReLU fused.  The weight tile of 64 output channels is loaded once per workgroup.
//
// Row-window form (DR).  When a window row is at most 16 bytes (Kw <= 8 bf16 / 16 int8) and
// consecutive windows start a whole number of dwords apart (Sw * element size a multiple of 4),
// the contraction index is laid out as (c, dx, dy padded to 16 bytes): the 16 bytes an MFMA lane
// needs for position y and row (c, dx) are then the 16 bytes of the staged input row starting at
// column y*Sw - Pw, so the B fragments are read straight from the staged rows with the columns
// past Kw masked to zero, and no [position][k] tile is formed at all.  The first data column of a
// staged row is Pw, which puts every window on a dword boundary (16-byte LDS reads off a dword
// boundary are several times slower); the staged data may then sit off a dword boundary and is
// written with stores aligned to the element only, which the hardware's unaligned mode allows
// and which are few.  The weights get a second copy in that order, zero in the padding.
#include "common.h"

#include <limits.h>

#include <mutex>

namespace gs {

struct SmallCArgs {
  ConvArgs c;
  int K, Kp;        // contraction length and its padding to whole 32-byte MFMA steps (elements)
  int pitch, XO;    // LDS input-row pitch (elements) and first data column
  int wpb;          // LDS bytes per weight / tile row: Kp * esz + 16
  int tile_bytes;   // LDS bytes of the [128][wpb] tile region (at least the four staging areas)
  int xtiles;       // 128-position tasks per output row
  int otiles;       // 64-channel tiles
  int64_t tasks;    // N * Ho * xtiles * otiles
  int vec_ok;       // input rows are whole 16-byte vectors
  uint32_t dr_mask[4];   // row-window form: keeps the first Kw elements of a 16-byte window
  FastDiv dvpr, dW, dhalo, dKh, dT, dKw, dchunk;
};

constexpr int kSmallCBatch = 4;   // 16-byte vectors a thread stages per task
constexpr int kSmallCThreads = 512;

template <typename TR, bool DR>
__global__ void __launch_bounds__(kSmallCThreads) conv_smallc_kernel(SmallCArgs p) {
  constexpr int NT = kSmallCThreads;
  using T = typename std::conditional<TR::kEsz == 1, uint8_t, uint16_t>::type;
  constexpr int ESZ = TR::kEsz;
  constexpr int EPV = 16 / ESZ;
  constexpr int RS = 32 * 4 + 16;          // epilogue staging row stride in bytes
  typedef T outv_t __attribute__((ext_vector_type(EPV)));
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const ConvArgs& a = p.c;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nrows = a.C * a.Kh;
  const int row_bytes = p.pitch * ESZ;
  // LDS: weights [64][wpb] | tile [128][wpb] (reused as 4 staging areas) | input rows (+ zero row) | table
  uint8_t* wl = lds;
  uint8_t* tl = wl + 64 * p.wpb;
  T* stage = reinterpret_cast<T*>(tl + p.tile_bytes);
  const int zero_row = nrows * p.pitch;
  uint32_t* tab = reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(stage) +
                                              round_up(int64_t(nrows + 1) * row_bytes, 16));
  const T* in = static_cast<const T*>(a.act);
  const int vpr = a.W * ESZ / 16;
  const int halo = p.pitch - a.W;
  const bool vec_ok = p.vec_ok != 0;

  // Workgroup b runs on XCD b % 8.  Within each round of gridDim.x tasks an XCD takes a contiguous
  // run of them, so that the input rows shared by neighbouring output rows meet in one L2.
  int64_t task = blockIdx.x;
  if (gridDim.x % 8 == 0) task = int64_t(blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
  if (task >= p.tasks) return;
  // task -> (o tile, n, x, position tile): the channel tile changes slowest so that a workgroup
  // almost never reloads its weights
  const int64_t per_o = p.tasks / p.otiles;
  auto decode = [&](int64_t t, int* ot, int* n, int* ho, int* xt) {
    *ot = int(t / per_o);
    int64_t r = t - int64_t(*ot) * per_o;
    *xt = int(r % p.xtiles);
    r /= p.xtiles;
    *ho = int(r % a.Ho);
    *n = int(r / a.Ho);
  };

  // -- written once: padding cells, zero row, table k -> LDS byte offset of (c, dx, dy) at column 0
  for (int id = tid; id < nrows * halo; id += NT) {
    uint32_t r, h;
    p.dhalo.divmod(uint32_t(id), &r, &h);
    stage[int(r) * p.pitch + (int(h) < p.XO ? int(h) : a.W + int(h))] = T(0);
  }
  for (int id = tid; id < p.pitch; id += NT) stage[zero_row + id] = T(0);
  for (int k = tid; !DR && k < p.Kp; k += NT) {
    int off = zero_row;
    if (k < p.K) {
      uint32_t c, t, dx, dy;
      p.dT.divmod(uint32_t(k), &c, &t);
      p.dKw.divmod(t, &dx, &dy);
      off = (int(c) * a.Kh + int(dx)) * p.pitch + p.XO - a.Pw + int(dy);
    }
    tab[k] = uint32_t(off * ESZ);
  }

  i32x4 val[kSmallCBatch];
  auto issue_loads = [&](int64_t t) {
    int ot, n, ho, xt;
    decode(t, &ot, &n, &ho, &xt);
    const int nvec = nrows * vpr;
#pragma unroll
    for (int u = 0; u < kSmallCBatch; ++u) {
      val[u] = i32x4{0, 0, 0, 0};
      if (u * NT < nvec) {                             // uniform: skip batches past the last vector
        const int id = u * NT + tid;
        uint32_t r, v, c, dx;
        p.dvpr.divmod(uint32_t(id), &r, &v);
        p.dKh.divmod(r, &c, &dx);
        const int ih = ho * a.Sh + int(dx) - a.Ph;
        if (id < nvec && ih >= 0 && ih < a.H)
          val[u] = *reinterpret_cast<const i32x4*>(in + ((int64_t(n) * a.C + int(c)) * a.H + ih) * a.W + int(v) * EPV);
      }
    }
  };
  if (vec_ok) issue_loads(task);

  int cur_ot = -1;
  for (; task < p.tasks; task += gridDim.x) {
    int ot, n, ho, xt;
    decode(task, &ot, &n, &ho, &xt);
    const int y0 = xt * 128;
    const int npos = a.Wo - y0 < 128 ? a.Wo - y0 : 128;
    __syncthreads();                                   // the previous task is out of LDS
    if (ot != cur_ot) {                                // weight tile: rows past O and columns past K are zero
      cur_ot = ot;
      const T* wsrc = static_cast<const T*>(a.wr);     // ((O rounded up to 64),(Kp)), zero padded
      for (int id = tid; id < 64 * (p.Kp / EPV); id += NT) {
        const int r = id / (p.Kp / EPV), v = id - r * (p.Kp / EPV);
        *reinterpret_cast<i32x4*>(wl + r * p.wpb + v * 16) =
            *reinterpret_cast<const i32x4*>(wsrc + (int64_t(ot) * 64 + r) * p.Kp + v * EPV);
      }
    }
    // -- stage the input rows (c, dx): image row ho*Sh + dx - Ph of channel c
    if (vec_ok) {
      const int nvec = nrows * vpr;
#pragma unroll
      for (int u = 0; u < kSmallCBatch; ++u) {
        const int id = u * NT + tid;
        if (u * NT < nvec && id < nvec) {
          uint32_t r, v;
          p.dvpr.divmod(uint32_t(id), &r, &v);
          typedef int32_t word_t __attribute__((aligned(1)));   // aligned to the element only
          word_t* d = reinterpret_cast<word_t*>(reinterpret_cast<uint8_t*>(stage) +
                                                (int(r) * p.pitch + p.XO) * ESZ + int(v) * 16);
          d[0] = val[u][0];
          d[1] = val[u][1];
          d[2] = val[u][2];
          d[3] = val[u][3];
        }
      }
    } else {
      for (int id = tid; id < nrows * a.W; id += NT) {
        uint32_t r, x, c, dx;
        p.dW.divmod(uint32_t(id), &r, &x);
        p.dKh.divmod(r, &c, &dx);
        const int ih = ho * a.Sh + int(dx) - a.Ph;
        stage[int(r) * p.pitch + p.XO + int(x)] =
            (ih >= 0 && ih < a.H) ? in[((int64_t(n) * a.C + int(c)) * a.H + ih) * a.W + int(x)] : T(0);
      }
    }
    __syncthreads();
    if (vec_ok && task + gridDim.x < p.tasks) issue_loads(task + gridDim.x);
    // -- gather the [position][k] tile: item = (position, 16-byte chunk of k)
    if constexpr (!DR) {
      const int nchunk = p.Kp / EPV;
      const int items = npos * nchunk;
      for (int id = tid; id < items; id += NT) {
        uint32_t pos, j;
        p.dchunk.divmod(uint32_t(id), &pos, &j);
        const uint32_t shift = uint32_t((y0 + int(pos)) * a.Sw * ESZ);
        typedef uint32_t tabv_t __attribute__((ext_vector_type(EPV)));
        const tabv_t offs = *reinterpret_cast<const tabv_t*>(tab + int(j) * EPV);
        outv_t v;
#pragma unroll
        for (int i = 0; i < EPV; ++i)
          v[i] = *reinterpret_cast<const T*>(reinterpret_cast<const uint8_t*>(stage) + offs[i] + shift);
        *reinterpret_cast<outv_t*>(tl + int(pos) * p.wpb + int(j) * 16) = v;
      }
      __syncthreads();
    }
    // -- multiply: wave w owns positions 32 (w % 4) .. + 31 and channels 32 (w / 4) .. + 31
    const int pb_ = wave & 3, ob_ = wave >> 2;
    typename TR::accv_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
    if (pb_ * 32 < npos) {
      const uint8_t* ap = wl + (ob_ * 32 + (lane & 31)) * p.wpb + (lane >> 5) * 16;
      const int ksteps = p.Kp * ESZ / 32;
      if constexpr (DR) {
        // K step ks holds input rows 2 ks and 2 ks + 1 (the row after the last is the zero row);
        // lanes past the last position read the last position's windows and are not stored.
        typedef i32x4 win_t __attribute__((aligned(4)));   // windows start on dword boundaries
        const int pos = pb_ * 32 + (lane & 31);
        const uint8_t* bp = reinterpret_cast<const uint8_t*>(stage) +
                            (p.XO - a.Pw + (y0 + (pos < npos ? pos : npos - 1)) * a.Sw) * ESZ +
                            (lane >> 5) * row_bytes;
        const i32x4 keep = {int(p.dr_mask[0]), int(p.dr_mask[1]), int(p.dr_mask[2]), int(p.dr_mask[3])};
        for (int ks = 0; ks < ksteps; ++ks) {
          const i32x4 b = *reinterpret_cast<const win_t*>(bp + ks * 2 * row_bytes) & keep;
          const i32x4 a0 = *reinterpret_cast<const i32x4*>(ap + ks * 32);
          acc = TR::mfma(a0, b, acc);
        }
      } else {
        const uint8_t* bp = tl + (pb_ * 32 + (lane & 31)) * p.wpb + (lane >> 5) * 16;
        for (int ks = 0; ks < ksteps; ++ks) {
          const i32x4 b = *reinterpret_cast<const i32x4*>(bp + ks * 32);
          const i32x4 a0 = *reinterpret_cast<const i32x4*>(ap + ks * 32);
          acc = TR::mfma(a0, b, acc);
        }
      }
    }
    if constexpr (!DR) __syncthreads();                // the tile is free: it becomes the staging areas
    // -- epilogue: out[((n*O + o)*Ho + ho)*Wo + y]
    if (pb_ * 32 < npos) {
      uint8_t* st = tl + wave * (32 * RS);
      const int64_t row0 = ((int64_t(n) * a.O) * a.Ho + ho) * a.Wo + y0 + pb_ * 32;   // o = 0
      const int64_t ostride = int64_t(a.Ho) * a.Wo;
      const bool vec_out = a.Wo % 4 == 0;
      {
        const int m = ob_;
        if (vec_out) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int r = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            *reinterpret_cast<typename TR::acc_t*>(st + r * RS + (lane & 31) * 4) = acc[v];
          }
          const int gq = lane & 7, rsub = lane >> 3;   // 8 groups of 4 positions, 8 rows per step
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const int r = it * 8 + rsub;
            const int o = ot * 64 + m * 32 + r;
            const i32x4 raw = *reinterpret_cast<const i32x4*>(st + r * RS + gq * 16);
            if (o < a.O && pb_ * 32 + gq * 4 < npos) {
              const int64_t addr = row0 + int64_t(o) * ostride + gq * 4;
              if constexpr (__is_same(typename TR::acc_t, int32_t)) {
                i32x4 r4 = raw;
                if (a.residual) r4 += *reinterpret_cast<const i32x4*>(static_cast<const int32_t*>(a.residual) + addr);
                if (a.relu) {
#pragma unroll
                  for (int e = 0; e < 4; ++e) r4[e] = r4[e] > 0 ? r4[e] : 0;
                }
                *reinterpret_cast<i32x4*>(static_cast<int32_t*>(a.out) + addr) = r4;
              } else {
                float f[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) f[e] = __int_as_float(raw[e]);
                if (a.out_dtype == GS_F32) {
                  if (a.residual) {
                    const i32x4 q = *reinterpret_cast<const i32x4*>(static_cast<const float*>(a.residual) + addr);
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[e] += __int_as_float(q[e]);
                  }
                  i32x4 w4;
#pragma unroll
                  for (int e = 0; e < 4; ++e) w4[e] = __float_as_int(a.relu ? fmaxf(f[e], 0.0f) : f[e]);
                  *reinterpret_cast<i32x4*>(static_cast<float*>(a.out) + addr) = w4;
                } else {
                  if (a.residual) {
                    const uint2 q = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.residual) + addr);
                    f[0] += __uint_as_float(q.x << 16); f[1] += __uint_as_float(q.x & 0xffff0000u);
                    f[2] += __uint_as_float(q.y << 16); f[3] += __uint_as_float(q.y & 0xffff0000u);
                  }
#pragma unroll
                  for (int e = 0; e < 4; ++e) f[e] = a.relu ? fmaxf(f[e], 0.0f) : f[e];
                  uint2 w2;
                  w2.x = pack_bf16x2(f[0], f[1]);
                  w2.y = pack_bf16x2(f[2], f[3]);
                  *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + addr) = w2;
                }
              }
            }
          }
        } else {
          const int pos = pb_ * 32 + (lane & 31);
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int o = ot * 64 + m * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (pos < npos && o < a.O)
              store_result<typename TR::acc_t>(a.out, a.residual, a.out_dtype,
                                               row0 + int64_t(o) * ostride + (lane & 31), acc[v], a.relu);
          }
        }
      }
    }
  }
}

// Natural-order copy of the weights for the kernel above: ((O rounded up to 64),(Kp)), zeros in
// the padding.  `w` is ((O),(C,Kh,Kw)) = ((O),(K)) already.
template <typename T>
__global__ void __launch_bounds__(256)
conv_smallc_pack_kernel(const T* __restrict__ w, T* __restrict__ wn, int O, int K, int Kp, int O64) {
  const int64_t total = int64_t(O64) * Kp;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    const int k = int(f % Kp);
    const int64_t o = f / Kp;
    wn[f] = (o < O && k < K) ? w[o * K + k] : T(0);
  }
}

// Row-window copy: ((O rounded up to 64),(C*Kh rounded up to 2, 16 bytes)): element dy of row
// r = c*Kh + dx is w[o][c][dx][dy], zeros for dy >= Kw and in the padding row.
template <typename T>
__global__ void __launch_bounds__(256)
conv_smallc_pack_rows_kernel(const T* __restrict__ w, T* __restrict__ wn, int O, int nrows, int Kw,
                             int rows2, int O64) {
  constexpr int G = 16 / int(sizeof(T));
  const int64_t total = int64_t(O64) * rows2 * G;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    const int dy = int(f % G);
    const int64_t t = f / G;
    const int r = int(t % rows2);
    const int64_t o = t / rows2;
    wn[f] = (o < O && r < nrows && dy < Kw) ? w[(o * nrows + r) * Kw + dy] : T(0);
  }
}

static int smallc_kp(int in_dtype, int C, int Kh, int Kw) {
  const int per = in_dtype == GS_I8 ? 32 : 16;
  return int(round_up(int64_t(C) * Kh * Kw, per));
}

bool conv_is_smallc(int in_dtype, int C) { return C * int(dtype_size(in_dtype)) < 32 && C > 0; }

// The row-window copy exists when a window row fits 16 bytes (whether it is used depends on the
// stride, which the packing call does not know).
static bool smallc_has_rows_copy(int in_dtype, int Kw) { return Kw * int(dtype_size(in_dtype)) <= 16; }
static size_t smallc_natural_bytes(int in_dtype, int O, int C, int Kh, int Kw) {
  return size_t(round_up(O, 64)) * smallc_kp(in_dtype, C, Kh, Kw) * dtype_size(in_dtype);
}
static size_t smallc_rows_offset(int in_dtype, int O, int C, int Kh, int Kw) {
  return size_t(round_up(int64_t(smallc_natural_bytes(in_dtype, O, C, Kh, Kw)), 256));
}

size_t conv_smallc_weight_bytes(int in_dtype, int O, int C, int Kh, int Kw) {
  if (!conv_is_smallc(in_dtype, C)) return 0;
  if (!smallc_has_rows_copy(in_dtype, Kw)) return smallc_natural_bytes(in_dtype, O, C, Kh, Kw);
  return smallc_rows_offset(in_dtype, O, C, Kh, Kw) + size_t(round_up(O, 64)) * round_up(C * Kh, 2) * 16;
}

hipError_t launch_conv_smallc_pack(const void* w, void* wn, int in_dtype, int O, int C, int Kh, int Kw,
                                   hipStream_t s) {
  const int K = C * Kh * Kw, Kp = smallc_kp(in_dtype, C, Kh, Kw), O64 = int(round_up(O, 64));
  const int64_t total = int64_t(O64) * Kp;
  if (total == 0) return hipSuccess;
  const int64_t b = ceil_div(total, 256);
  const dim3 grid(unsigned(b < 4096 ? b : 4096));
  if (in_dtype == GS_I8)
    hipLaunchKernelGGL((conv_smallc_pack_kernel<uint8_t>), grid, dim3(256), 0, s,
                       static_cast<const uint8_t*>(w), static_cast<uint8_t*>(wn), O, K, Kp, O64);
  else
    hipLaunchKernelGGL((conv_smallc_pack_kernel<uint16_t>), grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wn), O, K, Kp, O64);
  if (smallc_has_rows_copy(in_dtype, Kw)) {
    const int nrows = C * Kh, rows2 = int(round_up(nrows, 2));
    void* wrows = static_cast<uint8_t*>(wn) + smallc_rows_offset(in_dtype, O, C, Kh, Kw);
    const int64_t b2 = ceil_div(int64_t(O64) * rows2 * 16 / int64_t(dtype_size(in_dtype)), 256);
    const dim3 grid2(unsigned(b2 < 4096 ? b2 : 4096));
    if (in_dtype == GS_I8)
      hipLaunchKernelGGL((conv_smallc_pack_rows_kernel<uint8_t>), grid2, dim3(256), 0, s,
                         static_cast<const uint8_t*>(w), static_cast<uint8_t*>(wrows), O, nrows, Kw, rows2, O64);
    else
      hipLaunchKernelGGL((conv_smallc_pack_rows_kernel<uint16_t>), grid2, dim3(256), 0, s,
                         static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wrows), O, nrows, Kw, rows2, O64);
  }
  return hipGetLastError();
}

static int smallc_num_cus() {
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

// `a.wr` must point at the natural-order weight copy.  Returns hipErrorInvalidValue when the
// shape does not fit (LDS), so that the caller can fall back.
template <typename TR>
static hipError_t launch_smallc_t(const ConvArgs& a, hipStream_t s) {
  constexpr int ESZ = TR::kEsz;
  constexpr int EPV = 16 / ESZ, EPD = 4 / ESZ;
  SmallCArgs p;
  p.c = a;
  p.K = a.C * a.Kh * a.Kw;
  p.Kp = smallc_kp(a.in_dtype, a.C, a.Kh, a.Kw);
  // Row-window form: windows a whole number of dwords apart, a window row within 16 bytes.
  const bool dr = smallc_has_rows_copy(a.in_dtype, a.Kw) && (a.Sw * ESZ) % 4 == 0;
  if (dr) {
    p.Kp = int(round_up(a.C * a.Kh, 2)) * EPV;
    p.c.wr = static_cast<const uint8_t*>(a.wr) + smallc_rows_offset(a.in_dtype, a.O, a.C, a.Kh, a.Kw);
    for (int d = 0; d < 4; ++d) {
      uint32_t m = 0;
      for (int e = 0; e < EPD; ++e)
        if (d * EPD + e < a.Kw) m |= (ESZ == 2 ? 0xffffu : 0xffu) << (e * ESZ * 8);
      p.dr_mask[d] = m;
    }
  }
  p.wpb = p.Kp * ESZ + 16;
  // First data column of a staged row.  Row-window form: exactly Pw, so that window y starts
  // y*Sw elements into the row, on a dword boundary (the staged data itself may then sit off one).
  p.XO = dr ? a.Pw : int(round_up(a.Pw, EPD));
  const int64_t reach = int64_t(p.XO) - a.Pw + int64_t(a.Wo - 1) * a.Sw + a.Kw;
  const int64_t width = reach > p.XO + a.W ? reach : p.XO + a.W;
  p.pitch = int(round_up(width, EPD));
  if ((p.pitch / EPD) % 2 == 0) p.pitch += EPD;        // an odd number of dwords spreads the gather over banks
  const int nrows = a.C * a.Kh;
  p.vec_ok = ((a.W * ESZ) % 16 == 0 && reinterpret_cast<uintptr_t>(a.act) % 16 == 0 &&
              int64_t(nrows) * (a.W * ESZ / 16) <= kSmallCThreads * kSmallCBatch) ? 1 : 0;
  const int64_t stage_bytes = round_up(int64_t(nrows + 1) * p.pitch * ESZ, 16);
  constexpr int kStaging = (kSmallCThreads / 64) * 32 * (32 * 4 + 16);   // one staging area per wave
  p.tile_bytes = (!dr && 128 * p.wpb > kStaging) ? 128 * p.wpb : kStaging;
  const int64_t lds_bytes = 64 * int64_t(p.wpb) + p.tile_bytes + stage_bytes + int64_t(p.Kp) * 4;
  if (lds_bytes > 96 * 1024 || (int64_t(nrows) + 1) * p.pitch * ESZ > (1 << 20)) return hipErrorInvalidValue;
  p.xtiles = int(ceil_div(a.Wo, 128));
  p.otiles = int(ceil_div(a.O, 64));
  p.tasks = int64_t(a.N) * a.Ho * p.xtiles * p.otiles;
  if (p.tasks == 0) return hipSuccess;
  if (p.tasks > (int64_t(1) << 40)) return hipErrorInvalidValue;
  p.dvpr = FastDiv::make(uint32_t(a.W * ESZ / 16 > 0 ? a.W * ESZ / 16 : 1));
  p.dW = FastDiv::make(uint32_t(a.W));
  p.dhalo = FastDiv::make(uint32_t(p.pitch - a.W > 0 ? p.pitch - a.W : 1));
  p.dKh = FastDiv::make(uint32_t(a.Kh));
  p.dT = FastDiv::make(uint32_t(a.Kh * a.Kw));
  p.dKw = FastDiv::make(uint32_t(a.Kw));
  p.dchunk = FastDiv::make(uint32_t(p.Kp / EPV));
  auto kern = dr ? conv_smallc_kernel<TR, true> : conv_smallc_kernel<TR, false>;
  static std::once_flag once[2];
  static hipError_t attr_status[2] = {hipSuccess, hipSuccess};
  std::call_once(once[dr], [&]() {
    attr_status[dr] = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
  });
  if (attr_status[dr] != hipSuccess) return attr_status[dr];
  int per_cu = int((160 * 1024) / (lds_bytes + 512));
  per_cu = per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu;
  int64_t grid = int64_t(smallc_num_cus()) * per_cu;
  if (grid > p.tasks) grid = p.tasks;
  grid = ceil_div(p.tasks, ceil_div(p.tasks, grid));
  hipLaunchKernelGGL(kern, dim3(unsigned(grid)), dim3(kSmallCThreads), size_t(lds_bytes), s, p);
  return hipGetLastError();
}

hipError_t launch_conv_smallc(const ConvArgs& a, hipStream_t s) {
  if (!conv_is_smallc(a.in_dtype, a.C)) return hipErrorInvalidValue;
  return a.in_dtype == GS_I8 ? launch_smallc_t<I8Traits>(a, s) : launch_smallc_t<Bf16Traits>(a, s);
}

}  // namespace gs
