// Host side of the direct 2D convolution of Fig. 2a: weight packing, kernel selection, and the
// combine step of split channel sums.
//
//   out[n,o,x,y] = sum_{c,dx,dy} act[n,c,Sh*x+dx-Ph,Sw*y+dy-Pw] * w[o,c,dx,dy]
//
// Kernels, in the order they are tried:
//   * conv_smallc_kernel  (conv_smallc.hip)  fewer input channels than one 32-byte chunk;
//   * conv_direct4_kernel (conv4_kernel.h)   eight waves, producers and consumers; may split the
//                                            channel sum among workgroups;
//   * conv_direct3_kernel (conv_kernels.h)   four waves doing everything, same LDS layout;
//   * conv_direct_kernel  (conv_kernels.h)   the simple general kernel.
// All of them put output channels on MFMA rows and flattened output positions (n, x, y) on MFMA
// columns (lanes), which makes the (N,O,H',W') store of the listing coalesced, read weights from
// the packed copy [o][tap][channel] and form windows out of an LDS patch [row][pixel][channel].
#include "conv_kernels.h"

#include <array>
#include <map>
#include <mutex>

namespace gs {

static int conv_max_rows_scan(const ConvArgs& a, int64_t M, int HWo, int TP);

// wr[o][tap][c] = w[o][c][tap] for c < C, zero for C <= c < Cpad.  With `wb` (channel counts
// that are whole chunks, C == Cpad) also the blocked copy (see conv_blocked_weight_offset):
// element e of 16-byte piece i of block (ob, chunk, tap) is
// w[ob * 32 + i / 2][chunk * CCH + h * G + e][tap], G = elements in 16 bytes, CCH = 2 G,
// h = (i % 2) ^ (((r >> 2) ^ (r >> 3)) & 1) with r = i / 2 -- the swizzle the consumers'
// fragment reads undo; rows past O are zero.
template <typename T>
__global__ void __launch_bounds__(256)
conv_repack_kernel(const T* __restrict__ w, T* __restrict__ wr, T* __restrict__ wb, int O, int C, int T_,
                   int Cpad) {
  const int64_t total = int64_t(O) * T_ * Cpad;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    const int c = int(f % Cpad);
    const int64_t ot = f / Cpad;
    const int tap = int(ot % T_);
    const int64_t o = ot / T_;
    wr[f] = c < C ? w[(o * C + c) * T_ + tap] : T(0);
  }
  if (!wb) return;
  constexpr int G = 16 / int(sizeof(T)), CCH = 2 * G;
  const int nchunk = C / CCH;
  const int64_t total_b = round_up(O, 32) * T_ * C;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total_b;
       f += int64_t(gridDim.x) * blockDim.x) {
    const int e = int(f % G);
    const int i = int((f / G) % 64);
    const int64_t blk = f / (G * 64);
    const int tap = int(blk % T_);
    const int chunk = int((blk / T_) % nchunk);
    const int64_t ob = blk / T_ / nchunk;
    const int r = i >> 1, h = (i & 1) ^ (((r >> 2) ^ (r >> 3)) & 1);
    const int64_t o = ob * 32 + r;
    const int c = chunk * CCH + h * G + e;
    wb[f] = o < O ? w[(o * C + c) * T_ + tap] : T(0);
  }
}

static int conv_cpad(int in_dtype, int C) {
  const int per_step = in_dtype == GS_I8 ? 32 : 16;   // channels in 32 bytes
  return int(round_up(C, per_step));
}

size_t conv_smallc_weight_offset(int in_dtype, int O, int C, int Kh, int Kw) {
  return size_t(round_up(int64_t(O) * Kh * Kw * conv_cpad(in_dtype, C) * int64_t(dtype_size(in_dtype)), 256));
}

// The two copies in front of the blocked one.
static size_t conv_weight_front_bytes(int in_dtype, int O, int C, int Kh, int Kw) {
  const size_t tap_major = size_t(O) * Kh * Kw * conv_cpad(in_dtype, C) * dtype_size(in_dtype);
  const size_t natural = conv_smallc_weight_bytes(in_dtype, O, C, Kh, Kw);
  return natural ? conv_smallc_weight_offset(in_dtype, O, C, Kh, Kw) + natural : tap_major;
}

size_t conv_blocked_weight_bytes(int in_dtype, int O, int C, int Kh, int Kw) {
  if (C != conv_cpad(in_dtype, C)) return 0;
  return size_t(round_up(O, 32)) * Kh * Kw * C * dtype_size(in_dtype);
}

size_t conv_blocked_weight_offset(int in_dtype, int O, int C, int Kh, int Kw) {
  return size_t(round_up(int64_t(conv_weight_front_bytes(in_dtype, O, C, Kh, Kw)), 256));
}

size_t conv_weight_workspace(int in_dtype, int O, int C, int Kh, int Kw) {
  const size_t blocked = conv_blocked_weight_bytes(in_dtype, O, C, Kh, Kw);
  return blocked ? conv_blocked_weight_offset(in_dtype, O, C, Kh, Kw) + blocked
                 : conv_weight_front_bytes(in_dtype, O, C, Kh, Kw);
}

hipError_t launch_conv_repack(const void* w, void* wr, int in_dtype, int O, int C, int Kh, int Kw,
                              hipStream_t s) {
  const int Cpad = conv_cpad(in_dtype, C);
  const int64_t total = round_up(O, 32) * Kh * Kw * Cpad;   // the longer of the kernel's two loops
  if (int64_t(O) * Kh * Kw * Cpad == 0) return hipSuccess;
  const int64_t b = ceil_div(total, 256);
  const dim3 grid(unsigned(b < 65536 ? b : 65536));
  uint8_t* wb = conv_blocked_weight_bytes(in_dtype, O, C, Kh, Kw)
                    ? static_cast<uint8_t*>(wr) + conv_blocked_weight_offset(in_dtype, O, C, Kh, Kw)
                    : nullptr;
  if (in_dtype == GS_I8)
    hipLaunchKernelGGL((conv_repack_kernel<uint8_t>), grid, dim3(256), 0, s,
                       static_cast<const uint8_t*>(w), static_cast<uint8_t*>(wr), wb, O, C, Kh * Kw, Cpad);
  else
    hipLaunchKernelGGL((conv_repack_kernel<uint16_t>), grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wr),
                       reinterpret_cast<uint16_t*>(wb), O, C, Kh * Kw, Cpad);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && conv_is_smallc(in_dtype, C))
    e = launch_conv_smallc_pack(w, static_cast<uint8_t*>(wr) + conv_smallc_weight_offset(in_dtype, O, C, Kh, Kw),
                                in_dtype, O, C, Kh, Kw, s);
  return e;
}

// Host: most patch rows any tile of TP positions needs, or -1 if a tile spans too many images.
// The scan over tiles is remembered per shape so that repeated calls cost a map lookup.
int conv_max_rows(const ConvArgs& a, int64_t M, int HWo, int TP) {
  static std::mutex mu;
  static std::map<std::array<int64_t, 7>, int> memo;
  const std::array<int64_t, 7> key = {M, HWo, a.Wo, a.Sh, a.Ph, a.Kh, TP};
  {
    std::lock_guard<std::mutex> lock(mu);
    auto it = memo.find(key);
    if (it != memo.end()) return it->second;
  }
  const int r = conv_max_rows_scan(a, M, HWo, TP);
  std::lock_guard<std::mutex> lock(mu);
  memo[key] = r;
  return r;
}

static int conv_max_rows_scan(const ConvArgs& a, int64_t M, int HWo, int TP) {
  int best = 0;
  SegTable t;
  for (int64_t m0 = 0; m0 < M; m0 += TP) {
    const int64_t mend = m0 + TP < M ? m0 + TP : M;
    if ((mend - 1) / HWo - m0 / HWo + 1 > kMaxSeg) return -1;
    build_segments(int(m0), int(mend), HWo, a.Wo, a.Sh, a.Ph, a.Kh, &t);
    if (t.rowbase[t.nseg] > best) best = t.rowbase[t.nseg];
  }
  return best;
}

int conv_num_cus() {
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

template <typename TR, int TO, int TP, int WO, int WP, int CB>
static hipError_t launch_conv_cfg(const ConvArgs& a, const ConvGeom& g, size_t lds_bytes,
                                  hipStream_t s) {
  auto kern = conv_direct_kernel<TR, TO, TP, WO, WP, CB>;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&]() {
    attr_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, int(kLdsLimit));
  });
  if (attr_status != hipSuccess) return attr_status;
  const int64_t tiles = ceil_div(g.M, TP) * ceil_div(a.O, TO);
  if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3(unsigned(tiles)), dim3(256), lds_bytes, s, a, g);
  return hipGetLastError();
}

static size_t conv_lds_bytes(int TO, int T, int CB, int rows, int PW) {
  return 256 + size_t(TO) * (T * CB + 16) + size_t(rows) * PW * (CB + 16);
}

template <typename TR, int TO, int TP, int WO, int WP>
static hipError_t launch_conv_tile(const ConvArgs& a, ConvGeom g, hipStream_t s) {
  g.max_rows = conv_max_rows(a, g.M, g.HWo, TP);
  if (g.max_rows < 0) return hipErrorInvalidValue;
  const int cbytes = a.Cpad * TR::kEsz;
  // Largest channel chunk that divides the padded channel count and leaves room for two
  // workgroups per compute unit; failing that, the largest that fits at all.
  const int cands[3] = {128, 64, 32};
  for (int pass = 0; pass < 2; ++pass) {
    const size_t limit = pass == 0 ? kLdsLimit / 2 : kLdsLimit;
    for (int ci = 0; ci < 3; ++ci) {
      const int CB = cands[ci];
      if (cbytes % CB) continue;
      const size_t need = conv_lds_bytes(TO, g.T, CB, g.max_rows, g.PW);
      if (need > limit) continue;
      if (CB == 128) return launch_conv_cfg<TR, TO, TP, WO, WP, 128>(a, g, need, s);
      if (CB == 64) return launch_conv_cfg<TR, TO, TP, WO, WP, 64>(a, g, need, s);
      return launch_conv_cfg<TR, TO, TP, WO, WP, 32>(a, g, need, s);
    }
  }
  return hipErrorInvalidValue;
}

// Pipelined kernel instances (conv3_inst.hip), one per element type and tile shape.
hipError_t launch_conv3_bf16_t0(const ConvArgs&, const ConvGeom&, hipStream_t);
hipError_t launch_conv3_bf16_t1(const ConvArgs&, const ConvGeom&, hipStream_t);
hipError_t launch_conv3_bf16_t2(const ConvArgs&, const ConvGeom&, hipStream_t);
hipError_t launch_conv3_i8_t0(const ConvArgs&, const ConvGeom&, hipStream_t);
hipError_t launch_conv3_i8_t1(const ConvArgs&, const ConvGeom&, hipStream_t);
hipError_t launch_conv3_i8_t2(const ConvArgs&, const ConvGeom&, hipStream_t);

// 64 x 256 or 64 x 128 tiles: whichever needs less time by rounds x cost per tile, a wide tile
// costing 1.44 narrow ones (measured: 196 wide tiles of 256 channels at 14x14 take 23.7 us in one
// round, the same layer in 392 narrow tiles 33.0 us in two).  Few tiles therefore go narrow (more
// compute units busy): 256 channels at 14x14, batch 32, 17.9 us in 196 narrow tiles against 23.7
// in 100 wide ones with a two-way split of the channel sum; 512 channels at 7x7, batch 64, with a
// residual, 28 us in 200 narrow tiles against 34 in 104 wide ones split two ways.
static bool conv_prefers_wide_tile(int64_t M, int O) {
  const int64_t cus = 256;
  const int64_t wide = ceil_div(M, 256) * ceil_div(O, 64), narrow = ceil_div(M, 128) * ceil_div(O, 64);
  return double(ceil_div(wide, cus)) * 1.44 < double(ceil_div(narrow, cus));
}

template <typename TR>
static hipError_t launch_conv3(const ConvArgs& a, const ConvGeom& g, hipStream_t s) {
  constexpr bool i8 = TR::kEsz == 1;
  if (a.C % (16 / TR::kEsz) != 0 || a.C != a.Cpad) return hipErrorInvalidValue;
  // Tile shapes: 64 channels x 256 positions (three weight buffers fit, the best pipeline) while
  // that still gives most compute units a tile; 64 x 128 for small feature maps; 128 x 128 last.
  auto t0 = [&]() { return i8 ? launch_conv3_i8_t0(a, g, s) : launch_conv3_bf16_t0(a, g, s); };
  auto t1 = [&]() { return i8 ? launch_conv3_i8_t1(a, g, s) : launch_conv3_bf16_t1(a, g, s); };
  auto t2 = [&]() { return i8 ? launch_conv3_i8_t2(a, g, s) : launch_conv3_bf16_t2(a, g, s); };
  hipError_t e = hipErrorInvalidValue;
  const bool wide = conv_prefers_wide_tile(g.M, a.O);
  e = wide ? t1() : t2();
  if (e != hipErrorInvalidValue) return e;
  e = wide ? t2() : t1();
  if (e != hipErrorInvalidValue) return e;
  return a.O > 64 ? t0() : e;
}

// Combines the partial sums of a split channel sum: out = cvt(relu(sum_k partial[k] + residual)).
template <typename AccT>
__global__ void __launch_bounds__(256)
conv_splitk_finish_kernel(const AccT* __restrict__ partial, int ksplit, int64_t total,
                          const void* __restrict__ residual, void* __restrict__ out, int out_dtype,
                          int relu) {
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total;
       i += int64_t(gridDim.x) * blockDim.x) {
    AccT v = partial[i];
    for (int k = 1; k < ksplit; ++k) v += partial[int64_t(k) * total + i];
    store_result<AccT>(out, residual, out_dtype, i, v, relu);
  }
}

// Same, four results per thread; total and all pointers are multiples of four elements.
template <typename AccT>
__global__ void __launch_bounds__(256)
conv_splitk_finish_vec_kernel(const AccT* __restrict__ partial, int ksplit, int64_t total,
                              const void* __restrict__ residual, void* __restrict__ out, int out_dtype,
                              int relu) {
  typedef AccT acc4_t __attribute__((ext_vector_type(4)));
  const int64_t nvec = total / 4;
  for (int64_t q = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; q < nvec;
       q += int64_t(gridDim.x) * blockDim.x) {
    acc4_t v = __builtin_nontemporal_load(reinterpret_cast<const acc4_t*>(partial) + q);
    for (int k = 1; k < ksplit; ++k)
      v += __builtin_nontemporal_load(reinterpret_cast<const acc4_t*>(partial + int64_t(k) * total) + q);
    if constexpr (__is_same(AccT, int32_t)) {
      if (residual) v += reinterpret_cast<const acc4_t*>(residual)[q];
      if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0 ? v[e] : 0;
      }
      reinterpret_cast<acc4_t*>(out)[q] = v;
    } else if (out_dtype == GS_F32) {
      if (residual) v += reinterpret_cast<const acc4_t*>(residual)[q];
      if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
      }
      reinterpret_cast<acc4_t*>(out)[q] = v;
    } else {
      if (residual) {
        const i32x2 r = reinterpret_cast<const i32x2*>(residual)[q];
        v[0] += __uint_as_float(uint32_t(r.x) << 16); v[1] += __uint_as_float(uint32_t(r.x) & 0xffff0000u);
        v[2] += __uint_as_float(uint32_t(r.y) << 16); v[3] += __uint_as_float(uint32_t(r.y) & 0xffff0000u);
      }
      if (relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
      }
      const i32x2 w = {int32_t(pack_bf16x2(v[0], v[1])), int32_t(pack_bf16x2(v[2], v[3]))};
      reinterpret_cast<i32x2*>(out)[q] = w;
    }
  }
}

int conv_pick_ksplit(int in_dtype, int N, int C, int O, int Ho, int Wo) {
  const int64_t M = int64_t(N) * Ho * Wo;
  const int nchunk = conv_cpad(in_dtype, C) / (in_dtype == GS_I8 ? 32 : 16);
  const int64_t tiles = ceil_div(M, conv_prefers_wide_tile(M, O) ? 256 : 128) * ceil_div(O, 64);
  const int cus = 256;
  if (tiles * 4 <= cus && nchunk % 16 == 0) return 4;
  if (tiles * 2 <= cus && nchunk % 8 == 0) return 2;
  return 1;
}

template <typename TR>
static hipError_t launch_conv_t(const ConvArgs& a_in, hipStream_t s) {
  ConvArgs a = a_in;
  if (a.ksplit < 2 || !a.partial) {
    a.ksplit = 1;
    a.partial = nullptr;
  }
  ConvGeom g;
  g.T = a.Kh * a.Kw;
  g.XO = int(round_up(a.Pw, 2));
  g.PW = int(round_up(g.XO + a.W + a.Pw, 2));
  g.HWo = a.Ho * a.Wo;
  g.M = int64_t(a.N) * g.HWo;
  g.pair_ok = (a.W % 2 == 0) ? 1 : 0;
  g.max_rows = 0;
  g.tps = 0;
  g.rb_shift = 0;
  g.pos_major = 0;
  g.dHWo = FastDiv::make(uint32_t(g.HWo > 0 ? g.HWo : 1));
  g.dWo = FastDiv::make(uint32_t(a.Wo > 0 ? a.Wo : 1));
  if (g.M == 0 || a.O == 0) return hipSuccess;
  if (a.wnat) {                        // fewer channels than a chunk: windows formed as im2col rows in LDS
    ConvArgs b = a;
    b.wr = a.wnat;
    const hipError_t es = launch_conv_smallc(b, s);
    if (es != hipErrorInvalidValue) return es;
  }
  hipError_t e = launch_conv3<TR>(a, g, s);
  if (a.ksplit > 1) {
    if (e == hipSuccess) {
      using AccT = typename TR::acc_t;
      const int64_t total = g.M * a.O;
      const size_t osz = dtype_size(a.out_dtype);
      const bool vec = total % 4 == 0 && reinterpret_cast<uintptr_t>(a.partial) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(a.out) % (4 * osz) == 0 &&
                       reinterpret_cast<uintptr_t>(a.residual) % (4 * osz) == 0;
      const int64_t b = ceil_div(vec ? total / 4 : total, 256);
      const dim3 grid(unsigned(b < 4096 ? b : 4096));
      if (vec)
        hipLaunchKernelGGL((conv_splitk_finish_vec_kernel<AccT>), grid, dim3(256), 0, s,
                           static_cast<const AccT*>(a.partial), a.ksplit, total, a.residual, a.out,
                           a.out_dtype, a.relu);
      else
        hipLaunchKernelGGL((conv_splitk_finish_kernel<AccT>), grid, dim3(256), 0, s,
                           static_cast<const AccT*>(a.partial), a.ksplit, total, a.residual, a.out,
                           a.out_dtype, a.relu);
      return hipGetLastError();
    }
    if (e != hipErrorInvalidValue) return e;
    a.ksplit = 1;                      // no splitting kernel takes this shape: plain path
    a.partial = nullptr;
    e = launch_conv3<TR>(a, g, s);
  }
  if (e != hipErrorInvalidValue) return e;
  if (a.O > 64) {
    e = launch_conv_tile<TR, 128, 128, 2, 2>(a, g, s);
    if (e != hipErrorInvalidValue) return e;
  }
  e = launch_conv_tile<TR, 64, 128, 1, 4>(a, g, s);
  if (e != hipErrorInvalidValue) return e;
  return launch_conv_tile<TR, 64, 64, 2, 2>(a, g, s);
}

hipError_t launch_conv(const ConvArgs& a, hipStream_t s) {
  return a.in_dtype == GS_I8 ? launch_conv_t<I8Traits>(a, s) : launch_conv_t<Bf16Traits>(a, s);
}

}  // namespace gs
