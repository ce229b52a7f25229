// 2D convolution of Fig. 2a with the windows formed on chip (implicit im2col).
//
//   out[n,o,x,y] = sum_{c,dx,dy} act[n,c,Sh*x+dx-Ph,Sw*y+dy-Pw] * w[o,c,dx,dy]
//
// The contraction is the same `compute dotProd (cartProd windows weights)` as the dense kernel,
// with MFMA rows = output channels o and MFMA columns = flattened output positions
// m = (n, x, y).  Putting the positions on the lanes makes the (N,O,H',W') store of the listing
// (its squeeze + transpose (0 3 1 2) tail) a coalesced store, because for fixed (n, o) the
// positions are contiguous in memory.
//
// A workgroup (4 waves) owns TO output channels x TP consecutive positions.  For every chunk of
// input channels it stages in LDS
//   * the input patch those positions need: whole input rows including the halo, stored
//     [row][pixel][channel] with the channel fastest.  The NCHW -> channel-fastest transposition
//     happens in registers between the coalesced global loads (lanes along W) and the 16-byte
//     LDS writes.  Padded cells are written as zeros, so padding costs nothing later;
//   * the weight slab [o][tap][channel] from a repacked copy of the weights (workspace).
// A window element is then just an address into the patch: lane (position) base + tap offset,
// read 16 bytes (8 bf16 / 16 int8 channels) at a time as the MFMA B operand.  The K order is
// (channel chunk, dx, dy, channel) -- a reordering of the dotProd sum, exact for integers.
//
// A tile of consecutive positions may span several images (small feature maps); the patch is
// then a list of row segments, one per image, described by a small table in LDS.
#include "common.h"

#include <array>
#include <map>
#include <mutex>

namespace gs {

constexpr int kMaxSeg = 16;

struct ConvGeom {
  int T;            // taps = Kh * Kw
  int XO;           // patch columns left of input column 0 (>= Pw, even)
  int PW;           // patch width in pixels (even)
  int HWo;          // Ho * Wo
  int64_t M;        // N * Ho * Wo
  int max_rows;     // most patch rows any tile needs
  int pair_ok;      // W even: pixel pairs may be loaded with one access
};

struct SegTable {
  int nseg;
  int n_first;
  int rowbase[kMaxSeg + 1];
  int ihlo[kMaxSeg];
};

static int conv_max_rows_scan(const ConvArgs& a, int64_t M, int HWo, int TP);

// Row segments of the tile of positions [m0, mend): one per image it touches.
__host__ __device__ inline void build_segments(int64_t m0, int64_t mend, int HWo, int Wo, int Sh,
                                               int Ph, int Kh, SegTable* t) {
  const int n_first = int(m0 / HWo), n_last = int((mend - 1) / HWo);
  t->n_first = n_first;
  t->nseg = n_last - n_first + 1;
  int rows = 0;
  for (int s = 0; s < t->nseg && s < kMaxSeg; ++s) {
    const int64_t img0 = int64_t(n_first + s) * HWo;
    const int pa = int((m0 > img0 ? m0 : img0) - img0);
    const int64_t e = mend < img0 + HWo ? mend : img0 + HWo;
    const int pb = int(e - 1 - img0);
    const int ho_a = pa / Wo, ho_b = pb / Wo;
    t->rowbase[s] = rows;
    t->ihlo[s] = ho_a * Sh - Ph;
    rows += (ho_b - ho_a) * Sh + Kh;
  }
  t->rowbase[t->nseg < kMaxSeg ? t->nseg : kMaxSeg] = rows;
}

// wr[o][tap][c] = w[o][c][tap] for c < C, zero for C <= c < Cpad.
template <typename T>
__global__ void __launch_bounds__(256)
conv_repack_kernel(const T* __restrict__ w, T* __restrict__ wr, int O, int C, int T_, int Cpad) {
  const int64_t total = int64_t(O) * T_ * Cpad;
  for (int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; f < total;
       f += int64_t(gridDim.x) * blockDim.x) {
    const int c = int(f % Cpad);
    const int64_t ot = f / Cpad;
    const int tap = int(ot % T_);
    const int64_t o = ot / T_;
    wr[f] = c < C ? w[(o * C + c) * T_ + tap] : T(0);
  }
}

static int conv_cpad(int in_dtype, int C) {
  const int per_step = in_dtype == GS_I8 ? 32 : 16;   // channels in 32 bytes
  return int(round_up(C, per_step));
}

size_t conv_weight_workspace(int in_dtype, int O, int C, int Kh, int Kw) {
  return size_t(O) * Kh * Kw * conv_cpad(in_dtype, C) * dtype_size(in_dtype);
}

hipError_t launch_conv_repack(const void* w, void* wr, int in_dtype, int O, int C, int Kh, int Kw,
                              hipStream_t s) {
  const int Cpad = conv_cpad(in_dtype, C);
  const int64_t total = int64_t(O) * Kh * Kw * Cpad;
  if (total == 0) return hipSuccess;
  const int64_t b = ceil_div(total, 256);
  const dim3 grid(unsigned(b < 65536 ? b : 65536));
  if (in_dtype == GS_I8)
    hipLaunchKernelGGL((conv_repack_kernel<uint8_t>), grid, dim3(256), 0, s,
                       static_cast<const uint8_t*>(w), static_cast<uint8_t*>(wr), O, C, Kh * Kw, Cpad);
  else
    hipLaunchKernelGGL((conv_repack_kernel<uint16_t>), grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(w), static_cast<uint16_t*>(wr), O, C, Kh * Kw, Cpad);
  return hipGetLastError();
}

// CB = channel-chunk bytes per pixel (32, 64 or 128); WO x WP waves over (channels, positions).
template <typename TR, int TO, int TP, int WO, int WP, int CB>
__global__ void __launch_bounds__(256) conv_direct_kernel(ConvArgs a, ConvGeom g) {
  static_assert(WO * WP == 4, "four waves");
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int ESZ = TR::kEsz;
  constexpr int G = 16 / ESZ;            // channels per 16-byte vector
  constexpr int CCH = CB / ESZ;          // channels per chunk
  constexpr int NCG = CB / 16;           // 16-byte vectors per pixel per chunk
  constexpr int PIXB = CB + 16;          // LDS bytes per patch pixel (odd multiple of 16)
  constexpr int WOT = TO / WO, WPT = TP / WP;
  constexpr int MI = WOT / 32, NJ = WPT / 32;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wo = wave / WP, wp = wave % WP;
  const int64_t tiles_m = ceil_div(g.M, TP);
  const int64_t m0 = (blockIdx.x % tiles_m) * TP;
  const int o0 = int(blockIdx.x / tiles_m) * TO;
  const int64_t mend = m0 + TP < g.M ? m0 + TP : g.M;

  const int wrow = g.T * CB + 16;        // LDS bytes per weight row (odd multiple of 16)
  SegTable* seg = reinterpret_cast<SegTable*>(lds);
  uint8_t* wlds = lds + 256;
  uint8_t* plds = wlds + TO * wrow;

  if (tid == 0) build_segments(m0, mend, g.HWo, a.Wo, a.Sh, a.Ph, a.Kh, seg);
  __syncthreads();
  const int nseg = seg->nseg, n_first = seg->n_first;
  const int total_rows = seg->rowbase[nseg];

  // Patch address of this lane's positions (window origin), one per position block.
  int pbase[NJ];
  int64_t out_base[NJ];
  bool pos_ok[NJ];
#pragma unroll
  for (int n = 0; n < NJ; ++n) {
    const int64_t m = m0 + wp * WPT + n * 32 + (lane & 31);
    pos_ok[n] = m < g.M;
    pbase[n] = 0;
    out_base[n] = 0;
    if (pos_ok[n]) {
      const int img = int(m / g.HWo), p = int(m % g.HWo);
      const int ho = p / a.Wo, wo_ = p % a.Wo;
      const int s = img - n_first;
      const int row = seg->rowbase[s] + (ho * a.Sh - a.Ph - seg->ihlo[s]);
      const int col = wo_ * a.Sw - a.Pw + g.XO;
      pbase[n] = (row * g.PW + col) * PIXB;
      out_base[n] = int64_t(img) * a.O * g.HWo + p;
    }
  }

  typename TR::accv_t acc[MI][NJ];
#pragma unroll
  for (int m = 0; m < MI; ++m)
#pragma unroll
    for (int n = 0; n < NJ; ++n)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[m][n][v] = 0;

  const uint8_t* act = static_cast<const uint8_t*>(a.act);
  const uint8_t* wr = static_cast<const uint8_t*>(a.wr);
  const int XG = g.PW / 2;
  const int64_t plane = int64_t(a.H) * a.W;
  const int64_t wr_row = int64_t(g.T) * a.Cpad * ESZ;   // bytes per output channel in wr

  for (int c0 = 0; c0 < a.Cpad; c0 += CCH) {
    // ---- weights: [o][tap][CB bytes] --------------------------------------------------------
    const int w_items = TO * g.T * NCG;
    for (int it = tid; it < w_items; it += 256) {
      const int v = it % NCG, ot = it / NCG;
      const int tap = ot % g.T, o = ot / g.T;
      i32x4 val = {0, 0, 0, 0};
      if (o0 + o < a.O)
        val = *reinterpret_cast<const i32x4*>(wr + (o0 + o) * wr_row +
                                              (int64_t(tap) * a.Cpad + c0) * ESZ + v * 16);
      *reinterpret_cast<i32x4*>(wlds + o * wrow + tap * CB + v * 16) = val;
    }
    // ---- patch: [row][pixel][CB bytes], transposed from NCHW in registers ----------------------
    const int p_items = total_rows * XG * NCG;
    for (int it = tid; it < p_items; it += 256) {
      const int xg = it % XG, rc = it / XG;
      const int cg = rc % NCG, r = rc / NCG;
      int s = 0;
      while (s + 1 < nseg && seg->rowbase[s + 1] <= r) ++s;
      const int ih = seg->ihlo[s] + (r - seg->rowbase[s]);
      const int iw = 2 * xg - g.XO;
      // e[t]: channel t of this group, low half = pixel iw, high half = pixel iw + 1.
      uint32_t e[G];
#pragma unroll
      for (int t = 0; t < G; ++t) e[t] = 0;
      if (ih >= 0 && ih < a.H && iw + 1 >= 0 && iw < a.W) {
        const int cbase = c0 + cg * G;
        const uint8_t* src = act + ((int64_t(n_first + s) * a.C + cbase) * plane +
                                    int64_t(ih) * a.W + iw) * ESZ;
        const bool ok0 = iw >= 0, ok1 = iw + 1 < a.W;
#pragma unroll
        for (int t = 0; t < G; ++t) {
          if (cbase + t < a.C) {
            const uint8_t* q = src + int64_t(t) * plane * ESZ;
            uint32_t two = 0;
            if constexpr (ESZ == 2) {
              if (g.pair_ok && ok0) {   // W even and iw even: both pixels inside, 4-byte aligned
                two = *reinterpret_cast<const uint32_t*>(q);
              } else {
                if (ok0) two = *reinterpret_cast<const uint16_t*>(q);
                if (ok1) two |= uint32_t(*reinterpret_cast<const uint16_t*>(q + 2)) << 16;
              }
            } else {
              if (g.pair_ok && ok0) {
                two = *reinterpret_cast<const uint16_t*>(q);
              } else {
                if (ok0) two = q[0];
                if (ok1) two |= uint32_t(q[1]) << 8;
              }
            }
            e[t] = two;
          }
        }
      }
      i32x4 v0, v1;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if constexpr (ESZ == 2) {
          v0[d] = int32_t((e[2 * d] & 0xffffu) | (e[2 * d + 1] << 16));
          v1[d] = int32_t((e[2 * d] >> 16) | (e[2 * d + 1] & 0xffff0000u));
        } else {
          v0[d] = int32_t((e[4 * d] & 0xffu) | ((e[4 * d + 1] & 0xffu) << 8) |
                          ((e[4 * d + 2] & 0xffu) << 16) | ((e[4 * d + 3] & 0xffu) << 24));
          v1[d] = int32_t(((e[4 * d] >> 8) & 0xffu) | (((e[4 * d + 1] >> 8) & 0xffu) << 8) |
                          (((e[4 * d + 2] >> 8) & 0xffu) << 16) | (((e[4 * d + 3] >> 8) & 0xffu) << 24));
        }
      }
      uint8_t* dst = plds + (int64_t(r) * g.PW + 2 * xg) * PIXB + cg * 16;
      *reinterpret_cast<i32x4*>(dst) = v0;
      *reinterpret_cast<i32x4*>(dst + PIXB) = v1;
    }
    __syncthreads();

    // ---- MFMA over taps and the chunk's channels --------------------------------------------------
    const int half = (lane >> 5) * 16;
    for (int kh = 0; kh < a.Kh; ++kh) {
      for (int kw = 0; kw < a.Kw; ++kw) {
        const int tap = kh * a.Kw + kw;
        const int tapoff = (kh * g.PW + kw) * PIXB + half;
        const uint8_t* wtap = wlds + (wo * WOT + (lane & 31)) * wrow + tap * CB + half;
#pragma unroll
        for (int ks = 0; ks < CB / 32; ++ks) {
          i32x4 af[MI], bf[NJ];
#pragma unroll
          for (int m = 0; m < MI; ++m)
            af[m] = *reinterpret_cast<const i32x4*>(wtap + m * 32 * wrow + ks * 32);
#pragma unroll
          for (int n = 0; n < NJ; ++n)
            bf[n] = *reinterpret_cast<const i32x4*>(plds + pbase[n] + tapoff + ks * 32);
#pragma unroll
          for (int m = 0; m < MI; ++m)
#pragma unroll
            for (int n = 0; n < NJ; ++n) acc[m][n] = TR::mfma(af[m], bf[n], acc[m][n]);
        }
      }
    }
    __syncthreads();
  }

  // ---- epilogue: out[(img*O + o)*HWo + p], lanes along p ---------------------------------------------
#pragma unroll
  for (int n = 0; n < NJ; ++n) {
    if (!pos_ok[n]) continue;
#pragma unroll
    for (int m = 0; m < MI; ++m) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int o = o0 + wo * WOT + m * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (o < a.O)
          store_result<typename TR::acc_t>(a.out, a.residual, a.out_dtype,
                                           out_base[n] + int64_t(o) * g.HWo, acc[m][n][v], a.relu);
      }
    }
  }
}

// Host: most patch rows any tile of TP positions needs, or -1 if a tile spans too many images.
// The scan over tiles is remembered per shape so that repeated calls cost a map lookup.
static int conv_max_rows(const ConvArgs& a, int64_t M, int HWo, int TP) {
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
    build_segments(m0, mend, HWo, a.Wo, a.Sh, a.Ph, a.Kh, &t);
    if (t.rowbase[t.nseg] > best) best = t.rowbase[t.nseg];
  }
  return best;
}

constexpr int kLdsLimit = 160 * 1024;

template <typename TR, int TO, int TP, int WO, int WP, int CB>
static hipError_t launch_conv_cfg(const ConvArgs& a, const ConvGeom& g, size_t lds_bytes,
                                  hipStream_t s) {
  auto kern = conv_direct_kernel<TR, TO, TP, WO, WP, CB>;
  static size_t attr_bytes = 0;
  if (lds_bytes > attr_bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, int(kLdsLimit));
    if (e != hipSuccess) return e;
    attr_bytes = kLdsLimit;
  }
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

template <typename TR>
static hipError_t launch_conv_t(const ConvArgs& a, hipStream_t s) {
  ConvGeom g;
  g.T = a.Kh * a.Kw;
  g.XO = int(round_up(a.Pw, 2));
  g.PW = int(round_up(g.XO + a.W + a.Pw, 2));
  g.HWo = a.Ho * a.Wo;
  g.M = int64_t(a.N) * g.HWo;
  g.pair_ok = (a.W % 2 == 0) ? 1 : 0;
  g.max_rows = 0;
  if (g.M == 0 || a.O == 0) return hipSuccess;
  hipError_t e = hipErrorInvalidValue;
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
