// One translation unit per (element type, tile shape) of the pipelined convolution kernel, so
// that the many template instances compile in parallel.  Built several times with different
// -DGS_CONV3_TRAITS / -DGS_CONV3_TILE / -DGS_CONV3_NAME (see build.py).
#include "conv4_kernel.h"

#include <mutex>

namespace gs {

// Pipelined kernel launcher: returns hipErrorInvalidValue when this shape does not fit it.
template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW, int D>
static hipError_t launch_conv3_cfg(const ConvArgs& a, ConvGeom g, hipStream_t s) {
  constexpr int MAXI = VW * TR::kEsz >= 16 ? 1 : (VW * TR::kEsz >= 8 ? 2 : 3);   // bounds the register ring
  g.max_rows = conv_max_rows(a, g.M, g.HWo, TP);
  if (g.max_rows < 0) return hipErrorInvalidValue;
  const int64_t items = int64_t(g.max_rows) * (a.W / VW) * 2;
  if (items > 256 * MAXI) return hipErrorInvalidValue;
  const size_t stage_bytes = 4 * 32 * size_t(TP / WP * 4 + 16);   // epilogue staging, one region per wave
  size_t patch_bytes = 2 * size_t(g.max_rows) * g.PW * 48;
  if (patch_bytes < stage_bytes) patch_bytes = stage_bytes;
  const size_t lds_bytes = 1024 + 3 * size_t(a.Kh * a.Kw) * TO * 32 + patch_bytes;
  if (lds_bytes > size_t(kLdsLimit)) return hipErrorInvalidValue;
  auto kern = conv_direct3_kernel<TR, TO, TP, WO, WP, VW, KH, KW, MAXI, D>;
  static std::once_flag once;              // the attribute is set once, whichever thread comes first
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&]() {
    attr_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, int(kLdsLimit));
  });
  if (attr_status != hipSuccess) return attr_status;
  const int64_t tiles = ceil_div(g.M, TP) * ceil_div(a.O, TO);
  const int64_t per_cu = lds_bytes <= size_t(kLdsLimit) / 2 ? 2 : 1;
  const int64_t grid = tiles < per_cu * conv_num_cus() ? tiles : per_cu * conv_num_cus();
  hipLaunchKernelGGL(kern, dim3(unsigned(grid)), dim3(256), lds_bytes, s, a, g);
  return hipGetLastError();
}

// Producer / consumer kernel (eight waves): returns hipErrorInvalidValue when the shape does not
// fit it.  Three weight buffers when the output-channel tile is 64 wide, two when it is 128.
template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW, int MAXI, int D, bool FLAT>
static hipError_t launch_conv4_ring(const ConvArgs& a, const ConvGeom& g, size_t lds_bytes, hipStream_t s) {
  constexpr int NWB = TO <= 64 ? 3 : 2;
  auto kern = conv_direct4_kernel<TR, TO, TP, WO, WP, VW, KH, KW, MAXI, NWB, D, FLAT>;
  static std::once_flag once;              // the attribute is set once, whichever thread comes first
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&]() {
    attr_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, int(kLdsLimit));
  });
  if (attr_status != hipSuccess) return attr_status;
  const int64_t tiles = ceil_div(g.M, g.tps) * ceil_div(a.O, TO) * (a.ksplit > 1 ? a.ksplit : 1);
  const int64_t grid = tiles < conv_num_cus() ? tiles : conv_num_cus();
  hipLaunchKernelGGL(kern, dim3(unsigned(grid)), dim3(512), lds_bytes, s, a, g);
  return hipGetLastError();
}

// Ring depth: four chunks of loads in flight; two when the channel chunks per work item are only
// a multiple of two (int8 with 64 channels) -- instantiated for int8 only, to bound compile time.
template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW, int MAXI, bool FLAT = false>
static hipError_t launch_conv4_cfg(const ConvArgs& a, const ConvGeom& g, size_t lds_bytes, hipStream_t s) {
  const int per_item = a.Cpad / (32 / TR::kEsz) / (a.ksplit > 1 ? a.ksplit : 1);
  if (per_item % 4 == 0)
    return launch_conv4_ring<TR, TO, TP, WO, WP, VW, KH, KW, MAXI, 4, FLAT>(a, g, lds_bytes, s);
  if constexpr (TR::kEsz == 1) {
    if (per_item % 2 == 0)
      return launch_conv4_ring<TR, TO, TP, WO, WP, VW, KH, KW, MAXI, 2, FLAT>(a, g, lds_bytes, s);
  }
  return hipErrorInvalidValue;
}

// Picks the shape of the producers' items: a producer thread moves one or two items of VW pixels
// x 8 (16) channels per chunk.
template <typename TR, int TO, int TP, int WO, int WP, int KH, int KW>
static hipError_t launch_conv4(const ConvArgs& a, ConvGeom g, hipStream_t s) {
  constexpr int NWB = TO <= 64 ? 3 : 2;
  const int ksplit = a.ksplit > 1 ? a.ksplit : 1;
  const int nchunk = a.Cpad / (32 / TR::kEsz);
  if (nchunk % (2 * ksplit) != 0) return hipErrorInvalidValue;   // the ring holds two or four chunks
  // the producers read the blocked weight copy, by 32-bit byte offsets
  if (!a.wblk) return hipErrorInvalidValue;
  if (round_up(a.O, 32) * a.Kh * a.Kw * a.Cpad * TR::kEsz >= (int64_t(1) << 32)) return hipErrorInvalidValue;
  // Positions per tile: TP, or fewer (in steps that keep each wave's share a multiple of 4) when
  // that lowers rounds x tile cost.  A tile's cost is half fixed (the MFMA blocks stay TP wide) and
  // half proportional to its positions (patch traffic, write-back), and with unit strides 7 % less
  // for a tile of whole output rows, which needs one patch row fewer and whose items have no
  // partial rows (strided layers, whose patches are four times larger, measured no better)
  // (measured: 64 channels at 56x56, batch 64, 30.4 us in tiles of 224 positions, 31.9 in tiles of
  // 208; 128 channels at 28x28 24.7 us at 224, 24.9 at 208, 27.2 at 240, 26.9 at 256).
  g.tps = TP;
  {
    const int64_t per_m = ceil_div(a.O, TO) * ksplit, cus = conv_num_cus();
    auto cost = [&](int tps) {
      const double c = double(ceil_div(ceil_div(g.M, tps) * per_m, cus)) * (TP + tps);
      return (tps % a.Wo == 0 && a.Sh * a.Sw == 1) ? c * 0.93 : c;
    };
    for (int tps = TP - 4 * WP; tps >= TP / 2; tps -= 4 * WP)
      if (cost(tps) < cost(g.tps)) g.tps = tps;
  }
  g.max_rows = conv_max_rows(a, g.M, g.HWo, g.tps);
  if (g.max_rows < 0) return hipErrorInvalidValue;
  // Tile order.  An XCD (private L2) owns a contiguous range of tiles.  Channel tile first: its
  // workgroups share a channel tile's weights, and every channel tile re-reads the input.
  // Position tile first: they share a patch, and every XCD reads all the weights -- once if they
  // stay in its L2 (4 MB), else once per position tile.  Take the order that fetches less.
  {
    const double in_b = double(a.N) * a.C * a.H * a.W * TR::kEsz;
    const double w_b = double(a.O) * a.C * a.Kh * a.Kw * TR::kEsz;
    const int64_t n_ot = ceil_div(a.O, TO), tiles_m = ceil_div(g.M, g.tps);
    const double ch_first = in_b * double(n_ot) + w_b * (n_ot < 8 ? 8.0 / double(n_ot) : 1.0);
    const double pos_first = in_b + w_b * 8.0 * (w_b > 3.0e6 ? double(ceil_div(tiles_m, 8)) : 1.0);
    g.pos_major = (n_ot > 1 && pos_first < ch_first) ? 1 : 0;
    g.dTiles = FastDiv::make(uint32_t(g.pos_major ? n_ot : tiles_m));
  }
  g.dW = FastDiv::make(uint32_t(a.W));
  g.dXG = FastDiv::make(1);
  // Patch row pitch: g.PW pixels of 48 bytes with g.PW * 3 / 2 odd, so that consecutive patch rows
  // of one pixel column fall on different 16-byte bank groups (the producers' LDS stores).
  while ((g.PW * 3 / 2) % 2 == 0) g.PW += 2;
  const size_t stage_bytes = 4 * 32 * size_t(TP / WP * 4 + 16);   // epilogue staging, one region per wave
  const size_t patch_bytes = 2 * size_t(g.max_rows) * g.PW * 48;
  const size_t lds_bytes = 1024 + NWB * size_t(a.Kh * a.Kw) * TO * 32 + patch_bytes + stage_bytes;
  if (lds_bytes > size_t(kLdsLimit)) return hipErrorInvalidValue;
  // A producer thread issues 8 (16 for int8) loads per item whatever the item's width, and those
  // instructions are what limits it: one item per thread beats two.  Aligned items (VW pixels of
  // one row, W a multiple of VW) are tried narrowest first, which keeps the most lanes busy; then
  // items of 4 or 8 pixels consecutive in memory, which cross row ends and need no alignment;
  // then two items per thread.
  // Aligned items come in blocks of 2^rb_shift patch rows (see the kernel): the largest block
  // of up to 8 rows whose padding still leaves one item per thread.
  auto items_rb = [&](int vw, int sh) { return ((int64_t(g.max_rows) + (1 << sh) - 1) >> sh << sh) * (a.W / vw) * 2; };
  auto pick_rb = [&](int vw, int maxi) {
    for (int sh = 3; sh > 0; --sh)
      if (items_rb(vw, sh) <= 192 * maxi) return sh;
    return 0;
  };
  auto items = [&](int vw) { return int64_t(g.max_rows) * (a.W / vw) * 2; };
  // Every segment of a tile (one per image it touches) may end with a partial flat item per
  // channel group.
  const int64_t segs = (g.tps + g.HWo - 2) / g.HWo + 1;
  auto flat_items = [&](int vw) { return 2 * ((int64_t(g.max_rows) * a.W + vw - 1) / vw + segs); };
#define GS_TRY(VW_, MAXI_)                                                                   \
  if (a.W % VW_ == 0 && items(VW_) <= 192 * MAXI_) {                                        \
    g.rb_shift = pick_rb(VW_, MAXI_);                                                        \
    g.dXG = FastDiv::make(uint32_t(a.W / VW_));                                              \
    return launch_conv4_cfg<TR, TO, TP, WO, WP, VW_, KH, KW, MAXI_>(a, g, lds_bytes, s);      \
  }
#define GS_TRY_FLAT(VW_, MAXI_)                                                              \
  if (a.W >= VW_ && flat_items(VW_) <= 192 * MAXI_)                                         \
    return launch_conv4_cfg<TR, TO, TP, WO, WP, VW_, KH, KW, MAXI_, true>(a, g, lds_bytes, s);
  GS_TRY(1, 1) GS_TRY(2, 1) GS_TRY(4, 1) GS_TRY(8, 1)
  GS_TRY_FLAT(4, 1) GS_TRY_FLAT(8, 1)
  GS_TRY(1, 2) GS_TRY(2, 2) GS_TRY(4, 2)   // (8, 2) would need 256 ring registers
  GS_TRY_FLAT(4, 2)
#undef GS_TRY
#undef GS_TRY_FLAT
  return hipErrorInvalidValue;
}

template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW>
static hipError_t launch_conv3_depth(const ConvArgs& a, const ConvGeom& g, hipStream_t s) {
  const int nchunk = a.Cpad / (32 / TR::kEsz);
  if (nchunk < 2) return hipErrorInvalidValue;
  if (nchunk % 2 == 0) return launch_conv3_cfg<TR, TO, TP, WO, WP, VW, KH, KW, 2>(a, g, s);
  return hipErrorInvalidValue;   // odd chunk counts take the general kernel
}

template <typename TR, int TO, int TP, int WO, int WP, int VW>
static hipError_t launch_conv3_taps(const ConvArgs& a, const ConvGeom& g, hipStream_t s) {
  if (a.Kh == 3 && a.Kw == 3) return launch_conv3_depth<TR, TO, TP, WO, WP, VW, 3, 3>(a, g, s);
  return launch_conv3_depth<TR, TO, TP, WO, WP, VW, 0, 0>(a, g, s);
}

template <typename TR, int TO, int TP, int WO, int WP>
static hipError_t launch_conv3_vw(const ConvArgs& a, const ConvGeom& g, hipStream_t s) {
  constexpr int ESZ = TR::kEsz;
  {
    const hipError_t e = (a.Kh == 3 && a.Kw == 3) ? launch_conv4<TR, TO, TP, WO, WP, 3, 3>(a, g, s)
                                                  : launch_conv4<TR, TO, TP, WO, WP, 0, 0>(a, g, s);
    if (e != hipErrorInvalidValue) return e;
  }
  if (a.ksplit > 1) return hipErrorInvalidValue;   // only the kernel above splits the channel sum
  // Widest pixel vector whose loads stay aligned: W (hence every row start) a multiple of it.
  if (a.W % 8 == 0) return launch_conv3_taps<TR, TO, TP, WO, WP, 8>(a, g, s);
  if (a.W % 4 == 0) return launch_conv3_taps<TR, TO, TP, WO, WP, 4>(a, g, s);
  if (a.W % 2 == 0) return launch_conv3_taps<TR, TO, TP, WO, WP, 2>(a, g, s);
  (void)ESZ;
  return launch_conv3_taps<TR, TO, TP, WO, WP, 1>(a, g, s);
}


#if GS_CONV3_TILE == 0
#define GS_TILE 128, 128, 2, 2
#elif GS_CONV3_TILE == 1
#define GS_TILE 64, 256, 1, 4
#else
#define GS_TILE 64, 128, 1, 4
#endif

hipError_t GS_CONV3_NAME(const ConvArgs& a, const ConvGeom& g, hipStream_t s) {
  return launch_conv3_vw<GS_CONV3_TRAITS, GS_TILE>(a, g, s);
}

}  // namespace gs
