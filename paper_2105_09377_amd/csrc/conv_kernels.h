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
#pragma once
#include "common.h"

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
  int tps;          // producer/consumer kernel: positions a tile covers (<= its MFMA width TP)
  int rb_shift;     // producer/consumer kernel: log2 of the patch rows per block of producer items
  int pos_major;    // producer/consumer kernel: tiles numbered position tile first (all channel tiles of a
                    // position tile are neighbours) instead of channel tile first
  FastDiv dHWo, dWo;  // division by Ho*Wo and by Wo
  FastDiv dTiles, dXG, dW;   // producer/consumer kernel: by position tiles (channel tiles if pos_major), pixel groups per row, W
};

struct SegTable {
  int nseg;
  int n_first;
  int rowbase[kMaxSeg + 1];
  int ihlo[kMaxSeg];
};

// Row segments of the tile of positions [m0, mend): one per image it touches.
__host__ __device__ inline void build_segments(int m0, int mend, int HWo, int Wo, int Sh, int Ph,
                                               int Kh, SegTable* t) {
  const int n_first = m0 / HWo, n_last = (mend - 1) / HWo;
  t->n_first = n_first;
  t->nseg = n_last - n_first + 1;
  int rows = 0;
  for (int s = 0; s < t->nseg && s < kMaxSeg; ++s) {
    const int img0 = (n_first + s) * HWo;
    const int pa = (m0 > img0 ? m0 : img0) - img0;
    const int e = mend < img0 + HWo ? mend : img0 + HWo;
    const int pb = e - 1 - img0;
    const int ho_a = pa / Wo, ho_b = pb / Wo;
    t->rowbase[s] = rows;
    t->ihlo[s] = ho_a * Sh - Ph;
    rows += (ho_b - ho_a) * Sh + Kh;
  }
  t->rowbase[t->nseg < kMaxSeg ? t->nseg : kMaxSeg] = rows;
}

constexpr int kLdsLimit = 160 * 1024;

// Host: most patch rows any tile of TP positions needs (memoised per shape), or -1 if a tile would
// span more images than the segment table holds.  Defined in conv.hip.
int conv_max_rows(const ConvArgs& a, int64_t M, int HWo, int TP);
int conv_num_cus();

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

  if (tid == 0) build_segments(int(m0), int(mend), g.HWo, a.Wo, a.Sh, a.Ph, a.Kh, seg);
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

// ---------------------------------------------------------------------------------------------
// Pipelined, persistent kernel.  Same tiling and LDS patch idea as conv_direct_kernel, with
//   * persistent workgroups: each walks tiles id, id + grid, ... so that loads for the next tile
//     are in flight while the current one is computed;
//   * 32-byte channel chunks (16 bf16 / 32 int8 channels).  Patch data travels global ->
//     registers -> LDS through a ring of D register sets: the load for chunk k + D is issued as
//     soon as chunk k has been written to LDS, which puts D chunks (several microseconds) of
//     memory latency cover between a load and its use.  The ring runs across tile boundaries;
//   * weights stream global -> LDS directly (global_load_lds) two chunks ahead, through three
//     LDS buffers; they are re-read per tile from L2;
//   * wide patch loads: one item = G channels x VW consecutive pixels of one input row, loaded
//     as G accesses of VW pixels (up to 16 bytes) and transposed in registers into VW
//     channel-fastest 16-byte vectors;
//   * padding: the two patch buffers are zero-filled at the start of every tile and the loads
//     only ever write real pixels.
// Weight slab layout in LDS: [tap][o][32 bytes], 16-byte column c of row o at position
// c ^ (((o >> 2) ^ (o >> 3)) & 1), which makes the 16-byte fragment reads of 8 (and of 16)
// consecutive rows hit distinct bank groups
//// bank groups although rows are only 32 bytes apart.
//   * barriers that wait for LDS traffic only, with explicit vector-memory waits sized so that
//     exactly the weight chunk needed next has landed while the ring loads stay in flight.  This
//     relies on every wave issuing the same, statically known sequence of vector-memory
//     instructions per chunk: [weights of chunk k+2] [ring load of chunk k+1+D], each of fixed
//     length (out-of-range work is redirected to valid addresses instead of being skipped).
// Requires C % G == 0, W % VW == 0, D >= 2 and (C / chunk channels) % D == 0; the host checks and
// otherwise uses conv_direct_kernel.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(1))) const void* conv_gptr_t;
typedef __attribute__((address_space(3))) void* conv_lptr_t;

#define CONV3_BARRIER() lds_barrier()
#define CONV3_WAIT() wait_vmem<kWaitWeights>()

// Same table as build_segments, built by the first lanes of a wave in parallel: lane s fills
// segment s, lane 0 then turns the row counts into prefix sums.  Call with tid < 64.
__device__ __forceinline__ void build_segments_wave(int lane, int m0, int mend, const ConvGeom& g,
                                                    int Sh, int Ph, int Kh, SegTable* t) {
  const int n_first = int(g.dHWo.div(uint32_t(m0))), n_last = int(g.dHWo.div(uint32_t(mend - 1)));
  const int nseg = n_last - n_first + 1;
  if (lane < nseg && lane < kMaxSeg) {
    const int img0 = (n_first + lane) * g.HWo;
    const int pa = (m0 > img0 ? m0 : img0) - img0;
    const int e = mend < img0 + g.HWo ? mend : img0 + g.HWo;
    const int pb = e - 1 - img0;
    const int ho_a = int(g.dWo.div(uint32_t(pa))), ho_b = int(g.dWo.div(uint32_t(pb)));
    t->ihlo[lane] = ho_a * Sh - Ph;
    t->rowbase[lane + 1] = (ho_b - ho_a) * Sh + Kh;      // row count for now
  }
  if (lane == 0) {
    t->n_first = n_first;
    t->nseg = nseg;
    t->rowbase[0] = 0;
  }
  __builtin_amdgcn_wave_barrier();
  if (lane == 0) {
    int rows = 0;
    for (int s = 0; s < nseg && s < kMaxSeg; ++s) {
      rows += t->rowbase[s + 1];
      t->rowbase[s + 1] = rows;
    }
  }
}

// Ring registers of the patch prefetch: one load of LB bytes.  Ordinary loads, so the compiler
// tracks them and inserts the waits itself; the kernel keeps every path from a load to its use
// free of branches so that those waits name the exact number of younger loads instead of
// draining all of them.
template <int LB> struct RingReg;
template <> struct RingReg<16> {
  i32x4 v;
  __device__ __forceinline__ void load(const uint8_t* p) { v = *reinterpret_cast<const i32x4*>(p); }
  __device__ __forceinline__ uint32_t word(int k) const { return uint32_t(v[k]); }
};
template <> struct RingReg<8> {
  uint2 v;
  __device__ __forceinline__ void load(const uint8_t* p) { v = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ uint32_t word(int k) const { return k == 0 ? v.x : v.y; }
};
template <> struct RingReg<4> {
  uint32_t v;
  __device__ __forceinline__ void load(const uint8_t* p) { v = *reinterpret_cast<const uint32_t*>(p); }
  __device__ __forceinline__ uint32_t word(int) const { return v; }
};
template <> struct RingReg<2> {
  uint32_t v;
  __device__ __forceinline__ void load(const uint8_t* p) { v = *reinterpret_cast<const uint16_t*>(p); }
  __device__ __forceinline__ uint32_t word(int) const { return v; }
};
template <> struct RingReg<1> {
  uint32_t v;
  __device__ __forceinline__ void load(const uint8_t* p) { v = *p; }
  __device__ __forceinline__ uint32_t word(int) const { return v; }
};

template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW, int MAXI, int D>
__global__ void __launch_bounds__(256) conv_direct3_kernel(ConvArgs a, ConvGeom g) {
  static_assert(WO * WP == 4, "four waves");
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  constexpr int ESZ = TR::kEsz;
  constexpr int G = 16 / ESZ;            // channels per 16-byte vector
  constexpr int CCH = 32 / ESZ;          // channels per chunk
  constexpr int PIXB = 48;               // LDS bytes per patch pixel: 32 + 16 pad (odd multiple of 16)
  constexpr int WOT = TO / WO, WPT = TP / WP;
  constexpr int MI = WOT / 32, NJ = WPT / 32;
  constexpr int OB = TO / 32;            // 32-row weight blocks per tap
  constexpr int LB = VW * ESZ;           // bytes per patch load

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wo = wave / WP, wp = wave % WP;
  // Everything below fits 32 bits (the host refuses tensors of 2^31 elements or more), and
  // 64-bit integer division is a long software routine on this hardware.
  const int M = int(g.M);
  const int tiles_m = (M + TP - 1) / TP;
  const int n_tiles = tiles_m * ((a.O + TO - 1) / TO);
  const FastDiv dTiles = FastDiv::make(uint32_t(tiles_m));
  const int Kh = KH ? KH : a.Kh, Kw = KW ? KW : a.Kw;
  const int T = Kh * Kw;

  const int wbytes = T * TO * 32;                     // one weight buffer
  const int pbytes = g.max_rows * g.PW * PIXB;        // one patch buffer
  SegTable* segs = reinterpret_cast<SegTable*>(lds);  // [2]: current and next tile
  uint8_t* wl = lds + 1024;                           // [3][wbytes], 1 KB aligned
  uint8_t* pl = wl + 3 * wbytes;                      // [2][pbytes]

  const uint8_t* act = static_cast<const uint8_t*>(a.act);
  const uint8_t* wr = static_cast<const uint8_t*>(a.wr);
  const int64_t plane = int64_t(a.H) * a.W * ESZ;     // bytes per channel plane
  const int64_t wr_row = int64_t(T) * a.Cpad * ESZ;   // bytes per output channel in wr
  const int XGn = a.W / VW;                           // pixel groups per row
  const FastDiv dXG = FastDiv::make(uint32_t(XGn));
  const int nchunk = a.Cpad / CCH;
  const int n_wq = T * OB;

  // Per-tile descriptors of this thread's patch items (global source, LDS destination).
  struct Items {
    const uint8_t* src[MAXI];
    int dst[MAXI];
    uint32_t okbits;          // bit i: item i exists
  };
  auto make_items = [&](const SegTable* seg, Items& it) {
    const int nseg = seg->nseg;
    const int n_items = seg->rowbase[nseg] * XGn * 2;   // 2 channel groups per chunk
    it.okbits = 0;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      const int id = tid + 256 * i;
      it.src[i] = act;
      it.dst[i] = 512;          // dummy area (VW * 48 bytes at most)
      if (id < n_items) {
        const int rc = int(dXG.div(uint32_t(id))), xg = id - rc * XGn;
        const int cg = rc & 1, r = rc >> 1;
        int s = 0;
        while (s + 1 < nseg && seg->rowbase[s + 1] <= r) ++s;
        const int ih = seg->ihlo[s] + (r - seg->rowbase[s]);
        if (ih >= 0 && ih < a.H) {
          it.okbits |= 1u << i;
          it.src[i] = act + (int64_t(seg->n_first + s) * a.C + cg * G) * plane +
                      (int64_t(ih) * a.W + xg * VW) * ESZ;
          it.dst[i] = int(pl - lds) + (r * g.PW + g.XO + xg * VW) * PIXB + cg * 16;
        }
      }
    }
  };
  // Weight DMA sources of this lane for output-channel tile o0: instruction q covers tap q / OB,
  // rows (q % OB) * 32 .. + 31; lane i fills (row i / 2, position i % 2).
  const int wrow = lane >> 1;
  const int wcol = ((lane & 1) ^ (((wrow >> 2) ^ (wrow >> 3)) & 1)) * 16;
  struct WSrc { const uint8_t* p[OB]; };
  auto make_wsrc = [&](int o0, WSrc& w) {
#pragma unroll
    for (int b = 0; b < OB; ++b) {
      int o = o0 + b * 32 + wrow;
      o = o < a.O ? o : a.O - 1;                      // rows past O are never stored
      w.p[b] = wr + o * wr_row + wcol;
    }
  };
  // Every wave issues NWI weight instructions per chunk (static when the taps are static); the
  // surplus ones repeat the last block, which rewrites the same bytes.
  constexpr int NWI = KH > 0 ? (KH * KW * OB + 3) / 4 : 0;
  // The source table is picked element by element (use_next ? next : current): handing the
  // lambda a reference chosen at run time would force both tables into scratch memory, and
  // scratch loads share the counter that the prefetched global loads are tracked with.
  WSrc wcur, wnxt;
  const uint32_t wl_addr = lds_addr_of(wl);
  auto issue_weights = [&](bool use_next, int chunk, int slot) {
    const int64_t coff = int64_t(chunk) * CCH * ESZ;
    const uint8_t* tab[OB];
#pragma unroll
    for (int b = 0; b < OB; ++b) tab[b] = use_next ? wnxt.p[b] : wcur.p[b];
    auto one = [&](int q) {
      const int tap = q / OB, b = q % OB;
      const uint8_t* src = tab[0];
#pragma unroll
      for (int bb = 1; bb < OB; ++bb) src = (b == bb) ? tab[bb] : src;
      lds_dma16(src + int64_t(tap) * a.Cpad * ESZ + coff, wl_addr + slot * wbytes + q * 1024);
    };
    if constexpr (KH > 0) {
#pragma unroll
      for (int k = 0; k < NWI; ++k) {
        const int q = wave + 4 * k;
        one(q < n_wq ? q : n_wq - 1);
      }
    } else {
      for (int q = wave; q < n_wq; q += 4) one(q);
    }
  };

  RingReg<LB> preg[D][MAXI][G];
  Items cur, nxt;
  auto load_patch = [&](bool use_next, int chunk, auto slot_) {
    constexpr int slot = decltype(slot_)::value;
    const int64_t coff = int64_t(chunk) * CCH * plane;
    // Unconditional: items that do not exist read valid dummy addresses (never stored), so
    // that every wave has the same number of loads in flight.
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      const uint8_t* src = use_next ? nxt.src[i] : cur.src[i];
#pragma unroll
      for (int t = 0; t < G; ++t) preg[slot][i][t].load(src + coff + t * plane);
    }
  };
  // Unconditional as well: items that do not exist write into a 512-byte dummy area behind the
  // segment tables, so that no branch separates a ring load from its use.
  auto store_patch = [&](const Items& it, auto slot_, int buf) {
    constexpr int slot = decltype(slot_)::value;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      uint8_t* pb = lds + it.dst[i] + (((it.okbits >> i) & 1u) ? buf * pbytes : 0);
#pragma unroll
      for (int p = 0; p < VW; ++p) {
        i32x4 v;   // pixel p: element t = channel t of the group
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          uint32_t w = 0;
#pragma unroll
          for (int e = 0; e < 4 / ESZ; ++e) {
            const int t = d * (4 / ESZ) + e;
            const int boff = p * ESZ;
            const uint32_t word = preg[slot][i][t].word(boff / 4);
            const uint32_t val = (word >> ((boff % 4) * 8)) & (ESZ == 2 ? 0xffffu : 0xffu);
            w |= val << (e * ESZ * 8);
          }
          v[d] = int32_t(w);
        }
        *reinterpret_cast<i32x4*>(pb + p * PIXB) = v;
      }
    }
  };

  // A-fragment address inside a 1 KB weight block: row (lane % 32), column lane / 32, swizzled.
  const int afrag = (lane & 31) * 32 + (((lane >> 5) ^ ((((lane & 31) >> 2) ^ ((lane & 31) >> 3)) & 1)) << 4) +
                    wo * (WOT / 32) * 1024;

  auto tile_range = [&](int tile, int* m0, int* mend, int* o0) {
    const int to = int(dTiles.div(uint32_t(tile)));
    *m0 = (tile - to * tiles_m) * TP;
    *o0 = to * TO;
    *mend = *m0 + TP < M ? *m0 + TP : M;
  };

  // ---- prologue: descriptors of the first tile, first D patch chunks and 2 weight chunks in flight ---
  int tile = blockIdx.x;
  if (tile >= n_tiles) return;
  int m0, mend, o0;
  tile_range(tile, &m0, &mend, &o0);
  if (tid < 64) build_segments_wave(tid, m0, mend, g, a.Sh, a.Ph, a.Kh, &segs[0]);
  __syncthreads();
  make_items(&segs[0], cur);
  make_wsrc(o0, wcur);
  nxt = cur;
  static_for<D>([&](auto d_) { load_patch(false, decltype(d_)::value, d_); });
  int wslot = 0;                                       // LDS weight buffer of the current chunk
  wnxt = wcur;
  issue_weights(false, 0, 0);
  issue_weights(false, 1, 1);
  wait_vmem<0>();
  int cur_seg = 0;
  // Vector-memory instructions a wave issues after a weight chunk and before that chunk must
  // have landed: ring load, next weight chunk, ring load.
  constexpr int RL = MAXI * G;
  constexpr int kWaitWeights = KH > 0 ? 2 * RL + NWI : 0;

  for (; tile < n_tiles; tile += gridDim.x) {
    const SegTable* seg = &segs[cur_seg];
    const int next_tile = tile + int(gridDim.x);
    const bool has_next = next_tile < n_tiles;
    int nm0 = m0, nmend = mend, no0 = o0;
    if (has_next) {
      tile_range(next_tile, &nm0, &nmend, &no0);
      if (tid < 64) build_segments_wave(tid, nm0, nmend, g, a.Sh, a.Ph, a.Kh, &segs[cur_seg ^ 1]);
    }
    {  // zero both patch buffers: halo columns and out-of-image rows stay zero for every chunk
      const i32x4 z = {0, 0, 0, 0};
      for (int off = tid * 16; off < 2 * pbytes; off += 256 * 16) *reinterpret_cast<i32x4*>(pl + off) = z;
    }
    CONV3_BARRIER();
    if (has_next) {
      make_items(&segs[cur_seg ^ 1], nxt);
      make_wsrc(no0, wnxt);
    } else {          // nothing follows: surplus prefetches re-read this tile (never consumed)
      nxt = cur;
      wnxt = wcur;
    }

    // Per-lane window origins in the patch, and output addresses.
    int pbase[NJ];
    uint32_t out_base[NJ];
    bool pos_ok[NJ];
#pragma unroll
    for (int n = 0; n < NJ; ++n) {
      const int m = m0 + wp * WPT + n * 32 + (lane & 31);
      pos_ok[n] = m < M;
      pbase[n] = (lane >> 5) * 16;
      out_base[n] = 0;
      if (pos_ok[n]) {
        const int img = int(g.dHWo.div(uint32_t(m))), p = m - img * g.HWo;
        const int ho = int(g.dWo.div(uint32_t(p))), wo_ = p - ho * a.Wo;
        const int s = img - seg->n_first;
        const int row = seg->rowbase[s] + (ho * a.Sh - a.Ph - seg->ihlo[s]);
        const int col = wo_ * a.Sw - a.Pw + g.XO;
        pbase[n] += (row * g.PW + col) * PIXB;
        out_base[n] = uint32_t(img) * uint32_t(a.O) * uint32_t(g.HWo) + uint32_t(p);
      }
    }

    typename TR::accv_t acc[MI][NJ];
    static_for<MI>([&](auto m_) {
      static_for<NJ>([&](auto n_) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[decltype(m_)::value][decltype(n_)::value][v] = 0;
      });
    });

    // Chunk 0 of this tile goes to LDS now; its ring slot is refilled with chunk D.
    store_patch(cur, std::integral_constant<int, 0>{}, 0);
    load_patch(D >= nchunk, D >= nchunk ? D - nchunk : D, std::integral_constant<int, 0>{});
    CONV3_WAIT();
    CONV3_BARRIER();

    for (int cb = 0; cb < nchunk; cb += D) {
      static_for<D>([&](auto d_) {
        constexpr int d = decltype(d_)::value;
        const int ch = cb + d;
        const int buf = ch & 1;
        const uint8_t* wb = wl + wslot * wbytes + afrag;
        const uint8_t* pb = pl + buf * pbytes;
        auto tap_step = [&](int kh, int kw) {
          const int tap = kh * Kw + kw;
          const int tapoff = (kh * g.PW + kw) * PIXB;
          i32x4 af[MI], bf[NJ];
#pragma unroll
          for (int m = 0; m < MI; ++m)
            af[m] = *reinterpret_cast<const i32x4*>(wb + (tap * OB + m) * 1024);
#pragma unroll
          for (int n = 0; n < NJ; ++n)
            bf[n] = *reinterpret_cast<const i32x4*>(pb + pbase[n] + tapoff);
#pragma unroll
          for (int m = 0; m < MI; ++m)
#pragma unroll
            for (int n = 0; n < NJ; ++n) acc[m][n] = TR::mfma(af[m], bf[n], acc[m][n]);
        };
        if constexpr (KH > 0) {
          // Static taps: fragments of tap t+1 are requested before the MFMAs of tap t.
          constexpr int NT = KH * KW;
          const uint32_t wa = lds_addr_of(wb);
          const uint32_t pa = lds_addr_of(pb);
          constexpr int PD = 1;                    // taps requested ahead of the one being multiplied
          i32x4 fr[PD + 1][MI + NJ];
          auto request = [&](int tap, int slot) {
            const int kh = tap / KW, kw = tap - kh * KW;
            const uint32_t tapoff = uint32_t((kh * g.PW + kw) * PIXB);
#pragma unroll
            for (int m = 0; m < MI; ++m) lds_read_pinned(fr[slot][m], wa + (tap * OB + m) * 1024);
#pragma unroll
            for (int n = 0; n < NJ; ++n) lds_read_pinned(fr[slot][MI + n], pa + pbase[n] + tapoff);
          };
          static_for<(PD < NT ? PD : NT)>([&](auto t_) { request(decltype(t_)::value, decltype(t_)::value); });
          static_for<NT>([&](auto t_) {
            constexpr int t = decltype(t_)::value;
            constexpr int slot = t % (PD + 1);
            if constexpr (t + PD < NT) request(t + PD, (t + PD) % (PD + 1));
            constexpr int ahead = (NT - 1 - t) < PD ? (NT - 1 - t) : PD;   // taps requested after tap t
            lds_wait_tied<ahead * (MI + NJ), MI + NJ>(fr[slot]);
#pragma unroll
            for (int m = 0; m < MI; ++m)
#pragma unroll
              for (int n = 0; n < NJ; ++n)
                acc[m][n] = TR::mfma(fr[slot][m], fr[slot][MI + n], acc[m][n]);
          });
        } else {
          for (int kh = 0; kh < Kh; ++kh)
            for (int kw = 0; kw < Kw; ++kw) tap_step(kh, kw);
        }
        // Next chunk of this tile: registers -> LDS; then the weights two chunks ahead (wrapping
        // into the next tile's first chunks) -- their LDS buffer held chunk ch-1, which every wave
        // left behind at the last barrier; then refill the ring slot D chunks ahead.  This order
        // (weights before ring load) keeps the ring loads the youngest requests at their use.
        if (ch + 1 < nchunk) {
          constexpr int ns = (d + 1) % D;
          store_patch(cur, std::integral_constant<int, ns>{}, buf ^ 1);
        }
        {
          const int wch = ch + 2;
          const int slot2 = wslot + 2 >= 3 ? wslot - 1 : wslot + 2;
          const bool wrap = wch >= nchunk;
          issue_weights(wrap, wrap ? wch - nchunk : wch, slot2);
        }
        wslot = wslot + 1 >= 3 ? 0 : wslot + 1;
        if (ch + 1 < nchunk) {
          constexpr int ns = (d + 1) % D;
          const int lch = ch + 1 + D;
          load_patch(lch >= nchunk, lch >= nchunk ? lch - nchunk : lch, std::integral_constant<int, ns>{});
          CONV3_WAIT();
        }
        CONV3_BARRIER();
      });
    }

    // ---- epilogue ---------------------------------------------------------------------------------
    // out[(img*O + o)*HWo + p].  When 4 consecutive positions are contiguous and aligned in the
    // output (H'*W' a multiple of 4), each wave stages one 32-channel block of its results in a
    // private LDS region as 32-bit values and writes it back 4 positions per lane; otherwise
    // every lane stores its own elements.
    if (g.HWo % 4 == 0) {
      constexpr int RS = WPT * 4 + 16;                 // staging row stride in bytes
      constexpr int GR = WPT / 4;                      // 4-position groups per row
      constexpr int ROWS_PER_IT = 64 / GR;
      uint8_t* stage_base = pl;   // the patch buffers are idle now; they are cleared again per tile
      uint8_t* stage = stage_base + wave * (32 * RS);
      // This lane's group of 4 positions is the same for every row it writes back.
      const int gq = lane % GR, rsub = lane / GR;
      const int mm = m0 + wp * WPT + gq * 4;
      const bool grp_ok = mm < M;
      const int gimg = int(g.dHWo.div(uint32_t(grp_ok ? mm : 0)));
      const uint32_t gbase = uint32_t(gimg) * uint32_t(a.O) * uint32_t(g.HWo) + uint32_t(mm - gimg * g.HWo);
      auto write_back = [&](auto kind_) {
        constexpr int kind = decltype(kind_)::value;   // 0: int32, 1: f32, 2: bf16
        static_for<MI>([&](auto m_) {
          constexpr int m = decltype(m_)::value;
          static_for<NJ>([&](auto n_) {
            constexpr int n = decltype(n_)::value;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int r = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
              *reinterpret_cast<typename TR::acc_t*>(stage + r * RS + (n * 32 + (lane & 31)) * 4) = acc[m][n][v];
            }
          });
#pragma unroll
          for (int it = 0; it < 32 / ROWS_PER_IT; ++it) {
            const int r = it * ROWS_PER_IT + rsub;
            const int o = o0 + wo * WOT + m * 32 + r;
            const i32x4 raw = *reinterpret_cast<const i32x4*>(stage + r * RS + gq * 16);
            if (grp_ok && o < a.O) {
              const uint32_t addr = gbase + uint32_t(o) * uint32_t(g.HWo);
              if constexpr (kind == 0) {
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
                if constexpr (kind == 1) {
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
                  if (a.relu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) f[e] = fmaxf(f[e], 0.0f);
                  }
                  uint2 w2;
                  w2.x = pack_bf16x2(f[0], f[1]);
                  w2.y = pack_bf16x2(f[2], f[3]);
                  *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + addr) = w2;
                }
              }
            }
          }
        });
      };
      if constexpr (__is_same(typename TR::acc_t, int32_t)) {
        write_back(std::integral_constant<int, 0>{});
      } else {
        if (a.out_dtype == GS_BF16) write_back(std::integral_constant<int, 2>{});
        else write_back(std::integral_constant<int, 1>{});
      }
    } else {
      static_for<NJ>([&](auto n_) {
        constexpr int n = decltype(n_)::value;
        static_for<MI>([&](auto m_) {
          constexpr int m = decltype(m_)::value;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int o = o0 + wo * WOT + m * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (pos_ok[n] && o < a.O)
              store_result<typename TR::acc_t>(a.out, a.residual, a.out_dtype,
                                               out_base[n] + uint32_t(o) * uint32_t(g.HWo), acc[m][n][v],
                                               a.relu);
          }
        });
      });
    }
    CONV3_BARRIER();   // staging regions are reused as patch buffers by the next tile

    // rotate to the next tile
    cur = nxt;
    wcur = wnxt;
    m0 = nm0; mend = nmend; o0 = no0;
    cur_seg ^= 1;
  }
}

}  // namespace gs
