// Producer / consumer form of the direct convolution (Fig. 2a with the windows formed on chip).
//
// Same tiling and LDS layout as conv_direct3_kernel (conv_kernels.h), but a workgroup has eight
// waves, two per SIMD, with fixed roles:
//   * waves 0-3, the consumers, only read MFMA fragments from LDS, multiply, and write results;
//   * waves 4-7, the producers, only move data: activation rows global -> registers (a ring two
//     or four chunks deep) -> transposed 16-byte LDS writes, and weight slabs global -> LDS
//     directly.
// A SIMD therefore always has a wave with MFMAs to issue next to a wave doing address, packing
// and memory work, and the hardware interleaves them; with four do-everything waves those phases
// ran one after the other.  One workgroup barrier per channel chunk hands a filled patch / weight
// buffer from the producers to the consumers and a drained one back.  The producers run through
// tile boundaries without a gap (chunk 0 of the next tile is stored during the last chunk of this
// one), so the consumers' epilogue overlaps the producers' work for the next tile; the epilogue
// stages results in an LDS region of its own for that reason.
//
// Work items (position tile, channel tile, split of the channel sum) are dealt so that each XCD
// owns a contiguous range of them; a tile may cover fewer positions than its MFMA width (g.tps);
// producer items are VW pixels of a row or, in the FLAT form, VW pixels consecutive in memory.
#pragma once
#include "conv_kernels.h"

#include <limits.h>

namespace gs {

// Row segments of a tile of positions [m0, mend), computed on the fly (no table): the tile touches
// images n_first .. n_first + nseg - 1; segment s holds the input rows ihlo .. ihlo + rows - 1 of
// its image, stored in the patch from row `base` on.
struct TileSegs {
  int m0, mend, n_first, nseg;
};
__device__ __forceinline__ TileSegs tile_segs(int m0, int mend, const ConvGeom& g) {
  TileSegs t;
  t.m0 = m0;
  t.mend = mend;
  t.n_first = int(g.dHWo.div(uint32_t(m0)));
  t.nseg = int(g.dHWo.div(uint32_t(mend - 1))) - t.n_first + 1;
  return t;
}
__device__ __forceinline__ void seg_extent(const TileSegs& t, int s, const ConvGeom& g, int Sh, int Ph,
                                           int Kh, int* ihlo, int* rows) {
  const int img0 = (t.n_first + s) * g.HWo;
  const int pa = (t.m0 > img0 ? t.m0 : img0) - img0;
  const int e = t.mend < img0 + g.HWo ? t.mend : img0 + g.HWo;
  const int pb = e - 1 - img0;
  const int ho_a = int(g.dWo.div(uint32_t(pa))), ho_b = int(g.dWo.div(uint32_t(pb)));
  *ihlo = ho_a * Sh - Ph;
  *rows = (ho_b - ho_a) * Sh + Kh;
}
// Patch row r -> (segment, input row); returns false past the last row.
__device__ __forceinline__ bool seg_of_row(const TileSegs& t, int r, const ConvGeom& g, int Sh, int Ph,
                                           int Kh, int* seg, int* ih) {
  int base = 0;
  for (int s = 0; s < t.nseg; ++s) {
    int ihlo, rows;
    seg_extent(t, s, g, Sh, Ph, Kh, &ihlo, &rows);
    if (r < base + rows) {
      *seg = s;
      *ih = ihlo + (r - base);
      return true;
    }
    base += rows;
  }
  return false;
}

// FLAT: a producer item is VW pixels that are consecutive in memory (the valid rows of a segment
// are one contiguous range of the channel plane) rather than VW pixels of one row, so rows whose
// width is not a multiple of VW are still moved with wide loads.  Such loads are aligned to the
// element size only, and each pixel of an item has its own LDS destination.
template <typename TR, int TO, int TP, int WO, int WP, int VW, int KH, int KW, int MAXI, int NWB, int D,
          bool FLAT = false>
__global__ void __launch_bounds__(512) conv_direct4_kernel(ConvArgs a, ConvGeom g) {
  static_assert(WO * WP == 4, "four consumer waves");
  static_assert(NWB == 2 || NWB == 3, "weight buffers");
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  static_assert(D == 2 || D == 4, "ring depth: chunks of patch loads in flight per thread");
  constexpr int ESZ = TR::kEsz;
  constexpr int G = 16 / ESZ;            // channels per 16-byte vector
  constexpr int CCH = 32 / ESZ;          // channels per chunk
  constexpr int PIXB = 48;               // LDS bytes per patch pixel: 32 + 16 pad (odd multiple of 16)
  constexpr int WOT = TO / WO, WPT = TP / WP;
  constexpr int MI = WOT / 32, NJ = WPT / 32;
  constexpr int OB = TO / 32;            // 32-row weight blocks per tap
  constexpr int LB = VW * ESZ;           // bytes per patch load
  constexpr int RS = WPT * 4 + 16;       // epilogue staging row stride in bytes

  const int tid = threadIdx.x, lane = tid & 63;
  // The role must be a scalar (wave-uniform) value: a wave that ran the other role's code with
  // all lanes masked off would still arrive at its barriers.
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool producer = wave >= 4;
  const int M = int(g.M);
  // A tile covers g.tps <= TP positions (a multiple of 8), dealt to the consumer wave columns in
  // groups of eight (the first columns take the odd groups), so that every wave's share starts and
  // ends on a multiple of 8; the MFMA blocks are TP wide and the columns past a wave's share are
  // computed on a valid stand-in position and dropped.  The host shrinks tiles when that fills
  // more compute units.
  const int tps = g.tps;
  const int tiles_m = (M + tps - 1) / tps;
  // A work item ("tile" below) is (position tile, channel tile, K split): the split index runs
  // fastest so that workgroups launched together share a patch.
  const int ksplit = a.ksplit, kshift = ksplit == 4 ? 2 : ksplit == 2 ? 1 : 0;
  const int n_ot = (a.O + TO - 1) / TO;
  const int n_tiles = tiles_m * n_ot * ksplit;
  const FastDiv dTiles = g.dTiles;
  const int Kh = KH ? KH : a.Kh, Kw = KW ? KW : a.Kw;
  const int T = Kh * Kw;
  const int nchunk = a.Cpad / CCH / ksplit;   // chunks per work item: a multiple of D (checked by the host)

  const int wbytes = T * TO * 32;                     // one weight buffer
  const int pbytes = g.max_rows * g.PW * PIXB;        // one patch buffer
  uint8_t* wl = lds + 1024;                           // [NWB][wbytes], 1 KB aligned; dummy area at lds + 512
  uint8_t* pl = wl + NWB * wbytes;                    // [2][pbytes]
  uint8_t* sl = pl + 2 * pbytes;                      // [4][32 * RS] epilogue staging

  // Work item i runs on XCD i % 8 (workgroups are dealt to the 8 XCDs, each with its own L2, in
  // turn, and the grid is a multiple of 8 or a single round).  `lg` renumbers the items so that an
  // XCD owns a contiguous range of the (channel tile, position tile, split) order: its workgroups
  // then share one or two channel tiles' weights and neighbouring patches in that L2.
  const int xcd_per = n_tiles >> 3, xcd_rem = n_tiles & 7;
  auto lg = [&](int i) {
    const int x = i & 7;
    return x * xcd_per + (x < xcd_rem ? x : xcd_rem) + (i >> 3);
  };
  auto tile_range = [&](int item, int* m0, int* mend, int* o0) {
    const int tile = lg(item) >> kshift;
    const int q = int(dTiles.div(uint32_t(tile)));
    // channel tile first: tile = to * tiles_m + mt; position tile first: tile = mt * n_ot + to
    const int to = g.pos_major ? tile - q * n_ot : q;
    const int mt = g.pos_major ? q : tile - q * tiles_m;
    *m0 = mt * tps;
    *o0 = to * TO;
    *mend = *m0 + tps < M ? *m0 + tps : M;
  };

  int tile = blockIdx.x;
  if (tile >= n_tiles) return;
  // The patch buffers start as zeros (the halo columns are never written again): every thread
  // clears its share and all meet at a barrier -- the producers after they have sent off their
  // first weight transfers and patch loads, which touch other LDS or none and so are under way
  // while the buffers are cleared.
  auto clear_patch_buffers = [&]() {
    const i32x4 z = {0, 0, 0, 0};
    for (int off = tid * 16; off < 2 * pbytes; off += 512 * 16) *reinterpret_cast<i32x4*>(pl + off) = z;
    lds_barrier();
  };

  if (producer) {
    // =========================================================================================
    // Producers.  Three cursors walk the same sequence of (tile, chunk) units, each a fixed
    // distance ahead of the consumers: stores 1 unit, weight transfers NWB - 1 units, patch loads
    // 1 + D units.  Everything that depends on the tile only (item sources and destinations,
    // weight rows, rows to clear) is worked out once, when the load cursor enters the tile, and
    // handed down to the other cursors; a chunk step itself is loads at a scalar base plus fixed
    // per-lane offsets, byte permutes, LDS stores at immediate offsets and a few scalar updates.
    // =========================================================================================
    // Wave 4 moves the weights; waves 5-7 move the patches (192 threads, numbered by ptid).  A
    // wave's vector-memory operations complete in order on one counter, so a wave that waited for
    // its weight transfers would also wait for every patch load it issued before them: with the
    // roles apart, patch loads keep the whole ring depth to arrive.
    const int pwave = wave - 4;
    const int ptid = tid - 320;
    constexpr int PT = 192;                             // patch threads
    const uint8_t* act = static_cast<const uint8_t*>(a.act);
    const uint8_t* wr = static_cast<const uint8_t*>(a.wblk);   // 1 KB blocks [O / 32][chunk][tap]
    const int64_t plane = int64_t(a.H) * a.W * ESZ;     // bytes per channel plane
    const uint32_t wr_chunk = uint32_t(T) * 1024u;       // bytes of one chunk of a 32-channel block
    const uint32_t wr_blk = uint32_t(a.Cpad / CCH) * wr_chunk;   // and of all its chunks
    const int n_oblk = (a.O + 31) / 32;
    const int XGn = a.W / VW;                           // pixel groups per row
    const FastDiv dXG = g.dXG;
    const int n_wq = T * OB;
    const int64_t chunk_bytes = int64_t(CCH) * plane;   // activations: one chunk further
    constexpr int ND = FLAT ? VW : 1;                   // LDS destinations kept per item
    const FastDiv dW = g.dW;
    const int pl_off = int(pl - lds);

    // Patch items of a tile, per thread.  The tensors have fewer than 2^31 elements (host check),
    // so byte offsets from the tensor's start fit 32 bits.
    struct Loads {
      uint32_t off[MAXI][G];    // item i, channel t of the group: byte offset within the chunk
    };
    struct Stores {
      int dst[2][MAXI][ND];     // LDS byte offset per patch buffer; the dummy area if the item does not exist
      int m0, mend;             // the tile's positions (for the rows to clear)
    };
    // Aligned items (VW pixels of one row): what does not depend on the tile.  Item id is
    // (pixel group, block of g.rb patch rows, row within the block, channel group) with the last
    // two running fastest, so that the 16 lanes an LDS store serves together write rows of one
    // pixel column: the row pitch (g.PW pixels of 48 bytes, g.PW * 3 / 2 odd) puts eight
    // consecutive rows on eight different even 16-byte bank groups and the channel group on the
    // odd ones.  (Lanes along a row, 8 pixels = 384 bytes apart, would share two bank groups.)
    int item_r[MAXI], item_dst[MAXI];
    uint32_t item_koff[MAXI];
    if constexpr (!FLAT) {
      const int rb_shift = g.rb_shift;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const int id = ptid + PT * i;
        const int cg = id & 1, q = id >> 1;
        const int q2 = q >> rb_shift;
        const int r_hi = int(dXG.div(uint32_t(q2))), xg = q2 - r_hi * XGn;
        item_r[i] = (r_hi << rb_shift) + (q & ((1 << rb_shift) - 1));
        item_dst[i] = pl_off + (item_r[i] * g.PW + g.XO + xg * VW) * PIXB + cg * 16;
        item_koff[i] = uint32_t(cg * G) * uint32_t(plane) + uint32_t(xg * VW * ESZ);
      }
    }
    auto make_items = [&](int tile_, Loads& lo, Stores& so) {
      int m0_, mend_, o0_;
      tile_range(tile_, &m0_, &mend_, &o0_);
      const TileSegs ts = tile_segs(m0_, mend_, g);
      so.m0 = m0_;
      so.mend = mend_;
      if constexpr (FLAT) {
        // Segment s contributes ceil(L / VW) items per channel group, L = pixels of its valid
        // rows; the last item of a range is moved back to end with the range (it overlaps its
        // neighbour, which is written twice with the same data) so that no load leaves the range.
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
          uint32_t off0 = 0;
          int dst[ND];
#pragma unroll
          for (int e = 0; e < ND; ++e) dst[e] = 512 + e * PIXB;   // dummy area
          bool found = false;
          int rem = ptid + PT * i, base = 0;
          for (int s_ = 0; s_ < ts.nseg; ++s_) {
            int ihlo, rows;
            seg_extent(ts, s_, g, a.Sh, a.Ph, a.Kh, &ihlo, &rows);
            const int vlo = ihlo > 0 ? ihlo : 0;
            const int vhi = ihlo + rows < a.H ? ihlo + rows : a.H;
            const int L = vhi > vlo ? (vhi - vlo) * a.W : 0;
            const int cnt = (L + VW - 1) / VW;
            if (!found && rem < 2 * cnt) {
              found = true;
              const int cg = rem >= cnt ? 1 : 0, k = rem - cg * cnt;
              const int f0 = vlo * a.W + (k * VW < L - VW ? k * VW : L - VW);
              off0 = uint32_t((int64_t(ts.n_first + s_) * a.C + cg * G) * plane + int64_t(f0) * ESZ);
#pragma unroll
              for (int e = 0; e < ND; ++e) {
                const int row = int(dW.div(uint32_t(f0 + e))), col = f0 + e - row * a.W;
                dst[e] = pl_off + ((base + row - ihlo) * g.PW + g.XO + col) * PIXB + cg * 16;
              }
            }
            rem -= 2 * cnt;
            base += rows;
          }
#pragma unroll
          for (int t = 0; t < G; ++t) lo.off[i][t] = off0 + uint32_t(t * plane);
#pragma unroll
          for (int e = 0; e < ND; ++e) {
            so.dst[0][i][e] = dst[e];
            so.dst[1][i][e] = dst[e] + (found ? pbytes : 0);
          }
        }
        return;
      } else {
        // One segment (the tile lies within one image): patch row r is input row ihlo + r.
        int ihlo1 = 0, rows1 = 0;
        if (ts.nseg == 1) seg_extent(ts, 0, g, a.Sh, a.Ph, a.Kh, &ihlo1, &rows1);
        const uint32_t img1 = uint32_t(ts.n_first) * uint32_t(a.C) * uint32_t(plane);
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
          uint32_t off0 = 0;
          bool ok = false;
          if (ts.nseg == 1) {                       // uniform
            const int ih = ihlo1 + item_r[i];
            ok = item_r[i] < rows1 && ih >= 0 && ih < a.H;
            off0 = item_koff[i] + img1 + uint32_t(ih) * uint32_t(a.W * ESZ);
          } else {
            int s_, ih;
            if (seg_of_row(ts, item_r[i], g, a.Sh, a.Ph, a.Kh, &s_, &ih) && ih >= 0 && ih < a.H) {
              ok = true;
              off0 = item_koff[i] + uint32_t(ts.n_first + s_) * uint32_t(a.C) * uint32_t(plane) +
                     uint32_t(ih) * uint32_t(a.W * ESZ);
            }
          }
          off0 = ok ? off0 : 0u;
#pragma unroll
          for (int t = 0; t < G; ++t) lo.off[i][t] = off0 + uint32_t(t) * uint32_t(plane);
          so.dst[0][i][0] = ok ? item_dst[i] : 512;            // else the dummy area (VW * 48 bytes at most)
          so.dst[1][i][0] = ok ? item_dst[i] + pbytes : 512;
        }
      }
    };
    // Rows of a tile's patch that lie outside their image (top / bottom padding) must read as
    // zeros; a row index may have held data of the previous tile, so they are cleared per tile
    // and buffer.  Data rows are overwritten in full and need no clearing.  The rows outside are
    // the first -ihlo and the last ihlo + rows - H rows of a segment: thread t clears pixel t.
    auto zero_invalid_rows = [&](const Stores& so, int buf) {
      const TileSegs ts = tile_segs(so.m0, so.mend, g);
      int base = 0;
      for (int s_ = 0; s_ < ts.nseg; ++s_) {
        int ihlo, rows;
        seg_extent(ts, s_, g, a.Sh, a.Ph, a.Kh, &ihlo, &rows);
        const int ntop = ihlo < 0 ? (-ihlo < rows ? -ihlo : rows) : 0;
        const int nbot = ihlo + rows > a.H ? (ihlo + rows - a.H < rows ? ihlo + rows - a.H : rows) : 0;
        for (int k = 0; k < ntop + nbot; ++k) {             // uniform; usually no iteration at all
          const int r = base + (k < ntop ? k : rows - nbot + (k - ntop));
          for (int x = ptid; x < g.PW; x += PT) {
            uint8_t* p = pl + buf * pbytes + (r * g.PW + x) * PIXB;
            const i32x4 z = {0, 0, 0, 0};
            *reinterpret_cast<i32x4*>(p) = z;
            *reinterpret_cast<i32x4*>(p + 16) = z;
          }
        }
        base += rows;
      }
    };
    // Weight transfers: instruction q of a chunk covers tap q / OB, rows (q % OB) * 32 .. + 31 of
    // the channel tile, which the blocked weight copy holds as 1 KB of consecutive bytes in the
    // order of the LDS block (row i / 2, swizzled position, for piece i): lane i moves piece i.
    // With static taps the per-lane byte offsets of all of them are fixed per channel tile.
    constexpr int NWI = KH > 0 ? KH * KW * OB : 0;             // weight instructions per chunk (static taps)
    struct WSrc {
      uint32_t off[KH > 0 ? NWI : OB];   // static taps: per instruction; else per 32-row block
    };
    auto make_wsrc = [&](int tile_, WSrc& w) {
      int m0_, mend_, o0_;
      tile_range(tile_, &m0_, &mend_, &o0_);
      if constexpr (KH > 0) {
#pragma unroll
        for (int k = 0; k < NWI; ++k) {
          const int tap = k / OB, b = k % OB;
          int ob = o0_ / 32 + b;
          ob = ob < n_oblk ? ob : n_oblk - 1;             // blocks past O are never stored
          w.off[k] = uint32_t(ob) * wr_blk + uint32_t(tap) * 1024u + uint32_t(lane) * 16u;
        }
      } else {
#pragma unroll
        for (int b = 0; b < OB; ++b) {
          int ob = o0_ / 32 + b;
          ob = ob < n_oblk ? ob : n_oblk - 1;
          w.off[b] = uint32_t(ob) * wr_blk + uint32_t(lane) * 16u;
        }
      }
    };
    WSrc wld;
    const uint32_t wl_addr = lds_addr_of(wl);
    // `wbase` = wr + byte offset of the chunk within a 32-channel block (scalar).
    auto issue_weights = [&](const uint8_t* wbase, int slot) {
      if constexpr (KH > 0) {
#pragma unroll
        for (int k = 0; k < NWI; ++k) lds_dma16_off(wbase, wld.off[k], wl_addr + slot * wbytes + k * 1024);
      } else {
        for (int q = 0; q < n_wq; ++q) {
          const int tap = q / OB, b = q % OB;
          uint32_t off = wld.off[0];
#pragma unroll
          for (int bb = 1; bb < OB; ++bb) off = (b == bb) ? wld.off[bb] : off;
          lds_dma16_off(wbase + int64_t(tap) * 1024, off, wl_addr + slot * wbytes + q * 1024);
        }
      }
    };

    RingReg<LB> preg[D][MAXI][G];
    Loads ld;                 // items of the tile being loaded
    Stores st_next, st;       // of the tile being loaded and of the tile being stored
    auto split_of = [&](int item) { return lg(item) & (ksplit - 1); };
    // `abase` = act + byte offset of the chunk's first channel plane (scalar).
    auto load_patch = [&](const uint8_t* abase, auto slot_) {
      constexpr int slot = decltype(slot_)::value;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
#pragma unroll
        for (int t = 0; t < G; ++t) preg[slot][i][t].load(abase + ld.off[i][t]);
      }
    };
    // Items that do not exist read valid dummy addresses and write into a 512-byte dummy area
    // at lds + 512, so that no branch separates a ring load from its use.
    auto store_patch = [&](auto slot_, auto buf_) {
      constexpr int slot = decltype(slot_)::value, buf = decltype(buf_)::value;
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        uint8_t* pb = lds + st.dst[buf][i][0];
#pragma unroll
        for (int p = 0; p < VW; ++p) {
          i32x4 v;   // pixel p: element t = channel t of the group; one byte permute per two sources
          const int boff = p * ESZ, wi = boff / 4, bk = boff % 4;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            if constexpr (ESZ == 2) {
              const uint32_t c0 = preg[slot][i][2 * d].word(wi), c1 = preg[slot][i][2 * d + 1].word(wi);
              v[d] = int32_t(__builtin_amdgcn_perm(c1, c0, bk ? 0x07060302u : 0x05040100u));
            } else {
              const uint32_t sel = uint32_t((4 + bk) << 8 | bk);
              const uint32_t t01 = __builtin_amdgcn_perm(preg[slot][i][4 * d + 1].word(wi),
                                                         preg[slot][i][4 * d].word(wi), sel);
              const uint32_t t23 = __builtin_amdgcn_perm(preg[slot][i][4 * d + 3].word(wi),
                                                         preg[slot][i][4 * d + 2].word(wi), sel);
              v[d] = int32_t(__builtin_amdgcn_perm(t23, t01, 0x05040100u));
            }
          }
          if constexpr (FLAT) *reinterpret_cast<i32x4*>(lds + st.dst[buf][i][p]) = v;
          else *reinterpret_cast<i32x4*>(pb + p * PIXB) = v;
        }
      }
    };
    // Cursors.  Past the last tile a cursor keeps its descriptors and restarts at chunk 0 of its
    // last tile: surplus loads and weight transfers re-read valid addresses and are never
    // consumed; surplus stores are skipped.
    const int step = int(gridDim.x);
    struct Cursor {
      int tile, chunk;
      const uint8_t* base;      // scalar: start of the current chunk in the tensor the cursor reads
    };
    auto act_base = [&](int item) { return act + int64_t(split_of(item)) * nchunk * chunk_bytes; };
    auto w_base = [&](int item) { return wr + int64_t(split_of(item)) * nchunk * wr_chunk; };
    Cursor lc = {tile, 0, act_base(tile)}, wc = {tile, 0, w_base(tile)};
    int w_o0;                 // channel tile the weight offsets were made for
    {
      int m0_, mend_;
      tile_range(tile, &m0_, &mend_, &w_o0);
    }
    int sc_tile = tile, sc_chunk = 0;
    auto next_load = [&]() {
      lc.base += chunk_bytes;
      if (++lc.chunk == nchunk) {
        lc.chunk = 0;
        if (lc.tile + step < n_tiles) {
          lc.tile += step;
          make_items(lc.tile, ld, st_next);
        }
        lc.base = act_base(lc.tile);
      }
    };
    auto next_weights = [&]() {
      wc.base += wr_chunk;
      if (++wc.chunk == nchunk) {
        wc.chunk = 0;
        if (wc.tile + step < n_tiles) {
          wc.tile += step;
          int m0_, mend_, o0_;
          tile_range(wc.tile, &m0_, &mend_, &o0_);
          if (o0_ != w_o0) {                        // uniform; rare: an XCD's items share channel tiles
            w_o0 = o0_;
            make_wsrc(wc.tile, wld);
          }
        }
        wc.base = w_base(wc.tile);
      }
    };
    // The store cursor enters a tile D units after the load cursor did and, in program order,
    // before the load cursor can leave it (chunks per item are a multiple of D): the load
    // cursor's store descriptors are that tile's.
    auto next_store = [&]() {
      if (++sc_chunk == nchunk) {
        sc_chunk = 0;
        sc_tile += step;
        st = st_next;
      }
    };

    if (pwave == 0) {
      // ---- weight wave: NWB - 1 units ahead of the consumers ---------------------------------
      make_wsrc(tile, wld);
      static_for<NWB - 1>([&](auto k_) {
        issue_weights(wc.base, decltype(k_)::value);
        next_weights();
      });
      clear_patch_buffers();
      wait_vmem<0>();
      lds_barrier();                                     // B0
      int wslot = 0;                                     // LDS weight buffer of the current chunk
      // The next chunk's weights must have landed at the end of a period: with three buffers
      // they were sent a whole period earlier (only this period's transfers may be outstanding),
      // with two buffers in this period.
      constexpr int kWaitWeights = (KH > 0 && NWB == 3) ? NWI : 0;
      for (; tile < n_tiles; tile += step) {
        for (int ch = 0; ch < nchunk; ++ch) {
          const int slot2 = wslot + NWB - 1 >= NWB ? wslot - 1 : wslot + NWB - 1;
          issue_weights(wc.base, slot2);
          next_weights();
          wslot = wslot + 1 >= NWB ? 0 : wslot + 1;
          wait_vmem<kWaitWeights>();
          lds_barrier();
        }
      }
      wait_vmem<0>();
      return;
    }
    // ---- patch waves: ring primed, chunk 0 of the first tile in LDS ---------------------------
    make_items(tile, ld, st_next);
    st = st_next;
    static_for<D>([&](auto d_) {
      load_patch(lc.base, d_);
      next_load();
    });
    clear_patch_buffers();
    store_patch(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});   // nothing to clear: the buffers are zero
    next_store();
    load_patch(lc.base, std::integral_constant<int, 0>{});
    next_load();
    lds_barrier();                                       // B0: chunk 0 of the first tile is ready
    static_assert(D % 2 == 0, "the patch buffer of a stored unit follows from its ring slot");

    for (; tile < n_tiles; tile += step) {
      for (int cb = 0; cb < nchunk; cb += D) {
        static_for<D>([&](auto d_) {
          constexpr int d = decltype(d_)::value;      // the consumers multiply chunk cb + d now
          constexpr int ns = (d + 1) % D;             // ring slot of the unit stored (and refilled)
          // the unit after it: registers -> LDS.  Its chunk number is cb + d + 1 (mod the chunks
          // of an item, an even number), so its patch buffer is (d + 1) % 2.
          if (sc_tile < n_tiles) {
            if (sc_chunk <= 1) zero_invalid_rows(st, sc_chunk);   // first use of this buffer by the tile
            store_patch(std::integral_constant<int, ns>{}, std::integral_constant<int, (d + 1) & 1>{});
          }
          next_store();
          load_patch(lc.base, std::integral_constant<int, ns>{});
          next_load();
          lds_barrier();
        });
      }
    }
    wait_vmem<0>();
    return;
  }

  // ===========================================================================================
  // Consumers
  // ===========================================================================================
  const int wo = wave / WP, wp = wave % WP;
  const int wgroups = (tps >> 3) / WP, wextra = (tps >> 3) % WP;
  const int wstart = 8 * (wp * wgroups + (wp < wextra ? wp : wextra));     // first position of this wave column
  const int wpv = 8 * (wgroups + (wp < wextra ? 1 : 0));                   // and how many it covers
  // A-fragment address inside a 1 KB weight block: row (lane % 32), column lane / 32, swizzled.
  const int afrag = (lane & 31) * 32 + (((lane >> 5) ^ ((((lane & 31) >> 2) ^ ((lane & 31) >> 3)) & 1)) << 4) +
                    wo * (WOT / 32) * 1024;
  clear_patch_buffers();
  lds_barrier();                                         // B0
  int wslot = 0;
  const bool vec_epi = g.HWo % 4 == 0;
  int m0, mend, o0;
  for (; tile < n_tiles; tile += gridDim.x) {
    tile_range(tile, &m0, &mend, &o0);
    const TileSegs ts = tile_segs(m0, mend, g);
    // The extents of the tile's first two segments are the same for every lane (scalar work);
    // only tiles that touch more than two images walk the segments per lane.
    int ihlo0 = 0, rows0 = 0, ihlo1 = 0, rows1 = 0;
    seg_extent(ts, 0, g, a.Sh, a.Ph, a.Kh, &ihlo0, &rows0);
    if (ts.nseg > 1) seg_extent(ts, 1, g, a.Sh, a.Ph, a.Kh, &ihlo1, &rows1);
    // Per-lane window origins in the patch, and output addresses.
    int pbase[NJ];
    uint32_t out_base[NJ];
    bool pos_ok[NJ];
#pragma unroll
    for (int n = 0; n < NJ; ++n) {
      const int m = m0 + wstart + n * 32 + (lane & 31);
      pos_ok[n] = n * 32 + (lane & 31) < wpv && m < M;
      pbase[n] = (lane >> 5) * 16;
      out_base[n] = 0;
      if (pos_ok[n]) {
        const int img = int(g.dHWo.div(uint32_t(m))), p = m - img * g.HWo;
        const int ho = int(g.dWo.div(uint32_t(p))), wo_ = p - ho * a.Wo;
        const int si = img - ts.n_first;
        int base = si ? rows0 : 0, ihlo = si ? ihlo1 : ihlo0;   // patch rows in front of this image's segment
        if (ts.nseg > 2) {                             // uniform; small planes only
          int rows = 0;
          base = 0;
          for (int s = 0; s <= si; ++s) {
            base += rows;
            seg_extent(ts, s, g, a.Sh, a.Ph, a.Kh, &ihlo, &rows);
          }
        }
        const int row = base + (ho * a.Sh - a.Ph - ihlo);
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

    // Write-back geometry of this lane (vector epilogue): its group of 4 positions is the same
    // for every channel row it writes.
    constexpr int GR = WPT / 4;                      // 4-position groups per row
    constexpr int ROWS_PER_IT = 64 / GR;
    constexpr int NIT = 32 / ROWS_PER_IT;            // write-back steps per 32-channel block
    uint8_t* stage = sl + wave * (32 * RS);
    // Results of one 32x32 block (rows = positions, columns = channels: a lane holds, for channel
    // lane % 32, four consecutive positions per group of four registers) go to the staging rows
    // [channel][position] as 16-byte stores; rows are RS = 16 (mod 256) bytes apart, so the 16
    // lanes of a store pass hit 16 different bank groups.
    auto stage_block = [&](const typename TR::accv_t& c, int n) {
      uint8_t* row = stage + (lane & 31) * RS + (n * 32 + 4 * (lane >> 5)) * 4;
      static_for<4>([&](auto gi_) {
        constexpr int gi = decltype(gi_)::value;
        const auto q = __builtin_shufflevector(c, c, 4 * gi, 4 * gi + 1, 4 * gi + 2, 4 * gi + 3);
        *reinterpret_cast<i32x4*>(row + gi * 32) = __builtin_bit_cast(i32x4, q);
      });
    };
    // bfloat16 results of planes that are multiples of 8 go out 8 positions (16 bytes) per lane:
    // half as many store instructions, and a store costs the wave a few hundred cycles of issue
    // time whatever its width.
    const bool wide = vec_epi && ksplit == 1 && a.out_dtype == GS_BF16 && g.HWo % 8 == 0 &&
                      !__is_same(typename TR::acc_t, int32_t);
    const int pgw = wide ? 8 : 4;                    // positions per lane
    const int gq = wide ? lane % (GR / 2) : lane % GR, rsub = wide ? lane / (GR / 2) : lane / GR;
    const int mm = m0 + wstart + gq * pgw;
    const bool grp_ok = gq * pgw < wpv && mm < M;
    const int gimg = int(g.dHWo.div(uint32_t(grp_ok ? mm : 0)));
    const uint32_t gbase = uint32_t(gimg) * uint32_t(a.O) * uint32_t(g.HWo) + uint32_t(mm - gimg * g.HWo);
    // Destination: the output, or with a split channel sum this split's slice of the partials
    // (raw 32-bit sums; residual, ReLU and the conversion happen when the slices are combined).
    const bool split = ksplit > 1;
    void* const outp = split ? static_cast<void*>(static_cast<int32_t*>(a.partial) +
                                                   int64_t(lg(tile) & (ksplit - 1)) * a.N * a.O * g.HWo)
                             : a.out;
    const int odt = split ? (__is_same(typename TR::acc_t, int32_t) ? GS_I32 : GS_F32) : a.out_dtype;
    const bool relu = !split && a.relu;
    const bool has_res = !split && a.residual != nullptr;
    // bfloat16 residual values are requested before the last chunk's MFMAs and land under them;
    // 32-bit residuals (twice the registers) are requested per block inside the write-back.
    const bool res_early = has_res && odt == GS_BF16;
    uint2 resv[MI][NIT];
    auto request_residual = [&]() {
      static_for<MI>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const int o = o0 + wo * WOT + m * 32 + it * ROWS_PER_IT + rsub;
          const uint32_t addr = (grp_ok && o < a.O) ? gbase + uint32_t(o) * uint32_t(g.HWo) : 0u;
          resv[m][it] = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.residual) + addr);
        }
      });
    };
    // The same for 8 positions per lane: twice the rows per step, half the steps, 16 bytes each
    // (kept in two of the 8-byte registers).
    auto request_residual_wide = [&]() {
      static_for<MI>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
#pragma unroll
        for (int it = 0; it < NIT / 2; ++it) {
          const int o = o0 + wo * WOT + m * 32 + it * (2 * ROWS_PER_IT) + rsub;
          const uint32_t addr = (grp_ok && o < a.O) ? gbase + uint32_t(o) * uint32_t(g.HWo) : 0u;
          const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.residual) + addr);
          resv[m][2 * it] = make_uint2(r.x, r.y);
          resv[m][2 * it + 1] = make_uint2(r.z, r.w);
        }
      });
    };

    for (int ch = 0; ch < nchunk; ++ch) {
      const int buf = ch & 1;
      if (ch == nchunk - 1 && vec_epi && res_early) {
        if (wide) request_residual_wide();
        else request_residual();
      }
      const uint8_t* wb = wl + wslot * wbytes + afrag;
      const uint8_t* pb = pl + buf * pbytes;
      if constexpr (KH > 0) {
        // Static taps: fragments of tap t+1 are requested before the MFMAs of tap t.
        constexpr int NT = KH * KW;
        const uint32_t wa = lds_addr_of(wb);
        const uint32_t pa = lds_addr_of(pb);
        constexpr int PD = 2;                      // taps requested ahead of the one being multiplied
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
              acc[m][n] = TR::mfma(fr[slot][MI + n], fr[slot][m], acc[m][n]);
        });
      } else {
        for (int kh = 0; kh < Kh; ++kh)
          for (int kw = 0; kw < Kw; ++kw) {
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
              for (int n = 0; n < NJ; ++n) acc[m][n] = TR::mfma(bf[n], af[m], acc[m][n]);
          }
      }
      wslot = wslot + 1 >= NWB ? 0 : wslot + 1;
      lds_barrier();
    }

    // ---- epilogue: out[(img*O + o)*HWo + p] ------------------------------------------------------
    // Each wave stages one 32-channel block of its results in its LDS region as 32-bit values and
    // writes it back 4 positions per lane.  All reads of a block are requested before the first
    // is used, the residual values were requested before the last chunk's MFMAs, and ReLU is a
    // maximum with a run-time lower bound, so the write-back is straight-line code.
    if (vec_epi) {
      const int lo_i = relu ? 0 : INT_MIN;
      // ReLU as one maximum per value with a run-time second operand: zero, or a NaN, which
      // fmaxf ignores (it returns the other operand), so that nothing changes without ReLU.
      const float lo_f = relu ? 0.0f : __builtin_nanf("");
      auto write_back = [&](auto kind_) {
        constexpr int kind = decltype(kind_)::value;   // 0: int32, 1: f32, 2: bf16
        static_for<MI>([&](auto m_) {
          constexpr int m = decltype(m_)::value;
          static_for<NJ>([&](auto n_) {
            constexpr int n = decltype(n_)::value;
            stage_block(acc[m][n], n);
          });
          i32x4 raw[NIT];
#pragma unroll
          for (int it = 0; it < NIT; ++it)
            raw[it] = *reinterpret_cast<const i32x4*>(stage + (it * ROWS_PER_IT + rsub) * RS + gq * 16);
          i32x4 res4[kind == 2 ? 1 : NIT];
          if constexpr (kind != 2) {
            if (has_res) {
#pragma unroll
              for (int it = 0; it < NIT; ++it) {
                const int o = o0 + wo * WOT + m * 32 + it * ROWS_PER_IT + rsub;
                const uint32_t addr = (grp_ok && o < a.O) ? gbase + uint32_t(o) * uint32_t(g.HWo) : 0u;
                res4[it] = *reinterpret_cast<const i32x4*>(static_cast<const int32_t*>(a.residual) + addr);
              }
            }
          }
#pragma unroll
          for (int it = 0; it < NIT; ++it) {
            const int o = o0 + wo * WOT + m * 32 + it * ROWS_PER_IT + rsub;
            const uint32_t addr = gbase + uint32_t(o) * uint32_t(g.HWo);
            const bool ok = grp_ok && o < a.O;
            if constexpr (kind == 0) {
              i32x4 r4 = raw[it];
              if (has_res) r4 += res4[it];
#pragma unroll
              for (int e = 0; e < 4; ++e) r4[e] = r4[e] > lo_i ? r4[e] : lo_i;
              if (ok) *reinterpret_cast<i32x4*>(static_cast<int32_t*>(outp) + addr) = r4;
            } else {
              float f[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) f[e] = __int_as_float(raw[it][e]);
              if constexpr (kind == 1) {
                if (has_res) {
#pragma unroll
                  for (int e = 0; e < 4; ++e) f[e] += __int_as_float(res4[it][e]);
                }
                i32x4 w4;
#pragma unroll
                for (int e = 0; e < 4; ++e) w4[e] = __float_as_int(fmaxf(f[e], lo_f));
                if (ok) *reinterpret_cast<i32x4*>(static_cast<float*>(outp) + addr) = w4;
              } else {
                if (has_res) {
                  const uint32_t qx = resv[m][it].x, qy = resv[m][it].y;
                  f[0] += __uint_as_float(qx << 16); f[1] += __uint_as_float(qx & 0xffff0000u);
                  f[2] += __uint_as_float(qy << 16); f[3] += __uint_as_float(qy & 0xffff0000u);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) f[e] = fmaxf(f[e], lo_f);
                uint2 w2;
                w2.x = pack_bf16x2(f[0], f[1]);
                w2.y = pack_bf16x2(f[2], f[3]);
                if (ok) *reinterpret_cast<uint2*>(static_cast<uint16_t*>(outp) + addr) = w2;
              }
            }
          }
        });
      };
      // bfloat16, 8 positions per lane
      auto write_back_wide = [&]() {
        constexpr int RPI = 2 * ROWS_PER_IT, NW = NIT / 2;
        static_for<MI>([&](auto m_) {
          constexpr int m = decltype(m_)::value;
          static_for<NJ>([&](auto n_) {
            constexpr int n = decltype(n_)::value;
            stage_block(acc[m][n], n);
          });
          i32x4 raw[NW][2];
#pragma unroll
          for (int it = 0; it < NW; ++it) {
            const uint8_t* src = stage + (it * RPI + rsub) * RS + gq * 32;
            raw[it][0] = *reinterpret_cast<const i32x4*>(src);
            raw[it][1] = *reinterpret_cast<const i32x4*>(src + 16);
          }
#pragma unroll
          for (int it = 0; it < NW; ++it) {
            const int o = o0 + wo * WOT + m * 32 + it * RPI + rsub;
            const uint32_t addr = gbase + uint32_t(o) * uint32_t(g.HWo);
            const bool ok = grp_ok && o < a.O;
            float f[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = __int_as_float(raw[it][e / 4][e % 4]);
            if (has_res) {
#pragma unroll
              for (int h = 0; h < 2; ++h) {
                const uint32_t qx = resv[m][2 * it + h].x, qy = resv[m][2 * it + h].y;
                f[4 * h + 0] += __uint_as_float(qx << 16); f[4 * h + 1] += __uint_as_float(qx & 0xffff0000u);
                f[4 * h + 2] += __uint_as_float(qy << 16); f[4 * h + 3] += __uint_as_float(qy & 0xffff0000u);
              }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = fmaxf(f[e], lo_f);
            i32x4 w4;
#pragma unroll
            for (int e = 0; e < 4; ++e) w4[e] = int32_t(pack_bf16x2(f[2 * e], f[2 * e + 1]));
            if (ok) *reinterpret_cast<i32x4*>(static_cast<uint16_t*>(outp) + addr) = w4;
          }
        });
      };
      if constexpr (__is_same(typename TR::acc_t, int32_t)) {
        write_back(std::integral_constant<int, 0>{});
      } else {
        if (wide) write_back_wide();
        else if (odt == GS_BF16) write_back(std::integral_constant<int, 2>{});
        else write_back(std::integral_constant<int, 1>{});
      }
    } else {
      // Planes whose size is not a multiple of four positions: the same staging, read back one
      // value per lane (lane % 32 = position, two channel rows per read) and stored one by one.
      static_for<MI>([&](auto m_) {
        constexpr int m = decltype(m_)::value;
        static_for<NJ>([&](auto n_) { stage_block(acc[m][decltype(n_)::value], decltype(n_)::value); });
        static_for<NJ>([&](auto n_) {
          constexpr int n = decltype(n_)::value;
          typename TR::acc_t val[16];
#pragma unroll
          for (int rr = 0; rr < 16; ++rr)
            val[rr] = *reinterpret_cast<const typename TR::acc_t*>(stage + (2 * rr + (lane >> 5)) * RS +
                                                                   (n * 32 + (lane & 31)) * 4);
          // The block's residual values are all requested before the first result is stored: a
          // wait for a load also waits for every store issued before it (one counter, in order),
          // so a load per result, each behind the previous store, costs a round trip per value.
          if (has_res) {
            uint32_t addr[16];
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
              const int o = o0 + wo * WOT + m * 32 + 2 * rr + (lane >> 5);
              addr[rr] = (pos_ok[n] && o < a.O) ? out_base[n] + uint32_t(o) * uint32_t(g.HWo) : 0u;
            }
            typename TR::acc_t res[16];
            if constexpr (__is_same(typename TR::acc_t, int32_t)) {
#pragma unroll
              for (int rr = 0; rr < 16; ++rr) res[rr] = static_cast<const int32_t*>(a.residual)[addr[rr]];
            } else if (odt == GS_F32) {
#pragma unroll
              for (int rr = 0; rr < 16; ++rr) res[rr] = static_cast<const float*>(a.residual)[addr[rr]];
            } else {
              uint16_t rb[16];
#pragma unroll
              for (int rr = 0; rr < 16; ++rr) rb[rr] = static_cast<const uint16_t*>(a.residual)[addr[rr]];
#pragma unroll
              for (int rr = 0; rr < 16; ++rr) res[rr] = bf16_bits_to_float(rb[rr]);
            }
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) val[rr] += res[rr];
          }
#pragma unroll
          for (int rr = 0; rr < 16; ++rr) {
            const int o = o0 + wo * WOT + m * 32 + 2 * rr + (lane >> 5);
            if (pos_ok[n] && o < a.O)
              store_result<typename TR::acc_t>(outp, nullptr, odt,
                                               out_base[n] + uint32_t(o) * uint32_t(g.HWo), val[rr], relu);
          }
        });
      });
    }
  }
}

}  // namespace gs
