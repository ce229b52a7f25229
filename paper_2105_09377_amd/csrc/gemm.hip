// `compute dotProd (cartProd a0 a1)` as an MFMA contraction:  C[i][j] = sum_k X[i][k] * Y[j][k].
//
// Both operands are K-contiguous (each access index of a0 / a1 owns one contiguous compute
// element), which is exactly the operand order the MFMA wants, so tiles are copied global -> LDS
// with 16-byte loads and no transposition.  A workgroup of 4 or 8 waves owns a BM x BN output tile
// (the concat-on-access-dimensions blocking of Sec. 5.4); the K loop walks 128-byte slabs (the
// pair/reduceSum blocking on the compute dimension), double-buffered in LDS with the next slab's
// global loads in flight while the current one feeds the MFMAs; fragment reads run one K step
// ahead of the MFMAs and the per-slab barrier sits under the slab's last MFMAs.  The kernels are
// written in bytes: a slab row is 128 bytes = 64 bf16 or 128 int8, one MFMA eats 32 bytes of K
// per row.
//
// Two kernels:
//   gemm_nt_dma_kernel     : aligned operands, K a whole number of 32-byte MFMA steps (the last
//                            slab may be short).  Slabs go global -> LDS
//                            directly (global_load_lds, 16 bytes per lane, no register staging);
//                            because such a load writes 64 x 16 contiguous bytes, rows cannot be
//                            padded, so bank conflicts are avoided by an XOR swizzle of the
//                            16-byte columns instead.
//   gemm_nt_checked_kernel : everything else (ragged K, unaligned rows), register-staged, checked.
//
// Result element (i, j) is stored at (j / jp) * (I * jp) + i * jp + (j % jp): jp = J gives the
// plain row-major ((I, J), ()) result; jp = H'*W' with j = flattened (n, h', w') and i = o gives
// the (N, O, H', W') layout of the convolution listings, i.e. the reshape/squeeze/transpose tail
// of Fig. 5 folded into the store.  Columns j sit on the lanes, so stores are coalesced along j.
//
// Workgroups are renumbered so that each of the 8 XCDs (which have private L2 caches and receive
// consecutive workgroup ids round-robin) works on a compact block of the tile grid.
#include "common.h"

#include <stdlib.h>

#include <mutex>

namespace gs {

constexpr int kSlabBytes = 128;             // K bytes per slab row
constexpr int kRowBytes = kSlabBytes + 16;  // LDS row stride: odd multiple of 16 B, conflict-free b128
constexpr int kXcds = 8;

// Map the hardware workgroup id to a tile so that an XCD's workgroups cover a compact region:
// XCD x gets the contiguous range of "logical" ids [x*n/8, (x+1)*n/8), and logical ids walk the
// grid in column bands of `band` tile rows.
__device__ inline void tile_of_block(int64_t bid, int64_t nblocks, int64_t tiles_i, int64_t tiles_j,
                                     int64_t* ti, int64_t* tj) {
  const int64_t per = nblocks / kXcds, rem = nblocks % kXcds;
  const int64_t x = bid % kXcds, l = bid / kXcds;
  // XCDs 0..rem-1 own (per + 1) ids.
  const int64_t logical = x * per + (x < rem ? x : rem) + l;
  constexpr int64_t band = 8;
  const int64_t band_size = band * tiles_j;
  const int64_t b = logical / band_size, r = logical % band_size;
  const int64_t rows_here = (b * band + band <= tiles_i) ? band : tiles_i - b * band;
  *ti = b * band + r % rows_here;
  *tj = r / rows_here;
}

// The rows [i0, ilim) and columns [j0, jlim) a tile may touch.  Unblocked: tile (ti, tj) starts at
// (ti * BM, tj * BN) and ends with the matrix.  Blocked: tiles are counted block by block
// (ceil(bm / BM) tile rows per block row) and end with their block; a tile past the end of a
// smaller last block is empty.
__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(v)));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(uint64_t(v) >> 32));
  return int64_t((uint64_t(hi) << 32) | lo);
}
struct TileBox {
  int64_t i0, j0, ilim, jlim;
};
__host__ __device__ inline int64_t tile_count(int64_t extent, int64_t block, int tile) {
  return block > 0 ? ceil_div(extent, block) * ceil_div(block, tile) : ceil_div(extent, tile);
}
__device__ inline void tile_span(int64_t t, int64_t extent, int64_t block, int tile, int64_t* lo, int64_t* lim) {
  if (block <= 0) {
    *lo = t * tile;
    *lim = extent;
    return;
  }
  const int64_t per = ceil_div(block, tile), b = t / per;
  *lo = b * block + (t - b * per) * tile;
  const int64_t end = (b + 1) * block;
  *lim = end < extent ? end : extent;
}
template <int BM, int BN>
__device__ inline TileBox tile_box(const GemmArgs& a, int64_t ti, int64_t tj) {
  TileBox b;
  tile_span(ti, a.I, a.bm, BM, &b.i0, &b.ilim);
  tile_span(tj, a.J, a.bn, BN, &b.j0, &b.jlim);
  return b;
}

// General (checked) load of one 16-byte chunk: zero beyond the row's K bytes, byte loads when the
// rows are not 16-byte aligned.  Used by the edge/unaligned kernel only.
template <bool VEC>
__device__ inline i32x4 load_chunk_checked(const uint8_t* row_ptr, int64_t kb, int64_t Kb,
                                           bool row_ok) {
  i32x4 v = {0, 0, 0, 0};
  if (!row_ok || kb >= Kb) return v;
  const int64_t nvalid = Kb - kb;
  if (VEC && nvalid >= 16) return *reinterpret_cast<const i32x4*>(row_ptr + kb);
  uint32_t w[4] = {0, 0, 0, 0};
  for (int t = 0; t < 16; ++t)
    if (t < nvalid) w[t >> 2] |= uint32_t(row_ptr[kb + t]) << (8 * (t & 3));
  v[0] = int32_t(w[0]); v[1] = int32_t(w[1]); v[2] = int32_t(w[2]); v[3] = int32_t(w[3]);
  return v;
}

// ---------------------------------------------------------------------------------------------
// Checked kernel: any K, any alignment.  64x64 tile, 4 waves of 32x32, register-staged slabs.
// ---------------------------------------------------------------------------------------------
template <typename TR, bool VEC>
__global__ void __launch_bounds__(256) gemm_nt_checked_kernel(GemmArgs a) {
  constexpr int BM = 64, BN = 64;
  constexpr int XCH = BM * 8 / 256, YCH = BN * 8 / 256;   // 16-byte chunks per thread per slab
  constexpr int kXBytes = BM * kRowBytes, kYBytes = BN * kRowBytes;
  constexpr int kBuf = kXBytes + kYBytes;
  __shared__ __attribute__((aligned(16))) uint8_t lds[2 * kBuf];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t tiles_j = tile_count(a.J, a.bn, BN);
  const TileBox box = tile_box<BM, BN>(a, blockIdx.x / tiles_j, blockIdx.x % tiles_j);
  const int64_t i0 = box.i0, j0 = box.j0;
  if (i0 >= box.ilim || j0 >= box.jlim) return;          // past the end of a smaller last block
  const int64_t Kb = a.K * TR::kEsz;
  const uint8_t* X = static_cast<const uint8_t*>(a.x);
  const uint8_t* Y = static_cast<const uint8_t*>(a.y);
  const int64_t ldxb = a.ldx * TR::kEsz, ldyb = a.ldy * TR::kEsz;
  const int nslab = int(ceil_div(Kb, kSlabBytes));

  typename TR::accv_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0;

  i32x4 xr[XCH], yr[YCH];
  auto load_slab = [&](int slab) {
    const int64_t k0 = int64_t(slab) * kSlabBytes;
#pragma unroll
    for (int r = 0; r < XCH; ++r) {
      const int c = tid + 256 * r, row = c >> 3, kc = c & 7;
      xr[r] = load_chunk_checked<VEC>(X + (i0 + row) * ldxb, k0 + kc * 16, Kb, i0 + row < box.ilim);
    }
#pragma unroll
    for (int r = 0; r < YCH; ++r) {
      const int c = tid + 256 * r, row = c >> 3, kc = c & 7;
      yr[r] = load_chunk_checked<VEC>(Y + (j0 + row) * ldyb, k0 + kc * 16, Kb, j0 + row < box.jlim);
    }
  };
  auto store_slab = [&](int buf) {
    uint8_t* xs = lds + buf * kBuf;
    uint8_t* ys = xs + kXBytes;
#pragma unroll
    for (int r = 0; r < XCH; ++r) {
      const int c = tid + 256 * r;
      *reinterpret_cast<i32x4*>(xs + (c >> 3) * kRowBytes + (c & 7) * 16) = xr[r];
    }
#pragma unroll
    for (int r = 0; r < YCH; ++r) {
      const int c = tid + 256 * r;
      *reinterpret_cast<i32x4*>(ys + (c >> 3) * kRowBytes + (c & 7) * 16) = yr[r];
    }
  };

  load_slab(0);
  store_slab(0);
  __syncthreads();
  constexpr int KST = TR::kStep, P = KST / 32;    // bytes of K per MFMA step; 16-byte pieces per lane
  const int frag_off = (lane & 31) * kRowBytes + (lane >> 5) * (KST / 2);
  for (int slab = 0; slab < nslab; ++slab) {
    if (slab + 1 < nslab) load_slab(slab + 1);
    const uint8_t* xs = lds + (slab & 1) * kBuf + wm * 32 * kRowBytes + frag_off;
    const uint8_t* ys = lds + (slab & 1) * kBuf + kXBytes + wn * 32 * kRowBytes + frag_off;
#pragma unroll
    for (int ks = 0; ks < kSlabBytes / KST; ++ks) {
      i32x4 xf[P], yf[P];
#pragma unroll
      for (int f = 0; f < P; ++f) {
        xf[f] = *reinterpret_cast<const i32x4*>(xs + ks * KST + f * 16);
        yf[f] = *reinterpret_cast<const i32x4*>(ys + ks * KST + f * 16);
      }
      acc = mfma_pieces<TR>(xf, yf, acc);
    }
    if (slab + 1 < nslab) store_slab((slab + 1) & 1);
    __syncthreads();
  }

  const int64_t j = j0 + wn * 32 + (lane & 31);
  if (j < box.jlim) {
    const int64_t jbase = (j / a.jp) * (a.I * a.jp) + (j % a.jp);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t i = i0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (i < box.ilim)
        store_result<typename TR::acc_t>(a.out, a.residual, a.out_dtype, jbase + i * a.jp, acc[v],
                                         a.relu);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS kernel.  LDS slab layout: row r at r*128 bytes, 16-byte column c of that row at
// position c ^ ((r / 2) % 8).  One transfer instruction fills 8 rows: lane i lands at
// (row i/8, position i%8) and therefore fetches global column (i%8) ^ swizzle(row).
// ---------------------------------------------------------------------------------------------

template <typename TR, int BM, int BN, int WGM, int WGN, int SB, int NS>
__global__ void __launch_bounds__(WGM * WGN * 64) gemm_nt_dma_kernel(GemmArgs a) {
  constexpr int NW = WGM * WGN;                   // waves per workgroup
  extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
  static_assert(SB == 64 || SB == 128, "K bytes per slab row");
  static_assert(NS >= 2, "slab buffers");
  constexpr int WM = BM / WGM, WN = BN / WGN;     // wave tile
  constexpr int MI = WM / 32, NJ = WN / 32;       // 32x32 MFMA blocks per wave
  constexpr int C = SB / 16;                      // 16-byte columns per slab row
  constexpr int RPB = 256 / SB;                   // slab rows per 256 bytes (one pass over the 64 banks)
  constexpr int RPI = 1024 / SB;                  // slab rows filled by one transfer instruction
  constexpr int XQ = BM / RPI / NW, YQ = BN / RPI / NW, Q = XQ + YQ;   // transfer instructions per wave and slab
  static_assert(BM % (RPI * NW) == 0 && BN % (RPI * NW) == 0, "tile rows must split over the waves");
  constexpr int kXBytes = BM * SB, kYBytes = BN * SB;
  constexpr int KST = TR::kStep;                  // bytes of K per row and MFMA
  constexpr int P = KST / 32;                     // 16-byte pieces a lane holds per operand block
  constexpr int KS = SB / KST;                    // MFMA K steps per slab

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int64_t tiles_i = tile_count(a.I, a.bm, BM), tiles_j = tile_count(a.J, a.bn, BN);
  int64_t ti, tj;
  tile_of_block(blockIdx.x, gridDim.x, tiles_i, tiles_j, &ti, &tj);
  const TileBox box = tile_box<BM, BN>(a, ti, tj);
  // the tile origin is the same for every lane: say so, the transfers take their base in scalar registers
  const int64_t i0 = uniform64(box.i0), j0 = uniform64(box.j0);
  if (i0 >= box.ilim || j0 >= box.jlim) return;          // past the end of a smaller last block

  const uint8_t* X = static_cast<const uint8_t*>(a.x);
  const uint8_t* Y = static_cast<const uint8_t*>(a.y);
  const int64_t ldxb = a.ldx * TR::kEsz, ldyb = a.ldy * TR::kEsz;
  // K is a whole number of MFMA steps; the last slab may hold fewer than KS of them.
  const int64_t Kb = a.K * TR::kEsz;
  const int nslab = int(ceil_div(Kb, SB));
  const int tail_steps = int((Kb - int64_t(nslab - 1) * SB) / KST);   // 1..KS steps in the last slab

  // LDS slab layout: row r at r * SB bytes, its 16-byte column c at position c ^ swizzle(r) with
  // swizzle(r) = (r / RPB) % C.  The LDS has 64 four-byte banks and serves a 16-byte read 16 lanes
  // at a time; the 16 consecutive rows those lanes read in one K step then fall on 16 different
  // 16-byte bank groups.  A transfer instruction fills RPI consecutive rows: lane i lands at
  // (row i / C, position i % C) and therefore fetches global column (i % C) ^ swizzle(row).
  // Rows past the end of an operand are clamped: their products land in accumulators that are
  // never stored.
  const int lrow = lane / C;
  const int lcol = ((lane % C) ^ (((wave * RPI + lrow) / RPB) % C)) * 16;
  static_assert((NW * RPI / RPB) % C == 0, "the swizzle of a transfer's rows must not depend on q");
  // Sources are a wave-uniform 64-bit base (the tile's first row, advanced by the slab in scalar
  // registers) plus a 32-bit byte offset per lane and instruction (the host keeps 256 rows of
  // either operand below 4 GB).
  const uint8_t* const xbase = X + i0 * ldxb;
  const uint8_t* const ybase = Y + j0 * ldyb;
  uint32_t xoff[XQ], yoff[YQ];
#pragma unroll
  for (int q = 0; q < XQ; ++q) {
    int64_t row = (wave + q * NW) * RPI + lrow;
    row = i0 + row < box.ilim ? row : box.ilim - 1 - i0;
    xoff[q] = uint32_t(row * ldxb + lcol);
  }
#pragma unroll
  for (int q = 0; q < YQ; ++q) {
    int64_t row = (wave + q * NW) * RPI + lrow;
    row = j0 + row < box.jlim ? row : box.jlim - 1 - j0;
    yoff[q] = uint32_t(row * ldyb + lcol);
  }
  // In a short last slab the 16-byte columns past K are not multiplied; their lanes re-read
  // column 0 of the slab instead of running past the end of the row (and of the matrix).
  const uint32_t tail_fix = (lcol >= tail_steps * KST) ? uint32_t(lcol) : 0u;
  // LDS: [X buffers 0 .. NS-1 | Y buffers 0 .. NS-1].
  constexpr int kYBase = NS * kXBytes;
  static_assert((MI - 1) * 32 * SB < 65536 && (NJ - 1) * 32 * SB < 65536, "blocks by immediate offset");
  const uint32_t lds0 = lds_addr_of(lds);
  // Transfer instruction idx (0 .. Q - 1) of slab `slab` into buffer `buf`.
  auto issue_one = [&](int slab, int buf, auto idx_) {
    constexpr int idx = decltype(idx_)::value;
    const int64_t k0 = int64_t(slab) * SB;
    const uint32_t fix = slab == nslab - 1 ? tail_fix : 0u;
    if constexpr (idx < XQ)
      lds_dma16_off(xbase + k0, xoff[idx] - fix, lds0 + buf * kXBytes + (wave + idx * NW) * 1024);
    else
      lds_dma16_off(ybase + k0, yoff[idx - XQ] - fix,
                    lds0 + kYBase + buf * kYBytes + (wave + (idx - XQ) * NW) * 1024);
  };

  typename TR::accv_t acc[MI][NJ];
  static_for<MI>([&](auto m_) {
    static_for<NJ>([&](auto n_) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[decltype(m_)::value][decltype(n_)::value][v] = 0;
    });
  });

  // Fragment addresses in the buffer being multiplied: row (lane % 32) of a 32-row block, 16-byte
  // columns P*(2*ks + lane/32) + f for the pieces f < P, swizzled; one address register per
  // operand, K step and piece, moved to the next buffer once per slab; the 32-row blocks of a wave
  // by immediate offset.
  const uint8_t* xa[KS * P];
  const uint8_t* ya[KS * P];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int f = 0; f < P; ++f) {
      const int koff = ((P * (2 * ks + (lane >> 5)) + f) ^ (((lane & 31) / RPB) % C)) << 4;
      xa[ks * P + f] = lds + (wm * WM + (lane & 31)) * SB + koff;
      ya[ks * P + f] = lds + kYBase + (wn * WN + (lane & 31)) * SB + koff;
    }
  // The K loop is software-pipelined by hand.  Slabs s+1 .. s+NS-1 are in flight (or landed)
  // while slab s is multiplied.  The fragments of K step k + 1 are requested before the MFMAs of
  // step k are issued (two register sets; scheduling barriers keep the compiler from undoing that
  // order, its own wait-count insertion does the rest), and the workgroup barrier of a slab sits
  // in front of the MFMAs of its LAST step, so those MFMAs cover the barrier and the latency of
  // the next slab's first fragments.  At that barrier every wave has (a) received all of its
  // fragments of the current slab (lgkmcnt 0), so its buffer may be overwritten by slab s+NS, and
  // (b) waited for its own direct-to-LDS transfers of slab s+1 (vmcnt: the counter belongs to the
  // issuing wave and transfers complete in order), so after the barrier all of that slab is in LDS.
  // The fragment reads are ordinary loads, not asm: a register written by an asm read would be
  // "defined" for the compiler at once, and copies it makes of such a register (across the loop's
  // back edge, under register pressure) would run before the data has arrived.  The loop bodies
  // are free of branches (steady state and drain are separate loops) so that the accumulators
  // stay in place.
  i32x4 fr[2][(MI + NJ) * P];
  auto request = [&](auto ks_, auto slot_) {
    constexpr int ks = decltype(ks_)::value, slot = decltype(slot_)::value;
#pragma unroll
    for (int m = 0; m < MI; ++m)
#pragma unroll
      for (int f = 0; f < P; ++f)
        fr[slot][m * P + f] = *reinterpret_cast<const i32x4*>(xa[ks * P + f] + m * 32 * SB);
#pragma unroll
    for (int n = 0; n < NJ; ++n)
#pragma unroll
      for (int f = 0; f < P; ++f)
        fr[slot][(MI + n) * P + f] = *reinterpret_cast<const i32x4*>(ya[ks * P + f] + n * 32 * SB);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto multiply = [&](auto slot_) {
    constexpr int slot = decltype(slot_)::value;
#pragma unroll
    for (int m = 0; m < MI; ++m)
#pragma unroll
      for (int n = 0; n < NJ; ++n)
        acc[m][n] = mfma_pieces<TR>(&fr[slot][m * P], &fr[slot][(MI + n) * P], acc[m][n]);
    __builtin_amdgcn_sched_barrier(0);
  };
  using I0 = std::integral_constant<int, 0>;
  static_assert(KS % 2 == 0, "register sets alternate per K step and restart with every slab");
  int s = 0, buf = 0;               // slab being multiplied and its buffer (s % NS)
  // One full slab (another slab follows it).  ISSUE: slab s + NS exists and is requested.
  auto full_slab = [&](auto issue_) {
    constexpr bool ISSUE = decltype(issue_)::value;
    static_for<KS>([&](auto ks_) {
      constexpr int ks = decltype(ks_)::value;
      constexpr int slot = ks & 1;
      if constexpr (ks + 1 < KS) {
        request(std::integral_constant<int, ks + 1>{}, std::integral_constant<int, slot ^ 1>{});
        multiply(std::integral_constant<int, slot>{});
      } else {
        // slabs s+1 .. min(s+NS-1, last) are outstanding; s+1 must have landed
        if constexpr (ISSUE) wait_vmem<(NS - 2) * Q>();
        else wait_vmem<0>();
        lds_barrier_tracked();         // lgkmcnt(0), then the workgroup barrier
        const int done_buf = buf;
        const bool wrap = buf + 1 == NS;
        buf = wrap ? 0 : buf + 1;
        const int dx = wrap ? -(NS - 1) * kXBytes : kXBytes, dy = wrap ? -(NS - 1) * kYBytes : kYBytes;
#pragma unroll
        for (int k = 0; k < KS * P; ++k) {
          xa[k] += dx;
          ya[k] += dy;
        }
        request(I0{}, std::integral_constant<int, slot ^ 1>{});
        // the transfers of slab s + NS, into the buffer just drained, go between this step's MFMAs
        static_for<(MI * NJ > (ISSUE ? Q : 0) ? MI * NJ : Q)>([&](auto i_) {
          constexpr int i = decltype(i_)::value;
          if constexpr (i < MI * NJ) {
            constexpr int m = i / NJ, n = i % NJ;
            acc[m][n] = mfma_pieces<TR>(&fr[slot][m * P], &fr[slot][(MI + n) * P], acc[m][n]);
          }
          if constexpr (ISSUE && i < Q) issue_one(s + NS, done_buf, i_);
          __builtin_amdgcn_sched_barrier(0);
        });
        ++s;
      }
    });
  };

  static_for<NS>([&](auto b_) {
    if (decltype(b_)::value < nslab)
      static_for<Q>([&](auto idx_) { issue_one(decltype(b_)::value, decltype(b_)::value, idx_); });
  });
  // Arguments that only the epilogue reads are fetched here: a scalar load left pending across
  // the K loop would make every wait for LDS fragments a wait for everything (scalar loads return
  // out of order on the same counter).
  asm volatile("" ::"s"(a.relu), "s"(a.vj), "s"(a.jp), "s"(a.residual), "s"(a.out), "s"(a.out_dtype));
  if (nslab >= NS) wait_vmem<(NS - 1) * Q>();
  else wait_vmem<0>();
  lds_barrier_tracked();
  request(I0{}, I0{});
  while (s + NS < nslab) full_slab(std::true_type{});     // steady state
  while (s + 1 < nslab) full_slab(std::false_type{});     // drain: nothing left to request
  static_for<KS>([&](auto ks_) {    // last slab: 1..KS steps; its first fragments are on their way
    constexpr int ks = decltype(ks_)::value;
    constexpr int slot = ks & 1;
    if (ks < tail_steps) {                         // uniform
      if constexpr (ks + 1 < KS) {
        if (ks + 1 < tail_steps)
          request(std::integral_constant<int, ks + 1>{}, std::integral_constant<int, slot ^ 1>{});
      }
      multiply(std::integral_constant<int, slot>{});
    }
  });
  __syncthreads();   // every wave is done with the slabs: their memory becomes epilogue staging

  // Epilogue: lane holds column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4 of each block.
  // Results larger than the last-level cache are streamed past L2.
  const bool stream_out = a.I * a.J * 4 > (int64_t(128) << 20);

  // Vector write-back (a.vj = 8 or 4 consecutive columns j are contiguous and aligned in the
  // result): each wave stages one 32-row block of its results in the slab memory, which no wave
  // reads any more, as 32-bit values and writes it back a.vj columns per lane, so a store
  // instruction carries 16 (or 8) bytes per lane instead of one element.
  if (a.vj > 1) {
    constexpr int RS = WN * 4 + 16;                 // staging row stride in bytes
    static_assert(NW * 32 * RS <= NS * (kXBytes + kYBytes), "staging must fit in the slab buffers");
    uint8_t* stage = lds + wave * (32 * RS);
    const bool has_res = a.residual != nullptr;
    auto write_back = [&](auto vj_, auto kind_) {
      constexpr int VJ = decltype(vj_)::value;       // columns per lane
      constexpr int kind = decltype(kind_)::value;   // 0: int32, 1: f32, 2: bf16
      constexpr int NV = VJ / 4;                     // 16-byte pieces of 32-bit values per lane
      constexpr int LPR = WN / VJ, RPP = 64 / LPR, NP = 32 / RPP;   // lanes per row, rows per pass, passes
      const int cq = lane % LPR, rsub = lane / LPR;
      const int64_t jg = j0 + wn * WN + cq * VJ;
      const bool j_ok = jg < box.jlim;
      const int64_t jq = j_ok ? jg : 0;
      const int64_t jbase = (jq / a.jp) * (a.I * a.jp) + (jq % a.jp);
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
        i32x4 raw[NP][NV];
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
          for (int q = 0; q < NV; ++q)
            raw[p][q] = *reinterpret_cast<const i32x4*>(stage + (p * RPP + rsub) * RS + cq * VJ * 4 + q * 16);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const int64_t i = i0 + wm * WM + m * 32 + p * RPP + rsub;
          const bool ok = j_ok && i < box.ilim;
          const int64_t addr = ok ? jbase + i * a.jp : 0;
          if constexpr (kind == 2) {
            float f[VJ];
#pragma unroll
            for (int e = 0; e < VJ; ++e) f[e] = __int_as_float(raw[p][e >> 2][e & 3]);
            if (has_res) {
              uint32_t rq[VJ / 2];
              if constexpr (VJ == 8) {
                const i32x4 t = *reinterpret_cast<const i32x4*>(static_cast<const uint16_t*>(a.residual) + addr);
                rq[0] = t[0]; rq[1] = t[1]; rq[2] = t[2]; rq[3] = t[3];
              } else {
                const uint2 t = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.residual) + addr);
                rq[0] = t.x; rq[1] = t.y;
              }
#pragma unroll
              for (int e = 0; e < VJ / 2; ++e) {
                f[2 * e] += __uint_as_float(rq[e] << 16);
                f[2 * e + 1] += __uint_as_float(rq[e] & 0xffff0000u);
              }
            }
            uint32_t w[VJ / 2];
#pragma unroll
            for (int e = 0; e < VJ / 2; ++e) {
              const float lo = a.relu ? fmaxf(f[2 * e], 0.0f) : f[2 * e];
              const float hi = a.relu ? fmaxf(f[2 * e + 1], 0.0f) : f[2 * e + 1];
              w[e] = pack_bf16x2(lo, hi);
            }
            if (ok) {
              uint16_t* dst = static_cast<uint16_t*>(a.out) + addr;
              if constexpr (VJ == 8) {
                const i32x4 w4 = {int(w[0]), int(w[1]), int(w[2]), int(w[3])};
                if (stream_out) __builtin_nontemporal_store(w4, reinterpret_cast<i32x4*>(dst));
                else *reinterpret_cast<i32x4*>(dst) = w4;
              } else {
                const i32x2 w2 = {int(w[0]), int(w[1])};
                if (stream_out) __builtin_nontemporal_store(w2, reinterpret_cast<i32x2*>(dst));
                else *reinterpret_cast<i32x2*>(dst) = w2;
              }
            }
          } else {
#pragma unroll
            for (int q = 0; q < NV; ++q) {
              i32x4 r4 = raw[p][q];
              if (has_res) {
                const i32x4 t = *reinterpret_cast<const i32x4*>(static_cast<const int32_t*>(a.residual) + addr + q * 4);
                if constexpr (kind == 0) {
                  r4 += t;
                } else {
#pragma unroll
                  for (int e = 0; e < 4; ++e) r4[e] = __float_as_int(__int_as_float(r4[e]) + __int_as_float(t[e]));
                }
              }
              if (a.relu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  if constexpr (kind == 0) r4[e] = r4[e] > 0 ? r4[e] : 0;
                  else r4[e] = __float_as_int(fmaxf(__int_as_float(r4[e]), 0.0f));
                }
              }
              if (ok) {
                i32x4* dst = reinterpret_cast<i32x4*>(static_cast<int32_t*>(a.out) + addr + q * 4);
                if (stream_out) __builtin_nontemporal_store(r4, dst);
                else *dst = r4;
              }
            }
          }
        }
      });
    };
    using c8 = std::integral_constant<int, 8>;
    using c4 = std::integral_constant<int, 4>;
    if constexpr (__is_same(typename TR::acc_t, int32_t)) {
      if (a.vj == 8) write_back(c8{}, std::integral_constant<int, 0>{});
      else write_back(c4{}, std::integral_constant<int, 0>{});
    } else if (a.out_dtype == GS_BF16) {
      if (a.vj == 8) write_back(c8{}, std::integral_constant<int, 2>{});
      else write_back(c4{}, std::integral_constant<int, 2>{});
    } else {
      if (a.vj == 8) write_back(c8{}, std::integral_constant<int, 1>{});
      else write_back(c4{}, std::integral_constant<int, 1>{});
    }
    return;
  }
  static_for<NJ>([&](auto n_) {
    constexpr int n = decltype(n_)::value;
    const int64_t j = j0 + wn * WN + n * 32 + (lane & 31);
    const bool j_ok = j < box.jlim;
    const int64_t jbase = (j / a.jp) * (a.I * a.jp) + (j % a.jp);
    static_for<MI>([&](auto m_) {
      constexpr int m = decltype(m_)::value;
      const int64_t ibase = i0 + wm * WM + m * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int64_t i = ibase + 8 * (v >> 2) + (v & 3);
        if (j_ok && i < box.ilim)
          store_result<typename TR::acc_t>(a.out, a.residual, a.out_dtype, jbase + i * a.jp,
                                           acc[m][n][v], a.relu, stream_out);
      }
    });
  });
}

template <typename TR, int BM, int BN, int WGM, int WGN, int SB, int NS>
static hipError_t launch_dma(const GemmArgs& a, hipStream_t s) {
  constexpr int lds_bytes = NS * (BM + BN) * SB;
  static_assert(lds_bytes <= 160 * 1024, "LDS of a compute unit");
  auto kern = gemm_nt_dma_kernel<TR, BM, BN, WGM, WGN, SB, NS>;
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [&]() {
    attr_status = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int64_t tiles = tile_count(a.I, a.bm, BM) * tile_count(a.J, a.bn, BN);
  if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3(unsigned(tiles)), dim3(WGM * WGN * 64), lds_bytes, s, a);
  return hipGetLastError();
}

// Tile choice of the direct-to-LDS kernel.
template <typename TR>
static hipError_t launch_dma_tiles(const GemmArgs& a, hipStream_t s) {
  const int64_t t128 = tile_count(a.I, a.bm, 128) * tile_count(a.J, a.bn, 128);
  const int64_t t256 = tile_count(a.I, a.bm, 256) * tile_count(a.J, a.bn, 256);
  // extent a tile can fill: the block when the result is cut into blocks
  const int64_t fi = a.bm > 0 && a.bm < a.I ? a.bm : a.I, fj = a.bn > 0 && a.bn < a.J ? a.bn : a.J;
  if (t256 >= 256 && fi >= 256 && fj >= 256) return launch_dma<TR, 256, 256, 2, 4, 128, 2>(a, s);
  // few rows (a convolution's output channels against many positions): tiles 64 rows tall
  if (a.I <= 64 && ceil_div(fj, 256) * ceil_div(a.J, fj) >= 192) return launch_dma<TR, 64, 256, 1, 4, 128, 2>(a, s);
  if (t128 >= 192 && (a.bm <= 0 || fi >= 128) && (a.bn <= 0 || fj >= 128)) return launch_dma<TR, 128, 128, 2, 2, 128, 2>(a, s);
  return launch_dma<TR, 64, 64, 2, 2, 128, 2>(a, s);
}

template <typename TR>
static hipError_t launch_t(const GemmArgs& a, hipStream_t s) {
  const bool vec = (a.ldx * TR::kEsz) % 16 == 0 && (a.ldy * TR::kEsz) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(a.x) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(a.y) % 16 == 0;
  // whole MFMA steps, and 256 rows of either operand within reach of a 32-bit byte offset
  const bool dma = vec && a.K > 0 && (a.K * TR::kEsz) % TR::kStep == 0 && a.ldx * TR::kEsz < (int64_t(1) << 23) &&
                   a.ldy * TR::kEsz < (int64_t(1) << 23);
  if (dma) {
    // Columns per lane of the vector write-back: groups of vj columns must not straddle a jp
    // boundary or the end of the result, and must be 16-byte (8-byte for 4 bfloat16) aligned.
    GemmArgs v = a;
    v.vj = 1;
    const size_t osz = dtype_size(a.out_dtype);
    for (int cand = 8; cand >= 4 && v.vj == 1; cand /= 2) {
      const size_t al = cand * osz < 16 ? cand * osz : 16;
      if (a.jp % cand == 0 && a.J % cand == 0 && a.bn % cand == 0 && reinterpret_cast<uintptr_t>(a.out) % al == 0 &&
          reinterpret_cast<uintptr_t>(a.residual) % al == 0)
        v.vj = cand;
    }
    return launch_dma_tiles<TR>(v, s);
  }
  const int64_t tiles = tile_count(a.I, a.bm, 64) * tile_count(a.J, a.bn, 64);
  if (tiles > 0x7fffffff) return hipErrorInvalidValue;
  if (vec)
    hipLaunchKernelGGL((gemm_nt_checked_kernel<TR, true>), dim3(unsigned(tiles)), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((gemm_nt_checked_kernel<TR, false>), dim3(unsigned(tiles)), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  if (a.I == 0 || a.J == 0) return hipSuccess;
  if (ceil_div(a.I, 64) * ceil_div(a.J, 64) > 0x7fffffff) return hipErrorInvalidValue;
  if (a.in_dtype == GS_I8) return launch_t<I8Traits>(a, s);
  if (a.in_dtype == GS_F8) return launch_t<Fp8Traits>(a, s);
  return launch_t<Bf16Traits>(a, s);
}

}  // namespace gs
