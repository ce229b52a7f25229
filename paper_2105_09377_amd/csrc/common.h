// Shared device/host helpers for the gfx950 kernels: element types, conversions, MFMA traits.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "../../include/glenside.h"

namespace gs {

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;

// Compile-time loop: f(std::integral_constant<int, 0>) ... f(<N-1>).  Unlike `#pragma unroll`, which
// the optimiser may decline for large bodies, this always yields constant indices, so register
// arrays indexed by the loop variable never fall back to scratch memory.
template <int N, typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl<N>(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// Workgroup barrier that orders LDS traffic only.  `__syncthreads()` also waits for every global
// load of the wave, which would drain software prefetches that are meant to stay in flight
// across the barrier; this one waits for LDS operations alone.
__device__ __forceinline__ void lds_barrier() {
  // Written as one asm block: a compiler-level fence would also wait for every outstanding
  // global_load_lds transfer (they write LDS), which is exactly what must stay in flight.
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
// The same barrier from compiler builtins, for code whose LDS reads are ordinary loads: the
// compiler's wait-count bookkeeping sees this wait and does not repeat it (in full) later.
__device__ __forceinline__ void lds_barrier_tracked() {
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0); vmcnt and expcnt at their maxima = no wait
  __builtin_amdgcn_s_barrier();
}
// 16 bytes per lane, global -> LDS, without passing through registers: lane i of the wave lands at
// lds_base + 16 i (lds_base must be wave-uniform).  Written as asm rather than through the
// compiler builtin on purpose: the compiler orders every later LDS access after a builtin
// transfer by waiting for ALL outstanding vector-memory loads, which would also drain register
// prefetches that are meant to stay in flight.  The caller must wait for the transfer itself
// (wait_vmem) and synchronise before any wave reads the bytes.
__device__ __forceinline__ void lds_dma16(const void* gptr, uint32_t lds_base) {
  const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(base) : "memory", "m0");
}
// The same with the source given as a wave-uniform base plus a 32-bit byte offset per lane.
__device__ __forceinline__ void lds_dma16_off(const void* base, uint32_t byte_off, uint32_t lds_base) {
  const uint32_t lb = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(byte_off), "s"(base), "s"(lb) : "memory", "m0");
}
// Wait until at most N of this wave's vector-memory loads (which complete in order) are still
// outstanding.  N above the counter's range waits for more than necessary, never less.
template <int N>
__device__ __forceinline__ void wait_vmem() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N < 63 ? N : 63) : "memory");
}

// Hand-ordered LDS reads.  Left to itself the compiler emits "read fragments, wait, MFMAs" per
// K step, which puts the whole LDS latency in front of every group of MFMAs when a SIMD holds a
// single wave.  `lds_read_pinned` is an `asm volatile` read that stays where it is written, and
// `lds_wait_tied<N>(regs...)` waits until at most N LDS requests are outstanding (a wave's LDS
// requests complete in order) and makes every later use of `regs` depend on that wait, so code
// can request the fragments of step k+1, wait for those of step k only, and issue its MFMAs.
__device__ __forceinline__ void lds_read_pinned(i32x4& dst, uint32_t lds_byte_addr) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(lds_byte_addr) : "memory");
}
template <int N, int COUNT>
__device__ __forceinline__ void lds_wait_tied(i32x4* regs) {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N < 15 ? N : 15) : "memory");
#pragma unroll
  for (int i = 0; i < COUNT; ++i) asm volatile("" : "+v"(regs[i]));
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return uint32_t(uintptr_t((const __attribute__((address_space(3))) uint8_t*)p));
}

__host__ __device__ inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
__host__ __device__ inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// Division of 31-bit unsigned numbers by a run-time constant as multiply-high and shift (integer
// division is a ~40-instruction routine on this hardware).  With l = ceil(log2 d) and
// m = floor(2^(31+l) / d) + 1, floor(x / d) = (x * m) >> (31 + l) for every x < 2^31.
struct FastDiv {
  uint32_t d, mul, shift;   // shift = l - 1 applied to the high word; d == 1 is special-cased
  __host__ __device__ static FastDiv make(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;
    f.mul = d > 1 ? uint32_t(((uint64_t(1) << (31 + l)) / d) + 1) : 0;
    f.shift = l > 0 ? l - 1 : 0;
    return f;
  }
  __device__ __forceinline__ uint32_t div(uint32_t x) const {
    return d == 1 ? x : (__umulhi(x, mul) >> shift);
  }
  __device__ __forceinline__ void divmod(uint32_t x, uint32_t* q, uint32_t* r) const {
    *q = div(x);
    *r = x - *q * d;
  }
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// Two floats -> two bfloat16 (round to nearest even) packed in one dword, low half first.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__host__ __device__ inline size_t dtype_size(int dt) {
  return (dt == GS_I8 || dt == GS_F8) ? 1 : dt == GS_BF16 ? 2 : 4;
}

// bfloat16 is the upper half of an IEEE binary32.
__device__ inline float bf16_bits_to_float(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// Round to nearest, ties to even; NaN stays a quiet NaN.
__device__ inline uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// Element-type traits for the two contraction flavours.  One MFMA consumes 32 bytes of K per
// row: lanes 0-31 supply bytes [0,16), lanes 32-63 bytes [16,32) of the K step, for row/column
// (lane % 32).  The 32x32 result has column (lane % 32) and rows 8*(v/4) + 4*(lane/32) + v%4 in
// accumulator register v.
struct Bf16Traits {
  using acc_t = float;
  using accv_t = f32x16;
  static constexpr int kEsz = 2;
  static constexpr int kStep = 32;      // bytes of K per row that one MFMA consumes
  __device__ static inline accv_t mfma(const i32x4& a, const i32x4& b, const accv_t& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};

struct I8Traits {
  using acc_t = int32_t;
  using accv_t = i32x16;
  static constexpr int kEsz = 1;
  static constexpr int kStep = 32;
  __device__ static inline accv_t mfma(const i32x4& a, const i32x4& b, const accv_t& c) {
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
  }
};

// EXT: 8-bit floats (OCP e4m3).  One MFMA consumes 64 bytes of K per row: lanes 0-31 supply bytes
// [0,32), lanes 32-63 bytes [32,64) of the K step, as two 16-byte pieces each; both operands are
// cut the same way, so every byte of a row meets the byte of the same K index.  Unscaled (the
// block scales of the instruction are left at one).
typedef int32_t i32x8 __attribute__((ext_vector_type(8)));
struct Fp8Traits {
  using acc_t = float;
  using accv_t = f32x16;
  static constexpr int kEsz = 1;
  static constexpr int kStep = 64;
  __device__ static inline accv_t mfma(const i32x4* a, const i32x4* b, const accv_t& c) {
    const i32x8 x = {a[0][0], a[0][1], a[0][2], a[0][3], a[1][0], a[1][1], a[1][2], a[1][3]};
    const i32x8 y = {b[0][0], b[0][1], b[0][2], b[0][3], b[1][0], b[1][1], b[1][2], b[1][3]};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, c, 0, 0, 0, 0, 0, 0);
  }
};
// Fragments are arrays of 16-byte pieces: one piece for 32-byte K steps, two for 64-byte ones.
template <typename TR>
__device__ __forceinline__ typename TR::accv_t mfma_pieces(const i32x4* a, const i32x4* b,
                                                          const typename TR::accv_t& c) {
  if constexpr (TR::kStep == 32) return TR::mfma(a[0], b[0], c);
  else return TR::mfma(a, b, c);
}

// Epilogue shared by the contractions: optional residual, optional ReLU, store in the output
// type.  `addr` is an element offset.
// `stream`: the result is not read again soon (a large dense product): non-temporal stores keep
// it from displacing the operands in L2.
template <typename AccT>
__device__ __forceinline__ void store_result(void* out, const void* residual, int out_dtype,
                                             int64_t addr, AccT v, int relu, bool stream = false) {
  if constexpr (sizeof(AccT) == 4 && __is_same(AccT, int32_t)) {
    int32_t r = v;
    if (residual) r += static_cast<const int32_t*>(residual)[addr];
    if (relu) r = r > 0 ? r : 0;
    if (stream) __builtin_nontemporal_store(r, static_cast<int32_t*>(out) + addr);
    else static_cast<int32_t*>(out)[addr] = r;
  } else {
    float r = v;
    if (out_dtype == GS_F32) {
      if (residual) r += static_cast<const float*>(residual)[addr];
      if (relu) r = fmaxf(r, 0.0f);
      if (stream) __builtin_nontemporal_store(r, static_cast<float*>(out) + addr);
      else static_cast<float*>(out)[addr] = r;
    } else {
      if (residual) r += bf16_bits_to_float(static_cast<const uint16_t*>(residual)[addr]);
      if (relu) r = fmaxf(r, 0.0f);
      const uint16_t b = float_to_bf16_bits(r);
      if (stream) __builtin_nontemporal_store(b, static_cast<uint16_t*>(out) + addr);
      else static_cast<uint16_t*>(out)[addr] = b;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel launchers (defined in the .hip files).  All return hipError_t from the launch.
// ---------------------------------------------------------------------------------------------

struct WindowsArgs {      // generic N-d windows over the compute dims
  const void* in;
  void* out;
  int esz;                // element size in bytes
  int n_compute;          // number of windowed dims (1..4)
  int64_t outer;          // product of the access dims of `in`
  int64_t in_dim[4];      // b_i
  int64_t out_dim[4];     // b'_i
  int64_t win[4];         // w_i
  int64_t stride[4];
  int64_t pad_lo[4];
  uint32_t fill_bits;     // padded-cell value, in the low esz bytes
  int64_t out_row_stride; // elements between consecutive windows in `out` (>= prod w_i)
};
hipError_t launch_windows(const WindowsArgs& a, hipStream_t s);

struct MoveArgs {         // out[out_off + sum i_d os[d]] = in[in_off + sum i_d is[d]], 0 <= i_d < dims[d]
  const void* in;
  void* out;
  int esz;                // element size in bytes: 1, 2 or 4
  int rank;               // at most 8
  int64_t dims[8], is[8], os[8];   // extents and element strides, in the output's dimension order
  int64_t in_off, out_off;         // element offsets
};
hipError_t launch_move(const MoveArgs& a, hipStream_t s);
hipError_t launch_fill(void* out, int esz, int64_t n, uint32_t bits, hipStream_t s);

struct GemmArgs {         // C[i][j] = sum_k X[i][k] * Y[j][k]
  const void* x;          // I x K, row stride ldx elements
  const void* y;          // J x K, row stride ldy elements
  void* out;
  const void* residual;   // same addressing as out, may be null
  int in_dtype;           // GS_I8, GS_BF16 or GS_F8
  int out_dtype;
  int64_t I, J, K, ldx, ldy;
  int64_t jp;             // out element offset = (j / jp) * (I * jp) + i * jp + (j % jp)
  int relu;
  int vj;                 // set by launch_gemm: columns per lane of the vector write-back (1 = scalar)
  // Blocked evaluation (0 = off): the result is cut into blocks of bm x bn and no tile of a
  // kernel straddles a block boundary -- a workgroup's tile lies inside one block, whose K range
  // it walks from the first slice to the last.
  int64_t bm, bn;
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);

struct ConvArgs {
  const void* act;        // N x C x H x W
  const void* wr;         // repacked weights: O x (Kh*Kw) x Cpad, channel fastest, zero padded
  const void* wnat;       // fewer channels than a chunk: ((O up to 64s),(K up to 32 B)) copy, else null
  const void* wblk;       // whole chunks only (C == Cpad): the copy in 1 KB blocks (see conv_blocked_weight_offset), else null
  void* out;              // N x O x Ho x Wo
  const void* residual;
  int in_dtype, out_dtype;
  int N, C, H, W, O, Kh, Kw, Sh, Sw, Ph, Pw, Ho, Wo;
  int Cpad;               // channels per tap in `wr`
  int relu;
  int ksplit;             // 1, 2 or 4: the channel chunks are divided among ksplit workgroups
  void* partial;          // ksplit > 1: [ksplit][N*O*Ho*Wo] 32-bit partial sums
};
size_t conv_weight_workspace(int in_dtype, int O, int C, int Kh, int Kw);
// Few-channel inputs (conv_smallc.hip): a second, natural-order weight copy behind the first.
bool conv_is_smallc(int in_dtype, int C);
size_t conv_smallc_weight_bytes(int in_dtype, int O, int C, int Kh, int Kw);
size_t conv_smallc_weight_offset(int in_dtype, int O, int C, int Kh, int Kw);
// Channel counts that are whole chunks (32 bytes per tap): a third copy behind the others, cut
// into blocks of 1 KB = 32 output channels x one chunk of one tap, ordered [O / 32][chunk][tap],
// each block the exact image of the LDS block the convolution's weight transfers fill (lane i of a
// transfer moves bytes 16 i .. 16 i + 15), so that one transfer reads 1 KB of consecutive memory
// instead of 32 pieces of 32 bytes from 32 rows.  Bytes of that copy (0 if there is none) and its
// offset in the weight workspace.
size_t conv_blocked_weight_bytes(int in_dtype, int O, int C, int Kh, int Kw);
size_t conv_blocked_weight_offset(int in_dtype, int O, int C, int Kh, int Kw);
hipError_t launch_conv_smallc_pack(const void* w, void* wn, int in_dtype, int O, int C, int Kh, int Kw,
                                   hipStream_t s);
hipError_t launch_conv_smallc(const ConvArgs& a, hipStream_t s);   // reads a.wr = natural-order copy
hipError_t launch_conv_repack(const void* w, void* wr, int in_dtype, int O, int C, int Kh, int Kw,
                              hipStream_t s);
// Returns hipErrorInvalidValue if no tile configuration fits the LDS for this shape.  With
// a.ksplit > 1 and a.partial set, kernels that support it split the channel sum (Fig. 6's last
// blocking rule: partial dot products combined by reduceSum over a pair); others ignore it.
hipError_t launch_conv(const ConvArgs& a, hipStream_t s);
// Split the channel sum of this shape?  Returns 1, 2 or 4 (host heuristic: few tiles, many chunks).
int conv_pick_ksplit(int in_dtype, int N, int C, int O, int Ho, int Wo);

struct ReduceArgs {       // out[r] = reduce over `cols` contiguous values
  const void* in;
  void* out;
  int in_dtype, out_dtype, op;
  int64_t rows, cols;
  float scale;
};
hipError_t launch_reduce(const ReduceArgs& a, hipStream_t s);

struct WindowsReduceArgs {
  const void* in;
  void* out;
  int in_dtype, out_dtype, op;
  int n_compute;          // 1..3
  int64_t outer;
  int64_t in_dim[3], out_dim[3], win[3], stride[3], pad_lo[3];
  float scale;
};
hipError_t launch_windows_reduce(const WindowsReduceArgs& a, hipStream_t s);

struct DepthwiseArgs {    // out[n][c][y][x] = sum_{ky,kx} in[n][c][y*Sh-Ph+ky][x*Sw-Pw+kx] * w[c][ky][kx]
  const void* in;
  const void* w;
  void* out;
  int in_dtype, out_dtype, relu;
  int N, C, H, W, Ho, Wo, Kh, Kw, Sh, Sw, Ph, Pw;
};
hipError_t launch_depthwise(const DepthwiseArgs& a, hipStream_t s);

struct PairArgs {
  const void* a;
  const void* b;
  void* out;
  int dtype, op, relu;
  int64_t n;
};
hipError_t launch_pair_reduce(const PairArgs& a, hipStream_t s);

}  // namespace gs
