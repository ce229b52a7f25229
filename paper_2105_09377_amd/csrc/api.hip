// C ABI of the library: host-side validation of the access-pattern shape rules (Table 1, Table 2,
// Fig. 2, Fig. 5) and dispatch to the kernels.  Everything is checked before anything is
// launched, so every error path can be exercised on a host without a GPU.
#include "common.h"

#include <limits.h>
#include <string.h>

#include <mutex>

using namespace gs;

namespace {

int64_t prod(const int64_t* v, int n) {
  int64_t p = 1;
  for (int i = 0; i < n; ++i) p *= v[i];
  return p;
}

int64_t numel(const gs_ap* a) { return prod(a->shape, a->rank); }
int64_t access_numel(const gs_ap* a) { return prod(a->shape, a->n_access); }
int64_t compute_numel(const gs_ap* a) { return prod(a->shape + a->n_access, a->rank - a->n_access); }

// Structural check of one access pattern.  `need_data` = the kernels will dereference it.
int check_ap(const gs_ap* a, bool need_data) {
  if (!a) return GS_ERR_NULL;
  if (a->rank < 0 || a->rank > GS_MAX_RANK) return GS_ERR_RANK;
  if (a->n_access < 0 || a->n_access > a->rank) return GS_ERR_RANK;
  if (a->dtype < GS_I8 || a->dtype > GS_F8) return GS_ERR_DTYPE;
  if (a->reserved != 0) return GS_ERR_UNSUPPORTED;
  int64_t n = 1;
  for (int i = 0; i < a->rank; ++i) {
    if (a->shape[i] < 0) return GS_ERR_SHAPE;
    if (a->shape[i] > 0 && n > (int64_t(1) << 40) / a->shape[i]) return GS_ERR_UNSUPPORTED;
    n *= a->shape[i];
  }
  if (need_data && n > 0) {
    if (!a->data) return GS_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(a->data) % 16) return GS_ERR_UNSUPPORTED;
  }
  return GS_OK;
}

bool same_shape(const gs_ap* a, const gs_ap* b) {
  if (a->rank != b->rank) return false;
  for (int i = 0; i < a->rank; ++i)
    if (a->shape[i] != b->shape[i]) return false;
  return true;
}

// Do the bytes of two access patterns overlap?  (Empty tensors overlap nothing.)
bool overlaps(const gs_ap* a, const gs_ap* b) {
  const uint64_t na = uint64_t(numel(a)) * dtype_size(a->dtype), nb = uint64_t(numel(b)) * dtype_size(b->dtype);
  if (na == 0 || nb == 0) return false;
  const uintptr_t pa = reinterpret_cast<uintptr_t>(a->data), pb = reinterpret_cast<uintptr_t>(b->data);
  return pa < pb + nb && pb < pa + na;
}

uint32_t lowest_bits(int dtype) {
  switch (dtype) {
    case GS_I8: return 0x80u;
    case GS_I32: return 0x80000000u;
    case GS_BF16: return 0xff80u;       // -inf
    case GS_F8: return 0xfeu;           // -448: e4m3 has no infinity
    default: return 0xff800000u;        // -inf
  }
}

int launch_status(hipError_t e) {
  if (e == hipSuccess) return GS_OK;
  if (e == hipErrorInvalidValue) return GS_ERR_UNSUPPORTED;
  return GS_ERR_LAUNCH;
}

// Shape rule of `windows` with optional padding.  Fills dims of the result.
int windows_shape(const gs_ap* in, const int64_t* window, const int64_t* stride,
                  const int64_t* pad_lo, const int64_t* pad_hi, gs_ap* out) {
  int st = check_ap(in, false);
  if (st) return st;
  if (!window || !stride || !out) return GS_ERR_NULL;
  const int nc = in->rank - in->n_access;
  if (nc < 1) return GS_ERR_RANK;
  if (in->rank + nc > GS_MAX_RANK) return GS_ERR_RANK;
  out->dtype = in->dtype;
  out->rank = in->rank + nc;
  out->n_access = in->n_access + nc;
  out->reserved = 0;
  for (int i = 0; i < in->n_access; ++i) out->shape[i] = in->shape[i];
  for (int d = 0; d < nc; ++d) {
    const int64_t lo = pad_lo ? pad_lo[d] : 0, hi = pad_hi ? pad_hi[d] : 0;
    const int64_t b = in->shape[in->n_access + d] + lo + hi;
    if (lo < 0 || hi < 0 || window[d] < 1 || stride[d] < 1 || window[d] > b) return GS_ERR_SHAPE;
    out->shape[in->n_access + d] = ceil_div(b - (window[d] - 1), stride[d]);
    out->shape[in->n_access + nc + d] = window[d];
  }
  return GS_OK;
}

struct ConvShape {
  int N, C, H, W, O, Kh, Kw, Sh, Sw, Ph, Pw, Ho, Wo;
};

int conv_shape(const gs_ap* act, const gs_ap* w, const int64_t* stride, const int64_t* pad,
               ConvShape* cs) {
  int st = check_ap(act, false);
  if (st) return st;
  st = check_ap(w, false);
  if (st) return st;
  if (!stride || !pad) return GS_ERR_NULL;
  if (act->rank != 4 || act->n_access != 1 || w->rank != 4 || w->n_access != 1) return GS_ERR_RANK;
  if (act->dtype != w->dtype) return GS_ERR_DTYPE;
  if (act->dtype != GS_I8 && act->dtype != GS_BF16) return GS_ERR_DTYPE;
  for (int i = 0; i < 4; ++i)
    if (act->shape[i] > INT_MAX / 4 || w->shape[i] > INT_MAX / 4) return GS_ERR_UNSUPPORTED;
  if (act->shape[1] != w->shape[1]) return GS_ERR_SHAPE;   // window covers all C channels
  if (stride[0] < 1 || stride[1] < 1 || pad[0] < 0 || pad[1] < 0) return GS_ERR_SHAPE;
  if (stride[0] > 64 || stride[1] > 64 || pad[0] > 64 || pad[1] > 64) return GS_ERR_UNSUPPORTED;
  cs->N = int(act->shape[0]); cs->C = int(act->shape[1]);
  cs->H = int(act->shape[2]); cs->W = int(act->shape[3]);
  cs->O = int(w->shape[0]); cs->Kh = int(w->shape[2]); cs->Kw = int(w->shape[3]);
  cs->Sh = int(stride[0]); cs->Sw = int(stride[1]); cs->Ph = int(pad[0]); cs->Pw = int(pad[1]);
  if (cs->C < 1 || cs->Kh < 1 || cs->Kw < 1) return GS_ERR_SHAPE;
  if (cs->Kh > cs->H + 2 * cs->Ph || cs->Kw > cs->W + 2 * cs->Pw) return GS_ERR_SHAPE;
  cs->Ho = (cs->H + 2 * cs->Ph - cs->Kh) / cs->Sh + 1;
  cs->Wo = (cs->W + 2 * cs->Pw - cs->Kw) / cs->Sw + 1;
  if (int64_t(cs->N) * cs->O * cs->Ho * cs->Wo >= (int64_t(1) << 31)) return GS_ERR_UNSUPPORTED;
  if (int64_t(cs->N) * cs->C * cs->H * cs->W >= (int64_t(1) << 31)) return GS_ERR_UNSUPPORTED;
  return GS_OK;
}

int conv_check_io(const gs_ap* act, const gs_ap* w, const gs_ap* residual, int actfn,
                  const gs_ap* out, const ConvShape& cs) {
  int st = check_ap(act, true);
  if (st) return st;
  st = check_ap(w, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (actfn != GS_ACT_NONE && actfn != GS_ACT_RELU) return GS_ERR_UNSUPPORTED;
  if (out->rank != 4 || out->n_access != 4) return GS_ERR_RANK;
  const int64_t want[4] = {cs.N, cs.O, cs.Ho, cs.Wo};
  for (int i = 0; i < 4; ++i)
    if (out->shape[i] != want[i]) return GS_ERR_SHAPE;
  if (act->dtype == GS_I8 ? out->dtype != GS_I32
                          : (out->dtype != GS_F32 && out->dtype != GS_BF16))
    return GS_ERR_DTYPE;
  if (residual) {
    st = check_ap(residual, true);
    if (st) return st;
    if (!same_shape(residual, out)) return GS_ERR_SHAPE;
    if (residual->dtype != out->dtype) return GS_ERR_DTYPE;
  }
  return GS_OK;
}

// Row stride of the im2col matrix (and of the padded weight matrix): K rounded up to the 32-byte
// K step of the dense kernel.  Columns K..ld are zeros in both operands, so the contraction may
// run over ld columns and take the direct-to-LDS path.
int64_t im2col_ld(int dtype, int64_t K) { return round_up(K, 32 / int64_t(dtype_size(dtype))); }

}  // namespace

extern "C" {

const char* glenside_status_string(int status) {
  switch (status) {
    case GS_OK: return "ok";
    case GS_ERR_NULL: return "null pointer";
    case GS_ERR_RANK: return "rank or access split does not fit the operation";
    case GS_ERR_SHAPE: return "shape rule violated";
    case GS_ERR_DTYPE: return "element types do not fit the operation";
    case GS_ERR_UNSUPPORTED: return "valid program outside what the kernels cover";
    case GS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GS_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

int glenside_windows_out_shape(const gs_ap* in, const int64_t* window, const int64_t* stride,
                               const int64_t* pad_lo, const int64_t* pad_hi, gs_ap* out) {
  return windows_shape(in, window, stride, pad_lo, pad_hi, out);
}

int glenside_access_windows(const gs_ap* in, const int64_t* window, const int64_t* stride,
                            const int64_t* pad_lo, const int64_t* pad_hi, int pad_mode,
                            gs_ap* out, void* stream) {
  gs_ap want;
  int st = windows_shape(in, window, stride, pad_lo, pad_hi, &want);
  if (st) return st;
  if (pad_mode != GS_PAD_ZERO && pad_mode != GS_PAD_LOWEST) return GS_ERR_UNSUPPORTED;
  st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (out->rank != want.rank || out->n_access != want.n_access) return GS_ERR_RANK;
  if (!same_shape(out, &want)) return GS_ERR_SHAPE;
  if (out->dtype != in->dtype) return GS_ERR_DTYPE;
  const int nc = in->rank - in->n_access;
  if (nc > 4) return GS_ERR_UNSUPPORTED;
  WindowsArgs a;
  memset(&a, 0, sizeof(a));
  a.in = in->data;
  a.out = out->data;
  a.esz = int(dtype_size(in->dtype));
  a.n_compute = nc;
  a.outer = access_numel(in);
  int64_t k = 1;
  for (int d = 0; d < nc; ++d) {
    a.in_dim[d] = in->shape[in->n_access + d];
    a.out_dim[d] = want.shape[in->n_access + d];
    a.win[d] = window[d];
    a.stride[d] = stride[d];
    a.pad_lo[d] = pad_lo ? pad_lo[d] : 0;
    k *= window[d];
  }
  a.fill_bits = pad_mode == GS_PAD_LOWEST ? lowest_bits(in->dtype) : 0u;
  a.out_row_stride = k;
  return launch_status(launch_windows(a, static_cast<hipStream_t>(stream)));
}

int glenside_cartesian_dot(const gs_ap* a0, const gs_ap* a1, gs_ap* out, int act, void* workspace,
                           size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  int st = check_ap(a0, true);
  if (st) return st;
  st = check_ap(a1, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (act != GS_ACT_NONE && act != GS_ACT_RELU) return GS_ERR_UNSUPPORTED;
  // cartProd: compute shapes must be equal (Table 1).
  const int nc0 = a0->rank - a0->n_access, nc1 = a1->rank - a1->n_access;
  if (nc0 != nc1) return GS_ERR_SHAPE;
  for (int d = 0; d < nc0; ++d)
    if (a0->shape[a0->n_access + d] != a1->shape[a1->n_access + d]) return GS_ERR_SHAPE;
  // Result ((m.., n..), ()).
  if (out->rank != a0->n_access + a1->n_access || out->n_access != out->rank) return GS_ERR_RANK;
  for (int d = 0; d < a0->n_access; ++d)
    if (out->shape[d] != a0->shape[d]) return GS_ERR_SHAPE;
  for (int d = 0; d < a1->n_access; ++d)
    if (out->shape[a0->n_access + d] != a1->shape[d]) return GS_ERR_SHAPE;
  if (a0->dtype != a1->dtype) return GS_ERR_DTYPE;
  if (a0->dtype == GS_I8) {
    if (out->dtype != GS_I32) return GS_ERR_DTYPE;
  } else if (a0->dtype == GS_BF16 || a0->dtype == GS_F8) {
    if (out->dtype != GS_F32 && out->dtype != GS_BF16) return GS_ERR_DTYPE;
  } else {
    return GS_ERR_DTYPE;
  }
  GemmArgs g{};
  memset(&g, 0, sizeof(g));
  g.x = a0->data;
  g.y = a1->data;
  g.out = out->data;
  g.in_dtype = a0->dtype;
  g.out_dtype = out->dtype;
  g.I = access_numel(a0);
  g.J = access_numel(a1);
  g.K = compute_numel(a0);
  g.ldx = g.ldy = g.K;
  g.jp = g.J > 0 ? g.J : 1;
  g.relu = act == GS_ACT_RELU;
  return launch_status(launch_gemm(g, static_cast<hipStream_t>(stream)));
}

int glenside_cartesian_dot_blocked(const gs_ap* a0, const gs_ap* a1, int64_t tile_m, int64_t tile_n,
                                   int64_t tile_k, gs_ap* out, void* stream) {
  int st = check_ap(a0, true);
  if (st) return st;
  st = check_ap(a1, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  // The blocked form is stated for matrices: a0 ((M),(K)), a1 ((N),(K)), out ((M,N),()).
  if (a0->rank != 2 || a0->n_access != 1 || a1->rank != 2 || a1->n_access != 1) return GS_ERR_RANK;
  if (out->rank != 2 || out->n_access != 2) return GS_ERR_RANK;
  if (a0->shape[1] != a1->shape[1]) return GS_ERR_SHAPE;
  if (out->shape[0] != a0->shape[0] || out->shape[1] != a1->shape[0]) return GS_ERR_SHAPE;
  if (tile_m < 1 || tile_n < 1 || tile_k < 1) return GS_ERR_SHAPE;
  if (a0->dtype != a1->dtype) return GS_ERR_DTYPE;
  // Partial sums of the K blocks are folded in the result, which therefore has the accumulator's type.
  if (a0->dtype == GS_I8) {
    if (out->dtype != GS_I32) return GS_ERR_DTYPE;
  } else if (a0->dtype == GS_BF16 || a0->dtype == GS_F8) {
    if (out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else {
    return GS_ERR_DTYPE;
  }
  const int64_t M = a0->shape[0], N = a1->shape[0], K = a0->shape[1];
  if (M == 0 || N == 0) return GS_OK;
  const size_t esz = dtype_size(a0->dtype);
  // K slices that are whole 128-byte slabs of the contraction kernels (or a single slice): ONE
  // launch.  The result is cut into tile_m x tile_n blocks, every workgroup's tile lies inside one
  // block and walks that block's K slices in order, folding them in its accumulators (the
  // reduceSum (pair acc part) chain of Fig. 7, left to right).
  if (tile_k >= K || (tile_k * int64_t(esz)) % 128 == 0) {
    GemmArgs g{};
    memset(&g, 0, sizeof(g));
    g.x = a0->data;
    g.y = a1->data;
    g.out = out->data;
    g.in_dtype = a0->dtype;
    g.out_dtype = out->dtype;
    g.I = M;
    g.J = N;
    g.K = K;
    g.ldx = g.ldy = K;
    g.jp = N;
    g.bm = tile_m < M ? tile_m : 0;
    g.bn = tile_n < N ? tile_n : 0;
    return launch_status(launch_gemm(g, static_cast<hipStream_t>(stream)));
  }
  // Other slice lengths: one launch per (block, K slice) on views of the operands.
  const int64_t launches = ceil_div(M, tile_m) * ceil_div(N, tile_n) * (K > 0 ? ceil_div(K, tile_k) : 1);
  if (launches > 65536) return GS_ERR_UNSUPPORTED;
  for (int64_t m0 = 0; m0 < M; m0 += tile_m)
    for (int64_t n0 = 0; n0 < N; n0 += tile_n) {
      // dotProd over (slice a0 [m0,m1) x [k0,k1)) x (slice a1 [n0,n1) x [k0,k1)); the K blocks are
      // folded left to right as reduceSum (pair acc part), i.e. added to the block already stored.
      int64_t k0 = 0;
      do {
        GemmArgs g{};
        memset(&g, 0, sizeof(g));
        g.x = static_cast<const uint8_t*>(a0->data) + (m0 * K + k0) * esz;
        g.y = static_cast<const uint8_t*>(a1->data) + (n0 * K + k0) * esz;
        g.out = static_cast<uint8_t*>(out->data) + (m0 * N + n0) * 4;
        g.residual = k0 > 0 ? g.out : nullptr;
        g.in_dtype = a0->dtype;
        g.out_dtype = out->dtype;
        g.I = M - m0 < tile_m ? M - m0 : tile_m;
        g.J = N - n0 < tile_n ? N - n0 : tile_n;
        g.K = K - k0 < tile_k ? K - k0 : tile_k;
        g.ldx = g.ldy = K;
        g.jp = N;                         // rows of the block are N apart in the result
        st = launch_status(launch_gemm(g, static_cast<hipStream_t>(stream)));
        if (st) return st;
        k0 += tile_k;
      } while (k0 < K);
    }
  return GS_OK;
}

size_t glenside_conv2d_direct_workspace(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                                        const int64_t pad[2]) {
  ConvShape cs;
  if (conv_shape(act, w, stride, pad, &cs)) return 0;
  const int64_t wbytes = round_up(int64_t(conv_weight_workspace(act->dtype, cs.O, cs.C, cs.Kh, cs.Kw)), 256) + 256;
  const int ks = conv_pick_ksplit(act->dtype, cs.N, cs.C, cs.O, cs.Ho, cs.Wo);
  const int64_t scratch = ks > 1 ? int64_t(ks) * cs.N * cs.O * cs.Ho * cs.Wo * 4 : 0;
  return size_t(wbytes + scratch);
}

size_t glenside_conv2d_im2col_workspace(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                                        const int64_t pad[2]) {
  ConvShape cs;
  if (conv_shape(act, w, stride, pad, &cs)) return 0;
  const int64_t esz = int64_t(dtype_size(act->dtype));
  const int64_t K = int64_t(cs.C) * cs.Kh * cs.Kw, ld = im2col_ld(act->dtype, K);
  const int64_t M = int64_t(cs.N) * cs.Ho * cs.Wo;
  return size_t(round_up(M * ld * esz, 256) + round_up(int64_t(cs.O) * ld * esz, 256) + 256);
}

int glenside_conv2d_pack_weights(const gs_ap* w, void* packed, size_t packed_bytes, void* stream) {
  int st = check_ap(w, true);
  if (st) return st;
  if (w->rank != 4 || w->n_access != 1) return GS_ERR_RANK;
  if (w->dtype != GS_I8 && w->dtype != GS_BF16) return GS_ERR_DTYPE;
  for (int i = 0; i < 4; ++i)
    if (w->shape[i] > INT_MAX / 4) return GS_ERR_UNSUPPORTED;
  if (w->shape[1] < 1 || w->shape[2] < 1 || w->shape[3] < 1) return GS_ERR_SHAPE;
  const int O = int(w->shape[0]), C = int(w->shape[1]), Kh = int(w->shape[2]), Kw = int(w->shape[3]);
  const size_t need = size_t(round_up(int64_t(conv_weight_workspace(w->dtype, O, C, Kh, Kw)), 256)) + 256;
  if (!packed || packed_bytes < need || reinterpret_cast<uintptr_t>(packed) % 16)
    return GS_ERR_WORKSPACE;
  return launch_status(launch_conv_repack(w->data, packed, w->dtype, O, C, Kh, Kw,
                                          static_cast<hipStream_t>(stream)));
}

int glenside_conv2d_direct_packed(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                                  const int64_t pad[2], const gs_ap* residual, int actfn,
                                  gs_ap* out, void* packed, size_t packed_bytes,
                                  void* stream) {
  ConvShape cs;
  int st = conv_shape(act, w, stride, pad, &cs);
  if (st) return st;
  gs_ap wshape = *w;            // the packed form carries the data; only the shape is used
  wshape.data = packed;
  st = conv_check_io(act, &wshape, residual, actfn, out, cs);
  if (st) return st;
  // The packed weights must be there; the scratch behind them (split channel sums) is optional.
  const size_t wneed = size_t(round_up(int64_t(conv_weight_workspace(act->dtype, cs.O, cs.C, cs.Kh, cs.Kw)), 256)) + 256;
  const size_t need = glenside_conv2d_direct_workspace(act, w, stride, pad);
  if (!packed || packed_bytes < wneed || reinterpret_cast<uintptr_t>(packed) % 16)
    return GS_ERR_WORKSPACE;
  ConvArgs a;
  memset(&a, 0, sizeof(a));
  a.ksplit = 1;
  if (need > wneed && packed_bytes >= need) {
    a.ksplit = conv_pick_ksplit(act->dtype, cs.N, cs.C, cs.O, cs.Ho, cs.Wo);
    a.partial = static_cast<uint8_t*>(packed) + wneed;
  }
  a.act = act->data;
  a.wr = packed;
  a.out = out->data;
  a.residual = residual ? residual->data : nullptr;
  a.in_dtype = act->dtype;
  a.out_dtype = out->dtype;
  a.N = cs.N; a.C = cs.C; a.H = cs.H; a.W = cs.W; a.O = cs.O; a.Kh = cs.Kh; a.Kw = cs.Kw;
  a.Sh = cs.Sh; a.Sw = cs.Sw; a.Ph = cs.Ph; a.Pw = cs.Pw; a.Ho = cs.Ho; a.Wo = cs.Wo;
  a.Cpad = int(round_up(cs.C, act->dtype == GS_I8 ? 32 : 16));
  if (conv_is_smallc(act->dtype, cs.C))
    a.wnat = static_cast<const uint8_t*>(packed) + conv_smallc_weight_offset(act->dtype, cs.O, cs.C, cs.Kh, cs.Kw);
  if (conv_blocked_weight_bytes(act->dtype, cs.O, cs.C, cs.Kh, cs.Kw))
    a.wblk = static_cast<const uint8_t*>(packed) + conv_blocked_weight_offset(act->dtype, cs.O, cs.C, cs.Kh, cs.Kw);
  a.relu = actfn == GS_ACT_RELU;
  return launch_status(launch_conv(a, static_cast<hipStream_t>(stream)));
}

int glenside_conv2d_direct(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                           const int64_t pad[2], const gs_ap* residual, int actfn, gs_ap* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  // Validate everything first so that a bad call launches nothing, then run the two halves.
  ConvShape cs;
  int st = conv_shape(act, w, stride, pad, &cs);
  if (st) return st;
  st = conv_check_io(act, w, residual, actfn, out, cs);
  if (st) return st;
  const size_t need = glenside_conv2d_direct_workspace(act, w, stride, pad);
  if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16)
    return GS_ERR_WORKSPACE;
  st = glenside_conv2d_pack_weights(w, workspace, workspace_bytes, stream);
  if (st) return st;
  return glenside_conv2d_direct_packed(act, w, stride, pad, residual, actfn, out, workspace,
                                       workspace_bytes, stream);
}

}  // extern "C"

namespace {

// Scratch of glenside_conv2d_direct_static: the packed weights and the partial sums of a split
// channel sum, in device memory that belongs to the loaded library (one copy per GPU, held until
// the process ends) instead of memory the caller or the library allocates.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void* scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once

// Device address of the array on the current GPU.  The array's name is only a host-side handle:
// kernels and copies get this pointer.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GS_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GS_ERR_LAUNCH;
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return GS_OK;
}

}  // namespace

extern "C" {

size_t glenside_conv2d_direct_static_limit(void) { return kStaticScratchBytes; }

int glenside_conv2d_direct_static(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                                  const int64_t pad[2], const gs_ap* residual, int actfn,
                                  gs_ap* out, void* stream) {
  ConvShape cs;
  int st = conv_shape(act, w, stride, pad, &cs);
  if (st) return st;
  st = conv_check_io(act, w, residual, actfn, out, cs);
  if (st) return st;
  if (glenside_conv2d_direct_workspace(act, w, stride, pad) > kStaticScratchBytes) return GS_ERR_WORKSPACE;
  void* ws = nullptr;
  st = static_scratch(&ws);
  if (st) return st;
  return glenside_conv2d_direct(act, w, stride, pad, residual, actfn, out, ws, kStaticScratchBytes, stream);
}

int glenside_conv2d_im2col(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                           const int64_t pad[2], const gs_ap* residual, int actfn, gs_ap* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  ConvShape cs;
  int st = conv_shape(act, w, stride, pad, &cs);
  if (st) return st;
  st = conv_check_io(act, w, residual, actfn, out, cs);
  if (st) return st;
  const size_t need = glenside_conv2d_im2col_workspace(act, w, stride, pad);
  if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16)
    return GS_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t esz = int64_t(dtype_size(act->dtype));
  const int64_t K = int64_t(cs.C) * cs.Kh * cs.Kw, ld = im2col_ld(act->dtype, K);
  const int64_t M = int64_t(cs.N) * cs.Ho * cs.Wo;
  uint8_t* cols = static_cast<uint8_t*>(workspace);
  uint8_t* wpad = cols + round_up(M * ld * esz, 256);

  // flatten (windows (access activations 1) (C Kh Kw) (1 Sh Sw)), rows padded to 16 bytes.
  WindowsArgs wa;
  memset(&wa, 0, sizeof(wa));
  wa.in = act->data;
  wa.out = cols;
  wa.esz = int(esz);
  wa.n_compute = 3;
  wa.outer = cs.N;
  const int64_t in_dim[3] = {cs.C, cs.H, cs.W}, out_dim[3] = {1, cs.Ho, cs.Wo};
  const int64_t win[3] = {cs.C, cs.Kh, cs.Kw}, str[3] = {1, cs.Sh, cs.Sw}, plo[3] = {0, cs.Ph, cs.Pw};
  for (int d = 0; d < 3; ++d) {
    wa.in_dim[d] = in_dim[d]; wa.out_dim[d] = out_dim[d]; wa.win[d] = win[d];
    wa.stride[d] = str[d]; wa.pad_lo[d] = plo[d];
  }
  wa.fill_bits = 0;
  wa.out_row_stride = ld;
  hipError_t e = launch_windows(wa, s);
  if (e != hipSuccess) return launch_status(e);

  // flatten (access weights 1): already ((O),(K)) in memory; copied only when rows need padding.
  const void* wmat = w->data;
  if (ld != K) {
    WindowsArgs ww;
    memset(&ww, 0, sizeof(ww));
    ww.in = w->data;
    ww.out = wpad;
    ww.esz = int(esz);
    ww.n_compute = 1;
    ww.outer = cs.O;
    ww.in_dim[0] = K; ww.out_dim[0] = 1; ww.win[0] = K; ww.stride[0] = 1; ww.pad_lo[0] = 0;
    ww.out_row_stride = ld;
    e = launch_windows(ww, s);
    if (e != hipSuccess) return launch_status(e);
    wmat = wpad;
  }

  GemmArgs g{};
  memset(&g, 0, sizeof(g));
  g.x = wmat;
  g.y = cols;
  g.out = out->data;
  g.residual = residual ? residual->data : nullptr;
  g.in_dtype = act->dtype;
  g.out_dtype = out->dtype;
  g.I = cs.O;
  g.J = M;
  g.K = ld;   // the pad columns are zeros on both sides
  g.ldx = g.ldy = ld;
  g.jp = int64_t(cs.Ho) * cs.Wo;
  if (g.jp < 1) g.jp = 1;
  g.relu = actfn == GS_ACT_RELU;
  return launch_status(launch_gemm(g, s));
}

int glenside_reduce(const gs_ap* in, int op, float scale, gs_ap* out, void* stream) {
  int st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (op != GS_SUM && op != GS_MAX) return GS_ERR_UNSUPPORTED;
  if (out->rank != in->n_access || out->n_access != out->rank) return GS_ERR_RANK;
  for (int d = 0; d < out->rank; ++d)
    if (out->shape[d] != in->shape[d]) return GS_ERR_SHAPE;
  const bool is_int = in->dtype == GS_I8 || in->dtype == GS_I32;
  if (in->dtype == GS_I8) {
    if (out->dtype != (op == GS_SUM ? GS_I32 : GS_I8)) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_I32) {
    if (out->dtype != GS_I32) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_BF16) {
    if (out->dtype != GS_BF16 && out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_F32) {
    if (out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else {
    return GS_ERR_DTYPE;                 // 8-bit floats are contraction operands only
  }
  if ((is_int || op == GS_MAX) && scale != 1.0f) return GS_ERR_UNSUPPORTED;
  const int64_t cols = compute_numel(in);
  if (op == GS_MAX && cols == 0 && access_numel(in) > 0) return GS_ERR_SHAPE;   // max of nothing
  ReduceArgs a;
  memset(&a, 0, sizeof(a));
  a.in = in->data;
  a.out = out->data;
  a.in_dtype = in->dtype;
  a.out_dtype = out->dtype;
  a.op = op;
  a.rows = access_numel(in);
  a.cols = cols;
  a.scale = scale;
  return launch_status(launch_reduce(a, static_cast<hipStream_t>(stream)));
}

int glenside_depthwise_conv2d(const gs_ap* act, const gs_ap* w, const int64_t stride[2],
                              const int64_t pad[2], int act_fn, gs_ap* out, void* stream) {
  int st = check_ap(act, true);
  if (st) return st;
  st = check_ap(w, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (!stride || !pad) return GS_ERR_NULL;
  if (act->rank != 4 || act->n_access != 1 || w->rank != 3 || w->n_access != 1) return GS_ERR_RANK;
  if (out->rank != 4 || out->n_access != 4) return GS_ERR_RANK;
  if (act_fn != GS_ACT_NONE && act_fn != GS_ACT_RELU) return GS_ERR_UNSUPPORTED;
  if (act->dtype != w->dtype) return GS_ERR_DTYPE;
  if (act->dtype == GS_I8) {
    if (out->dtype != GS_I32) return GS_ERR_DTYPE;
  } else if (act->dtype == GS_BF16) {
    if (out->dtype != GS_BF16 && out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else {
    return GS_ERR_DTYPE;
  }
  const int64_t N = act->shape[0], C = act->shape[1], H = act->shape[2], W = act->shape[3];
  const int64_t Kh = w->shape[1], Kw = w->shape[2];
  if (w->shape[0] != C) return GS_ERR_SHAPE;
  if (stride[0] < 1 || stride[1] < 1 || pad[0] < 0 || pad[1] < 0 || Kh < 1 || Kw < 1) return GS_ERR_SHAPE;
  if (H + 2 * pad[0] < Kh || W + 2 * pad[1] < Kw) return GS_ERR_SHAPE;
  const int64_t Ho = (H + 2 * pad[0] - Kh) / stride[0] + 1, Wo = (W + 2 * pad[1] - Kw) / stride[1] + 1;
  if (out->shape[0] != N || out->shape[1] != C || out->shape[2] != Ho || out->shape[3] != Wo)
    return GS_ERR_SHAPE;
  if (N > (1 << 24) || C > (1 << 24) || H > (1 << 20) || W > (1 << 20) || Kh > 64 || Kw > 64 ||
      stride[0] > 64 || stride[1] > 64 || pad[0] >= Kh || pad[1] >= Kw)
    return GS_ERR_UNSUPPORTED;
  if (overlaps(act, out) || overlaps(w, out)) return GS_ERR_UNSUPPORTED;
  DepthwiseArgs d;
  memset(&d, 0, sizeof(d));
  d.in = act->data; d.w = w->data; d.out = out->data;
  d.in_dtype = act->dtype; d.out_dtype = out->dtype; d.relu = act_fn == GS_ACT_RELU;
  d.N = int(N); d.C = int(C); d.H = int(H); d.W = int(W); d.Ho = int(Ho); d.Wo = int(Wo);
  d.Kh = int(Kh); d.Kw = int(Kw); d.Sh = int(stride[0]); d.Sw = int(stride[1]);
  d.Ph = int(pad[0]); d.Pw = int(pad[1]);
  return launch_status(launch_depthwise(d, static_cast<hipStream_t>(stream)));
}

int glenside_windows_reduce(const gs_ap* in, const int64_t* window, const int64_t* stride,
                            const int64_t* pad_lo, const int64_t* pad_hi, int op, float scale,
                            gs_ap* out, void* stream) {
  gs_ap win;
  int st = windows_shape(in, window, stride, pad_lo, pad_hi, &win);
  if (st) return st;
  st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (op != GS_SUM && op != GS_MAX) return GS_ERR_UNSUPPORTED;
  const int nc = in->rank - in->n_access;
  if (nc > 3) return GS_ERR_UNSUPPORTED;
  // compute reduce (windows ...): ((a.., b'..), ()).
  if (out->rank != win.n_access || out->n_access != out->rank) return GS_ERR_RANK;
  for (int d = 0; d < out->rank; ++d)
    if (out->shape[d] != win.shape[d]) return GS_ERR_SHAPE;
  const bool is_int = in->dtype == GS_I8 || in->dtype == GS_I32;
  if (in->dtype == GS_I8) {
    if (out->dtype != (op == GS_SUM ? GS_I32 : GS_I8)) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_I32) {
    if (out->dtype != GS_I32) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_BF16) {
    if (out->dtype != GS_BF16 && out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else if (in->dtype == GS_F32) {
    if (out->dtype != GS_F32) return GS_ERR_DTYPE;
  } else {
    return GS_ERR_DTYPE;                 // 8-bit floats are contraction operands only
  }
  if ((is_int || op == GS_MAX) && scale != 1.0f) return GS_ERR_UNSUPPORTED;
  WindowsReduceArgs a;
  memset(&a, 0, sizeof(a));
  a.in = in->data;
  a.out = out->data;
  a.in_dtype = in->dtype;
  a.out_dtype = out->dtype;
  a.op = op;
  a.n_compute = nc;
  a.outer = access_numel(in);
  for (int d = 0; d < nc; ++d) {
    a.in_dim[d] = in->shape[in->n_access + d];
    a.out_dim[d] = win.shape[in->n_access + d];
    a.win[d] = window[d];
    a.stride[d] = stride[d];
    a.pad_lo[d] = pad_lo ? pad_lo[d] : 0;
  }
  a.scale = scale;
  return launch_status(launch_windows_reduce(a, static_cast<hipStream_t>(stream)));
}

int glenside_pair_reduce(const gs_ap* a, const gs_ap* b, int op, int act, gs_ap* out,
                         void* stream) {
  int st = check_ap(a, true);
  if (st) return st;
  st = check_ap(b, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (op != GS_SUM && op != GS_MAX) return GS_ERR_UNSUPPORTED;
  if (act != GS_ACT_NONE && act != GS_ACT_RELU) return GS_ERR_UNSUPPORTED;
  // pair needs two patterns of one shape (Table 1).  reduceSum then folds every compute
  // dimension, so the result is element-wise only for patterns with empty compute shape.
  if (a->rank != b->rank || a->n_access != b->n_access) return GS_ERR_RANK;
  if (a->n_access != a->rank || out->n_access != out->rank) return GS_ERR_RANK;
  if (!same_shape(a, b)) return GS_ERR_SHAPE;
  if (out->rank != a->rank) return GS_ERR_RANK;
  if (!same_shape(a, out)) return GS_ERR_SHAPE;
  if (a->dtype != b->dtype || a->dtype != out->dtype || a->dtype == GS_I8 || a->dtype == GS_F8)
    return GS_ERR_DTYPE;
  PairArgs p;
  memset(&p, 0, sizeof(p));
  p.a = a->data;
  p.b = b->data;
  p.out = out->data;
  p.dtype = a->dtype;
  p.op = op;
  p.relu = act == GS_ACT_RELU;
  p.n = numel(a);
  return launch_status(launch_pair_reduce(p, static_cast<hipStream_t>(stream)));
}

// ---------------------------------------------------------------------------------------------
// Table 1 transformers that move data
// ---------------------------------------------------------------------------------------------
}  // extern "C"

namespace {

void row_major_strides(const gs_ap* a, int64_t* st) {
  int64_t s = 1;
  for (int d = a->rank - 1; d >= 0; --d) {
    st[d] = s;
    s *= a->shape[d];
  }
}

// A box copy between two dense tensors: dims/strides given in the output's dimension order.
int run_move(const gs_ap* in, gs_ap* out, int rank, const int64_t* dims, const int64_t* is,
             const int64_t* os, int64_t in_off, int64_t out_off, void* stream) {
  if (overlaps(in, out)) return GS_ERR_UNSUPPORTED;    // a mover reads while it writes: never in place
  MoveArgs m;
  memset(&m, 0, sizeof(m));
  m.in = in->data;
  m.out = out->data;
  m.esz = int(dtype_size(in->dtype));
  m.rank = rank;
  for (int d = 0; d < rank; ++d) {
    m.dims[d] = dims[d];
    m.is[d] = is[d];
    m.os[d] = os[d];
  }
  m.in_off = in_off;
  m.out_off = out_off;
  return launch_status(launch_move(m, static_cast<hipStream_t>(stream)));
}

int check_result(const gs_ap* out, int dtype, int rank, int n_access, const int64_t* shape) {
  if (out->dtype != dtype) return GS_ERR_DTYPE;
  if (out->rank != rank || out->n_access != n_access) return GS_ERR_RANK;
  for (int d = 0; d < rank; ++d)
    if (out->shape[d] != shape[d]) return GS_ERR_SHAPE;
  return GS_OK;
}

}  // namespace

extern "C" {

int glenside_transpose(const gs_ap* in, const int64_t* perm, gs_ap* out, void* stream) {
  int st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (overlaps(in, out)) return GS_ERR_UNSUPPORTED;   // the result must not share bytes with an input
  if (!perm) return GS_ERR_NULL;
  bool seen[GS_MAX_RANK] = {false};
  int64_t shape[GS_MAX_RANK], ist[GS_MAX_RANK], is[GS_MAX_RANK], os[GS_MAX_RANK];
  row_major_strides(in, ist);
  for (int t = 0; t < in->rank; ++t) {
    if (perm[t] < 0 || perm[t] >= in->rank || seen[perm[t]]) return GS_ERR_SHAPE;
    seen[perm[t]] = true;
    shape[t] = in->shape[perm[t]];
    is[t] = ist[perm[t]];
  }
  st = check_result(out, in->dtype, in->rank, in->n_access, shape);
  if (st) return st;
  row_major_strides(out, os);
  return run_move(in, out, in->rank, shape, is, os, 0, 0, stream);
}

int glenside_slice(const gs_ap* in, int dim, int64_t lo, int64_t hi, gs_ap* out, void* stream) {
  int st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (overlaps(in, out)) return GS_ERR_UNSUPPORTED;   // the result must not share bytes with an input
  if (dim < 0 || dim >= in->rank) return GS_ERR_RANK;
  if (lo < 0 || lo > hi || hi > in->shape[dim]) return GS_ERR_SHAPE;
  int64_t shape[GS_MAX_RANK], is[GS_MAX_RANK], os[GS_MAX_RANK];
  for (int d = 0; d < in->rank; ++d) shape[d] = in->shape[d];
  shape[dim] = hi - lo;
  st = check_result(out, in->dtype, in->rank, in->n_access, shape);
  if (st) return st;
  row_major_strides(in, is);
  row_major_strides(out, os);
  return run_move(in, out, in->rank, shape, is, os, lo * is[dim], 0, stream);
}

int glenside_concat(const gs_ap* a, const gs_ap* b, int dim, gs_ap* out, void* stream) {
  int st = check_ap(a, true);
  if (st) return st;
  st = check_ap(b, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (overlaps(a, out) || overlaps(b, out)) return GS_ERR_UNSUPPORTED;   // the result must not share bytes with an input
  if (a->rank != b->rank || a->n_access != b->n_access) return GS_ERR_RANK;
  if (dim < 0 || dim >= a->rank) return GS_ERR_RANK;
  if (a->dtype != b->dtype) return GS_ERR_DTYPE;
  int64_t shape[GS_MAX_RANK], as[GS_MAX_RANK], bs[GS_MAX_RANK], os[GS_MAX_RANK];
  for (int d = 0; d < a->rank; ++d) {
    if (d != dim && a->shape[d] != b->shape[d]) return GS_ERR_SHAPE;
    shape[d] = a->shape[d];
  }
  shape[dim] = a->shape[dim] + b->shape[dim];
  st = check_result(out, a->dtype, a->rank, a->n_access, shape);
  if (st) return st;
  row_major_strides(a, as);
  row_major_strides(b, bs);
  row_major_strides(out, os);
  st = run_move(a, out, a->rank, a->shape, as, os, 0, 0, stream);
  if (st) return st;
  return run_move(b, out, b->rank, b->shape, bs, os, 0, a->shape[dim] * os[dim], stream);
}

int glenside_pad(const gs_ap* in, int dim, int64_t lo, int64_t hi, int pad_mode, gs_ap* out,
                 void* stream) {
  int st = check_ap(in, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (overlaps(in, out)) return GS_ERR_UNSUPPORTED;   // the result must not share bytes with an input
  if (dim < 0 || dim >= in->rank) return GS_ERR_RANK;
  if (lo < 0 || hi < 0) return GS_ERR_SHAPE;
  if (pad_mode != GS_PAD_ZERO && pad_mode != GS_PAD_LOWEST) return GS_ERR_UNSUPPORTED;
  int64_t shape[GS_MAX_RANK], is[GS_MAX_RANK], os[GS_MAX_RANK];
  for (int d = 0; d < in->rank; ++d) shape[d] = in->shape[d];
  shape[dim] = in->shape[dim] + lo + hi;
  st = check_result(out, in->dtype, in->rank, in->n_access, shape);
  if (st) return st;
  row_major_strides(in, is);
  row_major_strides(out, os);
  if (lo + hi > 0) {
    st = launch_status(launch_fill(out->data, int(dtype_size(in->dtype)), numel(out),
                                   pad_mode == GS_PAD_LOWEST ? lowest_bits(in->dtype) : 0u,
                                   static_cast<hipStream_t>(stream)));
    if (st) return st;
  }
  return run_move(in, out, in->rank, in->shape, is, os, 0, lo * os[dim], stream);
}

int glenside_pair(const gs_ap* a, const gs_ap* b, gs_ap* out, void* stream) {
  int st = check_ap(a, true);
  if (st) return st;
  st = check_ap(b, true);
  if (st) return st;
  st = check_ap(out, true);
  if (st) return st;
  if (overlaps(a, out) || overlaps(b, out)) return GS_ERR_UNSUPPORTED;   // the result must not share bytes with an input
  if (a->rank != b->rank || a->n_access != b->n_access) return GS_ERR_RANK;
  if (!same_shape(a, b)) return GS_ERR_SHAPE;
  if (a->dtype != b->dtype) return GS_ERR_DTYPE;
  if (a->rank + 1 > GS_MAX_RANK) return GS_ERR_RANK;
  int64_t shape[GS_MAX_RANK];
  for (int d = 0; d < a->n_access; ++d) shape[d] = a->shape[d];
  shape[a->n_access] = 2;
  for (int d = a->n_access; d < a->rank; ++d) shape[d + 1] = a->shape[d];
  st = check_result(out, a->dtype, a->rank + 1, a->n_access, shape);
  if (st) return st;
  // ((A..),(C..)) seen as [A][C]; the output as [A][2][C].
  const int64_t A = access_numel(a), C = compute_numel(a);
  const int64_t dims[2] = {A, C}, is[2] = {C, 1}, os[2] = {2 * C, 1};
  st = run_move(a, out, 2, dims, is, os, 0, 0, stream);
  if (st) return st;
  return run_move(b, out, 2, dims, is, os, 0, C, stream);
}

}  // extern "C"
