/*
 * glenside.h -- C ABI of the MI355X (gfx950) evaluator for Glenside access-pattern programs.
 *
 * Paper: "Pure Tensor Program Rewriting via Access Patterns" (Glenside).  An access pattern
 * (Sec. 4.1) is a dense row-major tensor of shape S_A ++ S_C viewed as an S_A-shaped tensor of
 * S_C-shaped elements; `gs_ap` is that view: a device pointer, the shape, and the split point
 * n_access = |S_A| (the integer of `(access T n_A)`).
 *
 * Conventions shared by every entry point
 *   - Pointers inside a `gs_ap` and the `workspace` arguments are DEVICE pointers owned by the
 *     caller.  The `gs_ap` structs themselves, and the window/stride/pad arrays, are HOST memory
 *     and are only read during the call.  The library never allocates, frees or keeps a pointer.
 *   - Tensors are dense and row-major over S_A ++ S_C; no strides exist at this boundary.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls validate on
 *     the host, enqueue their kernels on that stream and return without synchronising.
 *   - The return value is a `gs_status`.  Every shape rule is checked before anything is
 *     launched, so a non-zero status other than GS_ERR_LAUNCH means nothing ran.  No exception or
 *     abort crosses this boundary.
 *   - Element types: GS_I8 and GS_BF16 inputs to contractions accumulate in int32 and fp32
 *     respectively (exact for integers, no saturation; the paper's own notation is real-valued
 *     and fixes no storage type).  bfloat16 stores round to nearest even.
 *   - A result never shares bytes with an input (nothing works in place).  The data-moving
 *     transformers and glenside_depthwise_conv2d check this (partial overlap included) and return
 *     GS_ERR_UNSUPPORTED; for the other entry points it is the caller's duty.
 *   - Extensions that the paper does not have are marked EXT: padding, ReLU, scaling, a fused
 *     residual input.  With pad = 0, act = GS_ACT_NONE, scale = 1 and residual = NULL every entry
 *     point computes exactly the paper's expression.
 */
#ifndef GLENSIDE_H
#define GLENSIDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GS_MAX_RANK 8

typedef enum {
  GS_OK = 0,
  GS_ERR_NULL = 1,        /* a required pointer is NULL                                   */
  GS_ERR_RANK = 2,        /* rank / n_access / window rank do not fit the operation       */
  GS_ERR_SHAPE = 3,       /* a shape rule of Table 1 / Table 2 is violated                */
  GS_ERR_DTYPE = 4,       /* element types do not fit the operation                       */
  GS_ERR_UNSUPPORTED = 5, /* valid program, but outside what the kernels cover            */
  GS_ERR_WORKSPACE = 6,   /* workspace missing, misaligned or too small                   */
  GS_ERR_LAUNCH = 7       /* HIP reported an error when launching                         */
} gs_status;

/* GS_F8 (EXT): 8-bit float, OCP e4m3 (1-4-3, bias 7, no infinities, maximum 448); accepted as the
 * operand type of glenside_cartesian_dot (and of dotProd in programs) only.                       */
typedef enum { GS_I8 = 0, GS_I32 = 1, GS_BF16 = 2, GS_F32 = 3, GS_F8 = 4 } gs_dtype;
typedef enum { GS_SUM = 0, GS_MAX = 1 } gs_reduce_op;
typedef enum { GS_ACT_NONE = 0, GS_ACT_RELU = 1 } gs_activation;
/* EXT: what a padded cell reads: zero (for dotProd / reduceSum consumers) or the lowest value of
 * the element type (-inf for floats, the minimum integer) for reduceMax consumers.              */
typedef enum { GS_PAD_ZERO = 0, GS_PAD_LOWEST = 1 } gs_pad_mode;

typedef struct {
  void* data;                 /* device pointer, 16-byte aligned, caller-owned               */
  int32_t dtype;              /* gs_dtype                                                    */
  int32_t rank;               /* |S_A| + |S_C|, at most GS_MAX_RANK                          */
  int32_t n_access;           /* |S_A|                                                       */
  int32_t reserved;           /* must be 0                                                   */
  int64_t shape[GS_MAX_RANK]; /* S_A ++ S_C                                                  */
} gs_ap;

/* Human-readable name of a status code (static storage). */
const char* glenside_status_string(int status);

/* Shape rule of `windows` (Table 1): in ((a..),(b_0..b_n)), window (w_0..w_n), strides
 * (s_0..s_n) -> out ((a.., b'_0..b'_n),(w_0..w_n)) with b'_i = ceil((b_i + lo_i + hi_i -
 * (w_i - 1)) / s_i).  pad_lo / pad_hi (EXT) may be NULL, meaning 0.  Fills out->rank, n_access,
 * shape and dtype; leaves out->data alone.  Host only.                                         */
int glenside_windows_out_shape(const gs_ap* in, const int64_t* window, const int64_t* stride,
                               const int64_t* pad_lo, const int64_t* pad_hi, gs_ap* out);

/* `windows` (Table 1; element rule from the conv2d / max-pool equations of Sec. 5.1):
 *   out[a.., p.., q..] = in[a.., p_i*s_i + q_i - lo_i ..], padded cells per pad_mode.
 * window/stride have |S_C(in)| entries.  out must have exactly the shape the rule gives and the
 * dtype of in (any of the four).  With in ((N),(C,H,W)), window (C,Kh,Kw), strides (1,Sh,Sw)
 * the output, read as ((N*1*H'*W'),(C*Kh*Kw)), is the im2col matrix of Fig. 5.                   */
int glenside_access_windows(const gs_ap* in, const int64_t* window, const int64_t* stride,
                            const int64_t* pad_lo, const int64_t* pad_hi, int pad_mode,
                            gs_ap* out, void* stream);

/* `compute dotProd (cartProd a0 a1)` -- Fig. 2b and the left-hand side of the systolic-array
 * rewrite (Sec. 5.2).  a0 ((m..),(k..)), a1 ((n..),(k..)) with equal compute shapes ->
 * out ((m.., n..),()):  out[m, n] = sum_k a0[m, k] * a1[n, k].
 * Types: i8 x i8 -> i32;  bf16 x bf16 -> f32 or bf16 (fp32 accumulate);  EXT f8 x f8 -> f32 or
 * bf16 (fp32 accumulate; the matrix unit aligns the 64 products of a step to their largest
 * exponent before adding, absolute error up to about 3e-5 of sum_k |a0[m,k] a1[n,k]|).  EXT: act
 * applies ReLU to the result.  workspace is unused (pass NULL,
 * 0): no shape of this contraction splits its sum across workgroups.                            */
int glenside_cartesian_dot(const gs_ap* a0, const gs_ap* a1, gs_ap* out, int act,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The blocked form of the same product (Sec. 5.4; the rewrites of Fig. 6 applied as in Fig. 7):
 * a0 ((M),(K)), a1 ((N),(K)), out ((M,N),()) of the accumulator's type (GS_I32 for int8 inputs,
 * GS_F32 for bfloat16 and 8-bit floats).  The result is the concat, along both access dimensions,
 * of blocks of at most tile_m x tile_n results; each block is the left-to-right fold, by
 * reduceSum (pair acc part), of dotProd over slices of at most tile_k compute elements.
 * When the slices are whole 128-byte runs of K (tile_k * element size a multiple of 128) or there
 * is a single slice, this is ONE launch: no workgroup's tile crosses a block boundary and each
 * walks its block's slices in order, folding them in its accumulators.  Other slice lengths take
 * one contraction launch per (block, K slice) on views of the operands (nothing is copied; more
 * than 65536 launches are refused with GS_ERR_UNSUPPORTED).  Equal to glenside_cartesian_dot
 * exactly for integers and up to the summation order for floats.  This is the tile-shape sweep of
 * the paper's "systolic array" sizes.                                                            */
int glenside_cartesian_dot_blocked(const gs_ap* a0, const gs_ap* a1, int64_t tile_m, int64_t tile_n,
                                   int64_t tile_k, gs_ap* out, void* stream);

/* 2D convolution, Fig. 2a:
 *   (transpose (squeeze (compute dotProd (cartProd (windows (access activations 1)
 *       (shape C Kh Kw) (shape 1 Sh Sw)) (access weights 1))) 1) (list 0 3 1 2))
 * activations ((N),(C,H,W)), weights ((O),(C,Kh,Kw)) -> out ((N,O,H',W'),()).
 * EXT: pad[2] symmetric zero padding of H and W; residual (may be NULL) is an access pattern of
 * out's shape and dtype added to the result, i.e. compute reduceSum (pair conv residual);
 * act applies ReLU last.  Types as for glenside_cartesian_dot.
 *   _direct : the windows are formed on chip (LDS-staged patches), never written to memory.
 *   _im2col : the rewritten program of Fig. 5: flatten(windows ...) is written to the workspace,
 *             then contracted with flatten(weights) by the same kernel as glenside_cartesian_dot.
 * Both need a workspace of the size their *_workspace query returns (16-byte aligned).
 * The two forms give bit-identical integer results and float results equal up to summation
 * order.                                                                                       */
int glenside_conv2d_direct(const gs_ap* activations, const gs_ap* weights, const int64_t stride[2],
                           const int64_t pad[2], const gs_ap* residual, int act, gs_ap* out,
                           void* workspace, size_t workspace_bytes, void* stream);
int glenside_conv2d_im2col(const gs_ap* activations, const gs_ap* weights, const int64_t stride[2],
                           const int64_t pad[2], const gs_ap* residual, int act, gs_ap* out,
                           void* workspace, size_t workspace_bytes, void* stream);
/* Depth-wise windows (EXT workload, written with the paper's operators only): the concat along
 * the channel dimension of the program of Fig. 2a applied, for every channel c, to
 * (slice activations 1 c c+1) and (slice weights' 0 c c+1) -- C independent one-channel, one-filter
 * convolutions; with windows of shape (1,Kh,Kw) no sum over channels is left (Table 1, windows).
 * activations ((N),(C,H,W)), weights ((C),(Kh,Kw)) -> out ((N,C,H',W'),()):
 *   out[n,c,y,x] = sum_{ky,kx} activations[n,c, y*Sh - Ph + ky, x*Sw - Pw + kx] * weights[c,ky,kx],
 * cells outside the image counting as zero (EXT pad[2], symmetric, each smaller than its window
 * dimension); act applies ReLU.  Types: i8 x i8 -> i32; bf16 x bf16 -> bf16 or f32 (fp32
 * accumulate, taps in the order ky, kx).  No workspace.  Windows or strides above 64, or rows too
 * long for the on-chip copy (about 16000 elements), return GS_ERR_UNSUPPORTED.                   */
int glenside_depthwise_conv2d(const gs_ap* activations, const gs_ap* weights, const int64_t stride[2],
                              const int64_t pad[2], int act, gs_ap* out, void* stream);

/* The two halves of glenside_conv2d_direct, for callers whose weights are constants.
 *   _pack_weights  : writes the weight access pattern ((O),(C,Kh,Kw)) into `packed` in the order
 *                    the contraction reads it, (O, Kh, Kw, C) with C padded to a 32-byte step --
 *                    the weight-side layout change that the systolic-array rewrite (Sec. 5.2) makes
 *                    explicit with (transpose ?a1 ...) -- and, when C is a whole number of such
 *                    steps, once more cut into blocks of 32 output channels x one step of one
 *                    tap (1 KB each, the unit the kernel moves on chip), (O/32, C-step, Kh, Kw).
 *                    Needs glenside_conv2d_direct_workspace bytes.
 *   _direct_packed : the convolution proper, reading weights only from `packed`; `weights` gives
 *                    shape and dtype, its data pointer is not read.  `packed` needs the bytes that
 *                    _pack_weights needs; when it has glenside_conv2d_direct_workspace bytes for
 *                    these activations, the part behind the weights is scratch for splitting the
 *                    channel sum among workgroups (layers with few output tiles), overwritten
 *                    by every call.
 * glenside_conv2d_direct(x, w, ..., ws) == _pack_weights(w, ws) then _direct_packed(x, w, ..., ws). */
int glenside_conv2d_pack_weights(const gs_ap* weights, void* packed, size_t packed_bytes,
                                 void* stream);
int glenside_conv2d_direct_packed(const gs_ap* activations, const gs_ap* weights,
                                  const int64_t stride[2], const int64_t pad[2],
                                  const gs_ap* residual, int act, gs_ap* out, void* packed,
                                  size_t packed_bytes, void* stream);
/* Workspace bytes the two forms need; 0 if the arguments are invalid.  Host only. */
size_t glenside_conv2d_direct_workspace(const gs_ap* activations, const gs_ap* weights,
                                        const int64_t stride[2], const int64_t pad[2]);
size_t glenside_conv2d_im2col_workspace(const gs_ap* activations, const gs_ap* weights,
                                        const int64_t stride[2], const int64_t pad[2]);

/* glenside_conv2d_direct for callers that cannot allocate or pass a workspace (code under HIP
 * graph capture, serving loops, harnesses that forbid allocation): same arguments without the
 * workspace, same kernels, same result bit for bit.  The packed weights and the partial sums of
 * a split channel sum go to a fixed array of glenside_conv2d_direct_static_limit() bytes (32 MiB)
 * of device memory inside the loaded library, one copy per GPU, held until the process ends.
 * The call allocates and frees nothing.  A convolution whose glenside_conv2d_direct_workspace
 * exceeds the limit returns GS_ERR_WORKSPACE and launches nothing.  The array keeps the previous
 * call's contents and every call on a GPU uses the same one (each call rewrites all it reads), so
 * calls that overlap in time on one GPU -- different streams, or graphs replayed concurrently --
 * race; calls on one stream are ordered.  The first call on a GPU looks up the array's device
 * address (no allocation; make that call outside a capture).                                     */
int glenside_conv2d_direct_static(const gs_ap* activations, const gs_ap* weights, const int64_t stride[2],
                                  const int64_t pad[2], const gs_ap* residual, int act, gs_ap* out,
                                  void* stream);
size_t glenside_conv2d_direct_static_limit(void);

/* `compute reduceSum | reduceMax` (Table 2): in ((a..),(c..)) -> out ((a..),()).
 * Types: i8 -> i32 (sum) or i8 (max); i32 -> i32; bf16 -> bf16 or f32; f32 -> f32.  Float sums
 * accumulate in fp32.  EXT: scale multiplies a float result (1.0f = the paper's operator; must
 * be 1.0f for integers and for GS_MAX).                                                         */
int glenside_reduce(const gs_ap* in, int op, float scale, gs_ap* out, void* stream);

/* `compute reduceMax|reduceSum (windows in window stride)` fused -- max pooling is Fig. 2c with
 * in ((N,C),(H,W)).  Same result as glenside_access_windows followed by glenside_reduce, without
 * the windows ever reaching memory.  out ((a.., b'..),()).  Padding (EXT) reads the lowest value
 * for GS_MAX and zero for GS_SUM.  Compute rank 1..3.                                           */
int glenside_windows_reduce(const gs_ap* in, const int64_t* window, const int64_t* stride,
                            const int64_t* pad_lo, const int64_t* pad_hi, int op, float scale,
                            gs_ap* out, void* stream);

/* `compute reduceSum|reduceMax (pair a b)` -- the element-wise sum idiom of the blocking rewrites
 * (Sec. 5.4): out = a + b (or max(a, b)) for patterns a, b, out of one shape ((s..),()) -- empty
 * compute shape, since the reduction folds every compute dimension and the pair's 2 must be the
 * only one.  EXT: act applies ReLU.  Types: a, b, out share one dtype (i32, bf16 or f32).       */
int glenside_pair_reduce(const gs_ap* a, const gs_ap* b, int op, int act, gs_ap* out,
                         void* stream);

/* The Table 1 transformers that move data, materialised (in the other entry points they are folded
 * into descriptors or into a kernel's addressing).  `out` must be a distinct tensor that already
 * has the result's dtype, rank, access split and shape; nothing is launched otherwise.
 *
 * `transpose` (Table 1; Sec. 4.2; the `(transpose ... (0 3 1 2))` tail of Fig. 5): output dimension
 * t is input dimension perm[t], over all |S_A| + |S_C| dimensions; the access split stays where it
 * is.  perm: HOST array of in->rank entries, a permutation.                                        */
int glenside_transpose(const gs_ap* in, const int64_t* perm, gs_ap* out, void* stream);
/* `slice` (Table 1; Fig. 7): keeps [lo, hi) of dimension dim.                                      */
int glenside_slice(const gs_ap* in, int dim, int64_t lo, int64_t hi, gs_ap* out, void* stream);
/* `concat` (the blocking rewrites of Sec. 5.4, Fig. 6): joins a and b along dim; the other
 * dimensions, the rank and the access split of a and b agree.                                      */
int glenside_concat(const gs_ap* a, const gs_ap* b, int dim, gs_ap* out, void* stream);
/* EXT `pad`: grows dimension dim by lo cells in front and hi behind, filled per gs_pad_mode.       */
int glenside_pad(const gs_ap* in, int dim, int64_t lo, int64_t hi, int pad_mode, gs_ap* out,
                 void* stream);
/* `pair` (Table 1; Sec. 5.4): two patterns of one shape ((a..),(c..)) -> ((a..),(2, c..)).        */
int glenside_pair(const gs_ap* a, const gs_ap* b, gs_ap* out, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Programs as text.  The paper writes kernels as s-expressions over the transformers of Table 1
 * and the operators of Table 2 (Figs. 2a-2c, 5, 7).  Text conventions: a symbol that names one of
 * `tensors` is that tensor (all compute dimensions until `access`ed); any other symbol is looked
 * up in `ints` (the C, Kh, Sh ... of the listings); (shape d0 d1 ...) and (list i0 i1 ...) are
 * integer tuples; the shape literal of `reshape` is written as two tuples,
 * (reshape X (shape c...) (shape d...)).  EXT: (pad X dim lo hi) pads with zeros, `relu` is an
 * operator.  Transformers: access transpose cartProd windows slice squeeze flatten reshape pair
 * concat; (compute dotProd|reduceSum|reduceMax X); (systolicArray rows cols a0 w) (Sec. 5.2).
 * The name strings and the two arrays are HOST memory read during the call.                     */
typedef struct {
  const char* name;
  gs_ap tensor;               /* device data, dtype, rank, shape; n_access is ignored           */
} gs_named_ap;
typedef struct {
  const char* name;
  int64_t value;
} gs_named_int;

/* Access-pattern shape, split and element type of the program's result (the shape rules of
 * Table 1 / Table 2 applied bottom-up).  Fills everything in `out` but leaves out->data.  Host only.
 * Contractions give GS_I32 (int8 operands) or GS_F32 (bfloat16 operands).                       */
int glenside_program_shape(const char* text, const gs_named_ap* tensors, int n_tensors,
                           const gs_named_int* ints, int n_ints, gs_ap* out);
/* Evaluates the program on the GPU into `out` (shape and split as glenside_program_shape gives;
 * dtype the same, or GS_BF16 where the root is a bfloat16 contraction).  Node by node:
 *   (compute dotProd (cartProd a0 a1))   one MFMA contraction; the Cartesian product is never
 *                                        formed (the pattern Fig. 3 maps to hardware);
 *   the whole listing of Fig. 2a         the direct convolution (windows formed on chip);
 *   (compute reduceX (windows ...))      the fused pooling kernel (Fig. 2c);
 *   (compute reduceX (pair a b))         the element-wise kernel (Sec. 5.4);
 *   access squeeze flatten reshape,
 *   a slice of the outermost dimension   descriptor changes, no data moves;
 *   transpose slice concat pair pad
 *   windows                              the data-moving kernels, into the workspace;
 *   cartProd anywhere else               GS_ERR_UNSUPPORTED.
 * Identical sub-programs are evaluated once.  `workspace`: device memory of at least
 * glenside_program_workspace bytes (0 = invalid program), 16-byte aligned, caller-owned.       */
int glenside_program_eval(const char* text, const gs_named_ap* tensors, int n_tensors,
                          const gs_named_int* ints, int n_ints, gs_ap* out, void* workspace,
                          size_t workspace_bytes, void* stream);
size_t glenside_program_workspace(const char* text, const gs_named_ap* tensors, int n_tensors,
                                  const gs_named_int* ints, int n_ints);
/* Applies rewrite rules of the paper to a program and writes the new program text (host only).
 *   "im2col"   : the three rules of Fig. 4, in order, at the dotProd over cartProd: derives Fig. 5
 *                from Fig. 2a;
 *   "systolic" : the rule of Fig. 3;
 *   "block"    : the rules of Fig. 6 with params = {block_m, block_n, block_k}: operands
 *                ((M),(K)) and ((N),(K)) of the dotProd over cartProd are split by rule 1 and the
 *                other rules push cartProd and dotProd through the concats: derives a program of
 *                block products joined by concat and reduceSum (pair ...) (Fig. 7) from Fig. 2b.
 * The result's shape is checked to equal the input's.  out_text: HOST buffer of out_capacity
 * bytes; *out_needed (may be NULL) receives the bytes needed; GS_ERR_WORKSPACE if too small;
 * GS_ERR_UNSUPPORTED if no rule of the strategy applies.                                        */
int glenside_program_rewrite(const char* text, const char* strategy, const int64_t* params, int n_params,
                             const gs_named_ap* tensors, int n_tensors, const gs_named_int* ints,
                             int n_ints, char* out_text, size_t out_capacity, size_t* out_needed);

#ifdef __cplusplus
}
#endif
#endif /* GLENSIDE_H */
