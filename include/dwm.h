/*
 * libdwm -- forward 2-D convolution by the Decomposable Winograd Method (DWM) on
 * AMD MI355X (gfx950), C ABI.
 *
 * The method (paper Sec. 4.1): a kernel that is large and/or strided is split into
 * stride-1 sub-kernels ("parts") of size at most 3x3 -- taps are grouped by index
 * modulo the stride (eq. 12-14) and each group is cut into consecutive runs of three
 * (eq. 8-11) -- every part goes through a small Winograd F(2,l) (Sec. 3.1-3.2) and the
 * parts' results are summed (the five steps of Sec. 4.1 / Fig. 3: splitting,
 * transformation, calculation, detransformation, aggregation).  The result equals the
 * ordinary convolution in exact arithmetic.
 *
 * Semantics of the whole path: cross-correlation, identical to a framework conv2d with
 * no bias, dilation 1, groups 1, one stride for both dimensions and symmetric zero
 * padding:
 *     y[n,k,oh,ow] = sum_{c,r,q} xp[n,c,oh*stride+r,ow*stride+q] * w[k,c,r,q]
 * with xp = x zero-padded by `pad` on all four sides, OH = (H+2*pad-R)/stride+1 (same
 * for OW).  All tensors are dense float32: x[N][C][H][W], w[K][C][R][S], y[N][K][OH][OW].
 *
 * Memory and streams.  Every pointer named *_dev is DEVICE memory owned by the caller;
 * the library never allocates or frees device memory, never synchronises, and enqueues
 * all kernels on the hipStream_t passed as `stream` (a `void*`; NULL = default stream).
 * A plan is host memory owned by the library (create/destroy).  Kernel variants that move
 * the workspace layout ("contract", "split") can only be chosen BEFORE dwm_plan_set_workspace;
 * afterwards the layout is fixed and the plan may be reused for any number of calls.  Two calls
 * that use the same plan (hence the same workspace) must be ordered on one stream.
 *
 * Errors are return codes, never exceptions or aborts.  Launch errors reported by the
 * HIP runtime come back as DWM_ERR_HIP.
 */
#ifndef DWM_H_
#define DWM_H_

#include <stddef.h>

/* Exported symbols of the shared library. */
#define DWM_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dwm_plan dwm_plan_t;

typedef enum {
    DWM_OK = 0,
    DWM_ERR_INVALID_ARG = 1, /* null pointer; N,C,H,W,K,R,S < 1; stride < 1; pad < 0; empty output */
    DWM_ERR_UNSUPPORTED = 2, /* shape outside the limits stated at dwm_plan_create */
    DWM_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small */
    DWM_ERR_ALLOC = 4,       /* host allocation failed */
    DWM_ERR_HIP = 5          /* the HIP runtime reported an error */
} dwm_status_t;

/* What the planner decided (all host-side integers). */
typedef struct {
    int N, C, H, W, K, R, S, stride, pad;
    int OH, OW;               /* output size */
    int TH, TW;               /* 2x2 output tiles per image: ceil(OH/2), ceil(OW/2) */
    long long T;              /* N*TH*TW tiles */
    int n_parts;              /* sub-kernels (Sec. 4.1 "Splitting") */
    int n_classes;            /* distinct (len_h, len_w) among the parts */
    int n_planes;             /* Winograd-domain planes = sum over classes of (len_h+1)(len_w+1) */
    long long mults_per_tile; /* multiplications per 2x2 output tile per (k,c): sum over parts of
                                 (len_h+1)(len_w+1), the counting model of Table 3 */
    double direct_flops;      /* 2*N*K*C*R*S*OH*OW */
    double winograd_flops;    /* 2*mults_per_tile*C*K*T */
    int Kpad;                 /* rows per plane of the transformed filter (K rounded up) */
    long long Tpad;           /* tiles covered by the transformed input (T rounded up to 256) */
    long long Vblock;         /* floats of one block of the transformed input: all planes' rows for 64 tiles */
    int forward_path;         /* what dwm_conv_forward runs now: 0 = input transform + contraction,
                                 1 = single kernel (layers with few input channels) */
} dwm_plan_info_t;

/* One sub-kernel.  Its taps are w[.,.,stride*(off_h+a)+phase_h, stride*(off_w+b)+phase_w],
 * a < len_h, b < len_w; for output (oh,ow) it meets padded input
 * xp[stride*(oh+off_h+a)+phase_h][stride*(ow+off_w+b)+phase_w]. */
typedef struct {
    int phase_h, off_h, len_h;
    int phase_w, off_w, len_w;
    int cls;  /* class index: parts with equal (len_h, len_w) share transforms */
    int slot; /* position inside its class: reduction index l = slot*C + c */
} dwm_part_t;

/* One class = all parts with the same (len_h, len_w).  They use the same F(2,len)
 * matrices, so they are summed in the Winograd domain: the reduction of the class runs
 * over l = slot*C + c, l < L = n_parts*C (rounded up to Lpad with zeros).
 * Layouts (offsets in floats from the start of the buffer; fh <= len_h, fw <= len_w):
 *   transformed filter  Ugw[u_offset + ((fh*(len_w+1)+fw)*Kpad + k)*Lpad + l]
 *   transformed input   ws [(t/64)*Vblock + v_offset + ((fh*(len_w+1)+fw)*Lpad + l)*64 + t%64],
 *                       t = (n*TH + ty)*TW + tx: blocked by 64 tiles, so that what one workgroup
 *                       of the contraction reads per step is one contiguous run
 */
typedef struct {
    int len_h, len_w;
    int n_parts;
    int L, Lpad;
    long long u_offset, v_offset;
} dwm_class_t;

/* The single-kernel forward path (layers with few input channels) reads its own copy of the
 * transformed filter, kept in Ugw after the per-class layout above.  There, pieces of two and
 * three taps of a dimension form one family that shares the four frequencies of F(2,3)
 * (Sec. 3.2): a 2-tap piece is run as a 3-tap piece whose third tap is zero, so its fourth
 * product vanishes and is dropped -- a three-multiplication F(2,2), as Table 3 counts it.
 * One-tap pieces (two products, no transform) form the other family.  A "fused class" is a
 * pair of families; its rows are (part, channel) pairs, grouped by (len_h, len_w) and padded
 * to a multiple of four with rows of zeros.  Layout, filter k = 32*slice + 16*half + i:
 *   Ugw[uf_offset + (((slice*n_freq_h*n_freq_w + fh*n_freq_w + fw)*rows + row)*16 + i)*2 + half]
 * zero for k >= K, padding rows and frequencies a part does not have. */
typedef struct {
    int wide_h, wide_w;     /* 1: the family of 2- and 3-tap pieces, 0: one-tap pieces */
    int n_freq_h, n_freq_w; /* 4 or 2 */
    int first_row, rows;    /* rows of this class in the row numbering of dwm_plan_fused_row */
    long long uf_offset;    /* floats from the start of Ugw */
} dwm_fused_class_t;

typedef struct {
    int part;    /* index for dwm_plan_part */
    int channel; /* input channel */
    int real;    /* 0: padding row (zeros) */
} dwm_fused_row_t;

/*
 * Splitting, kernel side (Sec. 4.1: eq. 12 for the stride, eq. 8 for the size; the two
 * combined as its last paragraph says).  Where the single-kernel path applies, a phase's
 * taps are cut 3,...,3,2,2 instead of 3,...,3,3,1 (the same number of multiplications), so
 * that one-tap pieces only come from phases that hold a single tap.
 * Host only; no GPU call is made.
 * Limits: at most 16 one-dimensional pieces per dimension (e.g. R <= 48 at stride 1),
 * N*TH*TW and the element counts of x, w and y below 2^31 (the workspace may be larger: the transformed input
 * is addressed block by block, tested to 12 GiB).  Returns DWM_ERR_INVALID_ARG for
 * non-positive sizes, negative pad or an empty output, DWM_ERR_UNSUPPORTED beyond the limits.
 * *out is set only on DWM_OK and must be released with dwm_plan_destroy.
 */
DWM_API dwm_status_t dwm_plan_create(dwm_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                             int stride, int pad);
DWM_API dwm_status_t dwm_plan_destroy(dwm_plan_t* plan);

/* Introspection of the decomposition (host only). */
DWM_API dwm_status_t dwm_plan_info(const dwm_plan_t* plan, dwm_plan_info_t* info);
DWM_API dwm_status_t dwm_plan_part(const dwm_plan_t* plan, int i, dwm_part_t* part);     /* i < n_parts   */
DWM_API dwm_status_t dwm_plan_class(const dwm_plan_t* plan, int i, dwm_class_t* cls);   /* i < n_classes */
/* The single-kernel path's filter copy: counts (all 0 where the path does not apply), classes, rows. */
DWM_API dwm_status_t dwm_plan_fused_info(const dwm_plan_t* plan, int* n_classes, int* n_rows, int* n_slices);
DWM_API dwm_status_t dwm_plan_fused_class(const dwm_plan_t* plan, int i, dwm_fused_class_t* cls);
DWM_API dwm_status_t dwm_plan_fused_row(const dwm_plan_t* plan, int row, dwm_fused_row_t* out);

/* Bytes of the transformed filter Ugw and of the workspace (the transformed input V, plus
 * partial output tiles and arrival counters of the contraction's split tiles). */
DWM_API size_t dwm_plan_filter_bytes(const dwm_plan_t* plan);
DWM_API size_t dwm_plan_workspace_bytes(const dwm_plan_t* plan);

/* Hand the plan its workspace: caller-owned device memory, 256-byte aligned, at least
 * dwm_plan_workspace_bytes(plan) long, alive as long as the plan is used.  No GPU call. */
DWM_API dwm_status_t dwm_plan_set_workspace(dwm_plan_t* plan, void* ws_dev, size_t bytes);

/* Pick a kernel variant for a stage (for tuning and tests; the planner's own choice is the
 * default and variant < 0 restores it).
 *   "contract": tile shape / chunk depth of the contraction kernel: 10..19, the ids of the
 *               library's internal table of variants (a variant whose chunk depth does not divide
 *               the plan's reduction padding does not apply);
 *   "forward":  0 = input transform + contraction, 1 = single kernel (layers with few input channels
 *               only; the planner's choice where it applies);
 *   "input":    0, 1 = gather form of the input transform (blocks-fast / rows-fast workgroup order),
 *               2, 3 = LDS-staged form (channel groups fastest / blocks fastest; refused when the
 *               rows one block of 64 tiles needs do not fit in LDS);
 *   "input_cg": channels per workgroup of the LDS-staged form (0 = planner's choice);
 *   "split":    how the contraction shares out its tiles: 0 = planner's choice (whole tiles for every
 *               full round of the CUs + the remainder cut into equal ranges; with at most one long
 *               tile per CU, every tile cut into 2..8 ranges of its own), 1 = one round and a
 *               remainder are cut into equal ranges altogether, 2 = whole tiles only.  For tuning
 *               and tests; results are the same up to fp32 rounding.
 * The workspace size and layout depend on "contract" and "split": choose them BEFORE asking
 * dwm_plan_workspace_bytes.  DWM_ERR_INVALID_ARG for an unknown stage or a variant that does
 * not apply to this plan; DWM_ERR_WORKSPACE (nothing changed) for "contract" or "split" once
 * a workspace has been handed over. */
DWM_API dwm_status_t dwm_plan_set_variant(dwm_plan_t* plan, const char* stage, int variant);

/*
 * Transformation, kernel side (Sec. 4.1 "Transformation"; Sec. 3.1 eq. 4): for every part,
 * U = G g G^T with g the part's taps, written into Ugw_dev in the per-class layout above
 * (padding rows/columns are written as zeros).  w_dev is [K][C][R][S].  Asynchronous.
 */
DWM_API dwm_status_t dwm_filter_transform(const dwm_plan_t* plan, const float* w_dev, float* Ugw_dev, void* stream);

/*
 * The forward convolution (Sec. 4.1, all five steps on the input side): slices the
 * input per part and phase, V = B^T d B, per-plane contraction over (part, channel)
 * M = sum U .* V, detransformation A^T M A and aggregation over parts into y.
 * x_dev [N][C][H][W], Ugw_dev from dwm_filter_transform, y_dev [N][K][OH][OW] fully
 * overwritten.  Needs the workspace.  Asynchronous on `stream`.
 */
DWM_API dwm_status_t dwm_conv_forward(const dwm_plan_t* plan, const float* x_dev, const float* Ugw_dev,
                              float* y_dev, void* stream);

/*
 * dwm_conv_forward for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * plan's workspace is replaced by a fixed array of DWM_STATIC_SCRATCH_BYTES that lives in the
 * library's code object (one copy per GPU the library runs on, held until the process ends);
 * the plan needs no dwm_plan_set_workspace.  Nothing is allocated, on the device or the host.
 * DWM_ERR_WORKSPACE if dwm_plan_workspace_bytes(plan) exceeds DWM_STATIC_SCRATCH_BYTES
 * (dwm_static_scratch_bytes() returns the same figure at run time).  Layers that take the single-kernel
 * path use no scratch and are never refused.  All calls on one GPU share that GPU's array:
 * calls that may overlap (different streams, different threads) race; order them on one stream.
 * Results are those of dwm_conv_forward, bit for bit.
 */
#define DWM_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
DWM_API size_t dwm_static_scratch_bytes(void);
DWM_API dwm_status_t dwm_conv_forward_static(const dwm_plan_t* plan, const float* x_dev, const float* Ugw_dev,
                                             float* y_dev, void* stream);

/* The two stages of dwm_conv_forward on their own (for per-stage tests and timing):
 * dwm_input_transform fills the workspace with V (Sec. 4.1 "Splitting" of the input and
 * "Transformation"); dwm_contract_output reads V from the workspace and does the
 * "Calculation", "Detransformation" and "Aggregation" steps.  Calling them in this order
 * on one stream is exactly dwm_conv_forward.  dwm_contract_output may be repeated on the
 * same V; it must not be the first call on a fresh workspace (dwm_input_transform also
 * clears the arrival counters the contraction uses). */
DWM_API dwm_status_t dwm_input_transform(const dwm_plan_t* plan, const float* x_dev, void* stream);
DWM_API dwm_status_t dwm_contract_output(const dwm_plan_t* plan, const float* Ugw_dev, float* y_dev, void* stream);

/*
 * Gradient with respect to the input (the paper's backward pass: Sec. 3.1 eq. 5 for one
 * Winograd unit, Sec. 4.2 eq. 16-17 for the decomposition -- every part receives the whole
 * output gradient and the parts' input gradients are summed, which is the gradient of the
 * ordinary convolution):
 *     dx[n,c,ih,iw] = sum over (k,r,q,oh,ow) with oh*stride+r-pad == ih, ow*stride+q-pad == iw
 *                     of dy[n,k,oh,ow] * w[k,c,r,q]
 * It is computed as stride^2 stride-1 convolutions of dy, one per phase of the input
 * position modulo the stride (the phase grouping of Sec. 4.1, eq. 12-14, in mirror image),
 * each run through the forward machinery above and written to its own pixels of dx; phases
 * no tap reaches are written as zeros.  dx is fully overwritten, nothing is accumulated in
 * memory, results do not vary from run to run.
 * The plan takes the FORWARD layer's shape.  Limits: stride <= 8 and those of dwm_plan_create.
 * Memory, stream and error conventions are the same as for the forward calls; the workspace
 * (>= dwm_bwd_data_workspace_bytes, 256-byte aligned, non-null) holds the sub-convolutions'
 * transformed inputs: one after the other in the same space where the sub-convolutions run one
 * after the other, side by side where their contractions are launched together (stride > 1,
 * staged path).  Everything runs on the given stream.
 */
typedef struct dwm_bwd_data_plan dwm_bwd_data_plan_t;

typedef struct {
    int n_phases;                    /* stride^2 */
    int n_subconvs;                  /* phases that hold taps and pixels */
    long long mults_per_input_block; /* sum over sub-convolutions of their multiplications per 2x2 tile */
    double direct_flops;             /* 2*N*K*C*R*S*OH*OW, the same as the forward pass */
    double winograd_flops;           /* sum over sub-convolutions */
    int single_kernel;               /* 1: the path in use is the single kernel (see dwm_bwd_data_set_variant) */
} dwm_bwd_data_info_t;

typedef struct {
    int phase_h, phase_w; /* padded input position modulo the stride */
    int taps_h, taps_w;   /* taps of the kernel in that phase: ceil((R - phase_h)/stride), 0 if none */
    int first_h, first_w; /* first pixel of dx in the phase */
    int count_h, count_w; /* pixels of dx in the phase, per dimension */
    int has_subconv;      /* 1: a stride-1 convolution of taps_h x taps_w taps computes them; 0: zeros */
} dwm_bwd_phase_t;

DWM_API dwm_status_t dwm_bwd_data_plan_create(dwm_bwd_data_plan_t** out, int N, int C, int H, int W, int K, int R,
                                              int S, int stride, int pad);
DWM_API dwm_status_t dwm_bwd_data_plan_destroy(dwm_bwd_data_plan_t* plan);
DWM_API dwm_status_t dwm_bwd_data_plan_info(const dwm_bwd_data_plan_t* plan, dwm_bwd_data_info_t* info);
DWM_API dwm_status_t dwm_bwd_data_plan_phase(const dwm_bwd_data_plan_t* plan, int i, dwm_bwd_phase_t* out);
DWM_API size_t dwm_bwd_data_filter_bytes(const dwm_bwd_data_plan_t* plan);
DWM_API size_t dwm_bwd_data_workspace_bytes(const dwm_bwd_data_plan_t* plan);
DWM_API dwm_status_t dwm_bwd_data_set_workspace(dwm_bwd_data_plan_t* plan, void* ws_dev, size_t bytes);
/* stage "path": 0 = the sub-convolutions described above, 1 = the whole gradient in one kernel (all
 * phases and channels of dx as the columns of a single stride-1 correlation of dy whose window is
 * cut by eq. 8; for layers with few input channels; needs no workspace; DWM_ERR_UNSUPPORTED where
 * it does not apply: a window of fewer than two or more than eleven taps, more than 256 columns,
 * an image of dy of 2 GiB or more, a filter slice that does not fit in LDS -- windows of seven taps
 * and more), -1 = the planner's choice (1 where C <= 16, C*stride^2 <= 64, two workgroups fit a CU and at
 * least half of a workgroup's lanes hold a tile).
 * Both give the same dx up to fp32 summation order.  May be called at any time. */
DWM_API dwm_status_t dwm_bwd_data_set_variant(dwm_bwd_data_plan_t* plan, const char* stage, int variant);
/* w_dev is the forward layer's [K][C][R][S]; Ugw_dev (dwm_bwd_data_filter_bytes long) receives, per
 * phase, the transformed filter of that phase's flipped taps with filters and channels swapped.
 * Where no tap reaches any pixel of dx (stride above the kernel size on a narrow image) there is nothing to
 * transform: dwm_bwd_data_filter_bytes is 0 and Ugw_dev may be NULL here and in dwm_conv_backward_data, which
 * then writes zeros. */
DWM_API dwm_status_t dwm_bwd_data_filter_transform(const dwm_bwd_data_plan_t* plan, const float* w_dev, float* Ugw_dev,
                                                   void* stream);
/* dy_dev [N][K][OH][OW], dx_dev [N][C][H][W] (fully overwritten). */
DWM_API dwm_status_t dwm_conv_backward_data(const dwm_bwd_data_plan_t* plan, const float* dy_dev,
                                            const float* Ugw_dev, float* dx_dev, void* stream);

/*
 * Gradient with respect to the filter (the paper's backward pass: Sec. 3.1 eq. 5, second
 * formula, per Winograd unit; Sec. 4.2 eq. 18 for the decomposition):
 *     dw[k,c,r,q] = sum_{n,oh,ow} dy[n,k,oh,ow] * xp[n,c,oh*stride+r,ow*stride+q]
 * computed part by part as dg = G^T [ sum over tiles of (A dY A^T) .* V ] G with V = B^T d B the
 * forward pass's transformed input; the sum over tiles is a GEMM per Winograd-domain plane.
 * dw [K][C][R][S] is fully overwritten; results do not vary from run to run.
 * The plan takes the forward layer's shape; the workspace (dwm_bwd_filter_workspace_bytes,
 * 256-byte aligned) holds V, A dY A^T (not for layers with few input channels, where it is never
 * written to memory) and the partial sums.  Conventions as for the forward calls.
 */
typedef struct dwm_bwd_filter_plan dwm_bwd_filter_plan_t;

typedef struct {
    int n_planes;          /* Winograd-domain planes = GEMMs */
    int n_tiles;           /* 64x64 output tiles over all planes */
    int splits;            /* ranges the tile axis (the reduction) is cut into */
    double direct_flops;   /* 2*N*K*C*R*S*OH*OW */
    double winograd_flops; /* 2*mults_per_tile*C*K*T, as in the forward pass */
} dwm_bwd_filter_info_t;

DWM_API dwm_status_t dwm_bwd_filter_plan_create(dwm_bwd_filter_plan_t** out, int N, int C, int H, int W, int K,
                                                int R, int S, int stride, int pad);
DWM_API dwm_status_t dwm_bwd_filter_plan_destroy(dwm_bwd_filter_plan_t* plan);
DWM_API dwm_status_t dwm_bwd_filter_plan_info(const dwm_bwd_filter_plan_t* plan, dwm_bwd_filter_info_t* info);
DWM_API size_t dwm_bwd_filter_workspace_bytes(const dwm_bwd_filter_plan_t* plan);
DWM_API dwm_status_t dwm_bwd_filter_set_workspace(dwm_bwd_filter_plan_t* plan, void* ws_dev, size_t bytes);
/* x_dev [N][C][H][W], dy_dev [N][K][OH][OW], dw_dev [K][C][R][S]. */
DWM_API dwm_status_t dwm_conv_backward_filter(const dwm_bwd_filter_plan_t* plan, const float* x_dev,
                                              const float* dy_dev, float* dw_dev, void* stream);

/*
 * Half-precision forward path: the "DWM FP16" setting of the paper's accuracy table (Table 1,
 * discussed in Sec. 5.1).  x [N][C][H][W], w [K][C][R][S] and y [N][K][OH][OW] are dense IEEE
 * binary16 (dwm_half_t = the 16-bit pattern).  The paper does not say where its FP16 version
 * rounds; here the transformed filter U = G g G^T and the transformed input V = B^T d B are each
 * rounded ONCE to binary16 (nearest, ties to even) -- U from its exact value, V from B^T d B evaluated in
 * binary32, columns of the patch first, then rows (exact unless a sum spans more than 13 binades) --, their
 * products are summed over channels and parts in FP32 on the FP16 matrix cores, the output transform is
 * FP32 and y is rounded once.
 * The kernel is cut exactly as eq. 8 writes it (3,3,...,remainder), so that the rounding points
 * are those of the method as printed.
 *
 * Same conventions as the single-precision calls: the plan is host memory, every *_dev pointer is
 * caller-owned device memory, kernels go to `stream`, nothing is allocated or synchronised, errors
 * are return codes.  Workspace: dwm_f16_workspace_bytes, 256-byte aligned (V in binary16, partial
 * outputs, arrival counters).  U_dev: dwm_f16_filter_bytes (the staged path's U, then the single
 * kernel's copy where that path applies; dwm_f16_filter_transform writes both).
 * dwm_f16_set_variant(plan, "contract", v): v in 30..47 selects the contraction's tile shape
 * (v < 0: the planner's choice; before dwm_f16_set_workspace only); (plan, "input", v): 0 = gather form of the input transform,
 * 1 = LDS-staged form (C a multiple of 8, or at most 64, and a staged region that fits), v < 0: the planner's
 * choice; DWM_ERR_INVALID_ARG if the variant does not apply to the layer.
 * (plan, "forward", v): 0 = the staged path (input transform, then contraction: needs the workspace),
 * 1 = the single kernel for layers with few input channels (V stays in registers, the products go
 * straight into the 2x2 outputs, same rounding points; needs no workspace; applies with at most 127
 * channels, 512 reduction rows after padding every class to 16, a staged input region that fits in
 * LDS, and an image of y below 2 GiB), v < 0: the planner's choice (1 where it applies, C <= 16 and at
 * least half of a workgroup's lanes hold a tile); dwm_f16_plan_info's forward_path says which is in use.
 * (plan, "classes", v): 0 = always the general single kernel, v < 0: the one built for the layer's list
 * of classes where there is one (the same arithmetic in the same order: for tests).
 * dwm_f16_conv_forward_f32out is the same computation with y left in FP32 (not rounded): it
 * exists so that tests can compare everything before the last rounding.
 * dwm_f16_input_transform / dwm_f16_contract_output are the two stages of dwm_f16_conv_forward,
 * exposed for timing.
 */
typedef struct dwm_f16_plan dwm_f16_plan_t;
typedef unsigned short dwm_half_t;

DWM_API dwm_status_t dwm_f16_plan_create(dwm_f16_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                                         int stride, int pad);
DWM_API dwm_status_t dwm_f16_plan_destroy(dwm_f16_plan_t* plan);
DWM_API dwm_status_t dwm_f16_plan_info(const dwm_f16_plan_t* plan, dwm_plan_info_t* info);
DWM_API size_t dwm_f16_filter_bytes(const dwm_f16_plan_t* plan);
DWM_API size_t dwm_f16_workspace_bytes(const dwm_f16_plan_t* plan);
DWM_API dwm_status_t dwm_f16_set_workspace(dwm_f16_plan_t* plan, void* ws_dev, size_t bytes);
DWM_API dwm_status_t dwm_f16_set_variant(dwm_f16_plan_t* plan, const char* stage, int variant);
DWM_API dwm_status_t dwm_f16_filter_transform(const dwm_f16_plan_t* plan, const dwm_half_t* w_dev,
                                              dwm_half_t* U_dev, void* stream);
DWM_API dwm_status_t dwm_f16_conv_forward(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev,
                                          const dwm_half_t* U_dev, dwm_half_t* y_dev, void* stream);
DWM_API dwm_status_t dwm_f16_conv_forward_f32out(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev,
                                                 const dwm_half_t* U_dev, float* y_dev, void* stream);
DWM_API dwm_status_t dwm_f16_input_transform(const dwm_f16_plan_t* plan, const dwm_half_t* x_dev, void* stream);
DWM_API dwm_status_t dwm_f16_contract_output(const dwm_f16_plan_t* plan, const dwm_half_t* U_dev,
                                             dwm_half_t* y_dev, void* stream);

/*
 * The same path with bfloat16 storage (8 significant bits, binary32's exponent range) -- the other
 * 16-bit format the matrix cores take, and the one to use where binary16's range is too narrow.
 * Everything said above for dwm_f16_* holds with "bfloat16" for "binary16": x, w, y, U and V are
 * bfloat16 (dwm_bf16_t = the 16-bit pattern, the upper half of the binary32 pattern), U and V are
 * rounded once (nearest, ties to even), products are summed in FP32 on the bfloat16 matrix cores,
 * the output transform is FP32, y is rounded once; the kernel is cut as eq. 8 writes it.  Layouts,
 * workspace rules, variants (30..47) and error codes are those of the dwm_f16_* calls.
 */
typedef struct dwm_bf16_plan dwm_bf16_plan_t;
typedef unsigned short dwm_bf16_t;

DWM_API dwm_status_t dwm_bf16_plan_create(dwm_bf16_plan_t** out, int N, int C, int H, int W, int K, int R, int S,
                                          int stride, int pad);
DWM_API dwm_status_t dwm_bf16_plan_destroy(dwm_bf16_plan_t* plan);
DWM_API dwm_status_t dwm_bf16_plan_info(const dwm_bf16_plan_t* plan, dwm_plan_info_t* info);
DWM_API size_t dwm_bf16_filter_bytes(const dwm_bf16_plan_t* plan);
DWM_API size_t dwm_bf16_workspace_bytes(const dwm_bf16_plan_t* plan);
DWM_API dwm_status_t dwm_bf16_set_workspace(dwm_bf16_plan_t* plan, void* ws_dev, size_t bytes);
DWM_API dwm_status_t dwm_bf16_set_variant(dwm_bf16_plan_t* plan, const char* stage, int variant);
DWM_API dwm_status_t dwm_bf16_filter_transform(const dwm_bf16_plan_t* plan, const dwm_bf16_t* w_dev,
                                               dwm_bf16_t* U_dev, void* stream);
DWM_API dwm_status_t dwm_bf16_conv_forward(const dwm_bf16_plan_t* plan, const dwm_bf16_t* x_dev,
                                           const dwm_bf16_t* U_dev, dwm_bf16_t* y_dev, void* stream);
DWM_API dwm_status_t dwm_bf16_conv_forward_f32out(const dwm_bf16_plan_t* plan, const dwm_bf16_t* x_dev,
                                                  const dwm_bf16_t* U_dev, float* y_dev, void* stream);
DWM_API dwm_status_t dwm_bf16_input_transform(const dwm_bf16_plan_t* plan, const dwm_bf16_t* x_dev, void* stream);
DWM_API dwm_status_t dwm_bf16_contract_output(const dwm_bf16_plan_t* plan, const dwm_bf16_t* U_dev,
                                              dwm_bf16_t* y_dev, void* stream);

DWM_API const char* dwm_status_string(dwm_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* DWM_H_ */
