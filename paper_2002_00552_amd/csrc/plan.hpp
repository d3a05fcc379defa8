// Internal plan structures shared by the host planner and the kernel launchers.
// Everything a kernel needs about the decomposition travels BY VALUE in its kernel
// arguments (DevPlan / PlaneTable below), so the library owns no device memory.
#pragma once
#include <cstdint>
#ifdef __HIPCC__
#include <hip/hip_runtime.h>
#endif
#include "../../include/dwm.h"

struct dwm_plan;

namespace dwm {

constexpr int kMaxPieces = 16;  // one-dimensional pieces per dimension
constexpr int kMaxClasses = 9;  // (len_h, len_w) in {1,2,3}^2
constexpr int kMaxPlanes = 81;  // sum over classes of (len_h+1)(len_w+1) = (2+3+4)^2
constexpr int kKAlign = 128;    // Kpad is a multiple of this (largest K tile of any variant)
constexpr int kTAlign = 256;    // Tpad is a multiple of this (largest T tile of any variant)
constexpr int kLAlign = 16;     // Lpad is a multiple of this at least (smallest reduction chunk)

// A 1-D piece (Sec. 4.1): phase p, offset j inside the phase's tap list, length l.
struct DevPiece {
    int p, j, l;  // phase, first tap of the phase's tap list, length the transforms use
    int lr;       // taps the piece really has (l, except where a plan widens two-tap pieces to three)
};

// A class: the parts made of an h-piece of length lh and a w-piece of length lw.
// Pieces are stored sorted by length, so the class's h-pieces are ph[h0 .. h0+hn).
struct DevClass {
    int lh, lw;
    int h0, hn, w0, wn;
    int L, Lpad;
    int row0;    // first row of this class in the flattened (class, l) row space
    int plane0;  // first plane of this class
    long long u_off;         // floats
    int v_row0;              // first row of the class inside a V block (a row = 64 tiles)
    int pad2_;
};

// Where output pixel (oh, ow) of image n and filter k is written: element
// ((n*K + k)*YH + sy*oh + oy)*YW + sx*ow + ox of the destination.  The forward convolution
// writes densely (YH = OH, YW = OW, steps 1, offsets 0); the data gradient interleaves the
// outputs of its stride-1 sub-convolutions (one per input phase) into the gradient image.
struct OutMap {
    int YH, YW;
    int sy, oy, sx, ox;
};

struct DevPlan {
    int N, C, H, W, K, R, S, s;
    int Ph, Pw;  // the padded input starts Ph rows above and Pw columns left of the image (may be negative)
    int OH, OW, TH, TW;
    OutMap om;
    int T, Tpad, Kpad;
    int nh, nw;
    int ncls;
    int rows_total;  // sum over classes of Lpad
    int vblock_rows; // rows of one V block = sum over planes of Lpad
    DevPiece ph[kMaxPieces];
    DevPiece pw[kMaxPieces];
    DevClass cls[kMaxClasses];
};

// One Winograd-domain plane = (class, fh, fw): a [Kpad x Lpad] slice of U, a
// [Lpad x Tpad] slice of V, and the 2x2 pattern A^T[:,fh] (x) A^T[:,fw] with which its
// product enters the output tile (entries 0, +1, -1; packed two bits each).
struct DevPlaneEntry {
    uint32_t u_off64;  // offset into Ugw in units of 64 floats
    uint32_t v_off64;  // first row of the plane inside a V block (= offset in units of 64 floats)
    int32_t Lpad;
    int32_t coef;      // bits [2q+1:2q] of output q=2a+b: 0 -> 0, 1 -> +1, 3 -> -1
};

struct PlaneTable {
    int n;
    DevPlaneEntry e[kMaxPlanes];
};

// Shape of one contraction kernel variant: workgroup of WGM x WGN waves, each wave owning
// (32*WM) x (32*WN) of the (K tile) x (T tile); reduction staged LC steps at a time
// through NS LDS stages.
struct ContractVariant {
    int id, wgm, wgn, wm, wn, lc, ns;
    int kt() const { return 32 * wm * wgm; }
    int tt() const { return 32 * wn * wgn; }
};
constexpr ContractVariant kContractVariants[] = {
    {10, 2, 2, 1, 1, 16, 4}, {11, 2, 2, 1, 1, 32, 3}, {12, 2, 2, 1, 1, 64, 2}, {13, 4, 2, 1, 1, 32, 2},
    {14, 2, 4, 1, 1, 32, 3}, {15, 2, 2, 2, 1, 32, 2}, {16, 2, 2, 1, 2, 32, 2}, {17, 2, 2, 1, 1, 16, 2},
    {18, 2, 2, 1, 1, 32, 4}, {19, 2, 2, 1, 1, 64, 3},
    // half-precision contraction (half.hip): ids 30 and up
    {30, 2, 2, 1, 1, 16, 4}, {31, 2, 2, 1, 1, 32, 4}, {32, 2, 2, 1, 1, 64, 3}, {33, 2, 2, 1, 2, 32, 3},
    {34, 2, 2, 2, 1, 32, 3}, {35, 2, 2, 1, 2, 64, 2}, {36, 4, 2, 1, 1, 64, 2}, {37, 2, 4, 1, 1, 64, 2},
    {38, 4, 2, 1, 2, 32, 3}, {39, 2, 4, 2, 1, 32, 3}, {40, 4, 2, 1, 1, 64, 3}, {41, 4, 2, 1, 2, 64, 2},
    {42, 2, 2, 1, 1, 64, 5}, {43, 2, 2, 1, 1, 32, 8}, {44, 4, 2, 1, 1, 64, 4}, {45, 4, 2, 1, 2, 64, 3},
    {46, 4, 2, 1, 2, 32, 6}, {47, 2, 2, 1, 1, 64, 8},
};
constexpr int kFirstHalfVariant = 30, kLastHalfVariant = 47;
constexpr int kNumContractVariants = sizeof(kContractVariants) / sizeof(kContractVariants[0]);
constexpr int kNumCUs = 256;  // MI355X
// reduction steps a contraction's fp32 accumulator collects at most before it is folded into the outputs
constexpr int kFoldSteps = 256;

// How the (K tile, T tile) grid is shared out for one variant.  Workgroups 0..n_full-1
// each own one whole tile.  The remaining n_sk_tiles tiles (fewer than one per CU) are
// cut along the flattened (plane, chunk) iteration axis into sk_wgs equal ranges, one
// per extra workgroup, so that every CU ends up with the same amount of MFMA work; a
// tile shared by several workgroups is summed from per-workgroup partial outputs by
// whichever of them finishes last.  A layer with at most one (long) tile per CU has no
// whole-tile workgroups: each of its tiles is cut into sk_f ranges of its own.
struct ContractGeometry {
    int variant;
    int nkt, ntt, ntiles, full8;
    int n_iter;      // chunks per tile = sum over planes of Lpad/LC
    int n_full;      // whole-tile workgroups
    int n_sk_tiles;  // tiles handled by the stream-K workgroups
    int sk_wgs;      // stream-K workgroups
    int sk_ipw;      // iterations per stream-K workgroup
    int sk_maxc;     // partial-output slots per shared tile
    int sk_f;        // > 0: every stream-K tile is cut into sk_f ranges of sk_ipw iterations of its own
                     // (range g = piece g % sk_f of tile g / sk_f); 0: equal ranges of the flattened axis
    size_t partial_floats;
};

#ifdef __HIPCC__
// One 2x2 output tile through the output map; rows/columns past the output extent are dropped.
__device__ __forceinline__ void store_tile(float* __restrict__ y, const OutMap& M, int OH, int OW, size_t plane,
                                           int oh, int ow, float y00, float y01, float y10, float y11)
{
    float* yp = y + (plane * M.YH + (size_t)(M.sy * oh + M.oy)) * M.YW + (M.sx * ow + M.ox);
    const bool pair_ok = M.sx == 1 && ((M.YW | M.ox | OW) & 1) == 0;
    const size_t row = (size_t)M.sy * M.YW;
    if (pair_ok) {
        *reinterpret_cast<float2*>(yp) = make_float2(y00, y01);
        if (oh + 1 < OH) *reinterpret_cast<float2*>(yp + row) = make_float2(y10, y11);
    } else {
        yp[0] = y00;
        if (ow + 1 < OW) yp[M.sx] = y01;
        if (oh + 1 < OH) {
            yp[row] = y10;
            if (ow + 1 < OW) yp[row + M.sx] = y11;
        }
    }
}
#endif

// exact floor(n / d) for 0 <= n < 2^31, d >= 1, without a division
struct FastDiv {
    unsigned mul, shift;
    void init(unsigned d)
    {
        shift = 0;
        while ((1u << shift) < d) ++shift;
        mul = (unsigned)((((unsigned long long)1 << 32) * ((1ull << shift) - d)) / d + 1);
    }
#ifdef __HIPCC__
    __device__ __forceinline__ int div(int n) const
    {
        return (int)((__umulhi((unsigned)n, mul) + (unsigned)n) >> shift);
    }
#endif
};

// Geometry of the single-kernel forward path (fused.hip).  A wave owns 16
// tiles and 32 filters at a time; the pieces of 2 and 3 taps of a dimension form one family
// that shares the four F(2,3) frequencies (a 2-tap piece is a 3-tap piece whose last tap is
// zero: its fourth frequency vanishes and is skipped), one-tap pieces form the other.  A
// "class" here is a pair of families; its parts are ordered by (len_h, len_w) in groups whose
// rows (part, channel) are padded to a multiple of four, the reduction depth of one MFMA step.
constexpr int kFusedMaxSteps = 64;
constexpr int kFusedMaxRows = 4 * kFusedMaxSteps;
struct FusedClass {
    int wide_h, wide_w;  // 1: pieces of 2 or 3 taps (four frequencies), 0: one-tap pieces (two)
    int nfh, nfw;        // frequencies per dimension: 4 or 2
    int step0, nsteps;   // steps of four rows
    int row0, rows;      // first row, rows (a multiple of 4)
    long long uf_off;    // floats from the start of Ugw: UF[slice][plane][row][16 filters][2 halves]
};
struct FusedArgs {
    int BH, BW, nbh, nbw;           // block of tiles owned by a workgroup (BH*BW <= 64), blocks per image
    int nphase, lwp, lw_in, nrows;  // staged input region: 2*stride phases, floats per (row, phase), columns, rows
    int row_floats, chan_floats;    // LDS floats per staged row / per channel
    int tile_row_step;              // LDS floats between vertically adjacent tiles' patches
    int nslices;                    // ceil(K / 32)
    int slices_per_wg, nkw;         // K slices per workgroup, workgroups along K
    int wide;                       // 1: one class of two- and three-tap pieces only: patch rows are read as
                                    // pairs of adjacent words and operands are carried from slice to slice
    int nfc, rows_total;
    FusedClass fc[4];
    FastDiv div_bw, div_nphase;
    int roff[kMaxPieces][4], coff[kMaxPieces][4];  // LDS offset of patch row a / column b of a piece
    int step_type[kFusedMaxSteps];                    // len_h * 4 + len_w of the step's four rows
    unsigned short rowdesc[kFusedMaxRows];            // h piece | w piece << 4 | channel << 8 | real row << 15
    size_t lds_bytes;
};

// Geometry of the 16-bit single-kernel forward path (half_impl.inc), for layers with few input
// channels.  The decomposition is the 16-bit path's own (the kernel cut exactly as eq. 8 writes
// it; a class = the parts of one (len_h, len_w) with (len_h+1)(len_w+1) planes).  A wave owns 16
// tiles; a step is 16 reduction rows (part, channel) of one class -- the depth of the 16-bit
// 16x16x16 MFMA, four rows per lane -- and the products go straight into the 2x2 outputs: an
// output takes one MFMA for every plane whose A^T coefficient for it is not zero, with the sign on
// the transformed input.
constexpr int kF16MaxRows = 512;  // rows of all classes, each class padded to a multiple of 16
struct Fused16Class {
    int lh, lw;
    int row0, nsteps;   // first row in the padded row space, steps of 16 rows
    int L;              // real rows: parts * C
    int pad_;
    long long uf_off;   // 16-bit elements from the start of U: [block of 16 filters][step][plane][lane][4]
};
struct Fused16Args {
    int BH, BW, nbh, nbw;            // block of tiles of a workgroup (BH*BW <= 64), blocks per image
    int nphase, lwp, lw_in, nrows;   // staged input region: 2*stride column phases, floats per (row, phase), columns, rows
    int row_floats, chan_floats, tile_row_step;
    int patch_row_bytes;             // LDS bytes between the rows of a patch: stride * row_floats * 4
    int eff_pct;                     // lanes of a workgroup that hold a tile, in percent
    int nkb, slice_kb, nslices;      // blocks of 16 filters; blocks per pass over the classes and passes (set at launch)
    int ncls, rows_total;
    Fused16Class cls[kMaxClasses];
    FastDiv div_bw, div_nphase;
    int roff[kMaxPieces];            // LDS floats from a tile's base to row 0 of an h piece's patch
    int coff0[kMaxPieces], coff1[kMaxPieces];  // ... to column 0 / column 1 of a w piece's patch (columns 2, 3: one float on)
    unsigned short rowdesc[kF16MaxRows];       // h piece | w piece << 4 | channel << 8
    size_t lds_bytes, uf_halves;
};
bool fused16_setup(const dwm_plan& p, Fused16Args* out);

// Geometry of the LDS-staged input transform (transforms.hip): a workgroup stages the input
// rows that one 64-tile block needs, for `cg` channels, and builds every part's V from LDS.
struct InLdsArgs {
    int cg, ncg;                     // channels per workgroup, workgroups along C
    int nphase, lwp, lw_in;          // 2*stride phases, floats per (row, phase) (odd), staged columns
    int row_floats, chan_floats;     // LDS floats per staged row / per channel
    int max_rows;                    // most rows any block stages
    int foot_h;                      // rows one tile row needs: 2*stride*(ntr-1) + foot_h for ntr tile rows
    int rows_full;                   // rows of a whole image's tile rows
    FastDiv div_tw, div_th, div_lw, div_nphase, div_rows_full;
    int roff[kMaxPieces][4], coff[kMaxPieces][4];  // LDS offset of patch row a / column b of a piece
    size_t lds_bytes;
};

// Geometry of the single-kernel data gradient for layers with few input channels
// (backward_small.hip).  All phases of the gradient image are computed as ONE stride-1
// correlation of dy: pixel (stride*t + rho) of dx, for every residue rho, is a sum over the same
// window of dy, rows t - Lh .. t - Lh + nwh - 1, with the taps w[stride*(e_rho + Lh - j) + a_rho]
// at window position j (zero where the residue has no such tap).  The "filters" of that
// correlation are the columns f = (c*stride + rho_h)*stride + rho_w, its channels the K channels
// of dy; the window is cut into pieces of two and three taps (Sec. 4.1, eq. 8) and a tile of 2x2
// window positions produces a 2*stride x 2*stride block of every channel of dx.
constexpr int kBsMaxPieces = 4;  // pieces per dimension of the window (at most 11 taps)
constexpr int kBsMaxPairs = kBsMaxPieces * kBsMaxPieces;
constexpr int kBsMaxSlots = 8;   // (group of four channels, staged element) pairs per thread and chunk
struct BwdSmallArgs {
    int N, C, H, W, K, OH, OW, s;
    int nf, ncb;                                // columns C*s*s, blocks of 16 columns
    int nb, ncbp;                               // blocks a wave accumulates at once (1..3); ncb rounded up to whole groups
    int Lh, Lw, nwh, nww;                       // window offset and taps per dimension
    int nph, npw, npp;                          // pieces per dimension, pairs of pieces
    int jh[kBsMaxPieces], lh[kBsMaxPieces];     // first tap and length of the pieces
    int jw[kBsMaxPieces], lw[kBsMaxPieces];
    int ra_h[8], re_h[8], rn_h[8];              // per residue: tap residue a, shift e, taps n (0: none)
    int ra_w[8], re_w[8], rn_w[8];
    int four;                                   // some piece has three taps: four frequencies per dimension
    int TH, TW, BH, BW, nbh, nbw;               // tiles per image, block of tiles of a workgroup, blocks per image
    int eff_pct;                                // lanes of a workgroup that hold a tile, in percent
    // staged region of dy, per group of four channels: two planes (channel pairs) of [row][column parity][lwp]
    // elements of two floats
    int nrows, lw_in, lwp, row_elems, group_elems, tile_row_step;
    int glog, ck;                               // a chunk is 2^glog groups = ck channels of dy
    int nchunks, steps;                         // chunks, MFMA steps per chunk = pairs * groups
    int nelog;                                  // a thread stages 2^nelog elements of every group
    int xs_floats, us_floats;                   // LDS floats of one staged chunk of dy / of the filter copy
    int po0[kBsMaxPairs], po1[kBsMaxPairs];     // per pair of pieces: LDS byte offset of patch column 0 / 1, row 0
    FastDiv div_bw, div_lw;
    size_t lds_bytes, u_floats;
};

// Position of (plane, lane) inside one step of that kernel's filter copy: planes in groups of four, a
// lane's four planes adjacent (one 16-byte LDS read); the planes left over follow, 64 lanes each.
#ifdef __HIPCC__
__host__ __device__
#endif
inline int bs_upos(int planes, int plane, int lane)
{
    const int g4 = planes / 4;
    return plane < 4 * g4 ? (plane >> 2) * 256 + lane * 4 + (plane & 3) : g4 * 256 + (plane - 4 * g4) * 64 + lane;
}

// Several stride-1 sub-convolutions contracted in one launch (contract_batch.hip): their planes
// are concatenated in one PlaneTable, their (K tile, T tile) grids in one grid.
constexpr int kMaxBatch = 16;
struct BatchProb {
    int plane0, n_iter;  // first plane in the table, chunks per tile (sum over its planes of Lpad/LC)
    int tile0, vblock;   // first tile in the grid, floats of one 64-tile block of its V
    OutMap om;
    int OH, OW, TH, TW, T;
    int pad_;
    long long v_base;    // its V, in floats from the start of the workspace
};
struct BatchArgs {
    int K, nkt, nprob, ntiles;
    BatchProb p[kMaxBatch];
};

}  // namespace dwm

// The opaque plan of the C ABI.
struct dwm_plan {
    dwm::DevPlan d;
    dwm::PlaneTable planes;
    dwm_plan_info_t info;
    dwm_part_t parts[dwm::kMaxPieces * dwm::kMaxPieces];
    size_t filter_floats, v_floats;
    dwm::ContractGeometry geo;
    float* ws;
    size_t ws_bytes;
    int lgran;  // every class's Lpad is a multiple of this (16, 32 or 64)
    int variant_input;  // < 0: planner's choice
    int sk_mode;        // how leftover tiles are split (see contract_geometry)
    int variant_forward;  // < 0: planner's choice (single kernel where it applies), 0: staged, 1: single kernel
    bool fused_ok;        // the single-kernel path applies to this layer
    dwm::FusedArgs fused;
    size_t uf_gap, uf_begin;  // end of what precedes its filter copy in Ugw, first float of the copy
    bool inlds_ok;      // the LDS-staged input transform applies (its staged rows fit in LDS)
    bool skip_pad_rows; // the consumer of V never reads the rows past a class's reduction length: the
                        // LDS-staged input transform does not write their zeros
    dwm::InLdsArgs inlds;
    bool use_fused() const { return fused_ok && variant_forward != 0; }

    // workspace layout: [ V | partial outputs | arrival counters ]
    size_t ws_need_bytes() const { return (v_floats + geo.partial_floats) * sizeof(float) + counters_bytes(); }
    size_t counters_bytes() const { return ((size_t)geo.n_sk_tiles * sizeof(int) + 255) / 256 * 256; }
    // (given the workspace's base, so that a call may run on a workspace other than the plan's own)
    float* sk_partial(float* base) const { return base ? base + v_floats : nullptr; }
    int* sk_counters(float* base) const
    {
        return base ? reinterpret_cast<int*>(base + v_floats + geo.partial_floats) : nullptr;
    }
};

namespace dwm {
// What a plan is made from: the layer, where the padded input starts relative to the image,
// the output extent to compute and where the outputs go.
struct PlanSpec {
    int N, C, H, W, K, R, S, stride;
    int pad_h, pad_w;
    int OH, OW;
    OutMap om;
};
dwm_status_t plan_from_spec(dwm_plan_t** out, const PlanSpec& sp);
// For the filter gradient of layers with few channels: phases cut 3,...,3,2,2 and every two-tap
// piece transformed as a three-tap one (its third tap is a neighbour's, or lies past the kernel: the
// gradient of that tap is computed and dropped), so that all parts share the 16 planes of F(2,3)^2.
// Only the input transform and the tables of such a plan are used.
dwm_status_t plan_from_spec_widened(dwm_plan_t** out, const PlanSpec& sp);
// the same with the kernel cut exactly as eq. 8 writes it (3,3,...,remainder), staged path only
dwm_status_t plan_from_spec_as_printed(dwm_plan_t** out, const PlanSpec& sp);
// plan.cpp: geometry of a contraction variant for this plan; false if the variant does not apply
bool contract_geometry(const dwm_plan& p, int variant, ContractGeometry* out);
// transforms.hip, contract.hip
dwm_status_t launch_filter_transform(const dwm_plan& p, const float* w, float* U, void* stream);
// `ws` is the base of a workspace laid out as the plan says: V first, then the partial outputs and
// the arrival counters of the contraction's split tiles
dwm_status_t launch_input_transform(const dwm_plan& p, const float* x, float* ws, void* stream);
dwm_status_t launch_contract_output(const dwm_plan& p, const float* U, float* ws, float* y, void* stream);
bool input_lds_setup(const dwm_plan& p, InLdsArgs* out, int cg_wish);
// contract_batch.hip
dwm_status_t launch_contract_batch(const BatchArgs& a, const PlaneTable& pt, int lc, const float* U, const float* V,
                                   float* y, void* stream);
// setup.cpp / backward_small.hip: the single-kernel data gradient
bool bwd_small_setup(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, BwdSmallArgs* out);
dwm_status_t launch_bwd_small_filter(const BwdSmallArgs& a, int R, int S, const float* w, float* U, void* stream);
dwm_status_t launch_bwd_small(const BwdSmallArgs& a, const float* dy, const float* U, float* dx, void* stream);
// fused.hip
bool fused_setup(const dwm_plan& p, FusedArgs* out);
dwm_status_t launch_fused_filter(const dwm_plan& p, const float* w, float* U, void* stream);
dwm_status_t launch_fused_forward(const dwm_plan& p, const float* x, const float* U, float* y, void* stream);
}  // namespace dwm
