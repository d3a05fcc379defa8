// Internal plan structures shared by the host planner and the kernel launchers.
// Everything a kernel needs about the decomposition travels BY VALUE in its kernel
// arguments (DevPlan / PlaneTable below), so the library owns no device memory.
#pragma once
#include <cstdint>
#include "../../include/dwm.h"

namespace dwm {

constexpr int kMaxPieces = 16;  // one-dimensional pieces per dimension
constexpr int kMaxClasses = 9;  // (len_h, len_w) in {1,2,3}^2
constexpr int kMaxPlanes = 81;  // sum over classes of (len_h+1)(len_w+1) = (2+3+4)^2
constexpr int kKAlign = 128;    // Kpad is a multiple of this (largest K tile of any variant)
constexpr int kTAlign = 256;    // Tpad is a multiple of this (largest T tile of any variant)
constexpr int kLAlign = 16;     // Lpad is a multiple of this (largest reduction chunk)

// A 1-D piece (Sec. 4.1): phase p, offset j inside the phase's tap list, length l.
struct DevPiece {
    int p, j, l;
};

// A class: the parts made of an h-piece of length lh and a w-piece of length lw.
// Pieces are stored sorted by length, so the class's h-pieces are ph[h0 .. h0+hn).
struct DevClass {
    int lh, lw;
    int h0, hn, w0, wn;
    int L, Lpad;
    int row0;    // first row of this class in the flattened (class, l) row space
    int plane0;  // first plane of this class
    long long u_off, v_off;  // floats
};

struct DevPlan {
    int N, C, H, W, K, R, S, s, P;
    int OH, OW, TH, TW;
    int T, Tpad, Kpad;
    int nh, nw;
    int ncls;
    int rows_total;  // sum over classes of Lpad
    DevPiece ph[kMaxPieces];
    DevPiece pw[kMaxPieces];
    DevClass cls[kMaxClasses];
};

// One Winograd-domain plane = (class, fh, fw): a [Kpad x Lpad] slice of U, a
// [Lpad x Tpad] slice of V, and the 2x2 pattern A^T[:,fh] (x) A^T[:,fw] with which its
// product enters the output tile (entries 0, +1, -1; packed two bits each).
struct DevPlaneEntry {
    uint32_t u_off64;  // offset into Ugw in units of 64 floats
    uint32_t v_off64;  // offset into V   in units of 64 floats
    int32_t Lpad;
    int32_t coef;      // bits [2q+1:2q] of output q=2a+b: 0 -> 0, 1 -> +1, 3 -> -1
};

struct PlaneTable {
    int n;
    DevPlaneEntry e[kMaxPlanes];
};

}  // namespace dwm

// The opaque plan of the C ABI.
struct dwm_plan {
    dwm::DevPlan d;
    dwm::PlaneTable planes;
    dwm_plan_info_t info;
    dwm_part_t parts[dwm::kMaxPieces * dwm::kMaxPieces];
    size_t filter_floats, ws_floats;
    float* ws;
    int variant_input, variant_contract;  // < 0: planner's choice
};

namespace dwm {
// kernels.hip
dwm_status_t launch_filter_transform(const dwm_plan& p, const float* w, float* U, void* stream);
dwm_status_t launch_input_transform(const dwm_plan& p, const float* x, float* V, void* stream);
dwm_status_t launch_contract_output(const dwm_plan& p, const float* U, const float* V, float* y, void* stream);
}  // namespace dwm
