// How the Winograd-domain products decompose into int8 matrix-core GEMMs for the
// staged contraction kernel.  The work is cut into "units"; each unit is a short
// list of sub-products (activation plane x filter plane, summed over all input
// channels) whose weighted sum is one int32 plane of the workspace array M.
//
// Lossless: one unit per real 12-bit x 12-bit product, 46 in all (Section 3.4:
// 16 real entries + 10 complex entries x the three products of Section 3.1).
// With v = 64 h + l on both sides,
//     d*w = 4096 hh + 64 (ss - hh - ll) + ll = 4032 hh - 63 ll + 64 ss,   s = h + l,
// i.e. three int8 sub-products per unit (limb-level three-multiplication split).
// Unit q reads planes 3q, 3q+1, 3q+2 on both sides and writes plane q:
//   q < 16: the real entry q;   q = 16 + 3j + g: P1 = Dr Wr, P2 = Di Wi, P3 = (Dr+Di)(Wr+Wi)
//   of complex entry j; the output transform forms Re = P1 - P2, Im = P3 - P1 - P2 after
//   the channel sum, so the partial products stay separate until then (Section 3.4).
//
// Scaled (Section 4.2): filters are single int8 limbs, activations two limbs; Wr +- Wi would need
// nine bits, so a complex product is taken as its four real products.  36 units = the 36 planes:
//   u < 16: real entry u:  64 (Dh W) + (Dl W);
//   u = 16 + 2j + part: Re = Dr Wr + Di (-Wi), Im = Dr Wi + Di Wr of complex entry j, each with
//   the high-limb sub-products weighted by 64; the reciprocal r/2^q is applied to the finished sum.
#pragma once
#include "wg_internal.h"

namespace wg {

struct SubProduct {
    int a_plane, b_plane, weight;
};

__host__ __device__ constexpr int limb_weight(int limb) { return limb == 0 ? 4032 : (limb == 1 ? -63 : 64); }

template <int MODE> __host__ __device__ constexpr int num_units() { return MODE == WG_LOSSLESS ? 46 : 36; }

template <int MODE>
__host__ __device__ constexpr int num_subproducts(int unit) {
    return MODE == WG_LOSSLESS ? 3 : (unit < kRealEntries ? 2 : 4);
}

// the free entry (0..25) a unit belongs to (its row of the scaling table)
template <int MODE>
__host__ __device__ constexpr int unit_entry(int unit) {
    if (unit < kRealEntries) return unit;
    return MODE == WG_LOSSLESS ? kRealEntries + (unit - kRealEntries) / 3 : kRealEntries + (unit - kRealEntries) / 2;
}

template <int MODE>
__host__ __device__ constexpr SubProduct subproduct(int unit, int s) {
    SubProduct sp = {0, 0, 0};
    if (MODE == WG_LOSSLESS) {
        sp.a_plane = sp.b_plane = 3 * unit + s;
        sp.weight = limb_weight(s);
    } else if (unit < kRealEntries) {
        sp.a_plane = 2 * unit + s;      // high, low limb of D
        sp.b_plane = unit;
        sp.weight = s == 0 ? 64 : 1;
    } else {
        // activation planes 32+4j+{Re hi, Re lo, Im hi, Im lo}; filter planes 16+3j+{Re, Im, -Im}
        const int j = (unit - kRealEntries) >> 1, part = (unit - kRealEntries) & 1;
        const int d_is_im = s & 1, limb = s >> 1;     // order: (Dr hi, Di hi, Dr lo, Di lo)
        sp.a_plane = 32 + 4 * j + 2 * d_is_im + limb;
        sp.b_plane = 16 + 3 * j + (part == 0 ? (d_is_im ? 2 : 0) : (d_is_im ? 0 : 1));
        sp.weight = limb == 0 ? 64 : 1;
    }
    return sp;
}

// Planes of M: lossless 46 (one per unit), scaled 36.
__host__ __device__ inline int num_accumulator_planes(int mode) { return mode == WG_LOSSLESS ? 46 : 36; }

}  // namespace wg
