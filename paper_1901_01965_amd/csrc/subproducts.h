// How each Winograd-domain entry's product decomposes into int8 matrix-core
// sub-products, shared by the staged contraction kernel and the fused kernel.
#pragma once
#include "wg_internal.h"

namespace wg {

// One matrix-core sub-product: activation plane x filter plane, and the integer
// weights with which its channel sum enters Re and Im of the entry.
struct SubProduct {
    int a_plane, b_plane, w_re, w_im;
};

// v = 64 h + l on both sides gives  d*w = 4096 hh + 64 (ss - hh - ll) + ll
//                                       = 4032 hh - 63 ll + 64 ss,   s = h + l
// (the three-multiplication split of Section 3.1 applied to limbs).
__host__ __device__ constexpr int limb_weight(int limb) { return limb == 0 ? 4032 : (limb == 1 ? -63 : 64); }

template <int MODE>
__host__ __device__ constexpr int num_subproducts(int entry) {
    return MODE == WG_LOSSLESS ? (entry < kRealEntries ? 3 : 9) : (entry < kRealEntries ? 2 : 8);
}

template <int MODE>
__host__ __device__ constexpr SubProduct subproduct(int entry, int s) {
    SubProduct sp = {0, 0, 0, 0};
    if (MODE == WG_LOSSLESS) {
        if (entry < kRealEntries) {
            sp.a_plane = sp.b_plane = 3 * entry + s;
            sp.w_re = limb_weight(s);
            sp.w_im = 0;
        } else {
            // values 16+3j+{0,1,2} = Re, Im, Re+Im:  P1 = Dr Wr, P2 = Di Wi, P3 = (Dr+Di)(Wr+Wi)
            //   Re = P1 - P2,  Im = P3 - P1 - P2     (Section 3.1)
            const int j = entry - kRealEntries, g = s / 3, limb = s % 3;
            sp.a_plane = sp.b_plane = 3 * (16 + 3 * j + g) + limb;
            const int lw = limb_weight(limb);
            sp.w_re = g == 0 ? lw : (g == 1 ? -lw : 0);
            sp.w_im = g == 2 ? lw : -lw;
        }
    } else {
        if (entry < kRealEntries) {
            sp.a_plane = 2 * entry + s;      // high, low limb of D
            sp.b_plane = entry;
            sp.w_re = s == 0 ? 64 : 1;
            sp.w_im = 0;
        } else {
            // activation planes 32+4j+{Re hi, Re lo, Im hi, Im lo}; filter planes 16+3j+{Re, Im, -Im}
            //   Re = Dr Wr + Di (-Wi),  Im = Dr Wi + Di Wr
            const int j = entry - kRealEntries;
            const int part = s >> 2;          // 0: Re, 1: Im
            const int d_is_im = (s >> 1) & 1; // which D component
            const int limb = s & 1;
            sp.a_plane = 32 + 4 * j + 2 * d_is_im + limb;
            const int wsel = part == 0 ? (d_is_im ? 2 : 0) : (d_is_im ? 0 : 1);
            sp.b_plane = 16 + 3 * j + wsel;
            const int lw = limb == 0 ? 64 : 1;
            sp.w_re = part == 0 ? lw : 0;
            sp.w_im = part == 0 ? 0 : lw;
        }
    }
    return sp;
}

}  // namespace wg
