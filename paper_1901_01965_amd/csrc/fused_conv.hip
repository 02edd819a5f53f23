// The whole hot path in one kernel: input transform (Section 3.3-3.4) of a block
// of 16 tiles into int8 operand planes held in LDS, the Winograd-domain
// products of Section 3.4 against 32 filters on the int8 matrix cores, and the
// output transform accumulated on the fly, so neither the transformed
// activations nor the 36 accumulator planes ever travel through HBM.
//
// The output transform Y = A^T M A is linear in M, and M is a sum over input
// channels, so each finished row of M (for one 64-channel block) is reduced by
// the row rule of A^T at once and added into the 16 outputs of the tile.  That is
// valid for any number of channel blocks in lossless mode.  The reverse scaling of
// Section 4.2 is not linear (it rounds): with more than one channel block, scaled
// mode keeps the channel sums of all of a wave's entries in registers (18 sums of
// four registers per wave) across the channel blocks and scales and reduces them
// once at the end.
//
// This kernel is bound by vector ALU work (transform, limb re-assembly, output
// transform) and memory latency, not by the matrix cores, so it trades
// multiplications for vector work and traffic: a 12-bit x 12-bit
// product is taken as the four limb products hh, hl, lh, ll (two activation and
// two filter planes per value) and a complex product as its four real products,
// instead of the three-multiplication forms of Section 3.1 that the staged
// contraction kernel uses; those would need half again as many operand planes.
#include <atomic>
#include <type_traits>
#include <utility>

#include "kernel_common.h"

namespace wg {
namespace {


constexpr int kFusedTiles = kTileBlock;   // tiles per workgroup (rows of the 16x16x64 matrix-core product)
constexpr int kFusedFilters = 32;   // filters per workgroup: two 16-wide column blocks
constexpr int kFusedPlanes = 72;    // two-limb activation planes (kSplitTwoLimb)
constexpr int kLdsBytes = kFusedPlanes * kPlaneBytes;
constexpr int kParkBytes = 4 * 16 * 64 * 16;         // four waves x 16 outputs x 64 lanes x 4 registers
// How the activation patch reaches the transform threads (chosen on the host):
//   kLoadBytes:  one byte per load, any layout and channel count;
//   kLoadDwords: channels-last, C a multiple of 4: one 4-byte load per pixel and thread;
//   kLoadDirect: channels-last, C a multiple of 16, 16-byte aligned input: 16-byte pieces travel
//                from global memory straight into LDS (nine instructions per wave instead of
//                thirty-six), and the threads pick their four channels from there.
constexpr int kLoadBytes = 0, kLoadDwords = 1, kLoadDirect = 2;
constexpr int kRawWaveBytes = 4 * 36 * kCBlock;      // raw patches of a wave's four tiles: 36 pixels x 64 channels
constexpr int kRawBytes = 4 * kRawWaveBytes;
static_assert(kParkBytes <= kLdsBytes, "output staging reuses the operand planes' LDS");

// ---- per-entry programs ----------------------------------------------------------------
// An entry's product uses a few activation fragments (from LDS) and filter fragments (from
// the packed blob) and a short list of matrix-core instructions into a few accumulators.
//   lossless, real:    A = (h, l)  B = (h, l)          acc = (hh, hl+lh, ll)
//   lossless, complex: A = (Re h, Re l, Im h, Im l)  B = (Wr h, Wr l, Wi h, Wi l)
//                      acc 0-2: Dr*Wr, 3-5: Di*Wi, 6-8: Dr*Wi + Di*Wr, each as (hh, mid, ll)
//   scaled, real:      A = (h, l)  B = (W)             acc = (h, l)
//   scaled, complex:   B = (Wr, Wi, -Wi)               acc = (Re h, Re l, Im h, Im l)
//   scaled, complex, without the -Wi plane (kScaledTwoPlanes as MODE of the helpers below: a
//   third less filter traffic per complex entry for two subtractions per register):
//                      B = (Wr, Wi)                    acc = (Dr*Wr h, l, Im h, Im l, Di*Wi h, l)
constexpr int kScaledTwoPlanes = 2;
static_assert(kScaledTwoPlanes != WG_LOSSLESS && kScaledTwoPlanes != WG_SCALED, "a value of its own");
struct Op {
    int a, b, acc;
    bool init;   // first instruction into this accumulator (starts from zero)
};
constexpr bool is_real(int entry) { return entry < kRealEntries; }
template <int MODE> constexpr int num_a(int entry) { return is_real(entry) ? 2 : 4; }
template <int MODE> constexpr int num_b(int entry) {
    return MODE == WG_LOSSLESS ? (is_real(entry) ? 2 : 4) : (is_real(entry) ? 1 : (MODE == kScaledTwoPlanes ? 2 : 3));
}
template <int MODE> constexpr int num_ops(int entry) {
    return MODE == WG_LOSSLESS ? (is_real(entry) ? 4 : 16) : (is_real(entry) ? 2 : 8);
}
template <int MODE> constexpr int a_plane(int entry, int i) {
    return is_real(entry) ? 2 * entry + i : 32 + 4 * (entry - kRealEntries) + i;
}
template <int MODE> constexpr int b_plane(int entry, int i) {
    if (MODE == WG_LOSSLESS) {   // blob planes 3*value + {0: high limb, 1: low limb}
        if (is_real(entry)) return 3 * entry + i;
        const int value = 16 + 3 * (entry - kRealEntries) + (i >> 1);   // Re, then Im
        return 3 * value + (i & 1);
    }
    return is_real(entry) ? entry : 16 + 3 * (entry - kRealEntries) + i;
}
template <int MODE> constexpr Op entry_op(int entry, int i) {
    constexpr Op lossless_real[4] = {{0, 0, 0, true}, {0, 1, 1, true}, {1, 1, 2, true}, {1, 0, 1, false}};
    // dependent instructions into one accumulator are kept at least three apart
    constexpr Op lossless_complex[16] = {
        {0, 0, 0, true}, {0, 1, 1, true}, {1, 1, 2, true},    // Dr*Wr: hh, mid, ll
        {2, 2, 3, true}, {2, 3, 4, true}, {3, 3, 5, true},    // Di*Wi
        {0, 2, 6, true}, {0, 3, 7, true}, {1, 3, 8, true},    // Dr*Wi
        {1, 2, 7, false}, {1, 0, 1, false}, {3, 2, 4, false},
        {2, 1, 7, false}, {2, 0, 6, false}, {3, 1, 8, false}, {3, 0, 7, false}};
    constexpr Op scaled_real[2] = {{0, 0, 0, true}, {1, 0, 1, true}};
    constexpr Op scaled_complex[8] = {{0, 0, 0, true}, {1, 0, 1, true}, {0, 1, 2, true}, {1, 1, 3, true},
                                      {2, 2, 0, false}, {3, 2, 1, false}, {2, 0, 2, false}, {3, 0, 3, false}};
    constexpr Op two_planes_complex[8] = {{0, 0, 0, true}, {1, 0, 1, true}, {0, 1, 2, true}, {1, 1, 3, true},
                                          {2, 1, 4, true}, {3, 1, 5, true}, {2, 0, 2, false}, {3, 0, 3, false}};
    if (MODE == WG_LOSSLESS) return is_real(entry) ? lossless_real[i] : lossless_complex[i];
    if (MODE == kScaledTwoPlanes) return is_real(entry) ? scaled_real[i] : two_planes_complex[i];
    return is_real(entry) ? scaled_real[i] : scaled_complex[i];
}

// ---- which entries a wave owns, in order ---------------------------------------------------
// Half 0 owns rows 0,1,2 of M, half 1 rows 5 and 3; "half" 2 is all five rows, for a wave that
// owns every entry.  A real row RI (rows 0,1,2,5) holds entries 4RI..4RI+3 and the complex
// entry 16+RI; the complex row holds entries 20..25.
constexpr int kAllRows = 2;
constexpr int row_entries(int row) { return row < 4 ? 5 : 6; }
constexpr int row_entry(int row, int pos) {
    return row < 4 ? (pos < 4 ? 4 * row + pos : kRealEntries + row) : kRealEntries + 4 + pos;
}
constexpr int half_rows(int half) { return half == 0 ? 3 : (half == 1 ? 2 : 5); }
constexpr int half_row(int half, int i) { return half == 1 ? (i == 0 ? 3 : 4) : i; }
constexpr int half_entries(int half) { return half == 0 ? 15 : (half == 1 ? 11 : 26); }
struct Slot {
    int entry, row, pos;
    bool last_in_row;
};
constexpr Slot half_slot(int half, int i) {
    int n = 0;
    for (int r = 0; r < half_rows(half); ++r) {
        const int row = half_row(half, r);
        if (i < n + row_entries(row))
            return Slot{row_entry(row, i - n), row, i - n, i - n == row_entries(row) - 1};
        n += row_entries(row);
    }
    return Slot{0, 0, 0, false};
}
// index of the first filter fragment of slot i in the wave's fragment stream
template <int MODE> constexpr int b_start(int half, int i) {
    int n = 0;
    for (int s = 0; s < i; ++s) n += num_b<MODE>(half_slot(half, s).entry);
    return n;
}
// the slot that filter fragment f of the stream belongs to
template <int MODE> constexpr int b_slot_of(int half, int f) {
    int s = 0;
    while (b_start<MODE>(half, s + 1) <= f) ++s;
    return s;
}

// Direct global -> LDS transfer of the raw 6x6 patches of a wave's four tiles (one 64-channel
// block).  Instruction i (0..8) moves pixels 4i..4i+3 of the patch (pixel = 6 a + b): lane l
// carries 16 channels (piece l % 4) of tile (l % 16) / 4 at pixel 4i + l / 16, and the hardware
// puts lane l's piece at (wave-uniform destination) + 16 l.  The raw area of a wave is therefore
// [pixel][tile][64 channels], and transform thread (tile, channel quad) = lane reads its pixel
// p at p * 256 + 4 * lane: a wave reads 256 contiguous bytes.
struct DirectPatch {
    uint32_t pixel_off[9];   // byte offset of this lane's pixel (channel 0) for each instruction
    // (n, ty, tx): the tile this lane moves pieces of.  With j = lane / 16, instruction i covers
    // pixel 4i + j = 6a + b of the patch: a = {0,0,1,2,2,3,4,4,5}[i] + (i % 3 == 1 and j >= 2),
    // and b takes only three values per lane: j (i % 3 == 0), (j + 4) % 6 (i % 3 == 1) and j + 2
    // (i % 3 == 2).  Row terms follow each other by one clamped row step, so the whole table
    // costs four multiplications.
    __device__ inline void init(const Problem& p, int n, int ty, int tx, int lane) {
        const int h0 = 4 * ty - 1, w0 = 4 * tx - 1, j = lane >> 4;
        const uint32_t row_step = (uint32_t)(p.W * p.C);
        uint32_t row_term[6];
        row_term[0] = (uint32_t)(n * p.H + max(h0, 0)) * row_step;
#pragma unroll
        for (int a = 1; a < 6; ++a)   // rows clamp to [0, H-1]: the step is taken only inside the image
            row_term[a] = row_term[a - 1] + ((unsigned)(h0 + a - 1) < (unsigned)(p.H - 1) ? row_step : 0u);
        const int b1 = j < 2 ? j + 4 : j - 2;
        const uint32_t col_term[3] = {(uint32_t)(min(max(w0 + j, 0), p.W - 1) * p.C),
                                      (uint32_t)(min(max(w0 + b1, 0), p.W - 1) * p.C),
                                      (uint32_t)(min(max(w0 + j + 2, 0), p.W - 1) * p.C)};
        constexpr int a_base[9] = {0, 0, 1, 2, 2, 3, 4, 4, 5};
#pragma unroll
        for (int i = 0; i < 9; ++i) {
            uint32_t row = row_term[a_base[i]];
            if (i % 3 == 1) row = j >= 2 ? row_term[a_base[i] + 1] : row;
            pixel_off[i] = row + col_term[i % 3];
        }
    }
    // Pieces beyond C (the last channel block of a C that is not a multiple of 64) re-read
    // channel 0; bias_patch() discards them.
    __device__ inline void issue(const int8_t* __restrict__ x, const Problem& p, int cb, int lane,
                                 int8_t* raw_wave) const {
        const int c = cb * kCBlock + (lane & 3) * 16;
        const int8_t* src = x + (c < p.C ? c : 0);
#pragma unroll
        for (int i = 0; i < 9; ++i) __builtin_amdgcn_global_load_lds(src + pixel_off[i], raw_wave + i * 1024, 16, 0, 0);
    }
    __device__ inline static void read(const int8_t* raw_wave, int lane, uint32_t u[6][6]) {
#pragma unroll
        for (int a = 0; a < 6; ++a)
#pragma unroll
            for (int b = 0; b < 6; ++b)
                u[a][b] = *reinterpret_cast<const uint32_t*>(raw_wave + (6 * a + b) * 256 + 4 * lane);
    }
};

struct LaneContext {
    const int8_t* a_lds;        // this lane's 16-byte slot in plane 0
    const int8_t* b_glob;       // this lane's 16 bytes of filter plane 0, current channel block
    const ScaleEntry* table_k;  // scaling table row of this lane's filter (scaled mode)
    const uint32_t* parked;     // role-specialised kernels, scaled mode: see park_scales
};

constexpr int kFilterPrefetch = 16;   // filter fragments in flight per wave (covers L2 latency)

// value = 4096 hh + 64 mid + ll, modulo 2^32, as two shift-and-add instructions per register.
// The empty statement only pins the intermediate value, so that the compiler does not rewrite
// the expression as two shifts and a three-operand add.
__device__ inline v4i join_limbs(v4i hh, v4i mid, v4i ll) {
    v4i out;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int t = (hh[q] << 6) + mid[q];
        asm("" : "+v"(t));
        out[q] = (t << 6) + ll[q];
    }
    return out;
}

template <int MODE, int HALF>
struct ProductPhase {
    static constexpr int NE = half_entries(HALF);
    static constexpr int NB = b_start<MODE>(HALF, NE);
    static constexpr int NPRE = NB < kFilterPrefetch ? NB : kFilterPrefetch;
    v4i bring[kFilterPrefetch];

    // F-th filter fragment of this wave's stream.  A workgroup that covers more than 32 filters
    // goes through its entries once per 32 (pass F / NB); the wave's 16-filter fragment of the
    // next pass lies two fragments (2 * planes KB) further on in the blob.
    template <int F>
    __device__ inline static v4i load_b(const LaneContext& cx) {
        constexpr int pass = F / NB, f = F % NB;
        constexpr int slot = b_slot_of<MODE>(HALF, f);
        constexpr int plane = b_plane<MODE>(half_slot(HALF, slot).entry, f - b_start<MODE>(HALF, slot));
        constexpr int planes = MODE == WG_LOSSLESS ? 138 : 46;
        return *reinterpret_cast<const v4i*>(cx.b_glob + (pass * 2 * planes + plane) * kFilterFragBytes);
    }
    template <int SLOT, int I>
    __device__ inline static v4i load_a(const LaneContext& cx) {
        constexpr int plane = a_plane<MODE>(half_slot(HALF, SLOT).entry, I);
        return *reinterpret_cast<const v4i*>(cx.a_lds + plane * kPlaneBytes);
    }

    // Filter fragments do not depend on the transform phase: start them before it.
    __device__ inline void prefetch(const LaneContext& cx) {
        static_for<NPRE>([&](auto I) { bring[I] = load_b<I>(cx); });
    }
    static_assert(NB >= kFilterPrefetch || MODE != WG_LOSSLESS, "the ring is full from the first pass on");

    // One 64-channel block of this wave's rows.  Software pipeline over entries: while entry i's
    // matrix-core instructions run, entry i+1's activation fragments come from LDS, the filter
    // ring is refilled sixteen fragments ahead, and entry i-1's accumulators are joined,
    // (un)scaled and reduced into the outputs.
    // PASS of NPASS: which 32 of the workgroup's filters (see load_b).
    template <int PASS = 0, int NPASS = 1>
    __device__ inline void run(const LaneContext& cx, v4i (&Y)[16]) {
        constexpr int F0 = PASS * NB, FEND = NPASS * NB;   // this pass's place in the fragment stream
        v4i afr[2][4], acc[2][9], er[6], ei[6];
        static_for<num_a<MODE>(half_slot(HALF, 0).entry)>([&](auto I) { afr[0][I] = load_a<0, I>(cx); });
        static_for<NE + 1>([&](auto S) {
            constexpr int s = S;
            if constexpr (s < NE) {
                constexpr int entry = half_slot(HALF, s).entry;
                constexpr int b0 = b_start<MODE>(HALF, s);
                if constexpr (s + 1 < NE)
                    static_for<num_a<MODE>(half_slot(HALF, s + 1).entry)>(
                        [&](auto I) { afr[(s + 1) & 1][I] = load_a<s + 1, I>(cx); });
                static_for<num_ops<MODE>(entry)>([&](auto I) {
                    constexpr Op op = entry_op<MODE>(entry, I);
                    constexpr v4i zero = {0, 0, 0, 0};
                    acc[s & 1][op.acc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                        afr[s & 1][op.a], bring[(F0 + b0 + op.b) % kFilterPrefetch],
                        op.init ? zero : acc[s & 1][op.acc], 0, 0, 0);
                });
                static_for<num_b<MODE>(entry)>([&](auto I) {
                    if constexpr (F0 + b0 + I + kFilterPrefetch < FEND)
                        bring[(F0 + b0 + I) % kFilterPrefetch] = load_b<F0 + b0 + I + kFilterPrefetch>(cx);
                });
            }
            if constexpr (s > 0) {
                constexpr Slot sl = half_slot(HALF, s - 1);
                const v4i(&a)[9] = acc[(s - 1) & 1];
                v4i re, im = {0, 0, 0, 0};
                if constexpr (MODE == WG_LOSSLESS) {
                    if constexpr (is_real(sl.entry)) {
                        re = join_limbs(a[0], a[1], a[2]);
                    } else {   // Re = Dr Wr - Di Wi,  Im = Dr Wi + Di Wr
                        re = join_limbs(a[0] - a[3], a[1] - a[4], a[2] - a[5]);
                        im = join_limbs(a[6], a[7], a[8]);
                    }
                } else {
                    re = (a[0] << kByteLimbShift) + a[1];
                    if constexpr (!is_real(sl.entry)) im = (a[2] << kByteLimbShift) + a[3];
                    const ReverseScale unscale(cx.table_k[PASS * kFusedFilters * kEntries + sl.entry]);   // Section 4.2
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        re[q] = unscale(re[q]);
                        if constexpr (!is_real(sl.entry)) im[q] = unscale(im[q]);
                    }
                }
                er[sl.pos] = re;
                ei[sl.pos] = im;
                if constexpr (sl.last_in_row) finish_row<sl.row>(er, ei, Y);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
};

// Role-specialised kernels, scaled mode: the reverse-scaling factors (r, q) of the entries a
// product wave owns, read once at the start of the kernel (while the wave would only wait for
// the first operand planes) and parked in LDS as q << 8 | r, [slot][filter of the wave], so that
// the reverse scaling after the last channel block does not begin with a trip to L2.  Lane
// group g = lane / 16 reads slots g, 4 + g, 8 + g, 12 + g of filter lane % 16: ask() issues the
// four loads, park() writes what they brought, and a caller puts its first filter prefetch
// between the two so that one wait covers both.  Each wave writes and later reads its own 1 KB
// (16 slots x 16 filters; 2 KB for a wave that owns all 26 entries), in program order: no barrier.
constexpr int kParkedScaleBytes = 16 * 16 * 4;
template <int HALF>
struct ParkedScales {
    static constexpr int NE = ProductPhase<WG_SCALED, HALF>::NE;
    static constexpr int kRounds = (NE + 3) / 4;   // a wave that owns every entry: seven loads per lane, 2 KB
    static constexpr int kBytes = kRounds * 4 * 16 * 4;
    int2 rq[kRounds];
    __device__ inline void ask(const LaneContext& cx, int lane) {
        const int g = lane >> 4;
        static_for<kRounds>([&](auto J) {
            int entry = half_slot(HALF, 4 * J).entry;   // slot 4 J + g, clamped to the last slot
            static_for<3>([&](auto G) {
                constexpr int slot = 4 * J + G + 1 < NE ? 4 * J + G + 1 : NE - 1;
                if (g > G) entry = half_slot(HALF, slot).entry;
            });
            rq[J] = *reinterpret_cast<const int2*>(&cx.table_k[entry].r);
        });
    }
    __device__ inline void park(LaneContext& cx, int8_t* area, int lane) {
        uint32_t* const base = reinterpret_cast<uint32_t*>(area) + (lane & 15);
        const int g = lane >> 4;
        static_for<kRounds>([&](auto J) {
            if (4 * J + g < NE) base[(4 * J + g) * 16] = ((uint32_t)rq[J].y << 8) | (uint32_t)rq[J].x;   // r <= 255, q <= 7
        });
        cx.parked = base;
    }
};
template <int SLOT>
__device__ inline ReverseScale parked_scale(const LaneContext& cx) {
    const uint32_t v = cx.parked[SLOT * 16];
    return ReverseScale((int)(v & 0xffu), (int)(v >> 8));
}

// Scaled mode over several channel blocks: the products of every entry a wave owns accumulate
// in registers across the blocks (run, once per block), and the reverse scaling and the output
// transform are applied to the finished channel sums (finish, once).
template <int HALF>
struct ScaledSums {
    static constexpr int MODE = WG_SCALED;
    using Phase = ProductPhase<MODE, HALF>;
    static constexpr int NE = Phase::NE, NB = Phase::NB;
    static constexpr int sum_start(int slot) {   // first sum of a slot: one per real entry, Re and Im per complex
        int n = 0;
        for (int s = 0; s < slot; ++s) n += is_real(half_slot(HALF, s).entry) ? 1 : 2;
        return n;
    }
    static constexpr int kSums = sum_start(NE);

    // One channel block: each entry's limb products are formed from zero, and its value
    // 256 * high + low (byte limbs) joins the entry's running sum one entry later.
    template <int PASS = 0, int NPASS = 1>
    __device__ inline static void run(const LaneContext& cx, v4i (&bring)[kFilterPrefetch], v4i (&sums)[kSums]) {
        constexpr int F0 = PASS * NB, FEND = NPASS * NB;   // this pass's place in the fragment stream
        v4i afr[2][4], acc[2][4];
        static_for<num_a<MODE>(half_slot(HALF, 0).entry)>([&](auto I) { afr[0][I] = Phase::template load_a<0, I>(cx); });
        static_for<NE + 1>([&](auto S) {
            constexpr int s = S;
            if constexpr (s < NE) {
                constexpr int entry = half_slot(HALF, s).entry;
                constexpr int b0 = b_start<MODE>(HALF, s);
                if constexpr (s + 1 < NE)
                    static_for<num_a<MODE>(half_slot(HALF, s + 1).entry)>(
                        [&](auto I) { afr[(s + 1) & 1][I] = Phase::template load_a<s + 1, I>(cx); });
                static_for<num_ops<MODE>(entry)>([&](auto I) {
                    constexpr Op op = entry_op<MODE>(entry, I);
                    constexpr v4i zero = {0, 0, 0, 0};
                    acc[s & 1][op.acc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                        afr[s & 1][op.a], bring[(F0 + b0 + op.b) % kFilterPrefetch],
                        op.init ? zero : acc[s & 1][op.acc], 0, 0, 0);
                });
                static_for<num_b<MODE>(entry)>([&](auto I) {
                    if constexpr (F0 + b0 + I + kFilterPrefetch < FEND)
                        bring[(F0 + b0 + I) % kFilterPrefetch] = Phase::template load_b<F0 + b0 + I + kFilterPrefetch>(cx);
                });
            }
            if constexpr (s > 0) {
                constexpr int v = sum_start(s - 1);
                const v4i(&a)[4] = acc[(s - 1) & 1];
                sums[v] += (a[0] << kByteLimbShift) + a[1];
                if constexpr (!is_real(half_slot(HALF, s - 1).entry)) sums[v + 1] += (a[2] << kByteLimbShift) + a[3];
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }

    // After the last channel block: reverse scaling of the finished sums and the output transform.
    template <int PASS = 0, bool PARKED = false>
    __device__ inline static void finish(const LaneContext& cx, const v4i (&sums)[kSums], v4i (&Y)[16]) {
        v4i er[6], ei[6];
        static_for<NE>([&](auto S) {
            constexpr Slot sl = half_slot(HALF, S);
            constexpr int v = sum_start(S);
            v4i re = sums[v], im = {0, 0, 0, 0};
            if constexpr (!is_real(sl.entry)) im = sums[v + 1];
            const ReverseScale unscale = PARKED ? parked_scale<S>(cx)   // Section 4.2
                                                : ReverseScale(cx.table_k[PASS * kFusedFilters * kEntries + sl.entry]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                re[q] = unscale(re[q]);
                if constexpr (!is_real(sl.entry)) im[q] = unscale(im[q]);
            }
            er[sl.pos] = re;
            ei[sl.pos] = im;
            if constexpr (sl.last_in_row) {
                finish_row<sl.row>(er, ei, Y);
                // all rows in one wave: row by row, so that a row's sums are dead before the next row's work begins
                if constexpr (HALF == kAllRows) __builtin_amdgcn_sched_barrier(0);
            }
        });
    }
};
constexpr int kChannelSums = 18;
static_assert(ScaledSums<0>::kSums == kChannelSums && ScaledSums<1>::kSums == kChannelSums, "both halves keep 18 sums");

// Who a thread is when the four product waves store their outputs, and where its tile lies.
struct StoreContext {
    int8_t* lds;
    int tid, lane, wave, half, kblock;          // within the four waves that hold the outputs
    int my_n, my_row, my_col, my_origin;        // of tile (lane & 15): image, first output row and column, offset in y (-1: none)
    int rnd;                                    // rounding added before the final >> 4
    int32_t* y;
};

// Adds the two row halves and stores the 16 tiles x 32 filters (from kbase) whose partial outputs
// the four waves hold in Yp.  All four waves call it together (it contains one barrier).
// PART 1 / PART 2 (channels-last with K % 4 = 0 only): just the staging of Yp into LDS / just
// the adding and storing of what was staged, for callers that put their own barrier between
// the two and may run them on different waves.  PART 3: PART 2 for a caller whose waves own every
// entry and staged one finished copy (in the place of half 0): nothing is added.
template <int LAYOUT, bool Q8, int PART = 0>
__device__ __forceinline__ void store_block(const StoreContext& sc, const Problem& p, const Int8Epilogue& q8,
                                            const v4i (&Yp)[16], int kbase) {
    int8_t* const lds = sc.lds;
    const int tid = sc.tid, lane = sc.lane, wave = sc.wave, half = sc.half, kblock = sc.kblock;
    const int my_n = sc.my_n, my_row = sc.my_row, my_col = sc.my_col, my_origin = sc.my_origin, rnd = sc.rnd;
    int32_t* const y = sc.y;
    int* parki = reinterpret_cast<int*>(lds);
    (void)wave; (void)my_n;
    if (LAYOUT == WG_NHWC && (p.K & 3) == 0) {
        // Channels-last with K a multiple of four: outputs are staged filter-fastest,
        // stage[half][output 4i+j][tile][36] (32 filters, rows padded to 36 dwords so that the
        // four 16-lane groups of a wave land in different banks), then every thread adds the
        // halves for four consecutive filters and stores 16 bytes; eight lanes cover the 128
        // contiguous bytes this block owns of a pixel.
        constexpr int kRow = 36, kHalf = 16 * 16 * kRow;
        static_assert(2 * kHalf * 4 <= kLdsBytes, "staging fits the operand planes' LDS");
        // the second half's staged copy of four consecutive filters (none with PART 3)
        auto other_half = [&](int at) {
            if constexpr (PART == 3) return (v4i){0, 0, 0, 0};
            else return *reinterpret_cast<const v4i*>(parki + kHalf + at);
        };
        if constexpr (PART < 2) {
            int* dst = parki + half * kHalf + (4 * (lane >> 4)) * kRow + kblock * 16 + (lane & 15);
#pragma unroll
            for (int o = 0; o < 16; ++o)
#pragma unroll
                for (int q = 0; q < 4; ++q) dst[(o * 16 + q) * kRow] = Yp[o][q];
        }
        if constexpr (PART == 1) return;
        if constexpr (PART == 0) __syncthreads();
        // thread: filters 4*k4..4*k4+3; pass ps: output row i = ps/2, tile = 8*(ps%2) + px/4, column j = px%4
        const int k4 = tid & 7, px = tid >> 3, j = px & 3;
        const int kk = kbase + 4 * k4;
        if constexpr (Q8) {
            // finished int32 outputs of filters 4*g .. 4*g+3 of the block
            auto staged = [&](int o, int tile, int g) {
                const int at = (o * 16 + tile) * kRow + 4 * g;
                return (*reinterpret_cast<const v4i*>(parki + at) + other_half(at) + rnd) >> 4;
            };
            if (q8.pool) {
                // 16 tiles x 2x2 pooled pixels = 64 pixels; thread: four filters of pixels px and px + 32
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int pp = px + 32 * e, tile = pp >> 2, pi = (pp >> 1) & 1, pj = pp & 1;
                    v4i best = requantise(staged(4 * (2 * pi) + 2 * pj, tile, k4), q8);
                    best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi) + 2 * pj + 1, tile, k4), q8));
                    best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi + 1) + 2 * pj, tile, k4), q8));
                    best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi + 1) + 2 * pj + 1, tile, k4), q8));
                    const int n = __shfl(my_n, tile), row = __shfl(my_row, tile), col = __shfl(my_col, tile);
                    const bool ok = __shfl(my_origin, tile) >= 0 && row + 2 * pi < p.H && col + 2 * pj < p.W && kk < p.K;
                    const size_t at = (((size_t)n * (p.H >> 1) + (row >> 1) + pi) * (p.W >> 1) + (col >> 1) + pj) * p.K + kk;
                    if (ok) *reinterpret_cast<uint32_t*>(q8.out + at) = pack_bytes(best);
                }
                return;
            }
            // thread: 16 filters (half h16 of the block) of its own tile (lane & 15) at outputs
            // tid/32 and tid/32 + 8: sixteen lanes read sixteen tiles' rows, which fall in
            // different banks, and a thread stores 16 bytes where the alignment allows
            const int h16 = (tid >> 4) & 1, kq = kbase + 16 * h16;
            const bool vector_store = ((p.K & 15) | (reinterpret_cast<uintptr_t>(q8.out) & 15)) == 0;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int o = (tid >> 5) + 8 * e, i = o >> 2, jj = o & 3;
                uint32_t bytes[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) bytes[g] = pack_bytes(requantise(staged(o, lane & 15, 4 * h16 + g), q8));
                const bool ok = my_origin >= 0 && my_row + i < p.H && my_col + jj < p.W;
                int8_t* dst = q8.out + (size_t)my_origin + (size_t)(i * p.W + jj) * p.K + kq;
                if (ok && vector_store && kq < p.K) {
                    *reinterpret_cast<uint4*>(dst) = make_uint4(bytes[0], bytes[1], bytes[2], bytes[3]);
                } else if (ok) {
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        if (kq + 4 * g < p.K) reinterpret_cast<uint32_t*>(dst)[g] = bytes[g];
                }
            }
            return;
        }
        int32_t* first[2];   // output row 0 of the thread's two tiles (e = 0, 1); null where nothing is stored
        int rows[2];         // output rows of that tile inside the image
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int origin = __shfl(my_origin, 8 * e + (px >> 2));
            const bool ok = origin >= 0 && __shfl(my_col, 8 * e + (px >> 2)) + j < p.W && kk < p.K;
            first[e] = ok ? y + (size_t)origin + j * p.K + kk : nullptr;
            rows[e] = p.H - __shfl(my_row, 8 * e + (px >> 2));
        }
        const size_t row_pitch = (size_t)p.W * p.K;
        v4i v[8];
#pragma unroll
        for (int ps = 0; ps < 8; ++ps) {
            const int i = ps >> 1, tile = 8 * (ps & 1) + (px >> 2);
            const int at = ((4 * i + j) * 16 + tile) * kRow + 4 * k4;
            v[ps] = (*reinterpret_cast<const v4i*>(parki + at) + other_half(at) + rnd) >> 4;
        }
#pragma unroll
        for (int ps = 0; ps < 8; ++ps) {
            const int i = ps >> 1, e = ps & 1;
            if (first[e] != nullptr && i < rows[e]) *reinterpret_cast<v4i*>(first[e] + i * row_pitch) = v[ps];
        }
        return;
    }
    // General path: park[wave][output 0..15][lane] (four registers = four tiles each); the value
    // of (tile, output 4i+j, filter kl) sits in waves kl/16 and 2 + kl/16 at output 4i+j, lane
    // (tile/4)*16 + kl%16, register tile%4.  16 x 16 x 32 = 8192 results, 32 per thread.
    v4i* park = reinterpret_cast<v4i*>(lds);
#pragma unroll
    for (int i = 0; i < 16; ++i) park[(wave * 16 + i) * 64 + lane] = Yp[i];
    __syncthreads();
    if constexpr (Q8) {
        // One byte per (tile, output pixel, filter), in the order of the output layout; lg = log2
        // of the output pixels per tile side (4, or 2 after pooling).
        const int lg = q8.pool ? 1 : 2, side = 1 << lg, span = q8.pool ? 2 : 1;
        const int Ho = q8.pool ? p.H >> 1 : p.H, Wo = q8.pool ? p.W >> 1 : p.W;
        const int items = (16 * 32) << (2 * lg);
        for (int e = tid; e < items; e += 256) {
            int kl, tile, pi, pj;
            if constexpr (LAYOUT == WG_NHWC) {
                kl = e & 31; pj = (e >> 5) & (side - 1); pi = (e >> (5 + lg)) & (side - 1); tile = e >> (5 + 2 * lg);
            } else {
                pj = e & (side - 1); tile = (e >> lg) & 15; pi = (e >> (lg + 4)) & (side - 1); kl = e >> (2 * lg + 4);
            }
            int best = -129;
            for (int a = 0; a < span; ++a)
                for (int b = 0; b < span; ++b) {
                    const int o = 4 * (span * pi + a) + span * pj + b;
                    const int at = ((((kl >> 4) * 16 + o) * 64) + (tile >> 2) * 16 + (kl & 15)) * 4 + (tile & 3);
                    best = max(best, requantise((parki[at] + parki[at + 2 * 16 * 64 * 4] + rnd) >> 4, q8));
                }
            const int n = __shfl(my_n, tile), row = __shfl(my_row, tile), col = __shfl(my_col, tile);
            const bool ok = __shfl(my_origin, tile) >= 0 && row + span * pi < p.H && col + span * pj < p.W && kbase + kl < p.K;
            const int oh = (q8.pool ? row >> 1 : row) + pi, ow = (q8.pool ? col >> 1 : col) + pj;
            const size_t at = LAYOUT == WG_NHWC ? (((size_t)n * Ho + oh) * Wo + ow) * p.K + kbase + kl
                                                : (((size_t)n * p.K + kbase + kl) * Ho + oh) * Wo + ow;
            if (ok) q8.out[at] = (int8_t)best;
        }
        return;
    }
    int v[32];
    if constexpr (LAYOUT == WG_NHWC) {
        // thread: filter kl and output column j fixed; iteration it: tile it/2, output row 2(it%2) + tid/128
        const int kl = tid & 31, j = (tid >> 5) & 3, ih = tid >> 7;
        const int kk = kbase + kl;
        const int at0 = (((kl >> 4) * 16 + j) * 64 + (kl & 15)) * 4;
#pragma unroll
        for (int it = 0; it < 32; ++it) {
            const int tile = it >> 1, i = 2 * (it & 1) + ih;
            const int at = at0 + (4 * i * 64 + (tile >> 2) * 16) * 4 + (tile & 3);
            v[it] = (parki[at] + parki[at + 2 * 16 * 64 * 4] + rnd) >> 4;
        }
#pragma unroll
        for (int it = 0; it < 32; ++it) {
            const int tile = it >> 1, i = 2 * (it & 1) + ih;
            const int origin = __builtin_amdgcn_readlane(my_origin, tile);
            const int h = __builtin_amdgcn_readlane(my_row, tile) + i, w = __builtin_amdgcn_readlane(my_col, tile) + j;
            if (origin >= 0 && h < p.H && w < p.W && kk < p.K) y[(size_t)origin + (i * p.W + j) * p.K + kk] = v[it];
        }
    } else {
        // thread: tile, output row i and column j fixed; iteration it: filter it.  A wave writes one
        // output row of 16 consecutive tiles = 256 contiguous bytes.
        const int j = tid & 3, tile = (tid >> 2) & 15, i = tid >> 6;
        const int origin = __shfl(my_origin, tile), h = __shfl(my_row, tile) + i, w = __shfl(my_col, tile) + j;
        const bool ok = origin >= 0 && h < p.H && w < p.W;
        const int at0 = ((4 * i + j) * 64 + (tile >> 2) * 16) * 4 + (tile & 3);
#pragma unroll
        for (int it = 0; it < 32; ++it) {
            const int at = at0 + ((it >> 4) * 16 * 64 + (it & 15)) * 4;
            v[it] = (parki[at] + parki[at + 2 * 16 * 64 * 4] + rnd) >> 4;
        }
#pragma unroll
        for (int it = 0; it < 32; ++it)
            if (ok && kbase + it < p.K) y[(size_t)origin + ((size_t)(kbase + it) * p.H + i) * p.W + j] = v[it];
    }

}

// grid: (ceil(T/16), Kp/32), or Kp/64 for WIDE.  256 threads: in the transform phase one thread per (tile,
// four channels); in the product phase wave w owns filter block (w & 1) and half of the
// rows of M (w >> 1: rows 0,1,2 or rows 5,3); all four waves stage their partial outputs
// in LDS and the block stores the sums with full-line writes.
// SUMS: scaled mode keeps channel sums and scales them at the end (see ScaledSums): needed with
// more than one channel block, and used for every scaled WIDE workgroup.
// WIDE: the workgroup covers 64 filters instead of 32: the transform of a
// channel block is followed by two passes over the entries, one per 32 filters, each with its own
// outputs; used when there are more workgroups than compute units, where halving the number of
// repeated transforms outweighs the longer workgroup.
// Q8: the finished outputs are requantised (and pooled) to int8 at q8.out instead of stored to y.
// ENC: how the activation bytes are read (signed int8, or uint8 with a zero point: Section 4.1); the latter only
// with the load paths that select padding explicitly, and with blobs made from uint8 filters.
template <int LAYOUT, int LOAD, int MODE, bool SUMS, bool WIDE, bool Q8, class ENC = SignedInt8>
__device__ __forceinline__ void fused_conv_body(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                size_t table_off, size_t planes_off, int32_t* __restrict__ y,
                                                const Problem p, const Int8Epilogue q8, const ENC enc = ENC{}) {
    static_assert(LOAD != kLoadDirect || ENC::kMagic == kBlobMagic, "direct transfers deliver zero bytes for absent pixels");
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kblock = wave & 1, half = wave >> 1;
    // Workgroups are handed to the eight XCDs (each with its own L2) round-robin in launch order.
    // With several filter blocks and channel blocks, the grid is dealt out XCD-major instead, so
    // that an XCD runs consecutive tile blocks of as few filter blocks as possible at the same
    // time: a filter block's operand planes (46-138 KB per channel block) are then fetched into
    // one or two L2s instead of into all eight.  (With a single channel block the planes are
    // small and the order made no difference.)
    int bx = blockIdx.x, by = blockIdx.y;
    {
        const int total = gridDim.x * gridDim.y;
        if (gridDim.y >= 2 && p.CB >= 2 && (total & 7) == 0) {
            const int launch = blockIdx.y * gridDim.x + blockIdx.x;
            const int w = (launch & 7) * (total >> 3) + (launch >> 3);   // XCD-major position
            by = w / (int)gridDim.x;
            bx = w - by * (int)gridDim.x;
        }
    }
    const int tile0 = bx * kFusedTiles;
    constexpr int NPASS = WIDE ? 2 : 1;
    const int k0 = by * (kFusedFilters * NPASS);
    const int k = k0 + kblock * 16 + (lane & 15);

    // The activation patch of the first channel block does not depend on the blob and is the
    // longest wait of the kernel: its requests go out before anything else.
    DirectPatch direct;
    int8_t* raw_wave = lds + kLdsBytes + wave * kRawWaveBytes;
    if constexpr (LOAD == kLoadDirect) {
        const int dt = tile0 + 4 * wave + ((lane & 15) >> 2);   // the tile this lane moves pieces of
        int dn = 0, dty = 0, dtx = 0;
        if (dt < p.T) decode_tile(p, dt, dn, dty, dtx);
        direct.init(p, dn, dty, dtx, lane);
        direct.issue(x, p, 0, lane, raw_wave);
    }

    // transform-phase identity
    // every lane decodes tile (lane & 15) of the block once; the transform phase fetches the
    // coordinates of its own tile (tid / 16) from that lane
    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + (lane & 15) < p.T) decode_tile(p, tile0 + (lane & 15), my_n, my_ty, my_tx);
    const int a_tile = tid >> 4, a_cq = tid & 15;
    const int a_t = tile0 + a_tile;
    const int a_tx = __shfl(my_tx, a_tile), a_ty = __shfl(my_ty, a_tile), a_n = __shfl(my_n, a_tile);
    OperandSplitter<MODE == WG_SCALED ? kSplitByteLimbs : kSplitTwoLimb, LdsPlaneSink> out;
    out.sink.base = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;

    LaneContext cx;
    cx.a_lds = lds + lds_slot(lane >> 4, lane & 15) * 16;
    cx.table_k = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
    constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) +
                           filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, NP);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;

    v4i Yall[NPASS][16];
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass)
#pragma unroll
        for (int i = 0; i < 16; ++i) Yall[pass][i] = (v4i){0, 0, 0, 0};
    v4i (&Y)[16] = Yall[0];

    // The blob header is checked while the patch requests are in flight.
    constexpr bool VEC4 = LOAD == kLoadDwords;
    uint32_t patch[6][6];
    if constexpr (LOAD != kLoadDirect) {
        if (a_t < p.T) load_patch<LAYOUT, VEC4>(x, p, a_n, a_ty, a_tx, 4 * a_cq, patch, enc);
    }
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE, ENC::kMagic)) return;

    ProductPhase<MODE, 0> phase0;
    ProductPhase<MODE, 1> phase1;
    static_assert(!SUMS || MODE == WG_SCALED, "channel sums are kept apart in scaled mode only");
    v4i sums[SUMS ? NPASS : 1][SUMS ? kChannelSums : 1];
    if constexpr (SUMS) {
#pragma unroll
        for (int pass = 0; pass < NPASS; ++pass)
#pragma unroll
            for (int i = 0; i < kChannelSums; ++i) sums[pass][i] = (v4i){0, 0, 0, 0};
    }
    static_assert(ProductPhase<MODE, 0>::NPRE == kFilterPrefetch && ProductPhase<MODE, 1>::NPRE == kFilterPrefetch,
                  "the wait for the direct patch transfer counts the filter fragments requested after it");
    for (int cb = 0; cb < p.CB; ++cb) {
        cx.b_glob = b_lane + cb * b_block_stride;
        if (half == 0) phase0.prefetch(cx); else phase1.prefetch(cx);
        if (cb > 0) {   // everyone is done reading the previous block's planes
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
        }
        if constexpr (LOAD == kLoadDirect) {
            // the patch pieces were requested before the sixteen filter fragments above, and
            // loads complete in order; the pieces a thread reads were moved by its own wave
            asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            DirectPatch::read(raw_wave, lane, patch);
            if (cb + 1 < p.CB) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the raw area has been read
                direct.issue(x, p, cb + 1, lane, raw_wave);
            }
        }
        if (a_t < p.T) {
            bias_patch(p, a_ty, a_tx, cb * kCBlock + 4 * a_cq, patch, enc);
            transform_patch(patch, out, enc);
            if constexpr (LOAD != kLoadDirect) {
                if (cb + 1 < p.CB)   // next block's patch travels while this block's products run
                    load_patch<LAYOUT, VEC4>(x, p, a_n, a_ty, a_tx, (cb + 1) * kCBlock + 4 * a_cq, patch, enc);
            }
        }
        // the operand planes are complete once every wave's LDS writes have landed; global
        // requests (filter fragments, the next block's patch) stay in flight across the barrier
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        if constexpr (SUMS && WIDE) {
            if (half == 0) {
                ScaledSums<0>::template run<0, 2>(cx, phase0.bring, sums[0]);
                ScaledSums<0>::template run<1, 2>(cx, phase0.bring, sums[1]);
            } else {
                ScaledSums<1>::template run<0, 2>(cx, phase1.bring, sums[0]);
                ScaledSums<1>::template run<1, 2>(cx, phase1.bring, sums[1]);
            }
        } else if constexpr (SUMS) {
            if (half == 0) ScaledSums<0>::run(cx, phase0.bring, sums[0]); else ScaledSums<1>::run(cx, phase1.bring, sums[0]);
        } else if constexpr (WIDE) {
            if (half == 0) { phase0.template run<0, 2>(cx, Yall[0]); phase0.template run<1, 2>(cx, Yall[1]); }
            else           { phase1.template run<0, 2>(cx, Yall[0]); phase1.template run<1, 2>(cx, Yall[1]); }
        } else {
            if (half == 0) phase0.run(cx, Y); else phase1.run(cx, Y);
        }
    }
    if constexpr (SUMS) {
        if (half == 0) ScaledSums<0>::template finish<0>(cx, sums[0], Yall[0]);
        else           ScaledSums<1>::template finish<0>(cx, sums[0], Yall[0]);
        if constexpr (WIDE) {
            if (half == 0) ScaledSums<0>::template finish<1>(cx, sums[1], Yall[1]);
            else           ScaledSums<1>::template finish<1>(cx, sums[1], Yall[1]);
        }
    }

    // ---- add the two halves and store ------------------------------------------------------
    // Where tile (lane & 15) of this block starts in y (offsets fit 32 bits, checked on the
    // host; -1 marks tiles beyond T), and its first output row and column.
    const int my_row = 4 * my_ty, my_col = 4 * my_tx;
    int my_origin = -1;
    if (tile0 + (lane & 15) < p.T)
        my_origin = LAYOUT == WG_NHWC ? ((my_n * p.H + my_row) * p.W + my_col) * p.K
                                      : (my_n * p.K * p.H + my_row) * p.W + my_col;
    const int rnd = MODE == WG_SCALED ? 8 : 0;
    const StoreContext sc = {lds, tid, lane, wave, half, kblock, my_n, my_row, my_col, my_origin, rnd, y};
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
        __syncthreads();   // the operand planes (or the previous pass's staged outputs) are dead
        store_block<LAYOUT, Q8>(sc, p, q8, Yall[pass], k0 + pass * kFusedFilters);
    }
}

template <int LAYOUT, int LOAD, int MODE, bool SUMS, bool WIDE>
__global__ __launch_bounds__(256) void fused_conv_kernel(const int8_t* __restrict__ x,
                                                         const uint8_t* __restrict__ blob, size_t table_off,
                                                         size_t planes_off, int32_t* __restrict__ y, Problem p) {
    fused_conv_body<LAYOUT, LOAD, MODE, SUMS, WIDE, false>(x, blob, table_off, planes_off, y, p, Int8Epilogue{});
}

template <int LAYOUT, int LOAD, int MODE, bool SUMS, bool WIDE>
__global__ __launch_bounds__(256) void fused_conv_int8_kernel(const int8_t* __restrict__ x,
                                                              const uint8_t* __restrict__ blob, size_t table_off,
                                                              size_t planes_off, Problem p, Int8Epilogue q8) {
    fused_conv_body<LAYOUT, LOAD, MODE, SUMS, WIDE, true>(x, blob, table_off, planes_off, nullptr, p, q8);
}

template <int LAYOUT, int LOAD, int MODE, bool SUMS>
__global__ __launch_bounds__(256) void fused_conv_u8_kernel(const int8_t* __restrict__ x, ZeroPointU8 zero,
                                                            const uint8_t* __restrict__ blob, size_t table_off,
                                                            size_t planes_off, int32_t* __restrict__ y, Problem p) {
    fused_conv_body<LAYOUT, LOAD, MODE, SUMS, false, false, ZeroPointU8>(x, blob, table_off, planes_off, y, p, Int8Epilogue{}, zero);
}

// Product phase of the role-specialised kernel: the same arithmetic as ProductPhase / ScaledSums
// without their software pipelining (one set of fragments and accumulators, an eight-deep filter
// ring), because a product wave there has 256 registers and its waits are covered by the
// transform wave on the same SIMD.
// AHEAD: the activation fragments of the next entry are asked for before the current entry's
// matrix-core instructions (a second set of fragment registers), for callers whose product waves
// are the longer chain of the two roles.
// PIPE: an entry's vector work runs beside the next entry's matrix-core instructions (a second set of accumulators).
template <int MODE, int HALF, bool SUMS, int RING = 8, bool AHEAD = false, bool PIPE = false>
struct LeanProducts {
    // scaled mode with joined channel sums, or in a wave that owns every entry: complex entries without the -Wi plane
    static constexpr int PM = MODE == WG_SCALED && (SUMS || HALF == kAllRows) ? kScaledTwoPlanes : MODE;
    using Phase = ProductPhase<PM, HALF>;
    static constexpr int NE = Phase::NE, NB = Phase::NB;
    static constexpr int kRing = RING;
    static constexpr int kSums = SUMS ? ScaledSums<HALF>::kSums : 1;   // 18 per half, 36 for a wave that owns every entry
    v4i ring[kRing];

    __device__ inline void prefetch(const LaneContext& cx) {
        static_for<(NB < kRing ? NB : kRing)>([&](auto I) { ring[I] = Phase::template load_b<I>(cx); });
    }

    // sums: the 18 channel sums of ScaledSums (SUMS), else unused; Y: the outputs (not SUMS)
    __device__ inline void run(const LaneContext& cx, v4i (&sums)[kSums], v4i (&Y)[16]) {
        v4i er[6], ei[6];
        v4i afr2[AHEAD ? 2 : 1][4];
        if constexpr (AHEAD)
            static_for<num_a<PM>(half_slot(HALF, 0).entry)>([&](auto I) { afr2[0][I] = Phase::template load_a<0, I>(cx); });
        // the matrix-core part of slot S: activation fragments, products into acc, refill of the filter ring
        auto multiply = [&](auto S, v4i (&acc)[9]) {
            constexpr int s = S;
            constexpr int entry = half_slot(HALF, s).entry;
            constexpr int b0 = b_start<PM>(HALF, s);
            v4i (&afr)[4] = afr2[AHEAD ? (s & 1) : 0];
            if constexpr (!AHEAD) {
                static_for<num_a<PM>(entry)>([&](auto I) { afr[I] = Phase::template load_a<s, I>(cx); });
            } else if constexpr (s + 1 < NE) {
                static_for<num_a<PM>(half_slot(HALF, s + 1).entry)>(
                    [&](auto I) { afr2[(s + 1) & 1][I] = Phase::template load_a<s + 1, I>(cx); });
            }
            static_for<num_ops<PM>(entry)>([&](auto I) {
                constexpr Op op = entry_op<PM>(entry, I);
                constexpr v4i zero = {0, 0, 0, 0};
                acc[op.acc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(afr[op.a], ring[(b0 + op.b) % kRing],
                                                                    op.init ? zero : acc[op.acc], 0, 0, 0);
            });
            static_for<num_b<PM>(entry)>([&](auto I) {
                if constexpr (b0 + I + kRing < NB) ring[(b0 + I) % kRing] = Phase::template load_b<b0 + I + kRing>(cx);
            });
        };
        // the vector part of slot S: limbs joined; then into the channel sums, or reverse scaling and output transform
        auto reduce = [&](auto S, const v4i (&acc)[9]) {
            constexpr int s = S;
            constexpr Slot sl = half_slot(HALF, s);
            constexpr int entry = sl.entry;
            if constexpr (SUMS) {
                // joined values only; scaling (scaled mode) and the output transform wait for finish()
                constexpr int v = ScaledSums<HALF>::sum_start(s);
                if constexpr (MODE == WG_SCALED) {   // Re = Dr Wr - Di Wi,  Im = Dr Wi + Di Wr
                    if constexpr (is_real(entry)) {
                        sums[v] += (acc[0] << kByteLimbShift) + acc[1];
                    } else {
                        sums[v] += ((acc[0] - acc[4]) << kByteLimbShift) + (acc[1] - acc[5]);
                        sums[v + 1] += (acc[2] << kByteLimbShift) + acc[3];
                    }
                } else if constexpr (is_real(entry)) {
                    sums[v] += join_limbs(acc[0], acc[1], acc[2]);
                } else {
                    sums[v] += join_limbs(acc[0] - acc[3], acc[1] - acc[4], acc[2] - acc[5]);
                    sums[v + 1] += join_limbs(acc[6], acc[7], acc[8]);
                }
            } else {
                v4i re, im = {0, 0, 0, 0};
                if constexpr (MODE == WG_LOSSLESS) {
                    if constexpr (is_real(entry)) {
                        re = join_limbs(acc[0], acc[1], acc[2]);
                    } else {   // Re = Dr Wr - Di Wi,  Im = Dr Wi + Di Wr
                        re = join_limbs(acc[0] - acc[3], acc[1] - acc[4], acc[2] - acc[5]);
                        im = join_limbs(acc[6], acc[7], acc[8]);
                    }
                } else {
                    if constexpr (is_real(entry)) re = (acc[0] << kByteLimbShift) + acc[1];
                    else if constexpr (PM == kScaledTwoPlanes) re = ((acc[0] - acc[4]) << kByteLimbShift) + (acc[1] - acc[5]);
                    else re = (acc[0] << kByteLimbShift) + acc[1];
                    if constexpr (!is_real(entry)) im = (acc[2] << kByteLimbShift) + acc[3];
                    // Section 4.2 (a wave that owns every entry exists only where the factors were parked)
                    const ReverseScale unscale = HALF == kAllRows ? parked_scale<s>(cx) : ReverseScale(cx.table_k[entry]);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        re[q] = unscale(re[q]);
                        if constexpr (!is_real(entry)) im[q] = unscale(im[q]);
                    }
                }
                er[sl.pos] = re;
                ei[sl.pos] = im;
                if constexpr (sl.last_in_row) finish_row<sl.row>(er, ei, Y);
                if constexpr (HALF == kAllRows) {
                    // Pins the entry's value, and a finished row's outputs, to this place.  Left alone, the compiler moves
                    // the vector work of all 26 entries behind the last matrix-core instruction (into the block that
                    // stages the outputs) and keeps every accumulator alive until then.
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        asm volatile("" ::"v"(re[q]));
                        if constexpr (!is_real(entry)) asm volatile("" ::"v"(im[q]));
                    }
                    if constexpr (sl.last_in_row) {
#pragma unroll
                        for (int i = 0; i < 16; ++i)
#pragma unroll
                            for (int q = 0; q < 4; ++q) asm volatile("" ::"v"(Y[i][q]));
                    }
                }
            }
        };
        if constexpr (PIPE) {
            // slot s + 1's matrix-core instructions are issued before slot s's vector work, which then runs beside them
            v4i acc2[2][9];
            static_for<NE + 1>([&](auto S) {
                if constexpr (S < NE) multiply(S, acc2[S & 1]);
                if constexpr (S > 0) reduce(std::integral_constant<int, S - 1>{}, acc2[(S - 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
            });
        } else {
            static_for<NE>([&](auto S) {
                v4i acc[9];
                multiply(S, acc);
                reduce(S, acc);
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    }

    // SUMS, lossless mode, after the last channel block: the output transform of the channel sums
    // (it is linear, so it may as well run once on the sums as once per block).
    __device__ inline static void finish_lossless(const v4i (&sums)[kSums], v4i (&Y)[16]) {
        v4i er[6], ei[6];
        static_for<NE>([&](auto S) {
            constexpr Slot sl = half_slot(HALF, S);
            constexpr int v = ScaledSums<HALF>::sum_start(S);
            er[sl.pos] = sums[v];
            if constexpr (!is_real(sl.entry)) ei[sl.pos] = sums[v + 1];
            else                              ei[sl.pos] = (v4i){0, 0, 0, 0};
            if constexpr (sl.last_in_row) {
                finish_row<sl.row>(er, ei, Y);
                if constexpr (HALF == kAllRows) __builtin_amdgcn_sched_barrier(0);   // row by row (see ScaledSums::finish)
            }
        });
    }
};

// Scaled mode in the role-specialised kernel: every limb product of every entry a wave owns has
// its own matrix-core accumulator for the whole kernel (two per real entry: high and low
// activation limb; four per complex entry: Re and Im, each high and low; 36 per wave), so a
// channel block costs a product wave nothing but fragment loads and matrix-core instructions
// and the vector ALU is left to the transform wave.  The limbs are joined, the reverse scaling
// applied and the output transform run once, on the finished channel sums.
template <int HALF>
struct ResidentScaled {
    static constexpr int MODE = WG_SCALED;
    using Phase = ProductPhase<MODE, HALF>;
    static constexpr int NE = Phase::NE, NB = Phase::NB;
    static constexpr int kRing = 8;
    static constexpr int acc_start(int slot) {
        int n = 0;
        for (int s = 0; s < slot; ++s) n += is_real(half_slot(HALF, s).entry) ? 2 : 4;
        return n;
    }
    static constexpr int kAcc = acc_start(NE);
    v4i ring[kRing];

    __device__ inline void prefetch(const LaneContext& cx) {
        static_for<(NB < kRing ? NB : kRing)>([&](auto I) { ring[I] = Phase::template load_b<I>(cx); });
    }
    __device__ inline void run(const LaneContext& cx, v4i (&acc)[kAcc]) {
        static_for<NE>([&](auto S) {
            constexpr int s = S;
            constexpr int entry = half_slot(HALF, s).entry;
            constexpr int b0 = b_start<MODE>(HALF, s);
            constexpr int v = acc_start(s);
            v4i afr[4];
            static_for<num_a<MODE>(entry)>([&](auto I) { afr[I] = Phase::template load_a<s, I>(cx); });
            static_for<num_ops<MODE>(entry)>([&](auto I) {
                constexpr Op op = entry_op<MODE>(entry, I);
                acc[v + op.acc] = __builtin_amdgcn_mfma_i32_16x16x64_i8(afr[op.a], ring[(b0 + op.b) % kRing], acc[v + op.acc], 0, 0, 0);
            });
            static_for<num_b<MODE>(entry)>([&](auto I) {
                if constexpr (b0 + I + kRing < NB) ring[(b0 + I) % kRing] = Phase::template load_b<b0 + I + kRing>(cx);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    __device__ inline static void finish(const LaneContext& cx, const v4i (&acc)[kAcc], v4i (&Y)[16]) {
        v4i er[6], ei[6];
        static_for<NE>([&](auto S) {
            constexpr Slot sl = half_slot(HALF, S);
            constexpr int v = acc_start(S);
            v4i re = (acc[v] << kByteLimbShift) + acc[v + 1], im = {0, 0, 0, 0};
            if constexpr (!is_real(sl.entry)) im = (acc[v + 2] << kByteLimbShift) + acc[v + 3];
            const ReverseScale unscale = parked_scale<S>(cx);   // Section 4.2
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                re[q] = unscale(re[q]);
                if constexpr (!is_real(sl.entry)) im[q] = unscale(im[q]);
            }
            er[sl.pos] = re;
            ei[sl.pos] = im;
            if constexpr (sl.last_in_row) finish_row<sl.row>(er, ei, Y);
        });
    }
};
static_assert(ResidentScaled<0>::kAcc == 36 && ResidentScaled<1>::kAcc == 36, "both halves keep 36 accumulators");

// The same computation for layers with several channel blocks, with the two kinds of work on
// different waves.  Eight waves: waves 0-3 only transform (vector ALU), waves 4-7 only multiply
// (matrix cores, joins, output transform); each SIMD hosts one of each, so the transform of
// channel block cb + 1 runs under the products of block cb instead of before them, and a
// product wave's waits are filled with the transform wave's work.  The operand planes are
// double-buffered in LDS (2 x 72 KB); patches come through 4-byte or byte loads into the
// transform threads' registers, one channel block ahead.  One barrier per channel block:
// barrier j (j = 1..CB) publishes the planes of block j - 1 and frees the buffer that the
// products of block j - 2 were reading.  32 filters per workgroup (a second pass would not fit
// the 256 registers a wave has when two share a SIMD).
// PW = 8 (channels-last, 4-byte buffer loads, K % 4 = 0): eight product waves, twelve waves in all, 64 filters per workgroup.
// On deep layers the workgroup's pace is set by the transform waves and by what the compute unit's vector-memory path
// takes in, while the product waves of the eight-wave form idle half of the time: with two product waves per SIMD one
// transform (and one set of patch loads) serves twice the filters.  Product wave pw owns filter block pw % 4 and half
// pw / 4 of the entries.  Three waves per SIMD leave a wave 168 registers, so in both modes the product waves keep 18
// joined channel sums (scaled mode: instead of the 36 resident limb accumulators), with a loop per half so that each
// half is allocated registers on its own, and the transform waves form their patch offsets per load.  The two 32-filter
// halves stage their outputs in one operand buffer each and store at the same time.
#ifdef WG_TIMESTAMPS
// Development aid (never compiled into the library): per-wave sums of the time spent in each part of the channel-block loop.
__device__ unsigned long long* g_roles_stamps = nullptr;
#define WG_CLOCK() __builtin_amdgcn_s_memtime()
#define WG_SPENT(i, since) do { const unsigned long long now_ = WG_CLOCK(); spent[i] += now_ - (since); (since) = now_; } while (0)
#else
#define WG_SPENT(i, since) do { } while (0)
#endif

template <int LAYOUT, bool VEC4, int MODE, bool SUMS, bool Q8, int PW = 4>
__global__ __launch_bounds__(64 * (4 + PW)) void fused_conv_roles_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                                         size_t table_off, size_t planes_off, int32_t* __restrict__ y,
                                                                         Problem p, Int8Epilogue q8) {
    static_assert(PW == 4 || (PW == 8 && VEC4 && SUMS && LAYOUT == WG_NHWC), "eight product waves: channels-last, buffer loads, channel sums");
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int lane = threadIdx.x & 63, wave8 = threadIdx.x >> 6;
    const bool transforms = wave8 < 4;
    const int tid = threadIdx.x & 255, wave = wave8 & 3;   // within the role (PW = 8: within the four waves that store together)
    int bx = blockIdx.x, by = blockIdx.y;
    {
        const int total = gridDim.x * gridDim.y;
        if (gridDim.y >= 2 && (total & 7) == 0) {   // XCD-major order, as in fused_conv_body
            const int launch = blockIdx.y * gridDim.x + blockIdx.x;
            const int w = (launch & 7) * (total >> 3) + (launch >> 3);
            by = w / (int)gridDim.x;
            bx = w - by * (int)gridDim.x;
        }
    }
    const int tile0 = bx * kFusedTiles, k0 = by * (kFusedFilters * (PW / 4));
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + (lane & 15) < p.T) decode_tile(p, tile0 + (lane & 15), my_n, my_ty, my_tx);
#ifdef WG_TIMESTAMPS
    unsigned long long spent[4] = {0, 0, 0, 0}, mark = WG_CLOCK();
    const unsigned long long entered = mark;
    auto report = [&]() {
        if (g_roles_stamps != nullptr && lane == 0) {
            unsigned long long* o = g_roles_stamps + ((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 12 + wave8) * 8;
            o[0] = spent[0]; o[1] = spent[1]; o[2] = spent[2]; o[3] = spent[3]; o[4] = WG_CLOCK() - entered; o[6] = entered;
        }
    };
#endif

    if (transforms) {
        const int a_tile = tid >> 4, a_cq = tid & 15;
        const int a_t = tile0 + a_tile;
        const int a_tx = __shfl(my_tx, a_tile), a_ty = __shfl(my_ty, a_tile), a_n = __shfl(my_n, a_tile);
        OperandSplitter<MODE == WG_SCALED ? kSplitByteLimbs : kSplitTwoLimb, LdsPlaneSink> out;
        int8_t* const slot = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;
        uint32_t patch[6][6];
        // 4-byte pixel loads: the 36 offsets of the patch (relative to x: they fit 32 bits) are
        // formed once; a channel block is then a uniform offset on top of these.  Scaled mode,
        // where these waves set the pace, loads through the buffer descriptor (no select per
        // pixel); lossless mode, where the product waves do, measured 3 % faster with plain
        // loads from clamped addresses.
        constexpr bool kBuffer = VEC4 && (MODE == WG_SCALED || PW == 8);
        uint32_t pixel[VEC4 && PW == 4 ? 36 : 1];
        uint32_t row_off[PW == 8 ? 6 : 1], col_off[PW == 8 ? 6 : 1];   // PW = 8: offsets are formed per load (registers are scarce)
        const __amdgpu_buffer_rsrc_t xbuf = activation_buffer(x, p);
        auto request = [&](int cb) {
            if constexpr (PW == 8) {
                // channel groups beyond C (last block of a C that is not a multiple of 64: a uniform branch) get zeros
                const bool have = (cb + 1) * kCBlock <= p.C || cb * kCBlock + 4 * a_cq < p.C;
#pragma unroll
                for (int i = 0; i < 36; ++i) {
                    const uint32_t at = __builtin_elementwise_add_sat(row_off[i / 6], col_off[i % 6]);
                    patch[i / 6][i % 6] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xbuf, have ? at : kOutsideOffset, cb * kCBlock, 0);
                }
            } else if constexpr (kBuffer) {
                request_patch(xbuf, p, pixel, cb, 4 * a_cq, patch);
            } else if constexpr (VEC4) {
                const int c0 = cb * kCBlock + 4 * a_cq;
                const int8_t* base = x + (c0 < p.C ? c0 : 0);
#pragma unroll
                for (int i = 0; i < 36; ++i) patch[i / 6][i % 6] = *reinterpret_cast<const uint32_t*>(base + pixel[i]);
            } else {
                load_patch<LAYOUT, false>(x, p, a_n, a_ty, a_tx, cb * kCBlock + 4 * a_cq, patch);
            }
        };
        if constexpr (PW == 8) {
            const int h0 = 4 * a_ty - 1, w0 = 4 * a_tx - 1;
            const uint32_t image = (uint32_t)a_n * (uint32_t)p.H * (uint32_t)p.W * (uint32_t)p.C + (uint32_t)(4 * a_cq);
#pragma unroll
            for (int a = 0; a < 6; ++a) {
                row_off[a] = (unsigned)(h0 + a) < (unsigned)p.H ? image + (uint32_t)(h0 + a) * (uint32_t)p.W * (uint32_t)p.C : kOutsideOffset;
                col_off[a] = (unsigned)(w0 + a) < (unsigned)p.W ? (uint32_t)(w0 + a) * (uint32_t)p.C : kOutsideOffset;
            }
        } else if constexpr (kBuffer) {
            patch_offsets(p, a_n, a_ty, a_tx, 4 * a_cq, pixel);
        } else if constexpr (VEC4) {
            const int h0 = 4 * a_ty - 1, w0 = 4 * a_tx - 1;
            const uint32_t image = (uint32_t)a_n * (uint32_t)p.H * (uint32_t)p.W * (uint32_t)p.C;
#pragma unroll
            for (int a = 0; a < 6; ++a)
#pragma unroll
                for (int b = 0; b < 6; ++b)
                    pixel[6 * a + b] = image + ((uint32_t)min(max(h0 + a, 0), p.H - 1) * (uint32_t)p.W +
                                                (uint32_t)min(max(w0 + b, 0), p.W - 1)) * (uint32_t)p.C;
        }
        if (a_t < p.T) request(0);
        WG_SPENT(3, mark);
        for (int cb = 0; cb < p.CB; ++cb) {
            if (cb > 0) {   // barrier cb
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
            }
            WG_SPENT(0, mark);   // LDS writes landed + barrier
            out.sink.base = slot + (cb & 1) * kLdsBytes;
            if (a_t < p.T) {
#ifdef WG_TIMESTAMPS
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                WG_SPENT(1, mark);   // wait for the patch
#endif
                if constexpr (kBuffer) bias_buffer_patch(patch);
                else bias_patch(p, a_ty, a_tx, cb * kCBlock + 4 * a_cq, patch);
                transform_patch(patch, out);
                WG_SPENT(2, mark);   // transform
                if (cb + 1 < p.CB) request(cb + 1);
                WG_SPENT(3, mark);   // requests
            }
        }
#ifdef WG_TIMESTAMPS
        report();
#endif
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();   // barrier CB: the last block's planes are published
        __syncthreads();                // the two barriers of the product waves' store
        __syncthreads();
        return;
    }

    // PW = 4: wave = 2 half + kblock.  PW = 8: product wave pw = wave8 - 4 owns filter block pw % 4 and half pw / 4; the
    // waves of filter blocks 2 group, 2 group + 1 store together (`wave` counts within that group, as store_block expects)
    const int pw = wave8 - 4;
    const int kblock4 = PW == 8 ? (pw & 3) : (wave & 1), half = PW == 8 ? (pw >> 2) : (wave >> 1);
    const int kblock = kblock4 & 1, group = kblock4 >> 1;
    const int k = k0 + kblock4 * 16 + (lane & 15);
    LaneContext cx;
    cx.table_k = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
    cx.parked = nullptr;
    constexpr bool PARKED = SUMS && MODE == WG_SCALED;
    int8_t* const scale_area = lds + 2 * kLdsBytes + pw * kParkedScaleBytes;   // behind the two plane buffers: 1 KB per product wave
    constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) +
                           filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, NP);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;
    v4i Y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) Y[i] = (v4i){0, 0, 0, 0};
    // SUMS: the product waves do no output transform per block.  Scaled: all 36 limb-product
    // accumulators stay resident (PW = 4), or 18 joined channel sums (PW = 8: 168 registers per wave); lossless: 18
    // joined channel sums (54 accumulators would not fit).
    constexpr bool RESIDENT = SUMS && MODE == WG_SCALED && PW == 4;
    constexpr int kLeanRing = PW == 8 ? (MODE == WG_SCALED ? 10 : 6) : 8;
    std::conditional_t<RESIDENT, ResidentScaled<0>, LeanProducts<MODE, 0, SUMS, kLeanRing>> phase0;
    std::conditional_t<RESIDENT, ResidentScaled<1>, LeanProducts<MODE, 1, SUMS, kLeanRing>> phase1;
    constexpr int kSumRegs = RESIDENT ? 36 : (SUMS ? kChannelSums : 1);
    v4i sums[kSumRegs];
    if constexpr (SUMS) {
#pragma unroll
        for (int i = 0; i < kSumRegs; ++i) sums[i] = (v4i){0, 0, 0, 0};
    }
    if constexpr (PW == 8) {
        // one loop per half (the same barriers in both), so that each is allocated registers on its own
        auto blocks = [&](auto& phase, auto H) {
            // the first block's filter prefetch goes out between the request for the reverse-scaling factors and their parking
            ParkedScales<H> scales;
            if constexpr (PARKED) scales.ask(cx, lane);
            cx.b_glob = b_lane;
            phase.prefetch(cx);
            if constexpr (PARKED) scales.park(cx, scale_area, lane);
            for (int cb = 0; cb < p.CB; ++cb) {
                if (cb > 0) {
                    cx.b_glob = b_lane + cb * b_block_stride;
                    phase.prefetch(cx);
                }
                WG_SPENT(3, mark);   // ring prefetch issue
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();   // barrier cb + 1
                WG_SPENT(0, mark);   // barrier
                cx.a_lds = lds + (cb & 1) * kLdsBytes + lds_slot(lane >> 4, lane & 15) * 16;
                phase.run(cx, sums, Y);
                WG_SPENT(2, mark);   // products
            }
        };
        if (half == 0) blocks(phase0, std::integral_constant<int, 0>{}); else blocks(phase1, std::integral_constant<int, 1>{});
    } else {
        cx.b_glob = b_lane;
        if (half == 0) {
            ParkedScales<0> scales;
            if constexpr (PARKED) scales.ask(cx, lane);
            phase0.prefetch(cx);
            if constexpr (PARKED) scales.park(cx, scale_area, lane);
        } else {
            ParkedScales<1> scales;
            if constexpr (PARKED) scales.ask(cx, lane);
            phase1.prefetch(cx);
            if constexpr (PARKED) scales.park(cx, scale_area, lane);
        }
        for (int cb = 0; cb < p.CB; ++cb) {
            if (cb > 0) {
                cx.b_glob = b_lane + cb * b_block_stride;
                if (half == 0) phase0.prefetch(cx); else phase1.prefetch(cx);
            }
            WG_SPENT(3, mark);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();   // barrier cb + 1
            WG_SPENT(0, mark);
            cx.a_lds = lds + (cb & 1) * kLdsBytes + lds_slot(lane >> 4, lane & 15) * 16;
            if constexpr (RESIDENT) {
                if (half == 0) phase0.run(cx, sums); else phase1.run(cx, sums);
            } else {
                if (half == 0) phase0.run(cx, sums, Y); else phase1.run(cx, sums, Y);
            }
            WG_SPENT(2, mark);
        }
    }
#ifdef WG_TIMESTAMPS
    report();
#endif
    if constexpr (RESIDENT) {
        if (half == 0) ResidentScaled<0>::finish(cx, sums, Y);
        else           ResidentScaled<1>::finish(cx, sums, Y);
    } else if constexpr (SUMS && MODE == WG_SCALED) {
        if (half == 0) ScaledSums<0>::template finish<0, true>(cx, sums, Y);
        else           ScaledSums<1>::template finish<0, true>(cx, sums, Y);
    } else if constexpr (SUMS) {
        if (half == 0) LeanProducts<MODE, 0, true>::finish_lossless(sums, Y);
        else           LeanProducts<MODE, 1, true>::finish_lossless(sums, Y);
    }
    const int my_row = 4 * my_ty, my_col = 4 * my_tx;
    int my_origin = -1;
    if (tile0 + (lane & 15) < p.T)
        my_origin = LAYOUT == WG_NHWC ? ((my_n * p.H + my_row) * p.W + my_col) * p.K
                                      : (my_n * p.K * p.H + my_row) * p.W + my_col;
    if constexpr (PW == 8) {
        // the two 32-filter halves of the workgroup stage in one operand buffer each and store side by side (the host
        // gives this form only channels-last outputs with K % 4 = 0, the layout store_block's two parts exist for)
        const int gtid = (2 * half + kblock) * 64 + lane;
        const StoreContext sc = {lds + group * kLdsBytes, gtid, lane, 2 * half + kblock, half, kblock, my_n, my_row, my_col, my_origin,
                                 MODE == WG_SCALED ? 8 : 0, y};
        __syncthreads();   // the operand planes are dead
        store_block<LAYOUT, Q8, 1>(sc, p, q8, Y, k0 + group * kFusedFilters);
        __syncthreads();
        store_block<LAYOUT, Q8, 2>(sc, p, q8, Y, k0 + group * kFusedFilters);
#ifdef WG_TIMESTAMPS
        if (g_roles_stamps != nullptr && lane == 0)
            g_roles_stamps[((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 12 + wave8) * 8 + 5] = WG_CLOCK() - entered;
#endif
    } else {
        const StoreContext sc = {lds, tid, lane, wave, half, kblock, my_n, my_row, my_col, my_origin,
                                 MODE == WG_SCALED ? 8 : 0, y};
        __syncthreads();   // the operand planes are dead
        store_block<LAYOUT, Q8>(sc, p, q8, Y, k0);
#ifdef WG_TIMESTAMPS
        if (g_roles_stamps != nullptr && lane == 0)
            g_roles_stamps[((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 12 + wave8) * 8 + 5] = WG_CLOCK() - entered;
#endif
    }
}

template <int LAYOUT, bool VEC4, int MODE, bool SUMS, bool Q8, int PW = 4>
hipError_t launch_roles(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                        const Int8Epilogue& q8, hipStream_t s) {
    constexpr int lds_bytes = 2 * kLdsBytes + PW * kParkedScaleBytes;   // two plane buffers, the parked reverse-scaling factors
    static_assert(lds_bytes <= 160 * 1024, "fits the LDS of a compute unit");
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&fused_conv_roles_kernel<LAYOUT, VEC4, MODE, SUMS, Q8, PW>), lds_bytes)) return e;
    dim3 grid(ceil_div(p.T, kFusedTiles), p.Kp / (kFusedFilters * (PW / 4)));   // Kp is a multiple of 64
    fused_conv_roles_kernel<LAYOUT, VEC4, MODE, SUMS, Q8, PW><<<grid, 64 * (4 + PW), lds_bytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, p, q8);
    return hipGetLastError();
}

// Compute units of the current device (256 on MI355X), asked once.
int compute_units() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            return n;
        return 256;
    }();
    return cus;
}

// Barrier among the four transform waves of the streaming kernel (s_barrier would stop the product
// waves as well): a counter in LDS that only grows, four arrivals per use.  A wave arrives once its
// own LDS reads have returned and leaves when all four have arrived, so no wave writes the shared
// buffer while another still reads it.  Every transform wave runs the same (workgroup-uniform)
// sequence of uses, and all four are resident together, so the wait ends.
struct TransformWavesBarrier {
    uint32_t* counter;
    uint32_t arrivals;   // what the counter reads once everyone has arrived at the current use
    __device__ inline void sync(int lane) {
        arrivals += 4;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (lane == 0) __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        while ((int)(__hip_atomic_load(counter, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) - arrivals) < 0)
            __builtin_amdgcn_s_sleep(1);
        asm volatile("" ::: "memory");
    }
};

// The role-specialised kernel as a stream over tile blocks: a workgroup owns one 32-filter block
// and walks over many tile blocks (grid: about one workgroup per compute unit), so that the two
// roles also overlap across tile blocks and layers with a single channel block are pipelined
// too.  A unit u is one (tile block, channel block); the transform waves are one unit ahead of
// the product waves, and they also take over the second half of the store: at the end of a
// tile block the product waves only stage their outputs in LDS (in the buffer whose planes
// they have just consumed), and the transform waves add the halves and write them out while
// the product waves already multiply the next unit.
// Barriers, in the same order on both roles: U_u (u = 1..U) publishes the planes of unit u - 1 and
// frees the buffer of unit u - 2; after the last channel block of a tile block, D_u (every product
// wave has finished reading the planes) and S_u (the outputs are staged).
// The staged outputs of unit u - 2 and the planes of unit u share a buffer, and the four transform
// waves both read the former (each thread reads rows that other waves' plane writes cover) and
// write the latter: between the two they meet at a barrier of their own (TransformWavesBarrier;
// the product waves, which are multiplying unit u - 1 in the other buffer, do not take part).
// Channels-last, C % 4 = 0 (4-byte pixel loads), K % 4 = 0 (16-byte stores).
// WIDE: 64 filters per workgroup.  Each product wave owns every entry of its 16 filters (and keeps no
// channel sums: see the product side), so one transform serves twice the filters, no halves are added, and
// the workgroup stages one finished copy of its outputs (32 filters in the place of each half), which the
// transform waves write out.
template <int MODE, bool Q8, bool WIDE = false>
__global__ __launch_bounds__(512) void fused_conv_stream_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                                size_t table_off, size_t planes_off, int32_t* __restrict__ y,
                                                                Problem p, Int8Epilogue q8, int tile_blocks) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int lane = threadIdx.x & 63, wave8 = threadIdx.x >> 6;
    const bool transforms = wave8 < 4;
    const int tid = threadIdx.x & 255, wave = wave8 & 3;   // within the role
    const int k0 = blockIdx.y * kFusedFilters * (WIDE ? 2 : 1);
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    // this workgroup's tile blocks: blockIdx.x, blockIdx.x + gridDim.x, ...
    const int my_blocks = (tile_blocks - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int units = my_blocks * p.CB;
    const int rnd = MODE == WG_SCALED ? 8 : 0;
#ifdef WG_TIMESTAMPS
    // ticks per part of the unit loop, summed per wave: 8 numbers per wave, 12 wave slots per workgroup
    unsigned long long spent[6] = {0, 0, 0, 0, 0, 0}, mark = WG_CLOCK();
    const unsigned long long entered = mark;
    auto report = [&]() {
        if (g_roles_stamps != nullptr && lane == 0) {
            unsigned long long* o = g_roles_stamps + ((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 12 + wave8) * 8;
            for (int i = 0; i < 6; ++i) o[i] = spent[i];
            o[6] = WG_CLOCK() - entered;
            o[7] = (unsigned long long)units;
        }
    };
#endif

    if (transforms) {
        const int a_tile = tid >> 4, a_cq = tid & 15;
        OperandSplitter<MODE == WG_SCALED ? kSplitByteLimbs : kSplitTwoLimb, LdsPlaneSink> out;
        int8_t* const slot = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;
        uint32_t patch[6][6], pixel[36];
        int a_t = 0, a_ty = 0, a_tx = 0;
        // identity of the thread's tile in tile block tb, and the 36 pixel offsets of its patch
        auto enter_tile_block = [&](int tb) {
            a_t = tb * kFusedTiles + a_tile;
            int a_n = 0;
            a_ty = 0; a_tx = 0;
            if (a_t < p.T) decode_tile(p, a_t, a_n, a_ty, a_tx);
            patch_offsets(p, a_n, a_ty, a_tx, 4 * a_cq, pixel);
        };
        const __amdgpu_buffer_rsrc_t xbuf = activation_buffer(x, p);
        auto request = [&](int cb) { request_patch(xbuf, p, pixel, cb, 4 * a_cq, patch); };
        // adds the two halves staged in `buffer` for tile block tb and writes them out
        auto flush = [&](int tb, int buffer) {
            int n = 0, ty = 0, tx = 0;
            const int t = tb * kFusedTiles + (lane & 15);
            if (t < p.T) decode_tile(p, t, n, ty, tx);
            const int row = 4 * ty, col = 4 * tx;
            const int origin = t < p.T ? ((n * p.H + row) * p.W + col) * p.K : -1;
            v4i none[16];
            if constexpr (WIDE) {
                constexpr int kCopyBytes = 16 * 16 * 36 * 4;   // one staged copy of 32 filters (store_block's layout)
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const StoreContext sc = {lds + buffer * kLdsBytes + g * kCopyBytes, tid, lane, wave, 0, 0, n, row, col, origin, rnd, y};
                    store_block<WG_NHWC, Q8, 3>(sc, p, q8, none, k0 + g * kFusedFilters);
                }
            } else {
                const StoreContext sc = {lds + buffer * kLdsBytes, tid, lane, wave, 0, 0, n, row, col, origin, rnd, y};
                store_block<WG_NHWC, Q8, 2>(sc, p, q8, none, k0);
            }
        };
        TransformWavesBarrier among_us = {reinterpret_cast<uint32_t*>(lds + 2 * kLdsBytes), 0u};
        if (tid == 0) *among_us.counter = 0u;   // lands before the first s_barrier, long before the first use
        int cb = 0, jb = 0;   // unit u = (tile block number jb of this workgroup, channel block cb)
        if (units > 0) {
            enter_tile_block(blockIdx.x);
            request(0);
        }
        // was unit v the last channel block of its tile block?  v % CB == CB - 1, tracked without division:
        // last1 = for unit u - 1, last2 = for unit u - 2; tb1 / tb2 = their tile blocks
        bool last1 = false, last2 = false;
        int tb1 = 0, tb2 = 0;
        for (int u = 0; u <= units; ++u) {
            WG_SPENT(5, mark);   // requests
            if (u > 0) {   // U_u
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
            }
            WG_SPENT(0, mark);   // barrier U
            if (last2) {   // staged in the buffer of unit u - 2, which unit u is about to overwrite
                flush(tb2, u & 1);
                among_us.sync(lane);   // every transform wave has read its share before any of them writes planes
            }
            WG_SPENT(1, mark);   // flush
            const int tb = (int)blockIdx.x + jb * (int)gridDim.x;
            if (u < units) {
                out.sink.base = slot + (u & 1) * kLdsBytes;
                if (a_t < p.T) {
#ifdef WG_TIMESTAMPS
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                    WG_SPENT(2, mark);   // wait for the patch
#endif
                    bias_buffer_patch(patch);
                    transform_patch(patch, out);
                }
            }
            WG_SPENT(3, mark);   // transform
            const bool last0 = u < units && cb == p.CB - 1;
            if (u < units) {   // next unit's patch, asked for before the waits below so that they cover its latency
                if (++cb == p.CB) { cb = 0; ++jb; }
                if (u + 1 < units) {
                    if (cb == 0) enter_tile_block((int)blockIdx.x + jb * (int)gridDim.x);
                    if (a_t < p.T) request(cb);
                }
            }
            WG_SPENT(5, mark);   // requests
            if (last1) {   // D_{u-1}, S_{u-1}
                __syncthreads();
                __syncthreads();
            }
            WG_SPENT(4, mark);   // barriers D and S
            last2 = last1; tb2 = tb1;
            last1 = last0; tb1 = tb;
        }
        if (last2) flush(tb2, (units + 1) & 1);   // the last tile block, staged in the buffer of unit U - 1
#ifdef WG_TIMESTAMPS
        report();
#endif
        return;
    }

    // WIDE: wave w owns filters 16 w .. 16 w + 15 of the 64 and every entry; in the staging it stands where wave
    // (half = w / 2, kblock = w % 2) of a 32-filter workgroup stands, so that copy w / 2 holds filters 32 (w / 2) ..
    const int kblock = wave & 1, half = wave >> 1;
    const int k = k0 + (WIDE ? wave : kblock) * 16 + (lane & 15);
    LaneContext cx;
    cx.table_k = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
    cx.parked = nullptr;
    // behind the plane buffers and the barrier counter
    int8_t* const scale_area = lds + 2 * kLdsBytes + 64 + wave * (WIDE ? ParkedScales<kAllRows>::kBytes : kParkedScaleBytes);
    constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) +
                           filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, NP);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;
    if constexpr (WIDE) {
        // Every entry of 16 filters in one wave.  36 joined channel sums next to the fragments would not fit the registers,
        // so each channel block's products go through the reverse scaling and the output transform at once and the
        // outputs accumulate: exact in lossless mode (the transform is linear); in scaled mode the reverse scaling applies
        // to the channel sum (Section 4.2), so there the host uses this form for one-block layers only.
        // filter ring: lossless mode has twice the fragments per entry and the registers for twelve in flight
        LeanProducts<MODE, kAllRows, false, MODE == WG_SCALED ? 8 : 12, true, true> all;
        v4i unused[1];
        v4i Y[16];
        int cb = 0;
        if (units > 0) {
            cx.b_glob = b_lane;
            ParkedScales<kAllRows> scales;
            if constexpr (MODE == WG_SCALED) scales.ask(cx, lane);
            all.prefetch(cx);
            if constexpr (MODE == WG_SCALED) scales.park(cx, scale_area, lane);
        }
        for (int u = 0; u < units; ++u) {
            if (cb == 0) {
#pragma unroll
                for (int i = 0; i < 16; ++i) Y[i] = (v4i){0, 0, 0, 0};
            }
            WG_SPENT(5, mark);   // clearing the outputs
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();   // U_{u+1}
            WG_SPENT(0, mark);   // barrier U
            cx.a_lds = lds + (u & 1) * kLdsBytes + lds_slot(lane >> 4, lane & 15) * 16;
            all.run(cx, unused, Y);
            WG_SPENT(1, mark);   // products
            const bool last = cb == p.CB - 1;
            cb = last ? 0 : cb + 1;
            if (u + 1 < units) {   // the next unit's first filter fragments travel while this one is staged
                cx.b_glob = b_lane + cb * b_block_stride;
                all.prefetch(cx);
            }
            if (last) {
                WG_SPENT(2, mark);   // prefetch issue
                __syncthreads();   // D_u: every product wave has finished reading this unit's planes
                WG_SPENT(3, mark);   // barrier D
                const StoreContext sc = {lds + (u & 1) * kLdsBytes, tid, lane, wave, half, kblock, 0, 0, 0, -1, rnd, y};
                store_block<WG_NHWC, Q8, 1>(sc, p, q8, Y, k0);
                __syncthreads();   // S_u: staged
                WG_SPENT(4, mark);   // staging and barrier S
            }
        }
#ifdef WG_TIMESTAMPS
        report();
#endif
        return;
    }
    // 18 joined channel sums per wave in both modes (36 resident accumulators plus the outputs
    // would not fit the 256 registers here)
    // scaled mode has the registers for a second set of activation fragments (lossless mode would spill)
    LeanProducts<MODE, 0, true, 8, MODE == WG_SCALED> phase0;
    LeanProducts<MODE, 1, true, 8, MODE == WG_SCALED> phase1;
    constexpr int kSumRegs = kChannelSums;
    v4i sums[kSumRegs];
    v4i Y[16];
    int cb = 0;
    if (units > 0) {
        // the first unit's filter prefetch goes out between the request for the reverse-scaling factors and their parking
        cx.b_glob = b_lane;
        if (half == 0) {
            ParkedScales<0> scales;
            if constexpr (MODE == WG_SCALED) scales.ask(cx, lane);
            phase0.prefetch(cx);
            if constexpr (MODE == WG_SCALED) scales.park(cx, scale_area, lane);
        } else {
            ParkedScales<1> scales;
            if constexpr (MODE == WG_SCALED) scales.ask(cx, lane);
            phase1.prefetch(cx);
            if constexpr (MODE == WG_SCALED) scales.park(cx, scale_area, lane);
        }
    }
    for (int u = 0; u < units; ++u) {
        if (cb == 0) {
#pragma unroll
            for (int i = 0; i < kSumRegs; ++i) sums[i] = (v4i){0, 0, 0, 0};
        }
        WG_SPENT(5, mark);   // clearing the sums
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();   // U_{u+1}
        WG_SPENT(0, mark);   // barrier U
        cx.a_lds = lds + (u & 1) * kLdsBytes + lds_slot(lane >> 4, lane & 15) * 16;
        if (half == 0) phase0.run(cx, sums, Y); else phase1.run(cx, sums, Y);
        WG_SPENT(1, mark);   // products
        const bool last = cb == p.CB - 1;
        cb = last ? 0 : cb + 1;
        if (u + 1 < units) {   // the next unit's first filter fragments travel while this one is finished and staged
            cx.b_glob = b_lane + cb * b_block_stride;
            if (half == 0) phase0.prefetch(cx); else phase1.prefetch(cx);
        }
        if (last) {
#pragma unroll
            for (int i = 0; i < 16; ++i) Y[i] = (v4i){0, 0, 0, 0};
            if constexpr (MODE == WG_SCALED) {
                if (half == 0) ScaledSums<0>::template finish<0, true>(cx, sums, Y);
                else           ScaledSums<1>::template finish<0, true>(cx, sums, Y);
            } else {
                if (half == 0) LeanProducts<MODE, 0, true>::finish_lossless(sums, Y);
                else           LeanProducts<MODE, 1, true>::finish_lossless(sums, Y);
            }
            WG_SPENT(2, mark);   // finish
            __syncthreads();   // D_u: every product wave has finished reading this unit's planes
            WG_SPENT(3, mark);   // barrier D
            const StoreContext sc = {lds + (u & 1) * kLdsBytes, tid, lane, wave, half, kblock, 0, 0, 0, -1, rnd, y};
            store_block<WG_NHWC, Q8, 1>(sc, p, q8, Y, k0);
            __syncthreads();   // S_u: staged
            WG_SPENT(4, mark);   // staging and barrier S
        }
    }
#ifdef WG_TIMESTAMPS
    report();
#endif
}

// Workgroups per filter block of the streaming kernel: about one workgroup per compute unit in
// total (a test hook can set a smaller number, so that small problems stream, too).
std::atomic<int> g_stream_workgroups{0};
// Test hook for the streaming kernel's 64-filter form: 0 the library's choice, 1 wherever a layer streams, 2 never.
std::atomic<int> g_stream_variant{0};
int stream_workgroups(int tile_blocks, int filter_blocks) {
    const int forced = g_stream_workgroups.load(std::memory_order_relaxed);
    if (forced > 0) return std::max(1, std::min(tile_blocks, forced));
    // as many as the compute units allow, then as few as still finish in the same number of rounds
    const int wanted = std::max(1, compute_units() / filter_blocks);
    const int rounds = ceil_div(tile_blocks, wanted);
    return std::max(1, ceil_div(tile_blocks, rounds));
}

template <int MODE, bool Q8, bool WIDE = false>
hipError_t launch_stream(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                         const Int8Epilogue& q8, hipStream_t s) {
    // two plane buffers, the transform waves' barrier counter, the parked reverse-scaling factors
    constexpr int lds_bytes = 2 * kLdsBytes + 64 + 4 * (WIDE ? ParkedScales<kAllRows>::kBytes : kParkedScaleBytes);
    static_assert(lds_bytes <= 160 * 1024, "fits the LDS of a compute unit");
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&fused_conv_stream_kernel<MODE, Q8, WIDE>), lds_bytes)) return e;
    const int tile_blocks = ceil_div(p.T, kFusedTiles), filter_blocks = p.Kp / (kFusedFilters * (WIDE ? 2 : 1));   // Kp is a multiple of 64
    const int gx = stream_workgroups(tile_blocks, filter_blocks);
    fused_conv_stream_kernel<MODE, Q8, WIDE><<<dim3(gx, filter_blocks), 512, lds_bytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, p,
                                                                                           q8, tile_blocks);
    return hipGetLastError();
}

template <int LAYOUT, int LOAD, int MODE, bool SUMS, bool WIDE, bool Q8>
hipError_t launch(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                  const Int8Epilogue& q8, hipStream_t s) {
    constexpr int lds_bytes = kLdsBytes + (LOAD == kLoadDirect ? kRawBytes : 0);
    const void* kernel = Q8 ? reinterpret_cast<const void*>(&fused_conv_int8_kernel<LAYOUT, LOAD, MODE, SUMS, WIDE>)
                            : reinterpret_cast<const void*>(&fused_conv_kernel<LAYOUT, LOAD, MODE, SUMS, WIDE>);
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(kernel, lds_bytes)) return e;
    dim3 grid(ceil_div(p.T, kFusedTiles), p.Kp / (kFusedFilters * (WIDE ? 2 : 1)));
    if constexpr (Q8)
        fused_conv_int8_kernel<LAYOUT, LOAD, MODE, SUMS, WIDE><<<grid, 256, lds_bytes, s>>>(x, blob, bl.table_off, bl.planes_off, p, q8);
    else
        fused_conv_kernel<LAYOUT, LOAD, MODE, SUMS, WIDE><<<grid, 256, lds_bytes, s>>>(x, blob, bl.table_off, bl.planes_off, y, p);
    return hipGetLastError();
}

template <int LAYOUT, int LOAD, bool Q8>
hipError_t launch_mode(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                       int mode, const Int8Epilogue& q8, hipStream_t s) {
    // 64 filters per workgroup once the 32-filter grid would need more than one round of the
    // compute units (Kp is a multiple of 64).  Only the direct-transfer variants have the
    // registers for it (the others hold a patch in registers across the product phase).
    if constexpr (LOAD == kLoadDirect) {
        const long long workgroups = (long long)ceil_div(p.T, kFusedTiles) * (p.Kp / kFusedFilters);
        if (workgroups > compute_units()) {
            if (mode == WG_LOSSLESS) return launch<LAYOUT, LOAD, WG_LOSSLESS, false, true, Q8>(x, blob, bl, y, p, q8, s);
            // scaled mode keeps channel sums here also for a single channel block: the variant that
            // reduces each entry at once needs more registers than a wave has when it covers 64 filters
            return launch<LAYOUT, LOAD, WG_SCALED, true, true, Q8>(x, blob, bl, y, p, q8, s);
        }
    }
    if (mode == WG_LOSSLESS) return launch<LAYOUT, LOAD, WG_LOSSLESS, false, false, Q8>(x, blob, bl, y, p, q8, s);
    if (p.CB == 1) return launch<LAYOUT, LOAD, WG_SCALED, false, false, Q8>(x, blob, bl, y, p, q8, s);
    return launch<LAYOUT, LOAD, WG_SCALED, true, false, Q8>(x, blob, bl, y, p, q8, s);
}

std::atomic<int> g_scaled_variant{0};

template <bool Q8>
hipError_t launch_roles_mode(const int8_t* x, const uint8_t* b, const BlobLayout& bl, int32_t* y, const Problem& p,
                             int mode, const Int8Epilogue& q8, hipStream_t s, bool wide = false) {
    if (mode == WG_LOSSLESS && wide) return launch_roles<WG_NHWC, true, WG_LOSSLESS, true, Q8, 8>(x, b, bl, y, p, q8, s);
    if (mode == WG_LOSSLESS) return launch_roles<WG_NHWC, true, WG_LOSSLESS, true, Q8>(x, b, bl, y, p, q8, s);
    if (wide) return launch_roles<WG_NHWC, true, WG_SCALED, true, Q8, 8>(x, b, bl, y, p, q8, s);
    return launch_roles<WG_NHWC, true, WG_SCALED, true, Q8>(x, b, bl, y, p, q8, s);
}

template <bool Q8>
hipError_t launch_layout(const int8_t* x, const uint8_t* b, const BlobLayout& bl, int32_t* y, const Problem& p,
                         int layout, int mode, const Int8Epilogue& q8, hipStream_t s) {
    if (layout == WG_NHWC && p.C % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0)
        return launch_mode<WG_NHWC, kLoadDirect, Q8>(x, b, bl, y, p, mode, q8, s);
    if (layout == WG_NHWC && p.C % 4 == 0) return launch_mode<WG_NHWC, kLoadDwords, Q8>(x, b, bl, y, p, mode, q8, s);
    if (layout == WG_NHWC) return launch_mode<WG_NHWC, kLoadBytes, Q8>(x, b, bl, y, p, mode, q8, s);
    return launch_mode<WG_NCHW, kLoadBytes, Q8>(x, b, bl, y, p, mode, q8, s);
}

// ---- activations scaled as well (the remark that closes Section 4.1) --------------------------------------------
// Section 4.1 ends by noting that the analysis of Section 4.2 applies to B^T d B too (12 bits here for int8 data).
// The rule used is that section's with a tile in the place of an output feature map: at each of a tile's 26 free
// entries the largest max(|Re|, |Im|) over the input channels decides one factor n/2^p, Re and Im of every channel's
// value there are multiplied by it (round half up), and the channel sums are multiplied back by its reciprocal r/2^q
// after the filter's.  Both operands are then single int8 values: one matrix-core instruction per real product, 36
// operand planes instead of 72, channel sums accumulated by the matrix cores themselves.
//
// (n, p, r, q) for every possible maximum of int8 data, one byte each (n = 0: within the range, nothing applied).
constexpr int kActMax = 16 * 128;
struct ActScaleTable {
    uint32_t v[kActMax + 1];
};
constexpr ActScaleTable make_act_scale_table() {
    ActScaleTable t = {};
    for (int mx = 0; mx <= kActMax; ++mx) {
        uint32_t n = 0, p = 0, r = 1, q = 0;
        if (mx > kWeightRange) {
            const int num = kWeightRange * 128;
            int y = 0;
            while ((mx << (y + 1)) <= num) ++y;
            n = (uint32_t)((num * 8) / (mx << y));
            p = (uint32_t)(10 - y);
            for (int qq = 7; qq >= 0; --qq) {
                const uint32_t rr = ((2u << (p + qq)) + n) / (2 * n);
                if (rr <= 255) { r = rr; q = (uint32_t)qq; break; }
            }
        }
        t.v[mx] = n | (p << 8) | (r << 16) | (q << 24);
    }
    return t;
}
__device__ const ActScaleTable kActScale = make_act_scale_table();

constexpr int kActPlanes = 36;                       // 16 real entries, then (Re, Im) of each complex entry
static_assert(kActPlanes * kPlaneBytes <= kLdsBytes, "the single-limb planes lie where the two-limb planes do");
constexpr int kActNpOff = kLdsBytes;                 // v4i [tile][26]: (n, n), (half, half), (p, p) in 16-bit pairs
constexpr int kActRqOff = kActNpOff + 16 * kEntries * 16;   // uint32 [26][tile]: the table entry (r, q in its upper bytes)
constexpr int kActLdsBytes = kActRqOff + kEntries * 16 * 4;

__device__ inline s16x2 abs_max(Quad v) {
    const s16x2 zero = {0, 0};
    return __builtin_elementwise_max(__builtin_elementwise_max(v.a, zero - v.a), __builtin_elementwise_max(v.b, zero - v.b));
}
// transform_patch's receiver in the first pass: running maxima per free entry, two channels per register
struct MaxKeeper {
    s16x2* mx;
    __device__ inline void real_entry(int p, Quad v) const { mx[p] = __builtin_elementwise_max(mx[p], abs_max(v)); }
    __device__ inline void complex_entry(int j, Quad re, Quad im) const {
        mx[kRealEntries + j] = __builtin_elementwise_max(mx[kRealEntries + j], __builtin_elementwise_max(abs_max(re), abs_max(im)));
    }
};
// ... and in the second: every value times its tile's factor, rounded half up, as one int8 operand plane
struct ScaledPlanes {
    LdsPlaneSink sink;
    const v4i* np;   // this tile's 26 factors
    __device__ inline uint32_t scaled(int entry, Quad v) const {
        const v4i t = np[entry];
        const s16x2 mul = as_s16x2((uint32_t)t[0]), half = as_s16x2((uint32_t)t[1]), sh = as_s16x2((uint32_t)t[2]);
        return pack_low_bytes(Quad{(v.a * mul + half) >> sh, (v.b * mul + half) >> sh});
    }
    __device__ inline void real_entry(int p, Quad v) const { sink.put(p, scaled(p, v)); }
    __device__ inline void complex_entry(int j, Quad re, Quad im) const {
        sink.put(kRealEntries + 2 * j, scaled(kRealEntries + j, re));
        sink.put(kRealEntries + 2 * j + 1, scaled(kRealEntries + j, im));
    }
};

// Product phase: the channel sums of a wave's entries (18 of four registers) are the matrix cores' accumulators.
//   real:    sum += D W;    complex: Re += Dr Wr + Di (-Wi),  Im += Dr Wi + Di Wr
// Filter fragments come from the scaled blob in ProductPhase<WG_SCALED>'s order (W; Wr, Wi, -Wi).
template <int HALF>
struct BothScaledSums {
    using Phase = ProductPhase<WG_SCALED, HALF>;
    static constexpr int NE = Phase::NE, NB = Phase::NB;
    static constexpr int sum_start(int slot) { return ScaledSums<HALF>::sum_start(slot); }
    template <int SLOT, int I>
    __device__ inline static v4i load_a(const LaneContext& cx) {
        constexpr int entry = half_slot(HALF, SLOT).entry;
        constexpr int plane = is_real(entry) ? entry : kRealEntries + 2 * (entry - kRealEntries) + I;
        return *reinterpret_cast<const v4i*>(cx.a_lds + plane * kPlaneBytes);
    }
    __device__ inline static void run(const LaneContext& cx, v4i (&bring)[kFilterPrefetch], v4i (&sums)[kChannelSums]) {
        v4i afr[2][2];
        afr[0][0] = load_a<0, 0>(cx);
        if constexpr (!is_real(half_slot(HALF, 0).entry)) afr[0][1] = load_a<0, 1>(cx);
        static_for<NE>([&](auto S) {
            constexpr int s = S;
            constexpr int entry = half_slot(HALF, s).entry;
            constexpr int b0 = b_start<WG_SCALED>(HALF, s), v = sum_start(s);
            if constexpr (s + 1 < NE) {
                afr[(s + 1) & 1][0] = load_a<s + 1, 0>(cx);
                if constexpr (!is_real(half_slot(HALF, s + 1).entry)) afr[(s + 1) & 1][1] = load_a<s + 1, 1>(cx);
            }
            auto mac = [&](int a, int b, int sum) {
                sums[sum] = __builtin_amdgcn_mfma_i32_16x16x64_i8(afr[s & 1][a], bring[(b0 + b) % kFilterPrefetch], sums[sum], 0, 0, 0);
            };
            if constexpr (is_real(entry)) {
                mac(0, 0, v);
            } else {
                mac(0, 0, v);        // Dr Wr
                mac(0, 1, v + 1);    // Dr Wi
                mac(1, 2, v);        // Di (-Wi)
                mac(1, 0, v + 1);    // Di Wr
            }
            static_for<num_b<WG_SCALED>(entry)>([&](auto I) {
                if constexpr (b0 + I + kFilterPrefetch < NB)
                    bring[(b0 + I) % kFilterPrefetch] = Phase::template load_b<b0 + I + kFilterPrefetch>(cx);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    // After the last channel block: the filter's reverse scaling, then the tile's (register q of a lane belongs to
    // tile 4 (lane / 16) + q), and the output transform.
    __device__ inline static void finish(const LaneContext& cx, const uint32_t* rq_tab, int lane, const v4i (&sums)[kChannelSums],
                                         v4i (&Y)[16]) {
        v4i er[6], ei[6];
        static_for<NE>([&](auto S) {
            constexpr Slot sl = half_slot(HALF, S);
            constexpr int v = sum_start(S);
            v4i re = sums[v], im = {0, 0, 0, 0};
            if constexpr (!is_real(sl.entry)) im = sums[v + 1];
            const ReverseScale filter_side(cx.table_k[sl.entry]);
            const v4i rq = *reinterpret_cast<const v4i*>(rq_tab + sl.entry * 16 + 4 * (lane >> 4));
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const ReverseScale tile_side((int)(((uint32_t)rq[q] >> 16) & 255u), (int)((uint32_t)rq[q] >> 24));
                re[q] = tile_side(filter_side(re[q]));
                if constexpr (!is_real(sl.entry)) im[q] = tile_side(filter_side(im[q]));
            }
            er[sl.pos] = re;
            ei[sl.pos] = im;
            if constexpr (sl.last_in_row) finish_row<sl.row>(er, ei, Y);
        });
    }
};

// grid (ceil(T/16), Kp/32), 256 threads with the roles of fused_conv_body; the blob is a WG_SCALED one of signed int8
// filters.  Pass 1 transforms every channel block of the workgroup's 16 tiles and keeps the running maxima; each
// thread then looks up the factors of one or two (tile, entry) pairs; pass 2 transforms again (the patches now come
// from the caches), scales, and multiplies.  act_table (may be null) receives int32 [T][26][4] = (n, p, r, q).
template <int LAYOUT, int LOAD>
__global__ __launch_bounds__(256) void fused_conv_act_scaled_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                                    size_t table_off, size_t planes_off, int32_t* __restrict__ y,
                                                                    int32_t* __restrict__ act_table, const Problem p) {
    static_assert(LOAD != kLoadDirect, "the patch is held in registers");
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kblock = wave & 1, half = wave >> 1;
    const int tile0 = blockIdx.x * kFusedTiles, k0 = blockIdx.y * kFusedFilters;
    const int k = k0 + kblock * 16 + (lane & 15);
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, WG_SCALED)) return;

    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + (lane & 15) < p.T) decode_tile(p, tile0 + (lane & 15), my_n, my_ty, my_tx);
    const int a_tile = tid >> 4, a_cq = tid & 15;
    const int a_t = tile0 + a_tile;
    const int a_tx = __shfl(my_tx, a_tile), a_ty = __shfl(my_ty, a_tile), a_n = __shfl(my_n, a_tile);
    v4i* np_tab = reinterpret_cast<v4i*>(lds + kActNpOff);
    uint32_t* rq_tab = reinterpret_cast<uint32_t*>(lds + kActRqOff);
    constexpr bool VEC4 = LOAD == kLoadDwords;
    uint32_t patch[6][6];

    // ---- pass 1: largest magnitude per (tile, entry) over all channels --------------------------------------
    s16x2 mx[kEntries];
#pragma unroll
    for (int e = 0; e < kEntries; ++e) mx[e] = (s16x2){0, 0};
    if (a_t < p.T) {
        load_patch<LAYOUT, VEC4>(x, p, a_n, a_ty, a_tx, 4 * a_cq, patch);
        for (int cb = 0; cb < p.CB; ++cb) {
            bias_patch(p, a_ty, a_tx, cb * kCBlock + 4 * a_cq, patch);
            uint32_t now[6][6];
#pragma unroll
            for (int i = 0; i < 36; ++i) now[i / 6][i % 6] = patch[i / 6][i % 6];
            // the next block's patch, or the first block's again for pass 2, travels meanwhile
            load_patch<LAYOUT, VEC4>(x, p, a_n, a_ty, a_tx, (cb + 1 < p.CB ? cb + 1 : 0) * kCBlock + 4 * a_cq, patch);
            transform_patch(now, MaxKeeper{mx});
        }
    }
    // over the sixteen threads of a tile (consecutive lanes), two entries per register
    s16x2 pm[kEntries / 2];
#pragma unroll
    for (int j = 0; j < kEntries / 2; ++j) {
        pm[j] = (s16x2){max(mx[2 * j].x, mx[2 * j].y), max(mx[2 * j + 1].x, mx[2 * j + 1].y)};
#pragma unroll
        for (int off = 1; off < 16; off <<= 1)
            pm[j] = __builtin_elementwise_max(pm[j], as_s16x2((uint32_t)__shfl_xor((int)as_u32(pm[j]), off)));
    }
    {   // thread (tile, cq) looks up entry cq of its tile, and entry 16 + cq if there is one
        int mine[2] = {0, 0};
#pragma unroll
        for (int e = 0; e < kEntries; ++e)
            if (a_cq == (e & 15)) mine[e >> 4] = (e & 1) ? pm[e / 2].y : pm[e / 2].x;
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const int e = 16 * part + a_cq;
            if (e >= kEntries) break;
            const uint32_t entry = kActScale.v[min(mine[part], kActMax)];
            const uint32_t n = max(entry & 255u, 1u), sh = (entry >> 8) & 255u, hf = (1u << sh) >> 1;
            np_tab[a_tile * kEntries + e] = (v4i){(int)(n * 0x00010001u), (int)(hf * 0x00010001u), (int)(sh * 0x00010001u), 0};
            rq_tab[e * 16 + a_tile] = entry;
            if (act_table != nullptr && blockIdx.y == 0 && a_t < p.T)
                *reinterpret_cast<v4i*>(act_table + ((size_t)a_t * kEntries + e) * 4) =
                    (v4i){(int)(entry & 255u), (int)((entry >> 8) & 255u), (int)((entry >> 16) & 255u), (int)(entry >> 24)};
        }
    }
    __syncthreads();

    // ---- pass 2: scaled operands, products --------------------------------------------------------------------
    ScaledPlanes out;
    out.sink.base = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;
    out.np = np_tab + a_tile * kEntries;
    LaneContext cx;
    cx.a_lds = lds + lds_slot(lane >> 4, lane & 15) * 16;
    cx.table_k = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
    constexpr int NP = 46;
    const int8_t* b_lane = reinterpret_cast<const int8_t*>(blob + planes_off) + filter_plane_offset(0, 0, k, (lane >> 4) * 16, p.Kp, NP);
    const size_t b_block_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;
    ProductPhase<WG_SCALED, 0> phase0;
    ProductPhase<WG_SCALED, 1> phase1;
    v4i sums[kChannelSums];
#pragma unroll
    for (int i = 0; i < kChannelSums; ++i) sums[i] = (v4i){0, 0, 0, 0};
    for (int cb = 0; cb < p.CB; ++cb) {
        cx.b_glob = b_lane + cb * b_block_stride;
        if (half == 0) phase0.prefetch(cx); else phase1.prefetch(cx);
        if (cb > 0) {   // everyone is done reading the previous block's planes
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
        }
        if (a_t < p.T) {
            bias_patch(p, a_ty, a_tx, cb * kCBlock + 4 * a_cq, patch);
            transform_patch(patch, out);
            if (cb + 1 < p.CB) load_patch<LAYOUT, VEC4>(x, p, a_n, a_ty, a_tx, (cb + 1) * kCBlock + 4 * a_cq, patch);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        if (half == 0) BothScaledSums<0>::run(cx, phase0.bring, sums); else BothScaledSums<1>::run(cx, phase1.bring, sums);
    }
    v4i Y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) Y[i] = (v4i){0, 0, 0, 0};
    if (half == 0) BothScaledSums<0>::finish(cx, rq_tab, lane, sums, Y); else BothScaledSums<1>::finish(cx, rq_tab, lane, sums, Y);

    const int my_row = 4 * my_ty, my_col = 4 * my_tx;
    int my_origin = -1;
    if (tile0 + (lane & 15) < p.T)
        my_origin = LAYOUT == WG_NHWC ? ((my_n * p.H + my_row) * p.W + my_col) * p.K : (my_n * p.K * p.H + my_row) * p.W + my_col;
    const StoreContext sc = {lds, tid, lane, wave, half, kblock, my_n, my_row, my_col, my_origin, 8, y};
    __syncthreads();   // the operand planes are dead (the tables lie behind them)
    store_block<LAYOUT, false>(sc, p, Int8Epilogue{}, Y, k0);
}

template <int LAYOUT, int LOAD, int MODE, bool SUMS>
hipError_t launch_u8(const int8_t* x, ZeroPointU8 zero, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                     hipStream_t s) {
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&fused_conv_u8_kernel<LAYOUT, LOAD, MODE, SUMS>), kLdsBytes)) return e;
    dim3 grid(ceil_div(p.T, kFusedTiles), p.Kp / kFusedFilters);
    fused_conv_u8_kernel<LAYOUT, LOAD, MODE, SUMS><<<grid, 256, kLdsBytes, s>>>(x, zero, blob, bl.table_off, bl.planes_off, y, p);
    return hipGetLastError();
}

template <int LAYOUT, int LOAD>
hipError_t launch_u8_mode(const int8_t* x, ZeroPointU8 zero, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                          int mode, hipStream_t s) {
    if (mode == WG_LOSSLESS) return launch_u8<LAYOUT, LOAD, WG_LOSSLESS, false>(x, zero, blob, bl, y, p, s);
    if (p.CB == 1) return launch_u8<LAYOUT, LOAD, WG_SCALED, false>(x, zero, blob, bl, y, p, s);
    return launch_u8<LAYOUT, LOAD, WG_SCALED, true>(x, zero, blob, bl, y, p, s);
}

}  // namespace

// uint8 activations with a zero point: the four-wave kernel with the load paths that select padding pixels explicitly
// (they must read as the zero point, not as zero bytes), for every channel count the int9 path accepts.
hipError_t launch_fused_conv_u8(const uint8_t* x_u8, int zero_point, const void* blob, int32_t* y, const Problem& p, int layout,
                                int mode, hipStream_t s) {
    const BlobLayout bl = blob_layout(p.Kp, p.C, mode);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    const int8_t* x = reinterpret_cast<const int8_t*>(x_u8);
    const ZeroPointU8 zero = make_zero_point(zero_point);
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0)
        return launch_u8_mode<WG_NHWC, kLoadDwords>(x, zero, b, bl, y, p, mode, s);
    if (layout == WG_NHWC) return launch_u8_mode<WG_NHWC, kLoadBytes>(x, zero, b, bl, y, p, mode, s);
    return launch_u8_mode<WG_NCHW, kLoadBytes>(x, zero, b, bl, y, p, mode, s);
}

hipError_t launch_fused_conv_act_scaled(const int8_t* x, const void* blob, int32_t* y, int32_t* act_table, const Problem& p,
                                        int layout, hipStream_t s) {
    const BlobLayout bl = blob_layout(p.Kp, p.C, WG_SCALED);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    dim3 grid(ceil_div(p.T, kFusedTiles), p.Kp / kFusedFilters);
    auto go = [&](auto kernel) -> hipError_t {
        static LdsLimitOnce lds_limit;   // per kernel: the lambda's body is instantiated once per argument type
        if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(kernel), kActLdsBytes)) return e;
        kernel<<<grid, 256, kActLdsBytes, s>>>(x, b, bl.table_off, bl.planes_off, y, act_table, p);
        return hipGetLastError();
    };
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0)
        return go(&fused_conv_act_scaled_kernel<WG_NHWC, kLoadDwords>);
    if (layout == WG_NHWC) return go(&fused_conv_act_scaled_kernel<WG_NHWC, kLoadBytes>);
    return go(&fused_conv_act_scaled_kernel<WG_NCHW, kLoadBytes>);
}

#ifdef WG_TIMESTAMPS
extern "C" int winograd_debug_set_roles_stamps(void* dev_ptr) {
    return hipMemcpyToSymbol(HIP_SYMBOL(g_roles_stamps), &dev_ptr, sizeof dev_ptr) == hipSuccess ? 0 : -5;
}
#endif

void set_scaled_variant(int v) { g_scaled_variant.store(v, std::memory_order_relaxed); }
void set_stream_variant(int v) { g_stream_variant.store(v, std::memory_order_relaxed); }

void set_stream_workgroups(int n) { g_stream_workgroups.store(n > 0 ? n : 0, std::memory_order_relaxed); }

hipError_t launch_fused_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p, int layout, int mode,
                             const Int8Epilogue& q8, hipStream_t s) {
    if (layout == WG_NHWC && p.C <= kNarrowChannels) return launch_narrow_conv(x, blob, y, p, mode, q8, s);
    const BlobLayout bl = blob_layout(p.Kp, p.C, mode);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    // The streaming variant of the role-specialised kernel when every workgroup gets at least six
    // tile blocks to stream over (measured: +10-17 % on the large layers; with fewer, the fill
    // and drain of its pipeline cost more than the overlap saves), or when a test asks for it.
    const bool can_stream = layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0 && (p.K & 3) == 0;
    const int tile_blocks = ceil_div(p.T, kFusedTiles), filter_blocks = p.Kp / kFusedFilters;
    // The 64-filter form of that kernel (see below for when it applies) is also the fastest form for a layer with one
    // channel block as soon as the 32-filter grid exceeds one round of the compute units, whatever the number of tile
    // blocks per workgroup (56x56x64 at N = 12 .. 48: 8-30 % ahead of the limb-pair and 64-filter four-wave kernels).
    const int stream_variant = g_stream_variant.load(std::memory_order_relaxed);
    const bool whole64 = (p.K & 63) == 0 || (p.K & 63) > 32;   // padding to 64 filters adds no 32-filter block of nothing
    const bool wide_one_block = can_stream && p.CB == 1 && whole64 && stream_variant == 0 &&
                                (long long)tile_blocks * filter_blocks > compute_units();
    // Scaled mode, one channel block, a 32-filter grid of at most one round: the streaming kernel's 32-filter form with
    // one tile block per workgroup (its eight waves: four transform, four multiply) is 10-14 % ahead of the four-wave
    // kernel (56x56x64 at N = 8: 9.3 -> 8.5 us); lossless mode has the limb-pair kernel for these layers.
    const bool forced_stream = g_stream_workgroups.load(std::memory_order_relaxed) > 0;
    const bool narrow_one_round = can_stream && mode == WG_SCALED && p.CB == 1 && stream_variant == 0 && !forced_stream &&
                                  (long long)tile_blocks * filter_blocks <= compute_units();
    const bool streams = can_stream && (forced_stream || wide_one_block || narrow_one_round ||
                                        tile_blocks >= 6 * stream_workgroups(tile_blocks, filter_blocks));
    // Lossless mode, channels-last, one channel block, too few tile blocks to stream over: the limb-pair form (eight waves
    // per 16 tiles x 32 filters, lossless_conv.hip) against this file's four-wave forms, by rounds of the compute units:
    // measured on 56x56x64 layers, a round of the former takes 6.5 us, a round of the latter 7.4 us with 32 filters per
    // workgroup (a grid of at most one round) and 11.7 us with 64 filters.
    if (mode == WG_LOSSLESS && !streams) {
        const int form = lossless_pair_conv_choice(x, p, layout);   // 0: not applicable or switched off, 1: the library decides, 2: forced
        const long long w32 = (long long)tile_blocks * filter_blocks, cus = compute_units();
        const double pair_cost = 6.5 * (double)((w32 + cus - 1) / cus);
        const double here_cost = w32 <= cus ? 7.4 : 11.7 * (double)((w32 / 2 + cus - 1) / cus);
        if (form == 2 || (form == 1 && p.CB == 1 && pair_cost < here_cost)) return launch_lossless_pair_conv(x, blob, y, p, q8, s);
    }
    // Channels-last, K % 4 = 0, several channel blocks: the role-specialised kernel with eight product waves and 64 filters
    // per workgroup, as soon as the 32-filter grid would need more than one round of the compute units (with a 64-filter
    // grid of at most half the compute units the 32-filter form, which then fills the chip in one round, stays ahead).
    // Measured on the layers of the VGG-16-shaped stack at N = 16 and on the 128-, 256- and 512-channel configurations.
    // Scaled mode: 15-30 % faster than the streaming, 64-filter four-wave and 32-filter role-specialised forms wherever
    // there are two or more channel blocks.  Lossless mode (twice the matrix-core work and filter bytes per product):
    // +10-25 % with two or more channel blocks where the layer is too small to stream; where it streams, the streaming
    // kernel's 64-filter form is level (two blocks) or 4 % ahead (four blocks) and takes the layer.
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0 && (p.K & 3) == 0) {
        const int variant = g_scaled_variant.load(std::memory_order_relaxed);
        const long long wide_grid = (long long)tile_blocks * (p.Kp / (2 * kFusedFilters));
        // scaled mode also with one channel block, where the 64-filter grid is a single round and the 32-filter grid is not
        // (56x56x64 at N = 16: 11.4 -> 10.9 us against the streaming kernel's 64-filter form)
        const bool deep_enough = (p.CB >= 2 && (mode == WG_SCALED || !streams)) ||
                                 (mode == WG_SCALED && wide_grid <= compute_units());
        if (variant == 1 || (variant == 0 && deep_enough && 2 * wide_grid > compute_units()))
            return q8.out != nullptr ? launch_roles_mode<true>(x, b, bl, y, p, mode, q8, s, true)
                                     : launch_roles_mode<false>(x, b, bl, y, p, mode, q8, s, true);
    }
    if (streams) {
        // the 64-filter form: lossless mode, or one channel block (see the kernel), unless the padding to 64 filters
        // would add a 32-filter block of nothing
        const bool wide = !narrow_one_round && (mode == WG_LOSSLESS || p.CB == 1) &&
                          (stream_variant == 1 || (stream_variant == 0 && whole64));
        if (mode == WG_LOSSLESS) {
            if (wide) return q8.out ? launch_stream<WG_LOSSLESS, true, true>(x, b, bl, y, p, q8, s) : launch_stream<WG_LOSSLESS, false, true>(x, b, bl, y, p, q8, s);
            return q8.out ? launch_stream<WG_LOSSLESS, true>(x, b, bl, y, p, q8, s) : launch_stream<WG_LOSSLESS, false>(x, b, bl, y, p, q8, s);
        }
        if (wide) return q8.out ? launch_stream<WG_SCALED, true, true>(x, b, bl, y, p, q8, s) : launch_stream<WG_SCALED, false, true>(x, b, bl, y, p, q8, s);
        return q8.out ? launch_stream<WG_SCALED, true>(x, b, bl, y, p, q8, s) : launch_stream<WG_SCALED, false>(x, b, bl, y, p, q8, s);
    }
    // Transform and products on separate waves (channels-last with 4-byte pixel loads): with
    // several channel blocks and no more 32-filter workgroups than compute units (where the
    // 64-filter variant would leave units idle), and in scaled mode from four channel blocks on
    // when the grid is at least three rounds of the compute units (there the product waves do no
    // vector work per block; measured on 256- and 512-channel layers: 10 % faster than the
    // 64-filter variant, while in lossless mode, with two channel blocks, or with a grid of one
    // or two rounds the 64-filter variant stays ahead).
    const long long workgroups = (long long)ceil_div(p.T, kFusedTiles) * (p.Kp / kFusedFilters);
    if (layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0 && p.CB >= 2 &&
        (workgroups <= compute_units() || (mode == WG_SCALED && p.CB >= 4 && workgroups >= 3 * compute_units())))
        return q8.out != nullptr ? launch_roles_mode<true>(x, b, bl, y, p, mode, q8, s)
                                 : launch_roles_mode<false>(x, b, bl, y, p, mode, q8, s);
    return q8.out != nullptr ? launch_layout<true>(x, b, bl, y, p, layout, mode, q8, s)
                             : launch_layout<false>(x, b, bl, y, p, layout, mode, q8, s);
}

}  // namespace wg
