// The whole hot path in one kernel, lossless mode, for channels-last activations whose channel
// count is a multiple of four.
//
// A 12-bit Winograd-domain filter value W = 256 Wh + Wl (byte limbs) enters the matrix cores as TWO
// ROWS of the first operand: a fragment is 8 filters x (Wh, Wl) x 64 channels.  The second operand
// is one limb plane of the transformed activations of 16 tiles (B^T d B, Section 3.3-3.4, D = 256 Dh +
// Dl).  One v_mfma_i32_16x16x64_i8 then leaves, in each lane, the products Wh*Dx and Wl*Dx of two
// filters with one tile: all limbs of a product meet in one lane, so
//   W * D = 2^16 WhDh + 2^8 (WlDh + WhDl) + WlDl
// is three shift-and-add instructions per value and no data crosses lanes for it.
//
// Workgroup: 16 tiles x 32 filters, 512 threads = 8 waves, two per SIMD: a single wave issues a
// vector instruction every five to six clocks, two waves on a SIMD keep their own pace, so eight
// waves nearly double the vector rate of the transform and of the joins.
//   Transform phase: thread = (tile, four channels, half of the rows of B^T d B): waves w and w + 4 share
//   four tiles; one forms rows 0, 1, 2 of the transformed tile, the other row 5 and the complex row 3
//   (the column pass splits the same way, so only the unpacking is done twice).  Every thread writes
//   36 four-byte pieces of operand planes: LDS takes one write instruction per four clocks whatever
//   its width, so narrower writes from more threads would cost more than they save.  Raw patches travel
//   global -> LDS in 16-byte pieces through the buffer descriptor of the activation tensor, so pixels
//   outside the image (pad 1, ragged tiles) and tiles beyond the last one arrive as zeros.
//   Product phase: wave = (filter group of 8) x (half of the 26 free entries of Section 3.4: the 16
//   real ones cost two matrix-core instructions each, the 10 complex ones eight, 56 per half).  Each
//   finished row of M is reduced by the output transform A^T M A at once, so a wave ends with partial
//   outputs of 2 filters x 1 tile per lane.
//   Store: both halves are staged in LDS filter-fastest (in an area of their own, so no wave waits for
//   the others before staging), added, shifted and stored as whole 128-byte lines (16 bytes per lane) -
//   partial-line stores from the lanes' own two filters measured twice as slow.
// Several channel blocks: the output transform is linear, so every block's rows of M are reduced
// into the same 16 outputs.
#include <atomic>

#include "kernel_common.h"

namespace wg {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));

#ifdef WG_TIMESTAMPS
// Development aid (never compiled into the library): per-wave cycle counts at the phase boundaries.
__device__ unsigned long long* g_stamps = nullptr;
#define WG_STAMP(i)                                                                                        \
    do {                                                                                                   \
        if (g_stamps != nullptr && (threadIdx.x & 63) == 0)                                                \
            g_stamps[((blockIdx.y * gridDim.x + blockIdx.x) * 8 + (threadIdx.x >> 6)) * 8 + (i)] = __builtin_amdgcn_s_memtime(); \
    } while (0)
#else
#define WG_STAMP(i)
#endif

constexpr int kWaves = 8;
constexpr int kBlockFilters = 4 * kPairFilters;         // 32 filters per workgroup
constexpr int kActPlanes = 72;                          // byte-limb planes: real p: 2p, 2p+1; complex j: 32+4j + {Re h, Re l, Im h, Im l}
constexpr int kPlanesBytes = kActPlanes * kPlaneBytes;  // 72 KB
constexpr int kRawPixel = 4 * kCBlock;                  // raw patches of four tiles (waves w and w + 4): [pixel 0..35][tile][64 channels]
constexpr int kRawQuad = 36 * kRawPixel;                // 9 KB: nine 1 KB transfers
// output staging (after the products): stage[half][output o][tile][32 filters], tile rows 36 dwords apart and
// outputs 16*36 + 32 dwords apart, so that the 16-byte reads of a 16-lane group (two outputs x eight filter
// quads) fall into different banks
constexpr int kStageRow = 36, kStageOut = 16 * kStageRow + 32, kStageHalf = 16 * kStageOut;   // dwords
// LDS: [operand planes 72 KB][raw patches 36 KB, later the first part of the staged outputs][rest of the staged outputs]:
// the outputs are staged outside the operand planes, so a wave can stage its outputs while others still multiply
constexpr int kStageBytes = 2 * kStageHalf * 4;
static_assert(kStageBytes >= 4 * kRawQuad, "the staged outputs start in the raw patches' area");
constexpr int kLdsBytes = kPlanesBytes + kStageBytes;
static_assert(kLdsBytes <= 160 * 1024, "LDS of one compute unit");
constexpr int kLoadDwords = 1, kLoadDirect = 2;         // 4-byte loads into registers / 16-byte pieces straight into LDS

// ---- which entries a wave multiplies, in order -------------------------------------------------
// Half 0: rows 0, 1, 2 of M (five entries each: four real, then the complex M[row][3]) and M[3][0];
// half 1: M[3][1], M[3][2], M[3][5], M[3][3], M[3][4] and row 5.  56 matrix-core instructions each.
// Entry numbering as in the blob: real entries 0..15 (4 RI + CI over rows/columns 0,1,2,5), complex
// 16..19 = M[RI][3], 20..23 = M[3][CI], 24 = M[3][3], 25 = M[3][4].
struct Slot {
    int entry, row, pos;   // row 0..3: real rows 0,1,2,5; row 4: the complex row 3; pos: place in finish_row's arrays
    bool ends;             // last entry of its row in this half
};
constexpr int half_slots(int half) { return half == 0 ? 16 : 10; }
constexpr Slot half_slot(int half, int s) {
    if (half == 0) {
        if (s < 15) return Slot{s % 5 < 4 ? 4 * (s / 5) + s % 5 : 16 + s / 5, s / 5, s % 5, s % 5 == 4};
        return Slot{20, 4, 0, true};
    }
    // the complex row first: its reduction is the longest, and the last row's reduction has nothing to hide behind
    if (s < 5) return Slot{21 + s, 4, s + 1, s == 4};
    return Slot{s < 9 ? 7 + s : 19, 3, s - 5, s == 9};
}
constexpr bool real_entry(int e) { return e < kRealEntries; }
constexpr int entry_fragments(int e) { return real_entry(e) ? 1 : 2; }
constexpr int entry_value(int e) { return real_entry(e) ? e : 16 + 2 * (e - kRealEntries); }   // blob value index (Re; Im follows)
constexpr int entry_plane(int e) { return real_entry(e) ? 2 * e : 32 + 4 * (e - kRealEntries); }
constexpr int frag_start(int half, int s) {   // index of slot s's first fragment in the wave's fragment stream
    int n = 0;
    for (int i = 0; i < s; ++i) n += entry_fragments(half_slot(half, i).entry);
    return n;
}
constexpr int half_fragments(int half) { return frag_start(half, half_slots(half)); }
static_assert(half_fragments(0) + half_fragments(1) == kPairValues, "one fragment per Winograd-domain value");
constexpr int frag_value(int half, int f) {   // blob value index of fragment f of the stream
    int s = 0;
    while (frag_start(half, s + 1) <= f) ++s;
    return entry_value(half_slot(half, s).entry) + (f - frag_start(half, s));
}

// value = 2^16 hh + 2^8 (lh + hl) + ll for the two filters of a lane: wd = W x Dh, wl = W x Dl,
// registers (Wh0, Wl0, Wh1, Wl1) x D.
__device__ inline v2i join_pair(v4i wd, v4i wl) {
    v2i out;
#pragma unroll
    for (int f = 0; f < 2; ++f) {
        int t = (wd[2 * f] << 8) + (wd[2 * f + 1] + wl[2 * f]);
        asm("" : "+v"(t));   // keeps the two shift-and-add instructions apart
        out[f] = (t << 8) + wl[2 * f + 1];
    }
    return out;
}

struct WaveContext {
    const int8_t* act;   // this lane's 16 bytes of activation plane 0 (LDS)
    const int8_t* flt;   // this lane's 16 bytes of filter fragment 0 of the current channel block
};


constexpr int kRing = 10;   // filter fragments in flight per wave

template <int HALF>
struct Products {
    static constexpr int NS = half_slots(HALF), NF = half_fragments(HALF);
    // A wave gets 16-byte global loads at about 1 KB per 128 clocks, whatever else it does, so its 16 to 20 filter
    // fragments per channel block are requested well ahead: the first kRing before the transform, the others each
    // time a ring slot has been used.
    v4i ring[kRing];

    template <int F>
    __device__ inline static v4i fragment(const WaveContext& cx) {
        constexpr int offset = frag_value(HALF, F) * kFilterFragBytes;   // evaluated by the compiler
        return *reinterpret_cast<const v4i*>(cx.flt + offset);
    }
    template <int PLANE>
    __device__ inline static v4i activation(const WaveContext& cx) {
        return *reinterpret_cast<const v4i*>(cx.act + PLANE * kPlaneBytes);
    }
    // the first kRing fragments, one per call (I = 0 .. kRing - 1), pinned where the caller puts them
    template <int I>
    __device__ inline void prefetch_one(const WaveContext& cx) {
        __builtin_amdgcn_sched_barrier(0);
        ring[I] = fragment<I>(cx);
        __builtin_amdgcn_sched_barrier(0);
    }

    // One 64-channel block: entry s multiplies while entry s+1's activation fragments come from LDS,
    // the ring is refilled, and entry s-1 is joined and (at the end of a row of M) reduced into Y.
    __device__ inline void run(const WaveContext& cx, v2i (&Y)[16]) {
        v4i afr[2][4], acc[2][6];
        v2i er[6], ei[6];
        constexpr int e0 = half_slot(HALF, 0).entry;
        static_for<2 * entry_fragments(e0)>([&](auto I) { afr[0][I] = activation<entry_plane(e0) + I>(cx); });
        static_for<NS + 1>([&](auto S) {
            constexpr int s = S;
            if constexpr (s < NS) {
                constexpr int e = half_slot(HALF, s).entry, f0 = frag_start(HALF, s);
                if constexpr (s + 1 < NS) {
                    constexpr int en = half_slot(HALF, s + 1).entry;
                    static_for<2 * entry_fragments(en)>([&](auto I) { afr[(s + 1) & 1][I] = activation<entry_plane(en) + I>(cx); });
                }
                constexpr v4i zero = {0, 0, 0, 0};
                v4i (&a)[6] = acc[s & 1];
                const v4i (&d)[4] = afr[s & 1];
                const v4i w0 = ring[f0 % kRing];
                if constexpr (real_entry(e)) {
                    a[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[0], zero, 0, 0, 0);   // W x Dh
                    a[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[1], zero, 0, 0, 0);   // W x Dl
                } else {
                    // d = (Dr h, Dr l, Di h, Di l); Im = Wr Di + Wi Dr (a[0], a[1]), Re = Wr Dr (a[2], a[3]) - Wi Di (a[4], a[5]);
                    // instructions into the same accumulator are kept four apart
                    const v4i w1 = ring[(f0 + 1) % kRing];
                    a[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[2], zero, 0, 0, 0);
                    a[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[3], zero, 0, 0, 0);
                    a[2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[0], zero, 0, 0, 0);
                    a[3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0, d[1], zero, 0, 0, 0);
                    a[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, d[0], a[0], 0, 0, 0);
                    a[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, d[1], a[1], 0, 0, 0);
                    a[4] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, d[2], zero, 0, 0, 0);
                    a[5] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1, d[3], zero, 0, 0, 0);
                }
                static_for<entry_fragments(e)>([&](auto I) {
                    if constexpr (f0 + I + kRing < NF) ring[(f0 + I) % kRing] = fragment<f0 + I + kRing>(cx);
                });
            }
            if constexpr (s > 0) {
                constexpr Slot sl = half_slot(HALF, s - 1);
                const v4i (&a)[6] = acc[(s - 1) & 1];
                v2i re, im = {0, 0};
                if constexpr (real_entry(sl.entry)) {
                    re = join_pair(a[0], a[1]);
                } else {
                    re = join_pair(a[2] - a[4], a[3] - a[5]);
                    im = join_pair(a[0], a[1]);
                }
                if constexpr (HALF == 0 && sl.row == 4) {
                    // M[3][0] alone: in the row rule of A^T it only enters z0 = e0 + ..., which the column rule
                    // spreads as y0 += 2 Re z0, y1 -= 2 Im z0, y2 -= 2 Re z0, y3 += 2 Im z0 (first output column)
                    Y[0] += 2 * re;
                    Y[4] -= 2 * im;
                    Y[8] -= 2 * re;
                    Y[12] += 2 * im;
                } else {
                    er[sl.pos] = re;
                    ei[sl.pos] = im;
                    if constexpr (HALF == 1 && sl.row == 4 && sl.pos == 1) {   // M[3][0] belongs to the other half
                        er[0] = (v2i){0, 0};
                        ei[0] = (v2i){0, 0};
                    }
                    if constexpr (sl.ends) finish_row<sl.row>(er, ei, Y);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
};

// ---- the input transform, four channels per thread, half of the rows per thread ---------------------
// Activations are handled in the biased form u = x + 128 (one XOR on the raw bytes, so that unpacking
// is a zero extension); a constant patch maps to zero at every entry of B^T d B except (1,1), where
// the bias leaves 16 * 128 = 2048.  What lies outside the image arrived as zero bytes, i.e. x = 0
// after the XOR as well.
// The 1-D rule of B^T on a 6-vector (Section 3.4, the expansion of d' = B^T d):
//   t0 = v0 - v4, t1 = v1+v2+v3+v4, t2 = -v1+v2-v3+v4, t3 = (v4-v2) + i (v3-v1), t5 = v5 - v1.
// GROUP 0 forms rows 0, 1, 2 of the transformed tile (entries (r, 0..5) for r = 0, 1, 2: four real and one
// complex each), GROUP 1 row 5 and the complex row 3; of the column pass each group needs only its own rows.
// `tick` is called at ten places spread over the work (with std::integral_constant<int, 0..9>): the caller issues one
// global load at each, so that its requests enter the memory pipeline at the pace the pipeline takes them.
template <int GROUP, class Out, class Tick>
__device__ inline void transform_rows(const uint32_t (&u)[6][6], const Out& out, Tick&& tick) {
    Quad v[6][6];
    static_for<6>([&](auto A) {
#pragma unroll
        for (int b = 0; b < 6; ++b) v[A][b] = unpack_u8x4(u[A][b] ^ kBiasBytes);
        tick(A);
    });
    const s16x2 bias11 = {2048, 2048};
    auto row_rule = [](const Quad (&c)[6]) { return bt_rule(c[0], c[1], c[2], c[3], c[4], c[5]); };
    auto emit_real_row = [&](int ri, const Line& l) {
        out.real_entry(4 * ri + 0, l.t0);
        out.real_entry(4 * ri + 1, l.t1);
        out.real_entry(4 * ri + 2, l.t2);
        out.real_entry(4 * ri + 3, l.t5);
        out.complex_entry(ri, l.t3r, l.t3i);
    };
    if constexpr (GROUP == 0) {
        Quad r0[6], r1[6], r2[6];   // rows 0, 1, 2 of d' = B^T d, by column
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            const Quad s13 = v[1][b] + v[3][b], s24 = v[2][b] + v[4][b];
            r0[b] = v[0][b] - v[4][b];
            r1[b] = s24 + s13;
            r2[b] = s24 - s13;
        }
        tick(std::integral_constant<int, 6>{});
        emit_real_row(0, row_rule(r0));
        tick(std::integral_constant<int, 7>{});
        Line l1 = row_rule(r1);
        l1.t1 = Quad{l1.t1.a - bias11, l1.t1.b - bias11};
        emit_real_row(1, l1);
        tick(std::integral_constant<int, 8>{});
        emit_real_row(2, row_rule(r2));
        tick(std::integral_constant<int, 9>{});
    } else {
        Quad r5[6], ra_[6], rb_[6];   // row 5, and row 3 = ra + i rb
#pragma unroll
        for (int b = 0; b < 6; ++b) {
            r5[b] = v[5][b] - v[1][b];
            ra_[b] = v[4][b] - v[2][b];
            rb_[b] = v[3][b] - v[1][b];
        }
        tick(std::integral_constant<int, 6>{});
        emit_real_row(3, row_rule(r5));
        tick(std::integral_constant<int, 7>{});
        // the rule acts on the real and the imaginary part of row 3 separately; entries (3,3) and (3,4) mix them
        const Line ra = row_rule(ra_), rb = row_rule(rb_);
        out.complex_entry(4, ra.t0, rb.t0);
        out.complex_entry(5, ra.t1, rb.t1);
        out.complex_entry(6, ra.t2, rb.t2);
        tick(std::integral_constant<int, 8>{});
        out.complex_entry(7, ra.t5, rb.t5);
        out.complex_entry(8, ra.t3r - rb.t3i, rb.t3r + ra.t3i);
        out.complex_entry(9, ra.t3r + rb.t3i, rb.t3r - ra.t3i);
        tick(std::integral_constant<int, 9>{});
    }
}

// Offset (relative to x) of patch pixel `pixel` = 6a + b of tile (n, ty, tx), channel c; what does not
// exist (pixel >= 36, rows and columns outside the image, no tile) gets an offset no buffer can hold.
__device__ inline uint32_t pixel_offset(const Problem& p, bool tile_exists, int n, int ty, int tx, int pixel, int c) {
    const int a = (pixel * 43) >> 8, b = pixel - 6 * a;   // pixel / 6 for pixel < 48
    const int h = 4 * ty - 1 + a, w = 4 * tx - 1 + b;
    const bool inside = tile_exists && pixel < 36 && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W;
    return inside ? (uint32_t)(((n * p.H + h) * p.W + w) * p.C + c) : kOutsideOffset;
}

// 16 bytes per lane from the buffer straight into LDS: lane l's piece lands at lds_dst + 16 l (lds_dst uniform).
__device__ inline void buffer_to_lds_16(__amdgpu_buffer_rsrc_t buffer, int8_t* lds_dst, uint32_t voffset, int soffset) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(buffer, (__attribute__((address_space(3))) int8_t*)lds_dst, 16, voffset, soffset, 0, 0);
}

// grid (ceil(T/16), Kp/32), 512 threads.
template <int LOAD, bool Q8>
__global__ __launch_bounds__(512) void lossless_pair_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                            size_t pairs_off, int32_t* __restrict__ y, Problem p,
                                                            Int8Epilogue q8) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile0 = blockIdx.x * kTileBlock;
    const int k0 = blockIdx.y * kBlockFilters;
    const __amdgpu_buffer_rsrc_t xbuf = activation_buffer(x, p);
    WG_STAMP(0);

    // ---- the raw patch of the first channel block: the longest wait of the kernel, requested first ----
    // Transform thread: tile 4 (wave % 4) + lane / 16, channels 4 (lane % 16) .. + 3, rows by wave / 4.
    const int quad = wave & 3, half = wave >> 2;   // the same split serves the product phase: filters 8 quad .. + 7, half of the entries
    const int a_tile = 4 * quad + (lane >> 4), a_cq = lane & 15;
    int8_t* const raw_quad = lds + kPlanesBytes + quad * kRawQuad;
    uint32_t raw_off[LOAD == kLoadDirect ? 5 : 1];   // this lane's piece in each of the wave's transfers
    uint32_t pixel[LOAD == kLoadDwords ? 36 : 1];    // or this thread's 36 pixels
    uint32_t u[6][6];
    // Direct transfers: transfer i (0..8) moves pixels 4i .. 4i+3 of the four tiles: lane = 16 (pixel % 4) + 4 (tile % 4)
    // + piece of 16 channels, and the hardware puts lane l's 16 bytes at (uniform destination) + 16 l, so the raw area
    // is [pixel][tile % 4][64 channels].  Waves 0-3 issue transfers 0..4, waves 4-7 transfers 5..8.
    const int first_transfer = half == 0 ? 0 : 5, transfers = half == 0 ? 5 : 4;
    if constexpr (LOAD == kLoadDirect) {
        const int dt = tile0 + 4 * quad + ((lane >> 2) & 3);
        int dn = 0, dty = 0, dtx = 0;
        if (dt < p.T) decode_tile(p, dt, dn, dty, dtx);
#pragma unroll
        for (int j = 0; j < 5; ++j)
            raw_off[j] = pixel_offset(p, dt < p.T, dn, dty, dtx, 4 * (first_transfer + j) + (lane >> 4), 16 * (lane & 3));
    } else {
        const int at = tile0 + a_tile;
        int an = 0, aty = 0, atx = 0;
        if (at < p.T) decode_tile(p, at, an, aty, atx);
        patch_offsets(p, an, aty, atx, 4 * a_cq, pixel);
        if (at >= p.T) {
#pragma unroll
            for (int i = 0; i < 36; ++i) pixel[i] = kOutsideOffset;
        }
    }
    // Channel block cb.  In the last block of a C that is not a multiple of 64 (a uniform branch) lanes whose
    // channels lie beyond C ask for the outside offset and get zeros.
    auto request = [&](int cb) {
        const bool tail = (cb + 1) * kCBlock > p.C;
        if constexpr (LOAD == kLoadDirect) {
            const bool have = !tail || cb * kCBlock + 16 * (lane & 3) < p.C;
#pragma unroll
            for (int j = 0; j < 5; ++j)
                if (j < transfers)
                    buffer_to_lds_16(xbuf, raw_quad + (first_transfer + j) * 1024, have ? raw_off[j] : kOutsideOffset, cb * kCBlock);
        } else {
            const bool have = !tail || cb * kCBlock + 4 * a_cq < p.C;
#pragma unroll
            for (int i = 0; i < 36; ++i)
                u[i / 6][i % 6] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(xbuf, have ? pixel[i] : kOutsideOffset, cb * kCBlock, 0);
        }
    };
    request(0);
    // the blob header: requested now, looked at after the transform, so its latency hides behind the patch's
    __builtin_amdgcn_sched_barrier(0);
    const BlobHeaderWords header = read_blob_header(blob);
    __builtin_amdgcn_sched_barrier(0);

    // ---- identities of the two phases ------------------------------------------------------------------
    OperandSplitter<kSplitByteLimbs, LdsPlaneSink> out;
    out.sink.base = lds + lds_slot(a_cq >> 2, a_tile) * 16 + (a_cq & 3) * 4;
    WaveContext cx;
    cx.act = lds + lds_slot(lane >> 4, lane & 15) * 16;
    const int8_t* const flt0 = reinterpret_cast<const int8_t*>(blob + pairs_off) +
                               filter_pair_offset(0, 0, k0 + kPairFilters * quad, 0, 0, p.Kp) + (lane & 15) * kCBlock + (lane >> 4) * 16;
    const size_t flt_block = (size_t)(p.Kp >> 3) * kPairValues * kFilterFragBytes;
    cx.flt = flt0;

    v2i Y[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) Y[i] = (v2i){0, 0};

    Products<0> products0;
    Products<1> products1;
    WG_STAMP(1);
    for (int cb = 0; cb < p.CB; ++cb) {
        // This wave's share of the raw patch (or its 36 pixels) has arrived.  The filter fragments are only requested
        // now, so that at the start of the kernel, when every workgroup of the grid asks at once, the patches do not
        // share the memory system with them; the transform gives the fragments time enough to arrive.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if constexpr (LOAD == kLoadDirect) {
            // the raw pieces of a wave's tiles were moved by two waves; from the second block on the barrier also
            // says that everyone is done reading the previous block's planes
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            WG_STAMP(2);
#pragma unroll
            for (int i = 0; i < 36; ++i)
                u[i / 6][i % 6] = *reinterpret_cast<const uint32_t*>(raw_quad + i * kRawPixel + 4 * lane);
        } else if (cb > 0) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
        }
        // the first kRing filter fragments are requested at ten places spread over the transform
        static_assert(kRing == 10, "transform_rows calls its tick ten times");
        if (half == 0) transform_rows<0>(u, out, [&](auto I) { products0.template prefetch_one<I>(cx); });
        else           transform_rows<1>(u, out, [&](auto I) { products1.template prefetch_one<I>(cx); });
        if (cb == 0 && !blob_matches(header, p.K, p.C, WG_LOSSLESS)) return;   // uniform: nobody reaches the next barrier
        // the operand planes are complete once every wave's LDS writes have landed (and every wave has read its
        // raw patch); global requests stay in flight across the barrier
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        WG_STAMP(3);
        __builtin_amdgcn_s_barrier();
        WG_STAMP(4);
        if (cb + 1 < p.CB) request(cb + 1);   // travels while this block's products run
        if (half == 0) products0.run(cx, Y); else products1.run(cx, Y);
        cx.flt += flt_block;
        WG_STAMP(5);
    }

    // ---- stage both halves' partial outputs, add them, store whole lines ------------------------------
    // the staging area lies behind the operand planes (it begins where the raw patches were, which nobody reads
    // after the last transform), so a wave stages its outputs as soon as it has them
    int* const stage = reinterpret_cast<int*>(lds + kPlanesBytes);
    {
        // lane = tile (lane & 15) x filters 8 quad + 2 (lane / 16), + 1
        int* dst = stage + half * kStageHalf + (lane & 15) * kStageRow + 8 * quad + 2 * (lane >> 4);
#pragma unroll
        for (int o = 0; o < 16; ++o) *reinterpret_cast<v2i*>(dst + o * kStageOut) = Y[o];
    }
    __syncthreads();
    WG_STAMP(6);
    // thread: filters k0 + 4 k4 .. + 3 of output column j of tile `tile`; round r: output row r
    const int k4 = tid & 7, j = (tid >> 3) & 3, tile = tid >> 5;
    const int t = tile0 + tile, kk = k0 + 4 * k4;
    int n = 0, ty = 0, tx = 0;
    if (t < p.T) decode_tile(p, t, n, ty, tx);
    const int row = 4 * ty, col = 4 * tx + j;
    const bool live = t < p.T && col < p.W && kk < p.K;
    auto staged = [&](int o) {   // finished outputs of the thread's four filters at output o of its tile
        const int at = o * kStageOut + tile * kStageRow + 4 * k4;
        return (*reinterpret_cast<const v4i*>(stage + at) + *reinterpret_cast<const v4i*>(stage + kStageHalf + at)) >> 4;
    };
    if constexpr (!Q8) {
        int32_t* const first = y + ((size_t)(n * p.H + row) * p.W + col) * p.K + kk;
        const bool vector_store = (p.K & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        v4i v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = staged(4 * r + j);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (!live || row + r >= p.H) continue;
            int32_t* at = first + (size_t)r * p.W * p.K;
            if (vector_store) {
                *reinterpret_cast<v4i*>(at) = v[r];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (kk + q < p.K) at[q] = v[r][q];
            }
        }
    } else {
        // requantisation and clamp, then (a 4x4 tile holds whole 2x2 windows) the pooling maximum
        const bool word_store = (p.K & 3) == 0 && (reinterpret_cast<uintptr_t>(q8.out) & 3) == 0;
        auto put = [&](int8_t* at, v4i q) {
            if (word_store) {
                *reinterpret_cast<uint32_t*>(at) = pack_bytes(q);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (kk + e < p.K) at[e] = (int8_t)q[e];
            }
        };
        if (!q8.pool) {
            v4i v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = requantise(staged(4 * r + j), q8);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (live && row + r < p.H) put(q8.out + ((size_t)(n * p.H + row + r) * p.W + col) * p.K + kk, v[r]);
        } else if (j < 2) {
            // thread: pooled column j (0, 1) of its tile, both pooled rows
            const int Ho = p.H >> 1, Wo = p.W >> 1, ocol = 2 * tx + j;
#pragma unroll
            for (int pi = 0; pi < 2; ++pi) {
                v4i best = requantise(staged(4 * (2 * pi) + 2 * j), q8);
                best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi) + 2 * j + 1), q8));
                best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi + 1) + 2 * j), q8));
                best = __builtin_elementwise_max(best, requantise(staged(4 * (2 * pi + 1) + 2 * j + 1), q8));
                if (t < p.T && kk < p.K && ocol < Wo && 2 * ty + pi < Ho)
                    put(q8.out + ((size_t)(n * Ho + 2 * ty + pi) * Wo + ocol) * p.K + kk, best);
            }
        }
    }
    WG_STAMP(7);
}

template <int LOAD, bool Q8>
hipError_t launch(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                  const Int8Epilogue& q8, hipStream_t s) {
    static LdsLimitOnce lds_limit;   // per template instance
    if (hipError_t e = lds_limit.set(reinterpret_cast<const void*>(&lossless_pair_kernel<LOAD, Q8>), kLdsBytes)) return e;
    dim3 grid(ceil_div(p.T, kTileBlock), p.Kp / kBlockFilters);
    lossless_pair_kernel<LOAD, Q8><<<grid, 64 * kWaves, kLdsBytes, s>>>(x, blob, bl.pairs_off, y, p, q8);
    return hipGetLastError();
}

std::atomic<int> g_lossless_variant{0};

}  // namespace

#ifdef WG_TIMESTAMPS
extern "C" int winograd_debug_set_stamps(void* dev_ptr) {
    return hipMemcpyToSymbol(HIP_SYMBOL(g_stamps), &dev_ptr, sizeof dev_ptr) == hipSuccess ? 0 : -5;
}
#endif

void set_lossless_variant(int v) { g_lossless_variant.store(v, std::memory_order_relaxed); }

int lossless_pair_conv_choice(const int8_t* x, const Problem& p, int layout) {
    const int v = g_lossless_variant.load(std::memory_order_relaxed);
    const bool applies = layout == WG_NHWC && p.C % 4 == 0 && reinterpret_cast<uintptr_t>(x) % 4 == 0;
    if (v == 2 || !applies) return 0;
    return v == 1 ? 2 : 1;
}

hipError_t launch_lossless_pair_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p,
                                     const Int8Epilogue& q8, hipStream_t s) {
    const BlobLayout bl = blob_layout(p.Kp, p.C, WG_LOSSLESS);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    const bool direct = p.C % 16 == 0 && reinterpret_cast<uintptr_t>(x) % 16 == 0;
    if (q8.out != nullptr)
        return direct ? launch<kLoadDirect, true>(x, b, bl, y, p, q8, s) : launch<kLoadDwords, true>(x, b, bl, y, p, q8, s);
    return direct ? launch<kLoadDirect, false>(x, b, bl, y, p, q8, s) : launch<kLoadDwords, false>(x, b, bl, y, p, q8, s);
}

}  // namespace wg
