// The whole hot path for layers with at most four input channels (a network's first layer),
// channels-last.  With so few channels the Winograd-domain products (Section 3.4: 16 real and
// 10 complex per tile and channel pair) are a handful of multiply-adds per output, far too few
// to fill the 64-deep reduction of a matrix-core instruction, so this kernel keeps them on the
// vector ALU: the transformed activations and filters stay whole 12-bit numbers in 16-bit
// lanes (no limb split, Section 3.1 is not needed) and one `v_dot2_i32_i16` multiplies two
// channels at a time.
//
// One wave per workgroup and 8 to 32 tiles per wave (chosen on the host so that the waves fill
// the SIMDs evenly, two per SIMD).  Phase 1: lane = tile (the first lanes); the lane loads its 6x6
// patch (all channels packed in one dword per pixel), runs the input transform of Section 3.3
// and leaves the 36 real numbers of the 26 free entries in LDS.  Phase 2: lane = filter; the
// lane holds its filter's 36 Winograd-domain numbers (from the blob's narrow table) in
// registers, the wave walks over its tiles (every lane reads the same tile's numbers from
// LDS), forms the channel sums, applies the reverse scaling of Section 4.2 in scaled mode,
// runs the output transform and stores one output per lane: 64 consecutive filters of a
// pixel, i.e. full lines of the channels-last output.
#include "input_transform_core.h"
#include "output_transform_core.h"
#include "wg_internal.h"

#include <algorithm>

namespace wg {
namespace {

constexpr int kNarrowTiles = 32;                   // most tiles a wave takes
constexpr int kNarrowPieces = kNarrowValues / 2;   // 16-byte pieces per tile or filter: two values x four channels

// Receives the free entries from the input transform: value index = real entry p, or
// 16 + 2j (Re) and 17 + 2j (Im) of complex entry j, the order of the blob's narrow table.
struct ValueKeeper {
    Quad* v;
    __device__ inline void real_entry(int p, Quad q) const { v[p] = q; }
    __device__ inline void complex_entry(int j, Quad re, Quad im) const {
        v[16 + 2 * j] = re;
        v[17 + 2 * j] = im;
    }
};

// sum over the four channel slots of a (16-bit) x b (16-bit)
__device__ inline int dot4(uint32_t a01, uint32_t a23, uint32_t b01, uint32_t b23, int acc = 0) {
    return __builtin_amdgcn_sdot2(as_s16x2(a01), as_s16x2(b01), __builtin_amdgcn_sdot2(as_s16x2(a23), as_s16x2(b23), acc, false),
                                  false);
}

// The int8 epilogue on the output transform's 16 Y (before its rescale by 2^-4): the two nested
// floor divisions ((Y + rnd) >> 4, then (. + round) >> shift) are one, floor((Y + rnd + 16 round) /
// 2^(4 + shift)); then the clamp to [lo, 127].
__device__ inline int requantise_y16(int y16, int add, int shift, int lo) {
    return min(max((y16 + add) >> shift, lo), 127);   // the compiler picks v_med3_i32
}

// grid: (ceil(T/tiles_per_wave), Kp/64), 64 threads.
template <int MODE, bool Q8>
__global__ __launch_bounds__(64) void narrow_conv_kernel(const int8_t* __restrict__ x, const uint8_t* __restrict__ blob,
                                                         size_t table_off, size_t narrow_off, int32_t* __restrict__ y,
                                                         Problem p, Int8Epilogue q8, int tiles_per_wave) {
    __shared__ uint4 values[kNarrowPieces * kNarrowTiles];   // [piece][tile]
    const int lane = threadIdx.x;
    const int tile0 = blockIdx.x * tiles_per_wave;
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;

    // ---- phase 1: lane = tile -----------------------------------------------------------------
    int my_n = 0, my_ty = 0, my_tx = 0;
    if (tile0 + lane < p.T) decode_tile(p, tile0 + lane, my_n, my_ty, my_tx);   // else tile (0,0,0): loaded, never used
    if (lane < tiles_per_wave) {
        uint32_t u[6][6];
        load_patch<WG_NHWC, false>(x, p, my_n, my_ty, my_tx, 0, u);
        bias_patch(p, my_ty, my_tx, 0, u);
        Quad v[kNarrowValues];
        transform_patch(u, ValueKeeper{v});
#pragma unroll
        for (int i = 0; i < kNarrowPieces; ++i)
            values[i * kNarrowTiles + lane] =
                make_uint4(as_u32(v[2 * i].a), as_u32(v[2 * i].b), as_u32(v[2 * i + 1].a), as_u32(v[2 * i + 1].b));
    }

    // ---- phase 2: lane = filter ----------------------------------------------------------------
    const int k = blockIdx.y * 64 + lane;   // < Kp: the blob's tables are padded to Kp
    uint4 w[kNarrowPieces];
    {
        const uint4* mine = reinterpret_cast<const uint4*>(blob + narrow_off) + (size_t)k * kNarrowPieces;
#pragma unroll
        for (int i = 0; i < kNarrowPieces; ++i) w[i] = mine[i];
    }
    // reverse scaling factors r | q << 8 of this filter's 26 entries
    uint32_t rq[MODE == WG_SCALED ? kEntries : 1];
    if constexpr (MODE == WG_SCALED) {
        const ScaleEntry* tk = reinterpret_cast<const ScaleEntry*>(blob + table_off) + (size_t)k * kEntries;
#pragma unroll
        for (int e = 0; e < kEntries; ++e) rq[e] = (uint32_t)tk[e].r | ((uint32_t)tk[e].q << 8);
    }
    auto unscale = [&](int e, int m) {
        if constexpr (MODE == WG_SCALED) {
            // at most four channels: |m| <= 4 * 2047 * 127 < 2^21, so m * r + 2^(q-1) fits 32 bits and
            // the product is a 24-bit multiply
            const int r = (int)(rq[e] & 0xff), q = (int)(rq[e] >> 8);
            static_assert(2LL * kNarrowChannels * 2047 * 127 * 255 + 64 < (1LL << 31), "m * r + rnd fits int32");
            return (__mul24(m, r) + ((1 << q) >> 1)) >> q;
        } else {
            return m;
        }
    };
    __syncthreads();

    // int8 output: 16-byte stores need K % 16 = 0 and an aligned buffer; two staging buffers so
    // that a tile's bytes are not overwritten while the previous tile's are being read
    __shared__ __attribute__((aligned(16))) int8_t staging[Q8 ? 2 : 1][Q8 ? 16 * 64 : 16];
    const bool vector_store = Q8 && ((p.K & 15) | (reinterpret_cast<uintptr_t>(q8.out) & 15)) == 0;

    const int count = min(tiles_per_wave, p.T - tile0);
    const int rnd = MODE == WG_SCALED ? 8 : 0;
    for (int t = 0; t < count; ++t) {
        // all of the tile's numbers are requested before the first one is used, so the wave waits
        // for LDS once per tile
        uint4 v[kNarrowPieces];
#pragma unroll
        for (int i = 0; i < kNarrowPieces; ++i) v[i] = values[i * kNarrowTiles + t];
        __builtin_amdgcn_sched_barrier(0);
        int re[16], cr[10], ci[10];
#pragma unroll
        for (int i = 0; i < 8; ++i) {   // pieces 0..7: real entries 2i, 2i+1
            re[2 * i] = unscale(2 * i, dot4(v[i].x, v[i].y, w[i].x, w[i].y));
            re[2 * i + 1] = unscale(2 * i + 1, dot4(v[i].z, v[i].w, w[i].z, w[i].w));
        }
#pragma unroll
        for (int j = 0; j < 10; ++j) {   // piece 8 + j: (Re, Im) of complex entry j
            const uint4 a = v[8 + j], b = w[8 + j];
            cr[j] = unscale(16 + j, dot4(a.x, a.y, b.x, b.y) - dot4(a.z, a.w, b.z, b.w));
            ci[j] = unscale(16 + j, dot4(a.z, a.w, b.x, b.y, dot4(a.x, a.y, b.z, b.w)));
        }
        int out[4][4];   // out[j][i]: output row i, column j
        output_tile(re, cr, ci, out);

        const int n = __builtin_amdgcn_readlane(my_n, t);
        const int row = 4 * __builtin_amdgcn_readlane(my_ty, t), col = 4 * __builtin_amdgcn_readlane(my_tx, t);
        if constexpr (!Q8) {
            int32_t* dst = y + (((size_t)n * p.H + row) * p.W + col) * p.K + k;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (k < p.K && row + i < p.H && col + j < p.W) dst[(size_t)(i * p.W + j) * p.K] = (out[j][i] + rnd) >> 4;
        } else {
            // side x side output pixels per tile (2 x 2 after pooling), one byte per lane and pixel
            const int side = q8.pool ? 2 : 4, lg = q8.pool ? 1 : 2;
            const int Ho = p.H >> (q8.pool ? 1 : 0), Wo = p.W >> (q8.pool ? 1 : 0);
            const int orow = q8.pool ? row >> 1 : row, ocol = q8.pool ? col >> 1 : col;
            int8_t* tile_out = q8.out + (((size_t)n * Ho + orow) * Wo + ocol) * p.K;
            // With at most four input channels |y| < 2^21, so every shift from 22 on gives 0; capping it
            // at 24 changes no result and keeps 16 * round and 4 + shift within 32 bits for shifts up to 31.
            const int sh = min(q8.shift, 24);
            const int add = rnd + (sh > 0 ? 16 << (sh - 1) : 0), shift = 4 + sh;
            int8_t bytes[16];   // pixel (i, j) of the tile at 4 i + j; pooled: (pi, pj) at 2 pi + pj
            if (q8.pool) {
#pragma unroll
                for (int pi = 0; pi < 2; ++pi)
#pragma unroll
                    for (int pj = 0; pj < 2; ++pj) {
                        int best = -128;
#pragma unroll
                        for (int a = 0; a < 2; ++a)
#pragma unroll
                            for (int b = 0; b < 2; ++b)
                                best = max(best, requantise_y16(out[2 * pj + b][2 * pi + a], add, shift, q8.lo));
                        bytes[2 * pi + pj] = (int8_t)best;
                    }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) bytes[4 * i + j] = (int8_t)requantise_y16(out[j][i], add, shift, q8.lo);
            }
            if (vector_store) {
                // through LDS, so that a lane stores 16 consecutive filters of one pixel: stage[pixel][filter]
                int8_t* stage = staging[t & 1];
#pragma unroll
                for (int px = 0; px < 16; ++px)
                    if (px < side * side) stage[px * 64 + lane] = bytes[px];
                __syncthreads();   // one wave: orders the LDS writes before the reads
                const int px = lane >> 2, f0 = 16 * (lane & 3), i = px >> lg, j = px & (side - 1);
                if (px < side * side && orow + i < Ho && ocol + j < Wo && blockIdx.y * 64 + f0 < p.K)
                    *reinterpret_cast<uint4*>(tile_out + (size_t)(i * Wo + j) * p.K + blockIdx.y * 64 + f0) =
                        *reinterpret_cast<const uint4*>(stage + px * 64 + f0);
            } else {
#pragma unroll
                for (int px = 0; px < 16; ++px) {
                    const int i = px >> lg, j = px & (side - 1);
                    if (px < side * side && k < p.K && orow + i < Ho && ocol + j < Wo)
                        tile_out[(size_t)(i * Wo + j) * p.K + k] = bytes[px];
                }
            }
        }
    }
}

template <int MODE, bool Q8>
hipError_t launch(const int8_t* x, const uint8_t* blob, const BlobLayout& bl, int32_t* y, const Problem& p,
                  const Int8Epilogue& q8, hipStream_t s) {
    // Tiles per wave: the kernel is bound by vector instructions, so the waves should fill every
    // SIMD evenly: two waves on each of the 1,024 SIMDs (two cover each other's LDS and memory
    // waits; a third would only add transform phases with mostly idle lanes).
    const long long work = (long long)p.T * (p.Kp / 64);
    const int tiles = (int)std::min<long long>(kNarrowTiles, std::max<long long>(8, (work + 2047) / 2048));
    dim3 grid(ceil_div(p.T, tiles), p.Kp / 64);
    narrow_conv_kernel<MODE, Q8><<<grid, 64, 0, s>>>(x, blob, bl.table_off, bl.narrow_off, y, p, q8, tiles);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_narrow_conv(const int8_t* x, const void* blob, int32_t* y, const Problem& p, int mode,
                              const Int8Epilogue& q8, hipStream_t s) {
    static_assert(kFilterPad % 64 == 0, "a wave covers 64 filters of the padded filter count");
    const BlobLayout bl = blob_layout(p.Kp, p.C, mode);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (mode == WG_LOSSLESS)
        return q8.out != nullptr ? launch<WG_LOSSLESS, true>(x, b, bl, y, p, q8, s) : launch<WG_LOSSLESS, false>(x, b, bl, y, p, q8, s);
    return q8.out != nullptr ? launch<WG_SCALED, true>(x, b, bl, y, p, q8, s) : launch<WG_SCALED, false>(x, b, bl, y, p, q8, s);
}

}  // namespace wg
