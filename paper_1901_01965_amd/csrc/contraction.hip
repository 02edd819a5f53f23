// Winograd-domain contraction (Section 3.4): for every free entry of the transformed
// tile, the product of the transformed filter and activation summed over input
// channels, on the int8 matrix cores.  The work is cut into uniform units (see
// subproducts.h): lossless mode keeps the paper's three-multiplication forms
// (46 real 12-bit products, each as three int8 limb products); scaled mode
// (Section 4.2) uses single-limb filters and applies the reciprocal r/2^q to the
// finished sums.
//
// One workgroup owns one unit and a 128-tile x 128-filter block of it.  Each of
// the unit's sub-products is a [128 x C] x [C x 128] int8 GEMM.  Operand blocks
// of 64 channels travel from L2 straight into a six-stage LDS ring
// (global_load_lds_dwordx4, no register staging), several stages ahead of the
// matrix cores; every wave keeps a 64x64 block of v_mfma_i32_32x32x32_i8
// accumulators; the finished channel sum is folded into the unit's output with
// the sub-product's integer weight.
#include "subproducts.h"

namespace wg {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBlockTiles = 128, kBlockFilters = 128;
constexpr int kOperandBytes = 128 * kCBlock;        // one staged operand block: 128 rows x 64 bytes
constexpr int kStageBytes = 2 * kOperandBytes;      // activations + filters
constexpr int kStages = 6;
constexpr int kContractionLds = kStages * kStageBytes;   // 96 KB

// A staged row keeps its 64 bytes but stores 16-byte chunk c at position c ^ swizzle(row), which
// spreads the fragment reads of 16 consecutive rows over all banks.  The permutation is applied
// on the global side: the LDS side of a direct load is fixed (lane l lands at base + 16 l).
__device__ inline int swizzle(int row) { return (row ^ (row >> 2)) & 3; }

template <int MODE>
struct BlockLoader {
    const int8_t* V;
    const int8_t* U;
    size_t a_plane_stride, a_cb_stride, b_cb_stride;
    int a_off[2], b_off[2];   // this lane's source offsets inside plane 0, channel block 0
    int lds_off[2];           // wave-uniform destination of each instruction inside an operand block

    // wave w fills rows 32w..32w+31 of both operand blocks: two instructions of 16 rows each
    __device__ inline void init(const int8_t* V_, const int8_t* U_, const Problem& p, int t0, int k0, int wave,
                                int lane) {
        constexpr int NP = MODE == WG_LOSSLESS ? 138 : 46;
        V = V_; U = U_;
        a_plane_stride = (size_t)p.CB * p.Tp * kCBlock;
        a_cb_stride = (size_t)p.Tp * kCBlock;
        b_cb_stride = (size_t)(p.Kp >> 4) * NP * kFilterFragBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = wave * 32 + i * 16 + (lane >> 2);
            const int chunk = (lane & 3) ^ swizzle(row);
            // rows beyond the padded extent are clamped: their products are never stored
            const int t = min(t0 + row, p.Tp - 1), k = min(k0 + row, p.Kp - 1);
            a_off[i] = t * kCBlock + chunk * 16;
            b_off[i] = (int)filter_plane_offset(0, 0, k, chunk * 16, p.Kp, NP);
            lds_off[i] = (wave * 32 + i * 16) * kCBlock;
        }
    }
    __device__ inline void issue(int8_t* stage, int a_plane, int b_plane, int cb) const {
        const int8_t* A = V + a_plane * a_plane_stride + cb * a_cb_stride;
        const int8_t* B = U + cb * b_cb_stride + (size_t)b_plane * kFilterFragBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            __builtin_amdgcn_global_load_lds(A + a_off[i], stage + lds_off[i], 16, 0, 0);
            __builtin_amdgcn_global_load_lds(B + b_off[i], stage + kOperandBytes + lds_off[i], 16, 0, 0);
        }
    }
};

// Fragments of one staged block for one multiplying wave: for each of the two 32-channel steps,
// two activation and two filter fragments.  a_row/b_row: byte offset of this lane's row
// (lane % 32) in each operand block; sw = swizzle of that row (the same for the row 32 further
// on); half = lane / 32 selects the 16-byte half of a step.
struct Frags {
    v4i a[2][2], b[2][2];   // [step][fragment]
};
__device__ inline void read_frags(Frags& f, const int8_t* stage, int a_row, int b_row, int sw_a, int sw_b, int half) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int ca = ((2 * ks + half) ^ sw_a) * 16, cb = ((2 * ks + half) ^ sw_b) * 16;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            f.a[ks][i] = *reinterpret_cast<const v4i*>(stage + a_row + i * 32 * kCBlock + ca);
            f.b[ks][i] = *reinterpret_cast<const v4i*>(stage + kOperandBytes + b_row + i * 32 * kCBlock + cb);
        }
    }
}
__device__ inline void multiply(const Frags& f, v16i (&acc)[2][2], bool zero) {
    if (zero) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                constexpr v16i z = {0};
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.a[0][i], f.b[0][j], z, 0, 0, 0);
            }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.a[0][i], f.b[0][j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f.a[1][i], f.b[1][j], acc[i][j], 0, 0, 0);
}

// Which units each of the eight XCDs works on.  Workgroups are handed to the XCDs round-robin
// by linear index, and every XCD has its own L2: all blocks of one unit are therefore given to
// one XCD, back to back, so that an activation block (shared by the filter blocks of its row)
// and a filter block (shared by the tile blocks of its column) can hit in that L2.  Lossless
// units all cost the same (unit = xcd + 8 i).  Scaled units cost 2 (real) or 4 (complex part)
// sub-products: XCDs 0-3 take three complex parts and one real, XCDs 4-7 two and three.
constexpr int kXcds = 8;
template <int MODE> constexpr int units_per_xcd() { return MODE == WG_LOSSLESS ? 6 : 5; }
template <int MODE>
__device__ inline int unit_of(int xcd, int i) {
    if (MODE == WG_LOSSLESS) {
        const int u = xcd + kXcds * i;
        return u < num_units<MODE>() ? u : -1;
    }
    if (xcd < 4) return i < 3 ? kRealEntries + 4 * i + xcd : (i == 3 ? xcd : -1);
    const int x = xcd - 4;
    return i < 2 ? kRealEntries + 12 + 2 * x + i : 4 + 3 * x + (i - 2);
}

// grid: 8 XCDs x units per XCD x (tile blocks x filter blocks), one dimension.  512 threads:
// waves 0-3 multiply (one per SIMD, each a 64x64 quadrant of the block), waves 4-7 only move
// operands.  A wave issues in order, and a vector-memory instruction stalls at issue while the
// memory pipeline is full; keeping the loads in waves of their own lets the matrix-core
// instructions of the other wave on the same SIMD issue meanwhile.
//
// Stage f of a unit's stream = (sub-product f / CB, channel block f % CB); it lives in ring slot
// f % kStages.  Both roles pass one barrier per stage: barrier f tells the multiplying waves
// that stage f has landed, and the loading waves that the reads of stage f-1 are complete, so
// that its slot can take stage f + kStages - 1.
template <int MODE>
__global__ __launch_bounds__(512) void contraction_kernel(const int8_t* __restrict__ V,
                                                          const uint8_t* __restrict__ blob,
                                                          size_t table_off, size_t planes_off,
                                                          int32_t* __restrict__ M, Problem p) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    if (!blob_matches(reinterpret_cast<const BlobHeader*>(blob), p.K, p.C, MODE)) return;
    const int tile_blocks = (p.T + kBlockTiles - 1) / kBlockTiles;
    const int blocks_per_unit = tile_blocks * ((p.K + kBlockFilters - 1) / kBlockFilters);
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int unit = unit_of<MODE>(xcd, slot / blocks_per_unit);
    if (unit < 0) return;
    const int within = slot % blocks_per_unit;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int t0 = (within % tile_blocks) * kBlockTiles, k0 = (within / tile_blocks) * kBlockFilters;
    const int nsub = num_subproducts<MODE>(unit);
    const int total = nsub * p.CB;

    if (wave >= 4) {
        BlockLoader<MODE> loader;
        loader.init(V, reinterpret_cast<const int8_t*>(blob + planes_off), p, t0, k0, wave - 4, lane);
        int fs = 0, fcb = 0;   // sub-product and channel block of the next stage to request
        auto request = [&](int f) {
            const SubProduct sp = subproduct<MODE>(unit, fs);
            loader.issue(lds + (f % kStages) * kStageBytes, sp.a_plane, sp.b_plane, fcb);
            if (++fcb == p.CB) { fcb = 0; ++fs; }
        };
        for (int f = 0; f < kStages - 1; ++f) {
            if (f < total) request(f);
        }
        static_assert(kStages == 6, "the wait below covers up to four later stages");
        for (int f = 0; f < total; ++f) {
            // stage f has landed once only the requests of the (up to four) stages after it are
            // pending; every request is four load instructions per wave
            switch (min(total - 1 - f, kStages - 2)) {
                case 4:  asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
                case 3:  asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
                case 2:  asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
                case 1:  asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
                default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
            }
            __builtin_amdgcn_s_barrier();
            if (f + kStages - 1 < total) request(f + kStages - 1);
        }
        return;
    }

    const int wm = wave & 1, wn = wave >> 1;
    const int a_row = (wm * 64 + (lane & 31)) * kCBlock, b_row = (wn * 64 + (lane & 31)) * kCBlock;
    const int sw_a = swizzle(wm * 64 + (lane & 31)), sw_b = swizzle(wn * 64 + (lane & 31)), half = lane >> 5;

    v16i out[2][2], acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) out[i][j] = (v16i){0};

    // Consecutive sub-products of equal weight share one channel sum; it is folded into the
    // unit's output when the weight changes.  Lossless: every sub-product has its own weight and
    // |acc| <= 94 * 94 * 896 < 2^23, so a 24-bit multiply-add is exact modulo 2^32.  Scaled: the
    // weights are 64 and 1, a shift.
    int fs = 0, fcb = 0;       // sub-product and channel block of the stage being multiplied
    bool zero = true;
    auto multiply_stage = [&](const Frags& f) {
        multiply(f, acc, zero);
        zero = false;
        if (++fcb == p.CB) {
            fcb = 0;
            const int w = subproduct<MODE>(unit, fs).weight;
            ++fs;
            if (fs == nsub || subproduct<MODE>(unit, fs).weight != w) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            out[i][j][r] += MODE == WG_LOSSLESS ? __mul24(acc[i][j][r], w) : acc[i][j][r] << (w == 64 ? 6 : 0);
                zero = true;
            }
        }
    };
    // The fragments of stage f+1 are requested from LDS right after barrier f+1 and before the
    // matrix-core instructions of stage f are issued, so LDS latency hides behind them.
    Frags fa, fb;
    __builtin_amdgcn_s_barrier();   // barrier 0
    read_frags(fa, lds, a_row, b_row, sw_a, sw_b, half);
    for (int f = 0; f < total; f += 2) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // fa (stage f) is in registers
        if (f + 1 < total) {
            __builtin_amdgcn_s_barrier();
            read_frags(fb, lds + ((f + 1) % kStages) * kStageBytes, a_row, b_row, sw_a, sw_b, half);
        }
        multiply_stage(fa);
        if (f + 1 >= total) break;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // fb (stage f+1) is in registers
        if (f + 2 < total) {
            __builtin_amdgcn_s_barrier();
            read_frags(fa, lds + ((f + 2) % kStages) * kStageBytes, a_row, b_row, sw_a, sw_b, half);
        }
        multiply_stage(fb);
    }

    int32_t* Mu = M + (size_t)unit * p.Tp * p.Kp;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int k = k0 + wn * 64 + j * 32 + (lane & 31);
        if (k >= p.K) continue;
        ScaleEntry se = {0, 0, 1, 0};
        if (MODE == WG_SCALED)
            se = reinterpret_cast<const ScaleEntry*>(blob + table_off)[(size_t)k * kEntries + unit_entry<MODE>(unit)];
        const ReverseScale unscale(se);   // Section 4.2
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tb = t0 + wm * 64 + i * 32 + 4 * (lane >> 5);
            int32_t* m = Mu + (size_t)tb * p.Kp + k;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int v = out[i][j][r];
                if (MODE == WG_SCALED) v = unscale(v);
                const int dt = 8 * (r / 4) + (r % 4);
                if (tb + dt < p.T) m[dt * p.Kp] = v;
            }
        }
    }
}

// The 36 planes the output transform is defined on (real entry p: p; complex entry j:
// 16 + 2j + {Re, Im}) from the workspace planes: lossless Re = P1 - P2, Im = P3 - P1 - P2.
__device__ inline int accumulator_plane(const int32_t* M, size_t plane_stride, size_t at, int mode, int pl) {
    if (mode != WG_LOSSLESS || pl < kRealEntries) return M[pl * plane_stride + at];
    const int j = (pl - kRealEntries) >> 1;
    const int32_t* P = M + (size_t)(kRealEntries + 3 * j) * plane_stride + at;
    const int p1 = P[0], p2 = P[plane_stride], p3 = P[2 * plane_stride];
    return ((pl - kRealEntries) & 1) ? p3 - p1 - p2 : p1 - p2;
}

__global__ void unpack_accumulators_kernel(const int32_t* M, int32_t* dense, Problem p, int mode) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)kAccPlanes * p.T * p.K;
    if (i >= total) return;
    int k = (int)(i % p.K);
    int t = (int)((i / p.K) % p.T);
    int pl = (int)(i / ((size_t)p.K * p.T));
    dense[i] = accumulator_plane(M, (size_t)p.Tp * p.Kp, (size_t)t * p.Kp + k, mode, pl);
}

template <int MODE>
hipError_t configure_contraction() {
    static LdsLimitOnce lds_limit;
    return lds_limit.set(reinterpret_cast<const void*>(&contraction_kernel<MODE>), kContractionLds);
}

}  // namespace

hipError_t launch_contraction(const int8_t* V, const void* blob, int32_t* M, const Problem& p, int mode,
                              hipStream_t s) {
    if (hipError_t e = mode == WG_LOSSLESS ? configure_contraction<WG_LOSSLESS>() : configure_contraction<WG_SCALED>())
        return e;
    const BlobLayout bl = blob_layout(p.Kp, p.C, mode);
    const unsigned blocks = ceil_div(p.T, kBlockTiles) * ceil_div(p.K, kBlockFilters);
    const unsigned grid = kXcds * (mode == WG_LOSSLESS ? units_per_xcd<WG_LOSSLESS>() : units_per_xcd<WG_SCALED>()) * blocks;
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    if (mode == WG_LOSSLESS)
        contraction_kernel<WG_LOSSLESS><<<grid, 512, kContractionLds, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    else
        contraction_kernel<WG_SCALED><<<grid, 512, kContractionLds, s>>>(V, b, bl.table_off, bl.planes_off, M, p);
    return hipGetLastError();
}

hipError_t launch_unpack_accumulators(const int32_t* M, int32_t* dense, const Problem& p, int mode, hipStream_t s) {
    size_t total = (size_t)kAccPlanes * p.T * p.K;
    unpack_accumulators_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(M, dense, p, mode);
    return hipGetLastError();
}

}  // namespace wg
