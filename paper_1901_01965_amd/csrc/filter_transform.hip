// Filter transform W = G' g G'^T (G' = 4G, Section 3.3), the conjugate-aware
// selection of its 26 free entries (Section 3.4), the filter precision scaling
// of Section 4.2, and the split into int8 operand planes for the matrix cores.
// Runs once per layer; nothing here is on the per-inference path.
#include "wg_internal.h"

namespace wg {
namespace {

// The 1-D rule of G' on a real triple (x0,x1,x2):
//   0: 4 x0   1: x0+x1+x2   2: x0-x1+x2   3: (x0-x2) + i x1   [4: conj of 3]   5: 4 x2
// Free entries of W, in the library's order: re[0..15] = W[r][c], r,c in {0,1,2,5};
// complex cr/ci[0..3] = W[{0,1,2,5}][3], [4..7] = W[3][{0,1,2,5}], [8] = W[3][3], [9] = W[3][4].
__device__ inline void filter_entries(const int g[9], int re[16], int cr[10], int ci[10]) {
    int u[4][3];           // real rows 0,1,2,5 of G' g
    int a[3], b[3];        // row 3 of G' g = a + i b
    for (int col = 0; col < 3; ++col) {
        int g0 = g[col], g1 = g[3 + col], g2 = g[6 + col];
        u[0][col] = 4 * g0;
        u[1][col] = g0 + g1 + g2;
        u[2][col] = g0 - g1 + g2;
        u[3][col] = 4 * g2;
        a[col] = g0 - g2;
        b[col] = g1;
    }
    for (int ri = 0; ri < 4; ++ri) {
        int x0 = u[ri][0], x1 = u[ri][1], x2 = u[ri][2];
        re[4 * ri + 0] = 4 * x0;
        re[4 * ri + 1] = x0 + x1 + x2;
        re[4 * ri + 2] = x0 - x1 + x2;
        re[4 * ri + 3] = 4 * x2;
        cr[ri] = x0 - x2;
        ci[ri] = x1;
    }
    // row 3: the same rule on the complex triple a + i b
    cr[4] = 4 * a[0];            ci[4] = 4 * b[0];
    cr[5] = a[0] + a[1] + a[2];  ci[5] = b[0] + b[1] + b[2];
    cr[6] = a[0] - a[1] + a[2];  ci[6] = b[0] - b[1] + b[2];
    cr[7] = 4 * a[2];            ci[7] = 4 * b[2];
    cr[8] = a[0] - a[2] - b[1];  ci[8] = b[0] - b[2] + a[1];   // (x0-x2) + i x1
    cr[9] = a[0] - a[2] + b[1];  ci[9] = b[0] - b[2] - a[1];   // (x0-x2) - i x1
}

// How the stored filter bytes are read: signed int8, or uint8 minus a zero point (Section 4.1: int9).
struct FilterBytes {
    int is_unsigned, zero_point;
    __device__ inline int value(int8_t b) const { return is_unsigned ? (int)(uint8_t)b - zero_point : (int)b; }
};

__device__ inline void load_filter(const int8_t* w, FilterBytes fb, int k, int c, int K, int C, int layout, int g[9]) {
    if (k >= K || c >= C) {
        for (int i = 0; i < 9; ++i) g[i] = 0;
        return;
    }
    for (int i = 0; i < 9; ++i)
        g[i] = fb.value((layout == WG_NCHW) ? w[((size_t)k * C + c) * 9 + i] : w[((size_t)k * 9 + i) * C + c]);
}

__global__ void blob_init_kernel(uint8_t* blob, uint32_t magic, int K, int C, int mode, int Kp, int CB, size_t maxmag_off) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        BlobHeader* h = reinterpret_cast<BlobHeader*>(blob);
        h->magic = magic; h->version = kBlobVersion;
        h->K = K; h->C = C; h->mode = mode; h->range = kWeightRange;
        h->Kp = Kp; h->CB = CB; h->planes = num_filter_planes(mode);
        for (int j = 0; j < 55; ++j) h->reserved[j] = 0;
    }
    if (i < Kp * kEntries) reinterpret_cast<uint32_t*>(blob + maxmag_off)[i] = 0;
}

// Step 2 of Section 4.2: the largest magnitude over input channels at every
// (filter, entry); a complex entry counts max(|Re|, |Im|).  One wave per
// (filter, 64-channel block): shuffle reduction, then one atomic per entry.
__global__ __launch_bounds__(64) void filter_maxmag_kernel(const int8_t* w, FilterBytes fb, int K, int C, int layout,
                                                           uint32_t* maxmag) {
    int k = blockIdx.x, c = blockIdx.y * 64 + threadIdx.x;
    int g[9], re[16], cr[10], ci[10];
    load_filter(w, fb, k, c, K, C, layout, g);
    filter_entries(g, re, cr, ci);
    for (int e = 0; e < kEntries; ++e) {
        int m = e < 16 ? abs(re[e]) : max(abs(cr[e - 16]), abs(ci[e - 16]));
        for (int off = 32; off > 0; off >>= 1) m = max(m, __shfl_xor(m, off));
        if (threadIdx.x == 0) atomicMax(&maxmag[k * kEntries + e], (uint32_t)m);
    }
}

// Steps 3-4 of Section 4.2 and the reciprocal of its last paragraph.
//   mx <= range: no scaling.  Otherwise the largest n/2^p, n in 8..15, with n*mx <= range*2^p:
//   y = floor(log2(range*128/mx)), n = floor(range*1024 / (mx*2^y)), p = 10 - y.
//   Inverse: r = round(2^(p+q)/n) with the largest q <= 7 that keeps r <= 255.
__global__ void filter_table_kernel(const uint32_t* maxmag, ScaleEntry* table, int count, int mode) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    ScaleEntry s = {0, 0, 1, 0};
    int mx = (int)maxmag[i];
    if (mode == WG_SCALED && mx > kWeightRange) {
        const int num = kWeightRange * 128;          // mx <= 16 * 255 = 4080 < num / 2, so y >= 1 (int8 filters: mx <= 2048, y >= 2)
        int y = 0;
        while ((mx << (y + 1)) <= num) ++y;
        s.n = (num * 8) / (mx << y);
        s.p = 10 - y;
        for (int q = 7; q >= 0; --q) {
            int r = ((2 << (s.p + q)) + s.n) / (2 * s.n);
            if (r <= 255) { s.r = r; s.q = q; break; }
        }
    }
    table[i] = s;
}

__device__ inline int scale_half_up(int v, int n, int p) { return (v * n + (1 << (p - 1))) >> p; }

// Writes the operand planes.  One thread per (filter row k < Kp, channel c < 64*CB);
// rows and channels beyond K, C are written as zeros so the contraction needs no masks.
__global__ __launch_bounds__(256) void filter_pack_kernel(const int8_t* w, FilterBytes fb, int K, int C, int layout,
                                                          int mode, int Kp, int CB,
                                                          const ScaleEntry* table, int8_t* planes,
                                                          int16_t* narrow, int8_t* pairs) {
    int c = blockIdx.x * 64 + (threadIdx.x & 63);
    int k = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (k >= Kp) return;
    int g[9], re[16], cr[10], ci[10];
    load_filter(w, fb, k, c, K, C, layout, g);
    filter_entries(g, re, cr, ci);
    const size_t plane_stride = kFilterFragBytes;
    int8_t* base = planes + filter_plane_offset(0, c >> 6, k, c & 63, Kp, num_filter_planes(mode));
    // narrow table (C <= 4 only): the same values, unsplit, int16 [k][36][4]
    int16_t* wide = narrow != nullptr && c < kNarrowChannels ? narrow + (size_t)k * kNarrowValues * kNarrowChannels + c
                                                             : nullptr;
    if (mode == WG_LOSSLESS) {
        if (wide != nullptr) {
            for (int e = 0; e < 16; ++e) wide[e * kNarrowChannels] = (int16_t)re[e];
            for (int j = 0; j < 10; ++j) {
                wide[(16 + 2 * j) * kNarrowChannels] = (int16_t)cr[j];
                wide[(17 + 2 * j) * kNarrowChannels] = (int16_t)ci[j];
            }
        }
        // value v -> planes 3v: v>>6, 3v+1: v&63, 3v+2: their sum (Karatsuba's middle operand, Section 3.1)
        auto put = [&](int value_index, int v) {
            int hi = v >> 6, lo = v & 63;
            base[(size_t)(3 * value_index + 0) * plane_stride] = (int8_t)hi;
            base[(size_t)(3 * value_index + 1) * plane_stride] = (int8_t)lo;
            base[(size_t)(3 * value_index + 2) * plane_stride] = (int8_t)(hi + lo);
        };
        for (int e = 0; e < 16; ++e) put(e, re[e]);
        for (int j = 0; j < 10; ++j) {
            put(16 + 3 * j + 0, cr[j]);
            put(16 + 3 * j + 1, ci[j]);
            put(16 + 3 * j + 2, cr[j] + ci[j]);
        }
        // the same values as byte-limb pairs, v = 256 h + l (l the low byte, signed), limbs in neighbouring rows
        auto put_pair = [&](int value_index, int v) {
            int8_t* at = pairs + filter_pair_offset(value_index, c >> 6, k, 0, c & 63, Kp);
            at[0] = (int8_t)((v + 128) >> 8);
            at[kCBlock] = (int8_t)(v & 0xff);
        };
        for (int e = 0; e < 16; ++e) put_pair(e, re[e]);
        for (int j = 0; j < 10; ++j) {
            put_pair(16 + 2 * j, cr[j]);
            put_pair(17 + 2 * j, ci[j]);
        }
    } else {
        const ScaleEntry* tk = table + (size_t)k * kEntries;
        for (int e = 0; e < 16; ++e) {
            ScaleEntry s = tk[e];
            int v = s.n ? scale_half_up(re[e], s.n, s.p) : re[e];
            base[(size_t)e * plane_stride] = (int8_t)v;
            if (wide != nullptr) wide[e * kNarrowChannels] = (int16_t)v;
        }
        for (int j = 0; j < 10; ++j) {
            ScaleEntry s = tk[16 + j];
            int vr = s.n ? scale_half_up(cr[j], s.n, s.p) : cr[j];
            int vi = s.n ? scale_half_up(ci[j], s.n, s.p) : ci[j];
            base[(size_t)(16 + 3 * j + 0) * plane_stride] = (int8_t)vr;
            base[(size_t)(16 + 3 * j + 1) * plane_stride] = (int8_t)vi;
            base[(size_t)(16 + 3 * j + 2) * plane_stride] = (int8_t)(-vi);
            if (wide != nullptr) {
                wide[(16 + 2 * j) * kNarrowChannels] = (int16_t)vr;
                wide[(17 + 2 * j) * kNarrowChannels] = (int16_t)vi;
            }
        }
    }
}

__global__ void unpack_filter_planes_kernel(const int8_t* planes, const ScaleEntry* table, int8_t* dense,
                                            int32_t* table_out, int K, int C, int Kp, int CB, int nplanes) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)nplanes * K * C;
    if (i < total) {
        int c = (int)(i % C);
        int k = (int)((i / C) % K);
        int pl = (int)(i / ((size_t)C * K));
        dense[i] = planes[filter_plane_offset(pl, c >> 6, k, c & 63, Kp, nplanes)];
    }
    if (i < (size_t)K * kEntries) {
        ScaleEntry s = table[i];
        table_out[4 * i + 0] = s.n; table_out[4 * i + 1] = s.p;
        table_out[4 * i + 2] = s.r; table_out[4 * i + 3] = s.q;
    }
}

}  // namespace

hipError_t launch_filter_transform(const int8_t* w, int is_unsigned, int zero_point, int K, int C, int layout, int mode,
                                   void* blob_v, hipStream_t s) {
    const FilterBytes fb = {is_unsigned, zero_point};
    uint8_t* blob = static_cast<uint8_t*>(blob_v);
    const int Kp = ceil_div(K, kFilterPad) * kFilterPad, CB = ceil_div(C, kCBlock);
    const BlobLayout bl = blob_layout(Kp, C, mode);
    uint32_t* maxmag = reinterpret_cast<uint32_t*>(blob + bl.maxmag_off);
    ScaleEntry* table = reinterpret_cast<ScaleEntry*>(blob + bl.table_off);
    int8_t* planes = reinterpret_cast<int8_t*>(blob + bl.planes_off);
    const int entries = Kp * kEntries;
    blob_init_kernel<<<ceil_div(entries, 256), 256, 0, s>>>(blob, is_unsigned ? kBlobMagicInt9 : kBlobMagic, K, C, mode, Kp, CB,
                                                            bl.maxmag_off);
    if (mode == WG_SCALED)
        filter_maxmag_kernel<<<dim3(K, CB), 64, 0, s>>>(w, fb, K, C, layout, maxmag);
    filter_table_kernel<<<ceil_div(entries, 256), 256, 0, s>>>(maxmag, table, entries, mode);
    int16_t* narrow = C <= kNarrowChannels ? reinterpret_cast<int16_t*>(blob + bl.narrow_off) : nullptr;
    int8_t* pairs = reinterpret_cast<int8_t*>(blob + bl.pairs_off);
    filter_pack_kernel<<<dim3(CB, ceil_div(Kp, 4)), 256, 0, s>>>(w, fb, K, C, layout, mode, Kp, CB, table, planes, narrow, pairs);
    return hipGetLastError();
}

hipError_t launch_unpack_filter_planes(const void* blob_v, int8_t* dense, int32_t* table_out, int K, int C,
                                       int mode, hipStream_t s) {
    const uint8_t* blob = static_cast<const uint8_t*>(blob_v);
    const int Kp = ceil_div(K, kFilterPad) * kFilterPad, CB = ceil_div(C, kCBlock);
    const BlobLayout bl = blob_layout(Kp, C, mode);
    const int nplanes = num_filter_planes(mode);
    size_t total = (size_t)nplanes * K * C;
    size_t threads = total > (size_t)K * kEntries ? total : (size_t)K * kEntries;
    unpack_filter_planes_kernel<<<(unsigned)((threads + 255) / 256), 256, 0, s>>>(
        reinterpret_cast<const int8_t*>(blob + bl.planes_off),
        reinterpret_cast<const ScaleEntry*>(blob + bl.table_off), dense, table_out, K, C, Kp, CB, nplanes);
    return hipGetLastError();
}

}  // namespace wg
