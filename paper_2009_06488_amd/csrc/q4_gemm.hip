// 4-bit x 4-bit -> int32 matrix product for gfx950 (MI355X), and the same main loop fed by
// an im2col gather for convolution.
//
// What is computed: the first term of Eq. (2) of the paper (raw code products summed over
// the depth) on the int8 matrix cores, then the three zero-point terms of Eq. (2) / Eq. (3)
// in the epilogue:   C = raw - za * colsumB[n] - zb * rowsumA[m] + K * za * zb.
//
// Data path per workgroup (BM x BN output tile, depth step of 128 codes = 64 bytes per row):
//   HBM --16-byte loads--> registers --> LDS (still packed, two codes per byte, XOR-swizzled
//   16-byte chunks) --ds_read_b128--> registers --unpack--> v_mfma_i32_32x32x32_i8.
// The unpack is the widening step of Sec. 2.2 (4-bit codes zero-extended to 8 bits): one
// packed dword w gives (w & 0x0F0F0F0F) and ((w >> 4) & 0x0F0F0F0F).  These hold the even
// and the odd depth positions; since A and B are split the same way and a dot product does
// not depend on the order of its terms, no re-interleave is needed.
#include "q4_kernels.h"

namespace q4 {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kStepBytes = 64;               // bytes of depth per row per main-loop step
constexpr int kChunks = kStepBytes / 16;     // 16-byte chunks per row per step
constexpr uint32_t kLowNibbles = 0x0F0F0F0Fu;

enum LoadMode {
    kDenseAligned = 0,  // rows 16-byte aligned, ceil(K/2) a multiple of 16
    kDenseGeneric = 1,  // any alignment, any K
    kConvAligned = 2,   // C a multiple of 32: every 16-byte chunk lies inside one tap
    kConvGeneric = 3    // any C: gathered code by code
};

struct KernelArgs {
    const uint8_t *A;
    const uint8_t *B;
    int32_t *C;
    const int32_t *rowsumA;
    const int32_t *colsumB;
    int M, N, K;
    int kbytes;  // ceil(K/2)
    long lda, ldb, ldc;
    int za, zb;
    int tiles_m, tiles_n;
    ConvGeom g;
};

// XOR swizzle of the 16-byte chunk index inside a 64-byte LDS row.  For rows r..r+7 (and
// r..r+15) read at the same logical chunk the physical chunks fall into distinct banks.
__device__ __forceinline__ int swizzle(int row)
{
    return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1);
}

__device__ __forceinline__ uint32_t load_dword_guarded(const uint8_t *row, long b, long rowbytes, bool odd_k)
{
    const uint8_t *p = row + b;
    uint32_t v = 0;
    if (b + 4 <= rowbytes && (reinterpret_cast<uintptr_t>(p) & 3u) == 0) {
        v = *reinterpret_cast<const uint32_t *>(p);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (b + i < rowbytes) v |= static_cast<uint32_t>(p[i]) << (8 * i);
    }
    if (odd_k) {  // the pad nibble after the last code must not reach the product
        const long last = rowbytes - 1 - b;
        if (last >= 0 && last < 4) v &= ~(0xF0u << (8 * last));
    }
    return v;
}

// One 16-byte chunk of a dense packed row: bytes [kb, kb+16) of the row, zero past the end.
template <bool ALIGNED>
__device__ __forceinline__ uint4 load_dense_chunk(const uint8_t *row, int kb, int kbytes, bool odd_k)
{
    uint4 v = make_uint4(0, 0, 0, 0);
    if constexpr (ALIGNED) {
        if (kb < kbytes) v = *reinterpret_cast<const uint4 *>(row + kb);
    } else {
        if (kb < kbytes) {
            v.x = load_dword_guarded(row, kb, kbytes, odd_k);
            v.y = load_dword_guarded(row, kb + 4, kbytes, odd_k);
            v.z = load_dword_guarded(row, kb + 8, kbytes, odd_k);
            v.w = load_dword_guarded(row, kb + 12, kbytes, odd_k);
        }
    }
    return v;
}

// Where an output pixel's receptive field starts in the input.
struct PatchOrigin {
    long pixel0;  // n * H * W
    int ih0, iw0; // oh * sh - ph, ow * sw - pw
};

__device__ __forceinline__ PatchOrigin patch_origin(const ConvGeom &g, long m)
{
    PatchOrigin o;
    const int ow = static_cast<int>(m % g.OW);
    const long t = m / g.OW;
    const int oh = static_cast<int>(t % g.OH);
    o.pixel0 = (t / g.OH) * g.H * g.W;
    o.ih0 = oh * g.sh - g.ph;
    o.iw0 = ow * g.sw - g.pw;
    return o;
}

// 16-byte chunk of the virtual im2col row when C % 32 == 0: depth bytes [kb, kb+16) are 32
// channels of a single tap (kh, kw).
__device__ __forceinline__ uint4 load_conv_chunk_aligned(const uint8_t *x, const ConvGeom &g,
                                                         const PatchOrigin &o, int kb, int kbytes)
{
    uint4 v = make_uint4(0, 0, 0, 0);
    if (kb < kbytes) {
        const int kn = 2 * kb;
        const int tap = kn / g.C;
        const int c0 = kn - tap * g.C;
        const int kh = tap / g.KW;
        const int kw = tap - kh * g.KW;
        const int ih = o.ih0 + kh, iw = o.iw0 + kw;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
            const long e = ((o.pixel0 + static_cast<long>(ih) * g.W + iw) * g.C + c0) >> 1;
            v = *reinterpret_cast<const uint4 *>(x + e);
        } else {
            const uint32_t f = static_cast<uint32_t>(g.zx) * 0x11111111u;
            v = make_uint4(f, f, f, f);
        }
    }
    return v;
}

// Same chunk for any channel count: eight codes per dword gathered one by one.
__device__ __forceinline__ uint32_t load_conv_dword_generic(const uint8_t *x, const ConvGeom &g,
                                                            const PatchOrigin &o, int kn0, int K)
{
    uint32_t v = 0;
    int tap = kn0 / g.C;
    int c = kn0 - tap * g.C;
    int kh = tap / g.KW;
    int kw = tap - kh * g.KW;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (kn0 + j < K) {
            const int ih = o.ih0 + kh, iw = o.iw0 + kw;
            uint32_t code = static_cast<uint32_t>(g.zx);
            if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
                const long e = (o.pixel0 + static_cast<long>(ih) * g.W + iw) * g.C + c;
                code = (x[e >> 1] >> (4 * (e & 1))) & 15u;
            }
            v |= code << (4 * j);
        }
        if (++c == g.C) {
            c = 0;
            if (++kw == g.KW) {
                kw = 0;
                ++kh;
            }
        }
    }
    return v;
}

__device__ __forceinline__ v4i low_codes(const uint4 &p)
{
    v4i r;
    r[0] = p.x & kLowNibbles;
    r[1] = p.y & kLowNibbles;
    r[2] = p.z & kLowNibbles;
    r[3] = p.w & kLowNibbles;
    return r;
}

__device__ __forceinline__ v4i high_codes(const uint4 &p)
{
    v4i r;
    r[0] = (p.x >> 4) & kLowNibbles;
    r[1] = (p.y >> 4) & kLowNibbles;
    r[2] = (p.z >> 4) & kLowNibbles;
    r[3] = (p.w >> 4) & kLowNibbles;
    return r;
}

// Workgroup id -> output tile.  Consecutive workgroup ids land on different XCDs (each with
// its own L2), so ids are first regrouped so that one XCD owns a contiguous run of tiles,
// and a run walks the tile grid in column-major bands of kBand tile rows: the tiles in
// flight on one XCD then share A row-panels and B column-panels in that XCD's L2.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int kXcds = 8;
    constexpr int kBand = 8;
    const int nt = tiles_m * tiles_n;
    if (nt % kXcds == 0) pid = (pid % kXcds) * (nt / kXcds) + pid / kXcds;
    const int per_band = kBand * tiles_n;
    const int band = pid / per_band;
    const int first_m = band * kBand;
    const int band_rows = min(tiles_m - first_m, kBand);
    const int in_band = pid - band * per_band;
    tm = first_m + in_band % band_rows;
    tn = in_band / band_rows;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int MODE>
__global__ void __launch_bounds__(WAVES_M *WAVES_N * 64)
q4_gemm_kernel(const KernelArgs p)
{
    constexpr int T = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int NA = BM * kChunks / T, NB = BN * kChunks / T;
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 fragments");
    static_assert(BM * kChunks % T == 0 && BN * kChunks % T == 0, "tile rows must divide over the threads");
    constexpr bool kConv = (MODE == kConvAligned || MODE == kConvGeneric);
    constexpr bool kAligned = (MODE == kDenseAligned || MODE == kConvAligned);

    __shared__ uint4 lds[2][(BM + BN) * kChunks];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const bool odd_k = (p.K & 1) != 0;

    // ---- what this thread copies from HBM to LDS at every step
    const int chunk = tid % kChunks;  // same for all of a thread's slots (T is a multiple of kChunks)
    const uint8_t *a_row[NA];
    PatchOrigin a_org[NA];
    int a_lds[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row = (tid + i * T) / kChunks;
        const long m = min(static_cast<long>(m0 + row), static_cast<long>(p.M - 1));  // rows past M repeat the last one; never stored
        if constexpr (kConv) a_org[i] = patch_origin(p.g, m);
        else a_row[i] = p.A + m * p.lda;
        a_lds[i] = row * kChunks + (chunk ^ swizzle(row));
    }
    const uint8_t *b_row[NB];
    int b_lds[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int row = (tid + i * T) / kChunks;
        const long n = min(static_cast<long>(n0 + row), static_cast<long>(p.N - 1));
        b_row[i] = p.B + n * p.ldb;
        b_lds[i] = BM * kChunks + row * kChunks + (chunk ^ swizzle(row));
    }

    uint4 a_reg[NA], b_reg[NB];
    auto fetch = [&](int kt) {
        const int kb = kt * kStepBytes + chunk * 16;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if constexpr (MODE == kConvAligned) {
                a_reg[i] = load_conv_chunk_aligned(p.A, p.g, a_org[i], kb, p.kbytes);
            } else if constexpr (MODE == kConvGeneric) {
                a_reg[i] = make_uint4(0, 0, 0, 0);
                if (kb < p.kbytes) {
                    a_reg[i].x = load_conv_dword_generic(p.A, p.g, a_org[i], 2 * kb, p.K);
                    a_reg[i].y = load_conv_dword_generic(p.A, p.g, a_org[i], 2 * kb + 8, p.K);
                    a_reg[i].z = load_conv_dword_generic(p.A, p.g, a_org[i], 2 * kb + 16, p.K);
                    a_reg[i].w = load_conv_dword_generic(p.A, p.g, a_org[i], 2 * kb + 24, p.K);
                }
            } else {
                a_reg[i] = load_dense_chunk<kAligned>(a_row[i], kb, p.kbytes, odd_k);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) b_reg[i] = load_dense_chunk<kAligned>(b_row[i], kb, p.kbytes, odd_k);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA; ++i) lds[buf][a_lds[i]] = a_reg[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) lds[buf][b_lds[i]] = b_reg[i];
    };

    // ---- what this lane reads back for the matrix cores: row (lane % 32) of each 32-row
    // fragment, chunk 2*s + lane/32 of the step (s = 0, 1).
    const int frow = lane & 31;
    const int half = lane >> 5;
    const int fsw = swizzle(frow);
    int a_frag[2], b_frag[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int c = (2 * s + half) ^ fsw;
        a_frag[s] = (wm * WM + frow) * kChunks + c;
        b_frag[s] = BM * kChunks + (wn * WN + frow) * kChunks + c;
    }

    v16i acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int steps = (p.kbytes + kStepBytes - 1) / kStepBytes;
    fetch(0);
    stash(0);
    __syncthreads();

    for (int kt = 0; kt < steps; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < steps) fetch(kt + 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint4 pa[FM], pb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) pa[i] = lds[buf][a_frag[s] + i * 32 * kChunks];
#pragma unroll
            for (int j = 0; j < FN; ++j) pb[j] = lds[buf][b_frag[s] + j * 32 * kChunks];
            v4i alo[FM], ahi[FM], blo[FN], bhi[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                alo[i] = low_codes(pa[i]);
                ahi[i] = high_codes(pa[i]);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                blo[j] = low_codes(pb[j]);
                bhi[j] = high_codes(pb[j]);
            }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(alo[i], blo[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ahi[i], bhi[j], acc[i][j], 0, 0, 0);
                }
        }
        if (kt + 1 < steps) stash(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: zero-point terms of Eq. (2), then store.  In a 32x32 accumulator
    // fragment register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    const int kzz = p.K * p.za * p.zb;
#pragma unroll
    for (int j = 0; j < FN; ++j) {
        const int n = n0 + wn * WN + j * 32 + frow;
        if (n >= p.N) continue;
        const int col_term = kzz - p.za * p.colsumB[n];
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (m < p.M)
                    p.C[m * p.ldc + n] = acc[i][j][v] + col_term - p.zb * p.rowsumA[m];
            }
        }
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_tile(const GemmProblem &q, hipStream_t stream)
{
    KernelArgs a;
    a.A = q.A;
    a.B = q.B;
    a.C = q.C;
    a.rowsumA = q.rowsumA;
    a.colsumB = q.colsumB;
    a.M = q.M;
    a.N = q.N;
    a.K = q.K;
    a.kbytes = (q.K + 1) / 2;
    a.lda = q.lda;
    a.ldb = q.ldb;
    a.ldc = q.ldc;
    a.za = q.za;
    a.zb = q.zb;
    a.tiles_m = (q.M + BM - 1) / BM;
    a.tiles_n = (q.N + BN - 1) / BN;
    a.g = q.g;
    const dim3 grid(static_cast<unsigned>(a.tiles_m) * static_cast<unsigned>(a.tiles_n));
    const dim3 block(WAVES_M * WAVES_N * 64);

    const bool b_aligned = (reinterpret_cast<uintptr_t>(q.B) % 16 == 0) && (q.ldb % 16 == 0) && (a.kbytes % 16 == 0) && (q.K % 2 == 0);
    if (!q.is_conv) {
        const bool a_aligned = (reinterpret_cast<uintptr_t>(q.A) % 16 == 0) && (q.lda % 16 == 0);
        if (a_aligned && b_aligned)
            q4_gemm_kernel<BM, BN, WAVES_M, WAVES_N, kDenseAligned><<<grid, block, 0, stream>>>(a);
        else
            q4_gemm_kernel<BM, BN, WAVES_M, WAVES_N, kDenseGeneric><<<grid, block, 0, stream>>>(a);
    } else {
        const bool x_aligned = (reinterpret_cast<uintptr_t>(q.A) % 16 == 0) && (q.g.C % 32 == 0);
        if (x_aligned && b_aligned)
            q4_gemm_kernel<BM, BN, WAVES_M, WAVES_N, kConvAligned><<<grid, block, 0, stream>>>(a);
        else
            q4_gemm_kernel<BM, BN, WAVES_M, WAVES_N, kConvGeneric><<<grid, block, 0, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmProblem &p, int force_tile, hipStream_t stream)
{
    int tile = force_tile;
    if (tile < 0) {
        // Large tiles reuse operands best but need enough of them to fill 256 compute units.
        const long t_large = ((p.M + 255L) / 256) * ((p.N + 255L) / 256);
        const long t_medium = ((p.M + 127L) / 128) * ((p.N + 127L) / 128);
        if (t_large >= 256) tile = 0;
        else if (t_medium >= 128) tile = 1;
        else tile = 2;
    }
    switch (tile) {
    case 0: return launch_tile<256, 256, 2, 4>(p, stream);
    case 1: return launch_tile<128, 128, 2, 2>(p, stream);
    default: return launch_tile<64, 64, 2, 2>(p, stream);
    }
}

}  // namespace q4
