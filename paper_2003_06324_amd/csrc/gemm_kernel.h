// Tiled MFMA GEMM kernel for gfx950 (MI355X), wave64.
//
// One workgroup computes a BM x BN tile of C (the paper's block-level tile,
// Section 3.2 "tile"), walks K in chunks of BK (its "split"), stages the
// A and B chunks in LDS (its "load ... SH") with a double buffer, lets each
// wave own a (BM/WM) x (BN/WN) sub-tile built from 32x32 MFMA blocks held in
// accumulator registers (zero-filled first, stored last: its "epilog").
//
// LDS image of one operand chunk (the same bytes for f16 with BK = 64 and f32
// with BK = 32: a K-row of the chunk is 128 bytes = eight 16-byte granules):
//   K-contiguous operand (row-major A, column-major B): [tile row][128 B],
//     granule g of row r is stored at granule position g ^ (r & 7);
//   M/N-contiguous operand (column-major A, row-major B): [k][R elements],
//     granule g of k-row k is stored at position g ^ swz(k).
// Both images are produced either by direct 16-byte global->LDS loads (each
// wave fills 1 KiB of LDS per instruction, lane l writing bytes [16l, 16l+16),
// so the swizzle is applied by choosing which global granule a lane fetches)
// or, for ragged K tails and unaligned operands, by guarded element loads
// through registers that write the same positions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gemm_gfx950 {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

#define GEMM_LDS(T) __attribute__((address_space(3))) T
#define GEMM_GLB(T) __attribute__((address_space(1))) T

struct KernelArgs {
    const void *A;       // M x K
    const void *B;       // K x N
    float *C;            // row-major M x N, or the split-K workspace
    int64_t lda, ldb, ldc;
    int64_t split_stride;  // elements between consecutive K-slices of the workspace
    int M, N, K;
    int tiles_m, tiles_n;
    int kt_per_split;    // BK-chunks per K-slice (blockIdx.y selects the slice)
};

template <typename T> struct Elem;
template <> struct Elem<_Float16> { static constexpr int EPC = 8, BK = 64; };
template <> struct Elem<float>    { static constexpr int EPC = 4, BK = 32; };

// granule swizzle of an M/N-contiguous chunk, as a function of the k-row
template <typename T> __device__ __forceinline__ int swz_mc(int k);
template <> __device__ __forceinline__ int swz_mc<_Float16>(int k) { return (k & 3) << 1; }
template <> __device__ __forceinline__ int swz_mc<float>(int k) { return ((k >> 2) & 1) << 3; }

// ---------------------------------------------------------------------------
// Direct global->LDS loader for one operand chunk of R tile rows.
// ---------------------------------------------------------------------------
template <typename T, int R, int NW, bool KC>
struct DirectLoader {
    static constexpr int EPC = Elem<T>::EPC, BK = Elem<T>::BK;
    static constexpr int NLOADS = R / 8;  // 1 KiB wave-loads per chunk
    static constexpr int PER_WAVE = NLOADS / NW;
    static_assert(NLOADS % NW == 0 && PER_WAVE >= 1, "tile too small for this wave count");
    static constexpr int CPR = R / EPC;   // granules per k-row (M/N-contiguous image)

    const T *src[PER_WAVE];
    int64_t step;  // elements to advance per K chunk

    // base: operand pointer; ld: leading dimension; row0: first tile row (m or n);
    // rmax: matrix extent in that direction; k0: first k of the first chunk.
    __device__ __forceinline__ void init(const T *base, int64_t ld, int row0, int rmax, int k0,
                                         int wave, int lane)
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + i * NW;
            if (KC) {
                const int r = 8 * j + (lane >> 3);
                const int g = (lane & 7) ^ (lane >> 3);
                int row = row0 + r;
                row = row < rmax ? row : rmax - 1;  // rows past the edge re-read the last one
                src[i] = base + (int64_t)row * ld + k0 + g * EPC;
            } else {
                const int q = 64 * j + lane;
                const int kk = q / CPR;
                const int g = (q % CPR) ^ swz_mc<T>(kk);
                int m = row0 + g * EPC;
                m = m < rmax ? m : row0;  // granules past the edge re-read the first one
                src[i] = base + (int64_t)(k0 + kk) * ld + m;
            }
        }
        step = KC ? (int64_t)BK : (int64_t)BK * ld;
    }

    __device__ __forceinline__ void issue(GEMM_LDS(char) *dst, int wave)
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + i * NW;
            __builtin_amdgcn_global_load_lds((const GEMM_GLB(void) *)src[i],
                                             (GEMM_LDS(void) *)(dst + j * 1024), 16, 0, 0);
        }
    }

    __device__ __forceinline__ void advance()
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) src[i] += step;
    }
};

// ---------------------------------------------------------------------------
// Guarded loader through registers: any alignment, zero-fills outside the
// matrix and outside [.., kend).  Writes the same LDS image as DirectLoader.
// ---------------------------------------------------------------------------
template <typename T, int R, int NT, bool KC>
__device__ __forceinline__ void guarded_load(GEMM_LDS(char) *dst, const T *base, int64_t ld,
                                             int row0, int rmax, int k0, int kend, int tid)
{
    constexpr int EPC = Elem<T>::EPC, BK = Elem<T>::BK;
    constexpr int NGRAN = R * 8;
    constexpr int CPR = R / EPC;
    static_assert(NGRAN % NT == 0, "granules must divide over the threads");
#pragma unroll 2
    for (int i = 0; i < NGRAN / NT; ++i) {
        const int q = tid + i * NT;
        T v[EPC];
        int off;
        if (KC) {
            const int r = q >> 3, g = q & 7;
            const int row = row0 + r, k = k0 + g * EPC;
            const T *p = base + (int64_t)row * ld + k;
            const int nvalid = row < rmax ? kend - k : 0;
#pragma unroll
            for (int e = 0; e < EPC; ++e) v[e] = e < nvalid ? p[e] : (T)0;
            off = r * 128 + ((g ^ (r & 7)) << 4);
        } else {
            const int kk = q / CPR, g = q % CPR;
            const int k = k0 + kk, m = row0 + g * EPC;
            const T *p = base + (int64_t)k * ld + m;
            const int nvalid = k < kend ? rmax - m : 0;
#pragma unroll
            for (int e = 0; e < EPC; ++e) v[e] = e < nvalid ? p[e] : (T)0;
            off = kk * (CPR * 16) + ((g ^ swz_mc<T>(kk)) << 4);
        }
        uint4_t w;
        __builtin_memcpy(&w, v, 16);
        *(GEMM_LDS(uint4_t) *)(dst + off) = w;
    }
}

// ---------------------------------------------------------------------------
// MFMA operand fetch from the LDS image.  One "k-group" is 16 k for f16 and
// 8 k for f32; a chunk has 4 k-groups either way.
//   f16: returns the 8 halves lane l feeds to v_mfma_f32_32x32x16_f16 for
//        block row/column (l & 31): k = 16*kg + 8*(l >> 5) + 0..7.
//   f32: returns 4 floats; element t is what lane l feeds to the t-th
//        v_mfma_f32_32x32x2_f32 of the group: k = 8*kg + 4*(l >> 5) + t.
// ---------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<_Float16> { typedef half8_t type; };
template <> struct Frag<float> { typedef float4_t type; };

// r0: first tile row of the 32-row block inside the chunk image
template <typename T, int R, bool KC>
__device__ __forceinline__ typename Frag<T>::type fetch(const GEMM_LDS(char) *img, int r0, int kg,
                                                        int lane);

template <int R>
__device__ __forceinline__ half8_t fetch_f16_kc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    const int r = r0 + (lane & 31);
    const int g = 2 * kg + (lane >> 5);
    return *(const GEMM_LDS(half8_t) *)(img + r * 128 + ((g ^ (r & 7)) << 4));
}

template <int R>
__device__ __forceinline__ half8_t fetch_f16_mc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    // ds_read_b64_tr_b16: within each group of 16 lanes the 16 x 4 halves the
    // lanes point at are read as a [4][16] array (lane s supplies row s/4,
    // columns 4*(s%4)..+3) and lane i receives column i.  Rows are k, columns
    // are tile rows, so a lane ends up with 4 consecutive k of one tile row.
    constexpr int RB = R * 2;
    const int s = lane & 15;
    const int col = r0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int kq = 16 * kg + 8 * (lane >> 5) + (s >> 2);
    half8_t out;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int k = kq + 4 * t;
        const int off = k * RB + ((((col >> 3) ^ swz_mc<_Float16>(k))) << 4) + ((col & 7) << 1);
        short4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((GEMM_LDS(short4_t) *)(img + off));
        half4_t h;
        __builtin_memcpy(&h, &v, 8);
        out[4 * t + 0] = h[0];
        out[4 * t + 1] = h[1];
        out[4 * t + 2] = h[2];
        out[4 * t + 3] = h[3];
    }
    return out;
}

template <int R>
__device__ __forceinline__ float4_t fetch_f32_kc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    const int r = r0 + (lane & 31);
    const int g = 2 * kg + (lane >> 5);
    return *(const GEMM_LDS(float4_t) *)(img + r * 128 + ((g ^ (r & 7)) << 4));
}

template <int R>
__device__ __forceinline__ float4_t fetch_f32_mc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    constexpr int RB = R * 4;
    const int col = r0 + (lane & 31);
    float4_t out;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int k = 8 * kg + 4 * (lane >> 5) + t;
        const int off = k * RB + (((col >> 2) ^ swz_mc<float>(k)) << 4) + ((col & 3) << 2);
        out[t] = *(const GEMM_LDS(float) *)(img + off);
    }
    return out;
}

template <typename T, int R, bool KC> struct Fetch;
template <int R> struct Fetch<_Float16, R, true> {
    static __device__ __forceinline__ half8_t get(const GEMM_LDS(char) *i, int r0, int kg, int l) { return fetch_f16_kc<R>(i, r0, kg, l); }
};
template <int R> struct Fetch<_Float16, R, false> {
    static __device__ __forceinline__ half8_t get(const GEMM_LDS(char) *i, int r0, int kg, int l) { return fetch_f16_mc<R>(i, r0, kg, l); }
};
template <int R> struct Fetch<float, R, true> {
    static __device__ __forceinline__ float4_t get(const GEMM_LDS(char) *i, int r0, int kg, int l) { return fetch_f32_kc<R>(i, r0, kg, l); }
};
template <int R> struct Fetch<float, R, false> {
    static __device__ __forceinline__ float4_t get(const GEMM_LDS(char) *i, int r0, int kg, int l) { return fetch_f32_mc<R>(i, r0, kg, l); }
};

__device__ __forceinline__ void mma(float16_t &acc, const half8_t &a, const half8_t &b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(float16_t &acc, const float4_t &a, const float4_t &b)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// The kernel.  grid.x = 8 * ceil(tiles/8) workgroups, grid.y = K-slices.
// ---------------------------------------------------------------------------
template <typename T, int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool ALIGNED>
__global__ __launch_bounds__(WM *WN * 64) void gemm_tile_kernel(const KernelArgs p)
{
    constexpr int NW = WM * WN, NT = NW * 64;
    constexpr int BK = Elem<T>::BK;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be built from 32x32 blocks");
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
    typedef typename Frag<T>::type frag_t;

    __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE];
    GEMM_LDS(char) *lds = (GEMM_LDS(char) *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2):
    // give every XCD one contiguous run of tiles, and order tiles in bands of
    // GM tile rows so that tiles running together share A and B panels.
    const int ntiles = p.tiles_m * p.tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lin >= ntiles) return;
    constexpr int GM = 8;
    const int band = lin / (GM * p.tiles_n);
    const int first_m = band * GM;
    const int band_rows = (p.tiles_m - first_m) < GM ? (p.tiles_m - first_m) : GM;
    const int in_band = lin - band * GM * p.tiles_n;
    const int tile_m = first_m + in_band % band_rows;
    const int tile_n = in_band / band_rows;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // K range of this slice
    const int KT = (p.K + BK - 1) / BK;
    const int kt0 = blockIdx.y * p.kt_per_split;
    int kt1 = kt0 + p.kt_per_split;
    kt1 = kt1 < KT ? kt1 : KT;
    const int nkt = kt1 - kt0;
    const int kend = (kt1 * BK) < p.K ? (kt1 * BK) : p.K;

    const T *A = (const T *)p.A;
    const T *B = (const T *)p.B;

    DirectLoader<T, BM, NW, AKC> la;
    DirectLoader<T, BN, NW, BKC> lb;
    if (ALIGNED) {
        la.init(A, p.lda, m0, p.M, kt0 * BK, wave, lane);
        lb.init(B, p.ldb, n0, p.N, kt0 * BK, wave, lane);
    }

    float16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // stage chunk kt (absolute index) into buffer b
    auto stage = [&](int kt, int b) {
        GEMM_LDS(char) *dA = lds + b * STAGE;
        GEMM_LDS(char) *dB = dA + A_BYTES;
        const int k0 = kt * BK;
        if (ALIGNED && k0 + BK <= kend) {
            la.issue(dA, wave);
            lb.issue(dB, wave);
            la.advance();
            lb.advance();
        } else {
            guarded_load<T, BM, NT, AKC>(dA, A, p.lda, m0, p.M, k0, kend, tid);
            guarded_load<T, BN, NT, BKC>(dB, B, p.ldb, n0, p.N, k0, kend, tid);
        }
    };

    if (nkt > 0) {
        stage(kt0, 0);
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
        __syncthreads();
    }

    for (int it = 0; it < nkt; ++it) {
        const int cur = it & 1;
        if (it + 1 < nkt) stage(kt0 + it + 1, cur ^ 1);

        const GEMM_LDS(char) *iA = lds + cur * STAGE;
        const GEMM_LDS(char) *iB = iA + A_BYTES;
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
            frag_t a[FM], b[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) a[i] = Fetch<T, BM, AKC>::get(iA, wm * TM + i * 32, kg, lane);
#pragma unroll
            for (int j = 0; j < FN; ++j) b[j] = Fetch<T, BN, BKC>::get(iB, wn * TN + j * 32, kg, lane);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) mma(acc[i][j], a[i], b[j]);
        }
        // the next chunk has landed (own loads) and everyone is done reading this one
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
    }

    // epilogue: accumulator register r of lane l holds
    //   row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 block
    float *C = p.C + (int64_t)blockIdx.y * p.split_stride;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + wn * TN + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < p.M && col < p.N) C[(int64_t)row * p.ldc + col] = acc[i][j][r];
            }
        }
    }
}

}  // namespace gemm_gfx950
