// K split across the waves of a workgroup (the paper's three-dimensional arrangement of warps
// inside a block for small sizes, Section 5.3): each of the four waves owns the WHOLE BM x BN
// tile of C but only one of the four k-groups of every K slab, so a small tile still keeps
// four waves busy, every operand fragment a wave fetches feeds BM/32 or BN/32 matrix
// instructions instead of one, and the four partial tiles are summed inside the workgroup
// through LDS - no workspace in global memory, no second kernel.
//
// Operands are staged exactly as in gemm_tile_kernel (direct 16-byte global->LDS loads into a
// ring of five operand slots, same LDS images), one slab per step:
//   step t:  fetch this wave's k-group of slab t from LDS (landed, certified by barrier t);
//            issue X(t+2) into the spare slot; multiply slab t-1 meanwhile;
//            wait: own fetches done, all but the X(t+2) loads landed; barrier t+1;
//            issue Y(t+2) into X(t)'s slot, which every wave has finished reading.
// The kernel serves operands the direct loads serve (4-byte aligned, whole granules) and K a multiple of the slab; the host runs the
// two-dimensional tile of the same size otherwise.  M and N may be ragged (rows past the edge
// re-read a valid row, their results are dropped at the store).
#pragma once
#include "gemm_kernel.h"

namespace gemm_gfx950 {

// operand fetch with the k-group chosen at run time (it is the wave number here)
template <typename T, int R, bool KC>
__device__ __forceinline__ typename Frag<T>::type fetch_kg(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    if constexpr (sizeof(T) == 2 && !KC) {
        // the transposing read of fetch_f16_mc_kg with the k-group offset added at run time
        constexpr int RB = R * 2;
        const int s = lane & 15;
        const int col = r0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
        const int kl = 8 * (lane >> 5) + (s >> 2);
        const GEMM_LDS(char) *p =
            img + (kl + 16 * kg) * RB + ((((col >> 3) ^ swz_mc<_Float16, R / 8>(kl))) << 4) + ((col & 7) << 1);
        const half4_t lo = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4f16((GEMM_LDS(fp16x4_t) *)p));
        const half4_t hi =
            __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4f16((GEMM_LDS(fp16x4_t) *)(p + 4 * RB)));
        const half8_t out = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(typename Frag<T>::type, out);
    } else {
        return Fetch<T, R, KC>::get(img, r0, kg, lane);
    }
}

template <typename T, int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(256) void gemm_ksplit_kernel(const KernelArgs p)
{
    constexpr int NW = 4, NT = 256;
    constexpr int BK = Elem<T>::BK;
    constexpr int FM = BM / 32, FN = BN / 32;
    static_assert(KGS == NW, "one k-group of every slab per wave");
    static_assert(BM >= 64 && BN >= 64, "the LDS swizzles are defined for operands of 64 rows or more");
    constexpr int A_BYTES = BM * RBK, B_BYTES = BN * RBK;
    constexpr int SLOT = A_BYTES > B_BYTES ? A_BYTES : B_BYTES;
    constexpr int SW = BN + 8;                // staging row stride in words (see gemm_tile_kernel's epilogue)
    constexpr int STAGE = 32 * SW * 4;        // one wave's band of 32 rows
    constexpr int RING = NSLOT * SLOT;
    constexpr int LDS_BYTES = RING > NW * STAGE ? RING : NW * STAGE;
    typedef typename Frag<T>::type frag_t;
    constexpr int NVA = A_BYTES / 1024 / NW, NVB = B_BYTES / 1024 / NW;
    static_assert(NVA >= 1 && NVB >= 1, "tile too small for four loading waves");

    __shared__ __attribute__((aligned(1024))) char smem[LDS_BYTES];
    GEMM_LDS(char) *lds = (GEMM_LDS(char) *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // same work-item order as gemm_tile_kernel: one contiguous run per XCD, K-slice by K-slice
    const int ntiles = p.tiles_m * p.tiles_n;
    const int nwork = ntiles * p.splits;
    const int per_xcd = (nwork + 7) >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= nwork) return;
    const int slice = work / ntiles;
    const int lin = work - slice * ntiles;
    constexpr int GM = 8;
    const int band = lin / (GM * p.tiles_n);
    const int first_m = band * GM;
    const int band_rows = (p.tiles_m - first_m) < GM ? (p.tiles_m - first_m) : GM;
    const int in_band = lin - band * GM * p.tiles_n;
    const int tile_m = first_m + in_band % band_rows;
    const int tile_n = in_band / band_rows;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int KT = p.K / BK;  // K is a multiple of the slab here
    const int kt0 = slice * p.kt_per_split;
    int kt1 = kt0 + p.kt_per_split;
    kt1 = kt1 < KT ? kt1 : KT;
    const int n = kt1 - kt0;  // slabs of this slice, at least one

    const T *A = (const T *)p.A;
    const T *B = (const T *)p.B;
    const bool safe = p.safe != 0;

    float16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    DirectLoader<T, BM, NW, AKC> la;
    DirectLoader<T, BN, NW, BKC> lb;
    la.init(A, p.lda, m0, p.M, kt0 * BK, wave, lane);
    lb.init(B, p.ldb, n0, p.N, kt0 * BK, wave, lane);
    // ring order A(0) B(0) A(1) B(1) ...: slab h of that sequence goes to slot h % 5; past the
    // end of K the loaders re-fetch the last slab (never read), so the number of outstanding
    // loads at every counted wait is the same
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        if (h % 2 == 0) {
            la.issue(lds + h * SLOT, wave);
            la.advance(h / 2 + 1 < n);
        } else {
            lb.issue(lds + h * SLOT, wave);
            lb.advance(h / 2 + 1 < n);
        }
    }
    if (safe) {
        full_sync();
    } else {
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(NVA + NVB));  // slab 0 landed
        barrier_keep_loads();
    }

    auto fetch_all = [&](frag_t(&fa)[FM], frag_t(&fb)[FN], const GEMM_LDS(char) * iA, const GEMM_LDS(char) * iB) {
#pragma unroll
        for (int i = 0; i < FM; ++i) fa[i] = fetch_kg<T, BM, AKC>(iA, i * 32, wave, lane);
#pragma unroll
        for (int j = 0; j < FN; ++j) fb[j] = fetch_kg<T, BN, BKC>(iB, j * 32, wave, lane);
    };
    auto multiply = [&](const frag_t(&fa)[FM], const frag_t(&fb)[FN]) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) mma(acc[i][j], fa[i], fb[j]);
    };

    frag_t fa[2][FM], fb[2][FN];
    int sa = 0;  // slot of A(t); B(t) is the next one, the spare is sa + 4
    auto slot = [&](int d) -> GEMM_LDS(char) * {
        int x = sa + d;
        x = x >= NSLOT ? x - NSLOT : x;
        return lds + x * SLOT;
    };
    // one step; CUR selects the register set that receives slab t (the other holds slab t-1)
    auto step = [&](auto cur_tag, int t) {
        constexpr int CUR = decltype(cur_tag)::value;
        fetch_all(fa[CUR], fb[CUR], slot(0), slot(1));
        la.issue(slot(4), wave);
        la.advance(t + 3 < n);
        if (t > 0) multiply(fa[CUR ^ 1], fb[CUR ^ 1]);
        if (safe) {
            full_sync();
        } else {
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(NVA));  // own fetches done; all but A(t+2) landed
            barrier_keep_loads();
        }
        lb.issue(slot(0), wave);
        lb.advance(t + 3 < n);
        sa = sa + 2 >= NSLOT ? sa + 2 - NSLOT : sa + 2;
    };
    int t = 0;
    for (; t + 1 < n; t += 2) {
        step(std::integral_constant<int, 0>(), t);
        step(std::integral_constant<int, 1>(), t + 1);
    }
    if (t < n) {
        step(std::integral_constant<int, 0>(), t);
        multiply(fa[0], fb[0]);
    } else {
        multiply(fa[1], fb[1]);
    }
    // every direct load has landed (the redundant refills too) and every wave is done with the
    // ring before it is reused for the partial tiles (an explicit wait: the compiler does not
    // track the loads issued from inline assembly)
    full_sync();

    // Sum of the four partial tiles and store, one band of 32 rows at a time: every wave writes
    // its band as binary32 [32][BN + 8] into its own staging area (register r of lane l holds
    // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of a 32x32 block); then the 256 threads share
    // the band's 32 x BN/4 pieces of four columns: a thread adds the four partials of its piece
    // in wave order (so the result does not depend on timing) and stores it.
    float *C = p.C + (int64_t)slice * p.split_stride;
    _Float16 *Ch = (_Float16 *)p.C;
    GEMM_LDS(float) *stage = (GEMM_LDS(float) *)(lds + wave * STAGE);
    const GEMM_LDS(float) *stage0 = (const GEMM_LDS(float) *)lds;
    const int lrow = 4 * (lane >> 5), lcol = lane & 31;
    constexpr int PPR = BN / 4;              // pieces per row
    constexpr int PIECES = 32 * PPR;         // pieces per band
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        if (i > 0) __syncthreads();          // the previous band has been read
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                stage[(8 * (r >> 2) + (r & 3) + lrow) * SW + j * 32 + lcol] = acc[i][j][r];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < (PIECES + NT - 1) / NT; ++it) {
            const int q = it * NT + tid;
            if (PIECES % NT != 0 && q >= PIECES) break;
            const int row = q / PPR, c4 = (q % PPR) * 4;
            const GEMM_LDS(float) *src = stage0 + row * SW + c4;
            float4_t s = *(const GEMM_LDS(float4_t) *)src;
#pragma unroll
            for (int w = 1; w < NW; ++w) s += *(const GEMM_LDS(float4_t) *)(src + w * (STAGE / 4));
            const int grow = m0 + i * 32 + row, gcol = n0 + c4;
            if (grow >= p.M || gcol >= p.N) continue;
            if (p.out16) {
                _Float16 *dst = Ch + (int64_t)grow * p.ldc + gcol;
                half4_t h;
#pragma unroll
                for (int x = 0; x < 4; ++x) h[x] = (_Float16)s[x];
                if (p.rows16_c && gcol + 4 <= p.N) {
                    *(half4_t *)dst = h;     // rows of C on 16-byte boundaries: an 8-byte aligned piece
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (gcol + x < p.N) dst[x] = h[x];
                }
            } else {
                float *dst = C + (int64_t)grow * p.ldc + gcol;
                if (p.rows16_c && gcol + 4 <= p.N) {
                    *(float4_t *)dst = s;
                } else {
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        if (gcol + x < p.N) dst[x] = s[x];
                }
            }
        }
    }
}

}  // namespace gemm_gfx950
