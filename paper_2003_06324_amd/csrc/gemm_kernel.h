// Tiled MFMA GEMM kernel for gfx950 (MI355X), wave64.
//
// One workgroup computes a BM x BN tile of C (the paper's block-level tile,
// Section 3.2 "tile"), walks K in slabs of BK (its "split"), stages the A and B
// slabs in LDS (its "load ... SH") through a ring of operand slots that direct
// global->LDS loads keep full, lets each wave own a (BM/WM) x (BN/WN) sub-tile
// built from 32x32 MFMA blocks held in accumulator registers (zero-filled first,
// stored last: its "epilog").
//
// A slab is KGS "k-groups"; a k-group is what one MFMA step consumes per lane
// pair: 16 k for f16 (one v_mfma_f32_32x32x16_f16), 8 k for f32 (four
// v_mfma_f32_32x32x2_f32), i.e. 32 bytes per tile row either way.  So both
// types share one byte geometry: a slab row is 32*KGS bytes = 2*KGS granules of
// 16 bytes.
//
// LDS image of one operand slab:
//   K-contiguous operand (row-major A, column-major B): [tile row][32*KGS B],
//     granule g of row r is stored at granule position g ^ swz_kc(r);
//   M/N-contiguous operand (column-major A, row-major B): [k][R elements],
//     granule g of k-row k is stored at position g ^ swz_mc(k).
// The LDS serves 256 bytes per clock from 64 banks: a b128 read is processed
// 16 lanes at a time and a b64 read 32 lanes at a time, so the swizzles are
// chosen to spread every such lane group over all 64 banks.
//
// Both images are produced by direct 16-byte global->LDS loads (each wave fills
// 1 KiB of LDS per instruction, lane l writing bytes [16l, 16l+16), so the
// swizzle is applied by choosing which global granule a lane fetches; the
// global address of a granule needs 4-byte alignment only); for operands that
// are only 2-byte aligned by the same granules fetched through registers and
// written to the same positions; and for ragged K tails by guarded loads
// through registers.  The tile of C leaves through LDS as well when its rows
// allow 16-byte stores (see the epilogue).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace gemm_gfx950 {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef __fp16 fp16x4_t __attribute__((__vector_size__(4 * sizeof(__fp16))));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef int int4_t __attribute__((ext_vector_type(4)));

#define GEMM_LDS(T) __attribute__((address_space(3))) T

#ifndef GEMM_KGS
#define GEMM_KGS 4
#endif
constexpr int KGS = GEMM_KGS;    // k-groups per slab
constexpr int GPR = 2 * KGS;      // granules per row of a K-contiguous image
constexpr int RBK = 16 * GPR;     // bytes per row of a K-contiguous image
constexpr int NSLOT = 5;          // operand slots in the LDS ring of the direct-load pipeline

struct KernelArgs {
    const void *A;       // M x K
    const void *B;       // K x N
    float *C;            // row-major M x N (binary16 elements if out16), or the split-K workspace
    int64_t lda, ldb, ldc;
    int64_t split_stride;  // elements between consecutive K-slices of the workspace
    int M, N, K;
    int tiles_m, tiles_n;
    int kt_per_split;    // slabs per K-slice
    int splits;          // number of K-slices; the grid holds tiles_m * tiles_n * splits work items
    int ld32;            // 256 * ld * sizeof(element) < 2^31 for A and B: tile-local byte offsets fit 32 bits
    int out16;           // C holds binary16: the accumulators are rounded (to nearest even) at the store
    int stream_c;        // binary32 C, no K-slices, rows of C start on 128-byte lines: stores may be non-temporal
    int rows16_c;        // base and rows of C (or of the workspace) on 16-byte boundaries, ldc below 2^20
    int stage_c;         // interior tiles store through LDS in whole rows (needs rows16_c)
    int safe;            // every hand-over of an LDS buffer waits for all outstanding memory operations first
    unsigned long long *trace;  // profiling aid, normally null: 8 words per workgroup (see trace_mark)
    int trace_records;          // workgroups the trace buffer has room for
};

// Profiling aid: with a trace buffer set, thread 0 of every workgroup records the constant-rate
// (100 MHz) clock at the phase boundaries of its tile - 0 start, 1 first slab landed, 2 K loop
// done, 3 LDS free for the epilogue, 4 stores issued, 5 stores complete - and in word 7 where it
// ran (XCC id above bit 32, the hardware id register below).  Costs a scalar branch per mark.
__device__ __forceinline__ void trace_mark(const KernelArgs &p, int slot)
{
    if (p.trace != nullptr && threadIdx.x == 0 && (int)blockIdx.x < p.trace_records)
        p.trace[(size_t)blockIdx.x * 8 + slot] = wall_clock64();
}
__device__ __forceinline__ void trace_place(const KernelArgs &p)
{
    if (p.trace != nullptr && threadIdx.x == 0 && (int)blockIdx.x < p.trace_records) {
        const unsigned hw = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_ID: wave, SIMD, CU, SH, SE ...
        const unsigned xcc = __builtin_amdgcn_s_getreg((31 << 11) | 20);  // XCC_ID
        p.trace[(size_t)blockIdx.x * 8 + 7] = ((unsigned long long)xcc << 32) | hw;
    }
}

template <typename T> struct Elem;
template <> struct Elem<_Float16> { static constexpr int EPC = 8, KG = 16, BK = KG * KGS; };
template <> struct Elem<float>    { static constexpr int EPC = 4, KG = 8, BK = KG * KGS; };
// bfloat16 shares every byte of the binary16 path (loads, LDS images, fragment reads move bit
// patterns); only the MFMA instruction differs
template <> struct Elem<__bf16>   { static constexpr int EPC = 8, KG = 16, BK = KG * KGS; };

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }        // vmcnt(n)
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }  // vmcnt(n) lgkmcnt(0)

// Workgroup barrier that does not drain the vector-memory counter: direct loads for later
// slabs stay in flight across it.  The "memory" clobber keeps the compiler from moving LDS
// accesses over it; the waits that make the hand-over safe are issued by the caller.
__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_barrier" ::: "memory"); }

// The "safe" variant of a hand-over (run-time switch): wait for every outstanding memory and
// LDS operation of this wave, then a barrier.  The pipelines below hand buffers over with
// counted waits and a single barrier per slab; the paper notes (Section 4.1) that removing
// synchronisation is where races come from, so the same kernels can be run with every hand-over
// fully synchronised to compare against.
__device__ __forceinline__ void full_sync()
{
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    barrier_keep_loads();
}

// Granule swizzle of a K-contiguous image.  A b128 fragment read has 16 consecutive lanes
// on 16 consecutive rows at one logical granule; 16/GPR rows share a 256-byte bank period,
// so the row index above that picks the granule position.
__device__ __forceinline__ int swz_kc(int r) { return (r / (16 / GPR)) & (GPR - 1); }

// Granule swizzle of an M/N-contiguous image as a function of the k-row; CPR = granules
// per k-row.  f16 (transposing b64 reads, 32 lanes cover 4 k-rows x 64 bytes): the four
// rows go to four different 64-byte quarters of the bank space.  f32 (b32 reads, lanes
// 0-31 on row k, lanes 32-63 on row k+4): the two rows go to different 128-byte halves.
template <typename T, int CPR> __device__ __forceinline__ int swz_mc(int k)
{
    if (sizeof(T) == 2) return CPR >= 16 ? ((k & 3) << 2) : (((k >> 1) & 1) << 2);
    return ((k >> 2) & 1) << 3;
}

// ---------------------------------------------------------------------------
// Direct global->LDS loader for one operand slab of R tile rows.
// ---------------------------------------------------------------------------
template <typename T, int R, int NW, bool KC>
struct DirectLoader {
    static constexpr int EPC = Elem<T>::EPC, BK = Elem<T>::BK;
    static constexpr int NLOADS = R * RBK / 1024;  // 1 KiB wave-loads per slab
    static constexpr int PER_WAVE = NLOADS / NW;
    static_assert(NLOADS % NW == 0 && PER_WAVE >= 1, "tile too small for this wave count");
    static constexpr int CPR = R / EPC;            // granules per k-row (M/N-contiguous image)
    static constexpr int ROWS_PER_LOAD = 1024 / RBK;

    // Address of a lane's granule = wave-uniform base (scalar registers, advanced per slab)
    // + a 32-bit per-lane byte offset that never changes.  The loads are buffer loads
    // (scalar resource descriptor + vector offset), so the K loop spends no vector
    // instructions on pointers.  The base lives in the descriptor itself: words 0 and 1 are
    // the 48-bit address (stride and swizzle bits above it are zero), word 2 a 2 GiB window
    // (every offset used is below it and inside the operand by construction), word 3 the
    // 32-bit data format.
    int4_t rsrc;
    uint32_t off[PER_WAVE];
    int64_t step;  // bytes to advance per slab

    // origin: operand pointer; ld: leading dimension; row0: first tile row (m or n);
    // rmax: matrix extent in that direction; k0: first k of the first slab.
    // The host guarantees that R * ld * sizeof(T) is below 2^31.
    __device__ __forceinline__ void init(const T *origin, int64_t ld, int row0, int rmax, int k0,
                                         int wave, int lane)
    {
        const uint64_t base =
            (uint64_t)(uintptr_t)(KC ? origin + (int64_t)row0 * ld + k0 : origin + (int64_t)k0 * ld + row0);
        rsrc[0] = (int)(uint32_t)base;
        rsrc[1] = (int)(uint32_t)(base >> 32) & 0xffff;
        rsrc[2] = 0x7fffffff;
        rsrc[3] = 0x00020000;
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int j = wave + i * NW;
            if (KC) {
                const int r = ROWS_PER_LOAD * j + lane / GPR;
                const int g = (lane % GPR) ^ swz_kc(r);
                int row = r;
                row = row0 + row < rmax ? row : rmax - 1 - row0;  // rows past the edge re-read the last one
                off[i] = (uint32_t)(((int64_t)row * ld + g * EPC) * (int64_t)sizeof(T));
            } else {
                const int q = 64 * j + lane;
                const int kk = q / CPR;
                const int g = (q % CPR) ^ swz_mc<T, CPR>(kk);
                int m = g * EPC;
                m = row0 + m < rmax ? m : 0;  // granules past the edge re-read the first one
                off[i] = (uint32_t)(((int64_t)kk * ld + m) * (int64_t)sizeof(T));
            }
        }
        step = (KC ? (int64_t)BK : (int64_t)BK * ld) * (int64_t)sizeof(T);
    }

    // issue this wave's loads number [i0, i1) of the current slab into the slot at dst
    __device__ __forceinline__ void issue(GEMM_LDS(char) *dst, int wave, int i0 = 0, int i1 = PER_WAVE)
    {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            if (i < i0 || i >= i1) continue;
            issue1(dst, wave, i);
        }
    }

    // issue this wave's load number i (compile-time constant after unrolling)
    __device__ __forceinline__ void issue1(GEMM_LDS(char) *dst, int wave, int i)
    {
        // Issued as inline assembly on purpose.  If the compiler sees an LDS-DMA load it makes
        // every later LDS read it cannot prove disjoint wait for vmcnt(0), which would drain
        // the load pipeline at each operand fetch; the kernel orders loads and reads itself
        // (counted vmcnt waits + barrier).  The compiler's own vmcnt waits stay safe: loads
        // complete in order, so extra outstanding loads only make a counted wait stricter.
        const int j = wave + i * NW;
        const uint32_t lds_addr = (uint32_t)(uintptr_t)(dst + j * 1024);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :
                     : "s"(lds_addr), "v"(off[i]), "s"(rsrc)
                     : "memory", "m0");
    }

    // Same load with the LDS destination split into a per-wave run-time part (LDS address
    // of the ring + wave * 1024, held in a scalar register) and a compile-time byte offset
    // OFF of the slot inside the ring: M0 is then set with a single scalar add of an
    // immediate, and the K loop spends no other scalar work on LDS addresses.
    template <int OFF>
    __device__ __forceinline__ void issue_at(uint32_t wave_lds, int i)
    {
        asm volatile("s_add_i32 m0, %0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds"
                     :
                     : "s"(wave_lds), "i"(OFF + i * NW * 1024), "v"(off[i]), "s"(rsrc)
                     : "memory", "m0", "scc");
    }

    // The same granule through a register instead (operands whose rows are only 2-byte
    // aligned cannot use the direct loads): a 16-byte load that needs element alignment only,
    // and the store that puts it where the direct load would have put it.
    __device__ __forceinline__ uint4_t fetch1(int i) const
    {
        // a global-address-space pointer (a generic one would make this a flat load, which
        // also counts as an LDS operation and would be waited for at every operand fetch)
        typedef uint4_t granule_t __attribute__((aligned(2)));  // element alignment of the narrower type
        typedef const __attribute__((address_space(1))) char *gptr_t;
        const gptr_t base = (gptr_t)(uintptr_t)(((uint64_t)(uint32_t)rsrc[1] << 32) | (uint32_t)rsrc[0]);
        return *(const __attribute__((address_space(1))) granule_t *)(base + off[i]);
    }
    __device__ __forceinline__ void store1(GEMM_LDS(char) *dst, int wave, int lane, int i, const uint4_t &w) const
    {
        *(GEMM_LDS(uint4_t) *)(dst + (wave + i * NW) * 1024 + lane * 16) = w;
    }

    // move to the next slab if `more`, else stay (branch-free)
    __device__ __forceinline__ void advance(bool more)
    {
        uint64_t base = ((uint64_t)(uint32_t)rsrc[1] << 32) | (uint32_t)rsrc[0];
        base += more ? step : 0;
        rsrc[0] = (int)(uint32_t)base;
        rsrc[1] = (int)(uint32_t)(base >> 32);
    }
};

// ---------------------------------------------------------------------------
// Guarded loader through registers: any alignment, zero-fills outside the
// matrix and outside [.., kend).  Produces the same LDS image as DirectLoader,
// in two steps so that the global loads of the next slab can be in flight
// while the current one is multiplied: guarded_fetch (global -> registers) and
// staged_store (registers -> LDS).  A granule that lies fully inside the
// matrix is fetched with one 16-byte load (element-aligned only: the compiler
// picks the widest access the target allows), a ragged one element by element.
// ---------------------------------------------------------------------------
template <typename T, int R, int NT>
struct Staged {
    static constexpr int NGRAN = R * GPR;
    static constexpr int ITERS = (NGRAN + NT - 1) / NT;
    uint4_t v[ITERS];
};

// position of granule q of a slab: global pointer, number of valid elements, LDS byte offset
template <typename T, int R, bool KC>
__device__ __forceinline__ void granule_of(int q, const T *base, int64_t ld, int row0, int rmax, int k0,
                                           int kend, const T *&p, int &nvalid, int &off)
{
    constexpr int EPC = Elem<T>::EPC;
    constexpr int CPR = R / EPC;
    if (KC) {
        const int r = q / GPR, g = q % GPR;
        const int row = row0 + r, k = k0 + g * EPC;
        p = base + (int64_t)row * ld + k;
        nvalid = row < rmax ? kend - k : 0;
        off = r * RBK + ((g ^ swz_kc(r)) << 4);
    } else {
        const int kk = q / CPR, g = q % CPR;
        const int k = k0 + kk, m = row0 + g * EPC;
        p = base + (int64_t)k * ld + m;
        nvalid = k < kend ? rmax - m : 0;
        off = kk * (CPR * 16) + ((g ^ swz_mc<T, CPR>(kk)) << 4);
    }
}

// global -> registers: whole granules only (ragged ones are left zero, see staged_store)
template <typename T, int R, int NT, bool KC>
__device__ __forceinline__ void guarded_fetch(Staged<T, R, NT> &st, const T *base, int64_t ld,
                                              int row0, int rmax, int k0, int kend, int tid)
{
    constexpr int EPC = Elem<T>::EPC;
    constexpr int NGRAN = R * GPR;
#pragma unroll
    for (int i = 0; i < Staged<T, R, NT>::ITERS; ++i) {
        const int q = tid + i * NT;
        const T *p;
        int nvalid, off;
        granule_of<T, R, KC>(q, base, ld, row0, rmax, k0, kend, p, nvalid, off);
        if (NGRAN % NT != 0 && q >= NGRAN) nvalid = 0;
        uint4_t w = {0u, 0u, 0u, 0u};
        if (nvalid >= EPC) __builtin_memcpy(&w, p, 16);
        st.v[i] = w;
    }
}

// registers -> LDS; the few granules that straddle the matrix edge or the end of K are
// completed here, element by element, straight from global memory
template <typename T, int R, int NT, bool KC>
__device__ __forceinline__ void staged_store(GEMM_LDS(char) *dst, const Staged<T, R, NT> &st,
                                             const T *base, int64_t ld, int row0, int rmax, int k0,
                                             int kend, int tid)
{
    constexpr int EPC = Elem<T>::EPC;
    constexpr int NGRAN = R * GPR;
#pragma unroll
    for (int i = 0; i < Staged<T, R, NT>::ITERS; ++i) {
        const int q = tid + i * NT;
        if (NGRAN % NT != 0 && q >= NGRAN) break;
        const T *p;
        int nvalid, off;
        granule_of<T, R, KC>(q, base, ld, row0, rmax, k0, kend, p, nvalid, off);
        *(GEMM_LDS(uint4_t) *)(dst + off) = st.v[i];
        if (nvalid > 0 && nvalid < EPC) {
            GEMM_LDS(T) *d = (GEMM_LDS(T) *)(dst + off);
#pragma unroll 1
            for (int x = 0; x < nvalid; ++x) d[x] = p[x];
        }
    }
}

// ---------------------------------------------------------------------------
// MFMA operand fetch from the LDS image, k-group kg of the slab.
//   f16: returns the 8 halves lane l feeds to v_mfma_f32_32x32x16_f16 for
//        block row/column (l & 31): k = 16*kg + 8*(l >> 5) + 0..7.
//   f32: returns 4 floats; element t is what lane l feeds to the t-th
//        v_mfma_f32_32x32x2_f32 of the group: k = 8*kg + 4*(l >> 5) + t.
// ---------------------------------------------------------------------------
template <typename T> struct Frag;
template <> struct Frag<_Float16> { typedef half8_t type; };
template <> struct Frag<float> { typedef float4_t type; };
template <> struct Frag<__bf16> { typedef bf16x8_t type; };

// r0: first tile row of the 32-row block inside the slab image
template <int R>
__device__ __forceinline__ half8_t fetch_f16_kc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    const int r = r0 + (lane & 31);
    const int g = 2 * kg + (lane >> 5);
    return *(const GEMM_LDS(half8_t) *)(img + r * RBK + ((g ^ swz_kc(r)) << 4));
}

template <int R, int KG_>
__device__ __forceinline__ half8_t fetch_f16_mc_kg(const GEMM_LDS(char) *img, int r0, int lane)
{
    // ds_read_b64_tr_b16: within each group of 16 lanes the 16 x 4 halves the
    // lanes point at are read as a [4][16] array (lane s supplies row s/4,
    // columns 4*(s%4)..+3) and lane i receives column i.  Rows are k, columns
    // are tile rows, so a lane ends up with 4 consecutive k of one tile row.
    constexpr int RB = R * 2;
    const int s = lane & 15;
    const int col = r0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int kl = 8 * (lane >> 5) + (s >> 2);  // lane part of k; the rest (16*kg + 4*t) is a multiple of 4
    const GEMM_LDS(char) *p = img + kl * RB + ((((col >> 3) ^ swz_mc<_Float16, R / 8>(kl))) << 4) + ((col & 7) << 1);
    const half4_t lo = __builtin_bit_cast(
        half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4f16((GEMM_LDS(fp16x4_t) *)(p + (16 * KG_) * RB)));
    const half4_t hi = __builtin_bit_cast(
        half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4f16((GEMM_LDS(fp16x4_t) *)(p + (16 * KG_ + 4) * RB)));
    // the two 64-bit results are the low and high half of the 128-bit MFMA operand
    const half8_t out = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return out;
}

template <int R>
__device__ __forceinline__ half8_t fetch_f16_mc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    switch (kg) {  // kg is a compile-time constant at every call site
    case 0: return fetch_f16_mc_kg<R, 0>(img, r0, lane);
    case 1: return fetch_f16_mc_kg<R, 1>(img, r0, lane);
    case 2: return fetch_f16_mc_kg<R, 2>(img, r0, lane);
    default: return fetch_f16_mc_kg<R, 3>(img, r0, lane);
    }
}

template <int R>
__device__ __forceinline__ float4_t fetch_f32_kc(const GEMM_LDS(char) *img, int r0, int kg, int lane)
{
    const int r = r0 + (lane & 31);
    const int g = 2 * kg + (lane >> 5);
    return *(const GEMM_LDS(float4_t) *)(img + r * RBK + ((g ^ swz_kc(r)) << 4));
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
        const int off = k * RB + (((col >> 2) ^ swz_mc<float, R / 4>(k)) << 4) + ((col & 3) << 2);
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

template <int R, bool KC> struct Fetch<__bf16, R, KC> {
    static __device__ __forceinline__ bf16x8_t get(const GEMM_LDS(char) *i, int r0, int kg, int l)
    {
        return __builtin_bit_cast(bf16x8_t, Fetch<_Float16, R, KC>::get(i, r0, kg, l));
    }
};

__device__ __forceinline__ void mma(float16_t &acc, const bf16x8_t &a, const bf16x8_t &b)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
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
// The kernel.  grid.x = 8 * ceil(tiles * K-slices / 8) workgroups.
// ---------------------------------------------------------------------------
template <typename T, int BM, int BN, int WM, int WN, bool AKC, bool BKC, bool ALIGNED>
__global__ __launch_bounds__(WM *WN * 64) void gemm_tile_kernel(const KernelArgs p)
{
    constexpr int NW = WM * WN, NT = NW * 64;
    constexpr int BK = Elem<T>::BK;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    static_assert(TM % 32 == 0 && TN % 32 == 0, "wave tile must be built from 32x32 blocks");
    constexpr int A_BYTES = BM * RBK, B_BYTES = BN * RBK;
    constexpr int SLOT = A_BYTES > B_BYTES ? A_BYTES : B_BYTES;  // one operand slab
    constexpr int NBUF = ALIGNED ? NSLOT : 4;  // ring of five operand slots, or two buffers of (A, B)
    typedef typename Frag<T>::type frag_t;
    constexpr int NVA = A_BYTES / 1024 / NW;  // direct loads per wave per A slab
    constexpr int NVB = B_BYTES / 1024 / NW;
    static_assert(KGS == 4, "the pipeline below is written for four k-groups per slab");

    __shared__ __attribute__((aligned(1024))) char smem[NBUF * SLOT];
    GEMM_LDS(char) *lds = (GEMM_LDS(char) *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD
    // one contiguous run of work items, K-slice by K-slice (the tiles of one slice share that
    // slice's A and B panels; the same tile in another slice shares nothing), and within a
    // slice order tiles in bands of GM tile rows so that tiles running together share panels.
    const int ntiles = p.tiles_m * p.tiles_n;
    const int nwork = ntiles * p.splits;
    const int per_xcd = (nwork + 7) >> 3;
    const int work = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (work >= nwork) return;
    trace_mark(p, 0);
    trace_place(p);
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

    // K range of this slice
    const int KT = (p.K + BK - 1) / BK;
    const int kt0 = slice * p.kt_per_split;
    int kt1 = kt0 + p.kt_per_split;
    kt1 = kt1 < KT ? kt1 : KT;
    const int kend = (kt1 * BK) < p.K ? (kt1 * BK) : p.K;

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
    // Keeps the accumulators in the accumulation registers at this point (an empty asm with an
    // "a" constraint): without it the register allocator parks part of them in ordinary
    // vector registers across the guarded loop and spills the staging registers instead.
    auto pin_acc = [&]() {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) asm volatile("" : "+a"(acc[i][j]));
    };
    pin_acc();

    // One k-group of work in a fixed instruction order (the compiler may not move anything
    // across the fences): the m-th MFMA block (row m / FN of the wave's blocks) is followed by the m-th operand fetch of
    // the NEXT k-group (order a0, b0..b(FN-1), a1..a(FM-1): what the first MFMAs of that
    // k-group need comes first) and by its share of the NL direct loads `load(q)`, so LDS
    // reads and global loads trickle out between MFMAs instead of in bursts that would
    // fill the address queues and stall this wave's MFMA stream.
    auto kgroup = [&](const frag_t(&ca)[FM], const frag_t(&cb)[FN], frag_t(&na)[FM], frag_t(&nb)[FN],
                      const GEMM_LDS(char) * iA, const GEMM_LDS(char) * iB, int kg_next, bool fetch,
                      auto load, auto nl_tag) {
        constexpr int NL = decltype(nl_tag)::value;
        constexpr int NB = FM * FN, NF = FM + FN;
#pragma unroll
        for (int m = 0; m < NB; ++m) {
            // Blocks in boustrophedon order (row 0 left to right, row 1 right to left, ...): consecutive MFMAs share one
            // of their two operand registers, also across the turn of a row.  Each accumulator still gets its products in
            // ascending k, so results do not change; on data that throttles the clock it measures 0.4-0.9 % faster.
            const int mi = m / FN, mj = (mi & 1) ? FN - 1 - m % FN : m % FN;
            mma(acc[mi][mj], ca[mi], cb[mj]);
            // An MFMA is a pure operation to the optimiser, which would otherwise be free to
            // sink it below the fetches and loads that follow; the empty volatile asm is an
            // ordered use of the result and keeps the MFMA at this place in the stream.
            asm volatile("" : "+a"(acc[mi][mj]));
            if (fetch) {
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    // fetch f is issued with block m = f, leftovers with the last block
                    if ((f < NB ? f : NB - 1) != m) continue;
                    if (f == 0) na[0] = Fetch<T, BM, AKC>::get(iA, wm * TM, kg_next, lane);
                    else if (f <= FN) nb[f - 1] = Fetch<T, BN, BKC>::get(iB, wn * TN + (f - 1) * 32, kg_next, lane);
                    else na[f - FN] = Fetch<T, BM, AKC>::get(iA, wm * TM + (f - FN) * 32, kg_next, lane);
                }
            }
            if constexpr (NL > 0) {
#pragma unroll
                for (int q = 0; q < NL; ++q)
                    if (q * NB / NL == m) load(q);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    auto no_load = [](int) {};
    typedef std::integral_constant<int, 0> L0;

    int k_done = kt0 * BK;  // first k not yet accumulated
    // Registers of the guarded loop at the end.  When a fast path is followed by leftover k
    // (a ragged tail), it fetches the first leftover slab into them before its own last slab
    // is multiplied, so that the loads are not waited for in the open.
    Staged<T, BM, NT> sa_;
    Staged<T, BN, NT> sb_;
    bool staged_ready = false;
    auto prefetch_leftover = [&](int k_from) {
        if (k_from < kend) {
            guarded_fetch<T, BM, NT, AKC>(sa_, A, p.lda, m0, p.M, k_from, kend, tid);
            guarded_fetch<T, BN, NT, BKC>(sb_, B, p.ldb, n0, p.N, k_from, kend, tid);
            staged_ready = true;
        }
    };
    if (ALIGNED) {
        // Full slabs: direct global->LDS loads into a ring of NSLOT = 5 operand slots.  One
        // operand, called X below, goes first: slabs are fetched in the order X(0) Y(0) X(1)
        // Y(1) ..., slab number h going to slot h % 5, so tile t has X in slot 2t % 5 and Y
        // in the next one, and one slot is always spare.  Per tile t (four k-groups, operand
        // registers double-buffered):
        //   k-groups 0,1: MFMAs; fetch operands of the next k-group; issue X(t+2) into
        //                 the spare slot, half of its loads per k-group;
        //   k-group 2:    MFMAs; fetch operands of k-group 3;
        //   counted wait: everything but X(t+2) has landed, i.e. tile t+1 is complete;
        //   barrier:      every wave holds k-group 3 in registers, tile t's slots are free;
        //   k-group 3:    MFMAs; issue Y(t+2) into X(t)'s slot; fetch k-group 0 of tile t+1.
        // So loads are in flight all the time (32..96 KiB of the 160 KiB LDS), X slabs have
        // two tiles of MFMA time to land and Y slabs one.  Past the end of K the loaders
        // re-fetch the last slab (never read), which keeps the loop body branch-free and
        // the number of outstanding loads constant for the counted waits.
        // A granule of an M/N-contiguous operand that straddles the matrix edge is read whole (its
        // tail, padding or the start of the next k-row, only feeds tile rows that are never
        // stored); on the operand's last k-row that tail could lie past the operand, so a tile
        // with such granules leaves the slab holding that row to the guarded loop below.
        constexpr int EPC_ = Elem<T>::EPC;
        const bool edge_a = !AKC && p.M % EPC_ != 0 && m0 + BM > p.M;
        const bool edge_b = !BKC && p.N % EPC_ != 0 && n0 + BN > p.N;
        const bool narrow = (edge_a && p.lda < 2 * EPC_) || (edge_b && p.ldb < 2 * EPC_);
        int n = (kend - k_done) / BK;
        if ((edge_a || edge_b) && k_done + n * BK == p.K) --n;
        if (narrow) n = 0;
        if (n > 0) {
            DirectLoader<T, BM, NW, AKC> la;
            DirectLoader<T, BN, NW, BKC> lb;
            la.init(A, p.lda, m0, p.M, k_done, wave, lane);
            lb.init(B, p.ldb, n0, p.N, k_done, wave, lane);
            // The slot numbers repeat every NSLOT tiles, so the loop over tiles is unrolled
            // NSLOT times with every LDS address a compile-time constant (operand fetches
            // become base register + immediate, M0 values one scalar add).  With one wave per
            // SIMD every instruction between two MFMAs competes for that wave's issue slots
            // (about eight per 32-cycle MFMA), so address arithmetic in the loop shows up as
            // idle matrix cores.  What is left over after whole groups of NSLOT tiles runs
            // with slot numbers computed at run time.
            const uint32_t wave_lds = (uint32_t)(uintptr_t)lds + wave * 1024;
            // Ring order: the operand called X here goes first (X(0) Y(0) X(1) Y(1) ...), is
            // prefetched two tiles ahead into the spare slot and so has the longer time to
            // land; Y follows one tile ahead.  Which operand should be X is a measured choice:
            // B first gains 4-13% for the binary16 256x256 and 64x64 tiles on data that does
            // not throttle the clock, and loses 1-2% for the 128x128 tile and for binary32.
            constexpr bool BF = sizeof(T) == 2 && BM != 128;
            constexpr int PA = BF ? 1 : 0, PB = 1 - PA;  // position of A and B in a tile's slot pair
            constexpr int NVX = BF ? NVB : NVA, NVY = BF ? NVA : NVB;  // loads per wave and slab
            auto x_issue = [&](GEMM_LDS(char) *dst, int q) { if constexpr (BF) lb.issue1(dst, wave, q); else la.issue1(dst, wave, q); };
            auto y_issue = [&](GEMM_LDS(char) *dst, int q) { if constexpr (BF) la.issue1(dst, wave, q); else lb.issue1(dst, wave, q); };
            auto x_advance = [&](bool more) { if constexpr (BF) lb.advance(more); else la.advance(more); };
            auto y_advance = [&](bool more) { if constexpr (BF) la.advance(more); else lb.advance(more); };
            // X(0) Y(0) X(1) Y(1); the loaders then point at tile 2 (or the last tile)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
#pragma unroll
                for (int q = 0; q < (h % 2 == 0 ? NVX : NVY); ++q) {
                    if (h % 2 == 0) x_issue(lds + h * SLOT, q);
                    else y_issue(lds + h * SLOT, q);
                }
                if (h % 2 == 0) x_advance(h / 2 + 1 < n);
                else y_advance(h / 2 + 1 < n);
            }
            if (safe) {
                full_sync();
            } else {
                __builtin_amdgcn_s_waitcnt(waitcnt_vm(NVA + NVB));  // tile 0 landed
                barrier_keep_loads();
            }

            trace_mark(p, 1);
            frag_t fa[2][FM], fb[2][FN];
            {
                const GEMM_LDS(char) *cA = lds + PA * SLOT, *cB = lds + PB * SLOT;
                fa[0][0] = Fetch<T, BM, AKC>::get(cA, wm * TM, 0, lane);
#pragma unroll
                for (int j = 0; j < FN; ++j) fb[0][j] = Fetch<T, BN, BKC>::get(cB, wn * TN + j * 32, 0, lane);
#pragma unroll
                for (int i = 1; i < FM; ++i) fa[0][i] = Fetch<T, BM, AKC>::get(cA, wm * TM + i * 32, 0, lane);
            }
            // The k-groups of one steady-state tile; cX.. are the slots of this and the next tile.
            auto tile_kgroups = [&](const GEMM_LDS(char) * cA, const GEMM_LDS(char) * cB, const GEMM_LDS(char) * nA,
                                    const GEMM_LDS(char) * nB, auto load_x_lo, auto load_x_hi, auto load_y,
                                    const bool more) {
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 1, true, load_x_lo, std::integral_constant<int, NVX / 2>());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 2, true, load_x_hi, std::integral_constant<int, NVX - NVX / 2>());
                x_advance(more);
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 3, true, no_load, L0());
                // tile t+1 landed (all but the youngest NVX loads), own reads of tile t done
                if (safe) {
                    full_sync();
                } else {
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(NVX));
                    barrier_keep_loads();
                }
                kgroup(fa[1], fb[1], fa[0], fb[0], nA, nB, 0, true, load_y, std::integral_constant<int, NVY>());
                y_advance(more);
                if (safe) full_sync();
            };
            // One steady-state tile whose slot pair starts at slot SA (compile time).
            auto tile_body = [&](auto sa_tag, const bool more) {
                constexpr int SA = decltype(sa_tag)::value;
                constexpr int O0 = ((SA + 0) % NSLOT) * SLOT, O1 = ((SA + 1) % NSLOT) * SLOT;
                constexpr int O2 = ((SA + 2) % NSLOT) * SLOT, O3 = ((SA + 3) % NSLOT) * SLOT;
                constexpr int O4 = ((SA + 4) % NSLOT) * SLOT;
                auto load_x_lo = [&](int q) {
                    if constexpr (BF) lb.template issue_at<O4>(wave_lds, q); else la.template issue_at<O4>(wave_lds, q);
                };
                auto load_x_hi = [&](int q) {
                    if constexpr (BF) lb.template issue_at<O4>(wave_lds, NVX / 2 + q); else la.template issue_at<O4>(wave_lds, NVX / 2 + q);
                };
                auto load_y = [&](int q) {
                    if constexpr (BF) la.template issue_at<O0>(wave_lds, q); else lb.template issue_at<O0>(wave_lds, q);
                };
                tile_kgroups(lds + (PA ? O1 : O0), lds + (PB ? O1 : O0), lds + (PA ? O3 : O2), lds + (PB ? O3 : O2),
                             load_x_lo, load_x_hi, load_y, more);
            };
            static_assert(NSLOT == 5, "the slot sequence below is 0 2 4 1 3");
            // Constant addresses for five slots cost address registers (one base per 64 KiB of
            // immediate-offset range and per lane pattern); the 8-wave tiles, with 128 vector
            // registers per wave, would spill them, so they keep run-time slot numbers throughout.
            constexpr bool CONST_SLOTS = NW <= 4;
            const int nbody = n - 1;  // tiles 0 .. n-2 run a tile body, tile n-1 has nothing to load
            int t = 0;
            // whole groups whose loaders all still advance (tile t + 4 fetches tile t + 6 < n)
            for (; CONST_SLOTS && t + NSLOT + 2 < n; t += NSLOT) {
                tile_body(std::integral_constant<int, 0>(), true);
                tile_body(std::integral_constant<int, 2>(), true);
                tile_body(std::integral_constant<int, 4>(), true);
                tile_body(std::integral_constant<int, 1>(), true);
                tile_body(std::integral_constant<int, 3>(), true);
            }
            // the remaining bodies and the last tile, slot numbers at run time
            int sa = 0;  // first slot of tile t's pair
            auto slot = [&](int d) -> GEMM_LDS(char) * {
                int x = sa + d;
                x = x >= NSLOT ? x - NSLOT : x;
                return lds + x * SLOT;
            };
            for (; t < nbody; ++t) {
                GEMM_LDS(char) *s0 = slot(0), *spare = slot(4);
                auto load_x_lo = [&](int q) { x_issue(spare, q); };
                auto load_x_hi = [&](int q) { x_issue(spare, NVX / 2 + q); };
                auto load_y = [&](int q) { y_issue(s0, q); };
                tile_kgroups(slot(PA), slot(PB), slot(2 + PA), slot(2 + PB), load_x_lo, load_x_hi, load_y, t + 3 < n);
                sa = sa + 2 >= NSLOT ? sa + 2 - NSLOT : sa + 2;
            }
            prefetch_leftover(k_done + n * BK);
            {
                const GEMM_LDS(char) *cA = slot(PA), *cB = slot(PB);
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 1, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 2, true, no_load, L0());
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 3, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 0, false, no_load, L0());
            }
            k_done += n * BK;
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));  // drain the redundant refills
        }
    }
    if (!ALIGNED) {
        // Operands the direct loads do not serve (2-byte aligned, or forced): full slabs go through registers into two LDS
        // buffers (the same image as the direct loads make).  Per slab s: k-groups 0,1 multiply;
        // k-group 2 also writes slab s+1 (in registers since an earlier slab) to the other
        // buffer; wait for the own LDS traffic, one barrier; k-group 3 also issues the global
        // loads of a later slab into the freed registers and fetches slab s+1's first operands.
        // Rows (or whole granules) past the M/N edge re-read a valid one as in the direct
        // path.  A granule of an M/N-contiguous operand that straddles the edge is read whole:
        // its tail is the padding or the start of the next k-row, lands in tile rows past the
        // edge and only feeds results that are never stored.  On the operand's last k-row
        // that tail could lie past the end of the operand, so a tile with such granules leaves
        // the slab that holds the last k-row to the guarded loop below, which also takes
        // leading dimensions shorter than two granules or too long for 32-bit offsets.
        constexpr int EPC = Elem<T>::EPC;
        const bool edge_a = !AKC && p.M % EPC != 0 && m0 + BM > p.M;
        const bool edge_b = !BKC && p.N % EPC != 0 && n0 + BN > p.N;
        const bool narrow = (edge_a && p.lda < 2 * EPC) || (edge_b && p.ldb < 2 * EPC);
        int n = (kend - k_done) / BK;
        if ((edge_a || edge_b) && k_done + n * BK == p.K) --n;
        if (n > 0 && p.ld32 && !narrow) {
            DirectLoader<T, BM, NW, AKC> la;
            DirectLoader<T, BN, NW, BKC> lb;
            la.init(A, p.lda, m0, p.M, k_done, wave, lane);
            lb.init(B, p.ldb, n0, p.N, k_done, wave, lane);
            // DEPTH register sets: slab s waits in set s % DEPTH from the k-group 3 that issued
            // its loads (DEPTH slabs earlier) to the k-group 2 that writes it to LDS.  The small
            // tiles multiply a slab in far less than a global-load round trip, so they keep
            // several slabs in flight; the 256x256 tiles have no registers to spare and keep one.
            constexpr int DEPTH = BM * BN <= 64 * 64 ? 4 : (BM * BN <= 128 * 128 ? 3 : 1);
            uint4_t ra[DEPTH][NVA], rb[DEPTH][NVB];
            auto fetch_set = [&](auto set_tag) {
                constexpr int S = decltype(set_tag)::value;
                return [&](int q) {
                    if (q < NVA) ra[S][q] = la.fetch1(q);
                    else rb[S][q - NVA] = lb.fetch1(q - NVA);
                };
            };
            GEMM_LDS(char) *wA = lds, *wB = lds + SLOT;  // where the registers go next
            auto store_set = [&](auto set_tag) {
                constexpr int S = decltype(set_tag)::value;
                return [&](int q) {
                    if (q < NVA) la.store1(wA, wave, lane, q, ra[S][q]);
                    else lb.store1(wB, wave, lane, q - NVA, rb[S][q - NVA]);
                };
            };
            typedef std::integral_constant<int, NVA + NVB> LAB;
            typedef std::integral_constant<int, 0> SET0;
            // slab 0 -> set 0 -> first LDS buffer; then slabs 1 .. DEPTH into sets 1 .. DEPTH-1, 0
            // (past the end of K the loaders stay on the last slab, re-fetched and never used)
#pragma unroll
            for (int q = 0; q < NVA + NVB; ++q) fetch_set(SET0())(q);
            la.advance(1 < n);
            lb.advance(1 < n);
#pragma unroll
            for (int q = 0; q < NVA + NVB; ++q) store_set(SET0())(q);
            auto prologue_fetch = [&](auto d_tag) {
                constexpr int D = decltype(d_tag)::value;
#pragma unroll
                for (int q = 0; q < NVA + NVB; ++q) fetch_set(std::integral_constant<int, D % DEPTH>())(q);
                la.advance(D + 1 < n);
                lb.advance(D + 1 < n);
            };
            prologue_fetch(std::integral_constant<int, 1>());
            if constexpr (DEPTH >= 2) prologue_fetch(std::integral_constant<int, 2>());
            if constexpr (DEPTH >= 3) prologue_fetch(std::integral_constant<int, 3>());
            if constexpr (DEPTH >= 4) prologue_fetch(std::integral_constant<int, 4>());
            static_assert(DEPTH <= 4, "prologue written for up to four register sets");
            __syncthreads();

            frag_t fa[2][FM], fb[2][FN];
            fa[0][0] = Fetch<T, BM, AKC>::get(lds, wm * TM, 0, lane);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[0][j] = Fetch<T, BN, BKC>::get(lds + SLOT, wn * TN + j * 32, 0, lane);
#pragma unroll
            for (int i = 1; i < FM; ++i) fa[0][i] = Fetch<T, BM, AKC>::get(lds, wm * TM + i * 32, 0, lane);
            int cur = 0;
            int sl = 0;
            // multiplies slab sl, moves slab sl+1 (register set SET) to LDS, refills the set with
            // slab sl+1+DEPTH
            auto slab_body = [&](auto set_tag) {
                const GEMM_LDS(char) *cA = lds + (2 * cur) * SLOT, *cB = cA + SLOT;
                wA = lds + (2 * (cur ^ 1)) * SLOT;
                wB = wA + SLOT;
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 1, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 2, true, no_load, L0());
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 3, true, store_set(set_tag), LAB());
                // own LDS writes and reads done; the loads issued below stay in flight
                if (safe) {
                    full_sync();
                } else {
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));
                    barrier_keep_loads();
                }
                kgroup(fa[1], fb[1], fa[0], fb[0], wA, wB, 0, true, fetch_set(set_tag), LAB());
                if (safe) full_sync();
                la.advance(sl + 2 + DEPTH < n);
                lb.advance(sl + 2 + DEPTH < n);
                cur ^= 1;
                ++sl;
            };
            // sl is a multiple of DEPTH at the top of the loop, so slab sl+1+d sits in set (1+d) % DEPTH
            while (sl + DEPTH <= n - 1) {
                slab_body(std::integral_constant<int, 1 % DEPTH>());
                if constexpr (DEPTH >= 2) slab_body(std::integral_constant<int, 2 % DEPTH>());
                if constexpr (DEPTH >= 3) slab_body(std::integral_constant<int, 3 % DEPTH>());
                if constexpr (DEPTH >= 4) slab_body(std::integral_constant<int, 4 % DEPTH>());
            }
            if constexpr (DEPTH >= 2) {
                const int rest = n - 1 - sl;  // 0 .. DEPTH-1 slabs still have a successor
                if (rest > 0) slab_body(std::integral_constant<int, 1 % DEPTH>());
                if (rest > 1) slab_body(std::integral_constant<int, 2 % DEPTH>());
                if constexpr (DEPTH >= 4) {
                    if (rest > 2) slab_body(std::integral_constant<int, 3 % DEPTH>());
                }
            }
            prefetch_leftover(k_done + n * BK);
            {
                const GEMM_LDS(char) *cA = lds + (2 * cur) * SLOT, *cB = cA + SLOT;
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 1, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 2, true, no_load, L0());
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 3, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 0, false, no_load, L0());
            }
            k_done += n * BK;
            // the redundant last refill is still in flight: it targets registers only
        }
    }
    // Remaining slabs (a ragged K tail; everything for the tiles excluded above): guarded
    // loads through registers into one LDS buffer; the loads of slab s+1 are issued before
    // slab s is multiplied and written to LDS after it.
    if (k_done < kend) {
        __syncthreads();  // LDS is free (direct-load pipeline drained, all reads done)
        if (!staged_ready) {
            guarded_fetch<T, BM, NT, AKC>(sa_, A, p.lda, m0, p.M, k_done, kend, tid);
            guarded_fetch<T, BN, NT, BKC>(sb_, B, p.ldb, n0, p.N, k_done, kend, tid);
        }
        staged_store<T, BM, NT, AKC>(lds, sa_, A, p.lda, m0, p.M, k_done, kend, tid);
        staged_store<T, BN, NT, BKC>(lds + SLOT, sb_, B, p.ldb, n0, p.N, k_done, kend, tid);
        __syncthreads();
        for (; k_done < kend; k_done += BK) {
            const bool more = k_done + BK < kend;
            pin_acc();
            if (more) {
                guarded_fetch<T, BM, NT, AKC>(sa_, A, p.lda, m0, p.M, k_done + BK, kend, tid);
                guarded_fetch<T, BN, NT, BKC>(sb_, B, p.ldb, n0, p.N, k_done + BK, kend, tid);
            }
            {
                // same fixed-order k-groups as the last tile of the direct-load pipeline
                frag_t fa[2][FM], fb[2][FN];
                const GEMM_LDS(char) *cA = lds, *cB = lds + SLOT;
                fa[0][0] = Fetch<T, BM, AKC>::get(cA, wm * TM, 0, lane);
#pragma unroll
                for (int j = 0; j < FN; ++j) fb[0][j] = Fetch<T, BN, BKC>::get(cB, wn * TN + j * 32, 0, lane);
#pragma unroll
                for (int i = 1; i < FM; ++i) fa[0][i] = Fetch<T, BM, AKC>::get(cA, wm * TM + i * 32, 0, lane);
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 1, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 2, true, no_load, L0());
                kgroup(fa[0], fb[0], fa[1], fb[1], cA, cB, 3, true, no_load, L0());
                kgroup(fa[1], fb[1], fa[0], fb[0], cA, cB, 0, false, no_load, L0());
            }
            if (more) {
                __syncthreads();  // everyone is done reading this slab
                staged_store<T, BM, NT, AKC>(lds, sa_, A, p.lda, m0, p.M, k_done + BK, kend, tid);
                staged_store<T, BN, NT, BKC>(lds + SLOT, sb_, B, p.ldb, n0, p.N, k_done + BK, kend, tid);
                __syncthreads();
            }
        }
    }

    trace_mark(p, 2);
    // marks 4 and 5 of the profiling trace: all stores of this thread issued / complete
    auto trace_stores = [&]() {
        if (p.trace != nullptr) {
            trace_mark(p, 4);
            __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
            trace_mark(p, 5);
        }
    };
    // epilogue: accumulator register r of lane l holds
    //   row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 block
    float *C = p.C + (int64_t)slice * p.split_stride;
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass of hipcc does not know the buffer builtins
    // Tiles that lie fully inside C, with rows of C on 16-byte boundaries (host flag): the store
    // goes through LDS (the paper's epilogue via shared memory, Section 3.2 "Epilog" and
    // Listing 5, with the operand buffers reused once they have drained), so that each lane
    // writes 16 contiguous bytes of a row and a store instruction covers whole 128-byte lines:
    // a quarter of the store instructions for binary32 C, an eighth for binary16 C.  Each wave
    // stages its own sub-tile, one band of 32 rows at a time, in a private piece of LDS, as
    // binary32 [32][TN + 8]: the 8 words of padding put the two rows a write instruction covers
    // (four apart) into different halves of the 64 banks.  LDS operations of one wave execute in
    // order, so the bands need no barrier between them.
    if (p.stage_c && m0 + BM <= p.M && n0 + BN <= p.N) {
        constexpr int SW = TN + 8;                 // staging row stride in words
        constexpr int STAGE = 32 * SW * 4;         // bytes per wave
        static_assert(NW * STAGE <= NBUF * SLOT, "staging area does not fit the operand buffers");
        __syncthreads();  // every wave has read its last operands, every direct load has landed
        trace_mark(p, 3);
        GEMM_LDS(float) *stage = (GEMM_LDS(float) *)(lds + wave * STAGE);
        const int lrow = 4 * (lane >> 5), lcol = lane & 31;
        const int esz = p.out16 ? 2 : 4;
        const int ldcb = (int)p.ldc * esz;
        char *cbase = p.out16 ? (char *)((_Float16 *)p.C + (int64_t)m0 * p.ldc + n0)
                              : (char *)(C + (int64_t)m0 * p.ldc + n0);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)cbase, 0, 0x7fffffff, 0x00020000);
        auto band = [&](auto out16_tag, auto policy) {
            constexpr bool O16 = decltype(out16_tag)::value;
            constexpr int POLICY = decltype(policy)::value;
            constexpr int WPL = O16 ? 8 : 4;          // staged words per lane and store (16 bytes of C)
            constexpr int LPR = TN / WPL;             // lanes per row
            constexpr int RPI = 64 / LPR;             // rows per store instruction
            static_assert(64 % LPR == 0 && 32 % RPI == 0, "wave tile width not supported by the staged store");
            const int srow = lane / LPR, spiece = lane % LPR;
            const int voff = (wm * TM + srow) * ldcb + (wn * TN) * (O16 ? 2 : 4) + spiece * 16;
#pragma unroll
            for (int i = 0; i < FM; ++i) {
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        stage[(8 * (r >> 2) + (r & 3) + lrow) * SW + j * 32 + lcol] = acc[i][j][r];
#pragma unroll
                for (int it = 0; it < 32 / RPI; ++it) {
                    const GEMM_LDS(float) *src = stage + (it * RPI + srow) * SW + spiece * WPL;
                    const int soff = (i * 32 + it * RPI) * ldcb;
                    if constexpr (O16) {
                        const float4_t lo = *(const GEMM_LDS(float4_t) *)src;
                        const float4_t hi = *(const GEMM_LDS(float4_t) *)(src + 4);
                        half8_t h;
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            h[x] = (_Float16)lo[x];
                            h[4 + x] = (_Float16)hi[x];
                        }
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4_t, h), rsrc, voff, soff, POLICY);
                    } else {
                        const float4_t v = *(const GEMM_LDS(float4_t) *)src;
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4_t, v), rsrc, voff, soff, POLICY);
                    }
                }
            }
        };
        if (p.out16) band(std::true_type(), std::integral_constant<int, 0>());
        else if (p.stream_c) band(std::false_type(), std::integral_constant<int, 2>());
        else band(std::false_type(), std::integral_constant<int, 0>());
        trace_stores();
        return;
    }
#endif
    trace_mark(p, 3);
    if (p.out16) {
        // binary16 result (never combined with K-slices: those reduce from binary32 partials)
        _Float16 *Ch = (_Float16 *)p.C;
#if defined(__HIP_DEVICE_COMPILE__)
        if (p.ldc < (int64_t(1) << 20)) {
            // same range-checked descriptor as the binary32 edge-tile stores below
            const int ldc2 = (int)p.ldc * 2;
            const int rows_valid = p.M - m0 < BM ? p.M - m0 : BM;
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc((void *)(Ch + (int64_t)m0 * p.ldc + n0), 0, rows_valid * ldc2, 0x00020000);
            const int voff = (wm * TM + 4 * (lane >> 5)) * ldc2 + (wn * TN + (lane & 31)) * 2;
            int voffj[FN];
#pragma unroll
            for (int j = 0; j < FN; ++j)
                voffj[j] = n0 + wn * TN + j * 32 + (lane & 31) < p.N ? voff + j * 64 : (int)0x80000000;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int roff = (i * 32 + 8 * (r >> 2) + (r & 3)) * ldc2;
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const _Float16 h = (_Float16)acc[i][j][r];
                        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, h), rsrc, voffj[j] + roff, 0, 0);
                    }
                }
            trace_stores();
            return;
        }
#endif
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = n0 + wn * TN + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int row = m0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if (row < p.M && col < p.N) Ch[(int64_t)row * p.ldc + col] = (_Float16)acc[i][j][r];
                }
            }
        }
        trace_stores();
        return;
    }
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass of hipcc does not know the buffer builtins
    // Tiles that lie fully inside C (and whose byte offsets fit 32 bits) store through a
    // buffer descriptor based at the tile origin: the per-lane part of the address is one
    // 32-bit register, the row (i, r) a scalar offset and the column block j an immediate,
    // so a store costs an accumulator read, a scalar multiply shared by FN stores, and the
    // store itself - no per-store 64-bit address arithmetic, compares or exec masking.
    if (m0 + BM <= p.M && n0 + BN <= p.N && p.ldc < (int64_t(1) << 20)) {
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void *)(C + (int64_t)m0 * p.ldc + n0), 0, 0x7fffffff, 0x00020000);
        const int ldc4 = (int)p.ldc * 4;
        const int voff = (wm * TM + 4 * (lane >> 5)) * ldc4 + (wn * TN + (lane & 31)) * 4;
        // C is written once and never read here.  When every 128-byte piece a store instruction
        // writes is a whole cache line (host flag) the stores carry the non-temporal hint, which
        // keeps the result from displacing A and B panels in the L2 (8192^3: 1-6 % faster);
        // on partial lines the hint costs 10 %, and K-slice partials are re-read at once.
        auto store_all = [&](auto policy) {
            constexpr int POLICY = decltype(policy)::value;  // cache-policy operand: bit 1 = nt
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int soff = (i * 32 + 8 * (r >> 2) + (r & 3)) * ldc4;
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        // through a scalar temporary: a bit cast applied directly to a vector
                        // element expression reads element 0 with this compiler
                        const float v = acc[i][j][r];
                        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc, voff + j * 128, soff, POLICY);
                    }
                }
        };
        if (p.stream_c) store_all(std::integral_constant<int, 2>());
        else store_all(std::integral_constant<int, 0>());
        trace_stores();
        return;
    }
    // Edge tiles, same descriptor trick: the descriptor's range ends with the last valid row
    // (out-of-range buffer stores are discarded by the hardware) and lanes whose column is
    // past N get an offset that is out of range by itself.  The row offset goes into the
    // vector offset here, because the range check does not look at the scalar offset.
    if (p.ldc < (int64_t(1) << 20)) {
        const int ldc4 = (int)p.ldc * 4;
        const int rows_valid = p.M - m0 < BM ? p.M - m0 : BM;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void *)(C + (int64_t)m0 * p.ldc + n0), 0, rows_valid * ldc4, 0x00020000);
        const int voff = (wm * TM + 4 * (lane >> 5)) * ldc4 + (wn * TN + (lane & 31)) * 4;
        int voffj[FN];
#pragma unroll
        for (int j = 0; j < FN; ++j)
            voffj[j] = n0 + wn * TN + j * 32 + (lane & 31) < p.N ? voff + j * 128 : (int)0x80000000;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int roff = (i * 32 + 8 * (r >> 2) + (r & 3)) * ldc4;
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const float v = acc[i][j][r];
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), rsrc, voffj[j] + roff, 0, 0);
                }
            }
        trace_stores();
        return;
    }
#endif
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
    trace_stores();
}

}  // namespace gemm_gfx950
