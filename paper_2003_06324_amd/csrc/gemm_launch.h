// Host-side launcher shared by the per-tile instantiation files: maps the
// run-time (layout, alignment) choice onto the kernel template's booleans.
#pragma once
#include "gemm_kernel.h"
#include "gemm_ksplit_kernel.h"

#include <tuple>
#include <utility>

namespace gemm_gfx950 {

template <typename Tuple, size_t... I>
static void fill_argv(void **argv, Tuple &vals, std::index_sequence<I...>)
{
    ((argv[I] = (void *)&std::get<I>(vals)), ...);
}

// Enqueues one kernel and returns the status of this launch alone (an error some earlier,
// unrelated runtime call left pending in the calling thread is not picked up, unlike with
// hipGetLastError after a <<<>>> launch).
template <typename... Params, typename... Args>
static hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t s, Args... args)
{
    std::tuple<Params...> vals(args...);
    void *argv[sizeof...(Params)];
    fill_argv(argv, vals, std::index_sequence_for<Params...>());
    return hipLaunchKernel((const void *)kernel, grid, block, argv, 0, s);
}

template <typename T, int BM, int BN, int WM, int WN, bool AKC, bool BKC>
static hipError_t launch_aligned(bool aligned, dim3 grid, hipStream_t s, const KernelArgs &a)
{
    const dim3 block(WM * WN * 64);
    if (aligned) return launch_kernel(gemm_tile_kernel<T, BM, BN, WM, WN, AKC, BKC, true>, grid, block, s, a);
    return launch_kernel(gemm_tile_kernel<T, BM, BN, WM, WN, AKC, BKC, false>, grid, block, s, a);
}

// akc: A is K-contiguous (row-major); bkc: B is K-contiguous (column-major)
template <typename T, int BM, int BN, int WM, int WN>
hipError_t launch_tile(bool akc, bool bkc, bool aligned, dim3 grid, hipStream_t s, const KernelArgs &a)
{
    if (akc && bkc) return launch_aligned<T, BM, BN, WM, WN, true, true>(aligned, grid, s, a);
    if (akc && !bkc) return launch_aligned<T, BM, BN, WM, WN, true, false>(aligned, grid, s, a);
    if (!akc && bkc) return launch_aligned<T, BM, BN, WM, WN, false, true>(aligned, grid, s, a);
    return launch_aligned<T, BM, BN, WM, WN, false, false>(aligned, grid, s, a);
}

// K split across the waves of the workgroup; the caller passes operands the direct loads serve and a K
// that is a multiple of the slab (`aligned` is part of the common signature and always true here)
template <typename T, int BM, int BN>
hipError_t launch_ksplit(bool akc, bool bkc, bool aligned, dim3 grid, hipStream_t s, const KernelArgs &a)
{
    (void)aligned;
    const dim3 block(256);
    if (akc && bkc) return launch_kernel(gemm_ksplit_kernel<T, BM, BN, true, true>, grid, block, s, a);
    if (akc && !bkc) return launch_kernel(gemm_ksplit_kernel<T, BM, BN, true, false>, grid, block, s, a);
    if (!akc && bkc) return launch_kernel(gemm_ksplit_kernel<T, BM, BN, false, true>, grid, block, s, a);
    return launch_kernel(gemm_ksplit_kernel<T, BM, BN, false, false>, grid, block, s, a);
}

typedef hipError_t (*launch_fn)(bool, bool, bool, dim3, hipStream_t, const KernelArgs &);

#define GEMM_DECLARE_TILE(T, BM, BN, WM, WN) \
    extern template hipError_t launch_tile<T, BM, BN, WM, WN>(bool, bool, bool, dim3, hipStream_t, const KernelArgs &);
#define GEMM_INSTANTIATE_TILE(T, BM, BN, WM, WN) \
    template hipError_t launch_tile<T, BM, BN, WM, WN>(bool, bool, bool, dim3, hipStream_t, const KernelArgs &);
#define GEMM_DECLARE_KSPLIT(T, BM, BN) \
    extern template hipError_t launch_ksplit<T, BM, BN>(bool, bool, bool, dim3, hipStream_t, const KernelArgs &);
#define GEMM_INSTANTIATE_KSPLIT(T, BM, BN) \
    template hipError_t launch_ksplit<T, BM, BN>(bool, bool, bool, dim3, hipStream_t, const KernelArgs &);

}  // namespace gemm_gfx950
