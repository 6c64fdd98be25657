// Stand-alone microbenchmark, not part of the library: the rate of direct global->LDS loads
// (buffer_load_dwordx4 ... lds, the loads gemm_tile_kernel stages its operands with) per workgroup as a
// function of the waves that issue them, the loads each wave keeps in flight, the access pattern (1 KB
// contiguous per instruction, or 8 rows of 128 bytes as for a K-contiguous operand tile) and where the data
// comes from (a footprint the XCDs' L2s hold, one the memory-side cache holds, one only HBM holds).
// No LDS reads, no barriers, every workgroup streams a region of its own.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Wno-unused-value paper_2003_06324_amd/probes/dma_rate.hip -o /tmp/dma_rate && /tmp/dma_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef int int4_t __attribute__((ext_vector_type(4)));
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

template <int NW, int D, bool ROWS>
__global__ __launch_bounds__(NW * 64) void dma_kernel(const char *base, size_t per_wg, int iters, int ld)
{
    __shared__ __attribute__((aligned(1024))) char smem[NW * 16 * 1024];   // 16 KB ring per wave
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const char *mine = base + (size_t)blockIdx.x * per_wg;
    // one load instruction = 1 KB: contiguous, or 8 rows of 128 B at stride ld (a K-contiguous operand tile)
    // ROWS: the region is a matrix of rows of ld bytes; an instruction takes 128 bytes of 8 consecutive rows,
    // the next one the next 128 bytes of the same rows, and so on to the end of the rows
    const int voff = ROWS ? (lane >> 3) * ld + (lane & 7) * 16 : lane * 16;
    const size_t nchunks = per_wg / 1024 / NW;                  // instructions per wave and pass over the region
    const int per_row = ld / 128;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)mine, 0, 0x7fffffff, 0x00020000);
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem + wave * 16 * 1024;
    size_t c = 0;
    for (int it = 0; it < iters; ++it) {
        const size_t i = c * NW + wave;
        const uint32_t soff = ROWS ? (uint32_t)((i / per_row) * 8 * (size_t)ld + (i % per_row) * 128) : (uint32_t)(i * 1024);
        const uint32_t lds_addr = lds0 + (it & 15) * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                     : : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(D - 1));
        c = c + 1 < nchunks ? c + 1 : 0;
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
}

template <int NW, int D, bool ROWS> float run(const char *buf, size_t per_wg, int wgs, int iters, int ld)
{
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    for (int w = 0; w < 2; ++w) dma_kernel<NW, D, ROWS><<<wgs, NW * 64>>>(buf, per_wg, iters, ld);
    hipEventRecord(e0);
    dma_kernel<NW, D, ROWS><<<wgs, NW * 64>>>(buf, per_wg, iters, ld);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    if (hipGetLastError() != hipSuccess) { printf("launch error\n"); exit(1); }
    return ms;
}

template <int NW, bool ROWS> void sweep(const char *buf, size_t per_wg, int wgs, const char *what)
{
    const int iters = 4096 / NW * 4;
    const int ld = 8192;
    float ms[7];
    ms[0] = run<NW, 1, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[1] = run<NW, 2, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[2] = run<NW, 4, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[3] = run<NW, 8, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[4] = run<NW, 16, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[5] = run<NW, 32, ROWS>(buf, per_wg, wgs, iters, ld);
    ms[6] = run<NW, 60, ROWS>(buf, per_wg, wgs, iters, ld);
    printf("%-28s %s waves %d wgs %4d | GB/s per workgroup at 1,2,4,8,16,32,60 loads in flight per wave:", what, ROWS ? "rows " : "contig", NW, wgs);
    for (int i = 0; i < 7; ++i) printf(" %6.1f", (double)iters * NW * 1024 / (ms[i] * 1e-3) / 1e9);
    printf("\n"); fflush(stdout);
}

int main()
{
    const size_t total = (size_t)6 << 30;
    char *buf; if (hipMalloc(&buf, total) != hipSuccess) { printf("alloc failed\n"); return 1; }
    hipMemset(buf, 1, total); hipDeviceSynchronize();
    // footprint per workgroup: 256 KB (stays in the XCD's L2 with 32 workgroups per XCD: 8 MB > 4 MB... use 96 KB), 4 MB (memory-side cache), 16 MB (HBM)
    struct { size_t per; const char *what; } fp[] = {{(size_t)96 << 10, "96 KB/wg (L2)"}, {(size_t)768 << 10, "768 KB/wg (192 MB: MALL)"}, {(size_t)16 << 20, "16 MB/wg (4 GB: HBM)"}};
    for (auto &f : fp) {
        sweep<1, false>(buf, f.per, 256, f.what);
        sweep<4, false>(buf, f.per, 256, f.what);
        sweep<8, false>(buf, f.per, 256, f.what);
        sweep<4, true>(buf, f.per, 256, f.what);
    }
    // fewer busy CUs
    sweep<4, false>(buf, (size_t)768 << 10, 32, "768 KB/wg, 32 wgs");
    sweep<4, false>(buf, (size_t)16 << 20, 32, "16 MB/wg, 32 wgs");
    // two workgroups per CU
    sweep<4, false>(buf, (size_t)768 << 10, 512, "768 KB/wg, 512 wgs");
    return 0;
}
