// Stand-alone microbenchmark, not part of the library: streaming from the XCDs' L2s into LDS by the two ways the
// kernels stage operands -- direct global->LDS loads (buffer_load_dwordx4 ... lds), loads into registers followed
// by ds_write_b128 -- and both interleaved; 4 or 8 waves per workgroup, one workgroup per CU, loads issued in
// groups of 4 or 8 per wave with one wait per group.  Every workgroup reads 96 KB regions in rotation with the 31
// other workgroups of its XCD, so the data stays in that XCD's L2 and no line is seen twice by an L1.
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Wno-unused-value paper_2003_06324_amd/probes/load_paths.hip -o /tmp/load_paths && /tmp/load_paths
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef int int4_t __attribute__((ext_vector_type(4)));
#define LDSP(T) __attribute__((address_space(3))) T
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }
// MODE 0: D direct loads per iteration; 1: D register loads + writes; 2: D of each
template <int NW, int D, int MODE>
__global__ __launch_bounds__(NW * 64) void k(const char *base, size_t per_wg, int iters)
{
    __shared__ __attribute__((aligned(1024))) char smem[NW * 16 * 1024];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, 0x7fffffff, 0x00020000);
    // a pass over one region, then the region of the workgroup 8 further on (same XCD, so its L2 holds it; the L1 never sees a line twice)
    int region = blockIdx.x;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem + wave * 16 * 1024;
    LDSP(char) *lds = (LDSP(char) *)smem + wave * 16 * 1024;
    const int voff = lane * 16;
    const size_t nchunks = per_wg / 1024 / NW;
    size_t c = 0;
    for (int it = 0; it < iters; ++it) {
        int4_t r[D];
        if (MODE != 1) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const uint32_t soff = (uint32_t)((size_t)region * per_wg + (c * NW + wave) * 1024);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                             : : "s"(lds0 + d * 1024), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
                if (++c == nchunks) { c = 0; region = (region + 8) & 255; }
            }
        }
        if (MODE != 0) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                r[d] = *(const int4_t *)(base + (size_t)region * per_wg + (c * NW + wave) * 1024 + voff);
                if (++c == nchunks) { c = 0; region = (region + 8) & 255; }
            }
#pragma unroll
            for (int d = 0; d < D; ++d) *(LDSP(int4_t) *)(lds + (8 + d % 8) * 1024 + lane * 16) = r[d];
        }
        if (MODE == 0) __builtin_amdgcn_s_waitcnt(waitcnt_vm(D));   // previous iteration's loads done
    }
    __builtin_amdgcn_s_waitcnt(0x0070);
}
template <int NW, int D, int MODE> void run(const char *buf, size_t per_wg, const char *what)
{
    const int iters = 16384 / NW / D;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    for (int w = 0; w < 2; ++w) k<NW, D, MODE><<<256, NW * 64>>>(buf, per_wg, iters);
    hipEventRecord(e0);
    k<NW, D, MODE><<<256, NW * 64>>>(buf, per_wg, iters);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    const double kb = (double)iters * NW * D * (MODE == 2 ? 2 : 1);
    printf("%s waves %d, %d loads per iteration%s: %.1f GB/s per workgroup\n", what, NW, D, MODE == 2 ? " of each kind" : "", kb * 1024 / (ms * 1e-3) / 1e9);
    fflush(stdout);
}
int main()
{
    const size_t total = (size_t)256 << 20;
    char *buf; if (hipMalloc(&buf, total) != hipSuccess) return 1;
    hipMemset(buf, 1, total); hipDeviceSynchronize();
    const size_t per = (size_t)96 << 10;
    run<4, 4, 0>(buf, per, "direct   "); run<4, 8, 0>(buf, per, "direct   ");
    run<4, 4, 1>(buf, per, "registers"); run<4, 8, 1>(buf, per, "registers");
    run<4, 4, 2>(buf, per, "both     "); run<4, 8, 2>(buf, per, "both     ");
    run<8, 4, 0>(buf, per, "direct   "); run<8, 4, 1>(buf, per, "registers"); run<8, 4, 2>(buf, per, "both     ");
    return 0;
}
