// Register-only MFMA loop: what the matrix cores sustain on this part when nothing else runs.
//
//   hipcc -O3 --offload-arch=gfx950 -o mfma_ceiling paper_2003_06324_amd/probes/mfma_ceiling.hip
//   ./mfma_ceiling r      (operands ~N(0,1) rounded to binary16)
//   ./mfma_ceiling z      (all-zero operands)
//
// Every wave of every CU issues back-to-back independent v_mfma_f32_32x32x16_f16 (12 accumulators,
// 4 A x 3 B fragments held in registers, no memory traffic in the loop), one workgroup of four
// waves per CU, for about four seconds; socket power and XCD clocks are sampled with amd-smi
// half-way.  On random operands the part throttles itself far below the 2.4 GHz datasheet rate,
// which is the ceiling any FP16 GEMM on such data has on this part.
#include <hip/hip_runtime.h>
#include <chrono>
#include <cstdio>
#include <cstdlib>
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_loop(const half8_t *in, float *out, int iters)
{
    half8_t a[4], b[3];
    for (int i = 0; i < 4; ++i) a[i] = in[(threadIdx.x + 64 * i) & 1023];
    for (int i = 0; i < 3; ++i) b[i] = in[(threadIdx.x + 64 * i + 256) & 1023];
    float16_t acc[4][3];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 3; ++j)
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
                asm volatile("" : "+a"(acc[i][j]));  // keeps the accumulators where they are
            }
    }
    float s = 0;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 3; ++j)
            for (int r = 0; r < 16; ++r) s += acc[i][j][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main(int argc, char **argv)
{
    const bool zeros = argc > 1 && argv[1][0] == 'z';
    half8_t *in;
    float *out;
    CHECK(hipMalloc(&in, 1024 * sizeof(half8_t)));
    CHECK(hipMalloc(&out, 256 * 256 * sizeof(float)));
    static _Float16 h[8192];
    srand(1);
    for (int i = 0; i < 8192; ++i) {
        float s = 0;  // sum of 12 uniforms - 6: close to N(0,1)
        for (int t = 0; t < 12; ++t) s += rand() / (float)RAND_MAX;
        h[i] = zeros ? (_Float16)0.0f : (_Float16)(s - 6.0f);
    }
    CHECK(hipMemcpy(in, h, sizeof h, hipMemcpyHostToDevice));
    const int iters = 4000, grid = 256;
    const double flop = (double)grid * 4 * iters * 12 * 32768.0;  // per launch
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 3; ++w) mfma_loop<<<grid, 256>>>(in, out, iters);
    CHECK(hipDeviceSynchronize());
    const auto t0 = std::chrono::steady_clock::now();
    int n = 0;
    double gpu_ms = 0;
    bool sampled = false;
    while (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < 4.0) {
        CHECK(hipEventRecord(e0));
        for (int w = 0; w < 20; ++w) mfma_loop<<<grid, 256>>>(in, out, iters);
        CHECK(hipEventRecord(e1));
        if (!sampled && std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > 2.0) {
            sampled = true;  // the launches above are still running while this samples
            fflush(stdout);
            if (system("amd-smi metric -p -c --json | python3 -c \"import json,sys; g=json.load(sys.stdin)['gpu_data'][0]; "
                       "c=[v['clk']['value'] for k,v in g['clock'].items() if k.startswith('gfx_')]; "
                       "print('socket power', g['power']['socket_power']['value'], 'W, mean XCD clock %.0f MHz' % (sum(c)/len(c)))\"") != 0)
                printf("(amd-smi not usable here)\n");
        }
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        gpu_ms += ms;
        n += 20;
    }
    printf("%s operands, v_mfma_f32_32x32x16_f16 only: %.1f TFLOP/s sustained\n", zeros ? "zero" : "random",
           flop * n / gpu_ms / 1e9);
    return 0;
}
