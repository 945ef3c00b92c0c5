// Issue-rate microbenchmark for gfx950: how fast one SIMD issues dependent and independent chains of the
// instruction kinds the fused kernels are made of (packed 16-bit max/min, fp64 add/min, 32-bit integer ops,
// data-parallel lane moves, ds_swizzle), with one and two wavefronts per SIMD. Every workgroup runs the same
// straight-line loop; the cycle counter of one wavefront brackets ITER x 8 x CH x 2 instructions.
// Built and run by `python -m paper_2206_01288_amd.microbench`; its output backs the issue rates quoted in the
// design notes (they bound what straight-line code can reach; the roofline peak does not depend on them).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <math.h>
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b)
{ return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b))); }
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b)
{ return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b))); }

#define ITER 256
// KIND 0: pk max/min alternating, CH independent chains; 1: f64 add/min; 2: dpp mov (32-bit) chains; 3: u32 add
template <int KIND, int CH>
__global__ void k(uint32_t *out, uint64_t *cycles, uint32_t seed)
{
    uint32_t a[CH];
    double d[CH];
    for (int i = 0; i < CH; i++) { a[i] = seed * (threadIdx.x + 7 + i); d[i] = (double)a[i] * 1e-3; }
    uint32_t b = seed ^ 0x12345678u, c = seed * 3u;
    double e = (double)seed * 0.37;
    __syncthreads();
    uint64_t t0 = __builtin_readcyclecounter();
    for (int it = 0; it < ITER; it++) {
#pragma unroll
        for (int u = 0; u < 8; u++) {
#pragma unroll
            for (int i = 0; i < CH; i++) {
                if (KIND == 0) { a[i] = pk_max(a[i], b); a[i] = pk_min(a[i], c); }
                if (KIND == 1) { d[i] = d[i] + e; d[i] = fmin(d[i], 1e300); }
                if (KIND == 2) { a[i] = __builtin_amdgcn_update_dpp(0, a[i], 0xB1, 0xF, 0xF, true); a[i] = __builtin_amdgcn_update_dpp(0, a[i], 0x4E, 0xF, 0xF, true); }
                if (KIND == 3) { a[i] = a[i] + b; a[i] = a[i] ^ c; }
                if (KIND == 4) { a[i] = __builtin_amdgcn_ds_swizzle(a[i], 0x1F | (4 << 10)); a[i] = __builtin_amdgcn_ds_swizzle(a[i], 0x1F | (2 << 10)); }
            }
        }
        asm volatile("" ::: "memory");
    }
    uint64_t t1 = __builtin_readcyclecounter();
    uint32_t r = 0;
    for (int i = 0; i < CH; i++) r ^= a[i] ^ (uint32_t)d[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (threadIdx.x == 0 && blockIdx.x == 0) *cycles = t1 - t0;
}
template <int KIND, int CH>
void run(const char *name, int waves_per_simd, uint32_t *out, uint64_t *cyc)
{
    int threads = 64 * 4 * waves_per_simd;
    hipEvent_t s, e; hipEventCreate(&s); hipEventCreate(&e);
    hipLaunchKernelGGL((k<KIND, CH>), dim3(256), dim3(threads), 0, 0, out, cyc, 12345u);
    hipDeviceSynchronize();
    hipEventRecord(s);
    for (int i = 0; i < 20; i++) hipLaunchKernelGGL((k<KIND, CH>), dim3(256), dim3(threads), 0, 0, out, cyc, 12345u);
    hipEventRecord(e); hipDeviceSynchronize();
    float ms; hipEventElapsedTime(&ms, s, e); ms /= 20;
    uint64_t c; hipMemcpy(&c, cyc, 8, hipMemcpyDeviceToHost);
    double instr = (double)ITER * 8 * CH * 2;
    printf("%-10s chains=%d waves/SIMD=%d: %.1f us/launch, %.2f ns per instr per wave, counter %.2f ticks/instr\n", name, CH, waves_per_simd,
           ms * 1e3, ms * 1e6 / instr, (double)c / instr);
    fflush(stdout);
}
int main()
{
    uint32_t *out; uint64_t *cyc;
    hipMalloc(&out, 256 * 1024 * 4); hipMalloc(&cyc, 8);
    for (int w = 1; w <= 2; w++) {
        run<0, 1>("pk16", w, out, cyc); run<0, 2>("pk16", w, out, cyc); run<0, 4>("pk16", w, out, cyc);
        run<1, 1>("f64", w, out, cyc); run<1, 2>("f64", w, out, cyc); run<1, 4>("f64", w, out, cyc);
        run<2, 1>("dpp", w, out, cyc); run<2, 2>("dpp", w, out, cyc); run<2, 4>("dpp", w, out, cyc);
        run<3, 1>("u32", w, out, cyc); run<3, 4>("u32", w, out, cyc);
        run<4, 1>("swizzle", w, out, cyc); run<4, 4>("swizzle", w, out, cyc);
    }
    return 0;
}
