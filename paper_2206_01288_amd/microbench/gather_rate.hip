// Gather-rate microbenchmark for gfx950: how fast a CU serves the gathers of the general matching kernel. Every
// wavefront reads ROWS rows of a block the way k_match does: row r of the table (wavefront-uniform, as if it were the
// device of the block's row r) at 64 per-lane columns (the devices of the block's columns), entries of 2 or 4
// bytes, table of 1024 x 1024 entries; the columns are random, sorted, or the 64 consecutive ones. The sum of what
// was read is stored so that nothing is optimised away. Prints the time per launch and the cycles (at 2.4 GHz) a
// CU spends per 64-lane gather.
// Built and run by `python -m paper_2206_01288_amd.microbench`; its output backs the gather rate quoted in the
// design notes.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <stdlib.h>

#define N 1024
#define ROWS 64

template <typename T>
__global__ void k_gather(const T *__restrict__ tab, const int32_t *__restrict__ rows, const int32_t *__restrict__ cols,
                         uint32_t *__restrict__ out)
{
    const size_t wave = blockIdx.x;   // one wavefront per workgroup, as in k_match
    const int32_t *rr = rows + wave * ROWS;
    const uint32_t col = (uint32_t)cols[wave * 64 + threadIdx.x];
    uint32_t e[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; r++) e[r] = tab[(uint32_t)rr[r] * N + col];
    uint32_t m = 0xffffffffu;
#pragma unroll
    for (int r = 0; r < ROWS; r++) m = min(m, e[r]);
    out[wave * 64 + threadIdx.x] = m;
}

template <typename T>
static void run(const char *name, const char *order, const T *tab, const int32_t *rows, const int32_t *cols, uint32_t *out,
                int waves)
{
    hipEvent_t s, e;
    hipEventCreate(&s);
    hipEventCreate(&e);
    for (int i = 0; i < 3; i++) hipLaunchKernelGGL(k_gather<T>, dim3(waves), dim3(64), 0, 0, tab, rows, cols, out);
    hipDeviceSynchronize();
    hipEventRecord(s);
    const int reps = 10;
    for (int i = 0; i < reps; i++) hipLaunchKernelGGL(k_gather<T>, dim3(waves), dim3(64), 0, 0, tab, rows, cols, out);
    hipEventRecord(e);
    hipDeviceSynchronize();
    float ms;
    hipEventElapsedTime(&ms, s, e);
    ms /= reps;
    const double gathers_per_cu = (double)waves * ROWS / 256.0;
    printf("%-4s %-10s: %8.1f us/launch, %5.1f cycles per 64-lane gather and CU, %4.2f lanes per cycle and CU\n", name, order,
           ms * 1e3, ms * 1e-3 * 2.4e9 / gathers_per_cu, 64.0 / (ms * 1e-3 * 2.4e9 / gathers_per_cu));
    fflush(stdout);
}

static int cmp_i32(const void *a, const void *b) { return *(const int32_t *)a - *(const int32_t *)b; }

int main()
{
    const int waves = 4096 * 120;   // the blocks of one evaluation of 4096 candidates with 16 stages
    uint16_t *t16;
    uint32_t *t32, *out;
    int32_t *rows, *cols[3];
    hipMalloc(&t16, (size_t)N * N * 2);
    hipMalloc(&t32, (size_t)N * N * 4);
    hipMalloc(&out, (size_t)waves * 64 * 4);
    hipMalloc(&rows, (size_t)waves * ROWS * 4);
    for (int i = 0; i < 3; i++) hipMalloc(&cols[i], (size_t)waves * 64 * 4);
    hipMemset(t16, 1, (size_t)N * N * 2);
    hipMemset(t32, 1, (size_t)N * N * 4);
    int32_t *h = (int32_t *)malloc((size_t)waves * 64 * 4);
    uint64_t st = 88172645463325252ull;
    auto rnd = [&]() { st ^= st << 13; st ^= st >> 7; st ^= st << 17; return (uint32_t)(st >> 20); };
    for (size_t i = 0; i < (size_t)waves * ROWS; i++) h[i] = (int32_t)(rnd() % N);
    hipMemcpy(rows, h, (size_t)waves * ROWS * 4, hipMemcpyHostToDevice);
    for (size_t i = 0; i < (size_t)waves * 64; i++) h[i] = (int32_t)(rnd() % N);
    hipMemcpy(cols[0], h, (size_t)waves * 64 * 4, hipMemcpyHostToDevice);
    for (int w = 0; w < waves; w++) qsort(h + (size_t)w * 64, 64, 4, cmp_i32);
    hipMemcpy(cols[1], h, (size_t)waves * 64 * 4, hipMemcpyHostToDevice);
    for (int w = 0; w < waves; w++) {
        const int32_t first = h[(size_t)w * 64] % (N - 64);
        for (int c = 0; c < 64; c++) h[(size_t)w * 64 + c] = first + c;
    }
    hipMemcpy(cols[2], h, (size_t)waves * 64 * 4, hipMemcpyHostToDevice);
    const char *order[3] = {"random", "sorted", "contiguous"};
    for (int i = 0; i < 3; i++) {
        run<uint16_t>("u16", order[i], t16, rows, cols[i], out, waves);
        run<uint32_t>("u32", order[i], t32, rows, cols[i], out, waves);
    }
    free(h);
    return 0;
}
