// Stand-alone measurement behind the activation layout of the stream and team kernels: how long a compute
// unit takes per 16-byte-per-lane buffer load (one KiB per wave) for the access patterns a matrix-core operand
// can have, with 512 threads on every compute unit as in those kernels.  Build and run:
//   python -m paper_2306_17266_amd.build --tools && paper_2306_17266_amd/vmem_patterns
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, long bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x27000);
}
template <int AUX, int PATTERN>
__global__ __launch_bounds__(512, 2) void k(const char *buf, long per_wg, int iters, unsigned *out, long long *clk) {
    const char *base = buf + (long)blockIdx.x * per_wg;
    const __amdgpu_buffer_rsrc_t r = make_rsrc(base, per_wg);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // PATTERN 0: a wave reads 1 KiB contiguous.  1: 16 rows of 64 B, 176 B apart (operand order of a 3x3 conv, C = 88)
    // 2: the same rows with four neighbouring lanes on one row
    int off;
    if (PATTERN == 0) off = wave * 8192 + lane * 16;
    else if (PATTERN == 1) off = wave * 8192 + (lane & 15) * 176 + (lane >> 4) * 16;
    else off = wave * 8192 + (lane >> 2) * 176 + (lane & 3) * 16;
    u32x4_t acc = {0, 0, 0, 0};
    const long long t0 = clock64();
    const int span = (int)(per_wg / 8) - 4096;  // bytes a wave walks through
    int walk = 0;
    for (int it = 0; it < iters; ++it) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_amdgcn_raw_buffer_load_b128(r, off + walk + u * 1024 * (PATTERN == 0 ? 1 : 3), 0, AUX);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
        walk += 8 * 1024 * (PATTERN == 0 ? 1 : 3);
        if (walk + 8 * 1024 * 3 + 4096 > span) walk = 0;
    }
    const long long t1 = clock64();
    if (acc.x == 0x12345678u) out[0] = acc.y;
    if (tid == 0) clk[blockIdx.x] = t1 - t0;
}
template <int AUX, int PATTERN>
int run(const char *name, const char *buf, long per_wg, unsigned *out, long long *clk) {
    const int iters = 2000;
    for (int rep = 0; rep < 2; ++rep) {
        hipLaunchKernelGGL((k<AUX, PATTERN>), dim3(256), dim3(512), 0, 0, buf, per_wg, iters, out, clk);
        CK(hipDeviceSynchronize());
    }
    long long h[256];
    CK(hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost));
    double mean = 0; for (int i = 0; i < 256; ++i) mean += h[i] / 256.0;
    const double loads = (double)iters * 8 * 8;  // wave loads per CU
    printf("%-40s per_wg %6ld KiB: %7.1f clocks per wave load, %5.1f B/clock per CU\n", name, per_wg >> 10, mean / loads, loads * 1024 / mean);
    return 0;
}
int main() {
    char *buf; unsigned *out; long long *clk;
    const long total = 256L << 20;
    CK(hipMalloc((void **)&buf, total)); CK(hipMemset(buf, 1, total));
    CK(hipMalloc((void **)&out, 64)); CK(hipMalloc((void **)&clk, 256 * 8));
    for (long per_wg : {16L << 10 << 3, 1L << 20}) {  // 128 KiB per WG (beyond the L1), 1 MiB per WG (256 MiB in all: beyond the L2s)
        run<0, 0>("plain, contiguous", buf, per_wg, out, clk);
        run<16, 0>("sc1, contiguous", buf, per_wg, out, clk);
        run<0, 1>("plain, operand order of 16 pixels", buf, per_wg, out, clk);
        run<16, 1>("sc1, operand order of 16 pixels", buf, per_wg, out, clk);
        run<16, 2>("sc1, four lanes per pixel", buf, per_wg, out, clk);
    }
    return 0;
}
