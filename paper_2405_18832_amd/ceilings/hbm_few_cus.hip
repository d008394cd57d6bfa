// HBM streaming rate per CU when only S CUs stream (one block per CU): W wavefronts per block, each keeping
// PF loads of 1 KiB (16 B per lane) in flight over its own contiguous region.  Shows what a few CUs set aside
// for weight streaming could deliver while the others do matrix work.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
template <int PF>
__global__ __launch_bounds__(1024) void k(const uint4* __restrict__ src, uint4* out, long per_wave_vec, int chunk_steps) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, W = blockDim.x >> 6;
    const uint4* p = src + ((size_t)blockIdx.x * W + wave) * per_wave_vec + lane;
    const long steps = per_wave_vec / 64;
    uint4 acc = make_uint4(0, 0, 0, 0);
    uint4 v[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) v[i] = p[(long)i * 64];
    long s = 0;
    for (; s + 2 * PF <= steps; s += PF) {
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            acc.x ^= v[i].x; acc.y ^= v[i].y; acc.z ^= v[i].z; acc.w ^= v[i].w;
            v[i] = p[(s + PF + i) * 64];
        }
    }
#pragma unroll
    for (int i = 0; i < PF; ++i) { acc.x ^= v[i].x; acc.y ^= v[i].y; }
    if (acc.x == 0x12345678) out[threadIdx.x] = acc;
}
template <int PF>
void run(const uint4* src, uint4* out, int S, int W, size_t total_bytes) {
    // every configuration reads the same total: split over S * W wavefronts
    const long per_wave_vec = (long)(total_bytes / 16 / ((size_t)S * W)) / (64 * PF) * (64 * PF);
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(k<PF>, dim3(S), dim3(W * 64), 0, 0, src, out, per_wave_vec, 0); CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    hipLaunchKernelGGL(k<PF>, dim3(S), dim3(W * 64), 0, 0, src, out, per_wave_vec, 0);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    const double bytes = (double)per_wave_vec * 16 * S * W;
    printf("S=%3d CUs, %2d waves/CU, PF=%2d (%3d KiB in flight/CU): %.3f ms, %.2f TB/s, %.1f GB/s per CU\n", S, W, PF, W * PF, ms,
           bytes / (ms * 1e-3) / 1e12, bytes / (ms * 1e-3) / 1e9 / S);
    fflush(stdout);
}
int main() {
    uint4* src; uint4* out;
    const size_t bytes = (size_t)2 << 30;
    CK(hipMalloc(&src, bytes)); CK(hipMemset(src, 1, bytes)); CK(hipMalloc(&out, 1 << 20));
    for (int S : {8, 16, 32, 64, 256}) {
        const size_t tot = S >= 64 ? bytes : bytes / 4;
        run<4>(src, out, S, 8, tot); run<8>(src, out, S, 8, tot); run<16>(src, out, S, 8, tot);
        run<8>(src, out, S, 16, tot); run<16>(src, out, S, 16, tot); run<4>(src, out, S, 4, tot);
    }
    return 0;
}
