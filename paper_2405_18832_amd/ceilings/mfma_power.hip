// What the chip sustains under its power management: a register-only MFMA loop on random bf16 operands, and the
// same loop mixed with LDS reads and global -> LDS copies at the rates of the LDS-tiled product, each run for
// about 80 ms.  8 wavefronts per CU; per step each wavefront issues 32 MFMA 16x16x32 (or 16 of 32x32x16), NR
// ds_read_b128 whose results feed the MFMAs, and NC 1 KiB global -> LDS copies from an L2-resident buffer.  No
// barriers, no epilogues, no misses: an upper bound for a kernel with that instruction mix.  The shader clock
// is measured (s_memtime against the 100 MHz wall clock); the published peak assumes 2.4 GHz.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef void __attribute__((address_space(3))) * lptr_t;
__device__ __forceinline__ uint32_t lds_address(const void* p) { return static_cast<uint32_t>(reinterpret_cast<size_t>((lptr_t)(p))); }
__device__ __forceinline__ void copy16_to_lds(const void* src, uint32_t lds_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory");
}
__device__ inline unsigned hashu(unsigned x){ x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }

// NR: LDS reads per step (0, 4, 8, 12); NC: copies per step (0 or 4); K32: 32x32x16 instead of 16x16x32
template <int NR, int NC, int K32>
__global__ __launch_bounds__(512) void k(const uint4* __restrict__ src, float* out, int steps, long long* clk, int constant_operands) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // 96 KiB operand area + 32 KiB copy landing area
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // random bf16 data in the operand area
    for (int i = threadIdx.x; i < 24576; i += 512) {      // 96 KiB: 12 KiB per wavefront
        const unsigned h = hashu(i * 2654435761u + blockIdx.x);
        reinterpret_cast<uint32_t*>(smem)[i] = constant_operands ? 0x3f803f80u   // every operand 1.0: nothing toggles
                                                                  : ((h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u));   // magnitudes around 0.5 - 2
    }
    __syncthreads();
    bf16x8 w[4], x[8];
    const unsigned char* base = smem + (wave * 12 * 64 + lane) * 16;       // 12 KiB per wavefront
    for (int i = 0; i < 4; ++i) w[i] = *reinterpret_cast<const bf16x8*>(base + i * 1024);
    for (int i = 0; i < 8; ++i) x[i] = *reinterpret_cast<const bf16x8*>(base + (4 + i) * 1024);
    const uint4* gp = src + (size_t)blockIdx.x * 4096 + wave * 512 + lane;   // 64 KiB per block (8 KiB per wavefront), L2 resident
    const uint32_t land = lds_address(smem) + 98304 + wave * 4096;   // 32 KiB behind the operand area
    f32x4 acc[4][8];
    f32x16 acc32[2][4];
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0, 0, 0, 0};
    for (int i = 0; i < 2; ++i) for (int j = 0; j < 4; ++j) for (int q = 0; q < 16; ++q) acc32[i][j][q] = 0;
    long long c0 = clock64(), w0 = wall_clock64();
    for (int s = 0; s < steps; ++s) {
        const unsigned char* b2 = base + ((s & 1) ? 0 : 0);
        if (NC > 0) {
#pragma unroll
            for (int c = 0; c < NC; ++c) copy16_to_lds(gp + ((s & 1) * 4 + c) * 64, land + c * 1024);   // index < 8 * 64 + 63 inside the wavefront's 512
        }
        if (NR >= 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i] = *reinterpret_cast<const bf16x8*>(b2 + i * 1024);
        }
        if (NR >= 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = *reinterpret_cast<const bf16x8*>(b2 + (4 + i) * 1024);
        }
        if (NR >= 12) {
#pragma unroll
            for (int i = 4; i < 8; ++i) x[i] = *reinterpret_cast<const bf16x8*>(b2 + (4 + i) * 1024);
        }
        if (K32) {
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        acc32[nb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[2 * nb + kh], x[2 * rb + kh], acc32[nb][rb], 0, 0, 0);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[i], x[j], acc[i][j], 0, 0, 0);
        }
        if (NC > 0) __builtin_amdgcn_s_waitcnt(0x0F70 | NC);   // the previous step's copies have landed
        asm volatile("" ::: "memory");
    }
    long long c1 = clock64(), w1 = wall_clock64();
    float sum = 0;
    for (int i = 0; i < 4; ++i) for (int j = 0; j < 8; ++j) sum += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    for (int i = 0; i < 2; ++i) for (int j = 0; j < 4; ++j) for (int q = 0; q < 16; ++q) sum += acc32[i][j][q];
    if (sum == 12345.678f) out[threadIdx.x] = sum;
    if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}
template <int NR, int NC, int K32>
void run(const uint4* src, float* out, long long* clk, int constant_operands = 0) {
    const int steps = 150000, blocks = 256;   // ~80 ms: long enough for the power management to settle
    auto kern = k<NR, NC, K32>;
    CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), 131072, 0, src, out, 1000, clk, constant_operands); CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), 131072, 0, src, out, steps, clk, constant_operands);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    long long h[2]; CK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
    const double flops = (double)steps * 32 * 16384.0 * 8 * blocks;
    printf("%s mfma %s, %2d LDS reads (%3d KiB/step/CU), %d copies (%2d KiB/step/CU): %.1f ms, %.0f TFLOP/s (%.3f of 2500), clock %.3f GHz, %.0f clk/step\n",
           constant_operands ? "constant operands," : "random operands,  ", K32 ? "32x32x16" : "16x16x32", NR, NR * 8, NC, NC * 8, ms, flops / (ms * 1e-3) / 1e12, flops / (ms * 1e-3) / 2.5e15,
           (double)h[0] / (double)h[1] * 0.1, (double)h[0] / steps);
    fflush(stdout);
}
int main() {
    uint4* src; float* out; long long* clk;
    CK(hipMalloc(&src, (size_t)256 * 65536)); CK(hipMemset(src, 0x5a, (size_t)256 * 65536)); CK(hipMalloc(&out, 1 << 20)); CK(hipMalloc(&clk, 64));
        run<0, 0, 0>(src, out, clk, 1);
    run<0, 0, 0>(src, out, clk); run<4, 0, 0>(src, out, clk); run<8, 0, 0>(src, out, clk); run<12, 0, 0>(src, out, clk);
    run<0, 4, 0>(src, out, clk); run<8, 4, 0>(src, out, clk); run<12, 4, 0>(src, out, clk);
    run<0, 0, 1>(src, out, clk); run<12, 0, 1>(src, out, clk); run<12, 4, 1>(src, out, clk);
    run<0, 0, 0>(src, out, clk); run<12, 4, 0>(src, out, clk);
    return 0;
}
