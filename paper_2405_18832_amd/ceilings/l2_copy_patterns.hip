// What the memory system delivers to a CU for the access pattern of the LDS-tiled product, without any matrix
// work: 8 wavefronts per CU issue 1 KiB wavefront loads (16 B per lane), 4 per wavefront and k-step (32 KiB per CU
// and step, half of it a row panel, half a weight panel), D steps in flight, one barrier per step, 256 blocks.
// MODE 0: global -> LDS copies; MODE 1: global -> VGPR loads.  The 32 blocks of an XCD share panels as a 4 x 8
// patch of output tiles does.  Patterns differ in where consecutive k-steps of a panel lie in memory: contiguous,
// or the row panels k-step-major over all rows of a 32768-row layer (2 MiB from step to step), or over 4096 rows.
// Prints bytes per (measured) shader clock and CU.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef void __attribute__((address_space(3))) * lptr_t;
__device__ __forceinline__ uint32_t lds_address(const void* p) { return static_cast<uint32_t>(reinterpret_cast<size_t>((lptr_t)(p))); }
__device__ __forceinline__ void copy16_to_lds(const void* src, uint32_t lds_base) {
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(dst) : "memory");
}
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

template <int MODE, int D, int BAR>
__global__ __launch_bounds__(512) void k(const uint4* __restrict__ src, uint4* out, int steps, const long* __restrict__ bases, long rstep, long rpiece, long cstep, long cpiece, int wrap, long long* clk) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = blockIdx.x;
    // all in uint4 units (64 per KiB)
    const uint4* rp = src + bases[2 * b] + (2 * wave) * rpiece + lane;
    const uint4* cp = src + bases[2 * b + 1] + (2 * wave) * cpiece + lane;
    const uint32_t l0 = lds_address(smem) + wave * 4096;
    uint4 acc = make_uint4(0, 0, 0, 0);
    long long c0 = clock64(), w0 = wall_clock64();
    if (MODE == 0) {
        auto issue = [&](int s) {
            const long o = (s % wrap); const int st = s % (D + 1);
            copy16_to_lds(rp + o * rstep, l0 + st * 32768);
            copy16_to_lds(rp + o * rstep + rpiece, l0 + st * 32768 + 1024);
            copy16_to_lds(cp + o * cstep, l0 + st * 32768 + 2048);
            copy16_to_lds(cp + o * cstep + cpiece, l0 + st * 32768 + 3072);
        };
        for (int s = 0; s < D; ++s) issue(s);
        for (int s = 0; s < steps; ++s) {
            issue(s + D);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 * D));
            if (BAR) asm volatile("s_barrier" ::: "memory");
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    } else {
        uint4 v[D + 1][4];
        auto issue = [&](int s, int slot) {
            const long o = (s % wrap);
            v[slot][0] = rp[o * rstep]; v[slot][1] = rp[o * rstep + rpiece]; v[slot][2] = cp[o * cstep]; v[slot][3] = cp[o * cstep + cpiece];
        };
#pragma unroll
        for (int s = 0; s < D; ++s) issue(s, s);
        for (int s = 0; s < steps; s += D + 1) {
#pragma unroll
            for (int q = 0; q < D + 1; ++q) {
                issue(s + q + D, (q + D) % (D + 1));
#pragma unroll
                for (int j = 0; j < 4; ++j) { acc.x ^= v[q][j].x; acc.y ^= v[q][j].y; acc.z ^= v[q][j].z; acc.w ^= v[q][j].w; }
                if (BAR) asm volatile("s_barrier" ::: "memory");
            }
        }
    }
    long long c1 = clock64(), w1 = wall_clock64();
    __syncthreads();
    if (MODE == 0) acc = *reinterpret_cast<uint4*>(smem + threadIdx.x * 16);
    if (acc.x == 0x7fffffff) out[threadIdx.x] = acc;
    if (b == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}


struct Pat { const char* name; long rstep, rpiece, cstep, cpiece; int wrap; long bases[512]; };
template <int MODE, int D, int BAR>
void run(const uint4* src, uint4* out, long long* clk, long* dbases, const Pat& p) {
    const int steps = 24000, blocks = 256;
    auto kern = k<MODE, D, BAR>;
    const int lds = (D + 1) * 32768;
    CK(hipMemcpy(dbases, p.bases, sizeof(p.bases), hipMemcpyHostToDevice));
    CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), lds, 0, src, out, 240, dbases, p.rstep, p.rpiece, p.cstep, p.cpiece, p.wrap, clk); CK(hipDeviceSynchronize());
    CK(hipEventRecord(a));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), lds, 0, src, out, steps, dbases, p.rstep, p.rpiece, p.cstep, p.cpiece, p.wrap, clk);
    CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
    float ms; CK(hipEventElapsedTime(&ms, a, b));
    long long h[2]; CK(hipMemcpy(h, clk, 16, hipMemcpyDeviceToHost));
    const double ghz = (double)h[0] / (double)h[1] * 0.1;   // wall clock: 100 MHz
    const double bytes = (double)steps * 32768;
    printf("%-34s %s D=%d bar=%d: %.3f ms, clock %.2f GHz, %.1f B/clk/CU, %.0f clk/step, aggregate %.1f TB/s\n", p.name,
           MODE == 0 ? "->LDS " : "->VGPR", D, BAR, ms, ghz, bytes / (double)h[0], (double)h[0] / steps, bytes * 256 / (ms * 1e-3) / 1e12);
    fflush(stdout);
}

int main() {
    uint4* src; uint4* out; long long* clk; long* dbases;
    const size_t bytes = (size_t)1 << 30;   // 1 GiB
    CK(hipMalloc(&src, bytes)); CK(hipMemset(src, 1, bytes)); CK(hipMalloc(&out, 1 << 20)); CK(hipMalloc(&clk, 64)); CK(hipMalloc(&dbases, 512 * 8));
    const long KB = 64;            // uint4 per KiB
    static Pat ps[10];
    int np = 0;
    auto patch = [](int b, int& xcd, int& mi, int& ni) { xcd = b & 7; const int idx = b >> 3; mi = idx >> 3; ni = idx & 7; };
    {   // contiguous panels, 4x8 patch, 64 steps per panel (12 MiB per XCD)
        Pat& p = ps[np++]; p = Pat{"both panels contiguous, 64 steps", 16 * KB, KB, 16 * KB, KB, 64, {}};
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 64 * 16 * KB; p.bases[2 * b + 1] = (long)(32 + x * 8 + ni) * 64 * 16 * KB; }
    }
    {   // second product with h k-step-major over all rows: [256 steps][32768 rows][32] (2 MiB per step), W2 fragments [128 nb][256 kb] KiB
        Pat& p = ps[np++]; p = Pat{"rows k-major/32768, frags 256K", 2048 * KB, KB, KB, 256 * KB, 256, {}};
        const long wbase = 512 * 1024 * KB;     // weights behind the 512 MiB of h
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 16 * KB; p.bases[2 * b + 1] = wbase + (long)(ni * 16) * 256 * KB; }
    }
    {   // first product with x k-step-major over all rows: [64 steps][32768][32], W1 fragments [512 nb][64 kb] KiB; 8 of 32 column tiles
        Pat& p = ps[np++]; p = Pat{"rows k-major/32768, frags 64K", 2048 * KB, KB, KB, 64 * KB, 64, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 16 * KB; p.bases[2 * b + 1] = wbase + (long)(ni * 16) * 64 * KB; }
    }
    {   // second product, weights tile-contiguous: [8 column tiles][256 kb][16 frags] KiB, h as now
        Pat& p = ps[np++]; p = Pat{"rows k-major/32768, weights contig", 2048 * KB, KB, 16 * KB, KB, 256, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 16 * KB; p.bases[2 * b + 1] = wbase + (long)ni * 256 * 16 * KB; }
    }
    {   // second product, both tile-contiguous: rows [row tile][256 kb][16 KiB]
        Pat& p = ps[np++]; p = Pat{"rows blocked, weights contig", 16 * KB, KB, 16 * KB, KB, 256, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 256 * 16 * KB; p.bases[2 * b + 1] = wbase + (long)ni * 256 * 16 * KB; }
    }

    {   // second product as the library lays it out: rows in blocks of 256 (16 KiB per step), packed weight fragments
        Pat& p = ps[np++]; p = Pat{"rows blocked, frags 256K (2nd)", 16 * KB, KB, KB, 256 * KB, 256, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 256 * 16 * KB; p.bases[2 * b + 1] = wbase + (long)(ni * 16) * 256 * KB; }
    }
    {   // first product as the library lays it out (64 steps)
        Pat& p = ps[np++]; p = Pat{"rows blocked, frags 64K (1st)", 16 * KB, KB, KB, 64 * KB, 64, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)(x * 4 + mi) * 64 * 16 * KB; p.bases[2 * b + 1] = wbase + (long)(ni * 16) * 64 * KB; }
    }
    {   // h k-step-major with a smaller stride between steps (as if A were 4096 rows: 256 KiB)
        Pat& p = ps[np++]; p = Pat{"rows k-major/4096, frags 256K", 256 * KB, KB, KB, 256 * KB, 256, {}};
        const long wbase = 512 * 1024 * KB;
        for (int b = 0; b < 256; ++b) { int x, mi, ni; patch(b, x, mi, ni); p.bases[2 * b] = (long)((x * 4 + mi) % 16) * 16 * KB; p.bases[2 * b + 1] = wbase + (long)(ni * 16) * 256 * KB; }
    }
    for (int i = 0; i < np; ++i) {
        run<0, 3, 1>(src, out, clk, dbases, ps[i]);
        run<1, 2, 1>(src, out, clk, dbases, ps[i]);
    }
    return 0;
}
