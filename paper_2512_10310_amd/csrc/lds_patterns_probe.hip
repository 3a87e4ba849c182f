// Measurement helper, a program of its own (not part of libevl.so): the LDS access patterns of
// attn_kernel<128>, one kernel per pattern and nothing else in it, so that one counter pass
// (rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS SQ_INSTS_LDS) names the accesses that
// run into bank conflicts:
//   k_read / v_read : the operand reads of the two MFMA blocks of the loop (swizzled K rows,
//                     [half][channel] V words), against lane-linear reads of the same width
//   tab_read<S>     : the prologue's reads of the cos/sin table, token rows S pairs apart
//                     (64: rows 512 bytes apart; 66: the padded rows the kernel uses)
//   stage_write / stage_read : the epilogue's staging of bf16 rows (row stride 272 bytes)
//   fill            : the direct global -> LDS loads that fill the tile ring
// Each kernel is one work-group of 8 waves doing its pattern a fixed number of times.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
constexpr int D = 128, KN = 64, CH = 16, NW = 8, ITER = 2000;
#define SINK(v) asm volatile("" ::"v"(v))

__device__ __forceinline__ void prep(int &lane, int &wave, int &j, int &h) {
    lane = threadIdx.x & 63; wave = threadIdx.x >> 6; j = lane & 31; h = lane >> 5;
}
// K operand reads: row krow(j), chunk (2ks+h)^gj, two 32-key blocks
__global__ __launch_bounds__(512) void k_read(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    const int krow = 16 * (j >> 4) + 8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3);
    const int gj = j & 15;
    int off[8];
    for (int ks = 0; ks < 8; ++ks) off[ks] = krow * (D * 2) + (((2 * ks + h) ^ gj) & (CH - 1)) * 16;
    float acc = 0;
    for (int it = 0; it < ITER; ++it) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                bf16x8 a = *(const bf16x8 *)(smem + kb * 32 * (D * 2) + off[ks]);
                SINK(a);
            }
    }
    out[threadIdx.x] = acc;
}
// V operand reads: [page][block][h][j]
__global__ __launch_bounds__(512) void v_read(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    const int v_read_off = h * 512 + j * 16;
    for (int it = 0; it < ITER; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            bf16x8 a = *(const bf16x8 *)(smem + v_read_off + (u / 4) * 4096 + (u % 4) * 1024);
            SINK(a);
        }
    }
    out[threadIdx.x] = 0;
}
// reference: lane-linear 16-byte reads
__global__ __launch_bounds__(512) void linear_read(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    for (int it = 0; it < ITER; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            bf16x8 a = *(const bf16x8 *)(smem + lane * 16 + u * 1024);
            SINK(a);
        }
    }
    out[threadIdx.x] = 0;
}
// prologue cos/sin table reads: float2 trow[16*ks + e], row of token (row / 7), token stride STRIDE float2
template <int STRIDE>
__global__ __launch_bounds__(512) void tab_read(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    const float2 *tab = (const float2 *)smem;
    const int tok = (wave * 32 + j) / 7;
    const float2 *trow = tab + tok * STRIDE + 8 * h;
    float acc = 0;
    for (int it = 0; it < ITER / 4; ++it) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float2 cs = trow[16 * ks + e];
                SINK(cs.x); SINK(cs.y);
            }
    }
    out[threadIdx.x] = acc;
}
// epilogue staging: bf16x4 writes at (row j)*RS + (db*32 + 8a + 4h)*2, then whole-row bf16x8 reads
template <int RS>
__global__ __launch_bounds__(512) void stage_write(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    unsigned char *stg = smem + wave * (32 * RS);
    bf16x4 ob; for (int e = 0; e < 4; ++e) ob[e] = (bf16)1.0f;
    for (int it = 0; it < ITER / 4; ++it) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                *(bf16x4 *)(stg + j * RS + (db * 32 + 8 * a + 4 * h) * 2) = ob;
                asm volatile("" ::: "memory");
            }
    }
    out[threadIdx.x] = 0;
}
template <int RS>
__global__ __launch_bounds__(512) void stage_read(float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    unsigned char *stg = smem + wave * (32 * RS);
    for (int it = 0; it < ITER / 4; ++it) {
#pragma unroll
        for (int r8 = 0; r8 < 8; ++r8) {
            const int r = r8 * 4 + lane / 16, c = lane % 16;
            bf16x8 v = *(const bf16x8 *)(stg + r * RS + c * 16);
            SINK(v);
        }
    }
    out[threadIdx.x] = 0;
}
// direct global -> LDS fills as in the kernel (K swizzled source offsets; LDS side is lane-linear)
__global__ __launch_bounds__(512) void fill(const unsigned char *src, float *out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    int lane, wave, j, h; prep(lane, wave, j, h);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    for (int it = 0; it < ITER / 8; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + wave * 4096 + u * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(lane * 16 + u * 1024), "s"(src) : "memory");
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    out[threadIdx.x] = 0;
}
int main() {
    float *out; unsigned char *src;
    hipMalloc(&out, 4096); hipMalloc(&src, 1 << 20); hipMemset(src, 0, 1 << 20);
    const size_t lds = 96 * 1024;
#define RUN(k, ...) do { hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); \
    hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b); hipLaunchKernelGGL(k, dim3(1), dim3(512), lds, 0, __VA_ARGS__); hipDeviceSynchronize(); \
    hipEventRecord(a); hipLaunchKernelGGL(k, dim3(1), dim3(512), lds, 0, __VA_ARGS__); hipEventRecord(b); hipDeviceSynchronize(); float ms; hipEventElapsedTime(&ms, a, b); \
    printf("%-28s %.1f us\n", #k, ms * 1e3); fflush(stdout); } while (0)
    RUN(linear_read, out);
    RUN(k_read, out);
    RUN(v_read, out);
    RUN((tab_read<64>), out);
    RUN((tab_read<66>), out);
    RUN((stage_write<272>), out);
    RUN((stage_read<272>), out);
    RUN(fill, src, out);
    hipError_t e = hipGetLastError();
    printf("status %s\n", hipGetErrorString(e));
    return e != hipSuccess;
}
