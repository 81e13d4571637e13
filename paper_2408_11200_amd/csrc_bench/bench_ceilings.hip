// Instruction-rate ceilings of one MI355X compute unit, measured the way the layer kernels use the
// hardware: independent fp32 multiply-adds, LDS reads of 4 / 8 / 16 bytes per lane, LDS writes, LDS
// floating-point atomic adds, an LDS read-modify-write, and the 4x4x1 fp32 matrix-core instruction
// (independent, and as dependent chains of five).  One workgroup per CU (256 workgroups), every wave
// in an 8 KB LDS region of its own, unit-stride addresses (no bank conflicts).  Part of the benchmark
// library (kan_bench.h: kan_bench_ceiling); `python bench.py --ceilings` prints the table.
#include <hip/hip_runtime.h>
#include "kan_bench.h"

namespace {
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));

// MODE 0: v_fma_f32  1: ds_read_b32  2: ds_read_b64  3: ds_read_b128  4: ds_write_b32  5: ds_write_b128
// 6: ds_add_f32 (no return)  7: v_mfma_f32_4x4x1 independent  8: the same in two chains of five from zero
// 11: ds_read_b32 + add + ds_write_b32
template <int MODE>
__global__ __launch_bounds__(1024) void ceiling_kernel(float *out, int iters)
{
    extern __shared__ float sm[];
    for (int i = threadIdx.x; i < 32768; i += blockDim.x) sm[i] = 0.0f;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // each wave works in its own 8 KB region (16 waves -> 128 KB)
    unsigned a4 = (unsigned)(wave * 8192 + lane * 4);
    unsigned a8 = (unsigned)(wave * 8192 + lane * 8);
    unsigned a16 = (unsigned)(wave * 8192 + lane * 16);
    float v0 = lane * 0.5f, v1 = 1.0f, v2 = 2.0f, v3 = 3.0f, v4 = 0.1f, v5 = 0.2f, v6 = 0.3f, v7 = 0.4f;
    f4 d0 = {0, 0, 0, 0}, d1 = d0, d2 = d0, d3 = d0, d4 = d0, d5 = d0, d6 = d0, d7 = d0;
    f4 q0 = d0;
    f2 p0 = {0, 0};
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 0) {
            asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n"
                         "v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n"
                         : "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3), "+v"(v4), "+v"(v5), "+v"(v6), "+v"(v7) : "v"(0.999f), "v"(0.001f));
        } else if constexpr (MODE == 1) {
            float b0, b1, b2, b3, b4, b5, b6, b7;
            asm volatile("ds_read_b32 %0, %8 offset:0\n ds_read_b32 %1, %8 offset:256\n ds_read_b32 %2, %8 offset:512\n ds_read_b32 %3, %8 offset:768\n"
                         "ds_read_b32 %4, %8 offset:1024\n ds_read_b32 %5, %8 offset:1280\n ds_read_b32 %6, %8 offset:1536\n ds_read_b32 %7, %8 offset:1792\n s_waitcnt lgkmcnt(0)"
                         : "=v"(b0), "=v"(b1), "=v"(b2), "=v"(b3), "=v"(b4), "=v"(b5), "=v"(b6), "=v"(b7) : "v"(a4));
            v0 += b0 + b7;
        } else if constexpr (MODE == 2) {
            f2 b0, b1, b2, b3, b4, b5, b6, b7;
            asm volatile("ds_read_b64 %0, %8 offset:0\n ds_read_b64 %1, %8 offset:512\n ds_read_b64 %2, %8 offset:1024\n ds_read_b64 %3, %8 offset:1536\n"
                         "ds_read_b64 %4, %8 offset:2048\n ds_read_b64 %5, %8 offset:2560\n ds_read_b64 %6, %8 offset:3072\n ds_read_b64 %7, %8 offset:3584\n s_waitcnt lgkmcnt(0)"
                         : "=v"(b0), "=v"(b1), "=v"(b2), "=v"(b3), "=v"(b4), "=v"(b5), "=v"(b6), "=v"(b7) : "v"(a8));
            p0 += b0 + b7;
        } else if constexpr (MODE == 3) {
            f4 b0, b1, b2, b3, b4, b5, b6, b7;
            asm volatile("ds_read_b128 %0, %8 offset:0\n ds_read_b128 %1, %8 offset:1024\n ds_read_b128 %2, %8 offset:2048\n ds_read_b128 %3, %8 offset:3072\n"
                         "ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %8 offset:5120\n ds_read_b128 %6, %8 offset:6144\n ds_read_b128 %7, %8 offset:7168\n s_waitcnt lgkmcnt(0)"
                         : "=v"(b0), "=v"(b1), "=v"(b2), "=v"(b3), "=v"(b4), "=v"(b5), "=v"(b6), "=v"(b7) : "v"(a16));
            q0 += b0 + b7;
        } else if constexpr (MODE == 4) {
            asm volatile("ds_write_b32 %0, %1 offset:0\n ds_write_b32 %0, %1 offset:256\n ds_write_b32 %0, %1 offset:512\n ds_write_b32 %0, %1 offset:768\n"
                         "ds_write_b32 %0, %1 offset:1024\n ds_write_b32 %0, %1 offset:1280\n ds_write_b32 %0, %1 offset:1536\n ds_write_b32 %0, %1 offset:1792\n s_waitcnt lgkmcnt(0)"
                         :: "v"(a4), "v"(v0) : "memory");
        } else if constexpr (MODE == 5) {
            asm volatile("ds_write_b128 %0, %1 offset:0\n ds_write_b128 %0, %1 offset:1024\n ds_write_b128 %0, %1 offset:2048\n ds_write_b128 %0, %1 offset:3072\n"
                         "ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:5120\n ds_write_b128 %0, %1 offset:6144\n ds_write_b128 %0, %1 offset:7168\n s_waitcnt lgkmcnt(0)"
                         :: "v"(a16), "v"(d0) : "memory");
        } else if constexpr (MODE == 6) {
            asm volatile("ds_add_f32 %0, %1 offset:0\n ds_add_f32 %0, %1 offset:256\n ds_add_f32 %0, %1 offset:512\n ds_add_f32 %0, %1 offset:768\n"
                         "ds_add_f32 %0, %1 offset:1024\n ds_add_f32 %0, %1 offset:1280\n ds_add_f32 %0, %1 offset:1536\n ds_add_f32 %0, %1 offset:1792\n s_waitcnt lgkmcnt(0)"
                         :: "v"(a4), "v"(v1) : "memory");
        } else if constexpr (MODE == 7) {
            d0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v1, d0, 4, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v2, d1, 4, 1, 0);
            d2 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v3, d2, 4, 2, 0);
            d3 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v4, d3, 4, 3, 0);
            d4 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v5, d4, 4, 4, 0);
            d5 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v6, d5, 4, 5, 0);
            d6 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v7, d6, 4, 6, 0);
            d7 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v1, d7, 4, 7, 0);
        } else if constexpr (MODE == 8) {
            // two chains of five dependent MFMAs starting from zero, result folded into d0/d1 by VALU adds
            f4 z = {0, 0, 0, 0};
            f4 t0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v1, z, 4, 0, 0);
            f4 t1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v0, v2, z, 4, 0, 0);
            t0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v3, v1, t0, 4, 0, 0);
            t1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v3, v2, t1, 4, 0, 0);
            t0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v4, v1, t0, 4, 0, 0);
            t1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v4, v2, t1, 4, 0, 0);
            t0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v5, v1, t0, 4, 0, 0);
            t1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v5, v2, t1, 4, 0, 0);
            t0 = __builtin_amdgcn_mfma_f32_4x4x1f32(v6, v1, t0, 4, 0, 0);
            t1 = __builtin_amdgcn_mfma_f32_4x4x1f32(v6, v2, t1, 4, 0, 0);
            d0 += t0; d1 += t1;
            asm volatile("" : "+v"(v0));
        } else if constexpr (MODE == 11) {
            float b0, b1, b2, b3;
            asm volatile("ds_read_b32 %0, %4 offset:0\n ds_read_b32 %1, %4 offset:256\n ds_read_b32 %2, %4 offset:512\n ds_read_b32 %3, %4 offset:768\n s_waitcnt lgkmcnt(0)"
                         : "=v"(b0), "=v"(b1), "=v"(b2), "=v"(b3) : "v"(a4) : "memory");
            b0 += v1; b1 += v1; b2 += v1; b3 += v1;
            asm volatile("ds_write_b32 %4, %0 offset:0\n ds_write_b32 %4, %1 offset:256\n ds_write_b32 %4, %2 offset:512\n ds_write_b32 %4, %3 offset:768\n"
                         :: "v"(b0), "v"(b1), "v"(b2), "v"(b3), "v"(a4) : "memory");
        }
    }
    __syncthreads();
    float r = v0 + v1 + v2 + v3 + v4 + v5 + v6 + v7 + q0[0] + q0[3] + p0[0] + p0[1];
    f4 s = d0 + d1 + d2 + d3 + d4 + d5 + d6 + d7;
    r += s[0] + s[1] + s[2] + s[3] + sm[threadIdx.x];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
}


struct Mode { int id; const char *name; const char *unit; double units_per_thread_iter; void (*kern)(float *, int); };
const Mode kModes[] = {
    {0, "v_fma_f32 x8", "FMA", 8, ceiling_kernel<0>},
    {1, "ds_read_b32 x8", "B", 32, ceiling_kernel<1>},
    {2, "ds_read_b64 x8", "B", 64, ceiling_kernel<2>},
    {3, "ds_read_b128 x8", "B", 128, ceiling_kernel<3>},
    {4, "ds_write_b32 x8", "B", 32, ceiling_kernel<4>},
    {5, "ds_write_b128 x8", "B", 128, ceiling_kernel<5>},
    {6, "ds_add_f32 x8", "B", 32, ceiling_kernel<6>},
    {7, "v_mfma_f32_4x4x1 x8 independent", "FMA", 8.0 * 256 / 64, ceiling_kernel<7>},
    {8, "v_mfma_f32_4x4x1 two chains of five", "FMA", 10.0 * 256 / 64, ceiling_kernel<8>},
    {11, "ds_read_b32 x4 + add + ds_write_b32 x4", "B", 32, ceiling_kernel<11>},
};
}  // namespace

extern "C" int kan_bench_ceiling_count(void) { return (int)(sizeof(kModes) / sizeof(kModes[0])); }

extern "C" int kan_bench_ceiling(int index, int threads_per_cu, int iters, const char **name, const char **unit,
                                 double *per_cu_per_second, double *ms)
{
    if (index < 0 || index >= kan_bench_ceiling_count() || iters < 1 || !per_cu_per_second) return KAN_ERR_INVALID_ARG;
    if (threads_per_cu != 256 && threads_per_cu != 512 && threads_per_cu != 1024) return KAN_ERR_INVALID_ARG;
    const Mode &m = kModes[index];
    constexpr int kLds = 131072, kBlocks = 256;
    float *out = nullptr;
    if (hipMalloc(&out, (size_t)kBlocks * 1024 * sizeof(float)) != hipSuccess) return KAN_ERR_HIP;
    hipEvent_t e0, e1;
    int rc = KAN_OK;
    float t = 0.0f;
    if (hipEventCreate(&e0) != hipSuccess) { (void)hipFree(out); return KAN_ERR_HIP; }
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); (void)hipFree(out); return KAN_ERR_HIP; }
    if (hipFuncSetAttribute((const void *)m.kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLds) != hipSuccess) rc = KAN_ERR_HIP;
    if (rc == KAN_OK) {
        m.kern<<<kBlocks, threads_per_cu, kLds>>>(out, 10);             // warm-up
        if (hipDeviceSynchronize() != hipSuccess) rc = KAN_ERR_HIP;
    }
    if (rc == KAN_OK) {
        (void)hipEventRecord(e0);
        m.kern<<<kBlocks, threads_per_cu, kLds>>>(out, iters);
        (void)hipEventRecord(e1);
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&t, e0, e1) != hipSuccess) rc = KAN_ERR_HIP;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(out);
    if (rc != KAN_OK) return rc;
    if (name) *name = m.name;
    if (unit) *unit = m.unit;
    if (ms) *ms = t;
    *per_cu_per_second = (double)iters * threads_per_cu * m.units_per_thread_iter / (t * 1e-3);
    return KAN_OK;
}
