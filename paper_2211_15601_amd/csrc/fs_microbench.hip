// Measurement support: three micro-benchmarks that give the solve kernel's ceilings on the device
// it runs on -- fp32 fused multiply-add issue rate, per-lane 16-byte gathers from a cache-resident
// array (the access pattern of the tri-linear lookup: every SIMD lane its own address) and the
// same gathers from LDS.  Not part of the articulation path itself.
#include "../../include/fastsnarf_bench.h"

#include <hip/hip_runtime.h>

namespace {

__device__ __forceinline__ unsigned lcg(unsigned &s)
{
    s = s * 1664525u + 1013904223u;
    return s >> 8;
}

// pattern 0: every lane reads a random 16-byte piece; 1: 8 adjacent lanes read one aligned 128-byte line;
// 2: every lane reads, with six consecutive instructions, the six 16-byte pieces of a random pair of adjacent 48-byte
// records (what a lane of the solve kernel does for each of the four (x, y) corners of a grid cell)
template <int PAT>
__global__ __launch_bounds__(256) void mb_gather(const float4 *__restrict__ a, unsigned npieces, int iters,
                                                 float4 *__restrict__ sink)
{
    const unsigned lane = threadIdx.x & 63, tid = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned s = tid * 2654435761u + 12345u;
    unsigned s8 = (tid >> 3) * 2654435761u + 77u;
    float4 acc = make_float4(0, 0, 0, 0);
    for (int i = 0; i < iters; ++i) {
        if (PAT == 2) {
            const float4 *p = a + (lcg(s) % (npieces / 3 - 2)) * 3;
#pragma unroll
            for (int u = 0; u < 6; ++u) {
                const float4 v = p[u];
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned idx = PAT == 0 ? lcg(s) % npieces : (lcg(s8) % (npieces / 8)) * 8 + (lane & 7);
            const float4 v = a[idx];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    if (acc.x == 123.456f) sink[tid] = acc;    // never true: keeps the loads alive
}

__global__ __launch_bounds__(256) void mb_lds(int iters, float4 *__restrict__ sink)
{
    __shared__ float4 sm[3072];   // 48 KiB
    for (int i = threadIdx.x; i < 3072; i += 256) sm[i] = make_float4((float)i, 1, 2, 3);
    __syncthreads();
    const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
    unsigned s = tid * 2654435761u + 12345u;
    float4 acc = make_float4(0, 0, 0, 0);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float4 v = sm[lcg(s) % 3072];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    if (acc.x == 123.456f) sink[tid] = acc;
}

__global__ __launch_bounds__(256) void mb_fma(int iters, float *__restrict__ sink)
{
    float a0 = (float)threadIdx.x, a1 = 1, a2 = 2, a3 = 3, a4 = 4, a5 = 5, a6 = 6, a7 = 7;
    const float b = 1.0001f, c = 0.5f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            a0 = __builtin_fmaf(a0, b, c); a1 = __builtin_fmaf(a1, b, c); a2 = __builtin_fmaf(a2, b, c);
            a3 = __builtin_fmaf(a3, b, c); a4 = __builtin_fmaf(a4, b, c); a5 = __builtin_fmaf(a5, b, c);
            a6 = __builtin_fmaf(a6, b, c); a7 = __builtin_fmaf(a7, b, c);
        }
    }
    const float r = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
    if (r == 123.456f) sink[threadIdx.x] = r;
}

template <class F>
bool time_ms(F launch, float *ms)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return false;
    launch();
    bool ok = hipDeviceSynchronize() == hipSuccess;
    ok = ok && hipEventRecord(e0, nullptr) == hipSuccess;
    for (int r = 0; r < 5; ++r) launch();
    ok = ok && hipEventRecord(e1, nullptr) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
    ok = ok && hipEventElapsedTime(ms, e0, e1) == hipSuccess;
    *ms /= 5.0f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ok && hipGetLastError() == hipSuccess;
}

}  // namespace

extern "C" fs_status fs_microbench(int32_t which, int64_t array_bytes, double *result)
{
    if (!result) return FS_E_ARG;
    *result = 0.0;
    const int blocks = 256 * 8, iters = 64;
    float4 *sink = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&sink), sizeof(float4) * blocks * 256) != hipSuccess) {
        (void)hipGetLastError();
        return FS_E_ALLOC;
    }
    float ms = 0.0f;
    bool ok = false;
    fs_status st = FS_OK;
    if (which == FS_MB_GATHER_LANE || which == FS_MB_GATHER_LINE || which == FS_MB_GATHER_SEGMENT) {
        if (array_bytes < 4096 || array_bytes > (1ll << 32)) {
            st = FS_E_SHAPE;
        } else {
            float4 *a = nullptr;
            if (hipMalloc(reinterpret_cast<void **>(&a), (size_t)array_bytes) != hipSuccess) {
                (void)hipGetLastError();
                st = FS_E_ALLOC;
            } else {
                (void)hipMemset(a, 0, (size_t)array_bytes);
                const unsigned np = (unsigned)(array_bytes / 16);
                if (which == FS_MB_GATHER_LANE)
                    ok = time_ms([&] { mb_gather<0><<<blocks, 256>>>(a, np, iters, sink); }, &ms);
                else if (which == FS_MB_GATHER_LINE)
                    ok = time_ms([&] { mb_gather<1><<<blocks, 256>>>(a, np, iters, sink); }, &ms);
                else
                    ok = time_ms([&] { mb_gather<2><<<blocks, 256>>>(a, np, iters, sink); }, &ms);
                (void)hipFree(a);
                // lane accesses per second (8 per round, 6 for the record pairs)
                if (ok) *result = (double)blocks * 256 * iters * (which == FS_MB_GATHER_SEGMENT ? 6 : 8) / (ms * 1e-3);
            }
        }
    } else if (which == FS_MB_LDS_GATHER) {
        ok = time_ms([&] { mb_lds<<<blocks, 256>>>(iters, sink); }, &ms);
        if (ok) *result = (double)blocks * 256 * iters * 8 / (ms * 1e-3);
    } else if (which == FS_MB_FMA) {
        const int fi = 2048;
        ok = time_ms([&] { mb_fma<<<256 * 16, 256>>>(fi, reinterpret_cast<float *>(sink)); }, &ms);
        if (ok) *result = (double)(256 * 16) * 256 * fi * 128 * 2 / (ms * 1e-3);       // flop per second
    } else {
        st = FS_E_ARG;
    }
    (void)hipFree(sink);
    if (st != FS_OK) return st;
    return ok ? FS_OK : FS_E_DEVICE;
}
