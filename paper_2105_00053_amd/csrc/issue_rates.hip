// Instruction-issue microbenchmarks: the rates the roofline discussion of the kernels leans on,
// measured on the machine the kernels run on.  Not part of the library boundary: bench.py --issue-rates
// loads this file's own small shared object and prints what it returns.
//
// Each kernel keeps 16 independent dependency chains per lane in registers and repeats one instruction on
// them, 4096 x 16 times per lane, on 8 workgroups of 256 lanes per compute unit (two waves per SIMD, enough
// to cover the issue latency of a dependent chain of 16).  Rate = lanes x repeats / time, in lane-operations
// per second; for the 16-bit dot product one lane-operation is two multiply-accumulates.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef short short2_t __attribute__((ext_vector_type(2)));
constexpr int REPEATS = 4096;
constexpr int CHAINS = 16;
constexpr int THREADS = 256;

__global__ __launch_bounds__(THREADS) void dot2_rate_kernel(int* out, int a0, int b0) {
    int acc[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) acc[i] = (int)threadIdx.x + i;
    const int a = a0 + (int)threadIdx.x, b = b0 ^ (int)threadIdx.x;
    for (int it = 0; it < REPEATS; ++it) {
#pragma unroll
        for (int i = 0; i < CHAINS; ++i)
            acc[i] = __builtin_amdgcn_sdot2(__builtin_bit_cast(short2_t, a), __builtin_bit_cast(short2_t, b + i), acc[i], false);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) s ^= acc[i];
    out[blockIdx.x * THREADS + threadIdx.x] = s;
}

__global__ __launch_bounds__(THREADS) void fma64_rate_kernel(int* out, int a0, int b0) {
    double acc[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) acc[i] = (double)((int)threadIdx.x + i);
    const double a = 1.0 + 1e-9 * a0, b = 1e-3 * (b0 + (int)threadIdx.x);
    for (int it = 0; it < REPEATS; ++it) {
#pragma unroll
        for (int i = 0; i < CHAINS; ++i) acc[i] = __builtin_fma(acc[i], a, b);
    }
    double s = 0;
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) s += acc[i];
    out[blockIdx.x * THREADS + threadIdx.x] = (int)s;
}

__global__ __launch_bounds__(THREADS) void add32_rate_kernel(int* out, int a0, int b0) {
    uint32_t acc[CHAINS];
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) acc[i] = threadIdx.x + i;
    const uint32_t b = (uint32_t)b0 ^ threadIdx.x;
    for (int it = 0; it < REPEATS; ++it) {
#pragma unroll
        for (int i = 0; i < CHAINS; ++i) acc[i] = (acc[i] ^ b) + (uint32_t)a0;  // xor + add: counted as two operations, one instruction if the compiler fuses them
    }
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < CHAINS; ++i) s ^= acc[i];
    out[blockIdx.x * THREADS + threadIdx.x] = (int)s;
}

// 16-byte LDS reads in the access pattern of the GEMM tiles (16 distinct addresses per wave, the rest broadcast)
__global__ __launch_bounds__(THREADS) void lds128_rate_kernel(int* out, int a0, int) {
    __shared__ int4 buf[2048];
    for (int i = threadIdx.x; i < 2048; i += THREADS) buf[i] = make_int4(i, i + 1, i + 2, a0);
    __syncthreads();
    int4 acc = make_int4(0, 0, 0, 0);
    const int idx = threadIdx.x & 15;
    for (int it = 0; it < REPEATS; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int4 v = buf[(idx + i * 16 + it * 3) & 2047];
            acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
        }
    }
    out[blockIdx.x * THREADS + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

// v_mfma_i32_32x32x32_i8 from registers: 8 independent accumulator blocks per wave, one wave per SIMD
typedef int rate_v4i __attribute__((ext_vector_type(4)));
typedef int rate_v16i __attribute__((ext_vector_type(16)));
constexpr int MFMA_CHAINS = 8;
__global__ __launch_bounds__(THREADS, 1) void mfma_i8_rate_kernel(int* out, int a0, int b0) {
    rate_v16i acc[MFMA_CHAINS];
#pragma unroll
    for (int i = 0; i < MFMA_CHAINS; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    const rate_v4i a = {a0 + (int)threadIdx.x, a0, 3, 5}, b = {7, b0 ^ (int)threadIdx.x, 11, 13};
    for (int it = 0; it < REPEATS; ++it) {
#pragma unroll
        for (int i = 0; i < MFMA_CHAINS; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < MFMA_CHAINS; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s ^= acc[i][r];
    out[blockIdx.x * THREADS + threadIdx.x] = s;
}

template <class K>
int time_kernel(K kernel, int blocks, int* out, float* ms) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(THREADS), 0, 0, out, 3, 5);
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    hipEventRecord(e0, 0);
    for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(kernel, dim3(blocks), dim3(THREADS), 0, 0, out, 3, 5);
    hipEventRecord(e1, 0);
    if (hipEventSynchronize(e1) != hipSuccess) return 1;
    hipEventElapsedTime(ms, e0, e1);
    *ms /= 5;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace

// rates[0]: v_dot2_i32_i16 lane-operations/s, [1]: fp64 fma lane-operations/s, [2]: 32-bit integer
// operations/s (xor + add pairs, two operations per pair), [3]: LDS bytes/s through 16-byte reads, [4]: int8
// operations/s of v_mfma_i32_32x32x32_i8 (2 per multiply-accumulate).  info[0] = compute units,
// info[1] = clock in kHz as the runtime reports it.  Returns 0 on success.
extern "C" int pnn_issue_rates(double* rates, int* info) {
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, 0) != hipSuccess) return 1;
    info[0] = p.multiProcessorCount;
    info[1] = p.clockRate;
    const int blocks = p.multiProcessorCount * 8;
    int* out = nullptr;
    if (hipMalloc(&out, (size_t)blocks * THREADS * sizeof(int)) != hipSuccess) return 1;
    const double lane_ops = (double)blocks * THREADS * REPEATS * CHAINS;
    float ms = 0;
    int bad = 0;
    bad |= time_kernel(dot2_rate_kernel, blocks, out, &ms);
    rates[0] = lane_ops / (ms * 1e-3);
    bad |= time_kernel(fma64_rate_kernel, blocks, out, &ms);
    rates[1] = lane_ops / (ms * 1e-3);
    bad |= time_kernel(add32_rate_kernel, blocks, out, &ms);
    rates[2] = 2 * lane_ops / (ms * 1e-3);
    bad |= time_kernel(lds128_rate_kernel, blocks, out, &ms);
    rates[3] = (double)blocks * THREADS * REPEATS * 8 * 16 / (ms * 1e-3);
    bad |= time_kernel(mfma_i8_rate_kernel, p.multiProcessorCount, out, &ms);  // one workgroup of four waves per compute unit
    rates[4] = 2.0 * p.multiProcessorCount * (THREADS / 64) * (double)REPEATS * MFMA_CHAINS * 32768.0 / (ms * 1e-3);
    hipFree(out);
    return bad;
}
