// What one MI355X actually delivers on the two resources the scoring kernels are bound by, measured with loops
// shaped like theirs -- measurement tooling, not part of libaif:
//   aifcal_mfma: bf16 32x32x16 MFMAs back to back on every SIMD, four independent accumulators per wave, the A
//                operand either held in registers or read from LDS for every MFMA (the MLP chain's and the attention
//                kernels' pattern), operands constant or random (switching activity sets the board's power, and the
//                power limit sets the clock);
//   aifcal_copy: a plain 16-bytes-per-lane device copy, and a read-only pass over the same buffer.
// Each reports a rate and the shader clock during the run (cycle counter against the 100 MHz wall counter).
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int FRAGS = 16;        // 1 KB A fragments per block in LDS

template <bool FROM_LDS>
__global__ __launch_bounds__(256) void k_mfma_loop(const uint4 *__restrict__ a_src, const uint4 *__restrict__ b_src, int iters,
                                                   float *__restrict__ out, unsigned long long *__restrict__ ticks)
{
    __shared__ uint4 sa[FRAGS * 64];
    const int lane = threadIdx.x & 63;
    for (int i = threadIdx.x; i < FRAGS * 64; i += 256) sa[i] = a_src[i];
    bf16x8 b[2], a[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = __builtin_bit_cast(bf16x8, b_src[(threadIdx.x + 256 * i) % (FRAGS * 64)]);
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, a_src[(threadIdx.x * 3 + 64 * i) % (FRAGS * 64)]);
    f32x16 acc[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    __syncthreads();
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int f = 0; f < FRAGS; ++f) {
            bf16x8 av;
            if constexpr (FROM_LDS) av = __builtin_bit_cast(bf16x8, sa[f * 64 + lane]);
            else av = a[f & 3];
            acc[f & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b[f & 1], acc[f & 3], 0, 0, 0);
        }
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

// four independent 16-byte loads in flight per thread before the first store; streaming (non-temporal) stores
// How much vector-ALU work fits beside the MFMAs of the same SIMD: groups of {1 MFMA, NF v_fma_f32, NE v_exp_f32}, all
// independent of one another, three waves per SIMD (the attention kernel's occupancy), constant operands (full clock).
template <int NF, int NE, int WITH_MFMA>
__global__ __launch_bounds__(768) void k_coissue(float *__restrict__ out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(threadIdx.x * 0.001f + i);
        b[i] = (__bf16)(i * 0.5f);
    }
    f32x16 acc[2];
    for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (threadIdx.x + i) + 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if constexpr (WITH_MFMA) acc[r & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[r & 1], 0, 0, 0);
#pragma unroll
            for (int v = 0; v < NF; ++v) {
                const int i = (r * NF + v) & 15;
                x[i] = fmaf(x[i], 0.999f, 0.001f);
            }
#pragma unroll
            for (int v = 0; v < NE; ++v) {
                const int i = (r * NE + v + 5) & 15;
                x[i] = __builtin_amdgcn_exp2f(x[i]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = 0.f;
    for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    for (int i = 0; i < 16; ++i) s += x[i];
    out[(size_t)blockIdx.x * 768 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void k_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = src[i + j * stride];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v[j]), (u32x4 *)(dst + i + j * stride));
        }
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// the same bytes with every block working through a contiguous run of 64 KB at a time (DRAM pages and channels see
// long runs instead of one 4 KB line per block and trip), plain or streaming stores
template <bool NT>
__global__ __launch_bounds__(256) void k_copy_runs(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    constexpr size_t RUN = 4096;                      // 16-byte pieces per run: 64 KB
    const size_t n_runs = n16 / RUN;
    for (size_t r = blockIdx.x; r < n_runs; r += gridDim.x) {
        const uint4 *s = src + r * RUN;
        uint4 *d = dst + r * RUN;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = s[(t * 4 + j) * 256 + threadIdx.x];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (NT) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v[j]), (u32x4 *)(d + (t * 4 + j) * 256 + threadIdx.x));
                else d[(t * 4 + j) * 256 + threadIdx.x] = v[j];
            }
        }
    }
    for (size_t i = n_runs * RUN + (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// write-only: 64 KB runs per block, plain or streaming stores
template <bool NT>
__global__ __launch_bounds__(256) void k_fill_runs(uint4 *__restrict__ dst, size_t n16, uint32_t seed)
{
    constexpr size_t RUN = 4096;
    const size_t n_runs = n16 / RUN;
    const uint4 v = make_uint4(seed, threadIdx.x, blockIdx.x, seed ^ 0x9E3779B9u);
    for (size_t r = blockIdx.x; r < n_runs; r += gridDim.x) {
        uint4 *d = dst + r * RUN;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if constexpr (NT) __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4 *)(d + j * 256 + threadIdx.x));
            else d[j * 256 + threadIdx.x] = v;
        }
    }
}

__global__ __launch_bounds__(256) void k_read(const uint4 *__restrict__ src, size_t n16, uint32_t *__restrict__ out)
{
    uint32_t acc = 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345u) out[0] = acc;      // practically never: keeps the loads alive
}

#define CAL_TRY(e)                        \
    do {                                  \
        if ((e) != hipSuccess) return 1;  \
    } while (0)

}  // namespace

extern "C" {

// a_bits, b_bits: DEVICE, 16 KB each (FRAGS x 64 lanes x 8 bf16), the operands' bit patterns (zeros, constants or
// random values: the caller's choice).  blocks_per_cu blocks of four waves per compute unit.  Out (HOST): TFLOP/s
// and the shader clock in MHz during the loop.  Returns 0 on success.
__attribute__((visibility("default"))) int aifcal_mfma(const void *a_bits, const void *b_bits, int from_lds, int blocks_per_cu,
                                                       int iters, double *tflops, double *mhz)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount * blocks_per_cu;
    float *out = nullptr;
    unsigned long long *ticks = nullptr, h[2] = {0, 0};
    CAL_TRY(hipMalloc((void **)&out, (size_t)blocks * 256 * 4));
    CAL_TRY(hipMalloc((void **)&ticks, 16));
    hipEvent_t e0, e1;
    CAL_TRY(hipEventCreate(&e0));
    CAL_TRY(hipEventCreate(&e1));
    auto go = [&](int n) {
        if (from_lds)
            hipLaunchKernelGGL(k_mfma_loop<true>, dim3(blocks), dim3(256), 0, 0, (const uint4 *)a_bits, (const uint4 *)b_bits, n, out, ticks);
        else
            hipLaunchKernelGGL(k_mfma_loop<false>, dim3(blocks), dim3(256), 0, 0, (const uint4 *)a_bits, (const uint4 *)b_bits, n, out, ticks);
    };
    go(iters / 10 + 1);                       // warm-up
    CAL_TRY(hipDeviceSynchronize());
    CAL_TRY(hipEventRecord(e0, 0));
    go(iters);
    CAL_TRY(hipEventRecord(e1, 0));
    CAL_TRY(hipEventSynchronize(e1));
    float ms = 0.f;
    CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
    CAL_TRY(hipMemcpy(h, ticks, 16, hipMemcpyDeviceToHost));
    *tflops = (double)blocks * 4 * iters * FRAGS * 32768.0 / (ms * 1e-3) / 1e12;
    *mhz = h[1] ? 100.0 * (double)h[0] / (double)h[1] : 0.0;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(out);
    (void)hipFree(ticks);
    return 0;
}

// src, dst: DEVICE buffers of `bytes` (a multiple of 16).  Out (HOST): GB/s of the copy counting bytes read plus
// bytes written, and GB/s of a read-only pass.  Returns 0 on success.
__attribute__((visibility("default"))) int aifcal_copy(const void *src, void *dst, size_t bytes, int reps, double *gbs_copy,
                                                       double *gbs_read)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount * 8;
    const size_t n16 = bytes / 16;
    uint32_t *flag = nullptr;
    CAL_TRY(hipMalloc((void **)&flag, 4));
    hipEvent_t e0, e1;
    CAL_TRY(hipEventCreate(&e0));
    CAL_TRY(hipEventCreate(&e1));
    float ms = 0.f;
    hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, (const uint4 *)src, (uint4 *)dst, n16);
    CAL_TRY(hipDeviceSynchronize());
    CAL_TRY(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, (const uint4 *)src, (uint4 *)dst, n16);
    CAL_TRY(hipEventRecord(e1, 0));
    CAL_TRY(hipEventSynchronize(e1));
    CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
    *gbs_copy = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;
    // the best of the three forms of the copy is the figure reported
    for (int form = 0; form < 2; ++form) {
        auto go = [&]() {
            if (form) hipLaunchKernelGGL(k_copy_runs<true>, dim3(blocks), dim3(256), 0, 0, (const uint4 *)src, (uint4 *)dst, n16);
            else hipLaunchKernelGGL(k_copy_runs<false>, dim3(blocks), dim3(256), 0, 0, (const uint4 *)src, (uint4 *)dst, n16);
        };
        go();
        CAL_TRY(hipDeviceSynchronize());
        CAL_TRY(hipEventRecord(e0, 0));
        for (int i = 0; i < reps; ++i) go();
        CAL_TRY(hipEventRecord(e1, 0));
        CAL_TRY(hipEventSynchronize(e1));
        CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
        const double g = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;
        if (g > *gbs_copy) *gbs_copy = g;
    }
    CAL_TRY(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(k_read, dim3(blocks), dim3(256), 0, 0, (const uint4 *)src, n16, flag);
    CAL_TRY(hipEventRecord(e1, 0));
    CAL_TRY(hipEventSynchronize(e1));
    CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
    *gbs_read = (double)bytes * reps / (ms * 1e-3) / 1e9;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(flag);
    return 0;
}

// ns_out (HOST, 8 values): nanoseconds per group and SIMD of {MFMA}, {MFMA + 4 fma}, {MFMA + 4 exp}, {MFMA + 4 fma + 4 exp},
// {MFMA + 8 fma + 8 exp}, and without the MFMA {4 fma + 4 exp}, {8 fma + 8 exp}, {16 fma}.  Returns 0 on success.
__attribute__((visibility("default"))) int aifcal_coissue(double *ns_out)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount, iters = 4000;
    float *out = nullptr;
    CAL_TRY(hipMalloc((void **)&out, (size_t)blocks * 768 * 4));
    hipEvent_t e0, e1;
    CAL_TRY(hipEventCreate(&e0));
    CAL_TRY(hipEventCreate(&e1));
    auto timed = [&](auto kern, double *ns) -> int {
        for (int rep = 0; rep < 3; ++rep) hipLaunchKernelGGL(kern, dim3(blocks), dim3(768), 0, 0, out, iters);
        CAL_TRY(hipDeviceSynchronize());
        CAL_TRY(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(768), 0, 0, out, iters);
        CAL_TRY(hipEventRecord(e1, 0));
        CAL_TRY(hipEventSynchronize(e1));
        float ms = 0.f;
        CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
        *ns = ms * 1e6 / ((double)iters * 8 * 3);       // groups issued on one SIMD: 3 waves x iters x 8
        return 0;
    };
    for (int w = 0; w < 10; ++w) {                      // let the clocks rise
        double d;
        if (timed(k_coissue<4, 4, 1>, &d)) return 1;
    }
    if (timed(k_coissue<0, 0, 1>, ns_out + 0) || timed(k_coissue<4, 0, 1>, ns_out + 1) || timed(k_coissue<0, 4, 1>, ns_out + 2) ||
        timed(k_coissue<4, 4, 1>, ns_out + 3) || timed(k_coissue<8, 8, 1>, ns_out + 4) || timed(k_coissue<4, 4, 0>, ns_out + 5) ||
        timed(k_coissue<8, 8, 0>, ns_out + 6) || timed(k_coissue<16, 0, 0>, ns_out + 7))
        return 1;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    (void)hipFree(out);
    return 0;
}

// dst: DEVICE buffer of `bytes`.  Out (HOST): GB/s of a write-only pass (the better of plain and streaming stores).
__attribute__((visibility("default"))) int aifcal_fill(void *dst, size_t bytes, int reps, double *gbs_write)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount * 8;
    const size_t n16 = bytes / 16;
    hipEvent_t e0, e1;
    CAL_TRY(hipEventCreate(&e0));
    CAL_TRY(hipEventCreate(&e1));
    *gbs_write = 0.0;
    for (int form = 0; form < 2; ++form) {
        auto go = [&](int i) {
            if (form) hipLaunchKernelGGL(k_fill_runs<true>, dim3(blocks), dim3(256), 0, 0, (uint4 *)dst, n16, (uint32_t)i);
            else hipLaunchKernelGGL(k_fill_runs<false>, dim3(blocks), dim3(256), 0, 0, (uint4 *)dst, n16, (uint32_t)i);
        };
        go(0);
        CAL_TRY(hipDeviceSynchronize());
        CAL_TRY(hipEventRecord(e0, 0));
        for (int i = 0; i < reps; ++i) go(i + 1);
        CAL_TRY(hipEventRecord(e1, 0));
        CAL_TRY(hipEventSynchronize(e1));
        float ms = 0.f;
        CAL_TRY(hipEventElapsedTime(&ms, e0, e1));
        const double g = (double)bytes * reps / (ms * 1e-3) / 1e9;
        if (g > *gbs_write) *gbs_write = g;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return 0;
}

}  // extern "C"
