// The key-tile loop of the resident target-attention kernel (Eq. 3 with the candidate as the query; heads of 64,
// 16 key tiles per item: the default workload's shape) in isolation, and the cost of its vector instructions one by one --
// measurement tooling, part of libaif_calib, not of libaif.
//   aifcal_attn_loop:  K and V fragments of one request resident in LDS, every wave walks items of 16 key tiles with
//                      the kernel's schedule (score product of tile t + 1 interleaved with the exponentials of tile t,
//                      conversions, second product with the row sums' fp32 adds between its MFMAs).  Parts of the loop can be left
//                      out (timing only: the results are then meaningless), which prices each part; the operand values
//                      come from the caller (zeros hold the full clock, random values meet the power limit).
//   aifcal_valu_costs: sixteen independent instructions of one kind per group, three waves per SIMD, with and without
//                      one MFMA per group: what an instruction costs and how much of an MFMA it hides.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int NKT = 16, FR = 8, JS = 4, FT = 2;         // key tiles per item; 1 KB fragments per key tile: 4 of K, 4 of V
constexpr int LDS_BYTES = NKT * FR * 1024;

// parts of the loop that can be left out
constexpr int NO_SUMS = 1, NO_EXP = 2, NO_LDS = 4, NO_CVT = 8, SUMS_AS_DOTS = 16;

template <int I0, int N> __device__ __forceinline__ float sum_pairs(const bf16x8 &a, float acc)
{
    bf16x2 one;
    one[0] = (__bf16)1.0f;
    one[1] = (__bf16)1.0f;
#pragma unroll
    for (int i = I0; i < I0 + N; ++i) {
        bf16x2 p;
        p[0] = a[2 * i];
        p[1] = a[2 * i + 1];
        acc = __builtin_amdgcn_fdot2_f32_bf16(one, p, acc, false);
    }
    return acc;
}

#define SLOT_END __builtin_amdgcn_sched_barrier(0)
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

template <int WAVES, int LEAVE_OUT>
__global__ __launch_bounds__(WAVES * 64) void k_attn_loop(const uint4 *__restrict__ kv, const uint4 *__restrict__ qsrc,
                                                          float *__restrict__ out, int items)
{
    extern __shared__ __align__(16) char lds[];
    for (int i = threadIdx.x; i < LDS_BYTES / 16; i += WAVES * 64) ((uint4 *)lds)[i] = kv[i];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const char *kbase = lds + lane * 16;
    bf16x8 q[JS];
    for (int j = 0; j < JS; ++j) q[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j) & 4095]);
    float tot = 0.f;
    for (int it = 0; it < items; ++it) {
        f32x16 O[FT];
        for (int ft = 0; ft < FT; ++ft)
            for (int i = 0; i < 16; ++i) O[ft][i] = 0.f;
        float l = 0.f, l4[4] = {0.f, 0.f, 0.f, 0.f};
        bf16x8 kf[JS], vf[2 * FT];
        f32x16 S, S1;
        auto step = [&](int kt, const f32x16 &Sin, f32x16 &Sout, bool next) {
            const char *vbase = kbase + (kt * FR + JS) * 1024;
            if constexpr (!(LEAVE_OUT & NO_LDS)) {
#pragma unroll
                for (int i = 0; i < 2 * FT; ++i) vf[i] = *(const bf16x8 *)(vbase + i * 1024);
            }
            const int kn = kt + 2 < NKT ? kt + 2 : NKT - 1;
            SLOT_END;
            float p[16];
#pragma unroll
            for (int j = 0; j < JS; ++j) {
                if (next) {
                    if (j == 0) {
                        f32x16 Z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) Z[i] = 0.f;
                        Sout = MFMA(kf[0], q[0], Z);
                    } else
                        Sout = MFMA(kf[j], q[j], Sout);
                    if constexpr (!(LEAVE_OUT & NO_LDS)) kf[j] = *(const bf16x8 *)(kbase + (kn * FR + j) * 1024);
                }
#pragma unroll
                for (int v = 4 * j; v < 4 * (j + 1); ++v) {
                    if constexpr (LEAVE_OUT & NO_EXP) p[v] = Sin[v];
                    else {
                        p[v] = __builtin_amdgcn_exp2f(Sin[v]);
                        asm volatile("" : "+v"(p[v]));
                    }
                }
                SLOT_END;
            }
            bf16x8 P0, P1;
            if constexpr (LEAVE_OUT & NO_CVT) {
#pragma unroll
                for (int v = 0; v < 16; ++v) asm volatile("" ::"v"(p[v]));
                P0 = q[0];
                P1 = q[1];
            } else {
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    P0[v] = (__bf16)p[v];
                    P1[v] = (__bf16)p[8 + v];
                }
            }
            SLOT_END;
#pragma unroll
            for (int i = 0; i < 2 * FT; ++i) {
                O[i % FT] = MFMA(vf[i], i < FT ? P0 : P1, O[i % FT]);
                if constexpr (LEAVE_OUT & SUMS_AS_DOTS) {       // the rounded weights, two a v_dot2c_f32_bf16
                    if (i == 0) l = sum_pairs<0, 2>(P0, l);
                    if (i == 1) l = sum_pairs<2, 2>(P0, l);
                    if (i == 2) l = sum_pairs<0, 2>(P1, l);
                    if (i == 3) l = sum_pairs<2, 2>(P1, l);
                } else if constexpr (!(LEAVE_OUT & NO_SUMS)) {  // the kernel's: fp32 adds of the weights before rounding
#pragma unroll
                    for (int v = 4 * i; v < 4 * (i + 1); ++v) l4[v & 3] += p[v];
                }
                SLOT_END;
            }
        };
#pragma unroll
        for (int j = 0; j < JS; ++j) kf[j] = *(const bf16x8 *)(kbase + j * 1024);
#pragma unroll
        for (int i = 0; i < 2 * FT; ++i) vf[i] = *(const bf16x8 *)(kbase + (JS + i) * 1024);
#pragma unroll
        for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
        for (int j = 0; j < JS; ++j) S = MFMA(kf[j], q[j], S);
#pragma unroll
        for (int j = 0; j < JS; ++j) kf[j] = *(const bf16x8 *)(kbase + (FR + j) * 1024);
        SLOT_END;
        int kt = 0;
        for (; kt + 2 < NKT; kt += 2) {
            step(kt, S, S1, true);
            step(kt + 1, S1, S, true);
        }
        step(kt, S, S1, true);
        step(kt + 1, S1, S, false);
        if constexpr (!(LEAVE_OUT & SUMS_AS_DOTS)) l = (LEAVE_OUT & NO_SUMS) ? 1.0f + O[0][0] : (l4[0] + l4[1]) + (l4[2] + l4[3]);
        l += __shfl_xor(l, 32, 64);
        const float inv = 1.0f / l;
        for (int ft = 0; ft < FT; ++ft)
            for (int i = 0; i < 16; ++i) tot += O[ft][i] * inv;
#pragma unroll
        for (int j = 0; j < JS; ++j) q[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j + 64 * (it + 1)) & 4095]);
    }
    out[(size_t)blockIdx.x * WAVES * 64 + threadIdx.x] = tot;
}

// The same work with TWO 32-candidate tiles a wave (tiles a and b), each the other's partner in the pipeline: while the
// vector ALU takes the exponentials of one tile's scores the matrix cores form the other's, and a K or V fragment read
// from LDS serves both -- half the LDS reads per candidate, one S buffer per tile instead of two.
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_attn_loop2(const uint4 *__restrict__ kv, const uint4 *__restrict__ qsrc,
                                                           float *__restrict__ out, int items)
{
    extern __shared__ __align__(16) char lds[];
    for (int i = threadIdx.x; i < LDS_BYTES / 16; i += WAVES * 64) ((uint4 *)lds)[i] = kv[i];
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const char *kbase = lds + lane * 16;
    bf16x8 qa[JS], qb[JS];
    for (int j = 0; j < JS; ++j) {
        qa[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j) & 4095]);
        qb[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j + 2048) & 4095]);
    }
    float tot = 0.f;
    for (int it = 0; it < items; ++it) {
        f32x16 Oa[FT], Ob[FT];
        for (int ft = 0; ft < FT; ++ft)
            for (int i = 0; i < 16; ++i) Oa[ft][i] = Ob[ft][i] = 0.f;
        float la[4] = {0.f, 0.f, 0.f, 0.f}, lb[4] = {0.f, 0.f, 0.f, 0.f};
        bf16x8 kf[JS], vf[2 * FT];
        f32x16 Sa, Sb;
        // one phase: the S product of `other` (scores into So, query qo) beside the exponentials of Sin, then the
        // second product of Sin's tile into O; REFILL_K: the K fragments are the next key tile's from here on;
        // REFILL_V: so are the V fragments
        auto phase = [&](const f32x16 &Sin, f32x16 &So, const bf16x8(&qo)[JS], f32x16(&O)[FT], float(&l4)[4], bool s_next, int k_refill,
                         int v_refill) {
            float p[16];
#pragma unroll
            for (int j = 0; j < JS; ++j) {
                if (s_next) {
                    if (j == 0) {
                        f32x16 Z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) Z[i] = 0.f;
                        So = MFMA(kf[0], qo[0], Z);
                    } else
                        So = MFMA(kf[j], qo[j], So);
                    if (k_refill >= 0) kf[j] = *(const bf16x8 *)(kbase + (k_refill * FR + j) * 1024);
                }
#pragma unroll
                for (int v = 4 * j; v < 4 * (j + 1); ++v) {
                    p[v] = __builtin_amdgcn_exp2f(Sin[v]);
                    asm volatile("" : "+v"(p[v]));
                }
                SLOT_END;
            }
            bf16x8 P0, P1;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                P0[v] = (__bf16)p[v];
                P1[v] = (__bf16)p[8 + v];
            }
            SLOT_END;
#pragma unroll
            for (int i = 0; i < 2 * FT; ++i) {
                O[i % FT] = MFMA(vf[i], i < FT ? P0 : P1, O[i % FT]);
                if (v_refill >= 0) vf[i] = *(const bf16x8 *)(kbase + (v_refill * FR + JS + i) * 1024);
#pragma unroll
                for (int v = 4 * i; v < 4 * (i + 1); ++v) l4[v & 3] += p[v];
                SLOT_END;
            }
        };
#pragma unroll
        for (int j = 0; j < JS; ++j) kf[j] = *(const bf16x8 *)(kbase + j * 1024);
#pragma unroll
        for (int i = 0; i < 2 * FT; ++i) vf[i] = *(const bf16x8 *)(kbase + (JS + i) * 1024);
#pragma unroll
        for (int i = 0; i < 16; ++i) Sa[i] = 0.f;
#pragma unroll
        for (int j = 0; j < JS; ++j) Sa = MFMA(kf[j], qa[j], Sa);
        SLOT_END;
        for (int kt = 0; kt < NKT; ++kt) {
            const int kn = kt + 1 < NKT ? kt + 1 : NKT - 1;
            // tile a's weights and second product beside tile b's scores (same key tile); K moves on to the next key tile
            phase(Sa, Sb, qb, Oa, la, true, kn, -1);
            // tile b's weights and second product beside tile a's scores of the next key tile; V moves on
            phase(Sb, Sa, qa, Ob, lb, kt + 1 < NKT, -1, kn);
        }
        float l0 = (la[0] + la[1]) + (la[2] + la[3]), l1 = (lb[0] + lb[1]) + (lb[2] + lb[3]);
        l0 += __shfl_xor(l0, 32, 64);
        l1 += __shfl_xor(l1, 32, 64);
        const float i0 = 1.0f / l0, i1 = 1.0f / l1;
        for (int ft = 0; ft < FT; ++ft)
            for (int i = 0; i < 16; ++i) tot += Oa[ft][i] * i0 + Ob[ft][i] * i1;
#pragma unroll
        for (int j = 0; j < JS; ++j) {
            qa[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j + 64 * (it + 1)) & 4095]);
            qb[j] = __builtin_bit_cast(bf16x8, qsrc[(threadIdx.x * JS + j + 2048 + 64 * (it + 1)) & 4095]);
        }
    }
    out[(size_t)blockIdx.x * WAVES * 64 + threadIdx.x] = tot;
}

// OP: 0 v_fma_f32, 1 v_exp_f32, 2 v_cvt_pk_bf16_f32, 3 v_dot2c_f32_bf16
template <int OP, int WITH_MFMA>
__global__ __launch_bounds__(768) void k_valu_cost(float *__restrict__ out, int iters)
{
    float x[16];
    unsigned y[16];
    for (int i = 0; i < 16; ++i) {
        x[i] = 0.001f * (threadIdx.x + i) + 0.5f;
        y[i] = 0x3f803f80u + i;
    }
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(threadIdx.x * 0.001f + i);
        b[i] = (__bf16)(i * 0.5f);
    }
    f32x16 acc[2];
    for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if constexpr (WITH_MFMA) acc[r & 1] = MFMA(a, b, acc[r & 1]);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if constexpr (OP == 0) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(x[i]) : "v"(x[(i + 1) & 15]));
                if constexpr (OP == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
                if constexpr (OP == 2) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(y[i]) : "v"(x[i]), "v"(x[(i + 1) & 15]));
                if constexpr (OP == 3) asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(x[i]) : "v"(y[i]), "v"(y[(i + 1) & 15]));
            }
            SLOT_END;
        }
    }
    float s = 0.f;
    for (int n = 0; n < 2; ++n)
        for (int i = 0; i < 16; ++i) s += acc[n][i];
    for (int i = 0; i < 16; ++i) s += x[i] + (float)y[i];
    out[(size_t)blockIdx.x * 768 + threadIdx.x] = s;
}

#define CAL_TRY(e)                        \
    do {                                  \
        if ((e) != hipSuccess) return 1;  \
    } while (0)

struct Timer {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int init() { return hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess; }
    ~Timer()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace

extern "C" {

// kv: DEVICE, 128 KB of bf16 (the request's K and V fragments); q: DEVICE, 64 KB of bf16 (queries).  ns_out (HOST, 11
// values): nanoseconds per key tile and SIMD of the whole loop at 3, 2 and 1 waves per SIMD, then at 3 waves per SIMD
// without the row sums, without the exponentials, without the conversions, without the LDS reads, with the MFMAs
// alone, with the row sums as two-term dot products of the rounded weights (eight v_dot2c_f32_bf16 a key tile: the
// kernel's former way), the whole loop once more, and two candidate tiles a wave at 2 waves per SIMD (k_attn_loop2; per 32
// candidates).  Returns 0 on success.
__attribute__((visibility("default"))) int aifcal_attn_loop(const void *kv, const void *q, double *ns_out)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount, items = 64;
    float *out = nullptr;
    CAL_TRY(hipMalloc((void **)&out, (size_t)blocks * 768 * 4));
    Timer t;
    if (t.init()) return 1;
    auto timed = [&](auto kern, int waves, double *ns) -> int {
        CAL_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES));
        for (int rep = 0; rep < 3; ++rep)
            hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * 64), LDS_BYTES, 0, (const uint4 *)kv, (const uint4 *)q, out, items);
        CAL_TRY(hipDeviceSynchronize());
        CAL_TRY(hipEventRecord(t.e0, 0));
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * 64), LDS_BYTES, 0, (const uint4 *)kv, (const uint4 *)q, out, items);
        CAL_TRY(hipEventRecord(t.e1, 0));
        CAL_TRY(hipEventSynchronize(t.e1));
        float ms = 0.f;
        CAL_TRY(hipEventElapsedTime(&ms, t.e0, t.e1));
        *ns = ms * 1e6 / ((double)items * NKT * (waves / 4));
        return 0;
    };
    double warm;
    for (int w = 0; w < 6; ++w)                         // let the clocks settle
        if (timed(k_attn_loop<12, 0>, 12, &warm)) return 1;
    int rc = timed(k_attn_loop<12, 0>, 12, ns_out + 0) || timed(k_attn_loop<8, 0>, 8, ns_out + 1) || timed(k_attn_loop<4, 0>, 4, ns_out + 2) ||
             timed(k_attn_loop<12, NO_SUMS>, 12, ns_out + 3) || timed(k_attn_loop<12, NO_EXP>, 12, ns_out + 4) ||
             timed(k_attn_loop<12, NO_CVT>, 12, ns_out + 5) || timed(k_attn_loop<12, NO_LDS>, 12, ns_out + 6) ||
             timed(k_attn_loop<12, NO_SUMS | NO_EXP | NO_CVT | NO_LDS>, 12, ns_out + 7) ||
             timed(k_attn_loop<12, SUMS_AS_DOTS>, 12, ns_out + 8) || timed(k_attn_loop<12, 0>, 12, ns_out + 9) ||
             timed(k_attn_loop2<8>, 8, ns_out + 10);
    ns_out[10] *= 0.5;          // two candidate tiles a wave: per 32 candidates, like the others
    (void)hipFree(out);
    return rc;
}

// ns_out (HOST, 8 values): nanoseconds per group of sixteen instructions and SIMD for v_fma_f32, v_exp_f32,
// v_cvt_pk_bf16_f32, v_dot2c_f32_bf16, then the same four with one 32x32x16 bf16 MFMA per group.  Returns 0 on success.
__attribute__((visibility("default"))) int aifcal_valu_costs(double *ns_out)
{
    int dev = 0;
    hipDeviceProp_t prop;
    CAL_TRY(hipGetDevice(&dev));
    CAL_TRY(hipGetDeviceProperties(&prop, dev));
    const int blocks = prop.multiProcessorCount, iters = 4000;
    float *out = nullptr;
    CAL_TRY(hipMalloc((void **)&out, (size_t)blocks * 768 * 4));
    Timer t;
    if (t.init()) return 1;
    auto timed = [&](auto kern, double *ns) -> int {
        for (int rep = 0; rep < 3; ++rep) hipLaunchKernelGGL(kern, dim3(blocks), dim3(768), 0, 0, out, iters);
        CAL_TRY(hipDeviceSynchronize());
        CAL_TRY(hipEventRecord(t.e0, 0));
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(768), 0, 0, out, iters);
        CAL_TRY(hipEventRecord(t.e1, 0));
        CAL_TRY(hipEventSynchronize(t.e1));
        float ms = 0.f;
        CAL_TRY(hipEventElapsedTime(&ms, t.e0, t.e1));
        *ns = ms * 1e6 / ((double)iters * 4 * 3);       // groups issued on one SIMD: 3 waves x iters x 4
        return 0;
    };
    double warm;
    for (int w = 0; w < 10; ++w)
        if (timed(k_valu_cost<1, 0>, &warm)) return 1;
    int rc = timed(k_valu_cost<0, 0>, ns_out + 0) || timed(k_valu_cost<1, 0>, ns_out + 1) || timed(k_valu_cost<2, 0>, ns_out + 2) ||
             timed(k_valu_cost<3, 0>, ns_out + 3) || timed(k_valu_cost<0, 1>, ns_out + 4) || timed(k_valu_cost<1, 1>, ns_out + 5) ||
             timed(k_valu_cost<2, 1>, ns_out + 6) || timed(k_valu_cost<3, 1>, ns_out + 7);
    (void)hipFree(out);
    return rc;
}

}  // extern "C"
