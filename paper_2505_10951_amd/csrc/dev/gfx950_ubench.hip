// Micro-benchmarks for gfx950 (MI355X) that fixed design choices of the attention and projection kernels: LDS read
// rates of ds_read_b128 for the lane-to-address patterns that were considered, the issue rate of the 32x32x16 bf16
// matrix instruction with one and two wavefronts per SIMD, the cost of the vector instructions of the softmax, how
// matrix and vector work of different wavefronts overlap, and a synthetic 64-key tile step (operand reads through a
// rolling window, two products, dependent softmax, copies, scalar overhead, barrier) to see what the hardware allows
// the real step.  Development aid, not part of the library: nothing links against it.  All kernels read and write
// only their own LDS and the buffers allocated below; LDS content and results are meaningless.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_2505_10951_amd/csrc/dev/gfx950_ubench.hip -o /tmp/gfx950_ubench && /tmp/gfx950_ubench
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)

// ---- unit rates ------------------------------------------------------------------------------------------------
// mode: address pattern for ds_read_b128; 8 independent reads in flight per wave
__global__ void __launch_bounds__(512) lds_read_kernel(int mode, int iters, unsigned long long *cycles, uint4 *sink)
{
    __shared__ __attribute__((aligned(1024))) char smem[65536];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 65536 / 16; i += blockDim.x) reinterpret_cast<uint4 *>(smem)[i] = make_uint4(i, i + 1, i + 2, i + 3);
    __syncthreads();
    int off;
    switch (mode) {
        case 0: off = lane * 16; break;                                           // linear
        case 1: off = (lane & 31) * 32 + (lane >> 5) * 16; break;                 // 32B stride, halves interleaved
        case 2: off = (lane & 15) * 16 + (lane >> 4) * 512; break;                // 16 lanes contiguous, groups 512 apart
        case 3: off = (lane & 7) * 16 + (lane >> 3) * 256; break;                 // 8 lanes contiguous, groups 256 apart
        case 4: off = lane * 256; break;                                          // worst: same banks
        case 5: off = ((lane & 31) * 16) + (lane >> 5) * 1024; break;             // halves 1 KiB apart
        case 6: off = (lane & 3) * 16 + (lane >> 2) * 64; break;                  // = linear
        case 7: off = (lane * 16) ^ ((lane >> 4) << 4); break;
        case 8: off = (lane & 31) * 128 + (((lane >> 5) ^ (lane & 7) ^ ((lane >> 3) & 1)) * 16); break;   // gemm swizzle
        case 9: off = (lane & 31) * 128 + (((lane >> 5) ^ ((lane >> 1) & 7)) * 16); break;
        case 10: off = (lane & 31) * 128 + (((lane >> 5) ^ (lane & 7)) * 16); break;
        case 11: off = (lane & 31) * 128 + (lane >> 5) * 16; break;   // no swizzle
        default: off = lane * 16; break;
    }
    off = (off + wave * 1024) & 0x3FF0;
    const unsigned addr = (unsigned)(size_t)(smem) + off;   // LDS byte address (flat->lds low bits)
    typedef __attribute__((ext_vector_type(4))) unsigned int u4;
    u4 r0, r1, r2, r3, r4, r5, r6, r7;
    u4 acc = {0, 0, 0, 0};
    __syncthreads();
    unsigned long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:4096\n ds_read_b128 %2, %8 offset:8192\n ds_read_b128 %3, %8 offset:12288\n"
            "ds_read_b128 %4, %8 offset:16384\n ds_read_b128 %5, %8 offset:20480\n ds_read_b128 %6, %8 offset:24576\n ds_read_b128 %7, %8 offset:28672\n"
            "s_waitcnt lgkmcnt(0)\n"
            : "=v"(r0), "=v"(r1), "=v"(r2), "=v"(r3), "=v"(r4), "=v"(r5), "=v"(r6), "=v"(r7) : "v"(addr) : "memory");
        acc ^= r0 ^ r7;
    }
    unsigned long long t1 = clock64();
    if (lane == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
    acc ^= r1 ^ r2 ^ r3 ^ r4 ^ r5 ^ r6;
    sink[blockIdx.x * 512 + tid] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
}

template <int NCHAIN>
__global__ void __launch_bounds__(512) mfma_kernel(int iters, unsigned long long *cycles, float *sink)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(lane + i); b[i] = (__bf16)(float)(lane - i); }
    f32x16 acc[NCHAIN];
    for (int c = 0; c < NCHAIN; ++c) for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    unsigned long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) acc[u % NCHAIN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[u % NCHAIN], 0, 0, 0);
    }
    unsigned long long t1 = clock64();
    if (lane == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
    float s = 0;
    for (int c = 0; c < NCHAIN; ++c) for (int r = 0; r < 16; ++r) s += acc[c][r];
    sink[blockIdx.x * 512 + tid] = s;
}

// op 0: v_exp_f32, 1: v_fma_f32, 2: cvt_pk_bf16, 3: v_max_f32, 4: dot2c
template <int op>
__global__ void __launch_bounds__(512) valu_kernel(int iters, unsigned long long *cycles, float *sink)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * (lane + i);
    unsigned long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (op == 0) x[i] = __builtin_amdgcn_exp2f(x[i]);
                else if (op == 1) x[i] = x[i] * 0.999f + 0.001f;
                else if (op == 3) x[i] = fmaxf(x[i], x[(i + 1) & 7] * 0.5f);
                else if (op == 2) { typedef __attribute__((ext_vector_type(2))) __bf16 b2; b2 p; p[0] = (__bf16)x[i]; p[1] = (__bf16)x[(i + 1) & 7]; x[i] = __builtin_bit_cast(float, p); }
                else { typedef __attribute__((ext_vector_type(2))) __bf16 b2; b2 p = __builtin_bit_cast(b2, x[i]); b2 one; one[0] = (__bf16)1.f; one[1] = (__bf16)1.f; x[i] = __builtin_amdgcn_fdot2_f32_bf16(p, one, x[i], false); }
            }
        }
    }
    unsigned long long t1 = clock64();
    if (lane == 0) cycles[blockIdx.x * 8 + wave] = t1 - t0;
    float s = 0;
    for (int i = 0; i < 8; ++i) s += x[i];
    sink[blockIdx.x * 512 + tid] = s;
}

static int run_unit_rates()
{
    unsigned long long *d_cyc;
    void *d_sink;
    const int blocks = 256;
    CHECK(hipMalloc(&d_cyc, blocks * 8 * sizeof(unsigned long long)));
    CHECK(hipMalloc(&d_sink, blocks * 512 * 16));
    std::vector<unsigned long long> h(blocks * 8);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    auto report = [&](const char *name, double units_per_wave_iter, int iters, int waves, const char *unit) {
        CHECK(hipDeviceSynchronize());
        CHECK(hipMemcpy(h.data(), d_cyc, blocks * 8 * sizeof(unsigned long long), hipMemcpyDeviceToHost));
        double avg = 0;
        for (int i = 0; i < waves; ++i) avg += (double)h[i];
        avg /= waves;
        printf("%-44s cycles/wave %10.0f  -> %8.2f %s per clk per CU (%d waves/CU)\n", name, avg, units_per_wave_iter * iters * waves / avg, unit, waves);
    };
    const int iters = 2000;
    for (int threads : {256, 512}) {
        for (int mode = 0; mode < 12; ++mode) {
            CHECK(hipEventRecord(e0));
            hipLaunchKernelGGL(lds_read_kernel, dim3(blocks), dim3(threads), 0, 0, mode, iters, d_cyc, (uint4 *)d_sink);
            CHECK(hipEventRecord(e1));
            char nm[64]; snprintf(nm, 64, "ds_read_b128 pattern %d threads %d", mode, threads);
            report(nm, 8.0 * 1024, iters, threads / 64, "B");
            { float ms; CHECK(hipEventElapsedTime(&ms, e0, e1)); printf("   wall %.3f ms -> %.1f B/ns per CU\n", ms, 8.0*1024*iters*(threads/64)/ (ms*1e6)); }
        }

    }
    if (getenv("LDS_ONLY")) return 0;
    for (int threads : {256, 512}) {
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(mfma_kernel<1>, dim3(blocks), dim3(threads), 0, 0, iters, d_cyc, (float *)d_sink);
        CHECK(hipEventRecord(e1));
        report("mfma 32x32x16 bf16 chain=1", 16.0 * 32768, iters, threads / 64, "flop");
        float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
        printf("   wall %.3f ms -> %.1f TFLOP/s whole chip\n", ms, 16.0 * 32768 * iters * (threads / 64) * blocks / ms / 1e9);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(mfma_kernel<4>, dim3(blocks), dim3(threads), 0, 0, iters, d_cyc, (float *)d_sink);
        CHECK(hipEventRecord(e1));
        report("mfma 32x32x16 bf16 chain=4", 16.0 * 32768, iters, threads / 64, "flop");
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        printf("   wall %.3f ms -> %.1f TFLOP/s whole chip\n", ms, 16.0 * 32768 * iters * (threads / 64) * blocks / ms / 1e9);
    }
    const char *opn[] = {"v_exp_f32", "v_fma_f32", "v_cvt_pk_bf16_f32", "v_max_f32(+mul)", "v_dot2c_f32_bf16"};
#define VALU(op) { CHECK(hipEventRecord(e0)); hipLaunchKernelGGL(valu_kernel<op>, dim3(blocks), dim3(256), 0, 0, iters, d_cyc, (float *)d_sink); CHECK(hipEventRecord(e1)); report(opn[op], 32.0 * 64, iters, 4, "lane-ops"); float ms; CHECK(hipEventElapsedTime(&ms, e0, e1)); printf("   wall %.3f ms -> %.2f wave-instr/ns per CU\n", ms, 32.0*iters*4/(ms*1e6)); }
    VALU(0) VALU(1) VALU(2) VALU(3) VALU(4)
    return 0;
}

// ---- overlap and step models ------------------------------------------------------------------------------------
__device__ inline void mfma_phase(f32x16 &acc, const bf16x8 &a, const bf16x8 &b, int n)
{
#pragma unroll
    for (int u = 0; u < 16; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
__device__ inline void valu_phase(float (&x)[32], float c, float m)
{
#pragma unroll
    for (int i = 0; i < 32; ++i) x[i] = __builtin_amdgcn_exp2f(x[i] * c - m);
#pragma unroll
    for (int i = 0; i < 32; i += 2) { x[i] = x[i] + x[i + 1]; x[i + 1] = x[i + 1] * 0.5f + x[i]; }
}

// mode 0: all waves MFMA only; 1: all waves VALU only; 2: waves 0-3 MFMA only, 4-7 VALU only;
// 3: every wave [MFMA16, VALU] same order; 4: waves 4-7 start with VALU (opposite phase); 5: mode 3 + setprio on waves 0-3
template <int MODE>
__global__ void __launch_bounds__(512) overlap_kernel(int iters, float *sink)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(lane + i); b[i] = (__bf16)(0.01f * (lane - i)); }
    f32x16 acc;
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float x[32];
    for (int i = 0; i < 32; ++i) x[i] = 0.001f * (lane + i);
    const bool first = wave < 4;
    if (MODE == 5) { if (first) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0); }
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0 || (MODE == 2 && first)) { mfma_phase(acc, a, b, 16); mfma_phase(acc, a, b, 16); }
        else if (MODE == 1 || (MODE == 2 && !first)) { valu_phase(x, 0.999f, 0.001f); }
        else if (MODE == 3 || MODE == 5) { mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); valu_phase(x, 0.999f, 0.001f); __builtin_amdgcn_sched_barrier(0); mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); }
        else if (MODE == 4) {
            if (first) { mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); valu_phase(x, 0.999f, 0.001f); __builtin_amdgcn_sched_barrier(0); mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); }
            else { valu_phase(x, 0.999f, 0.001f); __builtin_amdgcn_sched_barrier(0); mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); mfma_phase(acc, a, b, 16); __builtin_amdgcn_sched_barrier(0); }
        }
    }
    float s = 0;
    for (int r = 0; r < 16; ++r) s += acc[r];
    for (int i = 0; i < 32; ++i) s += x[i];
    sink[blockIdx.x * 512 + tid] = s;
}

// Closer to the kernel: per iteration K-operand reads (rolling window of 8), 16 MFMA, VALU, V-operand reads, 16 MFMA,
// optional barrier.  LDS content is irrelevant.
template <bool BARRIER, bool LDSREAD, int NV, bool DEP, int NDMA = 0, int NSALU = 0>
__global__ void __launch_bounds__(512) step_kernel(int iters, float *sink, const char *gsrc = nullptr)
{
    __shared__ __attribute__((aligned(1024))) char smem[65536];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < 65536 / 16; i += blockDim.x) reinterpret_cast<uint4 *>(smem)[i] = make_uint4(0x3f803f80, 0x3f803f80, 0x3f803f80, 0x3f803f80);
    __syncthreads();
    bf16x8 b;
    for (int i = 0; i < 8; ++i) b[i] = (__bf16)(0.01f * (lane - i));
    f32x16 acc, acc2;
    for (int r = 0; r < 16; ++r) { acc[r] = 0.f; acc2[r] = 0.f; }
    float x[32];
    for (int i = 0; i < 32; ++i) x[i] = 0.001f * (lane + i);
    bf16x8 frag[8];
    for (int i = 0; i < 8; ++i) frag[i] = b;
    int sacc_s = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int it = 0; it < iters; ++it) {
        const char *buf = smem + (it & 1) * 32768 + lane * 16;
        if (NDMA > 0) {
            char *other = smem + ((it + 1) & 1) * 32768;
#pragma unroll
            for (int j = 0; j < NDMA; ++j) {
                const int u = wave_u + 8 * j;
                const char *src = gsrc + (size_t)((blockIdx.x * 7 + it * 3 + u) & 1023) * 1024 + lane * 16;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)(other + (u & 31) * 1024), 16, 0, 0);
            }
        }
        if (NSALU > 0) {
#pragma unroll
            for (int j = 0; j < NSALU; ++j) { sacc_s = sacc_s * 3 + j; asm volatile("" : "+s"(sacc_s)); }
        }
        if (LDSREAD) {
#pragma unroll
            for (int i = 0; i < 8; ++i) frag[i] = *reinterpret_cast<const bf16x8 *>(buf + i * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        f32x16 accb;
        if (DEP) { for (int r = 0; r < 16; ++r) { acc[r] = 0.f; accb[r] = 0.f; } }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (DEP && i >= 8) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i & 7], b, accb, 0, 0, 0);
            else acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i & 7], b, acc, 0, 0, 0);
            if (LDSREAD) frag[i & 7] = *reinterpret_cast<const bf16x8 *>(buf + (i + 8) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        bf16x8 pb[4] = {b, b, b, b};
        if (DEP) {
            typedef __attribute__((ext_vector_type(2))) __bf16 b2;
            float psum = 0.f;
            b2 ones; ones[0] = (__bf16)1.f; ones[1] = (__bf16)1.f;
#pragma unroll
            for (int r = 0; r < 32; r += 2) {
                b2 pk;
                const float s0 = (r < 16) ? acc[r] : accb[r - 16], s1 = (r < 16) ? acc[r + 1] : accb[r - 15];
                pk[0] = (__bf16)__builtin_amdgcn_exp2f(s0 * 0.01f - x[0]);
                pk[1] = (__bf16)__builtin_amdgcn_exp2f(s1 * 0.01f - x[0]);
                psum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, psum, false);
                pb[r >> 3][r & 7] = pk[0]; pb[r >> 3][(r & 7) + 1] = pk[1];
            }
            x[1] += psum;
        } else {
#pragma unroll
            for (int v = 0; v < NV; ++v) valu_phase(x, 0.999f, 0.001f);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[i & 7], pb[i >> 2], acc2, 0, 0, 0);
            if (LDSREAD && i < 8) frag[i & 7] = *reinterpret_cast<const bf16x8 *>(buf + (i + 24) * 1024);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (NDMA > 0) __builtin_amdgcn_s_waitcnt(0x0F70);
        if (BARRIER) __syncthreads();
    }
    float s = (float)sacc_s;
    for (int r = 0; r < 16; ++r) s += acc[r] + acc2[r];
    for (int i = 0; i < 32; ++i) s += x[i];
    sink[blockIdx.x * 512 + tid] = s;
}

template <bool BARRIER, bool LDSREAD, int NV, bool DEP = false, int NDMA = 0, int NSALU = 0>
void run_step(const char *name, int threads, float *d_sink, const char *gsrc = nullptr)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int iters = 4000, blocks = 256;
    hipLaunchKernelGGL((step_kernel<BARRIER, LDSREAD, NV, DEP, NDMA, NSALU>), dim3(blocks), dim3(threads), 0, 0, 100, d_sink, gsrc);
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL((step_kernel<BARRIER, LDSREAD, NV, DEP, NDMA, NSALU>), dim3(blocks), dim3(threads), 0, 0, iters, d_sink, gsrc);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-60s threads %d: %.1f ns per iteration\n", name, threads, ms * 1e6 / iters);
}

template <int MODE>
void run(const char *name, int threads, float *d_sink)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int iters = 4000, blocks = 256;
    hipLaunchKernelGGL(overlap_kernel<MODE>, dim3(blocks), dim3(threads), 0, 0, 100, d_sink);
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(overlap_kernel<MODE>, dim3(blocks), dim3(threads), 0, 0, iters, d_sink);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("%-60s threads %d: %.1f ns per iteration\n", name, threads, ms * 1e6 / iters);
}

static int run_step_models()
{
    float *d_sink; CHECK(hipMalloc(&d_sink, 256 * 512 * 4));
    run<0>("MFMA only (32 per iter per wave)", 256, d_sink);
    run<0>("MFMA only (32 per iter per wave)", 512, d_sink);
    run<1>("VALU only (32 fma+exp, 32 add/fma per iter per wave)", 256, d_sink);
    run<1>("VALU only", 512, d_sink);
    run<2>("waves 0-3 MFMA only, waves 4-7 VALU only", 512, d_sink);
    run<3>("each wave MFMA16, VALU, MFMA16 (same order)", 256, d_sink);
    run<3>("each wave MFMA16, VALU, MFMA16 (same order)", 512, d_sink);
    run<4>("waves 4-7 in opposite phase", 512, d_sink);
    run<5>("same order + setprio on waves 0-3", 512, d_sink);
    run_step<false, false, 1>("step: no lds, no barrier, 1x valu", 512, d_sink);
    run_step<true, false, 1>("step: no lds, barrier, 1x valu", 512, d_sink);
    run_step<false, true, 1>("step: lds reads, no barrier, 1x valu", 512, d_sink);
    run_step<true, true, 1>("step: lds reads, barrier, 1x valu", 512, d_sink);
    run_step<true, true, 2>("step: lds reads, barrier, 2x valu", 512, d_sink);
    run_step<true, true, 1>("step: lds reads, barrier, 1x valu", 256, d_sink);
    run_step<true, true, 1, true>("step: lds reads, barrier, DEPENDENT softmax", 512, d_sink);
    run_step<false, true, 1, true>("step: lds reads, no barrier, DEPENDENT softmax", 512, d_sink);
    run_step<true, true, 1, true>("step: lds reads, barrier, DEPENDENT softmax", 256, d_sink);
    char *gsrc; CHECK(hipMalloc(&gsrc, 1024 * 1024 + 4096)); CHECK(hipMemset(gsrc, 0, 1024 * 1024 + 4096));
    run_step<true, true, 1, true, 4, 0>("DEP + 4 DMA per wave", 512, d_sink, gsrc);
    run_step<true, true, 1, true, 0, 60>("DEP + 60 SALU", 512, d_sink, gsrc);
    run_step<true, true, 1, true, 0, 200>("DEP + 200 SALU", 512, d_sink, gsrc);
    run_step<true, true, 1, true, 4, 60>("DEP + 4 DMA + 60 SALU", 512, d_sink, gsrc);
    run_step<true, true, 1, true, 4, 60>("DEP + 4 DMA + 60 SALU", 256, d_sink, gsrc);
    return 0;
}

int main()
{
    const int rc = run_unit_rates();
    return rc ? rc : run_step_models();
}
