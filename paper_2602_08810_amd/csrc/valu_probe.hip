// Issue-rate probe for the vector ALU of gfx950: a stand-alone program, not part of the scan library.
//
// The selective-scan kernels are bound by vector-ALU issue, not by HBM, so their roofline needs the rates at which a
// SIMD really issues the instruction kinds they are made of.  Each case below runs a loop of one instruction kind,
// 64 instructions per loop pass on CH independent registers per lane, with 1, 2 or 4 wavefronts resident per SIMD
// (256 compute units x 4 SIMDs; one 256-thread workgroup puts one wavefront on each SIMD of a unit), and prints the
// time per wavefront-instruction per SIMD in cycles of the nominal 2.4 GHz clock.  CH = 8 gives the issue rate;
// CH = 1 is a dependent chain and gives the latency from an instruction to the next one that needs its result.
//
//     hipcc --offload-arch=gfx950 -O3 valu_probe.hip -o valu_probe && ./valu_probe
#include <hip/hip_runtime.h>
#include <cstdio>

enum Kind { FMA, MUL, MUL_SGPR, CNDMASK_SGPR, MUL_DPP, MAX, CVT_PK_BF16, EXP, RCP };

template <int KIND, int CH>
__global__ __launch_bounds__(256) void k_probe(float *out, int iters, float seed, float sval, unsigned long long mask) {
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = seed + threadIdx.x * 1e-3f + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 64 / CH; ++r) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const float other = v[(i + 3) & 7];        // an operand from another chain (not written while CH == 1)
                if (KIND == FMA) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(v[i]) : "v"(other));
                if (KIND == MUL) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[i]) : "v"(other));
                if (KIND == MUL_SGPR) asm volatile("v_mul_f32 %0, %1, %0" : "+v"(v[i]) : "s"(sval));
                if (KIND == CNDMASK_SGPR) asm volatile("v_cndmask_b32 %0, %0, %1, %2" : "+v"(v[i]) : "v"(other), "s"(mask));
                // the lanes are permuted on the operand from the other chain, which is never written within the three
                // instructions before (a DPP read needs two wait states after a write of its register)
                if (KIND == MUL_DPP) asm volatile("v_mul_f32_dpp %0, %1, %0 row_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(v[i]) : "v"(other));
                if (KIND == MAX) asm volatile("v_max_f32 %0, %0, %1" : "+v"(v[i]) : "v"(other));
                if (KIND == CVT_PK_BF16) asm volatile("v_cvt_pk_bf16_f32 %0, %0, %1" : "+v"(v[i]) : "v"(other));
                if (KIND == EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(v[i]));
                if (KIND == RCP) asm volatile("v_rcp_f32 %0, %0" : "+v"(v[i]));
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

static bool ok(hipError_t e, const char *what) {
    if (e != hipSuccess) { std::fprintf(stderr, "valu_probe: %s: %s\n", what, hipGetErrorString(e)); return false; }
    return true;
}

template <int KIND, int CH>
static bool run(const char *name, float *out, int waves_per_simd) {
    const int blocks = 256 * waves_per_simd, iters = 1000;
    hipEvent_t e0, e1;
    if (!ok(hipEventCreate(&e0), "event") || !ok(hipEventCreate(&e1), "event")) return false;
    hipLaunchKernelGGL((k_probe<KIND, CH>), dim3(blocks), dim3(256), 0, 0, out, 10, 1.0f, 0.999f, 0x5555555555555555ull);
    if (!ok(hipEventRecord(e0), "record")) return false;
    hipLaunchKernelGGL((k_probe<KIND, CH>), dim3(blocks), dim3(256), 0, 0, out, iters, 1.0f, 0.999f, 0x5555555555555555ull);
    if (!ok(hipEventRecord(e1), "record") || !ok(hipEventSynchronize(e1), "sync")) return false;
    float ms = 0.0f;
    if (!ok(hipEventElapsedTime(&ms, e0, e1), "elapsed")) return false;
    const double per_simd = ms * 1e-3 * 2.4e9 / (double(waves_per_simd) * iters * 64.0);
    std::printf("%-28s chains %d  waves/SIMD %d  %6.2f cycles per instruction and SIMD  (%6.2f per wavefront)\n", name, CH,
                waves_per_simd, per_simd, per_simd * waves_per_simd);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    return true;
}

int main() {
    float *out = nullptr;
    if (!ok(hipMalloc(&out, 1024 * 256 * sizeof(float)), "hipMalloc")) return 1;
    bool good = true;
    for (int w : {1, 2, 4}) {
        good = good && run<FMA, 8>("v_fma_f32", out, w) && run<MUL, 8>("v_mul_f32", out, w) &&
               run<MUL_SGPR, 8>("v_mul_f32, scalar operand", out, w) && run<CNDMASK_SGPR, 8>("v_cndmask_b32", out, w) &&
               run<MUL_DPP, 8>("v_mul_f32_dpp", out, w) && run<MAX, 8>("v_max_f32", out, w) &&
               run<CVT_PK_BF16, 8>("v_cvt_pk_bf16_f32", out, w) && run<EXP, 8>("v_exp_f32", out, w) && run<RCP, 8>("v_rcp_f32", out, w);
    }
    good = good && run<FMA, 1>("v_fma_f32", out, 1) && run<MUL_DPP, 1>("v_mul_f32_dpp", out, 1) && run<EXP, 1>("v_exp_f32", out, 1);
    good = good && ok(hipDeviceSynchronize(), "sync");
    (void)hipFree(out);
    return good ? 0 : 1;
}
