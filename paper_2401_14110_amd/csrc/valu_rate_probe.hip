// valu_rate_probe.hip -- measures the VALU issue rate of gfx950 for the instruction classes the
// LBA kernels are built from.  Stand-alone program (not part of the library):
//   hipcc -O3 --offload-arch=gfx950 valu_rate_probe.hip -o valu_rate_probe && ./valu_rate_probe
// Each lane runs NCH independent register chains; one "group" is one instruction sequence applied
// to one chain by one wave.  Reported: SIMD cycles per group at 2.4 GHz with W workgroups of 256
// lanes per CU (= W waves per SIMD), and the lane-ops per clock per CU that corresponds to.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>

enum { OP_FMA, OP_MUL, OP_ADD, OP_AND_V, OP_AND_S, OP_XOR_V, OP_ADDU_V, OP_MED3, OP_MAX, OP_BFE, OP_ADD3,
       OP_CMP, OP_LDEXP, OP_PKFMA16, MIX_MFA_DEP, MIX_MFA, MIX_FA, MIX_MFAC, MIX_RNE };

template <int OP, int NCH>
__global__ void __launch_bounds__(256) probe(float* out, int iters, float a, float b, uint32_t mask) {
    float x[NCH], q[NCH];
    float vm = __uint_as_float(mask);
    asm volatile("" : "+v"(vm));
    for (int i = 0; i < NCH; ++i) { x[i] = (float)(threadIdx.x + i) * 1e-3f; q[i] = 0.0f; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (OP == MIX_MFA_DEP) {                 // dependent order: mul, fma, and per chain
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    asm volatile("v_mul_f32 %0, %1, %2" : "=v"(q[i]) : "v"(a), "v"(b));
                    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[i]) : "v"(vm), "v"(q[i]));
                    asm volatile("v_and_b32 %0, %1, %0" : "+v"(x[i]) : "v"(vm));
                }
            } else if (OP >= MIX_MFA) {              // phased order: all muls, all fmas, all ands ...
                if (OP != MIX_FA) {
#pragma unroll
                    for (int i = 0; i < NCH; ++i) asm volatile("v_mul_f32 %0, %1, %2" : "=v"(q[i]) : "v"(a), "v"(b));
                }
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    if (OP == MIX_FA) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                    else asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[i]) : "v"(vm), "v"(q[i]));
                }
                if (OP == MIX_RNE) {
#pragma unroll
                    for (int i = 0; i < NCH; ++i) asm volatile("v_bfe_u32 %0, %1, 16, 1" : "=v"(q[i]) : "v"(x[i]));
#pragma unroll
                    for (int i = 0; i < NCH; ++i) asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(q[i]), "v"(vm));
                }
#pragma unroll
                for (int i = 0; i < NCH; ++i) asm volatile("v_and_b32 %0, %1, %0" : "+v"(x[i]) : "v"(vm));
                if (OP == MIX_MFAC) {
#pragma unroll
                    for (int i = 0; i < NCH; ++i) asm volatile("v_med3_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                }
            } else {
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    if (OP == OP_FMA) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                    if (OP == OP_MUL) asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x[i]) : "v"(a));
                    if (OP == OP_ADD) asm volatile("v_add_f32 %0, %1, %0" : "+v"(x[i]) : "v"(a));
                    if (OP == OP_AND_V) asm volatile("v_and_b32 %0, %1, %0" : "+v"(x[i]) : "v"(vm));
                    if (OP == OP_AND_S) asm volatile("v_and_b32 %0, %1, %0" : "+v"(x[i]) : "s"(mask));
                    if (OP == OP_XOR_V) asm volatile("v_xor_b32 %0, %1, %0" : "+v"(x[i]) : "v"(vm));
                    if (OP == OP_ADDU_V) asm volatile("v_add_u32 %0, %1, %0" : "+v"(x[i]) : "v"(vm));
                    if (OP == OP_MED3) asm volatile("v_med3_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                    if (OP == OP_MAX) asm volatile("v_max_f32 %0, %1, %0" : "+v"(x[i]) : "v"(a));
                    if (OP == OP_BFE) asm volatile("v_bfe_u32 %0, %0, 3, 1" : "+v"(x[i]));
                    if (OP == OP_ADD3) asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                    if (OP == OP_CMP) asm volatile("v_cmp_lt_f32 vcc, %0, %1" ::"v"(x[i]), "v"(a) : "vcc");
                    if (OP == OP_LDEXP) asm volatile("v_ldexp_f32 %0, %0, 1" : "+v"(x[i]));
                    if (OP == OP_PKFMA16) asm volatile("v_pk_fma_f16 %0, %0, %1, %2" : "+v"(x[i]) : "v"(a), "v"(b));
                }
            }
        }
    }
    float s = 0;
    for (int i = 0; i < NCH; ++i) s += x[i] + q[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int OP, int NCH>
static void run(const char* name, int ops, int waves_per_simd) {
    const int blocks = 256 * waves_per_simd, iters = 2000;
    float* out = nullptr;
    if (hipMalloc(&out, (size_t)blocks * 256 * sizeof(float)) != hipSuccess) { printf("hipMalloc failed\n"); return; }
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    probe<OP, NCH><<<blocks, 256>>>(out, 10, 1.0f, 0.5f, 0xffff0000u);
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0);
    probe<OP, NCH><<<blocks, 256>>>(out, iters, 1.0f, 0.5f, 0xffff0000u);
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    const double groups = (double)blocks * 4 * iters * 4 * NCH;
    const double cyc = (ms * 1e-3 * 2.4e9) * 256 * 4 / groups;
    printf("%-28s chains=%2d waves/SIMD=%d  %6.2f SIMD-cycles/group (%d instr)  %6.1f lane-ops/clk/CU\n",
           name, NCH, waves_per_simd, cyc, ops, 256.0 * ops / cyc);
    (void)hipFree(out);
}

int main() {
    for (int w : {2, 4, 8}) {
        run<OP_FMA, 8>("v_fma_f32", 1, w); run<OP_MUL, 8>("v_mul_f32", 1, w); run<OP_ADD, 8>("v_add_f32", 1, w);
        run<OP_AND_V, 8>("v_and_b32 (vgpr)", 1, w); run<OP_AND_S, 8>("v_and_b32 (sgpr operand)", 1, w);
        run<OP_XOR_V, 8>("v_xor_b32 (vgpr)", 1, w); run<OP_ADDU_V, 8>("v_add_u32 (vgpr)", 1, w);
        run<OP_MED3, 8>("v_med3_f32", 1, w); run<OP_MAX, 8>("v_max_f32", 1, w); run<OP_BFE, 8>("v_bfe_u32", 1, w);
        run<OP_ADD3, 8>("v_add3_u32", 1, w); run<OP_CMP, 8>("v_cmp_lt_f32", 1, w); run<OP_LDEXP, 8>("v_ldexp_f32", 1, w);
        run<OP_PKFMA16, 8>("v_pk_fma_f16", 1, w);
    }
    for (int w : {1, 2, 3, 4, 6, 8}) {
        run<MIX_MFA_DEP, 16>("mul,fma,and dependent", 3, w);
        run<MIX_MFA, 16>("mul|fma|and phased", 3, w);
        run<MIX_FA, 16>("fma|and phased", 2, w);
        run<MIX_MFAC, 16>("mul|fma|and|med3 phased", 4, w);
        run<MIX_RNE, 16>("mul|fma|bfe|add3|and phased", 5, w);
    }
    return 0;
}
