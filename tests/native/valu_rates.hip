// Issue rate of the vector-ALU instructions the field kernels are made of, on the
// GPU this runs on: every kernel is a long unrolled run of one instruction on four
// independent registers per lane, launched with 1, 2 and 4 wavefronts per SIMD.
// The figures behind the integer-ALU roof used in bench.py (one v_mad_u64_u32 per
// lane per clock) and behind "a multiplication costs its instruction count".
//
//   hipcc -O3 --offload-arch=gfx950 tests/native/valu_rates.hip -o _work/valu_rates && _work/valu_rates
//
// Measurement support, not part of the library; nothing links against it.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#define ITERS 2048
#define UNROLL 16

// NAME: kernel suffix; TYPE: type of the four registers written; SRC: type of the two sources; ASM: four instances
// of the instruction on %0..%3, sources %4, %5
#define RATE_KERNEL(NAME, TYPE, SRC, INIT, ASM, CLOBBER)                                                 \
    __global__ void k_##NAME(uint32_t* out, uint32_t seed) {                                             \
        TYPE a0 = (TYPE)(INIT + threadIdx.x), a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3;                      \
        SRC x = (SRC)(seed | 1), y = (SRC)(threadIdx.x | 0x30000003u);                                    \
        for (int it = 0; it < ITERS; ++it) {                                                             \
            _Pragma("unroll") for (int u = 0; u < UNROLL; ++u) {                                         \
                asm volatile(ASM : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(x), "v"(y) : CLOBBER);   \
            }                                                                                            \
        }                                                                                                \
        out[blockIdx.x * blockDim.x + threadIdx.x] = (uint32_t)(a0 + a1 + a2 + a3);                      \
    }

#define FOUR(I) I(0) "\n" I(1) "\n" I(2) "\n" I(3)
#define I_MAD64(n) "v_mad_u64_u32 %" #n ", vcc, %4, %5, %" #n
#define I_ADD64(n) "v_lshl_add_u64 %" #n ", %" #n ", 0, %5"
#define I_LSHR64(n) "v_lshrrev_b64 %" #n ", 3, %" #n
#define I_MULLO(n) "v_mul_lo_u32 %" #n ", %" #n ", %5"
#define I_MULHI(n) "v_mul_hi_u32 %" #n ", %" #n ", %5"
#define I_ADD(n) "v_add_u32 %" #n ", %" #n ", %5"
#define I_SUB(n) "v_sub_u32 %" #n ", %" #n ", %5"
#define I_AND(n) "v_and_b32 %" #n ", %" #n ", %5"
#define I_XOR(n) "v_xor_b32 %" #n ", %" #n ", %5"
#define I_LSHR(n) "v_lshrrev_b32 %" #n ", 3, %" #n
#define I_MOV(n) "v_mov_b32 %" #n ", %5"
#define I_ADD3(n) "v_add3_u32 %" #n ", %" #n ", %4, %5"
#define I_BITOP3(n) "v_bitop3_b32 %" #n ", %" #n ", %4, %5 bitop3:0x96"
#define I_ALIGNBIT(n) "v_alignbit_b32 %" #n ", %" #n ", %4, 7"
#define I_PERM(n) "v_perm_b32 %" #n ", %" #n ", %4, %5"
#define I_BFI(n) "v_bfi_b32 %" #n ", %" #n ", %4, %5"
#define I_FMA32(n) "v_fma_f32 %" #n ", %" #n ", %4, %5"
#define I_FMA64(n) "v_fma_f64 %" #n ", %" #n ", %4, %5"

RATE_KERNEL(mad_u64_u32, uint64_t, uint32_t, seed, FOUR(I_MAD64), "vcc")
RATE_KERNEL(lshl_add_u64, uint64_t, uint64_t, seed, FOUR(I_ADD64), "memory")
RATE_KERNEL(lshrrev_b64, uint64_t, uint32_t, seed, FOUR(I_LSHR64), "memory")
RATE_KERNEL(mul_lo_u32, uint32_t, uint32_t, seed, FOUR(I_MULLO), "memory")
RATE_KERNEL(mul_hi_u32, uint32_t, uint32_t, seed, FOUR(I_MULHI), "memory")
RATE_KERNEL(add_u32, uint32_t, uint32_t, seed, FOUR(I_ADD), "memory")
RATE_KERNEL(sub_u32, uint32_t, uint32_t, seed, FOUR(I_SUB), "memory")
RATE_KERNEL(and_b32, uint32_t, uint32_t, seed, FOUR(I_AND), "memory")
RATE_KERNEL(xor_b32, uint32_t, uint32_t, seed, FOUR(I_XOR), "memory")
RATE_KERNEL(lshrrev_b32, uint32_t, uint32_t, seed, FOUR(I_LSHR), "memory")
RATE_KERNEL(mov_b32, uint32_t, uint32_t, seed, FOUR(I_MOV), "memory")
RATE_KERNEL(add3_u32, uint32_t, uint32_t, seed, FOUR(I_ADD3), "memory")
RATE_KERNEL(bitop3_b32, uint32_t, uint32_t, seed, FOUR(I_BITOP3), "memory")
RATE_KERNEL(alignbit_b32, uint32_t, uint32_t, seed, FOUR(I_ALIGNBIT), "memory")
RATE_KERNEL(perm_b32, uint32_t, uint32_t, seed, FOUR(I_PERM), "memory")
RATE_KERNEL(bfi_b32, uint32_t, uint32_t, seed, FOUR(I_BFI), "memory")
RATE_KERNEL(fma_f32, float, float, 1.0f, FOUR(I_FMA32), "memory")
RATE_KERNEL(fma_f64, double, double, 1.0, FOUR(I_FMA64), "memory")

// carry chain: v_add_co_u32 followed by three v_addc_co_u32
__global__ void k_addc_co_u32(uint32_t* out, uint32_t seed) {
    uint32_t a0 = seed + threadIdx.x, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, y = threadIdx.x | 0xf0000003u;
    for (int it = 0; it < ITERS; ++it) {
        _Pragma("unroll") for (int u = 0; u < UNROLL; ++u) {
            asm volatile("v_add_co_u32 %0, vcc, %0, %4\nv_addc_co_u32 %1, vcc, %1, %4, vcc\nv_addc_co_u32 %2, vcc, %2, %4, vcc\n"
                         "v_addc_co_u32 %3, vcc, %3, %4, vcc"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(y) : "vcc");
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3;
}

typedef void (*kernel_t)(uint32_t*, uint32_t);

static int run(kernel_t kern, const char* name, int waves_per_simd, uint32_t* d) {
    const int blocks = 256 * waves_per_simd;  // 256 compute units x 4 SIMDs x waves_per_simd wavefronts, four per workgroup
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), 0, 0, d, 12345u);
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    (void)hipEventRecord(e0);
    for (int r = 0; r < 5; ++r) hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), 0, 0, d, 12345u);
    (void)hipEventRecord(e1);
    if (hipEventSynchronize(e1) != hipSuccess) return 1;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    ms /= 5;
    const double lane_ops = (double)blocks * 256 * (double)ITERS * UNROLL * 4;
    const double wave_instr_per_simd = lane_ops / 64.0 / 1024.0;
    printf("%-14s waves/SIMD=%d %8.3f ms %7.2f T lane-op/s %6.2f cycles per wave-instruction per SIMD at 2.4 GHz\n", name,
           waves_per_simd, ms, lane_ops / (ms * 1e-3) / 1e12, ms * 1e-3 * 2.4e9 / wave_instr_per_simd);
    fflush(stdout);
    return 0;
}

int main() {
    hipDeviceProp_t p;
    if (hipGetDeviceProperties(&p, 0) != hipSuccess) return 1;
    printf("device %s, %d compute units, clock %d kHz\n", p.gcnArchName, p.multiProcessorCount, p.clockRate);
    uint32_t* d;
    if (hipMalloc(&d, (size_t)256 * 4 * 256 * 4) != hipSuccess) return 1;
    struct { kernel_t k; const char* name; } all[] = {
        {k_mad_u64_u32, "mad_u64_u32"}, {k_addc_co_u32, "addc_co_u32"}, {k_lshl_add_u64, "lshl_add_u64"},
        {k_lshrrev_b64, "lshrrev_b64"}, {k_mul_lo_u32, "mul_lo_u32"}, {k_mul_hi_u32, "mul_hi_u32"},
        {k_add_u32, "add_u32"}, {k_sub_u32, "sub_u32"}, {k_and_b32, "and_b32"}, {k_xor_b32, "xor_b32"},
        {k_lshrrev_b32, "lshrrev_b32"}, {k_mov_b32, "mov_b32"}, {k_add3_u32, "add3_u32"}, {k_bitop3_b32, "bitop3_b32"},
        {k_alignbit_b32, "alignbit_b32"}, {k_perm_b32, "perm_b32"}, {k_bfi_b32, "bfi_b32"}, {k_fma_f32, "fma_f32"},
        {k_fma_f64, "fma_f64"}};
    for (int w : {1, 2, 4})
        for (auto& e : all)
            if (run(e.k, e.name, w, d)) return 1;
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    printf("done\n");
    return 0;
}
