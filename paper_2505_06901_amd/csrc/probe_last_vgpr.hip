// Measurement program (not part of libecco): does an instruction give the same result when one of its source operands
// sits in the LAST vector register of the wavefront's allocation as when the same value sits in another register?
//
// Found while looking for the cause of kernels whose results changed from launch to launch: on the MI355X boxes this
// library was developed on, the 64-bit shifts (v_lshlrev_b64, v_lshrrev_b64, v_ashrrev_i64) do not, when the shift
// AMOUNT is in the last register of the allocation and the SIMD holds more than one wavefront.  The register itself
// holds the right value (a move reads it back correctly, wait states in front of the shift change nothing), a 32-bit
// shift, an add or a 64-bit multiply-add by the same register are right, and the register before the last is right:
// the amount seems to be fetched as a register pair whose second half lies outside the wavefront's allocation.
// The compiler does not avoid the register; paper_2505_06901_amd/build.py checks every kernel of the library for it.
//
// Each case runs its instruction twice per iteration: with the operand moved into the named register (followed by
// eight wait states), and with the operand in a register the compiler picks; the two results must agree.  A kernel's
// allocation is set by naming its top register in a clobber list.  256 workgroups; every LDS address is in bounds.
// Build: python -m paper_2505_06901_amd.build   Run: ./paper_2505_06901_amd/probe_last_vgpr [iterations]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                    \
    do {                                                                         \
        hipError_t e_ = (x);                                                     \
        if (e_ != hipSuccess) {                                                  \
            std::printf("%s: %s\n", #x, hipGetErrorString(e_));                  \
            return 1;                                                            \
        }                                                                        \
    } while (0)

namespace {

// NAME: kernel name.  REG: the register under test.  TOP: the highest register of the allocation (named in a clobber
// list once, so that the allocation is TOP + 1 registers).  TYPE: C type of the result.  INSN: the instruction, with
// %0 the result, X the operand under test, %2 a 64-bit and %3 a 32-bit further operand.
#define PROBE_KERNEL(NAME, REG, TOP, TYPE, INSN_REG, INSN_ANY)                                                            \
    __global__ __launch_bounds__(1024) void NAME(unsigned long long* out, int iters) {                                    \
        asm volatile("v_mov_b32 v" #TOP ", 0" ::: "v" #TOP);                                                              \
        unsigned long long bad = 0;                                                                                       \
        uint32_t r = threadIdx.x * 747796405u + blockIdx.x * 7919u + 1u;                                                  \
        for (int it = 0; it < iters; ++it) {                                                                              \
            r = r * 1664525u + 1013904223u;                                                                               \
            const uint32_t val = r, other = r * 2246822519u + 7u;                                                         \
            const uint64_t wide = ((uint64_t)other << 32) | (r ^ 0x9E3779B9u);                                            \
            TYPE a, b;                                                                                                    \
            asm volatile("v_mov_b32 v" #REG ", %1\n\ts_nop 7\n\t" INSN_REG : "=&v"(a) : "v"(val), "v"(wide), "v"(other)    \
                         : "v" #REG, "s20", "s21");                                                                       \
            asm volatile(INSN_ANY : "=&v"(b) : "v"(val), "v"(wide), "v"(other) : "s20", "s21");                           \
            bad += (a != b);                                                                                              \
            r ^= (uint32_t)a;                                                                                             \
        }                                                                                                                 \
        if (bad) atomicAdd(out, bad);                                                                                     \
        if (r == 77u) atomicAdd(out + 1, 1ull); /* keeps the loop alive */                                                \
    }

// 64-bit shifts by the last register of allocations of 64, 104, 120 and 128 registers
PROBE_KERNEL(shl64_last_of_64, 63, 63, uint64_t, "v_lshlrev_b64 %0, v63, %2", "v_lshlrev_b64 %0, %1, %2")
PROBE_KERNEL(shl64_last_of_104, 103, 103, uint64_t, "v_lshlrev_b64 %0, v103, %2", "v_lshlrev_b64 %0, %1, %2")
PROBE_KERNEL(shl64_last_of_120, 119, 119, uint64_t, "v_lshlrev_b64 %0, v119, %2", "v_lshlrev_b64 %0, %1, %2")
PROBE_KERNEL(shl64_last_of_128, 127, 127, uint64_t, "v_lshlrev_b64 %0, v127, %2", "v_lshlrev_b64 %0, %1, %2")
PROBE_KERNEL(shr64_last_of_120, 119, 119, uint64_t, "v_lshrrev_b64 %0, v119, %2", "v_lshrrev_b64 %0, %1, %2")
PROBE_KERNEL(sar64_last_of_120, 119, 119, uint64_t, "v_ashrrev_i64 %0, v119, %2", "v_ashrrev_i64 %0, %1, %2")
// the same shift by other registers of a 120-register allocation
PROBE_KERNEL(shl64_v118_of_120, 118, 119, uint64_t, "v_lshlrev_b64 %0, v118, %2", "v_lshlrev_b64 %0, %1, %2")
PROBE_KERNEL(shl64_v112_of_120, 112, 119, uint64_t, "v_lshlrev_b64 %0, v112, %2", "v_lshlrev_b64 %0, %1, %2")
// v119 used, but the allocation is 128: not the last register
PROBE_KERNEL(shl64_v119_of_128, 119, 127, uint64_t, "v_lshlrev_b64 %0, v119, %2", "v_lshlrev_b64 %0, %1, %2")
// other instructions with a source in the last register of 120
PROBE_KERNEL(shl32_last_of_120, 119, 119, uint32_t, "v_lshlrev_b32 %0, v119, %3", "v_lshlrev_b32 %0, %1, %3")
PROBE_KERNEL(add32_last_of_120, 119, 119, uint32_t, "v_add_u32 %0, v119, %3", "v_add_u32 %0, %1, %3")
PROBE_KERNEL(mad64_last_of_120, 119, 119, uint64_t, "v_mad_u64_u32 %0, s[20:21], v119, %3, %2", "v_mad_u64_u32 %0, s[20:21], %1, %3, %2")
PROBE_KERNEL(madi64_last_of_120, 119, 119, uint64_t, "v_mad_i64_i32 %0, s[20:21], %3, v119, %2", "v_mad_i64_i32 %0, s[20:21], %3, %1, %2")
PROBE_KERNEL(alignbit_last_of_120, 119, 119, uint32_t, "v_alignbit_b32 %0, %3, %3, v119", "v_alignbit_b32 %0, %3, %3, %1")
PROBE_KERNEL(fma_mix_last_of_120, 119, 119, uint32_t, "v_fma_mix_f32 %0, v119, %3, %3 op_sel:[1,0,0] op_sel_hi:[1,1,0]",
             "v_fma_mix_f32 %0, %1, %3, %3 op_sel:[1,0,0] op_sel_hi:[1,1,0]")

struct Case {
    const char* what;
    const void* fn;
    int threads;
};

}  // namespace

int main(int argc, char** argv) {
    int iters = argc > 1 ? std::atoi(argv[1]) : 2000;
    if (iters < 1 || iters > 100000) iters = 2000;
    unsigned long long* d;
    CK(hipMalloc(&d, 16));
    const Case cases[] = {
        {"v_lshlrev_b64, amount in v63, the last of 64 registers", (const void*)shl64_last_of_64, 1024},
        {"v_lshlrev_b64, amount in v103, the last of 104", (const void*)shl64_last_of_104, 1024},
        {"v_lshlrev_b64, amount in v119, the last of 120", (const void*)shl64_last_of_120, 1024},
        {"v_lshlrev_b64, amount in v127, the last of 128", (const void*)shl64_last_of_128, 1024},
        {"v_lshrrev_b64, amount in v119, the last of 120", (const void*)shr64_last_of_120, 1024},
        {"v_ashrrev_i64, amount in v119, the last of 120", (const void*)sar64_last_of_120, 1024},
        {"v_lshlrev_b64, amount in v119 of 120, 8 wavefronts", (const void*)shl64_last_of_120, 512},
        {"v_lshlrev_b64, amount in v119 of 120, 4 wavefronts", (const void*)shl64_last_of_120, 256},
        {"v_lshlrev_b64, amount in v118 of 120", (const void*)shl64_v118_of_120, 1024},
        {"v_lshlrev_b64, amount in v112 of 120", (const void*)shl64_v112_of_120, 1024},
        {"v_lshlrev_b64, amount in v119 of 128", (const void*)shl64_v119_of_128, 1024},
        {"v_lshlrev_b32, amount in v119, the last of 120", (const void*)shl32_last_of_120, 1024},
        {"v_add_u32, source in v119, the last of 120", (const void*)add32_last_of_120, 1024},
        {"v_mad_u64_u32, factor in v119, the last of 120", (const void*)mad64_last_of_120, 1024},
        {"v_mad_i64_i32, factor in v119, the last of 120", (const void*)madi64_last_of_120, 1024},
        {"v_alignbit_b32, amount in v119, the last of 120", (const void*)alignbit_last_of_120, 1024},
        {"v_fma_mix_f32, factor in v119, the last of 120", (const void*)fma_mix_last_of_120, 1024},
    };
    std::printf("probe_last_vgpr: %d iterations per lane, 256 workgroups; results that differ between the operand in the named "
                "register and in a register of the compiler's choice\n", iters);
    for (const Case& c : cases) {
        CK(hipMemset(d, 0, 16));
        void* args[] = {(void*)&d, (void*)&iters};
        CK(hipLaunchKernel(c.fn, dim3(256), dim3(c.threads), args, 0, 0));
        CK(hipDeviceSynchronize());
        unsigned long long h[2];
        CK(hipMemcpy(h, d, 16, hipMemcpyDeviceToHost));
        const double total = 1.0 * iters * 256 * c.threads;
        std::printf("  %-56s %12llu of %.0f (%.2f %%)\n", c.what, h[0], total, 100.0 * (double)h[0] / total);
        std::fflush(stdout);
    }
    CK(hipFree(d));
    return 0;
}
