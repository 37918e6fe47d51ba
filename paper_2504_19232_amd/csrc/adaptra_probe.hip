// adaptra_probe.hip -- issue-rate probes for the integer vector instructions the recurrence
// kernels are made of (gfx950).  Measurement aid only (include/adaptra_testing.h): a roofline
// against "the integer VALU peak" needs to know what that peak is for the instructions really
// issued, and the counters of the recurrence kernel can only be read against kernels whose
// instruction counts are known by construction.
//
// Every probe keeps eight independent registers per lane and issues one instruction (or one
// short group) per register, 32 times per loop trip, so neither dependency latency nor the
// loop's own scalar instructions limit it; there is no memory traffic except in the forward-step
// mix, which runs the hot kernel's LDS ring accesses on a private ring.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adaptra.h"
#include "adaptra_internal.h"
#include "adaptra_testing.h"

namespace {

constexpr int kProbeBlock = 256;
constexpr int kRegs = 8;              // independent registers per lane
constexpr int kRepeat = 32;           // groups of kRegs instructions per loop trip
constexpr int kStepRepeat = 4;        // forward-step mix: sweeps of kRegs steps per loop trip
constexpr int kStepValu = 5;          // vector instructions of one forward step

// The single-instruction mixes: name, assembly, vector instructions per statement.  Operands:
// %0 the lane's register (read and written), %1 another VGPR, %2 a 32-bit SGPR, %3 a 64-bit
// SGPR pair, %4 a third VGPR.  Statements that touch vcc or scc say so in the clobber list
// (a select fed by s_bfe_i64 changes scc, which the loop's own compare also uses).
#define ADAPTRA_PROBE_TABLE(X)                                                                        \
    X(ADAPTRA_PROBE_ADD_VGPR, "v_add_u32 %0, %0, %1")                                                 \
    X(ADAPTRA_PROBE_ADD_SGPR, "v_add_u32 %0, %2, %0")                                                 \
    X(ADAPTRA_PROBE_ADD_INLINE, "v_add_u32 %0, 4, %0")                                                \
    X(ADAPTRA_PROBE_ADD_LITERAL, "v_add_u32 %0, 0x12345, %0")                                         \
    X(ADAPTRA_PROBE_ADD_E64, "v_add_u32_e64 %0, %0, %1")                                              \
    X(ADAPTRA_PROBE_SUB, "v_sub_u32 %0, %0, %1")                                                      \
    X(ADAPTRA_PROBE_ADD_CO, "v_add_co_u32 %0, vcc, %0, %1")                                           \
    X(ADAPTRA_PROBE_ADD3, "v_add3_u32 %0, %0, %1, %4")                                                \
    X(ADAPTRA_PROBE_MAX, "v_max_i32 %0, %0, %1")                                                      \
    X(ADAPTRA_PROBE_MAX_SGPR, "v_max_i32 %0, %2, %0")                                                 \
    X(ADAPTRA_PROBE_MAX_E64, "v_max_i32_e64 %0, %0, %1")                                              \
    X(ADAPTRA_PROBE_MAX_U32, "v_max_u32 %0, %0, %1")                                                  \
    X(ADAPTRA_PROBE_MIN, "v_min_i32 %0, %0, %1")                                                      \
    X(ADAPTRA_PROBE_MAX3, "v_max3_i32 %0, %0, %1, %4")                                                \
    X(ADAPTRA_PROBE_MED3, "v_med3_i32 %0, %0, %1, %4")                                                \
    X(ADAPTRA_PROBE_AND, "v_and_b32 %0, %0, %1")                                                      \
    X(ADAPTRA_PROBE_OR, "v_or_b32 %0, %0, %1")                                                        \
    X(ADAPTRA_PROBE_XOR, "v_xor_b32 %0, %0, %1")                                                      \
    X(ADAPTRA_PROBE_LSHL, "v_lshlrev_b32 %0, 1, %0")                                                  \
    X(ADAPTRA_PROBE_MOV, "v_mov_b32 %0, %1")                                                          \
    X(ADAPTRA_PROBE_CNDMASK, "v_cndmask_b32 %0, %0, %1, vcc")                                         \
    X(ADAPTRA_PROBE_CNDMASK_SGPR, "v_cndmask_b32_e64 %0, %0, %1, %3")                                 \
    X(ADAPTRA_PROBE_CNDMASK_BFE, "s_bfe_i64 vcc, %3, 0x10005\n\tv_cndmask_b32 %0, %0, %1, vcc")       \
    X(ADAPTRA_PROBE_CMP_CNDMASK, "v_cmp_gt_i32 vcc, %0, %1\n\tv_cndmask_b32 %0, %0, %1, vcc")       \
    X(ADAPTRA_PROBE_ADD_MAX_ALT, "v_add_u32 %0, %0, %1\n\tv_max_i32 %0, %0, %4")

template <int MIX>
__device__ __forceinline__ void probe_statement(int &v, int other, int third, int c, unsigned long long mask);
#define ADAPTRA_PROBE_DEFINE(mix, text)                                                                              \
    template <>                                                                                                      \
    __device__ __forceinline__ void probe_statement<mix>(int &v, int other, int third, int c, unsigned long long mask) { \
        asm volatile(text : "+v"(v) : "v"(other), "s"(c), "s"(mask), "v"(third) : "vcc", "scc");                     \
    }
ADAPTRA_PROBE_TABLE(ADAPTRA_PROBE_DEFINE)
#undef ADAPTRA_PROBE_DEFINE

template <int MIX>
__global__ __launch_bounds__(kProbeBlock) void k_valu_probe(int iters, int c, int d, unsigned long long mask, int *out) {
    int v[kRegs];
#pragma unroll
    for (int j = 0; j < kRegs; ++j) v[j] = (int)threadIdx.x + j;
    const int other = (int)threadIdx.x ^ d, third = (int)threadIdx.x * 3 + d;
    int scalar_sink = 0;
    // vcc is set once, before the loop: nothing in that mix's loop writes it (the loop's own
    // compare goes through scc)
    if constexpr (MIX == ADAPTRA_PROBE_CNDMASK) asm volatile("s_mov_b64 vcc, %0" : : "s"(mask) : "vcc");
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < kRepeat; ++u) {
#pragma unroll
            for (int j = 0; j < kRegs; ++j) {
                if constexpr (MIX == ADAPTRA_PROBE_ADD_MAX) {
                    v[j] = (v[j] + c > d + j) ? v[j] + c : d + j;
                } else if constexpr (MIX == ADAPTRA_PROBE_ADD_MAX_BATCH || MIX == ADAPTRA_PROBE_ADD_MAX_BATCH_NOP ||
                                     MIX == ADAPTRA_PROBE_ADD_MAX_ALT_DENSE) {
                    // the same eight adds and eight maxes as the alternating mix in ONE statement:
                    // the adds first (with or without an s_nop behind every instruction), or
                    // alternating without the s_nop the compiler puts between two asm statements
                    if (j == 0) {
#define ADAPTRA_A(r) "v_add_u32 %" #r ", %" #r ", %8\n\t"
#define ADAPTRA_M(r) "v_max_i32 %" #r ", %" #r ", %9\n\t"
#define ADAPTRA_N "s_nop 0\n\t"
#define ADAPTRA_REGS : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) : "v"(other), "v"(third)
                        if constexpr (MIX == ADAPTRA_PROBE_ADD_MAX_BATCH)
                            asm volatile(ADAPTRA_A(0) ADAPTRA_A(1) ADAPTRA_A(2) ADAPTRA_A(3) ADAPTRA_A(4) ADAPTRA_A(5) ADAPTRA_A(6) ADAPTRA_A(7)
                                         ADAPTRA_M(0) ADAPTRA_M(1) ADAPTRA_M(2) ADAPTRA_M(3) ADAPTRA_M(4) ADAPTRA_M(5) ADAPTRA_M(6) ADAPTRA_M(7)
                                         ADAPTRA_REGS);
                        else if constexpr (MIX == ADAPTRA_PROBE_ADD_MAX_BATCH_NOP)
                            asm volatile(ADAPTRA_A(0) ADAPTRA_N ADAPTRA_A(1) ADAPTRA_N ADAPTRA_A(2) ADAPTRA_N ADAPTRA_A(3) ADAPTRA_N
                                         ADAPTRA_A(4) ADAPTRA_N ADAPTRA_A(5) ADAPTRA_N ADAPTRA_A(6) ADAPTRA_N ADAPTRA_A(7) ADAPTRA_N
                                         ADAPTRA_M(0) ADAPTRA_N ADAPTRA_M(1) ADAPTRA_N ADAPTRA_M(2) ADAPTRA_N ADAPTRA_M(3) ADAPTRA_N
                                         ADAPTRA_M(4) ADAPTRA_N ADAPTRA_M(5) ADAPTRA_N ADAPTRA_M(6) ADAPTRA_N ADAPTRA_M(7) ADAPTRA_N
                                         ADAPTRA_REGS);
                        else
                            asm volatile(ADAPTRA_A(0) ADAPTRA_M(0) ADAPTRA_A(1) ADAPTRA_M(1) ADAPTRA_A(2) ADAPTRA_M(2) ADAPTRA_A(3) ADAPTRA_M(3)
                                         ADAPTRA_A(4) ADAPTRA_M(4) ADAPTRA_A(5) ADAPTRA_M(5) ADAPTRA_A(6) ADAPTRA_M(6) ADAPTRA_A(7) ADAPTRA_M(7)
                                         ADAPTRA_REGS);
#undef ADAPTRA_A
#undef ADAPTRA_M
#undef ADAPTRA_N
#undef ADAPTRA_REGS
                    }
                } else if constexpr (MIX == ADAPTRA_PROBE_READLANE) {
                    int s;
                    asm volatile("v_readlane_b32 %0, %1, 3" : "=s"(s) : "v"(v[j]));
                    scalar_sink ^= s;
                } else {
                    probe_statement<MIX>(v[j], other, third, c, mask);
                }
            }
        }
    }
    int r = scalar_sink;
#pragma unroll
    for (int j = 0; j < kRegs; ++j) r ^= v[j];
    if (r == 0x7fffffff && c == 0x12345) out[0] = r;      // never in practice: keeps the registers alive
}

// The forward step of the scenario-lanes kernel, instruction for instruction: the addend from a
// vector register, the select of a link without slack (mask bit -> scalar pair -> v_cndmask_b32), the
// max, the ring offset advanced with the carry trick, the write of the result and the read of a
// value for a later step, each with its own address add.  Eight "stages" share one ring of
// eight slots [slot][lane]; a value read in a step is used by the same step of the next sweep,
// fourteen LDS operations later (s_waitcnt lgkmcnt(14)).
#define ADAPTRA_PROBE_STEP(j, jp)                                  \
    "v_add_u32 %[t], %[L" #j "], %[vadd]\n\t"                      \
    "s_bfe_i64 %[pair], %[mask], 0x1000" #j "\n\t"                 \
    "s_waitcnt lgkmcnt(14)\n\t"                                    \
    "v_cndmask_b32_e64 %[o], %[x" #j "], %[L" #jp "], %[pair]\n\t" \
    "s_add_u32 %[soff], %[soff], 0x100\n\t"                        \
    "s_cmov_b32 %[soff], %[bias]\n\t"                              \
    "v_max_i32 %[L" #j "], %[t], %[o]\n\t"                         \
    "v_add_u32 %[a], %[soff], %[ring]\n\t"                         \
    "ds_write_b32 %[a], %[L" #j "]\n\t"                            \
    "v_add_u32 %[a], %[soff], %[ring]\n\t"                         \
    "ds_read_b32 %[x" #j "], %[a]\n\t"

__global__ __launch_bounds__(kProbeBlock) void k_forward_step_probe(int iters, int c, unsigned long long mask, int *out) {
    extern __shared__ int probe_lds[];
    const unsigned ring_bytes = kRegs * 256u;
    const unsigned bias = 0u - ring_bytes;
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    typedef __attribute__((address_space(3))) int lds_int;
    const unsigned ring = (unsigned)(size_t)(lds_int *)probe_lds + wave * ring_bytes + lane * 4u + ring_bytes;
    for (unsigned s = 0; s < kRegs; ++s) probe_lds[(wave * kRegs + s) * 64 + lane] = (int)(lane + s);
    int L0 = 0, L1 = 1, L2 = 2, L3 = 3, L4 = 4, L5 = 5, L6 = 6, L7 = 7;
    int x0 = 0, x1 = 0, x2 = 0, x3 = 0, x4 = 0, x5 = 0, x6 = 0, x7 = 0;
    unsigned soff = bias;
    int t, o, vadd = c;
    asm volatile("" : "+v"(vadd));                        // the addend in a vector register
    unsigned a;
    unsigned long long pair;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < kStepRepeat; ++u) {
            asm volatile(ADAPTRA_PROBE_STEP(0, 7) ADAPTRA_PROBE_STEP(1, 0) ADAPTRA_PROBE_STEP(2, 1) ADAPTRA_PROBE_STEP(3, 2)
                         ADAPTRA_PROBE_STEP(4, 3) ADAPTRA_PROBE_STEP(5, 4) ADAPTRA_PROBE_STEP(6, 5) ADAPTRA_PROBE_STEP(7, 6)
                         : [L0] "+v"(L0), [L1] "+v"(L1), [L2] "+v"(L2), [L3] "+v"(L3), [L4] "+v"(L4), [L5] "+v"(L5),
                           [L6] "+v"(L6), [L7] "+v"(L7), [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3),
                           [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6), [x7] "+v"(x7), [soff] "+s"(soff),
                           [t] "=&v"(t), [o] "=&v"(o), [a] "=&v"(a), [pair] "=&s"(pair)
                         : [vadd] "v"(vadd), [mask] "s"(mask), [bias] "s"(bias), [ring] "v"(ring)
                         : "scc", "memory");
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int r = L0 ^ L1 ^ L2 ^ L3 ^ L4 ^ L5 ^ L6 ^ L7 ^ x0 ^ x1 ^ x2 ^ x3 ^ x4 ^ x5 ^ x6 ^ x7;
    if (r == 0x7fffffff && c == 0x12345) out[0] = r;      // never in practice
}
#undef ADAPTRA_PROBE_STEP

template <int MIX>
void launch_probe(int blocks, int iters, int *scratch, hipStream_t st) {
    hipLaunchKernelGGL((k_valu_probe<MIX>), dim3(blocks), dim3(kProbeBlock), 0, st, iters, 1, -5, 0x5555aaaa3333ccccull, scratch);
}

}  // namespace

extern "C" int adaptra_valu_probe(int32_t mix, int32_t blocks, int32_t iters, int32_t *scratch, void *stream,
                                  int64_t *valu_instructions) {
    if (blocks < 1 || iters < 1 || !scratch || mix < 0 || mix >= ADAPTRA_PROBE_MIXES) return ADAPTRA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int64_t per_wave = (int64_t)iters * kRepeat * kRegs;
    switch (mix) {
#define ADAPTRA_PROBE_CASE(m, text) \
    case m: launch_probe<m>(blocks, iters, scratch, st); break;
        ADAPTRA_PROBE_TABLE(ADAPTRA_PROBE_CASE)
#undef ADAPTRA_PROBE_CASE
        case ADAPTRA_PROBE_ADD_MAX: launch_probe<ADAPTRA_PROBE_ADD_MAX>(blocks, iters, scratch, st); break;
        case ADAPTRA_PROBE_READLANE: launch_probe<ADAPTRA_PROBE_READLANE>(blocks, iters, scratch, st); break;
        case ADAPTRA_PROBE_ADD_MAX_BATCH: launch_probe<ADAPTRA_PROBE_ADD_MAX_BATCH>(blocks, iters, scratch, st); break;
        case ADAPTRA_PROBE_ADD_MAX_BATCH_NOP: launch_probe<ADAPTRA_PROBE_ADD_MAX_BATCH_NOP>(blocks, iters, scratch, st); break;
        case ADAPTRA_PROBE_ADD_MAX_ALT_DENSE: launch_probe<ADAPTRA_PROBE_ADD_MAX_ALT_DENSE>(blocks, iters, scratch, st); break;
        default:
            hipLaunchKernelGGL(k_forward_step_probe, dim3(blocks), dim3(kProbeBlock), (kProbeBlock / 64) * kRegs * 256, st,
                               iters, 1, 0x5555aaaa3333ccccull, scratch);
            per_wave = (int64_t)iters * kStepRepeat * kRegs * kStepValu;
            break;
    }
    ADAPTRA_CHECK_LAUNCH();
    if (mix == ADAPTRA_PROBE_ADD_MAX || mix == ADAPTRA_PROBE_CMP_CNDMASK || mix == ADAPTRA_PROBE_ADD_MAX_ALT ||
        mix == ADAPTRA_PROBE_ADD_MAX_BATCH || mix == ADAPTRA_PROBE_ADD_MAX_BATCH_NOP || mix == ADAPTRA_PROBE_ADD_MAX_ALT_DENSE)
        per_wave *= 2;                            // two vector instructions per statement
    if (valu_instructions) *valu_instructions = per_wave * (int64_t)blocks * (kProbeBlock / 64);
    return ADAPTRA_OK;
}
