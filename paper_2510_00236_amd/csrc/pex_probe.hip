// pex_probe.hip -- what the MFMA pipes of this chip sustain when nothing else happens: the ceiling against which the
// contraction kernels are also reported.  The datasheet rate (2.5 PFLOP/s dense bf16) assumes the peak clock; under a
// full MFMA load with realistic operand values the chip settles at a lower one (with all-zero or all-one operands the
// same loop reaches 2.47 PFLOP/s), and that, not an issue limit, is what bounds a kernel that keeps the pipes busy.
// The probe has the register shape of the 256 x 256 tile kernel (8 waves per workgroup, one workgroup per compute
// unit, per wave 8 x 4 accumulators of v_mfma_f32_16x16x32_bf16 fed by 8 + 4 operand fragments, the same back-and-
// forth order of the MFMAs) and issues nothing but those MFMAs; the operands come from a caller-supplied buffer (their
// values matter: switching activity sets the power and with it the clock) and alternate between two register sets.
// For the record: the 32x32x16 form of the instruction sustains 1.80 PFLOP/s in this loop, this one 2.07-2.11.
#include "pex_internal.h"

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float float4_t;
typedef __attribute__((ext_vector_type(4))) unsigned int uint4_t;

constexpr int PROBE_WAVES = 8, PROBE_FM = 8, PROBE_FN = 4, PROBE_SETS = 2;
constexpr int PROBE_FRAGS = PROBE_SETS * (PROBE_FM + PROBE_FN);   // 16-byte fragments a lane loads

__global__ __launch_bounds__(PROBE_WAVES * 64, 1) void mfma_probe_kernel(const uint4_t* __restrict__ operands, int iters,
                                                                         float* __restrict__ sink)
{
    const int lane_global = blockIdx.x * blockDim.x + threadIdx.x;
    bf16x8_t a[PROBE_SETS][PROBE_FM], b[PROBE_SETS][PROBE_FN];
    const uint4_t* src = operands + (size_t)(threadIdx.x % (PROBE_WAVES * 64)) * PROBE_FRAGS;
#pragma unroll
    for (int s = 0; s < PROBE_SETS; ++s) {
#pragma unroll
        for (int i = 0; i < PROBE_FM; ++i) a[s][i] = __builtin_bit_cast(bf16x8_t, src[s * (PROBE_FM + PROBE_FN) + i]);
#pragma unroll
        for (int j = 0; j < PROBE_FN; ++j) b[s][j] = __builtin_bit_cast(bf16x8_t, src[s * (PROBE_FM + PROBE_FN) + PROBE_FM + j]);
    }
    float4_t acc[PROBE_FM][PROBE_FN];
#pragma unroll
    for (int i = 0; i < PROBE_FM; ++i)
#pragma unroll
        for (int j = 0; j < PROBE_FN; ++j) acc[i][j] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < PROBE_SETS; ++s)
#pragma unroll
            for (int i = 0; i < PROBE_FM; ++i)
#pragma unroll
                for (int jj = 0; jj < PROBE_FN; ++jj) {
                    const int j = (i & 1) ? PROBE_FN - 1 - jj : jj;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s][i], b[s][j], acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
    }
    float total = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_FM; ++i)
#pragma unroll
        for (int j = 0; j < PROBE_FN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) total += acc[i][j][r];
    sink[lane_global] = total;
}

}  // namespace

size_t probe_operand_bytes() { return (size_t)PROBE_WAVES * 64 * PROBE_FRAGS * 16; }
size_t probe_sink_floats(int workgroups) { return (size_t)workgroups * PROBE_WAVES * 64; }
double probe_flop(int workgroups, int iters)
{
    return (double)workgroups * PROBE_WAVES * (double)iters * PROBE_SETS * PROBE_FM * PROBE_FN * (2.0 * 16 * 16 * 32);
}

hipError_t launch_mfma_probe(const void* operands, int workgroups, int iters, float* sink, hipStream_t stream)
{
    mfma_probe_kernel<<<dim3(workgroups), dim3(PROBE_WAVES * 64), 0, stream>>>((const uint4_t*)operands, iters, sink);
    return hipGetLastError();
}

}  // namespace pex
