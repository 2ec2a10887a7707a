// Register-only matrix-core loops: what the contraction step of the product kernels could reach on this part if
// nothing but its MFMA instruction ran.  One wavefront per SIMD with all 256 accumulator registers in use, exactly
// the register shape of the product kernels' wavefront tiles, operands loaded once and then held in registers:
//   kind 0 : V_MFMA_F32_32X32X2_F32,  4 x 4 accumulator blocks, 64 MFMAs per pass (one 8-k chunk of the fp32 kernel)
//   kind 1 : V_MFMA_F32_16X16X32_BF16, 8 x 8 accumulator blocks, 128 MFMAs per pass (one K-tile of the bf16 kernel: the two
//            k-steps of a block back to back, as that kernel issues them -- the second MFMA then takes the first one's
//            result as its addend without a trip through the register file, which on random operands sustains about
//            6 % more than the same MFMAs issued k-step by k-step)
// The rate depends on the operand values (a matrix core working on zeros draws far less power than one working on
// random data, and under the power limit the clock follows), so the caller brings the operands.
// The result is a measurement aid for the profiler leg: it computes nothing a caller would want.
#include "launchers.hpp"

namespace fsrgemm {
namespace {

constexpr int kThreads = 256;

template <int KIND>
__global__ __launch_bounds__(kThreads) void mfma_ceiling_kernel(const u32x4 *__restrict__ operands, float *__restrict__ sink, int passes)
{
    const int lane = threadIdx.x & 63;
    float s = 0.f;
    if constexpr (KIND == 0) {
        // 16 + 16 operand values per lane: fragment q of 8 (4 of A, 4 of B), four k-steps each, from piece q * 64 + lane
        float a[4][4], b[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4 va = operands[q * 64 + lane], vb = operands[(4 + q) * 64 + lane];
#pragma unroll
            for (int t = 0; t < 4; ++t) a[q][t] = __builtin_bit_cast(float, va[t]), b[q][t] = __builtin_bit_cast(float, vb[t]);
        }
        f32x16 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
                asm volatile("" : "+a"(acc[i][j]));
            }
        for (int p = 0; p < passes; ++p) {
#pragma unroll
            for (int m = 0; m < 64; ++m) {
                const int t = m >> 4, i = (m >> 2) & 3, j = m & 3;
                asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[i][t]), "v"(b[j][t]));
            }
        }
        // the last MFMAs retire before the accumulators are read (the compiler does not know what wrote them);
        // the empty statements make every read of a block depend on a statement that follows the wait
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                asm volatile("" : "+a"(acc[i][j]));
#pragma unroll
                for (int r = 0; r < 16; ++r) s += acc[i][j][r];
            }
    } else {
        bf16x8 a[2][8], b[2][8];        // [k-step][block row / column]: fragment q of 32, from piece q * 64 + lane
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            a[q >> 3][q & 7] = __builtin_bit_cast(bf16x8, operands[q * 64 + lane]);
            b[q >> 3][q & 7] = __builtin_bit_cast(bf16x8, operands[(16 + q) * 64 + lane]);
        }
        f32x4 acc[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                asm volatile("" : "+a"(acc[i][j]));
            }
        for (int p = 0; p < passes; ++p) {
#pragma unroll
            for (int m = 0; m < 128; ++m) {
                const int i = m >> 4, j = (m >> 1) & 7, kk = m & 1;
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(a[kk][i]), "v"(b[kk][j]));
            }
        }
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                asm volatile("" : "+a"(acc[i][j]));
                s += (acc[i][j][0] + acc[i][j][1]) + (acc[i][j][2] + acc[i][j][3]);
            }
    }
    sink[(int64_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

}  // namespace

// flop of one launch: workgroups x 4 wavefronts x passes x (64 MFMAs of 4096 | 128 MFMAs of 16384) flop
double mfma_ceiling_flop(int kind, int passes, int workgroups)
{
    return (double)workgroups * 4.0 * (double)passes * (kind == 0 ? 64.0 * 4096.0 : 128.0 * 16384.0);
}

const char *mfma_ceiling_kernel_name(int kind) { return kind == 0 ? "mfma_ceiling_kernel<0>" : "mfma_ceiling_kernel<1>"; }

hipError_t launch_mfma_ceiling(int kind, int passes, const void *operands, float *sink, int workgroups, hipStream_t s)
{
    const u32x4 *ops = static_cast<const u32x4 *>(operands);
    if (kind == 0) hipLaunchKernelGGL(mfma_ceiling_kernel<0>, dim3((unsigned)workgroups), dim3(kThreads), 0, s, ops, sink, passes);
    else hipLaunchKernelGGL(mfma_ceiling_kernel<1>, dim3((unsigned)workgroups), dim3(kThreads), 0, s, ops, sink, passes);
    return hipGetLastError();
}

}  // namespace fsrgemm
