// Measurement aid (not part of the method): the instruction mix of the prefill kernels' main loop without any global
// memory traffic, to find what the compute units sustain for it.  One workgroup of four waves per launch slot, each
// wave on a 64 x 64 output tile (2 x 2 MFMA tiles of 32 x 32) walking over groups of 8 steps of 16, as
// moe_prefill_kernel does for quantisation groups of 128:
//   level 0: the MFMAs alone, operands in registers (four independent accumulator chains)
//   level 1: + the two A fragments of every step read from LDS (ds_read_b128)
//   level 2: + the two B fragments of every step unpacked from 4-bit codes (3 shifts and 4 and-or per fragment)
//   level 3: + the fold of every group's partial sums into the accumulators (16 FMAs per tile and group)
//   level 4: + per group, the store of the next activation tile into the other half of an LDS double buffer (four
//            16-byte stores per thread) and the workgroup barrier that publishes it
// Every level runs with two workgroups per compute unit (two waves per SIMD), as the kernel does.  The kernel reports
// its own cycle count and wall-clock time, so the clock the chip sustained under that load is known.
#include "tq_device.h"

using namespace tqdev;

namespace {

template <int LEVEL>
__global__ void __launch_bounds__(256, 2) issue_probe_kernel(float* __restrict__ out, int iters, uint32_t mask, uint32_t magic_s,
                                                             const float* __restrict__ scales,
                                                             unsigned long long* __restrict__ clk)
{
    constexpr int MT = 2, NT = 2, GS = 8, ROWB = 272, BUFB = 32 * MT * ROWB;
    constexpr int NBUF = LEVEL >= 4 ? 2 : 1;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    for (int i = threadIdx.x; i < (NBUF * BUFB) / 4; i += blockDim.x) reinterpret_cast<uint32_t*>(lds)[i] = 0x3F803F80u + (i & 3);
    __syncthreads();
    u32x4 xr[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) { xr[m][0] = 0x3F803F80u; xr[m][1] = 0x3F803F81u; xr[m][2] = 0x3F803F82u; xr[m][3] = 0x3F803F83u; }
    const uint32_t wr_off = (threadIdx.x >> 4) * ROWB + (threadIdx.x & 15) * 16;      // 16 rows x 256 bytes per pass
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    uint32_t magic;
    asm volatile("v_mov_b32 %0, %1" : "=v"(magic) : "s"(magic_s));
    f32x16 acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][t][v] = 0.f;
    uint32_t w[NT][GS];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int s = 0; s < GS; ++s) w[t][s] = 0x12345678u * (threadIdx.x + 1) + t * 977 + s * 131;
    Frag areg[MT], breg[NT];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        areg[0].u[j] = 0x3F803F80u + j; areg[1].u[j] = 0x3F813F80u + j;
        breg[0].u[j] = 0x43014302u + j; breg[1].u[j] = 0x43034304u + j;
    }
    const uint8_t* base0 = lds + col * ROWB + hf * 16;
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        float sc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) sc[t] = scales[(it * NT + t) & 63];
        const uint8_t* base = base0 + (LEVEL >= 4 ? (it & 1) * BUFB : 0);
        f32x16 part[MT][NT];
#pragma unroll
        for (int ks = 0; ks < GS; ++ks) {
            Frag a[MT];
            bf16x8 b[NT];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (LEVEL >= 1) a[m].q = *reinterpret_cast<const u32x4*>(base + m * 32 * ROWB + ((ks + it) & 7) * 32);
                else a[m] = areg[m];
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (LEVEL >= 2) b[t] = unpack_word(w[t][ks] + it, mask, magic);
                else b[t] = breg[t].v;
            }
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    if (LEVEL >= 3) {
                        if (ks == 0) {
                            f32x16 z;
#pragma unroll
                            for (int v = 0; v < 16; ++v) z[v] = 0.f;
                            part[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m].v, b[t], z, 0, 0, 0);
                        } else {
                            part[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m].v, b[t], part[m][t], 0, 0, 0);
                        }
                    } else {
                        acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m].v, b[t], acc[m][t], 0, 0, 0);
                    }
                }
        }
        if (LEVEL >= 3) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[m][t][v] = fmaf(sc[t], part[m][t][v], acc[m][t][v]);
            if (LEVEL >= 4) {
                uint8_t* dst = lds + ((it + 1) & 1) * BUFB + wr_off;
#pragma unroll
                for (int m = 0; m < MT * 2; ++m) *reinterpret_cast<u32x4*>(dst + m * 16 * ROWB) = xr[m % MT];
                lds_barrier();
            }
        } else if (LEVEL < 2) {
            // keep the register operands loop-variant so that the steps are not merged
#pragma unroll
            for (int t = 0; t < NT; ++t) breg[t].u[0] ^= (uint32_t)(sc[t] != 7.f);
        }
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[m][t][v];
    if (s == 1.2345f) out[threadIdx.x] = s;      // practically never: keeps the result alive
}

}  // namespace

// MFMAs one wave issues per launch: iters groups of 8 steps on 2 x 2 tiles
extern "C" tq_status tq_debug_issue_probe(int32_t level, int32_t iters, void* scratch, size_t scratch_bytes, void* stream)
{
    if (!scratch) return TQ_ERR_NULL;
    if ((uintptr_t)scratch & 255) return TQ_ERR_ALIGN;
    if (level < 0 || level > 4 || iters < 1 || iters > (1 << 20)) return TQ_ERR_SHAPE;
    if (scratch_bytes < 4096) return TQ_ERR_WORKSPACE;
    const TqDeviceState* ds = nullptr;
    if (tqi_device_state(&ds) != TQ_OK) return TQ_ERR_HIP;
    // scratch: [0, 16) the two counters, [256, 512) 64 scales (whatever the caller left there: any finite values),
    // [1024, 2048) the never-written result
    unsigned long long* clk = reinterpret_cast<unsigned long long*>(scratch);
    const float* scales = reinterpret_cast<const float*>(reinterpret_cast<uint8_t*>(scratch) + 256);
    float* out = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(scratch) + 1024);
    const size_t smem = (level >= 4 ? 2 : 1) * 32 * 2 * 272 + 64;
    const dim3 grid(2 * ds->n_cu), block(256);
    hipStream_t st = (hipStream_t)stream;
    switch (level) {
    case 0: hipLaunchKernelGGL(issue_probe_kernel<0>, grid, block, smem, st, out, iters, 0x000F000Fu, 0x43004300u, scales, clk); break;
    case 1: hipLaunchKernelGGL(issue_probe_kernel<1>, grid, block, smem, st, out, iters, 0x000F000Fu, 0x43004300u, scales, clk); break;
    case 2: hipLaunchKernelGGL(issue_probe_kernel<2>, grid, block, smem, st, out, iters, 0x000F000Fu, 0x43004300u, scales, clk); break;
    case 3: hipLaunchKernelGGL(issue_probe_kernel<3>, grid, block, smem, st, out, iters, 0x000F000Fu, 0x43004300u, scales, clk); break;
    default: hipLaunchKernelGGL(issue_probe_kernel<4>, grid, block, smem, st, out, iters, 0x000F000Fu, 0x43004300u, scales, clk); break;
    }
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}
