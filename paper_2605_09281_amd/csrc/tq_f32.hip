// fp32-activation debug path of tq_moe_forward: exact (q - zero) * scale dequantisation, fp32 FMA
// accumulation, no rounding of intermediates below fp32.  One workgroup per (assignment row, four
// column-tile pairs); it reads the same packed blob as the MFMA path by index arithmetic.
// Built for checking the data flow at ~1e-6, not for speed.
#include "tq_common.h"

namespace {

struct F32Geom {
    int32_t ne, H, F, g, r, r16, k, S, cw;
    size_t expert_stride;
    TqFactorMap fm;
};

__device__ inline float silu_f32(float v) { return v / (1.0f + expf(-v)); }

// code i (0..7) of k-step w (0..3) of a chunk whose words are d[0..cw-1]: 4-bit slots (cw = 4) or dense 3- / 2-bit
// codes, as the layout text of the public header states them
__device__ inline uint32_t code_of_chunk(const uint32_t* d, int cw, int w, int i)
{
    if (cw == 4) return (d[w] >> (4 * tq_nibble_pos(i))) & 15u;
    const int P = 4 * w + (i >> 1), half = 16 * (i & 1);
    if (cw == 2) return (d[P / 8] >> (2 * (P % 8) + half)) & 3u;
    if (P < 15) return (d[P / 5] >> (3 * (P % 5) + half)) & 7u;
    return ((d[0] >> (15 + half)) & 1u) | (((d[1] >> (15 + half)) & 1u) << 1) | (((d[2] >> (15 + half)) & 1u) << 2);
}

// STAGE 0: gate/up + SwiGLU (input x gathered by token, output h32[slot][F])
// STAGE 1: down (input h32[slot][F], output yd[slot][H])
template <int STAGE>
__global__ void __launch_bounds__(256) f32_proj_kernel(F32Geom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                       const float* __restrict__ xin,
                                                       const int32_t* __restrict__ row_token,
                                                       const int32_t* __restrict__ offsets,
                                                       const int32_t* __restrict__ ctrl, float* __restrict__ out)
{
    extern __shared__ float smem[];
    const int K = sec.K;
    const int NA = STAGE == 0 ? 2 * G.r16 : G.r16;
    float* xs = smem;        // [K]
    float* ts = smem + K;    // [NA]
    const int slot = blockIdx.x;
    if (slot >= ctrl[3]) return;
    const int e = tq_find_expert(offsets, G.ne, slot);
    const float* xrow = STAGE == 0 ? xin + (size_t)row_token[slot] * G.H : xin + (size_t)slot * G.F;
    for (int kk = threadIdx.x; kk < K; kk += 256) xs[kk] = xrow[kk];
    __syncthreads();
    const uint8_t* rec = blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, hf = lane >> 5;
    // t[c] = sum_kk x[kk] * A[kk][c]
    if (G.r > 0) {
        const uint16_t* af = reinterpret_cast<const uint16_t*>(tq_afrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e));
        const uint8_t* af8 = reinterpret_cast<const uint8_t*>(af);       // fp8 factors: the same layout with 1-byte elements
        const float* sig = G.fm.fp8 ? tq_sig_base(blob, G.expert_stride, sec, G.fm, STAGE, e) : nullptr;
        const int ksteps = K / 16;
        for (int c = wave; c < NA; c += 4) {
            const int ta = c >> 5, cl = c & 31;
            float p = 0.f;
            for (int kk = lane; kk < K; kk += 64) {
                int s = kk >> 4, h2 = (kk >> 3) & 1, i = kk & 7;
                size_t ai = (((size_t)ta * ksteps + s) * 64 + h2 * 32 + cl) * 8 + i;
                p = fmaf(xs[kk], G.fm.fp8 ? tq_fp8_to_float(af8[ai]) : tq_half_bits_to_float(af[ai]), p);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) p += __shfl_xor(p, off);
            if (lane == 0) ts[c] = sig ? p * sig[c] : p;
        }
    }
    __syncthreads();
    const int pair = blockIdx.y * 4 + wave;
    if (pair >= sec.pairs) return;
    float res[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
        const uint32_t* cwp = reinterpret_cast<const uint32_t*>(rec + sec.codes);
        const uint32_t* szp = reinterpret_cast<const uint32_t*>(rec + sec.sz) + ((size_t)pair * sec.groups * 2 + tile) * 32 + col;
        float acc = 0.f, part = 0.f, s = 0.f, z = 0.f;
        int cur = -1;
        for (int c = 0; c < sec.chunks; ++c) {
            uint32_t wd[4] = {0, 0, 0, 0};
            {
                const size_t blk = ((size_t)pair * sec.chunks + c) * 2 + tile;      // (pair, chunk, tile)
                if (G.cw == 4) {
                    const uint4 v = reinterpret_cast<const uint4*>(cwp)[blk * 64 + lane];
                    wd[0] = v.x; wd[1] = v.y; wd[2] = v.z; wd[3] = v.w;
                } else {
                    for (int d = 0; d < G.cw; ++d) wd[d] = cwp[(blk * G.cw + d) * 64 + lane];
                }
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                int gi = (64 * c + 16 * w) / G.g;
                if (gi != cur) {
                    acc = fmaf(part, s, acc);
                    part = 0.f;
                    uint32_t sz = szp[(size_t)gi * 64];
                    s = tq_half_bits_to_float((uint16_t)(sz & 0xFFFF));
                    z = tq_half_bits_to_float((uint16_t)(sz >> 16));
                    cur = gi;
                }
                const int kk0 = 64 * c + 16 * w + 8 * hf;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float q = (float)code_of_chunk(wd, G.cw, w, i);
                    part = fmaf(xs[kk0 + i], q - z, part);
                }
            }
        }
        acc = fmaf(part, s, acc);
        if (G.r > 0) {
            const uint8_t* bbase = tq_bfrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e);
            const uint4* bf = reinterpret_cast<const uint4*>(bbase) + ((size_t)pair * (G.r16 / 16) * 2 + tile) * 64 + lane;
            const uint2* bf8 = reinterpret_cast<const uint2*>(bbase) + ((size_t)pair * (G.r16 / 16) * 2 + tile) * 64 + lane;
            const float* tp = ts + (STAGE == 0 ? tile * G.r16 : 0);
            float lr = 0.f;
            for (int st = 0; st < G.r16 / 16; ++st) {
                if (G.fm.fp8) {
                    const uint2 b = bf8[(size_t)st * 128];
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        lr = fmaf(tp[16 * st + 8 * hf + i], tq_fp8_to_float(((i < 4 ? b.x : b.y) >> (8 * (i & 3))) & 0xFF), lr);
                } else {
                    uint4 b = bf[(size_t)st * 128];
                    uint32_t bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        uint16_t hb = (uint16_t)(bw[i >> 1] >> (16 * (i & 1)));
                        lr = fmaf(tp[16 * st + 8 * hf + i], tq_half_bits_to_float(hb), lr);
                    }
                }
            }
            acc += lr;
        }
        acc += __shfl_xor(acc, 32);
        res[tile] = acc;
    }
    if (hf == 0) {
        if (STAGE == 0) {
            out[(size_t)slot * G.F + 32 * pair + col] = silu_f32(res[0]) * res[1];
        } else {
            out[(size_t)slot * G.H + 64 * pair + col] = res[0];
            out[(size_t)slot * G.H + 64 * pair + 32 + col] = res[1];
        }
    }
}

// y[t][c] = sum_j w[t][j] * yd[slot_of[t][j]][c] + sum_s yd[slot_of[t][k+s]][c], terms added in slot order
__global__ void __launch_bounds__(256) f32_combine_kernel(int T, int H, int k, int S,
                                                          const int32_t* __restrict__ slot_of,
                                                          const float* __restrict__ w,
                                                          const float* __restrict__ yd, float* __restrict__ y)
{
    const int t = blockIdx.x;
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= H) return;
    float acc = 0.f;
    for (int j = 0; j < k + S; ++j) {
        int slot = slot_of[(size_t)t * (k + S) + j];
        if (slot < 0) continue;
        float wj = j < k ? w[(size_t)t * k + j] : 1.0f;
        acc = fmaf(wj, yd[(size_t)slot * H + c], acc);
    }
    y[(size_t)t * H + c] = acc;
}

}  // namespace

tq_status tqi_forward_f32(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, const float* x,
                          int32_t T, float* y, uint8_t* ws, hipStream_t stream, const float* topk_w)
{
    F32Geom G;
    G.ne = L.E + L.S; G.H = L.H; G.F = L.F; G.g = L.g; G.r = L.r; G.r16 = L.r16; G.k = L.k; G.S = L.S;
    G.expert_stride = L.expert_stride; G.cw = L.cw; G.fm = L.fm;
    const int32_t* ctrl = reinterpret_cast<const int32_t*>(ws + W.ctrl);
    const int32_t* offsets = reinterpret_cast<const int32_t*>(ws + W.offsets);
    const int32_t* slot_of = reinterpret_cast<const int32_t*>(ws + W.slot_of);
    const int32_t* row_token = reinterpret_cast<const int32_t*>(ws + W.row_token);
    float* h32 = reinterpret_cast<float*>(ws + W.h);
    float* yd = reinterpret_cast<float*>(ws + W.yd);
    size_t sm0 = ((size_t)L.H + 2 * L.r16) * 4, sm1 = ((size_t)L.F + L.r16) * 4;
    if (sm0 > 160 * 1024 || sm1 > 160 * 1024) return TQ_ERR_UNSUPPORTED;
    if (sm0 > 48 * 1024)
        if (hipFuncSetAttribute((const void*)f32_proj_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm0) != hipSuccess) return TQ_ERR_HIP;
    if (sm1 > 48 * 1024)
        if (hipFuncSetAttribute((const void*)f32_proj_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm1) != hipSuccess) return TQ_ERR_HIP;
    hipLaunchKernelGGL(f32_proj_kernel<0>, dim3(W.a_tot, (L.gu.pairs + 3) / 4), dim3(256), sm0, stream, G, L.gu, blob, x,
                       row_token, offsets, ctrl, h32);
    TQ_CHECK_LAUNCH();
    tqi_record_stage(3, stream);
    hipLaunchKernelGGL(f32_proj_kernel<1>, dim3(W.a_tot, (L.d.pairs + 3) / 4), dim3(256), sm1, stream, G, L.d, blob, h32,
                       row_token, offsets, ctrl, yd);
    TQ_CHECK_LAUNCH();
    tqi_record_stage(5, stream);
    hipLaunchKernelGGL(f32_combine_kernel, dim3(T, (L.H + 255) / 256), dim3(256), 0, stream, T, L.H, L.k, L.S,
                       slot_of, topk_w, yd, y);
    TQ_CHECK_LAUNCH();
    tqi_record_stage(6, stream);
    return TQ_OK;
}
