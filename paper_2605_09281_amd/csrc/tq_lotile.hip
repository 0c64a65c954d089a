// LoTileMoE: the fused low-rank path over shared 2D-tiled factors (Section 3.2, Eq. 14-16; Appendix A.4).
//
//   X_proj = x (U Sigma)_reshape     [T, M rp]    dense bf16 MFMA product, K optionally split over planes
//   S[b]^(n) = sum_{t: n(b,t)=n} g[b,t] X_proj[b]^(m(b,t))     gather-scale-accumulate, fixed order
//   y = S V_flat                     [T, out]     dense bf16 MFMA product
//
// Both factors sit in the packed blob as bf16 in v_mfma_f32_32x32x16_bf16 B-operand fragment order (every
// tile's r columns / rows padded to rp = 16 ceil(r/16) with zeros), so a wave loads a fragment with one
// 16-byte load per lane.  The left operand goes through LDS in 128-wide chunks shared by the four waves of a
// workgroup; each wave owns two column tiles of the 32 x 256 output block.
#include "tq_device.h"

namespace {

using namespace tqdev;

constexpr uint32_t LT_MAGIC = 0x544C5154u;   // "TQLT"
constexpr int LT_HEADER = 256;
constexpr int LT_CK = 128;                   // contraction indices per staged chunk
constexpr int LT_ROWB = LT_CK * 2 + 16;      // padded LDS row
constexpr int LT_MAX_PLANES = 16;

struct LtLayout {
    int E, M, N, n_in, n_out, r, rp, k;
    int n1, nt1, steps1;      // B1 = (U Sigma)_reshape: n1 = M rp columns in nt1 tiles, steps1 = n_in / 16
    int k2, nt2, steps2;      // B2 = V_flat: k2 = N rp rows (steps2 = k2 / 16), nt2 = n_out / 32 column tiles
    size_t off_phi, off_b1, off_b2, total;
};

bool lt_make_layout(const tq_lotile_desc* d, LtLayout* L)
{
    if (!d) return false;
    if (d->n_experts < 1 || d->tiles_m < 1 || d->tiles_n < 1 || d->n_in < 32 || d->n_out < 32) return false;
    if (d->n_in % 32 || d->n_out % 32 || d->rank < 1 || d->rank > 256) return false;
    if (d->top_k < 1 || d->top_k > d->n_experts || d->flags != 0) return false;
    if ((int64_t)d->tiles_m * d->tiles_n > (1 << 20)) return false;
    L->E = d->n_experts; L->M = d->tiles_m; L->N = d->tiles_n; L->n_in = d->n_in; L->n_out = d->n_out;
    L->r = d->rank; L->rp = (d->rank + 15) / 16 * 16; L->k = d->top_k;
    L->n1 = L->M * L->rp; L->nt1 = (L->n1 + 31) / 32; L->steps1 = L->n_in / 16;
    L->k2 = L->N * L->rp; L->steps2 = L->k2 / 16; L->nt2 = L->n_out / 32;
    size_t off = LT_HEADER;
    L->off_phi = off; off += tq_align256((size_t)L->E * 2 * 4);
    L->off_b1 = off; off += tq_align256((size_t)L->nt1 * L->steps1 * 64 * 16);
    L->off_b2 = off; off += tq_align256((size_t)L->nt2 * L->steps2 * 64 * 16);
    L->total = off;
    return true;
}

struct LtWorkspace {
    size_t ctrl, xproj, s, total;
    int planes, ldx;       // planes of X_proj (K splits of the first product), its row length (32 nt1)
};

void lt_make_workspace(const LtLayout& L, int T, LtWorkspace* W)
{
    // split the contraction of the first product when there are too few output blocks to fill the chip
    const int rt = (T + 31) / 32, cb = (L.nt1 + 7) / 8;
    int planes = 1;
    const int chunks = (L.steps1 + 7) / 8;
    while (planes < LT_MAX_PLANES && planes * 2 <= chunks && (long)rt * cb * planes < 256) planes *= 2;
    W->planes = planes;
    W->ldx = 32 * L.nt1;
    size_t off = 0;
    W->ctrl = off; off += 256;
    W->xproj = off; off += tq_align256((size_t)planes * T * W->ldx * 4);
    W->s = off; off += tq_align256((size_t)T * L.k2 * 2);
    W->total = off;
}

// ---- pack -------------------------------------------------------------------------------------------------
__global__ void lt_pack_kernel(LtLayout L, const uint16_t* __restrict__ us, const uint16_t* __restrict__ v,
                               const int32_t* __restrict__ phi, uint8_t* __restrict__ packed,
                               int32_t* __restrict__ err_flag)
{
    const size_t n_b1 = (size_t)L.nt1 * L.steps1 * 64, n_b2 = (size_t)L.nt2 * L.steps2 * 64;
    const size_t total = n_b1 + n_b2 + (size_t)L.E;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        if (i < n_b1 + n_b2) {
            const bool first = i < n_b1;
            const size_t j = first ? i : i - n_b1;
            const int steps = first ? L.steps1 : L.steps2;
            const int lane = (int)(j % 64);
            const int s = (int)((j / 64) % steps);
            const int ct = (int)(j / 64 / steps);
            const int col = 32 * ct + (lane & 31), k0 = 16 * s + 8 * (lane >> 5);
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t pr[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int kk = k0 + 2 * q + h;
                    uint16_t hb = 0;      // fp16 bits
                    if (first) {          // B1[kk][col]: col = m rp + rho
                        const int m = col / L.rp, rho = col % L.rp;
                        if (col < L.n1 && rho < L.r) hb = us[((size_t)m * L.n_in + kk) * L.r + rho];
                    } else {              // B2[kk][col]: kk = n rp + rho
                        const int n = kk / L.rp, rho = kk % L.rp;
                        if (rho < L.r) hb = v[((size_t)n * L.r + rho) * L.n_out + col];
                    }
                    pr[h] = f2bf_bits(tq_half_bits_to_float(hb));
                }
                w[q] = pr[0] | (pr[1] << 16);
            }
            u32x4 o = {w[0], w[1], w[2], w[3]};
            *reinterpret_cast<u32x4*>(packed + (first ? L.off_b1 : L.off_b2) + j * 16) = o;
        } else {
            const int e = (int)(i - n_b1 - n_b2);
            int m = phi[2 * e], n = phi[2 * e + 1];
            if (m < 0 || m >= L.M || n < 0 || n >= L.N) {
                if (err_flag) atomicOr(err_flag, 1);
                m = min(max(m, 0), L.M - 1);
                n = min(max(n, 0), L.N - 1);
            }
            int32_t* dst = reinterpret_cast<int32_t*>(packed + L.off_phi) + 2 * e;
            dst[0] = m;
            dst[1] = n;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 16) {
        const int32_t hdr[16] = {(int32_t)LT_MAGIC, 1, L.E, L.M, L.N, L.n_in, L.n_out, L.r, L.rp, 0, 0, 0, 0, 0, 0, 0};
        reinterpret_cast<int32_t*>(packed)[threadIdx.x] = hdr[threadIdx.x];
    }
}

// ---- dense product C[T, 32 nt] = A[T, 16 steps] B, B in fragment order ----------------------------------------
// grid (column blocks of 8 tiles, row tiles of 32, K splits); OUT_BF16: C bf16 [T][ldc], else fp32 planes
// [split][T][ldc].  Columns at or beyond ncols are not stored.
template <bool OUT_BF16>
__global__ void __launch_bounds__(256) lt_gemm_kernel(const uint16_t* __restrict__ A, int lda, int T,
                                                      const u32x4* __restrict__ bfrag, int steps, int ntiles,
                                                      void* __restrict__ C, int ldc, int ncols)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * 32 * LT_ROWB];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int row0 = blockIdx.y * 32;
    const int split = blockIdx.z, nsplit = gridDim.z;
    const int nchunks_all = (steps + 7) / 8;
    const int c0 = (int)((long)split * nchunks_all / nsplit), c1 = (int)((long)(split + 1) * nchunks_all / nsplit);
    // this wave's two column tiles (clamped: a tile past the end repeats the last one and is not stored)
    int ct[2];
    bool live[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int t = blockIdx.x * 8 + wave * 2 + j;
        live[j] = t < ntiles;
        ct[j] = live[j] ? t : ntiles - 1;
    }
    // staging: 32 rows x 16 segments of 16 bytes per chunk, two per thread
    const int srow = tid >> 4, sseg = tid & 15;
    const uint16_t* arow[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) arow[p] = A + (size_t)min(row0 + srow + 16 * p, T - 1) * lda;
    u32x4 xr[2];
    auto load_chunk = [&](int c) {
        const int kk = min(c * LT_CK + sseg * 8, steps * 16 - 8);
#pragma unroll
        for (int p = 0; p < 2; ++p) xr[p] = *reinterpret_cast<const u32x4*>(arow[p] + kk);
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 2; ++p)
            *reinterpret_cast<u32x4*>(lds + buf * 32 * LT_ROWB + (srow + 16 * p) * LT_ROWB + sseg * 16) = xr[p];
    };
    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    if (c0 < c1) {
        load_chunk(c0);
        store_chunk(0);
        lds_barrier();
        for (int c = c0; c < c1; ++c) {
            const int buf = (c - c0) & 1;
            u32x4 bq[8][2];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    bq[ks][j] = bfrag[((size_t)ct[j] * steps + min(c * 8 + ks, steps - 1)) * 64 + lane];
            load_chunk(min(c + 1, c1 - 1));
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                if (c * 8 + ks < steps) {
                    Frag xa, b0, b1;
                    xa.q = *reinterpret_cast<const u32x4*>(lds + buf * 32 * LT_ROWB + col * LT_ROWB + ks * 32 + hf * 16);
                    b0.q = bq[ks][0];
                    b1.q = bq[ks][1];
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa.v, b0.v, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa.v, b1.v, acc[1], 0, 0, 0);
                }
            }
            store_chunk(buf ^ 1);
            lds_barrier();
        }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int c = 32 * ct[j] + col;
        if (!live[j] || c >= ncols) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = row0 + 8 * (v / 4) + 4 * hf + (v % 4);
            if (m < T) {
                if (OUT_BF16) reinterpret_cast<uint16_t*>(C)[(size_t)m * ldc + c] = (uint16_t)f2bf_bits(acc[j][v]);
                else reinterpret_cast<float*>(C)[((size_t)split * T + m) * ldc + c] = acc[j][v];
            }
        }
    }
}

// ---- S[b][n rp + rho] = sum_t [n(b,t) == n] g[b,t] sum_planes X_proj[b][m(b,t) rp + rho]   (Eq. 16) ----------
__global__ void __launch_bounds__(256) lt_gather_kernel(LtLayout L, const int32_t* __restrict__ phi,
                                                        const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                        const float* __restrict__ xproj, int planes, int ldx, int T,
                                                        uint16_t* __restrict__ S, int32_t* __restrict__ err)
{
    __shared__ int32_t tm[64], tn[64];
    __shared__ float tg[64];
    const int b = blockIdx.x;
    for (int t0 = 0; t0 < L.k; t0 += 64) {      // top_k beyond 64 is handled in rounds
        __syncthreads();
        const int t = t0 + threadIdx.x;
        if (threadIdx.x < 64 && t < L.k) {
            const int e = idx[(size_t)b * L.k + t];
            if (e >= 0 && e < L.E) {
                tm[threadIdx.x] = phi[2 * e];
                tn[threadIdx.x] = phi[2 * e + 1];
                tg[threadIdx.x] = w[(size_t)b * L.k + t];
            } else {
                tm[threadIdx.x] = 0;
                tn[threadIdx.x] = -1;           // matches no column tile
                tg[threadIdx.x] = 0.f;
                atomicOr(err, 1);
            }
        }
        __syncthreads();
        const int nt = min(64, L.k - t0);
        for (int c = threadIdx.x; c < L.k2; c += blockDim.x) {
            const int n = c / L.rp, rho = c % L.rp;
            float sum = 0.f;
            for (int t2 = 0; t2 < nt; ++t2) {
                if (tn[t2] == n) {
                    float xp = 0.f;
                    for (int p = 0; p < planes; ++p) xp += xproj[((size_t)p * T + b) * ldx + tm[t2] * L.rp + rho];
                    sum = fmaf(tg[t2], xp, sum);
                }
            }
            // rounds after the first add to what the previous ones left (kept in fp32 in the plane-0 tail is not
            // possible here, so top_k > 64 re-reads the bf16 value: exact enough for the rare case)
            if (t0 > 0) sum += bf_lo((uint32_t)S[(size_t)b * L.k2 + c]);
            S[(size_t)b * L.k2 + c] = (uint16_t)f2bf_bits(sum);
        }
    }
}

__global__ void lt_clear_kernel(int32_t* ctrl)
{
    if (threadIdx.x < 64) ctrl[threadIdx.x] = 0;
}

}  // namespace

extern "C" size_t tq_lotile_packed_size(const tq_lotile_desc* desc)
{
    LtLayout L;
    return lt_make_layout(desc, &L) ? L.total : 0;
}

extern "C" tq_status tq_lotile_pack(const tq_lotile_desc* desc, const uint16_t* us, const uint16_t* v,
                                    const int32_t* phi, void* packed, size_t packed_bytes, int32_t* err_flag,
                                    void* stream)
{
    if (!desc || !us || !v || !phi || !packed) return TQ_ERR_NULL;
    LtLayout L;
    if (!lt_make_layout(desc, &L)) return TQ_ERR_SHAPE;
    if (((uintptr_t)packed & 255) || (((uintptr_t)us | (uintptr_t)v | (uintptr_t)phi) & 15)) return TQ_ERR_ALIGN;
    if (packed_bytes < L.total) return TQ_ERR_WORKSPACE;
    hipLaunchKernelGGL(lt_pack_kernel, dim3(1024), dim3(256), 0, (hipStream_t)stream, L, us, v, phi, (uint8_t*)packed,
                       err_flag);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

extern "C" size_t tq_lotile_workspace_size(const tq_lotile_desc* desc, int32_t T)
{
    LtLayout L;
    if (!lt_make_layout(desc, &L) || T < 0 || T > (1 << 24)) return 0;
    LtWorkspace W;
    lt_make_workspace(L, T, &W);
    return W.total;
}

extern "C" tq_status tq_lotile_forward(const tq_lotile_desc* desc, const void* packed, const void* x,
                                       const int32_t* topk_idx, const float* topk_w, int32_t T, void* y,
                                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (!desc || !packed || !x || !topk_idx || !topk_w || !y || !workspace) return TQ_ERR_NULL;
    LtLayout L;
    if (!lt_make_layout(desc, &L) || T < 0 || T > (1 << 24)) return TQ_ERR_SHAPE;
    if (((uintptr_t)packed | (uintptr_t)workspace) & 255) return TQ_ERR_ALIGN;
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)topk_idx | (uintptr_t)topk_w) & 15) return TQ_ERR_ALIGN;
    LtWorkspace W;
    lt_make_workspace(L, T, &W);
    if (workspace_bytes < W.total) return TQ_ERR_WORKSPACE;
    if (T == 0) return TQ_OK;
    hipStream_t st = (hipStream_t)stream;
    uint8_t* ws = (uint8_t*)workspace;
    const uint8_t* pk = (const uint8_t*)packed;
    int32_t* ctrl = (int32_t*)(ws + W.ctrl);
    float* xproj = (float*)(ws + W.xproj);
    uint16_t* S = (uint16_t*)(ws + W.s);
    const int rt = (T + 31) / 32;
    if (rt > 65535) return TQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(lt_clear_kernel, dim3(1), dim3(64), 0, st, ctrl);
    TQ_CHECK_LAUNCH();
    // step one: the global projection on every row tile's factor
    hipLaunchKernelGGL(lt_gemm_kernel<false>, dim3((L.nt1 + 7) / 8, rt, W.planes), dim3(256), 0, st,
                       (const uint16_t*)x, L.n_in, T, (const u32x4*)(pk + L.off_b1), L.steps1, L.nt1, (void*)xproj, W.ldx,
                       W.ldx);
    TQ_CHECK_LAUNCH();
    // step two: routing-weighted selection and accumulation into the compact buffer
    hipLaunchKernelGGL(lt_gather_kernel, dim3(T), dim3(256), 0, st, L, (const int32_t*)(pk + L.off_phi), topk_idx, topk_w,
                       (const float*)xproj, W.planes, W.ldx, T, S, ctrl);
    TQ_CHECK_LAUNCH();
    // step three: output reconstruction
    hipLaunchKernelGGL(lt_gemm_kernel<true>, dim3((L.nt2 + 7) / 8, rt, 1), dim3(256), 0, st, (const uint16_t*)S, L.k2, T,
                       (const u32x4*)(pk + L.off_b2), L.steps2, L.nt2, y, L.n_out, L.n_out);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}
