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

#include <algorithm>
#include <vector>

namespace {

using namespace tqdev;

constexpr uint32_t LT_MAGIC = 0x544C5154u;   // "TQLT"
constexpr int LT_HEADER = 256;
constexpr int LT_SPC = 8;                    // MFMA steps per staged chunk
constexpr int LT_CK = 16 * LT_SPC;           // contraction indices per staged chunk
constexpr int LT_ROWB = LT_CK * 2 + 16;      // padded LDS row
constexpr int LT_MAX_PLANES = 16;

struct LtLayout {
    int E, M, N, n_in, n_out, r, rp, k;
    int n1, nt1, steps1;      // B1 = (U Sigma)_reshape: n1 = M rp columns in nt1 tiles, steps1 = n_in / 16
    int k2, nt2, steps2;      // B2 = V_flat: k2 = N rp rows (steps2 = k2 / 16), nt2 = n_out / 32 column tiles
    size_t off_phi, off_sigma, off_b1, off_b2, total;
    int fp8;                  // factors stored as fp8 E4M3 with an fp32 copy of the fp16 Sigma (else bf16, no Sigma)
    int nsp1, nsp2;           // fp8: step pairs per column tile (one 16-byte lane load holds two steps)
};

bool lt_make_layout(const tq_lotile_desc* d, LtLayout* L)
{
    if (!d) return false;
    if (d->n_experts < 1 || d->tiles_m < 1 || d->tiles_n < 1 || d->n_in < 32 || d->n_out < 32) return false;
    if (d->n_in % 32 || d->n_out % 32 || d->rank < 1 || d->rank > 256) return false;
    if (d->top_k < 1 || d->top_k > d->n_experts || d->top_k > 1024 || (d->flags & ~TQ_LOTILE_FP8)) return false;
    if ((int64_t)d->tiles_m * d->tiles_n > (1 << 20)) return false;
    L->E = d->n_experts; L->M = d->tiles_m; L->N = d->tiles_n; L->n_in = d->n_in; L->n_out = d->n_out;
    L->r = d->rank; L->rp = (d->rank + 15) / 16 * 16; L->k = d->top_k;
    L->n1 = L->M * L->rp; L->nt1 = (L->n1 + 31) / 32; L->steps1 = L->n_in / 16;
    L->k2 = L->N * L->rp; L->steps2 = L->k2 / 16; L->nt2 = L->n_out / 32;
    size_t off = LT_HEADER;
    L->off_phi = off; off += tq_align256((size_t)L->E * 2 * 4);
    L->fp8 = (d->flags & TQ_LOTILE_FP8) != 0;
    L->nsp1 = (L->steps1 + 1) / 2; L->nsp2 = (L->steps2 + 1) / 2;
    L->off_sigma = off; off += L->fp8 ? tq_align256((size_t)L->rp * 4) : 0;
    L->off_b1 = off; off += tq_align256((size_t)L->nt1 * (L->fp8 ? L->nsp1 : L->steps1) * 64 * 16);
    L->off_b2 = off; off += tq_align256((size_t)L->nt2 * (L->fp8 ? L->nsp2 : L->steps2) * 64 * 16);
    L->total = off;
    return true;
}

struct LtWorkspace {
    size_t ctrl, xproj, s, total;
    int mt;                // row sub-tiles of 32 per workgroup (1 for decode batches, else 2)
    int ntw1, planes;      // first product: column tiles per wave, K splits (= planes of X_proj)
    int ntw2;              // second product: column tiles per wave
    int ldx;               // row length of X_proj (32 nt1)
};

void lt_make_workspace(const LtLayout& L, int T, LtWorkspace* W)
{
    W->mt = T <= 32 ? 1 : 2;
    const int bm = 32 * W->mt, rt = (T + bm - 1) / bm;
    // first product: as many column tiles per wave as there are (up to 3), and the contraction split over
    // planes when there are too few output blocks to fill the chip
    W->ntw1 = std::min(3, (L.nt1 + 3) / 4);
    const int cb1 = (L.nt1 + 4 * W->ntw1 - 1) / (4 * W->ntw1), chunks = (L.steps1 + LT_SPC - 1) / LT_SPC;
    int planes = 1;
    while (planes < LT_MAX_PLANES && planes * 2 <= chunks && (long)rt * cb1 * planes < 256) planes *= 2;
    W->planes = planes;
    // second product: its contraction is short, so narrower workgroups fill the chip instead
    int ntw2 = std::min(3, (L.nt2 + 3) / 4);
    while (ntw2 > 1 && (long)rt * ((L.nt2 + 4 * ntw2 - 1) / (4 * ntw2)) < 256) --ntw2;
    W->ntw2 = ntw2;
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

// fp8 factors: bytes are only rearranged (two MFMA steps per 16-byte lane load), Sigma is widened to fp32
__global__ void lt_pack_fp8_kernel(LtLayout L, const uint8_t* __restrict__ u8, const uint16_t* __restrict__ sigma,
                                   const uint8_t* __restrict__ v8, const int32_t* __restrict__ phi,
                                   uint8_t* __restrict__ packed, int32_t* __restrict__ err_flag)
{
    const size_t n_b1 = (size_t)L.nt1 * L.nsp1 * 64, n_b2 = (size_t)L.nt2 * L.nsp2 * 64;
    const size_t total = n_b1 + n_b2 + (size_t)L.E + (size_t)L.rp;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        if (i < n_b1 + n_b2) {
            const bool first = i < n_b1;
            const size_t j = first ? i : i - n_b1;
            const int nsp = first ? L.nsp1 : L.nsp2, steps = first ? L.steps1 : L.steps2;
            const int lane = (int)(j % 64);
            const int sp = (int)((j / 64) % nsp);
            const int ct = (int)(j / 64 / nsp);
            const int col = 32 * ct + (lane & 31);
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                const int s = 2 * sp + b / 8, kk = 16 * s + 8 * (lane >> 5) + (b & 7);
                uint32_t byte = 0;
                if (s < steps) {
                    if (first) {          // B1[kk][col]: col = m rp + rho
                        const int m = col / L.rp, rho = col % L.rp;
                        if (col < L.n1 && rho < L.r) byte = u8[((size_t)m * L.n_in + kk) * L.r + rho];
                    } else {              // B2[kk][col]: kk = n rp + rho
                        const int n = kk / L.rp, rho = kk % L.rp;
                        if (rho < L.r) byte = v8[((size_t)n * L.r + rho) * L.n_out + col];
                    }
                }
                w[b / 4] |= byte << (8 * (b & 3));
            }
            u32x4 o = {w[0], w[1], w[2], w[3]};
            *reinterpret_cast<u32x4*>(packed + (first ? L.off_b1 : L.off_b2) + j * 16) = o;
        } else if (i < n_b1 + n_b2 + (size_t)L.E) {
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
        } else {
            const int rho = (int)(i - n_b1 - n_b2 - (size_t)L.E);
            reinterpret_cast<float*>(packed + L.off_sigma)[rho] = rho < L.r ? tq_half_bits_to_float(sigma[rho]) : 0.f;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < 16) {
        const int32_t hdr[16] = {(int32_t)LT_MAGIC, 1, L.E, L.M, L.N, L.n_in, L.n_out, L.r, L.rp, 1, 0, 0, 0, 0, 0, 0};
        reinterpret_cast<int32_t*>(packed)[threadIdx.x] = hdr[threadIdx.x];
    }
}

// ---- dense product C[T, 32 nt] = A[T, 16 steps] B, B in fragment order ----------------------------------------
// grid (column blocks of 4 NTW tiles, row tiles of 32 MT rows, K splits).  A workgroup stages its rows of A
// through LDS in 128-wide chunks; wave w owns NTW column tiles and all MT row sub-tiles, so a B fragment (one
// 16-byte load per lane, prefetched four steps ahead) feeds MT MFMAs and an A fragment (one LDS read) NTW of them.
// OUT_BF16: C bf16 [T][ldc], else fp32 planes [split][T][ldc].
struct LtGemmArgs {
    const uint16_t* A;
    int lda, T;
    const u32x4* bfrag;
    int steps, ntiles;    // MFMA steps of the contraction, column tiles of B
    int nsp;              // fp8 only: step pairs per column tile
    void* C;
    int ldc;
    int32_t* clear;       // not null: the first workgroup zeroes this word (the operator's error flag)
};

template <int MT, int NTW, bool OUT_BF16, bool FP8>
__global__ void __launch_bounds__(256) lt_gemm_kernel(LtGemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    constexpr int BM = 32 * MT, NSEG = LT_CK / 8, RPP = 256 / NSEG, NP = BM / RPP, BUF = BM * LT_ROWB, PF = 4, SPC = LT_SPC;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int row0 = blockIdx.y * BM, T = a.T, steps = a.steps;
    const int split = blockIdx.z, nsplit = gridDim.z;
    const int nchunks_all = (steps + SPC - 1) / SPC;
    const int c0 = (int)((long)split * nchunks_all / nsplit), c1 = (int)((long)(split + 1) * nchunks_all / nsplit);
    if (a.clear && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) *a.clear = 0;
    // this wave's column tiles (a tile past the end repeats the last one and is not stored)
    int ct[NTW];
    bool live[NTW];
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        const int t = (blockIdx.x * 4 + wave) * NTW + j;
        live[j] = t < a.ntiles;
        ct[j] = live[j] ? t : a.ntiles - 1;
    }
    // staging: BM rows x NSEG segments of 16 bytes per chunk, NP per thread
    const int srow = tid / NSEG, sseg = tid % NSEG;
    const uint16_t* arow[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) arow[p] = a.A + (size_t)min(row0 + srow + RPP * p, T - 1) * a.lda;
    u32x4 xr[NP];
    // a chunk that reaches past the contraction length is filled with zeros there (when it is written to LDS: a
    // select right after the load would wait for it), so the step loop needs no guard
    bool xr_inside = true;
    auto load_chunk = [&](int c) {
        const int k0 = c * LT_CK + sseg * 8;
        xr_inside = k0 < steps * 16;
        const int kk = xr_inside ? k0 : 0;
#pragma unroll
        for (int p = 0; p < NP; ++p) xr[p] = *reinterpret_cast<const u32x4*>(arow[p] + kk);
    };
    auto store_chunk = [&](int buf) {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<u32x4*>(lds + buf * BUF + (srow + RPP * p) * LT_ROWB + sseg * 16) = xr_inside ? xr[p] : z;
    };
    f32x16 acc[MT][NTW];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NTW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (c0 < c1) {
        const int s_last = min(c1 * SPC, steps) - 1;      // steps past it multiply zeros: any valid fragment serves
        u32x4 bq[PF][NTW];
        // bf16 factors: slot = one step; fp8 factors: slot = a pair of steps in one 16-byte load
        auto load_b = [&](int slot, int s) {
            const int sc = min(s, s_last);
#pragma unroll
            for (int j = 0; j < NTW; ++j)
                bq[slot][j] = FP8 ? a.bfrag[((size_t)ct[j] * a.nsp + (sc >> 1)) * 64 + lane]
                                  : a.bfrag[((size_t)ct[j] * steps + sc) * 64 + lane];
        };
        // first chunk's A loads, then the B prefetch, then the A store: the loads outstanding on entry to the loop
        // are the same four B slots, in the same order, as at its back edge (the wait counts are derived from the
        // weaker of the two states), and neither set of loads waits for the other
        load_chunk(c0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < PF; ++i) load_b(i, c0 * SPC + (FP8 ? 2 * i : i));
        __builtin_amdgcn_sched_barrier(0);
        store_chunk(0);
        lds_barrier();
        for (int c = c0; c < c1; ++c) {
            const int buf = (c - c0) & 1;
            load_chunk(min(c + 1, c1 - 1));
            // the scheduling barriers keep this order: the next step's A fragments and the B fragments four steps
            // ahead are requested around each step's MFMAs, not gathered at the end of the chunk
            Frag xa[2][MT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
                xa[0][i].q = *reinterpret_cast<const u32x4*>(lds + buf * BUF + (32 * i + col) * LT_ROWB + hf * 16);
#pragma unroll
            for (int ks = 0; ks < SPC; ++ks) {
                if (ks < SPC - 1) {
#pragma unroll
                    for (int i = 0; i < MT; ++i)
                        xa[(ks + 1) & 1][i].q = *reinterpret_cast<const u32x4*>(lds + buf * BUF + (32 * i + col) * LT_ROWB +
                                                                               (ks + 1) * 32 + hf * 16);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < NTW; ++j) {
                    Frag b;
                    if (FP8) {
                        const u32x4 raw = bq[(ks >> 1) % PF][j];
                        b.v = (ks & 1) ? fp8x8_to_bf8(raw[2], raw[3]) : fp8x8_to_bf8(raw[0], raw[1]);
                    } else {
                        b.q = bq[ks % PF][j];
                    }
#pragma unroll
                    for (int i = 0; i < MT; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[ks & 1][i].v, b.v, acc[i][j], 0, 0, 0);
                }
                if (!FP8) load_b(ks % PF, c * SPC + ks + PF);
                else if (ks & 1) load_b((ks >> 1) % PF, c * SPC + ks - 1 + 2 * PF);
                __builtin_amdgcn_sched_barrier(0);
            }
            store_chunk(buf ^ 1);
            lds_barrier();
        }
    }
#pragma unroll
    for (int j = 0; j < NTW; ++j) {
        if (!live[j]) continue;
        const int c = 32 * ct[j] + col;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = row0 + 32 * i + 8 * (v / 4) + 4 * hf + (v % 4);
                if (m < T) {
                    if (OUT_BF16) reinterpret_cast<uint16_t*>(a.C)[(size_t)m * a.ldc + c] = (uint16_t)f2bf_bits(acc[i][j][v]);
                    else reinterpret_cast<float*>(a.C)[((size_t)split * T + m) * a.ldc + c] = acc[i][j][v];
                }
            }
    }
}

template <int MT, int NTW, bool OUT_BF16, bool FP8>
tq_status lt_launch_gemm_inst(const LtGemmArgs& a, int planes, hipStream_t st)
{
    auto kern = lt_gemm_kernel<MT, NTW, OUT_BF16, FP8>;
    constexpr size_t smem = 2 * 32 * MT * LT_ROWB;      // at most 34 KB: inside the default dynamic-LDS limit
    const int rt = (a.T + 32 * MT - 1) / (32 * MT), cb = (a.ntiles + 4 * NTW - 1) / (4 * NTW);
    if (rt > 65535) return TQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3(cb, rt, planes), dim3(256), smem, st, a);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

template <bool OUT_BF16, bool FP8>
tq_status lt_launch_gemm(const LtGemmArgs& a, int mt, int ntw, int planes, hipStream_t st)
{
    if (mt == 1) {
        if (ntw == 1) return lt_launch_gemm_inst<1, 1, OUT_BF16, FP8>(a, planes, st);
        if (ntw == 2) return lt_launch_gemm_inst<1, 2, OUT_BF16, FP8>(a, planes, st);
        return lt_launch_gemm_inst<1, 3, OUT_BF16, FP8>(a, planes, st);
    }
    if (mt == 2) {
        if (ntw == 1) return lt_launch_gemm_inst<2, 1, OUT_BF16, FP8>(a, planes, st);
        if (ntw == 2) return lt_launch_gemm_inst<2, 2, OUT_BF16, FP8>(a, planes, st);
        return lt_launch_gemm_inst<2, 3, OUT_BF16, FP8>(a, planes, st);
    }
    return TQ_ERR_UNSUPPORTED;
}

// ---- S[b][n rp + rho] = sum_t [n(b,t) == n] g[b,t] sum_planes X_proj[b][m(b,t) rp + rho]   (Eq. 16) ----------
// A workgroup takes `tb` consecutive tokens: their selections are resolved to (m, n, g) once, into LDS (one
// dependent chain of loads instead of one per selection), then one thread per (token, four columns of S) adds the
// matching slices: selections in ascending t, planes in ascending order.
constexpr int LT_GATHER_TAB = 1024;      // selections per workgroup held in LDS (tb * top_k)

__global__ void __launch_bounds__(256) lt_gather_kernel(LtLayout L, const int32_t* __restrict__ phi,
                                                        const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                        const float* __restrict__ xproj, int planes, int ldx, int T, int tb,
                                                        const float* __restrict__ sigma, uint16_t* __restrict__ S,
                                                        int32_t* __restrict__ err)
{
    __shared__ int32_t tm[LT_GATHER_TAB], tn[LT_GATHER_TAB];
    __shared__ float tg[LT_GATHER_TAB];
    const int b0 = blockIdx.x * tb, nb = min(tb, T - b0), k = L.k;
    for (int i = threadIdx.x; i < nb * k; i += blockDim.x) {
        const int e = idx[(size_t)b0 * k + i];
        int m = 0, n = -1;                  // -1 matches no column tile
        float g = 0.f;
        if (e >= 0 && e < L.E) {
            const int2 mn = *reinterpret_cast<const int2*>(phi + 2 * e);
            m = mn.x;
            n = mn.y;
            g = w[(size_t)b0 * k + i];
        } else {
            atomicOr(err, 1);
        }
        tm[i] = m;
        tn[i] = n;
        tg[i] = g;
    }
    __syncthreads();
    const int q4 = L.k2 / 4;
    for (int it = threadIdx.x; it < nb * q4; it += blockDim.x) {
        const int bl = it / q4, c = (it % q4) * 4, b = b0 + bl;
        const int n = c / L.rp, rho = c % L.rp;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        for (int t = 0; t < k; ++t) {
            if (tn[bl * k + t] != n) continue;
            const float g = tg[bl * k + t];
            const float* src = xproj + (size_t)b * ldx + tm[bl * k + t] * L.rp + rho;
            float4 xp = {0.f, 0.f, 0.f, 0.f};
            // planes is a power of two: four loads in flight at a time, added in ascending order
            const size_t ps = (size_t)T * ldx;
            int p = 0;
            for (; p + 4 <= planes; p += 4) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(src + (size_t)(p + u) * ps);
#pragma unroll
                for (int u = 0; u < 4; ++u) { xp.x += v[u].x; xp.y += v[u].y; xp.z += v[u].z; xp.w += v[u].w; }
            }
            for (; p < planes; ++p) {
                const float4 v = *reinterpret_cast<const float4*>(src + (size_t)p * ps);
                xp.x += v.x; xp.y += v.y; xp.z += v.z; xp.w += v.w;
            }
            s0 = fmaf(g, xp.x, s0); s1 = fmaf(g, xp.y, s1); s2 = fmaf(g, xp.z, s2); s3 = fmaf(g, xp.w, s3);
        }
        if (sigma) {      // mixed-precision factors: X_proj was formed on U alone, Sigma scales its rank components
            const float4 sg = *reinterpret_cast<const float4*>(sigma + rho);
            s0 *= sg.x; s1 *= sg.y; s2 *= sg.z; s3 *= sg.w;
        }
        uint2 o = {pack_bf2(s0, s1), pack_bf2(s2, s3)};
        *reinterpret_cast<uint2*>(S + (size_t)b * L.k2 + c) = o;
    }
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
    if (!lt_make_layout(desc, &L) || L.fp8) return TQ_ERR_SHAPE;
    if (((uintptr_t)packed & 255) || (((uintptr_t)us | (uintptr_t)v | (uintptr_t)phi) & 15)) return TQ_ERR_ALIGN;
    if (packed_bytes < L.total) return TQ_ERR_WORKSPACE;
    hipLaunchKernelGGL(lt_pack_kernel, dim3(1024), dim3(256), 0, (hipStream_t)stream, L, us, v, phi, (uint8_t*)packed,
                       err_flag);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

extern "C" tq_status tq_lotile_pack_fp8(const tq_lotile_desc* desc, const uint8_t* u8, const uint16_t* sigma,
                                        const uint8_t* v8, const int32_t* phi, void* packed, size_t packed_bytes,
                                        int32_t* err_flag, void* stream)
{
    if (!desc || !u8 || !sigma || !v8 || !phi || !packed) return TQ_ERR_NULL;
    LtLayout L;
    if (!lt_make_layout(desc, &L) || !L.fp8) return TQ_ERR_SHAPE;
    if (((uintptr_t)packed & 255) || (((uintptr_t)u8 | (uintptr_t)v8 | (uintptr_t)sigma | (uintptr_t)phi) & 15)) return TQ_ERR_ALIGN;
    if (packed_bytes < L.total) return TQ_ERR_WORKSPACE;
    hipLaunchKernelGGL(lt_pack_fp8_kernel, dim3(1024), dim3(256), 0, (hipStream_t)stream, L, u8, sigma, v8, phi,
                       (uint8_t*)packed, err_flag);
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
    tqi_record_stage(0, st);
    // step one: the global projection on every row tile's factor (its first workgroup clears the error flag)
    LtGemmArgs g1 = {(const uint16_t*)x, L.n_in, T, (const u32x4*)(pk + L.off_b1), L.steps1, L.nt1, L.nsp1, (void*)xproj, W.ldx, ctrl};
    tq_status rc = L.fp8 ? lt_launch_gemm<false, true>(g1, W.mt, W.ntw1, W.planes, st)
                         : lt_launch_gemm<false, false>(g1, W.mt, W.ntw1, W.planes, st);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(1, st);
    // step two: routing-weighted selection and accumulation into the compact buffer
    const int q4 = L.k2 / 4;
    const int tb = std::max(1, std::min({T / 256, std::max(1, 512 / q4), LT_GATHER_TAB / L.k}));
    hipLaunchKernelGGL(lt_gather_kernel, dim3((T + tb - 1) / tb), dim3(256), 0, st, L, (const int32_t*)(pk + L.off_phi),
                       topk_idx, topk_w, (const float*)xproj, W.planes, W.ldx, T, tb,
                       L.fp8 ? (const float*)(pk + L.off_sigma) : nullptr, S, ctrl);
    TQ_CHECK_LAUNCH();
    tqi_record_stage(2, st);
    // step three: output reconstruction
    LtGemmArgs g2 = {(const uint16_t*)S, L.k2, T, (const u32x4*)(pk + L.off_b2), L.steps2, L.nt2, L.nsp2, y, L.n_out, nullptr};
    rc = L.fp8 ? lt_launch_gemm<true, true>(g2, W.mt, W.ntw2, 1, st) : lt_launch_gemm<true, false>(g2, W.mt, W.ntw2, 1, st);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(3, st);
    return TQ_OK;
}

// ---- offline helpers (host only) --------------------------------------------------------------------------------
extern "C" tq_status tq_lotile_grid(int32_t n_experts, int32_t* tiles_m, int32_t* tiles_n)
{
    if (!tiles_m || !tiles_n) return TQ_ERR_NULL;
    if (n_experts < 1) return TQ_ERR_SHAPE;
    // the integer closest to sqrt(E): the m with m(m-1) < E <= m(m+1) (ties cannot occur: sqrt(E) = m + 1/2 has no
    // integer solution)
    int32_t m = 1;
    while ((int64_t)m * (m + 1) < n_experts) ++m;
    *tiles_m = m;
    *tiles_n = (n_experts + m - 1) / m;
    return TQ_OK;
}

extern "C" tq_status tq_lotile_place(const int32_t* ideal, int32_t n_experts, int32_t tiles_m, int32_t tiles_n,
                                     int32_t* phi)
{
    if (!ideal || !phi) return TQ_ERR_NULL;
    if (n_experts < 1 || tiles_m < 1 || tiles_n < 1) return TQ_ERR_SHAPE;
    if ((int64_t)tiles_m * tiles_n < n_experts || (int64_t)tiles_m * tiles_n > (1 << 20)) return TQ_ERR_SHAPE;
    const int M = tiles_m, N = tiles_n;
    std::vector<uint8_t> taken((size_t)M * N, 0);
    for (int k = 0; k < n_experts; ++k) {
        const int am = std::min(std::max(ideal[2 * k], 0), M - 1), an = std::min(std::max(ideal[2 * k + 1], 0), N - 1);
        bool placed = false;
        // rings of growing Chebyshev distance around the anchor, each scanned row by row; the grid has a free cell
        // (M N >= E), and every cell lies on a ring of distance below max(M, N)
        for (int rho = 0; rho < std::max(M, N) && !placed; ++rho) {
            for (int m = std::max(am - rho, 0); m <= std::min(am + rho, M - 1) && !placed; ++m) {
                const bool edge_row = (m == am - rho) || (m == am + rho);
                for (int n = std::max(an - rho, 0); n <= std::min(an + rho, N - 1); ++n) {
                    if (!edge_row && n != an - rho && n != an + rho) continue;      // interior of the ring's square
                    if (taken[(size_t)m * N + n]) continue;
                    taken[(size_t)m * N + n] = 1;
                    phi[2 * k] = m;
                    phi[2 * k + 1] = n;
                    placed = true;
                    break;
                }
            }
        }
        if (!placed) return TQ_ERR_RANGE;       // cannot happen with M N >= E
    }
    return TQ_OK;
}

