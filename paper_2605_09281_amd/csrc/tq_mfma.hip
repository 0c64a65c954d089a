// bf16 path of tq_moe_forward for gfx950: fused int4 dequant x bf16 MFMA grouped GEMM with the
// rank-r correction and the zero-point correction folded into the same tile loop.
//
// How a projection out[m][n] = sum_kk x[m][kk] (q[n][kk] - z[n][G]) s[n][G] + (x A)[m][:] B[:][n] is evaluated:
//   * the 4-bit codes are turned into bf16 values 128 + q with one and-or per pair (0x4300 | q is
//     exactly 128 + q in bf16), fed to v_mfma_f32_32x32x16_bf16 against the bf16 activations, and the
//     fp32 partial sum of one quantisation group is scaled by s[n][G] on the accumulator;
//   * what that leaves, -(128 + z) s times the group sum of x, is a rank-(K/g) term.  The group sums are
//     computed once per row by aug_kernel, split into bf16 hi + lo parts (the coefficient likewise), and
//     contracted by three extra MFMA steps per 16 groups;
//   * the low-rank term is r/16 more MFMA steps on t = x A (computed by aug_kernel with MFMA as well)
//     against B converted fp16 -> bf16 on the fly.
// Activations are staged through LDS (shared by the four waves of a workgroup); the packed codes are
// already in MFMA fragment order and go straight from global memory to registers.
#include "tq_device.h"

#include <type_traits>

namespace {

using namespace tqdev;

// ------------------------------------------------------------------------------------------------
// aug_kernel: per 32-row tile, the augmented activation row
//   xaug[slot] = [ hi(xsum_0..G-1) | lo(xsum) | hi(xsum) | 0.. (to a multiple of 16) | t = x A (NA values) | 0.. ]
// STAGE 0: x rows gathered by token, A = [gate | up] factors (NA = 2 r16).  STAGE 1: h rows, down factors.
// NAT = column tiles of t per pass over x, UNR = steps whose loads are issued together.
template <int STAGE, int NAT, int UNR>
__global__ void __launch_bounds__(256) aug_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                  const uint16_t* __restrict__ xin,
                                                  const int32_t* __restrict__ row_token,
                                                  const int32_t* __restrict__ tile_e,
                                                  const int32_t* __restrict__ tile_row0,
                                                  const int32_t* __restrict__ offsets,
                                                  const int32_t* __restrict__ ctrl, int ctrl_idx,
                                                  uint16_t* __restrict__ xaug, int ka)
{
    constexpr int MT = 1;
    // One workgroup per tile of 32 rows; its four waves split the contraction at unit (= group)
    // boundaries so that enough loads are in flight, and their partial t tiles are summed through LDS.
    __shared__ float red[4][16][64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x;
    if (tile >= ctrl[ctrl_idx]) return;
    const int e = tile_e[tile], slot0 = tile_row0[tile];
    const int rows = min(32 * MT, offsets[e + 1] - slot0);
    const int col = lane & 31, hf = lane >> 5;
    const int K = sec.K, NA = STAGE == 0 ? 2 * G.r16 : G.r16;
    const int groups = sec.groups, GS = G.g / 16, ksteps = K / 16;
    const int ZT = tq_zero_terms(K, G.g);
    const uint16_t* xrow[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int m = min(32 * i + col, rows - 1);
        xrow[i] = STAGE == 0 ? xin + (size_t)row_token[slot0 + m] * K : xin + (size_t)(slot0 + m) * K;
    }
    const u32x4* af = reinterpret_cast<const u32x4*>(tq_afrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e));
    uint16_t* orow = xaug + (size_t)(slot0 + col) * ka;     // row 32 i + col is at orow + 32 i ka
    const int unit_steps = (G.g < 64 ? 64 : G.g) / 16;
    const int NU = ksteps / unit_steps;
    const int sb = (wave * NU / 4) * unit_steps, se = ((wave + 1) * NU / 4) * unit_steps;

    const int na_tiles = (G.r > 0) ? sec.na_tiles : 0;
    for (int ta0 = 0; ta0 == 0 || ta0 < na_tiles; ta0 += NAT) {
        f32x16 acc[MT][NAT];
        float gsum[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            gsum[i] = 0.f;
#pragma unroll
            for (int j = 0; j < NAT; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        }
        for (int s0 = sb; s0 < se; s0 += UNR) {
            Frag xa[MT][UNR];
            u32x4 aq[UNR][NAT];
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    xa[i][u].q = *reinterpret_cast<const u32x4*>(xrow[i] + 16 * (s0 + u) + 8 * hf);
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int j = 0; j < NAT; ++j)
                    if (ta0 + j < na_tiles) aq[u][j] = af[((size_t)(ta0 + j) * ksteps + s0 + u) * 64 + lane];
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int s = s0 + u;
                if (ta0 == 0) {
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) gsum[i] += bf_lo(xa[i][u].u[j]) + bf_hi(xa[i][u].u[j]);
                    if ((s + 1) % GS == 0) {
                        const int gi = s / GS;
#pragma unroll
                        for (int i = 0; i < MT; ++i) {
                            float tot = gsum[i] + __shfl_xor(gsum[i], 32);
                            if (hf == 0 && 32 * i + col < rows) {
                                uint32_t hi = f2bf_bits(tot);
                                uint32_t lo = f2bf_bits(tot - __uint_as_float(hi << 16));
                                // block of 16 groups: hi | lo | hi
                                uint16_t* zb = orow + (size_t)32 * i * ka + 48 * (gi >> 4) + (gi & 15);
                                zb[0] = (uint16_t)hi;
                                zb[16] = (uint16_t)lo;
                                zb[32] = (uint16_t)hi;
                            }
                            gsum[i] = 0.f;
                        }
                    }
                }
#pragma unroll
                for (int j = 0; j < NAT; ++j)
                    if (ta0 + j < na_tiles) {
                        const bf16x8 a8 = half8_to_bf8(aq[u][j]);
#pragma unroll
                        for (int i = 0; i < MT; ++i)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[i][u].v, a8, acc[i][j], 0, 0, 0);
                    }
            }
        }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NAT; ++j) {
                if (ta0 + j < na_tiles) {      // uniform over the workgroup
#pragma unroll
                    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[i][j][v];
                    __syncthreads();
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int v = 4 * q + wave;
                        const float sum = (red[0][v][lane] + red[1][v][lane]) + (red[2][v][lane] + red[3][v][lane]);
                        const int c = 32 * (ta0 + j) + col;
                        const int m2 = 32 * i + 8 * (v / 4) + 4 * hf + (v % 4);
                        if (c < NA && m2 < rows) xaug[(size_t)(slot0 + m2) * ka + ZT + c] = (uint16_t)f2bf_bits(sum);
                    }
                    __syncthreads();
                }
            }
    }
    // the padding must be finite (it meets zero weights in the MFMA): write zeros
    if (hf == 0 && wave == 0) {
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            if (32 * i + col >= rows) continue;
            uint16_t* o = orow + (size_t)32 * i * ka;
            for (int gi = groups; gi < 16 * ((groups + 15) / 16); ++gi) {
                uint16_t* zb = o + 48 * (gi >> 4) + (gi & 15);
                zb[0] = 0; zb[16] = 0; zb[32] = 0;
            }
            for (int kk = ZT + ((G.r > 0) ? NA : 0); kk < ka; ++kk) o[kk] = 0;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// aug_staged_kernel: the same result as aug_kernel for groups of at most 128, with the activation rows read in
// whole 4-group chunks by all threads (each row's chunk is one contiguous run of up to 1 KB instead of
// 16 bytes per lane and step) and staged through LDS; wave w of the workgroup owns group w of every chunk.
template <int STAGE, int NAT, int GS>
__global__ void __launch_bounds__(256, NAT == 1 ? 3 : 2) aug_staged_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                            const uint16_t* __restrict__ xin,
                                                            const int32_t* __restrict__ row_token,
                                                            const int32_t* __restrict__ tile_e,
                                                            const int32_t* __restrict__ tile_row0,
                                                            const int32_t* __restrict__ offsets,
                                                            const int32_t* __restrict__ ctrl,
                                                            uint16_t* __restrict__ xaug, int ka, int cps,
                                                            float* __restrict__ tslice)
{
    constexpr int CK = 4 * GS * 16;        // contraction indices per chunk (four groups)
    constexpr int CKB = CK * 2;            // bytes of one row's chunk
    constexpr int ROWB = CKB + 16;         // padded LDS row
    constexpr int SPR = CKB / 16;          // 16-byte segments per row
    constexpr int RPP = 256 / SPR;         // rows per pass
    constexpr int NP = 32 / RPP;           // passes
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];     // 32 x ROWB (one buffer: the next chunk waits
                                                                       // in registers); reused for the reduction
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int tile = blockIdx.x;
    if (tile >= ctrl[1]) return;
    const int e = tile_e[tile], slot0 = tile_row0[tile];
    const int rows = min(32, offsets[e + 1] - slot0);
    const int col = lane & 31, hf = lane >> 5;
    const int K = sec.K, NA = STAGE == 0 ? 2 * G.r16 : G.r16;
    const int groups = sec.groups, ksteps = K / 16;
    const int ZT = tq_zero_terms(K, G.g);
    const int nchunks = (groups + 3) / 4;
    const int na_tiles = (G.r > 0) ? sec.na_tiles : 0;
    const uint8_t* rec = blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride;
    // layers without factors have an empty fragment section: their (unconditional, unused) fragment loads all read
    // the first kilobyte of the codes instead of running past the record
    const u32x4* af = reinterpret_cast<const u32x4*>(na_tiles > 0 ? tq_afrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e)
                                                                  : rec + sec.codes) + lane;
    const size_t af_live = na_tiles > 0 ? 1 : 0;
    uint16_t* orow = xaug + (size_t)(slot0 + col) * ka;
    const bool writer = (hf == 0) && (col < rows);

    const int prow = tid / SPR, seg = tid % SPR;
    uint32_t roff[NP];                     // byte offset of this thread's rows in xin
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int m = min(p * RPP + prow, rows - 1);
        const uint32_t src = STAGE == 0 ? (uint32_t)row_token[slot0 + m] : (uint32_t)(slot0 + m);
        roff[p] = src * (uint32_t)(K * 2);
    }
    const uint8_t* xb = reinterpret_cast<const uint8_t*>(xin);
    u32x4 xr[NP];
    auto load_chunk = [&](int c) {
        // the last chunk may be short: segments past the row end re-read the last valid one (never used)
        const int kb = min(c * CKB + seg * 16, K * 2 - 16);
#pragma unroll
        for (int p = 0; p < NP; ++p) xr[p] = *reinterpret_cast<const u32x4*>(xb + roff[p] + (uint32_t)kb);
    };
    auto store_chunk = [&]() {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<u32x4*>(lds + (p * RPP + prow) * ROWB + seg * 16) = xr[p];
    };

    f32x16 acc[NAT];
#pragma unroll
    for (int j = 0; j < NAT; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    // With few row tiles the contraction is cut into slices of cps chunks, one workgroup (blockIdx.y) each: the group
    // sums of a slice are final, its part of t goes to tslice and aug_slices_kernel adds the parts up.
    const int c_begin = blockIdx.y * cps, c_end = min(nchunks, c_begin + cps);
    load_chunk(c_begin);
    store_chunk();
    lds_barrier();
    for (int c = c_begin; c < c_end; ++c) {
        const int gi = 4 * c + wave;
        // The factor fragments of this chunk are requested BEFORE the next chunk's rows: loads return in order, and
        // behind the gathered rows (memory-side cache or HBM) these L2 hits would wait for them.  Unconditional
        // with a clamped group, so that the compiler can count them.
        // (four column tiles at groups of 128 are 128 registers of fragments: they come in two halves, the second one
        // requested after the first one's MFMAs)
        constexpr int NJ = (NAT * GS > 16) ? NAT / 2 : NAT;
        u32x4 aq[GS][NJ];
        const int gic = min(gi, groups - 1);
        auto load_aq = [&](int j0) {
#pragma unroll
            for (int ks = 0; ks < GS; ++ks)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    aq[ks][j] = af[((size_t)min(j0 + j, max(na_tiles, 1) - 1) * ksteps + gic * GS + ks) * 64 * af_live];
        };
        load_aq(0);
        if constexpr (NJ == NAT) load_chunk(min(c + 1, c_end - 1));
        // every wave copies its group's fragments out of the one LDS buffer (clamped for a group past the end),
        // then the buffer is free for the next chunk
        Frag xa[GS];
#pragma unroll
        for (int ks = 0; ks < GS; ++ks)
            xa[ks].q = *reinterpret_cast<const u32x4*>(lds + col * ROWB + (wave * GS + ks) * 32 + hf * 16);
        lds_barrier();
        if (gi < groups) {
            float gsum = 0.f;
#pragma unroll
            for (int ks = 0; ks < GS; ++ks)
#pragma unroll
                for (int j = 0; j < 4; ++j) gsum += bf_lo(xa[ks].u[j]) + bf_hi(xa[ks].u[j]);
            const float tot = gsum + __shfl_xor(gsum, 32);
            if (writer) {
                const uint32_t hi = f2bf_bits(tot);
                const uint32_t lo = f2bf_bits(tot - __uint_as_float(hi << 16));
                uint16_t* zb = orow + 48 * (gi >> 4) + (gi & 15);        // block of 16 groups: hi | lo | hi
                zb[0] = (uint16_t)hi;
                zb[16] = (uint16_t)lo;
                zb[32] = (uint16_t)hi;
            }
            // NAT is the number of column tiles of t whenever there are factors at all, so one uniform test covers
            // the block (a test per MFMA turns into a copy of the accumulator per MFMA)
            if (na_tiles > 0) {
#pragma unroll
                for (int j0 = 0; j0 < NAT; j0 += NJ) {
                    if (j0 > 0) load_aq(j0);
                    // two halves: the next chunk's rows are requested behind the second half's fragments (in front
                    // of them they would hold those L2 hits back until the rows have arrived)
                    if (NJ != NAT && j0 + NJ >= NAT) load_chunk(min(c + 1, c_end - 1));
#pragma unroll
                    for (int ks = 0; ks < GS; ++ks)
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            acc[j0 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[ks].v, half8_to_bf8(aq[ks][j]), acc[j0 + j], 0, 0, 0);
                }
            }
        }
        store_chunk();
        lds_barrier();
    }
    // sum the four waves' partial t tiles through LDS (the staging buffers are free now) and write them out
    float* red = reinterpret_cast<float*>(lds);       // [4][16][64]
#pragma unroll
    for (int j = 0; j < NAT; ++j) {
        if (j < na_tiles) {                           // uniform over the workgroup
#pragma unroll
            for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = acc[j][v];
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int v = 4 * q + wave;
                const float sum = (red[(0 * 16 + v) * 64 + lane] + red[(1 * 16 + v) * 64 + lane]) +
                                  (red[(2 * 16 + v) * 64 + lane] + red[(3 * 16 + v) * 64 + lane]);
                const int cc = 32 * j + col;
                const int m2 = 8 * (v / 4) + 4 * hf + (v % 4);
                if (tslice) tslice[((((size_t)tile * gridDim.y + blockIdx.y) * NAT + j) * 16 + v) * 64 + lane] = sum;
                else if (cc < NA && m2 < rows) xaug[(size_t)(slot0 + m2) * ka + ZT + cc] = (uint16_t)f2bf_bits(sum);
            }
            __syncthreads();
        }
    }
    // the padding must be finite (it meets zero weights in the MFMA): write zeros
    if (writer && wave == 0 && blockIdx.y == 0) {
        for (int gi = groups; gi < 16 * ((groups + 15) / 16); ++gi) {
            uint16_t* zb = orow + 48 * (gi >> 4) + (gi & 15);
            zb[0] = 0; zb[16] = 0; zb[32] = 0;
        }
        for (int kk = ZT + ((G.r > 0) ? NA : 0); kk < ka; ++kk) orow[kk] = 0;
    }
}

// Sum of the slices of t that aug_staged_kernel left in tslice ([tile][slice][NAT][16][64] fp32, in the accumulator
// layout of the 32x32 MFMA), in slice order, rounded to bf16 into the rows of xaug.  One workgroup per tile, column
// tile of t and four accumulator registers; eight slices are requested at a time.
__global__ void __launch_bounds__(256) aug_slices_kernel(const float* __restrict__ tslice, int nsl, int nat, int NA, int ZT,
                                                         const int32_t* __restrict__ tile_e,
                                                         const int32_t* __restrict__ tile_row0,
                                                         const int32_t* __restrict__ offsets,
                                                         const int32_t* __restrict__ ctrl,
                                                         uint16_t* __restrict__ xaug, int ka)
{
    const int tile = blockIdx.x, j = blockIdx.y;
    if (tile >= ctrl[1]) return;
    const int e = tile_e[tile], slot0 = tile_row0[tile];
    const int rows = min(32, offsets[e + 1] - slot0);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int v = 4 * blockIdx.z + wave;
    const float* src = tslice + (((size_t)tile * nsl * nat + j) * 16 + v) * 64 + lane;
    const size_t stride = (size_t)nat * 1024;
    float sum = 0.f;
    for (int s0 = 0; s0 < nsl; s0 += 8) {
        float part[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) part[u] = src[(size_t)min(s0 + u, nsl - 1) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (s0 + u < nsl) sum += part[u];
    }
    const int cc = 32 * j + col;
    const int m2 = 8 * (v / 4) + 4 * hf + (v % 4);
    if (cc < NA && m2 < rows) xaug[(size_t)(slot0 + m2) * ka + ZT + cc] = (uint16_t)f2bf_bits(sum);
}

// ------------------------------------------------------------------------------------------------
// The grouped GEMM.  Workgroup = 4*WM waves sharing one row tile of BM = 32*MT*WM rows; wave (wm, wn) owns
// rows [32*MT*wm, 32*MT*(wm+1)) of the tile and column-tile pair 4*nb + wn (64 output columns; in
// stage 0 that is 32 gate + the matching 32 up columns).
//   STAGE 0: out = h[slot][F] bf16 = silu(gate) * up
//   STAGE 1: out = yd[split][slot][H] fp32, split = blockIdx.z covering a slice of K
// GS = quantisation group in MFMA steps (g/16).  A "unit" is max(g, 64) contraction indices.
// CW = 32-bit words of codes per lane, tile and 64-wide chunk: 4 (4-bit slots), 3 or 2 (dense 3- / 2-bit codes).
// Staging units between two workgroup barriers of moe_mfma_kernel: the 32-row tile is bound by the weight stream, and
// a barrier per unit would tie its four waves to the slowest arrival of every unit; with four units per barrier (two
// for groups of 128 and 256: LDS) they drift apart inside a chunk.  Larger tiles keep one unit per barrier (LDS per
// workgroup).  The 32-row tile is also compiled for four waves per SIMD (groups of 128 run as half-group units of the
// instantiation for groups of 64, see G2): its waves stall on their own operands, and more of them hide that.
constexpr int mfma_chunk_units(int MT, int GS) { return MT == 1 ? (GS >= 8 ? 2 : 4) : 1; }

// G2 (with GS = 4 on the 32-row tile): the layer's groups are 128 wide and a unit is HALF a group - the partial sums
// run over two units (even unit: start, odd unit: fold) and both units read the group's scale.  Half the registers
// of codes and staging per unit, which is what lets groups of 128 run at four waves per SIMD like groups of 64.
template <int MT, int WM, int STAGE, int GS, int CW = 4, bool G2 = false>
__global__ void __launch_bounds__(256 * WM, (MT == 2 && WM == 1) ? 2 : (MT == 1 && GS <= 4) ? 4 : (MT == 1 && GS == 8) ? 3 : 1) moe_mfma_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                       const uint16_t* __restrict__ xin,
                                                       const uint16_t* __restrict__ xaug,
                                                       const int32_t* __restrict__ row_token,
                                                       const int32_t* __restrict__ tile_e,
                                                       const int32_t* __restrict__ tile_row0,
                                                       const int32_t* __restrict__ offsets,
                                                       const int32_t* __restrict__ ctrl, int ctrl_idx,
                                                       void* __restrict__ out, int ka, int nsplit)
{
    constexpr int BM = 32 * MT * WM;
    constexpr int NTHR = 256 * WM;
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int UC = UNIT_K / 64;     // 64-wide chunks (one u32x4 of codes per lane and tile) per unit
    constexpr int US = UNIT_K / 16;     // MFMA steps per unit
    constexpr int NG = US / GS;         // quantisation groups per unit
    constexpr int ROWB = UNIT_K * 2 + 16;   // LDS bytes per activation row (16 B pad: conflict-free b128 reads)
    constexpr int BUFB = BM * ROWB;
    constexpr int CH = mfma_chunk_units(MT, GS);   // units per chunk: two chunks of CH unit buffers, a barrier per chunk
    constexpr int TPR = UNIT_K / 8;     // threads (16-byte segments) per row when loading a unit
    constexpr int RPP = NTHR / TPR;     // rows per pass
    constexpr int NP = BM / RPP;        // passes
    using WT = std::conditional_t<CW == 4, u32x4, uint32_t>;      // register type of the packed codes
    constexpr int WN = CW == 4 ? UC : UC * CW;                    // and how many of them one tile of a unit takes

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int32_t* tokx = reinterpret_cast<int32_t*>(lds + 2 * CH * BUFB);   // [BM] source row of the main operand
    int32_t* toka = tokx + BM;                                    // [BM] row in xaug

    const int K = sec.K;
    // XCD-aware mapping: consecutive workgroup ids go to the 8 XCDs in turn, each with its own L2.  Ids are
    // laid out so that, within a block of 8 row tiles, XCD x works on row tile x of the block and walks through
    // all its column blocks itself: the activation tile is then re-read from that XCD's L2 instead of from memory
    // by all 8.
    const int nb_count = (sec.pairs + 3) / 4;
    const int wg = blockIdx.x;
    const int grp = wg / (8 * nb_count), rem = wg - grp * (8 * nb_count);
    const int nb = rem >> 3;
    const int rt = grp * 8 + (rem & 7);
    const int tid = threadIdx.x;
    if (rt >= ctrl[ctrl_idx]) return;
    const int e = tile_e[rt], slot0 = tile_row0[rt];
    const int rows = min(BM, offsets[e + 1] - slot0);
    const int wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wn = wave & 3, wm = wave >> 2;
    const int pair_raw = nb * 4 + wn;
    const bool active = pair_raw < sec.pairs;
    const int pair = active ? pair_raw : sec.pairs - 1;
    const int split = blockIdx.z;

    if (tid < BM) {
        int r = min(tid, rows - 1);
        tokx[tid] = STAGE == 0 ? row_token[slot0 + r] : slot0 + r;
        toka[tid] = slot0 + r;
    }
    lds_barrier();

    const uint8_t* rec = blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride;
    const u32x4* codes = reinterpret_cast<const u32x4*>(rec + sec.codes) + (size_t)pair * sec.chunks * 128 + lane;
    const uint32_t* codes32 = reinterpret_cast<const uint32_t*>(rec + sec.codes) + (size_t)pair * sec.chunks * (2 * CW * 64) + lane;
    const uint32_t* szp = reinterpret_cast<const uint32_t*>(rec + sec.sz) + (size_t)pair * sec.groups * 64 + col;
    const u32x4* zcp = reinterpret_cast<const u32x4*>(tq_zc_base(G, blob, sec, STAGE, e)) + (size_t)pair * sec.zfrag * 128 + lane;
    const u32x4* bfr = reinterpret_cast<const u32x4*>(G.r > 0 ? tq_bfrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e)
                                                               : rec + sec.bfrag) + (size_t)pair * (G.r16 / 16) * 128 + lane;

    const int NU = K / UNIT_K;
    constexpr int UPG = G2 ? 2 : 1;      // units per group where a unit is a part of one: splits fall on whole groups
    const int u0 = UPG * (int)((long)split * (NU / UPG) / nsplit), u1 = UPG * (int)((long)(split + 1) * (NU / UPG) / nsplit);
    const int nmain = u1 - u0;
    const int naug = (split == 0) ? ka / UNIT_K : 0;
    const int nsteps = nmain + naug;

    u32x4 xr[NP];
    // ---- staging helpers: steps 0..naug-1 are units of the augmented rows (zero-point and low-rank terms; they go
    //      first so that the latency of their operands overlaps with the start-up of the main stream), the
    //      remaining steps are the main units u0, u0+1, ...
    auto load_step_to = [&](u32x4 (&dst)[NP], int st) {
        const bool is_main = st >= naug;
        const uint16_t* base = is_main ? xin : xaug;
        const int32_t* tok = is_main ? tokx : toka;
        const size_t stride = is_main ? (size_t)K : (size_t)ka;
        const size_t koff = (size_t)(is_main ? u0 + st - naug : st) * UNIT_K;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            int row = p * RPP + tid / TPR, seg = tid % TPR;
            dst[p] = *reinterpret_cast<const u32x4*>(base + (size_t)tok[row] * stride + koff + seg * 8);
        }
    };
    auto load_step = [&](int st) { load_step_to(xr, st); };
    // step st lives in unit buffer (st mod 2 CH): chunk parity times CH plus the position inside the chunk
    auto store_step_from = [&](const u32x4 (&src)[NP], int st) {
        const int buf = st % (2 * CH);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            int row = p * RPP + tid / TPR, seg = tid % TPR;
            *reinterpret_cast<u32x4*>(lds + buf * BUFB + row * ROWB + seg * 16) = src[p];
        }
    };
    auto store_step = [&](int st) { store_step_from(xr, st); };
    // Steps are staged one chunk ahead: step st requests step st + CH at its start and writes it at its end, into the
    // chunk that nobody reads before the next barrier; the barrier stands at the end of every chunk.
    auto end_step = [&](int st) {
        store_step(st + CH);     // past the last step this refills an idle buffer with the last step: harmless
        if ((st + 1) % CH == 0) lds_barrier();
    };
    auto load_w = [&](WT (&dst)[2][WN], int u) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < UC; ++c) {
                if constexpr (CW == 4) {
                    dst[t][c] = codes[((size_t)(u * UC + c) * 2 + t) * 64];
                } else {
#pragma unroll
                    for (int d = 0; d < CW; ++d) dst[t][c * CW + d] = codes32[(((size_t)(u * UC + c) * 2 + t) * CW + d) * 64];
                }
            }
    };
    auto load_sz = [&](uint32_t (&dst)[NG][2], int u) {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
            for (int t = 0; t < 2; ++t) dst[gi][t] = szp[((size_t)((G2 ? u >> 1 : u) * NG + gi) * 2 + t) * 32];
    };

    f32x16 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mt][t][v] = 0.f;

    // the or-operand of the unpack lives in a vector register (only one scalar operand fits the and-or
    // encoding); the move is opaque to the compiler so that it does not fold the value back into a literal
    uint32_t magic_v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(G.unpack_magic));

    WT wq[2][2][WN];
    uint32_t szq[2][NG][2];
    f32x16 part2[G2 ? MT : 1][2];      // G2: the group's partial sums between its two units

    // ---- prologue ---------------------------------------------------------------------------------
    // Prefetches are issued unconditionally with clamped indices (a repeated, unused load at the tail): a load
    // under a condition makes the compiler wait for ALL outstanding loads at every later use, which would
    // drain the prefetch queue once per unit.
    const int ulast = u1 - 1;
    {
        // the whole first chunk is requested at once, ahead of the first weights
        u32x4 x0[CH][NP];
#pragma unroll
        for (int c = 0; c < CH; ++c) load_step_to(x0[c], min(c, nsteps - 1));
        load_w(wq[0], min(u0, ulast)); load_sz(szq[0], min(u0, ulast));
        load_w(wq[1], min(u0 + 1, ulast)); load_sz(szq[1], min(u0 + 1, ulast));
#pragma unroll
        for (int c = 0; c < CH; ++c) store_step_from(x0[c], c);
    }
    lds_barrier();

    auto lds_frag = [&](int buf, int mt, int kstep) -> bf16x8 {
        Frag f;
        f.q = *reinterpret_cast<const u32x4*>(lds + buf * BUFB + (32 * (MT * wm + mt) + col) * ROWB + (kstep * 16 + 8 * hf) * 2);
        return f.v;
    };

    // ---- main units ---------------------------------------------------------------------------------
    auto main_unit = [&](int mu, auto slot_tag) {      // mu: index of the main unit inside this split
        constexpr int SLOT = decltype(slot_tag)::value;
        const int st = naug + mu;
        load_step(min(st + CH, nsteps - 1));
        WT wc[2][WN];
        uint32_t szc[NG][2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < WN; ++c) wc[t][c] = wq[SLOT][t][c];
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
            for (int t = 0; t < 2; ++t) szc[gi][t] = szq[SLOT][gi][t];
        load_w(wq[SLOT], min(u0 + mu + 2, ulast)); load_sz(szq[SLOT], min(u0 + mu + 2, ulast));
        const int buf = st % (2 * CH);
        if (active) {
            bf16x8 xa[2][MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xa[0][mt] = lds_frag(buf, mt, 0);
#pragma unroll
            for (int gi = 0; gi < NG; ++gi) {
                f32x16 part_loc[MT][2];
                auto& part = [&]() -> f32x16 (&)[MT][2] {
                    if constexpr (G2) return part2; else return part_loc;
                }();
#pragma unroll
                for (int ks = 0; ks < GS; ++ks) {
                    const int kidx = gi * GS + ks;
                    // fragments of the next step are requested before this step's MFMAs are issued
                    if (kidx + 1 < US) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) xa[(kidx + 1) & 1][mt] = lds_frag(buf, mt, kidx + 1);
                    }
                    bf16x8 bw[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if constexpr (CW == 4) bw[t] = unpack_word(word_of(wc[t][kidx / 4], kidx % 4), G.unpack_mask, magic_v);
                        else bw[t] = unpack_dense<CW>(&wc[t][(kidx / 4) * CW], kidx % 4, G.unpack_mask, magic_v);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            if (ks == 0 && !(G2 && SLOT == 1)) {      // (G2: the odd unit goes on with the even unit's sums)
                                f32x16 zero;
#pragma unroll
                                for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                                part[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[kidx & 1][mt], bw[t], zero, 0, 0, 0);
                            } else {
                                part[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[kidx & 1][mt], bw[t], part[mt][t], 0, 0, 0);
                            }
                        }
                    }
                }
                if (!(G2 && SLOT == 0)) {      // (G2: the group is complete after its odd unit)
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float s = tq_half_bits_to_float((uint16_t)(szc[gi][t] & 0xFFFF));
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[mt][t][v] = fmaf(s, part[mt][t][v], acc[mt][t][v]);
                    }
                }
            }
        }
        end_step(st);
    };

    // ---- augmented units: zero-point correction and the low-rank term ----------------------------------
    // All weight-side fragments of a unit are requested before its first MFMA: one exposed latency per unit
    // instead of one per step (and the first one coincides with the start-up of the main stream).
    const int ZT = tq_zero_terms(K, G.g);
    for (int st = 0; st < naug; ++st) {
        load_step(min(st + CH, nsteps - 1));
        const int buf = st % (2 * CH);
        if (active) {
            u32x4 fq[US][2];
            int kind[US];          // 0 skip, 1 zero-point step (both tiles), 2 low-rank tile 0, 3 low-rank tile 1, 4 both tiles
#pragma unroll
            for (int w = 0; w < US; ++w) {
                const int k0 = UNIT_K * st + 16 * w;
                kind[w] = 0;
                if (k0 < ZT) {
                    const int step = tq_zc_fragment(k0 / 16);
                    fq[w][0] = zcp[((size_t)step * 2 + 0) * 64];
                    fq[w][1] = zcp[((size_t)step * 2 + 1) * 64];
                    kind[w] = 1;
                } else if (G.r > 0 && k0 < ZT + G.r16) {
                    const int step = (k0 - ZT) / 16;
                    fq[w][0] = bfr[((size_t)step * 2 + 0) * 64];
                    if (STAGE == 1) { fq[w][1] = bfr[((size_t)step * 2 + 1) * 64]; kind[w] = 4; } else kind[w] = 2;
                } else if (STAGE == 0 && G.r > 0 && k0 < ZT + 2 * G.r16) {
                    const int step = (k0 - ZT - G.r16) / 16;
                    fq[w][1] = bfr[((size_t)step * 2 + 1) * 64];
                    kind[w] = 3;
                }
            }
#pragma unroll
            for (int w = 0; w < US; ++w) {
                if (kind[w] == 0) continue;
                bf16x8 bw[2];
                if (kind[w] == 1) {
                    Frag f0, f1;
                    f0.q = fq[w][0]; f1.q = fq[w][1];
                    bw[0] = f0.v; bw[1] = f1.v;
                } else {
                    if (kind[w] != 3) bw[0] = half8_to_bf8(fq[w][0]);
                    if (kind[w] != 2) bw[1] = half8_to_bf8(fq[w][1]);
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    bf16x8 xa = lds_frag(buf, mt, w);
                    if (kind[w] != 3) acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, bw[0], acc[mt][0], 0, 0, 0);
                    if (kind[w] != 2) acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, bw[1], acc[mt][1], 0, 0, 0);
                }
            }
        }
        end_step(st);
    }

    int mu = 0;
    for (; mu + 1 < nmain; mu += 2) {
        main_unit(mu, std::integral_constant<int, 0>{});
        main_unit(mu + 1, std::integral_constant<int, 1>{});
    }
    if (mu < nmain) main_unit(mu, std::integral_constant<int, 0>{});

    // ---- epilogue (full tiles take a path without per-row tests) ----------------------------------------
    if (!active) return;
    const bool full = rows == BM;
    if (STAGE == 0) {
        uint16_t* h = reinterpret_cast<uint16_t*>(out) + (size_t)slot0 * G.F + 32 * pair + col;
        auto emit = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = 32 * (MT * wm + mt) + 8 * (v / 4) + 4 * hf + (v % 4);
                    if (FULL || m < rows)
                        h[(size_t)m * G.F] = (uint16_t)f2bf_bits(silu_mul(acc[mt][0][v], acc[mt][1][v]));
                }
        };
        if (full) emit(std::true_type{}); else emit(std::false_type{});
    } else {
        // unsplit tiles of 64 rows and more write their result as bf16, halving the traffic of this store and of the
        // combine pass; split-K planes (always on the 32-row path, on larger tiles when the batch leaves too few of
        // them to fill the chip) stay fp32
        auto emit = [&](auto full_tag, auto yd16_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            constexpr bool YD16 = decltype(yd16_tag)::value;
            using YT = std::conditional_t<YD16, uint16_t, float>;
            YT* yd = reinterpret_cast<YT*>(out) + (size_t)split * G.a_tot * G.H + (size_t)slot0 * G.H + 64 * pair + col;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = 32 * (MT * wm + mt) + 8 * (v / 4) + 4 * hf + (v % 4);
                    if (FULL || m < rows) {
                        if constexpr (YD16) {
                            yd[(size_t)m * G.H] = (uint16_t)f2bf_bits(acc[mt][0][v]);
                            yd[(size_t)m * G.H + 32] = (uint16_t)f2bf_bits(acc[mt][1][v]);
                        } else {
                            yd[(size_t)m * G.H] = acc[mt][0][v];
                            yd[(size_t)m * G.H + 32] = acc[mt][1][v];
                        }
                    }
                }
        };
        if (MT >= 2 && nsplit == 1) {
            if (full) emit(std::true_type{}, std::true_type{}); else emit(std::false_type{}, std::true_type{});
        } else {
            if (full) emit(std::true_type{}, std::false_type{}); else emit(std::false_type{}, std::false_type{});
        }
    }
}

// y[t][c] = bf16( sum_j w[t][j] * sum_s yd[s][slot_of[t][j]][c] + shared ), terms in slot order.
// YD16: yd is one plane of bf16 (written by the 64-row and larger tiles), else nsplit planes of fp32.
template <bool YD16>
__global__ void __launch_bounds__(256) combine_bf16_kernel(int T, int H, int k, int S, int nsplit, size_t plane,
                                                           const int32_t* __restrict__ slot_of,
                                                           const float* __restrict__ w,
                                                           const void* __restrict__ ydv, uint16_t* __restrict__ y)
{
    const int t = blockIdx.x;
    constexpr int VW = YD16 ? 8 : 4;
    const int c = (blockIdx.y * 256 + threadIdx.x) * VW;
    if (c >= H) return;
    float a[VW];
#pragma unroll
    for (int i = 0; i < VW; ++i) a[i] = 0.f;
    for (int j = 0; j < k + S; ++j) {
        const int slot = slot_of[(size_t)t * (k + S) + j];
        if (slot < 0) continue;
        const float wj = j < k ? w[(size_t)t * k + j] : 1.0f;
        if constexpr (YD16) {
            // every row is read exactly once: non-temporal
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(ydv) + (size_t)slot * H + c));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[2 * i] = fmaf(wj, bf_lo(v[i]), a[2 * i]);
                a[2 * i + 1] = fmaf(wj, bf_hi(v[i]), a[2 * i + 1]);
            }
        } else {
            const float* yd = reinterpret_cast<const float*>(ydv);
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            for (int sp = 0; sp < nsplit; ++sp) {
                const float4 v = *reinterpret_cast<const float4*>(yd + (size_t)sp * plane + (size_t)slot * H + c);
                s0 += v.x; s1 += v.y; s2 += v.z; s3 += v.w;
            }
            a[0] = fmaf(wj, s0, a[0]); a[1] = fmaf(wj, s1, a[1]); a[2] = fmaf(wj, s2, a[2]); a[3] = fmaf(wj, s3, a[3]);
        }
    }
    if constexpr (YD16) {
        u32x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = pack_bf2(a[2 * i], a[2 * i + 1]);
        *reinterpret_cast<u32x4*>(y + (size_t)t * H + c) = o;
    } else {
        uint2 o;
        o.x = pack_bf2(a[0], a[1]);
        o.y = pack_bf2(a[2], a[3]);
        *reinterpret_cast<uint2*>(y + (size_t)t * H + c) = o;
    }
}

template <int MT, int WM, int STAGE, int GS, int CW = 4, bool G2 = false>
tq_status launch_main(const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin, const uint16_t* xaug,
                      const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                      const int32_t* offsets, const int32_t* ctrl, int ctrl_idx, void* out, int ka, int nsplit,
                      int row_tiles, hipStream_t st)
{
    constexpr int BM = 32 * MT * WM;
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int ROWB = UNIT_K * 2 + 16;
    const size_t smem = (size_t)2 * mfma_chunk_units(MT, GS) * BM * ROWB + (size_t)2 * BM * 4;
    auto kern = moe_mfma_kernel<MT, WM, STAGE, GS, CW, G2>;      // dynamic-LDS limit: raised once per device by tqi_setup_mfma
    const int nb_count = (sec.pairs + 3) / 4;
    const long n_wg = (long)((row_tiles + 7) / 8) * 8 * nb_count;
    if (n_wg > 0x7FFFFFFF || nb_count > 65535) return TQ_ERR_UNSUPPORTED;
    dim3 grid((unsigned)n_wg, 1, nsplit);
    hipLaunchKernelGGL(kern, grid, dim3(256 * WM), smem, st, G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl,
                       ctrl_idx, out, ka, nsplit);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

template <int MT, int WM, int STAGE>
tq_status launch_main_gs(int gs, int cw, const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin, const uint16_t* xaug,
                         const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                         const int32_t* offsets, const int32_t* ctrl, int ctrl_idx, void* out, int ka, int nsplit,
                         int row_tiles, hipStream_t st)
{
#define TQ_CASE(GSV)                                                                                              \
    case GSV:                                                                                                     \
        return launch_main<MT, WM, STAGE, GSV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, ctrl_idx, \
                                           out, ka, nsplit, row_tiles, st)
    if (cw != 4) {      // dense codes: groups of 64 and 128
        if constexpr (MT == 1) {      // groups of 128 on the 32-row tile: units of half a group (see G2)
            if (gs == 8 && cw == 3)
                return launch_main<MT, WM, STAGE, 4, 3, true>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl,
                                                              ctrl_idx, out, ka, nsplit, row_tiles, st);
            if (gs == 8 && cw == 2)
                return launch_main<MT, WM, STAGE, 4, 2, true>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl,
                                                              ctrl_idx, out, ka, nsplit, row_tiles, st);
        }
#define TQ_DENSE(GSV, CWV)                                                                                                   \
    if (gs == GSV && cw == CWV)                                                                                              \
        return launch_main<MT, WM, STAGE, GSV, CWV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, ctrl_idx, \
                                                    out, ka, nsplit, row_tiles, st)
        TQ_DENSE(4, 3); TQ_DENSE(4, 2);
        if constexpr (MT != 1) { TQ_DENSE(8, 3); TQ_DENSE(8, 2); }      // (the 32-row tile took its groups of 128 above)
#undef TQ_DENSE
        return TQ_ERR_UNSUPPORTED;
    }
    if constexpr (MT == 1) {
        // groups of 128 on the 32-row tile: units of half a group (see G2)
        if (gs == 8)
            return launch_main<MT, WM, STAGE, 4, 4, true>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl,
                                                          ctrl_idx, out, ka, nsplit, row_tiles, st);
    }
    switch (gs) {
        TQ_CASE(2);
        TQ_CASE(4);
        case 8:
            if constexpr (MT != 1) {      // (the 32-row tile took its groups of 128 above)
                return launch_main<MT, WM, STAGE, 8>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, ctrl_idx,
                                                     out, ka, nsplit, row_tiles, st);
            }
            break;
        case 16:
            if constexpr (MT == 1) {
                return launch_main<MT, WM, STAGE, 16>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, ctrl_idx,
                                                      out, ka, nsplit, row_tiles, st);
            }
            break;      // groups of 256 with large tiles go through the <4, 1> instantiation
    }
#undef TQ_CASE
    return TQ_ERR_UNSUPPORTED;
}

template <int MT, int WM, int STAGE, int GS, int CW = 4, bool G2 = false>
bool raise_lds_limit_main()
{
    constexpr int BM = 32 * MT * WM;
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int ROWB = UNIT_K * 2 + 16;
    constexpr size_t smem = (size_t)2 * mfma_chunk_units(MT, GS) * BM * ROWB + (size_t)2 * BM * 4;
    if (smem <= 64 * 1024) return true;
    return hipFuncSetAttribute((const void*)moe_mfma_kernel<MT, WM, STAGE, GS, CW, G2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)smem) == hipSuccess;
}

template <int STAGE>
tq_status launch_aug(const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin, const int32_t* row_token,
                const int32_t* tile_e, const int32_t* tile_row0, const int32_t* offsets, const int32_t* ctrl,
                uint16_t* xaug, int ka, int rt32, float* tslice, size_t tslice_bytes, hipStream_t st)
{
    // fewer column tiles leave registers for more loads in flight; eight steps at a time need units of 128
    const int nat = G.r > 0 ? sec.na_tiles : 0;
    const int gs = G.g / 16;
    // the staged variant: groups up to 128, at most four column tiles of t, 32-bit byte offsets of the rows
    const uint64_t span = (uint64_t)(STAGE == 0 ? G.a_tot / (G.k + G.S) : G.a_tot) * sec.K * 2;
    if (gs <= 8 && nat <= 4 && span < (1ull << 32)) {
        // A workgroup per row tile walks the whole contraction, some 3 us of dependent latency per chunk: with fewer
        // tiles than workgroup slots (a medium batch on a layer of few experts, a small one on many experts) the
        // contraction is cut into slices of at least 512 indices until about 512 workgroups exist, and a second launch
        // adds the slices of t up.
        const int natv = nat <= 1 ? 1 : nat == 2 ? 2 : 4;
        const int nchunks = (sec.groups + 3) / 4, ck = 4 * G.g;
        const int tiles_est = std::max(1, std::min(rt32, (int)G.a_tot));
        int cps = nchunks, nsl = 1;
        // (measured: a gain up to 128 row tiles on every layer shape, up to 160 only on contractions of 4096 and more;
        // beyond that the tiles alone fill the chip and the second launch is a loss)
        if (rt32 <= 128 || (rt32 <= TQ_AUG_SLICE_MAX_TILES && sec.K >= 4096)) {
            const int want = (512 + tiles_est - 1) / tiles_est;
            cps = std::max((nchunks + want - 1) / want, (512 + ck - 1) / ck);
            nsl = (nchunks + cps - 1) / cps;
            if (nat > 0 && (size_t)rt32 * nsl * natv * 4096 > tslice_bytes) { cps = nchunks; nsl = 1; }
        }
        float* ts = (nsl > 1 && nat > 0) ? tslice : nullptr;
#define TQ_AUGS(NATV, GSV)                                                                                          \
    hipLaunchKernelGGL((aug_staged_kernel<STAGE, NATV, GSV>), dim3(rt32, nsl), dim3(256),                       \
                       std::max<size_t>((size_t)32 * (4 * GSV * 32 + 16), 4 * 16 * 64 * sizeof(float)) /* staging | reduction */, \
                       st, G, sec, blob, xin, row_token, tile_e, tile_row0, offsets, ctrl, xaug, ka, cps, ts)
        if (nat <= 1) { if (gs == 8) TQ_AUGS(1, 8); else if (gs == 4) TQ_AUGS(1, 4); else TQ_AUGS(1, 2); }
        else if (nat == 2) { if (gs == 8) TQ_AUGS(2, 8); else if (gs == 4) TQ_AUGS(2, 4); else TQ_AUGS(2, 2); }
        else { if (gs == 8) TQ_AUGS(4, 8); else if (gs == 4) TQ_AUGS(4, 4); else TQ_AUGS(4, 2); }
#undef TQ_AUGS
        TQ_CHECK_LAUNCH();
        if (ts) {
            hipLaunchKernelGGL(aug_slices_kernel, dim3(rt32, nat, 4), dim3(256), 0, st, (const float*)ts, nsl, natv,
                               STAGE == 0 ? 2 * G.r16 : G.r16, tq_zero_terms(sec.K, G.g), tile_e, tile_row0, offsets, ctrl,
                               xaug, ka);
            TQ_CHECK_LAUNCH();
        }
        return TQ_OK;
    }
    const bool deep = (G.g < 64 ? 64 : G.g) % 128 == 0;
#define TQ_AUG(NATV, UNRV)                                                                                        \
    hipLaunchKernelGGL((aug_kernel<STAGE, NATV, UNRV>), dim3(rt32), dim3(256), 0, st, G, sec, blob, xin, row_token, \
                       tile_e, tile_row0, offsets, ctrl, 1, xaug, ka)
    if (nat <= 1 && deep) TQ_AUG(1, 8);
    else if (nat <= 1) TQ_AUG(1, 4);
    else if (nat == 2 && deep) TQ_AUG(2, 8);
    else if (nat == 2) TQ_AUG(2, 4);
    else TQ_AUG(4, 4);
#undef TQ_AUG
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

}  // namespace

tq_status tqi_setup_mfma()
{
    bool ok = true;
#define TQ_BOTH(MT, GS) ok = ok && raise_lds_limit_main<MT, 1, 0, GS>() && raise_lds_limit_main<MT, 1, 1, GS>()
    TQ_BOTH(1, 2); TQ_BOTH(1, 4); TQ_BOTH(1, 16);
    ok = ok && raise_lds_limit_main<1, 1, 0, 4, 4, true>() && raise_lds_limit_main<1, 1, 1, 4, 4, true>();
    ok = ok && raise_lds_limit_main<1, 1, 0, 4, 3, true>() && raise_lds_limit_main<1, 1, 1, 4, 3, true>();
    ok = ok && raise_lds_limit_main<1, 1, 0, 4, 2, true>() && raise_lds_limit_main<1, 1, 1, 4, 2, true>();
    TQ_BOTH(2, 2); TQ_BOTH(2, 4); TQ_BOTH(2, 8);
    TQ_BOTH(4, 16);
#undef TQ_BOTH
#define TQ_DENSE(MT, GS, CW) ok = ok && raise_lds_limit_main<MT, 1, 0, GS, CW>() && raise_lds_limit_main<MT, 1, 1, GS, CW>()
    TQ_DENSE(1, 4, 3); TQ_DENSE(1, 4, 2);
    TQ_DENSE(2, 4, 3); TQ_DENSE(2, 8, 3); TQ_DENSE(2, 4, 2); TQ_DENSE(2, 8, 2);
#undef TQ_DENSE
    return ok ? TQ_OK : TQ_ERR_HIP;
}

// Tile choice of the bf16 forward: rows per expert on average decide between the 32-row tile and the large tiles;
// decode batches (a handful of rows per expert) take the weight-streaming 16-row path when the layer allows it.
static bool bf16_large_tiles_rows(const TqLayout& L, int64_t a_tot, int flags);
static bool bf16_large_tiles(const TqLayout& L, const TqWorkspace& W, int flags) { return bf16_large_tiles_rows(L, W.a_tot, flags); }
static bool bf16_large_tiles_rows(const TqLayout& L, int64_t a_tot, int flags)
{
    // measured crossover of the two tilings (four layer shapes, batches swept across it): a layer of 8 wide experts
    // changes over between 28 rows per expert (32-row kernel 11 % ahead) and 30 (large tiles 13 % ahead: by then
    // most experts hold more than 32 rows, a second tile for the 32-row kernel); the 128-expert layer (hidden size
    // 4096) between 16 rows (32-row kernel 4 % ahead) and 20 (large tiles 4 % ahead, 5.5 % at 24); the 60- and
    // 66-expert layers (hidden size 2048) between 24 rows (32-row kernel 4-5 % ahead) and 32 (large tiles 3 % ahead).
    // (Before the 32-row kernel was compiled for more waves per SIMD and its pre-pass cut over K, these crossovers
    // lay at 12 to 16 rows.)
    const int64_t avg_rows = a_tot / (L.E + L.S);
    bool large = avg_rows >= (L.E + L.S <= 16 ? 30 : L.H <= 2048 ? 28 : 20);
    if (flags & TQ_FLAG_FORCE_SMALL_TILE) large = false;
    if (flags & TQ_FLAG_FORCE_LARGE_TILE) large = true;
    return large;
}

bool tqi_bf16_takes_skinny(const TqLayout& L, const TqWorkspace& W, int flags) { return tqi_bf16_rows_take_skinny(L, W.a_tot, flags); }

bool tqi_bf16_rows_take_skinny(const TqLayout& L, int64_t a_tot, int flags)
{
    // The decode kernels pay where a few large experts hold a handful of rows each: measured against the 32-row
    // kernel they are 20-35 % ahead up to 8 rows per expert on layers of 8 to 32 experts and fall behind at 12 (an
    // expert with more than 16 rows streams its weights once per 16-row tile: 190 against 173 us, 224 against 172 us).
    // With 8 experts they stay ahead up to 12 rows (181 against 230 us) and lose at 14 (281 against 231 us: some
    // expert then holds more than 16).  On layers of 60 and more experts every (tile, column pair) costs them the same
    // time whether the tile holds one row or sixteen - 5 us on a contraction of 4096, half of that up to 2048, where a
    // wave's slice is 256 wide - so how long they stay ahead goes by the hidden size: with 4096 up to 3 rows per
    // expert on average (128 experts: 124 against 149 us at 1 row, 179 against 192 at 3, 212 against 196 at 4), with
    // 2048 up to 8 (60 experts, groups of 64: 94 against 120 us at 1 row, 122 against 142 at 8; 66 experts, groups of
    // 128: 76 against 91 at 2 rows, level at 8).
    const int64_t avg_rows = a_tot / (L.E + L.S);
    const int ne = L.E + L.S;
    const bool few_rows = ne <= 32 ? avg_rows <= (ne <= 8 ? 12 : 10) : a_tot <= (L.H <= 2048 ? 8 : 3) * (int64_t)ne;
    bool skinny = !bf16_large_tiles_rows(L, a_tot, flags) && few_rows && !(flags & TQ_FLAG_FORCE_SMALL_TILE);
    if (flags & TQ_FLAG_FORCE_SKINNY) skinny = true;
    // (dense codes and fp8 factors follow the same rule: the parts the tiled kernels derive per call are laid out in
    // the workspace exactly when this returns false)
    return skinny && a_tot <= TQ_SKINNY_MAX_ROWS && tqi_skinny_supported(L);
}

tq_status tqi_forward_bf16(const TqLayout& L, const TqWorkspace& W, int flags, const uint8_t* blob,
                           const uint16_t* x, int32_t T, uint16_t* y, uint8_t* ws, hipStream_t stream,
                           const float* topk_w)
{
    if (L.r16 > 128) return TQ_ERR_UNSUPPORTED;
    MGeom G;
    G.ne = L.E + L.S; G.H = L.H; G.F = L.F; G.g = L.g; G.r = L.r; G.r16 = L.r16; G.k = L.k; G.S = L.S;
    G.a_tot = W.a_tot; G.expert_stride = L.expert_stride; G.fm = L.fm;
    G.unpack_mask = L.cw == 4 ? 0x000F000Fu : L.cw == 3 ? 0x00070007u : 0x00030003u;
    G.unpack_magic = 0x43004300u;
    G.zc_ws = nullptr; G.zc_stride = 0; G.zc_d_off = 0;
    const int32_t* ctrl = reinterpret_cast<const int32_t*>(ws + W.ctrl);
    const int32_t* offsets = reinterpret_cast<const int32_t*>(ws + W.offsets);
    const int32_t* slot_of = reinterpret_cast<const int32_t*>(ws + W.slot_of);
    const int32_t* row_token = reinterpret_cast<const int32_t*>(ws + W.row_token);
    const int32_t* tile_e = reinterpret_cast<const int32_t*>(ws + W.tile_e);
    const int32_t* tile_row0 = reinterpret_cast<const int32_t*>(ws + W.tile_row0);
    uint16_t* xaug_gu = reinterpret_cast<uint16_t*>(ws + W.xaug_gu);
    uint16_t* xaug_d = reinterpret_cast<uint16_t*>(ws + W.xaug_d);
    uint16_t* h = reinterpret_cast<uint16_t*>(ws + W.h);
    float* yd = reinterpret_cast<float*>(ws + W.yd);

    const bool large = bf16_large_tiles(L, W, flags);
    const int rt32 = W.a_tot / 32 + L.E + L.S;     // upper bounds on the number of row tiles
    const int rt128 = W.a_tot / 128 + L.E + L.S;
    const int rt64 = W.a_tot / 64 + L.E + L.S;
    const int gs = L.g / 16;
    const bool persist = tqi_prefill_supported(L, W, T);

    // decode batches (a handful of rows per expert): the weight-streaming 16-row path, no pre-pass over K
    if (tqi_bf16_takes_skinny(L, W, flags)) {
        int nsplit_sk = 1;
        tq_status rs = tqi_forward_skinny(L, W, blob, x, T, ws, stream, &nsplit_sk);
        if (rs != TQ_OK) return rs;
        tqi_record_stage(5, stream);
        hipLaunchKernelGGL(combine_bf16_kernel<false>, dim3(T, (L.H / 4 + 255) / 256), dim3(256), 0, stream, T, L.H, L.k, L.S,
                           nsplit_sk, (size_t)W.a_tot * L.H, slot_of, topk_w, yd, y);
        TQ_CHECK_LAUNCH();
        tqi_record_stage(6, stream);
        return TQ_OK;
    }

    tq_status rc;
    if (L.fm.fp8) {
        // fp8 factors: the tiled kernels read fp16 fragments, expanded into the workspace for this call
        if (W.fac_bytes == 0) return TQ_ERR_UNSUPPORTED;
        rc = tqi_expand_fp8_factors(L, W, blob, ws, stream);
        if (rc != TQ_OK) return rc;
        G.fm = W.fac_fm;
        G.fm.fbase = ws + W.fac_ws;
    }
    if (L.cw != 4) {
        // dense codes: the blob stores no zero-point coefficient fragments; the tiled kernels read them from the workspace
        if (W.zc_stride == 0 || gs == 16) return TQ_ERR_UNSUPPORTED;
        rc = tqi_derive_zc(L, W, blob, ws, stream);
        if (rc != TQ_OK) return rc;
        G.zc_ws = ws + W.zc_ws; G.zc_stride = W.zc_stride; G.zc_d_off = W.zc_d_off;
    }
    rc = launch_aug<0>(G, L.gu, blob, x, row_token, tile_e, tile_row0, offsets, ctrl, xaug_gu, W.ka_gu, rt32,
                       reinterpret_cast<float*>(ws + W.tpart), W.tpart_bytes, stream);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(2, stream);
    // many rows per expert: persistent 64-row-tile workgroups (tq_prefill.hip) when the layer qualifies, else one
    // workgroup per 64-row tile; groups of 256 need more registers than two workgroups per CU leave and run
    // as four waves of 128x64 on 128-row tiles
    if (large && gs == 16)
        rc = launch_main<4, 1, 0, 16>(G, L.gu, blob, x, xaug_gu, row_token, tile_e + W.rt_max, tile_row0 + W.rt_max,
                                      offsets, ctrl, 2, h, W.ka_gu, 1, rt128, stream);
    else if (large && persist)
        rc = tqi_forward_prefill_stage(0, L, W, G, blob, x, xaug_gu, row_token, tile_e + 3 * (size_t)W.rt_max,
                                       tile_row0 + 3 * (size_t)W.rt_max, offsets, ctrl, 5, h, stream);
    else if (large)
        // 64-row tiles, four waves of 64x64: two such workgroups share a CU and run out of phase, so one's
        // per-unit tail (fold, staging store, barrier) overlaps the other's MFMAs
        rc = launch_main_gs<2, 1, 0>(gs, L.cw, G, L.gu, blob, x, xaug_gu, row_token, tile_e + 3 * (size_t)W.rt_max,
                                     tile_row0 + 3 * (size_t)W.rt_max, offsets, ctrl, 5, h, W.ka_gu, 1, rt64, stream);
    else
        rc = launch_main_gs<1, 1, 0>(gs, L.cw, G, L.gu, blob, x, xaug_gu, row_token, tile_e, tile_row0, offsets, ctrl, 1, h, W.ka_gu, 1,
                                  rt32, stream);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(3, stream);
    rc = launch_aug<1>(G, L.d, blob, h, row_token, tile_e, tile_row0, offsets, ctrl, xaug_d, W.ka_d, rt32,
                       reinterpret_cast<float*>(ws + W.tpart), W.tpart_bytes, stream);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(4, stream);
    int nsplit = 1;
    if (!large && W.a_tot <= TQ_SPLITK_MAX_ROWS) {
        // few rows: split the long contraction of the down projection so the grid fills the chip
        const int unit_k = L.g < 64 ? 64 : L.g;
        const int nu = L.F / unit_k;
        const int64_t base = (int64_t)((L.d.pairs + 3) / 4) * (rt32 < L.E + L.S ? rt32 : L.E + L.S);
        int want = (int)((1024 + base - 1) / base);
        nsplit = want < 1 ? 1 : want > TQ_MAX_SPLIT ? TQ_MAX_SPLIT : want;
        if (nsplit > nu) nsplit = nu;
    }
    if (large && gs != 16 && W.a_tot <= TQ_SPLITK_MAX_ROWS) {
        // a medium batch on a layer of few, wide experts leaves the 64-row tiling a few hundred (tile, column block)
        // items that each walk the whole long contraction: one or two per workgroup, finishing far apart.  Split
        // over K into about 1500 workgroups of the one-item kernel instead (fp32 planes, summed by the combine), each
        // with at least 2048 contraction indices: on short contractions (layers of many narrow experts, measured at
        // 1408) the planes cost more than the balance gains.
        const int64_t items = (int64_t)((L.d.pairs + 3) / 4) * rt64;
        if (items < 1024) {
            int want = (int)((1536 + items - 1) / items);
            if (want > TQ_MAX_SPLIT) want = TQ_MAX_SPLIT;
            if (want > L.F / 2048) want = L.F / 2048;
            if (want > 1) nsplit = want;
        }
    }
    if (large && gs == 16)
        rc = launch_main<4, 1, 1, 16>(G, L.d, blob, h, xaug_d, row_token, tile_e + W.rt_max, tile_row0 + W.rt_max,
                                      offsets, ctrl, 2, yd, W.ka_d, 1, rt128, stream);
    else if (large && persist && nsplit == 1)
        rc = tqi_forward_prefill_stage(1, L, W, G, blob, h, xaug_d, row_token, tile_e + 3 * (size_t)W.rt_max,
                                       tile_row0 + 3 * (size_t)W.rt_max, offsets, ctrl, 5, yd, stream);
    else if (large)
        rc = launch_main_gs<2, 1, 1>(gs, L.cw, G, L.d, blob, h, xaug_d, row_token, tile_e + 3 * (size_t)W.rt_max,
                                     tile_row0 + 3 * (size_t)W.rt_max, offsets, ctrl, 5, yd, W.ka_d, nsplit, rt64, stream);
    else
        rc = launch_main_gs<1, 1, 1>(gs, L.cw, G, L.d, blob, h, xaug_d, row_token, tile_e, tile_row0, offsets, ctrl, 1, yd, W.ka_d,
                                  nsplit, rt32, stream);
    if (rc != TQ_OK) return rc;
    tqi_record_stage(5, stream);
    if (large && nsplit == 1)
        hipLaunchKernelGGL(combine_bf16_kernel<true>, dim3(T, (L.H / 8 + 255) / 256), dim3(256), 0, stream, T, L.H, L.k,
                           L.S, 1, (size_t)0, slot_of, topk_w, yd, y);
    else
        hipLaunchKernelGGL(combine_bf16_kernel<false>, dim3(T, (L.H / 4 + 255) / 256), dim3(256), 0, stream, T, L.H, L.k,
                           L.S, nsplit, (size_t)W.a_tot * L.H, slot_of, topk_w, yd, y);
    TQ_CHECK_LAUNCH();
    tqi_record_stage(6, stream);
    return TQ_OK;
}
