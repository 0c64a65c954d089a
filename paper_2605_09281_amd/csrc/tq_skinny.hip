// Decode path of tq_moe_forward (few rows per expert): the projection is bound by streaming the packed
// weights from HBM once, so the kernel is built around that stream.
//
//   * A row tile holds at most 16 assignment rows of one expert.  Its activations for the whole
//     contraction range of the workgroup (up to 4096 values per row) are staged in LDS ONCE.
//   * A workgroup has 8 waves; wave w owns a 512-wide slice (256 on contractions up to 2048) of the contraction range and walks over the
//     workgroup's column-tile pairs, streaming its slice of the packed codes (already in MFMA fragment
//     order) straight from global memory into registers, one pair ahead.  No barrier in that stream.
//   * Codes go to v_mfma_f32_32x32x16_bf16 as 128 + q (rows 16..31 of the tile are padding); each
//     quantisation group's fp32 partial sum is folded as  acc += s * part - s (128 + z) * xsum, with the
//     group sums of the activations computed once per workgroup by an MFMA against a matrix of ones.
//   * The 8 partial results of a pair are summed across the waves through LDS in a fixed order (the
//     "wavefront reduction"), then SwiGLU (stage 0) or the store of the split-K plane (stage 1).
//   * The low-rank intermediate t = x A is produced per 256-wide slice by skinny_pre_kernel (for decode batches
//     proper the gate/up slices come per assignment from the permutation's launch instead); a workgroup
//     adds the slices of its own range, so a split contraction needs no global reduction: the partial
//     t of a split times B lands in that split's output plane, and the planes are summed by the combine.
#include "tq_device.h"

#include <algorithm>
#include <type_traits>

using namespace tqdev;

namespace {

constexpr int SK_NW = 8;        // waves per workgroup
constexpr int SK_RED_BYTES = SK_NW * 7 * 2 * 64 * 4;   // per wave: 7 of its 8 row groups, 2 tiles, 64 lanes

__device__ inline int row_of_v(int v, int hf) { return 8 * (v >> 2) + 4 * hf + (v & 3); }

// Partial low-rank intermediate of one 16-row tile over one 256-wide slice of the contraction:
//   tpart[tile][slice][ta][v][lane] = sum_{kk in slice} x[row(v, lane)][kk] * A[kk][32 ta + lane % 32]   (fp32)
// One wave per (tile, slice, ta); all of its loads are in flight at once.
constexpr int SK_PRE_K = 256;

template <int STAGE, bool FP8>
__global__ void __launch_bounds__(64) skinny_pre_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                        const uint16_t* __restrict__ xin,
                                                        const int32_t* __restrict__ row_token,
                                                        const int32_t* __restrict__ tile_e,
                                                        const int32_t* __restrict__ tile_row0,
                                                        const int32_t* __restrict__ offsets,
                                                        const int32_t* __restrict__ ctrl, float* __restrict__ tpart,
                                                        int n_slices, int na_tiles)
{
    const int tile = blockIdx.x, slice = blockIdx.y, ta = blockIdx.z, lane = threadIdx.x;
    if (tile >= ctrl[4]) return;
    const int e = tile_e[tile], slot0 = tile_row0[tile];
    const int rows = min(16, offsets[e + 1] - slot0);
    const int col = lane & 31, hf = lane >> 5;
    const int K = sec.K, ksteps = K / 16;
    const int r = min(col & 15, rows - 1);
    const uint16_t* xrow = STAGE == 0 ? xin + (size_t)row_token[slot0 + r] * K : xin + (size_t)(slot0 + r) * K;
    const u32x4* af = reinterpret_cast<const u32x4*>(tq_afrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e));
    constexpr int NS = SK_PRE_K / 16;
    const int s0 = slice * NS;
    const int n = min(NS, ksteps - s0);
    Frag xa[NS];
    u32x4 aq[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u)
        if (u < n) {
            xa[u].q = *reinterpret_cast<const u32x4*>(xrow + 16 * (s0 + u) + 8 * hf);
            const size_t f = (size_t)ta * ksteps + s0 + u;                  // fragment; fp8 fragments are half as long
            aq[u] = af[FP8 ? f * 32 + (lane >> 1) : f * 64 + lane];
        }
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int u = 0; u < NS; ++u)
        if (u < n)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[u].v, FP8 ? fp8_frag_to_bf8(aq[u], lane) : half8_to_bf8(aq[u]), acc,
                                                          0, 0, 0);
    float* dst = tpart + (((size_t)tile * n_slices + slice) * na_tiles + ta) * 512 + lane;
#pragma unroll
    for (int v = 0; v < 8; ++v) dst[v * 64] = acc[v];
}

// STAGE 0: out = h[slot][F] bf16 = silu(gate) * up.   STAGE 1: out = yd[split][slot][H] fp32.
// CW: 32-bit words of codes per lane, tile and 64-wide chunk: 4 (4-bit slots), 3 or 2 (dense 3- / 2-bit codes).
// DEAL: the workgroups share out the (tile, split) combinations that exist among themselves (1-D grid) instead of
// taking the one their 3-D block index names; see below.
// WK: contraction indices per wave (512, or 256 on contractions of at most 2048 so that all eight waves have a slice).
template <int STAGE, int GS, int CW, bool DEAL, int WK>
__global__ void __launch_bounds__(512) moe_skinny_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob,
                                                         const uint16_t* __restrict__ xin,
                                                         const int32_t* __restrict__ row_token,
                                                         const int32_t* __restrict__ tile_e,
                                                         const int32_t* __restrict__ tile_row0,
                                                         const int32_t* __restrict__ offsets,
                                                         const int32_t* __restrict__ ctrl,
                                                         const float* __restrict__ tpart, int n_slices, int na_tiles,
                                                         void* __restrict__ out, int32_t* __restrict__ pair_cnt,
                                                         int units_per_split, int RB, int red_off, int xs_off, int mb_off,
                                                         const int32_t* __restrict__ row_src, int nsplit,
                                                         const int32_t* __restrict__ tile_rows)
{
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int UC = UNIT_K / 64;
    constexpr int US = UNIT_K / 16;
    constexpr int NG = US / GS;
    constexpr int UPW = WK / UNIT_K;   // units per wave
    using WT = std::conditional_t<CW == 4, u32x4, uint32_t>;      // register type of the packed codes
    constexpr int WN = CW == 4 ? UC : UC * CW;                    // and how many of them one tile of a unit takes

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    float* red = reinterpret_cast<float*>(lds + red_off);
    float* xs = reinterpret_cast<float*>(lds + xs_off);
    uint16_t* tbuf = reinterpret_cast<uint16_t*>(lds + red_off);   // [16][NA] bf16; lives only before the pair loop

    // Which (row tile, split) this workgroup works on, its number `part` among the g_wg workgroups on it:
    //  * 3-D grid (layers of few experts, where the host knows how many tiles will exist): blockIdx itself;
    //  * DEAL, 1-D grid (many small experts, most of the tiles the host has to allow for are empty): the
    //    workgroups are shared out among the combinations that EXIST, a number only the device knows.  Each of the
    //    n_v combinations gets G = grid / n_v consecutive workgroups (consecutive ids sit on different XCDs, so a
    //    combination's weight stream is spread over all of them), the first grid mod n_v one more from the end.
    //    (A template argument, not a run-time switch or the only form: the kernel is short of scalar registers, and
    //    the second form measured 1-2 % slower per stage on the 8-expert decode layer in every spelling tried; its
    //    surplus workgroups leave inside the block below because the same test further down cost the down stage 70
    //    more spilled scalar registers.)
    int rt, split, part, g_wg;
    if constexpr (!DEAL) {
        rt = blockIdx.y;
        if (rt >= ctrl[4]) return;
        split = blockIdx.z;
        part = blockIdx.x;
        g_wg = gridDim.x;
    } else {
        const int n_t = ctrl[4], n_v = n_t * nsplit;
        if (n_v == 0) return;
        const int G_lo = (int)gridDim.x / n_v, n_full = G_lo * n_v;      // the grid has at least n_v workgroups
        const bool extra = (int)blockIdx.x >= n_full;
        const int vt = extra ? (int)blockIdx.x - n_full : (int)blockIdx.x / G_lo;
        part = extra ? G_lo : (int)blockIdx.x % G_lo;
        if (part >= sec.pairs) return;      // more workgroups on this combination than it has pairs
        g_wg = G_lo + (vt < (int)gridDim.x - n_full ? 1 : 0);
        rt = vt % n_t;
        split = vt / n_t;
    }
    const int e = tile_e[rt], slot0 = tile_row0[rt];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int K = sec.K, NU = K / UNIT_K;
    const int NA = STAGE == 0 ? 2 * G.r16 : G.r16;
    const int n_lr = (G.r > 0) ? NA / 16 : 0;       // low-rank MFMA steps; step j is applied by wave j
    const int ub = split * units_per_split;
    const int ue = min(NU, ub + units_per_split);
    const int range_k = (ue - ub) * UNIT_K;
    int nuw = min(UPW, ue - (ub + wave * UPW));     // units of this wave (0 for idle waves)
    if (nuw < 0) nuw = 0;
    const int wk0 = wave * UPW * US;                // first MFMA step of this wave inside the workgroup's range
    // Column-tile pairs are dealt out dynamically among the g_wg workgroups of this (tile, split): the first one is the
    // workgroup's number among them, every further one comes from a counter (cleared by the permutation), fetched one pair
    // ahead of its use so that the weight prefetch knows where to go.  Workgroups that get a better share of the
    // memory system take more pairs, and all of them finish together.
    const int npairs = sec.pairs;
    const int p0 = part;
    int32_t* cnt = pair_cnt + (size_t)rt * TQ_MAX_SPLIT + split;
    int* pq = reinterpret_cast<int*>(lds + mb_off);            // two mailbox words
    int got_v = 0;
    if (tid == 0) got_v = g_wg + atomicAdd(cnt, 1);

    const uint8_t* rec = blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride;
    const u32x4* codes = reinterpret_cast<const u32x4*>(rec + sec.codes) + lane;
    const uint32_t* szp = reinterpret_cast<const uint32_t*>(rec + sec.sz) + col;
    const u32x4* bfr = reinterpret_cast<const u32x4*>(G.r > 0 ? tq_bfrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e)
                                                               : rec + sec.bfrag);
    const bool fp8 = G.fm.fp8 != 0;
    // fragment f of the right factors: 64 lanes x 16 bytes (fp16), or 64 x 8 bytes (fp8: lanes 2j, 2j + 1 share a word)
    const int b_per = fp8 ? 32 : 64, b_lane = fp8 ? (lane >> 1) : lane;

    // Unit and pair indices are clamped into the valid range instead of guarding the loads: a load under a
    // condition makes the compiler wait for ALL outstanding loads at every later use, which would drain the
    // one-pair-ahead prefetch at every unit.  Clamped loads repeat a neighbour's line (cache hit) and are unused.
    const uint32_t* codes32 = reinterpret_cast<const uint32_t*>(rec + sec.codes) + lane;      // dense layouts
    auto load_w = [&](WT (&dst)[2][WN], int pair, int u) {       // unit u of this wave, both tiles
        const int chunk0 = min(ub + wave * UPW + u, ue - 1) * UC;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < UC; ++c) {    // read once, never again: the non-temporal hint keeps the stream out of the caches
                if constexpr (CW == 4) {
                    dst[t][c] = __builtin_nontemporal_load(&codes[(((size_t)pair * sec.chunks + chunk0 + c) * 2 + t) * 64]);
                } else {
#pragma unroll
                    for (int d = 0; d < CW; ++d)
                        dst[t][c * CW + d] = __builtin_nontemporal_load(
                            &codes32[((((size_t)pair * sec.chunks + chunk0 + c) * 2 + t) * CW + d) * 64]);
                }
            }
    };
    auto load_sz = [&](uint32_t (&dst)[NG][2], int pair, int u) {
        const int g0 = min(ub + wave * UPW + u, ue - 1) * NG;
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
            for (int t = 0; t < 2; ++t) dst[gi][t] = szp[(((size_t)pair * sec.groups + g0 + gi) * 2 + t) * 32];
    };

    // the or-operand of the unpack in a vector register (see unpack_word): opaque move, not folded to a literal
    uint32_t magic_v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(G.unpack_magic));

    // ---- 1. activations of the tile for the workgroup's contraction range -> LDS (row stride RB = 2*range + 16 bytes:
    //         the rows read by one ds_read_b128 fall into different bank groups).  Only the rows that exist are
    //         staged; the MFMA rows beyond them re-read the last one and their results are never stored.
    //         Everything the set-up needs (these rows, the low-rank slices) is requested and awaited BEFORE the first
    //         weights are asked for: at kernel start every workgroup asks for its first pair at once, and small
    //         loads queued behind that burst would arrive only after it.
    // (DEAL reads the tile's row count from the tile table: its tile index already waited for a load, and offsets
    // would be one more in the chain)
    const int rows = DEAL ? tile_rows[rt] : min(16, offsets[e + 1] - slot0);
    const int gran = range_k / 8;                 // 16-byte chunks per row
    const int total = rows * gran;
    auto stage_load = [&](int c0, u32x4 (&v)[4], int (&dst)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = min(c0 + j * 512 + tid, total - 1);
            const int row = c / gran, kg = c - row * gran;
            const size_t src_row = STAGE == 0 ? (size_t)row_token[slot0 + row] : (size_t)(slot0 + row);
            v[j] = *reinterpret_cast<const u32x4*>(xin + src_row * K + (size_t)ub * UNIT_K + (size_t)kg * 8);
            dst[j] = row * RB + kg * 16;
        }
    };
    u32x4 xv0[4];
    int xd0[4];
    stage_load(0, xv0, xd0);

    // ---- the slices of the low-rank intermediate: up to 16 per workgroup range and column tile of t.  Requested
    //         before the weights as well, and unconditionally (layers without factors read a valid dummy word with
    //         weight zero).
    // Sigma of fp8 factors for this lane's columns of t (requested with the slices; 1 otherwise, from a valid dummy word)
    float sgv[4];
    {
        const float* sp = fp8 ? tq_sig_base(blob, G.expert_stride, sec, G.fm, STAGE, e) : reinterpret_cast<const float*>(ctrl);
#pragma unroll
        for (int ta = 0; ta < 4; ++ta) sgv[ta] = sp[fp8 ? min(32 * ta + col, NA - 1) : 0];
    }
    float tv[4][16];
    {
        const int sl0 = (ub * UNIT_K) / SK_PRE_K;
        const int nsl = (range_k + SK_PRE_K - 1) / SK_PRE_K;
        const float* tp = n_lr > 0 ? tpart : reinterpret_cast<const float*>(ctrl);
        const size_t live = n_lr > 0 ? 1 : 0;
        if (STAGE == 0 && row_src) {
            // slices stored per assignment (they came with the permutation's launch): this lane's value of step
            // `wave` belongs to row row_of_v(wave, hf) of the tile; padding rows repeat the last one
            const int m = min(row_of_v(wave, hf), rows - 1);
            const size_t v = (size_t)row_src[slot0 + m];
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int sl = 0; sl < 16; ++sl) {
                    const size_t idx = ((v * n_slices + sl0 + min(sl, nsl - 1)) * na_tiles + min(ta, max(na_tiles, 1) - 1)) * 32 + col;
                    tv[ta][sl] = tp[idx * live];
                }
        } else {
#pragma unroll
            for (int ta = 0; ta < 4; ++ta)
#pragma unroll
                for (int sl = 0; sl < 16; ++sl) {
                    const size_t idx = (((size_t)rt * n_slices + sl0 + min(sl, nsl - 1)) * na_tiles + min(ta, max(na_tiles, 1) - 1)) * 512 + wave * 64 + lane;
                    tv[ta][sl] = tp[idx * live];
                }
        }
    }

#pragma unroll
    for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4*>(lds + xd0[j]) = xv0[j];
    for (int c0 = 4 * 512; c0 < total; c0 += 4 * 512) {      // more than four chunks per thread: the rare tall tiles
        u32x4 v[4];
        int dst[4];
        stage_load(c0, v, dst);
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4*>(lds + dst[j]) = v[j];
    }
    float tsum[4] = {0.f, 0.f, 0.f, 0.f};
    {
        const int nsl = (range_k + SK_PRE_K - 1) / SK_PRE_K;
#pragma unroll
        for (int ta = 0; ta < 4; ++ta)
#pragma unroll
            for (int sl = 0; sl < 16; ++sl) tsum[ta] += sl < nsl ? tv[ta][sl] : 0.f;
    }
    // the first pair's codes: their latency hides behind the rest of the set-up (group sums, t fragments)
    WT wq[UPW][2][WN];
    uint32_t szq[UPW][NG][2];
#pragma unroll
    for (int u = 0; u < UPW; ++u) { load_w(wq[u], p0, u); load_sz(szq[u], p0, u); }
    // low-rank B fragments ride in the same prefetch (one pair ahead); waves without a low-rank step, and layers
    // without factors, read a valid dummy location
    const int steps_per_tile = G.r16 / 16;
    const int lr_t = (STAGE == 0 && wave >= steps_per_tile) ? 1 : 0;
    const int lr_step = (G.r > 0) ? min(wave - lr_t * steps_per_tile, steps_per_tile - 1) : 0;
    const u32x4* bsrc = (G.r > 0) ? bfr + b_lane : codes;
    const size_t bstride = (G.r > 0) ? (size_t)steps_per_tile * 2 * b_per : (size_t)0;      // dummy reads stay in the first 2 KB of the codes
    auto load_b = [&](u32x4 (&dst)[2], int pair) {
        if (STAGE == 0) {
            dst[0] = bsrc[(size_t)pair * bstride + ((size_t)lr_step * 2 + lr_t) * b_per];
            dst[1] = dst[0];
        } else {
            dst[0] = bsrc[(size_t)pair * bstride + ((size_t)lr_step * 2 + 0) * b_per];
            dst[1] = bsrc[(size_t)pair * bstride + ((size_t)lr_step * 2 + 1) * b_per];
        }
    };
    auto b_operand = [&](const u32x4& raw) -> bf16x8 { return fp8 ? fp8_frag_to_bf8(raw, lane) : half8_to_bf8(raw); };
    u32x4 bq[2];
    load_b(bq, p0);

    if (tid == 0) pq[0] = got_v;
    lds_barrier();
    const int xrow_off = min(col & 15, rows - 1) * RB;
    auto lds_x = [&](int kl) -> bf16x8 {       // fragment of MFMA step kl (relative to the workgroup's range)
        Frag f;
        f.q = *reinterpret_cast<const u32x4*>(lds + xrow_off + (kl * 16 + 8 * hf) * 2);
        return f.v;
    };

    // ---- 2. group sums of the activations (MFMA against ones: every column of the result holds the row sums)
    {
        Frag ones;
#pragma unroll
        for (int j = 0; j < 4; ++j) ones.u[j] = 0x3F803F80u;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            if (u < nuw) {
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    f32x16 sD;
#pragma unroll
                    for (int v = 0; v < 16; ++v) sD[v] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < GS; ++ks)
                        sD = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_x(wk0 + u * US + gi * GS + ks), ones.v, sD, 0, 0, 0);
                    if (col == 0) {
                        const int gl = (wave * UPW + u) * NG + gi;      // group index inside the workgroup's range
#pragma unroll
                        for (int v = 0; v < 8; ++v) xs[gl * 16 + row_of_v(v, hf)] = sD[v];
                    }
                }
            }
        }
    }
    // ---- 3. low-rank intermediate: add the slices of this range, round to bf16, keep it as MFMA fragments
    Frag tf;
#pragma unroll
    for (int j = 0; j < 4; ++j) tf.u[j] = 0;
    if (n_lr > 0) {
        const int m = row_of_v(wave, hf);          // wave w owns result rows row_of_v(w, hf)
#pragma unroll
        for (int ta = 0; ta < 4; ++ta) {
            const int c = 32 * ta + col;
            if (ta < na_tiles && c < NA) tbuf[m * NA + c] = (uint16_t)f2bf_bits(fp8 ? tsum[ta] * sgv[ta] : tsum[ta]);
        }
        lds_barrier();
        if (wave < n_lr) tf.q = *reinterpret_cast<const u32x4*>(tbuf + (col & 15) * NA + 16 * wave + 8 * hf);
    }
    lds_barrier();     // xs is complete; tbuf has been read: the reduction buffer may be reused

    // ---- 4. the stream over this workgroup's column-tile pairs
    int pnext_raw = pq[0];
    int it = 0;
    for (int pair = p0; pair < npairs;) {
        const int pnext = pnext_raw < npairs ? pnext_raw : pair;     // nothing left: re-request this pair (its scales and
                                                                     // factors hit the cache; the codes are fetched again, once
                                                                     // per workgroup: measured cheaper than a guarded prefetch)
        int fetched = 0;
        if (tid == 0) fetched = g_wg + atomicAdd(cnt, 1);       // the pair after the next one
        float acc8[2][8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 8; ++v) acc8[t][v] = 0.f;
#pragma unroll
        for (int u = 0; u < UPW; ++u) {
            WT wc[2][WN];
            uint32_t szc[NG][2];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int c = 0; c < WN; ++c) wc[t][c] = wq[u][t][c];
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                for (int t = 0; t < 2; ++t) szc[gi][t] = szq[u][gi][t];
            load_w(wq[u], pnext, u);
            load_sz(szq[u], pnext, u);
            if (u < nuw) {
                bf16x8 xq[2];
                xq[0] = lds_x(wk0 + u * US);
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    f32x16 part[2];
#pragma unroll
                    for (int ks = 0; ks < GS; ++ks) {
                        const int kidx = gi * GS + ks;
                        if (kidx + 1 < US) xq[(kidx + 1) & 1] = lds_x(wk0 + u * US + kidx + 1);   // next step's fragment
                        const bf16x8 xa = xq[kidx & 1];
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            bf16x8 bw;
                            if constexpr (CW == 4) bw = unpack_word(word_of(wc[t][kidx / 4], kidx % 4), G.unpack_mask, magic_v);
                            else bw = unpack_dense<CW>(&wc[t][(kidx / 4) * CW], kidx % 4, G.unpack_mask, magic_v);
                            if (ks == 0) {
                                f32x16 zero;
#pragma unroll
                                for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                                part[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, bw, zero, 0, 0, 0);
                            } else {
                                part[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, bw, part[t], 0, 0, 0);
                            }
                        }
                    }
                    // fold the group: acc += s * part + c * xsum, c = -s (128 + z)
                    const int gl = (wave * UPW + u) * NG + gi;
                    const float4 x0 = *reinterpret_cast<const float4*>(xs + gl * 16 + 4 * hf);
                    const float4 x1 = *reinterpret_cast<const float4*>(xs + gl * 16 + 8 + 4 * hf);
                    const float xv[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const float s = tq_half_bits_to_float((uint16_t)(szc[gi][t] & 0xFFFF));
                        const float z = tq_half_bits_to_float((uint16_t)(szc[gi][t] >> 16));
                        const float c = -s * (128.0f + z);
#pragma unroll
                        for (int v = 0; v < 8; ++v) acc8[t][v] = fmaf(c, xv[v], fmaf(s, part[t][v], acc8[t][v]));
                    }
                }
            }
        }
        // low-rank step `wave` (stage 0: steps below r16/16 feed the gate tile, the others the up tile)
        {
            u32x4 bc[2] = {bq[0], bq[1]};
            load_b(bq, pnext);
            if (wave < n_lr) {
                f32x16 zero;
#pragma unroll
                for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                if (STAGE == 0) {
                    const f32x16 lr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf.v, b_operand(bc[0]), zero, 0, 0, 0);
#pragma unroll
                    for (int v = 0; v < 8; ++v) {
                        if (lr_t == 0) acc8[0][v] += lr[v]; else acc8[1][v] += lr[v];
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const f32x16 lr = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tf.v, b_operand(bc[t]), zero, 0, 0, 0);
#pragma unroll
                        for (int v = 0; v < 8; ++v) acc8[t][v] += lr[v];
                    }
                }
            }
        }
        // ---- wavefront reduction: wave w keeps row group v = w and publishes its other seven
        {
            float* mine = red + wave * (7 * 2 * 64);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    if (v != wave) {
                        const int slot = v < wave ? v : v - 1;
                        mine[(t * 7 + slot) * 64 + lane] = acc8[t][v];
                    }
                }
            if (tid == 0) pq[(it + 1) & 1] = fetched;
        }
        lds_barrier();
        {
            float own[2] = {0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 8; ++v)
                    if (v == wave) own[t] = acc8[t][v];
            float tot[2] = {0.f, 0.f};
            for (int ww = 0; ww < SK_NW; ++ww) {           // fixed order: run-to-run identical sums
                if (ww == wave) {
                    tot[0] += own[0];
                    tot[1] += own[1];
                } else {
                    const int slot = wave < ww ? wave : wave - 1;
                    const float* src = red + ww * (7 * 2 * 64);
                    tot[0] += src[(0 * 7 + slot) * 64 + lane];
                    tot[1] += src[(1 * 7 + slot) * 64 + lane];
                }
            }
            const int m = row_of_v(wave, hf);
            if (m < rows) {
                if (STAGE == 0) {
                    const float hv = silu_mul(tot[0], tot[1]);
                    reinterpret_cast<uint16_t*>(out)[(size_t)(slot0 + m) * G.F + 32 * pair + col] = (uint16_t)f2bf_bits(hv);
                } else {
                    float* yd = reinterpret_cast<float*>(out) + (size_t)split * G.a_tot * G.H + (size_t)(slot0 + m) * G.H + 64 * pair + col;
                    yd[0] = tot[0];
                    yd[32] = tot[1];
                }
            }
        }
        lds_barrier();
        pair = pnext_raw;
        pnext_raw = pq[(it + 1) & 1];
        ++it;
    }
}

template <int STAGE, int GS, int CW, int WK>
tq_status launch_skinny(const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin,
                        const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                        const int32_t* offsets, const int32_t* ctrl, float* tpart, int n_slices, int na_tiles,
                        void* out, int32_t* pair_cnt, int row_tiles, int nsplit, int units_per_split,
                        hipStream_t st, const int32_t* row_src, const int32_t* tile_rows)
{
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    const int range_k = units_per_split * UNIT_K;
    const int RB = range_k * 2 + 16;
    const int red_off = 16 * RB;
    const int xs_off = red_off + SK_RED_BYTES;
    const int mb_off = xs_off + (range_k / G.g) * 16 * 4;      // mailbox of the pair scheduler
    const size_t smem = (size_t)mb_off + 16;
    if (smem > 160 * 1024) return TQ_ERR_UNSUPPORTED;
    // one workgroup per compute unit (a workgroup fills a CU's LDS; fewer, longer workgroups amortise the set-up -
    // activation staging, group sums - over more pairs)
    const TqDeviceState* ds = nullptr;
    if (tqi_device_state(&ds) != TQ_OK) return TQ_ERR_HIP;
    dim3 grid;
    int deal_nsplit = 0;
    if (G.ne <= 32) {
        // few experts: nearly all of them receive rows, the host's count of the tiles is good
        const int tiles_est = (int)std::min<int64_t>(G.a_tot, std::min(G.ne, row_tiles));
        long total = (long)sec.pairs * tiles_est * nsplit;
        int ppw = (int)((total + ds->n_cu - 1) / ds->n_cu);
        ppw = std::max(1, std::min(ppw, sec.pairs));
        grid = dim3((sec.pairs + ppw - 1) / ppw, row_tiles, nsplit);
        if (grid.y > 65535) return TQ_ERR_UNSUPPORTED;
    } else {
        // many experts: at least one workgroup per (tile, split) that may exist; the kernel shares them out among
        // those that do
        const long n_wg = std::max<long>(ds->n_cu, (long)row_tiles * nsplit);
        if (n_wg > 0x7FFFFFFF) return TQ_ERR_UNSUPPORTED;
        grid = dim3((unsigned)n_wg);
        deal_nsplit = nsplit;
    }
    // (dynamic-LDS limit of both instantiations: raised once per device by tqi_setup_skinny)
    if (deal_nsplit == 0)
        hipLaunchKernelGGL((moe_skinny_kernel<STAGE, GS, CW, false, WK>), grid, dim3(512), smem, st, G, sec, blob, xin, row_token, tile_e,
                           tile_row0, offsets, ctrl, (const float*)tpart, n_slices, na_tiles, out, pair_cnt, units_per_split,
                           RB, red_off, xs_off, mb_off, row_src, deal_nsplit, tile_rows);
    else
        hipLaunchKernelGGL((moe_skinny_kernel<STAGE, GS, CW, true, WK>), grid, dim3(512), smem, st, G, sec, blob, xin, row_token, tile_e,
                           tile_row0, offsets, ctrl, (const float*)tpart, n_slices, na_tiles, out, pair_cnt, units_per_split,
                           RB, red_off, xs_off, mb_off, row_src, deal_nsplit, tile_rows);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

template <int STAGE>
tq_status launch_skinny_gs(int gs, int cw, const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin,
                           const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                           const int32_t* offsets, const int32_t* ctrl, float* tpart, int n_slices, int na_tiles,
                           void* out, int32_t* pair_cnt, int row_tiles, int nsplit, int units_per_split,
                           hipStream_t st, const int32_t* row_src, const int32_t* tile_rows, int wave_k)
{
#define TQ_SK(GSV, CWV)                                                                                                   \
    do {                                                                                                                  \
        if (wave_k == 256 && GSV * 16 <= 256)                                                                             \
            return launch_skinny<STAGE, GSV, CWV, (GSV * 16 <= 256 ? 256 : 512)>(                                         \
                G, sec, blob, xin, row_token, tile_e, tile_row0, offsets, ctrl, tpart, n_slices, na_tiles, out, pair_cnt, \
                row_tiles, nsplit, units_per_split, st, row_src, tile_rows);                                              \
        return launch_skinny<STAGE, GSV, CWV, 512>(G, sec, blob, xin, row_token, tile_e, tile_row0, offsets, ctrl, tpart,  \
                                                   n_slices, na_tiles, out, pair_cnt, row_tiles, nsplit, units_per_split, \
                                                   st, row_src, tile_rows);                                               \
    } while (0)
    if (cw == 4) {
        switch (gs) {
            case 2: TQ_SK(2, 4);
            case 4: TQ_SK(4, 4);
            case 8: TQ_SK(8, 4);
            case 16: TQ_SK(16, 4);
        }
    } else if (cw == 3) {      // dense codes: groups of 64 and 128
        if (gs == 4) TQ_SK(4, 3);
        if (gs == 8) TQ_SK(8, 3);
    } else if (cw == 2) {
        if (gs == 4) TQ_SK(4, 2);
        if (gs == 8) TQ_SK(8, 2);
    }
#undef TQ_SK
    return TQ_ERR_UNSUPPORTED;
}

// contraction indices per wave of a stage: 512, or 256 on contractions of at most 2048 - a workgroup works on one
// column-tile pair at a time, and with 512-wide slices a contraction of 1536 would leave five of its eight waves idle
inline int wave_k_of(int K, int g) { return (K <= 2048 && g <= 256) ? 256 : 512; }

// contraction split of one stage: nsplit workgroups along K, each a whole number of wave slices
inline void plan_split(int K, int g, int* nsplit, int* units_per_split)
{
    const int unit_k = g < 64 ? 64 : g;
    const int upw = wave_k_of(K, g) / unit_k;
    const int nu = K / unit_k;
    const int max_units = SK_NW * upw;
    int ns = (nu + max_units - 1) / max_units;
    int ups = (nu + ns - 1) / ns;
    ups = (ups + upw - 1) / upw * upw;
    *nsplit = (nu + ups - 1) / ups;
    *units_per_split = ups;
}

}  // namespace

tq_status tqi_setup_skinny()
{
    bool ok = true;
#define TQ_ATTR(ST, GS, CW, DL, WK)                                                                                  \
    ok = ok && hipFuncSetAttribute((const void*)moe_skinny_kernel<ST, GS, CW, DL, WK>,                                  \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess
#define TQ_ONE(ST, GS, CW)                                                                                           \
    TQ_ATTR(ST, GS, CW, false, 512); TQ_ATTR(ST, GS, CW, true, 512);                                                 \
    TQ_ATTR(ST, GS, CW, false, (GS * 16 <= 256 ? 256 : 512)); TQ_ATTR(ST, GS, CW, true, (GS * 16 <= 256 ? 256 : 512))
    TQ_ONE(0, 2, 4); TQ_ONE(0, 4, 4); TQ_ONE(0, 8, 4); TQ_ONE(0, 16, 4);
    TQ_ONE(1, 2, 4); TQ_ONE(1, 4, 4); TQ_ONE(1, 8, 4); TQ_ONE(1, 16, 4);
    TQ_ONE(0, 4, 3); TQ_ONE(0, 8, 3); TQ_ONE(1, 4, 3); TQ_ONE(1, 8, 3);
    TQ_ONE(0, 4, 2); TQ_ONE(0, 8, 2); TQ_ONE(1, 4, 2); TQ_ONE(1, 8, 2);
#undef TQ_ONE
#undef TQ_ATTR
    return ok ? TQ_OK : TQ_ERR_HIP;
}

// Whether the decode path can run this layer (LDS budget, one workgroup must span the whole hidden size).
bool tqi_skinny_supported(const TqLayout& L)
{
    if (L.r16 > 64) return false;
    if (L.cw != 4 && L.g != 64 && L.g != 128) return false;
    int ns, ups;
    plan_split(L.H, L.g, &ns, &ups);
    if (ns != 1) return false;
    const int unit_k = L.g < 64 ? 64 : L.g;
    auto smem = [&](int units) {
        const int range_k = units * unit_k;
        return (size_t)16 * (range_k * 2 + 16) + SK_RED_BYTES + (size_t)(range_k / L.g) * 64 + 16;
    };
    if (smem(ups) > 160 * 1024) return false;
    plan_split(L.F, L.g, &ns, &ups);
    if (ns > TQ_MAX_SPLIT || smem(ups) > 160 * 1024) return false;
    return true;
}

tq_status tqi_forward_skinny(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, const uint16_t* x,
                             int32_t T, uint8_t* ws, hipStream_t stream, int* nsplit_out)
{
    MGeom G;
    G.ne = L.E + L.S; G.H = L.H; G.F = L.F; G.g = L.g; G.r = L.r; G.r16 = L.r16; G.k = L.k; G.S = L.S;
    G.a_tot = W.a_tot; G.expert_stride = L.expert_stride; G.fm = L.fm;
    G.unpack_mask = L.cw == 4 ? 0x000F000Fu : L.cw == 3 ? 0x00070007u : 0x00030003u;
    G.unpack_magic = 0x43004300u;
    G.zc_ws = nullptr; G.zc_stride = 0; G.zc_d_off = 0;
    const int32_t* ctrl = reinterpret_cast<const int32_t*>(ws + W.ctrl);
    const int32_t* offsets = reinterpret_cast<const int32_t*>(ws + W.offsets);
    const int32_t* row_token = reinterpret_cast<const int32_t*>(ws + W.row_token);
    const int32_t* tile_e = reinterpret_cast<const int32_t*>(ws + W.tile_e) + 2 * (size_t)W.rt_max;      // 16-row tiling
    const int32_t* tile_row0 = reinterpret_cast<const int32_t*>(ws + W.tile_row0) + 2 * (size_t)W.rt_max;
    const int32_t* tile_rows = tile_row0 + (size_t)TQ_N_TILINGS * W.rt_max;      // row counts of the same tiling
    uint16_t* h = reinterpret_cast<uint16_t*>(ws + W.h);
    float* yd = reinterpret_cast<float*>(ws + W.yd);
    float* tpart = reinterpret_cast<float*>(ws + W.tpart);
    const int gs = L.g / 16;
    const int rt16 = W.a_tot / 16 + L.E + L.S;

    int ns, ups;
    plan_split(L.H, L.g, &ns, &ups);
    const int sl_gu = (L.H + SK_PRE_K - 1) / SK_PRE_K, sl_d = (L.F + SK_PRE_K - 1) / SK_PRE_K;
    const int nat_gu = L.r > 0 ? L.gu.na_tiles : 0, nat_d = L.r > 0 ? L.d.na_tiles : 0;
    // decode batches proper: the gate/up slices were computed per assignment in the permutation's launch
    const bool by_assign = tqi_pre_by_assign(L, W);
    const int32_t* row_src = by_assign ? reinterpret_cast<const int32_t*>(ws + W.row_src) : nullptr;
    if (L.r > 0 && !by_assign) {
        if (L.fm.fp8)
            hipLaunchKernelGGL((skinny_pre_kernel<0, true>), dim3(rt16, sl_gu, nat_gu), dim3(64), 0, stream, G, L.gu, blob, x, row_token,
                               tile_e, tile_row0, offsets, ctrl, tpart, sl_gu, nat_gu);
        else
            hipLaunchKernelGGL((skinny_pre_kernel<0, false>), dim3(rt16, sl_gu, nat_gu), dim3(64), 0, stream, G, L.gu, blob, x, row_token,
                               tile_e, tile_row0, offsets, ctrl, tpart, sl_gu, nat_gu);
        TQ_CHECK_LAUNCH();
    }
    tqi_record_stage(2, stream);
    int32_t* pair_cnt = reinterpret_cast<int32_t*>(ws + W.sk_cnt);
    if (W.sk_cnt_n < 2 * W.rt_max * TQ_MAX_SPLIT) return TQ_ERR_UNSUPPORTED;
    tq_status rc = launch_skinny_gs<0>(gs, L.cw, G, L.gu, blob, x, row_token, tile_e, tile_row0, offsets, ctrl, tpart, sl_gu, nat_gu,
                                       h, pair_cnt, rt16, 1, ups, stream, row_src, tile_rows, wave_k_of(L.H, L.g));
    if (rc != TQ_OK) return rc;
    tqi_record_stage(3, stream);
    if (L.r > 0) {
        if (L.fm.fp8)
            hipLaunchKernelGGL((skinny_pre_kernel<1, true>), dim3(rt16, sl_d, nat_d), dim3(64), 0, stream, G, L.d, blob, h, row_token,
                               tile_e, tile_row0, offsets, ctrl, tpart, sl_d, nat_d);
        else
            hipLaunchKernelGGL((skinny_pre_kernel<1, false>), dim3(rt16, sl_d, nat_d), dim3(64), 0, stream, G, L.d, blob, h, row_token,
                               tile_e, tile_row0, offsets, ctrl, tpart, sl_d, nat_d);
        TQ_CHECK_LAUNCH();
    }
    tqi_record_stage(4, stream);
    plan_split(L.F, L.g, &ns, &ups);
    rc = launch_skinny_gs<1>(gs, L.cw, G, L.d, blob, h, row_token, tile_e, tile_row0, offsets, ctrl, tpart, sl_d, nat_d, yd,
                             pair_cnt + (size_t)W.rt_max * TQ_MAX_SPLIT, rt16, ns, ups, stream, nullptr, tile_rows, wave_k_of(L.F, L.g));
    if (rc != TQ_OK) return rc;
    *nsplit_out = ns;
    return TQ_OK;
}
