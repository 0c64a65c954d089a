// Prefill (many rows per expert) grouped GEMM of the bf16 path: persistent workgroups.
//
// Same arithmetic as moe_mfma_kernel<2, 1, ...> (64-row tiles, four waves of 64x64, int4 -> bf16 unpack with
// the group scale folded on the fp32 accumulator, zero-point and low-rank terms as extra MFMA steps on the
// augmented rows), but a workgroup walks through a list of (row tile, column block) items instead of ending
// after one.  What a fresh workgroup pays per tile - the chain of dependent loads tile table -> row ids ->
// first operands, an empty prefetch queue, the operands of the correction steps - is paid once per
// workgroup here: while the last unit of an item is multiplied, the first activation unit, the first two
// weight units and the correction operands of the NEXT item are already in flight, and its row ids were
// fetched an item earlier.
//
// Items are dealt out statically.  Workgroup ids go round-robin over the 8 XCDs (each with its own L2);
// XCD x takes the x-th eighth of the row tiles, a contiguous range, and its workgroups walk (row tile, column
// block) in row-tile-major order, so the workgroups of one XCD are on a few neighbouring row tiles at any time:
// they share their activations in that L2, and neighbouring tiles mostly share an expert's weights there too.
// (With few row tiles the XCDs share out the column blocks of every tile instead: see by_cols.)
#include "tq_device.h"

#include <type_traits>

namespace {

using namespace tqdev;

__device__ inline uint32_t opaque_mov(uint32_t x)
{
    uint32_t y;
    asm volatile("v_mov_b32 %0, %1" : "=v"(y) : "v"(x));
    return y;
}

struct WSrc {                // weight-side operand bases of one (expert, column pair): wave-uniform
    const u32x4* codes;
    const uint32_t* codes32;   // the same part seen as dwords (dense 2- / 3-bit layouts)
    const uint32_t* sz;
    const u32x4* zc;
    const u32x4* bf;
};

// CW: 32-bit words of codes per lane, tile and 64-wide chunk: 4 (4-bit slots), 3 or 2 (dense 3- / 2-bit codes).
template <int STAGE, int GS, int CW = 4>
__global__ void __launch_bounds__(256, 2)
moe_prefill_kernel(MGeom G, TqSection sec, const uint8_t* __restrict__ blob, const uint16_t* __restrict__ xin,
                   const uint16_t* __restrict__ xaug, const int32_t* __restrict__ row_token,
                   const int32_t* __restrict__ tile_e, const int32_t* __restrict__ tile_row0,
                   const int32_t* __restrict__ offsets, const int32_t* __restrict__ ctrl, int ctrl_idx,
                   void* __restrict__ out, int ka)
{
    constexpr int MT = 2, BM = 64, NTHR = 256;
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int UC = UNIT_K / 64;     // 64-wide chunks (one u32x4 of codes per lane and tile) per unit
    constexpr int US = UNIT_K / 16;     // MFMA steps per unit
    constexpr int NG = US / GS;         // quantisation groups per unit
    constexpr int ROWB = UNIT_K * 2 + 16;   // LDS bytes per activation row (16 B pad: conflict-free b128 reads)
    constexpr int BUFB = BM * ROWB;
    constexpr int TPR = UNIT_K / 8;     // threads (16-byte segments) per row when loading a unit
    constexpr int RPP = NTHR / TPR;     // rows per pass
    constexpr int NP = BM / RPP;        // passes
    using WT = std::conditional_t<CW == 4, u32x4, uint32_t>;      // register type of the packed codes
    constexpr int WN = CW == 4 ? UC : UC * CW;                    // and how many of them one tile of a unit takes

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    int32_t* tok = reinterpret_cast<int32_t*>(lds + 2 * BUFB);   // [item parity][0: source row, 1: xaug row][BM]

    const int K = sec.K;
    const int nb_count = (sec.pairs + 3) / 4;
    const int xcd = blockIdx.x & 7, wgx = gridDim.x >> 3;
    const int ntiles = ctrl[ctrl_idx];
    const int last_row = ctrl[3] - 1;       // last assignment row the permutation filled in
    const int per_x = (ntiles + 7) >> 3;
    const int tiles_x = min(max(ntiles - xcd * per_x, 0), per_x);
    // With few row tiles an eighth of them per XCD is a poor deal (12 tiles: six XCDs with two each, two with
    // none).  Then XCD x takes the column blocks x, x + 8, ... of EVERY row tile instead, whenever that leaves the
    // busiest XCD at least a tenth fewer items; still row-tile-major, so its workgroups stay on neighbouring tiles.
    const int nbx_max = (nb_count + 7) >> 3;
    const bool by_cols = (long long)ntiles * nbx_max * 10 <= (long long)per_x * nb_count * 9;
    const int nbx = xcd < nb_count ? (nb_count - xcd + 7) >> 3 : 0;
    const int items_x = by_cols ? ntiles * nbx : tiles_x * nb_count;
    int q = blockIdx.x >> 3;
    if (q >= items_x) return;
    // The two workgroups of a CU: the one launched first wins every issue arbitration (oldest first) and runs
    // a third faster, which unbalances the static deal.  The second half of the grid shares CUs with the first
    // half, so the halves take turns at a raised wave priority, switching every 2^13 ticks of the 100 MHz clock.
    const bool young = q >= (wgx >> 1);

    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int wn = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int prow = tid / TPR, seg = tid % TPR;
    const uint32_t lds_wr = (uint32_t)(prow * ROWB + seg * 16);
    const uint32_t lds_rd = (uint32_t)(col * ROWB + hf * 16);

    const int nmain = K / UNIT_K;
    const int naug = ka / UNIT_K;
    const int ZT = tq_zero_terms(K, G.g);

    // ---- item bookkeeping (everything wave-uniform) ---------------------------------------------------
    auto tile_of = [&](int qq) { return by_cols ? qq / nbx : xcd * per_x + qq / nb_count; };
    auto nb_of = [&](int qq) { return by_cols ? xcd + 8 * (qq % nbx) : qq % nb_count; };
    auto make_src = [&](int e, int nb, bool& active) {
        const int pair_raw = nb * 4 + wn;
        active = pair_raw < sec.pairs;
        const int pair = active ? pair_raw : sec.pairs - 1;
        const uint8_t* rec = blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride;
        WSrc s;
        s.codes = reinterpret_cast<const u32x4*>(rec + sec.codes) + (size_t)pair * sec.chunks * 128;
        s.codes32 = reinterpret_cast<const uint32_t*>(rec + sec.codes) + (size_t)pair * sec.chunks * (2 * CW * 64);
        s.sz = reinterpret_cast<const uint32_t*>(rec + sec.sz) + (size_t)pair * sec.groups * 64;
        s.zc = reinterpret_cast<const u32x4*>(tq_zc_base(G, blob, sec, STAGE, e)) + (size_t)pair * sec.zfrag * 128;
        s.bf = reinterpret_cast<const u32x4*>(G.r > 0 ? tq_bfrag_base(blob, G.expert_stride, sec, G.fm, STAGE, e) : rec + sec.bfrag) +
               (size_t)pair * (G.r16 / 16) * 128;
        return s;
    };
    // row ids of a tile: rows past the end of the expert read the following (valid, finite) rows; their
    // results are never stored.  The clamp is the last row that exists: when the permutation dropped an invalid
    // expert index there are fewer rows than assignments, and the row tables beyond them are not written.
    auto row_ids = [&](int slot0, int& tx, int& ta) {
        ta = min(slot0 + (tid & (BM - 1)), last_row);
        tx = STAGE == 0 ? row_token[ta] : ta;
    };

    u32x4 xr[NP];
    uint32_t xvoff[NP];          // byte offset of this thread's segment in each pass, relative to xsb
    const uint8_t* xsb;          // wave-uniform base of the unit being prefetched
    auto set_rows = [&](int par, int which, uint32_t row_bytes) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            xvoff[p] = (uint32_t)tok[(par * 2 + which) * BM + p * RPP + prow] * row_bytes + (uint32_t)seg * 16u;
    };
    auto load_x = [&]() {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            uint32_t o = xvoff[p];
            asm volatile("" : "+v"(o));      // keeps the offset a 32-bit register operand next to the scalar base
            xr[p] = *reinterpret_cast<const u32x4*>(xsb + o);
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
            *reinterpret_cast<u32x4*>(lds + buf * BUFB + p * RPP * ROWB + lds_wr) = xr[p];
    };
    auto load_w = [&](WT (&dst)[2][WN], const WSrc& s, int u) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < UC; ++c) {
                if constexpr (CW == 4) {
                    dst[t][c] = s.codes[((size_t)(u * UC + c) * 2 + t) * 64 + lane];
                } else {
#pragma unroll
                    for (int d = 0; d < CW; ++d)
                        dst[t][c * CW + d] = s.codes32[(((size_t)(u * UC + c) * 2 + t) * CW + d) * 64 + lane];
                }
            }
    };
    auto load_sz = [&](uint32_t (&dst)[NG][2], const WSrc& s, int u) {
#pragma unroll
        for (int gi = 0; gi < NG; ++gi)
#pragma unroll
            for (int t = 0; t < 2; ++t) dst[gi][t] = s.sz[((size_t)(u * NG + gi) * 2 + t) * 32 + col];
    };
    // operands of the correction steps of augmented unit `st`: every step loads two fragments from a valid
    // address whether it is used or not (loads under a condition would drain the prefetch queue)
    u32x4 fq[US][2];
    auto load_fq = [&](const WSrc& s, int st) {
#pragma unroll
        for (int w = 0; w < US; ++w) {
            const int k0 = UNIT_K * st + 16 * w;
            const bool zp = k0 < ZT;
            int step = zp ? k0 / 16 : (k0 - ZT) / 16;
            const int nlr = G.r16 / 16;
            if (!zp) { if (step >= nlr) step -= nlr; if (step >= nlr) step = 0; }
            const u32x4* base = (zp || G.r == 0) ? s.zc : s.bf;
            if (zp) step = tq_zc_fragment(step);
            if (!zp && G.r == 0) step = 0;
            fq[w][0] = base[((size_t)step * 2 + 0) * 64 + lane];
            fq[w][1] = base[((size_t)step * 2 + 1) * 64 + lane];
        }
    };

    f32x16 acc[MT][2];
    auto clear_acc = [&]() {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][t][v] = 0.f;
    };
    clear_acc();

    // the or-operand of the unpack lives in a vector register (only one scalar operand fits the and-or
    // encoding); the move is opaque to the compiler so that it does not fold the value back into a literal
    uint32_t magic_v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(magic_v) : "s"(G.unpack_magic));

    WT wq[2][2][WN];
    uint32_t szq[2][NG][2];

    // ---- start-up: the only place where the chain of dependent loads is exposed -------------------------
    int cur_e, cur_slot0, cur_nb, cur_rows;
    int nxt_e, nxt_slot0;
    {
        const int rt = tile_of(q);
        cur_e = __builtin_amdgcn_readfirstlane(tile_e[rt]);
        cur_slot0 = __builtin_amdgcn_readfirstlane(tile_row0[rt]);
        cur_nb = nb_of(q);
        cur_rows = min(BM, __builtin_amdgcn_readfirstlane(offsets[cur_e + 1]) - cur_slot0);
        const int rtn = tile_of(min(q + wgx, items_x - 1));
        nxt_e = __builtin_amdgcn_readfirstlane(tile_e[rtn]);
        nxt_slot0 = __builtin_amdgcn_readfirstlane(tile_row0[rtn]);
        int tx, ta;
        row_ids(cur_slot0, tx, ta);
        if (tid < BM) { tok[tid] = tx; tok[BM + tid] = ta; }
    }
    bool cur_active;
    WSrc cur = make_src(cur_e, cur_nb, cur_active);
    lds_barrier();
    set_rows(0, 1, (uint32_t)ka * 2u);
    xsb = reinterpret_cast<const uint8_t*>(xaug);
    load_x();
    load_w(wq[0], cur, 0); load_sz(szq[0], cur, 0);
    load_w(wq[1], cur, 1); load_sz(szq[1], cur, 1);
    load_fq(cur, 0);
    store_x(0);
    lds_barrier();

    int gstep = 0;      // steps done so far; step s reads LDS buffer s & 1
    int par = 0;        // parity of the current item (selects its row ids in LDS)

    for (;;) {
        const int qn = q + wgx;
        const bool has_next = qn < items_x;
        // next item: its tile header was fetched one item ago, its row ids are requested now and written to
        // LDS after the augmented units; the header of the item after it is requested now as well
        const int nxt_nb = has_next ? nb_of(qn) : cur_nb;
        bool nxt_active;
        const WSrc nxt = make_src(nxt_e, nxt_nb, nxt_active);
        int ntx, nta;
        row_ids(nxt_slot0, ntx, nta);
        const int noffs_v = offsets[nxt_e + 1];
        const int rtnn = tile_of(min(qn + wgx, items_x - 1));
        const int nn_e_v = tile_e[rtnn], nn_slot0_v = tile_row0[rtnn];

        // ---- augmented units: zero-point correction and the low-rank term ------------------------------
        for (int st = 0; st < naug; ++st) {
            if (st + 1 < naug) {
                xsb = reinterpret_cast<const uint8_t*>(xaug) + (size_t)(st + 1) * UNIT_K * 2;
            } else {
                set_rows(par, 0, (uint32_t)K * 2u);
                xsb = reinterpret_cast<const uint8_t*>(xin);
            }
            load_x();
            const int buf = gstep & 1;
            if (cur_active) {
#pragma unroll
                for (int w = 0; w < US; ++w) {
                    const int k0 = UNIT_K * st + 16 * w;
                    // 1: zero-point step (both tiles), 2: low-rank on tile 0, 3: low-rank on tile 1, 4: on both
                    int kind = 0;
                    if (k0 < ZT) kind = 1;
                    else if (G.r > 0 && k0 < ZT + G.r16) kind = STAGE == 1 ? 4 : 2;
                    else if (STAGE == 0 && G.r > 0 && k0 < ZT + 2 * G.r16) kind = 3;
                    if (kind == 0) continue;
                    bf16x8 bw[2];
                    if (kind == 1) {
                        Frag f0, f1;
                        f0.q = fq[w][0]; f1.q = fq[w][1];
                        bw[0] = f0.v; bw[1] = f1.v;
                    } else {
                        bw[0] = half8_to_bf8(fq[w][0]);
                        bw[1] = half8_to_bf8(fq[w][1]);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        Frag xa;
                        xa.q = *reinterpret_cast<const u32x4*>(lds + buf * BUFB + mt * 32 * ROWB + w * 32 + lds_rd);
                        if (kind != 3) acc[mt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa.v, bw[0], acc[mt][0], 0, 0, 0);
                        if (kind != 2) acc[mt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa.v, bw[1], acc[mt][1], 0, 0, 0);
                    }
                }
            }
            if (st + 1 < naug) load_fq(cur, st + 1);
            store_x((gstep + 1) & 1);
            lds_barrier();
            ++gstep;
        }

        // row ids of the next item (visible to everyone after the next barrier; first used at the last unit)
        if (tid < BM) {
            tok[((par ^ 1) * 2 + 0) * BM + tid] = ntx;
            tok[((par ^ 1) * 2 + 1) * BM + tid] = nta;
        }
        const int nxt_rows = min(BM, __builtin_amdgcn_readfirstlane(noffs_v) - nxt_slot0);
        const int nn_e = __builtin_amdgcn_readfirstlane(nn_e_v), nn_slot0 = __builtin_amdgcn_readfirstlane(nn_slot0_v);

        // ---- main units ----------------------------------------------------------------------------------
        const bool upper = cur_rows > 32;
        auto main_unit = [&](int mu, auto slot_tag) {
            constexpr int SLOT = decltype(slot_tag)::value;
#ifndef TQ_PRIO_GS
#define TQ_PRIO_GS 8
#endif
            if constexpr (GS >= TQ_PRIO_GS) {     // measured: pays with groups of 128 (-4 %), costs with groups of 64 (+9 %)
                const bool hi = (((__builtin_amdgcn_s_memrealtime() >> 13) & 1) != 0) != young;
                if (hi) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0);
            }
            // activation prefetch one unit ahead (at the last unit a harmless reload of itself: the first unit of
            // the next item is fetched after the loop, where registers are free to recompute the row offsets)
            xsb = reinterpret_cast<const uint8_t*>(xin) + (size_t)min(mu + 1, nmain - 1) * UNIT_K * 2;
            load_x();
            WT wc[2][WN];
            uint32_t szc[NG][2];
            // The copies are opaque moves: the slot is dead afterwards, so the prefetch below can land in the very
            // same registers.  Left to itself the compiler keeps the old values in place instead and renames the
            // slot, and then has to move freshly requested registers at the loop end, which waits for those loads.
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int c = 0; c < WN; ++c) {
                    if constexpr (CW == 4) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) wc[t][c][i] = opaque_mov(wq[SLOT][t][c][i]);
                    } else {
                        wc[t][c] = opaque_mov(wq[SLOT][t][c]);
                    }
                }
#pragma unroll
            for (int gi = 0; gi < NG; ++gi)
#pragma unroll
                for (int t = 0; t < 2; ++t) szc[gi][t] = opaque_mov(szq[SLOT][gi][t]);
            {
                // two units ahead; past the end of this item that is unit SLOT of the next one, so that its
                // units 0 and 1 land in slots 0 and 1 whatever the parity of the unit count
                const bool here = mu + 2 < nmain;
                const WSrc& s = here ? cur : nxt;
                const int u = here ? mu + 2 : SLOT;
                load_w(wq[SLOT], s, u); load_sz(szq[SLOT], s, u);
            }
            const int buf = gstep & 1;
            if (cur_active) {
                bf16x8 xa[2][MT];
                f32x16 part[MT][2];
                auto read_a = [&](int kk, int m0, int m1) {
#pragma unroll
                    for (int mt = m0; mt < m1; ++mt) {
                        Frag f;
                        f.q = *reinterpret_cast<const u32x4*>(lds + buf * BUFB + mt * 32 * ROWB + kk * 32 + lds_rd);
                        xa[kk & 1][mt] = f.v;
                    }
                };
                read_a(0, 0, 1);
                if (upper) read_a(0, 1, MT);
#pragma unroll
                for (int kidx = 0; kidx < US; ++kidx) {
                    const int gi = kidx / GS, ks = kidx % GS;
                    // fragments of the next step are requested before this step's MFMAs are issued
                    if (kidx + 1 < US) read_a(kidx + 1, 0, 1);
                    bf16x8 bw[2];
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if constexpr (CW == 4) bw[t] = unpack_word(word_of(wc[t][kidx / 4], kidx % 4), G.unpack_mask, magic_v);
                        else bw[t] = unpack_dense<CW>(&wc[t][(kidx / 4) * CW], kidx % 4, G.unpack_mask, magic_v);
                    }
                    auto mfmas = [&](int m0, int m1) {
#pragma unroll
                        for (int mt = m0; mt < m1; ++mt) {
#pragma unroll
                            for (int t = 0; t < 2; ++t) {
                                if (ks == 0) {
                                    f32x16 zero;
#pragma unroll
                                    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                                    part[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[kidx & 1][mt], bw[t], zero, 0, 0, 0);
                                } else {
                                    part[mt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[kidx & 1][mt], bw[t], part[mt][t], 0, 0, 0);
                                }
                            }
                        }
                    };
                    auto fold = [&](int m0, int m1) {        // the group is complete: fold it with its scale
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const float s = tq_half_bits_to_float((uint16_t)(szc[gi][t] & 0xFFFF));
#pragma unroll
                            for (int mt = m0; mt < m1; ++mt)
#pragma unroll
                                for (int v = 0; v < 16; ++v) acc[mt][t][v] = fmaf(s, part[mt][t][v], acc[mt][t][v]);
                        }
                    };
                    mfmas(0, 1);
                    if (ks == GS - 1) fold(0, 1);
                    // a tile of at most 32 rows runs the MFMAs of its first row block only (one wave-uniform branch
                    // around each block of the second one's)
                    if (upper) {
                        if (kidx + 1 < US) read_a(kidx + 1, 1, MT);
                        mfmas(1, MT);
                        if (ks == GS - 1) fold(1, MT);
                    }
                }
            }
            if (mu + 1 < nmain) {
                store_x((gstep + 1) & 1);
                lds_barrier();
                ++gstep;
            }
        };
        // The first pair stands outside the loop (there are at least two units): the wait counts the compiler
        // derives at the loop head are the minimum over all ways in, and the way in from the augmented units has
        // fewer loads in flight than the steady state, which would shorten the prefetch distance of every unit.
        main_unit(0, std::integral_constant<int, 0>{});
        main_unit(1, std::integral_constant<int, 1>{});
        int mu = 2;
        for (; mu + 1 < nmain; mu += 2) {
            main_unit(mu, std::integral_constant<int, 0>{});
            main_unit(mu + 1, std::integral_constant<int, 1>{});
        }
        if (mu < nmain) main_unit(mu, std::integral_constant<int, 0>{});

        // the first augmented unit of the next item and its correction operands travel during the epilogue
        // (when there is no next item this reloads the current one: harmless)
        set_rows(has_next ? par ^ 1 : par, 1, (uint32_t)ka * 2u);
        xsb = reinterpret_cast<const uint8_t*>(xaug);
        load_x();
        load_fq(nxt, 0);

        // ---- epilogue (full tiles take a path without per-row tests) ---------------------------------------
        // Addresses are a per-item scalar row pointer plus ONE per-lane offset: spelled any other way the
        // compiler hoists thirty-odd per-row offsets out of the item loop, spills them, and every reload in the
        // epilogue then waits for all the stores issued before it.
        if (cur_active) {
            const int pair = cur_nb * 4 + wn;
            const bool full = cur_rows == BM;
            const size_t row_bytes = (size_t)(STAGE == 0 ? G.F : G.H) * 2;
            uint8_t* obase = reinterpret_cast<uint8_t*>(out) + (size_t)cur_slot0 * row_bytes +
                             (size_t)(STAGE == 0 ? 32 : 64) * pair * 2;
            uint32_t lane_off = (uint32_t)(4 * hf) * (uint32_t)row_bytes + (uint32_t)col * 2u;
            asm volatile("" : "+v"(lane_off));
            auto emit = [&](auto full_tag) {
                constexpr bool FULL = decltype(full_tag)::value;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int mrow = 32 * mt + 8 * (v / 4) + (v % 4);      // + 4 hf: in lane_off
                        uint8_t* rowp = obase + (size_t)mrow * row_bytes;        // wave-uniform
                        if (FULL || mrow + 4 * hf < cur_rows) {
                            if (STAGE == 0) {
                                *reinterpret_cast<uint16_t*>(rowp + lane_off) =
                                    (uint16_t)f2bf_bits(silu_mul(acc[mt][0][v], acc[mt][1][v]));
                            } else {
                                *reinterpret_cast<uint16_t*>(rowp + lane_off) = (uint16_t)f2bf_bits(acc[mt][0][v]);
                                *reinterpret_cast<uint16_t*>(rowp + lane_off + 64) = (uint16_t)f2bf_bits(acc[mt][1][v]);
                            }
                        }
                    }
            };
            if (full) emit(std::true_type{}); else emit(std::false_type{});
        }
        if (!has_next) break;
        clear_acc();
        store_x((gstep + 1) & 1);
        lds_barrier();
        ++gstep;
        q = qn;
        cur = nxt; cur_active = nxt_active; cur_nb = nxt_nb;
        cur_e = nxt_e; cur_slot0 = nxt_slot0; cur_rows = nxt_rows;
        nxt_e = nn_e;
        nxt_slot0 = nn_slot0;
        par ^= 1;
    }
}

template <int STAGE, int GS, int CW = 4>
tq_status launch_prefill(const MGeom& G, const TqSection& sec, const uint8_t* blob, const uint16_t* xin,
                         const uint16_t* xaug, const int32_t* row_token, const int32_t* tile_e,
                         const int32_t* tile_row0, const int32_t* offsets, const int32_t* ctrl, int ctrl_idx,
                         void* out, int ka, hipStream_t st)
{
    constexpr int BM = 64;
    constexpr int UNIT_K = (GS * 16 < 64) ? 64 : GS * 16;
    constexpr int ROWB = UNIT_K * 2 + 16;
    const size_t smem = (size_t)2 * BM * ROWB + (size_t)4 * BM * 4;
    const TqDeviceState* ds = nullptr;
    if (tqi_device_state(&ds) != TQ_OK) return TQ_ERR_HIP;
    const int n_cu = ds->n_cu;
    const int grid = (2 * n_cu) / 8 * 8;     // two workgroups per CU, a whole number per XCD
    hipLaunchKernelGGL((moe_prefill_kernel<STAGE, GS, CW>), dim3(grid), dim3(256), smem, st, G, sec, blob, xin, xaug, row_token,
                       tile_e, tile_row0, offsets, ctrl, ctrl_idx, out, ka);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

}  // namespace

bool tqi_prefill_supported(const TqLayout& L, const TqWorkspace& W, int32_t T)
{
    const int gs = L.g / 16;
    if (gs != 2 && gs != 4 && gs != 8) return false;
    const int unit = L.g < 64 ? 64 : L.g;
    if (L.H / unit < 2 || L.F / unit < 2) return false;            // the weight prefetch runs two units ahead
    // 32-bit byte offsets of activation rows
    const uint64_t lim = 1ull << 32;
    if ((uint64_t)T * L.H * 2 >= lim || (uint64_t)W.a_tot * L.F * 2 >= lim) return false;
    if ((uint64_t)W.a_tot * W.ka_gu * 2 >= lim || (uint64_t)W.a_tot * W.ka_d * 2 >= lim) return false;
    return true;
}

tq_status tqi_forward_prefill_stage(int stage, const TqLayout& L, const TqWorkspace& W, const MGeom& G,
                                    const uint8_t* blob, const uint16_t* xin, const uint16_t* xaug,
                                    const int32_t* row_token, const int32_t* tile_e, const int32_t* tile_row0,
                                    const int32_t* offsets, const int32_t* ctrl, int ctrl_idx, void* out,
                                    hipStream_t st)
{
    const int gs = L.g / 16;
    const TqSection& sec = stage == 0 ? L.gu : L.d;
    const int ka = stage == 0 ? W.ka_gu : W.ka_d;
#define TQ_CASE(GSV)                                                                                                  \
    case GSV:                                                                                                         \
        return stage == 0 ? launch_prefill<0, GSV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, \
                                                   ctrl_idx, out, ka, st)                                             \
                          : launch_prefill<1, GSV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, \
                                                   ctrl_idx, out, ka, st)
    if (L.cw != 4) {      // dense codes: groups of 64 and 128
#define TQ_DENSE(GSV, CWV)                                                                                                  \
    if (gs == GSV && L.cw == CWV)                                                                                           \
        return stage == 0 ? launch_prefill<0, GSV, CWV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, \
                                                        ctrl_idx, out, ka, st)                                              \
                          : launch_prefill<1, GSV, CWV>(G, sec, blob, xin, xaug, row_token, tile_e, tile_row0, offsets, ctrl, \
                                                        ctrl_idx, out, ka, st)
        TQ_DENSE(4, 3); TQ_DENSE(8, 3); TQ_DENSE(4, 2); TQ_DENSE(8, 2);
#undef TQ_DENSE
        return TQ_ERR_UNSUPPORTED;
    }
    switch (gs) {
        TQ_CASE(2);
        TQ_CASE(4);
        TQ_CASE(8);
    }
#undef TQ_CASE
    return TQ_ERR_UNSUPPORTED;
}
