// Internal definitions shared by the HIP translation units of libtileq: blob layout arithmetic,
// workspace carve-up, and a few device helpers.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "tileq.h"

#define TQ_BLOB_MAGIC 0x31425154u /* "TQB1" */
#define TQ_BLOB_VERSION 4u
#define TQ_HEADER_BYTES 256
#define TQ_STATIC_SCRATCH_BYTES TQ_STATIC_SCRATCH_MAX   /* size of the static scratch array (tileq.h) */

// error-flag bits written by kernels into the first int32 of the workspace / into err_flag
#define TQ_FLAG_BIT_RANGE 1
#define TQ_FLAG_BIT_BLOB 2

struct TqSection {
    // geometry of one section (GU or D) of an expert record
    int32_t pairs;   // column-tile pairs
    int32_t K;       // contraction length
    int32_t chunks;  // K / 64
    int32_t groups;  // K / g
    int32_t na_tiles;  // 32-wide tiles of the A-factor columns
    int32_t zfrag;     // fragments of the zero-point coefficients per pair and tile: 2 * ceil(groups / 16) (hi, lo)
    int32_t zsteps;    // of which the blob stores: zfrag, or 0 (dense codes: the tiled kernels derive them per call)
    // byte offsets from the start of the expert record
    size_t codes, sz, zc, bfrag, afrag, sig, end;     // sig: fp32 Sigma of fp8 factors (empty otherwise)
};

// Where the factor fragments of an expert live: inside its record, or (shared 2D-tiled factors) in per-tile blocks
// behind the records, found through the placement table.  Index 0: section GU, 1: section D.
struct TqFactorMap {
    int32_t shared, M, N, fp8;             // fp8: one byte per factor element and a Sigma table
    size_t phi_off;                       // byte offsets from the start of the blob
    size_t apool[2], astride[2];          // block m of the left factors at apool + m * astride (afrag layout)
    size_t bpool[2], bstride[2];          // block n of the right factors at bpool + n * bstride (bfrag layout)
    size_t sig_off[2];                    // shared fp8 factors: fp32 Sigma of section GU / D (one table for all tiles)
    const uint8_t* fbase;                 // null: the offsets above count from the blob; else from this device address
                                          // (fp16 fragments expanded from fp8 factors into the workspace)
};

struct TqLayout {
    int32_t E, S, k, H, F, g, bits, r, r16;
    TqFactorMap fm;
    int32_t cw;      // 32-bit words of codes per (lane, 64-wide chunk, tile): 4 (4-bit slots), 3 or 2 (dense 3- / 2-bit)
    int32_t flags;   // the descriptor's
    TqSection gu, d;
    size_t expert_stride;
    size_t total_bytes;
};

struct TqBlobHeader {
    uint32_t magic, version;
    int32_t n_experts, n_shared, hidden, ffn, group, bits, rank, r16;
    int32_t code_words, factor_fp8;     // TqLayout::cw, TqFactorMap::fp8
    int32_t tiles_m, tiles_n;           // 0, 0: per-expert factors
    uint64_t expert_stride, total_bytes;
    uint64_t off[10];  // gu.codes, gu.sz, gu.zc, gu.bfrag, gu.afrag, then the same five of d
};
static_assert(sizeof(TqBlobHeader) <= TQ_HEADER_BYTES, "header too large");

__host__ __device__ inline size_t tq_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Returns false if the descriptor is outside what the layout supports.
__host__ inline bool tq_make_layout(const tq_layer_desc* d, TqLayout* L)
{
    if (!d) return false;
    if (d->n_experts < 1 || d->n_shared < 0 || d->top_k < 1 || d->top_k > d->n_experts) return false;
    if (d->n_experts > 1024 || d->n_shared > 64) return false;
    if (d->hidden < 64 || d->ffn < 64 || d->hidden % 64 || d->ffn % 64) return false;
    if (d->hidden > (1 << 16) || d->ffn > (1 << 17)) return false;
    if (!(d->group == 32 || d->group == 64 || d->group == 128 || d->group == 256)) return false;
    if (d->hidden % d->group || d->ffn % d->group) return false;
    const bool dense = (d->flags & TQ_FLAG_DENSE_CODES) != 0;
    if (dense ? (d->bits != 2 && d->bits != 3) : (d->bits != 3 && d->bits != 4)) return false;
    if (dense && d->group < 64) return false;       // dense codes: groups of 64 and more
    if (d->rank < 0 || d->rank > 256) return false;
    if (d->act_dtype != TQ_ACT_BF16 && d->act_dtype != TQ_ACT_FP32) return false;
    const bool shared = d->tiles_m > 0 || d->tiles_n > 0;
    const bool fp8 = (d->flags & TQ_FLAG_FP8_FACTORS) != 0;
    if (fp8 && d->rank < 1) return false;
    const size_t fb = fp8 ? 1 : 2;       // bytes per factor element
    if (d->tiles_m < 0 || d->tiles_n < 0 || (shared && (d->tiles_m < 1 || d->tiles_n < 1))) return false;
    if (shared && (d->rank < 1 || d->tiles_m > 4096 || d->tiles_n > 4096)) return false;
    L->E = d->n_experts; L->S = d->n_shared; L->k = d->top_k; L->H = d->hidden; L->F = d->ffn;
    L->g = d->group; L->bits = d->bits; L->r = d->rank; L->r16 = (d->rank + 15) / 16 * 16;
    L->cw = dense ? d->bits : 4;
    L->flags = d->flags;
    size_t off = 0;
    auto fill = [&](TqSection& s, int pairs, int K, int na) {
        s.pairs = pairs; s.K = K; s.chunks = K / 64; s.groups = K / L->g; s.na_tiles = (na + 31) / 32;
        s.codes = off; off += (size_t)pairs * s.chunks * 512 * L->cw;
        s.sz = off;    off += (size_t)pairs * s.groups * 256;
        s.zfrag = 2 * ((s.groups + 15) / 16);
        s.zsteps = dense ? 0 : s.zfrag;     // only the MFMA prefill kernels read this part
        s.zc = off;    off += (size_t)pairs * s.zsteps * 2048;
        // shared factors: the records hold no factor parts (their geometry, na_tiles, still describes the blocks)
        s.bfrag = off; off += shared ? 0 : (size_t)pairs * (L->r16 / 16) * 1024 * fb;
        s.afrag = off; off += shared ? 0 : (size_t)s.na_tiles * (K / 16) * 512 * fb;
        s.sig = off;   off += (fp8 && !shared) ? tq_align256((size_t)na * 4) : 0;
        s.end = off;
    };
    fill(L->gu, L->F / 32, L->H, 2 * L->r16);
    fill(L->d, L->H / 64, L->F, L->r16);
    L->expert_stride = tq_align256(off);
    L->total_bytes = TQ_HEADER_BYTES + (size_t)(L->E + L->S) * L->expert_stride;
    TqFactorMap& fm = L->fm;
    fm = TqFactorMap{};
    fm.fp8 = fp8 ? 1 : 0;
    if (shared) {
        fm.shared = 1; fm.M = d->tiles_m; fm.N = d->tiles_n;
        size_t o = L->total_bytes;
        fm.phi_off = o; o += tq_align256((size_t)(L->E + L->S) * 8);
        const TqSection* secs[2] = {&L->gu, &L->d};
        for (int i = 0; i < 2; ++i) {
            fm.astride[i] = (size_t)secs[i]->na_tiles * (secs[i]->K / 16) * 512 * fb;
            fm.bstride[i] = (size_t)secs[i]->pairs * (L->r16 / 16) * 1024 * fb;
            fm.apool[i] = o; o += (size_t)fm.M * fm.astride[i];
            fm.bpool[i] = o; o += (size_t)fm.N * fm.bstride[i];
            fm.sig_off[i] = o; o += fp8 ? tq_align256((size_t)(i == 0 ? 2 : 1) * L->r16 * 4) : 0;
        }
        L->total_bytes = tq_align256(o);
    }
    return true;
}

// Correction step s of the K-order (per block of 16 groups: hi(c) against hi(xsum), hi(c) against lo(xsum), lo(c)
// against hi(xsum)) -> stored fragment of the zc part (per block: hi, lo)
__host__ __device__ inline int tq_zc_fragment(int step) { const int b = step / 3; return 2 * b + (step - 3 * b == 2 ? 1 : 0); }

// position of code i (0..7, consecutive kk) inside a packed 32-bit word, in nibbles
__host__ __device__ inline int tq_nibble_pos(int i) { return (i >> 1) + 4 * (i & 1); }

// ------------------------------------------------------------------------------------------------
// Workspace of tq_moe_forward.  All offsets are multiples of 256 bytes.
struct TqWorkspace {
    size_t ctrl;        // int32[64]: [0] error flag, [1] row tiles (32-row), [2] (128-row), [3] rows, [4] (16-row), [5] (64-row)
    size_t offsets;     // int32 [E+S+1]
    size_t slot_of;     // int32 [T*(k+S)]
    size_t row_token;   // int32 [A_tot]
    size_t row_w;       // float [A_tot]
    size_t row_src;     // int32 [A_tot]  assignment behind each slot: t * k + j (routed), T * k + s * T + t (shared expert s)
    size_t tile_e;      // int32 [4][RT]  expert of each row tile, for the 32-, 128-, 16- and 64-row tilings
    size_t tile_row0;   // int32 [4][RT]  first slot of each row tile, followed by int32 [4][RT] its number of rows
    size_t hist;        // int32 [nblk][E] permutation scratch
    size_t xaug_gu;     // bf16 [A_tot][ka_gu]   (bf16 path)
    size_t xaug_d;      // bf16 [A_tot][ka_d]
    size_t h;           // bf16 [A_tot][F]  or fp32 [A_tot][F]
    size_t yd;          // fp32 [nsplit][A_tot][H]
    size_t tpart;       // fp32 partial low-rank intermediates (only for small batches): slices of the decode path's
    size_t tpart_bytes; // pre-pass, or of the tiled kernels' pre-pass when it cuts the contraction
    size_t zc_ws;       // dense codes on the tiled kernels: the zero-point coefficient fragments the blob does not store,
    size_t zc_stride;   // derived per call: [E+S] records of zc_stride bytes, section GU at 0, section D at zc_d_off
    size_t zc_d_off;
    size_t fac_ws;      // fp8 factors on the tiled kernels: fp16 fragments expanded per call; fac_fm describes them
    size_t fac_bytes;   // (offsets from the start of fac_ws; 0 bytes when not laid out)
    TqFactorMap fac_fm;
    size_t sk_cnt;      // decode path: next-pair counters [2 stages][rt_max][TQ_MAX_SPLIT], cleared by the permutation
    int32_t sk_cnt_n;   // their number (0 when the batch is too large for the decode path)
    size_t total;
    int32_t a_tot, rt_max, nblk, ka_gu, ka_d, nsplit_max;
};

#define TQ_N_TILINGS 4      // row tilings with a tile table: 32, 128, 16, 64 rows (in this order)
#define TQ_PERM_CHUNK 256   // assignments handled by one permutation block
#define TQ_MAX_SPLIT 8      // K-splits of the down projection on the small-tile path
#define TQ_SKINNY_MAX_ROWS 1024   // assignment rows up to which the decode (16-row tile) path is considered
#define TQ_AUG_SLICE_MAX_TILES 160   // 32-row tiles up to which the tiled kernels' pre-pass is cut over K
#define TQ_SPLITK_MAX_ROWS 4096   // assignment rows up to which the 32-row path may split the down projection's K

__host__ __device__ inline int tq_pad64(int v) { return (v + 63) / 64 * 64; }
// augmented-K length: three bf16 split terms per quantisation group (zero-point correction; groups in blocks
// of 16, each block laid out hi | lo | hi) followed by the rank-r intermediate, the whole padded to one
// staging unit (max(g, 64))
__host__ __device__ inline int tq_zero_terms(int K, int g) { return 48 * ((K / g + 15) / 16); }
__host__ __device__ inline int tq_aug_len(int K, int g, int n_lr)
{
    const int unit = g < 64 ? 64 : g;
    return (tq_zero_terms(K, g) + n_lr + unit - 1) / unit * unit;
}

struct TqLayout;
bool tqi_bf16_rows_take_skinny(const TqLayout& L, int64_t a_tot, int flags);      // the path rule (tq_mfma.hip)
bool tqi_skinny_supported(const TqLayout& L);

__host__ inline void tq_make_workspace(const TqLayout& L, int act_dtype, int32_t T, TqWorkspace* W)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += tq_align256(bytes); return o; };
    int64_t a_tot = (int64_t)T * (L.k + L.S);
    W->a_tot = (int32_t)a_tot;
    W->rt_max = (int32_t)(a_tot / 16 + L.E + L.S + 1);
    W->nblk = (int32_t)(((int64_t)T * L.k + TQ_PERM_CHUNK - 1) / TQ_PERM_CHUNK);
    if (W->nblk < 1) W->nblk = 1;
    W->ka_gu = tq_aug_len(L.H, L.g, 2 * L.r16);
    W->ka_d = tq_aug_len(L.F, L.g, L.r16);
    W->nsplit_max = TQ_MAX_SPLIT;
    W->ctrl = take(64 * sizeof(int32_t));
    W->offsets = take((size_t)(L.E + L.S + 1) * 4);
    W->slot_of = take((size_t)a_tot * 4);
    W->row_token = take((size_t)a_tot * 4);
    W->row_w = take((size_t)a_tot * 4);
    W->row_src = take((size_t)a_tot * 4);
    W->tile_e = take((size_t)TQ_N_TILINGS * W->rt_max * 4);
    W->tile_row0 = take((size_t)2 * TQ_N_TILINGS * W->rt_max * 4);      // first slots, then row counts
    W->hist = take((size_t)W->nblk * L.E * 4);
    if (act_dtype == TQ_ACT_BF16) {
        W->xaug_gu = take((size_t)a_tot * W->ka_gu * 2);
        W->xaug_d = take((size_t)a_tot * W->ka_d * 2);
        W->h = take((size_t)a_tot * L.F * 2);
        // the small-tile path may split the down projection's K; the large-tile path never does
        size_t planes = (a_tot <= TQ_SPLITK_MAX_ROWS) ? TQ_MAX_SPLIT : 1;
        W->yd = take(planes * (size_t)a_tot * L.H * 4);
        W->tpart = off; W->tpart_bytes = 0;
        if (L.r > 0) {
            if (a_tot <= TQ_SKINNY_MAX_ROWS) {
                const size_t slices = (size_t)((L.H > L.F ? L.H : L.F) + 255) / 256;
                const size_t nat = (size_t)(2 * L.r16 + 31) / 32;
                W->tpart_bytes = (size_t)(a_tot / 16 + L.E + L.S) * slices * nat * 512 * 4;
            }
            // pre-pass of the tiled kernels cut over K (at most TQ_AUG_SLICE_MAX_TILES row tiles): slices of at least
            // 512 indices, up to 512 + tiles (tile, slice) parts, each the 32x32 fp32 column tiles of t
            const size_t rt32 = (size_t)(a_tot / 32 + L.E + L.S);
            const size_t cps_min = (size_t)(512 + 4 * L.g - 1) / (4 * L.g);
            const size_t ch_gu = (size_t)(L.gu.groups + 3) / 4, ch_d = (size_t)(L.d.groups + 3) / 4;
            const size_t ch = ch_gu > ch_d ? ch_gu : ch_d;
            const size_t nsl_max = (ch + cps_min - 1) / cps_min;
            if (rt32 <= TQ_AUG_SLICE_MAX_TILES && nsl_max > 1) {
                const size_t nat = (size_t)(2 * L.r16 + 31) / 32, natv = nat <= 1 ? 1 : nat == 2 ? 2 : 4;
                size_t parts = rt32 * nsl_max;
                if (parts > 512 + rt32) parts = 512 + rt32;
                if (parts * natv * 4096 > W->tpart_bytes) W->tpart_bytes = parts * natv * 4096;
            }
            if (W->tpart_bytes) W->tpart = take(W->tpart_bytes);
        }
        // dense codes / fp8 factors on the tiled kernels (every batch the decode kernels do not take)
        const bool tiled = !tqi_bf16_rows_take_skinny(L, a_tot, L.flags);
        W->zc_ws = off; W->zc_stride = 0; W->zc_d_off = 0;
        if (L.cw != 4 && tiled) {
            W->zc_d_off = (size_t)L.gu.pairs * L.gu.zfrag * 2048;
            W->zc_stride = W->zc_d_off + (size_t)L.d.pairs * L.d.zfrag * 2048;
            W->zc_ws = take((size_t)(L.E + L.S) * W->zc_stride);
        }
        W->fac_ws = off; W->fac_bytes = 0; W->fac_fm = TqFactorMap{};
        if (L.fm.fp8 && tiled) {
            TqFactorMap& f = W->fac_fm;
            f.shared = 1; f.fp8 = 0;
            f.M = L.fm.shared ? L.fm.M : L.E + L.S;       // per-expert factors: one block per expert, identity placement
            f.N = L.fm.shared ? L.fm.N : L.E + L.S;
            size_t o = 0;
            f.phi_off = o; o += tq_align256((size_t)(L.E + L.S) * 8);
            const TqSection* secs[2] = {&L.gu, &L.d};
            for (int i = 0; i < 2; ++i) {
                f.astride[i] = (size_t)secs[i]->na_tiles * (secs[i]->K / 16) * 1024;
                f.bstride[i] = (size_t)secs[i]->pairs * (L.r16 / 16) * 2048;
                f.apool[i] = o; o += (size_t)f.M * f.astride[i];
                f.bpool[i] = o; o += (size_t)f.N * f.bstride[i];
            }
            W->fac_bytes = o;
            W->fac_ws = take(o);
        }
        W->sk_cnt = off;
        W->sk_cnt_n = 0;
        if (a_tot <= TQ_SKINNY_MAX_ROWS) {
            W->sk_cnt_n = 2 * W->rt_max * TQ_MAX_SPLIT;
            W->sk_cnt = take((size_t)W->sk_cnt_n * 4);
        }
    } else {
        W->xaug_gu = W->xaug_d = off;
        W->zc_ws = off; W->zc_stride = 0; W->zc_d_off = 0;
        W->fac_ws = off; W->fac_bytes = 0; W->fac_fm = TqFactorMap{};
        W->tpart = off; W->tpart_bytes = 0;
        W->sk_cnt = off;
        W->sk_cnt_n = 0;
        W->h = take((size_t)a_tot * L.F * 4);
        W->yd = take((size_t)a_tot * L.H * 4);
    }
    W->total = off;
}

// ------------------------------------------------------------------------------------------------
#ifdef __HIPCC__
__device__ inline float tq_half_bits_to_float(uint16_t h)
{
    return __half2float(__ushort_as_half(h));
}

// one fp8 E4M3 code (low byte of b) -> fp32, exact (the hardware conversion of gfx950, OCP E4M3)
__device__ inline float tq_fp8_to_float(uint32_t b)
{
    return __builtin_amdgcn_cvt_pk_f32_fp8(b, false)[0];
}

// base of the left (afrag layout) / right (bfrag layout) factor fragments of expert e in section sec_id (0 GU, 1 D)
__device__ inline const uint8_t* tq_afrag_base(const uint8_t* blob, size_t expert_stride, const TqSection& sec,
                                               const TqFactorMap& fm, int sec_id, int e)
{
    if (!fm.shared) return blob + TQ_HEADER_BYTES + (size_t)e * expert_stride + sec.afrag;
    const uint8_t* b = fm.fbase ? fm.fbase : blob;
    const int m = reinterpret_cast<const int32_t*>(b + fm.phi_off)[2 * e];
    return b + fm.apool[sec_id] + (size_t)m * fm.astride[sec_id];
}
__device__ inline const uint8_t* tq_bfrag_base(const uint8_t* blob, size_t expert_stride, const TqSection& sec,
                                               const TqFactorMap& fm, int sec_id, int e)
{
    if (!fm.shared) return blob + TQ_HEADER_BYTES + (size_t)e * expert_stride + sec.bfrag;
    const uint8_t* b = fm.fbase ? fm.fbase : blob;
    const int n = reinterpret_cast<const int32_t*>(b + fm.phi_off)[2 * e + 1];
    return b + fm.bpool[sec_id] + (size_t)n * fm.bstride[sec_id];
}

// fp32 Sigma of the fp8 factors of expert e in section sec_id: NA values (gate then up in GU)
__device__ inline const float* tq_sig_base(const uint8_t* blob, size_t expert_stride, const TqSection& sec,
                                           const TqFactorMap& fm, int sec_id, int e)
{
    if (fm.shared) return reinterpret_cast<const float*>(blob + fm.sig_off[sec_id]);
    return reinterpret_cast<const float*>(blob + TQ_HEADER_BYTES + (size_t)e * expert_stride + sec.sig);
}

// expert owning slot `s`: largest e with offsets[e] <= s (offsets is non-decreasing, n+1 entries)
__device__ inline int tq_find_expert(const int32_t* __restrict__ offsets, int n, int s)
{
    int lo = 0, hi = n;  // invariant: offsets[lo] <= s < offsets[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (offsets[mid] <= s) lo = mid; else hi = mid;
    }
    return lo;
}
#endif

// Decode batches: the low-rank intermediate of gate/up, t = x A_e, computed per ASSIGNMENT (it needs the routing
// table only, not the permutation) so that it can share the permutation's launch:
//   tpart[v][slice][ta][c] = sum over the 256-wide slice of x[token(v)][kk] * A_e(v)[kk][32 ta + c]   (fp32)
// v = t * k + j for routed assignments, T * k + s * T + t for shared expert s.
#define TQ_PRE_ASSIGN_MAX_ROWS 256    // assignment rows up to which the decode path takes this form (A_e is read per row;
                                      // measured: saves 7 % of the step at 96 rows, 5 % at 160, 1-2 % at 256)
struct TqPreByAssign {
    const uint16_t* x;       // [T][H] bf16
    const uint8_t* blob;
    size_t expert_stride;
    TqSection sec;           // section GU
    TqFactorMap fm;
    float* tpart;
    int32_t H, n_slices, na_tiles, a_tot;
};

// Routing inputs of tq_route_moe_forward: when the single-wave permutation runs (one chunk of assignments) and the
// routing is a few scores per token (tqi_route_fusable), the permutation's launch computes the routing itself and writes
// topk_idx / topk_w as outputs.
struct TqRouteIn {
    const float* logits;     // [T][E]
    const float* bias;       // [E] or null
    int32_t* idx_out;        // [T][k]
    float* w_out;            // [T][k]
};
inline bool tqi_route_fusable(int64_t T, int E, int S, int k, int nblk)
{
    // (one lane scans a token's E scores k times: beyond a few experts the routing kernel, a wave per token, is faster)
    return nblk == 1 && T >= 1 && T <= 64 && E <= 16 && T * k <= TQ_PERM_CHUNK && (int64_t)S * T <= 4096;
}

// internal entry points implemented across the translation units (host side)
tq_status tqi_launch_permute(const int32_t* topk_idx, const float* topk_w, int32_t T, int32_t E, int32_t S,
                             int32_t k, int32_t* offsets, int32_t* slot_of, int32_t slot_stride,
                             int32_t* src_of, int32_t* row_token, float* row_w, int32_t* tile_e,
                             int32_t* tile_row0, int32_t rt_max, int32_t* ctrl, int32_t* err_flag,
                             int32_t* hist, int32_t nblk, const void* blob, const TqLayout* L,
                             int32_t* zero_buf, int32_t zero_n, hipStream_t stream,
                             const TqPreByAssign* pre = nullptr, int tilings = (1 << TQ_N_TILINGS) - 1,
                             const TqRouteIn* route = nullptr);
// fills W.fac_ws with fp16 fragments (Sigma folded into the left factors) and the placement table (fp8 factors on the
// tiled kernels)
tq_status tqi_expand_fp8_factors(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, uint8_t* ws, hipStream_t stream);
// fills W.zc_ws from the blob's scale / zero part (dense codes on the tiled kernels)
tq_status tqi_derive_zc(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, uint8_t* ws, hipStream_t stream);
// whether the bf16 forward of this batch runs on the decode kernels, and whether its gate/up pre-pass is by assignment
bool tqi_bf16_takes_skinny(const TqLayout& L, const TqWorkspace& W, int flags);
inline bool tqi_pre_by_assign(const TqLayout& L, const TqWorkspace& W) { return L.r > 0 && W.a_tot <= TQ_PRE_ASSIGN_MAX_ROWS; }
tq_status tqi_forward_f32(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, const float* x,
                          int32_t T, float* y, uint8_t* ws, hipStream_t stream, const float* topk_w);
tq_status tqi_forward_bf16(const TqLayout& L, const TqWorkspace& W, int flags, const uint8_t* blob,
                           const uint16_t* x, int32_t T, uint16_t* y, uint8_t* ws, hipStream_t stream,
                           const float* topk_w);

bool tqi_skinny_supported(const TqLayout& L);
tq_status tqi_forward_skinny(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, const uint16_t* x,
                             int32_t T, uint8_t* ws, hipStream_t stream, int* nsplit_out);

// Per-device state, set up once per device under a lock by the first entry point that needs it (or by tq_init):
// the CU count, the raised dynamic-LDS limits of the kernels that need more than the default, and the address of
// the library's static scratch array on that device.
struct TqDeviceState {
    int n_cu;
    void* scratch;          // device address of the static scratch array (each device holds its own copy)
};
tq_status tqi_device_state(const TqDeviceState** out);
// each translation unit raises the dynamic-LDS limit of its own kernel instantiations (current device)
tq_status tqi_setup_mfma();
tq_status tqi_setup_skinny();

// profiling aid: stage-boundary events registered through tq_set_profile_events (nullptr when off)
void tqi_record_stage(int stage, hipStream_t stream);

#define TQ_CHECK_LAUNCH()                                         \
    do {                                                          \
        if (hipGetLastError() != hipSuccess) return TQ_ERR_HIP;   \
    } while (0)
