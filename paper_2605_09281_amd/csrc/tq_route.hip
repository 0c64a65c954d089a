// tq_route (top-k selection and routing weights) and the token -> expert permutation with
// prefix-sum offsets (histogram, scan, stable scatter) that tq_permute exports and tq_moe_forward
// runs as its first step.
#include "tq_common.h"

namespace {

constexpr int kMaxPerLane = 16;  // E <= 64 * 16

// One wavefront per token.  Lane l holds the scores of experts l, l+64, l+128, ... (PL of them: the per-lane scans
// are unrolled to the number of experts a lane can hold, not to the maximum).
// Each of the k rounds takes the wave-wide maximum under the order (score desc, index asc).
// One selection round over the scores a wave holds (lane l: experts l, l + 64, ...; `taken` marks the ones already
// chosen or past E): the wave-wide maximum under the order (score desc, index asc), marked as taken in its lane.
template <int PL>
__device__ inline void wave_select_round(const float (&v)[PL], uint32_t& taken, int lane, float& bv, int& be)
{
    // best candidate of this lane: ascending index scan with a strict compare keeps the lowest index
    bv = 0.f;
    be = 0x7FFFFFFF;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        if (!((taken >> i) & 1u)) {
            if (be == 0x7FFFFFFF || v[i] > bv) { bv = v[i]; be = lane + 64 * i; }
        }
    }
    // wave-wide arg-max under (score desc, index asc); lanes with nothing left carry index INT_MAX
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(bv, off);
        int oe = __shfl_xor(be, off);
        bool take = (oe != 0x7FFFFFFF) && (be == 0x7FFFFFFF || ov > bv || (ov == bv && oe < be));
        if (take) { bv = ov; be = oe; }
    }
    if ((be & 63) == lane) taken |= 1u << (be >> 6);
}

template <int PL>
__device__ inline void wave_load_scores(const float* __restrict__ logits_row, const float* __restrict__ bias, int E, int lane,
                                        float (&v)[PL], uint32_t& taken)
{
    taken = 0;
#pragma unroll
    for (int i = 0; i < PL; ++i) {
        int e = lane + 64 * i;
        float s = -INFINITY;
        if (e < E) {
            s = logits_row[e];
            if (bias) s = s + bias[e];
        } else {
            taken |= 1u << i;
        }
        v[i] = s;
    }
}

template <int PL>
__global__ void __launch_bounds__(256) route_kernel(const float* __restrict__ logits,
                                                    const float* __restrict__ bias, int T, int E, int k,
                                                    int32_t* __restrict__ topk_idx, float* __restrict__ topk_w)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (t >= T) return;
    float v[PL];
    uint32_t taken;
    wave_load_scores<PL>(logits + (size_t)t * E, bias, E, lane, v, taken);
    float first = 0.f, denom = 0.f, my_p = 0.f;
    for (int j = 0; j < k; ++j) {
        float bv;
        int be;
        wave_select_round<PL>(v, taken, lane, bv, be);
        if (j == 0) first = bv;
        float p = expf(bv - first);       // the same value in every lane
        denom += p;
        if (lane == j) my_p = p;          // lane j keeps the unnormalised weight of slot j (k <= 64)
        if (lane == 0) topk_idx[(size_t)t * k + j] = be;
    }
    if (lane < k) topk_w[(size_t)t * k + lane] = my_p / denom;
}

// The routing of a decode batch inside the permutation's launch (at most 64 tokens and 16 experts): one LANE per
// token scans its scores serially, the same order (score desc, index asc) and the same arithmetic as route_kernel,
// so the results are identical bit for bit.  Scores are staged in LDS (row stride E + 1: conflict-free); the results
// land in LDS (ridx, rw: [T * k]) for the permutation that follows and in memory for the caller.
__device__ inline void route_small(const TqRouteIn& R, int T, int E, int k, float* sc, int32_t* ridx, float* rw, int lane)
{
    // at most 64 x 16 scores: all of a lane's loads are in flight at once
    {
        constexpr int NL = 16;
        float lv[NL], bv[NL];
        const int n = T * E;
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = min(u * 64 + lane, n - 1);
            lv[u] = R.logits[i];
            bv[u] = R.bias ? R.bias[i % E] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = u * 64 + lane;
            if (i < n) {
                float s = lv[u];
                if (R.bias) s = s + bv[u];
                sc[(i / E) * (E + 1) + i % E] = s;
            }
        }
    }
    __syncthreads();
    if (lane < T) {
        uint64_t taken = 0;
        float first = 0.f, denom = 0.f;
        const float* row = sc + lane * (E + 1);
        for (int j = 0; j < k; ++j) {
            float bv = 0.f;
            int be = -1;
            for (int e = 0; e < E; ++e) {
                const float s = row[e];
                if (!((taken >> e) & 1ull) && (be < 0 || s > bv)) { bv = s; be = e; }
            }
            taken |= 1ull << be;
            if (j == 0) first = bv;
            const float p = expf(bv - first);
            denom += p;
            ridx[lane * k + j] = be;
            rw[lane * k + j] = p;
        }
        for (int j = 0; j < k; ++j) rw[lane * k + j] = rw[lane * k + j] / denom;
    }
    __syncthreads();
    for (int a = lane; a < T * k; a += 64) {
        R.idx_out[a] = ridx[a];
        R.w_out[a] = rw[a];
    }
}

// The expert of assignment (t, j) recomputed by one wave from the token's scores (E <= 64): the workgroups that share
// the permutation's launch cannot wait for its routing results.
__device__ inline int route_expert_of(const TqRouteIn& R, int t, int j, int E, int lane)
{
    float v[1];
    uint32_t taken;
    wave_load_scores<1>(R.logits + (size_t)t * E, R.bias, E, lane, v, taken);
    int be = 0;
    for (int q = 0; q <= j; ++q) {
        float bv;
        wave_select_round<1>(v, taken, lane, bv, be);
    }
    return be;
}

// ---------------------------------------------------------------------------------------------
// Permutation.  Assignments are cut into chunks of TQ_PERM_CHUNK; one wavefront per chunk.
//   hist_kernel:    per-chunk histogram over experts (also validates the blob header)
//   scan_kernel:    per expert, exclusive scan over chunks; offsets; row-tile tables
//   scatter_kernel: stable placement, chunk by chunk, 64 assignments per round in order
// permute_small_kernel does all of it in one wavefront when there is a single chunk (decode batches).
//
// Row-tile tables: for each tiling (32, 128, 16, 64 rows) the list of (expert, first slot) of every tile,
// expert-major; their lengths go to ctrl[1], ctrl[2], ctrl[4], ctrl[5]; ctrl[3] = number of rows in total.
__device__ inline int tile_rows_of(int which) { return which == 0 ? 32 : which == 1 ? 128 : which == 2 ? 16 : 64; }
__device__ inline int tile_ctrl_of(int which) { return which == 0 ? 1 : which == 1 ? 2 : which == 2 ? 4 : 5; }

__device__ inline int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    return v;
}

// One wavefront: out[0..n] = exclusive prefix sum of f(in[i]); returns the total.  in/out live in LDS.
template <typename F>
__device__ inline int wave_excl_scan(const int32_t* in, int32_t* out, int n, int lane, F f)
{
    int carry = 0;
    for (int i0 = 0; i0 < n; i0 += 64) {
        int i = i0 + lane;
        int v = i < n ? f(in[i]) : 0;
        int inc = wave_incl_scan(v, lane);
        if (i < n) out[i] = carry + inc - v;
        carry += __shfl(inc, 63);
    }
    if (lane == 0) out[n] = carry;
    return carry;
}

__device__ inline bool blob_header_ok(const TqBlobHeader* hdr, const TqBlobHeader& expect)
{
    return hdr->magic == expect.magic && hdr->version == expect.version && hdr->n_experts == expect.n_experts &&
           hdr->n_shared == expect.n_shared && hdr->hidden == expect.hidden && hdr->ffn == expect.ffn &&
           hdr->group == expect.group && hdr->bits == expect.bits && hdr->rank == expect.rank &&
           hdr->code_words == expect.code_words && hdr->factor_fp8 == expect.factor_fp8 && hdr->tiles_m == expect.tiles_m && hdr->tiles_n == expect.tiles_n &&
           hdr->expert_stride == expect.expert_stride;
}

__global__ void __launch_bounds__(64) hist_kernel(const int32_t* __restrict__ idx, int64_t n_assign, int E,
                                                  int32_t* __restrict__ hist, int32_t* __restrict__ err_flag,
                                                  const TqBlobHeader* __restrict__ hdr, TqBlobHeader expect,
                                                  int check_blob)
{
    extern __shared__ int32_t cnt[];
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) cnt[e] = 0;
    __syncthreads();
    const int64_t a0 = (int64_t)blockIdx.x * TQ_PERM_CHUNK;
    bool bad = false;
    for (int i = lane; i < TQ_PERM_CHUNK; i += 64) {
        int64_t a = a0 + i;
        if (a < n_assign) {
            int e = idx[a];
            if (e >= 0 && e < E) atomicAdd(&cnt[e], 1); else bad = true;
        }
    }
    __syncthreads();
    for (int e = lane; e < E; e += 64) hist[(size_t)blockIdx.x * E + e] = cnt[e];
    if (bad && err_flag) atomicOr(err_flag, TQ_FLAG_BIT_RANGE);
    if (check_blob && blockIdx.x == 0 && lane == 0) {
        if (!blob_header_ok(hdr, expect) && err_flag) atomicOr(err_flag, TQ_FLAG_BIT_BLOB);
    }
}

// writes the row-tile tables from offs[0..ne] (LDS); `sm_base` is LDS scratch of TQ_N_TILINGS*(ne+1) ints;
// tile_row0 holds 2 * TQ_N_TILINGS * rt_max ints: the first slots, then the row counts
__device__ inline void build_tile_tables(const int32_t* offs, int32_t* sm_base, int ne, int32_t* tile_e,
                                         int32_t* tile_row0, int rt_max, int32_t* ctrl, int tid, int nthreads,
                                         int tilings = (1 << TQ_N_TILINGS) - 1)
{
    // per tiling: tiles of expert e = ceil(count/bm); scan by wavefront `which` (or by wave 0 in turn)
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    for (int which = wave; which < TQ_N_TILINGS; which += nwaves) {
        if (!((tilings >> which) & 1)) continue;       // tilings no kernel of this forward reads (their counts stay 0)
        const int bm = tile_rows_of(which);
        int32_t* base = sm_base + which * (ne + 1);
        int carry = 0;
        for (int i0 = 0; i0 < ne; i0 += 64) {
            int i = i0 + lane;
            int v = i < ne ? (offs[i + 1] - offs[i] + bm - 1) / bm : 0;
            int inc = wave_incl_scan(v, lane);
            if (i < ne) base[i] = carry + inc - v;
            carry += __shfl(inc, 63);
        }
        if (lane == 0) { base[ne] = carry; ctrl[tile_ctrl_of(which)] = carry < rt_max ? carry : rt_max; }
    }
    __syncthreads();
    // one entry per thread: the expert of tile n is found by bisection over the per-expert first tiles
    for (int which = 0; which < TQ_N_TILINGS; ++which) {
        if (!((tilings >> which) & 1)) continue;
        const int bm = tile_rows_of(which);
        const int32_t* base = sm_base + which * (ne + 1);
        const int total = base[ne] < rt_max ? base[ne] : rt_max;
        int32_t* te = tile_e + (size_t)which * rt_max;
        int32_t* tr = tile_row0 + (size_t)which * rt_max;
        for (int n = tid; n < total; n += nthreads) {
            int lo = 0, hi = ne - 1;          // largest e with base[e] <= n (experts without rows share a base)
            while (lo < hi) {
                int mid = (lo + hi + 1) >> 1;
                if (base[mid] <= n) lo = mid; else hi = mid - 1;
            }
            te[n] = lo;
            tr[n] = offs[lo] + (n - base[lo]) * bm;
            // the tile's row count, behind the first-slot tables: saves the decode kernels a dependent load of offsets
            tr[n + (size_t)TQ_N_TILINGS * rt_max] = min(bm, offs[lo + 1] - tr[n]);
        }
    }
}

// One wavefront per routed expert: hist[b][e] becomes the number of assignments of expert e in chunks
// before b, and counts[e] their total.
__global__ void __launch_bounds__(64) chunk_scan_kernel(int32_t* __restrict__ hist, int nblk, int E,
                                                        int32_t* __restrict__ counts)
{
    const int e = blockIdx.x, lane = threadIdx.x;
    int run = 0;
    for (int b0 = 0; b0 < nblk; b0 += 64) {
        int b = b0 + lane;
        int v = b < nblk ? hist[(size_t)b * E + e] : 0;
        int inc = wave_incl_scan(v, lane);
        if (b < nblk) hist[(size_t)b * E + e] = run + inc - v;
        run += __shfl(inc, 63);
    }
    if (lane == 0) counts[e] = run;
}

// Single block of 1024 threads: expert offsets from the counts (left in offsets[1..E] by chunk_scan_kernel
// when hist is null, else computed here from the few chunks of hist) and the row-tile tables.
__global__ void __launch_bounds__(1024) scan_kernel(int32_t* __restrict__ hist, int nblk, int E, int S, int T,
                                                    int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ tile_e, int32_t* __restrict__ tile_row0,
                                                    int rt_max, int32_t* __restrict__ ctrl, int check_blob)
{
    extern __shared__ int32_t sm[];   // counts[ne] | offs[ne+1] | tile scratch TQ_N_TILINGS*(ne+1)
    const int ne = E + S;
    int32_t* counts = sm;
    int32_t* offs = sm + ne;
    int32_t* tsm = offs + ne + 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (hist) {
        // few chunks: the per-expert scan over chunks is one wave round per expert, done here
        for (int e = wave; e < E; e += 16) {
            int run = 0;
            for (int b0 = 0; b0 < nblk; b0 += 64) {
                int b = b0 + lane;
                int v = b < nblk ? hist[(size_t)b * E + e] : 0;
                int inc = wave_incl_scan(v, lane);
                if (b < nblk) hist[(size_t)b * E + e] = run + inc - v;
                run += __shfl(inc, 63);
            }
            if (lane == 0) counts[e] = run;
        }
        for (int s = tid; s < S; s += 1024) counts[E + s] = T;
    } else {
        for (int e = tid; e < ne; e += 1024) counts[e] = e < E ? offsets[e + 1] : T;
    }
    __syncthreads();
    if (wave == 0) {
        int total = wave_excl_scan(counts, offs, ne, lane, [](int v) { return v; });
        if (lane == 0 && ctrl) ctrl[3] = total;
    }
    __syncthreads();
    for (int e = tid; e <= ne; e += 1024) offsets[e] = offs[e];
    if (tile_e) build_tile_tables(offs, tsm, ne, tile_e, tile_row0, rt_max, ctrl, tid, 1024);
    // blob / descriptor mismatch (found by hist_kernel, which ran before): no row tiles and no rows, so that every
    // later kernel of the forward ends at once instead of indexing the blob with the wrong geometry
    __syncthreads();
    if (check_blob && ctrl && tid == 0 && (ctrl[0] & TQ_FLAG_BIT_BLOB)) { ctrl[1] = 0; ctrl[2] = 0; ctrl[3] = 0; ctrl[4] = 0; ctrl[5] = 0; }
}

// stable placement of one chunk of assignments by one wavefront; cursor[e] (LDS) = next free slot of expert e.
// `sync` orders this wavefront's reads of cursor before its writes and the writes before the next round's reads: a
// workgroup barrier where the workgroup is this one wave, a wave-level fence where several waves each place a chunk
// of their own (their trip counts differ, so they cannot meet at a workgroup barrier).
template <typename Sync>
__device__ inline void scatter_chunk(const int32_t* __restrict__ idx, const float* __restrict__ w, int64_t a0,
                                     int64_t n_assign, int E, int k, int32_t* cursor, int lane,
                                     int32_t* __restrict__ slot_of, int slot_stride, int32_t* __restrict__ src_of,
                                     int32_t* __restrict__ row_token, float* __restrict__ row_w, Sync sync)
{
    for (int i0 = 0; i0 < TQ_PERM_CHUNK; i0 += 64) {
        if (a0 + i0 >= n_assign) break;
        int64_t a = a0 + i0 + lane;
        int e = -1;
        if (a < n_assign) {
            e = idx[a];
            if (e < 0 || e >= E) e = -1;
        }
        // rank of this lane among the lanes of the round that hold the same expert and come before it
        // lanes holding the same expert: intersect, bit by bit of e, the ballots that agree with this lane
        uint64_t same = __ballot(e >= 0);
        for (int bit = 0; (1 << bit) < E; ++bit) {
            const uint64_t bal = __ballot((e >> bit) & 1);
            same &= ((e >> bit) & 1) ? bal : ~bal;
        }
        const int before = __popcll(same & ((1ull << lane) - 1ull));
        const bool last = (same >> lane) <= 1ull;      // no higher lane with this expert
        const int slot = e >= 0 ? cursor[e] + before : -1;
        sync();
        if (e >= 0 && last) cursor[e] = slot + 1;   // the last lane of each expert moves its cursor
        sync();
        if (a < n_assign) {
            int t = (int)(a / k), j = (int)(a % k);
            if (slot_of) slot_of[(size_t)t * slot_stride + j] = slot;
            if (slot >= 0) {
                if (src_of) src_of[slot] = (int32_t)a;
                if (row_token) row_token[slot] = t;
                if (row_w) row_w[slot] = w ? w[a] : 1.0f;
            }
        }
    }
}

__global__ void __launch_bounds__(64) scatter_kernel(const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                     int64_t n_assign, int E, int S, int T, int k,
                                                     const int32_t* __restrict__ hist,
                                                     const int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ slot_of, int slot_stride,
                                                     int32_t* __restrict__ src_of, int32_t* __restrict__ row_token,
                                                     float* __restrict__ row_w)
{
    extern __shared__ int32_t cursor[];   // next free slot of each expert for this chunk
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += 64) cursor[e] = offsets[e] + hist[(size_t)blockIdx.x * E + e];
    __syncthreads();
    scatter_chunk(idx, w, (int64_t)blockIdx.x * TQ_PERM_CHUNK, n_assign, E, k, cursor, lane, slot_of, slot_stride,
                  src_of, row_token, row_w, [] { __syncthreads(); });
    // shared experts: every token, weight 1, identity order
    if (S > 0) {
        const int64_t total = (int64_t)S * T;
        for (int64_t i = (int64_t)blockIdx.x * 64 + lane; i < total; i += (int64_t)gridDim.x * 64) {
            int s = (int)(i / T), t = (int)(i % T);
            int slot = offsets[E + s] + t;
            if (slot_of) slot_of[(size_t)t * slot_stride + k + s] = slot;
            if (src_of) src_of[slot] = (int32_t)(n_assign + i);
            if (row_token) row_token[slot] = t;
            if (row_w) row_w[slot] = 1.0f;
        }
    }
}

// Batches of 2 to TQ_PERM_MID_CHUNKS chunks (a few thousand assignments): the whole permutation in ONE workgroup of 16
// waves instead of four launches (clear, histogram, scan, scatter) that each cost a few microseconds of latency for
// microseconds of work.  Wave w takes chunks w, w + 16, ...; the per-chunk histograms live in LDS and turn, after the
// scans, into the per-chunk cursors.  Same slots as the several-launch path: chunk-major, stable inside a chunk.
constexpr int TQ_PERM_MID_CHUNKS = 16;      // measured: 16 chunks -2 % on the step, 32 chunks +1 % against the several launches
__global__ void __launch_bounds__(1024) permute_mid_kernel(const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                           int n_assign, int nblk, int E, int S, int T, int k,
                                                           int32_t* __restrict__ offsets, int32_t* __restrict__ slot_of,
                                                           int slot_stride, int32_t* __restrict__ src_of,
                                                           int32_t* __restrict__ row_token, float* __restrict__ row_w,
                                                           int32_t* __restrict__ tile_e, int32_t* __restrict__ tile_row0,
                                                           int rt_max, int32_t* __restrict__ ctrl,
                                                           int32_t* __restrict__ err_flag,
                                                           const TqBlobHeader* __restrict__ hdr, TqBlobHeader expect,
                                                           int check_blob, int32_t* __restrict__ zero_buf, int zero_n,
                                                           int tilings)
{
    extern __shared__ int32_t sm[];   // counts[ne] | offs[ne+1] | tile scratch TQ_N_TILINGS*(ne+1) | flags[1] | hist[nblk][E]
    const int ne = E + S;
    int32_t* counts = sm;
    int32_t* offs = counts + ne;
    int32_t* tsm = offs + ne + 1;
    int32_t* flagw = tsm + TQ_N_TILINGS * (ne + 1);
    int32_t* hist = flagw + 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    TqBlobHeader hv = expect;
    if (check_blob && tid == 0) hv = *hdr;
    if (ctrl && tid < 64) ctrl[tid] = 0;
    for (int i = tid; i < zero_n; i += 1024) zero_buf[i] = 0;
    if (tid == 0) {
        if (err_flag && err_flag != ctrl) *err_flag = 0;
        *flagw = 0;
    }
    for (int i = tid; i < nblk * E; i += 1024) hist[i] = 0;
    __syncthreads();
    // per-chunk histograms
    bool bad = false;
    for (int b = wave; b < nblk; b += 16) {
        for (int i = lane; i < TQ_PERM_CHUNK; i += 64) {
            const int a = b * TQ_PERM_CHUNK + i;
            if (a < n_assign) {
                const int e = idx[a];
                if (e >= 0 && e < E) atomicAdd(&hist[b * E + e], 1); else bad = true;
            }
        }
    }
    if (bad) atomicOr(flagw, TQ_FLAG_BIT_RANGE);
    if (check_blob && tid == 0 && !blob_header_ok(&hv, expect)) atomicOr(flagw, TQ_FLAG_BIT_BLOB);
    __syncthreads();
    // per expert: exclusive scan over the chunks (at most 16: one round of a wave), total into counts
    for (int e = wave; e < E; e += 16) {
        const int v = lane < nblk ? hist[lane * E + e] : 0;
        const int inc = wave_incl_scan(v, lane);
        if (lane < nblk) hist[lane * E + e] = inc - v;
        if (lane == 63) counts[e] = inc;
    }
    for (int sidx = tid; sidx < S; sidx += 1024) counts[E + sidx] = T;
    __syncthreads();
    if (wave == 0) {
        const int total = wave_excl_scan(counts, offs, ne, lane, [](int v) { return v; });
        if (lane == 0 && ctrl) ctrl[3] = total;
    }
    __syncthreads();
    for (int e = tid; e <= ne; e += 1024) offsets[e] = offs[e];
    if (tile_e) build_tile_tables(offs, tsm, ne, tile_e, tile_row0, rt_max, ctrl, tid, 1024, tilings);
    for (int i = tid; i < nblk * E; i += 1024) hist[i] += offs[i % E];      // the chunks' cursors
    __syncthreads();
    for (int b = wave; b < nblk; b += 16)
        scatter_chunk(idx, w, (int64_t)b * TQ_PERM_CHUNK, n_assign, E, k, hist + b * E, lane, slot_of, slot_stride, src_of,
                      row_token, row_w, [] {
                          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                          __builtin_amdgcn_wave_barrier();
                          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                      });
    for (int i = tid; i < S * T; i += 1024) {      // shared experts: every token, weight 1, identity order
        const int sidx = i / T, t = i % T;
        const int slot = offs[E + sidx] + t;
        if (slot_of) slot_of[(size_t)t * slot_stride + k + sidx] = slot;
        if (src_of) src_of[slot] = n_assign + i;
        if (row_token) row_token[slot] = t;
        if (row_w) row_w[slot] = 1.0f;
    }
    const int flags = *flagw;
    if (flags && tid == 0 && err_flag) atomicOr(err_flag, flags);
    // a blob that does not belong to the descriptor: no row tiles and no rows, so that every later kernel of the
    // forward ends at once instead of indexing the blob with the wrong geometry
    if ((flags & TQ_FLAG_BIT_BLOB) && ctrl && tid == 0) { ctrl[1] = 0; ctrl[2] = 0; ctrl[3] = 0; ctrl[4] = 0; ctrl[5] = 0; }
}

__device__ inline void permute_small_body(const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                           int n_assign, int E, int S, int T, int k,
                                                           int32_t* __restrict__ offsets, int32_t* __restrict__ slot_of,
                                                           int slot_stride, int32_t* __restrict__ src_of,
                                                           int32_t* __restrict__ row_token, float* __restrict__ row_w,
                                                           int32_t* __restrict__ tile_e, int32_t* __restrict__ tile_row0,
                                                           int rt_max, int32_t* __restrict__ ctrl,
                                                           int32_t* __restrict__ err_flag,
                                                           const TqBlobHeader* __restrict__ hdr, TqBlobHeader expect,
                                                           int check_blob, int32_t* __restrict__ zero_buf, int zero_n,
                                                           int tilings)
{
    extern __shared__ int32_t sm[];   // counts[ne] | offs[ne+1] | cursor[E] | tile scratch 3*(ne+1)
    const int ne = E + S, lane = threadIdx.x;
    int32_t* counts = sm;
    int32_t* offs = counts + ne;
    int32_t* cursor = offs + ne + 1;
    int32_t* tsm = cursor + E;
    // everything this wave reads from memory is requested first (one round trip instead of three): the
    // assignments and weights of up to four rounds of 64, and the blob header
    constexpr int NR = TQ_PERM_CHUNK / 64;
    int ev[NR];
    float wv[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        ev[j] = -2;                                  // past the end: neither counted nor flagged
        wv[j] = 1.0f;
    }
    if (n_assign > 0) {                              // an empty batch has no first element to clamp to
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int a = j * 64 + lane;
            const int ac = min(a, n_assign - 1);
            const int ej = idx[ac];
            const float wj = w ? w[ac] : 1.0f;
            if (a < n_assign) { ev[j] = ej; wv[j] = wj; }
        }
    }
    TqBlobHeader hv = expect;
    if (check_blob) hv = *hdr;
    if (ctrl) ctrl[lane] = 0;
    for (int i = lane; i < zero_n; i += 64) zero_buf[i] = 0;
    for (int e = lane; e < ne; e += 64) counts[e] = e < E ? 0 : T;
    __syncthreads();
    bool bad = false;
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        if (ev[j] >= 0 && ev[j] < E) atomicAdd(&counts[ev[j]], 1);
        else if (ev[j] != -2) { bad = true; ev[j] = -1; }
    }
    __syncthreads();
    int flags = __ballot(bad) ? TQ_FLAG_BIT_RANGE : 0;
    if (check_blob && !blob_header_ok(&hv, expect)) flags |= TQ_FLAG_BIT_BLOB;
    int total = wave_excl_scan(counts, offs, ne, lane, [](int v) { return v; });
    __syncthreads();
    for (int e = lane; e <= ne; e += 64) offsets[e] = offs[e];
    for (int e = lane; e < E; e += 64) cursor[e] = offs[e];
    __syncthreads();
    if (ctrl && lane == 0) ctrl[3] = total;
    if (tile_e) build_tile_tables(offs, tsm, ne, tile_e, tile_row0, rt_max, ctrl, lane, 64, tilings);
    __syncthreads();
    // stable placement, 64 assignments per round in order (same ranking as scatter_chunk, from registers)
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        if (j * 64 >= n_assign) break;
        const int a = j * 64 + lane;
        const int e = ev[j] >= 0 ? ev[j] : -1;
        uint64_t same = __ballot(e >= 0);
        for (int bit = 0; (1 << bit) < E; ++bit) {
            const uint64_t bal = __ballot((e >> bit) & 1);
            same &= ((e >> bit) & 1) ? bal : ~bal;
        }
        const int before = __popcll(same & ((1ull << lane) - 1ull));
        const bool last = (same >> lane) <= 1ull;
        const int slot = e >= 0 ? cursor[e] + before : -1;
        __syncthreads();
        if (e >= 0 && last) cursor[e] = slot + 1;
        __syncthreads();
        if (a < n_assign) {
            const int t = a / k, jj = a % k;
            if (slot_of) slot_of[(size_t)t * slot_stride + jj] = slot;
            if (slot >= 0) {
                if (src_of) src_of[slot] = (int32_t)a;
                if (row_token) row_token[slot] = t;
                if (row_w) row_w[slot] = wv[j];
            }
        }
    }
    for (int i = lane; i < S * T; i += 64) {
        int s = i / T, t = i % T;
        int slot = offs[E + s] + t;
        if (slot_of) slot_of[(size_t)t * slot_stride + k + s] = slot;
        if (src_of) src_of[slot] = n_assign + i;
        if (row_token) row_token[slot] = t;
        if (row_w) row_w[slot] = 1.0f;
    }
    if (flags && lane == 0 && err_flag) atomicOr(err_flag, flags);
    // a blob that does not belong to the descriptor must not be indexed with the descriptor's geometry: with no
    // row tiles and no rows every later kernel of the forward ends at once
    if ((flags & TQ_FLAG_BIT_BLOB) && ctrl && lane == 0) { ctrl[1] = 0; ctrl[2] = 0; ctrl[3] = 0; ctrl[4] = 0; ctrl[5] = 0; }
}

// One wavefront per (assignment v, 256-wide slice, 32-column tile of t): see TqPreByAssign.  Plain fp32 FMAs on the
// exact values of x (bf16) and A (fp16, or fp8 with FP8), the two halves of a 16-wide step in the two halves of the wave.
template <bool FP8>
__device__ inline void pre_by_assign_block(const TqPreByAssign& P, const int32_t* __restrict__ idx, int T, int E, int k,
                                           int b, int lane, const TqRouteIn* route = nullptr)
{
    const int ta = b % P.na_tiles;
    const int slice = (b / P.na_tiles) % P.n_slices;
    const int v = b / (P.na_tiles * P.n_slices);
    if (v >= P.a_tot) return;
    int e, t;
    if (v < T * k) {
        t = v / k;
        e = route ? route_expert_of(*route, t, v % k, E, lane) : idx[v];
        if (e < 0 || e >= E) return;      // dropped assignments have no row
    }
    else { const int q = v - T * k; e = E + q / T; t = q % T; }
    const int col = lane & 31, hf = lane >> 5;
    const int ksteps = P.H / 16;
    const uint16_t* xrow = P.x + (size_t)t * P.H;
    const uint4* af = reinterpret_cast<const uint4*>(tq_afrag_base(P.blob, P.expert_stride, P.sec, P.fm, 0, e));
    constexpr int NS = 16;                       // steps per slice
    const int s0 = slice * NS;
    uint4 xa[NS], aq[NS];
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        const int sidx = min(s0 + u, ksteps - 1);
        xa[u] = *reinterpret_cast<const uint4*>(xrow + 16 * sidx + 8 * hf);
        const size_t f = (size_t)ta * ksteps + sidx;       // fragment; fp8 fragments: 8 bytes per lane, two lanes per word
        aq[u] = af[FP8 ? f * 32 + (lane >> 1) : f * 64 + lane];
    }
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < NS; ++u) {
        if (s0 + u < ksteps) {
            const uint32_t xw[4] = {xa[u].x, xa[u].y, xa[u].z, xa[u].w};
            const uint32_t aw[4] = {aq[u].x, aq[u].y, aq[u].z, aq[u].w};
            if (FP8) {
                const uint32_t d[2] = {(lane & 1) ? aw[2] : aw[0], (lane & 1) ? aw[3] : aw[1]};
#pragma unroll
                for (int j = 0; j < 4; ++j) {      // elements 2j, 2j + 1: bytes 2 (j % 2), 2 (j % 2) + 1 of word j / 2
                    const auto a2 = (j & 1) ? __builtin_amdgcn_cvt_pk_f32_fp8(d[j >> 1], true)
                                            : __builtin_amdgcn_cvt_pk_f32_fp8(d[j >> 1], false);
                    acc = fmaf(__uint_as_float(xw[j] << 16), a2[0], acc);
                    acc = fmaf(__uint_as_float(xw[j] & 0xFFFF0000u), a2[1], acc);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc = fmaf(__uint_as_float(xw[j] << 16), tq_half_bits_to_float((uint16_t)(aw[j] & 0xFFFF)), acc);
                    acc = fmaf(__uint_as_float(xw[j] & 0xFFFF0000u), tq_half_bits_to_float((uint16_t)(aw[j] >> 16)), acc);
                }
            }
        }
    }
    acc += __shfl_xor(acc, 32);
    if (hf == 0) P.tpart[(((size_t)v * P.n_slices + slice) * P.na_tiles + ta) * 32 + col] = acc;
}

template <bool FP8>
__global__ void __launch_bounds__(64) pre_by_assign_kernel(TqPreByAssign P, const int32_t* __restrict__ idx, int T, int E, int k,
                                                           const TqBlobHeader* __restrict__ hdr, TqBlobHeader expect,
                                                           int check_blob)
{
    if (check_blob && !blob_header_ok(hdr, expect)) return;      // a blob of another layer is not indexed
    pre_by_assign_block<FP8>(P, idx, T, E, k, blockIdx.x, threadIdx.x);
}

// The whole permutation for a few chunks of assignments in ONE wavefront (one launch instead of five); with
// PRE != 0 the other workgroups of the launch compute the gate/up low-rank intermediate by assignment (1: fp16
// factors, 2: fp8 factors).
// With ROUTE the launch also does the routing (route_small; idx and w are then unused).
template <int PRE, bool ROUTE>
__global__ void __launch_bounds__(64) permute_small_kernel(const int32_t* __restrict__ idx, const float* __restrict__ w,
                                                           int n_assign, int E, int S, int T, int k,
                                                           int32_t* __restrict__ offsets, int32_t* __restrict__ slot_of,
                                                           int slot_stride, int32_t* __restrict__ src_of,
                                                           int32_t* __restrict__ row_token, float* __restrict__ row_w,
                                                           int32_t* __restrict__ tile_e, int32_t* __restrict__ tile_row0,
                                                           int rt_max, int32_t* __restrict__ ctrl,
                                                           int32_t* __restrict__ err_flag,
                                                           const TqBlobHeader* __restrict__ hdr, TqBlobHeader expect,
                                                           int check_blob, int32_t* __restrict__ zero_buf, int zero_n,
                                                           TqPreByAssign P, int tilings, TqRouteIn R, int route_off)
{
    if (PRE != 0 && blockIdx.x > 0) {
        if (check_blob && !blob_header_ok(hdr, expect)) return;      // a blob of another layer is not indexed
        pre_by_assign_block<PRE == 2>(P, idx, T, E, k, blockIdx.x - 1, threadIdx.x, ROUTE ? &R : nullptr);
        return;
    }
    if (ROUTE) {
        extern __shared__ int32_t sm_all[];
        float* sc = reinterpret_cast<float*>(sm_all + route_off);
        int32_t* ridx = sm_all + route_off + 64 * 17;
        float* rw = reinterpret_cast<float*>(ridx + TQ_PERM_CHUNK);
        route_small(R, T, E, k, sc, ridx, rw, threadIdx.x);
        __syncthreads();
        idx = ridx;
        w = rw;
    }
    permute_small_body(idx, w, n_assign, E, S, T, k, offsets, slot_of, slot_stride, src_of, row_token, row_w, tile_e,
                       tile_row0, rt_max, ctrl, err_flag, hdr, expect, check_blob, zero_buf, zero_n, tilings);
}

__global__ void clear_ctrl_kernel(int32_t* ctrl, int32_t* err_flag, int32_t* zero_buf, int zero_n)
{
    if (threadIdx.x < 64 && ctrl) ctrl[threadIdx.x] = 0;
    for (int i = threadIdx.x; i < zero_n; i += blockDim.x) zero_buf[i] = 0;
    if (threadIdx.x == 0 && err_flag && err_flag != ctrl) *err_flag = 0;
}

}  // namespace

tq_status tqi_launch_permute(const int32_t* topk_idx, const float* topk_w, int32_t T, int32_t E, int32_t S,
                             int32_t k, int32_t* offsets, int32_t* slot_of, int32_t slot_stride,
                             int32_t* src_of, int32_t* row_token, float* row_w, int32_t* tile_e,
                             int32_t* tile_row0, int32_t rt_max, int32_t* ctrl, int32_t* err_flag,
                             int32_t* hist, int32_t nblk, const void* blob, const TqLayout* L,
                             int32_t* zero_buf, int32_t zero_n, hipStream_t stream, const TqPreByAssign* pre, int tilings,
                             const TqRouteIn* route)
{
    const int64_t n_assign = (int64_t)T * k;
    const int64_t n_pre = pre ? (int64_t)pre->a_tot * pre->n_slices * pre->na_tiles : 0;
    if (n_pre > 0x3FFFFFFF) return TQ_ERR_UNSUPPORTED;
    TqBlobHeader expect = {};
    int check = 0;
    if (blob && L) {
        check = 1;
        expect.magic = TQ_BLOB_MAGIC; expect.version = TQ_BLOB_VERSION;
        expect.n_experts = L->E; expect.n_shared = L->S; expect.hidden = L->H; expect.ffn = L->F;
        expect.group = L->g; expect.bits = L->bits; expect.rank = L->r; expect.expert_stride = L->expert_stride;
        expect.code_words = L->cw; expect.factor_fp8 = L->fm.fp8; expect.tiles_m = L->fm.M; expect.tiles_n = L->fm.N;
    }
    const int ne = E + S;
    if (nblk == 1 && (int64_t)S * T <= 4096) {
        const int sm_words = ne + (ne + 1) + E + TQ_N_TILINGS * (ne + 1);
        const bool fused = route != nullptr;
        if (fused && !tqi_route_fusable(T, E, S, k, nblk)) return TQ_ERR_UNSUPPORTED;
        const size_t sm = ((size_t)sm_words + (fused ? 64 * 17 + 2 * TQ_PERM_CHUNK : 0)) * 4;
        const int pre_kind = n_pre > 0 ? (pre->fm.fp8 ? 2 : 1) : 0;
        const TqRouteIn R = fused ? *route : TqRouteIn{};
        const TqPreByAssign P = n_pre > 0 ? *pre : TqPreByAssign{};
#define TQ_PS(PREV, ROUTEV)                                                                                               \
        hipLaunchKernelGGL((permute_small_kernel<PREV, ROUTEV>), dim3(1 + (unsigned)n_pre), dim3(64), sm, stream, topk_idx, \
                           topk_w, (int)n_assign, E, S, T, k, offsets, slot_of, slot_stride, src_of, row_token, row_w,     \
                           tile_e, tile_row0, rt_max, ctrl, err_flag, (const TqBlobHeader*)blob, expect, check, zero_buf,  \
                           (int)zero_n, P, tilings, R, sm_words)
        if (fused) {
            if (pre_kind == 2) TQ_PS(2, true); else if (pre_kind == 1) TQ_PS(1, true); else TQ_PS(0, true);
        } else {
            if (pre_kind == 2) TQ_PS(2, false); else if (pre_kind == 1) TQ_PS(1, false); else TQ_PS(0, false);
        }
#undef TQ_PS
        TQ_CHECK_LAUNCH();
        return TQ_OK;
    }
    if (route) return TQ_ERR_UNSUPPORTED;      // the caller routes by itself when the single-wave permutation does not run
    if (n_pre > 0) {      // the permutation takes several launches: the pre-pass gets its own
        if (pre->fm.fp8)
            hipLaunchKernelGGL(pre_by_assign_kernel<true>, dim3((unsigned)n_pre), dim3(64), 0, stream, *pre, topk_idx, T, E, k,
                               (const TqBlobHeader*)blob, expect, check);
        else
            hipLaunchKernelGGL(pre_by_assign_kernel<false>, dim3((unsigned)n_pre), dim3(64), 0, stream, *pre, topk_idx, T, E, k,
                               (const TqBlobHeader*)blob, expect, check);
        TQ_CHECK_LAUNCH();
    }
    const size_t sm_mid = ((size_t)ne + (ne + 1) + TQ_N_TILINGS * (ne + 1) + 1 + (size_t)nblk * E) * 4;
    if (nblk <= TQ_PERM_MID_CHUNKS && sm_mid <= 64 * 1024 && (int64_t)S * T <= 0x3FFFFFFF) {
        hipLaunchKernelGGL(permute_mid_kernel, dim3(1), dim3(1024), sm_mid, stream, topk_idx, topk_w, (int)n_assign, (int)nblk, E, S,
                           T, k, offsets, slot_of, slot_stride, src_of, row_token, row_w, tile_e, tile_row0, rt_max, ctrl,
                           err_flag, (const TqBlobHeader*)blob, expect, check, zero_buf, (int)zero_n, tilings);
        TQ_CHECK_LAUNCH();
        return TQ_OK;
    }
    if (ctrl) {
        hipLaunchKernelGGL(clear_ctrl_kernel, dim3(1), dim3(64), 0, stream, ctrl, err_flag, zero_buf, (int)zero_n);
        TQ_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(hist_kernel, dim3(nblk), dim3(64), (size_t)E * 4, stream, topk_idx, n_assign, E, hist,
                       err_flag, (const TqBlobHeader*)blob, expect, check);
    TQ_CHECK_LAUNCH();
    const size_t sm_scan = ((size_t)ne + (ne + 1) + TQ_N_TILINGS * (ne + 1)) * 4;
    const bool split_scan = nblk > 64;
    if (split_scan) {
        hipLaunchKernelGGL(chunk_scan_kernel, dim3(E), dim3(64), 0, stream, hist, nblk, E, offsets + 1);
        TQ_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), sm_scan, stream, split_scan ? nullptr : hist, nblk, E, S, T,
                       offsets, tile_e, tile_row0, rt_max, ctrl, check && err_flag == ctrl ? 1 : 0);
    TQ_CHECK_LAUNCH();
    hipLaunchKernelGGL(scatter_kernel, dim3(nblk), dim3(64), (size_t)E * 4, stream, topk_idx, topk_w, n_assign, E,
                       S, T, k, hist, offsets, slot_of, slot_stride, src_of, row_token, row_w);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

extern "C" tq_status tq_route(const float* logits, const float* bias, int32_t T, int32_t E, int32_t k,
                              int32_t* topk_idx, float* topk_w, void* stream)
{
    if (!logits || !topk_idx || !topk_w) return TQ_ERR_NULL;
    if (T < 0 || E < 1 || k < 1 || k > E) return TQ_ERR_SHAPE;
    if (E > 64 * kMaxPerLane || k > 64) return TQ_ERR_UNSUPPORTED;
    if (((uintptr_t)logits | (uintptr_t)topk_idx | (uintptr_t)topk_w | (uintptr_t)bias) & 3) return TQ_ERR_ALIGN;
    if (T == 0) return TQ_OK;
    const int per_lane = (E + 63) / 64;
    const dim3 grid((T + 3) / 4), block(256);
    hipStream_t st = (hipStream_t)stream;
    if (per_lane == 1) hipLaunchKernelGGL(route_kernel<1>, grid, block, 0, st, logits, bias, T, E, k, topk_idx, topk_w);
    else if (per_lane == 2) hipLaunchKernelGGL(route_kernel<2>, grid, block, 0, st, logits, bias, T, E, k, topk_idx, topk_w);
    else if (per_lane <= 4) hipLaunchKernelGGL(route_kernel<4>, grid, block, 0, st, logits, bias, T, E, k, topk_idx, topk_w);
    else hipLaunchKernelGGL(route_kernel<kMaxPerLane>, grid, block, 0, st, logits, bias, T, E, k, topk_idx, topk_w);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

extern "C" size_t tq_permute_workspace_size(int32_t T, int32_t E, int32_t k)
{
    if (T < 0 || E < 1 || k < 1) return 0;
    int64_t nblk = ((int64_t)T * k + TQ_PERM_CHUNK - 1) / TQ_PERM_CHUNK;
    if (nblk < 1) nblk = 1;
    return tq_align256((size_t)nblk * E * 4);
}

extern "C" tq_status tq_permute(const int32_t* topk_idx, int32_t T, int32_t E, int32_t k, int32_t* offsets,
                                int32_t* slot_of, int32_t* src_of, int32_t* err_flag, void* workspace,
                                size_t workspace_bytes, void* stream)
{
    if (!topk_idx || !offsets || !slot_of || !src_of || !workspace) return TQ_ERR_NULL;
    if (T < 0 || E < 1 || E > 1024 || k < 1 || k > E) return TQ_ERR_SHAPE;
    if (workspace_bytes < tq_permute_workspace_size(T, E, k)) return TQ_ERR_WORKSPACE;
    if (((uintptr_t)topk_idx | (uintptr_t)offsets | (uintptr_t)slot_of | (uintptr_t)src_of |
         (uintptr_t)err_flag | (uintptr_t)workspace) & 3)
        return TQ_ERR_ALIGN;
    int64_t nblk = ((int64_t)T * k + TQ_PERM_CHUNK - 1) / TQ_PERM_CHUNK;
    if (nblk < 1) nblk = 1;     // T == 0 runs the single-wave kernel with nothing to place: offsets become all zero
    return tqi_launch_permute(topk_idx, nullptr, T, E, 0, k, offsets, slot_of, k, src_of, nullptr, nullptr,
                              nullptr, nullptr, 0, nullptr, err_flag, (int32_t*)workspace, (int32_t)nblk, nullptr,
                              nullptr, nullptr, 0, (hipStream_t)stream);
}
