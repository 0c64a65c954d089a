/*
 * tileq.h — C ABI of the MI355X (gfx950) quantised-expert MoE forward with low-rank compensation.
 *
 * The operation (TileQ, arXiv 2605.09281): an MoE layer  MoE(X) = sum_{k in topK} G_k(X) * W_k(X)
 * (Eq. 3) whose expert weights are stored as "quantised residual + rank-r term",
 * W ~ Q(W - W_r) + U V (Eq. 2, Eq. 4), evaluated at inference as the quantised forward plus the
 * low-rank forward (Eq. 14).  The factors tq_pack_weights takes are the effective per-expert ones of Eq. 4 /
 * Algorithm 1: A_e = diag(s_e)^-1 U_{m(e)} Sigma  ([in, r]) and B_e = V_{n(e)} ([r, out]), with the
 * input-side scaling, Sigma and the position table folded offline; tq_pack_weights_shared takes the shared
 * factors U_m Sigma, V_n and the position table of Eq. 4 themselves, and TQ_FLAG_FP8_FACTORS keeps Sigma apart.
 * Each expert is a SwiGLU MLP (gate, up, down); each of the three projections is
 *     proj(v)[n] = sum_kk v[kk] * (q[n,kk] - zero[n,kk/g]) * scale[n,kk/g]
 *                + sum_rho ( sum_kk v[kk] * A[kk,rho] ) * B[rho,n]
 * with group-wise scales as in Appendix A.3 ("Basic Quantization"), h = silu(gate(x)) * up(x),
 * y_e = down(h), and  y[t] = sum_j w[t,j] * y_{idx[t,j]}(x[t]) + sum_{shared s} y_s(x[t]).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless it is said to be host.  Descriptors (tq_layer_desc,
 *    tq_weights_src, tq_weights_dst) are small host structs whose members are device pointers.
 *  - The caller owns every buffer.  The library allocates nothing, frees nothing and never
 *    synchronises; all work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream).  Outputs are valid once the stream has reached the end of the call.
 *  - Every entry point returns tq_status; argument errors are found on the host before any launch
 *    and nothing is enqueued then.  Launch failures map to TQ_ERR_HIP.
 *  - Device pointers must be 16-byte aligned; `packed` and `workspace` 256-byte aligned.
 *  - fp16 / bf16 values travel as uint16_t bit patterns.
 *
 * Canonical (unpacked) weights, expert-major, experts 0..E-1 routed then E..E+S-1 shared,
 * projection p in {0 gate, 1 up, 2 down}; gate/up are [N=F, K=H], down is [N=H, K=F]:
 *     codes  uint8  [E+S][3][N*K]     one code per byte (0..15, or 0..7 when bits == 3), row-major [N,K]
 *     scale  fp16   [E+S][3][N*K/g]   row-major [N, K/g]
 *     zero   fp16   [E+S][3][N*K/g]   row-major [N, K/g]
 *     A      fp16   [E+S][(2H+F)*r]   gate [H,r] | up [H,r] | down [F,r]
 *     B      fp16   [E+S][(2F+H)*r]   gate [r,F] | up [r,F] | down [r,H]
 *
 * Packed blob (what tq_pack_weights writes; the header carries a format version that tq_moe_forward checks on the
 * device together with the geometry).  256-byte header, then one record per expert
 * at  256 + e * expert_stride.  A record holds two sections, GU (gate and up interleaved; N2 = 2F
 * columns, K = H) and D (down; N2 = H columns, K = F), each made of five 256-byte aligned parts.
 * Columns are taken in tiles of 32 and tiles in pairs: in GU pair j = (gate rows 32j..32j+31,
 * up rows 32j..32j+31); in D pair j = (rows 64j..64j+31, rows 64j+32..64j+63).  `lane` runs over
 * 0..63, the column inside a tile is lane%32 and hf = lane/32 picks the upper or lower 8 of a 16-wide
 * contraction step.  r16 = rank rounded up to a multiple of 16.
 *   codes  uint32 [pairs][K/64][2 tiles][64 lanes][4]
 *          word w of (pair, chunk c, tile, lane) carries the 8 codes of column (tile, lane%32) at
 *          kk = 64c + 16w + 8hf + i, i = 0..7; code i sits in nibble position (i/2) + 4*(i%2), i.e.
 *          the nibbles from least significant upward hold i = 0,2,4,6,1,3,5,7.
 *   sz     uint32 [pairs][K/g][2 tiles][32]      low half = scale fp16 bits, high half = zero fp16 bits
 *   zc     bf16   [pairs][2*ceil(G/16)][2 tiles][64 lanes][8]   (G = K/g)   derived, written by pack only:
 *          c = -scale * (128 + zero), evaluated in fp32, split as hi = bf16(c) and lo = bf16(c - hi), both
 *          round-to-nearest-even.  Element i of (pair, fragment s, tile, lane) belongs to group 16*(s/2) + 8hf + i
 *          of column (tile, lane%32) and holds hi for even s, lo for odd s; 0 where the group >= G.
 *          (The MFMA path feeds the codes as 128 + q; c times the group sum of the activations is what that
 *          leaves to add.)
 *   bfrag  fp16   [pairs][r16/16][2 tiles][64 lanes][8]
 *          element i of (pair, step s, tile, lane) = B[rho = 16s + 8hf + i][column], 0 where rho >= r
 *   afrag  fp16   [ceil(NA/32)][K/16][64 lanes][8]   NA = 2*r16 in GU (gate factors then up factors), r16 in D
 *          element i of (tile ta, step s, lane) = A_p[kk = 16s + 8hf + i][rho] with column
 *          c = 32ta + lane%32, p = c / r16, rho = c % r16; 0 where rho >= r or c >= NA
 * The blob is position independent (offsets only) and may be stored and reloaded byte for byte.
 *
 * Dense codes (TQ_FLAG_DENSE_CODES, bits = 3 or 2): the codes part becomes
 *   codes  uint32 [pairs][K/64][2 tiles][cw][64 lanes]      cw = bits words per lane
 * and there is no zc part.  The 32 codes of (pair, chunk c, tile, lane), q[w][i] at kk = 64c + 16w + 8hf + i
 * (w = 0..3, i = 0..7), form 16 slots P = 4w + j holding the two codes lo = q[w][2j], hi = q[w][2j+1], always 16
 * bit positions apart so that one shift and one and-or yield two bf16 values:
 *   bits = 2:  slot P sits in word P / 8 at position p = 2 (P % 8): lo in bits [p+1 : p], hi in bits [p+17 : p+16].
 *   bits = 3:  slots 0..14 sit in word P / 5 at position p = 3 (P % 5): lo in bits [p+2 : p], hi in bits
 *              [p+18 : p+16]; slot 15 uses the two bits left in every word: bit b (0..2) of its lo code is bit 15
 *              of word b, bit b of its hi code is bit 31 of word b.
 */
#ifndef TILEQ_H
#define TILEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TQ_OK = 0,
    TQ_ERR_NULL = 1,        /* a required pointer is NULL */
    TQ_ERR_SHAPE = 2,       /* non-positive or inconsistent dimensions (H % g, F % g, top_k > E, ...) */
    TQ_ERR_ALIGN = 3,       /* a pointer misses its alignment */
    TQ_ERR_RANGE = 4,       /* a code above qmax or an expert index outside [0, E), found on the device */
    TQ_ERR_WORKSPACE = 5,   /* workspace or output buffer too small */
    TQ_ERR_UNSUPPORTED = 6, /* valid request this build has no kernel for */
    TQ_ERR_HIP = 7,         /* a HIP call or launch failed */
    TQ_ERR_BLOB = 8         /* the packed blob's header does not match the descriptor.  The header lives in device
                               memory, so the forward finds this on the device: it is reported through bit 1 of the
                               workspace's error flag (see tq_moe_forward), and host-side tools that hold a copy of
                               the header may return this code */
} tq_status;

enum { TQ_ACT_BF16 = 0, TQ_ACT_FP32 = 1 };

/* flags of tq_layer_desc (test hooks; 0 in production) */
enum {
    TQ_FLAG_FORCE_SMALL_TILE = 1, /* bf16 path: always the 32-row tile */
    TQ_FLAG_FORCE_LARGE_TILE = 2, /* bf16 path: always the large (64/128-row, prefill) tiles */
    TQ_FLAG_FORCE_SKINNY = 4,     /* bf16 path: the 16-row weight-streaming (decode) kernels whenever the layer
                                     and the batch (at most 1024 assignment rows) allow them */
    /* Not a test hook but part of the format: codes of `bits` = 2 or 3 bits stored densely (the bit-widths of
       Table 1; Appendix A.3 with d = 2 or 3) instead of in 4-bit slots.  Groups of 64 and more.  The blob then
       has no zc part and its size is the storage count of Appendix A.3 plus padding.  Kernels: the decode path
       (bf16 activations, a few rows per expert), the tiled bf16 kernels for every other batch (groups of 64
       and 128; the zero-point coefficient fragments the blob does not store are derived into the workspace on
       every such call, which tq_moe_workspace_size accounts for) and the fp32 debug path; what none of them covers
       (groups of 256 with bf16 activations) returns TQ_ERR_UNSUPPORTED before any launch. */
    TQ_FLAG_DENSE_CODES = 32,
    /* Part of the format as well: the low-rank factors stored as fp8 E4M3 codes with an fp16 diagonal Sigma per
       rank component (mixed-precision factor storage, end of Section 3.1; Appendix A.3 with d_low = 8).  The
       effective factors are A = fp8(A8) diag(sigma), B = fp8(B8): a projection's low-rank term is
       ((x fp8(A8)) * sigma) fp8(B8).  E4M3 as for tq_lotile_pack_fp8 (OCP variant without infinities; NaN codes
       are not supported).  The factor parts of the blob then hold one byte per element in the layouts above
       (bfrag8, afrag8: the fp16 layouts with 1-byte elements) plus
         sig    fp32   [NA]   per section: sigma widened to fp32, gate then up (r16 each) in GU, r16 in D, 0 beyond r
       behind them.  Requires rank >= 1.  Kernels: all paths (the tiled bf16 kernels read fp16 fragments expanded
       into the workspace on every call, which tq_moe_workspace_size accounts for). */
    TQ_FLAG_FP8_FACTORS = 64
};

typedef struct tq_layer_desc {
    int32_t n_experts; /* E  routed experts, >= 1 */
    int32_t n_shared;  /* S  always-on shared experts, >= 0 */
    int32_t top_k;     /* k  in [1, E] */
    int32_t hidden;    /* H  multiple of 64 and of group */
    int32_t ffn;       /* F  multiple of 64 and of group */
    int32_t group;     /* g  quantisation group along the contraction dim; 32, 64, 128 or 256 */
    int32_t bits;      /* 4, or 3 (codes 0..7 kept in 4-bit slots); with TQ_FLAG_DENSE_CODES: 3 or 2, stored densely */
    int32_t rank;      /* r  in [0, 256]; 0 = no low-rank term.  The bf16 path carries at most 128 rank columns
                          (TQ_ERR_UNSUPPORTED beyond); the fp32 debug path takes all of them */
    int32_t act_dtype; /* TQ_ACT_BF16: x, y bf16, MFMA path.  TQ_ACT_FP32: x, y fp32, exact-dequant debug path */
    int32_t flags;     /* TQ_FLAG_DENSE_CODES and / or test hooks */
    int32_t tiles_m;   /* 0: per-expert factors A_e, B_e.  M >= 1: shared 2D-tiled factors (Eq. 4): M left factors    */
    int32_t tiles_n;   /*    U_m Sigma and N right factors V_n per projection and a placement table phi (both 0 or   */
                       /*    both >= 1; see tq_pack_weights_shared)                                                   */
} tq_layer_desc;

typedef struct tq_weights_src { /* canonical layout above; A, B may be NULL when rank == 0 */
    const uint8_t *codes;
    const uint16_t *scale, *zero;
    const uint16_t *A, *B;     /* with TQ_FLAG_FP8_FACTORS: the same arrays as uint8 E4M3 codes (cast the pointers) */
    const uint16_t *sigma;     /* with TQ_FLAG_FP8_FACTORS: fp16 [E+S][3][r] (gate, up, down), else ignored */
} tq_weights_src;

typedef struct tq_weights_dst {
    uint8_t *codes;
    uint16_t *scale, *zero;
    uint16_t *A, *B;           /* with TQ_FLAG_FP8_FACTORS: uint8 arrays */
    uint16_t *sigma;           /* with TQ_FLAG_FP8_FACTORS: fp16 [E+S][3][r] */
} tq_weights_dst;

/* Text for a status code (static storage, host). */
const char *tq_status_str(tq_status s);

/* Per-device set-up for the CURRENT device: reads the CU count and raises the dynamic-LDS limit of the kernels
 * that need more than the default.  Idempotent and thread-safe.  Every entry point that launches kernels runs it
 * by itself on its first call on a device, so calling it is optional — except for callers whose FIRST call on a
 * device would be inside a stream capture: they call tq_init() once before capturing (the set-up makes
 * host-side HIP calls that do not belong in a captured region). */
tq_status tq_init(void);

/* Bytes of the packed blob for this layer; 0 if the descriptor is invalid.  Host only.  With r a multiple
 * of 32 and K/g a multiple of 16 this is 256 + (E+S) * 3HF * (4 + 32/g + 32/g + 16 r (1/H + 1/F)) / 8:
 * the per-expert low-rank storage count of Appendix A.3 with a 16-bit scale and a 16-bit zero per group
 * (4 + 32/g + 16 r (1/H + 1/F) bits per weight), plus the derived zc part (32/g bits per weight: two bf16 values per group). */
size_t tq_packed_size(const tq_layer_desc *desc);

/* Packs canonical weights into the blob (layout above).  `err_flag` (device int32, may be NULL) is set
 * to 1 by the kernel if any code exceeds qmax = 2^bits - 1; it is not cleared here, and the offending
 * code is stored masked to 4 bits.  Returns TQ_ERR_WORKSPACE if packed_bytes < tq_packed_size(). */
tq_status tq_pack_weights(const tq_layer_desc *desc, const tq_weights_src *src, void *packed,
                          size_t packed_bytes, int32_t *err_flag, void *stream);

/* Shared 2D-tiled factors of a layer (Section 3.1, Eq. 4: W_k = U_p Sigma V_q + quantised residual, {p, q} = phi(k);
 * Algorithm 1 stores per expert the residual and phi(k), and the factors once).  For each projection p in
 * {0 gate, 1 up, 2 down} with contraction length K_p (H, H, F) and output width N_p (F, F, H):
 *     us[p]  fp16 [M][K_p][r]     U_m Sigma, any per-row input scaling folded in
 *     v[p]   fp16 [N][r][N_p]     V_n
 *     phi    int32 [E+S][2]       expert -> (m, n), 0 <= m < M, 0 <= n < N (shared experts included)
 * All device pointers.  The layer then computes exactly what tq_pack_weights computes with the effective factors
 * A_e = us[p][m(e)], B_e = v[p][n(e)]. */
typedef struct tq_shared_factors {
    const uint16_t *us[3];     /* with TQ_FLAG_FP8_FACTORS: uint8 E4M3 codes of U_m (cast the pointers) */
    const uint16_t *v[3];      /* with TQ_FLAG_FP8_FACTORS: uint8 E4M3 codes of V_n */
    const int32_t *phi;
    const uint16_t *sigma;     /* with TQ_FLAG_FP8_FACTORS: fp16 [3][r], the diagonal Sigma of each projection's tiled
                                  decomposition, shared by all tiles; else ignored */
} tq_shared_factors;

/* As tq_pack_weights for a descriptor with tiles_m, tiles_n >= 1: src->codes / scale / zero as there (src->A, src->B
 * are ignored), the factors from `shared`.  The blob keeps one record of codes, scales and zero-points per expert
 * (parts codes, sz, zc only) and, behind the records, in this order: the placement table int32 [E+S][2] padded to
 * 256 bytes; for section GU (gate and up side by side) M blocks in the afrag layout, block m built from us[0][m]
 * and us[1][m], then N blocks in the bfrag layout from v[0][n] and v[1][n]; for section D M afrag blocks from
 * us[2][m] and N bfrag blocks from v[2][n]; the whole padded to 256 bytes.  Every block has exactly the layout
 * and size of that part of a per-expert record.  Its size is tq_packed_size(desc): with r a multiple of 32 the factors cost
 * 16 r (M (2 H + F) + N (2 F + H)) bits in total instead of 16 r (E+S) (3 H + 3 F), the shared count of Appendix A.3.
 * err_flag bit 0 is also set when a phi entry is outside the grid (it is then clamped into it).
 * Every kernel of tq_moe_forward finds an expert's factors through phi, so the forward accepts such a blob under
 * the same descriptor on every path (tiled bf16, decode, fp32). */
tq_status tq_pack_weights_shared(const tq_layer_desc *desc, const tq_weights_src *src, const tq_shared_factors *shared,
                                 void *packed, size_t packed_bytes, int32_t *err_flag, void *stream);

/* Exact inverse of tq_pack_weights (bit for bit on codes, scale, zero, A, B): recovers the per-expert stored
 * tuple of Algorithm 1 (quantised residual, effective factors) from the blob.  For tests and tools. */
tq_status tq_unpack_weights(const tq_layer_desc *desc, const void *packed, const tq_weights_dst *dst,
                            void *stream);

/* Routing (Eq. 3's top-K set and routing weights).  logits fp32 [T,E]; bias fp32 [E] or NULL, added to
 * the logits in fp32 before selection.  topk_idx int32 [T,k]: the k highest scores in descending order,
 * equal scores to the lower expert index.  topk_w fp32 [T,k]: softmax over the k selected scores (sums
 * to 1).  NaN logits are not supported.  E <= 1024 and k <= 64 (TQ_ERR_UNSUPPORTED beyond). */
tq_status tq_route(const float *logits, const float *bias, int32_t T, int32_t E, int32_t k,
                   int32_t *topk_idx, float *topk_w, void *stream);

/* Bytes of scratch tq_permute needs. Host only. */
size_t tq_permute_workspace_size(int32_t T, int32_t E, int32_t k);

/* Token -> expert permutation with prefix-sum offsets (the per-token expert dispatch of Appendix A.4, "vs.
 * Per-Token Expert Dispatch", done once for the whole batch): assignment a = t*k + j belongs to expert
 * topk_idx[a].  offsets int32 [E+1] = exclusive prefix sum of the per-expert counts; slot_of int32 [T*k]
 * = position of assignment a in expert-sorted order, stable (assignments of one expert keep their order
 * in a); src_of int32 [T*k] = its inverse.  err_flag as in tq_pack_weights, set when an index is outside
 * [0,E) (that assignment is then dropped from the counts).  Exported for bit-exact tests; tq_moe_forward
 * runs the same kernels internally. */
tq_status tq_permute(const int32_t *topk_idx, int32_t T, int32_t E, int32_t k, int32_t *offsets,
                     int32_t *slot_of, int32_t *src_of, int32_t *err_flag, void *workspace,
                     size_t workspace_bytes, void *stream);

/* Bytes of workspace tq_moe_forward needs for up to T tokens.  Host only; 0 if desc is invalid. */
size_t tq_moe_workspace_size(const tq_layer_desc *desc, int32_t T);

/* The expert forward (Eq. 3 over experts whose projections are Eq. 2 / Eq. 4, evaluated as Eq. 14's quantised
 * forward plus low-rank forward): permutation, gate/up with fused dequant + low-rank term + SwiGLU, down with the
 * same, routing-weighted combination.  x, y are [T,H] bf16 (act_dtype 0) or fp32 (act_dtype 1); y is
 * overwritten.  topk_idx / topk_w as produced by tq_route.  The first int32 of `workspace` is an error
 * flag: the kernels set bit 0 (value 1) on an out-of-range expert index (such assignments contribute nothing)
 * and bit 1 (value 2) when the blob's header does not match the descriptor (then no projection runs and y is
 * undefined).  The call clears the flag at its start and never reads it back — the caller may inspect it after
 * synchronising.  A workspace sized by tq_moe_workspace_size(desc, T) serves every batch of at most T tokens.
 * T == 0 is a no-op. */
tq_status tq_moe_forward(const tq_layer_desc *desc, const void *packed, const void *x,
                         const int32_t *topk_idx, const float *topk_w, int32_t T, void *y,
                         void *workspace, size_t workspace_bytes, void *stream);

/* tq_route followed by tq_moe_forward in one call, with the same results bit for bit (Eq. 3: the top-K set, the
 * routing weights and the weighted sum over the selected experts): logits fp32 [T,E] and bias fp32 [E] or NULL as
 * for tq_route; topk_idx int32 [T,k] and topk_w fp32 [T,k] are OUTPUTS here (device, 16-byte aligned), everything else
 * as for tq_moe_forward.  For decode batches (at most 64 tokens, at most 16 routed experts, at most 256 assignments)
 * the routing runs inside the permutation's launch, which saves one kernel launch per step; other batches run the
 * two steps one after the other. */
tq_status tq_route_moe_forward(const tq_layer_desc *desc, const void *packed, const void *x, const float *logits,
                               const float *bias, int32_t T, int32_t *topk_idx, float *topk_w, void *y,
                               void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory — code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc: tq_moe_forward without a workspace argument.  The same kernels run on a scratch array
 * of TQ_STATIC_SCRATCH_MAX bytes that lives inside the library (a static device array: every GPU the library runs
 * on holds its own copy until the process ends); the call allocates nothing and frees nothing.  All other arguments
 * as tq_moe_forward.  err_flag (device int32, 4-byte aligned, may be NULL) receives the error flag described there
 * at the end of the call.  Returns TQ_ERR_WORKSPACE, before any launch, when the batch needs more scratch than the
 * array holds, i.e. when tq_moe_workspace_size(desc, T) computed for exactly this T exceeds TQ_STATIC_SCRATCH_MAX
 * (decode batches and small prefill batches fit; use tq_moe_forward beyond).  Every call on one GPU uses that
 * GPU's single array: the call itself clears what must start at zero, but two calls that overlap in time on one
 * GPU (different streams or threads) race and must be serialised by the caller.  Callers whose first call on a
 * device is inside a stream capture call tq_init() before capturing. */
#define TQ_STATIC_SCRATCH_MAX (32u << 20)
tq_status tq_moe_forward_static(const tq_layer_desc *desc, const void *packed, const void *x,
                                const int32_t *topk_idx, const float *topk_w, int32_t T, void *y,
                                int32_t *err_flag, void *stream);

/* Profiling aid (not part of the method).  Registers up to TQ_N_STAGE_EVENTS hipEvent_t handles (host
 * array, copied) that tq_moe_forward records on its stream at the stage boundaries:
 *   0 entry, 1 after the permutation, 2 after the gate/up pre-pass (group sums and x A), 3 after gate/up,
 *   4 after the down pre-pass, 5 after down, 6 after the combination.
 * tq_lotile_forward records 0 at entry, 1 after the projection, 2 after the gather-accumulate, 3 after the output
 * product.  n == 0 switches it off.  Process-wide and not thread-safe: meant for one benchmark thread. */
#define TQ_N_STAGE_EVENTS 7
tq_status tq_set_profile_events(void *const *events, int32_t n);

/* Measurement aid (not part of the method): streams `bytes` (a multiple of 16) from src with 16-byte
 * accesses.  mode 0 copies them to dst (dst holds `bytes`); mode 1 only reads them (dst needs 16 bytes and
 * is practically never written); mode 2 reads them with the non-temporal hint, one contiguous slab per
 * workgroup (the access pattern of the decode kernels' weight stream).  Used to calibrate hardware byte counters against a transfer of known
 * size and to measure the streaming rate the memory system attains. */
tq_status tq_debug_stream(const void *src, void *dst, size_t bytes, int32_t mode, void *stream);

/* Measurement aid (not part of the method): runs the instruction mix of the prefill kernels' main loop with no
 * global memory traffic, on every compute unit at the kernels' occupancy.  level 0: MFMAs alone (operands in
 * registers); 1: + the A fragments read from LDS; 2: + the B fragments unpacked from 4-bit codes; 3: + the fold of
 * each group of 8 steps into the accumulators (the full mix); 4: + per group the store of the next activation tile
 * into an LDS double buffer and the workgroup barrier that publishes it.  Each wave issues 32 * iters MFMAs
 * (v_mfma_f32_32x32x16_bf16, 32768 flops each).  scratch (device, 256-byte aligned, at least 4096 bytes): on
 * return of the kernel its first two uint64 hold the shader-clock cycles and the 100 MHz wall-clock ticks one wave
 * spent in the loop; bytes [256, 512) are read as 64 fp32 scale values (any finite contents). */
tq_status tq_debug_issue_probe(int32_t level, int32_t iters, void *scratch, size_t scratch_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------------
 * LoTileMoE: the fused low-rank path over SHARED 2D-tiled factors (Section 3.2: Eq. 14 splits the layer into
 * QMoE + LoTileMoE; the construction ending in Eq. 15 defines it, Eq. 16 is the compact buffer used here,
 * Appendix A.4 its three steps).  One linear map whose input is shared by all experts:
 *     y[b] = sum_t g[b,t] * ( x[b] (U_m Sigma) ) V_n ,   (m, n) = phi(e[b,t])
 * evaluated as  X_proj = x (U Sigma)_reshape  [T, M r],  S[b]^(n) = sum_{t: n(b,t) = n} g[b,t] X_proj[b]^(m(b,t))
 * [T, N r],  y = S V_flat  [T, out]: two dense products and one gather-scale-accumulate, no per-expert loop.
 * Canonical inputs (device): us fp16 [M][n_in][r] = U_m Sigma, v fp16 [N][r][n_out] = V_n, phi int32 [E][2].
 * n_in and n_out are multiples of 32, 1 <= r <= 256, M N >= E is not required (phi may share tiles).
 * The packed form holds phi and both factors as bf16 (round to nearest even) in MFMA B-operand fragment
 * order: element i of (column tile ct, step s, lane) = B[kk = 16 s + 8 (lane / 32) + i][32 ct + lane % 32],
 * for B1 = (U Sigma)_reshape with every tile's r columns padded to rp = 16 ceil(r / 16) (zero), and for
 * B2 = V_flat with its N r rows padded likewise. */
/* flags bit: mixed-precision factors (end of Section 3.1; Appendix A.3, d_low = 8): U_m and V_n are stored as fp8
 * E4M3 (OCP 8-bit floating point, the variant without infinities: bias 7, S.1111.111 is NaN, largest finite 448)
 * and the diagonal Sigma [r], shared by all tiles, as fp16.  The operator is then
 *     y[b] = sum_t g[b,t] * ( (x[b] U_m) * Sigma ) V_n
 * and the packed form keeps the fp8 bytes (two MFMA steps per 16-byte fragment) next to an fp32 copy of Sigma. */
#define TQ_LOTILE_FP8 1

typedef struct tq_lotile_desc {
    int32_t n_experts; /* E */
    int32_t tiles_m;   /* M row tiles (shared left factors) */
    int32_t tiles_n;   /* N column tiles (shared right factors) */
    int32_t n_in;      /* i */
    int32_t n_out;     /* o */
    int32_t rank;      /* r */
    int32_t top_k;     /* experts per token, at most min(E, 1024) */
    int32_t flags;     /* 0, or TQ_LOTILE_FP8 */
} tq_lotile_desc;

/* Bytes of the packed factors.  Host only; 0 if desc is invalid. */
size_t tq_lotile_packed_size(const tq_lotile_desc *desc);

/* Packs us, v, phi (device) into `packed` (device, 256-byte aligned).  err_flag (device int32, may be
 * NULL): bit 0 is set when a phi entry is outside the M x N grid (it is then clamped into it). */
tq_status tq_lotile_pack(const tq_lotile_desc *desc, const uint16_t *us, const uint16_t *v, const int32_t *phi,
                         void *packed, size_t packed_bytes, int32_t *err_flag, void *stream);

/* As tq_lotile_pack for a descriptor with TQ_LOTILE_FP8: u8 [M][n_in][r] and v8 [N][r][n_out] are fp8 E4M3 bytes,
 * sigma [r] fp16 bit patterns (all device).  The bytes are rearranged, never re-rounded.  tq_lotile_pack rejects a
 * descriptor with the flag, this function one without it (TQ_ERR_SHAPE). */
tq_status tq_lotile_pack_fp8(const tq_lotile_desc *desc, const uint8_t *u8, const uint16_t *sigma, const uint8_t *v8,
                             const int32_t *phi, void *packed, size_t packed_bytes, int32_t *err_flag, void *stream);

/* Bytes of workspace tq_lotile_forward needs for up to T tokens.  Host only; 0 if desc is invalid. */
size_t tq_lotile_workspace_size(const tq_lotile_desc *desc, int32_t T);

/* y[T, n_out] bf16 = LoTileMoE(x[T, n_in] bf16) for topk_idx / topk_w [T, top_k] as produced by tq_route.
 * y is overwritten.  An expert index outside [0, E) contributes nothing and sets the first int32 of
 * `workspace` (cleared at the start of the call).  Sums run in a fixed order: results are reproducible.
 * T == 0 is a no-op. */
tq_status tq_lotile_forward(const tq_lotile_desc *desc, const void *packed, const void *x,
                            const int32_t *topk_idx, const float *topk_w, int32_t T, void *y,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Offline helpers for the shared-factor format (host only, no GPU work, host pointers; unlike the GPU entry
 * points these may use the host heap for their own bookkeeping).
 *
 * tq_lotile_grid: the near-square tile grid for E experts (Appendix B, Evaluation Details, "Tiling-size"): M = the integer closest to
 * sqrt(E), N = ceil(E / M), so that M N >= E.
 *
 * tq_lotile_place: the greedy 2D-tiling placement (Section 3.1, Step 4, Eq. 9-10).  ideal [E][2] holds each
 * expert's ideal tile (m_k, n_k) from the biclustering; experts are placed in index order; the anchor of an expert
 * is its ideal tile clamped into the grid; the unoccupied cell of the smallest Chebyshev distance rho = 0, 1, 2, ...
 * from the anchor is taken.  The paper leaves the order inside a ring open: here a ring is scanned row by row
 * (m ascending, n ascending within a row).  phi [E][2] receives the placement: no two experts share a cell.
 * TQ_ERR_SHAPE if M N < E. */
tq_status tq_lotile_grid(int32_t n_experts, int32_t *tiles_m, int32_t *tiles_n);
tq_status tq_lotile_place(const int32_t *ideal, int32_t n_experts, int32_t tiles_m, int32_t tiles_n, int32_t *phi);

/* Offline helper on the GPU (Section 3.1, "Plug-in", Eq. 13): rank-r approximation of a dense matrix by r
 * Gaussian-sketch rank-1 deflations, the replacement for the SVD of the tiled matrix W_big (Eq. 11).  For rank rho,
 * with the sketch vector s = sketch[rho] (standard normal draws, supplied by the caller so that the routine draws no
 * random numbers of its own):
 *     Q = (W W^T)^it W s,   U = Q / |Q|,   Sigma = |Q^T W| / |Q|,   V = Q^T W / |Q^T W|,   W <- W - U Sigma V.
 * W      fp32 [rows][cols], row-major, device, 16-byte aligned; cols a multiple of 4.  OVERWRITTEN: on return it
 *        holds the residual W - sum_rho U_rho Sigma_rho V_rho.
 * sketch fp32 [r][cols] device.   it >= 0 power iterations (Q is renormalised after each one, which changes none of
 *        U, Sigma, V).
 * U      fp32 [r][rows] (unit vectors), sigma fp32 [r], V fp32 [r][cols] (unit vectors), device.  A matrix that runs
 *        out of rank yields zero vectors and Sigma = 0 from there on.
 * workspace: tq_sketch_workspace_size(rows, cols) bytes, device, 256-byte aligned (0 = unsupported shape).
 * 1 <= r <= 4096, it <= 64.  Asynchronous on `stream`; all sums have a fixed order. */
size_t tq_sketch_workspace_size(int64_t rows, int64_t cols);
tq_status tq_sketch_lowrank(float *W, int64_t rows, int64_t cols, int32_t r, int32_t it, const float *sketch, float *U,
                            float *sigma, float *V, void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TILEQ_H */
