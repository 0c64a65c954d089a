// tq_pack_weights / tq_unpack_weights: canonical expert weights <-> the packed blob whose layout
// include/tileq.h specifies.  Pure index arithmetic; every element is moved bit for bit.
#include "tq_common.h"

namespace {

struct PackGeom {
    int32_t n_exp, H, F, g, r, r16, qmax, cw;
    TqSection gu, d;
    size_t expert_stride;
};

__global__ void write_header_kernel(TqBlobHeader hdr, uint8_t* blob)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        TqBlobHeader* out = reinterpret_cast<TqBlobHeader*>(blob);
        *out = hdr;
    }
}

// One thread per packed 32-bit code word.  PACK: gather 8 canonical bytes -> word.  !PACK: scatter.
template <bool PACK>
__global__ void codes_kernel(PackGeom G, uint8_t* __restrict__ blob, uint8_t* __restrict__ codes,
                             int32_t* __restrict__ err_flag)
{
    const size_t words_gu = (size_t)G.gu.pairs * G.gu.chunks * 512;  // 2 tiles * 64 lanes * 4 words
    const size_t words_d = (size_t)G.d.pairs * G.d.chunks * 512;
    const size_t per_exp = words_gu + words_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= words_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= words_gu;
    int word = (int)(w & 3);
    int lane = (int)((w >> 2) & 63);
    int tile = (int)((w >> 8) & 1);
    size_t pc = w >> 9;
    int chunk = (int)(pc % sec.chunks);
    int pair = (int)(pc / sec.chunks);
    int col = lane & 31, hf = lane >> 5;
    int kk = 64 * chunk + 16 * word + 8 * hf;
    int p, n, K = sec.K;
    if (!is_d) { p = tile; n = 32 * pair + col; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; }
    const size_t HF = (size_t)G.H * G.F;
    uint8_t* src = codes + ((size_t)e * 3 + p) * HF + (size_t)n * K + kk;
    uint32_t* dst = reinterpret_cast<uint32_t*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.codes) + w;
    if (PACK) {
        uint64_t v = *reinterpret_cast<const uint64_t*>(src);
        uint32_t out = 0;
        bool bad = false;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t c = (uint32_t)(v >> (8 * i)) & 0xFF;
            bad |= c > (uint32_t)G.qmax;
            out |= (c & 15u) << (4 * tq_nibble_pos(i));
        }
        *dst = out;
        if (bad && err_flag) atomicOr(err_flag, TQ_FLAG_BIT_RANGE);
    } else {
        uint32_t in = *dst;
        uint64_t v = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) v |= (uint64_t)((in >> (4 * tq_nibble_pos(i))) & 15u) << (8 * i);
        *reinterpret_cast<uint64_t*>(src) = v;
    }
}

// Dense codes (2 or 3 bits): one thread per (pair, chunk, tile, lane); it moves the lane's 32 codes between the
// canonical bytes and its CW words, which sit CW x 64 lanes apart ([cw][64 lanes] inside the tile's block).
template <bool PACK, int CW>
__global__ void dense_codes_kernel(PackGeom G, uint8_t* __restrict__ blob, uint8_t* __restrict__ codes,
                                   int32_t* __restrict__ err_flag)
{
    const size_t lanes_gu = (size_t)G.gu.pairs * G.gu.chunks * 128;   // 2 tiles * 64 lanes
    const size_t lanes_d = (size_t)G.d.pairs * G.d.chunks * 128;
    const size_t per_exp = lanes_gu + lanes_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= lanes_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= lanes_gu;
    int lane = (int)(w & 63);
    int tile = (int)((w >> 6) & 1);
    size_t pc = w >> 7;
    int chunk = (int)(pc % sec.chunks);
    int pair = (int)(pc / sec.chunks);
    int col = lane & 31, hf = lane >> 5;
    int p, n, K = sec.K;
    if (!is_d) { p = tile; n = 32 * pair + col; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; }
    const size_t HF = (size_t)G.H * G.F;
    uint8_t* src = codes + ((size_t)e * 3 + p) * HF + (size_t)n * K + 64 * chunk + 8 * hf;      // + 16 w + i
    uint32_t* dst = reinterpret_cast<uint32_t*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.codes) +
                    (pc * 2 + tile) * (size_t)(CW * 64) + lane;                                  // + 64 d
    constexpr uint32_t FM = (1u << CW) - 1;       // CW is also the number of bits per code
    uint32_t word[CW];
    if (PACK) {
#pragma unroll
        for (int d = 0; d < CW; ++d) word[d] = 0;
        bool bad = false;
#pragma unroll
        for (int ws = 0; ws < 4; ++ws) {
            const uint64_t v = *reinterpret_cast<const uint64_t*>(src + 16 * ws);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = (uint32_t)(v >> (16 * j)) & 0xFF, hi = (uint32_t)(v >> (16 * j + 8)) & 0xFF;
                bad |= lo > FM || hi > FM;
                const int P = 4 * ws + j;
                if (CW == 2) {
                    word[P / 8] |= ((lo & FM) | ((hi & FM) << 16)) << (2 * (P % 8));
                } else if (P < 15) {
                    word[P / 5] |= ((lo & FM) | ((hi & FM) << 16)) << (3 * (P % 5));
                } else {
#pragma unroll
                    for (int b = 0; b < 3; ++b) word[b % CW] |= (((lo >> b) & 1u) << 15) | (((hi >> b) & 1u) << 31);
                }
            }
        }
#pragma unroll
        for (int d = 0; d < CW; ++d) dst[64 * d] = word[d];
        if (bad && err_flag) atomicOr(err_flag, TQ_FLAG_BIT_RANGE);
    } else {
#pragma unroll
        for (int d = 0; d < CW; ++d) word[d] = dst[64 * d];
#pragma unroll
        for (int ws = 0; ws < 4; ++ws) {
            uint64_t v = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int P = 4 * ws + j;
                uint32_t lo, hi;
                if (CW == 2) {
                    const uint32_t t = word[P / 8] >> (2 * (P % 8));
                    lo = t & FM; hi = (t >> 16) & FM;
                } else if (P < 15) {
                    const uint32_t t = word[P / 5] >> (3 * (P % 5));
                    lo = t & FM; hi = (t >> 16) & FM;
                } else {
                    lo = hi = 0;
#pragma unroll
                    for (int b = 0; b < 3; ++b) {
                        lo |= ((word[b % CW] >> 15) & 1u) << b;
                        hi |= ((word[b % CW] >> 31) & 1u) << b;
                    }
                }
                v |= (uint64_t)lo << (16 * j) | (uint64_t)hi << (16 * j + 8);
            }
            *reinterpret_cast<uint64_t*>(src + 16 * ws) = v;
        }
    }
}

// One thread per (scale, zero) word.
template <bool PACK>
__global__ void sz_kernel(PackGeom G, uint8_t* __restrict__ blob, uint16_t* __restrict__ scale,
                          uint16_t* __restrict__ zero)
{
    const size_t n_gu = (size_t)G.gu.pairs * G.gu.groups * 64;
    const size_t n_d = (size_t)G.d.pairs * G.d.groups * 64;
    const size_t per_exp = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    int col = (int)(w & 31);
    int tile = (int)((w >> 5) & 1);
    size_t pg = w >> 6;
    int grp = (int)(pg % sec.groups);
    int pair = (int)(pg / sec.groups);
    int p, n;
    if (!is_d) { p = tile; n = 32 * pair + col; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; }
    const size_t HFg = (size_t)G.H * G.F / G.g;
    size_t ci = ((size_t)e * 3 + p) * HFg + (size_t)n * sec.groups + grp;
    uint32_t* dst = reinterpret_cast<uint32_t*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.sz) + w;
    if (PACK) {
        *dst = (uint32_t)scale[ci] | ((uint32_t)zero[ci] << 16);
    } else {
        uint32_t v = *dst;
        scale[ci] = (uint16_t)(v & 0xFFFF);
        zero[ci] = (uint16_t)(v >> 16);
    }
}


// Derived part (pack only): bf16 hi/lo split of c = -scale * (128 + zero), the coefficient of the group sum
// of the activations once the codes are fed to the MFMA as 128 + q.  One thread per 8-element fragment.
__device__ inline uint32_t bf16_rne_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ void zc_kernel(PackGeom G, uint8_t* __restrict__ blob, const uint16_t* __restrict__ scale,
                          const uint16_t* __restrict__ zero)
{
    const size_t n_gu = (size_t)G.gu.pairs * G.gu.zsteps * 128;
    const size_t n_d = (size_t)G.d.pairs * G.d.zsteps * 128;
    const size_t per_exp = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    int lane = (int)(w & 63);
    int tile = (int)((w >> 6) & 1);
    size_t ps = w >> 7;
    int step = (int)(ps % sec.zsteps);
    int pair = (int)(ps / sec.zsteps);
    int col = lane & 31, hf = lane >> 5;
    int p, n;
    if (!is_d) { p = tile; n = 32 * pair + col; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; }
    const size_t HFg = (size_t)G.H * G.F / G.g;
    const int which = step % 2, gblock = step / 2;       // fragment 0 of a block: hi, 1: lo
    uint16_t* dst = reinterpret_cast<uint16_t*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.zc) + w * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int grp = 16 * gblock + 8 * hf + i;
        uint16_t out = 0;
        if (grp < sec.groups) {
            size_t ci = ((size_t)e * 3 + p) * HFg + (size_t)n * sec.groups + grp;
            const float s = __half2float(__ushort_as_half(scale[ci]));
            const float z = __half2float(__ushort_as_half(zero[ci]));
            const float c = -s * (128.0f + z);
            const uint32_t hi = bf16_rne_bits(c);
            out = which == 0 ? (uint16_t)hi : (uint16_t)bf16_rne_bits(c - __uint_as_float(hi << 16));
        }
        dst[i] = out;
    }
}

// One thread per 8-element fragment of B.  Padding rows (rho >= r) are written as zero and skipped on unpack.
// ET: uint16_t (fp16 bit patterns) or uint8_t (fp8 E4M3 codes): the layout is the same with 2- or 1-byte elements.
template <bool PACK, typename ET>
__global__ void bfrag_kernel(PackGeom G, uint8_t* __restrict__ blob, ET* __restrict__ B)
{
    const int steps = G.r16 / 16;
    const size_t n_gu = (size_t)G.gu.pairs * steps * 128;
    const size_t n_d = (size_t)G.d.pairs * steps * 128;
    const size_t per_exp = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    int lane = (int)(w & 63);
    int tile = (int)((w >> 6) & 1);
    size_t ps = w >> 7;
    int step = (int)(ps % steps);
    int pair = (int)(ps / steps);
    int col = lane & 31, hf = lane >> 5;
    int p, n, N;
    if (!is_d) { p = tile; n = 32 * pair + col; N = G.F; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; N = G.H; }
    const size_t b_per_exp = (2 * (size_t)G.F + G.H) * G.r;
    const size_t b_off = (p == 0) ? 0 : (p == 1) ? (size_t)G.F * G.r : 2 * (size_t)G.F * G.r;
    ET* src = B + (size_t)e * b_per_exp + b_off;
    ET* dst = reinterpret_cast<ET*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.bfrag) + w * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int rho = 16 * step + 8 * hf + i;
        if (PACK) dst[i] = (rho < G.r) ? src[(size_t)rho * N + n] : (ET)0;
        else if (rho < G.r) src[(size_t)rho * N + n] = dst[i];
    }
}

// One thread per 8-element fragment of A.
template <bool PACK, typename ET>
__global__ void afrag_kernel(PackGeom G, uint8_t* __restrict__ blob, ET* __restrict__ A)
{
    const size_t n_gu = (size_t)G.gu.na_tiles * (G.gu.K / 16) * 64;
    const size_t n_d = (size_t)G.d.na_tiles * (G.d.K / 16) * 64;
    const size_t per_exp = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    int lane = (int)(w & 63);
    size_t ts = w >> 6;
    int ksteps = sec.K / 16;
    int step = (int)(ts % ksteps);
    int ta = (int)(ts / ksteps);
    int c = 32 * ta + (lane & 31), hf = lane >> 5;
    int na = is_d ? G.r16 : 2 * G.r16;
    int p = is_d ? 2 : (c / G.r16);
    int rho = c % G.r16;
    const bool live = (c < na) && (rho < G.r);
    const size_t a_per_exp = (2 * (size_t)G.H + G.F) * G.r;
    const size_t a_off = (p == 0) ? 0 : (p == 1) ? (size_t)G.H * G.r : 2 * (size_t)G.H * G.r;
    ET* src = A + (size_t)e * a_per_exp + a_off;
    ET* dst = reinterpret_cast<ET*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.afrag) + w * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int kk = 16 * step + 8 * hf + i;
        if (PACK) dst[i] = live ? src[(size_t)kk * G.r + rho] : (ET)0;
        else if (live) src[(size_t)kk * G.r + rho] = dst[i];
    }
}

// Sigma of fp8 factors: fp16 [n_exp][3][r] <-> the fp32 `sig` parts of the records (GU: gate then up, r16 each; D),
// each padded with zeros to 256 bytes.  With n_tables == 1 and shared factors the one table [3][r] goes behind the pools.
template <bool PACK>
__global__ void sig_kernel(PackGeom G, TqFactorMap fm, uint8_t* __restrict__ blob, uint16_t* __restrict__ sigma, int n_tables)
{
    const int n_gu = (int)(tq_align256((size_t)2 * G.r16 * 4) / 4), n_d = (int)(tq_align256((size_t)G.r16 * 4) / 4);
    const int per = n_gu + n_d;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per * n_tables) return;
    const int e = idx / per;
    int c = idx % per;
    const bool is_d = c >= n_gu;
    if (is_d) c -= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    float* dst = (fm.shared ? reinterpret_cast<float*>(blob + fm.sig_off[is_d])
                            : reinterpret_cast<float*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.sig)) + c;
    const int p = is_d ? 2 : c / G.r16, rho = c % G.r16;
    const bool live = c < (is_d ? G.r16 : 2 * G.r16) && rho < G.r;
    uint16_t* src = sigma + ((size_t)e * 3 + p) * G.r + rho;
    if (PACK) *dst = live ? __half2float(__ushort_as_half(*src)) : 0.f;
    else if (live) *src = __half_as_ushort(__float2half(*dst));      // exact: the value came from an fp16
}

// fp8 factor fragments of the blob -> fp16 fragments in the workspace, for the tiled kernels (which read fp16
// fragments): left factors with Sigma folded in, A16 = fp16(fp8(A8) * sigma) (one rounding to nearest), right factors
// exactly.  One thread per 8-element fragment of one block; blocks are experts (per-expert factors) or tiles.
// which: 0 left factors, 1 right factors.
__global__ void expand_fp8_kernel(PackGeom G, TqFactorMap src, TqFactorMap dstm, const uint8_t* __restrict__ blob,
                                  uint8_t* __restrict__ fbase, int which, int n_blocks)
{
    const size_t n_gu = which == 0 ? (size_t)G.gu.na_tiles * (G.gu.K / 16) * 64 : (size_t)G.gu.pairs * (G.r16 / 16) * 128;
    const size_t n_d = which == 0 ? (size_t)G.d.na_tiles * (G.d.K / 16) * 64 : (size_t)G.d.pairs * (G.r16 / 16) * 128;
    const size_t per = n_gu + n_d;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per * n_blocks) return;
    const int blk = (int)(idx / per);
    size_t w = idx % per;
    const bool is_d = w >= n_gu;
    if (is_d) w -= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    const uint8_t* sp;        // the block's fp8 fragments
    if (src.shared) sp = blob + (which == 0 ? src.apool[is_d] + (size_t)blk * src.astride[is_d] : src.bpool[is_d] + (size_t)blk * src.bstride[is_d]);
    else sp = blob + TQ_HEADER_BYTES + (size_t)blk * G.expert_stride + (which == 0 ? sec.afrag : sec.bfrag);
    uint8_t* dp = fbase + (which == 0 ? dstm.apool[is_d] + (size_t)blk * dstm.astride[is_d] : dstm.bpool[is_d] + (size_t)blk * dstm.bstride[is_d]);
    const uint2 raw = reinterpret_cast<const uint2*>(sp)[w];
    float sg = 1.f;
    if (which == 0) {
        // column of t this fragment belongs to: 32 ta + lane % 32; Sigma is stored per column (gate then up in GU)
        const int lane = (int)(w & 63), ta = (int)((w >> 6) / (sec.K / 16));
        const int c = 32 * ta + (lane & 31), na = is_d ? G.r16 : 2 * G.r16;
        const float* sig = src.shared ? reinterpret_cast<const float*>(blob + src.sig_off[is_d])
                                      : reinterpret_cast<const float*>(blob + TQ_HEADER_BYTES + (size_t)blk * G.expert_stride + sec.sig);
        sg = c < na ? sig[c] : 0.f;
    }
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const uint32_t b0 = ((i < 4 ? raw.x : raw.y) >> (8 * (i & 3))) & 0xFF, b1 = ((i < 4 ? raw.x : raw.y) >> (8 * ((i + 1) & 3))) & 0xFF;
        const uint32_t h0 = __half_as_ushort(__float2half(tq_fp8_to_float(b0) * sg));
        const uint32_t h1 = __half_as_ushort(__float2half(tq_fp8_to_float(b1) * sg));
        o[i >> 1] = h0 | (h1 << 16);
    }
    reinterpret_cast<uint4*>(dp)[w] = make_uint4(o[0], o[1], o[2], o[3]);
}

// placement table of the expanded factors: the blob's own (shared factors) or the identity (per-expert factors)
__global__ void expand_phi_kernel(TqFactorMap src, TqFactorMap dstm, const uint8_t* __restrict__ blob, uint8_t* __restrict__ fbase,
                                  int n_exp)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_exp) return;
    int32_t* dst = reinterpret_cast<int32_t*>(fbase + dstm.phi_off);
    if (src.shared) {
        const int32_t* p = reinterpret_cast<const int32_t*>(blob + src.phi_off);
        dst[2 * e] = p[2 * e]; dst[2 * e + 1] = p[2 * e + 1];
    } else {
        dst[2 * e] = e; dst[2 * e + 1] = e;
    }
}

// The same fragments as zc_kernel writes, computed from the blob's own sz part into a buffer outside the blob (dense
// codes on the tiled kernels: such blobs store no zc part).  One thread per (pair, block of 16 groups, tile, lane): it
// reads its 8 scale / zero words once and writes the hi and the lo fragment.
__global__ void zc_from_blob_kernel(PackGeom G, const uint8_t* __restrict__ blob, uint8_t* __restrict__ zc_ws,
                                    size_t zc_stride, size_t zc_d_off)
{
    const size_t n_gu = (size_t)G.gu.pairs * (G.gu.zfrag / 2) * 128;
    const size_t n_d = (size_t)G.d.pairs * (G.d.zfrag / 2) * 128;
    const size_t per_exp = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_exp * G.n_exp) return;
    const int e = (int)(idx / per_exp);
    size_t w = idx % per_exp;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    const int lane = (int)(w & 63), tile = (int)((w >> 6) & 1);
    const size_t ps = w >> 7;
    const int nblocks = sec.zfrag / 2;
    const int gblock = (int)(ps % nblocks), pair = (int)(ps / nblocks);
    const int col = lane & 31, hf = lane >> 5;
    const uint32_t* sz = reinterpret_cast<const uint32_t*>(blob + TQ_HEADER_BYTES + (size_t)e * G.expert_stride + sec.sz);
    uint32_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int grp = min(16 * gblock + 8 * hf + i, sec.groups - 1);
        v[i] = sz[(((size_t)pair * sec.groups + grp) * 2 + tile) * 32 + col];
    }
    uint16_t hi16[8], lo16[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int grp = 16 * gblock + 8 * hf + i;
        const float s = __half2float(__ushort_as_half((uint16_t)(v[i] & 0xFFFF)));
        const float z = __half2float(__ushort_as_half((uint16_t)(v[i] >> 16)));
        const float c = -s * (128.0f + z);
        const uint32_t hi = bf16_rne_bits(c);
        const bool live = grp < sec.groups;
        hi16[i] = live ? (uint16_t)hi : (uint16_t)0;
        lo16[i] = live ? (uint16_t)bf16_rne_bits(c - __uint_as_float(hi << 16)) : (uint16_t)0;
    }
    // fragment f of (pair, tile, lane) sits at ((pair * zfrag + f) * 2 + tile) * 64 + lane, 8 values each
    uint16_t* base = reinterpret_cast<uint16_t*>(zc_ws + (size_t)e * zc_stride + (is_d ? zc_d_off : 0));
    uint16_t* dh = base + ((((size_t)pair * sec.zfrag + 2 * gblock) * 2 + tile) * 64 + lane) * 8;
    uint16_t* dl = base + ((((size_t)pair * sec.zfrag + 2 * gblock + 1) * 2 + tile) * 64 + lane) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) { dh[i] = hi16[i]; dl[i] = lo16[i]; }
}

// Shared 2D-tiled factors.  Left factors: one thread per 8-element fragment of block (section, m); the block has the
// afrag layout, its columns being [gate factor | up factor] (r16 each) in section GU and the down factor in D.
template <typename ET>
__global__ void pool_afrag_kernel(PackGeom G, TqFactorMap fm, uint8_t* __restrict__ blob,
                                  const ET* __restrict__ us_g, const ET* __restrict__ us_u,
                                  const ET* __restrict__ us_d)
{
    const size_t n_gu = (size_t)G.gu.na_tiles * (G.gu.K / 16) * 64;     // fragments per block
    const size_t n_d = (size_t)G.d.na_tiles * (G.d.K / 16) * 64;
    const size_t per_m = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_m * fm.M) return;
    const int m = (int)(idx / per_m);
    size_t w = idx % per_m;
    const bool is_d = w >= n_gu;
    const TqSection& sec = is_d ? G.d : G.gu;
    if (is_d) w -= n_gu;
    const int lane = (int)(w & 63);
    const size_t ts = w >> 6;
    const int ksteps = sec.K / 16;
    const int step = (int)(ts % ksteps), ta = (int)(ts / ksteps);
    const int c = 32 * ta + (lane & 31), hf = lane >> 5;
    const int na = is_d ? G.r16 : 2 * G.r16;
    const int p = is_d ? 2 : (c / G.r16);
    const int rho = c % G.r16;
    const bool live = (c < na) && (rho < G.r);
    const ET* src = (p == 0 ? us_g : p == 1 ? us_u : us_d) + (size_t)m * sec.K * G.r;      // [K][r] of tile row m
    ET* dst = reinterpret_cast<ET*>(blob + fm.apool[is_d] + (size_t)m * fm.astride[is_d]) + w * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int kk = 16 * step + 8 * hf + i;
        dst[i] = live ? src[(size_t)kk * G.r + rho] : (ET)0;
    }
}

// Right factors: one thread per 8-element fragment of block (section, n), in the bfrag layout (tile 0 / 1 of a pair:
// gate / up factor in section GU, the two 32-column halves of the down factor's 64 columns in D).
template <typename ET>
__global__ void pool_bfrag_kernel(PackGeom G, TqFactorMap fm, uint8_t* __restrict__ blob,
                                  const ET* __restrict__ v_g, const ET* __restrict__ v_u,
                                  const ET* __restrict__ v_d)
{
    const int steps = G.r16 / 16;
    const size_t n_gu = (size_t)G.gu.pairs * steps * 128;
    const size_t n_d = (size_t)G.d.pairs * steps * 128;
    const size_t per_n = n_gu + n_d;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= per_n * fm.N) return;
    const int nt = (int)(idx / per_n);
    size_t w = idx % per_n;
    const bool is_d = w >= n_gu;
    if (is_d) w -= n_gu;
    const int lane = (int)(w & 63), tile = (int)((w >> 6) & 1);
    const size_t ps = w >> 7;
    const int step = (int)(ps % steps), pair = (int)(ps / steps);
    const int col = lane & 31, hf = lane >> 5;
    int p, n, N;
    if (!is_d) { p = tile; n = 32 * pair + col; N = G.F; }
    else       { p = 2;    n = 64 * pair + 32 * tile + col; N = G.H; }
    const ET* src = (p == 0 ? v_g : p == 1 ? v_u : v_d) + (size_t)nt * G.r * N;              // [r][N] of tile column nt
    ET* dst = reinterpret_cast<ET*>(blob + fm.bpool[is_d] + (size_t)nt * fm.bstride[is_d]) + w * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rho = 16 * step + 8 * hf + i;
        dst[i] = (rho < G.r) ? src[(size_t)rho * N + n] : (ET)0;
    }
}

__global__ void phi_kernel(TqFactorMap fm, int n_exp, int n_padded, uint8_t* __restrict__ blob, const int32_t* __restrict__ phi,
                           int32_t* __restrict__ err_flag)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_padded) return;
    int m = 0, n = 0;                    // entries of the padding behind the table are written as zeros
    if (e < n_exp) {
        m = phi[2 * e]; n = phi[2 * e + 1];
        if (m < 0 || m >= fm.M || n < 0 || n >= fm.N) {
            if (err_flag) atomicOr(err_flag, TQ_FLAG_BIT_RANGE);
            m = min(max(m, 0), fm.M - 1);
            n = min(max(n, 0), fm.N - 1);
        }
    }
    int32_t* dst = reinterpret_cast<int32_t*>(blob + fm.phi_off);
    dst[2 * e] = m;
    dst[2 * e + 1] = n;
}

inline PackGeom make_geom(const TqLayout& L)
{
    PackGeom G;
    G.n_exp = L.E + L.S; G.H = L.H; G.F = L.F; G.g = L.g; G.r = L.r; G.r16 = L.r16;
    G.qmax = (1 << L.bits) - 1;
    G.cw = L.cw;
    G.gu = L.gu; G.d = L.d; G.expert_stride = L.expert_stride;
    return G;
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

template <bool PACK>
tq_status run(const TqLayout& L, uint8_t* blob, uint8_t* codes, uint16_t* scale, uint16_t* zero,
              uint16_t* A, uint16_t* B, uint16_t* sigma, int32_t* err_flag, hipStream_t st)
{
    PackGeom G = make_geom(L);
    const size_t ne = G.n_exp;
    size_t n_codes = ((size_t)L.gu.pairs * L.gu.chunks + (size_t)L.d.pairs * L.d.chunks) * 512 * ne;
    size_t n_sz = ((size_t)L.gu.pairs * L.gu.groups + (size_t)L.d.pairs * L.d.groups) * 64 * ne;
    if (n_codes / 256 > 0x7FFFFFFFull) return TQ_ERR_UNSUPPORTED;
    if (L.cw == 4)
        hipLaunchKernelGGL(codes_kernel<PACK>, dim3(blocks_for(n_codes)), dim3(256), 0, st, G, blob, codes, err_flag);
    else if (L.cw == 3)
        hipLaunchKernelGGL((dense_codes_kernel<PACK, 3>), dim3(blocks_for(n_codes / 4)), dim3(256), 0, st, G, blob, codes, err_flag);
    else
        hipLaunchKernelGGL((dense_codes_kernel<PACK, 2>), dim3(blocks_for(n_codes / 4)), dim3(256), 0, st, G, blob, codes, err_flag);
    TQ_CHECK_LAUNCH();
    hipLaunchKernelGGL(sz_kernel<PACK>, dim3(blocks_for(n_sz)), dim3(256), 0, st, G, blob, scale, zero);
    TQ_CHECK_LAUNCH();
    if (PACK && L.cw == 4) {
        size_t n_zc = ((size_t)L.gu.pairs * L.gu.zsteps + (size_t)L.d.pairs * L.d.zsteps) * 128 * ne;
        hipLaunchKernelGGL(zc_kernel, dim3(blocks_for(n_zc)), dim3(256), 0, st, G, blob, scale, zero);
        TQ_CHECK_LAUNCH();
    }
    if (L.r > 0 && !L.fm.shared) {
        size_t n_b = ((size_t)L.gu.pairs + L.d.pairs) * (L.r16 / 16) * 128 * ne;
        size_t n_a = ((size_t)L.gu.na_tiles * (L.gu.K / 16) + (size_t)L.d.na_tiles * (L.d.K / 16)) * 64 * ne;
        if (L.fm.fp8) {
            hipLaunchKernelGGL((bfrag_kernel<PACK, uint8_t>), dim3(blocks_for(n_b)), dim3(256), 0, st, G, blob, (uint8_t*)B);
            TQ_CHECK_LAUNCH();
            hipLaunchKernelGGL((afrag_kernel<PACK, uint8_t>), dim3(blocks_for(n_a)), dim3(256), 0, st, G, blob, (uint8_t*)A);
            TQ_CHECK_LAUNCH();
            hipLaunchKernelGGL(sig_kernel<PACK>, dim3(blocks_for((tq_align256((size_t)8 * L.r16) + tq_align256((size_t)4 * L.r16)) / 4 * ne)),
                               dim3(256), 0, st, G, L.fm, blob, sigma, (int)ne);
            TQ_CHECK_LAUNCH();
        } else {
            hipLaunchKernelGGL((bfrag_kernel<PACK, uint16_t>), dim3(blocks_for(n_b)), dim3(256), 0, st, G, blob, B);
            TQ_CHECK_LAUNCH();
            hipLaunchKernelGGL((afrag_kernel<PACK, uint16_t>), dim3(blocks_for(n_a)), dim3(256), 0, st, G, blob, A);
            TQ_CHECK_LAUNCH();
        }
    }
    return TQ_OK;
}

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

}  // namespace

tq_status tqi_expand_fp8_factors(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, uint8_t* ws, hipStream_t stream)
{
    if (!L.fm.fp8 || W.fac_bytes == 0) return TQ_ERR_UNSUPPORTED;
    const PackGeom G = make_geom(L);
    uint8_t* fbase = ws + W.fac_ws;
    const size_t per_a = ((size_t)L.gu.na_tiles * (L.gu.K / 16) + (size_t)L.d.na_tiles * (L.d.K / 16)) * 64;
    const size_t per_b = ((size_t)L.gu.pairs + L.d.pairs) * (L.r16 / 16) * 128;
    hipLaunchKernelGGL(expand_phi_kernel, dim3(blocks_for((size_t)(L.E + L.S))), dim3(256), 0, stream, L.fm, W.fac_fm, blob, fbase,
                       L.E + L.S);
    TQ_CHECK_LAUNCH();
    hipLaunchKernelGGL(expand_fp8_kernel, dim3(blocks_for(per_a * W.fac_fm.M)), dim3(256), 0, stream, G, L.fm, W.fac_fm, blob, fbase,
                       0, W.fac_fm.M);
    TQ_CHECK_LAUNCH();
    hipLaunchKernelGGL(expand_fp8_kernel, dim3(blocks_for(per_b * W.fac_fm.N)), dim3(256), 0, stream, G, L.fm, W.fac_fm, blob, fbase,
                       1, W.fac_fm.N);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

tq_status tqi_derive_zc(const TqLayout& L, const TqWorkspace& W, const uint8_t* blob, uint8_t* ws, hipStream_t stream)
{
    if (W.zc_stride == 0) return TQ_ERR_UNSUPPORTED;
    const PackGeom G = make_geom(L);
    const size_t n = ((size_t)L.gu.pairs * (L.gu.zfrag / 2) + (size_t)L.d.pairs * (L.d.zfrag / 2)) * 128 * (L.E + L.S);
    hipLaunchKernelGGL(zc_from_blob_kernel, dim3(blocks_for(n)), dim3(256), 0, stream, G, blob, ws + W.zc_ws, W.zc_stride,
                       W.zc_d_off);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}

extern "C" size_t tq_packed_size(const tq_layer_desc* desc)
{
    TqLayout L;
    if (!tq_make_layout(desc, &L)) return 0;
    return L.total_bytes;
}

namespace {
tq_status pack_impl(const tq_layer_desc* desc, const tq_weights_src* src, const tq_shared_factors* shared, void* packed,
                    size_t packed_bytes, int32_t* err_flag, void* stream);
}

extern "C" tq_status tq_pack_weights(const tq_layer_desc* desc, const tq_weights_src* src, void* packed,
                                     size_t packed_bytes, int32_t* err_flag, void* stream)
{
    if (desc && (desc->tiles_m || desc->tiles_n)) return TQ_ERR_SHAPE;      // shared factors: tq_pack_weights_shared
    return pack_impl(desc, src, nullptr, packed, packed_bytes, err_flag, stream);
}

extern "C" tq_status tq_pack_weights_shared(const tq_layer_desc* desc, const tq_weights_src* src,
                                            const tq_shared_factors* shared, void* packed, size_t packed_bytes,
                                            int32_t* err_flag, void* stream)
{
    if (!shared) return TQ_ERR_NULL;
    if (desc && !(desc->tiles_m > 0 && desc->tiles_n > 0)) return TQ_ERR_SHAPE;
    for (int p = 0; p < 3; ++p) {
        if (!shared->us[p] || !shared->v[p]) return TQ_ERR_NULL;
        if ((((uintptr_t)shared->us[p]) | ((uintptr_t)shared->v[p])) & 15) return TQ_ERR_ALIGN;
    }
    if (!shared->phi) return TQ_ERR_NULL;
    if ((uintptr_t)shared->phi & 3) return TQ_ERR_ALIGN;
    return pack_impl(desc, src, shared, packed, packed_bytes, err_flag, stream);
}

namespace {
tq_status pack_impl(const tq_layer_desc* desc, const tq_weights_src* src, const tq_shared_factors* shared, void* packed,
                    size_t packed_bytes, int32_t* err_flag, void* stream)
{
    if (!desc || !src || !packed || !src->codes || !src->scale || !src->zero) return TQ_ERR_NULL;
    TqLayout L;
    if (!tq_make_layout(desc, &L)) return TQ_ERR_SHAPE;
    if (L.r > 0 && !L.fm.shared && (!src->A || !src->B)) return TQ_ERR_NULL;
    if (L.fm.fp8 && !(L.fm.shared ? shared->sigma : src->sigma)) return TQ_ERR_NULL;
    if (L.fm.fp8 && misaligned(L.fm.shared ? shared->sigma : src->sigma, 2)) return TQ_ERR_ALIGN;
    if (packed_bytes < L.total_bytes) return TQ_ERR_WORKSPACE;
    if (misaligned(packed, 256) || misaligned(src->codes, 16) || misaligned(src->scale, 16) ||
        misaligned(src->zero, 16) || (L.r > 0 && !L.fm.shared && (misaligned(src->A, 16) || misaligned(src->B, 16))) ||
        misaligned(err_flag, 4))
        return TQ_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    TqBlobHeader hdr = {};
    hdr.magic = TQ_BLOB_MAGIC; hdr.version = TQ_BLOB_VERSION;
    hdr.n_experts = L.E; hdr.n_shared = L.S; hdr.hidden = L.H; hdr.ffn = L.F; hdr.group = L.g;
    hdr.bits = L.bits; hdr.rank = L.r; hdr.r16 = L.r16; hdr.code_words = L.cw; hdr.factor_fp8 = L.fm.fp8;
    hdr.tiles_m = L.fm.M; hdr.tiles_n = L.fm.N;
    hdr.expert_stride = L.expert_stride; hdr.total_bytes = L.total_bytes;
    hdr.off[0] = L.gu.codes; hdr.off[1] = L.gu.sz; hdr.off[2] = L.gu.zc; hdr.off[3] = L.gu.bfrag; hdr.off[4] = L.gu.afrag;
    hdr.off[5] = L.d.codes; hdr.off[6] = L.d.sz; hdr.off[7] = L.d.zc; hdr.off[8] = L.d.bfrag; hdr.off[9] = L.d.afrag;
    hipLaunchKernelGGL(write_header_kernel, dim3(1), dim3(64), 0, st, hdr, (uint8_t*)packed);
    TQ_CHECK_LAUNCH();
    tq_status rc = run<true>(L, (uint8_t*)packed, const_cast<uint8_t*>(src->codes), const_cast<uint16_t*>(src->scale),
                             const_cast<uint16_t*>(src->zero), const_cast<uint16_t*>(src->A),
                             const_cast<uint16_t*>(src->B), const_cast<uint16_t*>(src->sigma), err_flag, st);
    if (rc != TQ_OK || !L.fm.shared) return rc;
    const PackGeom G = make_geom(L);
    const size_t n_a = ((size_t)L.gu.na_tiles * (L.gu.K / 16) + (size_t)L.d.na_tiles * (L.d.K / 16)) * 64 * L.fm.M;
    const size_t n_b = ((size_t)L.gu.pairs + L.d.pairs) * (L.r16 / 16) * 128 * L.fm.N;
    if (L.fm.fp8) {
        hipLaunchKernelGGL(pool_afrag_kernel<uint8_t>, dim3(blocks_for(n_a)), dim3(256), 0, st, G, L.fm, (uint8_t*)packed,
                           (const uint8_t*)shared->us[0], (const uint8_t*)shared->us[1], (const uint8_t*)shared->us[2]);
        TQ_CHECK_LAUNCH();
        hipLaunchKernelGGL(pool_bfrag_kernel<uint8_t>, dim3(blocks_for(n_b)), dim3(256), 0, st, G, L.fm, (uint8_t*)packed,
                           (const uint8_t*)shared->v[0], (const uint8_t*)shared->v[1], (const uint8_t*)shared->v[2]);
        TQ_CHECK_LAUNCH();
        hipLaunchKernelGGL(sig_kernel<true>, dim3(blocks_for((tq_align256((size_t)8 * L.r16) + tq_align256((size_t)4 * L.r16)) / 4)),
                           dim3(256), 0, st, G, L.fm, (uint8_t*)packed, const_cast<uint16_t*>(shared->sigma), 1);
        TQ_CHECK_LAUNCH();
    } else {
        hipLaunchKernelGGL(pool_afrag_kernel<uint16_t>, dim3(blocks_for(n_a)), dim3(256), 0, st, G, L.fm, (uint8_t*)packed,
                           shared->us[0], shared->us[1], shared->us[2]);
        TQ_CHECK_LAUNCH();
        hipLaunchKernelGGL(pool_bfrag_kernel<uint16_t>, dim3(blocks_for(n_b)), dim3(256), 0, st, G, L.fm, (uint8_t*)packed,
                           shared->v[0], shared->v[1], shared->v[2]);
        TQ_CHECK_LAUNCH();
    }
    const int n_padded = (int)(tq_align256((size_t)(L.E + L.S) * 8) / 8);
    hipLaunchKernelGGL(phi_kernel, dim3(blocks_for((size_t)n_padded)), dim3(256), 0, st, L.fm, L.E + L.S, n_padded,
                       (uint8_t*)packed, shared->phi, err_flag);
    TQ_CHECK_LAUNCH();
    return TQ_OK;
}
}  // namespace

extern "C" tq_status tq_unpack_weights(const tq_layer_desc* desc, const void* packed, const tq_weights_dst* dst,
                                       void* stream)
{
    if (!desc || !dst || !packed || !dst->codes || !dst->scale || !dst->zero) return TQ_ERR_NULL;
    TqLayout L;
    if (!tq_make_layout(desc, &L)) return TQ_ERR_SHAPE;
    if (L.r > 0 && !L.fm.shared && (!dst->A || !dst->B)) return TQ_ERR_NULL;      // shared factors: codes, scale, zero only
    if (L.fm.fp8 && !L.fm.shared && (!dst->sigma || misaligned(dst->sigma, 2))) return TQ_ERR_NULL;
    if (misaligned(packed, 256) || misaligned(dst->codes, 16) || misaligned(dst->scale, 16) ||
        misaligned(dst->zero, 16) || (L.r > 0 && !L.fm.shared && (misaligned(dst->A, 16) || misaligned(dst->B, 16))))
        return TQ_ERR_ALIGN;
    return run<false>(L, const_cast<uint8_t*>((const uint8_t*)packed), dst->codes, dst->scale, dst->zero, dst->A,
                      dst->B, dst->sigma, nullptr, (hipStream_t)stream);
}
