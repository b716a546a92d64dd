// k-means assignment (paper Sec. 4.1), and the fused encoder pass that follows it:
// centroid subtraction (Eq. 5), T rounds of 2-bit group quantization of the residual
// (Sec. 3.2 Eq. 1-2, applied progressively as in Sec. 4.2) and bit packing.
//
// Assignment = argmin_j ||x - c_j||^2 = argmax_j ( x.c_j - ||c_j||^2 / 2 ).
// The N x K matrix of scores is a dense contraction and runs on the matrix cores
// (v_mfma_f32_32x32x16_bf16; bf16 x bf16 products are exact in fp32), with the centroid
// table of the unit staged once per workgroup in LDS.  The MFMA is issued transposed
// (rows = centroids, columns = tokens) so that one lane owns one token and the argmax over
// centroids is a per-lane running maximum followed by a single exchange between the two
// lane halves.  A wavefront works on 64 tokens at a time: every centroid operand read from
// LDS feeds two MFMAs (two blocks of 32 tokens), which halves the LDS traffic per flop and
// gives two independent accumulation chains.  The term -||c||^2/2 enters through one extra
// MFMA step: a small kernel has split it, per centroid, into three bf16 pieces whose sum is
// the fp32 value exactly, and the matching token operand holds three ones.
//
// Exactness.  The reference result is the argmin of fp64 distances.  The fp32 scores
// carry a rounding error, so the kernel keeps the three largest scores per token
// (cluster index carried in the 7 low mantissa bits) and certifies the winner only
// when it leads by more than a bound on that error,
//     thr = 2^-14 * (||x||^2 / 2 + max_j ||c_j||^2),
// which covers the 131 accumulation roundings of half an ulp each plus the index tag for both
// scores (with more than 256 centroids the tag has 8 bits and the factor is 1.5 * 2^-14).  Otherwise the candidates are re-evaluated in fp64: the two leaders
// cooperatively by the wavefront, or, if the third score is inside the band as well,
// all K centroids with the channels summed in index order (the reference order).
// Equal fp64 distances go to the lower index.
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kAsgThreads = 256;
constexpr int kAsgWaves = kAsgThreads / 64;
constexpr int kAsgTile = 64;                    // tokens per wavefront step (two MFMA column blocks)
constexpr int kCPitch = 136;                    // bf16 elements per LDS centroid row (272 B): 128 + (hi, mid, lo of -||c||^2/2) + 5 zeros
constexpr int kPrepThreads = 256;

__device__ __forceinline__ void insert3(float v, int idx, float &b1, float &b2, float &b3,
                                        int &i1, int &i2) {
    if (v > b1) { b3 = b2; b2 = b1; i2 = i1; b1 = v; i1 = idx; }
    else if (v > b2) { b3 = b2; b2 = v; i2 = idx; }
    else if (v > b3) { b3 = v; }
}

__device__ __forceinline__ double shfl_xor_f64(double v, int m) { return __shfl_xor(v, m, 64); }
// Sum over each aligned group of 16 lanes, every lane getting the total, by data-parallel-primitive
// moves (VALU; the general lane exchange goes through the LDS pipe and its latency, four times in
// a row per table piece).  Pairings: lane ^ 1, lane ^ 2, then the mirror images inside 8 and
// inside 16 lanes, whose partners hold what lane ^ 4 and lane ^ 8 hold, so the sums are those of
// the xor butterfly bit for bit.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xf, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xf, 0xf, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double sum16_f64(double v) {
    v += dpp_f64<0xB1>(v);       // quad_perm [1,0,3,2]
    v += dpp_f64<0x4E>(v);       // quad_perm [2,3,0,1]
    v += dpp_f64<0x141>(v);      // row_half_mirror
    v += dpp_f64<0x140>(v);      // row_mirror
    return v;
}
__device__ __forceinline__ double readlane_f64(double v, int lane) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
template <bool V> struct BoolK { static constexpr bool value = V; };
// (a & mask) | (b & ~mask): v_bfi_b32
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }
// a constant the compiler must keep in a vector register (so that the other, scalar operand of a
// three-operand VALU instruction is the only one on the constant bus)
__device__ __forceinline__ uint32_t vgpr_const(uint32_t c) {
    uint32_t v;
    asm volatile("v_mov_b32 %0, %1" : "=v"(v) : "s"(c));
    return v;
}

// ---------------------------------------------------------------------------------------------
// Per centroid: nh = fp32(-||c||^2 / 2) from an fp64 sum, split into three bf16 pieces by
// truncation (8 significant bits each, so hi + mid + lo == nh exactly); rows K..Kpad-1 get a
// huge negative value so that they never win.  Per unit: an upper bound of max ||c||^2.
// One workgroup per unit, 16 lanes per row.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kPrepThreads)
void centroid_prep_kernel(const bf16_t *cent, int K, int Kpad, uint2 *nh3, float *cmax_out) {
    __shared__ uint32_t smax;
    const int h = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) smax = 0u;
    __syncthreads();
    const bf16_t *cg = cent + (int64_t)h * K * kHeadDim;
    for (int i = tid; i < Kpad * 16; i += kPrepThreads) {          // Kpad*16 is a multiple of 64: whole waves
        const int row = i >> 4, c16 = i & 15;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < K) v = *reinterpret_cast<const uint4 *>(cg + (int64_t)row * kHeadDim + c16 * 8);
        double s = 0.0;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double lo = (double)bf16_lo(w[e]), hi = (double)bf16_hi(w[e]);
            s += lo * lo; s += hi * hi;
        }
        s = sum16_f64(s);
        if (c16 == 0) {
            float nh = -3.0e38f;
            if (row < K) {
                nh = (float)(-0.5 * s);
                // upper bound of ||c||^2 in fp32 (one ulp up), kept as its bit pattern
                const float up = (float)s * (1.0f + 0x1p-22f);
                atomicMax(&smax, __float_as_uint(up));
            }
            const float hi = __uint_as_float(__float_as_uint(nh) & 0xffff0000u);
            const float r1 = nh - hi;
            const float mid = __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
            const float lo = __uint_as_float(__float_as_uint(r1 - mid) & 0xffff0000u);
            nh3[(int64_t)h * Kpad + row] =
                make_uint2((__float_as_uint(hi) >> 16) | (__float_as_uint(mid) & 0xffff0000u), __float_as_uint(lo) >> 16);
        }
    }
    __syncthreads();
    if (tid == 0) cmax_out[h] = __uint_as_float(smax);
}

// T rounds of Eq. 2 (b = 2: scale = max|r|, levels -1, 0, 1) on the 64 residuals r[] a lane
// holds of one token (channels 64*half ..), packed and stored as they are made.
// GL groups of NL elements lie inside the lane (B_ = 128: one group shared with the other half).
// TT > 0: the number of rounds is known at compile time (the loop unrolls, and the last round
// neither updates the residual nor takes the next maximum: a fifth of a round's instructions).
template <int B_, int TT>
__device__ __forceinline__ void quantize_token(float *r, int T, bool valid, int half, uint8_t *codes_tok,
                                               f16_t *scales_tok) {
    constexpr int G = kHeadDim / B_;                 // groups per token
    constexpr int GL = (B_ >= 64) ? 1 : 64 / B_;     // groups held by this lane
    constexpr int NL = (B_ >= 64) ? 64 : B_;         // elements per group in this lane
    auto round = [&](int t, auto last_k) {
        constexpr bool last = decltype(last_k)::value;
        uint32_t word[4];
        uint32_t sh[GL];
#pragma unroll
        for (int g = 0; g < GL; ++g) {
            float *rg = r + g * NL;
            float m = 0.0f;
#pragma unroll
            for (int i = 0; i < NL; i += 2) m = fmaxf(fmaxf(m, fabsf(rg[i])), fabsf(rg[i + 1]));
            if (B_ == 128) m = fmaxf(m, __shfl_xor(m, 32, 64));
            const float s32 = fminf(m, 65504.0f);
            sh[g] = f32_to_f16_bits(s32);
            const float sf = f16_bits_to_f32(sh[g]);
            const float inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
            // 8 levels -> one 16-bit field group: sum (q_i + 1) 4^i, exact in fp32.
            // |r / sf| <= 1 + 2^-11 unless the scale saturated, so the rounded level is already
            // in [-1, 1]; only a saturated group needs the clamp of Eq. 2.
            auto rounds = [&](auto clamp) {
#pragma unroll
                for (int o = 0; o < NL; o += 8) {
                    float cf = 21845.0f;             // 0x5555: the +1 of every field
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        float q = __builtin_rintf(rg[o + i] * inv);
                        if (decltype(clamp)::value) q = __builtin_amdgcn_fmed3f(q, -1.0f, 1.0f);
                        if (!last) rg[o + i] = __builtin_fmaf(-sf, q, rg[o + i]);
                        cf = __builtin_fmaf(q, (float)(1 << (2 * i)), cf);
                    }
                    const int e = g * NL + o;        // first channel (within the lane) of this field group
                    const uint32_t c16 = (uint32_t)cf;
                    if ((e >> 3) & 1) word[e >> 4] |= c16 << 16; else word[e >> 4] = c16;
                }
            };
            if (m > 65504.0f) rounds(BoolK<true>{}); else rounds(BoolK<false>{});
        }
        if (valid) {
            // word[] holds q + 1 per 2-bit field; the stored form is two's complement:
            // field 00 -> 11, 01 -> 00, 10 -> 01
#pragma unroll
            for (int wi = 0; wi < 4; ++wi) {
                const uint32_t lo = ~word[wi] & 0x55555555u;
                word[wi] = lo | (((~word[wi] >> 1) & lo) << 1);
            }
            *reinterpret_cast<uint4 *>(codes_tok + t * 32 + half * 16) = make_uint4(word[0], word[1], word[2], word[3]);
            f16_t *sp = scales_tok + t * G;
            if (B_ == 128) { if (half == 0) sp[0] = (f16_t)sh[0]; }
            else if (B_ == 64) sp[half] = (f16_t)sh[0];
            else if (B_ == 32)
                *reinterpret_cast<uint32_t *>(sp + half * 2) = sh[0] | (sh[GL - 1] << 16);
            else
                *reinterpret_cast<uint2 *>(sp + half * 4) =
                    make_uint2(sh[0] | (sh[1 % GL] << 16), sh[2 % GL] | (sh[3 % GL] << 16));
        }
    };
    if (TT > 0) {
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            if (t + 1 < TT) round(t, BoolK<false>{}); else round(t, BoolK<true>{});
        }
    } else {
        for (int t = 0; t < T; ++t) round(t, BoolK<false>{});
    }
}

// grid: x = unit, y = block of 256 * tiles_per_wave tokens.  With the unit as the fastest grid
// index and H a multiple of 8, all blocks of a unit run on one XCD and share its table in L2.
// T_: number of quantization rounds of the fused pass when known at compile time (0: a.T)
template <int B_, bool FUSED, bool NORMS_GIVEN, int T_>
__global__ __launch_bounds__(kAsgThreads, 2)
void assign_kernel(AssignArgs a, int Kpad, int tiles_per_wave) {
    constexpr bool norms_given = NORMS_GIVEN;
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t *lc = reinterpret_cast<bf16_t *>(smem);                       // [Kpad][kCPitch]
    bf16_t *lscr = lc + (size_t)Kpad * kCPitch;                          // [waves][128]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int h = blockIdx.x;
    const int K = a.K;
    const int64_t N = a.n_tokens;

    // ---- stage the centroid table (rows K.. are zero).  The norms either come from the
    // preparation kernel (norms_given: many workgroups per unit would each repeat the fp64 sums)
    // or are taken here while a row passes through (few workgroups per unit: one launch less): nh = fp32(-||c||^2 / 2) from an fp64 sum, split into three bf16 pieces by truncation
    // (8 significant bits each, so hi + mid + lo == nh exactly) that go into the row's padding;
    // rows K..Kpad-1 get a huge negative value so that they never win.  The largest ||c||^2 of the
    // unit (one ulp up) is needed for the error band of the certification.
    __shared__ uint32_t smax;
    if (tid == 0) smax = 0u;
    __syncthreads();
    const bf16_t *cg = a.cent + (int64_t)h * K * kHeadDim;
    // Eight 16-byte pieces per thread are requested before the first is used: taken one at a time
    // (load, store to LDS, norm) every piece waits a whole memory round trip (0.85 us measured),
    // which was most of what a workgroup with a single 256-token step spent on a 256-row table.
    constexpr int kStageBatch = 8;
    uint32_t up_max = 0u;          // this lane's largest ||c||^2 bound so far (bit pattern): one LDS atomic after the loop
    for (int i0 = tid; i0 < Kpad * 16; i0 += kAsgThreads * kStageBatch) {      // Kpad*16 is a multiple of the block: whole waves
        uint4 vb[kStageBatch];
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int i = i0 + u * kAsgThreads;
            const int row = i >> 4, c16 = i & 15;
            vb[u] = make_uint4(0u, 0u, 0u, 0u);
            if (i < Kpad * 16 && row < K) vb[u] = *reinterpret_cast<const uint4 *>(cg + (int64_t)row * kHeadDim + c16 * 8);
        }
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int i = i0 + u * kAsgThreads;
            if (i >= Kpad * 16) break;                                  // uniform
            const int row = i >> 4, c16 = i & 15;
            const uint4 v = vb[u];
            if (row < K && a.cent_copy && blockIdx.y == 0)              // the table's way out to the caller, for free
                *reinterpret_cast<uint4 *>(a.cent_copy + (int64_t)h * a.cent_copy_stride + (int64_t)row * kHeadDim + c16 * 8) = v;
            *reinterpret_cast<uint4 *>(lc + row * kCPitch + c16 * 8) = v;
            if (norms_given) continue;                                  // uniform
            double sq = 0.0;
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double lo = (double)bf16_lo(w[e]), hi = (double)bf16_hi(w[e]);
                sq += lo * lo; sq += hi * hi;
            }
            sq = sum16_f64(sq);
            if (c16 == 0) {
                float nh = -3.0e38f;
                if (row < K) {
                    nh = (float)(-0.5 * sq);
                    const float up = (float)sq * (1.0f + 0x1p-22f);      // upper bound of ||c||^2 in fp32, as its bit pattern
                    up_max = max(up_max, __float_as_uint(up));
                }
                const float hi = __uint_as_float(__float_as_uint(nh) & 0xffff0000u);
                const float r1 = nh - hi;
                const float mid = __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
                const float lo = __uint_as_float(__float_as_uint(r1 - mid) & 0xffff0000u);
                *reinterpret_cast<uint4 *>(lc + row * kCPitch + kHeadDim) =
                    make_uint4((__float_as_uint(hi) >> 16) | (__float_as_uint(mid) & 0xffff0000u), __float_as_uint(lo) >> 16, 0u, 0u);
            }
        }
    }
    if (!norms_given && up_max != 0u) atomicMax(&smax, up_max);
    if (norms_given)
        for (int row = tid; row < Kpad; row += kAsgThreads) {
            const uint2 p = a.nh3[(int64_t)h * Kpad + row];
            *reinterpret_cast<uint4 *>(lc + row * kCPitch + kHeadDim) = make_uint4(p.x, p.y, 0u, 0u);
        }
    __syncthreads();
    const float cmax = norms_given ? a.cmax[h] : __uint_as_float(smax);
    bf16_t *scr = lscr + wave * kHeadDim;
    // token operand of the extra MFMA step: three ones against (hi, mid, lo), lanes 0..31 only
    // 7 tag bits name a row among 256; with more rows the tag takes 8 (and the band below widens)
    const uint32_t tagbits = K > 256 ? 0xFFu : 0x7Fu;
    const uint32_t tagmask = vgpr_const(~tagbits);
    // +inf kept in a register the compiler cannot see through: med3(a, b, +inf) then stays one
    // instruction (as a constant it is rewritten into max(a, b) plus a NaN-quieting copy)
    const float pinf = __uint_as_float(vgpr_const(0x7f800000u));
    const uint4 ones = half ? make_uint4(0u, 0u, 0u, 0u) : make_uint4(0x3F803F80u, 0x00003F80u, 0u, 0u);

    const int64_t blk0 = (int64_t)blockIdx.y * tiles_per_wave * (kAsgWaves * kAsgTile);
    const bf16_t *xh = a.x + (int64_t)h * a.stride_head + half * 64;
    // this lane's 64 channels of its two tokens of a step (the MFMA B operands); a token past the
    // end of the chunk reads as zero
    auto load_x = [&](int64_t n0_, uint4 (&dst)[2][8]) {
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            const int64_t nn = n0_ + tb * 32 + col;
            const bf16_t *xp = xh + nn * a.stride_token;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                dst[tb][kk] = (nn < N) ? *reinterpret_cast<const uint4 *>(xp + kk * 8) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto step_start = [&](int k) {
        return k < tiles_per_wave ? blk0 + (int64_t)(k * kAsgWaves + wave) * kAsgTile : N;
    };
    // One step: 64 tokens.  Measured and left out, each without effect on the time of the pass:
    // requesting the next step's tokens a step ahead into a second register set; fetching the
    // tokens with whole rows per instruction through a staging area in LDS (each lane below reads
    // 16 bytes out of 64 different cache lines per instruction); more or fewer steps per workgroup.
    uint4 xa[2][8];
    for (int k = 0; k < tiles_per_wave; ++k) {
        const int64_t n0 = step_start(k);
        if (n0 >= N) break;                                  // uniform per wavefront
        load_x(n0, xa);
        int64_t n[2];
        bool valid[2];
        float xn[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            n[tb] = n0 + tb * 32 + col;
            valid[tb] = n[tb] < N;
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            float s = 0.0f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const uint32_t w[4] = {xa[tb][kk].x, xa[tb][kk].y, xa[tb][kk].z, xa[tb][kk].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bf16x2_t p = __builtin_bit_cast(bf16x2_t, w[e]);
                    s = __builtin_amdgcn_fdot2_f32_bf16(p, p, s, false);
                }
            }
            xn[tb] = s + __shfl_xor(s, 32, 64);
        }

        // ---- scores on the matrix cores, running top three per lane and token ----
        // Blocks of 32 centroids, software-pipelined: the MFMAs of block jb+1 are issued between
        // the VALU instructions that rank the scores of block jb (an MFMA occupies the matrix
        // pipe for 8 VALU issue slots), so one wavefront keeps both pipes busy.
        float b1[2] = {-INFINITY, -INFINITY}, b2[2] = {-INFINITY, -INFINITY}, b3[2] = {-INFINITY, -INFINITY};
        auto score_block = [&](int jb, floatx16_t (&acc)[2]) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc[0][r] = 0.0f; acc[1][r] = 0.0f; }
            const bf16_t *arow = lc + (jb * 32 + col) * kCPitch;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const bf16x8_t av = *reinterpret_cast<const bf16x8_t *>(arow + half * 64 + kk * 8);
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, xa[0][kk]), acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, __builtin_bit_cast(bf16x8_t, xa[1][kk]), acc[1], 0, 0, 0);
            }
            const bf16x8_t av = *reinterpret_cast<const bf16x8_t *>(arow + kHeadDim);
            const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, ones);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[1], 0, 0, 0);
        };
        auto rank_block = [&](int jb, const floatx16_t (&acc)[2]) {
            uint32_t tag0 = (uint32_t)jb << 4;
            asm volatile("" : "+s"(tag0));      // opaque: tag0 + r stays scalar arithmetic, the tag insert one v_and_or_b32
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // (score & ~0x7F) | tag: one v_and_or_b32, the tag is scalar arithmetic.
                    // max(a, b) is written med3(a, b, +inf): no NaN-quieting copy is needed.
                    const float v = __uint_as_float((__float_as_uint(acc[tb][r]) & tagmask) | (tag0 + r));
                    b3[tb] = __builtin_amdgcn_fmed3f(b2[tb], b3[tb], v);
                    b2[tb] = __builtin_amdgcn_fmed3f(b1[tb], b2[tb], v);
                    b1[tb] = __builtin_amdgcn_fmed3f(b1[tb], v, pinf);
                }
        };
        if (FUSED) {
            // the fused pass has no registers for a second set of accumulators
            floatx16_t acc[2];
            for (int jb = 0; jb < (Kpad >> 5); ++jb) { score_block(jb, acc); rank_block(jb, acc); }
        } else {
            // Software pipeline over groups of three k-steps (a block of 32 centroids is three
            // groups: 8 channel steps and the norm step).  The centroid operands of the NEXT group
            // are requested before the six MFMAs of the current one, whose issue slots are shared
            // with a third of the ranking of the PREVIOUS block; scheduling barriers keep each
            // part where it is written (left alone, the compiler reads every operand right
            // before its use and the LDS latency is exposed once per k-step).
            const int nb = Kpad >> 5;                    // even: Kpad is a multiple of 64
            floatx16_t accA[2], accB[2];
            bf16x8_t av[2][3];
            const bf16x8_t bones = __builtin_bit_cast(bf16x8_t, ones);
            auto load_group = [&](int jb, int g, bf16x8_t (&dst)[3]) {
                const bf16_t *arow = lc + (jb * 32 + col) * kCPitch;
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int kk = g * 3 + i;
                    dst[i] = *reinterpret_cast<const bf16x8_t *>(kk < 8 ? arow + half * 64 + kk * 8 : arow + kHeadDim);
                }
            };
            auto mfma_group = [&](int g, const bf16x8_t (&src)[3], floatx16_t (&acc)[2]) {
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    const int kk = g * 3 + i;
                    if (kk == 0) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) { acc[0][r] = 0.0f; acc[1][r] = 0.0f; }
                    }
                    const bf16x8_t b0 = kk < 8 ? __builtin_bit_cast(bf16x8_t, xa[0][kk < 8 ? kk : 0]) : bones;
                    const bf16x8_t b1 = kk < 8 ? __builtin_bit_cast(bf16x8_t, xa[1][kk < 8 ? kk : 0]) : bones;
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(src[i], b0, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(src[i], b1, acc[1], 0, 0, 0);
                }
            };
            // scores 11 c .. 11 c + 10 (of 32: 16 per token block) of a finished block
            auto rank_part = [&](int jb, const floatx16_t (&acc)[2], int c) {
                uint32_t tag0 = (uint32_t)jb << 4;
                asm volatile("" : "+s"(tag0));  // opaque, see rank_block
#pragma unroll
                for (int sidx = 11 * c; sidx < (c == 2 ? 32 : 11 * c + 11); ++sidx) {
                    const int tb = sidx >> 4, r = sidx & 15;
                    const float v = __uint_as_float((__float_as_uint(acc[tb][r]) & tagmask) | (tag0 + r));
                    b3[tb] = __builtin_amdgcn_fmed3f(b2[tb], b3[tb], v);
                    b2[tb] = __builtin_amdgcn_fmed3f(b1[tb], b2[tb], v);
                    b1[tb] = __builtin_amdgcn_fmed3f(b1[tb], v, pinf);
                }
            };
            auto interleave6 = [&]() {
#pragma unroll
                for (int i = 0; i < 6; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);
                }
            };
            // one block: its three groups; `prev` (if any) is ranked in their shadow; the operands
            // of the group after the current one are requested first (next_jb < 0: none)
            auto block_step = [&](int jb, floatx16_t (&acc)[2], int prev_jb, const floatx16_t (&prev)[2],
                                  int parity, bool more) {
#pragma unroll
                for (int g = 0; g < 3; ++g) {
                    const int cur = (parity + g) & 1;
                    if (g < 2) load_group(jb, g + 1, av[cur ^ 1]);
                    else if (more) load_group(jb + 1, 0, av[cur ^ 1]);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_group(g, av[cur], acc);
                    if (prev_jb >= 0) { rank_part(prev_jb, prev, g); interleave6(); }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            load_group(0, 0, av[0]);
            block_step(0, accA, -1, accB, 0, true);                 // groups 0..2: parities 0, 1, 0
            for (int jb = 1; jb + 1 < nb; jb += 2) {
                block_step(jb, accB, jb - 1, accA, 1, true);        // groups 3..5: parities 1, 0, 1
                block_step(jb + 1, accA, jb, accB, 0, true);
            }
            block_step(nb - 1, accB, nb - 2, accA, 1, false);
            rank_block(nb - 1, accB);
        }
        // tag -> centroid index: row 8*(r/4) + 4*half + r%4 of block jb
        auto tag_to_idx = [&](float v) {
            const uint32_t t = __float_as_uint(v) & tagbits;
            return (int)((t >> 4) * 32 + ((t >> 2) & 3) * 8 + half * 4 + (t & 3));
        };
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            if (n0 + tb * 32 >= N) break;                        // uniform: second block past the end
            float c1 = b1[tb], c2 = b2[tb], c3 = b3[tb];
            int i1 = tag_to_idx(c1), i2 = tag_to_idx(c2);
            {   // merge with the other half of the wavefront (same token, other centroids)
                const float p1 = __shfl_xor(c1, 32, 64), p2 = __shfl_xor(c2, 32, 64),
                            p3 = __shfl_xor(c3, 32, 64);
                const int q1 = __shfl_xor(i1, 32, 64), q2 = __shfl_xor(i2, 32, 64);
                insert3(p1, q1, c1, c2, c3, i1, i2);
                insert3(p2, q2, c1, c2, c3, i1, i2);
                insert3(p3, 0, c1, c2, c3, i1, i2);
            }
            const float thr = (K > 256 ? 0x1.8p-14f : 0x1p-14f) * (0.5f * xn[tb] + cmax);
            int id = i1;
            const bool amb = valid[tb] && (i2 < K) && !(c1 - c2 > thr);
            const bool full = !(c1 - c3 > thr);

            // ---- fp64 re-evaluation of tokens the fp32 scores cannot decide ----
            uint64_t mask = __ballot(amb) & 0xffffffffull;
            while (mask) {
                const int tk = __builtin_ctzll(mask);
                mask &= mask - 1;
                if (col == tk) {
#pragma unroll
                    for (int kk = 0; kk < 8; ++kk)
                        *reinterpret_cast<uint4 *>(scr + half * 64 + kk * 8) = xa[tb][kk];
                }
                __builtin_amdgcn_wave_barrier();
                // the token's lane index is wave-uniform: plain lane reads, no exchange through LDS
                const int d1 = __builtin_amdgcn_readlane(i1, tk), d2 = __builtin_amdgcn_readlane(i2, tk);
                const int fl = __builtin_amdgcn_readlane((int)full, tk);
                int winner;
                if (!fl) {
                    const int cand = half ? d2 : d1;
                    const uint2 xv = *reinterpret_cast<const uint2 *>(scr + col * 4);
                    const uint2 cv = *reinterpret_cast<const uint2 *>(lc + cand * kCPitch + col * 4);
                    const double e0 = (double)bf16_lo(xv.x) - (double)bf16_lo(cv.x);
                    const double e1 = (double)bf16_hi(xv.x) - (double)bf16_hi(cv.x);
                    const double e2 = (double)bf16_lo(xv.y) - (double)bf16_lo(cv.y);
                    const double e3 = (double)bf16_hi(xv.y) - (double)bf16_hi(cv.y);
                    double d = e0 * e0; d += e1 * e1; d += e2 * e2; d += e3 * e3;
                    // the 32 lanes of a candidate: two rows of 16 summed by DPP moves, the two row
                    // sums read as scalars (no exchange through LDS: each cost a round trip, ten
                    // in a row per token).  Both candidates go through the same operations, so
                    // equal rows give equal sums.
                    d = sum16_f64(d);
                    const double D1 = readlane_f64(d, 0) + readlane_f64(d, 16);
                    const double D2 = readlane_f64(d, 32) + readlane_f64(d, 48);
                    winner = (D2 < D1 || (D2 == D1 && d2 < d1)) ? d2 : d1;
                } else {
                    double bd = INFINITY; int bj = 0x7fffffff;
                    for (int j = lane; j < K; j += 64) {
                        const bf16_t *cr = lc + j * kCPitch;
                        double acc = 0.0;
                        for (int c = 0; c < kHeadDim; c += 2) {
                            const uint32_t xw = *reinterpret_cast<const uint32_t *>(scr + c);
                            const uint32_t cw = *reinterpret_cast<const uint32_t *>(cr + c);
                            const double f0 = (double)bf16_lo(xw) - (double)bf16_lo(cw);
                            acc += f0 * f0;
                            const double f1 = (double)bf16_hi(xw) - (double)bf16_hi(cw);
                            acc += f1 * f1;
                        }
                        if (acc < bd) { bd = acc; bj = j; }
                    }
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1) {
                        const double od = shfl_xor_f64(bd, off);
                        const int oj = __shfl_xor(bj, off, 64);
                        if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
                    }
                    winner = bj;
                }
                if (col == tk) id = winner;
                __builtin_amdgcn_wave_barrier();
            }

            const int64_t hn = (int64_t)h * a.out_stride + n[tb];
            if (valid[tb] && half == 0) store_id(a.ids, hn * a.ids_step + a.ids_off, a.id_wide, (uint32_t)id);
            if (!FUSED) continue;

            // ---- Eq. 5: residual against the assigned centroid, then the T rounds ----
            float r[64];
            const bf16_t *crow = lc + id * kCPitch + half * 64;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const uint4 cv = *reinterpret_cast<const uint4 *>(crow + kk * 8);
                const uint32_t xw[4] = {xa[tb][kk].x, xa[tb][kk].y, xa[tb][kk].z, xa[tb][kk].w};
                const uint32_t cw[4] = {cv.x, cv.y, cv.z, cv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    r[kk * 8 + 2 * e] = bf16_lo(xw[e]) - bf16_lo(cw[e]);
                    r[kk * 8 + 2 * e + 1] = bf16_hi(xw[e]) - bf16_hi(cw[e]);
                }
            }
            const int T = T_ > 0 ? T_ : a.T;
            quantize_token<B_, T_>(r, T, valid[tb], half, a.codes + hn * T * 32, a.scales + hn * T * (kHeadDim / B_));
            __builtin_amdgcn_sched_barrier(0);       // keep the two tokens' passes apart: each needs most registers
        }
    }
}

static size_t assign_smem_bytes(int Kpad) {
    return (size_t)Kpad * kCPitch * 2 + (size_t)kAsgWaves * kHeadDim * 2;
}

template <int B_, bool FUSED, int T_>
static hipError_t launch_assign_t(const AssignArgs &a, hipStream_t s) {
    const int Kpad = (a.K + 63) & ~63;
    const size_t smem = assign_smem_bytes(Kpad);
    static LdsHighWater lds_limit[2] = {};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(&assign_kernel<B_, FUSED, true, T_>), smem, lds_limit[0]);
    if (e != hipSuccess) return e;
    e = ensure_dynamic_lds(reinterpret_cast<const void *>(&assign_kernel<B_, FUSED, false, T_>), smem, lds_limit[1]);
    if (e != hipSuccess) return e;
    // tokens per workgroup: 256 per step; more steps per workgroup amortise the table staging
    // once there are enough workgroups to fill the chip several times over
    const int64_t steps = (a.n_tokens + kAsgWaves * kAsgTile - 1) / (kAsgWaves * kAsgTile);
    int tpw = 1;
    while (tpw < 4 && (steps / (2 * tpw)) * a.H >= 2048) tpw *= 2;
    const int64_t gy = (steps + tpw - 1) / tpw;
    if (gy > 65535) return hipErrorInvalidValue;
    // the centroid norms: by a kernel of their own when there are many workgroups (each would
    // repeat the fp64 sums of its unit's table); inside the assignment kernel when there are few
    // (the extra launch then costs more than the repeated sums: 0.165 -> 0.154 ms per cfg2 encode;
    // the bound scales with the table size, measured at K = 64 and K = 512)
    const bool norms_given = (int64_t)a.H * gy * a.K > 2048 * 64;
    if (norms_given) {
        hipLaunchKernelGGL(centroid_prep_kernel, dim3((unsigned)a.H), dim3(kPrepThreads), 0, s, a.cent, a.K, Kpad,
                           a.nh3, a.cmax);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (norms_given)
        hipLaunchKernelGGL((assign_kernel<B_, FUSED, true, T_>), dim3((unsigned)a.H, (unsigned)gy), dim3(kAsgThreads), smem, s, a,
                           Kpad, tpw);
    else
        hipLaunchKernelGGL((assign_kernel<B_, FUSED, false, T_>), dim3((unsigned)a.H, (unsigned)gy), dim3(kAsgThreads), smem, s, a,
                           Kpad, tpw);
    return hipGetLastError();
}

// the fused pass with the round count of the measured configurations fixed at compile time
// (group 64: 1, 2 and 4 rounds; group 32: 3), any other count at run time
template <int B_>
static hipError_t launch_fused(const AssignArgs &a, hipStream_t s) {
    if (B_ == 64 && a.T == 1) return launch_assign_t<B_, true, (B_ == 64 ? 1 : 0)>(a, s);
    if (B_ == 64 && a.T == 2) return launch_assign_t<B_, true, (B_ == 64 ? 2 : 0)>(a, s);
    if (B_ == 64 && a.T == 4) return launch_assign_t<B_, true, (B_ == 64 ? 4 : 0)>(a, s);
    if (B_ == 32 && a.T == 3) return launch_assign_t<B_, true, (B_ == 32 ? 3 : 0)>(a, s);
    return launch_assign_t<B_, true, 0>(a, s);
}

hipError_t launch_assign(const AssignArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    if (!a.fused) return launch_assign_t<64, false, 0>(a, s);
    switch (a.B) {
        case 16: return launch_fused<16>(a, s);
        case 32: return launch_fused<32>(a, s);
        case 64: return launch_fused<64>(a, s);
        default: return launch_fused<128>(a, s);
    }
}

size_t assign_workspace_bytes(int H, int K) {
    const size_t Kpad = (size_t)((K + 63) & ~63);
    return ((size_t)H * Kpad * sizeof(uint2) + 255) / 256 * 256 + ((size_t)H * sizeof(float) + 255) / 256 * 256;
}
void assign_workspace_split(void *ws, int H, int K, uint2 **nh3, float **cmax) {
    const size_t Kpad = (size_t)((K + 63) & ~63);
    *nh3 = static_cast<uint2 *>(ws);
    *cmax = reinterpret_cast<float *>(static_cast<unsigned char *>(ws) + ((size_t)H * Kpad * sizeof(uint2) + 255) / 256 * 256);
}

}  // namespace qvg
