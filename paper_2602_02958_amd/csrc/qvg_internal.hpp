// Internal declarations shared by the HIP translation units of libqvg.
// Device helpers for the number formats and the launchers each .hip file defines.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qvg.h"

namespace qvg {

constexpr int kHeadDim = 128;      // only head_dim the kernels are written for
constexpr int kMaxStages = 8;
constexpr int kMaxSmooth = 4;       // smoothing stages (k-means rounds on the residual)
constexpr int kMaxTokensPerChunk = 1 << 20;
constexpr int kMaxClusters = 512;   // up to 256: one id byte per token and stage; beyond: two

typedef uint16_t bf16_t;           // bit pattern of a bfloat16
typedef uint16_t f16_t;            // bit pattern of an IEEE binary16

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2_t;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 halfx8_t;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 halfx2_t;

// ---- number formats -------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
// two fp32 -> packed bf16 (lo in bits 0..15), round to nearest even: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// two fp32 -> packed f16, round toward zero (saturates instead of overflowing): v_cvt_pkrtz_f16_f32
__device__ __forceinline__ uint32_t pack_f16x2_rtz(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}
// two fp32 -> packed f16, round to nearest even: v_cvt_pk_f16_f32 (values beyond 65504 become infinite)
__device__ __forceinline__ uint32_t pack_f16x2_rne(float lo, float hi) {
    const floatx2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, halfx2_t));
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {       // RNE (default mode)
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}

// ---- dequantization helpers shared by the decode and the fused attention kernels ----
__device__ __forceinline__ void unpack_bf16x8(const uint4 &c, float *acc) {
    acc[0] = bf16_lo(c.x); acc[1] = bf16_hi(c.x); acc[2] = bf16_lo(c.y); acc[3] = bf16_hi(c.y);
    acc[4] = bf16_lo(c.z); acc[5] = bf16_hi(c.z); acc[6] = bf16_lo(c.w); acc[7] = bf16_hi(c.w);
}
__device__ __forceinline__ uint4 pack_bf16x8(const float *acc) {
    return make_uint4(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                      pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7]));
}
// half of an f16 scale as fp32 (exact): the extracted levels below are 2q, not q
__device__ __forceinline__ float half_scale(uint32_t f16bits) { return 0.5f * f16_bits_to_f32(f16bits); }

// A 2-bit two's complement level (sign, nonzero) moved to bits 15..14 of a 16-bit half IS the
// f16 number 2q: 0b11 -> 0xC000 = -2, 0b01 -> 0x4000 = +2, 0b00 -> 0.  One shift and one mask
// therefore turn the fields at the same position of both halves of a 32-bit word into two f16
// operands, which v_fma_mix_f32 consumes directly: (s/2) * (2q) + acc, one rounding, the same
// value as fma(s, q, acc).  w = codes of stage t (low half) and stage t+1 (high half) of one
// token's 8 channels.
__device__ __forceinline__ void add_two_stages(float *acc, uint32_t w, float hs0, float hs1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const halfx2_t y = __builtin_bit_cast(halfx2_t, (w << (14 - 2 * i)) & 0xC000C000u);
        acc[i] = __builtin_fmaf(hs0, (float)y[0], acc[i]);
        acc[i] = __builtin_fmaf(hs1, (float)y[1], acc[i]);
    }
}
// w = codes of the same (last) stage of two different tokens: low half -> accA, high half -> accB.
__device__ __forceinline__ void add_last_stage_of_two_rows(float *accA, float *accB, uint32_t w,
                                                           float hsA, float hsB) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const halfx2_t y = __builtin_bit_cast(halfx2_t, (w << (14 - 2 * i)) & 0xC000C000u);
        accA[i] = __builtin_fmaf(hsA, (float)y[0], accA[i]);
        accB[i] = __builtin_fmaf(hsB, (float)y[1], accB[i]);
    }
}

// ---- cluster ids: bytes, or 16-bit words when the table has more than 256 rows ("wide") ----
__device__ __forceinline__ uint32_t load_id(const uint8_t *ids, int64_t i, int wide) {
    return wide ? (uint32_t)reinterpret_cast<const uint16_t *>(ids)[i] : (uint32_t)ids[i];
}
__device__ __forceinline__ void store_id(uint8_t *ids, int64_t i, int wide, uint32_t id) {
    if (wide) reinterpret_cast<uint16_t *>(ids)[i] = (uint16_t)id;
    else ids[i] = (uint8_t)id;
}

// ---- stored formats ---------------------------------------------------------
// fmt bit 0: scales are FP8 E4M3 bytes (else binary16); bit 1: 4-bit levels (else 2-bit)
constexpr int kFmtE4M3 = 1;
constexpr int kFmtInt4 = 2;

// E4M3 code of a non-negative scale (1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
// largest finite 448, subnormals m/8 * 2^-6) -> fp32, exact
__device__ __forceinline__ float e4m3_bits_to_f32(uint32_t b) {
    const float normal = __uint_as_float(((b & 0x7fu) << 20) + (120u << 23));
    return (b & 0x78u) ? normal : (float)(b & 7u) * 0x1p-9f;
}
// non-negative finite fp32 -> E4M3 code, round to nearest even, saturating at 448
__device__ __forceinline__ uint32_t f32_to_e4m3_bits(float a) {
    a = fminf(a, 448.0f);
    uint32_t u = __float_as_uint(a);
    u += 0x7ffffu + ((u >> 20) & 1u);                 // nearest even at 3 mantissa bits
    const uint32_t normal = (u >> 20) - (120u << 3);
    // below 2^-6 the grid is uniform with step 2^-9; 8 steps are the smallest normal, code 8
    return (a < 0x1p-6f) ? (uint32_t)__builtin_rintf(a * 512.0f) : normal;
}
template <bool FP8>
__device__ __forceinline__ float scale_bits_to_f32(uint32_t bits) {
    return FP8 ? e4m3_bits_to_f32(bits) : f16_bits_to_f32(bits);
}
// eight 4-bit two's complement levels of w (channel i in bits 4i..4i+3): acc += s * q
__device__ __forceinline__ void add_stage_int4(float *acc, uint32_t w, float s) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int q = ((int)(w << (28 - 4 * i))) >> 28;          // v_bfe_i32
        acc[i] = __builtin_fmaf(s, (float)q, acc[i]);
    }
}

// Raise a kernel's dynamic-LDS limit to `bytes` unless an earlier call on this device already raised
// it that far: the attribute belongs to the function (per device), not to the launch.  `mark` is a
// static of the calling launcher instance (one per kernel instance); a race between two first
// calls only sets the attribute twice.
struct LdsHighWater { size_t bytes[32]; };
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes, LdsHighWater &mark) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 32;
    if (tracked && bytes <= mark.bytes[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && tracked) mark.bytes[dev] = bytes;
    return e;
}

// ---- launchers (each returns a hipError_t from hipGetLastError) -----------
struct DecodeArgs {
    const bf16_t *cent; const uint8_t *ids; const uint8_t *codes; const f16_t *scales;
    bf16_t *out; int64_t n_tokens; int64_t chunk_len; int n_chunks; int H; int K; int B; int T;
    int64_t stride_head, stride_token;
    int S;      // smoothing stages: cent [H][n_chunks][S][K][d], ids [H][N][S]
    int fmt;    // kFmt* bits; scales then points at bytes, codes rows are 64 B per round with 4-bit levels
    int64_t kv_stride;     // tokens between consecutive units in ids / codes / scales (>= n_tokens)
    int chunk_stride;      // chunk tables between consecutive units in cent (>= n_chunks)
    int id_wide;           // ids are 16-bit words (K > 256)
};
hipError_t launch_decode(const DecodeArgs &a, hipStream_t s);

struct AssignArgs {
    const bf16_t *x; int64_t stride_head, stride_token; int64_t n_tokens;
    const bf16_t *cent; int H; int K; int B; int T;
    uint8_t *ids;            // always written
    uint8_t *codes; f16_t *scales;   // written when fused != 0
    int64_t out_stride;      // tokens between consecutive units in ids / codes / scales
    int ids_step, ids_off;   // a token has ids_step id bytes; this pass writes byte ids_off (smoothing stage)
    int fused;
    uint2 *nh3; float *cmax; // scratch of assign_workspace_bytes(H, K): split -||c||^2/2 per row, max ||c||^2 per unit
    bf16_t *cent_copy; int64_t cent_copy_stride;   // optional: the table also goes here, unit h at h * stride elements
                                                   // (written by the unit's first workgroup while it stages the table)
    int id_wide;             // ids are 16-bit words (K > 256)
};
// launches the centroid preparation and the assignment (fused with quantization when a.fused)
hipError_t launch_assign(const AssignArgs &a, hipStream_t s);
size_t assign_workspace_bytes(int H, int K);
void assign_workspace_split(void *ws, int H, int K, uint2 **nh3, float **cmax);

struct UpdateArgs {
    const bf16_t *x; int64_t stride_head, stride_token; int64_t n_tokens;
    const uint8_t *ids; int64_t ids_stride;      // tokens between consecutive units in ids
    int ids_step, ids_off;                       // id bytes per token, byte read by this pass
    const bf16_t *cent_prev; bf16_t *cent_out; int32_t *counts_out;
    int32_t *perm; int32_t *offsets;     // workspace: [H][N] and [H][K+1]
    int H; int K;
    int id_wide;                         // ids are 16-bit words (K > 256)
};
hipError_t launch_update(const UpdateArgs &a, hipStream_t s);

// out[h][n][:] = bf16( x[h][n][:] - cent[h][ids[h][n]][:] ), one fp32 subtraction (Eq. 5), for the
// next smoothing stage.  out is dense [H][N][128].
struct ResidualArgs {
    const bf16_t *x; int64_t stride_head, stride_token; int64_t n_tokens;
    const bf16_t *cent; const uint8_t *ids; int64_t ids_stride; int ids_step, ids_off;
    bf16_t *out; int H; int K; int id_wide;
};
hipError_t launch_residual(const ResidualArgs &a, hipStream_t s);

// Eq. 5 and the T rounds of Eq. 2 for a given assignment, for every stored format (the fused
// assignment kernel covers 2-bit levels with binary16 scales only).
struct QuantArgs {
    const bf16_t *x; int64_t stride_head, stride_token; int64_t n_tokens;
    const bf16_t *cent;                    // [H][K][d]
    const uint8_t *ids; int ids_step, ids_off;
    uint8_t *codes; void *scales; int64_t out_stride;     // tokens between units in ids / codes / scales
    int H; int K; int B; int T; int fmt; int id_wide;
};
hipError_t launch_quantize(const QuantArgs &a, hipStream_t s);

struct AttnArgs {
    const bf16_t *q; bf16_t *out; float *lse; int64_t n_q; int64_t n_kv; int64_t chunk_len;
    int n_chunks; int H; int K; int B; int T; float scale;
    const bf16_t *k_cent; const uint8_t *k_ids; const uint8_t *k_codes; const f16_t *k_scales;
    const bf16_t *v_cent; const uint8_t *v_ids; const uint8_t *v_codes; const f16_t *v_scales;
    int S;      // smoothing stages, layouts as in DecodeArgs
    int fmt;    // kFmt* bits, as in DecodeArgs
    int64_t kv_stride;     // tokens between consecutive units in ids / codes / scales (>= n_kv)
    int chunk_stride;      // chunk tables between consecutive units in the centroid arrays (>= n_chunks)
    const f16_t *rope;     // [n_kv][d/2][2] (cos, sin) applied to the decoded keys, or nullptr
    int id_wide;           // ids are 16-bit words (K > 256)
    const int32_t *q_len;  // [n_q] prefix length per query (clamped to 0 .. n_kv), or nullptr: all n_kv tokens
    float *out_f32;        // when set, the result goes here as fp32 [H][n_q][d] (not rounded to bf16) and `out` is not written
};
hipError_t launch_attn(const AttnArgs &a, hipStream_t s);
// The same attention with every tile decoded once per unit into a caller-lent workspace and shared
// by all query blocks (qvg_attn_slab.hip).  Workspace = running state of the queries (only when the
// cache needs more than one slab) + the operand images of a slab of whole chunks.
size_t attn_slab_state_bytes(int H, int64_t n_q);
size_t attn_slab_chunk_bytes(int H, int64_t chunk_len);
bool attn_slab_applicable(const AttnArgs &a, const void *ws, size_t ws_bytes);
hipError_t launch_attn_slab(const AttnArgs &a, void *ws, size_t ws_bytes, hipStream_t s);

// Rotary embedding of one lane's 8 decoded key channels (4 interleaved pairs): the values are
// first rounded to bf16 (what the stand-alone decoder stores), then each pair (x0, x1) becomes
// (x0 cos - x1 sin, x0 sin + x1 cos), one fp32 product and one fma per output.
// rp: the lane's 4 (cos, sin) binary16 pairs.
__device__ __forceinline__ void rope_rotate8(float *acc, const uint4 &rp) {
    const uint32_t w[4] = {rp.x, rp.y, rp.z, rp.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t pk = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
        const float x0 = bf16_lo(pk), x1 = bf16_hi(pk);
        const halfx2_t cs = __builtin_bit_cast(halfx2_t, w[i]);
        const float c = (float)cs[0], sn = (float)cs[1];
        const float t0 = x1 * sn, t1 = x1 * c;
        acc[2 * i] = __builtin_fmaf(x0, c, -t0);
        acc[2 * i + 1] = __builtin_fmaf(x0, sn, t1);
    }
}

// Merge of two partial attention results over disjoint key sets (rows of d = 128 channels)
struct MergeArgs {
    const bf16_t *oa; const float *lsea; const bf16_t *ob; const float *lseb;
    bf16_t *out; float *lse; int64_t rows;
};
hipError_t launch_attn_merge(const MergeArgs &a, hipStream_t s);

}  // namespace qvg
