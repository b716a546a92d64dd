// Pieces shared by the attention kernels that read the compressed cache: the tile walk over the
// chunks, what a thread loads for its part of a 64-token tile, the dequantization of Eq. 7 on
// those values, and the epilogue that normalises and stores a query's result.
#pragma once
#include <type_traits>

#include "qvg_internal.hpp"

namespace qvg {

constexpr int kAtThreads = 512;
constexpr int kAtWaves = kAtThreads / 64;
constexpr int kAtQPerBlock = 32 * kAtWaves;     // 256
constexpr int kAtKv = 64;
constexpr int kKtPitch = 136;      // bf16 per row of the K tile (272 B, 16-byte aligned, conflict-free)
constexpr int kVtPitch = 72;       // f16 per row of the transposed V tile (144 B)
constexpr int kKtElems = kAtKv * kKtPitch;
constexpr int kVtElems = kHeadDim * kVtPitch;
constexpr size_t kAtSmem = (size_t)2 * (kKtElems + kVtElems) * sizeof(uint16_t);

// acc + the eight f16 values of v, accumulated in fp32 (v_dot2_f32_f16 against ones)
__device__ __forceinline__ float sum_f16_pairs(const uint4 &v, float acc) {
    const halfx2_t ones = {(_Float16)1.0f, (_Float16)1.0f};
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2_t, v.x), ones, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2_t, v.y), ones, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2_t, v.z), ones, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2_t, v.w), ones, acc, false);
    return acc;
}

struct CacheSide {                 // one of K / V, already offset to this unit
    const bf16_t *cent;            // [n_chunks][K][d]
    const uint8_t *ids; const uint8_t *codes;
    const uint8_t *scales;         // binary16 or E4M3 bytes, per the format
    int wide;                      // ids are 16-bit words (more than 256 centroids)
};

struct Tile {                      // one 64-token tile; tiles never straddle a chunk
    int chunk; int t0, cend; bool valid;     // token indices fit 31 bits (checked by the caller)
};

struct Span {                      // the part of the cache a workgroup walks
    int64_t chunk_len, n_kv; int n_chunks;
};
__device__ __forceinline__ Span span_of(const AttnArgs &a) {
    Span s; s.chunk_len = a.chunk_len; s.n_kv = a.n_kv; s.n_chunks = a.n_chunks;
    return s;
}
__device__ __forceinline__ Tile first_tile(const Span &a) {
    Tile t;
    t.chunk = 0; t.t0 = 0; t.cend = (int)(a.chunk_len < a.n_kv ? a.chunk_len : a.n_kv); t.valid = true;
    return t;
}
__device__ __forceinline__ Tile next_tile(const Span &a, Tile t) {
    t.t0 += kAtKv;
    if (t.t0 >= t.cend) {
        t.chunk += 1;
        if (t.chunk >= a.n_chunks) { t.valid = false; t.chunk = a.n_chunks - 1; }
        else {
            const int64_t b = (int64_t)t.chunk * a.chunk_len;
            t.t0 = (int)b;
            t.cend = (int)((b + a.chunk_len < a.n_kv) ? b + a.chunk_len : a.n_kv);
        }
    }
    return t;
}

// Normalise and store one query's result: the lane holds channels 32*mb + 8*g + 4*half + 0..3 of its
// query.  bf16 (round to nearest even), or fp32 when a.out_f32 is set.  A query that saw no token
// at all (prefix length 0) gets a zero row and a log-sum-exp of -inf, which qvg_attn_merge takes
// as a weightless partial result.
__device__ __forceinline__ void store_result(const AttnArgs &a, int h, int64_t qrow, bool seen, bool qvalid,
                                             int half, const floatx16_t (&O)[4], float m, float l) {
    const float ltot = l + __shfl_xor(l, 32, 64);
    if (!qvalid) return;
    const float inv = seen ? 1.0f / ltot : 0.0f;
    const int64_t row = ((int64_t)h * a.n_q + qrow) * kHeadDim + half * 4;
    if (a.out_f32) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                float4 o;
                o.x = seen ? O[mb][4 * gq + 0] * inv : 0.0f; o.y = seen ? O[mb][4 * gq + 1] * inv : 0.0f;
                o.z = seen ? O[mb][4 * gq + 2] * inv : 0.0f; o.w = seen ? O[mb][4 * gq + 3] * inv : 0.0f;
                *reinterpret_cast<float4 *>(a.out_f32 + row + mb * 32 + gq * 8) = o;
            }
    } else {
        bf16_t *op = a.out + row;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const uint2 o = seen ? make_uint2(
                    pack_bf16x2(O[mb][4 * gq + 0] * inv, O[mb][4 * gq + 1] * inv),
                    pack_bf16x2(O[mb][4 * gq + 2] * inv, O[mb][4 * gq + 3] * inv)) : make_uint2(0u, 0u);
                *reinterpret_cast<uint2 *>(op + mb * 32 + gq * 8) = o;
            }
    }
    if (a.lse && half == 0)
        a.lse[(int64_t)h * a.n_q + qrow] = seen ? (m + __builtin_log2f(ltot)) * 0.6931471805599453f : -INFINITY;
}

// SM: how the smoothing stages are handled.  1: a single stage; 0: several, their number known at
// run time only (the rows are added as they arrive, which waits for every load where it is
// issued); 2..kMaxSmooth: that many stages, fixed at compile time (the rows stay packed in
// registers while the loads are in flight and are added, in stage order, when the tile is decoded).
template <int TM, int SM = 1>
struct Raw {                       // what one thread loads for its 2 tokens x 8 channels of one side
    uint32_t code[2][TM], sc[2][TM];
    uint4 cen[2];                  // one smoothing stage: the centroid row (8 bf16)
    float ci[2][8];                // SM == 0: the rows added in stage order (fp32)
    uint4 rows[2][SM > 1 ? SM : 1];     // SM > 1: the stages' rows
};

// ids of this thread's two tokens of a tile (0 for tokens past the chunk end / an invalid tile);
// with S smoothing stages a token has S id bytes, stage s in byte s of the result
// (ids of 16 bits, for tables of more than 256 rows: one stage here; with several stages the
// run-time-count path of load_raw reads them itself)
// The ids of a thread's two tokens, as stored: one load per token (the S id bytes of a token
// are contiguous; 1, 2 or 4 of them are one load when the array is aligned for it) and no
// arithmetic on what it returns.  The clamp to the table's last row is applied where the id is
// used (load_raw): applied here, every tile waited for the ids right after requesting them,
// and, the load counter being in order, for the codes, scales and rows requested just before.
// A token that does not exist reads the unit's token 0 instead (it exists), so that the load
// needs no branch; load_raw never uses such an id.
__device__ __forceinline__ void load_ids(const CacheSide &s, const Tile &t, int tp, int S,
                                         int wide, uint32_t id[2]) {
    const bool al = ((uintptr_t)s.ids & (uintptr_t)(S - 1)) == 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int n0 = t.t0 + 2 * tp + e;
        const int64_t n = (t.valid && n0 < t.cend) ? n0 : 0;
        if (wide) id[e] = load_id(s.ids, n, 1);
        else if (S == 1) id[e] = s.ids[n];
        else if (S == 2 && al) id[e] = *reinterpret_cast<const uint16_t *>(s.ids + n * 2);
        else if (S == 4 && al) id[e] = *reinterpret_cast<const uint32_t *>(s.ids + n * 4);
        else {
            id[e] = 0u;
            for (int st = 0; st < S; ++st) id[e] |= (uint32_t)s.ids[n * S + st] << (8 * st);
        }
    }
}

// FMT: stored format (kFmt* bits); with 4-bit levels a thread's 8 channels of a round are one
// 32-bit word, else one 16-bit word
template <int T_, int TM, int SM, int FMT>
__device__ __forceinline__ void load_raw(const CacheSide &s, const Tile &t, int tp, int c8, int T,
                                         int G, int g, int K, int S, const uint32_t id[2], Raw<TM, SM> &r) {
    const bf16_t *cent = s.cent + (int64_t)t.chunk * S * K * kHeadDim;      // [S][K][d] of this chunk
    const uint32_t kmax = (uint32_t)K - 1u;        // ids are clamped to the table's last row
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int n = t.t0 + 2 * tp + e;
        const bool ok = t.valid && n < t.cend;
#pragma unroll
        for (int k = 0; k < TM; ++k) { r.code[e][k] = 0u; r.sc[e][k] = 0u; }
        r.cen[e] = make_uint4(0u, 0u, 0u, 0u);
        if (SM == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) r.ci[e][i] = 0.0f;
        }
        if (SM > 1) {
#pragma unroll
            for (int st = 0; st < SM; ++st) r.rows[e][st] = make_uint4(0u, 0u, 0u, 0u);
        }
        if (ok) {
            constexpr bool FP8 = (FMT & kFmtE4M3) != 0, I4 = (FMT & kFmtInt4) != 0;
            typedef typename std::conditional<I4, uint32_t, uint16_t>::type code_t;
            typedef typename std::conditional<FP8, uint8_t, f16_t>::type scale_t;
            const code_t *cp = reinterpret_cast<const code_t *>(s.codes + (int64_t)n * T * (I4 ? 64 : 32)) + c8;
            const scale_t *sp = reinterpret_cast<const scale_t *>(s.scales) + (int64_t)n * T * G + g;
#pragma unroll
            for (int k = 0; k < TM; ++k)
                if (k < T) { r.code[e][k] = cp[k * 16]; r.sc[e][k] = sp[k * G]; }
            if (SM == 1) {
                r.cen[e] = *reinterpret_cast<const uint4 *>(cent + (int64_t)min(id[e], kmax) * kHeadDim + c8 * 8);
            } else if (SM > 1) {
#pragma unroll
                for (int st = 0; st < SM; ++st)
                    r.rows[e][st] = *reinterpret_cast<const uint4 *>(
                        cent + ((int64_t)st * K + min((id[e] >> (8 * st)) & 0xffu, kmax)) * kHeadDim + c8 * 8);
            } else {
                for (int st = 0; st < S; ++st) {
                    float row[8];
                    // 16-bit ids with several stages do not fit the packed word: read where they are used
                    const uint32_t sid = s.wide ? (uint32_t)reinterpret_cast<const uint16_t *>(s.ids)[(int64_t)n * S + st]
                                                : (id[e] >> (8 * st)) & 0xffu;
                    unpack_bf16x8(*reinterpret_cast<const uint4 *>(
                                      cent + ((int64_t)st * K + min(sid, kmax)) * kHeadDim + c8 * 8), row);
#pragma unroll
                    for (int i = 0; i < 8; ++i) r.ci[e][i] = st ? r.ci[e][i] + row[i] : row[i];
                }
            }
        }
    }
}

// fp32 decoded values of the thread's two tokens (tokens that do not exist decode to zero
// because their codes, scales and centroid were loaded as zero)
template <int T_, int TM, int SM = 1, int FMT = 0>
__device__ __forceinline__ void dequant2x8(const Raw<TM, SM> &r, int T, float *accA, float *accB) {
    if (SM == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { accA[i] = r.ci[0][i]; accB[i] = r.ci[1][i]; }
    } else if (SM > 1) {
        unpack_bf16x8(r.rows[0][0], accA);
        unpack_bf16x8(r.rows[1][0], accB);
#pragma unroll
        for (int st = 1; st < SM; ++st) {
            float ra[8], rb[8];
            unpack_bf16x8(r.rows[0][st], ra);
            unpack_bf16x8(r.rows[1][st], rb);
#pragma unroll
            for (int i = 0; i < 8; ++i) { accA[i] += ra[i]; accB[i] += rb[i]; }
        }
    } else {
        unpack_bf16x8(r.cen[0], accA);
        unpack_bf16x8(r.cen[1], accB);
    }
    if (FMT != 0) {
        constexpr bool FP8 = (FMT & kFmtE4M3) != 0;
#pragma unroll
        for (int t = 0; t < TM; ++t) {
            if (t < T) {
                const float sa = scale_bits_to_f32<FP8>(r.sc[0][t]), sb = scale_bits_to_f32<FP8>(r.sc[1][t]);
                if (FMT & kFmtInt4) {
                    add_stage_int4(accA, r.code[0][t], sa);
                    add_stage_int4(accB, r.code[1][t], sb);
                } else {
                    add_last_stage_of_two_rows(accA, accB, r.code[0][t] | (r.code[1][t] << 16), 0.5f * sa, 0.5f * sb);
                }
            }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t + 1 < TM; t += 2) {
        if (t + 1 < T) {
            add_two_stages(accA, r.code[0][t] | (r.code[0][t + 1] << 16),
                           half_scale(r.sc[0][t]), half_scale(r.sc[0][t + 1]));
            add_two_stages(accB, r.code[1][t] | (r.code[1][t + 1] << 16),
                           half_scale(r.sc[1][t]), half_scale(r.sc[1][t + 1]));
        }
    }
    if (T_ > 0) {
        if (T_ & 1)
            add_last_stage_of_two_rows(accA, accB, r.code[0][TM - 1] | (r.code[1][TM - 1] << 16),
                                       half_scale(r.sc[0][TM - 1]), half_scale(r.sc[1][TM - 1]));
    } else if (T & 1) {
#pragma unroll
        for (int t = 0; t < TM; t += 2)
            if (t == T - 1)
                add_last_stage_of_two_rows(accA, accB, r.code[0][t] | (r.code[1][t] << 16),
                                           half_scale(r.sc[0][t]), half_scale(r.sc[1][t]));
    }
}

// the (cos, sin) pairs of this thread's 8 channels of its two tokens of a tile (zero for tokens
// that do not exist: their decoded value is zero as well)
__device__ __forceinline__ void load_rope(const f16_t *rope, const Tile &t, int tp, int c8, uint4 rp[2]) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int n = t.t0 + 2 * tp + e;
        rp[e] = (t.valid && n < t.cend)
                    ? *reinterpret_cast<const uint4 *>(rope + (int64_t)n * kHeadDim + c8 * 8)
                    : make_uint4(0u, 0u, 0u, 0u);
    }
}

}  // namespace qvg
