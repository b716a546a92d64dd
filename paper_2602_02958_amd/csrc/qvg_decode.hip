// Decode kernel: replay of the stored stages (paper Sec. 4.2, Eq. 7; Sec. 4.3
// "Dequantization kernel": every stage in one pass, the running value in registers).
//
//   x_hat[n][c] = bf16( fma(s_T, q_T, ... fma(s_1, q_1, float(C[id_n][c])) ... ) )
//
// Per token-vector it reads 1 id byte, T*32 code bytes and T*(d/B) f16 scales, gathers one
// 256-byte centroid row and writes 256 bytes of bf16.  The centroid table of a chunk (at most
// 64 KB) is staged in LDS by the workgroup that decodes the chunk: gathering the rows from L2
// instead costs as much L2->CU traffic as the output itself and slows the writes measurably.
// The memory side is pure streaming; the instruction side is what has to be kept lean: a
// token costs 128*T field extractions and fmas (see add_two_stages for how a level becomes an
// fma operand in one instruction per element), so the per-lane addressing is reduced to 32-bit
// offsets from per-block (scalar) base pointers.
//
// With S > 1 smoothing stages a token has S ids and S centroid rows, added in stage order in fp32
// before the rounds; the S tables of a chunk sit in LDS together when they fit in 64 KB, else the
// rows are read from global memory (a general, slower variant of the same kernel).
// The other stored formats (FP8 E4M3 scale bytes, 4-bit levels; Sec. 5 "Implementation") are
// template variants of the same kernel: only the scale conversion and the field extraction differ.
// The caches may be allocated for more tokens than are decoded (unit strides in the arguments).
//
// Mapping: 16 lanes per token, 8 channels (one 16-byte store) per lane, so that a
// wavefront's store instruction covers 4 whole token rows = 1 KB contiguous.  A workgroup of
// 1024 threads walks its slice of a chunk 256 tokens per pass, 4 token rows per thread.
#include <type_traits>

#include "qvg_internal.hpp"

namespace qvg {

constexpr int kDecThreads = 1024;
constexpr int kDecRows = kDecThreads / 16;       // token rows per pass of a block (64)
constexpr int kDecUnroll = 4;
constexpr int kDecTokPerIter = kDecRows * kDecUnroll;      // 256 tokens per pass
constexpr int kXcds = 8;                         // MI355X: 8 XCDs, each with its own L2

// One pass of a block: 256 tokens, 4 rows per thread.  CHECK = false is the fast path for a pass
// whose tokens all exist (no per-row predication).  tab: the chunk's centroid table in LDS.
// SM: 1 = one smoothing stage, table in LDS; 2 = S stages, all tables in LDS (tab);
//     3 = S stages, tables read from global memory (cg).
// FMT: stored format (kFmt* bits).  4-bit levels: a lane's 8 channels of a round are one 32-bit
// word (16 words per token and round, so the offsets below are the same in units of the word).
// SC: number of smoothing stages when known at compile time (the loops over the stages unroll and
// their loads are issued together), 0 = run-time S.
// WIDE: ids are 16-bit words (more than 256 centroids; one stage, or several with the tables in
// global memory, which is where tables of that size always are).  A template parameter: as a
// run-time switch around the id load it cost the byte-id kernels 15 % (0.667 -> 0.767 ms at the
// cfg3 shape).
template <int T_, bool CHECK, int SM, int FMT, int SC, bool WIDE>
__device__ __forceinline__ void decode_pass(int T, int S_, uint32_t ln0, uint32_t n_left, uint32_t lane16,
                                            uint32_t G, uint32_t gidx, uint32_t kmax,
                                            const uint8_t *ids_b, const void *codes_v,
                                            const void *scales_v, const bf16_t *tab, const bf16_t *cg,
                                            bf16_t *out_b, int64_t stride_token) {
    constexpr int TM = T_ > 0 ? T_ : kMaxStages;
    constexpr bool FP8 = (FMT & kFmtE4M3) != 0, I4 = (FMT & kFmtInt4) != 0;
    typedef typename std::conditional<I4, uint32_t, uint16_t>::type code_t;
    typedef typename std::conditional<FP8, uint8_t, f16_t>::type scale_t;
    const code_t *codes_b = static_cast<const code_t *>(codes_v);
    const scale_t *scales_b = static_cast<const scale_t *>(scales_v);
    auto hs = [](uint32_t bits) { return 0.5f * scale_bits_to_f32<FP8>(bits); };
    const int S = SC > 0 ? SC : S_;
    // a token's ids packed into one word: 8 bits per stage, 16 with 16-bit ids
    constexpr int IB = (WIDE && SM != 1) ? 16 : 8;
    typedef typename std::conditional<(WIDE && SM != 1), uint64_t, uint32_t>::type idpack_t;
    constexpr uint32_t IMASK = (1u << IB) - 1u;
    idpack_t idv[kDecUnroll];
    uint32_t code[kDecUnroll][TM];
    uint32_t sc[kDecUnroll][TM];
    bool ok[kDecUnroll];
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        const uint32_t ln = ln0 + u * kDecRows;
        ok[u] = !CHECK || ln < n_left;
        if (CHECK) {
            idv[u] = 0u;
#pragma unroll
            for (int t = 0; t < TM; ++t) { code[u][t] = 0u; sc[u][t] = 0u; }
        }
        if (ok[u]) {
            if (SM == 1) idv[u] = WIDE ? (uint32_t)reinterpret_cast<const uint16_t *>(ids_b)[ln] : (uint32_t)ids_b[ln];
            else {                                   // up to four id bytes of the token, stage s in byte s
                idv[u] = 0u;
#pragma unroll
                for (int st = 0; st < (SC > 0 ? SC : kMaxSmooth); ++st)
                    if (st < S)
                        idv[u] |= (idpack_t)(WIDE ? (uint32_t)reinterpret_cast<const uint16_t *>(ids_b)[ln * (uint32_t)S + st]
                                                  : (uint32_t)ids_b[ln * (uint32_t)S + st]) << (IB * st);
            }
            const uint32_t co = ln * (uint32_t)T * 16u + lane16;       // in code words
            const uint32_t so = ln * (uint32_t)T * G + gidx;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                if (t < T) { code[u][t] = codes_b[co + t * 16]; sc[u][t] = scales_b[so + t * G]; }
        }
    }
    // rows are finished two at a time so that every shift+mask serves two 2-bit fields
#pragma unroll
    for (int up = 0; up < kDecUnroll; up += 2) {
        float accA[8], accB[8];
        // centroid rows; an id beyond the table (corrupt input) is clamped
        if (SM == 1) {
            unpack_bf16x8(*reinterpret_cast<const uint4 *>(tab + min((uint32_t)idv[up], kmax) * kHeadDim + lane16 * 8), accA);
            unpack_bf16x8(*reinterpret_cast<const uint4 *>(tab + min((uint32_t)idv[up + 1], kmax) * kHeadDim + lane16 * 8), accB);
        } else {
            // Eq. 7 with S tables: the rows are added in stage order in fp32
            const bf16_t *tb = (SM == 2) ? tab : cg;
            if (SC > 0) {
                uint4 wa[SC > 0 ? SC : 1], wb[SC > 0 ? SC : 1];
#pragma unroll
                for (int st = 0; st < SC; ++st) {
                    const uint32_t ia = min((uint32_t)(idv[up] >> (IB * st)) & IMASK, kmax) + (uint32_t)st * (kmax + 1u);
                    const uint32_t ib = min((uint32_t)(idv[up + 1] >> (IB * st)) & IMASK, kmax) + (uint32_t)st * (kmax + 1u);
                    wa[st] = *reinterpret_cast<const uint4 *>(tb + ia * kHeadDim + lane16 * 8);
                    wb[st] = *reinterpret_cast<const uint4 *>(tb + ib * kHeadDim + lane16 * 8);
                }
#pragma unroll
                for (int st = 0; st < SC; ++st) {
                    float ra[8], rb[8];
                    unpack_bf16x8(wa[st], ra);
                    unpack_bf16x8(wb[st], rb);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        accA[i] = st ? accA[i] + ra[i] : ra[i];
                        accB[i] = st ? accB[i] + rb[i] : rb[i];
                    }
                }
            } else {
                for (int st = 0; st < S; ++st) {
                    const uint32_t ia = min((uint32_t)(idv[up] >> (IB * st)) & IMASK, kmax) + (uint32_t)st * (kmax + 1u);
                    const uint32_t ib = min((uint32_t)(idv[up + 1] >> (IB * st)) & IMASK, kmax) + (uint32_t)st * (kmax + 1u);
                    float ra[8], rb[8];
                    unpack_bf16x8(*reinterpret_cast<const uint4 *>(tb + ia * kHeadDim + lane16 * 8), ra);
                    unpack_bf16x8(*reinterpret_cast<const uint4 *>(tb + ib * kHeadDim + lane16 * 8), rb);
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        accA[i] = st ? accA[i] + ra[i] : ra[i];
                        accB[i] = st ? accB[i] + rb[i] : rb[i];
                    }
                }
            }
        }
        if (I4) {
#pragma unroll
            for (int t = 0; t < TM; ++t)
                if (t < T) {
                    add_stage_int4(accA, code[up][t], scale_bits_to_f32<FP8>(sc[up][t]));
                    add_stage_int4(accB, code[up + 1][t], scale_bits_to_f32<FP8>(sc[up + 1][t]));
                }
        } else {
#pragma unroll
            for (int t = 0; t + 1 < TM; t += 2) {
                if (t + 1 < T) {
                    add_two_stages(accA, code[up][t] | (code[up][t + 1] << 16), hs(sc[up][t]), hs(sc[up][t + 1]));
                    add_two_stages(accB, code[up + 1][t] | (code[up + 1][t + 1] << 16),
                                   hs(sc[up + 1][t]), hs(sc[up + 1][t + 1]));
                }
            }
            if (T_ > 0) {
                if (T_ & 1)
                    add_last_stage_of_two_rows(accA, accB, code[up][TM - 1] | (code[up + 1][TM - 1] << 16),
                                               hs(sc[up][TM - 1]), hs(sc[up + 1][TM - 1]));
            } else if (T & 1) {
                // run-time stage count: the last odd stage sits at index T-1
#pragma unroll
                for (int t = 0; t < TM; t += 2)
                    if (t == T - 1)
                        add_last_stage_of_two_rows(accA, accB, code[up][t] | (code[up + 1][t] << 16),
                                                   hs(sc[up][t]), hs(sc[up + 1][t]));
            }
        }
        // the output is written once and not read again by this kernel: streaming stores
        typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
        if (ok[up]) {
            const uint4 o = pack_bf16x8(accA);
            __builtin_nontemporal_store(u32x4_t{o.x, o.y, o.z, o.w},
                reinterpret_cast<u32x4_t *>(out_b + ((int64_t)(ln0 + up * kDecRows) * stride_token + lane16 * 8)));
        }
        if (ok[up + 1]) {
            const uint4 o = pack_bf16x8(accB);
            __builtin_nontemporal_store(u32x4_t{o.x, o.y, o.z, o.w},
                reinterpret_cast<u32x4_t *>(out_b + ((int64_t)(ln0 + (up + 1) * kDecRows) * stride_token + lane16 * 8)));
        }
    }
}

// One workgroup = one slice of one chunk of one unit.  It stages the chunk's centroid table
// in LDS once (the only shared operand) and then streams its tokens.
template <int T_, int SM, int FMT, int SC, bool WIDE>   // T_ > 0: compile-time stage count; T_ == 0: run-time.  SM, FMT, SC, WIDE: see decode_pass
__global__ __launch_bounds__(kDecThreads)
void decode_kernel(DecodeArgs a, int slices, uint32_t slice_len, int n_blocks, int blocks_per_xcd) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t *tab = reinterpret_cast<bf16_t *>(smem);                 // [K][128]
    // Workgroups are dealt to the XCDs round-robin by their linear id; re-number them so that
    // each XCD walks one contiguous range of (unit, chunk, slice) and writes one contiguous
    // region of the output.
    const int w = (int)(blockIdx.x % kXcds) * blocks_per_xcd + (int)(blockIdx.x / kXcds);
    if (w >= n_blocks) return;
    const int per_unit = a.n_chunks * slices;
    const int h = w / per_unit;
    const int c = (w - h * per_unit) / slices;
    const int sl = w - h * per_unit - c * slices;
    const int64_t cbeg = (int64_t)c * a.chunk_len;
    const int64_t cend = (cbeg + a.chunk_len < a.n_tokens) ? cbeg + a.chunk_len : a.n_tokens;
    const int64_t tok0 = cbeg + (int64_t)sl * slice_len;
    if (tok0 >= cend) return;                                       // uniform: before any barrier
    const uint32_t n_left = (uint32_t)((cend - tok0 < slice_len) ? cend - tok0 : slice_len);

    const int T = T_ > 0 ? T_ : a.T;
    const uint32_t lane16 = threadIdx.x & 15;
    const uint32_t row = threadIdx.x >> 4;
    const uint32_t G = kHeadDim / a.B;
    const uint32_t gidx = (lane16 * 8) / a.B;     // scale group of this lane's 8 channels

    const int S = (SM == 1) ? 1 : (SC > 0 ? SC : a.S);
    const bf16_t *cg = a.cent + ((int64_t)h * a.chunk_stride + c) * S * a.K * kHeadDim;    // [S][K][128] of this chunk
    if (SM != 3) {   // stage the tables: S*K rows of 256 B, 16 B per thread and step
        for (int i = threadIdx.x; i < S * a.K * 16; i += kDecThreads)
            *reinterpret_cast<uint4 *>(tab + i * 8) = *reinterpret_cast<const uint4 *>(cg + i * 8);
    }
    __syncthreads();

    // per-block base pointers (uniform), per-lane 32-bit offsets
    const int64_t hn0 = (int64_t)h * a.kv_stride + tok0;
    const uint8_t *ids_b = a.ids + hn0 * S * (WIDE ? 2 : 1);
    const void *codes_b = a.codes + hn0 * T * ((FMT & kFmtInt4) ? 64 : 32);
    const void *scales_b = reinterpret_cast<const uint8_t *>(a.scales) + hn0 * T * G * ((FMT & kFmtE4M3) ? 1 : 2);
    bf16_t *out_b = a.out + (int64_t)h * a.stride_head + tok0 * a.stride_token;
    const uint32_t kmax = (uint32_t)a.K - 1u;

    for (uint32_t first = 0; first < n_left; first += kDecTokPerIter) {
        if (first + kDecTokPerIter <= n_left)
            decode_pass<T_, false, SM, FMT, SC, WIDE>(T, S, first + row, n_left, lane16, G, gidx, kmax, ids_b, codes_b, scales_b,
                                       tab, cg, out_b, a.stride_token);
        else
            decode_pass<T_, true, SM, FMT, SC, WIDE>(T, S, first + row, n_left, lane16, G, gidx, kmax, ids_b, codes_b, scales_b,
                                      tab, cg, out_b, a.stride_token);
    }
}

template <int T_, int SM, int FMT, int SC, bool WIDE>
static hipError_t launch_decode_w(const DecodeArgs &a, hipStream_t s) {
    // slices per chunk: enough workgroups to fill 256 CUs x 2 twice over, but as few as possible
    // beyond that (every workgroup re-reads the chunk's table; measured flat from 512 to 4096)
    const int64_t unit_chunks = (int64_t)a.H * a.n_chunks;
    const int64_t chunk = a.chunk_len < a.n_tokens ? a.chunk_len : a.n_tokens;
    int64_t slices = (1024 + unit_chunks - 1) / unit_chunks;
    const int64_t max_slices = (chunk + kDecTokPerIter - 1) / kDecTokPerIter;
    if (slices > max_slices) slices = max_slices;
    if (slices < 1) slices = 1;
    int64_t slice_len = (chunk + slices - 1) / slices;
    slice_len = (slice_len + kDecTokPerIter - 1) / kDecTokPerIter * kDecTokPerIter;
    slices = (chunk + slice_len - 1) / slice_len;
    const int64_t nb = unit_chunks * slices;
    if (nb > 0x7fffffff - kXcds) return hipErrorInvalidValue;
    const int bpx = (int)((nb + kXcds - 1) / kXcds);
    const size_t smem = (SM == 3) ? 16 : (size_t)(SM == 1 ? 1 : a.S) * a.K * kHeadDim * sizeof(bf16_t);
    static LdsHighWater lds_limit = {};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(&decode_kernel<T_, SM, FMT, SC, WIDE>), smem, lds_limit);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((decode_kernel<T_, SM, FMT, SC, WIDE>), dim3((unsigned)(bpx * kXcds)), dim3(kDecThreads), smem, s, a,
                       (int)slices, (uint32_t)slice_len, (int)nb, bpx);
    return hipGetLastError();
}

// 16-bit ids: one smoothing stage (SM == 1), or several with the tables in global memory (SM == 3:
// S tables of more than 256 rows never fit the 64 KB that SM == 2 keeps in LDS)
template <int T_, int SM, int FMT = 0, int SC = 0>
static hipError_t launch_decode_t(const DecodeArgs &a, hipStream_t s) {
    if ((SM == 1 || SM == 3) && a.id_wide) return launch_decode_w<T_, SM, FMT, SC, SM == 1 || SM == 3>(a, s);
    return launch_decode_w<T_, SM, FMT, SC, false>(a, s);
}

// the other stored formats: run-time round count, except the paper's own 2-bit / E4M3 / one round
template <int FMT>
static hipError_t launch_decode_fmt(const DecodeArgs &a, hipStream_t s) {
    if (a.S > 1) {
        if ((size_t)a.S * a.K * kHeadDim * sizeof(bf16_t) <= 65536) return launch_decode_t<0, 2, FMT>(a, s);
        // the paper's form with large tables (four stages, one round): counts fixed at compile time
        if ((FMT & kFmtE4M3) && a.S == 4 && a.T == 1) return launch_decode_t<1, 3, FMT, 4>(a, s);
        return launch_decode_t<0, 3, FMT>(a, s);
    }
    if (FMT == kFmtE4M3 && a.T == 1) return launch_decode_t<(FMT == kFmtE4M3 ? 1 : 0), 1, FMT>(a, s);
    return launch_decode_t<0, 1, FMT>(a, s);
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    switch (a.fmt) {
        case 0: break;
        case kFmtE4M3: return launch_decode_fmt<kFmtE4M3>(a, s);
        case kFmtInt4: return launch_decode_fmt<kFmtInt4>(a, s);
        default: return launch_decode_fmt<kFmtInt4 | kFmtE4M3>(a, s);
    }
    if (a.S > 1) {
        // several smoothing stages: every stage's table in LDS when they fit in 64 KB together
        if ((size_t)a.S * a.K * kHeadDim * sizeof(bf16_t) <= 65536) return launch_decode_t<0, 2>(a, s);
        return launch_decode_t<0, 3>(a, s);
    }
    switch (a.T) {
        case 1: return launch_decode_t<1, 1>(a, s);
        case 2: return launch_decode_t<2, 1>(a, s);
        case 3: return launch_decode_t<3, 1>(a, s);
        case 4: return launch_decode_t<4, 1>(a, s);
        default: return launch_decode_t<0, 1>(a, s);
    }
}

}  // namespace qvg
