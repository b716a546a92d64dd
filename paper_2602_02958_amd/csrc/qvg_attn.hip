// Attention that reads the compressed cache directly: O = softmax(scale * Q K_hat^T) V_hat,
// where K_hat / V_hat are the decoded values of paper Sec. 4.2 Eq. 7, rounded to bf16 as the
// stand-alone decoder stores them.  The decoded tiles live only in LDS.
//
// One workgroup = 4 wavefronts = 128 queries of one unit; it walks the cache chunk by chunk
// (each chunk has its own centroid tables) in tiles of 64 tokens:
//   1. all 256 threads decode the K tile (row-major) and the V tile (transposed) into LDS;
//   2. S^T = K_tile . Q^T on v_mfma_f32_32x32x16_bf16: rows = cache tokens, columns = queries,
//      so a lane owns one query and the soft-max statistics stay in the lane (one exchange
//      between the two lane halves per tile);
//   3. online soft-max in fp32 (base-2 exponent);
//   4. O^T += V_tile^T . P on v_mfma_f32_32x32x16_f16: the probabilities go in as f16 (11
//      significant bits; bf16's 8 would cost up to 2^-9 of |V| in the output), and the V tile,
//      first rounded to bf16 like the stand-alone decoder's output, is stored as f16, which
//      holds every bf16 value of magnitude 2^-14 .. 65504 exactly (larger ones saturate).
//      The lane's P values are already the B operand: the V tile is stored with the matching
//      token permutation, so no cross-lane traffic is needed.
// Only the two contractions use the matrix cores; the unpack / fma / soft-max work is VALU.
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kAtThreads = 256;
constexpr int kAtQPerBlock = 128;
constexpr int kAtKv = 64;
constexpr int kKtPitch = 136;      // bf16 per row of the K tile (272 B, 16-byte aligned, conflict-free)
constexpr int kVtPitch = 72;       // f16 per row of the transposed V tile (144 B)

struct CacheSide {                 // one of K / V, already offset to this unit
    const bf16_t *cent;            // [n_chunks][K][d]
    const uint8_t *ids; const uint8_t *codes; const f16_t *scales;
};

// Decode 4 consecutive tokens x 8 channels (chunk c8 of 16).  Tokens at or after `end`
// decode to zero.  hb[e][i]: bf16 bits of token tok0+e, channel 8*c8+i.
template <int T_>
__device__ __forceinline__ void dequant4x8(const CacheSide &s, const bf16_t *cent_chunk,
                                           int64_t tok0, int64_t end, int c8, int T, int B, int K,
                                           uint32_t hb[4][4]) {
    constexpr int TM = T_ > 0 ? T_ : kMaxStages;
    const int G = kHeadDim / B;
    const int g = (c8 * 8) / B;
    uint32_t idv[4];
    uint32_t code[4][TM], sc[4][TM];
    uint4 cen[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t n = tok0 + e;
        if (n < end) {
            idv[e] = min((uint32_t)s.ids[n], (uint32_t)(K - 1));   // stay inside the table
            const uint16_t *cp = reinterpret_cast<const uint16_t *>(s.codes + n * T * 32) + c8;
            const f16_t *sp = s.scales + n * T * G + g;
#pragma unroll
            for (int t = 0; t < TM; ++t)
                if (t < T) { code[e][t] = cp[t * 16]; sc[e][t] = sp[t * G]; }
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (tok0 + e < end)
            cen[e] = *reinterpret_cast<const uint4 *>(cent_chunk + (int64_t)idv[e] * kHeadDim + c8 * 8);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (tok0 + e < end) {
            float acc[8];
            acc[0] = bf16_lo(cen[e].x); acc[1] = bf16_hi(cen[e].x);
            acc[2] = bf16_lo(cen[e].y); acc[3] = bf16_hi(cen[e].y);
            acc[4] = bf16_lo(cen[e].z); acc[5] = bf16_hi(cen[e].z);
            acc[6] = bf16_lo(cen[e].w); acc[7] = bf16_hi(cen[e].w);
#pragma unroll
            for (int t = 0; t < TM; ++t) {
                if (t < T) {
                    const float sf = f16_bits_to_f32(sc[e][t]);
                    const uint32_t cw = code[e][t];
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        acc[i] = __builtin_fmaf(sf, (float)(((int)cw << (30 - 2 * i)) >> 30), acc[i]);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) hb[e][i] = pack_bf16x2(acc[2 * i], acc[2 * i + 1]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) hb[e][i] = 0u;
        }
    }
}

template <int T_>       // T_ > 0: compile-time stage count; 0: run-time (up to kMaxStages)
__global__ __launch_bounds__(kAtThreads, 2)
void attn_kernel(AttnArgs a) {
    __shared__ __align__(16) bf16_t Kt[kAtKv * kKtPitch];
    __shared__ __align__(16) uint16_t Vt[kHeadDim * kVtPitch];     // f16 bits

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int h = blockIdx.y;
    const int64_t qrow = (int64_t)blockIdx.x * kAtQPerBlock + wave * 32 + col;
    const bool qvalid = qrow < a.n_q;
    const int T = T_ > 0 ? T_ : a.T, B = a.B, K = a.K;
    const int G = kHeadDim / B;

    CacheSide ks, vs;
    ks.ids = a.k_ids + (int64_t)h * a.n_kv;  ks.codes = a.k_codes + (int64_t)h * a.n_kv * T * 32;
    ks.scales = a.k_scales + (int64_t)h * a.n_kv * T * G;
    ks.cent = a.k_cent + (int64_t)h * a.n_chunks * K * kHeadDim;
    vs.ids = a.v_ids + (int64_t)h * a.n_kv;  vs.codes = a.v_codes + (int64_t)h * a.n_kv * T * 32;
    vs.scales = a.v_scales + (int64_t)h * a.n_kv * T * G;
    vs.cent = a.v_cent + (int64_t)h * a.n_chunks * K * kHeadDim;

    // Q as the B operand of S^T = K Q^T: lane (col, half) holds Q[q][16*kk + 8*half .. +7].
    uint4 qa[8];
    {
        const bf16_t *qp = a.q + ((int64_t)h * a.n_q + qrow) * kHeadDim + half * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qa[kk] = qvalid ? *reinterpret_cast<const uint4 *>(qp + kk * 16) : make_uint4(0u, 0u, 0u, 0u);
    }
    floatx16_t O[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[mb][r] = 0.0f;
    float m = -INFINITY, l = 0.0f;
    const float scale2 = a.scale * 1.4426950408889634f;

    // thread -> (token quad, channel chunk) for the two tile layouts
    const int k_c8 = tid & 15, k_qd = tid >> 4;       // K tile: a row's 16 chunks are adjacent lanes
    const int v_qd = tid & 15, v_c8 = tid >> 4;       // V tile: a channel's 16 quads are adjacent lanes
    // position of quad v_qd in a transposed row: tokens 16*st + 8*a + 4*hh + e -> 16*st + 8*hh + 4*a + e
    const int v_pos = 16 * (v_qd >> 2) + 8 * (v_qd & 1) + 4 * ((v_qd >> 1) & 1);

    for (int c = 0; c < a.n_chunks; ++c) {
        const int64_t cbeg = (int64_t)c * a.chunk_len;
        const int64_t cend = (cbeg + a.chunk_len < a.n_kv) ? cbeg + a.chunk_len : a.n_kv;
        const bf16_t *kc = ks.cent + (int64_t)c * K * kHeadDim;
        const bf16_t *vc = vs.cent + (int64_t)c * K * kHeadDim;
        for (int64_t t0 = cbeg; t0 < cend; t0 += kAtKv) {
            __syncthreads();
            {
                uint32_t hb[4][4];
                dequant4x8<T_>(ks, kc, t0 + 4 * k_qd, cend, k_c8, T, B, K, hb);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *reinterpret_cast<uint4 *>(Kt + (4 * k_qd + e) * kKtPitch + k_c8 * 8) =
                        make_uint4(hb[e][0], hb[e][1], hb[e][2], hb[e][3]);
            }
            {
                uint32_t hb[4][4];
                dequant4x8<T_>(vs, vc, t0 + 4 * v_qd, cend, v_c8, T, B, K, hb);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < 4; ++i)      // bf16 pair -> f16 pair (exact in range)
                        hb[e][i] = pack_f16x2_rtz(bf16_lo(hb[e][i]), bf16_hi(hb[e][i]));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // channels 8*v_c8 + 2i (low halves) and + 2i + 1 (high halves) of 4 tokens
                    const uint32_t lo01 = (hb[0][i] & 0xffffu) | (hb[1][i] << 16);
                    const uint32_t lo23 = (hb[2][i] & 0xffffu) | (hb[3][i] << 16);
                    const uint32_t hi01 = (hb[0][i] >> 16) | (hb[1][i] & 0xffff0000u);
                    const uint32_t hi23 = (hb[2][i] >> 16) | (hb[3][i] & 0xffff0000u);
                    *reinterpret_cast<uint2 *>(Vt + (8 * v_c8 + 2 * i) * kVtPitch + v_pos) = make_uint2(lo01, lo23);
                    *reinterpret_cast<uint2 *>(Vt + (8 * v_c8 + 2 * i + 1) * kVtPitch + v_pos) = make_uint2(hi01, hi23);
                }
            }
            __syncthreads();

            // ---- S^T = K_tile . Q^T -------------------------------------
            floatx16_t S[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) S[nb][r] = 0.0f;
                const bf16_t *arow = Kt + (nb * 32 + col) * kKtPitch + half * 8;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const bf16x8_t av = *reinterpret_cast<const bf16x8_t *>(arow + kk * 16);
                    S[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        av, __builtin_bit_cast(bf16x8_t, qa[kk]), S[nb], 0, 0, 0);
                }
            }
            // ---- online soft-max (base 2) --------------------------------
            const int ntile = (int)((cend - t0 < kAtKv) ? cend - t0 : kAtKv);
            float tmax = -INFINITY;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kv = nb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    float z = S[nb][r] * scale2;
                    if (kv >= ntile) z = -INFINITY;
                    S[nb][r] = z;
                    tmax = fmaxf(tmax, z);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m, tmax);
            if (__ballot(m_new > m)) {                 // uniform: skip when no maximum moved
                const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                l *= alpha;
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) O[mb][r] *= alpha;
            }
            m = m_new;
            uint4 pb[4];
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(S[st >> 1][(st & 1) * 8 + e] - m);
                    l += p[e];
                }
                pb[st] = make_uint4(pack_f16x2_rtz(p[0], p[1]), pack_f16x2_rtz(p[2], p[3]),
                                    pack_f16x2_rtz(p[4], p[5]), pack_f16x2_rtz(p[6], p[7]));
            }
            // ---- O^T += V_tile^T . P --------------------------------------
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const uint16_t *vrow = Vt + (mb * 32 + col) * kVtPitch + half * 8;
#pragma unroll
                for (int st = 0; st < 4; ++st) {
                    const halfx8_t av = *reinterpret_cast<const halfx8_t *>(vrow + st * 16);
                    O[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                        av, __builtin_bit_cast(halfx8_t, pb[st]), O[mb], 0, 0, 0);
                }
            }
        }
    }
    // ---- normalise and store: lane holds channels 32*mb + 8*g + 4*half + 0..3 of its query ----
    const float ltot = l + __shfl_xor(l, 32, 64);
    if (qvalid) {
        const float inv = 1.0f / ltot;
        bf16_t *op = a.out + ((int64_t)h * a.n_q + qrow) * kHeadDim + half * 4;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint2 o = make_uint2(
                    pack_bf16x2(O[mb][4 * g + 0] * inv, O[mb][4 * g + 1] * inv),
                    pack_bf16x2(O[mb][4 * g + 2] * inv, O[mb][4 * g + 3] * inv));
                *reinterpret_cast<uint2 *>(op + mb * 32 + g * 8) = o;
            }
        if (a.lse && half == 0)
            a.lse[(int64_t)h * a.n_q + qrow] = (m + __builtin_log2f(ltot)) * 0.6931471805599453f;
    }
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t s) {
    if (a.n_q == 0) return hipSuccess;
    dim3 grid((unsigned)((a.n_q + kAtQPerBlock - 1) / kAtQPerBlock), (unsigned)a.H);
    switch (a.T) {
        case 1: hipLaunchKernelGGL(attn_kernel<1>, grid, dim3(kAtThreads), 0, s, a); break;
        case 2: hipLaunchKernelGGL(attn_kernel<2>, grid, dim3(kAtThreads), 0, s, a); break;
        case 3: hipLaunchKernelGGL(attn_kernel<3>, grid, dim3(kAtThreads), 0, s, a); break;
        case 4: hipLaunchKernelGGL(attn_kernel<4>, grid, dim3(kAtThreads), 0, s, a); break;
        default: hipLaunchKernelGGL(attn_kernel<0>, grid, dim3(kAtThreads), 0, s, a); break;
    }
    return hipGetLastError();
}

}  // namespace qvg
