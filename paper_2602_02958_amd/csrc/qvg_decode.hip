// Decode kernel: replay of the stored stages (paper Sec. 4.2, Eq. 7; Sec. 4.3
// "Dequantization kernel": every stage in one pass, the running value in registers).
//
//   x_hat[n][c] = bf16( fma(s_T, q_T, ... fma(s_1, q_1, float(C[id_n][c])) ... ) )
//
// Pure streaming, bound by HBM: per token-vector it reads 1 id byte, T*32 code
// bytes and T*(d/B) f16 scales, gathers one 256-byte centroid row (L2-resident:
// a table is at most 64 KB) and writes 256 bytes of bf16.
//
// Mapping: 16 lanes per token, 8 channels (one 16-byte store) per lane, so that a
// wavefront's store instruction covers 4 whole token rows = 1 KB contiguous.
// Each block walks kTokPerBlock tokens, kUnroll token rows in flight per thread.
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kDecThreads = 256;
constexpr int kDecRows = kDecThreads / 16;       // token rows per pass of a block
constexpr int kDecUnroll = 4;
constexpr int kDecTokPerBlock = kDecRows * kDecUnroll;

template <int T_>   // T_ > 0: compile-time stage count; T_ == 0: run-time
__global__ __launch_bounds__(kDecThreads)
void decode_kernel(DecodeArgs a) {
    const int T = T_ > 0 ? T_ : a.T;
    const int h = blockIdx.y;
    const int lane16 = threadIdx.x & 15;
    const int row = threadIdx.x >> 4;
    const int G = kHeadDim / a.B;
    const int gidx = (lane16 * 8) / a.B;          // scale group of this lane's 8 channels
    const int64_t tok0 = (int64_t)blockIdx.x * kDecTokPerBlock;

    uint32_t idv[kDecUnroll];
    uint32_t code[kDecUnroll][T_ > 0 ? T_ : kMaxStages];
    uint32_t sc[kDecUnroll][T_ > 0 ? T_ : kMaxStages];
    uint4 cen[kDecUnroll];
    bool ok[kDecUnroll];

#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        const int64_t n = tok0 + u * kDecRows + row;
        ok[u] = n < a.n_tokens;
        if (ok[u]) {
            const int64_t hn = (int64_t)h * a.n_tokens + n;
            idv[u] = min((uint32_t)a.ids[hn], (uint32_t)(a.K - 1));   // stay inside the table whatever the bytes hold
            const uint16_t *cp = reinterpret_cast<const uint16_t *>(a.codes + hn * T * 32) + lane16;
            const f16_t *sp = a.scales + hn * T * G + gidx;
#pragma unroll
            for (int t = 0; t < (T_ > 0 ? T_ : kMaxStages); ++t) {
                if (t < T) { code[u][t] = cp[t * 16]; sc[u][t] = sp[t * G]; }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        if (ok[u]) {
            const int64_t n = tok0 + u * kDecRows + row;
            const int64_t chunk = n / a.chunk_len;
            const bf16_t *crow = a.cent + (((int64_t)h * a.n_chunks + chunk) * a.K + idv[u]) * kHeadDim;
            cen[u] = *reinterpret_cast<const uint4 *>(crow + lane16 * 8);
        }
    }
#pragma unroll
    for (int u = 0; u < kDecUnroll; ++u) {
        if (!ok[u]) continue;
        const int64_t n = tok0 + u * kDecRows + row;
        float acc[8];
        acc[0] = bf16_lo(cen[u].x); acc[1] = bf16_hi(cen[u].x);
        acc[2] = bf16_lo(cen[u].y); acc[3] = bf16_hi(cen[u].y);
        acc[4] = bf16_lo(cen[u].z); acc[5] = bf16_hi(cen[u].z);
        acc[6] = bf16_lo(cen[u].w); acc[7] = bf16_hi(cen[u].w);
#pragma unroll
        for (int t = 0; t < (T_ > 0 ? T_ : kMaxStages); ++t) {
            if (t < T) {
                const float s = f16_bits_to_f32(sc[u][t]);
                const uint32_t cw = code[u][t];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float q = (float)((int)((cw >> (2 * i)) & 3u) - 1);
                    acc[i] = __builtin_fmaf(s, q, acc[i]);
                }
            }
        }
        uint4 o;
        o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
        bf16_t *orow = a.out + (int64_t)h * a.stride_head + n * a.stride_token;
        *reinterpret_cast<uint4 *>(orow + lane16 * 8) = o;
    }
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    dim3 grid((unsigned)((a.n_tokens + kDecTokPerBlock - 1) / kDecTokPerBlock), (unsigned)a.H);
    dim3 block(kDecThreads);
    switch (a.T) {
        case 1: hipLaunchKernelGGL(decode_kernel<1>, grid, block, 0, s, a); break;
        case 2: hipLaunchKernelGGL(decode_kernel<2>, grid, block, 0, s, a); break;
        case 3: hipLaunchKernelGGL(decode_kernel<3>, grid, block, 0, s, a); break;
        case 4: hipLaunchKernelGGL(decode_kernel<4>, grid, block, 0, s, a); break;
        default: hipLaunchKernelGGL(decode_kernel<0>, grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

}  // namespace qvg
