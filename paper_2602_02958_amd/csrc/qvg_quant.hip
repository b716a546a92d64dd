// Centroid subtraction (paper Eq. 5) and the T rounds of group quantization (Sec. 3.2 Eq. 1-2,
// applied progressively as in Sec. 4.2) for a GIVEN assignment, in every stored format:
// 2-bit or 4-bit levels (Sec. 5: INT2 / INT4), binary16 or FP8 E4M3 scales (Sec. 5
// "Implementation").  The encoder uses it after the assignment kernel whenever the format is
// not the one the fused assignment kernel writes (2-bit levels with binary16 scales).
//
// Per token it reads 256 B of x, one id and one centroid row (L2) and writes T*(d*b/8 + d/B
// scales): a streaming kernel.  Mapping: 16 lanes per token, 8 channels per lane, so a group of
// B channels is B/8 adjacent lanes and its maximum is a few lane exchanges.
//
// The integers are fixed by these rules (the same in every format): scale = max|r| / qmax with
// one correctly rounded fp32 division, saturated at the format's largest finite value and rounded
// to nearest even; q = round-half-even(r * (1/scale)) clamped to [-qmax, qmax], 1/scale one fp32
// division by the STORED scale; a zero scale gives q = 0; the next round sees fma(-scale, q, r).
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kQtThreads = 256;
constexpr int kQtTokens = kQtThreads / 16;      // tokens per pass of a block

template <int BITS, bool FP8, bool WIDE>       // WIDE: 16-bit ids (more than 256 centroids)
__global__ __launch_bounds__(kQtThreads)
void quantize_kernel(QuantArgs a, int passes) {
    const int h = blockIdx.x;
    const int lane16 = threadIdx.x & 15, row = threadIdx.x >> 4;
    const int B = a.B, T = a.T, G = kHeadDim / B;
    const int gl = B / 8;                          // lanes per group: 2, 4, 8 or 16
    const float qmax = (BITS == 4) ? 7.0f : 1.0f;
    constexpr int kCodeBytes = kHeadDim * BITS / 8;     // per token and round
    const bf16_t *cent = a.cent + (int64_t)h * a.K * kHeadDim;
    const uint32_t kmax = (uint32_t)a.K - 1u;

    for (int ps = 0; ps < passes; ++ps) {
        const int64_t n = ((int64_t)blockIdx.y * passes + ps) * kQtTokens + row;
        const bool valid = n < a.n_tokens;             // all 16 lanes of a token agree
        float r[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = 0.0f;
        const int64_t hn = (int64_t)h * a.out_stride + n;
        if (valid) {
            const uint32_t id = min(load_id(a.ids, hn * a.ids_step + a.ids_off, WIDE ? 1 : 0), kmax);
            const uint4 xv = *reinterpret_cast<const uint4 *>(a.x + (int64_t)h * a.stride_head + n * a.stride_token + lane16 * 8);
            const uint4 cv = *reinterpret_cast<const uint4 *>(cent + (int64_t)id * kHeadDim + lane16 * 8);
            const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w}, cw[4] = {cv.x, cv.y, cv.z, cv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                r[2 * e] = bf16_lo(xw[e]) - bf16_lo(cw[e]);               // Eq. 5, one fp32 subtraction
                r[2 * e + 1] = bf16_hi(xw[e]) - bf16_hi(cw[e]);
            }
        }
        for (int t = 0; t < T; ++t) {
            float m = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(r[i]));
            // maximum over the group's lanes (adjacent, aligned to the group size)
            for (int off = 1; off < gl; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
            const float s32 = m / qmax;
            uint32_t sbits; float sf;
            if (FP8) { sbits = f32_to_e4m3_bits(s32); sf = e4m3_bits_to_f32(sbits); }
            else { sbits = f32_to_f16_bits(fminf(s32, 65504.0f)); sf = f16_bits_to_f32(sbits); }
            const float inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
            uint32_t code = 0u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float q = __builtin_amdgcn_fmed3f(__builtin_rintf(r[i] * inv), -qmax, qmax);
                r[i] = __builtin_fmaf(-sf, q, r[i]);
                code |= ((uint32_t)(int)q & ((1u << BITS) - 1u)) << (BITS * i);     // two's complement field
            }
            if (valid) {
                uint8_t *cp = a.codes + (hn * T + t) * kCodeBytes + lane16 * BITS;
                if (BITS == 4) *reinterpret_cast<uint32_t *>(cp) = code;
                else *reinterpret_cast<uint16_t *>(cp) = (uint16_t)code;
                if ((lane16 & (gl - 1)) == 0) {
                    const int64_t so = (hn * T + t) * G + lane16 / gl;
                    if (FP8) static_cast<uint8_t *>(a.scales)[so] = (uint8_t)sbits;
                    else static_cast<f16_t *>(a.scales)[so] = (f16_t)sbits;
                }
            }
        }
    }
}

template <int BITS, bool FP8>
static hipError_t launch_quantize_t(const QuantArgs &a, hipStream_t s) {
    const int64_t steps = (a.n_tokens + kQtTokens - 1) / kQtTokens;
    int passes = 1;
    while (passes < 16 && (steps / (2 * passes)) * a.H >= 4096) passes *= 2;
    const int64_t gy = (steps + passes - 1) / passes;
    if (gy > 65535) return hipErrorInvalidValue;
    if (a.id_wide)
        hipLaunchKernelGGL((quantize_kernel<BITS, FP8, true>), dim3((unsigned)a.H, (unsigned)gy), dim3(kQtThreads), 0, s, a, passes);
    else
        hipLaunchKernelGGL((quantize_kernel<BITS, FP8, false>), dim3((unsigned)a.H, (unsigned)gy), dim3(kQtThreads), 0, s, a, passes);
    return hipGetLastError();
}

hipError_t launch_quantize(const QuantArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    switch (a.fmt) {
        case 0: return launch_quantize_t<2, false>(a, s);
        case kFmtE4M3: return launch_quantize_t<2, true>(a, s);
        case kFmtInt4: return launch_quantize_t<4, false>(a, s);
        default: return launch_quantize_t<4, true>(a, s);
    }
}

}  // namespace qvg
