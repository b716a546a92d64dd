// k-means assignment (paper Sec. 4.1), and the fused encoder pass that follows it:
// centroid subtraction (Eq. 5), T rounds of 2-bit group quantization of the residual
// (Sec. 3.2 Eq. 1-2, applied progressively as in Sec. 4.2) and bit packing.
//
// Assignment = argmin_j ||x - c_j||^2 = argmax_j ( x.c_j - ||c_j||^2 / 2 ).
// The N x K matrix of dot products is a dense contraction and runs on the matrix
// cores (v_mfma_f32_32x32x16_bf16; bf16 x bf16 products are exact in fp32), with the
// centroid table of the unit staged once per workgroup in LDS.  The MFMA is issued
// transposed (rows = centroids, columns = tokens) so that one lane owns one token and
// the argmax over centroids is a per-lane running maximum followed by a single
// exchange between the two lane halves.
//
// Exactness.  The reference result is the argmin of fp64 distances.  The fp32 scores
// carry a rounding error, so the kernel keeps the three largest scores per token
// (cluster index carried in the 7 low mantissa bits) and certifies the winner only
// when it leads by more than a bound on that error,
//     thr = 2^-14 * (||x||^2 / 2 + max_j ||c_j||^2),
// which covers 128 accumulation roundings of one ulp each plus the index tag for both
// scores.  Otherwise the candidates are re-evaluated in fp64: the two leaders
// cooperatively by the wavefront, or, if the third score is inside the band as well,
// all K centroids with the channels summed in index order (the reference order).
// Equal fp64 distances go to the lower index.
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kAsgThreads = 256;
constexpr int kAsgWaves = kAsgThreads / 64;
constexpr int kAsgTile = 32;                    // tokens per wavefront tile
constexpr int kAsgTokPerBlock = 256;
constexpr int kCPitch = 136;                    // bf16 elements per LDS centroid row (272 B)
constexpr uint32_t kTagMask = 0xFFFFFF80u;

__device__ __forceinline__ void insert3(float v, int idx, float &b1, float &b2, float &b3,
                                        int &i1, int &i2) {
    if (v > b1) { b3 = b2; b2 = b1; i2 = i1; b1 = v; i1 = idx; }
    else if (v > b2) { b3 = b2; b2 = v; i2 = idx; }
    else if (v > b3) { b3 = v; }
}

__device__ __forceinline__ double shfl_xor_f64(double v, int m) { return __shfl_xor(v, m, 64); }

// One round of 2-bit quantization of n_ consecutive residuals held by a lane
// (Eq. 2 with b = 2: scale = max|r|, levels -1, 0, 1).  m is the group maximum.
// Returns the f16 bits of the scale; codes are added into word[] (16 codes per word).
template <int N_>
__device__ __forceinline__ uint32_t quant_group(float *r, float m, uint32_t *word, int first) {
    const float s32 = fminf(m, 65504.0f);
    const uint32_t sh = f32_to_f16_bits(s32);
    const float sf = f16_bits_to_f32(sh);
    const float inv = (sf == 0.0f) ? 0.0f : 1.0f / sf;
#pragma unroll
    for (int i = 0; i < N_; ++i) {
        const float u = r[i] * inv;
        float q = __builtin_rintf(u);
        q = __builtin_amdgcn_fmed3f(q, -1.0f, 1.0f);
        r[i] = __builtin_fmaf(-sf, q, r[i]);
        const int e = first + i;
        word[e >> 4] += ((uint32_t)(int)q) << (2 * (e & 15));
    }
    return sh;
}

template <int B_, bool FUSED>
__global__ __launch_bounds__(kAsgThreads, 2)
void assign_kernel(AssignArgs a, int Kpad) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t *lc = reinterpret_cast<bf16_t *>(smem);                       // [Kpad][kCPitch]
    float *lcnh = reinterpret_cast<float *>(smem + (size_t)Kpad * kCPitch * 2);   // -||c||^2/2
    uint32_t *lcmax = reinterpret_cast<uint32_t *>(lcnh + Kpad);         // bits of max ||c||^2
    bf16_t *lscr = reinterpret_cast<bf16_t *>(lcmax + 4);                // [waves][128]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, col = lane & 31;
    const int h = blockIdx.y;
    const int K = a.K;
    const int64_t N = a.n_tokens;

    // ---- stage the centroid table and its norms -------------------------
    if (tid == 0) lcmax[0] = 0u;
    __syncthreads();
    const bf16_t *cg = a.cent + (int64_t)h * K * kHeadDim;
    for (int i = tid; i < Kpad * 16; i += kAsgThreads) {
        const int row = i >> 4, c16 = i & 15;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (row < K) v = *reinterpret_cast<const uint4 *>(cg + (int64_t)row * kHeadDim + c16 * 8);
        *reinterpret_cast<uint4 *>(lc + row * kCPitch + c16 * 8) = v;
        double s = 0.0;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double lo = (double)bf16_lo(w[e]), hi = (double)bf16_hi(w[e]);
            s += lo * lo; s += hi * hi;
        }
        s += shfl_xor_f64(s, 1); s += shfl_xor_f64(s, 2);
        s += shfl_xor_f64(s, 4); s += shfl_xor_f64(s, 8);
        if (c16 == 0) {
            if (row < K) {
                lcnh[row] = (float)(-0.5 * s);
                // upper bound of ||c||^2 in fp32 (one ulp up), kept as its bit pattern
                const float up = (float)s * (1.0f + 0x1p-22f);
                atomicMax(lcmax, __float_as_uint(up));
            } else {
                lcnh[row] = -3.0e38f;
            }
        }
    }
    __syncthreads();
    const float cmax = __uint_as_float(lcmax[0]);
    bf16_t *scr = lscr + wave * kHeadDim;

    const int64_t blk0 = (int64_t)blockIdx.x * kAsgTokPerBlock;
    for (int tile = wave; tile < kAsgTokPerBlock / kAsgTile; tile += kAsgWaves) {
        const int64_t n0 = blk0 + (int64_t)tile * kAsgTile;
        if (n0 >= N) break;                                  // uniform per wavefront
        const int64_t n = n0 + col;
        const bool valid = n < N;

        // ---- this lane's 64 channels of its token (the MFMA B operand) ----
        uint4 xa[8];
        {
            const bf16_t *xp = a.x + (int64_t)h * a.stride_head + n * a.stride_token + half * 64;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                xa[kk] = valid ? *reinterpret_cast<const uint4 *>(xp + kk * 8) : make_uint4(0u, 0u, 0u, 0u);
        }
        float xn = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const uint32_t w[4] = {xa[kk].x, xa[kk].y, xa[kk].z, xa[kk].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bf16x2_t p = __builtin_bit_cast(bf16x2_t, w[e]);
                xn = __builtin_amdgcn_fdot2_f32_bf16(p, p, xn, false);
            }
        }
        xn += __shfl_xor(xn, 32, 64);

        // ---- scores on the matrix cores, running top three per lane -------
        float b1 = -INFINITY, b2 = -INFINITY, b3 = -INFINITY;
        for (int jb = 0; jb < (Kpad >> 5); ++jb) {
            floatx16_t acc;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 v = *reinterpret_cast<const float4 *>(lcnh + jb * 32 + g * 8 + half * 4);
                acc[4 * g + 0] = v.x; acc[4 * g + 1] = v.y; acc[4 * g + 2] = v.z; acc[4 * g + 3] = v.w;
            }
            const bf16_t *arow = lc + (jb * 32 + col) * kCPitch + half * 64;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const bf16x8_t av = *reinterpret_cast<const bf16x8_t *>(arow + kk * 8);
                const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, xa[kk]);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
            }
            const uint32_t tag0 = (uint32_t)jb << 4;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float v = __uint_as_float((__float_as_uint(acc[r]) & kTagMask) | (tag0 + r));
                b3 = __builtin_amdgcn_fmed3f(b2, b3, v);
                b2 = __builtin_amdgcn_fmed3f(b1, b2, v);
                b1 = fmaxf(b1, v);
            }
        }
        // tag -> centroid index: row 8*(r/4) + 4*half + r%4 of block jb
        auto tag_to_idx = [&](float v) {
            const uint32_t t = __float_as_uint(v) & 0x7Fu;
            return (int)((t >> 4) * 32 + ((t >> 2) & 3) * 8 + half * 4 + (t & 3));
        };
        int i1 = tag_to_idx(b1), i2 = tag_to_idx(b2);
        {   // merge with the other half of the wavefront (same token, other centroids)
            const float p1 = __shfl_xor(b1, 32, 64), p2 = __shfl_xor(b2, 32, 64),
                        p3 = __shfl_xor(b3, 32, 64);
            const int q1 = __shfl_xor(i1, 32, 64), q2 = __shfl_xor(i2, 32, 64);
            insert3(p1, q1, b1, b2, b3, i1, i2);
            insert3(p2, q2, b1, b2, b3, i1, i2);
            insert3(p3, 0, b1, b2, b3, i1, i2);
        }
        const float thr = 0x1p-14f * (0.5f * xn + cmax);
        int id = i1;
        const bool amb = valid && (i2 < K) && !(b1 - b2 > thr);
        const bool full = !(b1 - b3 > thr);

        // ---- fp64 re-evaluation of tokens the fp32 scores cannot decide ----
        uint64_t mask = __ballot(amb) & 0xffffffffull;
        while (mask) {
            const int tk = __builtin_ctzll(mask);
            mask &= mask - 1;
            if (col == tk) {
#pragma unroll
                for (int kk = 0; kk < 8; ++kk)
                    *reinterpret_cast<uint4 *>(scr + half * 64 + kk * 8) = xa[kk];
            }
            __builtin_amdgcn_wave_barrier();
            const int c1 = __shfl(i1, tk, 64), c2 = __shfl(i2, tk, 64);
            const int fl = __shfl((int)full, tk, 64);
            int winner;
            if (!fl) {
                const int cand = half ? c2 : c1;
                const uint2 xv = *reinterpret_cast<const uint2 *>(scr + col * 4);
                const uint2 cv = *reinterpret_cast<const uint2 *>(lc + cand * kCPitch + col * 4);
                const double d0 = (double)bf16_lo(xv.x) - (double)bf16_lo(cv.x);
                const double d1 = (double)bf16_hi(xv.x) - (double)bf16_hi(cv.x);
                const double d2 = (double)bf16_lo(xv.y) - (double)bf16_lo(cv.y);
                const double d3 = (double)bf16_hi(xv.y) - (double)bf16_hi(cv.y);
                double d = d0 * d0; d += d1 * d1; d += d2 * d2; d += d3 * d3;
                d += shfl_xor_f64(d, 16); d += shfl_xor_f64(d, 8); d += shfl_xor_f64(d, 4);
                d += shfl_xor_f64(d, 2); d += shfl_xor_f64(d, 1);
                const double D1 = __shfl(d, 0, 64), D2 = __shfl(d, 32, 64);
                winner = (D2 < D1 || (D2 == D1 && c2 < c1)) ? c2 : c1;
            } else {
                double bd = INFINITY; int bj = 0x7fffffff;
                for (int j = lane; j < K; j += 64) {
                    const bf16_t *cr = lc + j * kCPitch;
                    double acc = 0.0;
                    for (int c = 0; c < kHeadDim; c += 2) {
                        const uint32_t xw = *reinterpret_cast<const uint32_t *>(scr + c);
                        const uint32_t cw = *reinterpret_cast<const uint32_t *>(cr + c);
                        const double e0 = (double)bf16_lo(xw) - (double)bf16_lo(cw);
                        acc += e0 * e0;
                        const double e1 = (double)bf16_hi(xw) - (double)bf16_hi(cw);
                        acc += e1 * e1;
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

        if (!FUSED) {
            if (valid && half == 0) a.ids[(int64_t)h * a.out_stride + n] = (uint8_t)id;
            continue;
        }

        // ---- Eq. 5: residual against the assigned centroid -----------------
        float r[64];
        {
            const bf16_t *crow = lc + id * kCPitch + half * 64;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const uint4 cv = *reinterpret_cast<const uint4 *>(crow + kk * 8);
                const uint32_t xw[4] = {xa[kk].x, xa[kk].y, xa[kk].z, xa[kk].w};
                const uint32_t cw[4] = {cv.x, cv.y, cv.z, cv.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    r[kk * 8 + 2 * e] = bf16_lo(xw[e]) - bf16_lo(cw[e]);
                    r[kk * 8 + 2 * e + 1] = bf16_hi(xw[e]) - bf16_hi(cw[e]);
                }
            }
        }
        // ---- T rounds of 2-bit group quantization, packed as they are made --
        constexpr int G = kHeadDim / B_;                 // groups per token
        constexpr int GL = (B_ >= 64) ? 1 : 64 / B_;     // groups held by this lane
        constexpr int NL = (B_ >= 64) ? 64 : B_;         // elements per group in this lane
        const int64_t hn = (int64_t)h * a.out_stride + n;
        if (valid && half == 0) a.ids[hn] = (uint8_t)id;
        for (int t = 0; t < a.T; ++t) {
            uint32_t word[4] = {0x55555555u, 0x55555555u, 0x55555555u, 0x55555555u};
            uint32_t sh[GL];
#pragma unroll
            for (int g = 0; g < GL; ++g) {
                float m = 0.0f;
#pragma unroll
                for (int i = 0; i < NL; ++i) m = fmaxf(m, fabsf(r[g * NL + i]));
                if (B_ == 128) m = fmaxf(m, __shfl_xor(m, 32, 64));
                sh[g] = quant_group<NL>(r + g * NL, m, word, g * NL);
            }
            if (valid) {
                uint8_t *cp = a.codes + (hn * a.T + t) * 32 + half * 16;
                // word[] holds q + 1 per 2-bit field (built with one shift-add per element);
                // the stored form is two's complement: field 00 -> 11, 01 -> 00, 10 -> 01
#pragma unroll
                for (int wi = 0; wi < 4; ++wi) {
                    const uint32_t lo = ~word[wi] & 0x55555555u;
                    word[wi] = lo | (((~word[wi] >> 1) & lo) << 1);
                }
                *reinterpret_cast<uint4 *>(cp) = make_uint4(word[0], word[1], word[2], word[3]);
                f16_t *sp = a.scales + (hn * a.T + t) * G;
                if (B_ == 128) { if (half == 0) sp[0] = (f16_t)sh[0]; }
                else if (B_ == 64) sp[half] = (f16_t)sh[0];
                else if (B_ == 32)
                    *reinterpret_cast<uint32_t *>(sp + half * 2) = sh[0] | (sh[1] << 16);
                else
                    *reinterpret_cast<uint2 *>(sp + half * 4) =
                        make_uint2(sh[0] | (sh[1] << 16), sh[2] | (sh[3] << 16));
            }
        }
    }
}

static size_t assign_smem_bytes(int Kpad) {
    return (size_t)Kpad * kCPitch * 2 + (size_t)Kpad * 4 + 16 + (size_t)kAsgWaves * kHeadDim * 2;
}

template <int B_, bool FUSED>
static hipError_t launch_assign_t(const AssignArgs &a, hipStream_t s) {
    const int Kpad = (a.K + 31) & ~31;
    const size_t smem = assign_smem_bytes(Kpad);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&assign_kernel<B_, FUSED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((a.n_tokens + kAsgTokPerBlock - 1) / kAsgTokPerBlock), (unsigned)a.H);
    hipLaunchKernelGGL((assign_kernel<B_, FUSED>), grid, dim3(kAsgThreads), smem, s, a, Kpad);
    return hipGetLastError();
}

hipError_t launch_assign(const AssignArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    if (!a.fused) return launch_assign_t<64, false>(a, s);
    switch (a.B) {
        case 16: return launch_assign_t<16, true>(a, s);
        case 32: return launch_assign_t<32, true>(a, s);
        case 64: return launch_assign_t<64, true>(a, s);
        default: return launch_assign_t<128, true>(a, s);
    }
}

}  // namespace qvg
