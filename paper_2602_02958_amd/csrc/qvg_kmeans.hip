// k-means update step (paper Sec. 4.1: the centroid is the mean of its group).
//
// The mean is defined with a fixed summation order - members in token order, fp64 -
// so that the result does not depend on scheduling.  Two kernels:
//   rank:  a stable counting sort of the token indices of one unit by cluster id
//          (16 wavefronts, each histogramming and then placing its own contiguous range
//          of tokens, ballot-built peer masks keeping equal ids in token order);
//   mean:  one wavefront per centroid adds its members in fp64, divides by the count, rounds
//          to fp32 and then to bf16: in token order for short lists, in four interleaved
//          partial sums for long ones when a test on the members' exponents shows that no
//          addition can round (then every order gives the same bits).
//          A group without members keeps its previous centroid.
// Also here: the residual pass that turns one smoothing stage's output into the next one's
// input (Eq. 5 on whole tensors, result rounded to bf16).
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kRankThreads = 1024;
constexpr int kRankWaves = kRankThreads / 64;      // the tokens of a unit are split into 16 ranges
constexpr int kRankKeep = 8;                        // ids a lane keeps in registers between passes

// Stable counting sort of token indices by cluster id, one workgroup per unit.
// Wavefront w owns the w-th contiguous range of tokens: it histograms the range, and after
// the scan (start of cluster k = tokens of lower clusters + tokens of k in earlier ranges) it
// places the range 64 tokens at a time.  Inside a step, lanes with equal ids are ranked by
// lane number (ballot-built peer masks), so equal ids keep their token order.
__global__ __launch_bounds__(kRankThreads)
void kmeans_rank_kernel(UpdateArgs a) {
    __shared__ int cnt[kRankWaves][256];      // histogram per range, then running cursor
    __shared__ int total[256];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int K = a.K;
    const int64_t N = a.n_tokens;
    const uint8_t *ids = a.ids + (int64_t)h * a.ids_stride * a.ids_step + a.ids_off;   // token n at ids[n * step]
    const int64_t step = a.ids_step;
    int32_t *perm = a.perm + (int64_t)h * N;
    int32_t *offs = a.offsets + (int64_t)h * (K + 1);

    for (int i = tid; i < kRankWaves * 256; i += kRankThreads) (&cnt[0][0])[i] = 0;
    __syncthreads();
    // range of this wavefront, a multiple of 64 tokens long
    const int64_t per = ((N + kRankWaves * 64 - 1) / (kRankWaves * 64)) * 64;
    const int64_t beg = (int64_t)w * per;
    const int64_t end = (beg + per < N) ? beg + per : N;
    const int steps = (int)((per + 63) / 64);
    const bool keep = steps <= kRankKeep;
    int kept[kRankKeep];
    // ids at or above K cannot come from the assignment; such tokens are left out (id = -1)
    if (keep) {
#pragma unroll
        for (int i = 0; i < kRankKeep; ++i) {
            const int64_t n = beg + (int64_t)i * 64 + lane;
            int id = -1;
            if (i < steps && n < end) { id = ids[n * step]; if (id >= K) id = -1; }
            kept[i] = id;
        }
#pragma unroll
        for (int i = 0; i < kRankKeep; ++i) if (kept[i] >= 0) atomicAdd(&cnt[w][kept[i]], 1);
    } else {
        for (int64_t n = beg + lane; n < end; n += 64) { const int id = ids[n * step]; if (id < K) atomicAdd(&cnt[w][id], 1); }
    }
    __syncthreads();
    if (tid < 256) {
        int t = 0;
        for (int r = 0; r < kRankWaves; ++r) t += cnt[r][tid];
        total[tid] = (tid < K) ? t : 0;
    }
    __syncthreads();
    if (tid < 64) {                       // exclusive scan of total[0..255] by one wavefront
        int v[4], run = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[i] = total[lane * 4 + i]; run += v[i]; }
        int incl = run;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        int start = incl - run;
#pragma unroll
        for (int i = 0; i < 4; ++i) { total[lane * 4 + i] = start; start += v[i]; }
    }
    __syncthreads();
    if (tid < 256) {
        // cursor of (range r, cluster tid) = start of the cluster + members in earlier ranges
        int run = total[tid], c = 0;
        for (int r = 0; r < kRankWaves; ++r) { const int t = cnt[r][tid]; cnt[r][tid] = run; run += t; c += t; }
        if (tid < K) {
            offs[tid] = total[tid];
            if (a.counts_out) a.counts_out[(int64_t)h * K + tid] = c;
            if (tid == K - 1) offs[K] = total[tid] + c;
        }
    }
    __syncthreads();

    int nxt = -1;
    if (!keep && beg + lane < end) { nxt = ids[(beg + lane) * step]; if (nxt >= K) nxt = -1; }
    for (int i = 0; i < steps; ++i) {
        const int64_t n = beg + (int64_t)i * 64 + lane;
        int id;
        if (keep) {
            id = -1;
#pragma unroll
            for (int j = 0; j < kRankKeep; ++j) if (j == i) id = kept[j];
        } else {
            id = nxt;
            const int64_t nn = n + 64;
            nxt = -1;
            if (nn < end) { nxt = ids[nn * step]; if (nxt >= K) nxt = -1; }
        }
        const bool valid = id >= 0;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot((id >> b) & 1);
            peers &= ((id >> b) & 1) ? m : ~m;
        }
        if (valid) {
            const int rank = __builtin_popcountll(peers & ((1ull << lane) - 1ull));
            const int start = cnt[w][id];             // read by all peers before the write below
            perm[start + rank] = (int32_t)n;
            if (rank == 0) cnt[w][id] = start + __builtin_popcountll(peers);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

constexpr int kMeanThreads = 256;           // 4 wavefronts = 4 centroids per block
constexpr int kMeanParallelMin = 96;        // member lists at least this long try the order-free path

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// One wavefront per centroid.  The defined result is the fp64 sum of the members in token order.
// Short lists are summed exactly like that (two channels per lane, 16 rows in flight).  A long list
// is latency-bound that way (one dependent fp64 add per member), so it is first summed in FOUR
// interleaved partial sums (lane = member slot x 8 channels, 16-byte row pieces), which is the same
// number whenever no addition rounds: every member is an integer multiple of 2^(emin-134) and every
// partial sum is below n * 256 * 2^(emax-134), with emin / emax the smallest / largest exponent
// field among the non-zero members of the channel, so if
//     ceil(log2 n) + 8 + emax - emin <= 53
// all partial sums of any order are exact in fp64.  The exponents are tracked alongside (packed
// 16-bit min / max of the magnitudes' bit patterns); a centroid with a channel that fails the
// test is summed again in token order.
__global__ __launch_bounds__(kMeanThreads)
void kmeans_mean_kernel(UpdateArgs a) {
    const int h = blockIdx.y, lane = threadIdx.x & 63;
    const int j = blockIdx.x * (kMeanThreads / 64) + (threadIdx.x >> 6);
    const int K = a.K;
    if (j >= K) return;
    const int64_t N = a.n_tokens;
    const int32_t *offs = a.offsets + (int64_t)h * (K + 1);
    const int32_t *perm = a.perm + (int64_t)h * N;
    const int beg = offs[j], end = offs[j + 1];
    const int64_t co = ((int64_t)h * K + j) * kHeadDim;
    if (end == beg) {
        *reinterpret_cast<uint32_t *>(a.cent_out + co + lane * 2) = *reinterpret_cast<const uint32_t *>(a.cent_prev + co + lane * 2);
        return;
    }
    const double c = (double)(end - beg);
    const bf16_t *xu = a.x + (int64_t)h * a.stride_head;

    if (end - beg >= kMeanParallelMin) {
        const int slot = lane >> 4, c8 = lane & 15;
        double s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) s[i] = 0.0;
        uint32_t amax[4] = {0u, 0u, 0u, 0u};                       // per 16-bit half: largest |bits|
        uint32_t amin[4] = {~0u, ~0u, ~0u, ~0u};                   // per half: smallest non-zero |bits|, minus 1
        const bf16_t *xb = xu + c8 * 8;
        for (int base = beg; base < end; base += 64) {
            const int mine = (base + lane < end) ? perm[base + lane] : 0;     // 64 member indices, one coalesced load
            const int cntm = (end - base < 64) ? end - base : 64;
            // slot s takes members s, s + 4, s + 8, .. of the group; 8 rows in flight per lane
            for (int i0 = 0; 4 * i0 < cntm; i0 += 8) {
                uint4 row[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int u = 4 * (i0 + i) + slot;
                    const int idx = __shfl(mine, u & 63, 64);
                    row[i] = (u < cntm) ? *reinterpret_cast<const uint4 *>(xb + (int64_t)idx * a.stride_token)
                                        : make_uint4(0u, 0u, 0u, 0u);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t w[4] = {row[i].x, row[i].y, row[i].z, row[i].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        s[2 * e] += (double)bf16_lo(w[e]);
                        s[2 * e + 1] += (double)bf16_hi(w[e]);
                        const uint32_t mag = w[e] & 0x7fff7fffu;
                        const ushort2_t m2 = __builtin_bit_cast(ushort2_t, mag);
                        amax[e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, amax[e]), m2));
                        const ushort2_t one = {1, 1};
                        amin[e] = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, amin[e]),
                                                                                         (ushort2_t)(m2 - one)));   // zero -> 0xffff
                    }
                }
            }
        }
        // the four slots hold partial results of the same channels: lanes l, l^16, l^32, l^48
        bool ok = true;
        int lg = 0;
        while ((1 << lg) < end - beg) ++lg;                          // ceil(log2 n)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint32_t mx = amax[e], mn = amin[e];
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                const uint32_t omx = __shfl_xor(mx, off, 64), omn = __shfl_xor(mn, off, 64);
                mx = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, mx), __builtin_bit_cast(ushort2_t, omx)));
                mn = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, mn), __builtin_bit_cast(ushort2_t, omn)));
            }
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const uint32_t big = (mx >> (16 * hf)) & 0xffffu, small1 = (mn >> (16 * hf)) & 0xffffu;
                if (small1 == 0xffffu) continue;                     // no non-zero member in this channel: the sum is zero
                const int eb = (int)(big >> 7) > 1 ? (int)(big >> 7) : 1;
                const int es = (int)((small1 + 1u) >> 7) > 1 ? (int)((small1 + 1u) >> 7) : 1;
                if (lg + 8 + eb - es > 53) ok = false;
            }
        }
        if (__all(ok)) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                s[i] += __shfl_xor(s[i], 16, 64);
                s[i] += __shfl_xor(s[i], 32, 64);
            }
            if (slot == 0) {
                float m[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) m[i] = (float)(s[i] / c);
                *reinterpret_cast<uint4 *>(a.cent_out + co + c8 * 8) = pack_bf16x8(m);
            }
            return;
        }
    }
    // token order: two channels per lane, 16 rows in flight
    double s0 = 0.0, s1 = 0.0;
    const bf16_t *xb = xu + lane * 2;
    for (int base = beg; base < end; base += 64) {
        // 64 member indices with one coalesced load, then broadcast lane by lane
        const int mine = (base + lane < end) ? perm[base + lane] : 0;
        const int cntm = (end - base < 64) ? end - base : 64;
        for (int u0 = 0; u0 < cntm; u0 += 16) {
            uint32_t wv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int idx = __shfl(mine, u0 + u, 64);
                wv[u] = (u0 + u < cntm)
                    ? *reinterpret_cast<const uint32_t *>(xb + (int64_t)idx * a.stride_token) : 0u;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (u0 + u < cntm) { s0 += (double)bf16_lo(wv[u]); s1 += (double)bf16_hi(wv[u]); }
        }
    }
    const float m0 = (float)(s0 / c), m1 = (float)(s1 / c);
    *reinterpret_cast<uint32_t *>(a.cent_out + co + lane * 2) = pack_bf16x2(m0, m1);
}

// Residual for the next smoothing stage: 16 lanes per token, 8 channels each.
__global__ __launch_bounds__(256)
void residual_kernel(ResidualArgs a) {
    const int h = blockIdx.y;
    const int64_t n = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c8 = threadIdx.x & 15;
    if (n >= a.n_tokens) return;
    int id = a.ids[((int64_t)h * a.ids_stride + n) * a.ids_step + a.ids_off];
    if (id >= a.K) id = a.K - 1;
    const uint4 xv = *reinterpret_cast<const uint4 *>(a.x + (int64_t)h * a.stride_head + n * a.stride_token + c8 * 8);
    const uint4 cv = *reinterpret_cast<const uint4 *>(a.cent + ((int64_t)h * a.K + id) * kHeadDim + c8 * 8);
    float xf[8], cf[8], r[8];
    unpack_bf16x8(xv, xf);
    unpack_bf16x8(cv, cf);
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = xf[i] - cf[i];
    *reinterpret_cast<uint4 *>(a.out + ((int64_t)h * a.n_tokens + n) * kHeadDim + c8 * 8) = pack_bf16x8(r);
}

hipError_t launch_residual(const ResidualArgs &a, hipStream_t s) {
    if (a.n_tokens == 0) return hipSuccess;
    dim3 grid((unsigned)((a.n_tokens + 15) / 16), (unsigned)a.H);
    hipLaunchKernelGGL(residual_kernel, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_update(const UpdateArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(kmeans_rank_kernel, dim3((unsigned)a.H), dim3(kRankThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((a.K + 3) / 4), (unsigned)a.H);
    hipLaunchKernelGGL(kmeans_mean_kernel, grid, dim3(kMeanThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace qvg
