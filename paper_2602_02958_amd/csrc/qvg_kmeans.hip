// k-means update step (paper Sec. 4.1: the centroid is the mean of its group).
//
// The mean is defined with a fixed summation order - members in token order, fp64 -
// so that the result does not depend on scheduling.  Two kernels:
//   rank:  a stable counting sort of the token indices of one unit by cluster id
//          (LDS histogram, scan, then one wavefront places 64 tokens per step using
//          ballot-built peer masks so that equal ids keep their token order);
//   mean:  one wavefront per centroid walks its members in that order, two channels
//          per lane (a 256-byte coalesced row per member), eight rows in flight,
//          adds in fp64, divides by the count, rounds to fp32 and then to bf16.
//          A group without members keeps its previous centroid.
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kRankThreads = 256;

__global__ __launch_bounds__(kRankThreads)
void kmeans_rank_kernel(UpdateArgs a) {
    __shared__ int cnt[256];
    __shared__ int cursor[256];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int K = a.K;
    const int64_t N = a.n_tokens;
    const uint8_t *ids = a.ids + (int64_t)h * a.ids_stride;
    int32_t *perm = a.perm + (int64_t)h * N;
    int32_t *offs = a.offsets + (int64_t)h * (K + 1);

    cnt[tid] = 0;
    __syncthreads();
    // ids at or above K cannot come from the assignment; such tokens are left out
    for (int64_t n = tid; n < N; n += kRankThreads) { const int id = ids[n]; if (id < K) atomicAdd(&cnt[id], 1); }
    __syncthreads();
    if (tid == 0) {                       // exclusive scan over at most 256 bins
        int run = 0;
        for (int j = 0; j < K; ++j) { cursor[j] = run; offs[j] = run; run += cnt[j]; }
        offs[K] = run;
    }
    __syncthreads();
    if (a.counts_out && tid < K) a.counts_out[(int64_t)h * K + tid] = cnt[tid];
    if (tid >= 64) return;                // placement: wavefront 0 only, tokens in order

    for (int64_t base = 0; base < N; base += 64) {
        const int64_t n = base + lane;
        const int id = (n < N) ? (int)ids[n] : 0;
        const bool valid = n < N && id < K;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t m = __ballot((id >> b) & 1);
            peers &= ((id >> b) & 1) ? m : ~m;
        }
        if (valid) {
            const uint64_t below = peers & ((1ull << lane) - 1ull);
            const int rank = __builtin_popcountll(below);
            const int start = cursor[id];             // read by all peers before the write below
            perm[start + rank] = (int32_t)n;
            if (rank == 0) cursor[id] = start + __builtin_popcountll(peers);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

constexpr int kMeanThreads = 256;           // 4 wavefronts = 4 centroids per block

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
    const int64_t co = ((int64_t)h * K + j) * kHeadDim + lane * 2;
    if (end == beg) {
        *reinterpret_cast<uint32_t *>(a.cent_out + co) = *reinterpret_cast<const uint32_t *>(a.cent_prev + co);
        return;
    }
    const bf16_t *xb = a.x + (int64_t)h * a.stride_head + lane * 2;
    double s0 = 0.0, s1 = 0.0;
    int i = beg;
    for (; i + 8 <= end; i += 8) {
        uint32_t w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            w[u] = *reinterpret_cast<const uint32_t *>(xb + (int64_t)perm[i + u] * a.stride_token);
#pragma unroll
        for (int u = 0; u < 8; ++u) { s0 += (double)bf16_lo(w[u]); s1 += (double)bf16_hi(w[u]); }
    }
    for (; i < end; ++i) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(xb + (int64_t)perm[i] * a.stride_token);
        s0 += (double)bf16_lo(w); s1 += (double)bf16_hi(w);
    }
    const double c = (double)(end - beg);
    const float m0 = (float)(s0 / c), m1 = (float)(s1 / c);
    *reinterpret_cast<uint32_t *>(a.cent_out + co) = pack_bf16x2(m0, m1);
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
