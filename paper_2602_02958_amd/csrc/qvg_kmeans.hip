// k-means update step (paper Sec. 4.1: the centroid is the mean of its group).
//
// The mean is defined with a fixed summation order - members in token order, fp64 -
// so that the result does not depend on scheduling.  Two kernels:
//   rank:  a stable counting sort of the token indices of one unit by cluster id
//          (16 wavefronts, each histogramming and then placing its own contiguous range
//          of tokens, ballot-built peer masks keeping equal ids in token order);
//   mean:  one wavefront per centroid walks its members in that order, two channels
//          per lane (a 256-byte coalesced row per member), up to 128 rows in flight,
//          adds in fp64, divides by the count, rounds to fp32 and then to bf16.
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

// WIDE: many members per centroid (few, long waves): see the comments inside
template <bool WIDE>
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
    double s0 = 0.0, s1 = 0.0;
    if (!WIDE) {
        // few members per centroid (many small waves): 16 rows in flight, few registers
        const bf16_t *xb = a.x + (int64_t)h * a.stride_head + lane * 2;
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
    } else {
        // Members are walked 64 at a time: one coalesced load brings their indices (one group
        // ahead), a constant-lane read moves each index into a scalar register, so the row address is
        // scalar arithmetic, and all 64 rows of the NEXT group are requested before the current
        // group is added.  The additions are strictly ordered (fp64, token order); with two groups
        // in flight they run in the shadow of the loads.
        const bf16_t *xu = a.x + (int64_t)h * a.stride_head;
        auto load64 = [&](int mine, int cntm, uint32_t (&wv)[64]) {
#pragma unroll
            for (int u = 0; u < 64; ++u) {
                const int idx = __builtin_amdgcn_readlane(mine, u);
                const bf16_t *row = xu + (int64_t)idx * a.stride_token;
                wv[u] = (u < cntm) ? *reinterpret_cast<const uint32_t *>(row + lane * 2) : 0u;   // uniform condition
            }
        };
        auto add64 = [&](int cntm, const uint32_t (&wv)[64]) {
            if (cntm == 64) {
#pragma unroll
                for (int u = 0; u < 64; ++u) { s0 += (double)bf16_lo(wv[u]); s1 += (double)bf16_hi(wv[u]); }
            } else {
#pragma unroll
                for (int u = 0; u < 64; ++u)
                    if (u < cntm) { s0 += (double)bf16_lo(wv[u]); s1 += (double)bf16_hi(wv[u]); }
            }
        };
        auto count_at = [&](int base) { return (end - base < 64) ? end - base : 64; };
        auto indices_at = [&](int base) { return (base + lane < end) ? perm[base + lane] : 0; };
        uint32_t wa[64], wb[64];
        int mine_b = indices_at(beg + 64);
        load64(indices_at(beg), count_at(beg), wa);
        for (int base = beg; base < end; base += 128) {
            // group B = [base + 64, base + 128), group A' = [base + 128, base + 192)
            const int mine_a = indices_at(base + 128);
            if (base + 64 < end) load64(mine_b, count_at(base + 64), wb);
            add64(count_at(base), wa);
            if (base + 64 >= end) break;
            mine_b = indices_at(base + 192);
            if (base + 128 < end) load64(mine_a, count_at(base + 128), wa);
            add64(count_at(base + 64), wb);
        }
    }
    const double c = (double)(end - beg);
    const float m0 = (float)(s0 / c), m1 = (float)(s1 / c);
    *reinterpret_cast<uint32_t *>(a.cent_out + co) = pack_bf16x2(m0, m1);
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
    // long member lists are latency-bound on their ordered sums: more rows in flight pays there
    if (a.n_tokens / a.K >= 48) hipLaunchKernelGGL(kmeans_mean_kernel<true>, grid, dim3(kMeanThreads), 0, s, a);
    else hipLaunchKernelGGL(kmeans_mean_kernel<false>, grid, dim3(kMeanThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace qvg
